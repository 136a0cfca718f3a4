/*
 * CPU oracle for KCache decode-step attention and its cache store.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path, is
 * never linked into it, and must not be called from any product code path.
 *
 * What it computes (paper section 3.1, Table 1 rows "S~ = TopN(softmax(Q K^T /
 * sqrt(d_h)))" and "A~ = S~ Part(V)", Figure 1 lower half, section 3.3 for the
 * per-(sequence, head) granularity):
 *
 *   for every sequence b and query head i, over the s_b cached positions,
 *     z[t]  = (q . K[t]) / sqrt(d_h)                  (scores)
 *     p[t]  = exp(z[t] - max z) / sum_t exp(z[t] - max z)   (softmax over ALL t)
 *     I     = the N positions with the largest p       (TopN)
 *     out   = sum_{t in I} p[t] * V[t]                 (partial V, weighted)
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - the kept weights are the full-context softmax values, not renormalised
 *     (the formula is literally TopN applied to the softmax output);
 *   - ordering is decided on z, which orders exactly like p in exact
 *     arithmetic (exp is strictly increasing), lower position wins a tie;
 *   - N_eff = min(N, s_b);
 *   - d_h is the per-head dimension;
 *   - grouped-query attention: query head i reads KV head i / (H / Hkv).
 *
 * Arithmetic: every stored 16-bit value is decoded exactly to double, all
 * sums and the softmax are in double.  No blocking, fusion or reordering.
 *
 * Parity pins (tests/test_oracle_pins.py): softmax sums to one, shift
 * invariance, N = s against a library attention routine, brute-force sort,
 * uniform-score closed form, two-score logistic closed form, GQA by head
 * repetition, ragged batch by independent calls, 16-bit decode against a
 * library decode; the conventional-attention routine against the same library
 * routine, a uniform-score closed form and the N = s case of the top-N routine;
 * the cache store (both forms) bit for bit against a slice assignment of rows with
 * distinct elements.
 * The no-renormalisation reading itself is "parity unpinned"
 * by the paper: only the literal formula fixes it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KCO_F16 0
#define KCO_BF16 1

/* IEEE binary16 bit pattern -> double, exact. */
static double kco_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int expo = (h >> 10) & 0x1f;
  int frac = h & 0x3ff;
  double v;
  if (expo == 0) {
    v = ldexp((double)frac, -24); /* subnormal: frac * 2^-10 * 2^-14 */
  } else if (expo == 31) {
    v = frac ? NAN : INFINITY;
  } else {
    v = ldexp((double)(frac + 1024), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
  }
  return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exact (sign, 8 exponent bits, 7 fraction bits). */
static double kco_bf16_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int expo = (h >> 7) & 0xff;
  int frac = h & 0x7f;
  double v;
  if (expo == 0) {
    v = ldexp((double)frac, -133); /* frac * 2^-7 * 2^-126 */
  } else if (expo == 255) {
    v = frac ? NAN : INFINITY;
  } else {
    v = ldexp((double)(frac + 128), expo - 134); /* (1 + frac/128) * 2^(expo-127) */
  }
  return sign ? -v : v;
}

static double kco_decode(uint16_t bits, int dtype) {
  return dtype == KCO_BF16 ? kco_bf16_to_double(bits) : kco_half_to_double(bits);
}

/*
 * 8-bit K storage (a variant outside the paper's own experiments; section 1 names
 * cache quantisation as the other way to cut the bytes a decode step moves).  The
 * code is OCP FP8 E4M3: 1 sign bit, 4 exponent bits with bias 7, 3 fraction bits,
 * no infinities, S.1111.111 is NaN, largest finite value 448.  A K element is
 * stored as code(k * 2^-e) for one integer e per cache and read back as
 * value(code) * 2^e.  The power-of-two scale makes every step exact, so the stored
 * byte is a pure function of the 16-bit input.
 */
static double kco_e4m3_to_double(uint8_t b) {
  int sign = (b >> 7) & 1;
  int expo = (b >> 3) & 0xf;
  int frac = b & 7;
  double v;
  if (expo == 15 && frac == 7) {
    v = NAN;
  } else if (expo == 0) {
    v = ldexp((double)frac, -9); /* subnormal: frac/8 * 2^-6 */
  } else {
    v = ldexp((double)(frac + 8), expo - 10); /* (1 + frac/8) * 2^(expo-7) */
  }
  return sign ? -v : v;
}

/* Nearest E4M3 code of x, ties to the even code, magnitudes above 448 saturate to
 * 448, NaN gives the NaN code.  Zero keeps its sign. */
static uint8_t kco_double_to_e4m3(double x) {
  uint8_t sign = signbit(x) ? 0x80 : 0;
  if (isnan(x)) return (uint8_t)(sign | 0x7f);
  double a = fabs(x);
  if (a >= 448.0) return (uint8_t)(sign | 0x7e);
  if (a == 0.0) return sign;
  int e;
  (void)frexp(a, &e); /* a = f * 2^e with f in [0.5, 1): a lies in [2^(e-1), 2^e) */
  int expo = e - 1;   /* floor(log2 a) */
  if (expo < -6) expo = -6; /* subnormal codes share the spacing of the smallest normals */
  /* spacing of the codes in this binade is 2^(expo-3); nearbyint rounds ties to even */
  double n = nearbyint(ldexp(a, 3 - expo)); /* 8..16 for normals, 0..8 below 2^-6 */
  double v = ldexp(n, expo - 3);            /* the rounded magnitude, exactly representable */
  if (v == 0.0) return sign;
  if (v < ldexp(1.0, -6)) return (uint8_t)(sign | (int)ldexp(v, 9)); /* subnormal: frac = v * 2^9 */
  (void)frexp(v, &e);
  int ve = e - 1;
  int frac = (int)(ldexp(v, 3 - ve)) - 8;
  return (uint8_t)(sign | ((ve + 7) << 3) | frac);
}

/* Exposed for the pins: decode of codes, and quantisation of 16-bit values k as
 * code(k * 2^-k_exp). */
void kcache_oracle_e4m3_decode(const uint8_t* codes, int64_t n, double* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = kco_e4m3_to_double(codes[i]);
}
void kcache_oracle_e4m3_quantise(const uint16_t* bits, int64_t n, int dtype, int k_exp,
                                 uint8_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = kco_double_to_e4m3(ldexp(kco_decode(bits[i], dtype), -k_exp));
}

/* Exposed so the decode can be pinned against a library conversion. */
void kcache_oracle_decode16(const uint16_t* bits, int64_t n, int dtype, double* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = kco_decode(bits[i], dtype);
}

typedef struct {
  double z;
  int32_t t;
} kco_scored;

/* Larger score first; equal scores: lower position first. */
static int kco_cmp_scored(const void* a, const void* b) {
  const kco_scored* x = (const kco_scored*)a;
  const kco_scored* y = (const kco_scored*)b;
  if (x->z > y->z) return -1;
  if (x->z < y->z) return 1;
  return (x->t > y->t) - (x->t < y->t);
}

static int kco_cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/*
 * One (sequence, query head) unit.
 *   q      [d]      stored 16-bit values
 *   K, V   [s][d]   rows of the shared KV head, position-major
 *   out    [d]      double
 *   idx    [N]      selected positions ascending, -1 beyond N_eff
 *   w      [N]      their softmax weights, 0 beyond N_eff
 *   z_out  [s]      optional (may be NULL): scaled scores
 *   p_out  [s]      optional (may be NULL): full softmax
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
/* K comes either as 16-bit values (K) or, when K8 is given, as E4M3 codes with the
 * cache's exponent k_exp. */
static int kco_unit(const uint16_t* q, const uint16_t* K, const uint8_t* K8, int k_exp,
                    const uint16_t* V, int dtype, int32_t s, int32_t d, int32_t N,
                    int renormalise, double* out, int32_t* idx, double* w, double* z_out,
                    double* p_out) {
  if (!q || (!K && !K8) || !V || !out || !idx || !w || s < 1 || d < 1 || N < 1) return -1;
  double* z = (double*)malloc(sizeof(double) * (size_t)s);
  double* p = (double*)malloc(sizeof(double) * (size_t)s);
  double* qd = (double*)malloc(sizeof(double) * (size_t)d);
  kco_scored* order = (kco_scored*)malloc(sizeof(kco_scored) * (size_t)s);
  if (!z || !p || !qd || !order) {
    free(z); free(p); free(qd); free(order);
    return -1;
  }
  for (int32_t c = 0; c < d; ++c) qd[c] = kco_decode(q[c], dtype);

  /* scores: z[t] = (q . K[t]) / sqrt(d_h) */
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  for (int32_t t = 0; t < s; ++t) {
    double acc = 0.0;
    for (int32_t c = 0; c < d; ++c) {
      const double k = K8 ? ldexp(kco_e4m3_to_double(K8[(size_t)t * d + c]), k_exp)
                          : kco_decode(K[(size_t)t * d + c], dtype);
      acc += qd[c] * k;
    }
    z[t] = acc * inv_sqrt_d;
  }

  /* softmax over all s positions */
  double m = z[0];
  for (int32_t t = 1; t < s; ++t)
    if (z[t] > m) m = z[t];
  double Z = 0.0;
  for (int32_t t = 0; t < s; ++t) {
    p[t] = exp(z[t] - m);
    Z += p[t];
  }
  for (int32_t t = 0; t < s; ++t) p[t] /= Z;

  /* TopN: order all positions by (score descending, position ascending) */
  for (int32_t t = 0; t < s; ++t) {
    order[t].z = z[t];
    order[t].t = t;
  }
  qsort(order, (size_t)s, sizeof(kco_scored), kco_cmp_scored);
  int32_t n_eff = N < s ? N : s;
  for (int32_t j = 0; j < n_eff; ++j) idx[j] = order[j].t;
  qsort(idx, (size_t)n_eff, sizeof(int32_t), kco_cmp_i32);
  for (int32_t j = n_eff; j < N; ++j) idx[j] = -1;

  /* weighted sum of the selected V rows; the weights are the full-context softmax values
     (NOT renormalised) unless the variant is asked for, which divides them by their sum */
  double kept = 0.0;
  for (int32_t j = 0; j < n_eff; ++j) kept += p[idx[j]];
  const double divisor = renormalise ? kept : 1.0;
  for (int32_t c = 0; c < d; ++c) out[c] = 0.0;
  for (int32_t j = 0; j < N; ++j) {
    if (j >= n_eff) {
      w[j] = 0.0;
      continue;
    }
    int32_t t = idx[j];
    w[j] = p[t] / divisor;
    for (int32_t c = 0; c < d; ++c) out[c] += w[j] * kco_decode(V[(size_t)t * d + c], dtype);
  }

  if (z_out) memcpy(z_out, z, sizeof(double) * (size_t)s);
  if (p_out) memcpy(p_out, p, sizeof(double) * (size_t)s);
  free(z); free(p); free(qd); free(order);
  return 0;
}

int kcache_oracle_unit(const uint16_t* q, const uint16_t* K, const uint16_t* V, int dtype,
                       int32_t s, int32_t d, int32_t N, double* out, int32_t* idx, double* w,
                       double* z_out, double* p_out) {
  return kco_unit(q, K, NULL, 0, V, dtype, s, d, N, 0, out, idx, w, z_out, p_out);
}

/*
 * Variant of the unit above in which the N kept weights are divided by their sum,
 * so that they add up to one.  The paper's formula does not do this (Table 1:
 * TopN applied to the softmax output); its passing remark in section 4 that TopN
 * acts as a regulariser of the softmax is the only hint at such a variant.  Everything up
 * to and including the selection is identical.
 */
int kcache_oracle_unit_renormalised(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                                    int dtype, int32_t s, int32_t d, int32_t N, double* out,
                                    int32_t* idx, double* w, double* z_out, double* p_out) {
  return kco_unit(q, K, NULL, 0, V, dtype, s, d, N, 1, out, idx, w, z_out, p_out);
}

/* The unit with its K rows stored as E4M3 codes K8 [s][d] and the exponent k_exp. */
int kcache_oracle_unit_k8(const uint16_t* q, const uint8_t* K8, int k_exp, const uint16_t* V,
                          int dtype, int32_t s, int32_t d, int32_t N, double* out, int32_t* idx,
                          double* w, double* z_out, double* p_out) {
  return kco_unit(q, NULL, K8, k_exp, V, dtype, s, d, N, 0, out, idx, w, z_out, p_out);
}

/*
 * One layer, whole batch.
 *   q         [B][H][d]
 *   K, V      [B][Hkv][S_cap][d]   (V read from ordinary host memory)
 *   seq_lens  [B]   1 <= s_b <= S_cap
 *   out       [B][H][d] double;  idx [B][H][N];  w [B][H][N]
 *   nthreads  units are independent; they are split over this many threads
 *             (the only parallelism).  <= 1 runs serially.
 * Returns 0, or -1 on bad arguments.
 */
int kcache_oracle_decode(const uint16_t* q, const uint16_t* K, const uint16_t* V, int dtype,
                         int32_t B, int32_t H, int32_t Hkv, int32_t S_cap, int32_t d,
                         const int32_t* seq_lens, int32_t N, double* out, int32_t* idx, double* w,
                         int nthreads) {
  if (!q || !K || !V || !seq_lens || !out || !idx || !w) return -1;
  if (B < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || S_cap < 1 || d < 1 || N < 1) return -1;
  for (int32_t b = 0; b < B; ++b)
    if (seq_lens[b] < 1 || seq_lens[b] > S_cap) return -1;
  const int32_t G = H / Hkv;
  int status = 0;
  int64_t units = (int64_t)B * H;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 1 ? nthreads : 1)
  for (int64_t u = 0; u < units; ++u) {
    int32_t b = (int32_t)(u / H), h = (int32_t)(u % H);
    int32_t hk = h / G;
    size_t kv_off = ((size_t)b * Hkv + hk) * (size_t)S_cap * d;
    int rc = kcache_oracle_unit(q + (size_t)u * d, K + kv_off, V + kv_off, dtype, seq_lens[b], d, N,
                                out + (size_t)u * d, idx + (size_t)u * N, w + (size_t)u * N, NULL,
                                NULL);
    if (rc != 0) {
#pragma omp atomic write
      status = -1;
    }
  }
  return status;
}

/*
 * Conventional decode attention, the baseline the method is compared with
 * (paper section 2: Attention(Q, K, V) = softmax(Q K^T / sqrt(d_h)) V; Table 1
 * rows "S = softmax(Q K^T / sqrt(d_h))" and "A = S V"; section 3.1 and the
 * caption of Table 2: the first L layers keep their V cache in HBM).  Every
 * position contributes; nothing is selected.  Written out on its own, not as a
 * call of the top-N routine, so that the two can be checked against each other.
 *   q [d], K [s][d], V [s][d] stored 16-bit values; out [d] double
 *   p_out [s] optional (may be NULL): the softmax
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int kcache_oracle_full_unit(const uint16_t* q, const uint16_t* K, const uint16_t* V, int dtype,
                            int32_t s, int32_t d, double* out, double* p_out) {
  if (!q || !K || !V || !out || s < 1 || d < 1) return -1;
  double* z = (double*)malloc(sizeof(double) * (size_t)s);
  if (!z) return -1;
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  for (int32_t t = 0; t < s; ++t) {
    double acc = 0.0;
    for (int32_t c = 0; c < d; ++c)
      acc += kco_decode(q[c], dtype) * kco_decode(K[(size_t)t * d + c], dtype);
    z[t] = acc * inv_sqrt_d;
  }
  double m = z[0];
  for (int32_t t = 1; t < s; ++t)
    if (z[t] > m) m = z[t];
  double Z = 0.0;
  for (int32_t t = 0; t < s; ++t) Z += exp(z[t] - m);
  for (int32_t c = 0; c < d; ++c) out[c] = 0.0;
  for (int32_t t = 0; t < s; ++t) {
    const double p = exp(z[t] - m) / Z;
    if (p_out) p_out[t] = p;
    for (int32_t c = 0; c < d; ++c) out[c] += p * kco_decode(V[(size_t)t * d + c], dtype);
  }
  free(z);
  return 0;
}

/*
 * Conventional attention for one layer, whole batch; same layouts, GQA mapping
 * and threading as kcache_oracle_decode.  out [B][H][d] double.
 */
int kcache_oracle_full_attention(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                                 int dtype, int32_t B, int32_t H, int32_t Hkv, int32_t S_cap,
                                 int32_t d, const int32_t* seq_lens, double* out, int nthreads) {
  if (!q || !K || !V || !seq_lens || !out) return -1;
  if (B < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || S_cap < 1 || d < 1) return -1;
  for (int32_t b = 0; b < B; ++b)
    if (seq_lens[b] < 1 || seq_lens[b] > S_cap) return -1;
  const int32_t G = H / Hkv;
  int status = 0;
  int64_t units = (int64_t)B * H;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 1 ? nthreads : 1)
  for (int64_t u = 0; u < units; ++u) {
    int32_t b = (int32_t)(u / H), h = (int32_t)(u % H);
    size_t kv_off = ((size_t)b * Hkv + h / G) * (size_t)S_cap * d;
    int rc = kcache_oracle_full_unit(q + (size_t)u * d, K + kv_off, V + kv_off, dtype,
                                     seq_lens[b], d, out + (size_t)u * d, NULL);
    if (rc != 0) {
#pragma omp atomic write
      status = -1;
    }
  }
  return status;
}

/*
 * Cache store (Figure 1 upper half and caption: every layer's K states are
 * pushed to the HBM cache, V states end up in CPU memory; in decode the new
 * token's states are appended the same way).
 *   k_new, v_new  [B][T][Hkv][d]  token-major, as a projection produces them
 *   k_cache, v_cache [B][Hkv][S_cap][d]
 *   pos [B]  first position written for each sequence; pos[b] + T <= S_cap
 * Pure data movement; bits are copied unchanged.
 */
int kcache_oracle_store(uint16_t* k_cache, uint16_t* v_cache, const uint16_t* k_new,
                        const uint16_t* v_new, const int32_t* pos, int32_t B, int32_t T,
                        int32_t Hkv, int32_t S_cap, int32_t d) {
  if (!k_cache || !v_cache || !k_new || !v_new || !pos) return -1;
  if (B < 1 || T < 1 || Hkv < 1 || S_cap < 1 || d < 1) return -1;
  for (int32_t b = 0; b < B; ++b)
    if (pos[b] < 0 || (int64_t)pos[b] + T > S_cap) return -1;
  for (int32_t b = 0; b < B; ++b)
    for (int32_t t = 0; t < T; ++t)
      for (int32_t hk = 0; hk < Hkv; ++hk)
        for (int32_t c = 0; c < d; ++c) {
          size_t src = (((size_t)b * T + t) * Hkv + hk) * d + c;
          size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + t)) * d + c;
          k_cache[dst] = k_new[src];
          v_cache[dst] = v_new[src];
        }
  return 0;
}

/*
 * The same store for a cache whose K rows are kept as E4M3 codes with exponent
 * k_exp (see kco_double_to_e4m3): K rows are quantised on the way in, V rows are
 * copied unchanged.  k8_cache [B][Hkv][S_cap][d] bytes.
 */
int kcache_oracle_store_k8(uint8_t* k8_cache, uint16_t* v_cache, const uint16_t* k_new,
                           const uint16_t* v_new, const int32_t* pos, int32_t B, int32_t T,
                           int32_t Hkv, int32_t S_cap, int32_t d, int dtype, int k_exp) {
  if (!k8_cache || !v_cache || !k_new || !v_new || !pos) return -1;
  if (B < 1 || T < 1 || Hkv < 1 || S_cap < 1 || d < 1) return -1;
  for (int32_t b = 0; b < B; ++b)
    if (pos[b] < 0 || (int64_t)pos[b] + T > S_cap) return -1;
  for (int32_t b = 0; b < B; ++b)
    for (int32_t t = 0; t < T; ++t)
      for (int32_t hk = 0; hk < Hkv; ++hk)
        for (int32_t c = 0; c < d; ++c) {
          size_t src = (((size_t)b * T + t) * Hkv + hk) * d + c;
          size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + t)) * d + c;
          k8_cache[dst] = kco_double_to_e4m3(ldexp(kco_decode(k_new[src], dtype), -k_exp));
          v_cache[dst] = v_new[src];
        }
  return 0;
}
