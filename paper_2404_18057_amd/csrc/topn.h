// Block-wide exact top-k selection over fp32 scores (paper section 3.1; Table 1
// row S~: the N largest softmax entries of a (sequence, head) are kept).
//
// Scores are mapped to unsigned keys whose integer order is the float order and
// ordered by (key descending, index ascending): "largest first, lower index on
// ties".  The k-th entry in that order is the threshold (T, T_idx); an entry is
// kept iff key > T or (key == T and index <= T_idx).
//
//   pass 1   LDS histogram of key bits 31..21 -> the bin holding the k-th entry;
//   resolve  the few entries of that bin are copied to an LDS list and ranked
//            against each other directly (all pairs, tie-break included), which
//            names the threshold entry without further passes;
//   fallback a bin too crowded for the list is split again on bits 20..10 and
//            resolved the same way; if even that bin is too crowded (many equal
//            scores) a third pass on bits 9..0 leaves exactly equal keys, which
//            are kept in index order by an ordered count;
//   emit     kept entries are written in ascending index order by an ordered
//            (ballot + prefix) compaction: nothing depends on the arrival order
//            of an atomic.
//
// Scores are read through a caller-supplied accessor keys(i), so they can live
// in LDS, in global memory, or behind a cache-bypassing load.
//
// The second half of the file holds the same selection for ONE wavefront (wave_topn, no
// workgroup barrier: several heads of a query group are selected at the same time by
// different wavefronts); it orders entries the same way and is described there.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kc {

constexpr int kTopNListCap = 512;

template <int NT>
struct alignas(16) TopNScratch {
  uint32_t hist[2048];
  uint32_t list_key[kTopNListCap];
  int list_idx[kTopNListCap];
  int list_rank[kTopNListCap];
  int wave_tot[NT / 64];
  int seg_a[NT / 64];
  int seg_b[NT / 64];
  float red_m[NT / 64];
  float red_l[NT / 64];
  float red_b[NT / 64];
  int bin, bin2, rank, list_cnt;
  uint32_t thr_key;
  int thr_idx;
};

__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;  // -0 and +0 are the same score
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Reads keys(i0), keys(i0 + stride), ... (U of them, 0 beyond n) before any is
// used, so that the read latencies overlap.
template <int U, typename Key>
__device__ __forceinline__ void load_keys(Key keys, int i0, int stride, int n, float (&v)[U]) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int i = i0 + u * stride;
    v[u] = (i < n) ? keys(i) : 0.f;
  }
}

// ---- wavefront primitives on DPP (no LDS traffic, a handful of cycles per step)

template <int CTRL>
__device__ __forceinline__ int dpp_i(int x) {  // lanes without a source read 0
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_bit_cast(float, dpp_i<CTRL>(__builtin_bit_cast(int, x)));
}

// Sum over the 64 lanes, returned to every lane.
__device__ __forceinline__ int wave_sum(int x) {
  x += dpp_i<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_i<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_i<0x141>(x);  // row_half_mirror
  x += dpp_i<0x140>(x);  // row_mirror: every lane of a 16-lane row holds the row sum
  return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) +
         __builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48);
}
__device__ __forceinline__ float wave_sum(float x) {
  x += dpp_f<0xB1>(x);
  x += dpp_f<0x4E>(x);
  x += dpp_f<0x141>(x);
  x += dpp_f<0x140>(x);
  const int xi = __builtin_bit_cast(int, x);
  return (__builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0)) +
          __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16))) +
         (__builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 32)) +
          __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 48)));
}
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_f<0xB1>(x));   // out-of-row sources cannot occur for these four patterns
  x = fmaxf(x, dpp_f<0x4E>(x));
  x = fmaxf(x, dpp_f<0x141>(x));
  x = fmaxf(x, dpp_f<0x140>(x));
  const int xi = __builtin_bit_cast(int, x);
  return fmaxf(fmaxf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0)),
                     __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16))),
               fmaxf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 32)),
                     __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 48))));
}

__device__ __forceinline__ float wave_min(float x) { return -wave_max(-x); }

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
  v += dpp_i<0x111>(v);  // row_shr:1
  v += dpp_i<0x112>(v);  // row_shr:2
  v += dpp_i<0x114>(v);  // row_shr:4
  v += dpp_i<0x118>(v);  // row_shr:8: inclusive scan inside each 16-lane row
  const int r0 = __builtin_amdgcn_readlane(v, 15), r1 = __builtin_amdgcn_readlane(v, 31),
            r2 = __builtin_amdgcn_readlane(v, 47);
  const int row = lane >> 4;
  return v + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

// Exclusive prefix sum of one int per thread over the block.
template <int NT>
__device__ __forceinline__ int block_excl_scan(int v, int* wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = wave_incl_scan(v, lane);
  __syncthreads();  // wave_tot may still be read from an earlier use
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int before = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) before += (w < wave) ? wave_tot[w] : 0;
  return before + inc - v;
}

// Finds, counting from the top bin, the bin that holds the k-th largest key:
// above(D) < k <= above(D) + hist[D].  Leaves D in sc->bin and k - above(D) in
// sc->rank; with k2 > 0 also the bin of the k2-th largest key in sc->bin2 (same scan).
// Ends with a barrier.
template <int NT, int NBINS>
__device__ __forceinline__ void find_bin(TopNScratch<NT>* sc, int k, int k2 = 0) {
  constexpr int PER = NBINS / NT;
  static_assert(NBINS % NT == 0, "bins must divide over the threads");
  const int top = NBINS - 1 - (int)threadIdx.x * PER;  // this thread owns top, top-1, ...
  int c[PER], mine = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    c[j] = (int)sc->hist[top - j];
    mine += c[j];
  }
  int above = block_excl_scan<NT>(mine, sc->wave_tot);
  const bool has_k = above < k && k <= above + mine;
  const bool has_k2 = k2 > 0 && above < k2 && k2 <= above + mine;
  if (has_k || has_k2) {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (has_k && above < k && k <= above + c[j]) {
        sc->bin = top - j;
        sc->rank = k - above;
      }
      if (has_k2 && above < k2 && k2 <= above + c[j]) sc->bin2 = top - j;
      above += c[j];
    }
  }
  __syncthreads();
}

// Merges one (max, sum of exp(. - max)) pair per thread into the block's pair,
// returned to every thread.  Two barriers.  A thread without data carries
// (-inf, 0); its term vanishes instead of becoming NaN.
template <int NT>
__device__ __forceinline__ float2 block_merge_stats(float m, float l, TopNScratch<NT>* sc) {
  const int tid = threadIdx.x;
  const float wm = wave_max(m);
  l = wave_sum(m == wm ? l : l * __expf(m - wm));  // (-inf, 0) lanes contribute 0
  __syncthreads();
  if ((tid & 63) == 0) {
    sc->red_m[tid >> 6] = wm;
    sc->red_l[tid >> 6] = l;
  }
  __syncthreads();
  float mm = sc->red_m[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) mm = fmaxf(mm, sc->red_m[w]);
  float ll = 0.f;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const float mw = sc->red_m[w];
    ll += (mw == mm) ? sc->red_l[w] : sc->red_l[w] * __expf(mw - mm);
  }
  return make_float2(mm, ll);
}

// The same with a third value per thread whose minimum over the block is returned in .z.
template <int NT>
__device__ __forceinline__ float3 block_merge_stats_min(float m, float l, float b,
                                                        TopNScratch<NT>* sc) {
  const int tid = threadIdx.x;
  const float wm = wave_max(m);
  l = wave_sum(m == wm ? l : l * __expf(m - wm));
  b = wave_min(b);
  __syncthreads();
  if ((tid & 63) == 0) {
    sc->red_m[tid >> 6] = wm;
    sc->red_l[tid >> 6] = l;
    sc->red_b[tid >> 6] = b;
  }
  __syncthreads();
  float mm = sc->red_m[0], bb = sc->red_b[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) {
    mm = fmaxf(mm, sc->red_m[w]);
    bb = fminf(bb, sc->red_b[w]);
  }
  float ll = 0.f;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const float mw = sc->red_m[w];
    ll += (mw == mm) ? sc->red_l[w] : sc->red_l[w] * __expf(mw - mm);
  }
  return make_float3(mm, ll, bb);
}

// Softmax partials of keys(0..n-1): (max, sum of exp(key - max)) to every thread.
// Each thread reduces its own keys around its own maximum, then the pairs merge.
template <int NT, typename Key>
__device__ __forceinline__ float2 block_softmax_stats(Key keys, int n, TopNScratch<NT>* sc) {
  constexpr int U = 8;
  float m = -INFINITY;
  for (int i0 = threadIdx.x; i0 < n; i0 += NT * U) {
    float v[U];
    load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + u * NT < n) m = fmaxf(m, v[u]);
  }
  float l = 0.f;
  for (int i0 = threadIdx.x; i0 < n; i0 += NT * U) {
    float v[U];
    load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + u * NT < n) l += __expf(v[u] - m);
  }
  return block_merge_stats<NT>(m, l, sc);
}

// Selects the k largest of keys(0..n-1) (1 <= k <= n), ties to the lower index,
// and calls emit(rank, index, score) for each kept entry, rank ascending with
// index.  All NT threads of the block must call it; it synchronises inside and
// ends with a barrier.  sc->hist is free for the caller once it returns.
//
// NORMALIZE: take keys relative to the smallest one (see below).  Worth its extra
// pass when the scores are a pre-filtered, narrow set (the merge of chunk lists);
// for the raw scores of a chunk the plain float key space resolves well enough.
//
// r2 / bound (optional, only without NORMALIZE): a value that at least r2 of the keys reach,
// namely the lower edge of the first-level bin that holds the r2-th largest key; -inf when
// no histogram is built (k == n).  Found by the scan that finds the k-th key's bin.
template <int NT, bool NORMALIZE, typename Key, typename Emit>
__device__ __forceinline__ void block_topn(Key keys, int n, int k, TopNScratch<NT>* sc,
                                           Emit emit, int r2 = 0, float* bound = nullptr) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NW = NT / 64, U = 8;
  if (bound) *bound = -INFINITY;
  if (k > n) k = n;      // never more than there is (callers pass k <= n; this keeps a
  if (k <= 0) {          // miscounted caller from reading the scratch of an empty selection)
    __syncthreads();
    return;
  }
  uint32_t T = 0;        // threshold in normalised key space; with k == n every entry is kept
  int T_idx = 0x7fffffff;
  int take_eq = -1;      // >= 0 only on the fallback path: entries == T kept in index order

  // Keys are taken relative to the smallest one and shifted up so that the largest
  // uses the top bit: the 2048 first-level bins then span exactly the range of the
  // scores at hand instead of the whole float line (a few entries per bin near the
  // threshold instead of hundreds).  The map is strictly increasing, so order and
  // equality of keys are unchanged.
  uint32_t kmin = 0;
  int lz = 0;
  if (NORMALIZE && k < n) {
    float lo = INFINITY, hi = -INFINITY;
    for (int i0 = tid; i0 < n; i0 += NT * U) {
      float v[U];
      load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (i0 + u * NT < n) {
          lo = fminf(lo, v[u]);
          hi = fmaxf(hi, v[u]);
        }
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    __syncthreads();
    if (lane == 0) {
      sc->red_m[wave] = lo;
      sc->red_l[wave] = hi;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      lo = fminf(lo, sc->red_m[w]);
      hi = fmaxf(hi, sc->red_l[w]);
    }
    kmin = score_key(lo);
    const uint32_t range = score_key(hi) - kmin;
    lz = range ? __builtin_clz(range) : 31;
  }
  auto nkey = [&](float v) { return (score_key(v) - kmin) << lz; };

  if (k < n) {
    // Entries whose key, shifted right by `shift`, equals `prefix` are copied to
    // the LDS list and ranked against each other directly (tie-break included);
    // the entry of rank r - 1 is the threshold.  Needs list_cnt == 0 on entry.
    auto resolve_in_list = [&](int shift, uint32_t prefix, int count, int r) {
      // pad to a multiple of 16 with entries that rank below everything, and clear
      // the rank accumulators
      const int padded = (count + 15) & ~15;
      for (int e = tid; e < padded; e += NT) {
        if (e >= count) {
          sc->list_key[e] = 0u;
          sc->list_idx[e] = 0x7fffffff;
        }
        sc->list_rank[e] = 0;
      }
      // append matching entries; one LDS atomic per wave and step, not per entry
      const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
      for (int i0 = tid; i0 - lane < n; i0 += NT * U) {  // whole waves stay in the loop
        float v[U];
        load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int i = i0 + u * NT;
          const uint32_t key = nkey(v[u]);
          const bool hit = i < n && (key >> shift) == prefix;
          const uint64_t hits = __ballot(hit);
          if (hits) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sc->list_cnt, __popcll(hits));
            base = __builtin_amdgcn_readfirstlane(base);
            if (hit) {
              const int p = base + __popcll(hits & lt_mask);
              sc->list_key[p] = key;
              sc->list_idx[p] = i;
            }
          }
        }
      }
      __syncthreads();
      // all-pairs ranking, spread over the whole block: thread t takes entry
      // t % padded and every (NT / padded)-th group of four of the others
      const uint4* lk = reinterpret_cast<const uint4*>(sc->list_key);
      const int4* li = reinterpret_cast<const int4*>(sc->list_idx);
      const int groups = padded >> 2;
      const int parts = NT / padded;           // >= 1 because padded <= kTopNListCap <= NT
      const int e = tid % padded, part = tid / padded;
      if (part < parts) {
        const uint32_t ke = sc->list_key[e];
        const int ie = sc->list_idx[e];
        int rank = 0;
        for (int j0 = part; j0 < groups; j0 += parts * 4) {
          uint4 kj[4];
          int4 ij[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {  // loads first: their latencies overlap
            const int j = j0 + q * parts;
            kj[q] = (j < groups) ? lk[j] : make_uint4(0, 0, 0, 0);
            ij[q] = (j < groups) ? li[j] : make_int4(0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            rank += (kj[q].x > ke) || (kj[q].x == ke && ij[q].x < ie);
            rank += (kj[q].y > ke) || (kj[q].y == ke && ij[q].y < ie);
            rank += (kj[q].z > ke) || (kj[q].z == ke && ij[q].z < ie);
            rank += (kj[q].w > ke) || (kj[q].w == ke && ij[q].w < ie);
          }
        }
        if (rank) atomicAdd(&sc->list_rank[e], rank);
      }
      __syncthreads();
      if (tid < count && sc->list_rank[tid] == r - 1) {
        sc->thr_key = sc->list_key[tid];
        sc->thr_idx = sc->list_idx[tid];
      }
      __syncthreads();
      T = sc->thr_key;
      T_idx = sc->thr_idx;
    };

    // level 1: key bits 31..21
    for (int i = tid; i < 2048; i += NT) sc->hist[i] = 0;
    if (tid == 0) sc->list_cnt = 0;
    __syncthreads();
    for (int i0 = tid; i0 < n; i0 += NT * U) {
      float v[U];
      load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (i0 + u * NT < n) atomicAdd(&sc->hist[nkey(v[u]) >> 21], 1u);
    }
    __syncthreads();
    const bool want_bound = !NORMALIZE && r2 > 0;
    find_bin<NT, 2048>(sc, k, want_bound ? (r2 < k ? r2 : k) : 0);
    const uint32_t d1 = (uint32_t)sc->bin;
    const int k1 = sc->rank;
    const int c1 = (int)sc->hist[d1];
    if (want_bound) {
      const uint32_t edge = (uint32_t)sc->bin2 << 21;  // smallest key of that bin
      *bound = __uint_as_float((edge & 0x80000000u) ? (edge & 0x7fffffffu) : ~edge);
    }
    if (c1 <= kTopNListCap) {
      resolve_in_list(21, d1, c1, k1);
    } else {
      __syncthreads();  // everyone has read hist[d1]
      // level 2: bits 20..10 among the keys of bin d1
      for (int i = tid; i < 2048; i += NT) sc->hist[i] = 0;
      __syncthreads();
      for (int i0 = tid; i0 < n; i0 += NT * U) {
        float v[U];
        load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t key = nkey(v[u]);
          if (i0 + u * NT < n && (key >> 21) == d1)
            atomicAdd(&sc->hist[(key >> 10) & 2047u], 1u);
        }
      }
      __syncthreads();
      find_bin<NT, 2048>(sc, k1);
      const uint32_t d2 = (d1 << 11) | (uint32_t)sc->bin;
      const int k2 = sc->rank;
      const int c2 = (int)sc->hist[sc->bin];
      if (c2 <= kTopNListCap) {
        resolve_in_list(10, d2, c2, k2);
      } else {
        __syncthreads();
        // level 3: bits 9..0 among the keys with the 22-bit prefix d2; what is left
        // after it are entries with exactly equal keys, kept in index order
        for (int i = tid; i < 1024; i += NT) sc->hist[i] = 0;
        __syncthreads();
        for (int i0 = tid; i0 < n; i0 += NT * U) {
          float v[U];
          load_keys<U>(keys, i0, NT, n, v);
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const uint32_t key = nkey(v[u]);
            if (i0 + u * NT < n && (key >> 10) == d2) atomicAdd(&sc->hist[key & 1023u], 1u);
          }
        }
        __syncthreads();
        find_bin<NT, 1024>(sc, k2);
        T = (d2 << 10) | (uint32_t)sc->bin;
        take_eq = sc->rank;
      }
    }
  }

  // ordered compaction: each wave owns a contiguous range of indices
  const int seg = (((n + NW - 1) / NW) + 63) & ~63;
  const int i_begin = wave * seg;
  const int i_end = (i_begin + seg < n) ? i_begin + seg : n;
  int ca = 0, cb = 0;  // ca: kept for sure; cb: entries == T (used on the fallback path)
  for (int i0 = i_begin + lane; i0 < i_end; i0 += 64 * U) {
    float v[U];
    load_keys<U>(keys, i0, 64, i_end, v);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * 64;
      const uint32_t key = nkey(v[u]);
      const bool in = i < i_end, gt = key > T, eq = key == T;
      ca += (in && (gt || (take_eq < 0 && eq && i <= T_idx))) ? 1 : 0;
      cb += (in && eq) ? 1 : 0;
    }
  }
  ca = wave_sum(ca);
  cb = wave_sum(cb);
  __syncthreads();
  if (lane == 0) {
    sc->seg_a[wave] = ca;
    sc->seg_b[wave] = cb;
  }
  __syncthreads();
  int a_before = 0, eq_before = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    a_before += (w < wave) ? sc->seg_a[w] : 0;
    eq_before += (w < wave) ? sc->seg_b[w] : 0;
  }
  int out_pos = a_before;
  if (take_eq >= 0) out_pos += eq_before < take_eq ? eq_before : take_eq;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  constexpr int EU = 4;
  for (int i00 = i_begin; i00 < i_end; i00 += 64 * EU) {
    float vv[EU];
#pragma unroll
    for (int u = 0; u < EU; ++u) {
      const int i = i00 + u * 64 + lane;
      vv[u] = (i < i_end) ? keys(i) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < EU; ++u) {
      const int i = i00 + u * 64 + lane;  // whole 64-groups beyond i_end select nothing
      const float v = vv[u];
      bool gt = false, eq = false;
      if (i < i_end) {
        const uint32_t key = nkey(v);
        gt = key > T;
        eq = key == T;
      }
      bool sel;
      if (take_eq < 0) {
        sel = gt || (eq && i <= T_idx);
      } else {
        const uint64_t eq_b = __ballot(eq);
        sel = gt || (eq && (eq_before + (int)__popcll(eq_b & lt_mask)) < take_eq);
        eq_before += (int)__popcll(eq_b);
      }
      const uint64_t sel_b = __ballot(sel);
      if (sel) emit(out_pos + __popcll(sel_b & lt_mask), i, v);
      out_pos += __popcll(sel_b);
    }
  }
  __syncthreads();
}

// ---- one wavefront selects on its own
//
// Exact top-k of keys(0..n-1) by ONE wavefront, ties to the lower index; emit(rank, index,
// score) as block_topn.  No workgroup barrier anywhere, so the wavefronts of a workgroup can
// each run it on different data at the same time: a workgroup that has scored G query heads
// against a chunk of K rows selects for all of them at once instead of head after head (the
// block-wide routine is bound by its barriers, not by its work).  A wavefront issues one
// vector instruction every four cycles, so what counts here is instructions per score: four
// passes over the scores, each a handful of instructions per score.
//
// hist: 512 words of LDS owned by the calling wavefront; free for the caller from the first
// emit on.
//
// Usual path (all scores finite): the scores are counted into 512 bins that divide
// [lo, hi] evenly.  bin(v) = int((v - lo) * 511 / (hi - lo)) never decreases with v
// (subtraction, multiplication by a positive factor and truncation are monotone in floating
// point), so the k-th largest score lies in the bin D where the count from the top reaches
// k, everything in a higher bin is kept and everything in a lower bin is not.  The few scores
// of bin D (at most 128, else the fallback) are ranked exactly among themselves by (key
// descending, index ascending); the one whose rank completes k is the threshold, and a final
// ordered pass keeps key > threshold key, or equal key and index <= threshold index.
//
// Fallback (NaN or infinity among the scores, all scores equal, or more than 128 in bin D):
// radix select on the order-preserving integer keys, 9 bits per pass (bits 31..23, 22..14,
// 13..5, then the last five): a pass counts the keys that match the prefix found so far,
// finds the bin of the k-th largest from the top and descends into it; it stops early when
// every key of that bin is kept; after the last pass the keys equal to the threshold are
// kept in index order.

// body(score, index, valid) for every index below n rounded up to a multiple of 64, U reads
// of the wavefront in flight; valid (index < n) is a constant true outside the last batch.
template <int U, typename Key, typename Body>
__device__ __forceinline__ void wave_for_each(Key keys, int n, int lane, Body body) {
  const int n_whole = n - n % (64 * U);
  int base = 0;
  for (; base < n_whole; base += 64 * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = keys(base + u * 64 + lane);
#pragma unroll
    for (int u = 0; u < U; ++u) body(v[u], base + u * 64 + lane, true);
  }
  if (base < n) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = base + u * 64 + lane;
      v[u] = i < n ? keys(i) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = base + u * 64 + lane;
      if (base + u * 64 < n) body(v[u], i, i < n);   // the same branch in every lane
    }
  }
}

// Count from the top over the 512 bins of hist: the bin where the running count reaches
// `need`, the count above it, and its own count; the same in every lane.
__device__ __forceinline__ void wave_find_bin(const uint32_t* hist, int need, int lane, int& bin,
                                              int& above, int& cnt) {
  // lane L owns the 8 bins 511 - 8 L ... 504 - 8 L (top down)
  const uint4* h4 = reinterpret_cast<const uint4*>(hist);
  const uint4 lo = h4[2 * (63 - lane)], hi = h4[2 * (63 - lane) + 1];
  const int c[8] = {(int)hi.w, (int)hi.z, (int)hi.y, (int)hi.x,
                    (int)lo.w, (int)lo.z, (int)lo.y, (int)lo.x};
  int mine = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) mine += c[j];
  const int incl = wave_incl_scan(mine, lane);
  const int above_lane = incl - mine;
  const bool has = above_lane < need && need <= incl;  // exactly one lane
  int b = 0, ab = 0, cn = 0;
  if (has) {
    int run = above_lane;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (run < need && need <= run + c[j]) {
        b = 511 - 8 * lane - j;
        ab = run;
        cn = c[j];
      }
      run += c[j];
    }
  }
  const int src = __builtin_ffsll((long long)__ballot(has)) - 1;
  bin = __builtin_amdgcn_readlane(b, src);
  above = __builtin_amdgcn_readlane(ab, src);
  cnt = __builtin_amdgcn_readlane(cn, src);
}

__device__ __forceinline__ void wave_zero_hist(uint32_t* hist, int lane) {
  uint4* h4 = reinterpret_cast<uint4*>(hist);
  h4[lane] = make_uint4(0, 0, 0, 0);
  h4[lane + 64] = make_uint4(0, 0, 0, 0);
}

// lo, hi: smallest and largest score; finite: no NaN or infinity among them (wave_minmax).
// SUMEXP: also returns the sum of exp(score - hi) over all scores in *sum_exp (added up in
// the final pass, which visits every score once in any case).
// r2 / bound (optional): *bound receives a value that at least r2 of the scores reach (one
// bin width below the lower edge of the bin that holds the r2-th largest: a score in that bin
// or above has (v - lo) * scale >= its bin number up to two roundings, far less than the one
// bin of slack), -inf when no histogram over [lo, hi] is built.
template <bool SUMEXP, typename Key, typename Emit>
__device__ __forceinline__ void wave_topn(Key keys, int n, int k, float lo, float hi, bool finite,
                                          uint32_t* hist, Emit emit, float* sum_exp = nullptr,
                                          int r2 = 0, float* bound = nullptr) {
  constexpr int U = 8, kList = 128;
  const int lane = threadIdx.x & 63;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  if (k > n) k = n;
  // kept: key > T, or key == T and (index <= T_idx, or among the first take_eq such keys when
  // take_eq >= 0)
  uint32_t T = 0;
  int T_idx = 0x7fffffff, take_eq = -1;   // as initialised: everything is kept
  bool done = k >= n;
  float bound_v = -INFINITY;
  if (!done && finite && hi > lo) {
    const float scale = 511.f / (hi - lo);   // 0 if the difference overflows: one bin, fallback
    auto bin_of = [&](float v) {
      const int b = (int)((v - lo) * scale);
      return b > 511 ? 511 : b;
    };
    wave_zero_hist(hist, lane);
    __builtin_amdgcn_wave_barrier();
    wave_for_each<U>(keys, n, lane, [&](float v, int, bool valid) {
      if (valid) atomicAdd(&hist[bin_of(v)], 1u);
    });
    __builtin_amdgcn_wave_barrier();
    int D, above, cnt;
    wave_find_bin(hist, k, lane, D, above, cnt);
    if (r2 > 0) {
      int D2, above2, cnt2;
      wave_find_bin(hist, r2 < n ? r2 : n, lane, D2, above2, cnt2);
      bound_v = D2 > 0 ? lo + (float)(D2 - 1) / scale : -INFINITY;
    }
    const int need = k - above;   // 1 <= need <= cnt: how many of bin D are kept
    if (cnt <= kList) {
      // the scores of bin D, in any order: key and index; hist[0] counts them
      uint32_t* l_key = hist + 1;
      int* l_idx = reinterpret_cast<int*>(hist) + 1 + kList;
      __builtin_amdgcn_wave_barrier();
      if (lane == 0) hist[0] = 0;
      __builtin_amdgcn_wave_barrier();
      wave_for_each<U>(keys, n, lane, [&](float v, int i, bool valid) {
        if (valid && bin_of(v) == D) {
          const uint32_t at = atomicAdd(&hist[0], 1u);
          if (at < (uint32_t)kList) {   // always: cnt of them exist
            l_key[at] = score_key(v);
            l_idx[at] = i;
          }
        }
      });
      __builtin_amdgcn_wave_barrier();
      // rank within the list; the entry of rank need - 1 is the threshold
      uint32_t my_key[2];
      int my_idx[2], rank[2] = {0, 0};
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int at = lane + 64 * e;
        my_key[e] = at < cnt ? l_key[at] : 0u;
        my_idx[e] = at < cnt ? l_idx[at] : 0;
      }
      for (int f = 0; f < cnt; ++f) {
        const uint32_t fk = l_key[f];
        const int fi = l_idx[f];
#pragma unroll
        for (int e = 0; e < 2; ++e)
          rank[e] += (fk > my_key[e] || (fk == my_key[e] && fi < my_idx[e])) ? 1 : 0;
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        if (lane + 64 * e < cnt && rank[e] == need - 1) {
          hist[300] = my_key[e];
          hist[301] = (uint32_t)my_idx[e];
        }
      }
      __builtin_amdgcn_wave_barrier();
      T = hist[300];
      T_idx = (int)hist[301];
      done = true;
    }
  }
  if (!done) {
    uint32_t prefix = 0;  // the bits of the threshold found so far
    int need = k;         // rank of the threshold among the keys that match the prefix
    int shift = 23;
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
      const int bits = pass < 3 ? 9 : 5;
      const uint32_t mask = (1u << bits) - 1u;
      __builtin_amdgcn_wave_barrier();
      wave_zero_hist(hist, lane);
      __builtin_amdgcn_wave_barrier();
      wave_for_each<U>(keys, n, lane, [&](float v, int, bool valid) {
        const uint32_t key = score_key(v);
        const bool match = pass == 0 || (key >> (shift + bits)) == prefix;
        if (valid && match) atomicAdd(&hist[(key >> shift) & mask], 1u);
      });
      __builtin_amdgcn_wave_barrier();
      int bin, above, cnt;
      wave_find_bin(hist, need, lane, bin, above, cnt);
      prefix = (prefix << bits) | ((uint32_t)bin & mask);
      need -= above;
      if (cnt == need || pass == 3) {
        T = shift ? prefix << shift : prefix;   // smallest key with this prefix
        if (cnt == need) {                      // every key >= T is kept
          T_idx = 0x7fffffff;
          take_eq = -1;
        } else {                                // last pass: keys == T, the first `need`
          T_idx = -1;
          take_eq = need;
        }
        break;
      }
      shift = pass < 2 ? shift - 9 : 0;
    }
  }
  __builtin_amdgcn_wave_barrier();
  // ordered compaction: index order is lane order within a step, steps in order
  int out_pos = 0, eq_seen = 0;
  float l = 0.f;
  wave_for_each<U>(keys, n, lane, [&](float v, int i, bool valid) {
    if (SUMEXP && valid) l += __expf(v - hi);
    const uint32_t key = score_key(v);
    bool sel = valid && (key > T || (key == T && i <= T_idx));
    if (take_eq >= 0) {
      const bool eq = valid && key == T;
      const uint64_t eq_b = __ballot(eq);
      if (eq) sel = eq_seen + (int)__popcll(eq_b & lt_mask) < take_eq;
      eq_seen += (int)__popcll(eq_b);
    }
    const uint64_t sel_b = __ballot(sel);
    if (sel) emit(out_pos + __popcll(sel_b & lt_mask), i, v);
    out_pos += __popcll(sel_b);
  });
  if (SUMEXP) *sum_exp = wave_sum(l);
  if (bound) *bound = bound_v;
}

// Smallest and largest of keys(0..n-1) and whether all of them are finite, to every lane.
template <typename Key>
__device__ __forceinline__ void wave_minmax(Key keys, int n, float& lo, float& hi, bool& finite) {
  const int lane = threadIdx.x & 63;
  float a = INFINITY, b = -INFINITY, big = 0.f;
  wave_for_each<8>(keys, n, lane, [&](float v, int, bool valid) {
    if (valid) {
      a = fminf(a, v);
      b = fmaxf(b, v);
      big = fmaxf(big, fabsf(v) < INFINITY ? 0.f : 1.f);   // 1 for NaN as well
    }
  });
  lo = wave_min(a);
  hi = wave_max(b);
  finite = __ballot(big != 0.f) == 0ull;
}

}  // namespace kc
