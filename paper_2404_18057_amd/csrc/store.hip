// Cache store: rows of a token-major tensor [B][T][Hkv][d] are written to the
// head-major cache [B][Hkv][S_cap][d] at positions pos[b] + t (paper Figure 1
// upper half: every layer pushes its K and V states; the V states end up in CPU
// memory.  Section 3.2: 2bsd bytes per block go device to host).
//
// The same kernel serves both halves: for K the destination is HBM, for V it is
// the mapped host cache, so V rows leave the GPU as posted PCIe writes without
// a staging copy.
//
// The V half is link bound (about 57 GB/s).  Its rows leave as posted PCIe writes, and
// posted writes beyond what the link drains back up into the write path they share with
// HBM traffic, so the number of workgroups that write to the host decides how much the
// store disturbs whatever runs beside it.  Measured on MI355X at config 5's layer (1.34 GB
// of V; conventional attention of another layer, 424 us alone, as the concurrent HBM-bound
// work; K store of the same call, 2.4 TB/s of rows alone):
//
//   workgroups | V alone  | K store beside it | V beside attention | attention beside it
//        4     | 45 GB/s  |    2.4 TB/s       |      27 GB/s       |     x 1.07
//        8     | 48 GB/s  |    2.3-2.4 TB/s   |      31 GB/s       |     x 1.21
//       20     | 54 GB/s  |    0.9-1.0 TB/s   |      37 GB/s       |     x 1.38
//       64     | 56 GB/s  |    0.2 TB/s       |      51 GB/s       |     x 1.42
//
// A layer's device-to-host copy has the whole next layer to hide under (paper section 3.2,
// equations (1)-(2)), so what counts is that it does not slow that layer down: the host
// destination gets a small fixed grid of 8 workgroups (128 KiB of writes in flight) that
// strides over the tiles; KC_OPT_HOST_STORE_BLOCKS changes it.
//
// The K half is a device-to-device relayout.  Measured on MI355X at config 5's layer
// (1.34 GB of rows) it moves 2.2-2.4 TB/s of rows, i.e. 4.4-4.7 TB/s of combined read and
// write traffic; a plain device copy of the same bytes (hipMemcpy device to device) reaches
// 2.6 TB/s of rows (5.2 TB/s combined, 65 % of the HBM peak: mixed read / write traffic
// pays for bus turnarounds), so the relayout runs at 86-89 % of what a copy can do here.
// Larger tiles (8 or 16 tokens, 4 or 16 heads per workgroup, up to 64 KiB in flight per
// workgroup) and non-temporal loads / stores were measured and gave nothing consistent
// (-30 % to +6 % depending on the shape), so the tile stays at 4 tokens x 16 heads.
#include "kc_internal.h"

namespace kc {
namespace {

constexpr int kHostStoreBlocks = 8;   // workgroups of a store whose destination is host memory
constexpr int kTokTile = 4;    // tokens per workgroup

// A row of D 16-bit values is LPR = D / 8 lanes x 16 bytes, so the 256 threads form
// 256 / LPR row groups.  A workgroup moves a tile of 4 tokens x HEADS KV heads in four
// passes; in each pass the row groups cover 4 tokens x (row groups / 4) heads.  For
// D = 128: 16 row groups, 4 tokens x 4 heads per pass - the 4 heads of a token are 1 KiB
// of contiguous source, the 4 tokens of a head are 1 KiB of contiguous destination.
//
// src2 / dst2, when not null, are a second tensor pair moved with the same
// indices (the K and V rows of a decode-step append in one launch).
//
// K8: the first pair is quantised on the way, 16-bit values in, OCP FP8 E4M3 codes of
// value * 2^-k_exp out (nearest, ties to even, saturating at 448; the power-of-two scale
// keeps every step exact).  A destination row is then 16 lanes x 8 bytes.

// E4M3 code of x: 1 sign, 4 exponent bits (bias 7), 3 fraction bits, no infinities.
__device__ __forceinline__ uint32_t quant_e4m3(float x) {
  const uint32_t u = __float_as_uint(x), sign = (u >> 24) & 0x80u, a = u & 0x7fffffffu;
  uint32_t code;
  if (a > 0x7f800000u) {
    code = 0x7fu;  // NaN
  } else if (a >= 0x43e00000u) {
    code = 0x7eu;  // |x| >= 448: the largest finite value
  } else if (a < 0x3c800000u) {
    // below 2^-6 the codes are 2^-9 apart (subnormals; 8 is the smallest normal's code)
    code = (uint32_t)__float2int_rn(__uint_as_float(a) * 512.f);
  } else {
    // round the 23 fraction bits to 3, ties to even; a carry moves into the exponent
    const uint32_t r = (a + 0x7ffffu + ((a >> 20) & 1u)) >> 20;
    code = r - (120u << 3);  // exponent bias 127 -> 7
  }
  return sign | code;
}

template <int DT>
__device__ __forceinline__ uint2 quant_row8(const uint4& v, int k_exp) {
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  uint32_t c[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float lo, hi;
    if constexpr (DT == 0) {
      const half2_t h = __builtin_bit_cast(half2_t, w[i]);
      lo = (float)h.x;
      hi = (float)h.y;
    } else {
      lo = __uint_as_float(w[i] << 16);
      hi = __uint_as_float(w[i] & 0xffff0000u);
    }
    c[2 * i] = quant_e4m3(ldexpf(lo, -k_exp));
    c[2 * i + 1] = quant_e4m3(ldexpf(hi, -k_exp));
  }
  return make_uint2(c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24),
                    c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24));
}

// K8: 0 = plain copy, 1 = quantise fp16 rows, 2 = quantise bf16 rows (LPR 16 only)
template <int K8, int LPR>
__global__ __launch_bounds__(256) void store_kernel(const uint4* __restrict__ src,
                                                    uint4* __restrict__ dst,
                                                    const uint4* __restrict__ src2,
                                                    uint4* __restrict__ dst2,
                                                    const int32_t* __restrict__ pos, int B, int T,
                                                    int Hkv, int S_cap, int t_tiles, int h_tiles,
                                                    unsigned total_tiles,
                                                    int* __restrict__ flags, int k_exp) {
  constexpr int HPP = 256 / LPR / kTokTile;  // heads per pass
  constexpr int kHeadTile = 4 * HPP;         // heads per workgroup
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const int ti = grp / HPP, hi = grp % HPP;
  for (unsigned tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
    const unsigned ht = tile % (unsigned)h_tiles;
    const unsigned rest = tile / (unsigned)h_tiles;
    const int tt = (int)(rest % (unsigned)t_tiles), b = (int)(rest / (unsigned)t_tiles);
    const int t = tt * kTokTile + ti;
    const long long p = (long long)pos[b] + t;
    const bool t_ok = t < T;
    const bool p_ok = p >= 0 && p < S_cap;
    if (t_ok && !p_ok && sub == 0 && hi == 0 && ht == 0) atomicOr(flags, kFlagBadPos);
    // all loads of the tile first, then all stores; everything stays in registers
    uint4 v0, v1, v2, v3, w0, w1, w2, w3;
    v0 = v1 = v2 = v3 = w0 = w1 = w2 = w3 = make_uint4(0, 0, 0, 0);
    const int hk0 = (int)ht * kHeadTile + hi;
    const bool row_ok = t_ok && p_ok;
    const bool ok0 = row_ok && hk0 < Hkv, ok1 = row_ok && hk0 + HPP < Hkv,
               ok2 = row_ok && hk0 + 2 * HPP < Hkv, ok3 = row_ok && hk0 + 3 * HPP < Hkv;
    const size_t from = (((size_t)b * T + t) * Hkv + hk0) * LPR + sub;
    const size_t fstep = (size_t)HPP * LPR;
    if (ok0) v0 = src[from];
    if (ok1) v1 = src[from + fstep];
    if (ok2) v2 = src[from + 2 * fstep];
    if (ok3) v3 = src[from + 3 * fstep];
    if (src2) {
      if (ok0) w0 = src2[from];
      if (ok1) w1 = src2[from + fstep];
      if (ok2) w2 = src2[from + 2 * fstep];
      if (ok3) w3 = src2[from + 3 * fstep];
    }
    const size_t to = (((size_t)b * Hkv + hk0) * S_cap + (size_t)(row_ok ? p : 0)) * LPR + sub;
    const size_t tstep = (size_t)HPP * S_cap * LPR;
    auto put = [&](bool ok, size_t at, const uint4& x) {
      if (!ok) return;
      if constexpr (K8 != 0)
        reinterpret_cast<uint2*>(dst)[at] = quant_row8<K8 - 1>(x, k_exp);
      else
        dst[at] = x;
    };
    put(ok0, to, v0);
    put(ok1, to + tstep, v1);
    put(ok2, to + 2 * tstep, v2);
    put(ok3, to + 3 * tstep, v3);
    if (src2) {
      if (ok0) dst2[to] = w0;
      if (ok1) dst2[to + tstep] = w1;
      if (ok2) dst2[to + 2 * tstep] = w2;
      if (ok3) dst2[to + 3 * tstep] = w3;
    }
  }
}

}  // namespace

hipError_t launch_store(const Shape& sh, const void* src, void* dst, const void* src2, void* dst2,
                        const int32_t* pos, int T, int* flags, int dst_is_host, hipStream_t st,
                        int k_fp8, int k_exp) {
  if (sh.B <= 0 || T <= 0 || sh.Hkv <= 0) return hipSuccess;
  if (sh.d != 64 && sh.d != 128 && sh.d != 256) return hipErrorInvalidValue;
  if (k_fp8 && sh.d != 128) return hipErrorInvalidValue;
  const int lpr = sh.d / 8;
  const long long head_tile = 4 * (256 / lpr / kTokTile);
  const long long t_tiles = (T + kTokTile - 1) / kTokTile;
  const long long h_tiles = (sh.Hkv + head_tile - 1) / head_tile;
  const long long tiles = (long long)sh.B * t_tiles * h_tiles;
  if (tiles > 0xffffffffLL) return hipErrorInvalidValue;
  long long blocks = tiles;
  const long long cap = dst_is_host ? (dst_is_host > 1 ? dst_is_host : kHostStoreBlocks) : 0x7fffffffLL;
  if (blocks > cap) blocks = cap;
#define KC_STORE(K8, LPR)                                                                       \
  hipLaunchKernelGGL((store_kernel<K8, LPR>), dim3((unsigned)blocks), dim3(256), 0, st,         \
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst),                  \
                     static_cast<const uint4*>(src2), static_cast<uint4*>(dst2), pos, sh.B, T,  \
                     sh.Hkv, sh.S_cap, (int)t_tiles, (int)h_tiles, (unsigned)tiles, flags, k_exp)
  if (k_fp8 && sh.dtype == 0)
    KC_STORE(1, 16);
  else if (k_fp8)
    KC_STORE(2, 16);
  else if (lpr == 8)
    KC_STORE(0, 8);
  else if (lpr == 16)
    KC_STORE(0, 16);
  else
    KC_STORE(0, 32);
#undef KC_STORE
  return hipGetLastError();
}

}  // namespace kc
