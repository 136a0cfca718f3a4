// Block-wide exact top-k selection over fp32 scores (paper section 3.1: "TopN
// selects the N most relevant results").
//
// Scores are mapped to unsigned keys whose integer order is the float order.
// The k-th largest key T is found by an 11 + 11 + 10 bit radix select with LDS
// histograms; the kept set is {key > T} plus the first (k - #{key > T})
// entries with key == T in index order, i.e. "largest first, lower index on
// ties".  Entries are emitted in ascending index order through an ordered
// (ballot + prefix) compaction, so nothing depends on the arrival order of an
// atomic.  The routine works on any flat pointer (LDS or global memory).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kc {

template <int NT>
struct TopNScratch {
  uint32_t hist[2048];
  int wave_tot[NT / 64];
  int seg_gt[NT / 64];
  int seg_eq[NT / 64];
  float red[NT / 64];
  int bin, rank;
};

__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;  // -0 and +0 are the same score
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  return v;
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
// sc->rank.  Ends with a barrier.
template <int NT, int NBINS>
__device__ __forceinline__ void find_bin(TopNScratch<NT>* sc, int k) {
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
  if (above < k && k <= above + mine) {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (above < k && k <= above + c[j]) {
        sc->bin = top - j;
        sc->rank = k - above;
      }
      above += c[j];
    }
  }
  __syncthreads();
}

template <int NT>
__device__ __forceinline__ float block_max(float m, TopNScratch<NT>* sc) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sc->red[threadIdx.x >> 6] = m;
  __syncthreads();
  m = sc->red[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) m = fmaxf(m, sc->red[w]);
  return m;
}

template <int NT>
__device__ __forceinline__ float block_sum(float v, TopNScratch<NT>* sc) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sc->red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) t += sc->red[w];
  return t;
}

// Selects the k largest of keys[0..n) (1 <= k <= n), ties to the lower index,
// and calls emit(rank, index, score) for each kept entry, rank ascending with
// index.  All NT threads of the block must call it; it synchronises inside.
template <int NT, typename Emit>
__device__ __forceinline__ void block_topn(const float* keys, int n, int k, TopNScratch<NT>* sc,
                                           Emit emit) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NW = NT / 64;
  uint32_t T = 0;       // threshold key; with k == n everything is kept
  int take_eq = 0;
  if (k < n) {
    // pass 1: key bits 31..21
    for (int i = tid; i < 2048; i += NT) sc->hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) atomicAdd(&sc->hist[score_key(keys[i]) >> 21], 1u);
    __syncthreads();
    find_bin<NT, 2048>(sc, k);
    const uint32_t d1 = (uint32_t)sc->bin;
    const int k1 = sc->rank;
    __syncthreads();
    // pass 2: bits 20..10 among the keys of bin d1
    for (int i = tid; i < 2048; i += NT) sc->hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) {
      const uint32_t key = score_key(keys[i]);
      if ((key >> 21) == d1) atomicAdd(&sc->hist[(key >> 10) & 2047u], 1u);
    }
    __syncthreads();
    find_bin<NT, 2048>(sc, k1);
    const uint32_t d2 = (d1 << 11) | (uint32_t)sc->bin;
    const int k2 = sc->rank;
    __syncthreads();
    // pass 3: bits 9..0 among the keys with the 22-bit prefix d2
    for (int i = tid; i < 1024; i += NT) sc->hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) {
      const uint32_t key = score_key(keys[i]);
      if ((key >> 10) == d2) atomicAdd(&sc->hist[key & 1023u], 1u);
    }
    __syncthreads();
    find_bin<NT, 1024>(sc, k2);
    T = (d2 << 10) | (uint32_t)sc->bin;
    take_eq = sc->rank;
  } else {
    take_eq = n;  // T = 0 is below every key: all entries count as "greater"
  }

  // ordered compaction: each wave owns a contiguous range of indices
  const int seg = (((n + NW - 1) / NW) + 63) & ~63;
  const int i_begin = wave * seg;
  const int i_end = (i_begin + seg < n) ? i_begin + seg : n;
  int cgt = 0, ceq = 0;
  for (int i = i_begin + lane; i < i_end; i += 64) {
    const uint32_t key = score_key(keys[i]);
    cgt += key > T;
    ceq += key == T;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    cgt += __shfl_xor(cgt, o, 64);
    ceq += __shfl_xor(ceq, o, 64);
  }
  __syncthreads();
  if (lane == 0) {
    sc->seg_gt[wave] = cgt;
    sc->seg_eq[wave] = ceq;
  }
  __syncthreads();
  int gt_before = 0, eq_before = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    gt_before += (w < wave) ? sc->seg_gt[w] : 0;
    eq_before += (w < wave) ? sc->seg_eq[w] : 0;
  }
  int out_pos = gt_before + (eq_before < take_eq ? eq_before : take_eq);
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int i0 = i_begin; i0 < i_end; i0 += 64) {
    const int i = i0 + lane;
    float v = 0.f;
    bool gt = false, eq = false;
    if (i < i_end) {
      v = keys[i];
      const uint32_t key = score_key(v);
      gt = key > T;
      eq = key == T;
    }
    const uint64_t eq_b = __ballot(eq);
    const bool sel = gt || (eq && (eq_before + __popcll(eq_b & lt_mask)) < take_eq);
    const uint64_t sel_b = __ballot(sel);
    if (sel) emit(out_pos + __popcll(sel_b & lt_mask), i, v);
    out_pos += __popcll(sel_b);
    eq_before += __popcll(eq_b);
  }
  __syncthreads();
}

}  // namespace kc
