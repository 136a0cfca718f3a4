// Softmax statistics and exact top-N selection for one (sequence, query head)
// unit per workgroup (paper section 3.1: "After the softmax operation, TopN
// selects the N most relevant results"; Table 1 row S~).
//
// exp is strictly increasing, so the N largest softmax values sit at the N
// largest scores: the selection runs on the fp32 scores, mapped to unsigned
// keys whose integer order is the float order.  The N-th largest key is found
// by an 11 + 11 + 10 bit radix select with LDS histograms; the kept set is
// {key > T} plus the first (N_eff - #{key > T}) positions with key == T in
// position order, which is exactly "largest first, lower position on ties".
// Positions are emitted ascending by an ordered (ballot / prefix) compaction, so
// the result does not depend on any atomic's arrival order.
#include "kc_internal.h"

namespace kc {
namespace {

constexpr int NT = kSelectThreads;
constexpr int NW = NT / 64;

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

// Exclusive prefix sum of one int per thread over the block; *total gets the sum.
__device__ __forceinline__ int block_excl_scan(int v, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = wave_incl_scan(v, lane);
  __syncthreads();  // wave_tot may still be read from a previous use
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    int t = wave_tot[w];
    before += (w < wave) ? t : 0;
    all += t;
  }
  *total = all;
  return before + inc - v;
}

// hist has NBINS counters.  Finds the bin D, counting from the top, that holds
// the k-th largest key: above(D) < k <= above(D) + hist[D].  Returns D and the
// rank still to resolve inside it (k - above(D)) through sh_bin / sh_k.
template <int NBINS>
__device__ __forceinline__ void find_bin(const uint32_t* hist, int k, int* wave_tot, int* sh_bin,
                                         int* sh_k) {
  constexpr int PER = NBINS / NT;
  static_assert(NBINS % NT == 0, "bins must divide over the threads");
  const int top = NBINS - 1 - (int)threadIdx.x * PER;  // this thread owns top, top-1, ...
  int c[PER], mine = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    c[j] = (int)hist[top - j];
    mine += c[j];
  }
  int total;
  int above = block_excl_scan(mine, wave_tot, &total);
  if (above < k && k <= above + mine) {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (above < k && k <= above + c[j]) {
        *sh_bin = top - j;
        *sh_k = k - above;
      }
      above += c[j];
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(NT) void select_kernel(const float* __restrict__ z,
                                                    const int32_t* __restrict__ seq_lens,
                                                    int32_t* __restrict__ idx,
                                                    float* __restrict__ wgt, int H, int S_cap,
                                                    int N, int u0) {
  __shared__ uint32_t hist[2048];
  __shared__ int wave_tot[NW];
  __shared__ float red[NW];
  __shared__ int sh_bin, sh_k;
  __shared__ int seg_gt[NW], seg_eq[NW];

  const int unit = u0 + blockIdx.x;
  const int b = unit / H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int s = seq_lens[b];
  s = s < 1 ? 0 : (s > S_cap ? S_cap : s);
  const int n_eff = N < s ? N : s;
  const float* __restrict__ zr = z + (size_t)unit * S_cap;
  int32_t* __restrict__ iu = idx + (size_t)unit * N;
  float* __restrict__ wu = wgt + (size_t)unit * N;

  for (int j = n_eff + tid; j < N; j += NT) {
    iu[j] = -1;
    wu[j] = 0.f;
  }
  if (n_eff == 0) return;

  // ---- pass 1: max score, histogram of key bits 31..21
  for (int i = tid; i < 2048; i += NT) hist[i] = 0;
  __syncthreads();
  float m = -INFINITY;
  for (int t = tid; t < s; t += NT) {
    float v = zr[t];
    m = fmaxf(m, v);
    atomicAdd(&hist[score_key(v) >> 21], 1u);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);
  find_bin<2048>(hist, n_eff, wave_tot, &sh_bin, &sh_k);
  const uint32_t d1 = (uint32_t)sh_bin;
  const int k1 = sh_k;
  __syncthreads();

  // ---- pass 2: sum of exp(z - m), histogram of bits 20..10 among keys in bin d1
  for (int i = tid; i < 2048; i += NT) hist[i] = 0;
  __syncthreads();
  float l = 0.f;
  for (int t = tid; t < s; t += NT) {
    float v = zr[t];
    l += __expf(v - m);
    uint32_t key = score_key(v);
    if ((key >> 21) == d1) atomicAdd(&hist[(key >> 10) & 2047u], 1u);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o, 64);
  __syncthreads();  // everyone has read red[] for the max
  if (lane == 0) red[wave] = l;
  __syncthreads();
  float Zsum = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) Zsum += red[w];
  find_bin<2048>(hist, k1, wave_tot, &sh_bin, &sh_k);
  const uint32_t d2 = (d1 << 11) | (uint32_t)sh_bin;
  const int k2 = sh_k;
  __syncthreads();

  // ---- pass 3: histogram of bits 9..0 among keys with the 22-bit prefix d2
  for (int i = tid; i < 1024; i += NT) hist[i] = 0;
  __syncthreads();
  for (int t = tid; t < s; t += NT) {
    uint32_t key = score_key(zr[t]);
    if ((key >> 10) == d2) atomicAdd(&hist[key & 1023u], 1u);
  }
  __syncthreads();
  find_bin<1024>(hist, k2, wave_tot, &sh_bin, &sh_k);
  const uint32_t T = (d2 << 10) | (uint32_t)sh_bin;  // the N_eff-th largest key
  const int take_eq = sh_k;                          // how many keys == T are kept

  // ---- ordered compaction: each wave owns a contiguous range of positions
  const int seg = (((s + NW - 1) / NW) + 63) & ~63;
  const int t_begin = wave * seg;
  const int t_end = (t_begin + seg < s) ? t_begin + seg : s;
  int cgt = 0, ceq = 0;
  for (int t = t_begin + lane; t < t_end; t += 64) {
    uint32_t key = score_key(zr[t]);
    cgt += key > T;
    ceq += key == T;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    cgt += __shfl_xor(cgt, o, 64);
    ceq += __shfl_xor(ceq, o, 64);
  }
  if (lane == 0) {
    seg_gt[wave] = cgt;
    seg_eq[wave] = ceq;
  }
  __syncthreads();
  int gt_before = 0, eq_before = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    gt_before += (w < wave) ? seg_gt[w] : 0;
    eq_before += (w < wave) ? seg_eq[w] : 0;
  }
  int out_pos = gt_before + (eq_before < take_eq ? eq_before : take_eq);
  const float inv_Z = 1.f / Zsum;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int t0 = t_begin; t0 < t_end; t0 += 64) {
    const int t = t0 + lane;
    float v = 0.f;
    bool gt = false, eq = false;
    if (t < t_end) {
      v = zr[t];
      uint32_t key = score_key(v);
      gt = key > T;
      eq = key == T;
    }
    const uint64_t eq_b = __ballot(eq);
    const bool sel = gt || (eq && (eq_before + __popcll(eq_b & lt_mask)) < take_eq);
    const uint64_t sel_b = __ballot(sel);
    if (sel) {
      const int p = out_pos + __popcll(sel_b & lt_mask);
      iu[p] = t;
      wu[p] = expf(v - m) * inv_Z;
    }
    out_pos += __popcll(sel_b);
    eq_before += __popcll(eq_b);
  }
}

}  // namespace

hipError_t launch_select(const Shape& sh, const float* z, const int32_t* seq_lens, int32_t* idx,
                         float* w, int u0, int count, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)count), dim3(NT), 0, st, z, seq_lens, idx, w,
                     sh.H, sh.S_cap, sh.N, u0);
  return hipGetLastError();
}

}  // namespace kc
