// V row pull and weighted sum: out = sum_j w[j] * V[idx[j]]
// (paper Figure 1 "VCache Pull"; Table 1 row A~ = S~ Part(V): 2bNd FLOPs, 2bNd
// bytes of V; section 3.2 equation (3): these bytes cross the host link).
//
// One workgroup per (sequence, query head).  A V row is 256 bytes = 16 lanes x
// 16 bytes, so a wave pulls 4 rows per load instruction and the workgroup's 16
// row slots each issue 8 independent loads before the first use: the link sees
// up to 128 outstanding 256-byte reads per workgroup, and every other resident
// workgroup adds its own.  The rows are read straight out of mapped, pinned
// host memory; nothing is staged in HBM.
#include "attn_common.h"

namespace kc {
namespace {

template <int DT>
__global__ __launch_bounds__(256) void gather_kernel(const uint16_t* __restrict__ V,
                                                     const int32_t* __restrict__ idx,
                                                     const float* __restrict__ wgt,
                                                     float* __restrict__ out, int H, int Hkv,
                                                     int S_cap, int N, int u0, int packed) {
  __shared__ float part[4][kHeadDim];
  const int unit = u0 + blockIdx.x;
  const int b = unit / H, h = unit - b * H;
  const int hk = h / (H / Hkv);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane & 15, rg = lane >> 4;
  const int slot = wave * 4 + rg;  // 16 row slots per workgroup

  const size_t base_row = packed ? (size_t)unit * N : ((size_t)b * Hkv + hk) * S_cap;
  const uint4* __restrict__ Vp = reinterpret_cast<const uint4*>(V) + base_row * 16 + sub;
  const int32_t* __restrict__ iu = idx + (size_t)unit * N;
  const float* __restrict__ wu = wgt + (size_t)unit * N;

  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;

  constexpr int UNR = 8;
  for (int j0 = slot; j0 < N; j0 += 16 * UNR) {
    int t[UNR];
    float w[UNR];
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + u * 16;
      t[u] = (j < N) ? iu[j] : -1;  // -1 marks the padding beyond N_eff
      w[u] = (j < N) ? wu[j] : 0.f;
      if (t[u] >= S_cap) t[u] = -1;  // a position outside the cache is never read
      if (packed && t[u] >= 0) t[u] = j;
    }
    if (t[0] < 0) break;  // positions are ascending with the padding at the end
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      v[u] = make_uint4(0, 0, 0, 0);
      if (t[u] >= 0) v[u] = Vp[(size_t)t[u] * 16];
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      if (t[u] >= 0) fma8<DT>(acc, v[u], w[u]);
  }

  // add the 4 row groups of the wave, then the 4 waves
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    acc[i] += __shfl_xor(acc[i], 16, 64);
    acc[i] += __shfl_xor(acc[i], 32, 64);
  }
  if (rg == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) part[wave][sub * 8 + i] = acc[i];
  }
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    const int c = threadIdx.x;
    out[(size_t)unit * kHeadDim + c] = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
  }
}

}  // namespace

hipError_t launch_gather(const Shape& sh, const void* v, const int32_t* idx, const float* w,
                         float* out, int u0, int count, int packed, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  const uint16_t* vp = static_cast<const uint16_t*>(v);
  if (sh.dtype == 0)
    hipLaunchKernelGGL((gather_kernel<0>), dim3((unsigned)count), dim3(256), 0, st, vp, idx, w,
                       out, sh.H, sh.Hkv, sh.S_cap, sh.N, u0, packed);
  else
    hipLaunchKernelGGL((gather_kernel<1>), dim3((unsigned)count), dim3(256), 0, st, vp, idx, w,
                       out, sh.H, sh.Hkv, sh.S_cap, sh.N, u0, packed);
  return hipGetLastError();
}

}  // namespace kc
