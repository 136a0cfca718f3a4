// Softmax statistics and exact top-N selection for one (sequence, query head)
// unit per workgroup, from scores that a separate K-scan launch left in HBM
// (paper section 3.1: "After the softmax operation, TopN selects the N most
// relevant results"; Table 1 row S~).  Used by the unfused path (staged gather,
// per-kernel measurements); the fused decode kernel selects on chip.
//
// exp is strictly increasing, so the N largest softmax values sit at the N
// largest scores: the selection runs on the fp32 scores (see topn.cuh).
#include "kc_internal.h"
#include "topn.cuh"

namespace kc {
namespace {

constexpr int NT = kSelectThreads;

__global__ __launch_bounds__(NT) void select_kernel(const float* __restrict__ z,
                                                    const int32_t* __restrict__ seq_lens,
                                                    int32_t* __restrict__ idx,
                                                    float* __restrict__ wgt, int H, int S_cap,
                                                    int N, int u0) {
  __shared__ TopNScratch<NT> sc;
  const int unit = u0 + blockIdx.x;
  const int b = unit / H;
  const int tid = threadIdx.x;
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

  auto key = [&](int t) { return zr[t]; };
  const float2 ml = block_softmax_stats<NT>(key, s, &sc);
  const float m = ml.x, inv_Z = 1.f / ml.y;
  block_topn<NT, false>(key, s, n_eff, &sc, [&](int r, int t, float v) {
    iu[r] = t;
    wu[r] = expf(v - m) * inv_Z;
  });
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
