// Softmax statistics and exact top-N selection for one (sequence, query head)
// unit per workgroup, from scores that a separate K-scan launch left in HBM
// (paper section 3.1; Table 1 row S~).  Used by the unfused path (staged gather,
// per-kernel measurements); the fused decode kernel selects on chip.
//
// exp is strictly increasing, so the N largest softmax values sit at the N
// largest scores: the selection runs on the fp32 scores (see topn.h).
#include "kc_internal.h"
#include "topn.h"

namespace kc {
namespace {

constexpr int NT = kSelectThreads;

__global__ __launch_bounds__(NT) void select_kernel(const float* __restrict__ z,
                                                    const int32_t* __restrict__ seq_lens,
                                                    int32_t* __restrict__ idx,
                                                    float* __restrict__ wgt, int H, int S_cap,
                                                    int N, int u0, int renorm) {
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
  float kept = 0.f;  // this thread's share of the kept softmax mass
  block_topn<NT, false>(key, s, n_eff, &sc, [&](int r, int t, float v) {
    const float w = expf(v - m) * inv_Z;
    iu[r] = t;
    wu[r] = w;
    kept += w;
  });
  if (renorm) {
    // variant: the kept weights are divided by their sum.  Entries were written by
    // whichever thread found them, so they are re-read around the L1.
    const float2 tot = block_merge_stats<NT>(0.f, kept, &sc);  // equal maxima: a plain sum
    const float inv = 1.f / tot.y;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int r = tid; r < n_eff; r += NT)
      wu[r] = __hip_atomic_load(&wu[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * inv;
  }
}

}  // namespace

hipError_t launch_select(const Shape& sh, const float* z, const int32_t* seq_lens, int32_t* idx,
                         float* w, int u0, int count, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)count), dim3(NT), 0, st, z, seq_lens, idx, w,
                     sh.H, sh.S_cap, sh.N, u0, sh.renorm);
  return hipGetLastError();
}

}  // namespace kc
