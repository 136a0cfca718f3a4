// Cache store: rows of a token-major tensor [B][T][Hkv][d] are written to the
// head-major cache [B][Hkv][S_cap][d] at positions pos[b] + t (paper Figure 1
// upper half: every layer pushes its K and V states; the V states end up in CPU
// memory.  Section 3.2: 2bsd bytes per block go device to host).
//
// The same kernel serves both halves: for K the destination is HBM, for V it is
// the mapped host cache, so V rows leave the GPU as posted PCIe writes without
// a staging copy.  Consecutive 16-lane groups write consecutive positions of
// one (sequence, KV head), i.e. one contiguous run of destination memory.
#include "kc_internal.h"

namespace kc {
namespace {

constexpr int kRowsPerBlock = 64;

__global__ __launch_bounds__(256) void store_kernel(const uint4* __restrict__ src,
                                                    uint4* __restrict__ dst,
                                                    const int32_t* __restrict__ pos, int B, int T,
                                                    int Hkv, int S_cap, long long total_rows,
                                                    int* __restrict__ flags) {
  const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const long long r0 = (long long)blockIdx.x * kRowsPerBlock + grp;
  uint4 v[4];
  long long d[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const long long r = r0 + i * 16;  // r = (b*Hkv + hk)*T + t
    d[i] = -1;
    if (r < total_rows) {
      const int t = (int)(r % T);
      const long long bh = r / T;
      const int hk = (int)(bh % Hkv), b = (int)(bh / Hkv);
      const long long p = (long long)pos[b] + t;
      if (p < 0 || p >= S_cap) {
        if (sub == 0) atomicOr(flags, kFlagBadPos);
      } else {
        d[i] = (bh * S_cap + p) * 16 + sub;
        v[i] = src[(((long long)b * T + t) * Hkv + hk) * 16 + sub];
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (d[i] >= 0) dst[d[i]] = v[i];
}

}  // namespace

hipError_t launch_store(const Shape& sh, const void* src, void* dst, const int32_t* pos, int T,
                        int* flags, hipStream_t st) {
  const long long rows = (long long)sh.B * T * sh.Hkv;
  if (rows <= 0) return hipSuccess;
  const long long blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(store_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), pos, sh.B, T,
                     sh.Hkv, sh.S_cap, rows, flags);
  return hipGetLastError();
}

}  // namespace kc
