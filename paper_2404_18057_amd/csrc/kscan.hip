// K scan: z[t] = (q . K[t]) / sqrt(d_h) over the whole cached context
// (paper section 3.1; Table 1 row S~: 2bsd FLOPs against 2bnhs bytes of K, an
// arithmetic intensity of about 1, so the kernel is a pure HBM read stream).
//
// Mapping for gfx950 (64-wide waves):
//   * one K row is 256 bytes = 16 lanes x 16 bytes, so a wave-wide dwordx4 load
//     covers 4 consecutive rows with fully coalesced 1 KiB requests;
//   * each lane multiplies its 8 values with the matching 8 values of q
//     (v_dot2_f32_f16 / v_dot2_f32_bf16, fp32 accumulation) and the 16 partial
//     sums of a row are added with four DPP steps inside the 16-lane DPP row;
//   * 16 loads (64 rows, 16 KiB per wave) are issued back to back before the
//     first use, which is what keeps enough bytes in flight per CU;
//   * the G query heads that share a KV head are scored from the same
//     registers, so each K row is read from HBM exactly once per group.
#include "attn_common.h"

namespace kc {
namespace {

template <int DT, int G>
__global__ __launch_bounds__(256) void kscan_kernel(const uint16_t* __restrict__ q,
                                                    const uint16_t* __restrict__ K,
                                                    const int32_t* __restrict__ seq_lens,
                                                    float* __restrict__ z, int H, int Hkv,
                                                    int kv_split, int S_cap, int kv0,
                                                    int chunks_per_unit, float scale,
                                                    int* __restrict__ flags) {
  const int chunk = blockIdx.x % chunks_per_unit;
  const int ku = kv0 + blockIdx.x / chunks_per_unit;
  const int b = ku / Hkv, hk = ku - b * Hkv;  // Hkv counts launch units per sequence
  const size_t kv_phys = (size_t)b * (Hkv / kv_split) + hk / kv_split;
  int s = seq_lens[b];
  if (s < 1 || s > S_cap) {
    if (threadIdx.x == 0 && chunk == 0) atomicOr(flags, kFlagBadSeqLen);
    s = s < 1 ? 0 : S_cap;
  }
  const int row0 = chunk * kScanRowsPerBlock;
  if (row0 >= s) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane & 15;  // which 16-byte piece of the row
  const int rg = lane >> 4;   // which of the 4 rows of one load

  uint4 qv[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qv[g] = *reinterpret_cast<const uint4*>(q + ((size_t)b * H + hk * G + g) * kHeadDim + sub * 8);

  const uint4* __restrict__ Kp =
      reinterpret_cast<const uint4*>(K + kv_phys * S_cap * kHeadDim);
  float* __restrict__ zu = z + ((size_t)b * H + hk * G) * S_cap;

  constexpr int kRowsPerWave = kScanRowsPerBlock / 4;
#pragma unroll 1
  for (int it = 0; it < kRowsPerWave / 64; ++it) {
    const int base = row0 + wave * kRowsPerWave + it * 64;
    if (base >= s) break;
    uint4 kr[16];
    if (base + 64 <= S_cap) {
      const uint4* p = Kp + (size_t)(base + rg) * 16 + sub;
#pragma unroll
      for (int u = 0; u < 16; ++u) kr[u] = load_stream16(p + u * 64);
    } else {  // last rows of the cache: never read beyond S_cap
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        int r = base + u * 4 + rg;
        r = r < S_cap ? r : S_cap - 1;
        kr[u] = Kp[(size_t)r * 16 + sub];
      }
    }
    float keep[G];
#pragma unroll
    for (int g = 0; g < G; ++g) keep[g] = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = row_sum<16>(dot8<DT>(kr[u], qv[g]));
        keep[g] = (sub == u) ? a : keep[g];
      }
    }
    // lane (rg, sub) now holds the score of row base + sub*4 + rg
    const int myrow = base + sub * 4 + rg;
    if (myrow < s) {
#pragma unroll
      for (int g = 0; g < G; ++g) zu[(size_t)g * S_cap + myrow] = keep[g] * scale;
    }
  }
}

template <int DT>
hipError_t launch_dt(const Shape& sh, const void* q, const void* k, const int32_t* seq_lens,
                     float* z, int kv0, int kv_count, int* flags, hipStream_t st) {
  // groups of 16 or 32 query heads run as 2 or 4 launch units of 8 heads per KV head
  const int split = kv_split_for(sh.H / sh.Hkv);
  const int G = sh.H / sh.Hkv / split, Hkv_l = sh.Hkv * split;
  kv0 *= split;
  kv_count *= split;
  const int chunks = (sh.S_cap + kScanRowsPerBlock - 1) / kScanRowsPerBlock;
  const dim3 grid((unsigned)(kv_count * chunks)), block(256);
  const float scale = 0.08838834764831845f;  // 1 / sqrt(128)
  const uint16_t* qp = static_cast<const uint16_t*>(q);
  const uint16_t* kp = static_cast<const uint16_t*>(k);
#define KC_LAUNCH(GG)                                                                          \
  hipLaunchKernelGGL((kscan_kernel<DT, GG>), grid, block, 0, st, qp, kp, seq_lens, z, sh.H,     \
                     Hkv_l, split, sh.S_cap, kv0, chunks, scale, flags)
  switch (G) {
    case 1: KC_LAUNCH(1); break;
    case 2: KC_LAUNCH(2); break;
    case 4: KC_LAUNCH(4); break;
    case 8: KC_LAUNCH(8); break;
    default: return hipErrorInvalidValue;
  }
#undef KC_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t launch_kscan(const Shape& sh, const void* q, const void* k, const int32_t* seq_lens,
                        float* z, int kv0, int kv_count, int* flags, hipStream_t st) {
  if (kv_count <= 0) return hipSuccess;
  return sh.dtype == 0 ? launch_dt<0>(sh, q, k, seq_lens, z, kv0, kv_count, flags, st)
                       : launch_dt<1>(sh, q, k, seq_lens, z, kv0, kv_count, flags, st);
}

}  // namespace kc
