// Conventional decode attention with the K and the V cache both in HBM:
// out = softmax(q K^T / sqrt(d_h)) V over all cached positions (paper section 2;
// Table 1 rows S and A of plain MHA).  It serves the layers whose V cache the
// method leaves in HBM (section 3.1 and the caption of Table 2: the leading L
// layers) and it is the baseline of the break-even analysis (section 3.2,
// equations (3)-(4)): per position it reads a K row and a V row, 512 bytes,
// where the KCache path reads 256 bytes from HBM and N rows over the host link.
//
// One launch per layer, split over the context like the fused KCache kernel:
//   1. a workgroup scores R positions of one (sequence, KV head) for the G query
//      heads of the group (scores to LDS);
//   2. per head: chunk maximum m, p = exp(z - m) in place, l = sum p;
//   3. it streams the chunk's V rows once and accumulates o = sum_t p[t] V[t] for
//      all G heads from the same registers;
//   4. (m, l, o) go to the workspace; the workgroup that completes a unit rescales
//      and adds the chunk results:  out = sum_c e^(m_c - M) o_c / sum_c e^(m_c - M) l_c.
// HBM bound: 512 bytes and 4 G d_h FLOPs per (KV head, position).
#include "attn_common.h"
#include "topn.h"

namespace kc {
namespace {

constexpr int AT = kFusedThreads;
constexpr int AW = AT / 64;

template <int D>
struct FullSmem {
  float z[kFusedZFloats];  // scores, then softmax numerators, [G][R]; reused by the merge
  TopNScratch<AT> sc;      // reduction scratch
  float red[AW * D];
  int last;
};

template <int DT, int G, int D>
__global__ __launch_bounds__(AT) __attribute__((amdgpu_waves_per_eu(4, 4))) void full_kernel(
    FullArgs a) {
  typedef RowLayout<D> RL;
  constexpr int LPR = RL::LPR, RPL = RL::RPL;
  __shared__ FullSmem<D> sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  // all chunks of a KV unit run on one XCD, unit u on XCD u % 8 (workgroups are
  // dealt to the XCDs round-robin in launch order); a.spread (a test option) deals the
  // chunks of a unit over all XCDs instead
  const int xcd = blockIdx.x % kXcds, in_xcd = blockIdx.x / kXcds;
  const int chunk = a.spread ? (int)(blockIdx.x % a.chunks_cap) : in_xcd % a.chunks_cap;
  const int ku = a.spread ? (int)(blockIdx.x / a.chunks_cap) : xcd + kXcds * (in_xcd / a.chunks_cap);
  if (ku >= a.kv_count) return;
  const int b = ku / a.Hkv, hk = ku - b * a.Hkv;  // a.Hkv counts launch units per sequence
  const size_t kv_phys = (size_t)b * (a.Hkv / a.kv_split) + hk / a.kv_split;
  const int R = a.R;
  int s = a.seq_lens[b];
  if (s < 1 || s > a.S_cap) {
    if (tid == 0 && chunk == 0) atomicOr(a.flags, kFlagBadSeqLen);
    s = s < 1 ? 0 : a.S_cap;
  }
  const int unit0 = b * a.H + hk * G;
  if (s == 0) {
    if (chunk == 0 && tid < D)
      for (int g = 0; g < G; ++g) a.out[(size_t)(unit0 + g) * D + tid] = 0.f;
    return;
  }
  const int row0 = chunk * R;
  if (row0 >= s) return;
  const int chunks_b = (s + R - 1) / R;
  const int n = (s - row0 < R) ? s - row0 : R;

  // ---------------- 1. scores -> LDS
  score_chunk<DT, G, AT, D>(a.q + (size_t)unit0 * D, a.K + kv_phys * a.S_cap * D, a.S_cap, s,
                            row0, R, a.scale, sm.z);
  __syncthreads();

  // ---------------- 2. per head: chunk maximum, numerators in place, their sum
#pragma unroll 1
  for (int g = 0; g < G; ++g) {
    float* zg = sm.z + g * R;
    float m = -INFINITY;
    for (int i = tid; i < n; i += AT) m = fmaxf(m, zg[i]);
    m = wave_max(m);
    if (lane == 0) sm.sc.red_m[wave] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < AW; ++w) m = fmaxf(m, sm.sc.red_m[w]);
    float l = 0.f;
    for (int i = tid; i < R; i += AT) {
      const float p = (i < n) ? __expf(zg[i] - m) : 0.f;  // rows beyond the length weigh nothing
      zg[i] = p;
      l += p;
    }
    l = wave_sum(l);
    if (lane == 0) sm.sc.red_l[wave] = l;
    __syncthreads();
    if (tid == 0) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < AW; ++w) t += sm.sc.red_l[w];
      const size_t slot = (size_t)(unit0 + g) * a.chunks_cap + chunk;
      st_dev(&a.part[slot].x, m);
      st_dev(&a.part[slot].y, t);
    }
    __syncthreads();  // red_m / red_l are reused by the next head
  }

  // ---------------- 3. o[g] = sum_t p[g][t] V[t]: the chunk's V rows are read once
  float acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
  {
    const uint4* __restrict__ Vp = reinterpret_cast<const uint4*>(a.V + kv_phys * a.S_cap * D);
    constexpr int ROWS = RL::ROWS, U = RL::LOADS;
    const int rows_per_wave = R / AW;
#pragma unroll 1
    for (int it = 0; it < rows_per_wave / ROWS; ++it) {
      const int local = wave * rows_per_wave + it * ROWS;
      const int base = row0 + local;
      if (base >= s) break;
      // rows per lane in flight; fewer when G accumulators need the registers
      constexpr int VB = (G >= 4 && U > 8) ? 8 : U;
#pragma unroll 1
      for (int h = 0; h < U; h += VB) {
        uint4 vr[VB];
        if (base + ROWS <= s) {
          const uint4* p = Vp + (size_t)(base + rg) * LPR + sub;
#pragma unroll
          for (int u = 0; u < VB; ++u) vr[u] = load_stream16(p + (h + u) * 64);
        } else {  // ragged end: rows at or beyond the length are neither read nor used
#pragma unroll
          for (int u = 0; u < VB; ++u) {
            const int r = base + (h + u) * RPL + rg;
            vr[u] = (r < s) ? Vp[(size_t)r * LPR + sub] : make_uint4(0, 0, 0, 0);
          }
        }
#pragma unroll
        for (int u = 0; u < VB; ++u) {
#pragma unroll
          for (int g = 0; g < G; ++g)
            fma8<DT>(acc[g], vr[u], sm.z[g * R + local + (h + u) * RPL + rg]);
        }
      }
    }
  }
  // add the row groups of a wave, then the waves; one head at a time through LDS
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int m = LPR; m < 64; m <<= 1) acc[g][i] += __shfl_xor(acc[g][i], m, 64);
    }
    if (rg == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) sm.red[wave * D + sub * 8 + i] = acc[g][i];
    }
    __syncthreads();
    if (tid < D) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < AW; ++w) t += sm.red[w * D + tid];
      st_dev(a.part_o + ((size_t)(unit0 + g) * a.chunks_cap + chunk) * D + tid, t);
    }
    __syncthreads();
  }

  // ---------------- 4. the workgroup that completes the unit combines the chunks
  // Every thread waits for the acknowledgement of its own write-through stores,
  // the barrier collects the workgroup, one thread takes the unit's ticket; the
  // last arriver's reads are issued after its ticket has returned.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) {
    const int ticket =
        __hip_atomic_fetch_add(a.counters + ku, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (ticket == chunks_b - 1);
    if (last) st_dev(a.counters + ku, 0);  // ready for the next launch
    sm.last = last;
  }
  __syncthreads();
  if (!sm.last) return;

  float* fac = sm.z;  // e^(m_c - M) per chunk, at most kFusedZFloats chunks at a time
  const int c_lane = tid % D, c_grp = tid / D;  // AT / D groups of D channels
  constexpr int GRPS = AT / D;
#pragma unroll 1
  for (int g = 0; g < G; ++g) {
    const size_t slot0 = (size_t)(unit0 + g) * a.chunks_cap;
    float m = -INFINITY, l = 0.f;
    for (int c = tid; c < chunks_b; c += AT) {
      const float mc = ld_dev(&a.part[slot0 + c].x), lc = ld_dev(&a.part[slot0 + c].y);
      const float mm = fmaxf(m, mc);
      l = (m == mm ? l : l * __expf(m - mm)) + (mc == mm ? lc : lc * __expf(mc - mm));
      m = mm;
    }
    const float2 ML = block_merge_stats<AT>(m, l, &sm.sc);
    float o = 0.f;
    for (int c0 = 0; c0 < chunks_b; c0 += kFusedZFloats) {
      const int cn = chunks_b - c0 < kFusedZFloats ? chunks_b - c0 : kFusedZFloats;
      __syncthreads();
      for (int c = tid; c < cn; c += AT) fac[c] = __expf(ld_dev(&a.part[slot0 + c0 + c].x) - ML.x);
      __syncthreads();
      constexpr int U = 8;
      for (int c = c_grp; c < cn; c += GRPS * U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int cc = c + u * GRPS;
          v[u] = (cc < cn) ? ld_dev(a.part_o + (slot0 + c0 + cc) * D + c_lane) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int cc = c + u * GRPS;
          if (cc < cn) o = fmaf(fac[cc], v[u], o);
        }
      }
    }
    sm.red[c_grp * D + c_lane] = o;
    __syncthreads();
    if (tid < D) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < GRPS; ++w) t += sm.red[w * D + tid];
      a.out[(size_t)(unit0 + g) * D + tid] = t / ML.y;
    }
    __syncthreads();
  }
}

template <int DT, int D>
hipError_t launch_dt(const FullArgs& a, int G, hipStream_t st) {
  const long long per_xcd = (long long)((a.kv_count + kXcds - 1) / kXcds) * a.chunks_cap;
  if (per_xcd * kXcds > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(per_xcd * kXcds)), block(AT);
  switch (G) {
    case 1: hipLaunchKernelGGL((full_kernel<DT, 1, D>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((full_kernel<DT, 2, D>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((full_kernel<DT, 4, D>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((full_kernel<DT, 8, D>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int DT>
hipError_t launch_d(const FullArgs& a, int G, hipStream_t st) {
  switch (a.d) {
    case 64: return launch_dt<DT, 64>(a, G, st);
    case 128: return launch_dt<DT, 128>(a, G, st);
    case 256: return launch_dt<DT, 256>(a, G, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// Positions per workgroup: 1024 (as in the fused KCache kernel), less when the
// group's scores would not fit the LDS buffer or the launch would be too small
// to fill the chip.
int full_rows_per_block(int kv_units, int G, int S_cap, int row_bytes) {
  int R = 1024 * kRowBytes / row_bytes;  // the same bytes per workgroup whatever the row size
  if (R * G > kFusedZFloats) R = kFusedZFloats / G;
  while (R > kFusedThreads && (int64_t)kv_units * ((S_cap + R - 1) / R) < 512) R /= 2;
  return R;
}

hipError_t launch_full(const FullArgs& a, int dtype, hipStream_t st) {
  if (a.kv_count <= 0) return hipSuccess;
  const int G = a.H / a.Hkv;
  if (a.R % kFusedThreads != 0 || a.R * G > kFusedZFloats) return hipErrorInvalidValue;
  return dtype == 0 ? launch_d<0>(a, G, st) : launch_d<1>(a, G, st);
}

}  // namespace kc
