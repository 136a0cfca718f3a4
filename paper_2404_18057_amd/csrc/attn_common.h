// Device helpers shared by the attention kernels of this library: the 256-byte
// row layout (16 lanes x 16 bytes), dot products and row reductions, the K scan
// of one chunk into LDS, and the cache-bypassing loads / stores used to hand
// data from one workgroup to another inside a launch.
#pragma once

#include "kc_internal.h"

namespace kc {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf162_t __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
  if constexpr (DT == 0) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b),
                                  acc, false);
  } else {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf162_t, a),
                                           __builtin_bit_cast(bf162_t, b), acc, false);
  }
}

template <int DT>
__device__ __forceinline__ float dot8(const uint4& k, const uint4& q) {
  float a = dot2<DT>(k.x, q.x, 0.f);
  a = dot2<DT>(k.y, q.y, a);
  a = dot2<DT>(k.z, q.z, a);
  return dot2<DT>(k.w, q.w, a);
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true);
  return x + __builtin_bit_cast(float, y);
}

// A cache row of D 16-bit values is LPR = D / 8 lanes x 16 bytes (8, 16 or 32 lanes for
// D = 64, 128, 256), so one wave-wide 16-byte load reads RPL = 64 / LPR rows.
template <int D>
struct RowLayout {
  static_assert(D == 64 || D == 128 || D == 256, "head dimension must be 64, 128 or 256");
  static constexpr int LPR = D / 8;
  static constexpr int RPL = 64 / LPR;
  // loads a lane keeps in flight per scan iteration, and the rows they cover (at most 64,
  // so that any chunk size that is a multiple of 64 rows per wave works)
  static constexpr int LOADS = LPR == 16 ? 16 : 8;  // (32-lane rows: fewer, their sums cost more registers)
  static constexpr int ROWS = LOADS * RPL;
};

// Sum over the LPR lanes that hold one row, returned to every one of them.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);  // row_half_mirror: 8 lanes
  if constexpr (LPR >= 16) x = dpp_add<0x140>(x);  // row_mirror: the 16 lanes of a DPP row
  if constexpr (LPR == 32) x += __shfl_xor(x, 16, 64);  // the neighbouring DPP row
  return x;
}

// acc[0..7] += w * (the 8 16-bit values of v)
template <int DT>
__device__ __forceinline__ void fma8(float (&acc)[8], const uint4& v, float w) {
  const uint32_t r[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float lo, hi;
    if constexpr (DT == 0) {
      half2_t h = __builtin_bit_cast(half2_t, r[i]);
      lo = (float)h.x;
      hi = (float)h.y;
    } else {
      lo = __uint_as_float(r[i] << 16);
      hi = __uint_as_float(r[i] & 0xffff0000u);
    }
    acc[2 * i] = fmaf(w, lo, acc[2 * i]);
    acc[2 * i + 1] = fmaf(w, hi, acc[2 * i + 1]);
  }
}

// Data that one workgroup hands to another inside the launch (chunk candidates
// and partials) is written through to memory and read around the per-XCD L2 with
// device-scope relaxed atomics (sc1 stores / loads).  That keeps the hand-over
// coherent across XCDs without the L2 write-back / invalidate walk that a
// release / acquire fence costs (about 1 us each, thousands per launch).
template <typename T>
__device__ __forceinline__ void st_dev(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T ld_dev(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Scores of the R positions [row0, row0 + R) of one (sequence, KV head) against
// the G query heads of its group, written to z[g * R + local] (LDS); local is the
// position relative to row0.  Called by all NT threads of the workgroup.
//
// For D = 128 a K row is 16 lanes x 16 bytes, so a wave-wide 16-byte load reads 4 rows
// as one coalesced 1 KiB request; 16 such loads are issued back to back (16 KiB per wave
// in flight) with the non-temporal hint.  Each lane multiplies its 8 values with
// q (fp32 accumulate); the partials of a row are added across its lanes with DPP.
// Rows at or beyond s are not loaded past S_cap and their scores are not defined.
template <int DT, int G, int NT, int D = kHeadDim>
__device__ __forceinline__ void score_chunk(const uint16_t* __restrict__ q_group,
                                            const uint16_t* __restrict__ K_unit, int S_cap, int s,
                                            int row0, int R, float scale, float* z) {
  typedef RowLayout<D> RL;
  // 32-lane rows with 8 heads: 8 query pieces and their 8 running scores per lane leave room
  // for 4 loads in flight, not 8 (the build spilled 184 bytes per lane otherwise)
  constexpr int LPR = RL::LPR, RPL = RL::RPL, U = (LPR == 32 && G >= 8) ? 4 : RL::LOADS;
  constexpr int ROWS = U * RPL;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  uint4 qv[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qv[g] = *reinterpret_cast<const uint4*>(q_group + (size_t)g * D + sub * 8);
  const uint4* __restrict__ Kp = reinterpret_cast<const uint4*>(K_unit);
  const int rows_per_wave = R / (NT / 64);  // a multiple of 64
#pragma unroll 1
  for (int it = 0; it < rows_per_wave / ROWS; ++it) {
    const int local = wave * rows_per_wave + it * ROWS;
    const int base = row0 + local;
    if (base >= s) break;
    uint4 kr[U];
    if (base + ROWS <= S_cap) {
      const uint4* p = Kp + (size_t)(base + rg) * LPR + sub;
#pragma unroll
      for (int u = 0; u < U; ++u) kr[u] = load_stream16(p + u * 64);
    } else {  // last rows of the cache: never read beyond S_cap
#pragma unroll
      for (int u = 0; u < U; ++u) {
        int r = base + u * RPL + rg;
        r = r < S_cap ? r : S_cap - 1;
        kr[u] = Kp[(size_t)r * LPR + sub];
      }
    }
    float keep[G];
#pragma unroll
    for (int g = 0; g < G; ++g) keep[g] = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float x = row_sum<LPR>(dot8<DT>(kr[u], qv[g]));
        keep[g] = (sub == u) ? x : keep[g];
      }
    }
    if (sub < U) {  // lane `sub` of a row group holds the row of load `sub`
#pragma unroll
      for (int g = 0; g < G; ++g) z[g * R + local + sub * RPL + rg] = keep[g] * scale;
    }
  }
}

// ---- K rows stored as OCP FP8 E4M3 codes (1 sign, 4 exponent bits with bias 7, 3
// fraction bits), 128 bytes per row.
//
// gfx950 converts two codes to two fp16 values in one instruction
// (v_cvt_scalef32_pk_f16_fp8; with a scale of 1 the result is value(code) exactly, checked
// for all finite codes on the hardware), which then go through the same packed dot product
// as a 16-bit K row.

// dot product of 4 E4M3 codes (one dword) with 4 16-bit values (qa: channels 0-1, qb: 2-3)
template <int DT>
__device__ __forceinline__ float dot4_e4m3(uint32_t w, uint32_t qa, uint32_t qb, float acc) {
  if constexpr (DT == 0) {
    const half2_t k01 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false);  // bytes 0, 1
    const half2_t k23 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true);   // bytes 2, 3
    acc = __builtin_amdgcn_fdot2(k01, __builtin_bit_cast(half2_t, qa), acc, false);
    return __builtin_amdgcn_fdot2(k23, __builtin_bit_cast(half2_t, qb), acc, false);
  } else {
    // bf16 queries: codes to fp32 (v_cvt_pk_f32_fp8, exact), whose upper halves are the
    // same values as bf16 (a code has 3 fraction bits), packed two to a register
    typedef float float2_t __attribute__((ext_vector_type(2)));
    const float2_t f01 = __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
    const float2_t f23 = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
    const uint32_t k01 = __builtin_amdgcn_perm(__float_as_uint(f01.y), __float_as_uint(f01.x),
                                               0x07060302u);  // (hi16(y) << 16) | hi16(x)
    const uint32_t k23 = __builtin_amdgcn_perm(__float_as_uint(f23.y), __float_as_uint(f23.x),
                                               0x07060302u);
    acc = dot2<1>(k01, qa, acc);
    return dot2<1>(k23, qb, acc);
  }
}

// Sum over the 8 lanes of half a DPP row, returned to every lane of the half row.
__device__ __forceinline__ float row8_sum(float x) {
  x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);  // row_half_mirror
  return x;
}

// score_chunk for a K cache of E4M3 codes.  A row is 8 lanes x 16 bytes,
// a wave-wide 16-byte load reads 8 rows; 8 loads (64 rows) are in flight per wave.  `scale`
// must carry 2^k_exp / sqrt(d_h).
template <int DT, int G, int NT>
__device__ __forceinline__ void score_chunk8(const uint16_t* __restrict__ q_group,
                                             const uint8_t* __restrict__ K_unit, int S_cap, int s,
                                             int row0, int R, float scale, float* z) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane & 7, rg = lane >> 3;
  uint4 qv[G][2];  // this lane's 16 channels of every head
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint4* qp = reinterpret_cast<const uint4*>(q_group + (size_t)g * kHeadDim + sub * 16);
    qv[g][0] = qp[0];
    qv[g][1] = qp[1];
  }
  const uint4* __restrict__ Kp = reinterpret_cast<const uint4*>(K_unit);  // 8 per row
  const int rows_per_wave = R / (NT / 64);  // a multiple of 64
#pragma unroll 1
  for (int it = 0; it < rows_per_wave / 64; ++it) {
    const int local = wave * rows_per_wave + it * 64;
    const int base = row0 + local;
    if (base >= s) break;
    uint4 kr[8];
    if (base + 64 <= S_cap) {
      const uint4* p = Kp + (size_t)(base + rg) * 8 + sub;
#pragma unroll
      for (int u = 0; u < 8; ++u) kr[u] = load_stream16(p + u * 64);
    } else {  // last rows of the cache: never read beyond S_cap
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int r = base + u * 8 + rg;
        r = r < S_cap ? r : S_cap - 1;
        kr[u] = Kp[(size_t)r * 8 + sub];
      }
    }
    float keep[G];
#pragma unroll
    for (int g = 0; g < G; ++g) keep[g] = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float x = dot4_e4m3<DT>(kr[u].x, qv[g][0].x, qv[g][0].y, 0.f);
        x = dot4_e4m3<DT>(kr[u].y, qv[g][0].z, qv[g][0].w, x);
        x = dot4_e4m3<DT>(kr[u].z, qv[g][1].x, qv[g][1].y, x);
        x = dot4_e4m3<DT>(kr[u].w, qv[g][1].z, qv[g][1].w, x);
        x = row8_sum(x);
        keep[g] = (sub == u) ? x : keep[g];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) z[g * R + local + sub * 8 + rg] = keep[g] * scale;
  }
}

constexpr int kXcds = 8;  // accelerator complex dies of an MI355X

}  // namespace kc
