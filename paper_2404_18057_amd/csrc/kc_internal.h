// Internal launch interface between the host side of libkcache and its kernels.
// Nothing here is part of the C ABI (include/kcache.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kc {

constexpr int kHeadDim = 128;           // d_h: one row = 128 16-bit values = 256 bytes
constexpr int kRowBytes = 256;
constexpr int kScanRowsPerBlock = 1024;  // K rows scored by one workgroup
constexpr int kSelectThreads = 512;
constexpr int kFusedThreads = 512;       // workgroup size of the fused decode kernel
constexpr int kFusedZFloats = 8192;      // fp32 scores one workgroup keeps in LDS ([G][R])

// 16-byte load that tells the caches the data will not be used again.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// bits of the device-check word
constexpr int kFlagBadSeqLen = 1;
constexpr int kFlagBadPos = 2;
constexpr int kFlagBadIndex = 4;  // a selected position fell outside [0, s): skipped, never read

// The kernels score at most 8 query heads from one pass over a K row.  Larger groups
// (16 or 32 query heads per KV head) run as 2 or 4 launch units per KV head, each with 8 of
// the group's heads: the launch then sees Hkv * split KV heads of group size 8, and unit
// (b, hk') reads the rows of physical head hk' / split.
inline int kv_split_for(int G) { return G > 8 ? G / 8 : 1; }

struct Shape {
  int B, H, Hkv, S_cap, N, dtype;
  int renorm = 0;  // 1: kept weights are divided by their sum
  int d = kHeadDim;  // head dimension (the store handles 64, 128, 256; the unfused kernels 128)
};

// Scores z[b][h][t] = (q[b][h] . K[b][h/G][t]) / sqrt(d_h) for the KV units
// [kv0, kv0 + kv_count) (a KV unit is one (sequence, KV head)); all G query
// heads of a unit are scored from one pass over its K rows.
hipError_t launch_kscan(const Shape& sh, const void* q, const void* k, const int32_t* seq_lens,
                        float* z, int kv0, int kv_count, int* flags, hipStream_t st);

// Softmax statistics over all s_b scores and exact top-N_eff selection for the
// query units [u0, u0 + count) (unit = b*H + h).  Writes ascending positions
// and their softmax weights, padded with -1 / 0 up to N.
hipError_t launch_select(const Shape& sh, const float* z, const int32_t* seq_lens, int32_t* idx,
                         float* w, int u0, int count, hipStream_t st);

// out[b][h][:] = sum_j w[j] * V[b][h/G][idx[j]][:].  `v` is the mapped host
// cache (or, with packed = 1, a device buffer holding row j of unit u at
// (u*N + j)*d).
hipError_t launch_gather(const Shape& sh, const void* v, const int32_t* idx, const float* w,
                         float* out, int u0, int count, int packed, hipStream_t st);

// Copy rows of src [B][T][Hkv][d] to dst [B][Hkv][S_cap][d] at pos[b] + t; src2 / dst2
// (may be null) are a second pair moved in the same launch.
// With k_fp8 the first pair is quantised on the way: 16-bit rows in, E4M3 codes of
// value * 2^-k_exp out (128 bytes per row).
hipError_t launch_store(const Shape& sh, const void* src, void* dst, const void* src2, void* dst2,
                        const int32_t* pos, int T, int* flags, int dst_is_host, hipStream_t st,
                        int k_fp8 = 0, int k_exp = 0);

// Fused decode kernel (decode_fused.hip): scan + local top-N per chunk, merge,
// V pull and weighted sum in one launch.
struct FusedArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;  // device-visible address of the mapped host cache
  const int32_t* seq_lens;
  float* out;
  int32_t* idx;
  float* w;
  float* cand_z;      // [units][chunks_cap][kk] chunk-local top scores
  int32_t* cand_pos;  // their positions
  float2* part;       // [units][chunks_cap] (max, sum of exp) of each chunk
  float* bound;       // [units][chunks_cap] a score that r of the chunk's rows reach (pruning)
  int* counters;      // [kv units] arrival tickets, zero between launches
  int* flags;
  int H, Hkv, S_cap, N;
  int R;           // positions per workgroup, a multiple of kFusedThreads, R * G <= kFusedZFloats
  int chunks_cap;  // ceil(S_cap / R)
  int kk;          // min(N, R): candidates kept per chunk
  int kv0;
  int kv_count;    // KV units of this launch
  int renorm;      // 1: kept weights are divided by their sum
  int kv_split;    // launch units per physical KV head (see kv_split_for)
  int k_fp8;       // 1: K rows are E4M3 codes (128 bytes per row); scale carries 2^k_exp
  int d;           // head dimension: 64, 128 or 256
  int dedup;       // 1: a group's heads pull the union of their V rows once
  int spread;      // 1: deal the chunks of a unit over all XCDs (test option, see fused_kernel)
  const int* plan; // dense numbering of the chunks that exist (launch_fused_plan), or null
  float scale;
};
int fused_rows_per_block(int kv_units, int G, int S_cap, int N, int k_row_bytes);
hipError_t launch_fused(const FusedArgs& a, int dtype, int kv_count, hipStream_t st);

// Dense numbering of the chunks that exist, for batches whose sequences are shorter than the
// cache's capacity (see fused_kernel).  fused_plan_items: ints the plan of such a launch
// occupies, or 0 when the launch shape does not take one (units per sequence not a multiple
// of eight, a single chunk of capacity, a small grid, sizes beyond the packing).
// launch_fused_plan fills it from the lengths in device memory; it must run before the fused
// launch that reads it, on the same stream, whenever the lengths may have changed.
size_t fused_plan_items(int B, int units_per_seq, int chunks_cap);
hipError_t launch_fused_plan(const int32_t* seq_lens, int B, int units_per_seq, int S_cap, int R,
                             int* plan, hipStream_t st);

// Conventional attention with K and V in HBM (full_attention.hip).
struct FullArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;  // device-visible [B][Hkv][S_cap][d]
  const int32_t* seq_lens;
  float* out;
  float2* part;   // [units][chunks_cap] (max, sum of exp(z - max)) of each chunk
  float* part_o;  // [units][chunks_cap][d] sum of exp(z - max) * V over the chunk
  int* counters;  // [kv units] arrival tickets, zero between launches
  int* flags;
  int H, Hkv, S_cap;
  int R;           // positions per workgroup, a multiple of kFusedThreads, R * G <= kFusedZFloats
  int chunks_cap;  // ceil(S_cap / R)
  int kv_count;
  int kv_split;    // launch units per physical KV head (see kv_split_for)
  int d;           // head dimension: 64, 128 or 256
  int spread;      // 1: deal the chunks of a unit over all XCDs (test option)
  float scale;
};
int full_rows_per_block(int kv_units, int G, int S_cap, int row_bytes);
hipError_t launch_full(const FullArgs& a, int dtype, hipStream_t st);

hipError_t launch_probe_read(const void* ptr, size_t bytes, uint32_t* sink, hipStream_t st);
hipError_t launch_probe_rows(const void* ptr, size_t total_rows, int64_t n_rows, uint32_t* sink,
                             hipStream_t st);

}  // namespace kc
