// Fused KCache decode attention: one launch per layer does the K scan, the
// softmax statistics, the top-N selection, the V pull and the weighted sum
// (paper section 3.1 and Table 1 rows S~ and A~; Figure 1 lower half).
//
// Why one kernel.  The K scan is a pure HBM read stream (arithmetic intensity
// about 1, Table 1) and the V pull is bound by the host link (section 3.2,
// equation (3)); they only overlap if some (sequence, head) units are already
// pulling V rows while others are still being scanned.  Writing all fp32
// scores back to HBM for a separate selection kernel costs the read stream
// about 15 % (measured: interleaved small writes), so the scores never leave
// the chip:
//
//   1. a workgroup scores R consecutive positions of one (sequence, KV head)
//      for all G query heads of the group and keeps the scores in LDS;
//   2. it reduces them to what the rest of the method needs: the chunk's
//      softmax partials (max, sum of exp) and its own top-min(N, R) scores
//      with their positions -- any member of the unit's global top-N is
//      necessarily in the top-N of its chunk under the same ordering, so the
//      union of the chunk lists is an exact candidate set;
//   3. the workgroup that finishes a unit last (ticket counter) merges the
//      chunk lists: combines the partials into the full-context softmax
//      normaliser, selects the final top-N among the candidates, writes
//      positions and weights, pulls the N rows of V from mapped host memory
//      and accumulates the output.  No workgroup ever waits for another.
//
// Units finish at different times (chunks of one unit are adjacent in the
// grid), so the V pulls of early units overlap the K scan of later ones.
//
// Steps 2 and 3 are done by the whole workgroup for a single query head (block_topn,
// pull_and_accumulate) and by one wavefront per head, all heads of a group at the same
// time, for grouped queries (wave_topn, wave_pull); a launch of a single round of workgroups
// uses the single-wavefront routines for a single head as well (see the kernel body).
#include "attn_common.h"
#include "topn.h"

namespace kc {
namespace {

#ifdef KC_TIMING  // developer build only: per-phase cycle sums in flags[32..]
#define KC_T(var) const unsigned long long var = wall_clock64()
// the sums of a workgroup are collected in LDS and added to the global slots when it ends, so
// that no phase waits for a contended global atomic of the phase before it
#define KC_TDECL __shared__ unsigned long long kc_tacc[9]; if (threadIdx.x == 0) { for (int i_ = 0; i_ < 9; ++i_) kc_tacc[i_] = 0; }
#define KC_TADD(slot, val) do { if (threadIdx.x == 0) kc_tacc[slot] += (unsigned long long)(val); } while (0)
#define KC_TFLUSH do { if (threadIdx.x == 0) { for (int i_ = 0; i_ < 9; ++i_) if (kc_tacc[i_]) atomicAdd(reinterpret_cast<unsigned long long*>(a.flags + 32) + i_, kc_tacc[i_]); } } while (0)
#else
#define KC_T(var)
#define KC_TDECL
#define KC_TADD(slot, val)
#define KC_TFLUSH
#endif

constexpr int FT = kFusedThreads;
constexpr int FW = FT / 64;

constexpr int kStage = 1024;  // entries of each of the two staging arrays inside hist[]
constexpr int kPlanSeqs = 2048;    // longest batch a launch plan is built for
constexpr int kPlanChunkBits = 12; // a plan entry is (unit of the XCD) << 12 | chunk
constexpr int kPruneCands = 2 * kFusedZFloats;  // candidates of a unit the pruned merge can take

template <int D>
struct Smem {
  float z[kFusedZFloats];  // scores of this chunk, [G][R]; reused for the merge
  TopNScratch<FT> sc;
  float red_out[FW * D];
  int last;
  int redo;  // grouped queries: a head's pruned merge did not fit, merge again without pruning
};

// V pull + weighted sum for one unit by the whole workgroup: FW * RPL row slots of LPR
// lanes (32 slots of 16 lanes for D = 128), 8 independent row reads per slot in flight.
// iu / wu may point to LDS or to global memory.
template <int DT, int D>
__device__ __forceinline__ void pull_and_accumulate(const uint4* __restrict__ Vp, const int32_t* iu,
                                                    const float* wu, int n_eff, int s, int* flags,
                                                    float* __restrict__ out_u, Smem<D>* sm) {
  constexpr int LPR = RowLayout<D>::LPR, RPL = RowLayout<D>::RPL;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int slot = wave * RPL + rg;
  constexpr int SLOTS = FW * RPL, UNR = 8;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int j0 = slot; j0 < n_eff; j0 += SLOTS * UNR) {
    int t[UNR];
    float w[UNR];
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + u * SLOTS;
      t[u] = (j < n_eff) ? iu[j] : -1;
      w[u] = (j < n_eff) ? wu[j] : 0.f;
      // the selection only emits positions below s; a row outside the unit is never read
      if (t[u] >= s) {
        atomicOr(flags, kFlagBadIndex);
        t[u] = -1;
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      v[u] = make_uint4(0, 0, 0, 0);
      if (t[u] >= 0) v[u] = Vp[(size_t)t[u] * LPR + sub];
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      if (t[u] >= 0) fma8<DT>(acc, v[u], w[u]);
  }
  // add the row groups of the wave (lanes that hold the same channels), then the waves
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) acc[i] += __shfl_xor(acc[i], m, 64);
  }
  if (rg == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) sm->red_out[wave * D + sub * 8 + i] = acc[i];
  }
  __syncthreads();
  if (threadIdx.x < D) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < FW; ++w) t += sm->red_out[w * D + threadIdx.x];
    out_u[threadIdx.x] = t;
  }
  __syncthreads();
}

// The same for one unit by ONE wavefront (no barrier): RPL row slots, 8 row reads per slot
// in flight.  il / wl: the unit's positions and weights in LDS.
template <int DT, int D>
__device__ __forceinline__ void wave_pull(const uint4* __restrict__ Vp, const int32_t* il,
                                          const float* wl, int n_eff, int s, int* flags,
                                          float* __restrict__ out_u) {
  constexpr int LPR = RowLayout<D>::LPR, RPL = RowLayout<D>::RPL;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPR, rg = lane / LPR;
  constexpr int UNR = 8;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int j0 = rg; j0 < n_eff; j0 += RPL * UNR) {
    int t[UNR];
    float w[UNR];
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + u * RPL;
      t[u] = (j < n_eff) ? il[j] : -1;
      w[u] = (j < n_eff) ? wl[j] : 0.f;
      if (t[u] >= s) {  // the selection only emits positions below s
        atomicOr(flags, kFlagBadIndex);
        t[u] = -1;
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      v[u] = make_uint4(0, 0, 0, 0);
      if (t[u] >= 0) v[u] = Vp[(size_t)t[u] * LPR + sub];
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      if (t[u] >= 0) fma8<DT>(acc, v[u], w[u]);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) acc[i] += __shfl_xor(acc[i], m, 64);
  }
  if (rg == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) out_u[sub * 8 + i] = acc[i];
  }
}

// What the wavefront that has selected a head's rows does next: st_w[r] / st_i[r] hold the
// weight and the candidate index of the r-th kept entry (LDS), kept this lane's share of the
// weights' sum.  Fetches the candidates' positions in one batch, renormalises if asked,
// writes the unit's lists and, unless the group's union is pulled afterwards, pulls and sums
// its V rows.
template <int DT, int D>
__device__ __forceinline__ void wave_finish_head(const FusedArgs& a, int unit, int N, int n_eff,
                                                 int M, int s, const int32_t* cp, float* st_w,
                                                 int32_t* st_i, float kept, bool dedup,
                                                 const uint4* __restrict__ Vp) {
  const int lane = threadIdx.x & 63;
  const float inv = a.renorm ? 1.f / wave_sum(kept) : 1.f;
  int32_t* iu = a.idx + (size_t)unit * N;
  float* wu = a.w + (size_t)unit * N;
  for (int r = lane; r < n_eff; r += 64) {
    const int ci = st_i[r];
    const int32_t t = ((unsigned)ci < (unsigned)M) ? ld_dev(cp + ci) : -1;
    const float w = a.renorm ? st_w[r] * inv : st_w[r];
    st_i[r] = t;
    st_w[r] = w;
    iu[r] = t;
    wu[r] = w;
  }
  for (int j = n_eff + lane; j < N; j += 64) {
    iu[j] = -1;
    wu[j] = 0.f;
  }
  if (!dedup) wave_pull<DT, D>(Vp, st_i, st_w, n_eff, s, a.flags, a.out + (size_t)unit * D);
}

// De-duplicated V pull for a group of G query heads (grouped-query attention): the heads
// of a group read the same V head, so a position that several of them selected is pulled
// over the host link once and accumulated into each head's output with that head's weight.
// (The paper only states that the method carries over to GQA, section 5; every head still
// makes its own selection.)  The union is built with a bitmap over the positions:
//   bm[w]          bit p % 32 of word p / 32 set iff some head kept position p
//   pf[w]          number of set bits before word w: the rank of a kept position in the
//                  union is pf[p / 32] + popcount(bits of its word below p)
//   upos[u]        position of the u-th row of the union (ascending)
//   wt[u * G + g]  weight of that row for head g, 0 if head g did not keep it
// idx / w: the group's positions and weights in global memory, [G][N], written earlier by
// this workgroup.  Needs G * n_eff <= 2 * FT, G * G * n_eff <= 2048 (wt lives in the
// histogram array), s <= 32 * kFusedZFloats / 2 (bm and pf share the score buffer).
template <int DT, int G, int D>
__device__ __forceinline__ void pull_union(const uint4* __restrict__ Vp, const int32_t* idx,
                                           const float* w, int N, int n_eff, int s,
                                           float* __restrict__ out_group, Smem<D>* sm) {
  constexpr int LPR = RowLayout<D>::LPR, RPL = RowLayout<D>::RPL;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  uint32_t* bm = reinterpret_cast<uint32_t*>(sm->z);
  int* pf = reinterpret_cast<int*>(sm->z) + kFusedZFloats / 2;
  float* wt = reinterpret_cast<float*>(sm->sc.hist);
  int* upos = reinterpret_cast<int*>(sm->sc.list_key);  // list_key, list_idx, list_rank: 1536 ints
  const int words = (s + 31) >> 5, total = G * n_eff;
  for (int i = tid; i < words; i += FT) bm[i] = 0u;
  for (int i = tid; i < total * G; i += FT) wt[i] = 0.f;
  // the lists were written by whichever threads found the entries: read them around the L1
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  int p[2];
  float wv[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int e = tid + k * FT;
    p[k] = -1;
    wv[k] = 0.f;
    if (e < total) {
      const int g = e / n_eff, j = e - g * n_eff;
      p[k] = ld_dev(idx + (size_t)g * N + j);
      wv[k] = ld_dev(w + (size_t)g * N + j);
      if (p[k] >= s) p[k] = -1;  // cannot happen for a finished selection; never index past s
    }
  }
#pragma unroll
  for (int k = 0; k < 2; ++k)
    if (p[k] >= 0) atomicOr(&bm[p[k] >> 5], 1u << (p[k] & 31));
  __syncthreads();
  // exclusive prefix of the word popcounts; each thread owns a contiguous run of words
  const int per = (words + FT - 1) / FT;
  int mine = 0;
  for (int i = 0; i < per; ++i) {
    const int wd = tid * per + i;
    mine += (wd < words) ? __popc(bm[wd]) : 0;
  }
  int before = block_excl_scan<FT>(mine, sm->sc.wave_tot);
  for (int i = 0; i < per; ++i) {
    const int wd = tid * per + i;
    if (wd < words) {
      pf[wd] = before;
      before += __popc(bm[wd]);
    }
  }
  if (tid == FT - 1) sm->sc.rank = before;  // rows in the union
  __syncthreads();
  const int U = sm->sc.rank;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    if (p[k] >= 0) {
      const int e = tid + k * FT, g = e / n_eff;
      const int u = pf[p[k] >> 5] + __popc(bm[p[k] >> 5] & ((1u << (p[k] & 31)) - 1u));
      wt[u * G + g] = wv[k];
      upos[u] = p[k];  // every head that kept the row writes the same value
    }
  }
  __syncthreads();

  const int slot = wave * RPL + rg;
  constexpr int SLOTS = FW * RPL, UNR = 4;
  float acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
  for (int u0 = slot; u0 < U; u0 += SLOTS * UNR) {
    uint4 v[UNR];
    int uu[UNR];
#pragma unroll
    for (int k = 0; k < UNR; ++k) {
      uu[k] = u0 + k * SLOTS;
      v[k] = make_uint4(0, 0, 0, 0);
      if (uu[k] < U) v[k] = Vp[(size_t)upos[uu[k]] * LPR + sub];
    }
#pragma unroll
    for (int k = 0; k < UNR; ++k) {
      if (uu[k] < U) {
#pragma unroll
        for (int g = 0; g < G; ++g) fma8<DT>(acc[g], v[k], wt[uu[k] * G + g]);
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int m = LPR; m < 64; m <<= 1) acc[g][i] += __shfl_xor(acc[g][i], m, 64);
    }
    if (rg == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) sm->red_out[wave * D + sub * 8 + i] = acc[g][i];
    }
    __syncthreads();
    if (tid < D) {
      float t = 0.f;
#pragma unroll
      for (int wv_ = 0; wv_ < FW; ++wv_) t += sm->red_out[wv_ * D + tid];
      out_group[(size_t)g * D + tid] = t;
    }
    __syncthreads();
  }
}

// Two workgroups per CU (4 waves per SIMD), not the three that registers and LDS
// would allow: measured on MI355X the launch is 3-7 % faster that way on the
// large workloads (fewer units in flight per XCD, so units complete and start
// pulling V earlier, and less contention for the CU while a workgroup selects).
template <int DT, int G, bool K8, int D>
__global__ __launch_bounds__(FT) __attribute__((amdgpu_waves_per_eu(4, 4))) void fused_kernel(
    FusedArgs a) {
  __shared__ Smem<D> sm;
  const int tid = threadIdx.x;
  // XCD-aware mapping.  Workgroups are handed to the 8 XCDs round-robin in launch
  // order, so block b runs on XCD b % 8.  All chunks of a KV unit are given to one
  // XCD (unit u lives on XCD u % 8): a unit then completes as soon as its own XCD
  // has scanned it, instead of waiting for the slowest of eight, and the merging
  // and pulling workgroups spread evenly over the XCDs.  (With chunks dealt over all
  // XCDs one slightly slower XCD ended up finishing - and therefore merging and
  // pulling - 80 % of all units, which made it slower still.)
  //
  // a.spread (KC_OPT_XCD_SPREAD, for tests) deals consecutive chunks of a unit to consecutive
  // workgroups instead, i.e. over all eight XCDs: slower, same results; it makes every
  // hand-over below cross XCD boundaries, so the tests can show that correctness does not
  // rest on the mapping.
  //
  // a.plan (batches that may be ragged).  The grid has a workgroup for every chunk of every
  // sequence's capacity, because the lengths live in device memory; a workgroup whose chunk
  // lies beyond its sequence's length exits at once, but it still takes a slot for the time of
  // a launch, in between the working ones (config 4: 47 % of the grid, 7 % of the launch).
  // plan_kernel therefore numbers the chunks that exist densely, in the same order: entry i
  // of the plan names the unit and chunk of the i-th workgroup of every XCD, plan[0] counts
  // them, and the workgroups left over come last in the grid and exit while the last units
  // finish.  For full-length sequences the numbering is the one above.
  int chunk, ku_rel;
  if (a.plan) {
    const unsigned i = blockIdx.x / kXcds;
    if (i >= (unsigned)a.plan[0]) return;
    const unsigned e = (unsigned)a.plan[1 + i];
    const unsigned per = (unsigned)a.Hkv / kXcds, uix = e >> kPlanChunkBits;
    const unsigned bq = uix / per;
    chunk = (int)(e & ((1u << kPlanChunkBits) - 1u));
    ku_rel = (int)(bq * (unsigned)a.Hkv + blockIdx.x % kXcds + kXcds * (uix - bq * per));
  } else {
    const unsigned in_xcd = a.spread ? blockIdx.x : blockIdx.x / kXcds;
    const unsigned group = in_xcd / (unsigned)a.chunks_cap;
    chunk = (int)(in_xcd - group * (unsigned)a.chunks_cap);
    ku_rel = a.spread ? (int)group : (int)(blockIdx.x % kXcds + kXcds * group);
    if (ku_rel >= a.kv_count) return;  // padding of the last group of eight units
  }
  const int ku = a.kv0 + ku_rel;
  const int b = ku / a.Hkv, hk = ku - b * a.Hkv;  // a.Hkv counts launch units per sequence
  const size_t kv_phys = (size_t)b * (a.Hkv / a.kv_split) + hk / a.kv_split;
  const int R = a.R, N = a.N, kk = a.kk;
  int s = a.seq_lens[b];
  if (s < 1 || s > a.S_cap) {
    if (tid == 0 && chunk == 0) atomicOr(a.flags, kFlagBadSeqLen);
    s = s < 1 ? 0 : a.S_cap;
  }
  const int unit0 = b * a.H + hk * G;  // first query head of the group
  if (s == 0) {                        // nothing cached: defined output, no work
    if (chunk == 0) {
      for (int g = 0; g < G; ++g) {
        for (int j = tid; j < N; j += FT) {
          a.idx[(size_t)(unit0 + g) * N + j] = -1;
          a.w[(size_t)(unit0 + g) * N + j] = 0.f;
        }
        if (tid < D) a.out[(size_t)(unit0 + g) * D + tid] = 0.f;
      }
    }
    return;
  }
  // grouped queries: 512 words per wavefront for the selections the wavefronts run on their own
  __shared__ uint32_t whist[G > 1 ? FW * 512 : 1];
  const int row0 = chunk * R;
  if (row0 >= s) return;
  const int chunks_b = (s + R - 1) / R;
  const int n = (s - row0 < R) ? s - row0 : R;  // valid rows of this chunk
  KC_TDECL
  KC_T(t0);

  // ---------------- 1. scores of R positions for the G heads of the group -> LDS
  if constexpr (K8)  // K rows are E4M3 codes, 128 bytes each
    score_chunk8<DT, G, FT>(a.q + (size_t)unit0 * D,
                            reinterpret_cast<const uint8_t*>(a.K) + kv_phys * a.S_cap * D,
                            a.S_cap, s, row0, R, a.scale, sm.z);
  else
    score_chunk<DT, G, FT, D>(a.q + (size_t)unit0 * D, a.K + kv_phys * a.S_cap * D, a.S_cap, s,
                              row0, R, a.scale, sm.z);
  __syncthreads();
  KC_T(t1);
  KC_TADD(0, t1 - t0);
  KC_TADD(7, 1);

  // ---------------- 2. per head: softmax partials and the chunk's own top-min(N, R)
  const bool lone = G == 1 && (long long)a.kv_count * a.chunks_cap <= 512;
  float* const stage_f = reinterpret_cast<float*>(sm.sc.hist);
  int32_t* const stage_i = reinterpret_cast<int32_t*>(sm.sc.hist) + kStage;
  const int k_loc = kk < n ? kk : n;
  const bool stage_loc = k_loc <= kStage;
  // Pruning bound for the merge.  A chunk with more rows than it may keep ("full") also
  // reports a score that at least r_bound of its rows reach, with r_bound * (number of full
  // chunks) >= N: the union of those rows alone has N members, so the unit's N-th largest
  // score is no smaller than the smallest of the reported values, and the merge can drop
  // every candidate below it before selecting.
  const int last_rows_b = s - (chunks_b - 1) * R;
  const int n_full = kk < R ? chunks_b - (last_rows_b > kk ? 0 : 1) : 0;
  const int r_bound = (n_full > 0 && n > kk) ? (N + n_full - 1) / n_full : 0;
  if constexpr (G > 1) {
    // Grouped queries: the G heads are independent, so each wavefront takes a head and does
    // its statistics and its selection alone, without a workgroup barrier, all heads at the
    // same time (head after head with the whole workgroup, the selection costs G times a
    // barrier-bound 8 us per chunk and outweighs the K scan it follows).
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll 1
    for (int g = wave; g < G; g += FW) {
      const float* zg = sm.z + g * R;
      const size_t slot = (size_t)(unit0 + g) * a.chunks_cap + chunk;
      auto key = [&](int i) { return zg[i]; };
      float m, z_lo, l, bound;
      bool finite;
      wave_minmax(key, n, z_lo, m, finite);
      float* cz = a.cand_z + slot * kk;
      int32_t* cp = a.cand_pos + slot * kk;
      wave_topn<true>(key, n, k_loc, z_lo, m, finite, whist + wave * 512,
                      [&](int r, int i, float v) {
                        st_dev(cz + r, v);
                        st_dev(cp + r, row0 + i);
                      }, &l, r_bound, &bound);
      if (lane == 0) {
        st_dev(&a.part[slot].x, m);
        st_dev(&a.part[slot].y, l);
        st_dev(a.bound + slot, bound);
      }
    }
    KC_T(t2w);
    KC_TADD(2, t2w - t1);
  } else if (lone) {
    // a launch of a single round of workgroups is bound by the latency of its steps, not by
    // HBM: the first wavefront selects alone (no barriers; 2-3 us instead of 7), the others
    // go on to the hand-over barrier
    if (tid < 64) {
      const size_t slot = (size_t)unit0 * a.chunks_cap + chunk;
      auto key = [&](int i) { return sm.z[i]; };
      float m, z_lo, l, bound;
      bool finite;
      wave_minmax(key, n, z_lo, m, finite);
      float* cz = a.cand_z + slot * kk;
      int32_t* cp = a.cand_pos + slot * kk;
      wave_topn<true>(key, n, k_loc, z_lo, m, finite, sm.sc.hist,
                      [&](int r, int i, float v) {
                        st_dev(cz + r, v);
                        st_dev(cp + r, row0 + i);
                      }, &l, r_bound, &bound);
      if (tid == 0) {
        st_dev(&a.part[slot].x, m);
        st_dev(&a.part[slot].y, l);
        st_dev(a.bound + slot, bound);
      }
    }
  } else {
#pragma unroll 1
  for (int g = 0; g < G; ++g) {
    const float* zg = sm.z + g * R;
    auto key = [&](int i) { return zg[i]; };
    const size_t slot = (size_t)(unit0 + g) * a.chunks_cap + chunk;
    KC_T(t2a);
    const float2 ml = block_softmax_stats<FT>(key, n, &sm.sc);
    KC_T(t2b);
    KC_TADD(1, t2b - t2a);
    if (tid == 0) {
      st_dev(&a.part[slot].x, ml.x);
      st_dev(&a.part[slot].y, ml.y);
    }
    float* cz = a.cand_z + slot * kk;
    int32_t* cp = a.cand_pos + slot * kk;
    float bound;
    block_topn<FT, false>(key, n, k_loc, &sm.sc, [&](int r, int i, float v) {
      if (stage_loc) {  // collect in LDS, then write whole lines
        stage_f[r] = v;
        stage_i[r] = row0 + i;
      } else {
        st_dev(cz + r, v);
        st_dev(cp + r, row0 + i);
      }
    }, r_bound, &bound);
    if (G == 1 && tid == 0) st_dev(a.bound + slot, bound);
    if (stage_loc) {
      for (int r = tid; r < k_loc; r += FT) {
        st_dev(cz + r, stage_f[r]);
        st_dev(cp + r, stage_i[r]);
      }
      __syncthreads();  // the staging area is the next head's histogram
    }
    KC_T(t2c);
    KC_TADD(2, t2c - t2b);
  }
  }
  KC_T(t3);

  // ---------------- 3. the workgroup that completes the unit merges and pulls V
  // Hand-over: every thread waits until its own write-through stores have been
  // acknowledged, the barrier collects the workgroup, then one thread takes the
  // unit's ticket.  The last arriver's reads (ld_dev) are issued after its ticket
  // has returned, so they see every other chunk's lists.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) {
    const int ticket =
        __hip_atomic_fetch_add(a.counters + ku, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (ticket == chunks_b - 1);
    if (last) st_dev(a.counters + ku, 0);  // ready for the next launch
    sm.last = last;
    sm.redo = 0;
  }
  __syncthreads();
  KC_T(t4);
  KC_TADD(3, t4 - t3);
  if (!sm.last) {
    KC_TFLUSH;
    return;
  }

  const int n_eff = N < s ? N : s;
  const int last_rows = s - (chunks_b - 1) * R;
  const int M = (chunks_b - 1) * kk + (kk < last_rows ? kk : last_rows);  // candidates
  const bool z_in_lds = M <= kFusedZFloats, pos_in_lds = 2 * M <= kFusedZFloats;
  const bool stage_out = n_eff <= kStage;
  // the merge may prune by the chunks' bounds when the candidates fit the registers of the
  // workgroup, 32 per thread (single-head units only: the grouped-query builds have no
  // registers to spare for it)
  const bool try_prune = G == 1 && M <= kPruneCands && stage_out && n_full > 0;
  const uint4* __restrict__ Vp =
      reinterpret_cast<const uint4*>(a.V) + kv_phys * a.S_cap * (D / 8);
  // grouped queries: pull the union of the group's rows once (see pull_union)
  const bool dedup = G > 1 && a.dedup && G * n_eff <= 2 * FT && G * G * n_eff <= 2048 &&
                     s <= 32 * (kFusedZFloats / 2);
  // Grouped queries, the usual sizes (the candidates of at least two heads fit the score
  // buffer, at most 256 rows kept): the heads are merged side by side, one wavefront per head,
  // as many heads per round as the score buffer holds candidates for.  (One wavefront works
  // through 1024 candidates in about 5 us, the whole workgroup takes about 10 us for any
  // number of them: with room for one head at a time the loop below is the faster one.)  The workgroup stages the candidates of
  // a round in LDS with all its threads; from there on a wavefront needs no barrier: the
  // normaliser from the chunk partials, the selection, the positions of the kept entries,
  // the lists in global memory and (unless the group's union is pulled) the V pull and sum.
  if constexpr (G > 1) {
    constexpr int kWaveKeep = 256;
    // First choice, pruned as for single heads (see "Pruning bound" above): every wavefront
    // streams the candidates of its head from memory, keeps those that reach the smallest
    // bound of the head's full chunks (ordered, with their candidate index) in its 1 / G of
    // the score buffer, and selects among the survivors, typically a few hundred however
    // many chunks the unit has; all heads at once.  A head whose survivors do not fit its
    // part of the buffer (or, with NaN scores, are fewer than the rows to keep) raises
    // sm.redo and the group is merged again by the paths below.
    if (n_full > 0 && n_eff <= kWaveKeep && G <= FW) {
      const int wave = tid >> 6, lane = tid & 63;
      constexpr int P = kFusedZFloats / G / 2;   // survivors a head may keep
      if (wave < G) {
        const int unit = unit0 + wave;
        const size_t slot0 = (size_t)unit * a.chunks_cap;
        const float* cz = a.cand_z + slot0 * kk;
        const int32_t* cp = a.cand_pos + slot0 * kk;
        float* zreg = sm.z + wave * (2 * P);
        int32_t* sreg = reinterpret_cast<int32_t*>(zreg) + P;
        // Every full chunk vouches for r_b of its scores reaching its bound, so the
        // need-th largest bound, need = ceil(N / r_b) chunks, is a value that N scores of the
        // unit reach (with more full chunks than rows to keep that is far tighter than the
        // smallest bound).  Found by bisection on the integer keys of up to 8 bounds a lane.
        constexpr int PBL = 8;
        const int r_b = (N + n_full - 1) / n_full, need = (N + r_b - 1) / r_b;
        const int pbn = (chunks_b + 63) / 64;
        float m = -INFINITY, l = 0.f, pb = INFINITY;
        uint32_t pk[PBL];
#pragma unroll
        for (int j = 0; j < PBL; ++j) pk[j] = 0u;   // below every key of a real bound
        for (int c = lane, j = 0; c < chunks_b; c += 64, ++j) {
          const float mc = ld_dev(&a.part[slot0 + c].x), lc = ld_dev(&a.part[slot0 + c].y);
          const float mm = fmaxf(m, mc);
          l = (m == mm ? l : l * __expf(m - mm)) + (mc == mm ? lc : lc * __expf(mc - mm));
          m = mm;
          if (c < chunks_b - 1 || last_rows > kk) {
            const float bc = ld_dev(a.bound + slot0 + c);
            pb = fminf(pb, bc);
#pragma unroll
            for (int jj = 0; jj < PBL; ++jj)
              if (jj == j) pk[jj] = score_key(bc);
          }
        }
        const float mx = wave_max(m);
        const float inv_Z = 1.f / wave_sum(m == mx ? l : l * __expf(m - mx));
        float L = wave_min(pb);   // the smallest bound: always valid
        if (pbn <= PBL && need < n_full) {
          uint32_t T = 0u;
#pragma unroll 1
          for (int bit = 31; bit >= 0; --bit) {
            const uint32_t cand_key = T | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int j = 0; j < PBL; ++j)
              if (j < pbn) cnt += pk[j] >= cand_key ? 1 : 0;
            if (wave_sum(cnt) >= need) T = cand_key;
          }
          // T is the need-th largest key; the bound it belongs to is the smallest one not below
          float at = INFINITY;
          for (int c = lane; c < chunks_b; c += 64)
            if (c < chunks_b - 1 || last_rows > kk) {
              const float bc = ld_dev(a.bound + slot0 + c);
              if (score_key(bc) >= T) at = fminf(at, bc);
            }
          at = wave_min(at);
          if (at < INFINITY && at > L) L = at;
        }
        if (!(L > -INFINITY)) L = -INFINITY;   // NaN or -inf: keep everything
        const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        constexpr int LB = 16;
        int Mp = 0;
        bool fits = true;
        for (int i0 = 0; i0 < M && fits; i0 += 64 * LB) {
          float zt[LB];
#pragma unroll
          for (int u = 0; u < LB; ++u) {
            const int i = i0 + u * 64 + lane;
            zt[u] = (i < M) ? ld_dev(cz + i) : -INFINITY;
          }
#pragma unroll
          for (int u = 0; u < LB; ++u) {
            const int i = i0 + u * 64 + lane;
            const bool keep = i < M && zt[u] >= L;
            const uint64_t b = __ballot(keep);
            const int cnt = __popcll(b);
            if (Mp + cnt > P) fits = false;   // the same in every lane
            if (keep && fits) {
              const int dst = Mp + __popcll(b & lt_mask);
              zreg[dst] = zt[u];
              sreg[dst] = i;
            }
            Mp += cnt;
          }
        }
        if (!fits || Mp < n_eff) {
          if (lane == 0) sm.redo = 1;
        } else {
          auto cand = [&](int i) { return zreg[i]; };
          float c_lo, c_hi;
          bool finite;
          wave_minmax(cand, Mp, c_lo, c_hi, finite);
          float* st_w = reinterpret_cast<float*>(whist + wave * 512);
          int32_t* st_i = reinterpret_cast<int32_t*>(whist + wave * 512) + kWaveKeep;
          float kept = 0.f;
          wave_topn<false>(cand, Mp, n_eff, c_lo, c_hi, finite, whist + wave * 512,
                           [&](int r, int i, float v) {
                             const float w = expf(v - mx) * inv_Z;
                             kept += w;
                             st_w[r] = w;
                             st_i[r] = sreg[i];
                           });
          wave_finish_head<DT, D>(a, unit, N, n_eff, M, s, cp, st_w, st_i, kept, dedup, Vp);
        }
      }
      __syncthreads();
      if (!sm.redo) {
        if (dedup)
          pull_union<DT, G, D>(Vp, a.idx + (size_t)unit0 * N, a.w + (size_t)unit0 * N, N, n_eff,
                               s, a.out + (size_t)unit0 * D, &sm);
        KC_TFLUSH;
        return;
      }
    }
    const int fit = M > 0 ? kFusedZFloats / M : 0;
    const int HR = fit < FW ? (fit < G ? fit : G) : (FW < G ? FW : G);
    if (HR >= 2 && n_eff <= kWaveKeep) {
      const int wave = tid >> 6, lane = tid & 63;
      constexpr int LB = 8;
#pragma unroll 1
      for (int g0 = 0; g0 < G; g0 += HR) {
        const int hr = G - g0 < HR ? G - g0 : HR;
        const int tot = hr * M;
        for (int e0 = tid; e0 < tot; e0 += FT * LB) {
          float zt[LB];
#pragma unroll
          for (int u = 0; u < LB; ++u) {
            const int e = e0 + u * FT;
            const int h = e / M, i = e - h * M;
            zt[u] = (e < tot)
                        ? ld_dev(a.cand_z + (size_t)(unit0 + g0 + h) * a.chunks_cap * kk + i)
                        : 0.f;
          }
#pragma unroll
          for (int u = 0; u < LB; ++u) {
            const int e = e0 + u * FT;
            if (e < tot) sm.z[e] = zt[u];
          }
        }
        __syncthreads();
        KC_T(w0);
        if (wave < hr) {
          const int unit = unit0 + g0 + wave;
          const size_t slot0 = (size_t)unit * a.chunks_cap;
          const int32_t* cp = a.cand_pos + slot0 * kk;
          const float* zl = sm.z + wave * M;
          float m = -INFINITY, l = 0.f;
          for (int c = lane; c < chunks_b; c += 64) {
            const float mc = ld_dev(&a.part[slot0 + c].x), lc = ld_dev(&a.part[slot0 + c].y);
            const float mm = fmaxf(m, mc);
            l = (m == mm ? l : l * __expf(m - mm)) + (mc == mm ? lc : lc * __expf(mc - mm));
            m = mm;
          }
          const float mx = wave_max(m);
          const float inv_Z = 1.f / wave_sum(m == mx ? l : l * __expf(m - mx));
          float* st_w = reinterpret_cast<float*>(whist + wave * 512);
          int32_t* st_i = reinterpret_cast<int32_t*>(whist + wave * 512) + kWaveKeep;
          float kept = 0.f;
          KC_T(w1);
          KC_TADD(4, w1 - w0);
          // (the staging arrays are the selection's histogram, dead by the time it emits)
          auto cand = [&](int i) { return zl[i]; };
          float c_lo, c_hi;
          bool finite;
          wave_minmax(cand, M, c_lo, c_hi, finite);
          wave_topn<false>(cand, M, n_eff, c_lo, c_hi, finite, whist + wave * 512,
                    [&](int r, int i, float v) {
                      const float w = expf(v - mx) * inv_Z;
                      kept += w;
                      st_w[r] = w;
                      st_i[r] = i;
                    });
          KC_T(w2);
          KC_TADD(5, w2 - w1);
          wave_finish_head<DT, D>(a, unit, N, n_eff, M, s, cp, st_w, st_i, kept, dedup, Vp);
          KC_T(w3);
          KC_TADD(6, w3 - w2);
          KC_TADD(8, 1);
        }
        __syncthreads();  // the next round overwrites the staged candidates
      }
      if (dedup)
        pull_union<DT, G, D>(Vp, a.idx + (size_t)unit0 * N, a.w + (size_t)unit0 * N, N, n_eff, s,
                             a.out + (size_t)unit0 * D, &sm);
      KC_TFLUSH;
      return;
    }
  }
#pragma unroll 1
  for (int g = 0; g < G; ++g) {
    const int unit = unit0 + g;
    const size_t slot0 = (size_t)unit * a.chunks_cap;
    // the unit's candidates are contiguous: every chunk but the last holds kk.
    // Everything the merge needs is requested in one batch of bypassing loads.
    const float* cz = a.cand_z + slot0 * kk;
    const int32_t* cp = a.cand_pos + slot0 * kk;
    // ZH: candidates per thread that the LDS buffer could also hold; the second half of zr
    // is used (big) only for units with more candidates than that
    constexpr int LB = 8, ZR = kPruneCands / FT, ZH = kFusedZFloats / FT;
    const bool big = M > kFusedZFloats;
    int32_t* pos_l = reinterpret_cast<int32_t*>(sm.z) + M;
    float pm = -INFINITY, pl = 0.f, pb = INFINITY;
    if (tid < chunks_b) {
      pm = ld_dev(&a.part[slot0 + tid].x);
      pl = ld_dev(&a.part[slot0 + tid].y);
      if (try_prune && (tid < chunks_b - 1 || last_rows > kk)) pb = ld_dev(a.bound + slot0 + tid);
    }
    float zr[G == 1 ? ZR : 1];  // pruned path: all candidates of the unit in registers, i = j * FT + tid
    if (G == 1 && try_prune) {
#pragma unroll
      for (int j = 0; j < ZH; ++j) {
        const int i = j * FT + tid;
        zr[j] = (i < M) ? ld_dev(cz + i) : -INFINITY;
      }
      if (big) {
#pragma unroll
        for (int j = ZH; j < ZR; ++j) {
          const int i = j * FT + tid;
          zr[j] = (i < M) ? ld_dev(cz + i) : -INFINITY;
        }
      }
    } else if (z_in_lds) {
      for (int i0 = tid; i0 < M; i0 += FT * LB) {
        float zt[LB];
        int32_t pr[LB];
#pragma unroll
        for (int u = 0; u < LB; ++u) {
          const int i = i0 + u * FT;
          zt[u] = (i < M) ? ld_dev(cz + i) : 0.f;
          pr[u] = (i < M && pos_in_lds) ? ld_dev(cp + i) : 0;
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) {
          const int i = i0 + u * FT;
          if (i < M) {
            sm.z[i] = zt[u];
            if (pos_in_lds) pos_l[i] = pr[u];
          }
        }
      }
    }
    float m = pm, l = pl;
    for (int c = tid + FT; c < chunks_b; c += FT) {  // more chunks than threads: rare
      const float mc = ld_dev(&a.part[slot0 + c].x), lc = ld_dev(&a.part[slot0 + c].y);
      const float mm = fmaxf(m, mc);
      l = (m == mm ? l : l * __expf(m - mm)) + (mc == mm ? lc : lc * __expf(mc - mm));
      m = mm;
      if constexpr (G == 1)
        if (try_prune && (c < chunks_b - 1 || last_rows > kk))
          pb = fminf(pb, ld_dev(a.bound + slot0 + c));
    }
    // full-context softmax normaliser from the chunk partials, and the pruning bound
    const float3 mZ = block_merge_stats_min<FT>(m, l, pb, &sm.sc);  // barriers inside
    const float mx = mZ.x, inv_Z = 1.f / mZ.y;
    KC_T(f1);
    KC_TADD(4, f1 - t4);

    // Pruned path: candidates below the bound cannot be among the N largest (see r_bound).
    // The survivors are compacted into LDS in candidate order (which is position order, so
    // ties still go to the lower position) together with their candidate index.
    int Mp = M;                                  // entries the selection runs over
    int32_t* src_l = reinterpret_cast<int32_t*>(sm.z) + kFusedZFloats / 2;
    bool pruned = false;
    if constexpr (G == 1) if (try_prune) {
      const int lane = tid & 63, wave = tid >> 6;
      const float L = mZ.z > -INFINITY ? mZ.z : -INFINITY;  // NaN or -inf: keep everything
      int* seg_cnt = sm.sc.list_rank;  // [ZR * FW] kept entries per (j, wave) segment
      int* seg_base = sm.sc.list_idx;
      const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
      for (int j = 0; j < ZH; ++j) {
        const uint64_t b = __ballot(zr[j] >= L);
        if (lane == 0) seg_cnt[j * FW + wave] = __popcll(b);
      }
      if (big) {
#pragma unroll
        for (int j = ZH; j < ZR; ++j) {
          const uint64_t b = __ballot(zr[j] >= L);
          if (lane == 0) seg_cnt[j * FW + wave] = __popcll(b);
        }
      }
      __syncthreads();
      if (wave == 0) {
        if (!big) {  // exclusive scan over the ZH * FW = 128 segments, two per lane
          const int c0 = seg_cnt[2 * lane], c1 = seg_cnt[2 * lane + 1];
          const int inc = wave_incl_scan(c0 + c1, lane);
          seg_base[2 * lane] = inc - c0 - c1;
          seg_base[2 * lane + 1] = inc - c1;
          if (lane == 63) sm.sc.rank = inc;
        } else {     // ZR * FW = 256 segments, four per lane
          int c[4], sum = 0;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            c[q] = seg_cnt[4 * lane + q];
            sum += c[q];
          }
          const int inc = wave_incl_scan(sum, lane);
          int before = inc - sum;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            seg_base[4 * lane + q] = before;
            before += c[q];
          }
          if (lane == 63) sm.sc.rank = inc;
        }
      }
      __syncthreads();
      Mp = sm.sc.rank;
      // scores and candidate indices side by side in LDS.  Fewer survivors than entries to
      // keep can only happen when scores are NaN (they compare false against the bound): the
      // ordinary selection below orders by key, NaN included, and always keeps n_eff entries.
      pruned = Mp <= kFusedZFloats / 2 && Mp >= n_eff;
      if (pruned) {
        auto place = [&](int j) {
          const bool keep = zr[j] >= L;
          const uint64_t b = __ballot(keep);
          if (keep) {
            const int dst = seg_base[j * FW + wave] + __popcll(b & lt_mask);
            sm.z[dst] = zr[j];
            src_l[dst] = j * FT + tid;
          }
        };
#pragma unroll
        for (int j = 0; j < ZH; ++j) place(j);
        if (big) {
#pragma unroll
          for (int j = ZH; j < ZR; ++j) place(j);
        }
      } else {  // the bound removed too little: select among all candidates as usual
        Mp = M;
        if (z_in_lds) {
#pragma unroll
          for (int j = 0; j < ZH; ++j) {
            const int i = j * FT + tid;
            if (i < M) sm.z[i] = zr[j];
          }
        }
      }
      __syncthreads();
    }

    int32_t* iu = a.idx + (size_t)unit * N;
    float* wu = a.w + (size_t)unit * N;
    // With room in the LDS staging arrays (N_eff <= kStage) the selection writes nothing to
    // global memory: weights and positions are collected in LDS and written out afterwards
    // in whole lines, and candidate positions that are not in LDS beside the scores are
    // fetched then, all kept entries in one round trip.
    const bool pos_here = pos_in_lds && !try_prune;   // positions were loaded into pos_l
    const bool pos_later = !pos_here && stage_out;
    float kept = 0.f;  // this thread's share of the kept softmax mass (renormalised variant)
    auto emit = [&](int r, int i, float v) {
      const float w = expf(v - mx) * inv_Z;
      kept += w;
      const int ci = pruned ? src_l[i] : i;      // index into the unit's candidate arrays
      if (stage_out) {
        stage_f[r] = w;
        stage_i[r] = pos_here ? pos_l[i] : ci;
      } else {
        wu[r] = w;
        iu[r] = pos_here ? pos_l[i] : ld_dev(cp + ci);
      }
    };
    if (lone && stage_out && (pruned || z_in_lds)) {
      if (tid < 64) {
        auto cand = [&](int i) { return sm.z[i]; };
        float c_lo, c_hi;
        bool finite;
        wave_minmax(cand, Mp, c_lo, c_hi, finite);
        wave_topn<false>(cand, Mp, n_eff, c_lo, c_hi, finite, sm.sc.hist, emit);
      }
      __syncthreads();
    } else if (pruned || z_in_lds)
      block_topn<FT, true>([&](int i) { return sm.z[i]; }, Mp, n_eff, &sm.sc, emit);
    else  // more candidates than the LDS buffer holds: read them around the L2 every pass
      block_topn<FT, true>([&](int i) { return ld_dev(cz + i); }, M, n_eff, &sm.sc, emit);
    if (stage_out) {
      for (int r = tid; r < n_eff; r += FT) {
        int32_t t = stage_i[r];
        if (pos_later) {  // t is an index into the unit's candidate arrays
          t = ((unsigned)t < (unsigned)M) ? ld_dev(cp + t) : -1;
          stage_i[r] = t;
        }
        iu[r] = t;
        if (!a.renorm) wu[r] = stage_f[r];
      }
      if (pos_later) __syncthreads();
    }
    if (a.renorm) {
      // variant: divide the kept weights by their sum (equal maxima make the merge a sum)
      const float inv = 1.f / block_merge_stats<FT>(0.f, kept, &sm.sc).y;
      if (stage_out) {
        for (int r = tid; r < n_eff; r += FT) {
          const float w = stage_f[r] * inv;
          stage_f[r] = w;
          wu[r] = w;
        }
      } else {  // written by whichever thread found the entry: re-read around the L1
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        for (int r = tid; r < n_eff; r += FT) wu[r] = ld_dev(wu + r) * inv;
        __builtin_amdgcn_s_waitcnt(0);
      }
      __syncthreads();
    }
    for (int j = n_eff + tid; j < N; j += FT) {
      iu[j] = -1;
      wu[j] = 0.f;
    }
    // block_topn ended with a barrier: positions and weights are visible to everyone
    KC_T(f2);
    KC_TADD(5, f2 - f1);
    if (!dedup)
      pull_and_accumulate<DT, D>(Vp, stage_out ? stage_i : iu, stage_out ? stage_f : wu, n_eff,
                                 s, a.flags, a.out + (size_t)unit * D, &sm);
    KC_T(f3);
    KC_TADD(6, f3 - f2);
    KC_TADD(8, 1);
  }
  if constexpr (G > 1) {
    if (dedup)
      pull_union<DT, G, D>(Vp, a.idx + (size_t)unit0 * N, a.w + (size_t)unit0 * N, N, n_eff, s,
                           a.out + (size_t)unit0 * D, &sm);
  }
  KC_TFLUSH;
}

// Fills the plan of a launch (see fused_kernel): one workgroup walks the lengths, builds the
// running count of chunks per sequence and writes one entry per chunk that exists, in the
// order an XCD's workgroups take them: sequence by sequence, within a sequence unit by unit
// (the units of that sequence on the XCD), within a unit chunk by chunk.  An entry packs
// (sequence * units-per-XCD + unit) << 12 | chunk; it is the same for all eight XCDs.
__global__ __launch_bounds__(FT) void plan_kernel(const int32_t* __restrict__ seq_lens, int B,
                                                  int per, int S_cap, int R,
                                                  int* __restrict__ plan) {
  __shared__ int pre[kPlanSeqs + 1];   // chunks (times units per XCD) before sequence b
  __shared__ int cnt[kPlanSeqs];       // chunks of sequence b
  __shared__ int wave_tot[FW];
  __shared__ int tile_total;
  const int tid = threadIdx.x;
  int carry = 0;
  for (int b0 = 0; b0 < B; b0 += FT) {
    const int b = b0 + tid;
    int c = 0;
    if (b < B) {
      int s = seq_lens[b];
      s = s < 1 ? 0 : (s > S_cap ? S_cap : s);
      c = (s + R - 1) / R;
      c = c < 1 ? 1 : c;  // an empty sequence keeps one chunk: it writes the defined empty result
      cnt[b] = c;
    }
    const int items = c * per;
    const int ex = block_excl_scan<FT>(items, wave_tot);
    if (b < B) pre[b] = carry + ex;
    if (tid == FT - 1) tile_total = ex + items;
    __syncthreads();
    carry += tile_total;
    __syncthreads();
  }
  if (tid == 0) {
    pre[B] = carry;
    plan[0] = carry;
  }
  __syncthreads();
  const int total = pre[B];
  for (int e = tid; e < total; e += FT) {
    int lo = 0, hi = B;  // largest b with pre[b] <= e
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pre[mid] <= e) lo = mid; else hi = mid;
    }
    const int rem = e - pre[lo], c = cnt[lo];
    const int jj = rem / c;
    plan[1 + e] = ((lo * per + jj) << kPlanChunkBits) | (rem - jj * c);
  }
}

template <int DT, bool K8, int D>
hipError_t launch_dt(const FusedArgs& a, int G, int kv_count, hipStream_t st) {
  // eight XCDs each get ceil(kv_count / 8) units' worth of blocks
  const long long per_xcd = (long long)((kv_count + kXcds - 1) / kXcds) * a.chunks_cap;
  if (per_xcd * kXcds > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(per_xcd * kXcds)), block(FT);
  switch (G) {
    case 1: hipLaunchKernelGGL((fused_kernel<DT, 1, K8, D>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((fused_kernel<DT, 2, K8, D>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((fused_kernel<DT, 4, K8, D>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((fused_kernel<DT, 8, K8, D>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int DT>
hipError_t launch_d(const FusedArgs& a, int G, int kv_count, hipStream_t st) {
  if (a.k_fp8) return a.d == 128 ? launch_dt<DT, true, 128>(a, G, kv_count, st) : hipErrorInvalidValue;
  switch (a.d) {
    case 64: return launch_dt<DT, false, 64>(a, G, kv_count, st);
    case 128: return launch_dt<DT, false, 128>(a, G, kv_count, st);
    case 256: return launch_dt<DT, false, 256>(a, G, kv_count, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// Positions per workgroup.  Smaller chunks let units finish (and start pulling V)
// earlier and more evenly, and leave fewer units in flight when the scan ends;
// larger chunks mean fewer workgroups paying the fixed selection and hand-over
// cost, and fewer candidates to merge.  Measured on MI355X, 256 KiB of K per workgroup
// (1024 rows of 16-bit values, 2048 rows of 8-bit codes) is the sweet spot
// as long as all of a unit's candidates fit the merging workgroup, ceil(S/R) * min(N, R) <=
// kFusedZFloats (its LDS buffer; twice that for single-head units with N <= 1024, whose merge
// first drops most candidates from registers); otherwise the smallest R that fits.  A group
// wants the candidates of all its heads in the buffer together, so that they merge side by
// side in one round (measured, G = 4: 4 x 8 KV heads x 131072, N 64: 254 -> 235 us with 2048
// rows; one sequence of 8192, N 256: 93 us with 512 rows, 66 us with 1024).
int fused_rows_per_block(int kv_units, int G, int S_cap, int N, int k_row_bytes) {
  const int cap = kFusedZFloats / G;
  const int64_t cands = G > 1 ? kFusedZFloats / G : N <= kStage ? kPruneCands : kFusedZFloats;
  const auto fits = [&](int r) { return (int64_t)((S_cap + r - 1) / r) * (N < r ? N : r) <= cands; };
  // the same K bytes per workgroup whatever the row size: an 8-bit K cache takes 2048 rows
  int R = 1024 * kRowBytes / k_row_bytes;  // 512 rows of 512 bytes ... 2048 rows of 128 bytes
  while (R < cap && !fits(R)) R *= 2;
  if (R > cap) R = cap;
  // small problems: more, smaller workgroups as long as the merge still fits
  while (R > kFusedThreads && (int64_t)kv_units * ((S_cap + R - 1) / R) < 512 && fits(R / 2))
    R /= 2;
  return R;
}

size_t fused_plan_items(int B, int units_per_seq, int chunks_cap) {
  if (B < 1 || B > kPlanSeqs || units_per_seq % kXcds != 0 || chunks_cap < 2 ||
      chunks_cap > (1 << kPlanChunkBits))
    return 0;
  const long long per_xcd = (long long)B * (units_per_seq / kXcds);
  if (per_xcd >= (1ll << (31 - kPlanChunkBits))) return 0;
  // a launch of fewer than four rounds of workgroups has nothing to gain
  if (per_xcd * chunks_cap * kXcds < 2048) return 0;
  return (size_t)(per_xcd * chunks_cap) + 1;
}

hipError_t launch_fused_plan(const int32_t* seq_lens, int B, int units_per_seq, int S_cap, int R,
                             int* plan, hipStream_t st) {
  if (B < 1 || B > kPlanSeqs || units_per_seq % kXcds != 0 || R < 1 || !plan)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(FT), 0, st, seq_lens, B, units_per_seq / kXcds,
                     S_cap, R, plan);
  return hipGetLastError();
}

hipError_t launch_fused(const FusedArgs& a, int dtype, int kv_count, hipStream_t st) {
  if (kv_count <= 0) return hipSuccess;
  const int G = a.H / a.Hkv;
  if (a.R % kFusedThreads != 0 || a.R * G > kFusedZFloats) return hipErrorInvalidValue;
  return dtype == 0 ? launch_d<0>(a, G, kv_count, st) : launch_d<1>(a, G, kv_count, st);
}

}  // namespace kc
