/*
 * libkcache: KCache decode-step attention for one MI355X (gfx950).
 *
 * The method (paper section 3.1, Figure 1, Table 1 "KCache MHA" rows): the K
 * cache of every layer stays in HBM, the V cache lives in CPU memory.  A decode
 * step scores the query against the whole K cache, takes the softmax over all
 * positions, keeps the N largest entries per (sequence, head), pulls only those
 * N rows of V across the host link and returns their weighted sum.
 *
 * Conventions of this C ABI
 *   - plain pointers and sizes only; "dev" = device (HBM) pointer, "host" =
 *     pinned, device-mapped host pointer (hipHostMalloc / torch pin_memory);
 *   - every call returns KC_OK (0) or a negative kc_status; the text of the
 *     last failure of a context is available from kcache_last_error();
 *   - arguments are validated on the host before anything is enqueued; nothing
 *     aborts or throws across the boundary;
 *   - calls enqueue work on the caller's HIP stream and do not synchronise with
 *     the host unless stated; the caller owns q / K / V / out memory, the
 *     library owns only its workspace, its side streams and events;
 *   - the store / attention / step calls never allocate: a context is sized beforehand
 *     with kcache_reserve (or the hint of kcache_create), and a call whose shape needs
 *     more fails with KC_ERR_WORKSPACE before anything is enqueued.  Setting
 *     KC_OPT_AUTO_GROW lets such a call grow the context instead, at the price of one
 *     device synchronisation each time it does;
 *   - a context is bound to one device and must not be used from two host
 *     threads at once.
 */
#ifndef KCACHE_H_
#define KCACHE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kc_ctx kc_ctx;

typedef enum { KC_F16 = 0, KC_BF16 = 1 } kc_dtype;

/* How the selected V rows cross the host link (Figure 1 "VCache Pull"; the
 * paper does not say which mechanism its engine uses):
 *   ZEROCOPY  the accumulate kernel reads the rows straight out of the mapped
 *             host cache (no host involvement, fully asynchronous);
 *   STAGED    indices go to the host, host threads pack the rows into a pinned
 *             staging buffer, one async copy brings them to HBM, a kernel
 *             accumulates.  This mode blocks the calling host thread until the
 *             indices have arrived. */
typedef enum { KC_GATHER_ZEROCOPY = 0, KC_GATHER_STAGED = 1 } kc_gather_mode;

typedef enum {
  KC_OK = 0,
  KC_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, H % Hkv != 0 ...     */
  KC_ERR_UNSUPPORTED = -2, /* head_dim not 64 / 128 / 256, group size H/Hkv not a
                              power of two up to 32, or a combination a path does
                              not serve (see the calls)                             */
  KC_ERR_NOT_PINNED = -3,  /* v_host is not device-mapped host memory (or, with
                              v_in_hbm, not device memory)                           */
  KC_ERR_WORKSPACE = -4,   /* the context is too small for the call (see kcache_reserve),
                              or its buffers could not be (re)allocated              */
  KC_ERR_HIP = -5,         /* a HIP runtime call failed; see kcache_last_error       */
  KC_ERR_DEVICE_CHECK = -6 /* a kernel found pos / seq_lens outside the cache        */
} kc_status;

/* One layer's cache.  Both buffers are owned by the caller.
 * Element (b, hk, t, c) of either cache is at ((b*Hkv + hk)*S_cap + t)*d + c, so
 * the K rows of one (sequence, KV head) form one contiguous stream and every V
 * row is one contiguous read of 2 d bytes, 256 for d = 128 (section 3.1: K in HBM, V in
 * CPU memory). */
typedef struct {
  void* k_dev;      /* dev   [B][Hkv][S_cap][d], 16-bit elements                     */
  void* v_host;     /* host  [B][Hkv][S_cap][d], same layout, pinned + mapped; with
                       v_in_hbm != 0 a dev pointer of the same layout instead        */
  int32_t B;        /* sequences                                                     */
  int32_t Hkv;      /* KV heads                                                      */
  int32_t S_cap;    /* capacity in positions                                         */
  int32_t d;        /* head dimension d_h: 64, 128 or 256 (a row is 2 d bytes)       */
  int32_t dtype;    /* kc_dtype of q, K, V                                           */
  int32_t v_in_hbm; /* 0: V in CPU memory (the method's default placement);
                       1: this layer keeps its V cache in HBM (section 3.1 and the
                       caption of Table 2: the first L layers)                      */
  int32_t k_fp8;    /* 0: K rows are `dtype` values, 2 d bytes each;
                       1: variant with an 8-bit K cache (section 1 names cache
                       quantisation as the other way to cut the bytes a decode step
                       moves): k_dev holds OCP FP8 E4M3 codes, 128 bytes per row,
                       element = value(code) * 2^k_exp.  kcache_prefill_store
                       quantises the 16-bit rows it is given (nearest, ties to even,
                       saturating at 448).  Needs d = 128; served by the fused
                       zero-copy decode path only                                  */
  int32_t k_exp;    /* the cache's power-of-two scale exponent, |k_exp| <= 32; used
                       only with k_fp8                                              */
} kc_layer_cache;

/* Identifiers for kcache_profile_read. */
typedef enum {
  KC_KERNEL_KSCAN = 0,   /* scores q.K^T / sqrt(d_h) over the context (HBM bound)    */
  KC_KERNEL_SELECT = 1,  /* softmax statistics + top-N select                        */
  KC_KERNEL_GATHER = 2,  /* V row pull + weighted sum (host-link bound)              */
  KC_KERNEL_STORE_K = 3, /* cache store, K half                                      */
  KC_KERNEL_STORE_V = 4, /* cache store, V half (device to host)                     */
  KC_KERNEL_FUSED = 5,   /* scan + select + V pull + weighted sum in one launch      */
  KC_KERNEL_FULL = 6,    /* conventional attention, K and V in HBM                   */
  KC_KERNEL_COUNT = 7
} kc_kernel_id;

/* Integer options for kcache_set_option. */
typedef enum {
  KC_OPT_PIPELINE_PARTS = 0, /* decode: split the (sequence, KV head) units into this
                                many parts so the V pull of one part overlaps the K
                                scan of the next; 0 = choose automatically            */
  KC_OPT_PROFILE = 1,        /* 1: bracket every kernel with HIP events (see
                                kcache_profile_read); 0: off (default)                */
  KC_OPT_STAGED_THREADS = 2, /* host threads packing rows in KC_GATHER_STAGED mode    */
  KC_OPT_FUSED = 3,          /* 1 (default): KC_GATHER_ZEROCOPY decodes run as one fused
                                launch per layer whose scores never leave the chip;
                                0: separate scan / select / gather launches            */
  KC_OPT_FUSED_ROWS = 4,     /* positions scored per workgroup of the fused launch and
                                of kcache_full_attention: a multiple of 512 with rows *
                                min(H/Hkv, 8) <= 8192 (ignored otherwise), or 0 = choose
                                from the shape (default)                               */
  KC_OPT_RENORMALIZE = 6,    /* 0 (default): the kept weights are the full-context softmax
                                values, as Table 1 writes them; 1: variant that divides
                                the N kept weights by their sum (section 4 remarks that
                                TopN acts as a regulariser of the softmax; the paper does not say
                                it renormalises)                                      */
  KC_OPT_STEP_LANES = 5,     /* kcache_decode_step / kcache_step_graph_create: streams a
                                step is spread over, so that the K scan of one launch
                                overlaps the tail (merge and V pull) of another.
                                0 (default): chosen from the shape - two lanes that each
                                take half of the batch through all layers in order when
                                the batch has at least two sequences and half of it still
                                covers the chip (256 workgroups), else one;
                                1: the layers one after another on the caller's stream;
                                2..4: that many lanes holding what KC_OPT_STEP_SPLIT says */
  KC_OPT_GQA_DEDUP = 8,      /* 1: with grouped queries the fused launch pulls the union of
                                the rows that the heads of a group selected, each row
                                once, instead of every head's rows separately (same
                                results up to summation order; pays when the heads of a
                                group attend to the same positions).  Used when
                                (H/Hkv)^2 * N <= 2048 and s <= 131072, otherwise the
                                per-head pull runs.  0 (default): per-head pulls       */
  KC_OPT_STEP_SPLIT = 7,     /* what an explicit number of lanes holds.  1 (default): the
                                sequences of the batch, a contiguous share per lane, each
                                share running through the layers in order on its own
                                stream - sequences are independent (section 3.3), so this
                                keeps every data dependency of a real decode step.
                                0: whole layers, dealt round-robin - only meaningful when
                                every layer's q is known up front, as in a benchmark of
                                the attention alone (in a model, layer l+1's query
                                depends on layer l's output)                           */
  KC_OPT_AUTO_GROW = 9,      /* 0 (default): a call whose shape needs more workspace,
                                tickets or staging than the context holds fails with
                                KC_ERR_WORKSPACE (size the context with kcache_reserve);
                                1: such a call grows the context itself, which
                                synchronises the device                                */
  KC_OPT_HOST_STORE_BLOCKS = 11, /* workgroups of the V half of a large kcache_prefill_store
                                (rows leave as posted PCIe writes): 0 (default) = the
                                library's choice, 2..4096 = that many.  More workgroups
                                do not make the link faster but do slow down HBM traffic
                                that runs at the same time                              */
  KC_OPT_LANE_STAGGER_US = 12, /* a step with more than one lane: lane i starts i / lanes of
                                this many microseconds late (a bounded wait on the GPU's
                                constant clock), so that the lanes' launches do not run
                                in step and the tail of one falls into the scan of
                                another.  -1 (default): derived from the shape, about 0.3
                                launch durations for the second of two lanes; 0: lanes
                                start together                                         */
  KC_OPT_XCD_SPREAD = 10     /* for tests.  0 (default): all workgroups that score one
                                (sequence, KV head) run on one of the eight XCDs, so the
                                results they hand to the finishing workgroup stay inside
                                one L2.  1: they are dealt over all XCDs (slower), so
                                every hand-over crosses XCD boundaries.  Results are bit
                                for bit the same                                       */
} kc_option;

/* Identifiers for kcache_stat. */
typedef enum {
  KC_STAT_REALLOCS = 0,        /* (re)allocations of workspace, tickets or staging buffers
                                  since the context was created (kcache_create's hint and
                                  kcache_reserve included)                              */
  KC_STAT_WORKSPACE_BYTES = 1, /* current workspace size                                */
  KC_STAT_TICKETS = 2,         /* current number of arrival tickets                     */
  KC_STAT_STEP_LANES = 3       /* value of KC_OPT_STEP_LANES                            */
} kc_stat;

/* Create a context on `device` (a HIP device ordinal) with a workspace of at
 * least workspace_bytes_hint bytes (0 is fine: kcache_reserve sizes it later).
 * *out is set only on success. */
int kcache_create(kc_ctx** out, int device, size_t workspace_bytes_hint);

/* Wait for the context's side streams, free its workspace.  NULL is accepted. */
int kcache_destroy(kc_ctx* ctx);

/* Upper bound of the device workspace one single-layer decode call of this shape needs
 * on any path for d = 128 and 16-bit K (the largest is the unfused one: fp32 scores
 * [B][H][S_cap] plus index / weight buffers [B][H][N]).  A hint for kcache_create; 0 on
 * invalid sizes.  kcache_reserve is the exact, shape-aware way to size a context. */
size_t kcache_workspace_bytes(int32_t B, int32_t H, int32_t S_cap, int32_t N);

/*
 * Sizes the context for every later call of this shape, so that none of them has to
 * allocate (and therefore synchronise): workspace, arrival tickets, the pinned and
 * device staging of KC_GATHER_STAGED, and the lane streams of a step.
 *   shape        B, Hkv, S_cap, d, dtype, v_in_hbm, k_fp8 are read; the pointers are not
 *   H, N         as for kcache_decode_attention
 *   gather_mode  the kc_gather_mode the calls will use
 *   step_layers  0: single-layer calls only; L > 0: also kcache_decode_step /
 *                kcache_step_graph_create over L layers of this shape
 * Takes the options in effect (KC_OPT_FUSED, KC_OPT_FUSED_ROWS, KC_OPT_STEP_LANES,
 * KC_OPT_STEP_SPLIT) into account: set them first.  Only ever grows the context; call it
 * once per shape that will be used.  May synchronise the device (it is the one place that
 * does); fails with KC_ERR_WORKSPACE while a step graph holds the buffers that would
 * have to move.
 */
int kcache_reserve(kc_ctx* ctx, const kc_layer_cache* shape, int32_t H, int32_t N,
                   int32_t gather_mode, int32_t step_layers);

/* Counters of the context, see kc_stat; -1 for an unknown identifier or a NULL context. */
int64_t kcache_stat(kc_ctx* ctx, int32_t which);

/* Lanes kcache_decode_step would use for L layers of this shape with the options in
 * effect (see KC_OPT_STEP_LANES); -1 on NULL arguments.  Host only. */
int32_t kcache_step_lanes_for(kc_ctx* ctx, const kc_layer_cache* shape, int32_t L, int32_t H);

/* Text of the last error recorded in this context ("" if none).  The pointer
 * stays valid until the next failing call on the context.  ctx == NULL returns
 * the text of the last failing kcache_create of the calling thread. */
const char* kcache_last_error(kc_ctx* ctx);

int kcache_set_option(kc_ctx* ctx, int32_t option, int64_t value);

/* Host-only shape check shared by the two calls below; touches no GPU state.
 * H and N are ignored when H == 0 (store-only check). */
int kcache_check_shapes(const kc_layer_cache* cache, int32_t H, int32_t N);

/*
 * Cache store (Figure 1 upper half and caption: each layer pushes its K and V
 * states; V is then copied to CPU memory asynchronously; in decode the new
 * token's states are appended the same way).  Writes T new tokens per sequence
 * at positions [pos[b], pos[b] + T).
 *   k_new_dev, v_new_dev  dev [B][T][Hkv][d], cache dtype (token-major)
 *   pos_dev               dev int32 [B]; the kernel skips (and flags, see
 *                         kcache_device_check) any row outside [0, S_cap)
 *   T                     >= 1
 *   stream                hipStream_t on which k_new / v_new / pos are ready
 *   done_event            optional hipEvent_t, recorded when the V rows have
 *                         been written to host memory
 * K rows are written into cache->k_dev on `stream`.  V rows are written to
 * cache->v_host by a kernel on an internal side stream ordered after `stream`;
 * later kcache_decode_attention calls on the same context wait for it on the
 * device.  The caller must keep v_new_dev alive until done_event (or a
 * kcache_synchronize) has completed.  With cache->v_in_hbm both halves are
 * written on `stream` by one launch.
 */
int kcache_prefill_store(kc_ctx* ctx, const kc_layer_cache* cache, const void* k_new_dev,
                         const void* v_new_dev, const int32_t* pos_dev, int32_t T, void* stream,
                         void* done_event);

/*
 * The same store for a caller that holds the positions on the host, as a serving loop does
 * for a prompt it is about to prefill (Figure 1 upper half; section 3.2, equations (1)-(2):
 * the V states of a layer are copied to CPU memory asynchronously, hidden under the next
 * layer's compute).  Knowing the positions on the host lets the V half go through the GPU's
 * copy engine (one strided device-to-host copy per (sequence, KV head)) instead of a kernel:
 * measured on MI355X it neither takes compute units nor slows HBM-bound work that runs beside
 * it, and keeps its own rate while such work runs.
 *   pos_host   host int32 [B], read during the call; [pos, pos + T) must fit the capacity
 *              (KC_ERR_INVALID_ARG otherwise, nothing is enqueued); at most 1024 sequences
 *   others     as for kcache_prefill_store
 * Small stores (decode appends) and layers with v_in_hbm take the same kernel path as
 * kcache_prefill_store.  Not meant for stream capture (the copies are issued by the host).
 */
int kcache_prefill_store_at(kc_ctx* ctx, const kc_layer_cache* cache, const void* k_new_dev,
                            const void* v_new_dev, const int32_t* pos_host, int32_t T,
                            void* stream, void* done_event);

/*
 * KCache attention for one layer and one decode step (section 3.1; Table 1 rows
 * S~ = TopN(softmax(Q K^T / sqrt(d_h))) and A~ = S~ Part(V); section 3.3 for
 * the per-(sequence, head) granularity).
 *   q_dev         dev [B][H][d], cache dtype
 *   H             query heads; H % Hkv == 0 and H / Hkv in {1, 2, 4, 8, 16, 32};
 *                 query head h reads KV head h / (H / Hkv).  Up to 8 heads of a
 *                 group are scored from one pass over the K rows; groups of 16 or
 *                 32 take 2 or 4 passes
 *   seq_lens_dev  dev int32 [B], 1 <= s_b <= S_cap, counts the current token,
 *                 whose K and V rows the caller has already stored
 *   N             >= 1; N_eff = min(N, s_b) positions are kept
 *   out_dev       dev fp32 [B][H][d]:  sum over the kept positions of
 *                 softmax(z)[t] * V[t]; the weights are the full-context
 *                 softmax values (not renormalised over the kept set)
 *   idx_out_dev   optional dev int32 [B][H][N]: kept positions, ascending,
 *                 -1 beyond N_eff; equal scores are broken towards the lower
 *                 position
 *   w_out_dev     optional dev fp32 [B][H][N]: matching weights, 0 beyond N_eff
 *   gather_mode   kc_gather_mode
 *   stream        hipStream_t; all results are complete in stream order
 * Scores and softmax are fp32; the selection is made on the fp32 scores.
 * Non-finite inputs: a NaN or infinity in q, K or V makes out / w_out of the units
 * it reaches unspecified (NaN as a rule), but never unsafe: every position in
 * idx_out stays in [-1, s_b), exactly N_eff of them are kept, and no row outside the
 * unit's cache is read.
 * A layer with cache->v_in_hbm is accepted too (its N rows then come from HBM);
 * KC_GATHER_STAGED is KC_ERR_UNSUPPORTED for such a layer.  Head dimensions 64 and
 * 256 and 8-bit K caches are served by the fused zero-copy path only (KC_OPT_FUSED
 * on, KC_GATHER_ZEROCOPY).
 */
int kcache_decode_attention(kc_ctx* ctx, const kc_layer_cache* cache, const void* q_dev, int32_t H,
                            const int32_t* seq_lens_dev, int32_t N, float* out_dev,
                            int32_t* idx_out_dev, float* w_out_dev, int32_t gather_mode,
                            void* stream);

/*
 * kcache_decode_attention for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results as kcache_decode_attention with KC_GATHER_ZEROCOPY on the fused
 * path, but the launch's scratch (chunk candidates, partials, arrival tickets) is a
 * fixed array inside the library's code object instead of the context's workspace,
 * and the call performs no hipMalloc / hipFree / event creation and no host
 * synchronisation.  Every GPU the library runs on holds its own copy of the array
 * until the process ends.
 *   - limit: the fused launch of the shape must need no more than
 *     kcache_static_scratch_bytes() (48 MiB) of scratch and at most 16384 (sequence,
 *     KV head) units; beyond that the call returns KC_ERR_WORKSPACE and enqueues
 *     nothing.  (Config 2's layer needs 17 MiB, config 4's at N = 128 34 MiB.)
 *   - all calls on one GPU share that GPU's array, whichever context or stream they
 *     come from: calls that overlap in time on one GPU race.  Calls on one stream are
 *     ordered and safe.  The tickets are cleared by a small kernel at the start of
 *     every call, so a previous call's leftovers do not matter.
 *   - KC_OPT_PROFILE does not time this call; KC_OPT_FUSED is ignored (always fused).
 */
int kcache_decode_attention_static(kc_ctx* ctx, const kc_layer_cache* cache, const void* q_dev,
                                   int32_t H, const int32_t* seq_lens_dev, int32_t N,
                                   float* out_dev, int32_t* idx_out_dev, float* w_out_dev,
                                   void* stream);
size_t kcache_static_scratch_bytes(void);

/*
 * Conventional decode attention for one layer whose V cache is in HBM
 * (cache->v_in_hbm == 1):  out = softmax(q K^T / sqrt(d_h)) V over all s_b cached
 * positions (section 2; Table 1, rows S and A of plain MHA).  This is what the
 * layers that keep V in HBM run (section 3.1; Table 2 caption) and the baseline
 * of the break-even analysis (section 3.2, equations (3)-(4)).
 *   q_dev, H, seq_lens_dev, stream   as for kcache_decode_attention
 *   out_dev                          dev fp32 [B][H][d]
 * Scores, softmax and accumulation are fp32.  Returns KC_ERR_INVALID_ARG when the
 * layer's V cache is not in HBM.
 */
int kcache_full_attention(kc_ctx* ctx, const kc_layer_cache* cache, const void* q_dev, int32_t H,
                          const int32_t* seq_lens_dev, float* out_dev, void* stream);

/*
 * A whole decode step in one call (Figure 1: every layer pushes the new token's K
 * and V states, then attends): for l = 0 .. L-1, in order, append layers[l]'s new
 * rows (T = 1, as kcache_prefill_store) and run its attention -- KCache top-N
 * (kcache_decode_attention, zero-copy gather) for a layer whose V cache is in host
 * memory, conventional attention (kcache_full_attention) for a layer with
 * v_in_hbm.  Same results as the per-layer calls; saves their host-side overhead
 * and is the unit that kcache_step_graph_create captures.
 *   layers        host array of L entries (read during the call only)
 *   H, N          as for kcache_decode_attention, shared by all layers
 *   pos_dev       dev int32 [B]: position written by the append (seq_lens - 1)
 *   seq_lens_dev  dev int32 [B]: lengths including the appended token
 */
typedef struct {
  kc_layer_cache cache;
  const void* k_new_dev; /* dev [B][1][Hkv][d] new K rows, or NULL: nothing is appended    */
  const void* v_new_dev; /* dev [B][1][Hkv][d] new V rows (NULL iff k_new_dev is NULL)     */
  const void* q_dev;     /* dev [B][H][d]                                                  */
  float* out_dev;        /* dev fp32 [B][H][d]                                             */
  int32_t* idx_out_dev;  /* optional dev int32 [B][H][N]; unused for v_in_hbm layers       */
  float* w_out_dev;      /* optional dev fp32 [B][H][N]; unused for v_in_hbm layers        */
} kc_step_layer;

int kcache_decode_step(kc_ctx* ctx, const kc_step_layer* layers, int32_t L, int32_t H,
                       const int32_t* pos_dev, const int32_t* seq_lens_dev, int32_t N,
                       void* stream);

/*
 * The same step captured once into a HIP graph and replayed with one launch per
 * decode step.  All pointers in `layers`, pos_dev and seq_lens_dev are baked into
 * the graph; their contents may change between launches (the context grows by
 * rewriting pos / seq_lens in place).  Options in effect at creation (rows, lanes)
 * stay in effect for the graph; profiling events are not part of it.  The graph
 * uses the context's workspace: do not run other calls of the same context
 * concurrently with a launch.  Destroy graphs before the context.
 */
typedef struct kc_step_graph kc_step_graph;
int kcache_step_graph_create(kc_ctx* ctx, const kc_step_layer* layers, int32_t L, int32_t H,
                             const int32_t* pos_dev, const int32_t* seq_lens_dev, int32_t N,
                             kc_step_graph** out);
int kcache_step_graph_launch(kc_ctx* ctx, kc_step_graph* graph, void* stream);
int kcache_step_graph_destroy(kc_ctx* ctx, kc_step_graph* graph);

/* Block until everything this context has enqueued (side streams included) is done. */
int kcache_synchronize(kc_ctx* ctx);

/* Synchronises, then reports whether any kernel since the last check met a
 * pos / seq_lens value outside the cache: KC_OK or KC_ERR_DEVICE_CHECK. */
int kcache_device_check(kc_ctx* ctx);

/* Per-kernel timing, active while KC_OPT_PROFILE is 1.  Synchronises, then
 * returns the sum of HIP-event durations (ms) and the number of launches of
 * `kernel` since the last kcache_profile_reset. */
int kcache_profile_read(kc_ctx* ctx, int32_t kernel, double* total_ms, int64_t* launches);
int kcache_profile_reset(kc_ctx* ctx);

/*
 * Bandwidth probes: the denominators the roofline fractions are quoted against.
 * read:  a streaming kernel sums `bytes` (multiple of 16) starting at `ptr`,
 *        device memory or mapped host memory, `iters` times; *gbps = bytes *
 *        iters / time.
 * rows:  the same kernel shape as the V pull: `n_rows` rows of 256 bytes at
 *        pseudo-random row offsets inside [ptr, ptr + bytes).
 * copy:  hipMemcpyAsync(dst, src, bytes) `iters` times (pinned H2D / D2H peak).
 * All three synchronise the stream.
 */
int kcache_probe_read(kc_ctx* ctx, const void* ptr, size_t bytes, int32_t iters, void* stream,
                      double* gbps);
int kcache_probe_rows(kc_ctx* ctx, const void* ptr, size_t bytes, int64_t n_rows, int32_t iters,
                      void* stream, double* gbps);
int kcache_probe_copy(kc_ctx* ctx, void* dst, const void* src, size_t bytes, int32_t iters,
                      void* stream, double* gbps);

const char* kcache_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KCACHE_H_ */
