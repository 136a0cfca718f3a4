// Host side of libkcache: argument validation, workspace, streams and events,
// the pipelining of K scan against V pull, and the C ABI of include/kcache.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <functional>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/kcache.h"
#include "kc_internal.h"

// ---- scratch of the entry point that allocates nothing (kcache_decode_attention_static).
// The array lives in the code object: every GPU the library runs on holds its own copy, at
// its own address, until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress, never an address: the device address is looked up once per
// device (static_scratch_for, called from kcache_create) and passed to the kernels like any
// other workspace.
constexpr size_t kStaticWorkBytes = (size_t)48 << 20;  // candidates, partials, positions, weights
constexpr size_t kStaticTickets = 16384;               // arrival counters, one int per KV unit
constexpr size_t kStaticScratchBytes = kStaticWorkBytes + kStaticTickets * sizeof(int);
static __device__ __align__(256) unsigned char kc_static_scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_create_error;

// Minimal persistent worker pool for the staged gather (host threads pack the
// selected V rows into one pinned buffer).
class Pool {
 public:
  explicit Pool(int n) {
    for (int i = 0; i < n; ++i) workers_.emplace_back([this] { run(); });
  }
  ~Pool() {
    {
      std::lock_guard<std::mutex> g(mu_);
      stop_ = true;
    }
    cv_.notify_all();
    for (auto& t : workers_) t.join();
  }
  int size() const { return (int)workers_.size(); }
  // Calls fn(i) for i in [0, n), spread over the workers and the caller.
  void parallel_for(int64_t n, const std::function<void(int64_t)>& fn) {
    if (n <= 0) return;
    {
      std::lock_guard<std::mutex> g(mu_);
      fn_ = &fn;
      next_.store(0);
      total_ = n;
      active_ = (int)workers_.size();
      ++epoch_;
    }
    cv_.notify_all();
    drain();
    std::unique_lock<std::mutex> l(mu_);
    done_cv_.wait(l, [this] { return active_ == 0; });
    fn_ = nullptr;
  }

 private:
  void drain() {
    for (;;) {
      int64_t i = next_.fetch_add(1);
      if (i >= total_) break;
      (*fn_)(i);
    }
  }
  void run() {
    uint64_t seen = 0;
    for (;;) {
      {
        std::unique_lock<std::mutex> l(mu_);
        cv_.wait(l, [&] { return stop_ || epoch_ != seen; });
        if (stop_) return;
        seen = epoch_;
      }
      drain();
      {
        std::lock_guard<std::mutex> g(mu_);
        if (--active_ == 0) done_cv_.notify_all();
      }
    }
  }
  std::vector<std::thread> workers_;
  std::mutex mu_;
  std::condition_variable cv_, done_cv_;
  const std::function<void(int64_t)>* fn_ = nullptr;
  std::atomic<int64_t> next_{0};
  int64_t total_ = 0;
  int active_ = 0;
  uint64_t epoch_ = 0;
  bool stop_ = false;
};

struct ProfRec {
  int kernel;
  hipEvent_t a, b;
};

constexpr int kMaxParts = 64;
constexpr int kMaxLanes = 4;
constexpr int kPosSlots = 8;     // stores with host-side positions that may be in flight at once
constexpr int kPosInts = 1024;   // sequences per such store

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices] = {};

// Device address of this device's copy of the scratch array.  `device` must be current.
hipError_t static_scratch_for(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> g(g_static_mu);
  if (!g_static_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(kc_static_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ptr[device] = p;
  }
  *out = g_static_ptr[device];
  return hipSuccess;
}

// Holds a lane back for `ticks` of the constant 100 MHz clock (see enqueue_step).  Bounded
// twice over: by the clock, and by an iteration cap that ends the loop even if the clock
// were to stand still.
__global__ __launch_bounds__(64) void stagger_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  for (int i = 0; i < (1 << 20) && (long long)wall_clock64() - t0 < ticks; ++i)
    __builtin_amdgcn_s_sleep(64);
}

// Writes up to 64 ints, handed over by value, to device memory: positions that the caller
// holds on the host reach the store kernel without a staging buffer whose reuse would have to
// be guarded.
struct IntPack {
  int32_t v[64];
};
__global__ __launch_bounds__(64) void set_ints_kernel(int32_t* dst, IntPack vals, int n) {
  if ((int)threadIdx.x < n) dst[threadIdx.x] = vals.v[threadIdx.x];
}

// Clears n ints.  A kernel, not hipMemsetAsync: memset nodes recorded into a captured graph
// have replayed wrongly on this platform.
__global__ __launch_bounds__(256) void zero_ints_kernel(int* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace

struct kc_ctx {
  int device = 0;
  hipStream_t side = nullptr;        // select + V pull of a part, while the next part is scanned
  hipStream_t store_side = nullptr;  // V half of the cache store
  hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_store = nullptr, ev_last = nullptr;
  hipEvent_t ev_part[kMaxParts] = {};
  bool store_pending = false, have_last = false;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  int* flags = nullptr;  // [0] device-check bits, [16] probe sink
  void* static_scratch = nullptr;  // this device's copy of kc_static_scratch
  int32_t* d_pos = nullptr;        // kPosSlots x kPosInts: positions of kcache_prefill_store_at
  int pos_slot = 0;
  std::string err;
  int parts = 0, profile = 0, staged_threads = 8, fused = 1, fused_rows = 0, step_lanes = 0,
      renorm = 0, step_split = 1, gqa_dedup = 0;
  int lane_stagger_us = -1;   // start of lane i is held back by i / lanes of this; 0 = no
                              // stagger, -1 = derived from the shape (see plan_step)
  int host_store_blocks = 0;  // workgroups of a V store to host memory; 0 = the kernel's default
  int xcd_spread = 0;      // test option: chunks of a unit dealt over all XCDs
  int auto_grow = 0;       // 1: a call may (re)allocate its scratch, synchronising the device
  bool reserving = false;  // inside kcache_create / kcache_reserve: growth is the point
  int64_t reallocs = 0;    // (re)allocations of workspace, tickets or staging since creation
  int graphs = 0;          // live step graphs: they hold addresses inside ws / counters
  bool capturing = false;  // a step is being captured into a graph: no profiling events
  hipStream_t lane[kMaxLanes] = {};  // streams of kcache_decode_step with more than one lane
  hipEvent_t ev_lane[kMaxLanes] = {};
  int* counters = nullptr;  // per KV unit arrival tickets of the fused kernel, zero when idle
  size_t counters_n = 0;
  std::vector<ProfRec> pending;
  std::vector<hipEvent_t> free_events;
  double prof_ms[KC_KERNEL_COUNT] = {};
  int64_t prof_n[KC_KERNEL_COUNT] = {};
  // staged gather
  Pool* pool = nullptr;
  int32_t* h_idx = nullptr;
  void* h_rows = nullptr;
  void* d_rows = nullptr;
  size_t staged_rows = 0;
};

namespace {

int fail(kc_ctx* c, int status, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c)
    c->err = buf;
  else
    g_create_error = buf;
  return status;
}

#define KC_HIP(c, call)                                                                    \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess)                                                                  \
      return fail((c), KC_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));         \
  } while (0)

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != dev) ok = hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

bool sizes_ok(int64_t B, int64_t H, int64_t S_cap, int64_t N) {
  return B >= 1 && H >= 1 && S_cap >= 1 && N >= 1 && B * H < (1ll << 31) &&
         B * H * S_cap < (1ll << 40) && B * H * N < (1ll << 36);
}

hipEvent_t get_event(kc_ctx* c) {
  if (!c->free_events.empty()) {
    hipEvent_t e = c->free_events.back();
    c->free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Brackets one kernel launch with events while profiling is on.
struct KernelTimer {
  kc_ctx* c;
  int id;
  hipStream_t st;
  hipEvent_t a = nullptr;
  KernelTimer(kc_ctx* c_, int id_, hipStream_t st_) : c(c_), id(id_), st(st_) {
    if (c->profile && !c->capturing && (a = get_event(c))) (void)hipEventRecord(a, st);
  }
  ~KernelTimer() {
    if (!a) return;
    hipEvent_t b = get_event(c);
    if (!b) {
      c->free_events.push_back(a);
      return;
    }
    (void)hipEventRecord(b, st);
    c->pending.push_back({id, a, b});
  }
};

int collect_profile(kc_ctx* c) {
  for (auto& r : c->pending) {
    float ms = 0.f;
    KC_HIP(c, hipEventSynchronize(r.b));
    KC_HIP(c, hipEventElapsedTime(&ms, r.a, r.b));
    c->prof_ms[r.kernel] += ms;
    c->prof_n[r.kernel] += 1;
    c->free_events.push_back(r.a);
    c->free_events.push_back(r.b);
  }
  c->pending.clear();
  return KC_OK;
}

// Growing a buffer frees the old one, which needs the device idle: that is allowed inside
// kcache_create / kcache_reserve, and inside the hot calls only with KC_OPT_AUTO_GROW.
int may_grow(kc_ctx* c, const char* what, size_t need, size_t have) {
  if (c->reserving || c->auto_grow) return KC_OK;
  return fail(c, KC_ERR_WORKSPACE, "%s: this call needs %zu, the context holds %zu.  Size the "
              "context first with kcache_reserve (or a workspace hint at kcache_create), or set "
              "KC_OPT_AUTO_GROW to let calls grow it, which synchronises the device", what, need,
              have);
}

int ensure_workspace(kc_ctx* c, size_t bytes) {
  if (bytes <= c->ws_bytes) return KC_OK;
  if (c->graphs > 0)
    return fail(c, KC_ERR_WORKSPACE, "the workspace would have to grow to %zu bytes while %d step "
                "graph(s) hold addresses inside it: destroy them first, or create the context "
                "with a larger workspace hint", bytes, c->graphs);
  int rc = may_grow(c, "workspace bytes", bytes, c->ws_bytes);
  if (rc != KC_OK) return rc;
  c->reallocs += 1;
  KC_HIP(c, hipDeviceSynchronize());
  if (c->ws) (void)hipFree(c->ws);
  c->ws = nullptr;
  c->ws_bytes = 0;
  hipError_t e = hipMalloc(&c->ws, bytes);
  if (e != hipSuccess)
    return fail(c, KC_ERR_WORKSPACE, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
  c->ws_bytes = bytes;
  return KC_OK;
}

int ensure_lanes(kc_ctx* c, int lanes) {  // stream / event creation does not synchronise
  for (int i = 0; i < lanes; ++i) {
    if (!c->lane[i]) KC_HIP(c, hipStreamCreateWithFlags(&c->lane[i], hipStreamNonBlocking));
    if (!c->ev_lane[i]) KC_HIP(c, hipEventCreateWithFlags(&c->ev_lane[i], hipEventDisableTiming));
  }
  return KC_OK;
}

int ensure_counters(kc_ctx* c, size_t n) {
  if (n <= c->counters_n) return KC_OK;
  if (c->graphs > 0)
    return fail(c, KC_ERR_WORKSPACE, "the ticket counters would have to grow while %d step "
                "graph(s) hold their address: destroy them first", c->graphs);
  int rc = may_grow(c, "arrival tickets", n, c->counters_n);
  if (rc != KC_OK) return rc;
  c->reallocs += 1;
  KC_HIP(c, hipDeviceSynchronize());
  if (c->counters) (void)hipFree(c->counters);
  c->counters = nullptr;
  c->counters_n = 0;
  hipError_t e = hipMalloc((void**)&c->counters, n * sizeof(int));
  if (e != hipSuccess)
    return fail(c, KC_ERR_WORKSPACE, "ticket counters for %zu units: %s", n, hipGetErrorString(e));
  KC_HIP(c, hipMemset(c->counters, 0, n * sizeof(int)));
  c->counters_n = n;
  return KC_OK;
}

// Workspace of the unfused path: fp32 scores [units][S_cap], positions and weights [units][N].
size_t unfused_bytes(size_t units, size_t S_cap, size_t N) {
  return round256(units * S_cap * sizeof(float)) + 2 * round256(units * N * sizeof(int32_t));
}

// Workspace of the fused path: chunk-local candidates (score + position), chunk
// partials, positions and weights.
size_t fused_bytes(size_t units, size_t chunks_cap, size_t kk, size_t N) {
  return 2 * round256(units * chunks_cap * kk * sizeof(float)) +
         round256(units * chunks_cap * sizeof(float2)) + round256(units * chunks_cap * sizeof(float)) +
         2 * round256(units * N * sizeof(int32_t));
}

int ensure_staged(kc_ctx* c, size_t rows) {
  if (!c->pool || c->pool->size() != std::max(0, c->staged_threads - 1)) {
    delete c->pool;
    c->pool = new Pool(std::max(0, c->staged_threads - 1));
  }
  if (rows <= c->staged_rows) return KC_OK;
  int rc = may_grow(c, "staging rows of the staged gather", rows, c->staged_rows);
  if (rc != KC_OK) return rc;
  c->reallocs += 1;
  KC_HIP(c, hipDeviceSynchronize());
  if (c->h_idx) (void)hipHostFree(c->h_idx);
  if (c->h_rows) (void)hipHostFree(c->h_rows);
  if (c->d_rows) (void)hipFree(c->d_rows);
  c->h_idx = nullptr;
  c->h_rows = c->d_rows = nullptr;
  c->staged_rows = 0;
  KC_HIP(c, hipHostMalloc((void**)&c->h_idx, rows * sizeof(int32_t), hipHostMallocDefault));
  KC_HIP(c, hipHostMalloc(&c->h_rows, rows * kc::kRowBytes, hipHostMallocDefault));
  hipError_t e = hipMalloc(&c->d_rows, rows * kc::kRowBytes);
  if (e != hipSuccess)
    return fail(c, KC_ERR_WORKSPACE, "staging of %zu rows: %s", rows, hipGetErrorString(e));
  c->staged_rows = rows;
  return KC_OK;
}

// Device-visible address of pinned, mapped host memory, or an error.
int mapped_host_pointer(kc_ctx* c, void* host, void** dev) {
  hipPointerAttribute_t attr;
  memset(&attr, 0, sizeof attr);
  hipError_t e = hipPointerGetAttributes(&attr, host);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, KC_ERR_NOT_PINNED, "v_host %p is not known to HIP (%s): it must be pinned, "
                "mapped host memory", host, hipGetErrorString(e));
  }
  if (attr.type != hipMemoryTypeHost)
    return fail(c, KC_ERR_NOT_PINNED, "v_host %p has memory type %d, expected pinned host memory",
                host, (int)attr.type);
  e = hipHostGetDevicePointer(dev, host, 0);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, KC_ERR_NOT_PINNED, "v_host %p is not mapped into the device: %s", host,
                hipGetErrorString(e));
  }
  return KC_OK;
}

// Device-visible address of a layer's V cache: the mapped host cache, or the
// device buffer of a layer that keeps V in HBM.
int v_pointer(kc_ctx* c, const kc_layer_cache* cache, void** dev) {
  if (!cache->v_in_hbm) return mapped_host_pointer(c, cache->v_host, dev);
  hipPointerAttribute_t attr;
  memset(&attr, 0, sizeof attr);
  hipError_t e = hipPointerGetAttributes(&attr, cache->v_host);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, KC_ERR_NOT_PINNED, "V cache %p is not known to HIP (%s): with v_in_hbm it must "
                "be device memory", cache->v_host, hipGetErrorString(e));
  }
  if (attr.type != hipMemoryTypeDevice)
    return fail(c, KC_ERR_NOT_PINNED, "V cache %p has memory type %d, expected device memory "
                "(v_in_hbm is set)", cache->v_host, (int)attr.type);
  *dev = cache->v_host;
  return KC_OK;
}

int shape_status(const kc_layer_cache* cache, int32_t H, int32_t N, const char** why) {
  *why = "";
  if (!cache) return *why = "cache is NULL", KC_ERR_INVALID_ARG;
  if (cache->B < 1 || cache->Hkv < 1 || cache->S_cap < 1)
    return *why = "B, Hkv and S_cap must be positive", KC_ERR_INVALID_ARG;
  if (cache->dtype != KC_F16 && cache->dtype != KC_BF16)
    return *why = "dtype must be KC_F16 or KC_BF16", KC_ERR_INVALID_ARG;
  if (cache->v_in_hbm != 0 && cache->v_in_hbm != 1)
    return *why = "v_in_hbm must be 0 or 1", KC_ERR_INVALID_ARG;
  if (cache->k_fp8 != 0 && cache->k_fp8 != 1)
    return *why = "k_fp8 must be 0 or 1", KC_ERR_INVALID_ARG;
  if (cache->k_fp8 && (cache->k_exp < -32 || cache->k_exp > 32))
    return *why = "k_exp must be in [-32, 32]", KC_ERR_INVALID_ARG;
  if (cache->d != 64 && cache->d != 128 && cache->d != 256)
    return *why = "head dimension must be 64, 128 or 256", KC_ERR_UNSUPPORTED;
  if (cache->k_fp8 && cache->d != kc::kHeadDim)
    return *why = "an 8-bit K cache needs head dimension 128", KC_ERR_UNSUPPORTED;
  if ((int64_t)cache->B * cache->Hkv * cache->S_cap >= (1ll << 40))
    return *why = "cache too large", KC_ERR_INVALID_ARG;
  if (H == 0) return KC_OK;
  if (H < 1 || N < 1) return *why = "H and N must be positive", KC_ERR_INVALID_ARG;
  if (H % cache->Hkv != 0) return *why = "H must be a multiple of Hkv", KC_ERR_INVALID_ARG;
  const int G = H / cache->Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16 && G != 32)
    return *why = "group size H/Hkv must be 1, 2, 4, 8, 16 or 32", KC_ERR_UNSUPPORTED;
  if (!sizes_ok(cache->B, H, cache->S_cap, N)) return *why = "sizes too large", KC_ERR_INVALID_ARG;
  return KC_OK;
}

int pick_parts(const kc_ctx* c, int kv_units, size_t k_bytes) {
  int p = c->parts;
  if (p <= 0) p = k_bytes >= ((size_t)256 << 20) ? 4 : 1;
  p = std::min(p, std::min(kv_units, kMaxParts));
  return std::max(p, 1);
}


// 1 / sqrt(d_h) for the supported head dimensions (exact constants, not a runtime sqrt).
float inv_sqrt_d(int d) { return d == 64 ? 0.125f : d == 256 ? 0.0625f : 0.08838834764831845f; }

// Sizes that a fused KCache launch of this shape needs.
struct FusedPlan {
  int R, chunks_cap, kk;
  size_t plan_items;  // ints of the launch plan (dense numbering of the chunks that exist), or 0
  size_t bytes;
};
// in_step: the launch is one of a whole step, where the launch plan is built once per lane
// and step; a single-layer call builds it every time (4-5 us), so it only takes one for
// batches of kPlanBatch sequences and more, where lengths that differ are to be expected.
constexpr int kPlanBatch = 32;
FusedPlan plan_fused(const kc_ctx* c, int B, int H, int Hkv, int S_cap, int N, int k_fp8, int d,
                     bool in_step = false) {
  const int split = kc::kv_split_for(H / Hkv), G = H / Hkv / split;  // per launch unit
  FusedPlan p;
  p.R = (c->fused_rows > 0 && c->fused_rows * G <= kc::kFusedZFloats)
            ? c->fused_rows
            : kc::fused_rows_per_block(B * Hkv * split, G, S_cap, N,
                                       k_fp8 ? d : 2 * d);
  p.chunks_cap = (S_cap + p.R - 1) / p.R;
  p.kk = std::min(N, p.R);
  p.plan_items = (c->xcd_spread || (!in_step && B < kPlanBatch))
                     ? 0
                     : kc::fused_plan_items(B, Hkv * split, p.chunks_cap);
  p.bytes = fused_bytes((size_t)B * H, p.chunks_cap, p.kk, N) +
            round256(p.plan_items * sizeof(int));
  return p;
}

// One fused KCache launch on `st` with its scratch carved out of `ws` and its tickets in
// `counters` (both exclusively this launch's until it has finished).
// `new_plan`: the launch plan in `ws` (if this shape takes one) is (re)built from the lengths
// first; false only when an earlier launch on `st` has built it in the same `ws` from the same
// lengths for the same shape (the layers of a step).
int enqueue_fused(kc_ctx* c, const kc_layer_cache* cache, const void* v_map, const void* q_dev,
                  int H, const int32_t* seq_lens_dev, int N, float* out_dev, int32_t* idx_out_dev,
                  float* w_out_dev, const FusedPlan& pl, void* ws, int* counters, hipStream_t st,
                  bool new_plan = true) {
  const int B = cache->B, Hkv = cache->Hkv, S_cap = cache->S_cap;
  const size_t units = (size_t)B * H;
  char* p = static_cast<char*>(ws);
  kc::FusedArgs a;
  a.q = static_cast<const uint16_t*>(q_dev);
  a.K = static_cast<const uint16_t*>(cache->k_dev);
  a.V = static_cast<const uint16_t*>(v_map);
  a.seq_lens = seq_lens_dev;
  a.out = out_dev;
  a.cand_z = reinterpret_cast<float*>(p);
  p += round256(units * pl.chunks_cap * pl.kk * sizeof(float));
  a.cand_pos = reinterpret_cast<int32_t*>(p);
  p += round256(units * pl.chunks_cap * pl.kk * sizeof(float));
  a.part = reinterpret_cast<float2*>(p);
  p += round256(units * pl.chunks_cap * sizeof(float2));
  a.bound = reinterpret_cast<float*>(p);
  p += round256(units * pl.chunks_cap * sizeof(float));
  a.idx = idx_out_dev ? idx_out_dev : reinterpret_cast<int32_t*>(p);
  p += round256(units * N * sizeof(int32_t));
  a.w = w_out_dev ? w_out_dev : reinterpret_cast<float*>(p);
  p += round256(units * N * sizeof(int32_t));
  a.plan = pl.plan_items ? reinterpret_cast<const int*>(p) : nullptr;
  a.counters = counters;
  a.flags = c->flags;
  a.kv_split = kc::kv_split_for(H / Hkv);
  a.H = H;
  a.Hkv = Hkv * a.kv_split;
  a.S_cap = S_cap;
  a.N = N;
  a.R = pl.R;
  a.chunks_cap = pl.chunks_cap;
  a.kk = pl.kk;
  a.kv0 = 0;
  a.kv_count = B * a.Hkv;
  a.renorm = c->renorm;
  a.k_fp8 = cache->k_fp8;
  a.d = cache->d;
  a.dedup = c->gqa_dedup;
  a.spread = c->xcd_spread;
  // 1 / sqrt(d_h), times the cache's 2^k_exp for an 8-bit K cache
  a.scale = ldexpf(inv_sqrt_d(cache->d), cache->k_fp8 ? cache->k_exp : 0);
  KernelTimer t(c, KC_KERNEL_FUSED, st);  // the plan, when one is built, is part of the launch's cost
  if (a.plan && new_plan)
    KC_HIP(c, kc::launch_fused_plan(seq_lens_dev, B, a.Hkv, S_cap, pl.R, const_cast<int*>(a.plan),
                                    st));
  KC_HIP(c, kc::launch_fused(a, cache->dtype, a.kv_count, st));
  return KC_OK;
}

struct FullPlan {
  int R, chunks_cap;
  size_t part_bytes, bytes;
};
FullPlan plan_full(const kc_ctx* c, int B, int H, int Hkv, int S_cap, int d = kc::kHeadDim) {
  const int split = kc::kv_split_for(H / Hkv), G = H / Hkv / split;  // per launch unit
  FullPlan p;
  p.R = (c->fused_rows > 0 && c->fused_rows * G <= kc::kFusedZFloats)
            ? c->fused_rows
            : kc::full_rows_per_block(B * Hkv * split, G, S_cap, 2 * d);
  p.chunks_cap = (S_cap + p.R - 1) / p.R;
  const size_t units = (size_t)B * H;
  p.part_bytes = round256(units * p.chunks_cap * sizeof(float2));
  p.bytes = p.part_bytes + round256(units * p.chunks_cap * d * sizeof(float));
  return p;
}

int enqueue_full(kc_ctx* c, const kc_layer_cache* cache, const void* v_map, const void* q_dev,
                 int H, const int32_t* seq_lens_dev, float* out_dev, const FullPlan& pl, void* ws,
                 int* counters, hipStream_t st) {
  kc::FullArgs a;
  a.q = static_cast<const uint16_t*>(q_dev);
  a.K = static_cast<const uint16_t*>(cache->k_dev);
  a.V = static_cast<const uint16_t*>(v_map);
  a.seq_lens = seq_lens_dev;
  a.out = out_dev;
  a.part = reinterpret_cast<float2*>(ws);
  a.part_o = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.part_bytes);
  a.counters = counters;
  a.flags = c->flags;
  a.kv_split = kc::kv_split_for(H / cache->Hkv);
  a.H = H;
  a.Hkv = cache->Hkv * a.kv_split;
  a.S_cap = cache->S_cap;
  a.R = pl.R;
  a.chunks_cap = pl.chunks_cap;
  a.kv_count = cache->B * a.Hkv;
  a.d = cache->d;
  a.spread = c->xcd_spread;
  a.scale = inv_sqrt_d(cache->d);
  KernelTimer t(c, KC_KERNEL_FULL, st);
  KC_HIP(c, kc::launch_full(a, cache->dtype, st));
  return KC_OK;
}

}  // namespace

extern "C" {

const char* kcache_version(void) { return "kcache-gfx950 0.1"; }

size_t kcache_workspace_bytes(int32_t B, int32_t H, int32_t S_cap, int32_t N) {
  if (!sizes_ok(B, H, S_cap, N)) return 0;
  const size_t units = (size_t)B * H;
  // the fused path never keeps more than min(N, R) candidates per R >= 512 positions
  const size_t chunks = ((size_t)S_cap + kc::kFusedThreads - 1) / kc::kFusedThreads;
  const size_t kk = std::min<size_t>(N, kc::kFusedThreads);
  return std::max(unfused_bytes(units, S_cap, N), fused_bytes(units, chunks, kk, N));
}

int kcache_check_shapes(const kc_layer_cache* cache, int32_t H, int32_t N) {
  const char* why;
  return shape_status(cache, H, N, &why);
}

int kcache_create(kc_ctx** out, int device, size_t workspace_bytes_hint) {
  if (!out) return fail(nullptr, KC_ERR_INVALID_ARG, "out is NULL");
  int count = 0;
  hipError_t e = hipGetDeviceCount(&count);
  if (e != hipSuccess || count < 1) {
    (void)hipGetLastError();
    return fail(nullptr, KC_ERR_HIP, "no HIP device available (%s)",
                e == hipSuccess ? "device count is 0" : hipGetErrorString(e));
  }
  if (device < 0 || device >= count)
    return fail(nullptr, KC_ERR_INVALID_ARG, "device %d outside [0, %d)", device, count);
  DeviceGuard g(device);
  if (!g.ok) return fail(nullptr, KC_ERR_HIP, "hipSetDevice(%d) failed", device);
  kc_ctx* c = new kc_ctx();
  c->device = device;
  auto bail = [&](const char* what, hipError_t err) {
    std::string msg = std::string(what) + ": " + hipGetErrorString(err);
    kcache_destroy(c);
    return fail(nullptr, KC_ERR_HIP, "%s", msg.c_str());
  };
  if ((e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking)) != hipSuccess)
    return bail("hipStreamCreate", e);
  if ((e = hipStreamCreateWithFlags(&c->store_side, hipStreamNonBlocking)) != hipSuccess)
    return bail("hipStreamCreate", e);
  hipEvent_t* evs[] = {&c->ev_fork, &c->ev_join, &c->ev_store, &c->ev_last};
  for (auto* ev : evs)
    if ((e = hipEventCreateWithFlags(ev, hipEventDisableTiming)) != hipSuccess)
      return bail("hipEventCreate", e);
  for (int i = 0; i < kMaxParts; ++i)
    if ((e = hipEventCreateWithFlags(&c->ev_part[i], hipEventDisableTiming)) != hipSuccess)
      return bail("hipEventCreate", e);
  if ((e = hipMalloc((void**)&c->flags, 256)) != hipSuccess) return bail("hipMalloc", e);
  if ((e = hipMemset(c->flags, 0, 256)) != hipSuccess) return bail("hipMemset", e);
  if ((e = static_scratch_for(device, &c->static_scratch)) != hipSuccess)
    return bail("hipGetSymbolAddress(static scratch)", e);
  if ((e = hipMalloc((void**)&c->d_pos, kPosSlots * kPosInts * sizeof(int32_t))) != hipSuccess)
    return bail("hipMalloc", e);
  if (workspace_bytes_hint) {
    c->reserving = true;
    int rc = ensure_workspace(c, workspace_bytes_hint);
    c->reserving = false;
    if (rc != KC_OK) {
      std::string msg = c->err;
      kcache_destroy(c);
      return fail(nullptr, rc, "%s", msg.c_str());
    }
  }
  *out = c;
  return KC_OK;
}

int kcache_destroy(kc_ctx* c) {
  if (!c) return KC_OK;
  DeviceGuard g(c->device);
  (void)hipDeviceSynchronize();
#ifdef KC_TIMING
  {
    unsigned long long d[9] = {};
    (void)hipMemcpy(d, c->flags + 32, sizeof d, hipMemcpyDeviceToHost);
    const double n = d[7] ? (double)d[7] : 1.0, f = d[8] ? (double)d[8] : 1.0;
    fprintf(stderr, "KC_TIMING us per workgroup (100 MHz clock): scan %.2f stats %.2f topn %.2f handover %.2f | "
            "per finisher head: load+merge %.2f topn %.2f pull %.2f (workgroups %llu, finisher heads %llu)\n",
            d[0] / n / 100., d[1] / n / 100., d[2] / n / 100., d[3] / n / 100., d[4] / f / 100., d[5] / f / 100.,
            d[6] / f / 100., d[7], d[8]);
  }
#endif
  delete c->pool;
  for (auto& r : c->pending) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  for (auto e : c->free_events) (void)hipEventDestroy(e);
  hipEvent_t evs[] = {c->ev_fork, c->ev_join, c->ev_store, c->ev_last};
  for (auto e : evs)
    if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_part)
    if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_lane)
    if (e) (void)hipEventDestroy(e);
  for (auto st : c->lane)
    if (st) (void)hipStreamDestroy(st);
  if (c->side) (void)hipStreamDestroy(c->side);
  if (c->store_side) (void)hipStreamDestroy(c->store_side);
  if (c->ws) (void)hipFree(c->ws);
  if (c->flags) (void)hipFree(c->flags);
  if (c->d_pos) (void)hipFree(c->d_pos);
  if (c->counters) (void)hipFree(c->counters);
  if (c->h_idx) (void)hipHostFree(c->h_idx);
  if (c->h_rows) (void)hipHostFree(c->h_rows);
  if (c->d_rows) (void)hipFree(c->d_rows);
  delete c;
  return KC_OK;
}

const char* kcache_last_error(kc_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int kcache_set_option(kc_ctx* c, int32_t option, int64_t value) {
  if (!c) return KC_ERR_INVALID_ARG;
  switch (option) {
    case KC_OPT_PIPELINE_PARTS:
      if (value < 0 || value > kMaxParts)
        return fail(c, KC_ERR_INVALID_ARG, "pipeline parts must be in [0, %d]", kMaxParts);
      c->parts = (int)value;
      return KC_OK;
    case KC_OPT_PROFILE:
      c->profile = value != 0;
      return KC_OK;
    case KC_OPT_FUSED:
      c->fused = value != 0;
      return KC_OK;
    case KC_OPT_GQA_DEDUP:
      c->gqa_dedup = value != 0;
      return KC_OK;
    case KC_OPT_STEP_SPLIT:
      if (value != 0 && value != 1)
        return fail(c, KC_ERR_INVALID_ARG, "step split must be 0 (layers) or 1 (sequences)");
      c->step_split = (int)value;
      return KC_OK;
    case KC_OPT_RENORMALIZE:
      c->renorm = value != 0;
      return KC_OK;
    case KC_OPT_STEP_LANES:
      if (value < 0 || value > kMaxLanes)
        return fail(c, KC_ERR_INVALID_ARG, "step lanes must be in [0, %d]", kMaxLanes);
      c->step_lanes = (int)value;
      return KC_OK;
    case KC_OPT_AUTO_GROW:
      c->auto_grow = value != 0;
      return KC_OK;
    case KC_OPT_LANE_STAGGER_US:
      if (value < -1 || value > 100000)
        return fail(c, KC_ERR_INVALID_ARG, "lane stagger must be -1 or in [0, 100000] microseconds");
      c->lane_stagger_us = (int)value;
      return KC_OK;
    case KC_OPT_HOST_STORE_BLOCKS:
      if (value < 0 || value > 4096)
        return fail(c, KC_ERR_INVALID_ARG, "host store workgroups must be in [0, 4096]");
      c->host_store_blocks = (int)value;
      return KC_OK;
    case KC_OPT_XCD_SPREAD:
      c->xcd_spread = value != 0;
      return KC_OK;
    case KC_OPT_FUSED_ROWS:
      if (value < 0 || value > kc::kFusedZFloats || value % kc::kFusedThreads != 0)
        return fail(c, KC_ERR_INVALID_ARG, "fused rows must be 0 or a multiple of %d up to %d",
                    kc::kFusedThreads, kc::kFusedZFloats);
      c->fused_rows = (int)value;
      return KC_OK;
    case KC_OPT_STAGED_THREADS:
      if (value < 1 || value > 256)
        return fail(c, KC_ERR_INVALID_ARG, "staged threads must be in [1, 256]");
      c->staged_threads = (int)value;
      return KC_OK;
    default:
      return fail(c, KC_ERR_INVALID_ARG, "unknown option %d", option);
  }
}

int kcache_prefill_store(kc_ctx* c, const kc_layer_cache* cache, const void* k_new_dev,
                         const void* v_new_dev, const int32_t* pos_dev, int32_t T, void* stream,
                         void* done_event) {
  if (!c) return KC_ERR_INVALID_ARG;
  const char* why;
  int rc = shape_status(cache, 0, 0, &why);
  if (rc != KC_OK) return fail(c, rc, "kcache_prefill_store: %s", why);
  if (!cache->k_dev || !cache->v_host || !k_new_dev || !v_new_dev || !pos_dev)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_prefill_store: NULL pointer argument");
  if (T < 1 || T > cache->S_cap)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_prefill_store: T = %d outside [1, S_cap = %d]", T,
                cache->S_cap);
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  void* v_map = nullptr;
  if ((rc = v_pointer(c, cache, &v_map)) != KC_OK) return rc;

  hipStream_t st = (hipStream_t)stream;
  const kc::Shape sh{cache->B, 0, cache->Hkv, cache->S_cap, 0, cache->dtype, 0, cache->d};
  if (cache->v_in_hbm) {
    // both caches in HBM: one launch over the whole grid on the caller's stream
    {
      KernelTimer t(c, KC_KERNEL_STORE_K, st);
      KC_HIP(c, kc::launch_store(sh, k_new_dev, cache->k_dev, v_new_dev, v_map, pos_dev, T,
                                 c->flags, 0, st, cache->k_fp8, cache->k_exp));
    }
    if (done_event) KC_HIP(c, hipEventRecord((hipEvent_t)done_event, st));
    return KC_OK;
  }
  if ((int64_t)cache->B * T * cache->Hkv <= 4096) {
    // a decode-step append: K and V rows in one small launch on the caller's stream
    // (too little data to be worth a second stream and two event waits)
    {
      KernelTimer t(c, KC_KERNEL_STORE_K, st);
      KC_HIP(c, kc::launch_store(sh, k_new_dev, cache->k_dev, v_new_dev, v_map, pos_dev, T,
                                 c->flags, 1, st, cache->k_fp8, cache->k_exp));
    }
    if (done_event) KC_HIP(c, hipEventRecord((hipEvent_t)done_event, st));
    return KC_OK;
  }
  // V first: the side stream starts as soon as the inputs are ready on `st`
  KC_HIP(c, hipEventRecord(c->ev_fork, st));
  KC_HIP(c, hipStreamWaitEvent(c->store_side, c->ev_fork, 0));
  {
    KernelTimer t(c, KC_KERNEL_STORE_V, c->store_side);
    KC_HIP(c, kc::launch_store(sh, v_new_dev, v_map, nullptr, nullptr, pos_dev, T, c->flags,
                               c->host_store_blocks > 1 ? c->host_store_blocks : 1, c->store_side));
  }
  KC_HIP(c, hipEventRecord(c->ev_store, c->store_side));
  c->store_pending = true;
  if (done_event) KC_HIP(c, hipEventRecord((hipEvent_t)done_event, c->store_side));
  {
    KernelTimer t(c, KC_KERNEL_STORE_K, st);
    KC_HIP(c, kc::launch_store(sh, k_new_dev, cache->k_dev, nullptr, nullptr, pos_dev, T,
                               c->flags, 0, st, cache->k_fp8, cache->k_exp));
  }
  return KC_OK;
}

int kcache_prefill_store_at(kc_ctx* c, const kc_layer_cache* cache, const void* k_new_dev,
                            const void* v_new_dev, const int32_t* pos_host, int32_t T,
                            void* stream, void* done_event) {
  if (!c) return KC_ERR_INVALID_ARG;
  const char* why;
  int rc = shape_status(cache, 0, 0, &why);
  if (rc != KC_OK) return fail(c, rc, "kcache_prefill_store_at: %s", why);
  if (!cache->k_dev || !cache->v_host || !k_new_dev || !v_new_dev || !pos_host)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_prefill_store_at: NULL pointer argument");
  if (T < 1 || T > cache->S_cap)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_prefill_store_at: T = %d outside [1, S_cap = %d]",
                T, cache->S_cap);
  const int B = cache->B, Hkv = cache->Hkv;
  if (B > kPosInts)
    return fail(c, KC_ERR_UNSUPPORTED, "kcache_prefill_store_at: at most %d sequences per call",
                kPosInts);
  for (int b = 0; b < B; ++b)
    if (pos_host[b] < 0 || (int64_t)pos_host[b] + T > cache->S_cap)
      return fail(c, KC_ERR_INVALID_ARG, "kcache_prefill_store_at: sequence %d: rows [%d, %d) do "
                  "not fit the capacity %d", b, pos_host[b], pos_host[b] + T, cache->S_cap);
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  void* v_map = nullptr;
  if ((rc = v_pointer(c, cache, &v_map)) != KC_OK) return rc;

  hipStream_t st = (hipStream_t)stream;
  // the positions, for the kernel that stores K (and V, where a kernel stores it)
  int32_t* pos_dev = c->d_pos + (size_t)c->pos_slot * kPosInts;
  c->pos_slot = (c->pos_slot + 1) % kPosSlots;
  for (int b0 = 0; b0 < B; b0 += 64) {
    IntPack pack;
    const int n = std::min(64, B - b0);
    for (int i = 0; i < 64; ++i) pack.v[i] = i < n ? pos_host[b0 + i] : 0;
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, st, pos_dev + b0, pack, n);
    KC_HIP(c, hipGetLastError());
  }
  const kc::Shape sh{B, 0, Hkv, cache->S_cap, 0, cache->dtype, 0, cache->d};
  const bool small = (int64_t)B * T * Hkv <= 4096;
  if (cache->v_in_hbm || small) {  // as kcache_prefill_store: one launch for both halves
    {
      KernelTimer t(c, KC_KERNEL_STORE_K, st);
      KC_HIP(c, kc::launch_store(sh, k_new_dev, cache->k_dev, v_new_dev, v_map, pos_dev, T,
                                 c->flags, cache->v_in_hbm ? 0 : 1, st, cache->k_fp8,
                                 cache->k_exp));
    }
    if (done_event) KC_HIP(c, hipEventRecord((hipEvent_t)done_event, st));
    return KC_OK;
  }
  // V half: the copy engine moves the rows of every (sequence, KV head), T rows of one head
  // out of the token-major source (pitch Hkv rows) into a dense run of the host cache
  KC_HIP(c, hipEventRecord(c->ev_fork, st));
  KC_HIP(c, hipStreamWaitEvent(c->store_side, c->ev_fork, 0));
  {
    KernelTimer t(c, KC_KERNEL_STORE_V, c->store_side);
    const size_t row = (size_t)cache->d * 2;
    for (int b = 0; b < B; ++b)
      for (int hk = 0; hk < Hkv; ++hk) {
        char* dst = static_cast<char*>(cache->v_host) +
                    (((size_t)b * Hkv + hk) * cache->S_cap + (size_t)pos_host[b]) * row;
        const char* src = static_cast<const char*>(v_new_dev) + ((size_t)b * T * Hkv + hk) * row;
        KC_HIP(c, hipMemcpy2DAsync(dst, row, src, (size_t)Hkv * row, row, (size_t)T,
                                   hipMemcpyDeviceToHost, c->store_side));
      }
  }
  KC_HIP(c, hipEventRecord(c->ev_store, c->store_side));
  c->store_pending = true;
  if (done_event) KC_HIP(c, hipEventRecord((hipEvent_t)done_event, c->store_side));
  {
    KernelTimer t(c, KC_KERNEL_STORE_K, st);
    KC_HIP(c, kc::launch_store(sh, k_new_dev, cache->k_dev, nullptr, nullptr, pos_dev, T,
                               c->flags, 0, st, cache->k_fp8, cache->k_exp));
  }
  return KC_OK;
}

int kcache_decode_attention(kc_ctx* c, const kc_layer_cache* cache, const void* q_dev, int32_t H,
                            const int32_t* seq_lens_dev, int32_t N, float* out_dev,
                            int32_t* idx_out_dev, float* w_out_dev, int32_t gather_mode,
                            void* stream) {
  if (!c) return KC_ERR_INVALID_ARG;
  const char* why;
  int rc = shape_status(cache, H == 0 ? -1 : H, N, &why);
  if (rc != KC_OK) return fail(c, rc, "kcache_decode_attention: %s", why);
  if (!cache->k_dev || !cache->v_host || !q_dev || !seq_lens_dev || !out_dev)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_decode_attention: NULL pointer argument");
  if (gather_mode != KC_GATHER_ZEROCOPY && gather_mode != KC_GATHER_STAGED)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_decode_attention: unknown gather mode %d",
                gather_mode);
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  if ((cache->k_fp8 || cache->d != kc::kHeadDim) &&
      (gather_mode == KC_GATHER_STAGED || !c->fused))
    return fail(c, KC_ERR_UNSUPPORTED, "kcache_decode_attention: 8-bit K caches and head "
                "dimensions other than 128 are served by the fused zero-copy path only");
  if (cache->v_in_hbm && gather_mode == KC_GATHER_STAGED)
    return fail(c, KC_ERR_UNSUPPORTED, "kcache_decode_attention: the staged gather needs the V "
                "cache in host memory");
  void* v_map = nullptr;
  if ((rc = v_pointer(c, cache, &v_map)) != KC_OK) return rc;

  const int B = cache->B, Hkv = cache->Hkv, S_cap = cache->S_cap, G = H / Hkv;
  const size_t units = (size_t)B * H;
  const int kv_units = B * Hkv;
  const bool staged = gather_mode == KC_GATHER_STAGED;
  const bool fused = !staged && c->fused;
  const FusedPlan pl = plan_fused(c, B, H, Hkv, S_cap, N, cache->k_fp8, cache->d);
  const size_t need = fused ? pl.bytes : unfused_bytes(units, S_cap, N);
  if ((rc = ensure_workspace(c, need)) != KC_OK) return rc;
  if (staged && (rc = ensure_staged(c, units * N)) != KC_OK) return rc;
  if (fused && (rc = ensure_counters(c, (size_t)kv_units * kc::kv_split_for(G))) != KC_OK)
    return rc;

  hipStream_t st = (hipStream_t)stream;
  const kc::Shape sh{B, H, Hkv, S_cap, N, cache->dtype, c->renorm};
  const int parts = pick_parts(c, kv_units, (size_t)kv_units * S_cap * kc::kRowBytes);

  // the workspace and the V rows must be free of earlier work of this context
  if (c->have_last) KC_HIP(c, hipStreamWaitEvent(st, c->ev_last, 0));
  if (c->store_pending) {
    KC_HIP(c, hipStreamWaitEvent(st, c->ev_store, 0));
    c->store_pending = false;
  }

  if (fused) {
    if ((rc = enqueue_fused(c, cache, v_map, q_dev, H, seq_lens_dev, N, out_dev, idx_out_dev,
                            w_out_dev, pl, c->ws, c->counters, st)) != KC_OK)
      return rc;
    KC_HIP(c, hipEventRecord(c->ev_last, st));
    c->have_last = true;
    return KC_OK;
  }

  char* wsp = static_cast<char*>(c->ws);
  float* z = reinterpret_cast<float*>(wsp);
  wsp += round256(units * S_cap * sizeof(float));
  int32_t* idx = idx_out_dev ? idx_out_dev : reinterpret_cast<int32_t*>(wsp);
  wsp += round256(units * N * sizeof(int32_t));
  float* w = w_out_dev ? w_out_dev : reinterpret_cast<float*>(wsp);

  auto part_range = [&](int p, int* kv0, int* cnt) {
    *kv0 = (int)((int64_t)kv_units * p / parts);
    *cnt = (int)((int64_t)kv_units * (p + 1) / parts) - *kv0;
  };

  if (!staged) {
    const bool overlap = parts > 1;
    hipStream_t tail = overlap ? c->side : st;
    if (overlap) {
      KC_HIP(c, hipEventRecord(c->ev_fork, st));
      KC_HIP(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
    }
    for (int p = 0; p < parts; ++p) {
      int kv0, cnt;
      part_range(p, &kv0, &cnt);
      {
        KernelTimer t(c, KC_KERNEL_KSCAN, st);
        KC_HIP(c, kc::launch_kscan(sh, q_dev, cache->k_dev, seq_lens_dev, z, kv0, cnt, c->flags,
                                   st));
      }
      if (overlap) {
        KC_HIP(c, hipEventRecord(c->ev_part[p], st));
        KC_HIP(c, hipStreamWaitEvent(c->side, c->ev_part[p], 0));
      }
      {
        KernelTimer t(c, KC_KERNEL_SELECT, tail);
        KC_HIP(c, kc::launch_select(sh, z, seq_lens_dev, idx, w, kv0 * G, cnt * G, tail));
      }
      {
        KernelTimer t(c, KC_KERNEL_GATHER, tail);
        KC_HIP(c, kc::launch_gather(sh, v_map, idx, w, out_dev, kv0 * G, cnt * G, 0, tail));
      }
    }
    if (overlap) {
      KC_HIP(c, hipEventRecord(c->ev_join, c->side));
      KC_HIP(c, hipStreamWaitEvent(st, c->ev_join, 0));
    }
  } else {
    // All scans and selects are enqueued up front; the host then packs part p
    // while the GPU is still scanning the later parts.
    for (int p = 0; p < parts; ++p) {
      int kv0, cnt;
      part_range(p, &kv0, &cnt);
      {
        KernelTimer t(c, KC_KERNEL_KSCAN, st);
        KC_HIP(c, kc::launch_kscan(sh, q_dev, cache->k_dev, seq_lens_dev, z, kv0, cnt, c->flags,
                                   st));
      }
      {
        KernelTimer t(c, KC_KERNEL_SELECT, st);
        KC_HIP(c, kc::launch_select(sh, z, seq_lens_dev, idx, w, kv0 * G, cnt * G, st));
      }
      const size_t off = (size_t)kv0 * G * N, n = (size_t)cnt * G * N;
      KC_HIP(c, hipMemcpyAsync(c->h_idx + off, idx + off, n * sizeof(int32_t),
                               hipMemcpyDeviceToHost, st));
      KC_HIP(c, hipEventRecord(c->ev_part[p], st));
    }
    const char* v_base = static_cast<const char*>(cache->v_host);
    char* rows = static_cast<char*>(c->h_rows);
    const int32_t* h_idx = c->h_idx;
    for (int p = 0; p < parts; ++p) {
      int kv0, cnt;
      part_range(p, &kv0, &cnt);
      KC_HIP(c, hipEventSynchronize(c->ev_part[p]));
      const int64_t u_first = (int64_t)kv0 * G, u_count = (int64_t)cnt * G;
      std::function<void(int64_t)> pack = [&](int64_t i) {
        const int64_t u = u_first + i;
        const int64_t b = u / H, hk = (u % H) / G;
        const char* src = v_base + ((b * Hkv + hk) * (int64_t)S_cap) * kc::kRowBytes;
        for (int j = 0; j < N; ++j) {
          const int32_t t = h_idx[u * N + j];
          if (t < 0) break;
          memcpy(rows + (u * N + j) * kc::kRowBytes, src + (int64_t)t * kc::kRowBytes,
                 kc::kRowBytes);
        }
      };
      c->pool->parallel_for(u_count, pack);
      const size_t off = (size_t)u_first * N * kc::kRowBytes, n = (size_t)u_count * N * kc::kRowBytes;
      if (p == 0) {
        KC_HIP(c, hipEventRecord(c->ev_fork, st));  // side must not run ahead of earlier work
        KC_HIP(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
      }
      KC_HIP(c, hipMemcpyAsync(static_cast<char*>(c->d_rows) + off, rows + off, n,
                               hipMemcpyHostToDevice, c->side));
      {
        KernelTimer t(c, KC_KERNEL_GATHER, c->side);
        KC_HIP(c, kc::launch_gather(sh, c->d_rows, idx, w, out_dev, (int)u_first, (int)u_count, 1,
                                    c->side));
      }
    }
    KC_HIP(c, hipEventRecord(c->ev_join, c->side));
    KC_HIP(c, hipStreamWaitEvent(st, c->ev_join, 0));
  }
  KC_HIP(c, hipEventRecord(c->ev_last, st));
  c->have_last = true;
  return KC_OK;
}

int kcache_full_attention(kc_ctx* c, const kc_layer_cache* cache, const void* q_dev, int32_t H,
                          const int32_t* seq_lens_dev, float* out_dev, void* stream) {
  if (!c) return KC_ERR_INVALID_ARG;
  const char* why;
  int rc = shape_status(cache, H == 0 ? -1 : H, 1, &why);
  if (rc != KC_OK) return fail(c, rc, "kcache_full_attention: %s", why);
  if (!cache->k_dev || !cache->v_host || !q_dev || !seq_lens_dev || !out_dev)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_full_attention: NULL pointer argument");
  if (cache->k_fp8)
    return fail(c, KC_ERR_UNSUPPORTED, "kcache_full_attention: 8-bit K caches are not supported");
  if (!cache->v_in_hbm)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_full_attention: this layer's V cache is in host "
                "memory (v_in_hbm is 0); use kcache_decode_attention");
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  void* v_map = nullptr;
  if ((rc = v_pointer(c, cache, &v_map)) != KC_OK) return rc;

  const FullPlan pl = plan_full(c, cache->B, H, cache->Hkv, cache->S_cap, cache->d);
  if ((rc = ensure_workspace(c, pl.bytes)) != KC_OK) return rc;
  if ((rc = ensure_counters(c, (size_t)cache->B * cache->Hkv *
                                   kc::kv_split_for(H / cache->Hkv))) != KC_OK)
    return rc;

  hipStream_t st = (hipStream_t)stream;
  if (c->have_last) KC_HIP(c, hipStreamWaitEvent(st, c->ev_last, 0));
  if (c->store_pending) {
    KC_HIP(c, hipStreamWaitEvent(st, c->ev_store, 0));
    c->store_pending = false;
  }
  if ((rc = enqueue_full(c, cache, v_map, q_dev, H, seq_lens_dev, out_dev, pl, c->ws, c->counters,
                         st)) != KC_OK)
    return rc;
  KC_HIP(c, hipEventRecord(c->ev_last, st));
  c->have_last = true;
  return KC_OK;
}

size_t kcache_static_scratch_bytes(void) { return kStaticWorkBytes; }

int kcache_decode_attention_static(kc_ctx* c, const kc_layer_cache* cache, const void* q_dev,
                                   int32_t H, const int32_t* seq_lens_dev, int32_t N,
                                   float* out_dev, int32_t* idx_out_dev, float* w_out_dev,
                                   void* stream) {
  if (!c) return KC_ERR_INVALID_ARG;
  const char* why;
  int rc = shape_status(cache, H == 0 ? -1 : H, N, &why);
  if (rc != KC_OK) return fail(c, rc, "kcache_decode_attention_static: %s", why);
  if (!cache->k_dev || !cache->v_host || !q_dev || !seq_lens_dev || !out_dev)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_decode_attention_static: NULL pointer argument");
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  void* v_map = nullptr;
  if ((rc = v_pointer(c, cache, &v_map)) != KC_OK) return rc;

  const int split = kc::kv_split_for(H / cache->Hkv);
  const size_t tickets = (size_t)cache->B * cache->Hkv * split;
  const FusedPlan pl = plan_fused(c, cache->B, H, cache->Hkv, cache->S_cap, N, cache->k_fp8, cache->d);
  if (pl.bytes > kStaticWorkBytes || tickets > kStaticTickets)
    return fail(c, KC_ERR_WORKSPACE, "kcache_decode_attention_static: this shape needs %zu bytes "
                "of scratch and %zu tickets, the static scratch holds %zu bytes and %zu tickets; "
                "use kcache_decode_attention", pl.bytes, tickets, kStaticWorkBytes, kStaticTickets);

  hipStream_t st = (hipStream_t)stream;
  if (c->store_pending) {  // V rows of an earlier store on the side stream
    KC_HIP(c, hipStreamWaitEvent(st, c->ev_store, 0));
    c->store_pending = false;
  }
  char* base = static_cast<char*>(c->static_scratch);
  int* counters = reinterpret_cast<int*>(base + kStaticWorkBytes);
  // the array keeps whatever the last call (or a call that was cut short) left: tickets
  // must start at zero
  hipLaunchKernelGGL(zero_ints_kernel, dim3((unsigned)((tickets + 255) / 256)), dim3(256), 0, st,
                     counters, (int)tickets);
  KC_HIP(c, hipGetLastError());
  const int saved_profile = c->profile;
  c->profile = 0;  // profiling events would be created on demand: nothing is allocated here
  rc = enqueue_fused(c, cache, v_map, q_dev, H, seq_lens_dev, N, out_dev, idx_out_dev, w_out_dev,
                     pl, base, counters, st);
  c->profile = saved_profile;
  return rc;
}

}  // extern "C"

struct kc_step_graph {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

namespace {

// How a step is spread over streams.
struct StepPlan {
  int lanes = 1;
  bool split_seq = false;  // lanes hold shares of the batch (true) or whole layers (false)
  long long stagger_ticks = 0;  // lane i starts i / lanes of this late (100 MHz ticks)
};

// Lanes that start together stay in step: their launches take equally long, so their tails
// (when HBM idles) coincide instead of falling into the other lane's scan.  Holding lane i
// back once by i / lanes of `stagger` keeps them out of step for the whole step.  Measured on
// MI355X with two lanes, a delay of about 0.3 launch durations is best (config 2: 10.85 ms
// per step against 11.09 without); a launch that shares HBM with the other lanes streams its
// K rows at about 6.6 TB/s / lanes.
long long stagger_ticks_for(const kc_ctx* c, const kc_layer_cache* shape, const StepPlan& p,
                            int32_t L) {
  if (p.lanes < 2 || c->lane_stagger_us == 0) return 0;
  if (c->lane_stagger_us > 0) return (long long)c->lane_stagger_us * 100;
  if (L < 4) return 0;  // nothing to keep out of step over a launch or two
  const double rows = (double)(p.split_seq ? (shape->B + p.lanes - 1) / p.lanes : shape->B) *
                      shape->Hkv * shape->S_cap;
  const double launch_us = rows * shape->d * (shape->k_fp8 ? 1 : 2) / (6.6e6 / p.lanes);
  const double us = std::min(0.3 * launch_us * p.lanes, 2000.0);  // lane 1 of 2: 0.3 launches
  return (long long)(us * 100.0);
}

// Lanes of a step of L layers over caches of this shape.  KC_OPT_STEP_LANES = 0 chooses:
// two lanes, each with half of the batch through all layers in order (sequences are
// independent, so every dependency of a real decode step is kept), as long as each lane's
// launches still cover the chip; otherwise one lane.  An explicit count is capped by what
// there is to split.
StepPlan plan_step(const kc_ctx* c, const kc_layer_cache* shape, int32_t L, int32_t H) {
  StepPlan p;
  const int B = shape ? std::max(shape->B, 1) : 1;
  if (c->step_lanes == 0) {
    p.split_seq = true;
    if (shape && B >= 2 && H >= 1 && shape->Hkv >= 1 && H % shape->Hkv == 0) {
      const int64_t chunks = (shape->S_cap + 1023) / 1024;
      const int64_t wgs_per_lane =
          (int64_t)(B / 2) * shape->Hkv * kc::kv_split_for(H / shape->Hkv) * chunks;
      if (wgs_per_lane >= 256) p.lanes = 2;
    }
    if (shape) p.stagger_ticks = stagger_ticks_for(c, shape, p, L);
    return p;
  }
  p.split_seq = c->step_split != 0;
  p.lanes = std::min(c->step_lanes, p.split_seq ? B : std::max(L, 1));
  if (shape) p.stagger_ticks = stagger_ticks_for(c, shape, p, L);
  return p;
}

// Workspace bytes and arrival tickets one lane of a step needs for a layer of this shape.
void step_layer_need(const kc_ctx* c, const kc_layer_cache& cache, int32_t H, int32_t N,
                     const StepPlan& sp, size_t* bytes, size_t* tickets) {
  // with sequences split over the lanes each launch covers a share of the batch
  const int nb_max = sp.split_seq ? (cache.B + sp.lanes - 1) / sp.lanes : cache.B;
  size_t need = 0;
  for (int nb = std::max(1, nb_max - 1); nb <= nb_max; ++nb)
    need = std::max(need, cache.v_in_hbm
                              ? plan_full(c, nb, H, cache.Hkv, cache.S_cap, cache.d).bytes
                              : plan_fused(c, nb, H, cache.Hkv, cache.S_cap, N, cache.k_fp8,
                                           cache.d, true).bytes);
  *bytes = std::max(*bytes, need);
  *tickets = std::max(*tickets, (size_t)nb_max * cache.Hkv * kc::kv_split_for(H / cache.Hkv));
}

// Validates a step and sizes what it needs; fills the device-visible V addresses.
int prepare_step(kc_ctx* c, const char* who, const kc_step_layer* layers, int32_t L, int32_t H,
                 const int32_t* pos_dev, const int32_t* seq_lens_dev, int32_t N, StepPlan* sp,
                 std::vector<void*>* v_maps, size_t* lane_bytes, size_t* lane_counters) {
  if (!layers || L < 1) return fail(c, KC_ERR_INVALID_ARG, "%s: no layers", who);
  if (!pos_dev || !seq_lens_dev) return fail(c, KC_ERR_INVALID_ARG, "%s: NULL pointer argument", who);
  size_t need = 0, kv_max = 0;
  v_maps->assign(L, nullptr);
  {
    const char* why0;
    int rc0 = shape_status(&layers[0].cache, H == 0 ? -1 : H, N, &why0);
    if (rc0 != KC_OK) return fail(c, rc0, "%s: layer 0: %s", who, why0);
  }
  *sp = plan_step(c, &layers[0].cache, L, H);
  const int lanes = sp->lanes;
  for (int l = 0; l < L; ++l) {
    const kc_step_layer& y = layers[l];
    const char* why;
    int rc = shape_status(&y.cache, H == 0 ? -1 : H, N, &why);
    if (rc != KC_OK) return fail(c, rc, "%s: layer %d: %s", who, l, why);
    if (!y.cache.k_dev || !y.cache.v_host || !y.q_dev || !y.out_dev)
      return fail(c, KC_ERR_INVALID_ARG, "%s: layer %d: NULL pointer argument", who, l);
    if ((y.k_new_dev == nullptr) != (y.v_new_dev == nullptr))
      return fail(c, KC_ERR_INVALID_ARG, "%s: layer %d: k_new_dev and v_new_dev must both be "
                  "given or both be NULL", who, l);
    if (y.cache.B != layers[0].cache.B)
      return fail(c, KC_ERR_INVALID_ARG, "%s: layer %d: B differs from layer 0", who, l);
    if (y.cache.k_fp8 && y.cache.v_in_hbm)
      return fail(c, KC_ERR_UNSUPPORTED, "%s: layer %d: 8-bit K caches are not supported by "
                  "conventional attention", who, l);
    if ((rc = v_pointer(c, &y.cache, &(*v_maps)[l])) != KC_OK) return rc;
    step_layer_need(c, y.cache, H, N, *sp, &need, &kv_max);
  }
  *lane_bytes = round256(need);
  *lane_counters = (kv_max + 63) & ~(size_t)63;
  int rc = ensure_workspace(c, *lane_bytes * lanes);
  if (rc != KC_OK) return rc;
  if ((rc = ensure_counters(c, *lane_counters * lanes)) != KC_OK) return rc;
  if (lanes > 1 && (rc = ensure_lanes(c, lanes)) != KC_OK) return rc;
  return KC_OK;
}

// Enqueues the step on `st` (and, with lanes > 1, on the lane streams forked from and
// joined back into `st`).  Allocates nothing: usable under stream capture.
int enqueue_step(kc_ctx* c, const kc_step_layer* layers, int32_t L, int32_t H,
                 const int32_t* pos_dev, const int32_t* seq_lens_dev, int32_t N,
                 const StepPlan& sp, const std::vector<void*>& v_maps, size_t lane_bytes,
                 size_t lane_counters, hipStream_t st) {
  const int lanes = sp.lanes;
  if (lanes > 1) {
    KC_HIP(c, hipEventRecord(c->ev_fork, st));
    for (int i = 0; i < lanes; ++i) KC_HIP(c, hipStreamWaitEvent(c->lane[i], c->ev_fork, 0));
    if (sp.stagger_ticks > 0) {  // see stagger_ticks_for
      for (int i = 1; i < lanes; ++i) {
        hipLaunchKernelGGL(stagger_kernel, dim3(1), dim3(64), 0, c->lane[i],
                           sp.stagger_ticks * i / lanes);
        KC_HIP(c, hipGetLastError());
      }
    }
  }
  // The launch plan of a lane's workspace (see enqueue_fused) stays valid from layer to layer
  // as long as the shape and the lengths it was built from are the same and nothing else
  // has used the workspace in between.
  struct PlanKey {
    int B = 0, units = 0, S_cap = 0, R = 0;
    const int32_t* lens = nullptr;
    bool operator==(const PlanKey& o) const {
      return B == o.B && units == o.units && S_cap == o.S_cap && R == o.R && lens == o.lens;
    }
  };
  PlanKey lane_plan[kMaxLanes];
  // one layer (or, with the batch split over the lanes, one share of its sequences)
  auto enqueue_layer = [&](const kc_step_layer& y, const void* v_map, const int32_t* pos,
                           const int32_t* lens, int ln) -> int {
    hipStream_t s = lanes > 1 ? c->lane[ln] : st;
    void* ws = static_cast<char*>(c->ws) + lane_bytes * ln;
    int* counters = c->counters + lane_counters * ln;
    if (y.k_new_dev) {
      const kc::Shape sh{y.cache.B, 0, y.cache.Hkv, y.cache.S_cap, 0, y.cache.dtype, 0, y.cache.d};
      KernelTimer t(c, KC_KERNEL_STORE_K, s);
      KC_HIP(c, kc::launch_store(sh, y.k_new_dev, y.cache.k_dev, y.v_new_dev,
                                 const_cast<void*>(v_map), pos, 1, c->flags,
                                 y.cache.v_in_hbm ? 0 : 1, s, y.cache.k_fp8, y.cache.k_exp));
    }
    if (y.cache.v_in_hbm) {
      const FullPlan pl = plan_full(c, y.cache.B, H, y.cache.Hkv, y.cache.S_cap, y.cache.d);
      lane_plan[ln] = PlanKey();  // conventional attention uses the same workspace
      return enqueue_full(c, &y.cache, v_map, y.q_dev, H, lens, y.out_dev, pl, ws, counters, s);
    }
    const FusedPlan pl =
        plan_fused(c, y.cache.B, H, y.cache.Hkv, y.cache.S_cap, N, y.cache.k_fp8, y.cache.d, true);
    PlanKey key;
    key.B = y.cache.B;
    key.units = y.cache.Hkv * kc::kv_split_for(H / y.cache.Hkv);
    key.S_cap = y.cache.S_cap;
    key.R = pl.R;
    key.lens = lens;
    const bool new_plan = !(key == lane_plan[ln]);
    lane_plan[ln] = key;
    return enqueue_fused(c, &y.cache, v_map, y.q_dev, H, lens, N, y.out_dev, y.idx_out_dev,
                         y.w_out_dev, pl, ws, counters, s, new_plan);
  };
  for (int l = 0; l < L; ++l) {
    const kc_step_layer& y = layers[l];
    if (!sp.split_seq || lanes == 1) {
      const int rc = enqueue_layer(y, v_maps[l], pos_dev, seq_lens_dev, l % lanes);
      if (rc != KC_OK) return rc;
      continue;
    }
    // lane i takes the sequences [b0, b1) of every layer: a view of the layer's tensors
    const int B = y.cache.B;
    const size_t kv_rows = (size_t)y.cache.Hkv * y.cache.S_cap;
    const size_t row_bytes = (size_t)y.cache.d * 2;
    for (int ln = 0; ln < lanes; ++ln) {
      const int b0 = (int)((int64_t)B * ln / lanes), b1 = (int)((int64_t)B * (ln + 1) / lanes);
      if (b1 <= b0) continue;
      kc_step_layer v = y;
      v.cache.B = b1 - b0;
      v.cache.k_dev = static_cast<char*>(y.cache.k_dev) +
                      (size_t)b0 * kv_rows * (y.cache.k_fp8 ? row_bytes / 2 : row_bytes);
      const void* v_map = static_cast<const char*>(v_maps[l]) + (size_t)b0 * kv_rows * row_bytes;
      const size_t tok = (size_t)b0 * y.cache.Hkv * row_bytes;  // new rows [B][1][Hkv][d]
      if (y.k_new_dev) {
        v.k_new_dev = static_cast<const char*>(y.k_new_dev) + tok;
        v.v_new_dev = static_cast<const char*>(y.v_new_dev) + tok;
      }
      v.q_dev = static_cast<const char*>(y.q_dev) + (size_t)b0 * H * row_bytes;
      v.out_dev = y.out_dev + (size_t)b0 * H * y.cache.d;
      if (y.idx_out_dev) v.idx_out_dev = y.idx_out_dev + (size_t)b0 * H * N;
      if (y.w_out_dev) v.w_out_dev = y.w_out_dev + (size_t)b0 * H * N;
      const int rc = enqueue_layer(v, v_map, pos_dev + b0, seq_lens_dev + b0, ln);
      if (rc != KC_OK) return rc;
    }
  }
  if (lanes > 1) {
    for (int i = 0; i < lanes; ++i) {
      KC_HIP(c, hipEventRecord(c->ev_lane[i], c->lane[i]));
      KC_HIP(c, hipStreamWaitEvent(st, c->ev_lane[i], 0));
    }
  }
  return KC_OK;
}

int wait_for_earlier_work(kc_ctx* c, hipStream_t st) {
  if (c->have_last) KC_HIP(c, hipStreamWaitEvent(st, c->ev_last, 0));
  if (c->store_pending) {
    KC_HIP(c, hipStreamWaitEvent(st, c->ev_store, 0));
    c->store_pending = false;
  }
  return KC_OK;
}

}  // namespace

extern "C" {

int kcache_reserve(kc_ctx* c, const kc_layer_cache* shape, int32_t H, int32_t N,
                   int32_t gather_mode, int32_t step_layers) {
  if (!c) return KC_ERR_INVALID_ARG;
  const char* why;
  int rc = shape_status(shape, H == 0 ? -1 : H, N, &why);
  if (rc != KC_OK) return fail(c, rc, "kcache_reserve: %s", why);
  if (gather_mode != KC_GATHER_ZEROCOPY && gather_mode != KC_GATHER_STAGED)
    return fail(c, KC_ERR_INVALID_ARG, "kcache_reserve: unknown gather mode %d", gather_mode);
  if (step_layers < 0) return fail(c, KC_ERR_INVALID_ARG, "kcache_reserve: step_layers < 0");
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  const int B = shape->B, Hkv = shape->Hkv, S_cap = shape->S_cap;
  const size_t units = (size_t)B * H;
  const bool plain_rows = !shape->k_fp8 && shape->d == kc::kHeadDim;  // what the unfused path serves
  // single-layer calls: the fused launch, conventional attention for a layer with V in HBM,
  // and the separate launches when they are selected (KC_OPT_FUSED off, or the staged gather)
  size_t bytes = plan_fused(c, B, H, Hkv, S_cap, N, shape->k_fp8, shape->d).bytes;
  if (shape->v_in_hbm && !shape->k_fp8)
    bytes = std::max(bytes, plan_full(c, B, H, Hkv, S_cap, shape->d).bytes);
  if (plain_rows && (!c->fused || gather_mode == KC_GATHER_STAGED))
    bytes = std::max(bytes, unfused_bytes(units, S_cap, N));
  size_t tickets = (size_t)B * Hkv * kc::kv_split_for(H / Hkv);
  // a whole step: one workspace and one set of tickets per lane
  StepPlan sp;
  if (step_layers > 0) {
    sp = plan_step(c, shape, step_layers, H);
    size_t lane_bytes = 0, lane_tickets = 0;
    step_layer_need(c, *shape, H, N, sp, &lane_bytes, &lane_tickets);
    bytes = std::max(bytes, round256(lane_bytes) * sp.lanes);
    tickets = std::max(tickets, ((lane_tickets + 63) & ~(size_t)63) * sp.lanes);
  }
  c->reserving = true;
  rc = ensure_workspace(c, bytes);
  if (rc == KC_OK) rc = ensure_counters(c, tickets);
  if (rc == KC_OK && gather_mode == KC_GATHER_STAGED && plain_rows && !shape->v_in_hbm)
    rc = ensure_staged(c, units * N);
  if (rc == KC_OK && sp.lanes > 1) rc = ensure_lanes(c, sp.lanes);
  c->reserving = false;
  return rc;
}

int64_t kcache_stat(kc_ctx* c, int32_t which) {
  if (!c) return -1;
  switch (which) {
    case KC_STAT_REALLOCS: return c->reallocs;
    case KC_STAT_WORKSPACE_BYTES: return (int64_t)c->ws_bytes;
    case KC_STAT_TICKETS: return (int64_t)c->counters_n;
    case KC_STAT_STEP_LANES: return c->step_lanes;
    default: return -1;
  }
}

int32_t kcache_step_lanes_for(kc_ctx* c, const kc_layer_cache* shape, int32_t L, int32_t H) {
  if (!c || !shape) return -1;
  return plan_step(c, shape, L, H).lanes;
}

int kcache_decode_step(kc_ctx* c, const kc_step_layer* layers, int32_t L, int32_t H,
                       const int32_t* pos_dev, const int32_t* seq_lens_dev, int32_t N,
                       void* stream) {
  if (!c) return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  std::vector<void*> v_maps;
  size_t lane_bytes = 0, lane_counters = 0;
  StepPlan sp;
  int rc = prepare_step(c, "kcache_decode_step", layers, L, H, pos_dev, seq_lens_dev, N, &sp,
                        &v_maps, &lane_bytes, &lane_counters);
  if (rc != KC_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = wait_for_earlier_work(c, st)) != KC_OK) return rc;
  if ((rc = enqueue_step(c, layers, L, H, pos_dev, seq_lens_dev, N, sp, v_maps, lane_bytes,
                         lane_counters, st)) != KC_OK)
    return rc;
  KC_HIP(c, hipEventRecord(c->ev_last, st));
  c->have_last = true;
  return KC_OK;
}

int kcache_step_graph_create(kc_ctx* c, const kc_step_layer* layers, int32_t L, int32_t H,
                             const int32_t* pos_dev, const int32_t* seq_lens_dev, int32_t N,
                             kc_step_graph** out) {
  if (!c) return KC_ERR_INVALID_ARG;
  if (!out) return fail(c, KC_ERR_INVALID_ARG, "kcache_step_graph_create: out is NULL");
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  std::vector<void*> v_maps;
  size_t lane_bytes = 0, lane_counters = 0;
  StepPlan sp;
  int rc = prepare_step(c, "kcache_step_graph_create", layers, L, H, pos_dev, seq_lens_dev, N,
                        &sp, &v_maps, &lane_bytes, &lane_counters);
  if (rc != KC_OK) return rc;
  // everything the context still has in flight is finished first, so that the captured
  // work depends on nothing outside the graph
  KC_HIP(c, hipDeviceSynchronize());
  c->have_last = false;
  c->store_pending = false;
  KC_HIP(c, hipStreamBeginCapture(c->side, hipStreamCaptureModeThreadLocal));
  c->capturing = true;
  rc = enqueue_step(c, layers, L, H, pos_dev, seq_lens_dev, N, sp, v_maps, lane_bytes,
                    lane_counters, c->side);
  c->capturing = false;
  hipGraph_t graph = nullptr;
  hipError_t e = hipStreamEndCapture(c->side, &graph);
  if (rc != KC_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipGetLastError();
    return rc;
  }
  if (e != hipSuccess || !graph)
    return fail(c, KC_ERR_HIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
  kc_step_graph* sg = new kc_step_graph();
  sg->graph = graph;
  e = hipGraphInstantiate(&sg->exec, graph, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    (void)hipGraphDestroy(graph);
    delete sg;
    return fail(c, KC_ERR_HIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
  }
  c->graphs += 1;
  *out = sg;
  return KC_OK;
}

int kcache_step_graph_launch(kc_ctx* c, kc_step_graph* sg, void* stream) {
  if (!c) return KC_ERR_INVALID_ARG;
  if (!sg || !sg->exec) return fail(c, KC_ERR_INVALID_ARG, "kcache_step_graph_launch: no graph");
  DeviceGuard g(c->device);
  if (!g.ok) return fail(c, KC_ERR_HIP, "hipSetDevice(%d) failed", c->device);
  hipStream_t st = (hipStream_t)stream;
  int rc = wait_for_earlier_work(c, st);
  if (rc != KC_OK) return rc;
  KC_HIP(c, hipGraphLaunch(sg->exec, st));
  KC_HIP(c, hipEventRecord(c->ev_last, st));
  c->have_last = true;
  return KC_OK;
}

int kcache_step_graph_destroy(kc_ctx* c, kc_step_graph* sg) {
  if (!sg) return KC_OK;
  if (c) {
    DeviceGuard g(c->device);
    (void)hipDeviceSynchronize();
    if (c->graphs > 0) c->graphs -= 1;
  }
  if (sg->exec) (void)hipGraphExecDestroy(sg->exec);
  if (sg->graph) (void)hipGraphDestroy(sg->graph);
  delete sg;
  return KC_OK;
}

int kcache_synchronize(kc_ctx* c) {
  if (!c) return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  KC_HIP(c, hipStreamSynchronize(c->side));
  KC_HIP(c, hipStreamSynchronize(c->store_side));
  for (auto st : c->lane)
    if (st) KC_HIP(c, hipStreamSynchronize(st));
  if (c->have_last) KC_HIP(c, hipEventSynchronize(c->ev_last));
  return KC_OK;
}

int kcache_device_check(kc_ctx* c) {
  if (!c) return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  KC_HIP(c, hipDeviceSynchronize());
  int host_flags = 0;
  KC_HIP(c, hipMemcpy(&host_flags, c->flags, sizeof(int), hipMemcpyDeviceToHost));
  if (host_flags == 0) return KC_OK;
  KC_HIP(c, hipMemset(c->flags, 0, sizeof(int)));
  return fail(c, KC_ERR_DEVICE_CHECK, "device check:%s%s%s",
              (host_flags & kc::kFlagBadSeqLen) ? " seq_lens outside [1, S_cap]" : "",
              (host_flags & kc::kFlagBadPos) ? " store position outside [0, S_cap)" : "",
              (host_flags & kc::kFlagBadIndex) ? " a selected position fell outside its sequence "
                                                 "(skipped, not read)" : "");
}

int kcache_profile_read(kc_ctx* c, int32_t kernel, double* total_ms, int64_t* launches) {
  if (!c || kernel < 0 || kernel >= KC_KERNEL_COUNT || !total_ms || !launches)
    return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  int rc = collect_profile(c);
  if (rc != KC_OK) return rc;
  *total_ms = c->prof_ms[kernel];
  *launches = c->prof_n[kernel];
  return KC_OK;
}

int kcache_profile_reset(kc_ctx* c) {
  if (!c) return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  int rc = collect_profile(c);
  if (rc != KC_OK) return rc;
  for (int i = 0; i < KC_KERNEL_COUNT; ++i) {
    c->prof_ms[i] = 0;
    c->prof_n[i] = 0;
  }
  return KC_OK;
}

static int timed_loop(kc_ctx* c, hipStream_t st, int iters, size_t bytes_per_iter, double* gbps,
                      const std::function<hipError_t()>& body) {
  hipEvent_t a = nullptr, b = nullptr;
  KC_HIP(c, hipEventCreate(&a));
  KC_HIP(c, hipEventCreate(&b));
  hipError_t e = body();  // warm-up, untimed
  if (e == hipSuccess) e = hipEventRecord(a, st);
  for (int i = 0; i < iters && e == hipSuccess; ++i) e = body();
  if (e == hipSuccess) e = hipEventRecord(b, st);
  if (e == hipSuccess) e = hipEventSynchronize(b);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (e != hipSuccess) return fail(c, KC_ERR_HIP, "probe failed: %s", hipGetErrorString(e));
  *gbps = ms > 0 ? (double)bytes_per_iter * iters / (ms * 1e-3) / 1e9 : 0.0;
  return KC_OK;
}

int kcache_probe_read(kc_ctx* c, const void* ptr, size_t bytes, int32_t iters, void* stream,
                      double* gbps) {
  if (!c || !ptr || !gbps || bytes < 16 || iters < 1) return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  hipStream_t st = (hipStream_t)stream;
  uint32_t* sink = reinterpret_cast<uint32_t*>(c->flags + 16);
  bytes &= ~(size_t)15;
  return timed_loop(c, st, iters, bytes, gbps,
                    [&] { return kc::launch_probe_read(ptr, bytes, sink, st); });
}

int kcache_probe_rows(kc_ctx* c, const void* ptr, size_t bytes, int64_t n_rows, int32_t iters,
                      void* stream, double* gbps) {
  if (!c || !ptr || !gbps || bytes < (size_t)kc::kRowBytes || n_rows < 1 || iters < 1)
    return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  hipStream_t st = (hipStream_t)stream;
  uint32_t* sink = reinterpret_cast<uint32_t*>(c->flags + 16);
  const size_t total_rows = bytes / kc::kRowBytes;
  return timed_loop(c, st, iters, (size_t)n_rows * kc::kRowBytes, gbps,
                    [&] { return kc::launch_probe_rows(ptr, total_rows, n_rows, sink, st); });
}

int kcache_probe_copy(kc_ctx* c, void* dst, const void* src, size_t bytes, int32_t iters,
                      void* stream, double* gbps) {
  if (!c || !dst || !src || !gbps || bytes < 1 || iters < 1) return KC_ERR_INVALID_ARG;
  DeviceGuard g(c->device);
  hipStream_t st = (hipStream_t)stream;
  return timed_loop(c, st, iters, bytes, gbps,
                    [&] { return hipMemcpyAsync(dst, src, bytes, hipMemcpyDefault, st); });
}

}  // extern "C"
