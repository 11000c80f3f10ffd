// C ABI of the CSER update (declared in include/cser.h; measurement entry points in include/cser_measure.h):
// argument checks, the context, the iteration counter of Algorithm 3 and the order in which the kernels are
// enqueued.  No arithmetic of the method happens on the host.

#include "../../include/cser_measure.h"
#include "cser_internal.h"

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

namespace {

thread_local std::string g_last_hip_error;

int hip_failed(hipError_t err, const char* what) {
  g_last_hip_error = std::string(what) + ": " + hipGetErrorString(err);
  return CSER_EHIP;
}

#define CSER_HIP(call)                                     \
  do {                                                     \
    hipError_t err__ = (call);                             \
    if (err__ != hipSuccess) return hip_failed(err__, #call); \
  } while (0)

constexpr size_t kMaxTimedLaunches = 4096;

struct Timer {
  std::vector<hipEvent_t> begin, end;   // pooled events, created on first use
  size_t used = 0;
  double total_ms = 0.0;
  uint64_t launches = 0;
};

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// A context's buffers and small arrays live on one device: calls must be made with it current.
bool on_its_device(int device) {
  int current = -1;
  return device < 0 || (hipGetDevice(&current) == hipSuccess && current == device);
}

// Non-temporal accesses pay once the state no longer fits the 256 MiB last-level cache (measured +10 % on the
// large workload); a smaller working set is better served by ordinary accesses, because x, e, m come back in
// the next iteration (+7 % at 110-250 MB).
bool wants_nontemporal(const cser_config& c, bool has_e, bool has_m, int setting) {
  if (setting >= 0) return setting != 0;
  const uint64_t arrays = 2u + (has_e ? 1u : 0u) + (has_m ? 1u : 0u);
  return static_cast<uint64_t>(c.W) * c.ld * 4u * arrays > (256ull << 20);
}

// Expected share of the blocks that need the worker mean in one launch: those C_step chose, and on an iteration
// whose reset is fused in, those C_reset chose (the two choices are independent).
double sync_share(uint64_t B, uint32_t k_step, uint32_t k_reset, bool fused_reset) {
  const double cs = static_cast<double>(k_step) / static_cast<double>(B);
  const double cr = fused_reset ? static_cast<double>(k_reset) / static_cast<double>(B) : 0.0;
  return cs + cr - cs * cr;
}

}  // namespace

struct cser_ctx {
  cser_config cfg;
  int device;                // the device that was current at cser_create
  float* x;
  float* e;
  float* m;
  uint64_t B;
  uint32_t k_step, k_reset;
  uint64_t t;
  bool vector_layout;        // block is a multiple of 4 columns: a 4-column group never straddles two blocks
  bool nontemporal;
  cser::Caps caps;
  uint8_t* mask_step;        // device, window * B bytes: C_step's masks for iterations win_t0 .. win_t0 + win_n - 1
  uint32_t window;           // iterations drawn per selector launch
  uint64_t win_t0;
  uint32_t win_n;            // 0: nothing drawn yet
  hipStream_t win_stream;    // stream the window was drawn on
  hipEvent_t win_done;       // recorded after the draw; other streams wait on it
  uint8_t* mask_reset;       // device, B bytes: C_reset's mask of an explicit cser_error_reset
  uint8_t* mask_reset_win;   // device, window * B bytes: C_reset's masks of the reset iterations inside the window
  uint64_t win_reset_t0;     // first reset iteration (multiple of H) in the window
  uint32_t win_reset_n;      // number of reset iterations in the window
  uint32_t* idx_reset;       // device, max(k_reset, 1) entries: the reset's block list in increasing order
  uint32_t* list_counts;     // device scratch of the ordered-list kernels
  uint8_t* mask_query;       // device scratch of cser_select_blocks, B bytes
  uint32_t* idx_query;       // device scratch of cser_select_blocks, max(k_step, k_reset, 1) entries
  hipStream_t query_stream;  // cser_select_blocks runs here
  cser::Tuning tuning;
  bool profiling;
  Timer timers[2];
  cser_counters counters;
};

namespace {

int record_begin(cser_ctx* ctx, int which, hipStream_t s, bool* timed) {
  *timed = false;
  if (!ctx->profiling) return CSER_OK;
  Timer& tm = ctx->timers[which];
  if (tm.used >= kMaxTimedLaunches) return CSER_OK;
  if (tm.used == tm.begin.size()) {
    hipEvent_t a, b;
    CSER_HIP(hipEventCreate(&a));
    hipError_t err = hipEventCreate(&b);
    if (err != hipSuccess) {
      (void)hipEventDestroy(a);
      return hip_failed(err, "hipEventCreate");
    }
    tm.begin.push_back(a);
    tm.end.push_back(b);
  }
  CSER_HIP(hipEventRecord(tm.begin[tm.used], s));
  *timed = true;
  return CSER_OK;
}

int record_end(cser_ctx* ctx, int which, hipStream_t s, bool timed) {
  if (!timed) return CSER_OK;
  Timer& tm = ctx->timers[which];
  CSER_HIP(hipEventRecord(tm.end[tm.used], s));
  tm.used += 1;
  return CSER_OK;
}

int drain_timer(Timer& tm) {
  for (size_t i = 0; i < tm.used; ++i) {
    CSER_HIP(hipEventSynchronize(tm.end[i]));
    float ms = 0.0f;
    CSER_HIP(hipEventElapsedTime(&ms, tm.begin[i], tm.end[i]));
    tm.total_ms += ms;
    tm.launches += 1;
  }
  tm.used = 0;
  return CSER_OK;
}

void free_device_arrays(cser_ctx* ctx) {
  if (ctx->mask_step) (void)hipFree(ctx->mask_step);
  if (ctx->mask_reset) (void)hipFree(ctx->mask_reset);
  if (ctx->mask_reset_win) (void)hipFree(ctx->mask_reset_win);
  if (ctx->win_done) (void)hipEventDestroy(ctx->win_done);
  if (ctx->idx_reset) (void)hipFree(ctx->idx_reset);
  if (ctx->list_counts) (void)hipFree(ctx->list_counts);
  if (ctx->mask_query) (void)hipFree(ctx->mask_query);
  if (ctx->idx_query) (void)hipFree(ctx->idx_query);
  if (ctx->query_stream) (void)hipStreamDestroy(ctx->query_stream);
  for (Timer& tm : ctx->timers) {
    for (hipEvent_t ev : tm.begin) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : tm.end) (void)hipEventDestroy(ev);
  }
}

int validate(const cser_config* c, const float* x, const float* e, const float* m) {
  if (!c || !x) return CSER_EINVAL;
  if (c->d == 0 || c->W == 0 || c->block == 0 || c->ld < c->d) return CSER_EINVAL;
  if (c->R_reset == 0) return CSER_EINVAL;
  if (!std::isfinite(c->lr)) return CSER_EINVAL;
  if (!(c->momentum >= 0.0f && c->momentum < 1.0f)) return CSER_EINVAL;
  if (!m && c->momentum != 0.0f) return CSER_EINVAL;
  if (!aligned(x, 4) || !aligned(e, 4) || !aligned(m, 4)) return CSER_EALIGN;
  const uint64_t B = ceil_div(c->d, c->block);
  if (B > 0xFFFFFFFFull) return CSER_ERANGE;
  if (c->d / 4 > 0xFFFFFFFFull) return CSER_ERANGE;
  if (c->block % 4 != 0 && c->d > 0xFFFFFFFFull) return CSER_ERANGE;   // the element-wise kernels index columns with 32 bits
  // one-wavefront workgroups: one per (worker, 256-column tile), at most 2^31 - 1 of them in a launch
  if (c->W <= 64 && ceil_div(c->d / 4, 64) * c->W > 0x7FFFFFFFull) return CSER_ERANGE;
  return CSER_OK;
}

int refresh_launch_shapes(cser_ctx* ctx) {
  ctx->nontemporal = wants_nontemporal(ctx->cfg, ctx->e != nullptr, ctx->m != nullptr, ctx->tuning.nontemporal);
  if (!ctx->vector_layout) {
    ctx->caps = cser::Caps();
    return CSER_OK;
  }
  CSER_HIP(cser::resolve_caps(ctx->cfg.W, ctx->e != nullptr, ctx->m != nullptr, ctx->nontemporal, ctx->tuning, &ctx->caps));
  return CSER_OK;
}

// The masks of iterations t .. t + window - 1 (stopping at the largest 64-bit t), and C_reset's masks of the
// reset iterations (multiples of H) among them, for the fused reset.
int draw_window(cser_ctx* ctx, uint64_t t, hipStream_t s) {
  ctx->win_n = 0;   // nothing usable until the draw below has been enqueued completely
  ctx->win_reset_n = 0;
  uint32_t count = ctx->window;
  if (UINT64_MAX - t < count - 1) count = static_cast<uint32_t>(UINT64_MAX - t) + 1u;
  CSER_HIP(cser::launch_selector(ctx->cfg.seed, 0u, t, 1u, count, static_cast<uint32_t>(ctx->B), ctx->k_step,
                                 ctx->mask_step, nullptr, s));
  uint32_t reset_n = 0;
  uint64_t reset_t0 = 0;
  const uint64_t H = ctx->cfg.H;
  if (H > 0 && ctx->tuning.fuse_reset) {
    const uint64_t last = t + (count - 1);
    const uint64_t rem = t % H;
    const uint64_t gap = rem == 0 ? 0 : H - rem;
    if (gap <= last - t) {
      reset_t0 = t + gap;
      reset_n = static_cast<uint32_t>((last - reset_t0) / H) + 1u;
      CSER_HIP(cser::launch_selector(ctx->cfg.seed, 1u, reset_t0, H, reset_n, static_cast<uint32_t>(ctx->B), ctx->k_reset,
                                     ctx->mask_reset_win, nullptr, s));
    }
  }
  CSER_HIP(hipEventRecord(ctx->win_done, s));
  ctx->win_t0 = t;
  ctx->win_n = count;
  ctx->win_reset_t0 = reset_t0;
  ctx->win_reset_n = reset_n;
  ctx->win_stream = s;
  ctx->counters.window_draws += 1;
  return CSER_OK;
}

}  // namespace

extern "C" {

int cser_create(const cser_config* cfg, float* x, float* e, float* m, void* hip_stream, cser_ctx** out) {
  if (!out) return CSER_EINVAL;
  *out = nullptr;
  const int bad = validate(cfg, x, e, m);
  if (bad != CSER_OK) return bad;

  cser_ctx* ctx = new (std::nothrow) cser_ctx();
  if (!ctx) return CSER_ENOMEM;
  ctx->cfg = *cfg;
  if (hipGetDevice(&ctx->device) != hipSuccess) ctx->device = -1;
  ctx->x = x;
  ctx->e = e;
  ctx->m = m;
  ctx->B = ceil_div(cfg->d, cfg->block);
  ctx->k_step = cfg->R_step == 0 ? 0u : static_cast<uint32_t>(ceil_div(ctx->B, cfg->R_step));
  ctx->k_reset = static_cast<uint32_t>(ceil_div(ctx->B, cfg->R_reset));
  ctx->t = 0;
  ctx->vector_layout = cfg->block % 4 == 0;
  ctx->profiling = false;
  std::memset(&ctx->counters, 0, sizeof(ctx->counters));

  // C_step's choice is a pure function of (seed, t): draw up to 32 iterations per selector launch
  // (fewer when B is so large that the masks would pass 64 MiB), so its latency is paid once per window
  ctx->window = 32;
  while (ctx->window > 1 && static_cast<uint64_t>(ctx->window) * ctx->B > (64ull << 20)) ctx->window /= 2;
  ctx->win_n = 0;
  ctx->win_t0 = 0;
  ctx->win_stream = nullptr;
  ctx->win_reset_t0 = 0;
  ctx->win_reset_n = 0;
  const uint32_t k_max = ctx->k_step > ctx->k_reset ? ctx->k_step : ctx->k_reset;
  hipError_t err = hipMalloc(reinterpret_cast<void**>(&ctx->mask_step), static_cast<uint64_t>(ctx->window) * ctx->B);
  if (err == hipSuccess) err = hipEventCreateWithFlags(&ctx->win_done, hipEventDisableTiming);
  if (err == hipSuccess && cfg->H > 0)
    err = hipMalloc(reinterpret_cast<void**>(&ctx->mask_reset_win), static_cast<uint64_t>(ctx->window) * ctx->B);
  if (err == hipSuccess) err = hipMalloc(reinterpret_cast<void**>(&ctx->mask_reset), ctx->B);
  if (err == hipSuccess) err = hipMalloc(reinterpret_cast<void**>(&ctx->mask_query), ctx->B);
  if (err == hipSuccess)
    err = hipMalloc(reinterpret_cast<void**>(&ctx->idx_reset), sizeof(uint32_t) * (ctx->k_reset ? ctx->k_reset : 1u));
  if (err == hipSuccess)
    err = hipMalloc(reinterpret_cast<void**>(&ctx->list_counts), sizeof(uint32_t) * cser::kOrderedListCounts);
  if (err == hipSuccess) err = hipMalloc(reinterpret_cast<void**>(&ctx->idx_query), sizeof(uint32_t) * (k_max ? k_max : 1u));
  if (err == hipSuccess) err = hipStreamCreateWithFlags(&ctx->query_stream, hipStreamNonBlocking);
  if (err != hipSuccess) {
    free_device_arrays(ctx);
    delete ctx;
    if (err == hipErrorOutOfMemory) return CSER_ENOMEM;
    return hip_failed(err, "allocating the context's device arrays");
  }
  int rc = refresh_launch_shapes(ctx);
  if (rc != CSER_OK) {
    free_device_arrays(ctx);
    delete ctx;
    return rc;
  }

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint64_t n = static_cast<uint64_t>(cfg->W - 1) * cfg->ld + cfg->d;   // up to the last row's last column
  if (e) err = cser::launch_fill_zero(e, n, s);
  if (err == hipSuccess && m) err = cser::launch_fill_zero(m, n, s);
  if (err != hipSuccess) {
    free_device_arrays(ctx);
    delete ctx;
    return hip_failed(err, "zero fill");
  }
  *out = ctx;
  return CSER_OK;
}

int cser_error_reset(cser_ctx* ctx, void* hip_stream) {
  if (!ctx || !on_its_device(ctx->device)) return CSER_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (ctx->k_reset == 0) return CSER_OK;
  // the mask from the blocks' side, then the chosen ids in increasing order: the kernel sweeps the rows forwards
  CSER_HIP(cser::launch_selector(ctx->cfg.seed, 1u, ctx->t, 0u, 1u, static_cast<uint32_t>(ctx->B), ctx->k_reset,
                                 ctx->mask_reset, nullptr, s));
  CSER_HIP(cser::launch_ordered_list(ctx->mask_reset, static_cast<uint32_t>(ctx->B), ctx->k_reset, ctx->list_counts,
                                     ctx->idx_reset, s));
  cser::ResetParams p;
  p.x = ctx->x;
  p.e = ctx->e;
  p.idx = ctx->idx_reset;
  p.ld = ctx->cfg.ld;
  p.d = ctx->cfg.d;
  p.W = ctx->cfg.W;
  p.block = ctx->cfg.block;
  p.k = ctx->k_reset;
  bool timed = false;
  int rc = record_begin(ctx, 1, s, &timed);
  if (rc != CSER_OK) return rc;
  CSER_HIP(cser::launch_reset(p, ctx->mask_reset, ctx->vector_layout, ctx->nontemporal, ctx->tuning, ctx->caps, s));
  ctx->counters.resets_separate += 1;
  return record_end(ctx, 1, s, timed);
}

int cser_step(cser_ctx* ctx, const float* g, void* hip_stream) {
  if (!ctx || !g || !on_its_device(ctx->device)) return CSER_EINVAL;
  if (!aligned(g, 4)) return CSER_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint64_t t = ctx->t + 1;
  if (ctx->win_n == 0 || t < ctx->win_t0 || t - ctx->win_t0 >= ctx->win_n) {
    const int rc = draw_window(ctx, t, s);
    if (rc != CSER_OK) return rc;
  } else if (s != ctx->win_stream) {
    CSER_HIP(hipStreamWaitEvent(s, ctx->win_done, 0));   // drawn on another stream: order after it
  }
  cser::StepParams p;
  p.g = g;
  p.m = ctx->m;
  p.x = ctx->x;
  p.e = ctx->e;
  p.mask = ctx->mask_step + (t - ctx->win_t0) * ctx->B;
  const bool reset_now = ctx->cfg.H > 0 && t % ctx->cfg.H == 0;
  const bool fused = reset_now && ctx->tuning.fuse_reset && ctx->win_reset_n > 0 && t >= ctx->win_reset_t0 &&
                     (t - ctx->win_reset_t0) / ctx->cfg.H < ctx->win_reset_n;
  p.reset_mask = fused ? ctx->mask_reset_win + ((t - ctx->win_reset_t0) / ctx->cfg.H) * ctx->B : nullptr;
  p.ld = ctx->cfg.ld;
  p.d = ctx->cfg.d;
  p.W = ctx->cfg.W;
  p.block = ctx->cfg.block;
  p.eta = ctx->cfg.lr;
  p.beta = ctx->cfg.momentum;
  bool timed = false;
  int rc = record_begin(ctx, 0, s, &timed);
  if (rc != CSER_OK) return rc;
  int used = 0;
  CSER_HIP(cser::launch_step(p, ctx->vector_layout, ctx->nontemporal, ctx->tuning, ctx->caps,
                             sync_share(ctx->B, ctx->k_step, ctx->k_reset, fused), &used, s));
  rc = record_end(ctx, 0, s, timed);
  if (rc != CSER_OK) return rc;
  ctx->t = t;
  ctx->counters.steps += 1;
  if (used == cser::kKernelTile) ctx->counters.launches_tile += 1;
  else if (used == cser::kKernelShared) ctx->counters.launches_shared += 1;
  else if (used == cser::kKernelSplit) ctx->counters.launches_split += 1;
  else ctx->counters.launches_general += 1;
  if (fused) ctx->counters.resets_fused += 1;
  if (reset_now && !fused) return cser_error_reset(ctx, hip_stream);
  return CSER_OK;
}

int cser_step_many(cser_ctx* ctx, const float* const* g_list, uint32_t n, void* hip_stream, uint32_t* done) {
  if (done) *done = 0;
  if (!ctx || (!g_list && n > 0)) return CSER_EINVAL;
  for (uint32_t i = 0; i < n; ++i) {
    const int rc = cser_step(ctx, g_list[i], hip_stream);
    if (rc != CSER_OK) return rc;
    if (done) *done = i + 1;
  }
  return CSER_OK;
}

int cser_destroy(cser_ctx* ctx) {
  if (!ctx) return CSER_OK;
  free_device_arrays(ctx);
  delete ctx;
  return CSER_OK;
}

int cser_select_blocks(const cser_ctx* ctx, int which, uint64_t t, uint32_t* idx_host, uint8_t* mask_host,
                       uint32_t* k_out) {
  if (!ctx || (which != 0 && which != 1) || !on_its_device(ctx->device)) return CSER_EINVAL;
  const uint32_t k = which == 0 ? ctx->k_step : ctx->k_reset;
  if (k_out) *k_out = k;
  hipStream_t s = ctx->query_stream;
  CSER_HIP(cser::launch_selector(ctx->cfg.seed, static_cast<uint32_t>(which), t, 0u, 1u, static_cast<uint32_t>(ctx->B), k,
                                 ctx->mask_query, ctx->idx_query, s));
  if (mask_host) CSER_HIP(hipMemcpyAsync(mask_host, ctx->mask_query, ctx->B, hipMemcpyDeviceToHost, s));
  if (idx_host && k) CSER_HIP(hipMemcpyAsync(idx_host, ctx->idx_query, sizeof(uint32_t) * k, hipMemcpyDeviceToHost, s));
  CSER_HIP(hipStreamSynchronize(s));
  return CSER_OK;
}

int cser_block_counts(const cser_ctx* ctx, uint64_t* B, uint32_t* k_step, uint32_t* k_reset) {
  if (!ctx) return CSER_EINVAL;
  if (B) *B = ctx->B;
  if (k_step) *k_step = ctx->k_step;
  if (k_reset) *k_reset = ctx->k_reset;
  return CSER_OK;
}

int cser_preset_csea(cser_config* cfg) {
  if (!cfg) return CSER_EINVAL;
  cfg->R_step = 0;
  cfg->H = 1;
  return CSER_OK;
}

int cser_preset_cser_pl(cser_config* cfg) {
  if (!cfg) return CSER_EINVAL;
  cfg->R_step = 0;
  return CSER_OK;
}

int cser_overall_ratio(const cser_config* cfg, double* ratio) {
  if (!cfg || !ratio || cfg->R_reset == 0) return CSER_EINVAL;
  double sent = 0.0;   // fraction of the elements sent per iteration
  if (cfg->R_step > 0) sent += 1.0 / static_cast<double>(cfg->R_step);
  if (cfg->H > 0) sent += 1.0 / (static_cast<double>(cfg->R_reset) * static_cast<double>(cfg->H));
  *ratio = sent > 0.0 ? 1.0 / sent : HUGE_VAL;
  return CSER_OK;
}

int cser_set_lr(cser_ctx* ctx, float lr) {
  if (!ctx || !std::isfinite(lr)) return CSER_EINVAL;
  ctx->cfg.lr = lr;
  return CSER_OK;
}

int cser_get_step(const cser_ctx* ctx, uint64_t* t) {
  if (!ctx || !t) return CSER_EINVAL;
  *t = ctx->t;
  return CSER_OK;
}

int cser_set_step(cser_ctx* ctx, uint64_t t) {
  if (!ctx) return CSER_EINVAL;
  ctx->t = t;
  return CSER_OK;
}

const char* cser_strerror(int status) {
  switch (status) {
    case CSER_OK: return "ok";
    case CSER_EINVAL: return "invalid argument";
    case CSER_EALIGN: return "misaligned pointer or size";
    case CSER_ENOMEM: return "out of memory";
    case CSER_EHIP: return "HIP runtime error (see cser_last_hip_error)";
    case CSER_ERANGE: return "size beyond the supported range";
    default: return "unknown status";
  }
}

const char* cser_last_hip_error(void) { return g_last_hip_error.c_str(); }

// ---------------------------------------------------------------- the entry point that allocates nothing
}  // extern "C"

namespace {

// Block masks of cser_step_static: C_step's in the first half, C_reset's in the second.  One copy per GPU, held
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels and
// launches use the device address looked up below.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[2u * CSER_STATIC_MAX_BLOCKS];

constexpr int kMaxStaticDevices = 64;

struct StaticDevice {
  unsigned char* scratch_ptr = nullptr;   // device address of `scratch` on this GPU
  // launch shapes by [W, or 0 beyond 16 workers][has e][has m][non-temporal]
  bool caps_known[17][2][2][2] = {};
  cser::Caps caps[17][2][2][2];
};

StaticDevice g_static_devices[kMaxStaticDevices];
std::mutex g_static_mutex;

// Set-up for the current device: the address of this GPU's copy of `scratch` (once per device) and the launch
// shapes of this (W, buffers) combination (once per combination); afterwards a lookup.
int static_setup(const cser_config& c, bool has_e, bool has_m, bool nontemporal, unsigned char** ptr, cser::Caps* caps) {
  int device = -1;
  CSER_HIP(hipGetDevice(&device));
  if (device < 0 || device >= kMaxStaticDevices) return CSER_ERANGE;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticDevice& sd = g_static_devices[device];
  if (sd.scratch_ptr == nullptr) {
    void* address = nullptr;
    CSER_HIP(hipGetSymbolAddress(&address, HIP_SYMBOL(scratch)));
    if (address == nullptr) return hip_failed(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
    sd.scratch_ptr = static_cast<unsigned char*>(address);
  }
  *ptr = sd.scratch_ptr;
  *caps = cser::Caps();
  if (c.block % 4 == 0) {
    const uint32_t w = c.W <= 16 ? c.W : 0u;
    cser::Caps& slot = sd.caps[w][has_e][has_m][nontemporal];
    if (!sd.caps_known[w][has_e][has_m][nontemporal]) {
      CSER_HIP(cser::resolve_caps(c.W, has_e, has_m, nontemporal, cser::Tuning(), &slot));
      sd.caps_known[w][has_e][has_m][nontemporal] = true;
    }
    *caps = slot;
  }
  return CSER_OK;
}

}  // namespace

extern "C" {

int cser_step_static(const cser_config* cfg, uint64_t t, float* x, float* e, float* m, const float* g,
                     void* hip_stream) {
  const int bad = validate(cfg, x, e, m);
  if (bad != CSER_OK) return bad;
  if (!g) return CSER_EINVAL;
  if (!aligned(g, 4)) return CSER_EALIGN;
  const uint64_t B = ceil_div(cfg->d, cfg->block);
  if (B > CSER_STATIC_MAX_BLOCKS) return CSER_ERANGE;
  const bool has_e = e != nullptr, has_m = m != nullptr;
  const bool nontemporal = wants_nontemporal(*cfg, has_e, has_m, -1);
  unsigned char* masks = nullptr;
  cser::Caps caps;
  int rc = static_setup(*cfg, has_e, has_m, nontemporal, &masks, &caps);
  if (rc != CSER_OK) return rc;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t k_step = cfg->R_step == 0 ? 0u : static_cast<uint32_t>(ceil_div(B, cfg->R_step));
  const uint32_t k_reset = static_cast<uint32_t>(ceil_div(B, cfg->R_reset));
  const bool reset_now = cfg->H > 0 && t % cfg->H == 0;
  uint8_t* mask_step = masks;
  uint8_t* mask_reset = masks + CSER_STATIC_MAX_BLOCKS;
  // every byte of a mask is written by the selector (a fill kernel, then the exceptions), so what an earlier
  // call left in the array does not matter
  CSER_HIP(cser::launch_selector(cfg->seed, 0u, t, 0u, 1u, static_cast<uint32_t>(B), k_step, mask_step, nullptr, s));
  if (reset_now)
    CSER_HIP(cser::launch_selector(cfg->seed, 1u, t, 0u, 1u, static_cast<uint32_t>(B), k_reset, mask_reset, nullptr, s));
  cser::StepParams p;
  p.g = g;
  p.m = m;
  p.x = x;
  p.e = e;
  p.mask = mask_step;
  p.reset_mask = reset_now ? mask_reset : nullptr;   // the error reset is carried out in the same kernel pass
  p.ld = cfg->ld;
  p.d = cfg->d;
  p.W = cfg->W;
  p.block = cfg->block;
  p.eta = cfg->lr;
  p.beta = cfg->momentum;
  CSER_HIP(cser::launch_step(p, cfg->block % 4 == 0, nontemporal, cser::Tuning(), caps,
                             sync_share(B, k_step, k_reset, reset_now), nullptr, s));
  return CSER_OK;
}

// ---------------------------------------------------------------- measurement only (cser_measure.h)

int cser_profile_enable(cser_ctx* ctx, int on) {
  if (!ctx) return CSER_EINVAL;
  ctx->profiling = on != 0;
  return CSER_OK;
}

int cser_profile_read(cser_ctx* ctx, int which, double* total_ms, uint64_t* launches) {
  if (!ctx || (which != 0 && which != 1)) return CSER_EINVAL;
  Timer& tm = ctx->timers[which];
  const int rc = drain_timer(tm);
  if (rc != CSER_OK) return rc;
  if (total_ms) *total_ms = tm.total_ms;
  if (launches) *launches = tm.launches;
  return CSER_OK;
}

int cser_profile_clear(cser_ctx* ctx) {
  if (!ctx) return CSER_EINVAL;
  for (Timer& tm : ctx->timers) {
    const int rc = drain_timer(tm);
    if (rc != CSER_OK) return rc;
    tm.total_ms = 0.0;
    tm.launches = 0;
  }
  return CSER_OK;
}

int cser_set_tuning(cser_ctx* ctx, int key, int64_t value) {
  if (!ctx || !on_its_device(ctx->device)) return CSER_EINVAL;
  cser::Tuning next = ctx->tuning;
  switch (key) {
    case CSER_TUNE_KERNEL:
      if (value < 0 || value > 4) return CSER_EINVAL;
      next.kernel = static_cast<int>(value);
      break;
    case CSER_TUNE_NONTEMPORAL:
      if (value < -1 || value > 1) return CSER_EINVAL;
      next.nontemporal = static_cast<int>(value);
      break;
    case CSER_TUNE_FUSE_RESET:
      next.fuse_reset = value != 0;
      break;
    case CSER_TUNE_TILE_WAVES_PER_CU:
      if (value < -1 || value > 64) return CSER_EINVAL;
      next.tile_waves_per_cu = static_cast<int>(value);
      break;
    case CSER_TUNE_SHARED_GROUPS_PER_CU:
      if (value < -1 || value > 64) return CSER_EINVAL;
      next.shared_groups_per_cu = static_cast<int>(value);
      break;
    default:
      return CSER_EINVAL;
  }
  const cser::Tuning before = ctx->tuning;
  ctx->tuning = next;
  const int rc = refresh_launch_shapes(ctx);
  if (rc != CSER_OK) {
    ctx->tuning = before;
    (void)refresh_launch_shapes(ctx);
    return rc;
  }
  ctx->win_n = 0;   // the window is redrawn with (or without) C_reset's masks
  return CSER_OK;
}

int cser_measure_counters(const cser_ctx* ctx, cser_counters* out) {
  if (!ctx || !out) return CSER_EINVAL;
  *out = ctx->counters;
  return CSER_OK;
}

int cser_measure_residency(const cser_ctx* ctx, cser_residency* out) {
  if (!ctx || !out) return CSER_EINVAL;
  const cser::Caps& c = ctx->caps;
  out->tile_lds = c.tile_lds;
  out->tile_groups_per_cu = c.tile_resident;
  out->shared_lds = c.shared_lds;
  out->shared_groups_per_cu = c.shared_resident;
  out->shared_reset_lds = c.shared_reset_lds;
  out->shared_reset_groups_per_cu = c.shared_reset_resident;
  out->reset_lds = c.reset_lds;
  out->reset_groups_per_cu = c.reset_resident;
  return CSER_OK;
}

int cser_measure_kernel_choice(const cser_config* cfg, int reset_iteration, int* kernel) {
  if (!cfg || !kernel || cfg->d == 0 || cfg->W == 0 || cfg->block == 0 || cfg->R_reset == 0) return CSER_EINVAL;
  const uint64_t B = ceil_div(cfg->d, cfg->block);
  const uint32_t k_step = cfg->R_step == 0 ? 0u : static_cast<uint32_t>(ceil_div(B, cfg->R_step));
  const uint32_t k_reset = static_cast<uint32_t>(ceil_div(B, cfg->R_reset));
  *kernel = cser::choose_step_kernel(cfg->d, cfg->W, cfg->block, cfg->block % 4 == 0,
                                     sync_share(B, k_step, k_reset, reset_iteration != 0), cser::Tuning());
  return CSER_OK;
}

int cser_copy_probe(void* dst, const void* src, uint64_t n_bytes, void* hip_stream) {
  if (!dst || !src) return CSER_EINVAL;
  if (!aligned(dst, 16) || !aligned(src, 16) || n_bytes % 16 != 0) return CSER_EALIGN;
  if (n_bytes / 16 / 256 > 0x7FFFFFFFull) return CSER_ERANGE;
  CSER_HIP(cser::launch_copy(dst, src, n_bytes, static_cast<hipStream_t>(hip_stream)));
  return CSER_OK;
}

}  // extern "C"
