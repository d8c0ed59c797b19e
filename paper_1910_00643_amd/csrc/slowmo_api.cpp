// C ABI of the Slow Momentum hot path: argument checking, workspace layout,
// tiling tables, per-call gradient-pointer table, counters.  All arithmetic on
// tensor elements happens in the kernels (slowmo_kernels.hip).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/slowmo.h"
#include "slowmo_kernels.h"
#include "slowmo_plan.h"

using namespace slowmo;

namespace {

constexpr int kSlots = 4;            // ring of per-call tables (mixing order, de-bias table)
constexpr int kGradSlots = 16;       // gradient-pointer tables kept on the device
constexpr size_t kSectionAlign = 256;

thread_local std::string g_err = "";

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// One slot of the mixing-table ring holds the entries of one mixing step.
size_t mixtab_bytes(int32_t m) { return static_cast<size_t>(m) * sizeof(MixEntry); }
// One slot of the de-bias ring: m * n_tensors destination pointers, then the m weights.
size_t ztab_bytes(int32_t m, int32_t n_tensors) {
  return static_cast<size_t>(m) * n_tensors * sizeof(void *) + static_cast<size_t>(m) * sizeof(float);
}

// Byte offsets of the sections of the caller's workspace.
struct Sections {
  size_t x0, u, h, v, xtab_t, gtab[kGradSlots], mixtab[kSlots], ztab[kSlots], slots, tensors, ltiles, otiles, btiles, rtiles, total;
};

Sections make_sections(const slowmo_config &c, int32_t n_tensors, const Layout &L, size_t n_ltiles,
                       size_t n_otiles, size_t n_btiles) {
  Sections s{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off += round_up(std::max<size_t>(bytes, 1), kSectionAlign);
    return at;
  };
  const size_t arena = static_cast<size_t>(L.d_pad) * sizeof(float);
  const size_t n_ptr = static_cast<size_t>(c.m) * n_tensors;
  const size_t outer_copies = c.no_average ? static_cast<size_t>(c.m) : 1;
  s.x0 = take(arena * outer_copies);
  s.u = take(arena * outer_copies);
  s.h = take(arena * c.m);
  s.v = take(c.base == SLOWMO_ADAM ? arena * c.m : 0);
  s.xtab_t = take(n_ptr * sizeof(void *));
  for (int i = 0; i < kGradSlots; ++i) s.gtab[i] = take(n_ptr * sizeof(void *));
  for (int i = 0; i < kSlots; ++i) s.mixtab[i] = take(mixtab_bytes(c.m));
  for (int i = 0; i < kSlots; ++i) s.ztab[i] = take(ztab_bytes(c.m, n_tensors));
  s.slots = take(n_ptr * sizeof(SlotInfo));
  s.tensors = take(static_cast<size_t>(n_tensors) * sizeof(TensorInfo));
  s.ltiles = take(n_ltiles * sizeof(TileRef));
  s.otiles = take(n_otiles * sizeof(TileRef));
  // big tiles and the ordinary tiles they leave over (at most all of them)
  s.btiles = take(n_btiles * sizeof(TileRef));
  s.rtiles = take(n_btiles ? n_otiles * sizeof(TileRef) : 0);
  s.total = off;
  return s;
}

bool finite_pos(float v) { return std::isfinite(v) && v > 0.f; }
bool unit_interval(float v) { return std::isfinite(v) && v >= 0.f && v < 1.f; }

// Returns an empty string if cfg / tensor list are usable.
std::string check_config(const slowmo_config *c, int32_t n_tensors, const int64_t *numel) {
  if (!c) return "cfg is NULL";
  if (!numel) return "numel is NULL";
  if (n_tensors < 1) return "n_tensors must be >= 1";
  if (c->m < 1 || c->m > SLOWMO_MAX_WORKERS) return "m must be in 1..SLOWMO_MAX_WORKERS";
  if (c->tau < 1) return "tau must be >= 1";
  if (!finite_pos(c->alpha)) return "alpha must be finite and > 0";
  if (!unit_interval(c->beta)) return "beta must satisfy 0 <= beta < 1";
  if (c->base != SLOWMO_SGD_NESTEROV && c->base != SLOWMO_ADAM) return "unknown base optimizer";
  if (c->policy != SLOWMO_BUF_RESET && c->policy != SLOWMO_BUF_MAINTAIN &&
      c->policy != SLOWMO_BUF_AVERAGE)
    return "unknown buffer policy";
  if (c->grad_dtype != SLOWMO_F32 && c->grad_dtype != SLOWMO_BF16) return "unknown gradient dtype";
  if (c->no_average != 0 && c->no_average != 1) return "no_average must be 0 or 1";
  if (c->no_average && c->policy == SLOWMO_BUF_AVERAGE)
    return "no_average cannot be combined with the AVERAGE buffer policy";
  if (!(std::isfinite(c->weight_decay) && c->weight_decay >= 0.f))
    return "weight_decay must be finite and >= 0";
  if (c->base == SLOWMO_SGD_NESTEROV) {
    if (!unit_interval(c->momentum)) return "momentum must satisfy 0 <= momentum < 1";
  } else {
    if (!unit_interval(c->beta1) || !unit_interval(c->beta2))
      return "beta1 and beta2 must satisfy 0 <= . < 1";
    if (!(std::isfinite(c->eps) && c->eps >= 0.f)) return "eps must be finite and >= 0";
  }
  int64_t total = 0;
  for (int32_t j = 0; j < n_tensors; ++j) {
    if (numel[j] < 0) return "numel has a negative entry";
    if (numel[j] > (int64_t(1) << 36)) return "a tensor exceeds 2^36 elements";
    total += numel[j];
  }
  if (total * c->m > (int64_t(1) << 44)) return "m * total elements exceeds 2^44";
  if (static_cast<int64_t>(c->m) * n_tensors > (int64_t(1) << 24))
    return "m * n_tensors exceeds 2^24";
  if (count_local_tiles(c->m, n_tensors, numel) > (int64_t(1) << 31) - 16)
    return "too many tiles for one launch (m * total elements too large)";
  return "";
}

int32_t env_flag(const char *name, int32_t dflt) {
  const char *s = std::getenv(name);
  if (!s || !*s) return dflt;
  return static_cast<int32_t>(std::strtol(s, nullptr, 10));
}

// A small host->device table that may change from call to call: a ring of
// device slots (inside the caller's workspace) with pinned staging copies,
// and one event per slot recorded after its upload, so that a staging copy is
// not rewritten while an earlier upload may still be reading it.
template <int N>
struct TableRing {
  void *d[N] = {};
  void *h[N] = {};
  hipEvent_t ev[N] = {};
  bool used[N] = {};     // the slot's device copy holds the table of its staging copy
  bool sent[N] = {};     // an upload from the slot's staging copy was enqueued (ev recorded)
  size_t len[N] = {};    // bytes of the table in each slot
  uint64_t key[N] = {};  // cheap fingerprint of the table in each slot
  int cur = -1;          // slot of the most recent upload, -1 = none

  hipError_t init(char *device_base, const size_t *offsets, size_t bytes) {
    for (int i = 0; i < N; ++i) {
      d[i] = device_base + offsets[i];
      hipError_t e = hipHostMalloc(&h[i], std::max<size_t>(bytes, 8), hipHostMallocDefault);
      if (e != hipSuccess) return e;
      e = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  // A few words of the table (first, last, two in between) mixed with its
  // length: distinct pointer tables differ there, so the full comparison
  // below runs for one candidate, not for every slot.
  static uint64_t fingerprint(const void *src, size_t bytes) {
    const size_t words = bytes / sizeof(uint64_t);
    uint64_t k = 0x9e3779b97f4a7c15ull ^ bytes;
    if (words == 0) return k;
    const size_t at[4] = {0, words / 3, 2 * words / 3, words - 1};
    for (size_t i : at) {
      uint64_t w;
      std::memcpy(&w, static_cast<const char *>(src) + i * sizeof(uint64_t), sizeof(w));
      k = (k ^ w) * 0xff51afd7ed558ccdull;
      k ^= k >> 32;
    }
    return k;
  }
  // Slot that already holds exactly this table (most recent first), or -1.
  // The staging copy of a slot always equals what its device copy holds once
  // the stream has reached the upload.
  int find(const void *src, size_t bytes) const {
    if (cur < 0) return -1;
    const uint64_t k = fingerprint(src, bytes);
    for (int i = 0; i < N; ++i) {
      const int slot = (cur - i + N) % N;
      if (used[slot] && key[slot] == k && len[slot] == bytes &&
          std::memcmp(h[slot], src, bytes) == 0)
        return slot;
    }
    return -1;
  }
  // The next slot's staging buffer, free to be written (waits until the
  // previous upload from it has been consumed); returns the slot or -1.
  int stage(hipError_t *err) {
    const int slot = (cur + 1) % N;
    if (sent[slot]) {
      *err = hipEventSynchronize(ev[slot]);
      if (*err != hipSuccess) return -1;
      sent[slot] = false;
    }
    used[slot] = false;
    return slot;
  }
  // Sends the first `bytes` of slot's staging buffer to `dst` (the slot's own
  // device copy when dst is NULL) and makes the slot the current one.
  hipError_t send(int slot, size_t bytes, void *dst, hipStream_t stream) {
    hipError_t e = hipMemcpyAsync(dst ? dst : d[slot], h[slot], bytes, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return e;
    e = hipEventRecord(ev[slot], stream);
    if (e != hipSuccess) return e;
    sent[slot] = true;
    used[slot] = dst == nullptr;  // a table sent elsewhere is not found again in this slot
    len[slot] = bytes;
    key[slot] = fingerprint(h[slot], bytes);
    cur = slot;
    return hipSuccess;
  }
  // Uploads `bytes` from src into the next slot; returns the slot or -1.
  int upload(const void *src, size_t bytes, hipStream_t stream, hipError_t *err) {
    const int slot = stage(err);
    if (slot < 0) return -1;
    std::memcpy(h[slot], src, bytes);
    *err = send(slot, bytes, nullptr, stream);
    return *err == hipSuccess ? slot : -1;
  }
  void destroy() {
    for (int i = 0; i < N; ++i) {
      if (ev[i]) (void)hipEventDestroy(ev[i]);
      if (h[i]) (void)hipHostFree(h[i]);
    }
  }
};

}  // namespace

struct slowmo_ctx {
  slowmo_config cfg{};
  int32_t n_tensors = 0;
  std::vector<int64_t> numel;
  Layout layout;
  int device = 0;

  // sections of the caller's workspace (device pointers)
  float *x0 = nullptr, *u = nullptr, *h = nullptr, *v = nullptr;
  float **d_xtab_t = nullptr;  // replica pointers, tensor-major
  SlotInfo *d_slots = nullptr;
  TensorInfo *d_tensors = nullptr;
  TileRef *d_ltiles = nullptr;
  TileRef *d_otiles = nullptr;
  int32_t n_ltiles = 0, n_otiles = 0;
  // With big tiles in use, the outer step and the fused last step run twice:
  // over the big tiles (whole kBigTile pieces of the tensors all of whose
  // replicas are 16-byte aligned) and over the ordinary tiles these leave
  // over.  Otherwise n_btiles = 0 and the rest list is the whole ordinary list.
  TileRef *d_btiles = nullptr, *d_rtiles = nullptr;
  int32_t n_btiles = 0, n_rtiles = 0;
  bool big_outer = false;  // the plain outer step uses them too (it gains only with many workers)
  bool big_forced = false; // SLOWMO_BIG_TILES=1: wherever the kernels allow

  TableRing<kGradSlots> gtab;  // gradient-pointer tables of recent calls (m * n_tensors each)
  TableRing<kSlots> mixtab;  // update order of the current mixing step (at most m entries)
  TableRing<kSlots> ztab;  // destination pointers and weights of the current de-bias call
  std::vector<float> w;  // push-sum weights (Algorithm C.1), 1 after every exact average
  std::vector<SlotInfo> slots;      // host copies of the per-slot / per-tensor tables
  std::vector<TensorInfo> tinfo;

  int64_t t = 0;  // outer iterations done
  int32_t k = 0;  // local steps in the current outer iteration
  int64_t l = 0;  // Adam steps counted by the bias correction
  bool buffers_zero = true;  // h (and v) are to be read as zero by the next local step
  bool params_aligned = true;  // every replica pointer is 16-byte aligned
  int32_t check_pointers = 1;  // 1: caller's tensors are checked at create; 2: also per call

  void *static_table = nullptr;  // this device's static scratch (slowmo_debias_static)

  // A call that launches several kernels and fails between two of them has
  // changed device memory halfway: the context then refuses further work.
  bool broken = false;
  // Test hook (SLOWMO_TEST_FAIL_LAUNCH=n, read at create): the n-th kernel
  // launch of this context (1-based) is not issued and reports a launch
  // failure instead, so the error paths can be driven from the host.
  int64_t fail_launch_at = 0, launches = 0;

  LaunchTuning tune{};
  std::string err;
};

namespace {

slowmo_status fail(slowmo_ctx *ctx, slowmo_status st, const std::string &msg) {
  if (ctx) {
    ctx->err = msg;
  } else {
    g_err = msg;
  }
  return st;
}

slowmo_status fail_hip(slowmo_ctx *ctx, hipError_t e, const char *what) {
  return fail(ctx, SLOWMO_ERR_HIP,
              std::string(what) + ": " + hipGetErrorName(e) + " (" + hipGetErrorString(e) + ")");
}

// Every kernel launch of a context goes through here (see fail_launch_at).
template <typename F>
hipError_t guarded(slowmo_ctx *ctx, F &&launch) {
  if (ctx->fail_launch_at > 0 && ++ctx->launches == ctx->fail_launch_at) return hipErrorLaunchFailure;
  return launch();
}

// Failure after at least one kernel of a multi-kernel call was launched.
slowmo_status fail_midway(slowmo_ctx *ctx, hipError_t e, const char *what) {
  ctx->broken = true;
  return fail(ctx, SLOWMO_ERR_HIP,
              std::string(what) + ": " + hipGetErrorName(e) + " (" + hipGetErrorString(e) +
                  ") after part of the call's kernels were launched; replicas and buffers are "
                  "partly updated and the context refuses further steps");
}

// A kernel that walks all workers per workgroup runs over the big tiles (if
// any) with `big`, then over the ordinary tiles they leave over with `rest`;
// both take (tiles, count) and return a hipError_t.  *launched counts the
// kernels of the current call issued so far: a failure after the first one is
// a failure halfway.
template <typename FB, typename FR>
slowmo_status run_tiled(slowmo_ctx *ctx, bool use_big, int *launched, const char *what, FB &&big,
                        FR &&rest) {
  for (int pass = 0; pass < 2; ++pass) {
    const bool b = pass == 0;
    if (b && !use_big) continue;
    const TileRef *tiles = b ? ctx->d_btiles : (use_big ? ctx->d_rtiles : ctx->d_otiles);
    const int32_t n = b ? ctx->n_btiles : (use_big ? ctx->n_rtiles : ctx->n_otiles);
    if (n <= 0) continue;
    const hipError_t e = guarded(ctx, [&] { return b ? big(tiles, n) : rest(tiles, n); });
    if (e != hipSuccess) return *launched ? fail_midway(ctx, e, what) : fail_hip(ctx, e, what);
    ++*launched;
  }
  return SLOWMO_OK;
}

const char *kBrokenMsg =
    "an earlier multi-kernel call failed halfway; the context's state is undefined: destroy it";

void release(slowmo_ctx *ctx) {
  ctx->gtab.destroy();
  ctx->mixtab.destroy();
  ctx->ztab.destroy();
  delete ctx;
}

}  // namespace

extern "C" {

const char *slowmo_version(void) { return "0.1.0 gfx950"; }

const char *slowmo_last_error(const slowmo_ctx *ctx) {
  return ctx ? ctx->err.c_str() : g_err.c_str();
}

size_t slowmo_state_bytes(const slowmo_config *cfg, int32_t n_tensors, const int64_t *numel) {
  std::string bad = check_config(cfg, n_tensors, numel);
  if (!bad.empty()) {
    g_err = bad;
    return 0;
  }
  Layout L = make_layout(n_tensors, numel);
  return make_sections(*cfg, n_tensors, L,
                       static_cast<size_t>(count_local_tiles(cfg->m, n_tensors, numel)),
                       static_cast<size_t>(count_outer_tiles(n_tensors, numel)),
                       static_cast<size_t>(count_big_tiles(n_tensors, numel)))
      .total;
}

static int64_t plan_query(bool local, int32_t m, int32_t n_tensors, const int64_t *numel,
                          slowmo_plan_run *out, int64_t cap) {
  if (m < 1 || n_tensors < 1 || !numel || cap < 0 || (cap > 0 && !out)) return -1;
  for (int32_t j = 0; j < n_tensors; ++j)
    if (numel[j] < 0) return -1;
  const int64_t total =
      local ? count_local_tiles(m, n_tensors, numel) : count_outer_tiles(n_tensors, numel);
  if (cap == 0) return total;
  if (total > (int64_t(1) << 31) - 16) return -1;
  std::vector<PlanRun> runs;
  if (local) {
    plan_local(m, n_tensors, numel, runs);
  } else {
    plan_outer(n_tensors, numel, runs);
  }
  for (int64_t i = 0; i < std::min<int64_t>(cap, runs.size()); ++i) {
    out[i] = {runs[i].tile, runs[i].worker, runs[i].tensor, runs[i].n, runs[i].offset};
  }
  return total;
}

int64_t slowmo_plan_local(int32_t m, int32_t n_tensors, const int64_t *numel, slowmo_plan_run *out,
                          int64_t cap) {
  return plan_query(true, m, n_tensors, numel, out, cap);
}

int64_t slowmo_plan_outer(int32_t m, int32_t n_tensors, const int64_t *numel, slowmo_plan_run *out,
                          int64_t cap) {
  return plan_query(false, m, n_tensors, numel, out, cap);
}

slowmo_status slowmo_check_device_range(const void *ptr, size_t bytes) {
  if (!ptr) return fail(nullptr, SLOWMO_ERR_ARG, "pointer is NULL");
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipGetDevice");
  const char *lo = static_cast<const char *>(ptr);
  const char *ends[2] = {lo, lo + (bytes ? bytes - 1 : 0)};
  for (const char *q : ends) {
    hipPointerAttribute_t at{};
    e = hipPointerGetAttributes(&at, q);
    if (e != hipSuccess) {
      (void)hipGetLastError();  // not sticky: the next call must not see it
      return fail(nullptr, SLOWMO_ERR_ARG,
                  "the range is not memory known to the HIP runtime (ordinary host memory?)");
    }
    if (at.type == hipMemoryTypeUnregistered)
      return fail(nullptr, SLOWMO_ERR_ARG, "the range is ordinary host memory, not device-accessible");
    if (at.type == hipMemoryTypeDevice && at.device != dev)
      return fail(nullptr, SLOWMO_ERR_ARG, "the range is memory of another device");
  }
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  e = hipMemGetAddressRange(&base, &size, const_cast<void *>(ptr));
  if (e != hipSuccess) {
    (void)hipGetLastError();  // no range information for this kind of memory: both ends were known
  } else if (lo + bytes > static_cast<const char *>(base) + size) {
    return fail(nullptr, SLOWMO_ERR_ARG, "the range runs past the end of its allocation");
  }
  return SLOWMO_OK;
}

slowmo_status slowmo_create(slowmo_ctx **out, const slowmo_config *cfg, int32_t n_tensors,
                            const int64_t *numel, float *const *params, void *state,
                            size_t state_bytes, void *stream_) {
  if (!out) return fail(nullptr, SLOWMO_ERR_ARG, "out is NULL");
  *out = nullptr;
  std::string bad = check_config(cfg, n_tensors, numel);
  if (!bad.empty()) return fail(nullptr, SLOWMO_ERR_ARG, bad);
  if (!params) return fail(nullptr, SLOWMO_ERR_ARG, "params is NULL");
  if (!state) return fail(nullptr, SLOWMO_ERR_ARG, "state is NULL");
  if (reinterpret_cast<uintptr_t>(state) % kSectionAlign)
    return fail(nullptr, SLOWMO_ERR_ALIGN, "state workspace must be 256-byte aligned");

  const int32_t m = cfg->m;
  const size_t n_ptr = static_cast<size_t>(m) * n_tensors;
  struct Span {
    uintptr_t lo, hi;
  };
  std::vector<Span> spans;
  for (size_t i = 0; i < n_ptr; ++i) {
    const int64_t n = numel[i % n_tensors];
    if (n == 0) continue;
    if (!params[i]) return fail(nullptr, SLOWMO_ERR_ARG, "a parameter pointer is NULL");
    uintptr_t p = reinterpret_cast<uintptr_t>(params[i]);
    if (p % sizeof(float)) return fail(nullptr, SLOWMO_ERR_ALIGN, "a parameter pointer is not 4-byte aligned");
    spans.push_back({p, p + static_cast<uintptr_t>(n) * sizeof(float)});
  }

  slowmo_ctx *ctx = new (std::nothrow) slowmo_ctx;
  if (!ctx) return fail(nullptr, SLOWMO_ERR_NOMEM, "host allocation failed");
  ctx->cfg = *cfg;
  ctx->n_tensors = n_tensors;
  ctx->numel.assign(numel, numel + n_tensors);
  ctx->layout = make_layout(n_tensors, numel);
  ctx->tune.xcd_remap = env_flag("SLOWMO_XCD_REMAP", 1) ? 1 : 0;
  ctx->tune.xcd_run = std::max(env_flag("SLOWMO_XCD_RUN", 0), 0);
  ctx->tune.nontemporal = env_flag("SLOWMO_NT", 1) ? 1 : 0;
  ctx->tune.fuse_last = env_flag("SLOWMO_FUSE_LAST", 1) ? 1 : 0;
  ctx->tune.fuse_mix = env_flag("SLOWMO_FUSE_MIX", 1) ? 1 : 0;
  ctx->tune.outer_lds = std::min(std::max(env_flag("SLOWMO_OUTER_LDS", 0), 0), 64 * 1024);
  // big tiles: -1 = by the worker count (see kBigFusedFromWorkers), 0 = never, 1 = always
  const int32_t big = env_flag("SLOWMO_BIG_TILES", -1);
  ctx->tune.big_tiles =
      ((big < 0 ? m >= kBigFusedFromWorkers : big != 0) && ctx->tune.nontemporal) ? 1 : 0;
  ctx->big_outer = ctx->tune.big_tiles && (big > 0 || m >= kBigOuterFromWorkers);
  ctx->big_forced = big > 0;
  ctx->fail_launch_at = env_flag("SLOWMO_TEST_FAIL_LAUNCH", 0);

  const int64_t n_ltiles = count_local_tiles(m, n_tensors, numel);
  const int64_t n_otiles = count_outer_tiles(n_tensors, numel);
  const Sections sec = make_sections(*cfg, n_tensors, ctx->layout, static_cast<size_t>(n_ltiles),
                                     static_cast<size_t>(n_otiles),
                                     static_cast<size_t>(count_big_tiles(n_tensors, numel)));
  if (state_bytes < sec.total) {
    delete ctx;
    return fail(nullptr, SLOWMO_ERR_NOMEM, "state workspace is smaller than slowmo_state_bytes()");
  }
  spans.push_back({reinterpret_cast<uintptr_t>(state), reinterpret_cast<uintptr_t>(state) + sec.total});
  std::sort(spans.begin(), spans.end(), [](const Span &a, const Span &b) { return a.lo < b.lo; });
  for (size_t i = 1; i < spans.size(); ++i) {
    if (spans[i].lo < spans[i - 1].hi) {
      delete ctx;
      return fail(nullptr, SLOWMO_ERR_ARG, "parameter tensors overlap each other or the workspace");
    }
  }

  // ---- from here on the device is needed -------------------------------------
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  hipError_t e = hipGetDevice(&ctx->device);
  if (e != hipSuccess) {
    delete ctx;
    return fail_hip(nullptr, e, "hipGetDevice");
  }
  ctx->check_pointers = env_flag("SLOWMO_CHECK_POINTERS", 1);
  if (ctx->check_pointers) {
    slowmo_status bad_ptr = slowmo_check_device_range(state, sec.total);
    for (size_t i = 0; i < n_ptr && bad_ptr == SLOWMO_OK; ++i) {
      const int64_t n = numel[i % n_tensors];
      if (n) bad_ptr = slowmo_check_device_range(params[i], static_cast<size_t>(n) * sizeof(float));
    }
    if (bad_ptr != SLOWMO_OK) {
      delete ctx;
      g_err = "parameter tensor or workspace: " + g_err;
      return bad_ptr;
    }
  }
  char *base = static_cast<char *>(state);
  ctx->x0 = reinterpret_cast<float *>(base + sec.x0);
  ctx->u = reinterpret_cast<float *>(base + sec.u);
  ctx->h = reinterpret_cast<float *>(base + sec.h);
  ctx->v = cfg->base == SLOWMO_ADAM ? reinterpret_cast<float *>(base + sec.v) : nullptr;
  ctx->d_xtab_t = reinterpret_cast<float **>(base + sec.xtab_t);
  ctx->d_slots = reinterpret_cast<SlotInfo *>(base + sec.slots);
  ctx->d_tensors = reinterpret_cast<TensorInfo *>(base + sec.tensors);
  ctx->d_ltiles = reinterpret_cast<TileRef *>(base + sec.ltiles);
  ctx->d_otiles = reinterpret_cast<TileRef *>(base + sec.otiles);
  ctx->n_ltiles = static_cast<int32_t>(n_ltiles);
  ctx->n_otiles = static_cast<int32_t>(n_otiles);
  ctx->d_btiles = reinterpret_cast<TileRef *>(base + sec.btiles);
  ctx->d_rtiles = reinterpret_cast<TileRef *>(base + sec.rtiles);

#define CREATE_HIP(call, what)              \
  do {                                      \
    hipError_t e_ = (call);                 \
    if (e_ != hipSuccess) {                 \
      release(ctx);                         \
      return fail_hip(nullptr, e_, what);   \
    }                                       \
  } while (0)

  CREATE_HIP(ctx->gtab.init(base, sec.gtab, n_ptr * sizeof(void *)), "gradient-pointer ring");
  CREATE_HIP(ctx->mixtab.init(base, sec.mixtab, mixtab_bytes(m)), "mixing-table ring");
  CREATE_HIP(ctx->ztab.init(base, sec.ztab, ztab_bytes(m, n_tensors)), "de-bias table ring");
  ctx->w.assign(m, 1.0f);
  // set-up for the entry point that may not allocate: this device's address of
  // the library's static scratch array (the create call runs with it current)
  CREATE_HIP(static_scratch(ctx->device, &ctx->static_table), "address of the static scratch array");

  // device tables
  const Layout &L = ctx->layout;
  std::vector<SlotInfo> &slots = ctx->slots;
  std::vector<TensorInfo> &tinfo = ctx->tinfo;
  slots.resize(n_ptr);
  tinfo.resize(n_tensors);
  std::vector<float *> xtab_t(n_ptr);
  for (int32_t j = 0; j < n_tensors; ++j) tinfo[j] = {L.arena_off[j], numel[j], 0, 1.0f, cfg->weight_decay};
  for (int32_t w = 0; w < m; ++w) {
    for (int32_t j = 0; j < n_tensors; ++j) {
      const size_t slot = static_cast<size_t>(w) * n_tensors + j;
      slots[slot] = {params[slot], static_cast<int64_t>(w) * L.d_pad + L.arena_off[j], numel[j],
                     cfg->weight_decay, 1.0f};
      xtab_t[static_cast<size_t>(j) * m + w] = params[slot];
      if (numel[j] && (reinterpret_cast<uintptr_t>(params[slot]) & 15)) {
        tinfo[j].unaligned = 1;
        ctx->params_aligned = false;
      }
    }
  }
  // tiles in launch order: worker-major, tensors in list order, pieces ascending
  std::vector<TileRef> lt, ot;
  lt.reserve(static_cast<size_t>(n_ltiles));
  ot.reserve(static_cast<size_t>(n_otiles));
  for (int32_t w = 0; w < m; ++w)
    for (int32_t j = 0; j < n_tensors; ++j)
      for (int64_t k = 0; k * kLocalTile < numel[j]; ++k)
        lt.push_back({w * n_tensors + j, static_cast<int32_t>(k)});
  for (int32_t j = 0; j < n_tensors; ++j)
    for (int64_t k = 0; k * kOuterTile < numel[j]; ++k) ot.push_back({j, static_cast<int32_t>(k)});
  if (!lt.empty())
    CREATE_HIP(hipMemcpyAsync(ctx->d_ltiles, lt.data(), lt.size() * sizeof(TileRef),
                              hipMemcpyHostToDevice, stream),
               "upload of the local-step tiles");
  if (!ot.empty())
    CREATE_HIP(hipMemcpyAsync(ctx->d_otiles, ot.data(), ot.size() * sizeof(TileRef),
                              hipMemcpyHostToDevice, stream),
               "upload of the outer-step tiles");
  std::vector<TileRef> bt, rt;
  if (ctx->tune.big_tiles) {
    constexpr int64_t per_big = kBigTile / kOuterTile;
    for (int32_t j = 0; j < n_tensors; ++j) {
      const int64_t n_big = tinfo[j].unaligned ? 0 : numel[j] / kBigTile;
      for (int64_t k = 0; k < n_big; ++k) bt.push_back({j, static_cast<int32_t>(k)});
      for (int64_t k = n_big * per_big; k * kOuterTile < numel[j]; ++k)
        rt.push_back({j, static_cast<int32_t>(k)});
    }
  }
  if (bt.empty() || (big < 0 && static_cast<int64_t>(bt.size()) < kBigMinTiles)) {
    ctx->d_rtiles = ctx->d_otiles;
    ctx->n_rtiles = ctx->n_otiles;
  } else {
    CREATE_HIP(hipMemcpyAsync(ctx->d_btiles, bt.data(), bt.size() * sizeof(TileRef),
                              hipMemcpyHostToDevice, stream),
               "upload of the big tiles");
    if (!rt.empty())
      CREATE_HIP(hipMemcpyAsync(ctx->d_rtiles, rt.data(), rt.size() * sizeof(TileRef),
                                hipMemcpyHostToDevice, stream),
                 "upload of the tiles the big ones leave over");
    ctx->n_btiles = static_cast<int32_t>(bt.size());
    ctx->n_rtiles = static_cast<int32_t>(rt.size());
  }
  CREATE_HIP(hipMemcpyAsync(ctx->d_tensors, tinfo.data(), tinfo.size() * sizeof(TensorInfo),
                            hipMemcpyHostToDevice, stream),
             "upload of the tensor table");
  CREATE_HIP(hipMemcpyAsync(ctx->d_slots, slots.data(), n_ptr * sizeof(SlotInfo),
                            hipMemcpyHostToDevice, stream),
             "upload of the slot table");
  CREATE_HIP(hipMemcpyAsync(ctx->d_xtab_t, xtab_t.data(), n_ptr * sizeof(float *),
                            hipMemcpyHostToDevice, stream),
             "upload of the replica pointers");

  // u_0 = 0, h = v = 0 (Algorithm 1, "Input"; Table C.1 caption)
  const size_t arena = static_cast<size_t>(L.d_pad) * sizeof(float);
  const size_t outer_copies = cfg->no_average ? static_cast<size_t>(m) : 1;
  CREATE_HIP(hipMemsetAsync(ctx->x0, 0, arena * outer_copies, stream), "clearing x0");
  CREATE_HIP(hipMemsetAsync(ctx->u, 0, arena * outer_copies, stream), "clearing u");
  CREATE_HIP(hipMemsetAsync(ctx->h, 0, arena * m, stream), "clearing h");
  if (ctx->v) CREATE_HIP(hipMemsetAsync(ctx->v, 0, arena * m, stream), "clearing v");
  // common starting point x_{0,0}: worker 0's replica, into x0 and every other replica
  {
    OuterArgs ia{};
    ia.tiles = ctx->d_otiles;
    ia.tensors = ctx->d_tensors;
    ia.xtab_t = ctx->d_xtab_t;
    ia.ntiles = ctx->n_otiles;
    ia.m = m;
    ia.x0 = ctx->x0;
    ia.d_pad = L.d_pad;
    CREATE_HIP(launch_init_broadcast(ia, static_cast<int32_t>(outer_copies), ctx->tune, stream),
               "copy of x_{0,0} into x0 and the replicas");
  }
  // the host-side tables above go out of scope: wait for their uploads
  CREATE_HIP(hipStreamSynchronize(stream), "hipStreamSynchronize");
#undef CREATE_HIP

  *out = ctx;
  return SLOWMO_OK;
}

extern "C++" {
namespace {

// Checks the arguments of a local step, uploads the gradient-pointer table if
// it changed and fills the kernel arguments.  *all_aligned tells whether every
// gradient pointer allows 16-byte vector loads.
slowmo_status prepare_local(slowmo_ctx *ctx, const void *const *grads, float lr,
                            hipStream_t stream, LocalArgs *out, bool *all_aligned) {
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!grads) return fail(ctx, SLOWMO_ERR_ARG, "grads is NULL");
  if (!finite_pos(lr)) return fail(ctx, SLOWMO_ERR_ARG, "lr must be finite and > 0");
  if (ctx->k >= ctx->cfg.tau)
    return fail(ctx, SLOWMO_ERR_STATE, "tau local steps already taken: slowmo_outer_step is due");
  const slowmo_config &c = ctx->cfg;
  const size_t n_ptr = static_cast<size_t>(c.m) * ctx->n_tensors;
  const size_t gsize = c.grad_dtype == SLOWMO_BF16 ? 2 : 4;
  uintptr_t low_bits = 0;
  for (size_t i = 0; i < n_ptr; ++i) {
    if (ctx->numel[i % ctx->n_tensors] == 0) continue;
    if (!grads[i]) return fail(ctx, SLOWMO_ERR_ARG, "a gradient pointer is NULL");
    if (reinterpret_cast<uintptr_t>(grads[i]) % gsize)
      return fail(ctx, SLOWMO_ERR_ALIGN, "a gradient pointer is not aligned to its element size");
    low_bits |= reinterpret_cast<uintptr_t>(grads[i]);
  }
  *all_aligned = (low_bits & (4 * gsize - 1)) == 0;

  // gradient-pointer table: reuse a device copy if one of the recent calls had these pointers
  int slot = ctx->gtab.find(grads, n_ptr * sizeof(void *));
  if (slot < 0) {
    hipError_t e = hipSuccess;
    if (ctx->check_pointers >= 2) {
      for (size_t i = 0; i < n_ptr; ++i) {
        const int64_t n = ctx->numel[i % ctx->n_tensors];
        if (n && slowmo_check_device_range(grads[i], static_cast<size_t>(n) * gsize) != SLOWMO_OK)
          return fail(ctx, SLOWMO_ERR_ARG, "gradient tensor: " + g_err);
      }
    }
    slot = ctx->gtab.upload(grads, n_ptr * sizeof(void *), stream, &e);
    if (slot < 0) return fail_hip(ctx, e, "upload of the gradient pointers");
  }

  LocalArgs a{};
  a.tiles = ctx->d_ltiles;
  a.slots = ctx->d_slots;
  a.ntiles = ctx->n_ltiles;
  a.gtab = static_cast<const void *const *>(ctx->gtab.d[slot]);
  a.h = ctx->h;
  a.v = ctx->v;
  a.lr = lr;
  a.wd = c.weight_decay;
  a.mu = c.momentum;
  if (c.base == SLOWMO_ADAM) {
    const double l_next = static_cast<double>(ctx->l + 1);
    a.b1 = c.beta1;
    a.b2 = c.beta2;
    a.omb1 = 1.0f - c.beta1;
    a.omb2 = 1.0f - c.beta2;
    a.eps = c.eps;
    // 1 / (1 - beta^l), l counting this step, in fp64, rounded once
    a.rc1 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(c.beta1), l_next)));
    a.rc2 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(c.beta2), l_next)));
  }
  *out = a;
  return SLOWMO_OK;
}

void finish_local(slowmo_ctx *ctx) {
  ctx->k += 1;
  ctx->l += 1;
  ctx->buffers_zero = false;
}

void finish_outer(slowmo_ctx *ctx) {
  ctx->k = 0;
  ctx->t += 1;
  // after the exact average every worker holds the same, unbiased point again
  if (!ctx->cfg.no_average) std::fill(ctx->w.begin(), ctx->w.end(), 1.0f);
  if (ctx->cfg.policy == SLOWMO_BUF_RESET) {  // Algorithm 1 line 2 of the next outer iteration
    ctx->buffers_zero = true;
    ctx->l = 0;
  }
}

}  // namespace
}  // extern "C++"

slowmo_status slowmo_local_step(slowmo_ctx *ctx, const void *const *grads, float lr,
                                void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  LocalArgs a{};
  bool aligned = false;
  slowmo_status st = prepare_local(ctx, grads, lr, stream, &a, &aligned);
  if (st != SLOWMO_OK) return st;
  const slowmo_config &c = ctx->cfg;
  // Under the reset policy the buffers written by the last step of an outer
  // iteration are discarded before they are read again: skip those stores.
  const bool dead_after = c.policy == SLOWMO_BUF_RESET && ctx->k == c.tau - 1;
  hipError_t e = guarded(ctx, [&] {
    return launch_local_step(a, c.base, c.grad_dtype == SLOWMO_BF16, ctx->buffers_zero, dead_after,
                             ctx->tune, stream);
  });
  if (e != hipSuccess) return fail_hip(ctx, e, "local-step kernel launch");
  finish_local(ctx);
  return SLOWMO_OK;
}

extern "C++" {
namespace {

OuterArgs outer_args(const slowmo_ctx *ctx, float lr) {
  const slowmo_config &c = ctx->cfg;
  OuterArgs a{};
  a.tiles = ctx->d_otiles;
  a.tensors = ctx->d_tensors;
  a.ntiles = ctx->n_otiles;
  a.xtab_t = ctx->d_xtab_t;
  a.m = c.m;
  a.x0 = ctx->x0;
  a.u = ctx->u;
  a.lr = lr;
  a.alpha = c.alpha;
  a.beta = c.beta;
  a.m_f = static_cast<float>(c.m);
  a.d_pad = ctx->layout.d_pad;
  if (c.policy == SLOWMO_BUF_AVERAGE) {  // Algorithm 1 line 2 of the next outer iteration
    a.avg_h = ctx->h;
    a.avg_v = ctx->v;  // nullptr unless Adam
  }
  return a;
}

// Lines 6-8 and the copy into the replicas.  *launched: kernels of the same
// call already issued (a failure is then a failure halfway).
slowmo_status run_outer(slowmo_ctx *ctx, float lr, int *launched, hipStream_t stream) {
  const slowmo_config &c = ctx->cfg;
  if (c.no_average) {  // Section 6: lines 7-8 per worker, no line 6
    OuterNoAvgArgs na{};
    na.tiles = ctx->d_ltiles;
    na.slots = ctx->d_slots;
    na.ntiles = ctx->n_ltiles;
    na.x0 = ctx->x0;
    na.u = ctx->u;
    na.lr = lr;
    na.alpha = c.alpha;
    na.beta = c.beta;
    const hipError_t e =
        guarded(ctx, [&] { return launch_outer_noavg_step(na, ctx->tune, stream); });
    if (e != hipSuccess)
      return *launched ? fail_midway(ctx, e, "outer-step kernel launch")
                       : fail_hip(ctx, e, "outer-step kernel launch");
    ++*launched;
    return SLOWMO_OK;
  }
  OuterArgs a = outer_args(ctx, lr);
  auto with = [&](const TileRef *tiles, int32_t n) {
    a.tiles = tiles;
    a.ntiles = n;
    return a;
  };
  // the big-tile kernel has no buffer average
  const bool use_big = ctx->n_btiles > 0 && ctx->big_outer && !a.avg_h;
  return run_tiled(
      ctx, use_big, launched, "outer-step kernel launch",
      [&](const TileRef *t, int32_t n) { return launch_outer_big(with(t, n), ctx->tune, stream); },
      [&](const TileRef *t, int32_t n) { return launch_outer_step(with(t, n), ctx->tune, stream); });
}

}  // namespace
}  // extern "C++"

slowmo_status slowmo_outer_step(slowmo_ctx *ctx, float lr, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!finite_pos(lr)) return fail(ctx, SLOWMO_ERR_ARG, "lr must be finite and > 0");
  if (ctx->k != ctx->cfg.tau)
    return fail(ctx, SLOWMO_ERR_STATE, "the outer step needs exactly tau local steps before it");
  int launched = 0;
  const slowmo_status st = run_outer(ctx, lr, &launched, static_cast<hipStream_t>(stream_));
  if (st != SLOWMO_OK) return st;
  finish_outer(ctx);
  return SLOWMO_OK;
}

slowmo_status slowmo_local_outer_step(slowmo_ctx *ctx, const void *const *grads, float lr,
                                      float outer_lr, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!finite_pos(outer_lr)) return fail(ctx, SLOWMO_ERR_ARG, "outer_lr must be finite and > 0");
  if (ctx->k != ctx->cfg.tau - 1)
    return fail(ctx, SLOWMO_ERR_STATE,
                "the fused step is the LAST local step of an outer iteration: tau-1 local steps "
                "must have been taken");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  LocalArgs a{};
  bool aligned = false;
  slowmo_status st = prepare_local(ctx, grads, lr, stream, &a, &aligned);
  if (st != SLOWMO_OK) return st;
  const slowmo_config &c = ctx->cfg;
  const bool bf16 = c.grad_dtype == SLOWMO_BF16;
  if (c.no_average || !aligned || !ctx->params_aligned || !ctx->tune.fuse_last) {
    // same two kernels as the separate calls
    hipError_t e = guarded(ctx, [&] {
      return launch_local_step(a, c.base, bf16, ctx->buffers_zero, c.policy == SLOWMO_BUF_RESET,
                               ctx->tune, stream);
    });
    if (e != hipSuccess) return fail_hip(ctx, e, "local-step kernel launch");
    int launched = 1;
    st = run_outer(ctx, outer_lr, &launched, stream);
    if (st != SLOWMO_OK) return st;
  } else {
    OuterArgs o = outer_args(ctx, outer_lr);
    auto with = [&](const TileRef *tiles, int32_t n) {
      o.tiles = tiles;
      o.ntiles = n;
      return o;
    };
    int launched = 0;
    // big tiles pay when the buffers of this step are dropped ("reset"); stores of
    // every worker's buffers inside the walk cost them their gain (measured: 2-10 %
    // slower than single-wave tiles under "maintain"), and the buffer average does
    // not fit their registers
    const bool use_big =
        ctx->n_btiles > 0 && (c.policy == SLOWMO_BUF_RESET ||
                              (ctx->big_forced && c.policy == SLOWMO_BUF_MAINTAIN));
    st = run_tiled(
        ctx, use_big, &launched, "fused local+outer kernel launch",
        [&](const TileRef *t, int32_t n) {
          return launch_local_outer_big(a, with(t, n), ctx->n_tensors, c.base, bf16,
                                        ctx->buffers_zero, c.policy, ctx->tune, stream);
        },
        [&](const TileRef *t, int32_t n) {
          return launch_local_outer_step(a, with(t, n), ctx->n_tensors, c.base, bf16,
                                         ctx->buffers_zero, c.policy, ctx->tune, stream);
        });
    if (st != SLOWMO_OK) return st;
  }
  finish_local(ctx);
  finish_outer(ctx);
  return SLOWMO_OK;
}

slowmo_status slowmo_lr_step_decay(float base_lr, float start_lr, int64_t warmup_steps,
                                   const int64_t *milestones, int32_t n_milestones, float factor,
                                   int64_t step, float *lr_out) {
  if (!lr_out || step < 0 || warmup_steps < 0 || n_milestones < 0 ||
      (n_milestones > 0 && !milestones))
    return fail(nullptr, SLOWMO_ERR_ARG, "bad arguments");
  if (!finite_pos(base_lr) || !std::isfinite(start_lr) || start_lr < 0.f ||
      !std::isfinite(factor) || factor <= 0.f || factor > 1.f)
    return fail(nullptr, SLOWMO_ERR_ARG,
                "base_lr must be finite and > 0, start_lr finite and >= 0, factor in (0, 1]");
  for (int32_t i = 0; i < n_milestones; ++i)
    if (milestones[i] < 0 || (i > 0 && milestones[i] <= milestones[i - 1]))
      return fail(nullptr, SLOWMO_ERR_ARG, "milestones must be >= 0 and ascend");
  double lr;
  if (step < warmup_steps) {  // Section 4: linear warm-up
    lr = static_cast<double>(start_lr) + (static_cast<double>(base_lr) - start_lr) *
                                             static_cast<double>(step) / static_cast<double>(warmup_steps);
  } else {                    // ... then one factor per milestone passed
    lr = base_lr;
    for (int32_t i = 0; i < n_milestones && milestones[i] <= step; ++i) lr *= static_cast<double>(factor);
  }
  *lr_out = static_cast<float>(lr);
  return SLOWMO_OK;
}

slowmo_status slowmo_lr_inverse_sqrt(float peak_lr, float init_lr, int64_t warmup_steps,
                                     int64_t step, float *lr_out) {
  if (!lr_out || step < 0 || warmup_steps < 0) return fail(nullptr, SLOWMO_ERR_ARG, "bad arguments");
  if (!finite_pos(peak_lr) || !std::isfinite(init_lr) || init_lr < 0.f)
    return fail(nullptr, SLOWMO_ERR_ARG, "peak_lr must be finite and > 0, init_lr finite and >= 0");
  double lr;
  if (step < warmup_steps) {  // Appendix A.3: linear warm-up
    lr = static_cast<double>(init_lr) + (static_cast<double>(peak_lr) - init_lr) *
                                            static_cast<double>(step) / static_cast<double>(warmup_steps);
  } else if (step == 0) {
    lr = peak_lr;
  } else {                    // ... then proportional to 1 / sqrt(step)
    lr = peak_lr * std::sqrt(static_cast<double>(warmup_steps) / static_cast<double>(step));
  }
  *lr_out = static_cast<float>(lr);
  return SLOWMO_OK;
}

slowmo_status slowmo_expgraph_in_peers(int32_t m, int64_t step, int32_t *in_peer) {
  if (m < 1 || step < 0 || !in_peer) return fail(nullptr, SLOWMO_ERR_ARG, "bad arguments");
  if (m == 1) {
    in_peer[0] = 0;
    return SLOWMO_OK;
  }
  int n_hops = 1;  // hops 2^0 .. 2^floor(log2(m-1))
  while ((int64_t(1) << n_hops) <= m - 1) ++n_hops;
  const int64_t hop = int64_t(1) << (step % n_hops);
  for (int32_t i = 0; i < m; ++i) in_peer[i] = static_cast<int32_t>(((i - hop) % m + m) % m);
  return SLOWMO_OK;
}

extern "C++" {
namespace {

// Ranges [first, last) of the mixing entries to run as separate launches: one
// per connected group of workers (a launch then walks only that group's
// replicas per tile, and fewer memory regions visited side by side measure
// faster), consecutive groups merged when there are more than kMaxMixLaunches.
constexpr size_t kMaxMixLaunches = 32;
std::vector<std::pair<int32_t, int32_t>> mix_launch_ranges(const std::vector<MixEntry> &seq) {
  std::vector<int32_t> starts;
  for (size_t i = 0; i < seq.size(); ++i)
    if (seq[i].flags & kMixGroupStart) starts.push_back(static_cast<int32_t>(i));
  std::vector<std::pair<int32_t, int32_t>> out;
  const size_t per = (starts.size() + kMaxMixLaunches - 1) / kMaxMixLaunches;  // groups per launch
  for (size_t g = 0; g < starts.size(); g += per) {
    const size_t g_end = std::min(g + per, starts.size());
    out.push_back({starts[g], g_end < starts.size() ? starts[g_end] : static_cast<int32_t>(seq.size())});
  }
  return out;
}

// The mixing order of one call, planned on the host and uploaded; nothing has
// been launched yet when stage_mix returns.
struct StagedMix {
  std::vector<std::pair<int32_t, int32_t>> ranges;  // one kernel launch each
  const MixEntry *d_seq = nullptr;
};

slowmo_status stage_mix(slowmo_ctx *ctx, const int32_t *in_peer, bool with_idle, hipStream_t stream,
                        StagedMix *out) {
  std::vector<MixEntry> seq;
  std::vector<float> share;
  plan_mix(ctx->cfg.m, in_peer, seq, share, with_idle);
  if (seq.empty() || ctx->n_otiles == 0) return SLOWMO_OK;  // nothing to launch
  hipError_t e = hipSuccess;
  const int slot = ctx->mixtab.upload(seq.data(), seq.size() * sizeof(MixEntry), stream, &e);
  if (slot < 0) return fail_hip(ctx, e, "upload of the mixing entries");
  out->d_seq = static_cast<const MixEntry *>(ctx->mixtab.d[slot]);
  out->ranges = mix_launch_ranges(seq);
  return SLOWMO_OK;
}

MixArgs mix_args(const slowmo_ctx *ctx) {
  MixArgs a{};
  a.tiles = ctx->d_otiles;
  a.tensors = ctx->d_tensors;
  a.xtab_t = ctx->d_xtab_t;
  a.ntiles = ctx->n_otiles;
  a.m = ctx->cfg.m;
  return a;
}

// Launches the gossip kernel once per group.  `launched`: kernels of this call
// already issued before (a failure is then a failure halfway).
slowmo_status run_mix(slowmo_ctx *ctx, const StagedMix &sm, int launched, hipStream_t stream) {
  MixArgs a = mix_args(ctx);
  for (const auto &r : sm.ranges) {
    a.seq = sm.d_seq + r.first;
    a.len = r.second - r.first;
    const hipError_t e = guarded(ctx, [&] { return launch_mix_step(a, ctx->tune, stream); });
    if (e != hipSuccess)
      return launched ? fail_midway(ctx, e, "mixing kernel launch")
                      : fail_hip(ctx, e, "mixing kernel launch");
    ++launched;
  }
  return SLOWMO_OK;
}

bool check_in_peer(const slowmo_ctx *ctx, const int32_t *in_peer) {
  for (int32_t i = 0; i < ctx->cfg.m; ++i)
    if (in_peer[i] < 0 || in_peer[i] >= ctx->cfg.m) return false;
  return true;
}

// the push-sum weights mix with the same P, in the same arithmetic as the replicas
void mix_weights(slowmo_ctx *ctx, const int32_t *in_peer) {
  const int32_t m = ctx->cfg.m;
  std::vector<int32_t> outdeg(m, 0);
  for (int32_t i = 0; i < m; ++i)
    if (in_peer[i] != i) ++outdeg[in_peer[i]];
  std::vector<float> w_new(m);
  for (int32_t i = 0; i < m; ++i) {
    const int32_t j = in_peer[i];
    float v = (1.0f / static_cast<float>(1 + outdeg[i])) * ctx->w[i];
    if (j != i) v = v + (1.0f / static_cast<float>(1 + outdeg[j])) * ctx->w[j];
    w_new[i] = v;
  }
  ctx->w.swap(w_new);
}

}  // namespace
}  // extern "C++"

slowmo_status slowmo_mix_step(slowmo_ctx *ctx, const int32_t *in_peer, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!in_peer) return fail(ctx, SLOWMO_ERR_ARG, "in_peer is NULL");
  if (!check_in_peer(ctx, in_peer))
    return fail(ctx, SLOWMO_ERR_ARG, "in_peer entries must lie in 0..m-1");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  StagedMix sm;
  slowmo_status st = stage_mix(ctx, in_peer, /*with_idle=*/false, stream, &sm);
  if (st == SLOWMO_OK) st = run_mix(ctx, sm, 0, stream);
  if (st != SLOWMO_OK) return st;
  mix_weights(ctx, in_peer);
  return SLOWMO_OK;
}

slowmo_status slowmo_local_mix_step(slowmo_ctx *ctx, const void *const *grads, float lr,
                                    const int32_t *in_peer, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!in_peer) return fail(ctx, SLOWMO_ERR_ARG, "in_peer is NULL");
  if (!check_in_peer(ctx, in_peer))
    return fail(ctx, SLOWMO_ERR_ARG, "in_peer entries must lie in 0..m-1");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  LocalArgs a{};
  bool aligned = false;
  slowmo_status st = prepare_local(ctx, grads, lr, stream, &a, &aligned);
  if (st != SLOWMO_OK) return st;
  const slowmo_config &c = ctx->cfg;
  const bool bf16 = c.grad_dtype == SLOWMO_BF16;
  const bool two_kernels = !aligned || !ctx->params_aligned || !ctx->tune.fuse_mix || ctx->n_otiles == 0;
  // both tables are on their way to the device before the first kernel is launched
  StagedMix sm;
  st = stage_mix(ctx, in_peer, /*with_idle=*/!two_kernels, stream, &sm);
  if (st != SLOWMO_OK) return st;
  if (two_kernels) {
    // same kernels as the separate calls
    const bool dead_after = c.policy == SLOWMO_BUF_RESET && ctx->k == c.tau - 1;
    const hipError_t e = guarded(ctx, [&] {
      return launch_local_step(a, c.base, bf16, ctx->buffers_zero, dead_after, ctx->tune, stream);
    });
    if (e != hipSuccess) return fail_hip(ctx, e, "local-step kernel launch");
    st = run_mix(ctx, sm, 1, stream);
    if (st != SLOWMO_OK) return st;
  } else {
    MixArgs x = mix_args(ctx);
    int launched = 0;
    for (const auto &r : sm.ranges) {
      x.seq = sm.d_seq + r.first;
      x.len = r.second - r.first;
      const hipError_t e = guarded(ctx, [&] {
        return launch_local_mix_step(a, x, ctx->layout.d_pad, ctx->n_tensors, c.base, bf16,
                                     ctx->buffers_zero, ctx->tune, stream);
      });
      if (e != hipSuccess)
        return launched ? fail_midway(ctx, e, "fused local+mixing kernel launch")
                        : fail_hip(ctx, e, "fused local+mixing kernel launch");
      ++launched;
    }
  }
  // counters and weights move only after the last launch was accepted
  finish_local(ctx);
  mix_weights(ctx, in_peer);
  return SLOWMO_OK;
}

int32_t slowmo_plan_mix(int32_t m, const int32_t *in_peer, slowmo_mix_entry *out) {
  static_assert(sizeof(slowmo_mix_entry) == sizeof(MixEntry), "public and internal entry differ");
  static_assert(SLOWMO_MIX_SAVE(5 << 6) == mix_save(5 << 6) && mix_save(5 << 6) == 5 &&
                    SLOWMO_MIX_OWN_SAVED(5 << 9) == mix_own_saved(5 << 9) &&
                    mix_own_saved(5 << 9) == 5 &&
                    SLOWMO_MIX_SOURCE_SAVED(5 << 12) == mix_src_saved(5 << 12) &&
                    mix_src_saved(5 << 12) == 5 && SLOWMO_MIX_SAVED_REGISTERS == kMixSaved &&
                    SLOWMO_MIX_GROUP_START == kMixGroupStart,
                "public and internal flags differ");
  if (m < 1 || m > SLOWMO_MAX_WORKERS || !in_peer || !out) return -1;
  for (int32_t i = 0; i < m; ++i)
    if (in_peer[i] < 0 || in_peer[i] >= m) return -1;
  std::vector<MixEntry> seq;
  std::vector<float> share;
  plan_mix(m, in_peer, seq, share);
  for (size_t i = 0; i < seq.size(); ++i)
    out[i] = {seq[i].node, seq[i].src, seq[i].a, seq[i].b, seq[i].flags, 0};
  return static_cast<int32_t>(seq.size());
}

slowmo_status slowmo_get_pushsum_weights(const slowmo_ctx *ctx, float *w) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (!w) return fail(const_cast<slowmo_ctx *>(ctx), SLOWMO_ERR_ARG, "w is NULL");
  std::memcpy(w, ctx->w.data(), ctx->w.size() * sizeof(float));
  return SLOWMO_OK;
}

extern "C++" {
namespace {

// z = x / w for every worker.  The table the kernel reads (m * n_tensors
// destination pointers, then the m weights) is written straight into a pinned
// staging buffer of the context and sent to `table_dev` (NULL: the staging
// slot's own device copy inside the workspace).  Allocates nothing.
slowmo_status debias_into(slowmo_ctx *ctx, float *const *z, void *table_dev, hipStream_t stream) {
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!z) return fail(ctx, SLOWMO_ERR_ARG, "z is NULL");
  const int32_t m = ctx->cfg.m, nt = ctx->n_tensors;
  const size_t n_ptr = static_cast<size_t>(m) * nt;
  for (size_t i = 0; i < n_ptr; ++i) {
    if (ctx->numel[i % nt] == 0) continue;
    if (!z[i]) return fail(ctx, SLOWMO_ERR_ARG, "a destination pointer is NULL");
    if (reinterpret_cast<uintptr_t>(z[i]) % sizeof(float))
      return fail(ctx, SLOWMO_ERR_ALIGN, "a destination pointer is not 4-byte aligned");
  }
  if (ctx->check_pointers >= 2) {
    for (size_t i = 0; i < n_ptr; ++i) {
      const int64_t n = ctx->numel[i % nt];
      if (n && slowmo_check_device_range(z[i], static_cast<size_t>(n) * sizeof(float)) != SLOWMO_OK)
        return fail(ctx, SLOWMO_ERR_ARG, "destination tensor: " + g_err);
    }
  }
  if (ctx->n_ltiles == 0) return SLOWMO_OK;
  hipError_t e = hipSuccess;
  const int slot = ctx->ztab.stage(&e);
  if (slot < 0) return fail_hip(ctx, e, "waiting for a staging buffer of the de-bias table");
  char *table = static_cast<char *>(ctx->ztab.h[slot]);
  std::memcpy(table, z, n_ptr * sizeof(void *));
  std::memcpy(table + n_ptr * sizeof(void *), ctx->w.data(), m * sizeof(float));
  e = ctx->ztab.send(slot, ztab_bytes(m, nt), table_dev, stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "upload of the de-bias table");
  const char *dev = static_cast<const char *>(table_dev ? table_dev : ctx->ztab.d[slot]);
  DebiasArgs a{};
  a.tiles = ctx->d_ltiles;
  a.slots = ctx->d_slots;
  a.ztab = reinterpret_cast<float *const *>(dev);
  a.w = reinterpret_cast<const float *>(dev + n_ptr * sizeof(void *));
  a.ntiles = ctx->n_ltiles;
  a.n_tensors = nt;
  e = guarded(ctx, [&] { return launch_debias(a, ctx->tune, stream); });
  if (e != hipSuccess) return fail_hip(ctx, e, "de-bias kernel launch");
  return SLOWMO_OK;
}

}  // namespace
}  // extern "C++"

slowmo_status slowmo_debias(slowmo_ctx *ctx, float *const *z, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  return debias_into(ctx, z, nullptr, static_cast<hipStream_t>(stream_));
}

slowmo_status slowmo_debias_static(slowmo_ctx *ctx, float *const *z, void *stream_) {
  static_assert(SLOWMO_STATIC_MAX_POINTERS == kStaticMaxPointers, "header and library disagree");
  static_assert(SLOWMO_MAX_WORKERS <= kStaticMaxWorkers, "weights must fit the static table");
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  const size_t n_ptr = static_cast<size_t>(ctx->cfg.m) * ctx->n_tensors;
  if (n_ptr > kStaticMaxPointers)
    return fail(ctx, SLOWMO_ERR_NOMEM,
                "m * n_tensors = " + std::to_string(n_ptr) + " exceeds SLOWMO_STATIC_MAX_POINTERS = " +
                    std::to_string(kStaticMaxPointers) + ": use slowmo_debias");
  int current = -1;
  const hipError_t e = hipGetDevice(&current);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipGetDevice");
  if (current != ctx->device)
    return fail(ctx, SLOWMO_ERR_STATE, "the context's device is not the current device");
  return debias_into(ctx, z, ctx->static_table, static_cast<hipStream_t>(stream_));
}

slowmo_status slowmo_set_tensor_hparams(slowmo_ctx *ctx, const float *weight_decay,
                                        const float *lr_scale, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  const int32_t nt = ctx->n_tensors, m = ctx->cfg.m;
  for (int32_t j = 0; j < nt; ++j) {
    if (weight_decay && !(std::isfinite(weight_decay[j]) && weight_decay[j] >= 0.f))
      return fail(ctx, SLOWMO_ERR_ARG, "weight_decay entries must be finite and >= 0");
    if (lr_scale && !finite_pos(lr_scale[j]))
      return fail(ctx, SLOWMO_ERR_ARG, "lr_scale entries must be finite and > 0");
  }
  // build the new tables aside; they replace the context's only if the upload succeeds
  std::vector<SlotInfo> slots = ctx->slots;
  std::vector<TensorInfo> tinfo = ctx->tinfo;
  for (int32_t j = 0; j < nt; ++j) {
    if (lr_scale) tinfo[j].lr_scale = lr_scale[j];
    if (weight_decay) tinfo[j].wd = weight_decay[j];
    for (int32_t w = 0; w < m; ++w) {
      SlotInfo &s = slots[static_cast<size_t>(w) * nt + j];
      if (weight_decay) s.wd = weight_decay[j];
      if (lr_scale) s.lr_scale = lr_scale[j];
    }
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  hipError_t e = hipMemcpyAsync(ctx->d_slots, slots.data(), slots.size() * sizeof(SlotInfo),
                                hipMemcpyHostToDevice, stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(ctx->d_tensors, tinfo.data(), tinfo.size() * sizeof(TensorInfo),
                       hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);  // the tables above go out of scope
  if (e != hipSuccess) return fail_hip(ctx, e, "upload of the per-tensor hyper-parameters");
  ctx->slots.swap(slots);
  ctx->tinfo.swap(tinfo);
  return SLOWMO_OK;
}

extern "C++" {
namespace {

// Header of an exported state blob (256 bytes), followed by the m push-sum
// weights (padded to a multiple of 256 bytes) and the x0, u, h, v arenas
// exactly as they lie in the workspace.
struct BlobHeader {
  char magic[8];
  uint32_t version;
  int32_t m, n_tensors, base, no_average, k, buffers_zero, reserved;
  int64_t d, d_pad, t, l;
  char pad_[256 - 8 - 4 * 8 - 8 * 4];
};
static_assert(sizeof(BlobHeader) == 256, "BlobHeader layout");
constexpr uint32_t kBlobVersion = 2;
constexpr char kBlobMagic[8] = {'S', 'L', 'O', 'W', 'M', 'O', 'S', 'T'};

struct BlobParts {
  size_t arena, outer_copies, n_v, weights, total;
};
BlobParts blob_parts(const slowmo_ctx *ctx) {
  BlobParts p;
  p.arena = static_cast<size_t>(ctx->layout.d_pad) * sizeof(float);
  p.outer_copies = ctx->cfg.no_average ? ctx->cfg.m : 1;
  p.n_v = ctx->v ? ctx->cfg.m : 0;
  p.weights = round_up(static_cast<size_t>(ctx->cfg.m) * sizeof(float), 256);
  p.total = sizeof(BlobHeader) + p.weights + p.arena * (2 * p.outer_copies + ctx->cfg.m + p.n_v);
  return p;
}

}  // namespace
}  // extern "C++"

size_t slowmo_export_bytes(const slowmo_ctx *ctx) { return ctx ? blob_parts(ctx).total : 0; }

slowmo_status slowmo_export_state(slowmo_ctx *ctx, void *dst, size_t bytes, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (!dst) return fail(ctx, SLOWMO_ERR_ARG, "dst is NULL");
  const BlobParts p = blob_parts(ctx);
  if (bytes < p.total) return fail(ctx, SLOWMO_ERR_NOMEM, "destination smaller than slowmo_export_bytes()");
  BlobHeader hd{};
  std::memcpy(hd.magic, kBlobMagic, 8);
  hd.version = kBlobVersion;
  hd.m = ctx->cfg.m;
  hd.n_tensors = ctx->n_tensors;
  hd.base = ctx->cfg.base;
  hd.no_average = ctx->cfg.no_average;
  hd.d = ctx->layout.d;
  hd.d_pad = ctx->layout.d_pad;
  hd.t = ctx->t;
  hd.l = ctx->l;
  hd.k = ctx->k;
  hd.buffers_zero = ctx->buffers_zero ? 1 : 0;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  char *out = static_cast<char *>(dst);
  hipError_t e = hipMemcpyAsync(out, &hd, sizeof(hd), hipMemcpyHostToDevice, stream);
  size_t off = sizeof(hd);
  if (e == hipSuccess)
    e = hipMemcpyAsync(out + off, ctx->w.data(), ctx->w.size() * sizeof(float),
                       hipMemcpyHostToDevice, stream);
  off += p.weights;
  auto put = [&](const float *src, size_t n) {
    if (e == hipSuccess && n)
      e = hipMemcpyAsync(out + off, src, n, hipMemcpyDeviceToDevice, stream);
    off += n;
  };
  put(ctx->x0, p.arena * p.outer_copies);
  put(ctx->u, p.arena * p.outer_copies);
  put(ctx->h, p.arena * ctx->cfg.m);
  put(ctx->v, p.arena * p.n_v);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);  // the header lives on this stack frame
  if (e != hipSuccess) return fail_hip(ctx, e, "state export");
  return SLOWMO_OK;
}

slowmo_status slowmo_import_state(slowmo_ctx *ctx, const void *src, size_t bytes, void *stream_) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (ctx->broken) return fail(ctx, SLOWMO_ERR_STATE, kBrokenMsg);
  if (!src) return fail(ctx, SLOWMO_ERR_ARG, "src is NULL");
  const BlobParts p = blob_parts(ctx);
  if (bytes < p.total) return fail(ctx, SLOWMO_ERR_ARG, "blob shorter than this context's state");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  BlobHeader hd{};
  hipError_t e = hipMemcpyAsync(&hd, src, sizeof(hd), hipMemcpyDeviceToHost, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "reading the blob header");
  if (std::memcmp(hd.magic, kBlobMagic, 8) != 0 || hd.version != kBlobVersion)
    return fail(ctx, SLOWMO_ERR_ARG, "not a state blob of this library version");
  if (hd.m != ctx->cfg.m || hd.n_tensors != ctx->n_tensors || hd.base != ctx->cfg.base ||
      hd.no_average != ctx->cfg.no_average || hd.d != ctx->layout.d || hd.d_pad != ctx->layout.d_pad)
    return fail(ctx, SLOWMO_ERR_ARG, "the blob was exported from a different configuration or tensor list");
  if (hd.k < 0 || hd.k > ctx->cfg.tau || hd.t < 0 || hd.l < 0 ||
      (hd.buffers_zero != 0 && hd.buffers_zero != 1))
    return fail(ctx, SLOWMO_ERR_ARG, "the blob's counters do not fit this configuration");
  const char *in = static_cast<const char *>(src);
  size_t off = sizeof(hd);
  std::vector<float> w(ctx->cfg.m);
  e = hipMemcpyAsync(w.data(), in + off, w.size() * sizeof(float), hipMemcpyDeviceToHost, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "reading the blob's push-sum weights");
  for (float wi : w)
    if (!finite_pos(wi)) return fail(ctx, SLOWMO_ERR_ARG, "the blob's push-sum weights are not positive");
  off += p.weights;
  // everything checkable has been checked: only now is the context touched
  bool copied = false;
  auto get = [&](float *dst, size_t n) {
    if (e == hipSuccess && n) {
      e = hipMemcpyAsync(dst, in + off, n, hipMemcpyDeviceToDevice, stream);
      copied = copied || e == hipSuccess;
    }
    off += n;
  };
  get(ctx->x0, p.arena * p.outer_copies);
  get(ctx->u, p.arena * p.outer_copies);
  get(ctx->h, p.arena * ctx->cfg.m);
  get(ctx->v, p.arena * p.n_v);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e != hipSuccess)
    return copied ? fail_midway(ctx, e, "state import") : fail_hip(ctx, e, "state import");
  ctx->t = hd.t;
  ctx->k = hd.k;
  ctx->l = hd.l;
  ctx->buffers_zero = hd.buffers_zero != 0;
  ctx->w.swap(w);
  return SLOWMO_OK;
}

slowmo_status slowmo_destroy(slowmo_ctx *ctx) {
  if (!ctx) return SLOWMO_OK;
  release(ctx);
  return SLOWMO_OK;
}

slowmo_status slowmo_get_buffer(slowmo_ctx *ctx, int32_t which, int32_t worker, int32_t tensor,
                                float **device_ptr) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (!device_ptr) return fail(ctx, SLOWMO_ERR_ARG, "device_ptr is NULL");
  if (tensor < 0 || tensor >= ctx->n_tensors) return fail(ctx, SLOWMO_ERR_ARG, "tensor index out of range");
  const int64_t off = ctx->layout.arena_off[tensor];
  switch (which) {
    case SLOWMO_BUF_X0:
    case SLOWMO_BUF_U: {
      int64_t woff = 0;
      if (ctx->cfg.no_average) {
        if (worker < 0 || worker >= ctx->cfg.m) return fail(ctx, SLOWMO_ERR_ARG, "worker index out of range");
        woff = static_cast<int64_t>(worker) * ctx->layout.d_pad;
      }
      *device_ptr = (which == SLOWMO_BUF_X0 ? ctx->x0 : ctx->u) + woff + off;
      return SLOWMO_OK;
    }
    case SLOWMO_BUF_H:
    case SLOWMO_BUF_V: {
      if (worker < 0 || worker >= ctx->cfg.m) return fail(ctx, SLOWMO_ERR_ARG, "worker index out of range");
      float *b = which == SLOWMO_BUF_H ? ctx->h : ctx->v;
      if (!b) return fail(ctx, SLOWMO_ERR_ARG, "this base optimizer has no v buffer");
      *device_ptr = b + static_cast<int64_t>(worker) * ctx->layout.d_pad + off;
      return SLOWMO_OK;
    }
    default: return fail(ctx, SLOWMO_ERR_ARG, "unknown buffer id");
  }
}

slowmo_status slowmo_get_counters(const slowmo_ctx *ctx, int64_t *t, int32_t *k, int64_t *l) {
  if (!ctx) return fail(nullptr, SLOWMO_ERR_ARG, "ctx is NULL");
  if (t) *t = ctx->t;
  if (k) *k = ctx->k;
  if (l) *l = ctx->l;
  return SLOWMO_OK;
}

}  // extern "C"
