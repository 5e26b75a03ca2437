// C ABI of the library (include/otas.h): argument validation, the host-side length schedule, the
// per-call plan upload, and the launch sequence of the token-adapted encoder block (Sec. III-B:
// normalisation -> attention -> [merge] -> normalisation -> MLP, prompting in front).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/otas.h"
#include "kernels.h"

using namespace otas;

namespace {

constexpr size_t kAlign = 256;
constexpr int64_t kRowPad = 256;              // activation buffers are padded to this many rows
constexpr size_t kPlanInts = (size_t)1 << 20;  // capacity of the device plan buffer (int32 entries)
constexpr int64_t kPlanSideMinRows = 32768;  // batches below this many rows plan inline (see run_layers)
constexpr int kStageSlots = 32;
constexpr size_t kSlotInts = kPlanInts / kStageSlots;
constexpr int kMaxLanes = 8;
// Split-K workspace: float rows of width D per (padded) token row of the batch.  Two for large batches; small
// batches, whose products leave most CUs idle and split up to eight ways, get up to eight (8192 rows in all).
inline int part_rows_factor(size_t rows) { return (int)std::min<size_t>(8, std::max<size_t>(2, 8192 / std::max<size_t>(rows, 1))); }

// Scratch of otas_token_merge_static: the merge lists of one call (src_list [rows] | row_ptr [rows + 64]).
// One copy per GPU, held until the process ends; every call on a GPU shares it.
constexpr int64_t kStaticMergeRows = OTAS_STATIC_MERGE_MAX_ROWS;
constexpr int kStaticMergeQueries = OTAS_STATIC_MERGE_MAX_QUERIES;
constexpr size_t kStaticRowPtrAt = (size_t)kStaticMergeRows;
constexpr size_t kStaticScratchInts = 2 * (size_t)kStaticMergeRows + 64;
constexpr int kMaxDevices = 64;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int removal_count(int n, int r, int n_lead) { return std::max(0, std::min(r, (n - n_lead) / 2)); }
// Workspace of otas_token_merge for the plan kernel's metric rows: none while no query of T tokens can
// overflow the kernel's LDS at any metric width.
inline size_t merge_rows_bytes(int64_t T) {
  return merge_plan_lds_bytes((int)std::min<int64_t>(T, OTAS_MAX_SEQ), 128) <= 160 * 1024
             ? 0 : align_up(merge_plan_rows_bytes(T, 128), kAlign);
}

}  // namespace

static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

namespace {
// Device address of `scratch` on each GPU (the array's name is only a host-side handle: every use of
// its memory from the host goes through the address looked up here, with that GPU current).
std::mutex g_scratch_mu;
int32_t* g_scratch_ptr[kMaxDevices] = {};

// Looks the address up once per device; `device` must be the current device.
otas_status scratch_address(int device, int32_t** out) {
  if (device < 0 || device >= kMaxDevices) return OTAS_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    int32_t* p = nullptr;
    if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return OTAS_EDEVICE;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return OTAS_OK;
}
}  // namespace

struct otas_ctx {
  otas_model_desc desc;
  std::vector<otas_layer_weights> layers;
  hipStream_t stream;
  int device;
  int32_t* d_plan;        // device plan buffer [kPlanInts]
  int32_t* d_scratch;     // this device's copy of the static scratch array (otas_token_merge_static)
  // Pinned host staging for the plan: a ring of kStageSlots slots of kSlotInts entries, so that the host
  // can enqueue that many calls ahead of the device (a host thread that is descheduled for tens of
  // milliseconds then costs nothing as long as the queue holds work).  Slot i may be overwritten once
  // h_done[i] has completed.  A plan larger than a slot uses the whole buffer and waits for the copy.
  int32_t* h_plan;
  hipEvent_t h_done[kStageSlots];
  bool h_used[kStageSlots];
  int h_next;
  // The merge plan of a layer needs only that layer's keys (the QKV projection), so it runs on a
  // second stream next to attention and the output projection: forked after the QKV GEMM, joined
  // before merge-apply.
  // A forward pass may also be cut into lanes (contiguous query ranges) that run side by side on
  // streams of their own, so that one lane's launch gaps, partial waves and latency-bound small
  // kernels overlap another lane's work.  Lane 0 runs on the caller's stream.
  struct Lane {
    hipStream_t main, side;
    hipEvent_t ev_fork, ev_join, ev_done;
  };
  Lane lane[8];
  hipEvent_t ev_begin;
  int lanes;   // requested lane count, 0 = chosen from the batch size
  int lanes_ready;   // lanes whose streams and events exist
  // optional per-launch timing (otas_timing_enable): one event pair per launch, summed per kind
  bool timing;
  float ev_overhead_ms;   // what an event pair reads around an empty launch (subtracted from every record)
  std::vector<hipEvent_t> ev_pool;
  std::vector<int> ev_kind;   // kind of the launch bracketed by ev_pool[2i], ev_pool[2i+1]
  // optional shader-clock probe (otas_clock_probe_start): its own stream and sample buffer, made at first use
  hipStream_t probe_stream;
  uint32_t* d_probe;      // [kProbeMaxSamples]
  int32_t probe_samples;  // samples of the probe in flight or finished and unread, 0 = none
};

namespace {

size_t elem_size(int dtype) { return dtype == OTAS_F32 ? 4 : 2; }

bool offsets_ok(const int32_t* off, int B) {
  if (off[0] != 0) return false;
  for (int q = 0; q < B; ++q)
    if (off[q + 1] < off[q]) return false;
  return true;
}

// Copies `count` ints to the device plan buffer at entry `at` through pinned staging.
otas_status upload_plan(otas_ctx* c, const int32_t* host, size_t count) {
  if (count > kPlanInts) return OTAS_ENOMEM;
  const size_t bytes = count * sizeof(int32_t);
  if (count > kSlotInts) {
    for (int j = 0; j < kStageSlots; ++j) {
      if (c->h_used[j] && hipEventSynchronize(c->h_done[j]) != hipSuccess) return OTAS_EDEVICE;
      c->h_used[j] = false;
    }
    std::memcpy(c->h_plan, host, bytes);
    if (hipMemcpyAsync(c->d_plan, c->h_plan, bytes, hipMemcpyHostToDevice, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess)
      return OTAS_EDEVICE;
    return OTAS_OK;
  }
  const int i = c->h_next;
  c->h_next = (c->h_next + 1) % kStageSlots;
  if (c->h_used[i] && hipEventSynchronize(c->h_done[i]) != hipSuccess) return OTAS_EDEVICE;
  int32_t* slot = c->h_plan + (size_t)i * kSlotInts;
  std::memcpy(slot, host, bytes);
  if (hipMemcpyAsync(c->d_plan, slot, bytes, hipMemcpyHostToDevice, c->stream) != hipSuccess) return OTAS_EDEVICE;
  if (hipEventRecord(c->h_done[i], c->stream) != hipSuccess) return OTAS_EDEVICE;
  c->h_used[i] = true;
  return OTAS_OK;
}
otas_status upload_plan(otas_ctx* c, const std::vector<int32_t>& host) {
  return upload_plan(c, host.data(), host.size());
}

struct WorkspaceLayout {
  size_t xa, xb, h, qkv, hid, part, sizes_a, sizes_b, src_list, row_ptr, total;
  int part_factor;   // float rows of the split-K buffer per token row
};

WorkspaceLayout forward_layout(const otas_model_desc& d, int64_t T0) {
  const size_t es = elem_size(d.dtype);
  const size_t rows = (size_t)((T0 + kRowPad - 1) / kRowPad * kRowPad);
  WorkspaceLayout w;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes, kAlign); return at; };
  w.xa = take(rows * d.D * sizeof(float));   // the residual stream is float for every dtype
  w.xb = take(rows * d.D * sizeof(float));
  w.h = take(rows * d.D * es);
  w.qkv = take(rows * 3 * d.D * es);
  w.hid = take(rows * d.F * es);
  w.part_factor = part_rows_factor(rows);
  w.part = take(d.dtype == OTAS_BF16 ? w.part_factor * rows * d.D * sizeof(float) : 0);   // split-K partial products
  w.sizes_a = take(rows * sizeof(int32_t));
  w.sizes_b = take(rows * sizeof(int32_t));
  w.src_list = take(rows * sizeof(int32_t));
  w.row_ptr = take((rows + kMaxLanes + 1) * sizeof(int32_t));   // one end entry per lane
  w.total = p;
  return w;
}

// A failing HIP call maps to OTAS_EDEVICE; with OTAS_DEBUG set in the environment it is also named
// on stderr.
inline bool hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  static const bool verbose = std::getenv("OTAS_DEBUG") != nullptr;
  if (verbose) std::fprintf(stderr, "otas: %s -> %s\n", what, hipGetErrorString(e));
  return false;
}
#define OTAS_HIP(expr)                              \
  do {                                              \
    if (!hip_ok((expr), #expr)) return OTAS_EDEVICE; \
  } while (0)

enum Kind { K_PREPEND = 0, K_LN, K_QKV, K_ATTN, K_PROJ, K_PLAN, K_APPLY, K_FC1, K_FC2, K_REDUCE, K_MISC, K_COUNT };
const char* const kKindNames[K_COUNT] = {"prompt_prepend", "layer_norm", "gemm_qkv", "attention", "gemm_proj",
                                         "merge_plan", "merge_apply", "gemm_fc1", "gemm_fc2", "splitk_reduce_ln",
                                         "misc"};

// Brackets one launch with an event pair when timing is on.
struct LaunchTimer {
  otas_ctx* c;
  bool on;
  hipStream_t st;
  LaunchTimer(otas_ctx* ctx, int kind, hipStream_t stream) : c(ctx), on(ctx->timing), st(stream) {
    if (!on) return;
    const size_t i = c->ev_kind.size();
    while (c->ev_pool.size() < 2 * (i + 1)) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
      c->ev_pool.push_back(e);
    }
    c->ev_kind.push_back(kind);
    idx = i;
    (void)hipEventRecord(c->ev_pool[2 * i], st);
  }
  ~LaunchTimer() {
    if (on) (void)hipEventRecord(c->ev_pool[2 * idx + 1], st);
  }
  size_t idx = 0;
};
#define OTAS_LAUNCH_ON(kind, stream, expr) \
  do {                                     \
    LaunchTimer _t(c, kind, stream);       \
    OTAS_HIP(expr);                        \
  } while (0)
#define OTAS_LAUNCH(kind, expr) OTAS_LAUNCH_ON(kind, c->stream, expr)

// Streams and events of lanes 0 .. n-1, created on first use (every stream at the default priority).
// Streams share a few hardware queues, so a context creates no more of them than it runs.
bool ensure_lanes(otas_ctx* c, int n) {
  for (int g = c->lanes_ready; g < n; ++g) {
    otas_ctx::Lane& ln = c->lane[g];
    bool ok = true;
    if (g > 0) ok = hipStreamCreateWithFlags(&ln.main, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&ln.side, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ln.ev_fork, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ln.ev_join, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ln.ev_done, hipEventDisableTiming) == hipSuccess;
    if (!ok) return false;   // otas_destroy releases what was created
    c->lanes_ready = g + 1;
  }
  return true;
}

}  // namespace

extern "C" {

const char* otas_strerror(otas_status s) {
  switch (s) {
    case OTAS_OK: return "ok";
    case OTAS_EINVAL: return "invalid argument";
    case OTAS_ESHAPE: return "shape does not match the model description";
    case OTAS_ENOMEM: return "workspace or plan buffer too small";
    case OTAS_EDEVICE: return "HIP runtime error";
    case OTAS_EUNSUPPORTED: return "size outside the supported range";
  }
  return "unknown status";
}

otas_status otas_schedule(int32_t n0, int32_t P, int32_t r, int32_t n_lead, int32_t L, int32_t* len_out) {
  if (!len_out || n0 < 0 || P < 0 || r < 0 || L < 0 || n_lead < 0 || n_lead > 1) return OTAS_EINVAL;
  if (n0 < n_lead) return OTAS_EINVAL;
  int n = n0 + P;
  len_out[0] = n;
  for (int l = 0; l < L; ++l) {
    n -= removal_count(n, r, n_lead);
    len_out[l + 1] = n;
  }
  return OTAS_OK;
}

otas_status otas_create(otas_ctx** out, const otas_model_desc* desc, const otas_layer_weights* layers,
                        void* hip_stream) {
  if (!out || !desc || !layers) return OTAS_EINVAL;
  *out = nullptr;
  const otas_model_desc& d = *desc;
  if (d.L <= 0 || d.D <= 0 || d.H <= 0 || d.F <= 0 || !(d.ln_eps >= 0.f)) return OTAS_EINVAL;
  if (d.dtype != OTAS_F32 && d.dtype != OTAS_BF16) return OTAS_EINVAL;
  if (d.n_lead < 0 || d.n_lead > 1) return OTAS_EUNSUPPORTED;
  if (d.D % d.H != 0) return OTAS_ESHAPE;
  const int dh = d.D / d.H;
  if (d.D % 8 != 0 || d.F % 8 != 0 || dh % 4 != 0 || dh > 128) return OTAS_EUNSUPPORTED;
  if (d.D > 8 * 64 * (d.dtype == OTAS_F32 ? 4 : 8)) return OTAS_EUNSUPPORTED;
  for (int l = 0; l < d.L; ++l) {
    const void* const* p = reinterpret_cast<const void* const*>(&layers[l]);
    for (size_t i = 0; i < sizeof(otas_layer_weights) / sizeof(void*); ++i)
      if (!p[i]) return OTAS_EINVAL;
  }
  otas_ctx* c = new (std::nothrow) otas_ctx();
  if (!c) return OTAS_ENOMEM;
  c->desc = d;
  c->layers.assign(layers, layers + d.L);
  c->stream = (hipStream_t)hip_stream;
  c->d_plan = nullptr;
  c->d_scratch = nullptr;
  c->h_plan = nullptr;
  for (int i = 0; i < kStageSlots; ++i) { c->h_done[i] = nullptr; c->h_used[i] = false; }
  c->h_next = 0;
  c->timing = false;
  c->ev_overhead_ms = 0.f;
  std::memset(c->lane, 0, sizeof(c->lane));
  c->ev_begin = nullptr;
  c->lanes = 0;
  c->lanes_ready = 0;
  c->probe_stream = nullptr;
  c->d_probe = nullptr;
  c->probe_samples = 0;
  bool ok = hipGetDevice(&c->device) == hipSuccess;
  ok = ok && scratch_address(c->device, &c->d_scratch) == OTAS_OK;   // the current device is c->device
  ok = ok && hipMalloc((void**)&c->d_plan, kPlanInts * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipHostMalloc((void**)&c->h_plan, kPlanInts * sizeof(int32_t), hipHostMallocDefault) == hipSuccess;
  for (int i = 0; i < kStageSlots && ok; ++i)
    ok = hipEventCreateWithFlags(&c->h_done[i], hipEventDisableTiming) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&c->ev_begin, hipEventDisableTiming) == hipSuccess;
  ok = ok && ensure_lanes(c, 1);
  if (!ok) {
    otas_destroy(c);
    return OTAS_EDEVICE;
  }
  *out = c;
  return OTAS_OK;
}

otas_status otas_destroy(otas_ctx* c) {
  if (!c) return OTAS_OK;
  if (c->stream || c->d_plan) (void)hipStreamSynchronize(c->stream);
  for (int g = 0; g < kMaxLanes; ++g) {
    otas_ctx::Lane& ln = c->lane[g];
    if (ln.main) { (void)hipStreamSynchronize(ln.main); (void)hipStreamDestroy(ln.main); }
    if (ln.side) { (void)hipStreamSynchronize(ln.side); (void)hipStreamDestroy(ln.side); }
    if (ln.ev_fork) (void)hipEventDestroy(ln.ev_fork);
    if (ln.ev_join) (void)hipEventDestroy(ln.ev_join);
    if (ln.ev_done) (void)hipEventDestroy(ln.ev_done);
  }
  if (c->ev_begin) (void)hipEventDestroy(c->ev_begin);
  for (int i = 0; i < kStageSlots; ++i)
    if (c->h_done[i]) (void)hipEventDestroy(c->h_done[i]);
  if (c->h_plan) (void)hipHostFree(c->h_plan);
  for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
  if (c->probe_stream) { (void)hipStreamSynchronize(c->probe_stream); (void)hipStreamDestroy(c->probe_stream); }
  if (c->d_probe) (void)hipFree(c->d_probe);
  if (c->d_plan) (void)hipFree(c->d_plan);
  delete c;
  return OTAS_OK;
}

size_t otas_workspace_bytes(const otas_ctx* c, int32_t B, int64_t T0) {
  if (!c || B <= 0 || T0 <= 0) return 0;
  return forward_layout(c->desc, T0).total;
}

size_t otas_merge_workspace_bytes(int32_t B, int64_t T) {
  if (B <= 0 || T <= 0) return 0;
  // src_list [T], row_ptr [T+1], and -- once a query can be too long for the plan kernel's LDS -- the
  // unit metric rows of all tokens at the widest metric (128)
  return align_up((size_t)T * 4, kAlign) + align_up((size_t)(T + 1) * 4, kAlign) + merge_rows_bytes(T);
}

}  // extern "C"

namespace {
// Body of otas_prompt_prepend and otas_prompt_prepend_pool: query q takes rows prm_beg[q] .. +prm_cnt[q]-1
// of `prompts` (prm_rows rows in all).
otas_status prepend_impl(otas_ctx* c, const void* tokens, const int32_t* tok_off, const void* prompts,
                         int64_t prm_rows, const int32_t* prm_beg, const int32_t* prm_cnt, int32_t B, void* out,
                         int32_t* out_off) {
  if (out == tokens || (prompts && out == prompts)) return OTAS_EINVAL;
  int max_n = 0;
  // plan: tok_off [B+1] | prm_beg [B] | prm_cnt [B] | out_off [B+1]
  std::vector<int32_t> plan(4 * (size_t)B + 2);
  out_off[0] = 0;
  for (int q = 0; q < B; ++q) {
    const int n = tok_off[q + 1] - tok_off[q], P = prm_cnt[q];
    if (n < c->desc.n_lead || P < 0) return OTAS_EINVAL;
    if (P > 0 && (!prompts || prm_beg[q] < 0 || (int64_t)prm_beg[q] + P > prm_rows)) return OTAS_EINVAL;
    out_off[q + 1] = out_off[q] + n + P;
    max_n = std::max(max_n, n + P);
  }
  std::memcpy(&plan[0], tok_off, (B + 1) * sizeof(int32_t));
  std::memcpy(&plan[B + 1], prm_beg, B * sizeof(int32_t));
  std::memcpy(&plan[2 * B + 1], prm_cnt, B * sizeof(int32_t));
  std::memcpy(&plan[3 * B + 1], out_off, (B + 1) * sizeof(int32_t));
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  otas_status st = upload_plan(c, plan);
  if (st != OTAS_OK) return st;
  const int32_t* dp = c->d_plan;
  OTAS_LAUNCH(K_PREPEND, launch_prepend(c->desc.dtype, tokens, prompts, out, dp, dp + (B + 1), dp + (2 * B + 1),
                                        dp + (3 * B + 1), B, max_n, c->desc.D, c->desc.n_lead, c->stream));
  return OTAS_OK;
}
}  // namespace

extern "C" {

otas_status otas_prompt_prepend(otas_ctx* c, const void* tokens, const int32_t* tok_off, const void* prompts,
                                const int32_t* prm_off, int32_t B, void* out, int32_t* out_off) {
  if (!c || !tokens || !tok_off || !prm_off || !out || !out_off || B <= 0) return OTAS_EINVAL;
  if (!offsets_ok(tok_off, B) || !offsets_ok(prm_off, B)) return OTAS_EINVAL;
  if (prm_off[B] > 0 && !prompts) return OTAS_EINVAL;
  std::vector<int32_t> cnt(B);
  for (int q = 0; q < B; ++q) cnt[q] = prm_off[q + 1] - prm_off[q];
  return prepend_impl(c, tokens, tok_off, prompts, prm_off[B], prm_off, cnt.data(), B, out, out_off);
}

otas_status otas_prompt_prepend_pool(otas_ctx* c, const void* tokens, const int32_t* tok_off, const void* pool,
                                     int64_t pool_rows, const int32_t* prompt_first, const int32_t* prompt_count,
                                     int32_t B, void* out, int32_t* out_off) {
  if (!c || !tokens || !tok_off || !prompt_first || !prompt_count || !out || !out_off || B <= 0 || pool_rows < 0)
    return OTAS_EINVAL;
  if (!offsets_ok(tok_off, B)) return OTAS_EINVAL;
  return prepend_impl(c, tokens, tok_off, pool, pool_rows, prompt_first, prompt_count, B, out, out_off);
}

}  // extern "C"

namespace {
// Body of otas_token_merge and otas_token_merge_static.  plan: host array of 4 B + 2 entries to fill
// (in_off [B+1] | out_off [B+1] | r_eff [B] | trace_off [B]); src_list / row_ptr: device lists of
// at least T and T + 1 entries; timed: bracket the launches with timing events when timing is on
// (creating events allocates, so the static entry point never does).
otas_status token_merge_impl(otas_ctx* c, const void* x, const void* metric, int32_t dm, const int32_t* sizes,
                             const int32_t* offsets, const int32_t* r, int32_t B, int32_t* plan, int32_t* src_list,
                             int32_t* row_ptr, float* rows, void* x_out, int32_t* sizes_out, int32_t* offsets_out,
                             int32_t* trace_src, int32_t* trace_dst, bool timed) {
  const int64_t T = offsets[B];
  const int n_lead = c->desc.n_lead;
  int32_t* in_off = &plan[0];
  int32_t* out_off = &plan[B + 1];
  int32_t* reff = &plan[2 * (B + 1)];
  int32_t* troff = &plan[2 * (B + 1) + B];
  int max_n = 0, tr = 0;
  out_off[0] = 0;
  for (int q = 0; q < B; ++q) {
    const int n = offsets[q + 1] - offsets[q];
    if (r[q] < 0) return OTAS_EINVAL;
    if (n > 0 && n < n_lead) return OTAS_EINVAL;
    if (n > OTAS_MAX_SEQ) return OTAS_EUNSUPPORTED;
    in_off[q] = offsets[q];
    reff[q] = removal_count(n, r[q], n_lead);
    troff[q] = tr;
    tr += reff[q];
    out_off[q + 1] = out_off[q] + n - reff[q];
    max_n = std::max(max_n, n);
  }
  in_off[B] = offsets[B];
  if (merge_plan_lds_bytes(max_n, dm) > 160 * 1024 && !rows) return OTAS_EUNSUPPORTED;   // no room for the metric rows
  std::memcpy(offsets_out, out_off, (B + 1) * sizeof(int32_t));
  const int64_t T_out = out_off[B];
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  otas_status st = upload_plan(c, plan, 4 * (size_t)B + 2);
  if (st != OTAS_OK) return st;
  const int32_t* dp = c->d_plan;
  const bool was_timing = c->timing;
  if (!timed) c->timing = false;
  st = [&]() -> otas_status {
    OTAS_LAUNCH(K_PLAN, launch_merge_plan(c->desc.dtype, metric, dm, 0, 1, dm, dp, dp + (B + 1), dp + 2 * (B + 1),
                                          dp + 2 * (B + 1) + B, B, max_n, n_lead, src_list, row_ptr, trace_src,
                                          trace_dst, rows, c->stream));
    OTAS_LAUNCH(K_APPLY, launch_merge_apply(c->desc.dtype, x, sizes, src_list, row_ptr, T, T_out, c->desc.D, x_out,
                                            sizes_out, c->stream));
    return OTAS_OK;
  }();
  c->timing = was_timing;
  return st;
}

otas_status token_merge_args_ok(otas_ctx* c, const void* x, const void* metric, int32_t dm, const int32_t* sizes,
                                const int32_t* offsets, const int32_t* r, int32_t B, void* x_out,
                                int32_t* sizes_out, int32_t* offsets_out, int32_t* trace_src, int32_t* trace_dst) {
  if (!c || !x || !metric || !offsets || !r || !x_out || !sizes_out || !offsets_out || B <= 0) return OTAS_EINVAL;
  if ((trace_src == nullptr) != (trace_dst == nullptr)) return OTAS_EINVAL;
  if (dm <= 0 || dm % 4 != 0 || dm > 128) return OTAS_EUNSUPPORTED;
  if (!offsets_ok(offsets, B)) return OTAS_EINVAL;
  if (x_out == x || (const void*)sizes_out == (const void*)sizes) return OTAS_EINVAL;
  if (offsets[B] <= 0) return OTAS_EINVAL;
  return OTAS_OK;
}
}  // namespace

extern "C" {

otas_status otas_token_merge(otas_ctx* c, const void* x, const void* metric, int32_t dm, const int32_t* sizes,
                             const int32_t* offsets, const int32_t* r, int32_t B, void* workspace,
                             size_t workspace_bytes, void* x_out, int32_t* sizes_out, int32_t* offsets_out,
                             int32_t* trace_src, int32_t* trace_dst) {
  otas_status st = token_merge_args_ok(c, x, metric, dm, sizes, offsets, r, B, x_out, sizes_out, offsets_out,
                                       trace_src, trace_dst);
  if (st != OTAS_OK) return st;
  if (!workspace || ((uintptr_t)workspace) % kAlign != 0) return OTAS_EINVAL;
  const int64_t T = offsets[B];
  if (workspace_bytes < otas_merge_workspace_bytes(B, T)) return OTAS_ENOMEM;
  std::vector<int32_t> plan(4 * (size_t)B + 2);
  int32_t* src_list = (int32_t*)workspace;
  int32_t* row_ptr = (int32_t*)((char*)workspace + align_up((size_t)T * 4, kAlign));
  float* rows = merge_rows_bytes(T) ? (float*)((char*)row_ptr + align_up((size_t)(T + 1) * 4, kAlign)) : nullptr;
  return token_merge_impl(c, x, metric, dm, sizes, offsets, r, B, plan.data(), src_list, row_ptr, rows, x_out,
                          sizes_out, offsets_out, trace_src, trace_dst, true);
}

otas_status otas_token_merge_static(otas_ctx* c, const void* x, const void* metric, int32_t dm,
                                    const int32_t* sizes, const int32_t* offsets, const int32_t* r, int32_t B,
                                    void* x_out, int32_t* sizes_out, int32_t* offsets_out, int32_t* trace_src,
                                    int32_t* trace_dst) {
  otas_status st = token_merge_args_ok(c, x, metric, dm, sizes, offsets, r, B, x_out, sizes_out, offsets_out,
                                       trace_src, trace_dst);
  if (st != OTAS_OK) return st;
  if (B > kStaticMergeQueries || (int64_t)offsets[B] > kStaticMergeRows) return OTAS_ENOMEM;
  if (!c->d_scratch) return OTAS_EDEVICE;
  int32_t plan[4 * kStaticMergeQueries + 2];   // on the stack: no host allocation either
  // Nothing in the lists has to start at zero: the plan kernel writes every entry of src_list [0, T)
  // and row_ptr [0, T_out) that the apply kernel reads, whatever an earlier call left there.
  // (no room for metric rows here: a query too long for the plan kernel's LDS is refused, EUNSUPPORTED)
  return token_merge_impl(c, x, metric, dm, sizes, offsets, r, B, plan, c->d_scratch,
                          c->d_scratch + kStaticRowPtrAt, nullptr, x_out, sizes_out, offsets_out, trace_src,
                          trace_dst, false);
}

namespace {
otas_status run_layers(otas_ctx* c, int32_t layer_begin, int32_t layer_end, const void* x0, bool x0_is_float,
                       const int32_t* sizes_in, const int32_t* offsets, const int32_t* r, int32_t B, uint32_t flags,
                       void* workspace, size_t workspace_bytes, void* x_out, int32_t* sizes_out,
                       int32_t* offsets_out, int32_t* trace_src, int32_t* trace_dst);
}

otas_status otas_encoder_forward(otas_ctx* c, const void* x0, const int32_t* offsets, const int32_t* r, int32_t B,
                                 uint32_t flags, void* workspace, size_t workspace_bytes, void* x_out,
                                 int32_t* sizes_out, int32_t* offsets_out, int32_t* trace_src, int32_t* trace_dst) {
  if (!c) return OTAS_EINVAL;
  return run_layers(c, 0, c->desc.L, x0, c->desc.dtype == OTAS_F32, nullptr, offsets, r, B, flags, workspace,
                    workspace_bytes, x_out, sizes_out, offsets_out, trace_src, trace_dst);
}

otas_status otas_encoder_layers(otas_ctx* c, int32_t layer_begin, int32_t layer_end, const void* x0,
                                const int32_t* sizes_in, const int32_t* offsets, const int32_t* r, int32_t B,
                                uint32_t flags, void* workspace, size_t workspace_bytes, void* x_out,
                                int32_t* sizes_out, int32_t* offsets_out, int32_t* trace_src, int32_t* trace_dst) {
  if (!c) return OTAS_EINVAL;
  return run_layers(c, layer_begin, layer_end, x0, true, sizes_in, offsets, r, B, flags, workspace, workspace_bytes,
                    x_out, sizes_out, offsets_out, trace_src, trace_dst);
}

}  // extern "C"

namespace {

// One lane's share of a forward pass: a contiguous range of queries that runs through the layers on
// its own stream, in its own rows of every workspace buffer, next to the other lanes.
struct LaneRun {
  int q0, q1, Bg;
  size_t plan_base;              // first entry of this lane's plan in the device plan buffer
  int64_t row0;                  // first packed row of the lane at the input (its rows in every buffer)
  int64_t rowL;                  // first packed row of the lane in the output
  std::vector<int64_t> T;        // packed rows of the lane entering layer l (l = 0 .. L)
  std::vector<int> max_n;        // longest query entering layer l
  std::vector<char> any_merge;
  int last_merge;
  // running state
  const int32_t* sizes_now;
  const void* x_cur;
  bool x_owned;
  bool ln1_done;   // the previous block's split-K reduce already wrote this block's LN1 output
};

otas_status run_layers(otas_ctx* c, int32_t layer_begin, int32_t layer_end, const void* x0, bool x0_is_float,
                       const int32_t* sizes_in, const int32_t* offsets, const int32_t* r, int32_t B, uint32_t flags,
                       void* workspace, size_t workspace_bytes, void* x_out, int32_t* sizes_out,
                       int32_t* offsets_out, int32_t* trace_src, int32_t* trace_dst) {
  if (!c || !x0 || !offsets || !r || !workspace || !x_out || !sizes_out || !offsets_out || B <= 0)
    return OTAS_EINVAL;
  if (layer_begin < 0 || layer_end > c->desc.L || layer_begin >= layer_end) return OTAS_EINVAL;
  if ((const void*)sizes_in == (const void*)sizes_out) return OTAS_EINVAL;
  if (flags & ~(uint32_t)(OTAS_FLAG_SIZE_BIAS | OTAS_FLAG_TRACE)) return OTAS_EINVAL;
  const bool trace = flags & OTAS_FLAG_TRACE;
  if (trace && (!trace_src || !trace_dst)) return OTAS_EINVAL;
  if (!offsets_ok(offsets, B)) return OTAS_EINVAL;
  if (x_out == x0 || ((uintptr_t)workspace) % kAlign != 0) return OTAS_EINVAL;
  const otas_model_desc& d = c->desc;
  const int L = layer_end - layer_begin, D = d.D, H = d.H, F = d.F, dh = D / H, n_lead = d.n_lead;
  const int64_t T0 = offsets[B];
  if (T0 <= 0) return OTAS_EINVAL;
  const WorkspaceLayout w = forward_layout(d, T0);
  if (workspace_bytes < w.total) return OTAS_ENOMEM;
  {
    const char* ws = (const char*)workspace;
    const char* xo = (const char*)x_out;
    if (xo >= ws && xo < ws + w.total) return OTAS_EINVAL;
  }

  // Schedule of the whole batch: lengths entering every layer, removal counts, and where each
  // (layer, query) starts in the trace (layer-major, then query).
  std::vector<int> len((size_t)(L + 1) * B), reff((size_t)L * B), troff((size_t)L * B);
  for (int q = 0; q < B; ++q) {
    const int n = offsets[q + 1] - offsets[q];
    if (r[q] < 0 || n <= 0 || n < n_lead) return OTAS_EINVAL;
    if (n > OTAS_MAX_SEQ) return OTAS_EUNSUPPORTED;
    len[q] = n;
  }
  int tr = 0;
  for (int l = 0; l < L; ++l) {
    int mx = 0;
    bool any = false;
    for (int q = 0; q < B; ++q) {
      const int n = len[(size_t)l * B + q];
      const int k = removal_count(n, r[q], n_lead);
      reff[(size_t)l * B + q] = k;
      troff[(size_t)l * B + q] = tr;
      tr += k;
      any = any || k > 0;
      mx = std::max(mx, n);
      len[(size_t)(l + 1) * B + q] = n - k;
    }
    // a query too long for the plan kernel's LDS keeps its metric rows in the (then unused) MLP hidden buffer,
    // F elements per token: that has to hold a metric row
    if (any && merge_plan_lds_bytes(mx, dh) > 160 * 1024 &&
        (size_t)d.F * elem_size(d.dtype) * 64 < merge_plan_rows_bytes(64, dh))
      return OTAS_EUNSUPPORTED;
  }
  offsets_out[0] = 0;
  for (int q = 0; q < B; ++q) offsets_out[q + 1] = offsets_out[q] + len[(size_t)L * B + q];

  // Lanes: contiguous query ranges with about equal token counts.
  int G = c->lanes > 0 ? c->lanes : 1;
  G = std::max(1, std::min(std::min(G, (int)B), kMaxLanes));
  std::vector<LaneRun> lanes(G);
  {
    int q = 0;
    for (int g = 0; g < G; ++g) {
      LaneRun& ln = lanes[g];
      ln.q0 = q;
      if (g == G - 1) q = B;
      else {
        const int64_t goal = T0 * (g + 1) / G;
        ++q;
        while (q < B - (G - 1 - g) && offsets[q] < goal) ++q;
      }
      ln.q1 = q;
      ln.Bg = ln.q1 - ln.q0;
      ln.row0 = offsets[ln.q0];
      ln.rowL = offsets_out[ln.q0];
    }
  }
  // Device plan.  Per lane (int32): off[l][Bg+1] for l = 0..L (relative to the lane's first row) |
  // r_eff[l][Bg] | trace_off[l][Bg].
  std::vector<int32_t> plan;
  for (LaneRun& ln : lanes) {
    const int Bg = ln.Bg;
    ln.plan_base = plan.size();
    plan.resize(ln.plan_base + (size_t)(L + 1) * (Bg + 1) + 2 * (size_t)L * Bg);
    int32_t* off = &plan[ln.plan_base];
    int32_t* pr = off + (size_t)(L + 1) * (Bg + 1);
    int32_t* pt = pr + (size_t)L * Bg;
    ln.T.assign(L + 1, 0);
    ln.max_n.assign(L + 1, 0);
    ln.any_merge.assign(L, 0);
    ln.last_merge = -1;
    for (int l = 0; l <= L; ++l) {
      int32_t* o = off + (size_t)l * (Bg + 1);
      o[0] = 0;
      for (int j = 0; j < Bg; ++j) {
        const int n = len[(size_t)l * B + ln.q0 + j];
        o[j + 1] = o[j] + n;
        ln.max_n[l] = std::max(ln.max_n[l], n);
      }
      ln.T[l] = o[Bg];
      if (l < L)
        for (int j = 0; j < Bg; ++j) {
          const int k = reff[(size_t)l * B + ln.q0 + j];
          pr[(size_t)l * Bg + j] = k;
          pt[(size_t)l * Bg + j] = troff[(size_t)l * B + ln.q0 + j];
          if (k > 0) { ln.any_merge[l] = 1; ln.last_merge = l; }
        }
    }
  }

  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  if (!ensure_lanes(c, G)) return OTAS_EDEVICE;

  otas_status st = upload_plan(c, plan);
  if (st != OTAS_OK) return st;
  // Everything below enqueues work.  If a HIP call fails after lanes or the plan stream were forked,
  // the library's own streams are drained before the error is returned, so that nothing of this call
  // is still running on them when the next call reuses the plan buffer and the workspace.
  const otas_status enq = [&]() -> otas_status {
  const int32_t* d_plan_base = c->d_plan;
  hipStream_t s0 = c->stream;   // lane 0 runs on the caller's stream
  // Lanes beyond the first run on streams of their own, forked here and joined at the end.
  if (G > 1) {
    OTAS_HIP(hipEventRecord(c->ev_begin, s0));
    for (int g = 1; g < G; ++g) OTAS_HIP(hipStreamWaitEvent(c->lane[g].main, c->ev_begin, 0));
  }

  char* ws = (char*)workspace;
  const size_t es = elem_size(d.dtype);
  const int dt = d.dtype;
  const bool size_bias = flags & OTAS_FLAG_SIZE_BIAS;
  const size_t es_in = x0_is_float ? sizeof(float) : es;

  // Token sizes: nullptr stands for "all 1" until the first merge (or the caller's sizes_in), so no
  // fill is needed; a lane's last merging layer writes straight into sizes_out.
  for (int g = 0; g < G; ++g) {
    LaneRun& ln = lanes[g];
    hipStream_t s = g == 0 ? s0 : c->lane[g].main;
    ln.sizes_now = sizes_in ? sizes_in + ln.row0 : nullptr;
    if (size_bias && !ln.sizes_now) {   // the attention bias reads sizes from the first layer on
      int32_t* sz = (int32_t*)(ws + w.sizes_a) + ln.row0;
      OTAS_LAUNCH_ON(K_MISC, s, launch_fill_i32(sz, 1, ln.T[0], s));
      ln.sizes_now = sz;
    }
    ln.x_cur = (const char*)x0 + (size_t)ln.row0 * D * es_in;   // residual stream entering the block
    ln.x_owned = false;   // x_cur is one of the workspace buffers, so it may be updated in place
    ln.ln1_done = false;
    if (!x0_is_float) {   // 16-bit tokens: widened into the workspace by the first block's LayerNorm
      float* xa = (float*)(ws + w.xa) + (size_t)ln.row0 * D;
      char* hbuf = ws + w.h + (size_t)ln.row0 * D * es;
      const otas_layer_weights& w0 = c->layers[layer_begin];
      OTAS_LAUNCH_ON(K_LN, s, launch_layer_norm_widen(ln.x_cur, w0.ln1_g, w0.ln1_b, hbuf, xa, ln.T[0], D, d.ln_eps, s));
      ln.x_cur = xa;
      ln.x_owned = true;
      ln.ln1_done = true;
    }
  }
  // The merge plan needs only this layer's keys, so it may run beside attention and the projection on a side
  // stream.  Measured on MI355X that pays only for the largest batches (ViT-H, 256 queries, 67 k rows: +0.9 %):
  // at ViT-B batch 64 and ViT-L batch 128 the plan's workgroups slow attention and the GEMMs next to them by as
  // much as hiding the plan saves (same images/s either way), a single forward pass is ~1 % quicker with the
  // plan inline, and every fork / join costs the host ~45 us per layer.  So smaller batches keep the plan on
  // the lane's own stream.
  const bool plan_inline = T0 < kPlanSideMinRows;
  for (int l = 0; l < L; ++l) {
    const otas_layer_weights& wl = c->layers[layer_begin + l];
    for (int g = 0; g < G; ++g) {
      LaneRun& ln = lanes[g];
      otas_ctx::Lane& hw = c->lane[g];
      hipStream_t s = g == 0 ? s0 : hw.main;
      const int Bg = ln.Bg;
      const int32_t* dp = d_plan_base + ln.plan_base;
      const int32_t* off_l = dp + (size_t)l * (Bg + 1);
      const int32_t* off_n = dp + (size_t)(l + 1) * (Bg + 1);
      const int32_t* d_reff = dp + (size_t)(L + 1) * (Bg + 1) + (size_t)l * Bg;
      const int32_t* d_tr = d_reff + (size_t)L * Bg;
      const int64_t T = ln.T[l], Tn = ln.T[l + 1];
      // the lane's rows of every buffer
      float* x_free[2] = {(float*)(ws + w.xa) + (size_t)ln.row0 * D, (float*)(ws + w.xb) + (size_t)ln.row0 * D};
      char* hbuf = ws + w.h + (size_t)ln.row0 * D * es;
      char* qkv = ws + w.qkv + (size_t)ln.row0 * 3 * D * es;
      char* hid = ws + w.hid + (size_t)ln.row0 * F * es;
      int32_t* sizes_buf[2] = {(int32_t*)(ws + w.sizes_a) + ln.row0, (int32_t*)(ws + w.sizes_b) + ln.row0};
      int32_t* src_list = (int32_t*)(ws + w.src_list) + ln.row0;
      int32_t* row_ptr = (int32_t*)(ws + w.row_ptr) + ln.row0 + g;   // one end entry per lane
      // normalisation -> QKV -> attention -> projection + residual
      if (!ln.ln1_done)
        OTAS_LAUNCH_ON(K_LN, s, launch_layer_norm(dt, true, ln.x_cur, wl.ln1_g, wl.ln1_b, hbuf, T, D, d.ln_eps, s));
      ln.ln1_done = false;
      OTAS_LAUNCH_ON(K_QKV, s, launch_linear(dt, hbuf, wl.w_qkv, wl.b_qkv, nullptr, qkv, T, 3 * D, D, EPI_NONE, s));
      // Attention and the merge plan both read only the QKV projection.  On one stream two kernels never overlap,
      // so where the plan stays on this stream and one kernel can hold both (bf16, head width 64), they go out
      // as ONE launch whose first workgroups are the plan's; it is recorded as an attention launch.
      const bool fuse = ln.any_merge[l] && plan_inline && attention_plan_takes(dt, ln.max_n[l], D, H);
      // Where the projection's launch below has workgroup slots to spare, the fused launch runs only the plan's
      // selection (the long part: keys, similarities, best matches) and the lists, which need nothing else, are
      // written by extra workgroups of the projection's launch: the plan's serial chain beside attention gets
      // shorter by a quarter.  The selection's result waits in the split-K partial buffer, idle between two MLPs.
      float* sel_best = (float*)(ws + w.part) + (size_t)w.part_factor * ln.row0 * D;
      int32_t* sel_bcol = (int32_t*)(sel_best + T);
      const bool tail = fuse && linear_plan_tail_fits(T, D, D, Bg);
      if (fuse) {
        OTAS_LAUNCH_ON(K_ATTN, s,
                       launch_attention_plan(qkv, ln.sizes_now, off_l, off_n, d_reff, d_tr, Bg, ln.max_n[l], D, H,
                                             size_bias, n_lead, hbuf, src_list, row_ptr,
                                             trace ? trace_src : nullptr, trace ? trace_dst : nullptr,
                                             tail ? sel_best : nullptr, tail ? sel_bcol : nullptr, s));
      } else {
        if (ln.any_merge[l]) {
          // fork: the merge plan reads only the keys just written; the lists it writes were last read by
          // the previous layer's merge-apply, which precedes this point on the lane's stream
          hipStream_t ps = plan_inline ? s : hw.side;
          if (!plan_inline) {
            OTAS_HIP(hipEventRecord(hw.ev_fork, s));
            OTAS_HIP(hipStreamWaitEvent(hw.side, hw.ev_fork, 0));
          }
          OTAS_LAUNCH_ON(K_PLAN, ps,
                         launch_merge_plan(dt, qkv, 3 * (int64_t)D, D, H, dh, off_l, off_n, d_reff, d_tr, Bg,
                                           ln.max_n[l], n_lead, src_list, row_ptr, trace ? trace_src : nullptr,
                                           trace ? trace_dst : nullptr, (float*)hid, ps));
          if (!plan_inline) OTAS_HIP(hipEventRecord(hw.ev_join, hw.side));
        }
        OTAS_LAUNCH_ON(K_ATTN, s,
                       launch_attention(dt, qkv, ln.sizes_now, off_l, Bg, ln.max_n[l], D, H, size_bias, hbuf, s));
      }
      // in-place residual is safe (each element is read then written by the same thread); the
      // caller's x0 is never written, so layer 0 writes into the workspace.
      void* x_attn = ln.x_owned ? const_cast<void*>(ln.x_cur) : (void*)x_free[0];
      if (tail) {
        const PlanTail pt{off_l, off_n, d_reff, d_tr, src_list, row_ptr, trace ? trace_src : nullptr,
                          trace ? trace_dst : nullptr, sel_best, sel_bcol, Bg};
        OTAS_LAUNCH_ON(K_PROJ, s, launch_linear_plan_tail(hbuf, wl.w_proj, wl.b_proj, (const float*)ln.x_cur, x_attn, T,
                                                          D, D, pt, ln.max_n[l], s));
      } else {
        OTAS_LAUNCH_ON(K_PROJ, s, launch_linear(dt, hbuf, wl.w_proj, wl.b_proj, (const float*)ln.x_cur, x_attn, T, D,
                                                D, EPI_RESIDUAL, s));
      }
      void* x_mlp = x_attn;
      // merging module
      if (ln.any_merge[l]) {
        void* x_other = (x_attn == (void*)x_free[0]) ? x_free[1] : x_free[0];
        if (!plan_inline) OTAS_HIP(hipStreamWaitEvent(s, hw.ev_join, 0));   // join
        int32_t* sizes_next = (l == ln.last_merge) ? sizes_out + ln.rowL
                                                   : (ln.sizes_now == sizes_buf[0] ? sizes_buf[1] : sizes_buf[0]);
        // merge-apply and the block's second LayerNorm in one pass over the rows
        OTAS_LAUNCH_ON(K_APPLY, s,
                       launch_merge_apply_ln(dt, (const float*)x_attn, ln.sizes_now, src_list, row_ptr, T, Tn, D,
                                             (float*)x_other, sizes_next, wl.ln2_g, wl.ln2_b, hbuf, d.ln_eps, s));
        ln.sizes_now = sizes_next;
        x_mlp = x_other;
      } else {
        OTAS_LAUNCH_ON(K_LN, s, launch_layer_norm(dt, true, x_mlp, wl.ln2_g, wl.ln2_b, hbuf, Tn, D, d.ln_eps, s));
      }
      // MLP + residual
      OTAS_LAUNCH_ON(K_FC1, s, launch_linear(dt, hbuf, wl.w_fc1, wl.b_fc1, nullptr, hid, Tn, F, D, EPI_GELU, s));
      void* x_next = (l == L - 1) ? (void*)((float*)x_out + (size_t)ln.rowL * D) : x_mlp;
      const int S = splitk_factor(dt, Tn, D, F, (int)std::min<int64_t>(8, w.part_factor * ln.T[0] / std::max<int64_t>(Tn, 1)));
      if (S > 1) {
        // few tiles, long K: S partial products, then one pass that adds them, the bias and the
        // residual and already applies the next block's first LayerNorm to the row in registers
        float* part = (float*)(ws + w.part) + (size_t)w.part_factor * ln.row0 * D;
        OTAS_LAUNCH_ON(K_FC2, s, launch_linear_splitk(hid, wl.w_fc2, part, Tn, D, F, S, s));
        const bool more = l + 1 < L;
        const otas_layer_weights* wn = more ? &c->layers[layer_begin + l + 1] : nullptr;
        OTAS_LAUNCH_ON(K_REDUCE, s,
                       launch_splitk_reduce_ln(part, S, wl.b_fc2, (const float*)x_mlp, (float*)x_next, Tn, D,
                                               more ? wn->ln1_g : nullptr, more ? wn->ln1_b : nullptr,
                                               more ? (void*)hbuf : nullptr, d.ln_eps, s));
        ln.ln1_done = more;
      } else {
        OTAS_LAUNCH_ON(K_FC2, s, launch_linear(dt, hid, wl.w_fc2, wl.b_fc2, (const float*)x_mlp, x_next, Tn, D, F,
                                               EPI_RESIDUAL, s));
      }
      ln.x_cur = x_next;
      ln.x_owned = true;
    }
  }
  for (int g = 0; g < G; ++g) {
    LaneRun& ln = lanes[g];
    hipStream_t s = g == 0 ? s0 : c->lane[g].main;
    if (ln.last_merge < 0) {   // nothing merged in this lane: the sizes are the input's
      if (sizes_in) OTAS_LAUNCH_ON(K_MISC, s, launch_copy_i32(sizes_in + ln.row0, sizes_out + ln.rowL, ln.T[L], s));
      else OTAS_LAUNCH_ON(K_MISC, s, launch_fill_i32(sizes_out + ln.rowL, 1, ln.T[L], s));
    }
    if (g > 0) {   // join
      OTAS_HIP(hipEventRecord(c->lane[g].ev_done, s));
      OTAS_HIP(hipStreamWaitEvent(s0, c->lane[g].ev_done, 0));
    }
  }
  return OTAS_OK;
  }();
  if (enq != OTAS_OK) {
    for (int g = 0; g < G; ++g) {
      if (g > 0 && c->lane[g].main) (void)hipStreamSynchronize(c->lane[g].main);
      if (c->lane[g].side) (void)hipStreamSynchronize(c->lane[g].side);
    }
  }
  return enq;
}
}  // namespace

extern "C" {

otas_status otas_encoder_forward_deep(otas_ctx* c, const void* x0, const int32_t* offsets, int32_t B, int32_t mode,
                                      const void* prompts, const int32_t* prompt_offsets, void* workspace,
                                      size_t workspace_bytes, void* x_out, int32_t* sizes_out, int32_t* offsets_out) {
  if (!c || !x0 || !offsets || !prompt_offsets || !workspace || !x_out || !sizes_out || !offsets_out || B <= 0)
    return OTAS_EINVAL;
  if (mode != OTAS_PROMPT_REPLACE && mode != OTAS_PROMPT_GROW) return OTAS_EINVAL;
  if (!offsets_ok(offsets, B) || !offsets_ok(prompt_offsets, B)) return OTAS_EINVAL;
  if (x_out == x0 || ((uintptr_t)workspace) % kAlign != 0) return OTAS_EINVAL;
  const bool grow = mode == OTAS_PROMPT_GROW;
  const otas_model_desc& d = c->desc;
  const int L = d.L, D = d.D, H = d.H, F = d.F, n_lead = d.n_lead, dt = d.dtype;
  const int64_t T0 = offsets[B];
  const int P_total = prompt_offsets[B];
  if (T0 <= 0) return OTAS_EINVAL;
  if (P_total > 0 && !prompts) return OTAS_EINVAL;

  // Length schedule: constant (replace) or + P_q per layer (grow); x0 holds layer 0's prompts.
  // Plan layout (int32): off[l][B+1] for l = 0..L-1 | prompt offsets [B+1].
  std::vector<int32_t> plan((size_t)(L + 1) * (B + 1));
  std::vector<int> max_n(L, 0);
  int max_p = 0;
  for (int l = 0; l < L; ++l) {
    int32_t* off = &plan[(size_t)l * (B + 1)];
    off[0] = 0;
    for (int q = 0; q < B; ++q) {
      const int n = offsets[q + 1] - offsets[q], P = prompt_offsets[q + 1] - prompt_offsets[q];
      if (n <= 0 || n < n_lead + P) return OTAS_EINVAL;   // x0 must already hold the P rows of layer 0
      const int nl = n + (grow ? l * P : 0);
      if (nl > OTAS_MAX_SEQ) return OTAS_EUNSUPPORTED;
      off[q + 1] = off[q] + nl;
      max_n[l] = std::max(max_n[l], nl);
      max_p = std::max(max_p, P);
    }
  }
  std::memcpy(&plan[(size_t)L * (B + 1)], prompt_offsets, (B + 1) * sizeof(int32_t));
  const int32_t* off_last = &plan[(size_t)(L - 1) * (B + 1)];
  const int64_t T_max = off_last[B];
  const WorkspaceLayout w = forward_layout(d, T_max);
  if (workspace_bytes < w.total) return OTAS_ENOMEM;
  {
    const char* ws = (const char*)workspace;
    const char* xo = (const char*)x_out;
    if (xo >= ws && xo < ws + w.total) return OTAS_EINVAL;
  }
  std::memcpy(offsets_out, off_last, (B + 1) * sizeof(int32_t));

  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  otas_status st = upload_plan(c, plan);
  if (st != OTAS_OK) return st;
  hipStream_t s = c->stream;
  char* ws = (char*)workspace;
  float* x_buf[2] = {(float*)(ws + w.xa), (float*)(ws + w.xb)};
  void* hbuf = ws + w.h;
  void* qkv = ws + w.qkv;
  void* hid = ws + w.hid;
  const int32_t* d_prm_off = c->d_plan + (size_t)L * (B + 1);
  const size_t es = elem_size(dt);

  const float* x_cur = (const float*)x0;   // float residual stream entering the block
  int cur = -1;                            // which workspace buffer holds x_cur (-1: the caller's x0)
  bool ln1_done = false;
  if (dt != OTAS_F32) {                    // 16-bit tokens: widened into the workspace by the first block's LayerNorm
    OTAS_LAUNCH(K_LN, launch_layer_norm_widen(x0, c->layers[0].ln1_g, c->layers[0].ln1_b, hbuf, x_buf[0], T0, D,
                                              d.ln_eps, s));
    x_cur = x_buf[0];
    cur = 0;
    ln1_done = true;
  }
  for (int l = 0; l < L; ++l) {
    const otas_layer_weights& wl = c->layers[l];
    const int32_t* off_l = c->d_plan + (size_t)l * (B + 1);
    const int64_t T = plan[(size_t)l * (B + 1) + B];
    if (l >= 1 && P_total > 0) {   // prompting module (cur >= 0 here: layer 0 wrote into the workspace)
      const char* pl = (const char*)prompts + (size_t)l * P_total * D * es;
      if (grow) {
        OTAS_LAUNCH(K_PREPEND, launch_deep_prompt(dt, x_cur, x_buf[cur ^ 1], pl, off_l - (B + 1), off_l, d_prm_off, B,
                                                  max_n[l], D, n_lead, true, s));
        cur ^= 1;
        x_cur = x_buf[cur];
      } else {
        OTAS_LAUNCH(K_PREPEND, launch_deep_prompt(dt, x_cur, x_buf[cur], pl, off_l, off_l, d_prm_off, B, max_p, D,
                                                  n_lead, false, s));
      }
    }
    if (!ln1_done) OTAS_LAUNCH(K_LN, launch_layer_norm(dt, true, x_cur, wl.ln1_g, wl.ln1_b, hbuf, T, D, d.ln_eps, s));
    ln1_done = false;
    OTAS_LAUNCH(K_QKV, launch_linear(dt, hbuf, wl.w_qkv, wl.b_qkv, nullptr, qkv, T, 3 * D, D, EPI_NONE, s));
    OTAS_LAUNCH(K_ATTN, launch_attention(dt, qkv, nullptr, off_l, B, max_n[l], D, H, false, hbuf, s));
    if (cur < 0) cur = 0;   // the caller's x0 is never written: layer 0 of an f32 model writes into the workspace
    OTAS_LAUNCH(K_PROJ, launch_linear(dt, hbuf, wl.w_proj, wl.b_proj, x_cur, x_buf[cur], T, D, D, EPI_RESIDUAL, s));
    x_cur = x_buf[cur];
    OTAS_LAUNCH(K_LN, launch_layer_norm(dt, true, x_cur, wl.ln2_g, wl.ln2_b, hbuf, T, D, d.ln_eps, s));
    OTAS_LAUNCH(K_FC1, launch_linear(dt, hbuf, wl.w_fc1, wl.b_fc1, nullptr, hid, T, F, D, EPI_GELU, s));
    void* x_next = (l == L - 1) ? x_out : (void*)x_buf[cur];
    // few rows, long K: split over K as in run_layers; the next block's LayerNorm is not folded into the reduce,
    // because that block first replaces or inserts prompt rows
    const int S = splitk_factor(dt, T, D, F, (int)std::min<int64_t>(8, w.part_factor * T_max / std::max<int64_t>(T, 1)));
    if (S > 1) {
      float* part = (float*)(ws + w.part);
      OTAS_LAUNCH(K_FC2, launch_linear_splitk(hid, wl.w_fc2, part, T, D, F, S, s));
      OTAS_LAUNCH(K_REDUCE, launch_splitk_reduce_ln(part, S, wl.b_fc2, x_cur, (float*)x_next, T, D, nullptr, nullptr,
                                                    nullptr, d.ln_eps, s));
    } else {
      OTAS_LAUNCH(K_FC2, launch_linear(dt, hid, wl.w_fc2, wl.b_fc2, x_cur, x_next, T, D, F, EPI_RESIDUAL, s));
    }
  }
  OTAS_LAUNCH(K_MISC, launch_fill_i32(sizes_out, 1, T_max, s));
  return OTAS_OK;
}

size_t otas_patch_embed_workspace_bytes(const otas_ctx* c, int32_t B, int32_t C, int32_t Hi, int32_t Wi, int32_t patch) {
  if (!c || B <= 0 || C <= 0 || patch <= 0 || Hi <= 0 || Wi <= 0 || Hi % patch || Wi % patch) return 0;
  const size_t rows = (size_t)B * (Hi / patch) * (Wi / patch), es = elem_size(c->desc.dtype);
  return align_up(rows * C * patch * patch * es, kAlign) + align_up(rows * c->desc.D * es, kAlign);
}

otas_status otas_patch_embed(otas_ctx* c, const void* images, int32_t B, int32_t C, int32_t Hi, int32_t Wi,
                             int32_t patch, const void* w_patch, const void* b_patch, const void* cls, const void* pos,
                             void* workspace, size_t workspace_bytes, void* tokens, int32_t* tok_offsets) {
  if (!c || !images || !w_patch || !b_patch || !pos || !workspace || !tokens || !tok_offsets) return OTAS_EINVAL;
  if (B <= 0 || C <= 0 || patch <= 0 || Hi <= 0 || Wi <= 0 || Hi % patch || Wi % patch) return OTAS_EINVAL;
  const int n_lead = c->desc.n_lead, D = c->desc.D, dt = c->desc.dtype;
  if (n_lead > 0 && !cls) return OTAS_EINVAL;
  if (((uintptr_t)workspace) % kAlign != 0 || tokens == images) return OTAS_EINVAL;
  const int N = (Hi / patch) * (Wi / patch), kp = C * patch * patch;
  if (n_lead + N > OTAS_MAX_SEQ) return OTAS_EUNSUPPORTED;
  if (kp % 8 != 0) return OTAS_EUNSUPPORTED;
  if (workspace_bytes < otas_patch_embed_workspace_bytes(c, B, C, Hi, Wi, patch)) return OTAS_ENOMEM;
  const size_t es = elem_size(dt);
  char* pm = (char*)workspace;
  char* proj = pm + align_up((size_t)B * N * kp * es, kAlign);
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  OTAS_LAUNCH(K_PREPEND, launch_patchify(dt, images, pm, B, C, Hi, Wi, patch, c->stream));
  OTAS_LAUNCH(K_MISC, launch_linear(dt, pm, w_patch, b_patch, nullptr, proj, (int64_t)B * N, D, kp, EPI_NONE, c->stream));
  OTAS_LAUNCH(K_PREPEND, launch_embed_finish(dt, proj, cls, pos, tokens, B, N, D, n_lead, c->stream));
  for (int q = 0; q <= B; ++q) tok_offsets[q] = q * (n_lead + N);
  return OTAS_OK;
}

otas_status otas_task_heads(otas_ctx* c, const float* x, const int32_t* offsets, const int32_t* task, int32_t B,
                            const otas_task_head* heads, int32_t n_tasks, const void* lnf_g, const void* lnf_b,
                            float* logits, int32_t k_max) {
  if (!c || !x || !offsets || !task || !heads || !lnf_g || !lnf_b || !logits || B <= 0 || n_tasks <= 0 || k_max <= 0)
    return OTAS_EINVAL;
  if (!offsets_ok(offsets, B)) return OTAS_EINVAL;
  for (int q = 0; q < B; ++q)
    if (task[q] < 0 || task[q] >= n_tasks || offsets[q + 1] <= offsets[q]) return OTAS_EINVAL;
  for (int t = 0; t < n_tasks; ++t)
    if (!heads[t].w || !heads[t].b || heads[t].classes <= 0 || heads[t].classes > k_max) return OTAS_EINVAL;
  // plan (int32): offsets [B] | task [B] | pad to 8 bytes | head records [n_tasks] of 6 ints
  const size_t o_task = B, o_heads = (2 * (size_t)B + 1) & ~(size_t)1;
  std::vector<int32_t> plan(o_heads + 6 * (size_t)n_tasks);
  std::memcpy(&plan[0], offsets, B * sizeof(int32_t));
  std::memcpy(&plan[o_task], task, B * sizeof(int32_t));
  for (int t = 0; t < n_tasks; ++t) {
    HeadRef r = {heads[t].w, heads[t].b, heads[t].classes, 0};
    static_assert(sizeof(HeadRef) == 6 * sizeof(int32_t), "head record layout");
    std::memcpy(&plan[o_heads + 6 * (size_t)t], &r, sizeof(r));
  }
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  otas_status st = upload_plan(c, plan);   // the plan buffer is 256-byte aligned, the records 8-byte
  if (st != OTAS_OK) return st;
  OTAS_LAUNCH(K_MISC, launch_task_heads(c->desc.dtype, x, c->d_plan, c->d_plan + o_task, c->d_plan + o_heads, lnf_g, lnf_b,
                                        B, c->desc.D, c->desc.ln_eps, logits, k_max, c->stream));
  return OTAS_OK;
}

otas_status otas_layer_norm(otas_ctx* c, const void* x, const void* g, const void* b, int64_t T, void* y) {
  if (!c || !x || !g || !b || !y || T < 0) return OTAS_EINVAL;
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  OTAS_LAUNCH(K_LN, launch_layer_norm(c->desc.dtype, c->desc.dtype == OTAS_F32, x, g, b, y, T, c->desc.D, c->desc.ln_eps, c->stream));
  return OTAS_OK;
}

otas_status otas_linear(otas_ctx* c, const void* x, const void* w, const void* b, const void* res, int64_t T,
                        int32_t N, int32_t K, int32_t epilogue, void* y) {
  if (!c || !x || !w || !b || !y || T < 0 || N <= 0 || K <= 0) return OTAS_EINVAL;
  if (epilogue < 0 || epilogue > 2 || (epilogue == EPI_RESIDUAL && !res)) return OTAS_EINVAL;
  if (N % 8 != 0 || K % 8 != 0) return OTAS_EUNSUPPORTED;
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  OTAS_LAUNCH(K_MISC, launch_linear(c->desc.dtype, x, w, b, (const float*)res, y, T, N, K, epilogue, c->stream));
  return OTAS_OK;
}

otas_status otas_linear_kernel(otas_ctx* c, int32_t kernel, const void* x, const void* w, const void* b,
                               const void* res, int64_t T, int32_t N, int32_t K, int32_t epilogue, void* y) {
  if (!c || !x || !w || !b || !y || T < 0 || N <= 0 || K <= 0) return OTAS_EINVAL;
  if (epilogue < 0 || epilogue > 2 || (epilogue == EPI_RESIDUAL && !res)) return OTAS_EINVAL;
  if (kernel < 0 || kernel >= GK_COUNT) return OTAS_EINVAL;
  if (N % 8 != 0 || K % 8 != 0) return OTAS_EUNSUPPORTED;
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  const hipError_t e = launch_linear_kernel(kernel, c->desc.dtype, x, w, b, (const float*)res, y, T, N, K, epilogue,
                                            c->stream);
  if (e == hipErrorInvalidValue) return OTAS_EUNSUPPORTED;   // the kernel does not take this shape / dtype
  return hip_ok(e, "launch_linear_kernel") ? OTAS_OK : OTAS_EDEVICE;
}

int32_t otas_linear_choice(const otas_ctx* c, int64_t T, int32_t N, int32_t K, int32_t epilogue) {
  if (!c || T < 0 || N <= 0 || K <= 0 || epilogue < 0 || epilogue > 2) return -1;
  return linear_kernel_choice(c->desc.dtype, T, N, K, epilogue);
}

otas_status otas_attention(otas_ctx* c, const void* qkv, const int32_t* sizes, const int32_t* offsets, int32_t B,
                           uint32_t flags, void* o) {
  if (!c || !qkv || !offsets || !o || B <= 0) return OTAS_EINVAL;
  if (!offsets_ok(offsets, B)) return OTAS_EINVAL;
  const bool size_bias = flags & OTAS_FLAG_SIZE_BIAS;
  if (size_bias && !sizes) return OTAS_EINVAL;
  int max_n = 0;
  for (int q = 0; q < B; ++q) max_n = std::max(max_n, offsets[q + 1] - offsets[q]);
  if (max_n > OTAS_MAX_SEQ) return OTAS_EUNSUPPORTED;
  std::vector<int32_t> plan(offsets, offsets + B + 1);
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  otas_status st = upload_plan(c, plan);
  if (st != OTAS_OK) return st;
  OTAS_LAUNCH(K_ATTN, launch_attention(c->desc.dtype, qkv, sizes, c->d_plan, B, max_n, c->desc.D, c->desc.H, size_bias, o,
                            c->stream));
  return OTAS_OK;
}

otas_status otas_timing_enable(otas_ctx* c, int32_t on) {
  if (!c) return OTAS_EINVAL;
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return OTAS_EDEVICE;
  c->timing = false;
  c->ev_kind.clear();
  if (on) {
    // Calibrate what an event pair adds to the launch it brackets, on kernels of known duration: one
    // wave that spins for 10 us and for 30 us of the device's constant-rate wall clock, 15 pairs each.
    // A pair reads spin + overhead + the dispatch's own ramp (launch to first instruction, last
    // instruction to completion), which a profiler counts as kernel time for every kernel: 1 us is
    // taken for it (a kernel-trace profiler reports 0.8 .. 1.9 us for an empty one-wave kernel on MI355X),
    // so overhead = median(reading - spin) - 1 us.  If the two spin lengths do not differ by 20 us within
    // 5 %, or the result is negative, nothing is subtracted (durations then read long, never short).
    c->timing = true;
    c->ev_overhead_ms = 0.f;
    int32_t* cell = c->d_plan + kPlanInts - 1;
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device) != hipSuccess || khz <= 0)
      khz = 100000;
    const double spin_us[2] = {10.0, 30.0};
    OTAS_HIP(launch_spin((int64_t)(spin_us[0] * khz / 1000.0), cell, c->stream));   // warm the code object
    for (int i = 0; i < 15; ++i)
      for (int j = 0; j < 2; ++j) OTAS_LAUNCH(K_MISC, launch_spin((int64_t)(spin_us[j] * khz / 1000.0), cell, c->stream));
    if (hipStreamSynchronize(c->stream) != hipSuccess) return OTAS_EDEVICE;
    std::vector<float> rd[2];
    for (size_t i = 0; i < c->ev_kind.size(); ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, c->ev_pool[2 * i], c->ev_pool[2 * i + 1]) != hipSuccess) return OTAS_EDEVICE;
      rd[i % 2].push_back(ms * 1e3f);
    }
    if (!rd[0].empty() && !rd[1].empty()) {
      std::sort(rd[0].begin(), rd[0].end());
      std::sort(rd[1].begin(), rd[1].end());
      const double m0 = rd[0][rd[0].size() / 2], m1 = rd[1][rd[1].size() / 2];
      const double step = m1 - m0, want = spin_us[1] - spin_us[0];
      const double over = 0.5 * ((m0 - spin_us[0]) + (m1 - spin_us[1])) - 1.0;
      if (step > 0.95 * want && step < 1.05 * want && over > 0.0) c->ev_overhead_ms = (float)(over * 1e-3);
    }
    c->ev_kind.clear();
  }
  return OTAS_OK;
}

otas_status otas_set_lanes(otas_ctx* c, int32_t lanes) {
  if (!c || lanes < 0 || lanes > kMaxLanes) return OTAS_EINVAL;
  c->lanes = lanes;
  return OTAS_OK;
}

int32_t otas_splitk_room(const otas_ctx* c, int64_t T0, int64_t M) {
  if (!c || T0 <= 0 || M <= 0) return 1;
  const size_t rows = (size_t)((T0 + kRowPad - 1) / kRowPad * kRowPad);
  return (int32_t)std::max<int64_t>(1, std::min<int64_t>(8, part_rows_factor(rows) * T0 / M));
}

int32_t otas_splitk_factor(const otas_ctx* c, int64_t M, int32_t N, int32_t K, int32_t max_split) {
  return c ? splitk_factor(c->desc.dtype, M, N, K, max_split) : 1;
}

float otas_timing_overhead_ms(const otas_ctx* c) { return c ? c->ev_overhead_ms : 0.f; }

otas_status otas_clock_probe_start(otas_ctx* c, int32_t samples) {
  if (!c || samples <= 0 || samples > OTAS_CLOCK_PROBE_MAX_SAMPLES) return OTAS_EINVAL;
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  if (!c->probe_stream) OTAS_HIP(hipStreamCreateWithFlags(&c->probe_stream, hipStreamNonBlocking));
  if (!c->d_probe) OTAS_HIP(hipMalloc((void**)&c->d_probe, (size_t)OTAS_CLOCK_PROBE_MAX_SAMPLES * sizeof(uint32_t)));
  OTAS_HIP(hipStreamSynchronize(c->probe_stream));   // an earlier probe has finished with the buffer
  OTAS_HIP(launch_clock_probe(c->d_probe, samples, c->probe_stream));
  c->probe_samples = samples;
  return OTAS_OK;
}

otas_status otas_clock_probe_read(otas_ctx* c, float* mhz, int32_t cap, int32_t* n) {
  if (!c || !mhz || !n || cap < 0) return OTAS_EINVAL;
  *n = 0;
  if (!c->probe_samples) return OTAS_OK;
  if (hipSetDevice(c->device) != hipSuccess) return OTAS_EDEVICE;
  OTAS_HIP(hipStreamSynchronize(c->probe_stream));
  const int32_t m = c->probe_samples < cap ? c->probe_samples : cap;
  std::vector<uint32_t> ticks((size_t)m);
  if (m) OTAS_HIP(hipMemcpy(ticks.data(), c->d_probe, (size_t)m * sizeof(uint32_t), hipMemcpyDeviceToHost));
  int khz = 0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device) != hipSuccess || khz <= 0) khz = 100000;
  for (int32_t i = 0; i < m; ++i)
    mhz[i] = ticks[i] ? (float)((double)kClockProbeClocks * (double)khz / 1000.0 / (double)ticks[i]) : 0.f;
  *n = m;
  c->probe_samples = 0;
  return OTAS_OK;
}

int32_t otas_timing_kinds(void) { return K_COUNT; }

const char* otas_timing_kind_name(int32_t kind) { return (kind >= 0 && kind < K_COUNT) ? kKindNames[kind] : ""; }

int32_t otas_timing_read_launches(otas_ctx* c, int32_t cap, int32_t* kinds, float* ms) {
  if (!c || cap < 0 || (cap > 0 && (!kinds || !ms))) return -1;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return -1;   // every lane and side stream has joined it
  const int32_t n = (int32_t)std::min<size_t>(c->ev_kind.size(), (size_t)cap);
  for (int32_t i = 0; i < n; ++i) {
    kinds[i] = c->ev_kind[i];
    if (hipEventElapsedTime(&ms[i], c->ev_pool[2 * i], c->ev_pool[2 * i + 1]) != hipSuccess) return -1;
    ms[i] = std::max(ms[i] - c->ev_overhead_ms, 0.0005f);
  }
  return (int32_t)c->ev_kind.size();
}

otas_status otas_timing_read(otas_ctx* c, double* total_ms, int64_t* launches) {
  if (!c || !total_ms || !launches) return OTAS_EINVAL;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return OTAS_EDEVICE;
  for (int k = 0; k < K_COUNT; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
  for (size_t i = 0; i < c->ev_kind.size(); ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev_pool[2 * i], c->ev_pool[2 * i + 1]) != hipSuccess) return OTAS_EDEVICE;
    total_ms[c->ev_kind[i]] += std::max(ms - c->ev_overhead_ms, 0.0005f);
    launches[c->ev_kind[i]] += 1;
  }
  c->ev_kind.clear();
  return OTAS_OK;
}

}  // extern "C"
