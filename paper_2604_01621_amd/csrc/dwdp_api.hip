// C-ABI entry points of libdwdp: argument checking, workspace, stream/event choreography
// of the layer-ahead prefetch pipeline.  All arithmetic lives in the kernels.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "dwdp_kernels.h"

using namespace dwdp;

struct dwdp_ctx {
  dwdp_config cfg{};
  int device = 0;
  hipStream_t compute = nullptr;
  hipStream_t copy = nullptr;
  hipStream_t aux = nullptr;  // runs the LDS-tiled GEMM chain beside the streaming chain
  hipEvent_t fork_ev = nullptr, join_ev = nullptr;
  int n_slots = 0;
  size_t rows_max = 0;
  void* ws[DWDP_N_WS] = {};
  int32_t* chunk_counts = nullptr;
  // LDS-tiled GEMM schedule (FP8): experts with more than stream_max_rows rows
  int stream_max_rows = -1;  // -1: the default for the weight format (see dwdp_set_stream_max_rows)
  int32_t* mid_expert = nullptr;  // row groups of the experts with 17 .. stream_max_rows rows
  int32_t* mid_row0 = nullptr;
  int32_t* n_mid = nullptr;
  int mid_cap = 0;
  int32_t* mt_expert = nullptr;
  int32_t* mt_row0 = nullptr;
  int32_t* n_mtiles = nullptr;
  int32_t* sched_sync = nullptr;  // ticket queues, error word and per-tile counters of the persistent tiled GEMM
  int mt_cap = 0;
  int n_cus = 256;
  int tile_schedule = DWDP_TILE_PER_ITEM;
  int tile_share_wgs = 0;  // 0: default share of a persistent tiled launch next to a streamed chain
  // prefetch engine: 0 = one hipMemcpyAsync per plan entry, 1 = one copy-plan kernel launch
  int copy_mode = 0;
  int copy_wgs = 256;
  struct PlanCache {
    std::vector<uintptr_t> key;      // the arguments the cached plan was built from
    bool valid = false;
    CopyUnit* units = nullptr;       // device
    CopyUnit* units_host = nullptr;  // pinned host image the device copy is uploaded from
    int n_units = 0;
  };
  std::vector<PlanCache> plan_cache;  // per layer
  struct Retired {
    CopyUnit* units;
    CopyUnit* units_host;
  };
  std::vector<Retired> retired;  // replaced plans, freed at destroy
  // double-buffer protocol
  std::vector<hipEvent_t> staged_ev;  // per layer: its prefetch copies are complete
  hipEvent_t done_ev[2] = {nullptr, nullptr};  // per staging buffer: its last reader finished
  bool done_valid[2] = {false, false};
  int pending_layer[2] = {-1, -1};  // layer prefetched into the buffer and not yet consumed
  // profiling
  bool prof = false;
  std::vector<hipEvent_t> prof_ev;
  std::vector<char> prof_has_aux;
  int prof_calls = 0;
  // timeline of prefetch copies and GEMM phases (both streams), relative to tl_base
  struct Span {
    int kind, layer;
    hipEvent_t a, b;
  };
  bool tl_on = false;
  hipEvent_t tl_base = nullptr;
  std::vector<Span> tl;
  std::string err;
};

static thread_local std::string g_create_err;

static dwdp_status fail(dwdp_ctx* ctx, dwdp_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx)
    ctx->err = buf;
  else
    g_create_err = buf;
  return st;
}

#define HIP_TRY(ctx, call)                                                                        \
  do {                                                                                            \
    hipError_t e_ = (call);                                                                       \
    if (e_ != hipSuccess) return fail(ctx, DWDP_EHIP, "%s: %s", #call, hipGetErrorString(e_));    \
  } while (0)

static dwdp_status check_config(const dwdp_config* c) {
  if (!c) return fail(nullptr, DWDP_EINVAL, "cfg is NULL");
  if (c->T_max < 0 || c->H <= 0 || c->I <= 0 || c->E <= 0 || c->K <= 0 || c->n_layers < 1)
    return fail(nullptr, DWDP_EINVAL, "non-positive size in cfg");
  if (c->score_fn != DWDP_SCORE_SOFTMAX && c->score_fn != DWDP_SCORE_SIGMOID)
    return fail(nullptr, DWDP_EINVAL, "score_fn must be DWDP_SCORE_SOFTMAX or DWDP_SCORE_SIGMOID");
  if (c->w_dtype != DWDP_W_BF16 && c->w_dtype != DWDP_W_FP8 && c->w_dtype != DWDP_W_MXFP4)
    return fail(nullptr, DWDP_EINVAL, "w_dtype must be DWDP_W_BF16, DWDP_W_FP8 or DWDP_W_MXFP4");
  if (c->has_shared != 0 && c->has_shared != 1) return fail(nullptr, DWDP_EINVAL, "has_shared must be 0 or 1");
  if (c->H % 128 || c->I % 128) return fail(nullptr, DWDP_ESHAPE, "H and I must be multiples of 128");
  if (c->E > 1024 || c->K > c->E || c->K > 32) return fail(nullptr, DWDP_ESHAPE, "need K <= E <= 1024 and K <= 32");
  if (c->n_group < 1 || c->n_group > 64 || c->E % c->n_group)
    return fail(nullptr, DWDP_ESHAPE, "n_group must divide E and be in [1,64]");
  if (c->topk_group < 1 || c->topk_group > c->n_group)
    return fail(nullptr, DWDP_ESHAPE, "topk_group must be in [1,n_group]");
  if (c->n_group > 1 && c->E / c->n_group < 2)
    return fail(nullptr, DWDP_ESHAPE, "group-limited routing needs at least 2 experts per group");
  if ((long)c->K > (long)c->topk_group * (c->E / c->n_group))
    return fail(nullptr, DWDP_ESHAPE, "K exceeds the experts of the kept groups");
  if ((long)c->T_max * c->K > (1L << 30)) return fail(nullptr, DWDP_ESHAPE, "T_max * K too large");
  {
    // the tiled GEMM addresses activations and one weight matrix with 32-bit byte offsets
    const long rows = (long)c->T_max * (c->K + c->has_shared);
    const long wide = c->H > c->I ? c->H : c->I;
    if (rows * wide >= (1L << 32) || 2L * c->I * c->H >= (1L << 32))
      return fail(nullptr, DWDP_ESHAPE, "T_max*(K+shared)*max(H,I) and 2*I*H must stay below 2^32");
  }
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_create(const dwdp_config* cfg, void* compute_stream, dwdp_ctx** out) {
  if (!out) return fail(nullptr, DWDP_EINVAL, "out is NULL");
  *out = nullptr;
  dwdp_status st = check_config(cfg);
  if (st != DWDP_OK) return st;
  dwdp_ctx* c = new (std::nothrow) dwdp_ctx();
  if (!c) return fail(nullptr, DWDP_ENOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->compute = (hipStream_t)compute_stream;
  c->n_slots = cfg->E + cfg->has_shared;
  const size_t T = (size_t)(cfg->T_max > 0 ? cfg->T_max : 1);
  const size_t K = cfg->K, H = cfg->H, I = cfg->I, E = cfg->E;
  c->rows_max = T * K + (cfg->has_shared ? T : 0);
  const bool fp8 = cfg->w_dtype != DWDP_W_BF16;  // FP8 activations and intermediates (FP8 and MXFP4 weights)
  size_t bytes[DWDP_N_WS];
  bytes[DWDP_WS_TOPK_IDS] = T * K * 4;
  bytes[DWDP_WS_TOPK_W] = T * K * 4;
  bytes[DWDP_WS_OFFSETS] = (E + 2) * 4;
  bytes[DWDP_WS_PERM] = T * K * 4;
  bytes[DWDP_WS_INV_PERM] = T * K * 4;
  bytes[DWDP_WS_XQ] = fp8 ? T * H : 0;
  // + 16: the tiled GEMM copies a row's scales three K blocks at a time and may read two floats past the last row
  bytes[DWDP_WS_XS] = fp8 ? T * (H / 128) * 4 + 16 : 0;
  bytes[DWDP_WS_HQ] = c->rows_max * I * (fp8 ? 1 : 4);
  bytes[DWDP_WS_HS] = fp8 ? c->rows_max * (I / 128) * 4 + 16 : 0;
  bytes[DWDP_WS_YP] = c->rows_max * H * (fp8 ? 2 : 4);
  bytes[DWDP_WS_SCHED] = 0;  // allocated below with the tile list (sched_sync)
  hipError_t e = hipGetDevice(&c->device);
  for (int i = 0; i < DWDP_N_WS && e == hipSuccess; i++)
    if (bytes[i]) e = hipMalloc(&c->ws[i], bytes[i]);
  const int chunk = permute_multi_chunk_tokens(cfg->E);
  const size_t n_chunks = (T + chunk - 1) / chunk;
  if (e == hipSuccess) e = hipMalloc((void**)&c->chunk_counts, n_chunks * E * 4);
  c->mt_cap = tile_mtiles_cap((int)c->rows_max, c->n_slots, 0);
  if (e == hipSuccess) e = hipMalloc((void**)&c->mt_expert, (size_t)c->mt_cap * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&c->mt_row0, (size_t)c->mt_cap * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&c->n_mtiles, 4);
  c->mid_cap = mid_groups_cap((int)c->rows_max, c->n_slots, 17);
  if (e == hipSuccess) e = hipMalloc((void**)&c->mid_expert, (size_t)c->mid_cap * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&c->mid_row0, (size_t)c->mid_cap * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&c->n_mid, 4);
  if (e == hipSuccess) e = hipMalloc((void**)&c->sched_sync, (size_t)tile_sync_words(c->mt_cap) * 4);
  if (e == hipSuccess) e = hipMemset(c->sched_sync, 0, (size_t)tile_sync_words(c->mt_cap) * 4);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, c->device);
  if (e == hipSuccess && c->n_cus < 8) c->n_cus = 8;
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->copy, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->fork_ev, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->join_ev, hipEventDisableTiming);
  c->plan_cache.resize(cfg->n_layers);
  c->staged_ev.assign(cfg->n_layers, nullptr);
  for (int l = 0; l < cfg->n_layers && e == hipSuccess; l++)
    e = hipEventCreateWithFlags(&c->staged_ev[l], hipEventDisableTiming);
  for (int b = 0; b < 2 && e == hipSuccess; b++) e = hipEventCreateWithFlags(&c->done_ev[b], hipEventDisableTiming);
  if (e != hipSuccess) {
    dwdp_status s = fail(nullptr, e == hipErrorOutOfMemory ? DWDP_ENOMEM : DWDP_EHIP, "dwdp_create: %s",
                         hipGetErrorString(e));
    dwdp_destroy(c);
    return s;
  }
  *out = c;
  return DWDP_OK;
}

extern "C" void dwdp_destroy(dwdp_ctx* c) {
  if (!c) return;
  if (c->compute || c->copy) (void)hipDeviceSynchronize();
  for (void* p : c->ws)
    if (p) (void)hipFree(p);
  if (c->chunk_counts) (void)hipFree(c->chunk_counts);
  if (c->mt_expert) (void)hipFree(c->mt_expert);
  if (c->mt_row0) (void)hipFree(c->mt_row0);
  if (c->n_mtiles) (void)hipFree(c->n_mtiles);
  if (c->sched_sync) (void)hipFree(c->sched_sync);
  if (c->mid_expert) (void)hipFree(c->mid_expert);
  if (c->mid_row0) (void)hipFree(c->mid_row0);
  if (c->n_mid) (void)hipFree(c->n_mid);
  for (auto& pc : c->plan_cache) {
    if (pc.units) (void)hipFree(pc.units);
    if (pc.units_host) (void)hipHostFree(pc.units_host);
  }
  for (auto& r : c->retired) {
    if (r.units) (void)hipFree(r.units);
    if (r.units_host) (void)hipHostFree(r.units_host);
  }
  for (hipEvent_t ev : c->staged_ev)
    if (ev) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : c->done_ev)
    if (ev) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : c->prof_ev)
    if (ev) (void)hipEventDestroy(ev);
  for (auto& sp : c->tl) {
    (void)hipEventDestroy(sp.a);
    (void)hipEventDestroy(sp.b);
  }
  if (c->tl_base) (void)hipEventDestroy(c->tl_base);
  if (c->copy) (void)hipStreamDestroy(c->copy);
  if (c->aux) (void)hipStreamDestroy(c->aux);
  if (c->fork_ev) (void)hipEventDestroy(c->fork_ev);
  if (c->join_ev) (void)hipEventDestroy(c->join_ev);
  delete c;
}

extern "C" const char* dwdp_last_error(const dwdp_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

// Open a timeline span on `s`: creates two events, records the first.  Returns the span index or -1.
static int tl_open(dwdp_ctx* ctx, int kind, int layer, hipStream_t s) {
  if (!ctx->tl_on || ctx->tl.size() >= (size_t)DWDP_TIMELINE_MAX) return -1;
  dwdp_ctx::Span sp{kind, layer, nullptr, nullptr};
  if (hipEventCreate(&sp.a) != hipSuccess) return -1;
  if (hipEventCreate(&sp.b) != hipSuccess) {
    (void)hipEventDestroy(sp.a);
    return -1;
  }
  (void)hipEventRecord(sp.a, s);
  ctx->tl.push_back(sp);
  return (int)ctx->tl.size() - 1;
}
static void tl_close(dwdp_ctx* ctx, int idx, hipStream_t s) {
  if (idx >= 0) (void)hipEventRecord(ctx->tl[idx].b, s);
}

static RouteParams route_params(const dwdp_config& c) {
  return RouteParams{c.E, c.K, c.n_group, c.topk_group, c.score_fn, c.routed_scale};
}

static dwdp_status check_T(dwdp_ctx* ctx, int32_t T) {
  if (T < 0) return fail(ctx, DWDP_EINVAL, "T is negative");
  if (T > ctx->cfg.T_max) return fail(ctx, DWDP_ESHAPE, "T = %d exceeds T_max = %d", T, ctx->cfg.T_max);
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_route(dwdp_ctx* ctx, const float* logits, const float* bias, int32_t T, int32_t* topk_ids,
                                  float* topk_w) {
  if (!ctx) return DWDP_EINVAL;
  dwdp_status st = check_T(ctx, T);
  if (st != DWDP_OK) return st;
  if (T == 0) return DWDP_OK;
  if (!logits || !topk_ids || !topk_w) return fail(ctx, DWDP_EINVAL, "dwdp_route: NULL pointer");
  launch_route(logits, ctx->cfg.score_fn == DWDP_SCORE_SIGMOID ? bias : nullptr, T, route_params(ctx->cfg), topk_ids,
               topk_w, ctx->compute);
  HIP_TRY(ctx, hipGetLastError());
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_permute(dwdp_ctx* ctx, const int32_t* topk_ids, int32_t T, int32_t* expert_offsets,
                                    int32_t* perm, int32_t* inv_perm) {
  if (!ctx) return DWDP_EINVAL;
  dwdp_status st = check_T(ctx, T);
  if (st != DWDP_OK) return st;
  if (!expert_offsets) return fail(ctx, DWDP_EINVAL, "dwdp_permute: expert_offsets is NULL");
  if (T > 0 && (!topk_ids || !perm || !inv_perm)) return fail(ctx, DWDP_EINVAL, "dwdp_permute: NULL pointer");
  launch_permute(topk_ids, T, ctx->cfg.E, ctx->cfg.K, ctx->cfg.has_shared, ctx->chunk_counts, expert_offsets, perm,
                 inv_perm, nullptr, 0, ctx->compute);
  HIP_TRY(ctx, hipGetLastError());
  return DWDP_OK;
}

// ---- the permutation without a context and without any allocation ----
// Scratch of dwdp_permute_static: the per-chunk expert histograms of the multi-workgroup
// permutation.  One copy per GPU, held until the process ends; every call on a GPU uses it.
__device__ __align__(256) static int32_t scratch[DWDP_STATIC_SCRATCH_BYTES / 4];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
int32_t* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, looked up once
}  // namespace

extern "C" dwdp_status dwdp_permute_static(const int32_t* topk_ids, int32_t T, int32_t E, int32_t K,
                                           int32_t has_shared, void* stream, int32_t* expert_offsets, int32_t* perm,
                                           int32_t* inv_perm) {
  if (T < 0 || E <= 0 || K <= 0 || (has_shared != 0 && has_shared != 1))
    return fail(nullptr, DWDP_EINVAL, "dwdp_permute_static: negative or zero size");
  if (E > 1024 || K > E || K > 32) return fail(nullptr, DWDP_ESHAPE, "dwdp_permute_static: need K <= E <= 1024, K <= 32");
  if ((long)T * K > (1L << 30)) return fail(nullptr, DWDP_ESHAPE, "dwdp_permute_static: T * K too large");
  if (!expert_offsets) return fail(nullptr, DWDP_EINVAL, "dwdp_permute_static: expert_offsets is NULL");
  if (T > 0 && (!topk_ids || !perm || !inv_perm)) return fail(nullptr, DWDP_EINVAL, "dwdp_permute_static: NULL pointer");
  const long chunk = permute_multi_chunk_tokens(E);
  const long need = T > permute_chunk_tokens(E) ? (T + chunk - 1) / chunk * E * 4 : 0;
  if (need > (long)DWDP_STATIC_SCRATCH_BYTES)
    return fail(nullptr, DWDP_ESHAPE, "dwdp_permute_static: T = %d with E = %d needs %ld bytes of scratch, the static "
                "array holds %d", T, E, need, (int)DWDP_STATIC_SCRATCH_BYTES);
  int dev = 0;
  HIP_TRY(nullptr, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, DWDP_ESHAPE, "dwdp_permute_static: device index %d", dev);
  int32_t* sp;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      // the array's name is a host-side handle; its address on the current GPU comes from the runtime
      void* p = nullptr;
      HIP_TRY(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) return fail(nullptr, DWDP_EHIP, "dwdp_permute_static: no device address for the scratch array");
      g_scratch_ptr[dev] = (int32_t*)p;
    }
    sp = g_scratch_ptr[dev];
  }
  launch_permute(topk_ids, T, E, K, has_shared, sp, expert_offsets, perm, inv_perm, nullptr, 0, (hipStream_t)stream);
  HIP_TRY(nullptr, hipGetLastError());
  return DWDP_OK;
}

// Profiling events per call: route, permute, quant, combine and end on the compute stream; the
// streaming chain's GEMM-1 start, GEMM-2 start and end on that chain's stream; the tiled chain's
// GEMM-1 start, GEMM-2 start and end on the compute stream.
constexpr int kProfMain = 6;
constexpr int kProfStreamEnd = kProfMain + 4;  // after the streaming chain's GEMM-2, on that chain's stream
constexpr int kProfPerCall = kProfMain + 1 + 3 + 1;
static inline hipEvent_t prof_event(dwdp_ctx* ctx, int idx) {
  return ctx->prof_ev[(size_t)ctx->prof_calls * kProfPerCall + idx];
}

extern "C" dwdp_status dwdp_moe_forward(dwdp_ctx* ctx, int32_t layer, const void* x, const float* logits,
                                        const float* bias, int32_t T, const dwdp_expert_ptrs* table, void* y) {
  if (!ctx) return DWDP_EINVAL;
  dwdp_status st = check_T(ctx, T);
  if (st != DWDP_OK) return st;
  const dwdp_config& c = ctx->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(ctx, DWDP_EINVAL, "layer %d outside [0,%d)", layer, c.n_layers);
  if (T > 0 && (!x || !logits || !table || !y)) return fail(ctx, DWDP_EINVAL, "dwdp_moe_forward: NULL pointer");
  hipStream_t s = ctx->compute;
  const int b = layer & 1;
  const bool consume = ctx->pending_layer[b] == layer;
  if (T == 0) {
    // nothing to compute, but the staging buffer is still released in stream order
    if (consume) HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->staged_ev[layer], 0));
    HIP_TRY(ctx, hipEventRecord(ctx->done_ev[b], s));
    ctx->done_valid[b] = true;
    if (consume) ctx->pending_layer[b] = -1;
    return DWDP_OK;
  }
  bool forked = false, released = false;
  auto enqueue = [&]() -> dwdp_status {
  const bool prof = ctx->prof && ctx->prof_calls < DWDP_PROFILE_MAX_CALLS;
  int32_t* ids = (int32_t*)ctx->ws[DWDP_WS_TOPK_IDS];
  float* tw = (float*)ctx->ws[DWDP_WS_TOPK_W];
  int32_t* off = (int32_t*)ctx->ws[DWDP_WS_OFFSETS];
  int32_t* perm = (int32_t*)ctx->ws[DWDP_WS_PERM];
  int32_t* inv = (int32_t*)ctx->ws[DWDP_WS_INV_PERM];

  GemmArgs ga{table, off, perm, ctx->n_slots, c.E, T, c.H, c.I, c.K};
  const bool mx = c.w_dtype == DWDP_W_MXFP4;
  const bool fp8 = c.w_dtype != DWDP_W_BF16;  // FP8 activations and intermediates (FP8 and MXFP4 weights)
  // Experts with 1..smr rows stream their weights; the others go through the LDS-tiled kernel
  // (FP8 and MXFP4 weights).
  const int rows = T * c.K + (c.has_shared ? T : 0);
  // Default threshold: 64 rows with FP8 weights (17 .. 64 rows go to the multi-tile streaming
  // items), 16 with MXFP4 weights (no multi-tile items there: larger experts go to the tiled kernels).
  const int smr = ctx->stream_max_rows >= 0 ? ctx->stream_max_rows : (mx ? 16 : 64);
  const bool use_stream = smr > 0;
  const bool use_mid = fp8 && !mx && smr > 16 && T > 16;
  // The tiled kernels are launched when an expert can have more than smr rows (it holds at most
  // T) -- and, when the row-group items exist as the alternative, only if the experts average at
  // least 16 rows: below that a tiled expert is a rare outlier (the shared expert, a hot routed
  // one), which the device-side rule of the list builder would send to the row groups anyway,
  // and the launch is skipped because even its surplus workgroups each need a whole compute unit
  // to start and exit (next to a prefetch copy that occupies every unit they wait for it to end).
  const bool use_tile = fp8 && T > smr && (!use_mid || (long)rows >= 16L * ctx->n_slots);
  TileSched ts{};
  if (use_tile) {
    ts.mt_expert = ctx->mt_expert;
    ts.mt_row0 = ctx->mt_row0;
    ts.n_mtiles = ctx->n_mtiles;
    ts.sync = ctx->sched_sync;
    ts.n_mt_max = tile_mtiles_cap(rows, ctx->n_slots, smr);
    ts.sync_words = tile_sync_words(ts.n_mt_max);
    // fewer tiled GEMM-1 items than half the compute units: not worth whole-unit workgroups
    const int p1 = c.I / 128;
    ts.min_tiles = use_mid ? (ctx->n_cus / 2 + p1 - 1) / p1 : 0;
    ts.wg_limit_full = ctx->n_cus;
    ts.wg_limit_shared = ctx->tile_share_wgs > 0 ? ctx->tile_share_wgs : ctx->n_cus * 13 / 16 / 8 * 8;
    ts.share_min_experts = 16;
  }
  if (use_mid) {
    ts.mid_expert = ctx->mid_expert;
    ts.mid_row0 = ctx->mid_row0;
    ts.n_mid = ctx->n_mid;
    ts.mid_min_rows = 17;
    // groups of the experts with 17 .. min(smr, T) rows
    ts.mid_cap = mid_groups_cap(rows, ctx->n_slots, 17);
  }
  // Two launches prepare the GEMMs: routing with the (independent) activation quantisation
  // riding along as extra workgroups, and the permutation, whose last single-workgroup step
  // also lists the M tiles of the tiled experts.
  if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_ROUTE), s));
  const float* rbias = c.score_fn == DWDP_SCORE_SIGMOID ? bias : nullptr;
  if (fp8)
    launch_route_quant(logits, rbias, T, route_params(c), ids, tw, x, c.H, (uint8_t*)ctx->ws[DWDP_WS_XQ],
                       (float*)ctx->ws[DWDP_WS_XS], s);
  else
    launch_route(logits, rbias, T, route_params(c), ids, tw, s);
  if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_PERMUTE), s));
  launch_permute(ids, T, c.E, c.K, c.has_shared, ctx->chunk_counts, off, perm, inv,
                 (use_tile || use_mid) ? &ts : nullptr, smr, s);
  if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_QUANT), s));
  // Only the grouped GEMMs read expert weights: the wait for the staged experts goes here.
  if (consume) HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->staged_ev[layer], 0));
  const int span = tl_open(ctx, DWDP_SPAN_GEMM, layer, s);
  // Two independent chains when both kernel families have work.  The tiled chain stays on the
  // compute stream and is enqueued first: its few, large workgroups need whole CUs, and once
  // the streaming kernel has filled the chip they would only get one when it drains.  The
  // streamed chain runs on aux behind a fork event (inheriting the wait above) and is joined
  // before the combine.
  const bool two = fp8 && use_tile && use_stream;
  hipStream_t sc = two ? ctx->aux : s;  // stream of the streaming chain
  if (two) {
    HIP_TRY(ctx, hipEventRecord(ctx->fork_ev, s));
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->aux, ctx->fork_ev, 0));
    forked = true;
  }
  if (fp8) {
    if (use_stream) {
      if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_GEMM1), sc));
      if (mx)
        launch_gemm1_mx(ga, smr, (const uint8_t*)ctx->ws[DWDP_WS_XQ], (const float*)ctx->ws[DWDP_WS_XS],
                        (uint8_t*)ctx->ws[DWDP_WS_HQ], (float*)ctx->ws[DWDP_WS_HS], sc);
      else
        launch_gemm1_fp8(ga, smr, ts, (const uint8_t*)ctx->ws[DWDP_WS_XQ], (const float*)ctx->ws[DWDP_WS_XS],
                         (uint8_t*)ctx->ws[DWDP_WS_HQ], (float*)ctx->ws[DWDP_WS_HS], sc);
      if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_GEMM2), sc));
      if (mx)
        launch_gemm2_mx(ga, smr, (const uint8_t*)ctx->ws[DWDP_WS_HQ], (const float*)ctx->ws[DWDP_WS_HS],
                        ctx->ws[DWDP_WS_YP], sc);
      else
        launch_gemm2_fp8(ga, smr, ts, (const uint8_t*)ctx->ws[DWDP_WS_HQ], (const float*)ctx->ws[DWDP_WS_HS],
                         ctx->ws[DWDP_WS_YP], sc);
      if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfStreamEnd), sc));
      if (two) HIP_TRY(ctx, hipEventRecord(ctx->join_ev, ctx->aux));
    } else if (prof) {
      HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_GEMM1), s));
      HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_GEMM2), s));
      HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfStreamEnd), s));
    }
    if (use_tile) {
      // one launch per GEMM (GEMM1_TILE and GEMM2_TILE timed separately), or with the fused
      // persistent schedule one launch for both (GEMM1_TILE is the whole launch, GEMM2_TILE zero)
      const uint8_t* xq = (const uint8_t*)ctx->ws[DWDP_WS_XQ];
      const float* xs = (const float*)ctx->ws[DWDP_WS_XS];
      uint8_t* hq = (uint8_t*)ctx->ws[DWDP_WS_HQ];
      float* hs = (float*)ctx->ws[DWDP_WS_HS];
      const int sched = ctx->tile_schedule == DWDP_TILE_PER_ITEM ? 0 : 1;
      const bool fused = ctx->tile_schedule == DWDP_TILE_PERSISTENT_FUSED;
      if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfMain + 1), s));
      launch_gemm_fp8_tile(ga, ts, mx, sched, fused ? 3 : 1, xq, xs, hq, hs, ctx->ws[DWDP_WS_YP], ctx->n_cus, s);
      if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfMain + 2), s));
      if (!fused) launch_gemm_fp8_tile(ga, ts, mx, sched, 2, xq, xs, hq, hs, ctx->ws[DWDP_WS_YP], ctx->n_cus, s);
      if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfMain + 3), s));
    }
    if (two) {
      HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->join_ev, 0));
      forked = false;
    }
  } else {
    if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_GEMM1), s));
    launch_gemm1_bf16(ga, x, ctx->ws[DWDP_WS_HQ], s);
    if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_GEMM2), s));
    launch_gemm2_bf16(ga, ctx->ws[DWDP_WS_HQ], ctx->ws[DWDP_WS_YP], s);
    if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfStreamEnd), s));
  }
  tl_close(ctx, span, s);
  // The layer's weights have been read once GEMM-2 is done: release the staging buffer here.
  HIP_TRY(ctx, hipEventRecord(ctx->done_ev[b], s));
  released = true;
  ctx->done_valid[b] = true;
  if (consume) ctx->pending_layer[b] = -1;
  if (prof) HIP_TRY(ctx, hipEventRecord(prof_event(ctx, DWDP_STAGE_COMBINE), s));
  launch_combine(ctx->ws[DWDP_WS_YP], !fp8, inv, tw, T, c.H, c.K, c.has_shared, y, s);
  if (prof) {
    HIP_TRY(ctx, hipEventRecord(prof_event(ctx, kProfMain), s));
    ctx->prof_has_aux[ctx->prof_calls] = (fp8 && use_tile) ? 1 : 0;
    ctx->prof_calls++;
  }
  HIP_TRY(ctx, hipGetLastError());
  return DWDP_OK;
  };
  st = enqueue();
  if (st != DWDP_OK) {
    // A HIP call failed half-way.  Leave the context in a state the next call can start from: the
    // second chain is joined back into the compute stream, and the staging buffer is released in
    // stream order (whatever was enqueued has been enqueued; the layer's result is not valid).
    // The message of the first failure is kept.
    if (forked && hipEventRecord(ctx->join_ev, ctx->aux) == hipSuccess) (void)hipStreamWaitEvent(s, ctx->join_ev, 0);
    if (!released && hipEventRecord(ctx->done_ev[b], s) == hipSuccess) ctx->done_valid[b] = true;
    if (consume) ctx->pending_layer[b] = -1;
    (void)hipGetLastError();
  }
  return st;
}

// The copy plan of paper Section 4.3.2 (Listing 1) in issue order, produced one entry at a time:
// parameters in turn; within a parameter the slices in turn; within a slice every peer once, in
// the caller's order.  Entry = (index into src/dst, byte offset inside the region, bytes).
namespace {
struct PlanWalk {
  const size_t* bytes;
  int n_peers, n_params;
  size_t slice;
  int p = 0, peer = 0;
  size_t off = 0;
  PlanWalk(const size_t* b, int peers, int params, size_t s) : bytes(b), n_peers(peers), n_params(params), slice(s) {
    skip_empty();
  }
  void skip_empty() {
    while (p < n_params && (bytes[p] == 0 || n_peers == 0)) p++;
  }
  bool done() const { return p >= n_params; }
  size_t region() const { return (size_t)peer * n_params + p; }
  size_t chunk() const {
    const size_t left = bytes[p] - off;
    return slice && slice < left ? slice : left;
  }
  void advance() {
    if (++peer < n_peers) return;
    peer = 0;
    off += chunk();
    if (off >= bytes[p]) {
      off = 0;
      p++;
      skip_empty();
    }
  }
};
}  // namespace

extern "C" dwdp_status dwdp_build_copy_plan(const void* const* src, void* const* dst, const size_t* bytes,
                                            int32_t n_peers, int32_t n_params, size_t slice_bytes, void** plan_dst,
                                            const void** plan_src, size_t* plan_bytes, size_t cap, size_t* n_out) {
  if (!src || !dst || !bytes || !n_out || n_peers < 0 || n_params < 0) return DWDP_EINVAL;
  if (cap > 0 && (!plan_dst || !plan_src || !plan_bytes)) return DWDP_EINVAL;
  size_t n = 0;
  for (PlanWalk w(bytes, n_peers, n_params, slice_bytes); !w.done(); w.advance(), n++) {
    if (n >= cap) continue;
    plan_dst[n] = (char*)dst[w.region()] + w.off;
    plan_src[n] = (const char*)src[w.region()] + w.off;
    plan_bytes[n] = w.chunk();
  }
  *n_out = n;
  return DWDP_OK;
}

static dwdp_status check_prefetch_args(dwdp_ctx* ctx, int32_t layer, const void* const* src, void* const* dst,
                                       const size_t* bytes, int32_t n_peers, int32_t n_params) {
  if (layer < 0 || layer >= ctx->cfg.n_layers)
    return fail(ctx, DWDP_EINVAL, "layer %d outside [0,%d)", layer, ctx->cfg.n_layers);
  if (!src || !dst || !bytes || n_peers < 0 || n_params < 0)
    return fail(ctx, DWDP_EINVAL, "prefetch: NULL pointer or negative count");
  for (int i = 0; i < n_peers * n_params; i++)
    if (bytes[i % n_params] && (!src[i] || !dst[i])) return fail(ctx, DWDP_EINVAL, "NULL region pointer at %d", i);
  return DWDP_OK;
}

// Device copy of a layer's plan for the copy-plan kernel, cut into units of at most 256 KiB so
// that the workgroups share evenly.  Built when the arguments differ from the cached ones: the
// units are written into a pinned host array and uploaded with an asynchronous copy on the copy
// stream, i.e. ordered before the kernel that reads them and after earlier launches that read
// the previous plan (same stream); nothing waits on the host.  A replaced plan's buffers are
// kept until dwdp_destroy (an upload or a launch may still be reading them).
static dwdp_status ensure_device_plan(dwdp_ctx* ctx, int32_t layer, const void* const* src, void* const* dst,
                                      const size_t* bytes, int32_t n_peers, int32_t n_params, size_t slice_bytes) {
  std::vector<uintptr_t> key;
  key.push_back((uintptr_t)n_peers);
  key.push_back((uintptr_t)n_params);
  key.push_back((uintptr_t)slice_bytes);
  for (int i = 0; i < n_peers * n_params; i++) {
    key.push_back((uintptr_t)src[i]);
    key.push_back((uintptr_t)dst[i]);
  }
  for (int p = 0; p < n_params; p++) key.push_back((uintptr_t)bytes[p]);
  dwdp_ctx::PlanCache& pc = ctx->plan_cache[layer];
  if (pc.valid && pc.key == key) return DWDP_OK;
  constexpr size_t kUnit = 256 << 10;
  size_t n_units = 0;
  for (PlanWalk w(bytes, n_peers, n_params, slice_bytes); !w.done(); w.advance())
    n_units += (w.chunk() + kUnit - 1) / kUnit;
  if (n_units > (size_t)1 << 30) return fail(ctx, DWDP_ESHAPE, "copy plan of %zu units is too long", n_units);
  if (pc.units) ctx->retired.push_back({pc.units, pc.units_host});
  pc.units = nullptr;
  pc.units_host = nullptr;
  pc.valid = false;
  pc.n_units = 0;
  if (n_units) {
    HIP_TRY(ctx, hipHostMalloc((void**)&pc.units_host, n_units * sizeof(CopyUnit), hipHostMallocDefault));
    HIP_TRY(ctx, hipMalloc((void**)&pc.units, n_units * sizeof(CopyUnit)));
    size_t u = 0;
    for (PlanWalk w(bytes, n_peers, n_params, slice_bytes); !w.done(); w.advance())
      for (size_t o = 0, c = w.chunk(); o < c; o += kUnit)
        pc.units_host[u++] = CopyUnit{(char*)dst[w.region()] + w.off + o, (const char*)src[w.region()] + w.off + o,
                                      c - o < kUnit ? c - o : kUnit};
    HIP_TRY(ctx, hipMemcpyAsync(pc.units, pc.units_host, n_units * sizeof(CopyUnit), hipMemcpyHostToDevice, ctx->copy));
  }
  pc.n_units = (int)n_units;
  pc.key = key;
  pc.valid = true;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_prepare_prefetch(dwdp_ctx* ctx, int32_t layer, const void* const* src, void* const* dst,
                                             const size_t* bytes, int32_t n_peers, int32_t n_params,
                                             size_t slice_bytes) {
  if (!ctx) return DWDP_EINVAL;
  dwdp_status st = check_prefetch_args(ctx, layer, src, dst, bytes, n_peers, n_params);
  if (st != DWDP_OK) return st;
  return ensure_device_plan(ctx, layer, src, dst, bytes, n_peers, n_params, slice_bytes);
}

extern "C" dwdp_status dwdp_prefetch_layer(dwdp_ctx* ctx, int32_t layer, const void* const* src, void* const* dst,
                                           const size_t* bytes, int32_t n_peers, int32_t n_params,
                                           size_t slice_bytes) {
  if (!ctx) return DWDP_EINVAL;
  dwdp_status st = check_prefetch_args(ctx, layer, src, dst, bytes, n_peers, n_params);
  if (st != DWDP_OK) return st;
  const int b = layer & 1;
  if (ctx->pending_layer[b] != -1)
    return fail(ctx, DWDP_ESTATE, "staging buffer %d still holds layer %d, which no dwdp_moe_forward has consumed", b,
                ctx->pending_layer[b]);
  if (ctx->copy_mode == DWDP_COPY_KERNEL) {
    st = ensure_device_plan(ctx, layer, src, dst, bytes, n_peers, n_params, slice_bytes);
    if (st != DWDP_OK) return st;
  }
  // double buffering: the buffer is free once its previous reader has finished
  if (ctx->done_valid[b]) HIP_TRY(ctx, hipStreamWaitEvent(ctx->copy, ctx->done_ev[b], 0));
  const int span = tl_open(ctx, DWDP_SPAN_COPY, layer, ctx->copy);
  if (ctx->copy_mode == DWDP_COPY_KERNEL) {
    launch_copy_plan(ctx->plan_cache[layer].units, ctx->plan_cache[layer].n_units, ctx->copy_wgs, ctx->copy);
    HIP_TRY(ctx, hipGetLastError());
  } else {
    for (PlanWalk w(bytes, n_peers, n_params, slice_bytes); !w.done(); w.advance())
      HIP_TRY(ctx, hipMemcpyAsync((char*)dst[w.region()] + w.off, (const char*)src[w.region()] + w.off, w.chunk(),
                                  hipMemcpyDeviceToDevice, ctx->copy));
  }
  tl_close(ctx, span, ctx->copy);
  HIP_TRY(ctx, hipEventRecord(ctx->staged_ev[layer], ctx->copy));
  ctx->pending_layer[b] = layer;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_merge_experts(dwdp_ctx* ctx, int32_t layer, const dwdp_expert_ptrs* table_host,
                                          int32_t n_slots, void* w13_out, float* s13_out, void* w2_out,
                                          float* s2_out, dwdp_expert_ptrs* merged_table_host) {
  if (!ctx) return DWDP_EINVAL;
  if (!table_host || !merged_table_host || !w13_out || !w2_out || n_slots < 0)
    return fail(ctx, DWDP_EINVAL, "dwdp_merge_experts: NULL pointer");
  const dwdp_config& c = ctx->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(ctx, DWDP_EINVAL, "layer %d outside [0,%d)", layer, c.n_layers);
  if (c.w_dtype == DWDP_W_MXFP4)
    return fail(ctx, DWDP_ESHAPE, "dwdp_merge_experts: the merge baseline is built for bf16 and FP8 weights");
  const bool fp8 = c.w_dtype == DWDP_W_FP8;
  if (fp8 && (!s13_out || !s2_out)) return fail(ctx, DWDP_EINVAL, "dwdp_merge_experts: scale outputs are NULL");
  // a pending prefetch of this layer: the merge reads the staged experts, so it waits for them
  // (the buffer stays the layer's until its dwdp_moe_forward has run)
  if (ctx->pending_layer[layer & 1] == layer) HIP_TRY(ctx, hipStreamWaitEvent(ctx->compute, ctx->staged_ev[layer], 0));
  const size_t el = fp8 ? 1 : 2;
  const size_t b13 = (size_t)2 * c.I * c.H * el, b2 = (size_t)c.H * c.I * el;
  const size_t n13 = (size_t)(2 * c.I / 128) * (c.H / 128) * 4, n2 = (size_t)(c.H / 128) * (c.I / 128) * 4;
  // one copy per run of experts that already lie back to back in the source (a resident
  // shard, one peer's staged shard): the merged image is the same, the call count is not
  auto field = [&](int e, int which) -> const char* {
    const dwdp_expert_ptrs& t = table_host[e];
    return (const char*)(which == 0 ? t.w13 : which == 1 ? (const void*)t.s13 : which == 2 ? t.w2 : (const void*)t.s2);
  };
  char* const outs[4] = {(char*)w13_out, (char*)s13_out, (char*)w2_out, (char*)s2_out};
  const size_t sizes[4] = {b13, n13, b2, n2};
  for (int which = 0; which < 4; which++) {
    if (!fp8 && (which & 1)) continue;  // no scales
    const size_t bytes = sizes[which];
    int e = 0;
    while (e < n_slots) {
      int f = e + 1;
      while (f < n_slots && field(f, which) == field(e, which) + (size_t)(f - e) * bytes) f++;
      HIP_TRY(ctx, hipMemcpyAsync(outs[which] + (size_t)e * bytes, field(e, which), (size_t)(f - e) * bytes,
                                  hipMemcpyDeviceToDevice, ctx->compute));
      e = f;
    }
  }
  for (int e = 0; e < n_slots; e++) {
    dwdp_expert_ptrs m{};
    m.w13 = outs[0] + (size_t)e * b13;
    m.w2 = outs[2] + (size_t)e * b2;
    if (fp8) {
      m.s13 = (const float*)(outs[1] + (size_t)e * n13);
      m.s2 = (const float*)(outs[3] + (size_t)e * n2);
    }
    merged_table_host[e] = m;
  }
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_set_copy_engine(dwdp_ctx* ctx, int32_t mode, int32_t n_workgroups) {
  if (!ctx) return DWDP_EINVAL;
  if (mode != DWDP_COPY_MEMCPY && mode != DWDP_COPY_KERNEL)
    return fail(ctx, DWDP_EINVAL, "dwdp_set_copy_engine: unknown mode %d", mode);
  if (mode == DWDP_COPY_KERNEL && (n_workgroups < 1 || n_workgroups > 65535))
    return fail(ctx, DWDP_EINVAL, "dwdp_set_copy_engine: n_workgroups must be in [1,65535]");
  ctx->copy_mode = mode;
  if (mode == DWDP_COPY_KERNEL) ctx->copy_wgs = n_workgroups;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_set_stream_max_rows(dwdp_ctx* ctx, int32_t max_rows) {
  if (!ctx) return DWDP_EINVAL;
  if (max_rows < 0) return fail(ctx, DWDP_EINVAL, "dwdp_set_stream_max_rows: negative");
  ctx->stream_max_rows = max_rows;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_set_tile_share(dwdp_ctx* ctx, int32_t n_workgroups) {
  if (!ctx) return DWDP_EINVAL;
  if (n_workgroups < 0 || n_workgroups % 8) return fail(ctx, DWDP_EINVAL, "dwdp_set_tile_share: need a multiple of 8");
  ctx->tile_share_wgs = n_workgroups;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_set_tile_schedule(dwdp_ctx* ctx, int32_t mode) {
  if (!ctx) return DWDP_EINVAL;
  if (mode != DWDP_TILE_PER_ITEM && mode != DWDP_TILE_PERSISTENT && mode != DWDP_TILE_PERSISTENT_FUSED)
    return fail(ctx, DWDP_EINVAL, "dwdp_set_tile_schedule: unknown mode %d", mode);
  ctx->tile_schedule = mode;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_pack_fp8_weight(dwdp_ctx* ctx, const void* src, void* dst, int64_t rows, int64_t cols) {
  if (!ctx) return DWDP_EINVAL;
  if (rows < 0 || cols < 0) return fail(ctx, DWDP_EINVAL, "dwdp_pack_fp8_weight: negative size");
  if (rows % 16 || cols % 128 || cols > (1 << 30))
    return fail(ctx, DWDP_ESHAPE, "dwdp_pack_fp8_weight: rows must be a multiple of 16 and cols of 128");
  if (rows * cols == 0) return DWDP_OK;
  if (!src || !dst || src == dst) return fail(ctx, DWDP_EINVAL, "dwdp_pack_fp8_weight: NULL or aliased pointers");
  launch_pack_fp8_tiles(src, dst, rows, (int)cols, ctx->compute);
  HIP_TRY(ctx, hipGetLastError());
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_pack_mxfp4_weight(dwdp_ctx* ctx, const void* src_codes, const void* src_scales,
                                              void* dst_codes, void* dst_scales, int64_t rows, int64_t cols) {
  if (!ctx) return DWDP_EINVAL;
  if (rows < 0 || cols < 0) return fail(ctx, DWDP_EINVAL, "dwdp_pack_mxfp4_weight: negative size");
  if (rows % 16 || cols % 128 || cols > (1 << 30))
    return fail(ctx, DWDP_ESHAPE, "dwdp_pack_mxfp4_weight: rows must be a multiple of 16 and cols of 128");
  if (rows * cols == 0) return DWDP_OK;
  if (!src_codes || !src_scales || !dst_codes || !dst_scales || src_codes == dst_codes || src_scales == dst_scales)
    return fail(ctx, DWDP_EINVAL, "dwdp_pack_mxfp4_weight: NULL or aliased pointers");
  launch_pack_mxfp4(src_codes, src_scales, dst_codes, dst_scales, rows, (int)cols, ctx->compute);
  HIP_TRY(ctx, hipGetLastError());
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_profile_enable(dwdp_ctx* ctx, int32_t on) {
  if (!ctx) return DWDP_EINVAL;
  if (on && ctx->prof_ev.empty()) {
    ctx->prof_ev.assign((size_t)DWDP_PROFILE_MAX_CALLS * kProfPerCall, nullptr);
    ctx->prof_has_aux.assign(DWDP_PROFILE_MAX_CALLS, 0);
    for (auto& ev : ctx->prof_ev) HIP_TRY(ctx, hipEventCreate(&ev));
  }
  ctx->prof = on != 0;
  ctx->prof_calls = 0;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_profile_read(dwdp_ctx* ctx, float* ms_sum, int32_t* n_calls) {
  if (!ctx) return DWDP_EINVAL;
  if (!ms_sum || !n_calls) return fail(ctx, DWDP_EINVAL, "dwdp_profile_read: NULL pointer");
  HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->aux));
  for (int s = 0; s < DWDP_N_STAGES; s++) ms_sum[s] = 0.f;
  for (int i = 0; i < ctx->prof_calls; i++) {
    const hipEvent_t* ev = &ctx->prof_ev[(size_t)i * kProfPerCall];
    for (int s = 0; s < kProfMain; s++) {
      float ms = 0.f;
      // GEMM-2 ends where the streaming chain ends, not where the combine starts (that is after the join)
      HIP_TRY(ctx, hipEventElapsedTime(&ms, ev[s], ev[s == DWDP_STAGE_GEMM2 ? kProfStreamEnd : s + 1]));
      ms_sum[s] += ms;
    }
    if (ctx->prof_has_aux[i]) {
      float ms = 0.f;
      HIP_TRY(ctx, hipEventElapsedTime(&ms, ev[kProfMain + 1], ev[kProfMain + 2]));
      ms_sum[DWDP_STAGE_GEMM1_TILE] += ms;
      HIP_TRY(ctx, hipEventElapsedTime(&ms, ev[kProfMain + 2], ev[kProfMain + 3]));
      ms_sum[DWDP_STAGE_GEMM2_TILE] += ms;
    }
  }
  *n_calls = ctx->prof_calls;
  ctx->prof_calls = 0;
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_timeline_enable(dwdp_ctx* ctx, int32_t on) {
  if (!ctx) return DWDP_EINVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->copy));
  for (auto& sp : ctx->tl) {
    (void)hipEventDestroy(sp.a);
    (void)hipEventDestroy(sp.b);
  }
  ctx->tl.clear();
  ctx->tl_on = on != 0;
  if (ctx->tl_on) {
    if (!ctx->tl_base) HIP_TRY(ctx, hipEventCreate(&ctx->tl_base));
    HIP_TRY(ctx, hipEventRecord(ctx->tl_base, ctx->compute));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
  }
  return DWDP_OK;
}

extern "C" dwdp_status dwdp_timeline_read(dwdp_ctx* ctx, int32_t* kind, int32_t* layer, float* start_ms,
                                          float* end_ms, int32_t cap, int32_t* n_out) {
  if (!ctx) return DWDP_EINVAL;
  if (!n_out || cap < 0 || (cap > 0 && (!kind || !layer || !start_ms || !end_ms)))
    return fail(ctx, DWDP_EINVAL, "dwdp_timeline_read: NULL pointer");
  HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->copy));
  const int n = (int)ctx->tl.size();
  for (int i = 0; i < n && i < cap; i++) {
    kind[i] = ctx->tl[i].kind;
    layer[i] = ctx->tl[i].layer;
    HIP_TRY(ctx, hipEventElapsedTime(&start_ms[i], ctx->tl_base, ctx->tl[i].a));
    HIP_TRY(ctx, hipEventElapsedTime(&end_ms[i], ctx->tl_base, ctx->tl[i].b));
  }
  *n_out = n;
  return DWDP_OK;
}

extern "C" void* dwdp_workspace_ptr(dwdp_ctx* ctx, int32_t which) {
  if (!ctx || which < 0 || which >= DWDP_N_WS) return nullptr;
  if (which == DWDP_WS_SCHED) return ctx->sched_sync;
  return ctx->ws[which];
}

extern "C" void* dwdp_copy_stream(dwdp_ctx* ctx) { return ctx ? (void*)ctx->copy : nullptr; }
