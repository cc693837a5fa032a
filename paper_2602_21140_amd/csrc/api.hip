// Context, map update (recovery step), graph replay and timing of the failure-remapped MoE layer.
#include <algorithm>
#include <mutex>
#include <new>
#include <utility>

#include "ctx.hpp"

namespace revive {


int fail(const revive_ctx* ctx, int status, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf; else noctx_error() = buf;
  return status;
}

int check_hip(const revive_ctx* ctx, hipError_t e, const char* what) {
  if (e == hipSuccess) return REVIVE_OK;
  return fail(ctx, REVIVE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

hipError_t allow_dynamic_lds(const void* kernel, size_t lds) {
  static std::mutex mu;
  static std::vector<std::pair<int, const void*>> done;  // (device, kernel) pairs already configured
  int dev = 0;
  hipError_t rc = hipGetDevice(&dev);
  if (rc != hipSuccess) return rc;
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& d : done)
    if (d.first == dev && d.second == kernel) return hipSuccess;
  rc = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  if (rc == hipSuccess) done.emplace_back(dev, kernel);
  return rc;
}

KernelTimer::KernelTimer(revive_ctx* c, int kernel, hipStream_t s) : ctx(c), stream(s) {
  if (!ctx->timing) return;
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone) return;
  if (ctx->slots_used == ctx->slots.size()) fold_timing(ctx);
  slot = &ctx->slots[ctx->slots_used++];
  slot->kernel = kernel;
  (void)hipEventRecord(slot->start, s);
}

KernelTimer::~KernelTimer() {
  if (slot) (void)hipEventRecord(slot->stop, stream);
}

int fold_timing(revive_ctx* ctx) {
  for (size_t i = 0; i < ctx->slots_used; ++i) {
    TimingSlot& s = ctx->slots[i];
    REVIVE_HIP(ctx, hipEventSynchronize(s.stop));
    float ms = 0.f;
    REVIVE_HIP(ctx, hipEventElapsedTime(&ms, s.start, s.stop));
    ctx->time_ms[s.kernel] += ms;
    ctx->time_n[s.kernel] += 1;
  }
  ctx->slots_used = 0;
  return REVIVE_OK;
}

}  // namespace revive

using namespace revive;

extern "C" {

int revive_create(const revive_config* cfg, revive_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return fail(nullptr, REVIVE_EINVAL, "revive_create: null argument");
  const revive_config& c = *cfg;
  const int64_t P = static_cast<int64_t>(c.n_ranks) * c.slots_per_rank;
  {
    int rc = check_config(c, &noctx_error());
    if (rc != REVIVE_OK) return rc;
  }

  revive_ctx* ctx = new (std::nothrow) revive_ctx();
  if (!ctx) return fail(nullptr, REVIVE_ENOMEM, "revive_create: out of host memory");
  ctx->cfg = c;
  ctx->P = static_cast<int>(P);
  ctx->elem = c.dtype == REVIVE_DTYPE_BF16 ? 2 : 4;

  MapLayout& m = ctx->map;
  m.off_count = 0;
  m.off_table = align_up(m.off_count + sizeof(int32_t) * c.E, 16);
  m.off_alive = align_up(m.off_table + sizeof(int32_t) * c.E * c.max_replicas, 16);
  m.off_lrank = align_up(m.off_alive + static_cast<size_t>(P), 16);
  m.off_nlive = align_up(m.off_lrank + sizeof(int32_t) * c.n_ranks, 16);
  m.bytes = align_up(m.off_nlive + 4 * sizeof(int32_t), 16);

  const int64_t N_max = static_cast<int64_t>(c.T_max) * c.k;
  const int tile_m = c.dtype == REVIVE_DTYPE_BF16 ? kTileM_bf16 : kTileM_f32;
  Workspace& w = ctx->ws;
  size_t off = 0;
  w.off_block_hist = off;
  off = align_up(off + sizeof(int32_t) * std::max<int64_t>(1, ceil_div(static_cast<int>(N_max), kDispatchChunk)) * P, 256);
  w.off_ticket = off;
  off = align_up(off + sizeof(uint32_t), 256);
  w.off_tiles = off;
  off = align_up(off + sizeof(MTile) * max_tiles(N_max, static_cast<int>(P), tile_m), 256);
  w.off_tile_count = off;
  off = align_up(off + 4 * sizeof(int32_t), 256);
  w.off_h = off;
  off = align_up(off + ctx->elem * N_max * c.I, 256);
  w.off_h_shared = off;
  off = align_up(off + ctx->elem * static_cast<size_t>(c.T_max) * c.I_shared, 256);
  w.bytes = off;

  int rc = check_hip(nullptr, hipGetDevice(&ctx->device), "hipGetDevice");
  if (rc == REVIVE_OK) rc = check_hip(nullptr, hipMalloc(reinterpret_cast<void**>(&ctx->d_map), m.bytes), "hipMalloc(map)");
  if (rc == REVIVE_OK) rc = check_hip(nullptr, hipMemset(ctx->d_map, 0, m.bytes), "hipMemset(map)");
  if (rc == REVIVE_OK)
    rc = check_hip(nullptr, hipMalloc(reinterpret_cast<void**>(&ctx->d_phys_to_logical), sizeof(int32_t) * P), "hipMalloc(p2l)");
  for (int i = 0; i < 2 && rc == REVIVE_OK; ++i) {
    rc = check_hip(nullptr, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_stage[i]), m.bytes, hipHostMallocDefault), "hipHostMalloc");
    if (rc == REVIVE_OK) rc = check_hip(nullptr, hipEventCreateWithFlags(&ctx->stage_done[i], hipEventDisableTiming), "hipEventCreate");
  }
  if (rc == REVIVE_OK) rc = init_static_dispatch_scratch(nullptr);
  if (rc != REVIVE_OK) {
    revive_destroy(ctx);
    return rc;
  }
  ctx->host_blob.assign(m.bytes, 0);
  *out = ctx;
  return REVIVE_OK;
}

int revive_destroy(revive_ctx* ctx) {
  if (!ctx) return REVIVE_OK;
  for (int i = 0; i < 2; ++i) {
    if (ctx->stage_done[i]) {
      if (ctx->stage_used[i]) (void)hipEventSynchronize(ctx->stage_done[i]);
      (void)hipEventDestroy(ctx->stage_done[i]);
    }
    if (ctx->h_stage[i]) (void)hipHostFree(ctx->h_stage[i]);
  }
  for (auto& s : ctx->slots) {
    (void)hipEventDestroy(s.start);
    (void)hipEventDestroy(s.stop);
  }
  if (ctx->d_map) (void)hipFree(ctx->d_map);
  if (ctx->d_phys_to_logical) (void)hipFree(ctx->d_phys_to_logical);
  delete ctx;
  return REVIVE_OK;
}

int revive_workspace_bytes(const revive_ctx* ctx, size_t* bytes) {
  if (!ctx || !bytes) return fail(ctx, REVIVE_EINVAL, "revive_workspace_bytes: null argument");
  *bytes = ctx->ws.bytes;
  return REVIVE_OK;
}

int revive_bind_workspace(revive_ctx* ctx, void* dev, size_t bytes) {
  if (!ctx || !dev) return fail(ctx, REVIVE_EINVAL, "revive_bind_workspace: null argument");
  if (bytes < ctx->ws.bytes) return fail(ctx, REVIVE_ENOMEM, "revive_bind_workspace: %zu bytes given, %zu needed", bytes, ctx->ws.bytes);
  if (reinterpret_cast<uintptr_t>(dev) % 256 != 0) return fail(ctx, REVIVE_EINVAL, "revive_bind_workspace: buffer must be 256-byte aligned");
  // the dispatch ticket must start at zero; every launch leaves it at zero again
  REVIVE_HIP(ctx, hipMemset(static_cast<uint8_t*>(dev) + ctx->ws.off_ticket, 0, sizeof(uint32_t)));
  ctx->d_ws = static_cast<uint8_t*>(dev);
  ctx->ws_bound = bytes;
  return REVIVE_OK;
}

int revive_set_placement(revive_ctx* ctx, const int32_t* phys_to_logical) {
  if (!ctx || !phys_to_logical) return fail(ctx, REVIVE_EINVAL, "revive_set_placement: null argument");
  const revive_config& c = ctx->cfg;
  std::vector<int32_t> full(c.E, 0);
  for (int p = 0; p < ctx->P; ++p) {
    const int32_t e = phys_to_logical[p];
    if (e < -1 || e >= c.E) return fail(ctx, REVIVE_EINVAL, "revive_set_placement: slot %d holds expert %d, outside [-1, %d)", p, e, c.E);
    if (e >= 0 && ++full[e] > c.max_replicas)
      return fail(ctx, REVIVE_EINVAL, "revive_set_placement: expert %d has more than max_replicas = %d copies", e, c.max_replicas);
  }
  ctx->phys_to_logical.assign(phys_to_logical, phys_to_logical + ctx->P);
  ctx->full_count = full;
  REVIVE_HIP(ctx, hipMemcpy(ctx->d_phys_to_logical, phys_to_logical, sizeof(int32_t) * ctx->P, hipMemcpyHostToDevice));
  ctx->placement_set = true;
  ctx->map_set = false;
  return REVIVE_OK;
}

int revive_update_map(revive_ctx* ctx, const uint8_t* rank_failed, revive_stream stream, revive_map_stats* stats) {
  return revive_update_map_experts(ctx, rank_failed, nullptr, stream, stats);
}

int revive_update_map_experts(revive_ctx* ctx, const uint8_t* rank_failed, const uint8_t* expert_failed, revive_stream stream,
                              revive_map_stats* stats) {
  if (!ctx || !rank_failed) return fail(ctx, REVIVE_EINVAL, "revive_update_map: null argument");
  if (!ctx->placement_set) return fail(ctx, REVIVE_ESTATE, "revive_update_map: call revive_set_placement first");
  const revive_config& c = ctx->cfg;

  // Build the new tables aside; nothing is committed until validation has passed.
  std::vector<uint8_t> blob(ctx->map.bytes, 0);
  revive_map_stats st{0, 0, 0, 0};
  int rc = build_tables(c, ctx->phys_to_logical.data(), rank_failed, expert_failed,
                        reinterpret_cast<int32_t*>(blob.data() + ctx->map.off_count),
                        reinterpret_cast<int32_t*>(blob.data() + ctx->map.off_table), blob.data() + ctx->map.off_alive, &st, &ctx->err);
  if (rc != REVIVE_OK) return rc;
  compacted_ranks(rank_failed, c.n_ranks, reinterpret_cast<int32_t*>(blob.data() + ctx->map.off_lrank),
                  reinterpret_cast<int32_t*>(blob.data() + ctx->map.off_nlive));

  const int b = ctx->stage_next;
  if (ctx->stage_used[b]) REVIVE_HIP(ctx, hipEventSynchronize(ctx->stage_done[b]));  // previous copy from this buffer
  std::memcpy(ctx->h_stage[b], blob.data(), blob.size());
  hipStream_t s = static_cast<hipStream_t>(stream);
  REVIVE_HIP(ctx, hipMemcpyAsync(ctx->d_map, ctx->h_stage[b], blob.size(), hipMemcpyHostToDevice, s));
  REVIVE_HIP(ctx, hipEventRecord(ctx->stage_done[b], s));
  ctx->stage_used[b] = true;
  ctx->stage_next = b ^ 1;
  ctx->host_blob.swap(blob);
  ctx->map_set = true;
  if (stats) *stats = st;
  return REVIVE_OK;
}

int revive_set_token_offset(revive_ctx* ctx, int64_t first_token) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_set_token_offset: null context");
  if (first_token < 0) return fail(ctx, REVIVE_EINVAL, "revive_set_token_offset: negative offset");
  ctx->token_offset = first_token;
  return REVIVE_OK;
}

int revive_get_map(const revive_ctx* ctx, int32_t* l2p_table, int32_t* l2p_count, uint8_t* slot_alive) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_get_map: null context");
  if (!ctx->map_set) return fail(ctx, REVIVE_ESTATE, "revive_get_map: no map has been built yet");
  const revive_config& c = ctx->cfg;
  if (l2p_count) std::memcpy(l2p_count, ctx->host_blob.data() + ctx->map.off_count, sizeof(int32_t) * c.E);
  if (l2p_table) std::memcpy(l2p_table, ctx->host_blob.data() + ctx->map.off_table, sizeof(int32_t) * c.E * c.max_replicas);
  if (slot_alive) std::memcpy(slot_alive, ctx->host_blob.data() + ctx->map.off_alive, ctx->P);
  return REVIVE_OK;
}

int revive_get_rank_map(const revive_ctx* ctx, int32_t* logical_rank, int32_t* n_live_ranks) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_get_rank_map: null context");
  if (!ctx->map_set) return fail(ctx, REVIVE_ESTATE, "revive_get_rank_map: no map has been built yet");
  if (logical_rank) std::memcpy(logical_rank, ctx->host_blob.data() + ctx->map.off_lrank, sizeof(int32_t) * ctx->cfg.n_ranks);
  if (n_live_ranks) std::memcpy(n_live_ranks, ctx->host_blob.data() + ctx->map.off_nlive, sizeof(int32_t));
  return REVIVE_OK;
}

// ---- data path entry points: argument checks, then the stage's launcher ----

static int check_call(revive_ctx* ctx, const char* who, int32_t T, bool need_ws) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "%s: null context", who);
  if (T < 0 || T > ctx->cfg.T_max) return fail(ctx, REVIVE_EINVAL, "%s: T = %d outside [0, T_max = %d]", who, T, ctx->cfg.T_max);
  if (need_ws && !ctx->d_ws) return fail(ctx, REVIVE_ESTATE, "%s: no workspace bound", who);
  return REVIVE_OK;
}

int revive_route(revive_ctx* ctx, const void* x, const void* w_router, float* logits, int32_t logits_given, int32_t T,
                 int32_t* topk_logical, float* topk_weight, int32_t* topk_phys, revive_stream stream) {
  int rc = check_call(ctx, "revive_route", T, false);
  if (rc != REVIVE_OK) return rc;
  if (!ctx->map_set) return fail(ctx, REVIVE_ESTATE, "revive_route: call revive_update_map first");
  if (!logits || !topk_logical || !topk_weight || !topk_phys) return fail(ctx, REVIVE_EINVAL, "revive_route: null output or logits");
  if (!logits_given && (!x || !w_router)) return fail(ctx, REVIVE_EINVAL, "revive_route: x and w_router are required unless logits are given");
  if (T == 0) return REVIVE_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!logits_given) {
    rc = launch_router_gemm(ctx, x, w_router, logits, T, s);
    if (rc != REVIVE_OK) return rc;
  }
  return launch_route_topk(ctx, logits, T, topk_logical, topk_weight, topk_phys, s);
}

int revive_dispatch(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int32_t T, void* x_perm,
                    int32_t* slot_offsets, int32_t* dst_row, int32_t* src_of, revive_stream stream) {
  int rc = check_call(ctx, "revive_dispatch", T, true);
  if (rc != REVIVE_OK) return rc;
  if (!slot_offsets) return fail(ctx, REVIVE_EINVAL, "revive_dispatch: null slot_offsets");
  if (T > 0 && (!x || !topk_phys || !x_perm || !dst_row || !src_of)) return fail(ctx, REVIVE_EINVAL, "revive_dispatch: null argument");
  return launch_dispatch(ctx, x, topk_phys, T, x_perm, slot_offsets, dst_row, src_of, static_cast<hipStream_t>(stream));
}

int revive_rank_offsets(revive_ctx* ctx, const int32_t* slot_offsets, int32_t* rank_offsets, revive_stream stream) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_rank_offsets: null context");
  if (!ctx->map_set) return fail(ctx, REVIVE_ESTATE, "revive_rank_offsets: call revive_update_map first");
  if (!slot_offsets || !rank_offsets) return fail(ctx, REVIVE_EINVAL, "revive_rank_offsets: null argument");
  return launch_rank_offsets(ctx, slot_offsets, rank_offsets, static_cast<hipStream_t>(stream));
}

int revive_dispatch_static(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int32_t T, void* x_perm,
                           int32_t* slot_offsets, int32_t* dst_row, int32_t* src_of, revive_stream stream) {
  int rc = check_call(ctx, "revive_dispatch_static", T, false);
  if (rc != REVIVE_OK) return rc;
  if (!slot_offsets) return fail(ctx, REVIVE_EINVAL, "revive_dispatch_static: null slot_offsets");
  if (T > 0 && (!x || !topk_phys || !x_perm || !dst_row || !src_of)) return fail(ctx, REVIVE_EINVAL, "revive_dispatch_static: null argument");
  return launch_dispatch_static(ctx, x, topk_phys, T, x_perm, slot_offsets, dst_row, src_of, static_cast<hipStream_t>(stream));
}

int revive_expert_ffn(revive_ctx* ctx, const void* x_perm, const int32_t* slot_offsets, const void* const* w_gate_up,
                      const void* const* w_down, void* y_perm, const void* x, const void* w_sh_gate_up,
                      const void* w_sh_down, void* y_shared, int32_t T, revive_stream stream) {
  int rc = check_call(ctx, "revive_expert_ffn", T, true);
  if (rc != REVIVE_OK) return rc;
  if (T == 0) return REVIVE_OK;
  if (!x_perm || !slot_offsets || !w_gate_up || !w_down || !y_perm) return fail(ctx, REVIVE_EINVAL, "revive_expert_ffn: null argument");
  if (y_shared) {
    if (ctx->cfg.I_shared == 0) return fail(ctx, REVIVE_EINVAL, "revive_expert_ffn: y_shared given but the layer has no shared expert");
    if (!x || !w_sh_gate_up || !w_sh_down) return fail(ctx, REVIVE_EINVAL, "revive_expert_ffn: shared expert needs x and both weight matrices");
  }
  return launch_expert_ffn(ctx, x_perm, slot_offsets, w_gate_up, w_down, y_perm, x, w_sh_gate_up, w_sh_down, y_shared, T,
                           static_cast<hipStream_t>(stream));
}

int revive_shared_ffn(revive_ctx* ctx, const void* x, const void* w_sh_gate_up, const void* w_sh_down, void* y_shared,
                      int32_t T, revive_stream stream) {
  int rc = check_call(ctx, "revive_shared_ffn", T, true);
  if (rc != REVIVE_OK) return rc;
  if (ctx->cfg.I_shared == 0) return fail(ctx, REVIVE_EINVAL, "revive_shared_ffn: the layer has no shared expert");
  if (T == 0) return REVIVE_OK;
  if (!x || !w_sh_gate_up || !w_sh_down || !y_shared) return fail(ctx, REVIVE_EINVAL, "revive_shared_ffn: null argument");
  return launch_shared_ffn(ctx, x, w_sh_gate_up, w_sh_down, y_shared, T, static_cast<hipStream_t>(stream));
}

int revive_expert_counts(revive_ctx* ctx, const int32_t* topk_logical, int32_t T, int64_t* counts, revive_stream stream) {
  int rc = check_call(ctx, "revive_expert_counts", T, false);
  if (rc != REVIVE_OK) return rc;
  if (!counts) return fail(ctx, REVIVE_EINVAL, "revive_expert_counts: null counts");
  if (T == 0) return REVIVE_OK;
  if (!topk_logical) return fail(ctx, REVIVE_EINVAL, "revive_expert_counts: null argument");
  return launch_expert_counts(ctx, topk_logical, T, counts, static_cast<hipStream_t>(stream));
}

int revive_combine(revive_ctx* ctx, const void* y_perm, const int32_t* dst_row, const float* topk_weight,
                   const void* y_shared, int32_t T, void* out, revive_stream stream) {
  int rc = check_call(ctx, "revive_combine", T, false);
  if (rc != REVIVE_OK) return rc;
  if (T == 0) return REVIVE_OK;
  if (!y_perm || !dst_row || !topk_weight || !out) return fail(ctx, REVIVE_EINVAL, "revive_combine: null argument");
  return launch_combine(ctx, y_perm, dst_row, topk_weight, y_shared, T, out, static_cast<hipStream_t>(stream));
}

// ---- graph replay ----

}  // extern "C"

struct revive_graph {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

extern "C" {

int revive_graph_begin(revive_ctx* ctx, revive_stream stream) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_graph_begin: null context");
  if (!stream) return fail(ctx, REVIVE_EINVAL, "revive_graph_begin: the default stream cannot be captured");
  REVIVE_HIP(ctx, hipStreamBeginCapture(static_cast<hipStream_t>(stream), hipStreamCaptureModeRelaxed));
  return REVIVE_OK;
}

int revive_graph_end(revive_ctx* ctx, revive_stream stream, revive_graph** out) {
  if (out) *out = nullptr;
  if (!ctx || !out) return fail(ctx, REVIVE_EINVAL, "revive_graph_end: null argument");
  hipGraph_t graph = nullptr;
  REVIVE_HIP(ctx, hipStreamEndCapture(static_cast<hipStream_t>(stream), &graph));
  hipGraphExec_t exec = nullptr;
  int rc = check_hip(ctx, hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0), "hipGraphInstantiate");
  if (rc != REVIVE_OK) {
    (void)hipGraphDestroy(graph);
    return rc;
  }
  revive_graph* g = new (std::nothrow) revive_graph();
  if (!g) {
    (void)hipGraphExecDestroy(exec);
    (void)hipGraphDestroy(graph);
    return fail(ctx, REVIVE_ENOMEM, "revive_graph_end: out of host memory");
  }
  g->graph = graph;
  g->exec = exec;
  *out = g;
  return REVIVE_OK;
}

int revive_graph_launch(revive_graph* g, revive_stream stream) {
  if (!g) return fail(nullptr, REVIVE_EINVAL, "revive_graph_launch: null graph");
  return check_hip(nullptr, hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)), "hipGraphLaunch");
}

uintptr_t revive_graph_exec_id(const revive_graph* g) { return g ? reinterpret_cast<uintptr_t>(g->exec) : 0; }

int revive_graph_destroy(revive_graph* g) {
  if (!g) return REVIVE_OK;
  (void)hipGraphExecDestroy(g->exec);
  (void)hipGraphDestroy(g->graph);
  delete g;
  return REVIVE_OK;
}

// ---- timing ----

int revive_set_kernel_timing(revive_ctx* ctx, int32_t enabled) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_set_kernel_timing: null context");
  if (enabled && ctx->slots.empty()) {
    ctx->slots.resize(kTimingPairs);
    for (auto& s : ctx->slots) {
      REVIVE_HIP(ctx, hipEventCreate(&s.start));
      REVIVE_HIP(ctx, hipEventCreate(&s.stop));
    }
  }
  if (!enabled && ctx->timing) {
    int rc = fold_timing(ctx);
    if (rc != REVIVE_OK) return rc;
  }
  ctx->timing = enabled != 0;
  return REVIVE_OK;
}

int revive_kernel_time(revive_ctx* ctx, int32_t kernel, double* total_ms, int64_t* launches) {
  if (!ctx || kernel < 0 || kernel >= REVIVE_K_COUNT) return fail(ctx, REVIVE_EINVAL, "revive_kernel_time: bad argument");
  int rc = fold_timing(ctx);
  if (rc != REVIVE_OK) return rc;
  if (total_ms) *total_ms = ctx->time_ms[kernel];
  if (launches) *launches = ctx->time_n[kernel];
  return REVIVE_OK;
}

int revive_reset_kernel_times(revive_ctx* ctx) {
  if (!ctx) return fail(ctx, REVIVE_EINVAL, "revive_reset_kernel_times: null context");
  int rc = fold_timing(ctx);
  for (int i = 0; i < REVIVE_K_COUNT; ++i) {
    ctx->time_ms[i] = 0;
    ctx->time_n[i] = 0;
  }
  return rc;
}

const char* revive_kernel_name(int32_t kernel) {
  static const char* names[REVIVE_K_COUNT] = {
      "router_gemm", "route_topk", "dispatch_index", "dispatch_permute",
      "ffn_tiles", "ffn_gate_up", "ffn_down", "ffn_shared_gate_up", "ffn_shared_down", "combine", "expert_counts"};
  return kernel >= 0 && kernel < REVIVE_K_COUNT ? names[kernel] : "?";
}

const char* revive_last_error(const revive_ctx* ctx) { return ctx ? ctx->err.c_str() : noctx_error().c_str(); }

}  // extern "C"
