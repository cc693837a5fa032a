// Internal context of the failure-remapped MoE layer library (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "map_host.hpp"
#include "revive.h"

namespace revive {

constexpr int kDispatchChunk = 1024;  // routed rows handled by one block of the count/place kernels
constexpr int kStaticDispatchChunks = 64;  // chunks the statically allocated dispatch scratch holds (65536 routed rows)
constexpr int kTimingPairs = 8192;    // event pairs kept before timing results are folded


// One row-tile of a grouped GEMM.  All row-tiles of a group (physical slot) carry the same
// record except for their position; tile_span() gives the rows of tile j.  The group's weight
// matrices ride along so that a workgroup needs one read to know everything about its tile.
struct MTile {
  int32_t group;
  int32_t group_begin;
  int32_t group_end;
  int32_t pad;          // (row-tiles of the group << 16) | position of this tile inside its group
  const void* w[2];     // the group's gate/up and down matrices (null when the caller uses a table)
};

// Rows [row_begin, row_end) of tile j of a group with rows [begin, end) cut into G = ceil(rows / tile_m)
// tiles.  Tiles are tile_m rows high except the last two, which share their rows about evenly (the
// first of them rounded up to 64 rows): a slot that overflows a tile by a few rows would otherwise
// get a second tile that streams the whole weight matrix for almost no work, ahead of and out of
// step with its neighbour, so that the weights come from HBM twice.  The split costs no extra
// MFMA time: the 32-row sub-tiles are dealt to two wavefront rows, and ceil(a/2) + ceil(b/2) over
// the two tiles is the same for both ways of cutting.
__host__ __device__ inline void tile_span(int begin, int end, int G, int j, int tile_m, int& row_begin, int& row_end) {
  if (G >= 2 && j >= G - 2) {
    const int base = begin + (G - 2) * tile_m;
    const int both = end - base;  // tile_m + rows of the last tile
    int a = ((both + 1) / 2 + 63) & ~63;
    if (a > tile_m) a = tile_m;
    row_begin = j == G - 2 ? base : base + a;
    row_end = j == G - 2 ? base + a : end;
  } else {
    row_begin = begin + j * tile_m;
    row_end = row_begin + tile_m < end ? row_begin + tile_m : end;
  }
}

// Device-resident map, one contiguous blob at a fixed address so that one copy updates it.
struct MapLayout {
  size_t off_count;   // int32 [E]
  size_t off_table;   // int32 [E * max_replicas]
  size_t off_alive;   // uint8 [P] (padded to 4)
  size_t off_lrank;   // int32 [R]: compacted logical rank of each simulated rank, -1 = failed
  size_t off_nlive;   // int32 [4]: [0] = number of live ranks
  size_t bytes;
};

struct Workspace {
  size_t off_block_hist;  // int32 [n_chunks_max * P]
  size_t off_ticket;      // uint32 [1] (+ padding): finished-workgroup counter of the dispatch index kernel, zero between launches
  size_t off_tiles;       // MTile [max_tiles_routed]
  size_t off_tile_count;  // int32 [4]
  size_t off_h;           // dtype [N_max * I]
  size_t off_h_shared;    // dtype [T_max * I_shared]
  size_t bytes;
};

struct TimingSlot {
  hipEvent_t start, stop;
  int kernel;
};

}  // namespace revive

struct revive_ctx {
  revive_config cfg;
  int device = 0;
  int P = 0;
  size_t elem = 2;  // bytes per element of dtype

  // host side of the map
  std::vector<int32_t> phys_to_logical;
  std::vector<int32_t> full_count;  // replicas per expert in the placement
  std::vector<uint8_t> host_blob;   // current tables, MapLayout order
  int64_t token_offset = 0;  // index of row 0 of x within the whole batch (replica rule of a microbatch)
  bool placement_set = false;
  bool map_set = false;

  // device side of the map (fixed addresses)
  revive::MapLayout map{};
  uint8_t* d_map = nullptr;
  int32_t* d_phys_to_logical = nullptr;
  // pinned staging, two buffers used alternately
  uint8_t* h_stage[2] = {nullptr, nullptr};
  hipEvent_t stage_done[2] = {nullptr, nullptr};
  bool stage_used[2] = {false, false};
  int stage_next = 0;

  // caller-owned scratch
  revive::Workspace ws{};
  uint8_t* d_ws = nullptr;
  size_t ws_bound = 0;

  // timing
  bool timing = false;
  std::vector<revive::TimingSlot> slots;
  size_t slots_used = 0;
  double time_ms[REVIVE_K_COUNT] = {0};
  int64_t time_n[REVIVE_K_COUNT] = {0};

  mutable std::string err;

  const int32_t* d_l2p_count() const { return reinterpret_cast<const int32_t*>(d_map + map.off_count); }
  const int32_t* d_l2p_table() const { return reinterpret_cast<const int32_t*>(d_map + map.off_table); }
  const uint8_t* d_slot_alive() const { return d_map + map.off_alive; }
  const int32_t* d_logical_rank() const { return reinterpret_cast<const int32_t*>(d_map + map.off_lrank); }
  const int32_t* d_n_live_ranks() const { return reinterpret_cast<const int32_t*>(d_map + map.off_nlive); }
};

namespace revive {

int fail(const revive_ctx* ctx, int status, const char* fmt, ...);
int check_hip(const revive_ctx* ctx, hipError_t e, const char* what);

// Brackets one kernel launch with timing events when timing is on and the stream is not capturing.
struct KernelTimer {
  revive_ctx* ctx;
  hipStream_t stream;
  TimingSlot* slot = nullptr;
  KernelTimer(revive_ctx* c, int kernel, hipStream_t s);
  ~KernelTimer();
};
int fold_timing(revive_ctx* ctx);

// Raises a kernel's dynamic-LDS limit to `lds` bytes on the current device.  Done once per kernel
// and device; safe to call from several host threads.
hipError_t allow_dynamic_lds(const void* kernel, size_t lds);

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Upper bound on row-tiles of a grouped GEMM over N rows in at most `groups` non-empty groups.
inline int max_tiles(int64_t n_rows, int groups, int tile_m) {
  return static_cast<int>(n_rows / tile_m) + groups;
}

// Data-path stages, one translation unit each.
int launch_router_gemm(revive_ctx*, const void* x, const void* w, float* logits, int T, hipStream_t);
int launch_route_topk(revive_ctx*, const float* logits, int T, int32_t* topk_logical, float* topk_weight,
                      int32_t* topk_phys, hipStream_t);
int launch_dispatch(revive_ctx*, const void* x, const int32_t* topk_phys, int T, void* x_perm,
                    int32_t* slot_offsets, int32_t* dst_row, int32_t* src_of, hipStream_t);
int init_static_dispatch_scratch(revive_ctx*);  // looks up this device's copy of the static scratch, once per device
int launch_dispatch_static(revive_ctx*, const void* x, const int32_t* topk_phys, int T, void* x_perm,
                           int32_t* slot_offsets, int32_t* dst_row, int32_t* src_of, hipStream_t);
int launch_rank_offsets(revive_ctx*, const int32_t* slot_offsets, int32_t* rank_offsets, hipStream_t);
int launch_expert_ffn(revive_ctx*, const void* x_perm, const int32_t* slot_offsets, const void* const* w_gate_up,
                      const void* const* w_down, void* y_perm, const void* x, const void* w_sh_gate_up,
                      const void* w_sh_down, void* y_shared, int T, hipStream_t);
int launch_shared_ffn(revive_ctx*, const void* x, const void* w_sh_gate_up, const void* w_sh_down, void* y_shared, int T,
                      hipStream_t);
int launch_expert_counts(revive_ctx*, const int32_t* topk_logical, int T, int64_t* counts, hipStream_t);
int launch_combine(revive_ctx*, const void* y_perm, const int32_t* dst_row, const float* topk_weight,
                   const void* y_shared, int T, void* out, hipStream_t);

}  // namespace revive

#define REVIVE_HIP(ctx, call)                                           \
  do {                                                                  \
    int _rc = revive::check_hip((ctx), (call), #call);                  \
    if (_rc != REVIVE_OK) return _rc;                                   \
  } while (0)
