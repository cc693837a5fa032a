// Host-only half of the library (see map_host.hpp): no GPU call, no HIP header.
#include "map_host.hpp"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <vector>

namespace revive {

int host_fail(std::string* err, int status, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  if (err) *err = buf;
  return status;
}

std::string& noctx_error() {
  static thread_local std::string text;
  return text;
}

// Ungrouped: at least k live experts.  Grouped: a group without live experts is kept only when
// fewer than topk_group groups have one, so the worst kept set is the topk_group live groups
// with the fewest live experts (or every live group when there are fewer than that).
bool enough_live(const revive_config& c, const int32_t* count) {
  if (c.n_group <= 1) {
    int live = 0;
    for (int e = 0; e < c.E; ++e) live += count[e] > 0;
    return live >= c.k;
  }
  const int gsz = c.E / c.n_group;
  std::vector<int> per;
  for (int g = 0; g < c.n_group; ++g) {
    int live = 0;
    for (int e = g * gsz; e < (g + 1) * gsz; ++e) live += count[e] > 0;
    if (live > 0) per.push_back(live);
  }
  std::sort(per.begin(), per.end());
  int reach = 0;
  for (size_t i = 0; i < per.size() && i < static_cast<size_t>(c.topk_group); ++i) reach += per[i];
  return reach >= c.k;
}

int build_tables(const revive_config& c, const int32_t* p2l, const uint8_t* rank_failed, const uint8_t* expert_failed,
                 int32_t* count, int32_t* table, uint8_t* alive, revive_map_stats* stats, std::string* err) {
  const int P = c.n_ranks * c.slots_per_rank;
  for (int r = 0; r < c.n_ranks; ++r)
    if (rank_failed[r] > 1) return host_fail(err, REVIVE_EINVAL, "rank_failed[%d] = %d is not 0 or 1", r, rank_failed[r]);
  if (expert_failed)
    for (int e = 0; e < c.E; ++e)
      if (expert_failed[e] > 1) return host_fail(err, REVIVE_EINVAL, "expert_failed[%d] = %d is not 0 or 1", e, expert_failed[e]);
  std::vector<int32_t> full(c.E, 0);
  std::fill(count, count + c.E, 0);
  std::fill(alive, alive + P, 0);
  std::fill(table, table + static_cast<size_t>(c.E) * c.max_replicas, -1);
  revive_map_stats st{0, 0, 0, 0};
  for (int p = 0; p < P; ++p) {  // ascending p => each expert's list is ascending
    const int32_t e = p2l[p];
    if (e < -1 || e >= c.E) return host_fail(err, REVIVE_EINVAL, "slot %d holds expert %d, outside [-1, %d)", p, e, c.E);
    if (e < 0) continue;
    if (++full[e] > c.max_replicas) return host_fail(err, REVIVE_EINVAL, "expert %d has more than max_replicas = %d copies", e, c.max_replicas);
    if (rank_failed[p / c.slots_per_rank]) continue;
    if (expert_failed && expert_failed[e]) continue;
    alive[p] = 1;
    table[static_cast<size_t>(e) * c.max_replicas + count[e]++] = p;
    ++st.n_live_slots;
  }
  for (int e = 0; e < c.E; ++e) {
    if (count[e] == 0) ++st.n_lost_experts;
    else {
      ++st.n_live_experts;
      if (count[e] < full[e]) ++st.n_degraded_experts;
    }
  }
  if (stats) *stats = st;
  if (!enough_live(c, count))
    return host_fail(err, REVIVE_EINSUFFICIENT_EXPERTS, "only %d live experts; a token could not be given k = %d of them",
                st.n_live_experts, c.k);
  return REVIVE_OK;
}

// Logical ranks after every failed rank has left the communication domain (Sec. 3.5): a failed
// rank holds no logical rank (-1) and every rank behind it moves down by one for each failed rank
// in front of it, the relative order of the survivors kept.  Removing the failed ranks one at a
// time with revive_compact_ranks gives the same table in whatever order they are taken.
void compacted_ranks(const uint8_t* rank_failed, int R, int32_t* logical_rank, int32_t* n_live) {
  int next = 0;
  for (int r = 0; r < R; ++r) logical_rank[r] = rank_failed[r] ? -1 : next++;
  *n_live = next;
}

int check_config(const revive_config& c, std::string* err) {
  const int64_t P = static_cast<int64_t>(c.n_ranks) * c.slots_per_rank;
  if (c.T_max < 0 || c.H <= 0 || c.E <= 0 || c.k <= 0 || c.I <= 0 || c.I_shared < 0 || c.n_ranks <= 0 ||
      c.slots_per_rank <= 0 || c.max_replicas <= 0)
    return host_fail(err, REVIVE_EINVAL, "config: sizes must be positive");
  if (c.E > kMaxE || P > kMaxP || c.k > kMaxK || c.k > c.E)
    return host_fail(err, REVIVE_EINVAL, "config: E <= %d, P <= %d, k <= min(%d, E) required", kMaxE, kMaxP, kMaxK);
  if (c.dtype != REVIVE_DTYPE_F32 && c.dtype != REVIVE_DTYPE_BF16)
    return host_fail(err, REVIVE_EINVAL, "config: dtype must be 0 (fp32) or 1 (bf16)");
  if (c.score_fn != REVIVE_SCORE_SOFTMAX && c.score_fn != REVIVE_SCORE_SIGMOID)
    return host_fail(err, REVIVE_EINVAL, "config: unknown score_fn");
  if (c.n_group < 1 || c.topk_group < 1 || c.topk_group > c.n_group || c.E % c.n_group != 0 || c.n_group > 32)
    return host_fail(err, REVIVE_EINVAL, "config: need 1 <= topk_group <= n_group <= 32 and n_group | E");
  if (c.H % 8 != 0) return host_fail(err, REVIVE_EINVAL, "config: H must be a multiple of 8");
  if (c.dtype == REVIVE_DTYPE_BF16 && (c.H % 64 != 0 || c.I % 64 != 0 || c.I_shared % 64 != 0))
    return host_fail(err, REVIVE_EINVAL, "config: bf16 needs H, I and I_shared multiples of 64");
  if (c.dtype == REVIVE_DTYPE_BF16) {
    // the GEMM addresses a weight matrix and one row-tile of activations with 32-bit byte offsets
    const int64_t widest = std::max<int64_t>(c.I, c.I_shared);
    const int64_t pad = 128;
    const int64_t gate_up_bytes = 2 * ((widest + pad - 1) / pad * pad) * c.H * 2;
    const int64_t down_bytes = ((static_cast<int64_t>(c.H) + pad - 1) / pad * pad) * widest * 2;
    const int64_t tile_bytes = 256 * std::max<int64_t>(c.H, widest) * 2;
    if (gate_up_bytes >= (1ll << 31) || down_bytes >= (1ll << 31) || tile_bytes >= (1ll << 31))
      return host_fail(err, REVIVE_EINVAL, "config: H * I too large for one expert matrix (2 GiB limit)");
  }
  if (c.dtype == REVIVE_DTYPE_F32 && (c.I % 4 != 0 || c.I_shared % 4 != 0))
    return host_fail(err, REVIVE_EINVAL, "config: fp32 needs I and I_shared multiples of 4");
  if (static_cast<int64_t>(c.T_max) * c.k >= (1ll << 30)) return host_fail(err, REVIVE_EINVAL, "config: T_max * k too large");
  // a row-tile record keeps the number of row-tiles of its slot and its own position in 16 bits each
  const int tile_m = c.dtype == REVIVE_DTYPE_BF16 ? kTileM_bf16 : kTileM_f32;
  if ((static_cast<int64_t>(c.T_max) * c.k + tile_m - 1) / tile_m >= kMaxTilesPerSlot)
    return host_fail(err, REVIVE_EINVAL, "config: T_max * k = %lld routed rows could put %d or more row-tiles of %d rows into one slot",
                static_cast<long long>(c.T_max) * c.k, kMaxTilesPerSlot, tile_m);
  return REVIVE_OK;
}

}  // namespace revive

using namespace revive;

extern "C" {

int revive_compact_ranks(int32_t* logical_rank, int32_t n, int32_t failed_device, int32_t switched_device) {
  if (!logical_rank || n <= 0 || failed_device < 0 || failed_device >= n || switched_device >= n || switched_device == failed_device)
    return host_fail(&noctx_error(), REVIVE_EINVAL, "revive_compact_ranks: bad argument");
  int gap = logical_rank[failed_device];
  if (gap < 0) return host_fail(&noctx_error(), REVIVE_EINVAL, "revive_compact_ranks: device %d holds no rank", failed_device);
  logical_rank[failed_device] = -1;
  if (switched_device >= 0) {  // the switched device moves into the hole and leaves its own behind
    const int old = logical_rank[switched_device];
    logical_rank[switched_device] = gap;
    gap = old;
  }
  if (gap >= 0)
    for (int d = 0; d < n; ++d)
      if (logical_rank[d] > gap) --logical_rank[d];
  return REVIVE_OK;
}

int revive_mask_every_nth(int32_t E, int32_t n, uint8_t* mask) {
  if (E <= 0 || n <= 0 || !mask) return host_fail(&noctx_error(), REVIVE_EINVAL, "revive_mask_every_nth: bad argument");
  for (int e = 0; e < E; ++e) mask[e] = e % n == 0;
  return REVIVE_OK;
}

int revive_mask_most_activated(const int64_t* counts, int32_t E, int32_t n_fail, uint8_t* mask) {
  if (!counts || !mask || E <= 0 || n_fail < 0 || n_fail > E) return host_fail(&noctx_error(), REVIVE_EINVAL, "revive_mask_most_activated: bad argument");
  std::vector<int> order(E);
  for (int e = 0; e < E; ++e) order[e] = e;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return counts[a] > counts[b]; });  // stable: ties by id
  std::fill(mask, mask + E, 0);
  for (int i = 0; i < n_fail; ++i) mask[order[i]] = 1;
  return REVIVE_OK;
}

int revive_build_map_experts(const revive_config* cfg, const int32_t* phys_to_logical, const uint8_t* rank_failed,
                             const uint8_t* expert_failed, int32_t* l2p_table, int32_t* l2p_count, uint8_t* slot_alive,
                             revive_map_stats* stats) {
  if (!cfg || !phys_to_logical || !rank_failed || !l2p_table || !l2p_count || !slot_alive)
    return host_fail(&noctx_error(), REVIVE_EINVAL, "revive_build_map: null argument");
  int rc = check_config(*cfg, &noctx_error());
  if (rc != REVIVE_OK) return rc;
  return build_tables(*cfg, phys_to_logical, rank_failed, expert_failed, l2p_count, l2p_table, slot_alive, stats, &noctx_error());
}

int revive_build_map(const revive_config* cfg, const int32_t* phys_to_logical, const uint8_t* rank_failed,
                     int32_t* l2p_table, int32_t* l2p_count, uint8_t* slot_alive, revive_map_stats* stats) {
  return revive_build_map_experts(cfg, phys_to_logical, rank_failed, nullptr, l2p_table, l2p_count, slot_alive, stats);
}

const char* revive_status_name(int status) {
  switch (status) {
    case REVIVE_OK: return "REVIVE_OK";
    case REVIVE_EINVAL: return "REVIVE_EINVAL";
    case REVIVE_ENOMEM: return "REVIVE_ENOMEM";
    case REVIVE_ESTATE: return "REVIVE_ESTATE";
    case REVIVE_EINSUFFICIENT_EXPERTS: return "REVIVE_EINSUFFICIENT_EXPERTS";
    case REVIVE_EHIP: return "REVIVE_EHIP";
    default: return "REVIVE_?";
  }
}

}  // extern "C"
