// Test driver for the library's host-only code (csrc/map_host.cpp), built by
// tests/test_host_sanitized_cpu.py with AddressSanitizer and UBSan.  Reads whitespace-separated
// cases from stdin and prints the results; holds no logic of its own.
//
//   map   E k n_group topk_group R S max_replicas  p2l[P]  rank_failed[R]  has_ef [ef[E]]
//           -> rc  live_slots live_experts lost degraded  count[E]  table[E*max_replicas]  alive[P]  lrank[R] n_live
//   ranks n failed switched  logical_rank[n]        -> rc  logical_rank[n]
//   nth   E n                                       -> rc  mask[E]
//   top   E n_fail counts[E]                        -> rc  mask[E]
#include <cstdint>
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "map_host.hpp"

int main() {
  std::string op;
  while (std::cin >> op) {
    if (op == "map") {
      revive_config c{};
      int has_ef = 0;
      std::cin >> c.E >> c.k >> c.n_group >> c.topk_group >> c.n_ranks >> c.slots_per_rank >> c.max_replicas;
      c.T_max = 16; c.H = 64; c.I = 64; c.I_shared = 0; c.score_fn = REVIVE_SCORE_SIGMOID; c.dtype = REVIVE_DTYPE_F32; c.route_scale = 1.f;
      const int P = c.n_ranks * c.slots_per_rank;
      std::vector<int32_t> p2l(P);
      for (auto& v : p2l) std::cin >> v;
      std::vector<uint8_t> rf(c.n_ranks), ef;
      for (auto& v : rf) { int t; std::cin >> t; v = static_cast<uint8_t>(t); }
      std::cin >> has_ef;
      if (has_ef) { ef.resize(c.E); for (auto& v : ef) { int t; std::cin >> t; v = static_cast<uint8_t>(t); } }
      // exactly-sized heap buffers: any write past the documented sizes is an AddressSanitizer report
      std::vector<int32_t> count(c.E, 77), table(static_cast<size_t>(c.E) * c.max_replicas, 77), lrank(c.n_ranks, 77);
      std::vector<uint8_t> alive(P, 77);
      revive_map_stats st{-1, -1, -1, -1};
      const int rc = revive_build_map_experts(&c, p2l.data(), rf.data(), has_ef ? ef.data() : nullptr, table.data(), count.data(),
                                              alive.data(), &st);
      int32_t n_live = -1;
      revive::compacted_ranks(rf.data(), c.n_ranks, lrank.data(), &n_live);
      std::printf("%d %d %d %d %d", rc, st.n_live_slots, st.n_live_experts, st.n_lost_experts, st.n_degraded_experts);
      for (int v : count) std::printf(" %d", v);
      for (int v : table) std::printf(" %d", v);
      for (int v : alive) std::printf(" %d", v);
      for (int v : lrank) std::printf(" %d", v);
      std::printf(" %d\n", n_live);
    } else if (op == "ranks") {
      int n, f, sw;
      std::cin >> n >> f >> sw;
      std::vector<int32_t> r(n);
      for (auto& v : r) std::cin >> v;
      const int rc = revive_compact_ranks(r.data(), n, f, sw);
      std::printf("%d", rc);
      for (int v : r) std::printf(" %d", v);
      std::printf("\n");
    } else if (op == "nth") {
      int E, n;
      std::cin >> E >> n;
      std::vector<uint8_t> m(E > 0 ? E : 1, 77);
      const int rc = revive_mask_every_nth(E, n, m.data());
      std::printf("%d", rc);
      for (int e = 0; e < E; ++e) std::printf(" %d", m[e]);
      std::printf("\n");
    } else if (op == "top") {
      int E, n_fail;
      std::cin >> E >> n_fail;
      std::vector<int64_t> cnt(E);
      for (auto& v : cnt) std::cin >> v;
      std::vector<uint8_t> m(E, 77);
      const int rc = revive_mask_most_activated(cnt.data(), E, n_fail, m.data());
      std::printf("%d", rc);
      for (int v : m) std::printf(" %d", v);
      std::printf("\n");
    } else {
      std::fprintf(stderr, "unknown op %s\n", op.c_str());
      return 2;
    }
  }
  return 0;
}
