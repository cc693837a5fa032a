// Host-only half of the library: limits, configuration checks, the map construction of the recovery
// step, rank compaction and the masks of the lost-expert study.  Nothing here touches the GPU or
// includes a HIP header, so this translation unit also builds with a plain C++ compiler (the CPU
// tests build it with AddressSanitizer and UBSan).
#pragma once

#include <cstdint>
#include <string>

#include "revive.h"

namespace revive {

constexpr int kMaxE = 512;
constexpr int kMaxP = 1024;
constexpr int kMaxK = 32;
// Tile heights of the grouped GEMMs (rows of one slot handled by one workgroup).
constexpr int kTileM_bf16 = 256;
constexpr int kTileM_f32 = 64;
constexpr int kMaxTilesPerSlot = 1 << 15;  // a row-tile record holds count and position in 16 bits each

// Formats an error text into *err (may be null) and returns `status`.
int host_fail(std::string* err, int status, const char* fmt, ...);

// Text of the last failure of a call that had no context (thread-local).
std::string& noctx_error();

int check_config(const revive_config& c, std::string* err);

// Worst case over all possible logits: can a token always be given k live experts?
bool enough_live(const revive_config& c, const int32_t* count);

// Host construction of the map tables from the static placement and the failure bytes.
// Writes count[E], table[E * max_replicas] (-1 padded) and alive[P].  stats (may be null) is
// filled even when REVIVE_EINSUFFICIENT_EXPERTS is returned.
int build_tables(const revive_config& c, const int32_t* p2l, const uint8_t* rank_failed, const uint8_t* expert_failed,
                 int32_t* count, int32_t* table, uint8_t* alive, revive_map_stats* stats, std::string* err);

// Logical ranks after every failed rank has left the communication domain (Sec. 3.5).
void compacted_ranks(const uint8_t* rank_failed, int R, int32_t* logical_rank, int32_t* n_live);

}  // namespace revive
