// Internal layout of the plan object shared by the host planner and the launch code.
#pragma once

#include <cstdint>
#include <vector>

#include "elaswave.h"

namespace ew {

// One unit of copy work for a workgroup: at most tile_elems elements of one segment.
// src_buf indexes the source pointer table (kSrcLive + old rank, kSrcSnap + owner, kSrcStage),
// dst_buf the destination table (new rank, or kDstStage).  32 bytes so that one record is a
// single aligned scalar load.
struct Tile {
  uint64_t src_off;  // elements
  uint64_t dst_off;  // elements
  uint32_t len;      // elements, 1..tile_elems
  uint16_t src_buf;
  uint16_t dst_buf;
  uint64_t pad;
};
static_assert(sizeof(Tile) == 32, "tile record must stay 32 bytes");

constexpr uint32_t kSrcLive = 0;
constexpr uint32_t kSrcSnap = EW_MAX_DP;
constexpr uint32_t kSrcStage = 2 * EW_MAX_DP;
constexpr uint32_t kNumSrc = 2 * EW_MAX_DP + 1;
constexpr uint32_t kDstStage = EW_MAX_DP;
constexpr uint32_t kNumDst = EW_MAX_DP + 1;

struct DeviceTiles {
  Tile *host = nullptr;  // pinned staging copy, kept until the plan is freed
  Tile *dev = nullptr;
  uint64_t count = 0;
};

}  // namespace ew

struct ew_plan_s {
  uint32_t old_dp = 0, new_dp = 0;
  uint64_t alive_mask = 0;
  uint64_t numel = 0;
  std::vector<uint64_t> old_len, new_len;      // shard lengths in elements
  std::vector<int32_t> new_rank_of, holder_of; // per old rank
  std::vector<ew_seg_t> segs;
  std::vector<uint64_t> pair_len, pair_off;    // [holder * new_dp + dst_rank]
  uint64_t stage_len = 0;
  uint64_t live_read = 0, snap_read = 0;       // bit j: some segment reads that buffer
  // device side (filled by ew_plan_upload)
  int device = -1;
  uint32_t tile_elems = 0;
  ew::DeviceTiles pack, unpack;
};

namespace ew {
// Cuts the plan's segments into tiles.  which = 0: non-LOCAL segments, source -> arena.
// which = 1: every segment, arena or local source -> new shard.
void build_tiles(const ew_plan_t &plan, int which, uint32_t tile_elems, std::vector<Tile> &out);
uint64_t count_tiles(const ew_plan_t &plan, int which, uint32_t tile_elems);
}  // namespace ew
