// Internal layout of the plan object shared by the host planner and the launch code.
//
// The plan is kept in run-length form: consecutive units (the paper's layers) of equal length
// split identically, so a run of n such units is stored as ONE unit's segments plus, for each
// segment, the distance its source / destination / arena offsets advance from one unit to the
// next.  A uniform interleave chunk gives two runs (the full units and the short last one)
// whatever the state size, so planning and the table upload cost microseconds, not a pass over
// 10^5 segments.  The explicit segment table of the C ABI is expanded from it on demand.
#pragma once

#include <cstdint>
#include <mutex>
#include <vector>

#include "elaswave.h"

namespace ew {

// A segment of the first unit of a run, with per-unit strides (all in elements).
struct RunSeg {
  uint64_t src_off, dst_off, stage_off, len;
  uint64_t src_stride, dst_stride, stage_stride;
  uint16_t src_owner, holder, dst_rank, flags;
};

struct Run {
  uint64_t n_units;   // consecutive units of this length
  uint64_t unit_len;  // elements
  uint32_t seg_begin, seg_end;  // range in ew_plan_s::run_segs
};

// ---- device tables ------------------------------------------------------------------------
// One unit of copy work for a workgroup: at most tile_elems elements of one segment of one
// unit.  A tile template belongs to a record (RunT); for repetition i of the record the offsets
// are off0 + i * stride.  src_buf indexes the source pointer table (kSrcLive + old rank,
// kSrcSnap + owner, kSrcStage), dst_buf the destination table (new rank, or kDstStage).
struct TileT {
  uint64_t src_off, dst_off;        // elements, unit 0 of the run
  uint64_t src_stride, dst_stride;  // elements per unit
  uint32_t len;                     // elements, 1..tile_elems
  uint16_t src_buf, dst_buf;
  uint64_t pad;
};
static_assert(sizeof(TileT) == 48, "tile template must stay 48 bytes");

// One record per (destination, run of equal units): the tiles that destination receives from the
// run, unit after unit.  Records are ordered destination-major (see build_tile_table).
struct RunT {
  uint64_t tile_begin;      // global id of the record's first tile
  uint64_t tile_end;        // one past its last tile (= the next record's tile_begin)
  uint32_t tiles_per_unit;  // templates per repetition (> 0)
  uint32_t templ_begin;     // index of the record's first template
  uint32_t div_magic;       // n / tiles_per_unit for 32-bit n without a division: see div_by_invariant
  uint8_t div_sh1, div_sh2;
  uint16_t pad;
};
static_assert(sizeof(RunT) == 32, "run record must stay 32 bytes (one aligned scalar load)");

constexpr uint32_t kSrcLive = 0;
constexpr uint32_t kSrcSnap = EW_MAX_DP;
constexpr uint32_t kSrcStage = 2 * EW_MAX_DP;
constexpr uint32_t kNumSrc = 2 * EW_MAX_DP + 1;
constexpr uint32_t kDstStage = EW_MAX_DP;
constexpr uint32_t kNumDst = EW_MAX_DP + 1;
constexpr int kNumTables = 3;  // pack, unpack, direct

// Tile id -> (buffers, offsets, length).  The one decoder, used by the copy kernel (where every
// operand is wave-uniform and lives in scalar registers) and by the host-side ew_plan_tiles.
struct TileRef {
  uint64_t src_off, dst_off;  // elements
  uint32_t len;
  uint16_t src_buf, dst_buf;
};

#if defined(__HIPCC__)
#define EW_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define EW_HD inline
#endif
// What a kernel needs to decode tile ids: the records, a coarse index over tile ids (entry b = the
// record holding tile b << shift, so the search below starts at most a few records early whatever
// the number of records: a plan with 1000 records decodes as fast as one with 14), the templates.
struct TableRef {
  const RunT *runs;
  const uint32_t *coarse;
  const TileT *templ;
  uint32_t nruns;
  uint32_t shift;
};

// Division of a 32-bit n by a divisor d >= 1 fixed in advance (Granlund and Montgomery, "Division by
// invariant integers using multiplication", 1994): with l = ceil(log2 d),
//   magic = floor(2^32 (2^l - d) / d) + 1,  sh1 = min(l, 1),  sh2 = l - sh1,
//   t = high half of n * magic,  n / d = (t + ((n - t) >> sh1)) >> sh2   exactly, for every n < 2^32.
// Five scalar instructions in a kernel, where a division costs forty and a trip through the vector unit.
inline void div_invariant_setup(uint32_t d, uint32_t &magic, uint8_t &sh1, uint8_t &sh2) {
  uint32_t l = 0;
  while (l < 32 && ((uint64_t)1 << l) < d) ++l;
  magic = (uint32_t)(((((uint64_t)1 << l) - d) << 32) / d + 1);
  sh1 = (uint8_t)(l < 1 ? l : 1);
  sh2 = (uint8_t)(l - sh1);
}
EW_HD uint32_t div_by_invariant(uint32_t n, uint32_t magic, uint32_t sh1, uint32_t sh2) {
  const uint32_t t = (uint32_t)(((uint64_t)n * magic) >> 32);
  return (t + ((n - t) >> sh1)) >> sh2;
}

// A record read as one 32-byte access (in a kernel: one scalar load and one wait, where member-wise
// reads inside the search loop below turn into three dependent loads).
EW_HD RunT load_run(const RunT *p) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef uint32_t u32x8 __attribute__((ext_vector_type(8), aligned(16)));
  const u32x8 raw = *reinterpret_cast<const u32x8 *>(p);
  RunT r;
  __builtin_memcpy(&r, &raw, sizeof(r));
  return r;
#else
  return *p;
#endif
}

EW_HD TileRef decode_tile(const TableRef &tb, uint64_t tile) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef uint32_t tid_t;  // a table that a kernel reads holds fewer than 2^31 tiles (ew_plan_upload)
#else
  typedef uint64_t tid_t;  // the host may decode larger ones
#endif
  const tid_t t = (tid_t)tile;
  uint32_t r = tb.coarse[t >> tb.shift];
  RunT run = load_run(tb.runs + r);
  while (t >= (tid_t)run.tile_end) run = load_run(tb.runs + ++r);  // usually no step: the index lands on the record

  const tid_t local = t - (tid_t)run.tile_begin;
  const uint64_t unit = ((uint64_t)local >> 32) == 0
                            ? (uint64_t)div_by_invariant((uint32_t)local, run.div_magic, run.div_sh1, run.div_sh2)
                            : (uint64_t)local / run.tiles_per_unit;
  const TileT tl = tb.templ[run.templ_begin + (uint32_t)(local - unit * run.tiles_per_unit)];
  TileRef ref;
  ref.src_off = tl.src_off + unit * tl.src_stride;
  ref.dst_off = tl.dst_off + unit * tl.dst_stride;
  ref.len = tl.len;
  ref.src_buf = tl.src_buf;
  ref.dst_buf = tl.dst_buf;
  return ref;
}

// Which tile workgroup w of an n-workgroup launch takes.  The hardware deals consecutive workgroup ids
// round-robin to the 8 XCDs, each with an L2 of its own, so with the identity mapping two neighbouring
// tiles never share an L2, and a 128-byte line that both touch (sources are only 32-byte aligned
// relative to the destination-aligned cuts) is fetched from memory twice.  With group g > 1, inside
// every block of 8*g consecutive workgroups XCD x takes the g consecutive tiles x*g .. x*g+g-1; the
// launch as a whole still walks the tiles in order.  A trailing partial block keeps the identity.
// The mapping is the first thing every workgroup computes, ahead of its only memory access, so a launch
// gets it prepared: no branch and no division in the kernel (a dozen scalar instructions).
struct XcdMap {
  uint32_t g;      // >= 1; 1 is the identity
  uint32_t n;      // workgroups of the launch (below 2^31)
  uint32_t magic;  // division by 8 g, see div_by_invariant
  uint8_t sh1, sh2;
  uint16_t pad;
};
inline XcdMap make_xcd_map(uint32_t g, uint32_t n) {
  XcdMap m;
  m.g = g < 1 ? 1u : (g > (1u << 24) ? (1u << 24) : g);
  m.n = n;
  div_invariant_setup(8u * m.g, m.magic, m.sh1, m.sh2);
  m.pad = 0;
  return m;
}
EW_HD uint32_t xcd_remap(uint32_t w, const XcdMap &m) {
  const uint32_t blk = 8u * m.g;
  const uint32_t base = div_by_invariant(w, m.magic, m.sh1, m.sh2) * blk;
  const uint32_t r = w - base;
  const uint32_t t = base + (r & 7) * m.g + (r >> 3);
  return base + blk <= m.n ? t : w;  // (base + blk stays below 2^31 + 2^27)
}

struct TileTable {       // host-side description of one (which, elem size) table
  std::vector<RunT> runs;
  std::vector<TileT> templ;
  std::vector<uint32_t> coarse;
  uint32_t shift = 0;
  uint64_t ntiles = 0;
  uint32_t tile_bytes = 0;  // nominal size of a tile (most tiles have it; none is larger)
  TableRef host_ref() const {
    return TableRef{runs.data(), coarse.data(), templ.data(), (uint32_t)runs.size(), shift};
  }
  // the same table inside the plan's single device buffer
  TableRef dev = {nullptr, nullptr, nullptr, 0, 0};
};

}  // namespace ew

struct ew_plan_s {
  uint32_t old_dp = 0, new_dp = 0;
  uint64_t alive_mask = 0;
  uint64_t numel = 0;
  uint64_t num_segs = 0;
  std::vector<uint64_t> old_len, new_len;       // shard lengths in elements
  std::vector<int32_t> new_rank_of, holder_of;  // per old rank
  std::vector<uint64_t> pair_len, pair_off;     // [holder * new_dp + dst_rank]
  uint64_t stage_len = 0;
  uint64_t live_read = 0, snap_read = 0;        // bit j: some segment reads that buffer
  std::vector<ew::Run> runs;
  std::vector<ew::RunSeg> run_segs;
  // explicit table, expanded on first request
  std::once_flag segs_once;
  std::vector<ew_seg_t> segs;
  // device side (filled by ew_plan_upload)
  bool uploaded = false;
  int device = -1;  // device that holds dev_buf; pack / unpack refuse to launch on another
  uint32_t tile_elems[2] = {0, 0};              // [0]: 2-byte elements, [1]: 4-byte elements
  ew::TileTable tables[3][2];                   // [which: 0 pack, 1 unpack, 2 direct][elem size index]
  void *host_buf = nullptr;                     // pinned staging copy, kept until the plan is freed
  void *dev_buf = nullptr;
};

namespace ew {
// Cuts the plan's run segments into tile templates.  which = 0 (pack): non-LOCAL segments, source ->
// arena.  which = 1 (unpack): every segment, arena or local source -> new shard.  which = 2 (direct):
// every segment, source -> new shard, no arena.
// Cuts inside a segment fall on multiples of align_elems in the destination buffer (0 or 1: none).
void build_tile_table(const ew_plan_t &plan, int which, uint32_t tile_elems, uint32_t align_elems,
                      TileTable &out);
}  // namespace ew
