// Unpack (Live Remap step 3 receiver side and step 4, Sec. 5.2) fused with the snapshot of the new
// shards (Sec. 5.1): every tile is loaded once and stored twice (new shard and its snapshot copy),
// and its bytes are folded into the checksum of the 1 MiB block of the NEW shard they land in, so
// the fresh snapshot of the new layout costs no second read pass.
//
// A block's words arrive from many tiles, possibly in pieces that are not word aligned (ragged
// units); both sum and xor decompose over bytes, so an element at byte offset o of its shard
// contributes  element << 8*(o mod 8)  to the record of block o >> 20.  Each workgroup writes its
// tile's (sum, xor) to the tile's slot of a scratch region; the rare tile that straddles a block
// boundary adds its upper part to the next block's record directly.  ew_fold_tiles_kernel then
// walks the slots in tile order and adds runs of equal (rank, block) to the records.  When no
// scratch region can be had (a stream under graph capture that would take the last region outside
// graphs), every workgroup adds its tile to the record itself: same bits, more atomics.
#include <cstring>
#include <type_traits>

#include "device_util.h"
#include "runtime.h"

// Cache policy of the store to the new shard and of the store to its snapshot copy (see StoreWindow).
// nt + sc1 on both, like the two-stream kernels: +1-1.5 % over nt alone now that tiles go to the XCDs
// in runs (6.07 -> 6.12 and 5.98 -> 6.07 TB/s on two sets of buffers); with tiles dealt out one by one
// it was neutral to -1 %, and giving the two stores different policies costs 1.5 % either way round.
#ifndef EW_FUSED_AUX1
#define EW_FUSED_AUX1 EW_STORE_AUX
#endif
#ifndef EW_FUSED_AUX2
#define EW_FUSED_AUX2 EW_STORE_AUX
#endif

namespace {

using ew::block_fold;
using ew::CopyTabs;
using ew::fold;
using ew::kThreads;
using ew::load16;
using ew::store16;
using ew::TableRef;
using ew::u32x4;

struct SnapTabs {
  char *snap[EW_MAX_DP];       // snapshot buffer of each new rank
  ew_cksum_t *rec[EW_MAX_DP];  // checksum records of each new rank
  uint32_t nblk[EW_MAX_DP];    // records per rank
};

__device__ __forceinline__ void add_to_record(ew_cksum_t *rec, uint64_t sum, uint64_t xr) {
  atomicAdd(reinterpret_cast<unsigned long long *>(&rec->sum), (unsigned long long)sum);
  atomicXor(reinterpret_cast<unsigned long long *>(&rec->xr), (unsigned long long)xr);
}

template <int ES, bool SLOTS>
__global__ __launch_bounds__(kThreads) void ew_unpack_snap_kernel(TableRef table, uint64_t tile_base, CopyTabs tabs,
                                                                  SnapTabs st, ew_cksum_t *__restrict__ slots,
                                                                  ew::XcdMap xcd) {
  __shared__ uint64_t lds_sum[kThreads / 64], lds_xor[kThreads / 64];
  __shared__ uint64_t lds_sum_hi[kThreads / 64], lds_xor_hi[kThreads / 64];
  typedef typename std::conditional<ES == 2, uint16_t, uint32_t>::type elem_t;
  const uint32_t tile = ew::xcd_remap(blockIdx.x, xcd);  // of this pass
  const ew::TileRef tl = ew::decode_tile(table, tile_base + tile);
  const char *sbase = tabs.src[tl.src_buf];
  char *dbase = tabs.dst[tl.dst_buf], *d2base = st.snap[tl.dst_buf];
  ew::want_scalars((uint64_t)sbase, (uint64_t)dbase, (uint64_t)d2base);
  const char *s = sbase + tl.src_off * ES;
  const uint64_t dbyte = tl.dst_off * ES;  // byte offset inside the new shard
  char *d = dbase + dbyte;
  char *d2 = d2base + dbyte;
  const uint32_t nbytes = tl.len * ES;
  const uint64_t boundary = ((dbyte >> 20) + 1) << 20;  // where the next checksum block starts
  const bool straddle = dbyte + nbytes > boundary;      // wave-uniform, rare
  uint64_t sum = 0, xr = 0, sum_hi = 0, xr_hi = 0;
  if ((((uintptr_t)s | (uintptr_t)d | (uintptr_t)d2 | dbyte) & 15u) == 0) {
    const u32x4 *sv = reinterpret_cast<const u32x4 *>(s);
    const uint32_t nvec = nbytes >> 4;
    const ew::StoreWindow<EW_FUSED_AUX1> out(d, nvec << 4);
    const ew::StoreWindow<EW_FUSED_AUX2> out2(d2, nvec << 4);
    for (uint32_t i = threadIdx.x; i < nvec; i += kThreads) {  // one trip for the default 4 KiB tile
      const u32x4 v = load16(sv + i);
      out.put(i << 4, v);
      out2.put(i << 4, v);
      if (straddle && dbyte + 16ull * i >= boundary)
        fold(v, sum_hi, xr_hi);
      else
        fold(v, sum, xr);
    }
    const uint32_t done = nvec << 4;
    const uint32_t rem = (nbytes - done) / ES;  // fewer than 16 trailing bytes: whole elements
    if (threadIdx.x < rem) {
      const elem_t e = reinterpret_cast<const elem_t *>(s + done)[threadIdx.x];
      reinterpret_cast<elem_t *>(d + done)[threadIdx.x] = e;
      reinterpret_cast<elem_t *>(d2 + done)[threadIdx.x] = e;
      const uint64_t o = dbyte + done + (uint64_t)threadIdx.x * ES;
      const uint64_t c = (uint64_t)e << (8 * (o & 7));
      if (o >= boundary) {
        sum_hi += c;
        xr_hi ^= c;
      } else {
        sum += c;
        xr ^= c;
      }
    }
  } else {
    const elem_t *se = reinterpret_cast<const elem_t *>(s);
    elem_t *de = reinterpret_cast<elem_t *>(d);
    elem_t *d2e = reinterpret_cast<elem_t *>(d2);
    for (uint32_t i = threadIdx.x; i < tl.len; i += kThreads) {
      const elem_t e = se[i];
      de[i] = e;
      d2e[i] = e;
      const uint64_t o = dbyte + (uint64_t)i * ES;
      const uint64_t c = (uint64_t)e << (8 * (o & 7));
      if (o >= boundary) {
        sum_hi += c;
        xr_hi ^= c;
      } else {
        sum += c;
        xr ^= c;
      }
    }
  }
  block_fold(sum, xr, lds_sum, lds_xor);
  if (threadIdx.x == 0) {
    if (SLOTS) {
      ew_cksum_t r;
      r.sum = sum;
      r.xr = xr;
      slots[tile] = r;
    } else {
      add_to_record(st.rec[tl.dst_buf] + (dbyte >> 20), sum, xr);
    }
  }
  if (straddle) {
    block_fold(sum_hi, xr_hi, lds_sum_hi, lds_xor_hi);
    if (threadIdx.x == 0) add_to_record(st.rec[tl.dst_buf] + (boundary >> 20), sum_hi, xr_hi);
  }
}

// Lane g walks the slots of tiles [g*per_lane, (g+1)*per_lane) of the pass and sums runs of tiles that share
// (new rank, block): tiles of a segment are adjacent, and tiles are numbered destination-major, so the keys
// never decrease along the lanes.  A run that ends inside a lane's range goes to its record at once; the
// run still open at the end of the range is first combined with the equal-keyed open runs of the following
// lanes of the wave (a segmented reduction with shuffles), and only the first lane of every key adds it to
// the record: one pair of atomics per (wave, block) instead of one per lane -- the atomics are what this
// kernel waits for.
template <int ES>
__global__ __launch_bounds__(kThreads) void ew_fold_tiles_kernel(TableRef table, uint64_t tile_base, uint64_t ntiles,
                                                                 uint32_t per_lane, SnapTabs st,
                                                                 const ew_cksum_t *__restrict__ slots) {
  const uint64_t g = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  uint64_t i = g * per_lane;  // may lie beyond the pass: such lanes only take part in the shuffles
  const uint64_t end = (i + per_lane < ntiles) ? i + per_lane : ntiles;
  uint32_t key_rank = 0;
  uint64_t key_blk = 0, sum = 0, xr = 0;
  bool open = false;
  for (; i < end; ++i) {
    const ew::TileRef tl = ew::decode_tile(table, tile_base + i);
    const uint64_t blk = (tl.dst_off * ES) >> 20;
    if (open && (tl.dst_buf != key_rank || blk != key_blk)) {
      add_to_record(st.rec[key_rank] + key_blk, sum, xr);
      sum = 0;
      xr = 0;
    }
    open = true;
    key_rank = tl.dst_buf;
    key_blk = blk;
    const ew_cksum_t r = slots[i];
    sum += r.sum;
    xr ^= r.xr;
  }
  // block numbers stay below 2^44 (byte offsets below 2^64), ranks below 2^7
  const uint64_t none = ~(uint64_t)0;
  const uint64_t key = open ? (((uint64_t)key_rank << 44) | key_blk) : none;
  const int lane = threadIdx.x & 63;
  for (int d = 1; d < 64; d <<= 1) {
    const uint64_t other_key = __shfl_down((unsigned long long)key, d, 64);
    const uint64_t other_sum = __shfl_down((unsigned long long)sum, d, 64);
    const uint64_t other_xr = __shfl_down((unsigned long long)xr, d, 64);
    if (lane + d < 64 && other_key == key) {  // equal keys are contiguous: lane + d lies in the same run
      sum += other_sum;
      xr ^= other_xr;
    }
  }
  const uint64_t prev_key = __shfl_up((unsigned long long)key, 1, 64);
  if (open && (lane == 0 || prev_key != key)) add_to_record(st.rec[key_rank] + key_blk, sum, xr);
}

// Zeroes every new rank's records: blockIdx.y = rank, 2 words per record.
__global__ __launch_bounds__(kThreads) void ew_zero_records_kernel(SnapTabs st) {
  const uint32_t k = blockIdx.y;
  const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < 2ull * st.nblk[k]) reinterpret_cast<uint64_t *>(st.rec[k])[i] = 0;
}

// One pass = the tiles [t0, t0 + n) whose slots fit the scratch region: the tile kernel in launches of at most
// `per_launch` tiles, then one fold over the whole pass.  Cutting the tile kernel's work into launches of
// about 1 GiB of destination (256 Ki tiles of 4 KiB, half a millisecond each) makes this kernel 0.7-0.9 %
// faster than one launch of 3 ms (7B stage, one process, same buffers: 128 Ki +0.7 %, 256 Ki +0.7-0.9 %,
// 512 Ki +0.4 %, 1 Mi +0.15 %, 64 Ki -0.2 %, 32 Ki -2.1 %), although every cut drains the GPU; the two-stream
// kernels gain nothing from it.  That is with the three streams in one 96-GiB region of the HBM (6.12 TB/s) or
// the two written ones in one (6.36: +0.75 %); with the three in three regions (6.59) the cut costs 0.4 %.
// Knob fused_pass_tiles.
template <int ES>
int launch_pass(const ew::TileTable &tt, uint64_t t0, uint64_t n, uint64_t per_launch, const CopyTabs &tabs,
                const SnapTabs &st, ew_cksum_t *slots, hipStream_t stream) {
  // Tiles per lane of the fold (knob fold_tiles_per_lane overrides).  With the lanes' open runs combined
  // across the wave before anything is added to a record, few tiles per lane are best: 1 / 2 / 4 / 8 / 16 / 32
  // per lane take 16.6 / 15.8 / 17.4 / 24.6 / 30.1 / 40.6 us on a pass of 1.76 M tiles and 3.6 / 3.8 / 4.9 /
  // 7.9 / 10.7 / 18.4 us on one of 1024 tiles (one pair of atomics per lane, as before: 366 / 171 / 81 / 53 /
  // 39 / 43 and 19 / 12 / 10 / 11 / 12 / 18 us).
  const int64_t knob = ew::knobs().fold_tiles_per_lane;
  const uint32_t kTilesPerLane = knob > 0 ? (uint32_t)knob : 2u;
  const uint64_t fold_grid = ((n + kTilesPerLane - 1) / kTilesPerLane + kThreads - 1) / kThreads;
  // Resident workgroups per CU can be capped by asking for unused dynamic LDS (knob fused_wgs_per_cu).
  // With tiles dealt to the XCDs one by one, six per CU were 1-5 % faster than the eight that fit
  // (three HBM streams per workgroup); with runs of tiles per XCD (xcd_remap) all eight are best
  // (7b stage, fp32: 5.97 / 5.98 / 5.85 / 5.62 TB/s at 8 / 7 / 6 / 5 per CU), so no cap by default.
  const uint32_t lds_pad = ew::occupancy_pad(ew::knobs().fused_wgs_per_cu, 8 * sizeof(uint64_t) * (kThreads / 64));
  const uint32_t group = ew::xcd_group_for((uint64_t)tt.tile_bytes);
  for (uint64_t off = 0; off < n; off += per_launch) {
    const uint32_t m = (uint32_t)(n - off < per_launch ? n - off : per_launch);
    const ew::XcdMap xcd = ew::make_xcd_map(group, m);
    if (slots)
      hipLaunchKernelGGL((ew_unpack_snap_kernel<ES, true>), dim3(m), dim3(kThreads), lds_pad, stream, tt.dev, t0 + off,
                         tabs, st, slots + off, xcd);
    else  // no scratch region: the workgroups add to the records themselves
      hipLaunchKernelGGL((ew_unpack_snap_kernel<ES, false>), dim3(m), dim3(kThreads), lds_pad, stream, tt.dev,
                         t0 + off, tabs, st, slots, xcd);
    EW_HIP(hipGetLastError());
  }
  if (!slots) return EW_OK;
  hipLaunchKernelGGL(ew_fold_tiles_kernel<ES>, dim3((uint32_t)fold_grid), dim3(kThreads), 0, stream, tt.dev, t0, n,
                     kTilesPerLane, st, slots);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

// which = 1: through the arena (stage); which = 2: every segment straight from its source
int unpack_snapshot(const ew_plan_t *plan, int which, const void *stage, const void *const *old_shards,
                    const void *const *snapshots, void *const *new_shards, void *const *new_snapshots,
                    ew_cksum_t *const *new_cksums, uint32_t elem_size, void *stream_) {
  if (!ew::tables_usable(plan) || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const int e = elem_size == 4 ? 1 : 0;
  const ew::TileTable &tt = plan->tables[which][e];
  if (tt.ntiles == 0) return EW_OK;
  if (!new_shards || !new_snapshots || !new_cksums) return EW_EINVAL;
  if (which == 1 && plan->stage_len > 0 && !stage) return EW_EINVAL;
  if ((uint64_t)plan->tile_elems[e] * elem_size > EW_CKSUM_BLOCK) return EW_EINVAL;  // a tile spans <= 2 blocks
  hipStream_t stream = (hipStream_t)stream_;
  CopyTabs tabs;
  const int rc = ew::fill_tabs(plan, old_shards, snapshots, tabs);
  if (rc != EW_OK) return rc;
  tabs.src[ew::kSrcStage] = (const char *)stage;
  SnapTabs st;
  std::memset(&st, 0, sizeof(st));
  uint32_t max_blk = 0;
  for (uint32_t k = 0; k < plan->new_dp; ++k) {
    if (plan->new_len[k] == 0) continue;
    if (!new_shards[k] || !new_snapshots[k] || !new_cksums[k]) return EW_EINVAL;
    const uint64_t nblk = (plan->new_len[k] * elem_size + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
    if (nblk > 0x3fffffffull) return EW_EINVAL;  // 2 words per record must fit the zero-fill grid
    tabs.dst[k] = (char *)new_shards[k];
    st.snap[k] = (char *)new_snapshots[k];
    st.rec[k] = new_cksums[k];
    st.nblk[k] = (uint32_t)nblk;
    if (st.nblk[k] > max_blk) max_blk = st.nblk[k];
  }
  ew::ScratchLease lease(stream);
  ew_cksum_t *slots = lease.slots();  // nullptr: launch_pass takes the scratch-free form
  if (ew::knobs().fused_mode == 1) slots = nullptr;
  hipLaunchKernelGGL(ew_zero_records_kernel, dim3((2 * max_blk + kThreads - 1) / kThreads, plan->new_dp),
                     dim3(kThreads), 0, stream, st);
  EW_HIP(hipGetLastError());
  const uint64_t per_pass = slots ? ew::kRegionSlots : 0x7fffffffull;
  uint64_t per_launch = per_pass;
  if (const int64_t cap = ew::knobs().fused_pass_tiles; cap > 0 && (uint64_t)cap < per_launch) per_launch = (uint64_t)cap;
  for (uint64_t t0 = 0; t0 < tt.ntiles; t0 += per_pass) {
    const uint64_t n = tt.ntiles - t0 < per_pass ? tt.ntiles - t0 : per_pass;
    const int prc = elem_size == 2 ? launch_pass<2>(tt, t0, n, per_launch, tabs, st, slots, stream)
                                   : launch_pass<4>(tt, t0, n, per_launch, tabs, st, slots, stream);
    if (prc != EW_OK) return prc;
  }
  return EW_OK;
}

}  // namespace

extern "C" {

int ew_unpack_snapshot(const ew_plan_t *plan, const void *stage, const void *const *old_shards,
                       const void *const *snapshots, void *const *new_shards, void *const *new_snapshots,
                       ew_cksum_t *const *new_cksums, uint32_t elem_size, void *stream) {
  return unpack_snapshot(plan, 1, stage, old_shards, snapshots, new_shards, new_snapshots, new_cksums, elem_size, stream);
}

int ew_reshard_snapshot(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
                        void *const *new_shards, void *const *new_snapshots, ew_cksum_t *const *new_cksums,
                        uint32_t elem_size, void *stream) {
  return unpack_snapshot(plan, 2, nullptr, old_shards, snapshots, new_shards, new_snapshots, new_cksums, elem_size,
                         stream);
}

}  // extern "C"
