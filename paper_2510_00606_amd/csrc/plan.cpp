// Host planner: Live Remap steps 1 and 2 (Sec. 5.2) under the interleaved ZeRO assignment
// (Sec. 6.3, Fig. 10b).  Integer arithmetic only, no GPU work.
//
// For every unit the old cuts (degree old_dp) and the new cuts (degree new_dp) are two sorted
// lists over the same element range; their common refinement, swept with two cursors, is the
// element-exact content of the overlap matrix M_overlap for that unit.  A refined interval is
// one segment: it lies in exactly one old piece (so it has one owner, one holder, one source
// buffer) and in exactly one new piece (one destination).  Offsets inside shards are running
// sums of piece lengths because a shard is the concatenation of its pieces in unit order.
#include <algorithm>
#include <cstring>
#include <new>

#include "plan_internal.h"

namespace {

// b_j = min(L, 8 * floor(j * ceil(L/8) / D)), j = 0..D
inline void piece_bounds(uint64_t L, uint32_t D, uint64_t *b) {
  const uint64_t n_gran = L / EW_GRANULE + (L % EW_GRANULE ? 1 : 0);
  for (uint32_t j = 0; j <= D; ++j) {
    const unsigned __int128 q = (unsigned __int128)j * n_gran / D;
    const uint64_t v = (uint64_t)q * EW_GRANULE;
    b[j] = v < L ? v : L;
  }
}

template <class UnitLen>
int build(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t n_units, UnitLen unit_len,
          ew_plan_t **out) {
  if (!out || old_dp == 0 || new_dp == 0 || old_dp > EW_MAX_DP || new_dp > EW_MAX_DP) return EW_EINVAL;
  if (old_dp < 64 && (alive_mask >> old_dp) != 0) return EW_EINVAL;

  // Step 1, integrity check: every failed rank's partition must exist in the snapshot kept by
  // its ring predecessor (worker i backs up worker (i+1) mod n, Sec. 5.1).
  auto alive = [&](uint32_t j) { return (alive_mask >> j) & 1u; };
  if (alive_mask == 0) return EW_EUNRECOVERABLE;
  ew_plan_t *p = new (std::nothrow) ew_plan_t();
  if (!p) return EW_ENOMEM;
  try {
    p->old_dp = old_dp;
    p->new_dp = new_dp;
    p->alive_mask = alive_mask;
    p->holder_of.assign(old_dp, -1);
    p->new_rank_of.assign(old_dp, -1);
    int32_t next_new = 0;
    for (uint32_t j = 0; j < old_dp; ++j) {
      if (alive(j)) {
        p->holder_of[j] = (int32_t)j;
        if ((uint32_t)next_new < new_dp) p->new_rank_of[j] = next_new++;
      } else {
        const uint32_t h = (j + old_dp - 1) % old_dp;
        if (!alive(h)) {
          delete p;
          return EW_EUNRECOVERABLE;
        }
        p->holder_of[j] = (int32_t)h;
      }
    }

    p->old_len.assign(old_dp, 0);
    p->new_len.assign(new_dp, 0);
    p->pair_len.assign((size_t)old_dp * new_dp, 0);
    p->pair_off.assign((size_t)old_dp * new_dp, 0);

    // Step 2: sweep the units.
    uint64_t ob[EW_MAX_DP + 1], nb[EW_MAX_DP + 1];
    uint64_t numel = 0;
    for (uint64_t u = 0; u < n_units; ++u) {
      const uint64_t L = unit_len(u);
      if (L == 0) continue;
      piece_bounds(L, old_dp, ob);
      piece_bounds(L, new_dp, nb);
      uint32_t j = 0, k = 0;
      while (j < old_dp && k < new_dp) {
        const uint64_t lo = std::max(ob[j], nb[k]);
        const uint64_t hi = std::min(ob[j + 1], nb[k + 1]);
        if (lo < hi) {
          ew_seg_t s;
          std::memset(&s, 0, sizeof(s));
          const uint32_t h = (uint32_t)p->holder_of[j];
          s.src_owner = (uint16_t)j;
          s.holder = (uint16_t)h;
          s.dst_rank = (uint16_t)k;
          s.len = hi - lo;
          s.src_off = p->old_len[j] + (lo - ob[j]);
          s.dst_off = p->new_len[k] + (lo - nb[k]);
          s.flags = 0;
          if (!alive(j)) {
            s.flags |= EW_SEG_SNAPSHOT;
            p->snap_read |= 1ull << j;
          } else {
            p->live_read |= 1ull << j;
          }
          if (p->new_rank_of[h] == (int32_t)k) {
            s.flags |= EW_SEG_LOCAL;
            s.stage_off = EW_NO_STAGE;
          } else {
            // offset inside the pair's message for now; the message base is added below
            uint64_t &pl = p->pair_len[(size_t)h * new_dp + k];
            s.stage_off = pl;
            pl += s.len;
          }
          p->segs.push_back(s);
        }
        const uint64_t oe = ob[j + 1], ne = nb[k + 1];
        if (oe <= ne) ++j;
        if (ne <= oe) ++k;
      }
      for (uint32_t r = 0; r < old_dp; ++r) p->old_len[r] += ob[r + 1] - ob[r];
      for (uint32_t r = 0; r < new_dp; ++r) p->new_len[r] += nb[r + 1] - nb[r];
      numel += L;
    }
    p->numel = numel;

    // Arena: one contiguous message per (holder -> destination) pair, sorted by (dst, holder).
    uint64_t off = 0;
    for (uint32_t k = 0; k < new_dp; ++k)
      for (uint32_t h = 0; h < old_dp; ++h) {
        const size_t idx = (size_t)h * new_dp + k;
        p->pair_off[idx] = off;
        off += p->pair_len[idx];
      }
    p->stage_len = off;
    for (ew_seg_t &s : p->segs)
      if (!(s.flags & EW_SEG_LOCAL)) s.stage_off += p->pair_off[(size_t)s.holder * new_dp + s.dst_rank];
  } catch (const std::bad_alloc &) {
    delete p;
    return EW_ENOMEM;
  }
  *out = p;
  return EW_OK;
}

}  // namespace

namespace ew {

uint64_t count_tiles(const ew_plan_t &plan, int which, uint32_t tile_elems) {
  uint64_t n = 0;
  for (const ew_seg_t &s : plan.segs) {
    if (which == 0 && (s.flags & EW_SEG_LOCAL)) continue;
    n += (s.len + tile_elems - 1) / tile_elems;
  }
  return n;
}

void build_tiles(const ew_plan_t &plan, int which, uint32_t tile_elems, std::vector<Tile> &out) {
  out.clear();
  out.reserve(count_tiles(plan, which, tile_elems));
  for (const ew_seg_t &s : plan.segs) {
    const bool local = (s.flags & EW_SEG_LOCAL) != 0;
    if (which == 0 && local) continue;
    const uint16_t data_buf =
        (uint16_t)((s.flags & EW_SEG_SNAPSHOT) ? kSrcSnap + s.src_owner : kSrcLive + s.holder);
    Tile t;
    std::memset(&t, 0, sizeof(t));
    uint64_t src, dst;
    if (which == 0) {  // source buffer -> arena
      t.src_buf = data_buf;
      t.dst_buf = (uint16_t)kDstStage;
      src = s.src_off;
      dst = s.stage_off;
    } else if (local) {  // source buffer -> new shard
      t.src_buf = data_buf;
      t.dst_buf = s.dst_rank;
      src = s.src_off;
      dst = s.dst_off;
    } else {  // arena -> new shard
      t.src_buf = (uint16_t)kSrcStage;
      t.dst_buf = s.dst_rank;
      src = s.stage_off;
      dst = s.dst_off;
    }
    for (uint64_t done = 0; done < s.len; done += tile_elems) {
      t.src_off = src + done;
      t.dst_off = dst + done;
      t.len = (uint32_t)std::min<uint64_t>(tile_elems, s.len - done);
      out.push_back(t);
    }
  }
}

}  // namespace ew

extern "C" {

int ew_plan(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t numel, uint64_t chunk,
            ew_plan_t **out) {
  if (chunk == 0) return EW_EINVAL;
  const uint64_t n_units = numel / chunk + (numel % chunk ? 1 : 0);
  return build(old_dp, new_dp, alive_mask, n_units,
               [=](uint64_t u) { return std::min(chunk, numel - u * chunk); }, out);
}

int ew_plan_bounds(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t n_units,
                   const uint64_t *unit_starts, ew_plan_t **out) {
  if (!unit_starts || unit_starts[0] != 0) return EW_EINVAL;
  for (uint64_t u = 0; u < n_units; ++u)
    if (unit_starts[u + 1] < unit_starts[u]) return EW_EINVAL;
  return build(old_dp, new_dp, alive_mask, n_units,
               [=](uint64_t u) { return unit_starts[u + 1] - unit_starts[u]; }, out);
}

uint64_t ew_plan_numel(const ew_plan_t *p) { return p ? p->numel : 0; }
uint32_t ew_plan_old_dp(const ew_plan_t *p) { return p ? p->old_dp : 0; }
uint32_t ew_plan_new_dp(const ew_plan_t *p) { return p ? p->new_dp : 0; }
uint64_t ew_plan_num_segs(const ew_plan_t *p) { return p ? p->segs.size() : 0; }
const ew_seg_t *ew_plan_segs(const ew_plan_t *p) { return p ? p->segs.data() : nullptr; }
uint64_t ew_plan_old_shard_len(const ew_plan_t *p, uint32_t r) {
  return (p && r < p->old_dp) ? p->old_len[r] : 0;
}
uint64_t ew_plan_new_shard_len(const ew_plan_t *p, uint32_t r) {
  return (p && r < p->new_dp) ? p->new_len[r] : 0;
}
int32_t ew_plan_new_rank_of(const ew_plan_t *p, uint32_t r) {
  return (p && r < p->old_dp) ? p->new_rank_of[r] : -1;
}
int32_t ew_plan_holder_of(const ew_plan_t *p, uint32_t r) {
  return (p && r < p->old_dp) ? p->holder_of[r] : -1;
}
uint64_t ew_plan_stage_len(const ew_plan_t *p) { return p ? p->stage_len : 0; }
uint64_t ew_plan_remote_elems(const ew_plan_t *p) { return p ? p->stage_len : 0; }
uint64_t ew_plan_pair_len(const ew_plan_t *p, uint32_t h, uint32_t k) {
  return (p && h < p->old_dp && k < p->new_dp) ? p->pair_len[(size_t)h * p->new_dp + k] : 0;
}
uint64_t ew_plan_pair_off(const ew_plan_t *p, uint32_t h, uint32_t k) {
  return (p && h < p->old_dp && k < p->new_dp) ? p->pair_off[(size_t)h * p->new_dp + k] : 0;
}

}  // extern "C"
