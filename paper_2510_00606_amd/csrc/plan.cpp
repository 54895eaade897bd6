// Host planner: Live Remap steps 1 and 2 (Sec. 5.2) under the interleaved ZeRO assignment
// (Sec. 6.3, Fig. 10b).  Integer arithmetic only, no GPU work.
//
// For one unit the old cuts (degree old_dp) and the new cuts (degree new_dp) are two sorted
// lists over the same element range; their common refinement, swept with two cursors, is the
// element-exact content of the overlap matrix M_overlap for that unit.  A refined interval is
// one segment: it lies in exactly one old piece (so it has one owner, one holder, one source
// buffer) and in exactly one new piece (one destination).  Offsets inside shards are running
// sums of piece lengths because a shard is the concatenation of its pieces in unit order; for
// a run of equal units they advance by the same amounts from unit to unit, which is what the
// run-length form records.
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

struct Builder {
  ew_plan_t *p;
  std::vector<uint64_t> old_cur, new_cur, pair_cur, pair_unit;

  explicit Builder(ew_plan_t *plan) : p(plan) {
    old_cur.assign(p->old_dp, 0);
    new_cur.assign(p->new_dp, 0);
    pair_cur.assign((size_t)p->old_dp * p->new_dp, 0);
    pair_unit.assign((size_t)p->old_dp * p->new_dp, 0);
  }

  // n consecutive units of L elements each, every one split over all old ranks and all new ranks
  void add_run(uint64_t L, uint64_t n) {
    if (L == 0 || n == 0) return;
    PieceList o, w;
    o.uniform(L, p->old_dp, 0, 0);
    w.uniform(L, p->new_dp, 0, 0);
    add_pieces(L, n, o, w);
  }

  // An ownership of one unit: piece i covers [b[i], b[i+1]) and belongs to rank r[i].  A rank owns
  // at most one piece of a unit.
  struct PieceList {
    uint64_t b[EW_MAX_DP + 2];
    uint16_t r[EW_MAX_DP + 1];
    uint32_t n = 0;
    // appends the uniform split of [base, base + L) over ranks rank0 .. rank0 + D - 1
    void uniform(uint64_t L, uint32_t D, uint64_t base, uint32_t rank0) {
      uint64_t pb[EW_MAX_DP + 1];
      piece_bounds(L, D, pb);
      for (uint32_t j = 0; j < D; ++j) {
        b[n] = base + pb[j];
        r[n] = (uint16_t)(rank0 + j);
        ++n;
      }
      b[n] = base + L;
    }
  };

  // n consecutive units of L elements each with the given old and new ownership
  void add_pieces(uint64_t L, uint64_t n, const PieceList &o, const PieceList &w) {
    if (L == 0 || n == 0) return;
    const uint32_t Dn = p->new_dp;
    const uint64_t *ob = o.b, *nb = w.b;
    ew::Run run;
    run.n_units = n;
    run.unit_len = L;
    run.seg_begin = (uint32_t)p->run_segs.size();
    std::fill(pair_unit.begin(), pair_unit.end(), 0);
    uint32_t oi = 0, ni = 0;
    while (oi < o.n && ni < w.n) {
      const uint64_t lo = std::max(ob[oi], nb[ni]);
      const uint64_t hi = std::min(ob[oi + 1], nb[ni + 1]);
      if (lo < hi) {
        const uint32_t j = o.r[oi], k = w.r[ni];
        ew::RunSeg s;
        std::memset(&s, 0, sizeof(s));
        const bool owner_alive = (p->alive_mask >> j) & 1u;
        const uint32_t h = (uint32_t)p->holder_of[j];
        s.src_owner = (uint16_t)j;
        s.holder = (uint16_t)h;
        s.dst_rank = (uint16_t)k;
        s.len = hi - lo;
        s.src_off = old_cur[j] + (lo - ob[oi]);
        s.dst_off = new_cur[k] + (lo - nb[ni]);
        s.src_stride = ob[oi + 1] - ob[oi];
        s.dst_stride = nb[ni + 1] - nb[ni];
        if (!owner_alive) {
          s.flags |= EW_SEG_SNAPSHOT;
          p->snap_read |= 1ull << j;
        } else {
          p->live_read |= 1ull << j;
        }
        if (p->new_rank_of[h] == (int32_t)k) {
          s.flags |= EW_SEG_LOCAL;
          s.stage_off = EW_NO_STAGE;
        } else {
          // position inside the pair's message; the message base is added by finish()
          const size_t idx = (size_t)h * Dn + k;
          s.stage_off = pair_cur[idx] + pair_unit[idx];
          pair_unit[idx] += s.len;
        }
        p->run_segs.push_back(s);
      }
      const uint64_t oe = ob[oi + 1], ne = nb[ni + 1];
      if (oe <= ne) ++oi;
      if (ne <= oe) ++ni;
    }
    run.seg_end = (uint32_t)p->run_segs.size();
    for (uint32_t i = run.seg_begin; i < run.seg_end; ++i) {
      ew::RunSeg &s = p->run_segs[i];
      if (!(s.flags & EW_SEG_LOCAL)) s.stage_stride = pair_unit[(size_t)s.holder * Dn + s.dst_rank];
    }
    for (uint32_t i = 0; i < o.n; ++i) old_cur[o.r[i]] += n * (ob[i + 1] - ob[i]);
    for (uint32_t i = 0; i < w.n; ++i) new_cur[w.r[i]] += n * (nb[i + 1] - nb[i]);
    for (size_t i = 0; i < pair_cur.size(); ++i) pair_cur[i] += n * pair_unit[i];
    p->numel += n * L;
    p->num_segs += n * (uint64_t)(run.seg_end - run.seg_begin);
    if (run.seg_end > run.seg_begin) p->runs.push_back(run);
  }

  // runs of equal-length units among units [u0, u1) of a boundary array, all with one ownership rule
  template <class Add>
  void for_runs(const uint64_t *starts, uint64_t u0, uint64_t u1, Add add) {
    uint64_t u = u0;
    while (u < u1) {
      const uint64_t L = starts[u + 1] - starts[u];
      uint64_t v = u + 1;
      while (v < u1 && starts[v + 1] - starts[v] == L) ++v;
      add(L, v - u);
      u = v;
    }
  }

  void finish() {
    const uint32_t Do = p->old_dp, Dn = p->new_dp;
    p->old_len = old_cur;
    p->new_len = new_cur;
    p->pair_len = pair_cur;
    p->pair_off.assign((size_t)Do * Dn, 0);
    // arena: one contiguous message per (holder -> destination) pair, sorted by (dst, holder)
    uint64_t off = 0;
    for (uint32_t k = 0; k < Dn; ++k)
      for (uint32_t h = 0; h < Do; ++h) {
        const size_t idx = (size_t)h * Dn + k;
        p->pair_off[idx] = off;
        off += p->pair_len[idx];
      }
    p->stage_len = off;
    for (ew::RunSeg &s : p->run_segs)
      if (!(s.flags & EW_SEG_LOCAL)) s.stage_off += p->pair_off[(size_t)s.holder * Dn + s.dst_rank];
  }
};

// Step 1, integrity check: every failed rank's partition must exist in the snapshot kept by its
// ring predecessor (worker i backs up worker (i+1) mod n, Sec. 5.1).  Also fixes the new rank
// numbering: survivors in order, densely from 0.
int new_plan(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, ew_plan_t **out) {
  if (!out || old_dp == 0 || new_dp == 0 || old_dp > EW_MAX_DP || new_dp > EW_MAX_DP) return EW_EINVAL;
  if (old_dp < 64 && (alive_mask >> old_dp) != 0) return EW_EINVAL;
  if (alive_mask == 0) return EW_EUNRECOVERABLE;
  auto alive = [&](uint32_t j) { return (alive_mask >> j) & 1u; };
  for (uint32_t j = 0; j < old_dp; ++j)
    if (!alive(j) && !alive((j + old_dp - 1) % old_dp)) return EW_EUNRECOVERABLE;
  ew_plan_t *p = new (std::nothrow) ew_plan_t();
  if (!p) return EW_ENOMEM;
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
      p->holder_of[j] = (int32_t)((j + old_dp - 1) % old_dp);
    }
  }
  *out = p;
  return EW_OK;
}

void expand_segs(ew_plan_t *p) {
  p->segs.reserve(p->num_segs);
  for (const ew::Run &run : p->runs)
    for (uint64_t i = 0; i < run.n_units; ++i)
      for (uint32_t r = run.seg_begin; r < run.seg_end; ++r) {
        const ew::RunSeg &t = p->run_segs[r];
        ew_seg_t s;
        std::memset(&s, 0, sizeof(s));
        s.src_off = t.src_off + i * t.src_stride;
        s.dst_off = t.dst_off + i * t.dst_stride;
        s.stage_off = (t.flags & EW_SEG_LOCAL) ? EW_NO_STAGE : t.stage_off + i * t.stage_stride;
        s.len = t.len;
        s.src_owner = t.src_owner;
        s.holder = t.holder;
        s.dst_rank = t.dst_rank;
        s.flags = t.flags;
        p->segs.push_back(s);
      }
}

}  // namespace

namespace ew {

// Tile order.  Tiles are numbered destination-major: for unpack, new rank by new rank (each new
// shard is written front to back); for pack, pair message by pair message in arena order.  Within
// a destination the runs follow each other, and within a run the units.  The workgroups in flight
// at any moment then write one sequential stream and read the two or three old shards that
// overlap it, which is what HBM likes: numbering tiles unit by unit instead makes up to
// old_dp + new_dp streams advance in lock step at equal offsets of equally sized buffers, and the
// identity plan of the 7B stage then copies at 4.8 TB/s instead of 6.3 (measured).
//
// Tile cuts.  A segment is cut so that every cut point inside it falls on a multiple of
// align_elems in the DESTINATION buffer (128 bytes by default): the first tile runs from the
// segment's start to the last such point within tile_elems, the following tiles are full and
// aligned, the last one takes the rest.  Neighbouring workgroups, which run on different XCDs with
// separate L2s, then never write parts of the same 128-byte line (measured: 4 % on the copy rate).
// The phase of a segment's destination offset changes from unit to unit by its stride, so the
// templates are laid down for a period of P consecutive units after which all phases repeat
// (P <= 128 bytes / 16 bytes = 8 when unit lengths are multiples of the 8-element granule; a
// group with a longer period is cut without alignment), and a record's "unit" is that period.
static uint64_t gcd_u64(uint64_t a, uint64_t b) {
  while (b) {
    const uint64_t t = a % b;
    a = b;
    b = t;
  }
  return a;
}

void build_tile_table(const ew_plan_t &plan, int which, uint32_t tile_elems, uint32_t align_elems,
                      TileTable &out) {
  out.runs.clear();
  out.templ.clear();
  out.ntiles = 0;
  if (align_elems == 0 || tile_elems % align_elems != 0) align_elems = 1;
  struct Item {
    uint32_t key, run, seg;
  };
  std::vector<Item> items;
  for (uint32_t ri = 0; ri < plan.runs.size(); ++ri) {
    const Run &run = plan.runs[ri];
    for (uint32_t r = run.seg_begin; r < run.seg_end; ++r) {
      const RunSeg &s = plan.run_segs[r];
      if (which == 0 && (s.flags & EW_SEG_LOCAL)) continue;
      const uint32_t key = which == 0 ? (uint32_t)s.dst_rank * EW_MAX_DP + s.holder : s.dst_rank;
      items.push_back({key, ri, r});
    }
  }
  std::stable_sort(items.begin(), items.end(), [](const Item &a, const Item &b) {
    return a.key != b.key ? a.key < b.key : (a.run != b.run ? a.run < b.run : a.seg < b.seg);
  });

  struct Piece {  // one segment of the group, as source -> destination of this table
    uint64_t src, dst, src_stride, dst_stride, len;
    uint16_t src_buf, dst_buf;
  };
  std::vector<Piece> group;
  size_t i = 0;
  while (i < items.size()) {
    const uint32_t key = items[i].key, ri = items[i].run;
    const Run &run = plan.runs[ri];
    group.clear();
    for (; i < items.size() && items[i].key == key && items[i].run == ri; ++i) {
      const RunSeg &s = plan.run_segs[items[i].seg];
      const bool local = (s.flags & EW_SEG_LOCAL) != 0;
      const uint16_t data_buf =
          (uint16_t)((s.flags & EW_SEG_SNAPSHOT) ? kSrcSnap + s.src_owner : kSrcLive + s.holder);
      Piece pc;
      pc.len = s.len;
      if (which == 0) {  // source buffer -> arena
        pc.src_buf = data_buf;
        pc.dst_buf = (uint16_t)kDstStage;
        pc.src = s.src_off;
        pc.dst = s.stage_off;
        pc.src_stride = s.src_stride;
        pc.dst_stride = s.stage_stride;
      } else if (local || which == 2) {  // source buffer -> new shard
        pc.src_buf = data_buf;
        pc.dst_buf = s.dst_rank;
        pc.src = s.src_off;
        pc.dst = s.dst_off;
        pc.src_stride = s.src_stride;
        pc.dst_stride = s.dst_stride;
      } else {  // arena -> new shard
        pc.src_buf = (uint16_t)kSrcStage;
        pc.dst_buf = s.dst_rank;
        pc.src = s.stage_off;
        pc.dst = s.dst_off;
        pc.src_stride = s.stage_stride;
        pc.dst_stride = s.dst_stride;
      }
      group.push_back(pc);
    }
    // period after which every piece's destination phase repeats
    uint64_t period = 1, align = align_elems;
    if (align > 1 && run.n_units > 1) {
      for (const Piece &pc : group) {
        const uint64_t ps = align / gcd_u64(pc.dst_stride % align, align);  // stride % align == 0 -> 1
        period = period / gcd_u64(period, ps) * ps;
        if (period > 8) break;
      }
      if (period > 8) {
        period = 1;
        align = 1;
      }
    }
    // lays down `units` consecutive units starting at unit `first` as one record repeated `reps` times
    auto emit = [&](uint64_t first, uint64_t units, uint64_t reps) {
      RunT rt;
      rt.tile_begin = out.ntiles;
      rt.templ_begin = (uint32_t)out.templ.size();
      for (uint64_t u = 0; u < units; ++u)
        for (const Piece &pc : group) {
          TileT t;
          std::memset(&t, 0, sizeof(t));
          t.src_buf = pc.src_buf;
          t.dst_buf = pc.dst_buf;
          t.src_stride = pc.src_stride * units;
          t.dst_stride = pc.dst_stride * units;
          const uint64_t src = pc.src + (first + u) * pc.src_stride;
          const uint64_t dst = pc.dst + (first + u) * pc.dst_stride;
          uint64_t done = 0;
          while (done < pc.len) {
            const uint64_t room = tile_elems - (dst + done) % align;  // up to the last aligned point
            const uint64_t n = std::min<uint64_t>(room, pc.len - done);
            t.src_off = src + done;
            t.dst_off = dst + done;
            t.len = (uint32_t)n;
            out.templ.push_back(t);
            done += n;
          }
        }
      rt.tiles_per_unit = (uint32_t)(out.templ.size() - rt.templ_begin);
      out.ntiles += (uint64_t)rt.tiles_per_unit * reps;
      rt.tile_end = out.ntiles;
      div_invariant_setup(rt.tiles_per_unit, rt.div_magic, rt.div_sh1, rt.div_sh2);
      rt.pad = 0;
      out.runs.push_back(rt);
    };
    const uint64_t whole = run.n_units / period, rest = run.n_units % period;
    if (whole > 0) emit(0, period, whole);
    if (rest > 0) emit(whole * period, rest, 1);
  }
  // coarse index: about four buckets per record
  out.shift = 0;
  while ((out.ntiles >> out.shift) > 4 * (uint64_t)out.runs.size() + 64) ++out.shift;
  out.coarse.assign((size_t)(out.ntiles >> out.shift) + 1, 0);
  uint32_t r = 0;
  for (size_t b = 0; b < out.coarse.size(); ++b) {
    const uint64_t t = (uint64_t)b << out.shift;
    while (r + 1 < out.runs.size() && out.runs[r + 1].tile_begin <= t) ++r;
    out.coarse[b] = r;
  }
}

}  // namespace ew

extern "C" {

int ew_plan(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t numel, uint64_t chunk,
            ew_plan_t **out) {
  if (chunk == 0) return EW_EINVAL;
  ew_plan_t *p = nullptr;
  const int rc = new_plan(old_dp, new_dp, alive_mask, &p);
  if (rc != EW_OK) return rc;
  try {
    Builder b(p);
    b.add_run(chunk, numel / chunk);
    b.add_run(numel % chunk, 1);
    b.finish();
  } catch (const std::bad_alloc &) {
    delete p;
    return EW_ENOMEM;
  }
  *out = p;
  return EW_OK;
}

int ew_plan_bounds(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t n_units,
                   const uint64_t *unit_starts, ew_plan_t **out) {
  if (!unit_starts || unit_starts[0] != 0) return EW_EINVAL;
  for (uint64_t u = 0; u < n_units; ++u)
    if (unit_starts[u + 1] < unit_starts[u]) return EW_EINVAL;
  ew_plan_t *p = nullptr;
  const int rc = new_plan(old_dp, new_dp, alive_mask, &p);
  if (rc != EW_OK) return rc;
  try {
    Builder b(p);
    b.for_runs(unit_starts, 0, n_units, [&](uint64_t L, uint64_t n) { b.add_run(L, n); });
    b.finish();
  } catch (const std::bad_alloc &) {
    delete p;
    return EW_ENOMEM;
  }
  *out = p;
  return EW_OK;
}

int ew_plan_migrate(uint32_t assignment, uint32_t dp, uint64_t n_src_units, const uint64_t *src_unit_starts,
                    uint64_t n_dst_units, const uint64_t *dst_unit_starts, uint64_t n_move, ew_plan_t **out) {
  if (assignment != EW_ASSIGN_INTERLEAVED && assignment != EW_ASSIGN_CONTIGUOUS) return EW_EINVAL;
  if (dp == 0 || 2 * dp > EW_MAX_DP || !src_unit_starts || !dst_unit_starts) return EW_EINVAL;
  if (src_unit_starts[0] != 0 || dst_unit_starts[0] != 0 || n_move > n_src_units) return EW_EINVAL;
  for (uint64_t u = 0; u < n_src_units; ++u)
    if (src_unit_starts[u + 1] < src_unit_starts[u]) return EW_EINVAL;
  for (uint64_t u = 0; u < n_dst_units; ++u)
    if (dst_unit_starts[u + 1] < dst_unit_starts[u]) return EW_EINVAL;
  // ranks 0..dp-1 are stage S, dp..2dp-1 stage S+1, before and after; everybody is alive
  ew_plan_t *p = nullptr;
  const uint64_t all = 2 * dp == 64 ? ~0ull : ((1ull << (2 * dp)) - 1);
  const int rc = new_plan(2 * dp, 2 * dp, all, &p);
  if (rc != EW_OK) return rc;
  try {
    Builder b(p);
    using PL = Builder::PieceList;
    const uint64_t keep = n_src_units - n_move;
    if (assignment == EW_ASSIGN_INTERLEAVED) {
      // every layer is split over the ranks of the stage that holds it (Fig. 10b): a moved layer's
      // piece j goes from rank j of stage S to rank j of stage S+1, nothing else changes owner
      auto add = [&](uint32_t old0, uint32_t new0) {
        return [&b, dp, old0, new0](uint64_t L, uint64_t n) {
          PL o, w;
          o.uniform(L, dp, 0, old0);
          w.uniform(L, dp, 0, new0);
          b.add_pieces(L, n, o, w);
        };
      };
      b.for_runs(src_unit_starts, 0, keep, add(0, 0));
      b.for_runs(src_unit_starts, keep, n_src_units, add(0, dp));
      b.for_runs(dst_unit_starts, 0, n_dst_units, add(dp, dp));
    } else {
      // each stage keeps one flat array cut into dp contiguous blocks (Fig. 10a): the two arrays,
      // laid end to end, form one unit whose cuts all move when the layers change sides
      const uint64_t A = src_unit_starts[n_src_units], B = dst_unit_starts[n_dst_units];
      const uint64_t M = A - src_unit_starts[keep];
      PL o, w;
      o.uniform(A, dp, 0, 0);
      o.uniform(B, dp, A, dp);
      w.uniform(A - M, dp, 0, 0);
      w.uniform(B + M, dp, A - M, dp);
      b.add_pieces(A + B, 1, o, w);
    }
    b.finish();
  } catch (const std::bad_alloc &) {
    delete p;
    return EW_ENOMEM;
  }
  *out = p;
  return EW_OK;
}

int ew_plan_tiles(const ew_plan_t *p, int which, uint32_t tile_elems, uint32_t align_elems, uint64_t first,
                  uint64_t count, ew_tile_t *out, uint64_t *total) {
  if (!p || which < 0 || which >= ew::kNumTables || tile_elems == 0 || tile_elems > (1u << 24)) return EW_EINVAL;
  if (count > 0 && !out) return EW_EINVAL;
  try {
    ew::TileTable tt;
    ew::build_tile_table(*p, which, tile_elems, align_elems, tt);
    if (total) *total = tt.ntiles;
    if (count == 0) return EW_OK;
    if (first > tt.ntiles || count > tt.ntiles - first) return EW_EINVAL;
    for (uint64_t i = 0; i < count; ++i) {
      const ew::TileRef r = ew::decode_tile(tt.host_ref(), first + i);
      out[i].src_off = r.src_off;
      out[i].dst_off = r.dst_off;
      out[i].len = r.len;
      out[i].src_buf = r.src_buf;
      out[i].dst_buf = r.dst_buf;
    }
  } catch (const std::bad_alloc &) {
    return EW_ENOMEM;
  }
  return EW_OK;
}

uint64_t ew_plan_numel(const ew_plan_t *p) { return p ? p->numel : 0; }
uint32_t ew_plan_old_dp(const ew_plan_t *p) { return p ? p->old_dp : 0; }
uint32_t ew_plan_new_dp(const ew_plan_t *p) { return p ? p->new_dp : 0; }
uint64_t ew_plan_num_segs(const ew_plan_t *p) { return p ? p->num_segs : 0; }
uint64_t ew_plan_num_runs(const ew_plan_t *p) { return p ? p->runs.size() : 0; }
const ew_seg_t *ew_plan_segs(const ew_plan_t *cp) {
  if (!cp) return nullptr;
  ew_plan_t *p = const_cast<ew_plan_t *>(cp);  // the cache is the only mutable part
  try {
    std::call_once(p->segs_once, expand_segs, p);
  } catch (const std::bad_alloc &) {
    return nullptr;
  }
  return p->segs.data();
}
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

uint64_t ew_tile_of_workgroup(uint64_t workgroup, uint64_t n_workgroups, uint32_t group) {
  // launches have fewer than 2^31 workgroups; beyond that nothing is remapped
  if (workgroup >= n_workgroups || n_workgroups > 0x7fffffffull) return workgroup;
  return ew::xcd_remap((uint32_t)workgroup, ew::make_xcd_map(group, (uint32_t)n_workgroups));
}

}  // extern "C"
