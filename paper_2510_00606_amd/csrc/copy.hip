// Tile-table-driven copy for gfx950: pack (Live Remap step 3, sender side) and unpack (receiver
// side and step 4), Sec. 5.2; the tile tables' life on the device (ew_plan_upload, ew_plan_free);
// and the plain copy that serves as the yardstick.  HBM-bandwidth bound: nothing here is a
// contraction, so no MFMA.
#include <cstring>
#include <new>

#include "device_util.h"
#include "runtime.h"

namespace {

using ew::CopyTabs;
using ew::kThreads;
using ew::kUnroll;
using ew::load16;
using ew::RunT;
using ew::store16;
using ew::TableRef;
using ew::TileT;
using ew::u32x4;

// One workgroup copies one tile: at most tile_elems elements of one segment of one unit, i.e. a
// plain contiguous copy between two buffers picked from the pointer tables.  The tile id is
// decoded against the run-length tables: record (one coarse-index lookup plus a short walk), unit
// inside the record (a multiply and two shifts prepared per record), tile template inside the unit.
// Everything up to the addresses is wave-uniform and runs on the scalar unit from cache-resident
// tables, so no per-tile record is streamed from HBM: about 95 scalar instructions and five round
// trips to the scalar cache (arguments, coarse index, record, template, the two buffer pointers) before
// the workgroup's vector load.  With a true division in the decode and in the workgroup -> tile mapping,
// member-wise reads of the record and one round trip per pointer it was 190 instructions, some on the
// vector unit, and nine round trips, and pack and unpack ran 1.3-1.5 % slower.  The default tile is
// 4 KiB: every lane moves one 128-bit vector, and the GPU is kept full by the sheer number of workgroups.
//
// There is no loop over tiles: every table load then precedes every store of the workgroup, which
// lets the compiler keep the decode on the scalar unit (a persistent loop forces vector loads of
// the tables, since a store might alias them: 3.9 instead of 6.2 TB/s).
template <int ES>
__global__ __launch_bounds__(kThreads) void ew_segcopy_kernel(TableRef table, CopyTabs tabs, ew::XcdMap xcd) {
  const ew::TileRef tl = ew::decode_tile(table, ew::xcd_remap(blockIdx.x, xcd));
  const char *sbase = tabs.src[tl.src_buf];
  char *dbase = tabs.dst[tl.dst_buf];
  ew::want_scalars((uint64_t)sbase, (uint64_t)dbase);
  const char *s = sbase + tl.src_off * ES;
  char *d = dbase + tl.dst_off * ES;
  const uint32_t nbytes = tl.len * ES;
  if ((((uintptr_t)s | (uintptr_t)d) & 15u) == 0) {
    const u32x4 *sv = reinterpret_cast<const u32x4 *>(s);
    const uint32_t nvec = nbytes >> 4;
    const ew::StoreWindow<> out(d, nvec << 4);
    uint32_t i = threadIdx.x;
    for (; i + (kUnroll - 1) * kThreads < nvec; i += kUnroll * kThreads) {  // tiles above 12 KiB only
      u32x4 v[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) v[u] = load16(sv + i + u * kThreads);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) out.put((i + u * kThreads) << 4, v[u]);
    }
    for (; i < nvec; i += kThreads) out.put(i << 4, load16(sv + i));
    // fewer than 16 trailing bytes: whole elements, one per lane
    const uint32_t done = nvec << 4;
    const uint32_t rem = (nbytes - done) / ES;
    if (threadIdx.x < rem) {
      if (ES == 2)
        reinterpret_cast<uint16_t *>(d + done)[threadIdx.x] = reinterpret_cast<const uint16_t *>(s + done)[threadIdx.x];
      else
        reinterpret_cast<uint32_t *>(d + done)[threadIdx.x] = reinterpret_cast<const uint32_t *>(s + done)[threadIdx.x];
    }
  } else {
    // a unit whose length is not a multiple of 8 elements shifts later pieces off the 16-byte
    // grid: element-wise copy (buffers are always element-aligned)
    if (ES == 2) {
      const uint16_t *se = reinterpret_cast<const uint16_t *>(s);
      uint16_t *de = reinterpret_cast<uint16_t *>(d);
      for (uint32_t i = threadIdx.x; i < tl.len; i += kThreads) de[i] = se[i];
    } else {
      const uint32_t *se = reinterpret_cast<const uint32_t *>(s);
      uint32_t *de = reinterpret_cast<uint32_t *>(d);
      for (uint32_t i = threadIdx.x; i < tl.len; i += kThreads) de[i] = se[i];
    }
  }
}

// Plain copy, one 128-bit vector per lane, no table and no fold, in one-wave workgroups (the fastest
// shape measured for a bare copy: 6.6 TB/s, against 6.5 with 256 lanes): the reference a profiler's
// byte counters and the other kernels' rates are calibrated against.
constexpr int kCopyThreads = 64;
__global__ __launch_bounds__(kCopyThreads) void ew_copy_kernel(const u32x4 *__restrict__ src,
                                                               u32x4 *__restrict__ dst, uint64_t nvec) {
  const uint64_t first = (uint64_t)blockIdx.x * kCopyThreads;  // the workgroup's first vector
  const uint64_t left = nvec - first;
  const ew::StoreWindow<> out(dst + first, (uint32_t)(left < kCopyThreads ? left : kCopyThreads) << 4);
  if (threadIdx.x < left) out.put(threadIdx.x << 4, load16(src + first + threadIdx.x));
}

void release_tables(ew_plan_t *plan) {
  if (plan->dev_buf) (void)hipFree(plan->dev_buf);
  if (plan->host_buf) (void)hipHostFree(plan->host_buf);
  plan->dev_buf = plan->host_buf = nullptr;
  plan->uploaded = false;
  plan->device = -1;
  for (int w = 0; w < ew::kNumTables; ++w)
    for (int e = 0; e < 2; ++e) plan->tables[w][e] = ew::TileTable();
}

int launch_segcopy(const ew::TileTable &tt, const CopyTabs &tabs, uint32_t elem_size, hipStream_t stream) {
  if (tt.ntiles == 0) return EW_OK;
  // One launch for the whole table (cutting it into launches of 64 Ki-512 Ki tiles, which gains the fused
  // unpack + snapshot kernel 0.7-0.9 %, changes nothing here down to 256 Ki tiles and costs 0.4-3 % below).
  const uint32_t grid = (uint32_t)tt.ntiles;  // ew_plan_upload refuses tables above 2^31-1 tiles
  const ew::XcdMap g = ew::make_xcd_map(ew::xcd_group_for((uint64_t)tt.tile_bytes), grid);
  if (elem_size == 2)
    hipLaunchKernelGGL(ew_segcopy_kernel<2>, dim3(grid), dim3(kThreads), 0, stream, tt.dev, tabs, g);
  else
    hipLaunchKernelGGL(ew_segcopy_kernel<4>, dim3(grid), dim3(kThreads), 0, stream, tt.dev, tabs, g);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

// Rounds a table's byte size up so that the next table starts 16-byte aligned.
size_t pad16(size_t n) { return (n + 15) & ~(size_t)15; }

}  // namespace

extern "C" {

void ew_plan_free(ew_plan_t *plan) {
  if (!plan) return;
  release_tables(plan);
  delete plan;
}

uint64_t ew_plan_num_tiles(const ew_plan_t *plan, int which, uint32_t elem_size) {
  if (!plan || which < 0 || which >= ew::kNumTables || (elem_size != 2 && elem_size != 4)) return 0;
  const int e = elem_size == 4 ? 1 : 0;
  if (plan->uploaded) return plan->tables[which][e].ntiles;
  const ew::Knobs &k = ew::knobs();
  const int64_t knob_elems = k.tile_elems;
  const uint32_t te = knob_elems > 0 ? (uint32_t)knob_elems : (uint32_t)(k.tile_bytes / elem_size);
  try {
    ew::TileTable tt;
    ew::build_tile_table(*plan, which, te, (uint32_t)(k.tile_align_bytes / elem_size), tt);
    return tt.ntiles;
  } catch (const std::bad_alloc &) {
    return 0;
  }
}

int ew_plan_upload(ew_plan_t *plan, uint32_t tile_elems, void *stream) {
  if (!plan) return EW_EINVAL;
  if (tile_elems > (1u << 24)) return EW_EINVAL;
  release_tables(plan);
  const ew::Knobs &k = ew::knobs();
  const int64_t knob_elems = k.tile_elems, knob_bytes = k.tile_bytes, knob_align = k.tile_align_bytes;
  if (tile_elems == 0 && knob_elems > 0) tile_elems = (uint32_t)knob_elems;
  size_t bytes = 0;
  try {
    for (int e = 0; e < 2; ++e) {
      const uint32_t es = e ? 4u : 2u;
      plan->tile_elems[e] = tile_elems ? tile_elems : (uint32_t)(knob_bytes / es);
      for (int w = 0; w < ew::kNumTables; ++w) {
        ew::TileTable &tt = plan->tables[w][e];
        ew::build_tile_table(*plan, w, plan->tile_elems[e], (uint32_t)(knob_align / es), tt);
        tt.tile_bytes = plan->tile_elems[e] * es;
        if (tt.ntiles > 0x7fffffffull) {  // tile ids are workgroup ids
          release_tables(plan);
          return EW_EINVAL;
        }
        bytes += tt.runs.size() * sizeof(RunT) + tt.templ.size() * sizeof(TileT) +
                 pad16(tt.coarse.size() * sizeof(uint32_t));
      }
    }
  } catch (const std::bad_alloc &) {
    release_tables(plan);
    return EW_ENOMEM;
  }
  if (bytes > 0) {
    if (hipGetDevice(&plan->device) != hipSuccess) {
      (void)hipGetLastError();
      plan->device = -1;
      return EW_EINVAL;
    }
    if (hipHostMalloc(&plan->host_buf, bytes, hipHostMallocDefault) != hipSuccess ||
        hipMalloc(&plan->dev_buf, bytes) != hipSuccess) {
      (void)hipGetLastError();
      release_tables(plan);
      return EW_ENOMEM;
    }
    size_t off = 0;
    char *h = (char *)plan->host_buf, *d = (char *)plan->dev_buf;
    for (int w = 0; w < ew::kNumTables; ++w)
      for (int e = 0; e < 2; ++e) {  // templates (48 B records) first keeps everything 16-byte aligned
        ew::TileTable &tt = plan->tables[w][e];
        const size_t tb = tt.templ.size() * sizeof(TileT), rb = tt.runs.size() * sizeof(RunT);
        const size_t cb = pad16(tt.coarse.size() * sizeof(uint32_t));
        tt.dev.nruns = (uint32_t)tt.runs.size();
        tt.dev.shift = tt.shift;
        std::memcpy(h + off, tt.templ.data(), tb);
        tt.dev.templ = (const TileT *)(d + off);
        off += tb;
        std::memcpy(h + off, tt.runs.data(), rb);
        tt.dev.runs = (const RunT *)(d + off);
        off += rb;
        std::memset(h + off, 0, cb);
        std::memcpy(h + off, tt.coarse.data(), tt.coarse.size() * sizeof(uint32_t));
        tt.dev.coarse = (const uint32_t *)(d + off);
        off += cb;
      }
    const hipError_t e =
        hipMemcpyAsync(plan->dev_buf, plan->host_buf, bytes, hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) {
      release_tables(plan);
      return ew::hip_fail(e, "hipMemcpyAsync(tile tables)");
    }
  }
  plan->uploaded = true;
  return EW_OK;
}

int ew_pack(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots, void *stage,
            uint32_t elem_size, void *stream) {
  if (!ew::tables_usable(plan) || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const ew::TileTable &tt = plan->tables[0][elem_size == 4 ? 1 : 0];
  if (tt.ntiles == 0) return EW_OK;
  if (!stage) return EW_EINVAL;
  CopyTabs tabs;
  const int rc = ew::fill_tabs(plan, old_shards, snapshots, tabs);
  if (rc != EW_OK) return rc;
  tabs.dst[ew::kDstStage] = (char *)stage;
  return launch_segcopy(tt, tabs, elem_size, (hipStream_t)stream);
}

int ew_unpack(const ew_plan_t *plan, const void *stage, const void *const *old_shards, const void *const *snapshots,
              void *const *new_shards, uint32_t elem_size, void *stream) {
  if (!ew::tables_usable(plan) || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const ew::TileTable &tt = plan->tables[1][elem_size == 4 ? 1 : 0];
  if (tt.ntiles == 0) return EW_OK;
  if (!new_shards) return EW_EINVAL;
  if (plan->stage_len > 0 && !stage) return EW_EINVAL;
  CopyTabs tabs;
  const int rc = ew::fill_tabs(plan, old_shards, snapshots, tabs);
  if (rc != EW_OK) return rc;
  tabs.src[ew::kSrcStage] = (const char *)stage;
  for (uint32_t k = 0; k < plan->new_dp; ++k) {
    if (plan->new_len[k] > 0 && !new_shards[k]) return EW_EINVAL;
    tabs.dst[k] = (char *)new_shards[k];
  }
  return launch_segcopy(tt, tabs, elem_size, (hipStream_t)stream);
}

int ew_reshard(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
               void *const *new_shards, uint32_t elem_size, void *stream) {
  if (!ew::tables_usable(plan) || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const ew::TileTable &tt = plan->tables[2][elem_size == 4 ? 1 : 0];
  if (tt.ntiles == 0) return EW_OK;
  if (!new_shards) return EW_EINVAL;
  CopyTabs tabs;
  const int rc = ew::fill_tabs(plan, old_shards, snapshots, tabs);
  if (rc != EW_OK) return rc;
  for (uint32_t k = 0; k < plan->new_dp; ++k) {
    if (plan->new_len[k] > 0 && !new_shards[k]) return EW_EINVAL;
    tabs.dst[k] = (char *)new_shards[k];
  }
  return launch_segcopy(tt, tabs, elem_size, (hipStream_t)stream);
}

int ew_memcpy(const void *src, void *dst, uint64_t nbytes, void *stream) {
  if (nbytes == 0) return EW_OK;
  if (!src || !dst || (nbytes & 15u) || (((uintptr_t)src | (uintptr_t)dst) & 15u)) return EW_EINVAL;
  const uint64_t nvec = nbytes >> 4;
  const uint64_t grid = (nvec + kCopyThreads - 1) / kCopyThreads;
  if (grid > 0x7fffffffull) return EW_EINVAL;
  hipLaunchKernelGGL(ew_copy_kernel, dim3((uint32_t)grid), dim3(kCopyThreads), 0, (hipStream_t)stream,
                     (const u32x4 *)src, (u32x4 *)dst, nvec);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

}  // extern "C"
