// HIP kernels for gfx950 (MI355X, wave64) and their launch code:
//   ew_segcopy_kernel   tile-table-driven copy: pack (Live Remap step 3, send side) and
//                       unpack (receive side + step 4), Sec. 5.2
//   ew_cksum_kernel     per-step snapshot copy fused with the per-block checksum (Sec. 5.1 and
//                       the "online verification" of the abstract); read-only form for verify
//   ew_compare_kernel   ordered list of blocks whose checksum changed
// All of them are HBM-bandwidth bound (no contraction anywhere, hence no MFMA): the work is
// 128-bit loads/stores, several in flight per lane, with a 64-bit integer fold on the side.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

#include "plan_internal.h"

namespace {

using ew::RunT;
using ew::TableRef;
using ew::TileT;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#ifndef EW_THREADS
#define EW_THREADS 256
#endif
#ifndef EW_UNROLL
#define EW_UNROLL 4
#endif
#ifndef EW_NT_LOAD
#define EW_NT_LOAD 1
#endif
#ifndef EW_NT_STORE
#define EW_NT_STORE 1
#endif
constexpr int kThreads = EW_THREADS;  // waves of 64
constexpr int kUnroll = EW_UNROLL;    // 16-byte loads in flight per lane in the unrolled body

thread_local std::string g_hip_error = "no HIP error recorded";

int hip_fail(hipError_t e, const char *what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return EW_EHIP;
}
#define EW_HIP(call)                                  \
  do {                                                \
    hipError_t e__ = (call);                          \
    if (e__ != hipSuccess) return hip_fail(e__, #call); \
  } while (0)

// process-wide launch-shape knobs (see ew_set_param)
int64_t g_cksum_sub_bytes = 65536; // bytes of a checksum block handled by one workgroup pass
int64_t g_cksum_wgs_per_cu = 0;    // 0 = one workgroup per sub-block, else persistent grid
int64_t g_cksum_mode = -1;         // -1 = slot kernel + fold for snapshot, atomic kernel for verify;
                                   // 0 / 1 force the slot / atomic kernel for both
int64_t g_tile_bytes = 4096;        // default copy tile: 256 lanes x one 128-bit vector
int64_t g_tile_elems = 0;           // > 0 overrides tile_bytes with a size in elements
int64_t g_tile_align_bytes = 128;   // tile cuts fall on multiples of this in the destination (0: off)

int num_cus() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return 256;
    cached[dev] = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  return cached[dev];
}

__device__ __forceinline__ u32x4 load16(const u32x4 *p) {
#if EW_NT_LOAD
  return __builtin_nontemporal_load(p);
#else
  return *p;
#endif
}
__device__ __forceinline__ void store16(u32x4 *p, u32x4 v) {
#if EW_NT_STORE
  __builtin_nontemporal_store(v, p);
#else
  *p = v;
#endif
}

// ------------------------------------------------------------------------------------------
// Segment copy.  One workgroup copies one tile: at most tile_elems elements of one segment of
// one unit, i.e. a plain contiguous copy between two buffers picked from the pointer tables.
// The tile id is decoded against the run-length tables: run (binary search over a handful of
// records), unit inside the run (one division), tile template inside the unit.  Everything up
// to the addresses is wave-uniform and runs on the scalar unit from scalar-cache-resident
// tables, so no per-tile record is streamed from HBM.  The default tile is 4 KiB: every lane
// moves one 128-bit vector, and the GPU is kept full by the sheer number of workgroups.
// ------------------------------------------------------------------------------------------
struct CopyTabs {
  const char *src[ew::kNumSrc];
  char *dst[ew::kNumDst];
};

template <int ES>
__global__ __launch_bounds__(kThreads) void ew_segcopy_kernel(TableRef table, CopyTabs tabs) {
  // No loop over tiles: every table load then precedes every store of the workgroup, which lets the
  // compiler keep the decode on the scalar unit (a persistent loop forces vector loads of the
  // tables, since a store might alias them: 3.9 instead of 6.2 TB/s).
  {
    const ew::TileRef tl = ew::decode_tile(table, blockIdx.x);
    const char *s = tabs.src[tl.src_buf] + tl.src_off * ES;
    char *d = tabs.dst[tl.dst_buf] + tl.dst_off * ES;
    const uint32_t nbytes = tl.len * ES;
    if ((((uintptr_t)s | (uintptr_t)d) & 15u) == 0) {
      const u32x4 *sv = reinterpret_cast<const u32x4 *>(s);
      u32x4 *dv = reinterpret_cast<u32x4 *>(d);
      const uint32_t nvec = nbytes >> 4;
      uint32_t i = threadIdx.x;
      for (; i + (kUnroll - 1) * kThreads < nvec; i += kUnroll * kThreads) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = load16(sv + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) store16(dv + i + u * kThreads, v[u]);
      }
      for (; i < nvec; i += kThreads) store16(dv + i, load16(sv + i));
      // fewer than 16 trailing bytes: whole elements, one per lane
      const uint32_t done = nvec << 4;
      const uint32_t rem = (nbytes - done) / ES;
      if (threadIdx.x < rem) {
        if (ES == 2)
          reinterpret_cast<uint16_t *>(d + done)[threadIdx.x] =
              reinterpret_cast<const uint16_t *>(s + done)[threadIdx.x];
        else
          reinterpret_cast<uint32_t *>(d + done)[threadIdx.x] =
              reinterpret_cast<const uint32_t *>(s + done)[threadIdx.x];
      }
    } else {
      // a unit whose length is not a multiple of 8 elements shifts later pieces off the
      // 16-byte grid: element-wise copy (buffers are always element-aligned)
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
}

// ------------------------------------------------------------------------------------------
// Snapshot + checksum.  A checksum block (1 MiB) is cut into sub-blocks of `sub` bytes
// (a power of two, 4 KiB..1 MiB); a workgroup streams one sub-block, folding the 64-bit
// words into (sum, xor) per lane, then across the wave with shuffles, then across the four
// waves through LDS.  With sub < 1 MiB the partial results of a block meet in its record
// through 64-bit atomics; sum and xor are commutative, so the bits do not depend on order.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void fold(u32x4 v, uint64_t &sum, uint64_t &xr) {
  const uint64_t w0 = (uint64_t)v.x | ((uint64_t)v.y << 32);
  const uint64_t w1 = (uint64_t)v.z | ((uint64_t)v.w << 32);
  sum += w0 + w1;
  xr ^= w0 ^ w1;
}

// Wave-wide fold of (sum, xor) with DPP moves: four row_shr steps inside each row of 16 lanes,
// then row_bcast:15 and row_bcast:31 carry the row totals across rows.  Lanes a move does not
// reach receive 0, the identity of both operations.  The wave's total ends up in lane 63.
// (Six cross-lane steps on the VALU; the LDS-crossbar shuffles they replace cost 15 % of a 4 KiB
// workgroup's run time.)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp_mov64(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_update_dpp(0u, (uint32_t)v, CTRL, ROW_MASK, 0xf, false);
  const uint32_t hi = __builtin_amdgcn_update_dpp(0u, (uint32_t)(v >> 32), CTRL, ROW_MASK, 0xf, false);
  return (uint64_t)lo | ((uint64_t)hi << 32);
}
constexpr int kWaveFoldLane = 63;
__device__ __forceinline__ void wave_fold(uint64_t &sum, uint64_t &xr) {
  sum += dpp_mov64<0x111, 0xf>(sum);  // row_shr:1
  xr ^= dpp_mov64<0x111, 0xf>(xr);
  sum += dpp_mov64<0x112, 0xf>(sum);  // row_shr:2
  xr ^= dpp_mov64<0x112, 0xf>(xr);
  sum += dpp_mov64<0x114, 0xf>(sum);  // row_shr:4
  xr ^= dpp_mov64<0x114, 0xf>(xr);
  sum += dpp_mov64<0x118, 0xf>(sum);  // row_shr:8
  xr ^= dpp_mov64<0x118, 0xf>(xr);
  sum += dpp_mov64<0x142, 0xa>(sum);  // row_bcast:15 into rows 1 and 3
  xr ^= dpp_mov64<0x142, 0xa>(xr);
  sum += dpp_mov64<0x143, 0xc>(sum);  // row_bcast:31 into rows 2 and 3
  xr ^= dpp_mov64<0x143, 0xc>(xr);
}

template <bool COPY, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void ew_cksum_kernel(const char *__restrict__ src,
                                                            char *__restrict__ dst, uint64_t nbytes,
                                                            ew_cksum_t *out, uint32_t sub,
                                                            uint32_t accumulate) {
  __shared__ uint64_t lds_sum[kThreads / 64];
  __shared__ uint64_t lds_xor[kThreads / 64];
  const uint64_t nsub = (nbytes + sub - 1) / sub;
  for (uint64_t c = blockIdx.x; c < nsub; c += gridDim.x) {
    const uint64_t begin = c * sub;
    const uint64_t left = nbytes - begin;
    const uint32_t n = left < sub ? (uint32_t)left : sub;
    uint64_t sum = 0, xr = 0;
    if (ALIGNED) {
      const u32x4 *sv = reinterpret_cast<const u32x4 *>(src + begin);
      u32x4 *dv = reinterpret_cast<u32x4 *>(dst + begin);
      const uint32_t nvec = n >> 4;
      uint32_t i = threadIdx.x;
      for (; i + (kUnroll - 1) * kThreads < nvec; i += kUnroll * kThreads) {
        u32x4 r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) r[u] = load16(sv + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          if (COPY) store16(dv + i + u * kThreads, r[u]);
          fold(r[u], sum, xr);
        }
      }
      for (; i < nvec; i += kThreads) {
        const u32x4 r = load16(sv + i);
        if (COPY) store16(dv + i, r);
        fold(r, sum, xr);
      }
      // fewer than 16 trailing bytes (only at the very end of the buffer): one lane copies
      // them and folds them as up to two zero-padded little-endian words
      const uint32_t done = nvec << 4;
      if (threadIdx.x == 0 && done < n) {
        uint64_t w[2] = {0, 0};
        for (uint32_t b = done; b < n; ++b) {
          const uint8_t v = (uint8_t)src[begin + b];
          if (COPY) dst[begin + b] = (char)v;
          w[(b - done) >> 3] |= (uint64_t)v << (8 * ((b - done) & 7));
        }
        sum += w[0] + w[1];
        xr ^= w[0] ^ w[1];
      }
    } else {
      // unaligned base: byte loads, one 64-bit word per lane per step
      const uint32_t nwords = (n + 7) >> 3;
      for (uint32_t wi = threadIdx.x; wi < nwords; wi += kThreads) {
        uint64_t w = 0;
        const uint32_t b0 = wi << 3;
        const uint32_t nb = (n - b0) < 8 ? (n - b0) : 8;
        for (uint32_t b = 0; b < nb; ++b) {
          const uint8_t v = (uint8_t)src[begin + b0 + b];
          if (COPY) dst[begin + b0 + b] = (char)v;
          w |= (uint64_t)v << (8 * b);
        }
        sum += w;
        xr ^= w;
      }
    }
    // wave fold
    wave_fold(sum, xr);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == kWaveFoldLane) {
      lds_sum[wave] = sum;
      lds_xor[wave] = xr;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      uint64_t s = 0, x = 0;
#pragma unroll
      for (int w = 0; w < kThreads / 64; ++w) {
        s += lds_sum[w];
        x ^= lds_xor[w];
      }
      ew_cksum_t *rec = out + (begin >> 20);
      if (accumulate) {
        atomicAdd(reinterpret_cast<unsigned long long *>(&rec->sum), (unsigned long long)s);
        atomicXor(reinterpret_cast<unsigned long long *>(&rec->xr), (unsigned long long)x);
      } else {
        rec->sum = s;
        rec->xr = x;
      }
    }
    __syncthreads();  // LDS is reused by the next sub-block of a persistent workgroup
  }
}

// Fast form of the same operation for 16-byte aligned buffers.  Measured on MI355X, a copy
// runs fastest as a flood of small workgroups in which every lane moves ONE 128-bit vector
// (4 KiB per 256-lane workgroup), and 64-bit atomics from many workgroups onto one checksum
// record serialise badly.  So: each workgroup folds its 4 KiB into one (sum, xor) pair and
// writes it to its own 16-byte slot of a scratch region (no atomics, no zero-fill), and
// ew_fold_kernel then folds the 256 slots of every 1 MiB block into the block's record.
template <bool COPY>
__global__ __launch_bounds__(kThreads) void ew_cksum_slots_kernel(const u32x4 *__restrict__ src,
                                                                  u32x4 *__restrict__ dst, uint64_t nbytes,
                                                                  ew_cksum_t *__restrict__ slots) {
  static_assert(kThreads == 256, "one slot per 4 KiB assumes 256 lanes x 16 bytes");
  __shared__ uint64_t lds_sum[kThreads / 64];
  __shared__ uint64_t lds_xor[kThreads / 64];
  const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  const uint64_t nvec = nbytes >> 4;
  uint64_t sum = 0, xr = 0;
  if (i < nvec) {
    const u32x4 v = load16(src + i);
    if (COPY) store16(dst + i, v);
    fold(v, sum, xr);
  } else if (i == nvec && (nbytes & 15u)) {
    // fewer than 16 trailing bytes: copied and folded as up to two zero-padded words
    const char *sb = reinterpret_cast<const char *>(src + nvec);
    char *db = reinterpret_cast<char *>(dst + nvec);
    uint64_t w[2] = {0, 0};
    for (uint32_t b = 0; b < (uint32_t)(nbytes & 15u); ++b) {
      const uint8_t v = (uint8_t)sb[b];
      if (COPY) db[b] = (char)v;
      w[b >> 3] |= (uint64_t)v << (8 * (b & 7));
    }
    sum = w[0] + w[1];
    xr = w[0] ^ w[1];
  }
  wave_fold(sum, xr);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == kWaveFoldLane) {
    lds_sum[wave] = sum;
    lds_xor[wave] = xr;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ew_cksum_t r;
    r.sum = lds_sum[0] + lds_sum[1] + lds_sum[2] + lds_sum[3];
    r.xr = lds_xor[0] ^ lds_xor[1] ^ lds_xor[2] ^ lds_xor[3];
    slots[blockIdx.x] = r;
  }
}

// One workgroup per checksum block: folds the block's slots (256 for a full block) into out[b].
__global__ __launch_bounds__(kThreads) void ew_fold_kernel(const ew_cksum_t *__restrict__ slots, uint64_t nslots,
                                                           ew_cksum_t *__restrict__ out) {
  __shared__ uint64_t lds_sum[kThreads / 64];
  __shared__ uint64_t lds_xor[kThreads / 64];
  constexpr uint32_t kSlotsPerBlock = EW_CKSUM_BLOCK / 4096;
  uint64_t sum = 0, xr = 0;
  for (uint32_t t = threadIdx.x; t < kSlotsPerBlock; t += kThreads) {
    const uint64_t sidx = (uint64_t)blockIdx.x * kSlotsPerBlock + t;
    if (sidx < nslots) {
      const ew_cksum_t r = slots[sidx];
      sum += r.sum;
      xr ^= r.xr;
    }
  }
  wave_fold(sum, xr);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == kWaveFoldLane) {
    lds_sum[wave] = sum;
    lds_xor[wave] = xr;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ew_cksum_t r = {0, 0};
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
      r.sum += lds_sum[w];
      r.xr ^= lds_xor[w];
    }
    out[blockIdx.x] = r;
  }
}

// ------------------------------------------------------------------------------------------
// Unpack fused with the snapshot of the new shards: every tile is loaded once and stored twice
// (new shard and its snapshot copy), and its bytes are folded into the checksum of the 1 MiB
// block of the NEW shard they land in, so the fresh snapshot of the new layout costs no second
// read pass.  A block's words arrive from many tiles, possibly in pieces that are not word
// aligned (ragged units); both sum and xor decompose over bytes, so an element at byte offset o
// of its shard contributes  element << 8*(o mod 8)  to the record of block o >> 20.
// Each workgroup writes its tile's (sum, xor) to the tile's slot; the rare tile that straddles a
// block boundary adds its upper part to the next block's record directly.  ew_fold_tiles_kernel
// then walks the slots in tile order and adds runs of equal (rank, block) to the records.
// ------------------------------------------------------------------------------------------
struct SnapTabs {
  char *snap[EW_MAX_DP];        // snapshot buffer of each new rank
  ew_cksum_t *rec[EW_MAX_DP];   // checksum records of each new rank
  uint32_t nblk[EW_MAX_DP];     // records per rank
};

// Workgroup-wide fold; the total is valid in thread 0.  Each call needs LDS cells of its own.
__device__ __forceinline__ void block_fold(uint64_t &sum, uint64_t &xr, uint64_t *lds_sum, uint64_t *lds_xor) {
  wave_fold(sum, xr);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == kWaveFoldLane) {
    lds_sum[wave] = sum;
    lds_xor[wave] = xr;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    sum = 0;
    xr = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
      sum += lds_sum[w];
      xr ^= lds_xor[w];
    }
  }
}

template <int ES>
__global__ __launch_bounds__(kThreads) void ew_unpack_snap_kernel(TableRef table, uint64_t tile_base, CopyTabs tabs,
                                                                  SnapTabs st, ew_cksum_t *__restrict__ slots) {
  __shared__ uint64_t lds_sum[kThreads / 64], lds_xor[kThreads / 64];
  __shared__ uint64_t lds_sum_hi[kThreads / 64], lds_xor_hi[kThreads / 64];
  typedef typename std::conditional<ES == 2, uint16_t, uint32_t>::type elem_t;
  const ew::TileRef tl = ew::decode_tile(table, tile_base + blockIdx.x);
  const char *s = tabs.src[tl.src_buf] + tl.src_off * ES;
  const uint64_t dbyte = tl.dst_off * ES;  // byte offset inside the new shard
  char *d = tabs.dst[tl.dst_buf] + dbyte;
  char *d2 = st.snap[tl.dst_buf] + dbyte;
  const uint32_t nbytes = tl.len * ES;
  const uint64_t boundary = ((dbyte >> 20) + 1) << 20;  // where the next checksum block starts
  const bool straddle = dbyte + nbytes > boundary;      // wave-uniform, rare
  uint64_t sum = 0, xr = 0, sum_hi = 0, xr_hi = 0;
  if ((((uintptr_t)s | (uintptr_t)d | (uintptr_t)d2 | dbyte) & 15u) == 0) {
    const u32x4 *sv = reinterpret_cast<const u32x4 *>(s);
    u32x4 *dv = reinterpret_cast<u32x4 *>(d);
    u32x4 *d2v = reinterpret_cast<u32x4 *>(d2);
    const uint32_t nvec = nbytes >> 4;
    for (uint32_t i = threadIdx.x; i < nvec; i += kThreads) {  // one trip for the default 4 KiB tile
      const u32x4 v = load16(sv + i);
      store16(dv + i, v);
      store16(d2v + i, v);
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
    ew_cksum_t r;
    r.sum = sum;
    r.xr = xr;
    slots[blockIdx.x] = r;
  }
  if (straddle) {
    block_fold(sum_hi, xr_hi, lds_sum_hi, lds_xor_hi);
    if (threadIdx.x == 0) {
      ew_cksum_t *rec = st.rec[tl.dst_buf] + (boundary >> 20);
      atomicAdd(reinterpret_cast<unsigned long long *>(&rec->sum), (unsigned long long)sum_hi);
      atomicXor(reinterpret_cast<unsigned long long *>(&rec->xr), (unsigned long long)xr_hi);
    }
  }
}

// Lane g adds the slots of tiles [g*per_lane, (g+1)*per_lane) of the pass to the records, one
// pair of atomics per run of tiles that share (new rank, block): tiles of a segment are adjacent.
template <int ES>
__global__ __launch_bounds__(kThreads) void ew_fold_tiles_kernel(TableRef table, uint64_t tile_base, uint64_t ntiles,
                                                                 uint32_t per_lane, SnapTabs st,
                                                                 const ew_cksum_t *__restrict__ slots) {
  const uint64_t g = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  uint64_t i = g * per_lane;
  const uint64_t end = (i + per_lane < ntiles) ? i + per_lane : ntiles;
  if (i >= end) return;
  uint32_t key_rank = 0;
  uint64_t key_blk = 0, sum = 0, xr = 0;
  bool open = false;
  for (; i < end; ++i) {
    const ew::TileRef tl = ew::decode_tile(table, tile_base + i);
    const uint64_t blk = (tl.dst_off * ES) >> 20;
    if (open && (tl.dst_buf != key_rank || blk != key_blk)) {
      ew_cksum_t *rec = st.rec[key_rank] + key_blk;
      atomicAdd(reinterpret_cast<unsigned long long *>(&rec->sum), (unsigned long long)sum);
      atomicXor(reinterpret_cast<unsigned long long *>(&rec->xr), (unsigned long long)xr);
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
  ew_cksum_t *rec = st.rec[key_rank] + key_blk;
  atomicAdd(reinterpret_cast<unsigned long long *>(&rec->sum), (unsigned long long)sum);
  atomicXor(reinterpret_cast<unsigned long long *>(&rec->xr), (unsigned long long)xr);
}

// Zeroes every new rank's records: blockIdx.y = rank, 2 words per record.
__global__ __launch_bounds__(kThreads) void ew_zero_records_kernel(SnapTabs st) {
  const uint32_t k = blockIdx.y;
  const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < 2ull * st.nblk[k]) reinterpret_cast<uint64_t *>(st.rec[k])[i] = 0;
}

// Plain copy, one 128-bit vector per lane and 4 KiB per workgroup like the tile copy, no table
// and no fold: the reference a profiler's byte counters and the other kernels' rates are
// calibrated against.
__global__ __launch_bounds__(kThreads) void ew_copy_kernel(const u32x4 *__restrict__ src,
                                                           u32x4 *__restrict__ dst, uint64_t nvec) {
  const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < nvec) store16(dst + i, load16(src + i));
}

__global__ __launch_bounds__(kThreads) void ew_zero_kernel(uint64_t *p, uint64_t nwords) {
  const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < nwords) p[i] = 0;
}

// Single workgroup: ascending list of differing blocks (stable compaction with ballots).
constexpr int kCmpThreads = 1024;
__global__ __launch_bounds__(kCmpThreads) void ew_compare_kernel(const ew_cksum_t *__restrict__ got,
                                                                 const ew_cksum_t *__restrict__ expect,
                                                                 uint64_t nblocks, uint64_t *n_bad,
                                                                 uint64_t *bad_blocks, ew_cksum_t *diffs,
                                                                 uint64_t cap) {
  __shared__ uint32_t wave_cnt[kCmpThreads / 64];
  __shared__ uint64_t base;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  for (uint64_t b0 = 0; b0 < nblocks; b0 += kCmpThreads) {
    const uint64_t b = b0 + threadIdx.x;
    ew_cksum_t g = {0, 0}, e = {0, 0};
    bool bad = false;
    if (b < nblocks) {
      g = got[b];
      e = expect[b];
      bad = (g.sum != e.sum) || (g.xr != e.xr);
    }
    const uint64_t ballot = __ballot(bad);
    if (lane == 0) wave_cnt[wave] = (uint32_t)__popcll(ballot);
    __syncthreads();
    uint64_t before = base, total = 0;
    for (int w = 0; w < kCmpThreads / 64; ++w) {
      if (w < wave) before += wave_cnt[w];
      total += wave_cnt[w];
    }
    if (bad) {
      const uint64_t slot = before + (uint64_t)__popcll(ballot & ((1ull << lane) - 1ull));
      if (slot < cap) {
        bad_blocks[slot] = b;
        diffs[slot].sum = g.sum - e.sum;
        diffs[slot].xr = g.xr ^ e.xr;
      }
    }
    __syncthreads();
    if (threadIdx.x == 0) base += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) *n_bad = base;
}

// ------------------------------------------------------------------------------------------
// launch helpers
// ------------------------------------------------------------------------------------------
void release_tables(ew_plan_t *plan) {
  if (plan->dev_buf) (void)hipFree(plan->dev_buf);
  if (plan->host_buf) (void)hipHostFree(plan->host_buf);
  plan->dev_buf = plan->host_buf = nullptr;
  plan->uploaded = false;
  for (int w = 0; w < 2; ++w)
    for (int e = 0; e < 2; ++e) plan->tables[w][e] = ew::TileTable();
}

int launch_segcopy(const ew::TileTable &tt, const CopyTabs &tabs, uint32_t elem_size, hipStream_t stream) {
  if (tt.ntiles == 0) return EW_OK;
  const uint32_t grid = (uint32_t)tt.ntiles;  // ew_plan_upload refuses tables above 2^31-1 tiles
  if (elem_size == 2)
    hipLaunchKernelGGL(ew_segcopy_kernel<2>, dim3(grid), dim3(kThreads), 0, stream, tt.dev, tabs);
  else
    hipLaunchKernelGGL(ew_segcopy_kernel<4>, dim3(grid), dim3(kThreads), 0, stream, tt.dev, tabs);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

int launch_zero(void *p, uint64_t nbytes, hipStream_t stream) {
  const uint64_t nwords = nbytes / 8;
  if (nwords == 0) return EW_OK;
  const uint64_t grid = (nwords + kThreads - 1) / kThreads;
  hipLaunchKernelGGL(ew_zero_kernel, dim3((uint32_t)grid), dim3(kThreads), 0, stream, (uint64_t *)p,
                     nwords);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

// ---- scratch for the per-workgroup checksum slots --------------------------------------------
// A fixed device array, so taking a snapshot never allocates.  It is cut into regions; a stream
// keeps the region it used last.  When a stream without a region asks for one and all are taken,
// the least recently used region changes hands, and the new owner's stream is first made to wait
// (hipStreamWaitEvent, no host blocking) for the event recorded after the region's last use, so
// two streams never touch a region at once.  A stream under graph capture can only use a region it
// already owns (its warm-up run claims one); otherwise ew_snapshot falls back to the atomic kernel,
// which needs no scratch.  One region (32 MiB) covers 8 GiB of input per pass; longer buffers are
// processed in several passes on the stream.
constexpr uint32_t kRegions = 4;
constexpr uint64_t kRegionSlots = 1ull << 21;                       // 32 MiB of 16-byte slots
constexpr uint64_t kPassBytes = kRegionSlots * 4096;                 // 8 GiB
__device__ __align__(256) ew_cksum_t g_slot_scratch[kRegions * kRegionSlots];

struct Region {
  hipStream_t owner = nullptr;
  bool taken = false;
  hipEvent_t done = nullptr;   // recorded on the owner's stream after each use
  bool recorded = false;
  uint64_t last_use = 0;
};
struct ScratchState {
  std::mutex mu;
  ew_cksum_t *base[64] = {nullptr};  // per device: address of that device's copy of the array
  Region region[64][kRegions];
  uint64_t clock = 0;
};
ScratchState g_scratch;

bool stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st != hipStreamCaptureStatusNone;
}

// Caller holds g_scratch.mu.  Returns the region's device address (and the region through *out), or
// nullptr when none can be had.
ew_cksum_t *acquire_region(hipStream_t stream, Region **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  if (!g_scratch.base[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_slot_scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch.base[dev] = (ew_cksum_t *)p;
  }
  Region *reg = g_scratch.region[dev];
  int pick = -1;
  for (uint32_t r = 0; r < kRegions && pick < 0; ++r)
    if (reg[r].taken && reg[r].owner == stream) pick = (int)r;
  for (uint32_t r = 0; r < kRegions && pick < 0; ++r)
    if (!reg[r].taken) pick = (int)r;
  if (pick < 0) {
    if (stream_is_capturing(stream)) return nullptr;  // cannot order a capture after outside work
    pick = 0;
    for (uint32_t r = 1; r < kRegions; ++r)
      if (reg[r].last_use < reg[pick].last_use) pick = (int)r;
    if (reg[pick].recorded && hipStreamWaitEvent(stream, reg[pick].done, 0) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
  }
  reg[pick].taken = true;
  reg[pick].owner = stream;
  *out = &reg[pick];
  return g_scratch.base[dev] + (uint64_t)pick * kRegionSlots;
}

// Caller holds g_scratch.mu; called after the last kernel of a call has been enqueued.
void release_region(Region *r, hipStream_t stream) {
  r->last_use = ++g_scratch.clock;
  if (stream_is_capturing(stream)) return;  // the graph's own ordering covers replays
  if (!r->done && hipEventCreateWithFlags(&r->done, hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    r->done = nullptr;
    return;
  }
  r->recorded = hipEventRecord(r->done, stream) == hipSuccess;
  if (!r->recorded) (void)hipGetLastError();
}

template <bool COPY>
int launch_cksum_atomic(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *out, hipStream_t stream) {
  const uint32_t sub = (uint32_t)g_cksum_sub_bytes;
  const uint64_t nblocks = (nbytes + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
  const uint32_t accumulate = sub < EW_CKSUM_BLOCK ? 1u : 0u;
  if (accumulate) {
    const int rc = launch_zero(out, nblocks * sizeof(ew_cksum_t), stream);
    if (rc != EW_OK) return rc;
  }
  uint64_t grid = (nbytes + sub - 1) / sub;
  if (g_cksum_wgs_per_cu > 0) {
    const uint64_t cap = (uint64_t)num_cus() * (uint64_t)g_cksum_wgs_per_cu;
    if (grid > cap) grid = cap;
  }
  if (grid > 0x7fffffffull) grid = 0x7fffffffull;
  const bool aligned = ((((uintptr_t)src) | (COPY ? (uintptr_t)dst : 0)) & 15u) == 0;
  if (aligned)
    hipLaunchKernelGGL((ew_cksum_kernel<COPY, true>), dim3((uint32_t)grid), dim3(kThreads), 0, stream,
                       (const char *)src, (char *)dst, nbytes, out, sub, accumulate);
  else
    hipLaunchKernelGGL((ew_cksum_kernel<COPY, false>), dim3((uint32_t)grid), dim3(kThreads), 0, stream,
                       (const char *)src, (char *)dst, nbytes, out, sub, accumulate);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

template <bool COPY>
int launch_cksum(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *out, hipStream_t stream) {
  const bool aligned = ((((uintptr_t)src) | (COPY ? (uintptr_t)dst : 0)) & 15u) == 0;
  // Read-only passes (verify) keep the streaming kernel: without stores to overlap, the wave-level
  // fold of a 4 KiB workgroup costs more than it saves (3.4 vs 6.2 TB/s measured).
  const int64_t mode = g_cksum_mode >= 0 ? g_cksum_mode : (COPY ? 0 : 1);
  if (!aligned || mode != 0) return launch_cksum_atomic<COPY>(src, dst, nbytes, out, stream);
  // the (slot kernel, fold kernel) pairs of one call must reach the stream back to back
  std::lock_guard<std::mutex> lock(g_scratch.mu);
  Region *region = nullptr;
  ew_cksum_t *slots = acquire_region(stream, &region);
  if (!slots) return launch_cksum_atomic<COPY>(src, dst, nbytes, out, stream);
  for (uint64_t off = 0; off < nbytes; off += kPassBytes) {
    const uint64_t n = nbytes - off < kPassBytes ? nbytes - off : kPassBytes;
    // one workgroup (and slot) per 4 KiB; a partial trailing vector belongs to lane n/16, which
    // the last workgroup always contains because ceil(n/4096)*256 > n/16 whenever 16 does not divide n
    const uint64_t grid = (n + 4095) / 4096;
    const uint64_t nblk = (n + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
    hipLaunchKernelGGL((ew_cksum_slots_kernel<COPY>), dim3((uint32_t)grid), dim3(kThreads), 0, stream,
                       (const u32x4 *)((const char *)src + off), (u32x4 *)(COPY ? (char *)dst + off : nullptr), n,
                       slots);
    EW_HIP(hipGetLastError());
    hipLaunchKernelGGL(ew_fold_kernel, dim3((uint32_t)nblk), dim3(kThreads), 0, stream, slots, grid,
                       out + off / EW_CKSUM_BLOCK);
    EW_HIP(hipGetLastError());
  }
  release_region(region, stream);
  return EW_OK;
}

int fill_tabs(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
              CopyTabs &tabs, bool need_local_only) {
  std::memset(&tabs, 0, sizeof(tabs));
  (void)need_local_only;
  for (uint32_t j = 0; j < plan->old_dp; ++j) {
    const void *live = old_shards ? old_shards[j] : nullptr;
    const void *snap = snapshots ? snapshots[j] : nullptr;
    if (((plan->live_read >> j) & 1) && !live) return EW_EINVAL;
    if (((plan->snap_read >> j) & 1) && !snap) return EW_EINVAL;
    tabs.src[ew::kSrcLive + j] = (const char *)live;
    tabs.src[ew::kSrcSnap + j] = (const char *)snap;
  }
  return EW_OK;
}

}  // namespace

extern "C" {

void ew_plan_free(ew_plan_t *plan) {
  if (!plan) return;
  release_tables(plan);
  delete plan;
}

uint64_t ew_plan_num_tiles(const ew_plan_t *plan, int which, uint32_t elem_size) {
  if (!plan || (which != 0 && which != 1) || (elem_size != 2 && elem_size != 4)) return 0;
  const int e = elem_size == 4 ? 1 : 0;
  if (plan->uploaded) return plan->tables[which][e].ntiles;
  const uint32_t te = g_tile_elems > 0 ? (uint32_t)g_tile_elems : (uint32_t)(g_tile_bytes / elem_size);
  try {
    ew::TileTable tt;
    ew::build_tile_table(*plan, which, te, (uint32_t)(g_tile_align_bytes / elem_size), tt);
    return tt.ntiles;
  } catch (const std::bad_alloc &) {
    return 0;
  }
}

int ew_plan_upload(ew_plan_t *plan, uint32_t tile_elems, void *stream) {
  if (!plan) return EW_EINVAL;
  if (tile_elems > (1u << 24)) return EW_EINVAL;
  release_tables(plan);
  if (tile_elems == 0 && g_tile_elems > 0) tile_elems = (uint32_t)g_tile_elems;
  size_t bytes = 0;
  try {
    for (int e = 0; e < 2; ++e) {
      const uint32_t es = e ? 4u : 2u;
      plan->tile_elems[e] = tile_elems ? tile_elems : (uint32_t)(g_tile_bytes / es);
      for (int w = 0; w < 2; ++w) {
        ew::TileTable &tt = plan->tables[w][e];
        ew::build_tile_table(*plan, w, plan->tile_elems[e], (uint32_t)(g_tile_align_bytes / es), tt);
        if (tt.ntiles > 0x7fffffffull) {  // tile ids are workgroup ids
          release_tables(plan);
          return EW_EINVAL;
        }
        bytes += tt.runs.size() * sizeof(RunT) + tt.templ.size() * sizeof(TileT) +
                 ((tt.coarse.size() * sizeof(uint32_t) + 15) & ~(size_t)15);
      }
    }
  } catch (const std::bad_alloc &) {
    release_tables(plan);
    return EW_ENOMEM;
  }
  if (bytes > 0) {
    if (hipHostMalloc(&plan->host_buf, bytes, hipHostMallocDefault) != hipSuccess ||
        hipMalloc(&plan->dev_buf, bytes) != hipSuccess) {
      release_tables(plan);
      return EW_ENOMEM;
    }
    size_t off = 0;
    char *h = (char *)plan->host_buf, *d = (char *)plan->dev_buf;
    for (int w = 0; w < 2; ++w)
      for (int e = 0; e < 2; ++e) {  // templates (48 B records) first keeps everything 16-byte aligned
        ew::TileTable &tt = plan->tables[w][e];
        const size_t tb = tt.templ.size() * sizeof(TileT), rb = tt.runs.size() * sizeof(RunT);
        const size_t cb = (tt.coarse.size() * sizeof(uint32_t) + 15) & ~(size_t)15;
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
    const hipError_t e = hipMemcpyAsync(plan->dev_buf, plan->host_buf, bytes, hipMemcpyHostToDevice,
                                        (hipStream_t)stream);
    if (e != hipSuccess) {
      release_tables(plan);
      return hip_fail(e, "hipMemcpyAsync(tile tables)");
    }
  }
  plan->uploaded = true;
  return EW_OK;
}

int ew_pack(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
            void *stage, uint32_t elem_size, void *stream) {
  if (!plan || !plan->uploaded || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const ew::TileTable &tt = plan->tables[0][elem_size == 4 ? 1 : 0];
  if (tt.ntiles == 0) return EW_OK;
  if (!stage) return EW_EINVAL;
  CopyTabs tabs;
  const int rc = fill_tabs(plan, old_shards, snapshots, tabs, false);
  if (rc != EW_OK) return rc;
  tabs.dst[ew::kDstStage] = (char *)stage;
  return launch_segcopy(tt, tabs, elem_size, (hipStream_t)stream);
}

int ew_unpack(const ew_plan_t *plan, const void *stage, const void *const *old_shards,
              const void *const *snapshots, void *const *new_shards, uint32_t elem_size,
              void *stream) {
  if (!plan || !plan->uploaded || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const ew::TileTable &tt = plan->tables[1][elem_size == 4 ? 1 : 0];
  if (tt.ntiles == 0) return EW_OK;
  if (!new_shards) return EW_EINVAL;
  if (plan->stage_len > 0 && !stage) return EW_EINVAL;
  CopyTabs tabs;
  const int rc = fill_tabs(plan, old_shards, snapshots, tabs, true);
  if (rc != EW_OK) return rc;
  tabs.src[ew::kSrcStage] = (const char *)stage;
  for (uint32_t k = 0; k < plan->new_dp; ++k) {
    if (plan->new_len[k] > 0 && !new_shards[k]) return EW_EINVAL;
    tabs.dst[k] = (char *)new_shards[k];
  }
  return launch_segcopy(tt, tabs, elem_size, (hipStream_t)stream);
}

int ew_unpack_snapshot(const ew_plan_t *plan, const void *stage, const void *const *old_shards,
                       const void *const *snapshots, void *const *new_shards, void *const *new_snapshots,
                       ew_cksum_t *const *new_cksums, uint32_t elem_size, void *stream_) {
  if (!plan || !plan->uploaded || (elem_size != 2 && elem_size != 4)) return EW_EINVAL;
  const int e = elem_size == 4 ? 1 : 0;
  const ew::TileTable &tt = plan->tables[1][e];
  if (tt.ntiles == 0) return EW_OK;
  if (!new_shards || !new_snapshots || !new_cksums) return EW_EINVAL;
  if (plan->stage_len > 0 && !stage) return EW_EINVAL;
  if ((uint64_t)plan->tile_elems[e] * elem_size > EW_CKSUM_BLOCK) return EW_EINVAL;  // a tile spans <= 2 blocks
  hipStream_t stream = (hipStream_t)stream_;
  CopyTabs tabs;
  const int rc = fill_tabs(plan, old_shards, snapshots, tabs, true);
  if (rc != EW_OK) return rc;
  tabs.src[ew::kSrcStage] = (const char *)stage;
  SnapTabs st;
  std::memset(&st, 0, sizeof(st));
  uint32_t max_blk = 0;
  for (uint32_t k = 0; k < plan->new_dp; ++k) {
    if (plan->new_len[k] == 0) continue;
    if (!new_shards[k] || !new_snapshots[k] || !new_cksums[k]) return EW_EINVAL;
    const uint64_t nblk = (plan->new_len[k] * elem_size + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
    if (nblk > 0xffffffffull) return EW_EINVAL;
    tabs.dst[k] = (char *)new_shards[k];
    st.snap[k] = (char *)new_snapshots[k];
    st.rec[k] = new_cksums[k];
    st.nblk[k] = (uint32_t)nblk;
    if (st.nblk[k] > max_blk) max_blk = st.nblk[k];
  }
  std::lock_guard<std::mutex> lock(g_scratch.mu);
  Region *region = nullptr;
  ew_cksum_t *slots = acquire_region(stream, &region);
  if (!slots) return EW_ENOMEM;  // only for a capturing stream that owns no region (see acquire_region)
  hipLaunchKernelGGL(ew_zero_records_kernel, dim3((2 * max_blk + kThreads - 1) / kThreads, plan->new_dp),
                     dim3(kThreads), 0, stream, st);
  EW_HIP(hipGetLastError());
  const uint32_t per_lane = 16;
  for (uint64_t t0 = 0; t0 < tt.ntiles; t0 += kRegionSlots) {
    const uint64_t n = tt.ntiles - t0 < kRegionSlots ? tt.ntiles - t0 : kRegionSlots;
    const uint64_t fold_grid = ((n + per_lane - 1) / per_lane + kThreads - 1) / kThreads;
    if (elem_size == 2) {
      hipLaunchKernelGGL(ew_unpack_snap_kernel<2>, dim3((uint32_t)n), dim3(kThreads), 0, stream, tt.dev, t0, tabs, st,
                         slots);
      EW_HIP(hipGetLastError());
      hipLaunchKernelGGL(ew_fold_tiles_kernel<2>, dim3((uint32_t)fold_grid), dim3(kThreads), 0, stream, tt.dev, t0, n,
                         per_lane, st, slots);
    } else {
      hipLaunchKernelGGL(ew_unpack_snap_kernel<4>, dim3((uint32_t)n), dim3(kThreads), 0, stream, tt.dev, t0, tabs, st,
                         slots);
      EW_HIP(hipGetLastError());
      hipLaunchKernelGGL(ew_fold_tiles_kernel<4>, dim3((uint32_t)fold_grid), dim3(kThreads), 0, stream, tt.dev, t0, n,
                         per_lane, st, slots);
    }
    EW_HIP(hipGetLastError());
  }
  release_region(region, stream);
  return EW_OK;
}

int ew_snapshot(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *cksums, void *stream) {
  if (nbytes == 0) return EW_OK;
  if (!src || !dst || !cksums) return EW_EINVAL;
  return launch_cksum<true>(src, dst, nbytes, cksums, (hipStream_t)stream);
}

int ew_verify(const void *buf, uint64_t nbytes, const ew_cksum_t *expect, ew_cksum_t *got,
              uint64_t *n_bad, uint64_t *bad_blocks, ew_cksum_t *diffs, uint64_t cap, void *stream) {
  if (!n_bad) return EW_EINVAL;
  if (nbytes > 0 && (!buf || !expect || !got)) return EW_EINVAL;
  if (cap > 0 && (!bad_blocks || !diffs)) return EW_EINVAL;
  if (nbytes > 0) {
    const int rc = launch_cksum<false>(buf, nullptr, nbytes, got, (hipStream_t)stream);
    if (rc != EW_OK) return rc;
  }
  const uint64_t nblocks = (nbytes + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
  hipLaunchKernelGGL(ew_compare_kernel, dim3(1), dim3(kCmpThreads), 0, (hipStream_t)stream, got, expect,
                     nblocks, n_bad, bad_blocks, diffs, cap);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

int ew_memcpy(const void *src, void *dst, uint64_t nbytes, void *stream) {
  if (nbytes == 0) return EW_OK;
  if (!src || !dst || (nbytes & 15u) || (((uintptr_t)src | (uintptr_t)dst) & 15u)) return EW_EINVAL;
  const uint64_t nvec = nbytes >> 4;
  const uint64_t grid = (nvec + kThreads - 1) / kThreads;
  if (grid > 0x7fffffffull) return EW_EINVAL;
  hipLaunchKernelGGL(ew_copy_kernel, dim3((uint32_t)grid), dim3(kThreads), 0, (hipStream_t)stream,
                     (const u32x4 *)src, (u32x4 *)dst, nvec);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

int ew_set_param(const char *name, int64_t value) {
  if (!name) return EW_EINVAL;
  if (!std::strcmp(name, "cksum_sub_bytes")) {
    if (value < 4096 || value > (int64_t)EW_CKSUM_BLOCK || (value & (value - 1))) return EW_EINVAL;
    g_cksum_sub_bytes = value;
  } else if (!std::strcmp(name, "cksum_wgs_per_cu")) {
    if (value < 0 || value > 64) return EW_EINVAL;
    g_cksum_wgs_per_cu = value;
  } else if (!std::strcmp(name, "cksum_mode")) {
    if (value < -1 || value > 1) return EW_EINVAL;
    g_cksum_mode = value;
  } else if (!std::strcmp(name, "tile_bytes")) {
    if (value < 256 || value > (1 << 24) || (value & 15)) return EW_EINVAL;
    g_tile_bytes = value;
  } else if (!std::strcmp(name, "tile_elems")) {
    if (value < 0 || value > (1 << 24)) return EW_EINVAL;
    g_tile_elems = value;
  } else if (!std::strcmp(name, "tile_align_bytes")) {
    if (value < 0 || value > 4096 || (value & (value - 1)) || (value && value < 16)) return EW_EINVAL;
    g_tile_align_bytes = value;
  } else {
    return EW_EINVAL;
  }
  return EW_OK;
}

int64_t ew_get_param(const char *name) {
  if (!name) return -1;
  if (!std::strcmp(name, "cksum_sub_bytes")) return g_cksum_sub_bytes;
  if (!std::strcmp(name, "cksum_wgs_per_cu")) return g_cksum_wgs_per_cu;
  if (!std::strcmp(name, "cksum_mode")) return g_cksum_mode;
  if (!std::strcmp(name, "tile_elems")) return g_tile_elems;
  if (!std::strcmp(name, "tile_bytes")) return g_tile_bytes;
  if (!std::strcmp(name, "tile_align_bytes")) return g_tile_align_bytes;
  return -1;
}

const char *ew_strerror(int code) {
  switch (code) {
    case EW_OK: return "ok";
    case EW_EINVAL: return "invalid argument";
    case EW_EUNRECOVERABLE:
      return "unrecoverable: no survivor, or a failed rank's snapshot holder (ring predecessor) failed too";
    case EW_ENOMEM: return "out of memory";
    case EW_EHIP: return g_hip_error.c_str();
    case EW_EINFEASIBLE: return "infeasible: no layer partition fits the stages' memory caps";
    default: return "unknown error code";
  }
}

const char *ew_version(void) { return "elaswave-mi355x 0.1 (gfx950)"; }

}  // extern "C"
