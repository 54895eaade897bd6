// Per-step snapshot copy fused with the per-block checksum (Sec. 5.1 and the online verification
// named in the abstract), its read-only form, and the ordered list of blocks whose checksum
// changed.  A block is EW_CKSUM_BLOCK = 1 MiB; its record is the wrapping sum and the xor of its
// little-endian 64-bit words, the last word zero-padded.  Both operations commute, so the bits do
// not depend on the order in which partial results meet.  HBM-bandwidth bound, no MFMA.
#include <atomic>

#include "device_util.h"
#include "runtime.h"

namespace {

using ew::block_fold;
using ew::fold;
using ew::kThreads;
using ew::kUnroll;
using ew::load16;
using ew::store16;
using ew::u32x4;

// Streaming form.  A block is cut into sub-blocks of `sub` bytes (a power of two, 4 KiB..1 MiB); a
// workgroup streams one sub-block, folding its words into (sum, xor) per lane, then across the
// workgroup.  With sub < 1 MiB the partial results of a block meet in its record through 64-bit
// atomics (the records are zeroed first).  Serves any alignment; it is the fast form for read-only
// passes and the fallback for copies.  (Dealing the sub-blocks to the XCDs in runs, which pays for the
// tile kernels and a little for the slot kernel below, changes nothing here: 6.26-6.43 TB/s for runs
// of 0-4 MiB at 64 KiB sub-blocks and four workgroups per CU.)
template <bool COPY, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void ew_cksum_kernel(const char *__restrict__ src, char *__restrict__ dst,
                                                            uint64_t nbytes, ew_cksum_t *out, uint32_t sub,
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
    block_fold(sum, xr, lds_sum, lds_xor);
    if (threadIdx.x == 0) {
      ew_cksum_t *rec = out + (begin >> 20);
      if (accumulate) {
        atomicAdd(reinterpret_cast<unsigned long long *>(&rec->sum), (unsigned long long)sum);
        atomicXor(reinterpret_cast<unsigned long long *>(&rec->xr), (unsigned long long)xr);
      } else {
        rec->sum = sum;
        rec->xr = xr;
      }
    }
    __syncthreads();  // LDS is reused by the next sub-block of a persistent workgroup
  }
}

// Fast form of the copy for 16-byte aligned buffers.  Measured on MI355X, a copy runs fastest as a
// flood of small workgroups in which every lane moves ONE 128-bit vector, and 64-bit atomics from
// many workgroups onto one checksum record serialise badly.  So: a workgroup of WAVES waves folds its
// WAVES KiB into one (sum, xor) pair and writes it to its own 16-byte slot of a scratch region (no
// atomics, no zero-fill), and ew_fold_kernel then folds the slots of every 1 MiB block into the
// block's record.  Two shapes: WAVES = 4 (the four waves meet in LDS; one slot per 4 KiB) and
// WAVES = 1 (the wave folds with DPP moves, lane 63 writes the slot: no LDS, no barrier; one slot per
// KiB).  Chunks go to the 8 XCDs in runs (xcd_remap, knob snapshot_xcd_group_kib).  Measured on
// 0.875 GB buffers, calls back to back, TB/s read + written: chunks dealt out one by one 6.58 (one
// wave) and 6.52 (four waves); runs of 128 KiB 6.60 and 6.63, runs of 16-32 KiB 6.0, runs of 8 MiB
// 6.05-6.3.  Four waves with runs of 128 KiB is the default for every size (+0.5 % at 0.875 GB, +1.5 %
// at 0.44 and 1 GB, +1 % at 100 MiB over one wave dealt one by one, and a quarter of the slots).
template <bool COPY, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void ew_cksum_slots_kernel(const u32x4 *__restrict__ src,
                                                                    u32x4 *__restrict__ dst, uint64_t nbytes,
                                                                    ew_cksum_t *__restrict__ slots, ew::XcdMap xcd) {
  static_assert(WAVES == 1 || 64 * WAVES == kThreads, "block_fold is written for kThreads lanes");
  const uint64_t chunk = ew::xcd_remap(blockIdx.x, xcd);  // which WAVES KiB of the buffer
  const uint64_t first = chunk * (64 * WAVES);  // the workgroup's first vector
  const uint64_t i = first + threadIdx.x;
  const uint64_t nvec = nbytes >> 4;
  uint64_t sum = 0, xr = 0;
  if (i < nvec) {
    const u32x4 v = load16(src + i);
    if (COPY) {
      const uint64_t left = nvec - first;
      const ew::StoreWindow<> out(dst + first, (uint32_t)(left < 64 * WAVES ? left : 64 * WAVES) << 4);
      out.put(threadIdx.x << 4, v);
    }
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
  if (WAVES == 1) {
    ew::wave_fold(sum, xr);
    if (threadIdx.x != ew::kWaveFoldLane) return;
  } else {
    __shared__ uint64_t lds_sum[WAVES];
    __shared__ uint64_t lds_xor[WAVES];
    block_fold(sum, xr, lds_sum, lds_xor);
    if (threadIdx.x != 0) return;
  }
  ew_cksum_t r;
  r.sum = sum;
  r.xr = xr;
  slots[chunk] = r;
}

// One workgroup per checksum block: folds the block's slots (per_block for a full block) into out[b].
__global__ __launch_bounds__(kThreads) void ew_fold_kernel(const ew_cksum_t *__restrict__ slots, uint64_t nslots,
                                                           uint32_t per_block, ew_cksum_t *__restrict__ out) {
  __shared__ uint64_t lds_sum[kThreads / 64];
  __shared__ uint64_t lds_xor[kThreads / 64];
  uint64_t sum = 0, xr = 0;
  for (uint32_t t = threadIdx.x; t < per_block; t += kThreads) {
    const uint64_t sidx = (uint64_t)blockIdx.x * per_block + t;
    if (sidx < nslots) {
      const ew_cksum_t r = slots[sidx];
      sum += r.sum;
      xr ^= r.xr;
    }
  }
  block_fold(sum, xr, lds_sum, lds_xor);
  if (threadIdx.x == 0) {
    ew_cksum_t r;
    r.sum = sum;
    r.xr = xr;
    out[blockIdx.x] = r;
  }
}

// Single workgroup: ascending list of differing blocks (stable compaction with ballots), with the
// (sum difference, xor difference) of each; *n_bad counts all of them, also those beyond cap.
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

template <bool COPY>
int launch_cksum_streaming(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *out, hipStream_t stream) {
  const ew::Knobs &k = ew::knobs();
  // A read-only pass over a large buffer runs as fewer, longer streams (see Knobs::verify_large_*).
  const bool large = !COPY && nbytes >= (uint64_t)k.verify_large_min_bytes;
  const int64_t resident = large ? k.verify_large_wgs_per_cu : k.verify_wgs_per_cu;
  uint32_t sub = (uint32_t)(large ? k.verify_large_sub_bytes : k.cksum_sub_bytes);
  if (large && resident > 0) {
    // the largest sub-block, down to 128 KiB, that still gives every resident workgroup five sub-blocks:
    // with three rounds or fewer the last, partly filled round shows (0.875 GB: 6.54 TB/s at 256 KiB, 6.16 at
    // 512 KiB; 0.44 GB: 6.03 at 128 KiB, 5.78 at 256 KiB)
    const uint64_t want = 5ull * (uint64_t)resident * (uint64_t)ew::num_cus();
    while (sub > 131072u && nbytes / sub < want) sub >>= 1;
  }
  const uint64_t nblocks = (nbytes + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
  const uint32_t accumulate = sub < EW_CKSUM_BLOCK ? 1u : 0u;
  if (accumulate) {
    const int rc = ew::launch_zero(out, nblocks * sizeof(ew_cksum_t), stream);
    if (rc != EW_OK) return rc;
  }
  uint64_t grid = (nbytes + sub - 1) / sub;
  if (k.cksum_wgs_per_cu > 0) {
    const uint64_t cap = (uint64_t)ew::num_cus() * (uint64_t)k.cksum_wgs_per_cu;
    if (grid > cap) grid = cap;
  }
  if (grid > 0x7fffffffull) grid = 0x7fffffffull;  // the kernel strides over what is left
  const bool aligned = ((((uintptr_t)src) | (COPY ? (uintptr_t)dst : 0)) & 15u) == 0;
  // A read-only pass runs faster with fewer of these workgroups resident per CU than the eight that fit
  // (four for small buffers: 6.33 -> 6.50 TB/s measured in one process; two for large ones); the copying
  // form wants all eight.
  const uint32_t lds_pad = COPY ? 0u : ew::occupancy_pad(resident, 4 * sizeof(uint64_t) * (kThreads / 64));
  if (aligned)
    hipLaunchKernelGGL((ew_cksum_kernel<COPY, true>), dim3((uint32_t)grid), dim3(kThreads), lds_pad, stream,
                       (const char *)src, (char *)dst, nbytes, out, sub, accumulate);
  else
    hipLaunchKernelGGL((ew_cksum_kernel<COPY, false>), dim3((uint32_t)grid), dim3(kThreads), lds_pad, stream,
                       (const char *)src, (char *)dst, nbytes, out, sub, accumulate);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

// Slot kernel + fold kernel over `slots` (room for max_slots of them), in as many passes as that takes.
template <bool COPY>
int launch_cksum_slots(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *out, ew_cksum_t *slots,
                       uint64_t max_slots, hipStream_t stream) {
  // one slot per KiB (one-wave workgroups) from snapshot_wave_min_bytes on, one per 4 KiB below
  const bool one_wave = nbytes >= (uint64_t)ew::knobs().snapshot_wave_min_bytes;
  const uint64_t slot_bytes = one_wave ? 1024 : 4096;
  const uint64_t pass_bytes = max_slots * slot_bytes;  // what the slots cover; a multiple of 1 MiB
  const uint64_t group_kib = (uint64_t)ew::knobs().snapshot_xcd_group_kib;
  const uint32_t xcd_group = group_kib ? (uint32_t)(group_kib * 1024 / slot_bytes) : 1u;
  for (uint64_t off = 0; off < nbytes; off += pass_bytes) {
    const uint64_t n = nbytes - off < pass_bytes ? nbytes - off : pass_bytes;
    // a partial trailing vector belongs to lane n/16, which the last workgroup always contains because
    // ceil(n/slot_bytes) * slot_bytes/16 > n/16 whenever 16 does not divide n
    const uint64_t grid = (n + slot_bytes - 1) / slot_bytes;
    const uint64_t nblk = (n + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
    const u32x4 *s = (const u32x4 *)((const char *)src + off);
    u32x4 *d = (u32x4 *)(COPY ? (char *)dst + off : nullptr);
    if (one_wave)
      hipLaunchKernelGGL((ew_cksum_slots_kernel<COPY, 1>), dim3((uint32_t)grid), dim3(64), 0, stream, s, d, n, slots,
                         ew::make_xcd_map(xcd_group, (uint32_t)grid));
    else
      hipLaunchKernelGGL((ew_cksum_slots_kernel<COPY, 4>), dim3((uint32_t)grid), dim3(256), 0, stream, s, d, n, slots,
                         ew::make_xcd_map(xcd_group, (uint32_t)grid));
    EW_HIP(hipGetLastError());
    hipLaunchKernelGGL(ew_fold_kernel, dim3((uint32_t)nblk), dim3(kThreads), 0, stream, slots, grid,
                       (uint32_t)(EW_CKSUM_BLOCK / slot_bytes), out + off / EW_CKSUM_BLOCK);
    EW_HIP(hipGetLastError());
  }
  return EW_OK;
}

template <bool COPY>
int launch_cksum(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *out, hipStream_t stream) {
  const bool aligned = ((((uintptr_t)src) | (COPY ? (uintptr_t)dst : 0)) & 15u) == 0;
  // Read-only passes (verify) keep the streaming kernel: with no stores for the fold to hide behind,
  // one slot per 4 KiB is the slower shape for them (4.4 TB/s), and a read-only slot kernel with 2, 4 or 8
  // vectors in flight per lane (one slot per 8-32 KiB) reaches 6.31-6.39 TB/s per call where the streaming
  // kernel in its shape for large buffers gives 6.47.
  const int64_t knob = ew::knobs().cksum_mode;
  const int64_t mode = knob >= 0 ? knob : (COPY ? 0 : 1);
  if (!aligned || mode != 0) return launch_cksum_streaming<COPY>(src, dst, nbytes, out, stream);
  // the lease keeps other calls off the region until this call's last kernel has been enqueued
  ew::ScratchLease lease(stream);
  ew_cksum_t *slots = lease.slots();
  if (!slots) return launch_cksum_streaming<COPY>(src, dst, nbytes, out, stream);  // needs no scratch
  return launch_cksum_slots<COPY>(src, dst, nbytes, out, slots, ew::kRegionSlots, stream);
}

// ---- the allocation-free entry point's own scratch ----------------------------------------------
// A fixed array of checksum slots for ew_snapshot_noalloc, apart from the leased regions above: no
// lease, no event, no lock.  In host code the array's name only stands for the symbol; the memory is
// reached through the per-device address that hipGetSymbolAddress returned for it.
constexpr uint64_t kNoAllocSlots = EW_NOALLOC_MAX_BYTES / 1024;  // one slot per KiB: 16 MiB of slots
static __device__ __align__(256) ew_cksum_t scratch[kNoAllocSlots];
constexpr int kNoAllocMaxDevices = 64;
std::atomic<ew_cksum_t *> g_noalloc_ptr[kNoAllocMaxDevices];  // zero-initialised; a race only repeats the query

// Address of the current device's copy of `scratch`, looked up on the first call on that device.
int noalloc_scratch(ew_cksum_t **out) {
  int dev = -1;
  EW_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kNoAllocMaxDevices) return EW_EINVAL;
  ew_cksum_t *p = g_noalloc_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void *q = nullptr;
    EW_HIP(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
    if (!q) return ew::hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch) returned no address");
    p = (ew_cksum_t *)q;
    g_noalloc_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return EW_OK;
}

}  // namespace

extern "C" {

int ew_snapshot_noalloc(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *cksums, void *stream) {
  if (nbytes == 0) return EW_OK;
  if (!src || !dst || !cksums) return EW_EINVAL;
  if (nbytes > EW_NOALLOC_MAX_BYTES) return EW_ETOOBIG;
  if ((((uintptr_t)src | (uintptr_t)dst) & 15u) != 0)  // the streaming kernel needs no scratch at all
    return launch_cksum_streaming<true>(src, dst, nbytes, cksums, (hipStream_t)stream);
  ew_cksum_t *slots = nullptr;
  const int rc = noalloc_scratch(&slots);
  if (rc != EW_OK) return rc;
  // Every slot the fold kernel reads was written by this call's slot kernel, so what earlier calls
  // left in the array never needs clearing.
  return launch_cksum_slots<true>(src, dst, nbytes, cksums, slots, kNoAllocSlots, (hipStream_t)stream);
}

int ew_snapshot(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *cksums, void *stream) {
  if (nbytes == 0) return EW_OK;
  if (!src || !dst || !cksums) return EW_EINVAL;
  return launch_cksum<true>(src, dst, nbytes, cksums, (hipStream_t)stream);
}

int ew_verify(const void *buf, uint64_t nbytes, const ew_cksum_t *expect, ew_cksum_t *got, uint64_t *n_bad,
              uint64_t *bad_blocks, ew_cksum_t *diffs, uint64_t cap, void *stream) {
  if (!n_bad) return EW_EINVAL;
  if (nbytes > 0 && (!buf || !expect || !got)) return EW_EINVAL;
  if (cap > 0 && (!bad_blocks || !diffs)) return EW_EINVAL;
  if (nbytes > 0) {
    const int rc = launch_cksum<false>(buf, nullptr, nbytes, got, (hipStream_t)stream);
    if (rc != EW_OK) return rc;
  }
  const uint64_t nblocks = (nbytes + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
  hipLaunchKernelGGL(ew_compare_kernel, dim3(1), dim3(kCmpThreads), 0, (hipStream_t)stream, got, expect, nblocks,
                     n_bad, bad_blocks, diffs, cap);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

}  // extern "C"
