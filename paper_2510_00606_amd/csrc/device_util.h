// Device-side building blocks shared by the gfx950 kernels (wave64): 128-bit streaming accesses
// and the (wrapping 64-bit sum, xor) fold of the per-block checksum.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ew {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;  // four waves of 64; at one 128-bit vector per lane a workgroup moves 4 KiB
#ifndef EW_UNROLL
#define EW_UNROLL 4
#endif
constexpr int kUnroll = EW_UNROLL;  // 128-bit loads in flight per lane where a workgroup moves more than that

// Every byte here is touched exactly once per kernel, so loads and stores carry the nontemporal
// hint and do not displace the tile tables from the caches.
__device__ __forceinline__ u32x4 load16(const u32x4 *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store16(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// The streaming stores of the hot kernels go through a buffer resource, because that is the form
// whose cache-policy bits the compiler lets a kernel choose: bit 0 = sc0, bit 1 = nt, bit 4 = sc1 of
// the instruction.  Measured on MI355X on the bare one-read-one-write and one-read-two-writes patterns
// (one vector per lane, nontemporal loads), stores with sc1 set run 1.5-2 % and 2-3 % faster than
// stores with nt alone (6.49 -> 6.61 and 6.08 -> 6.25 TB/s), and plain stores 3-5 % slower: sc1 makes
// the write leave the L2 for memory at once instead of lingering there as a dirty line.  On the real
// kernels (7B stage, one process, same buffers): snapshot +2 %, unpack +1 %, plain copy +1 %, fused
// unpack + snapshot +1-1.5 %, pack -0.5 %; sc1 without nt, which is fine on the bare patterns, loses 6-8 %
// on the tile kernels.
// A window is wave-uniform: base and size live in scalar registers; lanes address it with a 32-bit
// byte offset, and the hardware drops a store that falls outside [0, nbytes).
#ifndef EW_STORE_AUX
#define EW_STORE_AUX 18  // nt + sc1
#endif
template <int AUX = EW_STORE_AUX>
struct StoreWindow {
  __amdgpu_buffer_rsrc_t rsrc;
  __device__ __forceinline__ StoreWindow(void *base, uint32_t nbytes)
      : rsrc(__builtin_amdgcn_make_buffer_rsrc(base, 0, (int)nbytes, 0x00020000)) {}
  __device__ __forceinline__ void put(uint32_t byte_off, u32x4 v) const {
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)byte_off, 0, AUX);
  }
};

// Adds the two little-endian 64-bit words of a vector to a lane's running (sum, xor).
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
  // the 64-bit form moves the two halves as a register pair (built from two 32-bit moves and an or,
  // the sum of the pair cost two 64-bit additions per step)
  return __builtin_amdgcn_update_dpp((uint64_t)0, v, CTRL, ROW_MASK, 0xf, false);
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

// Workgroup-wide fold: waves through wave_fold, then the four wave totals through LDS.  The total
// is valid in thread 0 only.  Each call needs kThreads/64 LDS cells of its own per operand, and a
// caller that reuses them (a loop) puts a barrier between the calls.
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

// Wave-uniform values wanted in scalar registers at this point of the program: the scalar loads that
// produce them (here: entries of the pointer tables in the kernel arguments) are then issued together and
// waited for once, instead of one round trip to the scalar cache each at their first use.  A workgroup
// of the tile kernels lives for a few microseconds around one vector load, and what precedes that load
// shows in the rate.  Only for use AFTER a kernel's last table load: the compiler takes the statement for
// something that may write memory, and scalar loads of global memory behind it become vector loads.
// (Pointers go in as integers; the pointers themselves keep their address space.)
template <class T0, class T1>
__device__ __forceinline__ void want_scalars(T0 a, T1 b) {
  asm volatile("" ::"s"(a), "s"(b));
}
template <class T0, class T1, class T2>
__device__ __forceinline__ void want_scalars(T0 a, T1 b, T2 c) {
  asm volatile("" ::"s"(a), "s"(b), "s"(c));
}

}  // namespace ew
