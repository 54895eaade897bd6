// Host-side state shared by the translation units that launch kernels: HIP error capture, the
// process-wide launch-shape knobs, the fixed scratch array for per-workgroup checksum slots, and
// the pointer tables handed to the copy kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <mutex>

#include "plan_internal.h"

namespace ew {

// Records the failing call's message for ew_strerror(EW_EHIP) (per host thread); returns EW_EHIP.
int hip_fail(hipError_t e, const char *what);
const char *last_hip_error();

#define EW_HIP(call)                                        \
  do {                                                      \
    hipError_t e__ = (call);                                \
    if (e__ != hipSuccess) return ::ew::hip_fail(e__, #call); \
  } while (0)

// Launch-shape knobs behind ew_set_param / ew_get_param.  Each is an atomic of its own, so a launch
// on one host thread may read them while another thread sets one; a call reads every knob it needs
// once, so it never sees two values of the same knob.
typedef std::atomic<int64_t> Knob;
struct Knobs {
  Knob cksum_sub_bytes{65536};  // streaming checksum kernel: bytes of a block per workgroup pass
  Knob cksum_wgs_per_cu{0};     // streaming checksum kernel: 0 = one workgroup per sub-block,
                                // else a persistent grid of this many workgroups per CU
  Knob cksum_mode{-1};          // -1 = slot kernel + fold for snapshot, streaming kernel for verify;
                                // 0 / 1 force the slot / streaming kernel for both
  Knob snapshot_wave_min_bytes{(int64_t)1 << 62};  // snapshot: one-wave workgroups from this size on, 256 lanes below
                                                    // (default: never; see ew_cksum_slots_kernel)
  Knob snapshot_xcd_group_kib{128};  // snapshot slot kernel: KiB of consecutive chunks per XCD (0 = one by one)
  Knob tile_bytes{4096};        // default copy tile: 256 lanes x one 128-bit vector
  Knob tile_elems{0};           // > 0 overrides tile_bytes with a size in elements
  Knob tile_align_bytes{128};   // tile cuts fall on multiples of this in the destination (0: off)
  Knob xcd_group_kib{2048};     // KiB of consecutive tiles that one XCD takes (see xcd_remap); 0 = identity
  // Caps on the workgroups resident per CU (0 = all that fit) for the kernels that run faster with
  // fewer requests in flight.
  Knob fused_wgs_per_cu{0};     // fused unpack + snapshot (256 lanes; 8 fit): no cap since tiles go to XCDs in
                                // runs (with the identity mapping six per CU were 1-5 % faster than eight)
  Knob fold_tiles_per_lane{0};  // fused unpack + snapshot: tiles per lane of the fold kernel (0 = default)
  Knob fused_pass_tiles{262144};  // fused unpack + snapshot: at most this many tiles per launch of the tile kernel
                                  // (0 = what the scratch region holds); the fold follows once per region
  Knob fused_mode{0};           // fused unpack + snapshot: 0 = slot per tile + fold kernel, 1 = scratch-free (atomics)
  Knob verify_wgs_per_cu{4};    // read-only streaming checksum (256 lanes; 8 fit)
  // Read-only passes over large buffers run faster as fewer, longer streams: from verify_large_min_bytes on
  // they use verify_large_wgs_per_cu workgroups per CU and sub-blocks of up to verify_large_sub_bytes (halved,
  // down to 128 KiB, until every resident workgroup gets five of them) instead of verify_wgs_per_cu and
  // cksum_sub_bytes.  Per call on arrays of 0.44 / 0.875 / 1.75 GB: 5.94 / 6.35 / 6.57 TB/s in the small shape,
  // 6.03 / 6.54 / 6.81 in the large one; at 0.22 GB and below the small shape is equal or better.
  Knob verify_large_min_bytes{(int64_t)256 << 20};
  Knob verify_large_sub_bytes{524288};
  Knob verify_large_wgs_per_cu{2};
  Knob adam_xcd_group{256};     // optimizer step: consecutive workgroups (256 elements each) per XCD; 1 = one by one
  Knob adam_wgs_per_cu{10};     // optimizer step (one wave per workgroup; 32 fit)
};
Knobs &knobs();

int num_cus();

// The group argument of make_xcd_map for a kernel whose workgroups each cover unit_bytes of the
// destination (knob xcd_group_kib; 1 = identity).
uint32_t xcd_group_for(uint64_t unit_bytes);

// Dynamic LDS bytes that, requested per workgroup of a kernel with `static_lds` bytes of its own,
// leave room for exactly `wgs_per_cu` workgroups on a CU of the current device; 0 when no cap is
// wanted (wgs_per_cu <= 0) or none can be guaranteed.  Occupancy is capped with LDS nobody uses
// because nothing else limits it for these kernels (few registers, hardly any LDS).
uint32_t occupancy_pad(int64_t wgs_per_cu, uint32_t static_lds);

// Zero-fill by kernel (safe to record into a HIP graph); nbytes is a multiple of 8.
int launch_zero(void *p, uint64_t nbytes, hipStream_t stream);

// ---- scratch for per-workgroup checksum slots ---------------------------------------------------
// A fixed device array, so taking a snapshot never allocates.  It is cut into regions; a stream
// keeps the region it used last.  When a stream without a region asks for one and all are taken,
// the least recently used region changes hands, and the new owner's stream is first made to wait
// (hipStreamWaitEvent, no host blocking) for the event recorded after the region's last use, so
// two streams never touch a region at once.  A stream under graph capture can only use a region it
// already owns or one nobody has used yet; such a region stays with that stream (replays of the
// graph use it unseen) until ew_scratch_release says the graphs are gone, and one region per device
// always stays outside graphs so that eager calls on other streams keep working: the capture that
// would take the last one gets no region and its caller takes the scratch-free kernel instead.
// One region (32 MiB) holds 2^21 slots: 2 GiB of input for the snapshot kernel (one slot per wave and
// KiB), 2^21 tiles for the fused unpack (one slot per tile); longer inputs take several passes.
//
// Locking: one mutex per device, held only while a region is picked and while its hand-over event is
// recorded, never while kernels are enqueued.  A region is marked busy in between, so two host
// threads that share a stream get two regions (their kernel pairs may then interleave on the stream
// without touching each other's slots), and calls on different streams or devices enqueue at the
// same time.
constexpr uint32_t kRegions = 4;
constexpr uint64_t kRegionSlots = 1ull << 21;
struct Region;
struct DeviceScratch;
// A call's hold on a region.  The constructor picks a region for `stream` and marks it busy; the
// destructor (also on an early error return) records the event that later hand-overs wait for and
// clears the mark.  slots() is the region's device address, nullptr when none can be had (a stream
// under capture as described above, or a failing HIP call).
class ScratchLease {
 public:
  explicit ScratchLease(hipStream_t stream);
  ~ScratchLease();
  ScratchLease(const ScratchLease &) = delete;
  ScratchLease &operator=(const ScratchLease &) = delete;
  ew_cksum_t *slots() const { return slots_; }

 private:
  hipStream_t stream_;
  DeviceScratch *dev_ = nullptr;
  Region *region_ = nullptr;
  ew_cksum_t *slots_ = nullptr;
  bool capturing_ = false;
};

// The most leases ever held at once in this process (optionally reset to 0), and the call behind
// ew_scratch_release.
int64_t scratch_max_concurrent(bool reset);
int scratch_release(hipStream_t stream);

// ---- pointer tables of the tile-driven kernels, passed by value ----------------------------------
struct CopyTabs {
  const char *src[kNumSrc];
  char *dst[kNumDst];
};
// True if the plan's tables are uploaded and live on the current device.
bool tables_usable(const ew_plan_t *plan);
// Fills the live-shard and snapshot sources; EW_EINVAL if the plan reads a buffer that is null.
int fill_tabs(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots, CopyTabs &tabs);

}  // namespace ew
