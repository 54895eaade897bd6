// Host-side runtime shared by the kernel files: HIP error capture, launch-shape knobs, the scratch
// regions for per-workgroup checksum slots, and the small C-ABI calls that touch no kernel
// (ew_set_param, ew_get_param, ew_strerror, ew_version).
#include "runtime.h"

#include <atomic>
#include <condition_variable>
#include <cstring>
#include <string>

#include "device_util.h"

namespace ew {

namespace {

thread_local std::string g_hip_error = "no HIP error recorded";
Knobs g_knobs;

__global__ __launch_bounds__(kThreads) void ew_zero_kernel(uint64_t *p, uint64_t nwords) {
  const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < nwords) p[i] = 0;
}

// The slots of all regions.  In host code this name is only a handle for hipGetSymbolAddress; every
// use of the memory goes through the per-device address obtained there.
__device__ __align__(256) ew_cksum_t g_slot_scratch[kRegions * kRegionSlots];

constexpr int kMaxDevices = 64;

}  // namespace

struct Region {
  hipStream_t owner = nullptr;
  bool taken = false;
  bool busy = false;          // a host thread is between picking it and recording its event
  hipEvent_t done = nullptr;  // recorded on the owner's stream after each use
  bool recorded = false;
  bool in_graph = false;  // some captured graph uses it: its replays are invisible here, so it does not change hands
  uint64_t last_use = 0;
};

struct DeviceScratch {
  std::mutex mu;
  std::condition_variable freed;  // a busy region was given back
  ew_cksum_t *base = nullptr;     // address of this device's copy of the array
  Region region[kRegions];
  uint64_t clock = 0;
};

namespace {

DeviceScratch g_scratch[kMaxDevices];
// leases held right now over all devices, and the most ever held at once (ew_get_param
// "scratch_max_concurrent"): shows that calls on different streams enqueue side by side
std::atomic<int64_t> g_leases{0}, g_leases_max{0};

bool stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st != hipStreamCaptureStatusNone;
}

}  // namespace

int hip_fail(hipError_t e, const char *what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();  // reported here: the runtime's own record of it must not surface in a later call
  return EW_EHIP;
}

const char *last_hip_error() { return g_hip_error.c_str(); }

Knobs &knobs() { return g_knobs; }

int num_cus() {
  static std::atomic<int> cached[kMaxDevices];  // zero-initialised; a race only repeats the query
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return 256;
    n = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

uint32_t xcd_group_for(uint64_t unit_bytes) {
  const uint64_t kib = (uint64_t)g_knobs.xcd_group_kib.load();
  if (kib == 0 || unit_bytes == 0) return 1;
  const uint64_t g = kib * 1024 / unit_bytes;
  return g < 1 ? 1u : (g > (1u << 24) ? (1u << 24) : (uint32_t)g);
}

uint32_t occupancy_pad(int64_t wgs_per_cu, uint32_t static_lds) {
  if (wgs_per_cu <= 0 || wgs_per_cu > 64) return 0;
  static std::atomic<int> cached[kMaxDevices];  // LDS bytes per CU
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
  int lds = cached[dev].load(std::memory_order_relaxed);
  if (lds == 0) {
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess || lds <= 0) {
      (void)hipGetLastError();
      return 0;
    }
    cached[dev].store(lds, std::memory_order_relaxed);
  }
  // n workgroups fit and n + 1 do not when a workgroup's LDS lies between usable/(n+1) and usable/n.
  // Neither the usable size (measured on gfx950: a little under the 160 KiB reported) nor the
  // allocation granule is documented, so the request aims at the middle of that interval; a workgroup
  // may ask for at most 64 KiB in all.
  const int64_t n = wgs_per_cu, usable = (int64_t)lds - 4096, kMaxPerWorkgroup = 65536;
  const int64_t lo = usable / (n + 1), hi = usable / n;
  int64_t total = (lo + hi) / 2;
  if (total > kMaxPerWorkgroup) total = kMaxPerWorkgroup;
  const int64_t pad = (total - (int64_t)static_lds) & ~(int64_t)255;
  if (pad <= 0 || pad + (int64_t)static_lds <= lo + 256) return 0;  // no safe request: no cap
  return (uint32_t)pad;
}

int launch_zero(void *p, uint64_t nbytes, hipStream_t stream) {
  const uint64_t nwords = nbytes / 8;
  if (nwords == 0) return EW_OK;
  const uint64_t grid = (nwords + kThreads - 1) / kThreads;
  if (grid > 0x7fffffffull) return EW_EINVAL;
  hipLaunchKernelGGL(ew_zero_kernel, dim3((uint32_t)grid), dim3(kThreads), 0, stream, (uint64_t *)p, nwords);
  EW_HIP(hipGetLastError());
  return EW_OK;
}

ScratchLease::ScratchLease(hipStream_t stream) : stream_(stream) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return;
  }
  DeviceScratch &ds = g_scratch[dev];
  std::unique_lock<std::mutex> lock(ds.mu);
  if (!ds.base) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_slot_scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return;
    }
    ds.base = (ew_cksum_t *)p;
  }
  capturing_ = stream_is_capturing(stream);
  // hipStreamPerThread names a different stream in every host thread, so it never owns a region:
  // each of its calls goes through the event-ordered hand-over below
  const bool ownable = stream != hipStreamPerThread;
  Region *reg = ds.region;
  int pick = -1;
  for (;;) {
    for (uint32_t r = 0; r < kRegions && pick < 0 && ownable; ++r)
      if (reg[r].taken && !reg[r].busy && reg[r].owner == stream) pick = (int)r;
    for (uint32_t r = 0; r < kRegions && pick < 0; ++r)
      if (!reg[r].taken) pick = (int)r;
    if (pick >= 0) break;
    if (capturing_) return;  // a capture cannot be ordered after work outside it
    bool any_busy = false;
    for (uint32_t r = 0; r < kRegions; ++r) {
      if (reg[r].in_graph) continue;
      if (reg[r].busy) {
        any_busy = true;
        continue;
      }
      if (pick < 0 || reg[r].last_use < reg[pick].last_use) pick = (int)r;
    }
    if (pick >= 0) {
      // its last user was another stream (or this one's other region): wait for that use on the device
      if (reg[pick].recorded && hipStreamWaitEvent(stream, reg[pick].done, 0) != hipSuccess) {
        (void)hipGetLastError();
        return;
      }
      break;
    }
    if (!any_busy) return;  // cannot happen: one region always stays outside graphs
    ds.freed.wait(lock);    // every candidate is in another thread's hands for a few microseconds
  }
  if (capturing_ && !reg[pick].in_graph) {
    // this use would tie the region to a graph: refuse if it is the last one outside graphs
    uint32_t others_free = 0;
    for (uint32_t r = 0; r < kRegions; ++r)
      if ((int)r != pick && !reg[r].in_graph) ++others_free;
    if (others_free == 0) return;
  }
  // marked here, under the lock that the test above ran under, so two captures that start at the same
  // time cannot both take a "last but one" region; the graph's own ordering covers its replays
  if (capturing_) reg[pick].in_graph = true;
  reg[pick].taken = true;
  reg[pick].busy = true;
  reg[pick].owner = stream;
  dev_ = &ds;
  region_ = &reg[pick];
  slots_ = ds.base + (uint64_t)pick * kRegionSlots;
  const int64_t now = g_leases.fetch_add(1, std::memory_order_relaxed) + 1;
  int64_t seen = g_leases_max.load(std::memory_order_relaxed);
  while (now > seen && !g_leases_max.compare_exchange_weak(seen, now, std::memory_order_relaxed)) {
  }
}

// Runs after the last kernel of the call has been enqueued.
ScratchLease::~ScratchLease() {
  if (!region_) return;
  Region *r = region_;
  hipEvent_t ev = nullptr;
  bool recorded = false;
  if (!capturing_) {
    // the event is only ever touched by the thread that holds the busy mark
    ev = r->done;
    if (!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      ev = nullptr;
    }
    recorded = ev && hipEventRecord(ev, stream_) == hipSuccess;
    if (!recorded) {
      // no event to hand the region over with: leave it idle instead
      (void)hipGetLastError();
      (void)hipStreamSynchronize(stream_);
    }
  }
  {
    std::lock_guard<std::mutex> lock(dev_->mu);
    r->last_use = ++dev_->clock;
    if (!capturing_) {
      r->done = ev;
      r->recorded = recorded;
    }
    r->busy = false;
  }
  g_leases.fetch_sub(1, std::memory_order_relaxed);
  dev_->freed.notify_all();
}

int64_t scratch_max_concurrent(bool reset) {
  return reset ? g_leases_max.exchange(0, std::memory_order_relaxed) : g_leases_max.load(std::memory_order_relaxed);
}

int scratch_release(hipStream_t stream) {
  int dev = 0;
  EW_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return EW_EINVAL;
  DeviceScratch &ds = g_scratch[dev];
  std::lock_guard<std::mutex> lock(ds.mu);
  for (uint32_t r = 0; r < kRegions; ++r)
    if (ds.region[r].taken && ds.region[r].owner == stream && !ds.region[r].busy) ds.region[r].in_graph = false;
  return EW_OK;
}

bool tables_usable(const ew_plan_t *plan) {
  if (!plan || !plan->uploaded) return false;
  if (plan->device < 0) return true;  // nothing was uploaded: all tables are empty
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return dev == plan->device;
}

int fill_tabs(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots, CopyTabs &tabs) {
  std::memset(&tabs, 0, sizeof(tabs));
  for (uint32_t j = 0; j < plan->old_dp; ++j) {
    const void *live = old_shards ? old_shards[j] : nullptr;
    const void *snap = snapshots ? snapshots[j] : nullptr;
    if (((plan->live_read >> j) & 1) && !live) return EW_EINVAL;
    if (((plan->snap_read >> j) & 1) && !snap) return EW_EINVAL;
    tabs.src[kSrcLive + j] = (const char *)live;
    tabs.src[kSrcSnap + j] = (const char *)snap;
  }
  return EW_OK;
}

}  // namespace ew

extern "C" {

int ew_set_param(const char *name, int64_t value) {
  if (!name) return EW_EINVAL;
  ew::Knobs &k = ew::knobs();
  if (!std::strcmp(name, "cksum_sub_bytes")) {
    if (value < 4096 || value > (int64_t)EW_CKSUM_BLOCK || (value & (value - 1))) return EW_EINVAL;
    k.cksum_sub_bytes = value;
  } else if (!std::strcmp(name, "cksum_wgs_per_cu")) {
    if (value < 0 || value > 64) return EW_EINVAL;
    k.cksum_wgs_per_cu = value;
  } else if (!std::strcmp(name, "snapshot_wave_min_bytes")) {
    if (value < 0) return EW_EINVAL;
    k.snapshot_wave_min_bytes = value;
  } else if (!std::strcmp(name, "cksum_mode")) {
    if (value < -1 || value > 1) return EW_EINVAL;
    k.cksum_mode = value;
  } else if (!std::strcmp(name, "tile_bytes")) {
    if (value < 256 || value > (1 << 24) || (value & 15)) return EW_EINVAL;
    k.tile_bytes = value;
  } else if (!std::strcmp(name, "tile_elems")) {
    if (value < 0 || value > (1 << 24)) return EW_EINVAL;
    k.tile_elems = value;
  } else if (!std::strcmp(name, "fused_wgs_per_cu")) {
    if (value < 0 || value > 8) return EW_EINVAL;
    k.fused_wgs_per_cu = value;
  } else if (!std::strcmp(name, "snapshot_xcd_group_kib")) {
    if (value < 0 || value > (1 << 20)) return EW_EINVAL;
    k.snapshot_xcd_group_kib = value;
  } else if (!std::strcmp(name, "adam_xcd_group")) {
    if (value < 1 || value > (1 << 24)) return EW_EINVAL;
    k.adam_xcd_group = value;
  } else if (!std::strcmp(name, "xcd_group_kib")) {
    if (value < 0 || value > (1 << 20)) return EW_EINVAL;
    k.xcd_group_kib = value;
  } else if (!std::strcmp(name, "fold_tiles_per_lane")) {
    if (value < 0 || value > 1024) return EW_EINVAL;
    k.fold_tiles_per_lane = value;
  } else if (!std::strcmp(name, "fused_pass_tiles")) {
    if (value < 0 || value > 0x7fffffff) return EW_EINVAL;
    k.fused_pass_tiles = value;
  } else if (!std::strcmp(name, "fused_mode")) {
    if (value < 0 || value > 1) return EW_EINVAL;
    k.fused_mode = value;
  } else if (!std::strcmp(name, "verify_wgs_per_cu")) {
    if (value < 0 || value > 8) return EW_EINVAL;
    k.verify_wgs_per_cu = value;
  } else if (!std::strcmp(name, "verify_large_min_bytes")) {
    if (value < 0) return EW_EINVAL;
    k.verify_large_min_bytes = value;
  } else if (!std::strcmp(name, "verify_large_sub_bytes")) {
    if (value < 4096 || value > (int64_t)EW_CKSUM_BLOCK || (value & (value - 1))) return EW_EINVAL;
    k.verify_large_sub_bytes = value;
  } else if (!std::strcmp(name, "verify_large_wgs_per_cu")) {
    if (value < 0 || value > 8) return EW_EINVAL;
    k.verify_large_wgs_per_cu = value;
  } else if (!std::strcmp(name, "adam_wgs_per_cu")) {
    if (value < 0 || value > 32) return EW_EINVAL;
    k.adam_wgs_per_cu = value;
  } else if (!std::strcmp(name, "tile_align_bytes")) {
    if (value < 0 || value > 4096 || (value & (value - 1)) || (value && value < 16)) return EW_EINVAL;
    k.tile_align_bytes = value;
  } else if (!std::strcmp(name, "scratch_max_concurrent")) {
    if (value != 0) return EW_EINVAL;  // a statistic: it can only be reset
    (void)ew::scratch_max_concurrent(true);
  } else {
    return EW_EINVAL;
  }
  return EW_OK;
}

int64_t ew_get_param(const char *name) {
  if (!name) return -1;
  const ew::Knobs &k = ew::knobs();
  if (!std::strcmp(name, "cksum_sub_bytes")) return k.cksum_sub_bytes;
  if (!std::strcmp(name, "cksum_wgs_per_cu")) return k.cksum_wgs_per_cu;
  if (!std::strcmp(name, "cksum_mode")) return k.cksum_mode;
  if (!std::strcmp(name, "snapshot_wave_min_bytes")) return k.snapshot_wave_min_bytes;
  if (!std::strcmp(name, "tile_elems")) return k.tile_elems;
  if (!std::strcmp(name, "tile_bytes")) return k.tile_bytes;
  if (!std::strcmp(name, "tile_align_bytes")) return k.tile_align_bytes;
  if (!std::strcmp(name, "fused_wgs_per_cu")) return k.fused_wgs_per_cu;
  if (!std::strcmp(name, "xcd_group_kib")) return k.xcd_group_kib;
  if (!std::strcmp(name, "adam_xcd_group")) return k.adam_xcd_group;
  if (!std::strcmp(name, "snapshot_xcd_group_kib")) return k.snapshot_xcd_group_kib;
  if (!std::strcmp(name, "fold_tiles_per_lane")) return k.fold_tiles_per_lane;
  if (!std::strcmp(name, "fused_pass_tiles")) return k.fused_pass_tiles;
  if (!std::strcmp(name, "fused_mode")) return k.fused_mode;
  if (!std::strcmp(name, "verify_wgs_per_cu")) return k.verify_wgs_per_cu;
  if (!std::strcmp(name, "verify_large_min_bytes")) return k.verify_large_min_bytes;
  if (!std::strcmp(name, "verify_large_sub_bytes")) return k.verify_large_sub_bytes;
  if (!std::strcmp(name, "verify_large_wgs_per_cu")) return k.verify_large_wgs_per_cu;
  if (!std::strcmp(name, "adam_wgs_per_cu")) return k.adam_wgs_per_cu;
  if (!std::strcmp(name, "scratch_max_concurrent")) return ew::scratch_max_concurrent(false);
  return -1;
}

int ew_scratch_release(void *stream) { return ew::scratch_release((hipStream_t)stream); }

int ew_single_bit_flip(const ew_cksum_t *diff, uint32_t *lane, int32_t *direction) {
  if (!diff || !lane || !direction) return 0;
  const uint64_t x = diff->xr;
  if (x == 0 || (x & (x - 1)) != 0) return 0;  // not one-hot
  int32_t dir;
  if (diff->sum == x)
    dir = 1;
  else if (diff->sum == (uint64_t)0 - x)
    dir = -1;  // (bit 63: +x and -x coincide and read as +1)
  else
    return 0;
  *lane = (uint32_t)__builtin_ctzll(x);
  *direction = dir;
  return 1;
}

const char *ew_strerror(int code) {
  switch (code) {
    case EW_OK: return "ok";
    case EW_EINVAL: return "invalid argument";
    case EW_EUNRECOVERABLE:
      return "unrecoverable: no survivor, or a failed rank's snapshot holder (ring predecessor) failed too";
    case EW_ENOMEM: return "out of memory";
    case EW_EHIP: return ew::last_hip_error();
    case EW_EINFEASIBLE: return "infeasible: no layer partition fits the stages' memory caps";
    case EW_ETOOBIG:
      return "too big: the input exceeds the fixed scratch array of the allocation-free entry point "
             "(EW_NOALLOC_MAX_BYTES per call)";
    default: return "unknown error code";
  }
}

const char *ew_version(void) { return "elaswave-mi355x 0.1 (gfx950)"; }

}  // extern "C"
