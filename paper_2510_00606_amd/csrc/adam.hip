// Gradient-shipping snapshot (Sec. 5.1, Fig. 6): instead of copying a neighbour's Adam state every
// step, its GRADIENT shard is shipped (device to device, then device to host) and the optimizer
// update is replayed on the snapshot by the host CPU.  The replay must give the bits the owner's
// own update gave, so ONE element routine, made of single fp32 operations in a fixed order with
// contraction into fused multiply-adds switched off, is compiled for both sides:
//   ew_adam_kernel       the owner's step on its live shard (HBM bound: 30 B per element with fp32
//                        gradients: reads g, w, m, v, writes w, m, v and the bf16 copy)
//   ew_adam_replay_host  the same update on a host-resident snapshot, split over host threads
// plus ew_grad_ship (the two copies) and ew_checksum_host (block checksums of a host buffer, so a
// host snapshot can be verified against the live shard with ew_verify).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include "elaswave.h"
#include "runtime.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 64;    // one wave per workgroup: with eight streams per lane this shape measured best

__host__ __device__ inline float bits_to_f32(uint32_t u) {
  float f;
  __builtin_memcpy(&f, &u, 4);
  return f;
}
__host__ __device__ inline uint32_t f32_to_bits(float f) {
  uint32_t u;
  __builtin_memcpy(&u, &f, 4);
  return u;
}
// fp32 -> bf16, round to nearest even; NaNs stay quiet NaNs
__host__ __device__ inline uint16_t bf16_rne(float f) {
  const uint32_t u = f32_to_bits(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// The update of one element.  Every statement is one IEEE fp32 operation (division and square
// root correctly rounded on both sides); the pragma keeps the compilers from fusing any of them.
__host__ __device__ inline void adam_element(float &w, float &m, float &v, float g, const ew_adam_t &h,
                                             uint16_t &p) {
#pragma clang fp contract(off)
  const float t1 = h.beta1 * m;
  const float t2 = h.omb1 * g;
  m = t1 + t2;
  const float gg = g * g;
  const float t3 = h.beta2 * v;
  const float t4 = h.omb2 * gg;
  v = t3 + t4;
  const float vh = v * h.bias2;
  const float den = __builtin_sqrtf(vh) + h.eps;
  const float mh = m * h.bias1;
  const float upd = mh / den;
  const float dec = h.wd * w;
  const float dir = upd + dec;
  const float stepv = h.lr * dir;
  w = w - stepv;
  p = bf16_rne(w);
}

template <int GES>
__device__ __forceinline__ float load_grad(const void *g, uint64_t i) {
  if (GES == 4) return reinterpret_cast<const float *>(g)[i];
  return bits_to_f32((uint32_t) reinterpret_cast<const uint16_t *>(g)[i] << 16);
}

// One lane updates four consecutive elements: 128-bit loads of w, m, v (and g when fp32), 128-bit
// stores of w, m, v, one 64-bit store of the four bf16 values; 256 elements per one-wave workgroup.
template <int GES, bool VEC>
__global__ __launch_bounds__(kThreads) void ew_adam_kernel(uint16_t *__restrict__ p, float *__restrict__ w,
                                                           float *__restrict__ m, float *__restrict__ v,
                                                           const void *__restrict__ g, uint64_t n, ew_adam_t h,
                                                           ew::XcdMap xcd) {
  // workgroups go to the XCDs in runs of consecutive 256-element chunks (see ew::xcd_remap)
  const uint64_t lane = (uint64_t)(VEC ? ew::xcd_remap(blockIdx.x, xcd) : blockIdx.x) * kThreads + threadIdx.x;
  if (VEC) {
    const uint64_t i = lane * 4;
    if (i + 4 <= n) {
      f32x4 wv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(w + i));
      f32x4 mv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(m + i));
      f32x4 vv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(v + i));
      float gv[4];
      if (GES == 4) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(g) + i));
        gv[0] = t.x; gv[1] = t.y; gv[2] = t.z; gv[3] = t.w;
      } else {
        const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(reinterpret_cast<const uint16_t *>(g) + i));
        gv[0] = bits_to_f32(t.x << 16); gv[1] = bits_to_f32(t.x & 0xffff0000u);
        gv[2] = bits_to_f32(t.y << 16); gv[3] = bits_to_f32(t.y & 0xffff0000u);
      }
      float we[4] = {wv.x, wv.y, wv.z, wv.w}, me[4] = {mv.x, mv.y, mv.z, mv.w}, ve[4] = {vv.x, vv.y, vv.z, vv.w};
      uint16_t pe[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) adam_element(we[k], me[k], ve[k], gv[k], h, pe[k]);
      wv.x = we[0]; wv.y = we[1]; wv.z = we[2]; wv.w = we[3];
      mv.x = me[0]; mv.y = me[1]; mv.z = me[2]; mv.w = me[3];
      vv.x = ve[0]; vv.y = ve[1]; vv.z = ve[2]; vv.w = ve[3];
      __builtin_nontemporal_store(wv, reinterpret_cast<f32x4 *>(w + i));
      __builtin_nontemporal_store(mv, reinterpret_cast<f32x4 *>(m + i));
      __builtin_nontemporal_store(vv, reinterpret_cast<f32x4 *>(v + i));
      u32x2 pv;
      pv.x = (uint32_t)pe[0] | ((uint32_t)pe[1] << 16);
      pv.y = (uint32_t)pe[2] | ((uint32_t)pe[3] << 16);
      __builtin_nontemporal_store(pv, reinterpret_cast<u32x2 *>(p + i));
    } else {
      for (uint64_t e = i; e < n; ++e) {  // fewer than four trailing elements
        float we = w[e], me = m[e], ve = v[e];
        uint16_t pe;
        adam_element(we, me, ve, load_grad<GES>(g, e), h, pe);
        w[e] = we; m[e] = me; v[e] = ve; p[e] = pe;
      }
    }
  } else {
    // buffers that are not 16-byte aligned: one element per lane
    for (uint64_t e = lane; e < n; e += (uint64_t)gridDim.x * kThreads) {
      float we = w[e], me = m[e], ve = v[e];
      uint16_t pe;
      adam_element(we, me, ve, load_grad<GES>(g, e), h, pe);
      w[e] = we; m[e] = me; v[e] = ve; p[e] = pe;
    }
  }
}

void replay_range(uint16_t *p, float *w, float *m, float *v, const void *g, uint32_t ges, uint64_t lo, uint64_t hi,
                  const ew_adam_t &h) {
  if (ges == 4) {
    const float *gf = reinterpret_cast<const float *>(g);
    for (uint64_t e = lo; e < hi; ++e) adam_element(w[e], m[e], v[e], gf[e], h, p[e]);
  } else {
    const uint16_t *gb = reinterpret_cast<const uint16_t *>(g);
    for (uint64_t e = lo; e < hi; ++e) adam_element(w[e], m[e], v[e], bits_to_f32((uint32_t)gb[e] << 16), h, p[e]);
  }
}

template <class Fn>
int run_threads(uint64_t n_items, uint32_t n_threads, Fn fn) {  // fn(lo, hi) on disjoint ranges
  if (n_threads == 0) n_threads = std::max(1u, std::thread::hardware_concurrency());
  n_threads = (uint32_t)std::min<uint64_t>(n_threads, std::max<uint64_t>(1, n_items));
  if (n_threads <= 1) {
    fn((uint64_t)0, n_items);
    return EW_OK;
  }
  // The pool outlives the try block: if a thread cannot be started, those already running are joined
  // and the calling thread does the ranges that are left, so the work is still done exactly once.
  std::vector<std::thread> pool;
  const uint64_t per = (n_items + n_threads - 1) / n_threads;
  uint64_t next = 0;  // first item no thread has been given
  int rc = EW_OK;
  try {
    pool.reserve(n_threads);
    while (next < n_items) {
      const uint64_t hi = std::min<uint64_t>(n_items, next + per);
      pool.emplace_back(fn, next, hi);
      next = hi;
    }
  } catch (const std::bad_alloc &) {
    rc = EW_ENOMEM;
  } catch (const std::system_error &) {
    rc = EW_ENOMEM;
  }
  if (rc != EW_OK && next < n_items) {
    fn(next, n_items);
    rc = EW_OK;
  }
  for (auto &th : pool) th.join();
  return rc;
}

}  // namespace

extern "C" {

int ew_adam_hyper(float lr, float beta1, float beta2, float eps, float weight_decay, uint64_t step, ew_adam_t *out) {
  if (!out || step == 0 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return EW_EINVAL;
  out->lr = lr;
  out->beta1 = beta1;
  out->beta2 = beta2;
  out->omb1 = (float)(1.0 - (double)beta1);
  out->omb2 = (float)(1.0 - (double)beta2);
  out->eps = eps;
  out->wd = weight_decay;
  out->bias1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  out->bias2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  return EW_OK;
}

int ew_adam_step(void *p_bf16, float *w, float *m, float *v, const void *grad, uint32_t grad_elem_size, uint64_t n,
                 const ew_adam_t *h, void *stream) {
  if (!h || (grad_elem_size != 2 && grad_elem_size != 4)) return EW_EINVAL;
  if (n == 0) return EW_OK;
  if (!p_bf16 || !w || !m || !v || !grad) return EW_EINVAL;
  const uintptr_t all = (uintptr_t)w | (uintptr_t)m | (uintptr_t)v | (uintptr_t)grad | ((uintptr_t)p_bf16 << 1);
  const bool vec = (all & 15u) == 0;
  uint64_t grid = vec ? ((n + 3) / 4 + kThreads - 1) / kThreads : std::min<uint64_t>((n + kThreads - 1) / kThreads, 1u << 20);
  if (grid > 0x7fffffffull) return EW_EINVAL;
  uint16_t *p = (uint16_t *)p_bf16;
  hipStream_t s = (hipStream_t)stream;
  // Eight HBM streams per wave (four read, four written): with 10-12 one-wave workgroups resident per CU
  // the step runs 7 % faster than with the 32 that fit (6.05 -> 6.52 TB/s measured in one process;
  // 16: 5.6-6.3, 8: 6.0-6.2).  In one process on one set of buffers, eight timings each: 10 per CU
  // 6.44-6.49 TB/s, 12 per CU 6.18-6.47 (it wanders from one timing to the next), 14: 6.38-6.46.  Runs of
  // 256 consecutive workgroups per XCD add 1-1.5 % over one by one; runs of 64: 6.07-6.09, of 128: 6.26-6.44,
  // of 512 and more: 6.08-6.21.
  const uint32_t lds_pad = ew::occupancy_pad(ew::knobs().adam_wgs_per_cu, 0);
  const dim3 g((uint32_t)grid), b(kThreads);
  const ew::XcdMap xg = ew::make_xcd_map((uint32_t)ew::knobs().adam_xcd_group, (uint32_t)grid);  // in workgroups (256 elements each)
  if (grad_elem_size == 4) {
    if (vec) hipLaunchKernelGGL((ew_adam_kernel<4, true>), g, b, lds_pad, s, p, w, m, v, grad, n, *h, xg);
    else hipLaunchKernelGGL((ew_adam_kernel<4, false>), g, b, lds_pad, s, p, w, m, v, grad, n, *h, xg);
  } else {
    if (vec) hipLaunchKernelGGL((ew_adam_kernel<2, true>), g, b, lds_pad, s, p, w, m, v, grad, n, *h, xg);
    else hipLaunchKernelGGL((ew_adam_kernel<2, false>), g, b, lds_pad, s, p, w, m, v, grad, n, *h, xg);
  }
  EW_HIP(hipGetLastError());
  return EW_OK;
}

int ew_adam_replay_host(void *p_bf16, float *w, float *m, float *v, const void *grad, uint32_t grad_elem_size,
                        uint64_t n, const ew_adam_t *h, uint32_t n_threads) {
  if (!h || (grad_elem_size != 2 && grad_elem_size != 4)) return EW_EINVAL;
  if (n == 0) return EW_OK;
  if (!p_bf16 || !w || !m || !v || !grad) return EW_EINVAL;
  const ew_adam_t hh = *h;
  uint16_t *p = (uint16_t *)p_bf16;
  return run_threads(n, n_threads, [=](uint64_t lo, uint64_t hi) { replay_range(p, w, m, v, grad, grad_elem_size, lo, hi, hh); });
}

int ew_grad_ship(const void *grad_dev, void *peer_dev, void *host_buf, uint64_t nbytes, void *stream) {
  if (nbytes == 0) return EW_OK;
  if (!grad_dev || (!peer_dev && !host_buf)) return EW_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const void *from = grad_dev;
  if (peer_dev) {  // device-to-device hop to the worker that keeps the snapshot
    EW_HIP(hipMemcpyAsync(peer_dev, grad_dev, nbytes, hipMemcpyDeviceToDevice, s));
    from = peer_dev;
  }
  if (host_buf) EW_HIP(hipMemcpyAsync(host_buf, from, nbytes, hipMemcpyDeviceToHost, s));
  return EW_OK;
}

int ew_checksum_host(const void *buf, uint64_t nbytes, ew_cksum_t *cksums, uint32_t n_threads) {
  if (nbytes == 0) return EW_OK;
  if (!buf || !cksums) return EW_EINVAL;
  const uint64_t nblocks = (nbytes + EW_CKSUM_BLOCK - 1) / EW_CKSUM_BLOCK;
  const unsigned char *b = (const unsigned char *)buf;
  return run_threads(nblocks, n_threads, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t blk = lo; blk < hi; ++blk) {
      const uint64_t begin = blk * EW_CKSUM_BLOCK, end = std::min<uint64_t>(nbytes, begin + EW_CKSUM_BLOCK);
      uint64_t sum = 0, xr = 0, o = begin;
      for (; o + 8 <= end; o += 8) {
        uint64_t wd;
        std::memcpy(&wd, b + o, 8);  // little-endian host
        sum += wd;
        xr ^= wd;
      }
      if (o < end) {
        uint64_t wd = 0;
        std::memcpy(&wd, b + o, end - o);
        sum += wd;
        xr ^= wd;
      }
      cksums[blk].sum = sum;
      cksums[blk].xr = xr;
    }
  });
}

}  // extern "C"
