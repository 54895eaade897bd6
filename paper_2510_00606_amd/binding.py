"""ctypes binding of libelaswave.so: the same names as include/elaswave.h, argument marshalling
and buffer-size checks only.  Every step of the path runs in the library's HIP kernels; there is
no CPU fallback, and a missing library raises at first use.

Device buffers are passed either as integers (raw device addresses) or as objects with
`data_ptr()` (torch tensors); `stream` is a raw hipStream_t value (for torch:
`torch.cuda.current_stream().cuda_stream`) or None for the default stream.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

EW_OK, EW_EINVAL, EW_EUNRECOVERABLE, EW_ENOMEM, EW_EHIP, EW_EINFEASIBLE, EW_ETOOBIG = 0, -1, -2, -3, -4, -5, -6
EW_NOALLOC_MAX_BYTES = 1 << 30
EW_MAX_DP = 64
EW_GRANULE = 8
EW_CKSUM_BLOCK = 1 << 20
EW_SEG_SNAPSHOT, EW_SEG_LOCAL = 1, 2
EW_NO_STAGE = (1 << 64) - 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libelaswave.so")

SEG_DTYPE = np.dtype([("src_off", "<u8"), ("dst_off", "<u8"), ("stage_off", "<u8"), ("len", "<u8"),
                      ("src_owner", "<u2"), ("holder", "<u2"), ("dst_rank", "<u2"), ("flags", "<u2")])
TILE_DTYPE = np.dtype([("src_off", "<u8"), ("dst_off", "<u8"), ("len", "<u4"), ("src_buf", "<u2"), ("dst_buf", "<u2")])
CKSUM_DTYPE = np.dtype([("sum", "<u8"), ("xr", "<u8")])


class EwError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().ew_strerror(code).decode() if _lib is not None else "?"
        super().__init__(f"{where} failed: {msg} (code {code})")


_lib = None

_SIGNATURES = {
    "ew_plan": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64, C.POINTER(C.c_void_p)]),
    "ew_plan_bounds": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64, C.c_void_p, C.POINTER(C.c_void_p)]),
    "ew_plan_migrate": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64,
                                  C.POINTER(C.c_void_p)]),
    "ew_partition_layers": (C.c_int, [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.POINTER(C.c_double)]),
    "ew_plan_free": (None, [C.c_void_p]),
    "ew_plan_numel": (C.c_uint64, [C.c_void_p]),
    "ew_plan_old_dp": (C.c_uint32, [C.c_void_p]),
    "ew_plan_new_dp": (C.c_uint32, [C.c_void_p]),
    "ew_plan_num_segs": (C.c_uint64, [C.c_void_p]),
    "ew_plan_segs": (C.c_void_p, [C.c_void_p]),
    "ew_plan_old_shard_len": (C.c_uint64, [C.c_void_p, C.c_uint32]),
    "ew_plan_new_shard_len": (C.c_uint64, [C.c_void_p, C.c_uint32]),
    "ew_plan_new_rank_of": (C.c_int32, [C.c_void_p, C.c_uint32]),
    "ew_plan_holder_of": (C.c_int32, [C.c_void_p, C.c_uint32]),
    "ew_plan_stage_len": (C.c_uint64, [C.c_void_p]),
    "ew_plan_pair_len": (C.c_uint64, [C.c_void_p, C.c_uint32, C.c_uint32]),
    "ew_plan_pair_off": (C.c_uint64, [C.c_void_p, C.c_uint32, C.c_uint32]),
    "ew_plan_remote_elems": (C.c_uint64, [C.c_void_p]),
    "ew_plan_num_tiles": (C.c_uint64, [C.c_void_p, C.c_int, C.c_uint32]),
    "ew_plan_num_runs": (C.c_uint64, [C.c_void_p]),
    "ew_plan_tiles": (C.c_int, [C.c_void_p, C.c_int, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64, C.c_void_p,
                                C.POINTER(C.c_uint64)]),
    "ew_tile_of_workgroup": (C.c_uint64, [C.c_uint64, C.c_uint64, C.c_uint32]),
    "ew_plan_upload": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p]),
    "ew_pack": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]),
    "ew_unpack": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]),
    "ew_unpack_snapshot": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_uint32, C.c_void_p]),
    "ew_reshard": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]),
    "ew_reshard_snapshot": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                      C.c_void_p]),
    "ew_snapshot": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]),
    "ew_snapshot_noalloc": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]),
    "ew_scratch_release": (C.c_int, [C.c_void_p]),
    "ew_verify": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                            C.c_uint64, C.c_void_p]),
    "ew_single_bit_flip": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32), C.POINTER(C.c_int32)]),
    "ew_adam_hyper": (C.c_int, [C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_uint64, C.c_void_p]),
    "ew_adam_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64,
                               C.c_void_p, C.c_void_p]),
    "ew_adam_replay_host": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                      C.c_uint64, C.c_void_p, C.c_uint32]),
    "ew_grad_ship": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "ew_checksum_host": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32]),
    "ew_memcpy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "ew_set_param": (C.c_int, [C.c_char_p, C.c_int64]),
    "ew_get_param": (C.c_int64, [C.c_char_p]),
    "ew_strerror": (C.c_char_p, [C.c_int]),
    "ew_version": (C.c_char_p, []),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """Loads libelaswave.so on first use; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2510_00606_amd.build). "
                "There is no CPU fallback.")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(code: int, where: str):
    if code != EW_OK:
        raise EwError(code, where)


def _ptr(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _nbytes(x):
    """Size of a tensor-like buffer in bytes, or None for a raw address."""
    if isinstance(x, np.ndarray):
        return int(x.nbytes)
    if hasattr(x, "numel") and hasattr(x, "element_size"):
        return int(x.numel()) * int(x.element_size())
    return None


def _stream(stream) -> int:
    return 0 if stream is None else int(stream)


def _ptr_array(bufs, n):
    if bufs is None:
        bufs = [None] * n
    if len(bufs) != n:
        raise ValueError(f"expected {n} buffers, got {len(bufs)}")
    return (C.c_void_p * n)(*[_ptr(b) or None for b in bufs])


class Plan:
    """Owner of an ew_plan_t* (freed on close() / garbage collection)."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)

    # -- lifetime
    def close(self):
        if self._h:
            lib().ew_plan_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    @property
    def handle(self):
        if not self._h:
            raise ValueError("plan already freed")
        return self._h

    # -- queries
    @property
    def numel(self): return int(lib().ew_plan_numel(self.handle))
    @property
    def old_dp(self): return int(lib().ew_plan_old_dp(self.handle))
    @property
    def new_dp(self): return int(lib().ew_plan_new_dp(self.handle))
    @property
    def num_segs(self): return int(lib().ew_plan_num_segs(self.handle))
    @property
    def stage_len(self): return int(lib().ew_plan_stage_len(self.handle))
    @property
    def remote_elems(self): return int(lib().ew_plan_remote_elems(self.handle))

    def segs(self) -> np.ndarray:
        """Copy of the segment table as a structured numpy array."""
        n = self.num_segs
        if n == 0:
            return np.zeros(0, SEG_DTYPE)
        addr = lib().ew_plan_segs(self.handle)
        if not addr:
            raise MemoryError("ew_plan_segs: out of memory")
        buf = (C.c_char * (n * SEG_DTYPE.itemsize)).from_address(addr)
        return np.frombuffer(buf, dtype=SEG_DTYPE).copy()

    def tiles(self, which: int, tile_elems: int, align_elems: int = 0, first: int = 0, count=None) -> np.ndarray:
        """Copy tiles of the pack (0) / unpack (1) table, decoded on the host (all of them by default)."""
        total = C.c_uint64()
        _check(lib().ew_plan_tiles(self.handle, which, tile_elems, align_elems, 0, 0, None, C.byref(total)),
               "ew_plan_tiles")
        if count is None:
            count = total.value - first
        out = np.zeros(count, TILE_DTYPE)
        if count:
            _check(lib().ew_plan_tiles(self.handle, which, tile_elems, align_elems, first, count, out.ctypes.data,
                                       None), "ew_plan_tiles")
        return out

    def old_shard_len(self, r): return int(lib().ew_plan_old_shard_len(self.handle, r))
    def new_shard_len(self, r): return int(lib().ew_plan_new_shard_len(self.handle, r))
    def new_rank_of(self, r): return int(lib().ew_plan_new_rank_of(self.handle, r))
    def holder_of(self, r): return int(lib().ew_plan_holder_of(self.handle, r))
    def pair_len(self, h, k): return int(lib().ew_plan_pair_len(self.handle, h, k))
    def pair_off(self, h, k): return int(lib().ew_plan_pair_off(self.handle, h, k))
    def num_tiles(self, which, elem_size): return int(lib().ew_plan_num_tiles(self.handle, which, elem_size))
    @property
    def num_runs(self): return int(lib().ew_plan_num_runs(self.handle))


def ew_plan(old_dp, new_dp, alive_mask, numel, chunk) -> Plan:
    out = C.c_void_p()
    _check(lib().ew_plan(old_dp, new_dp, alive_mask, numel, chunk, C.byref(out)), "ew_plan")
    return Plan(out.value)


def ew_plan_bounds(old_dp, new_dp, alive_mask, unit_starts) -> Plan:
    starts = np.ascontiguousarray(unit_starts, dtype=np.uint64)
    if starts.ndim != 1 or len(starts) < 1:
        raise ValueError("unit_starts must hold n_units+1 values")
    out = C.c_void_p()
    _check(lib().ew_plan_bounds(old_dp, new_dp, alive_mask, len(starts) - 1, starts.ctypes.data, C.byref(out)),
           "ew_plan_bounds")
    return Plan(out.value)


EW_ASSIGN_INTERLEAVED, EW_ASSIGN_CONTIGUOUS = 0, 1


def ew_plan_migrate(assignment: int, dp: int, src_unit_starts, dst_unit_starts, n_move: int) -> Plan:
    src = np.ascontiguousarray(src_unit_starts, dtype=np.uint64)
    dst = np.ascontiguousarray(dst_unit_starts, dtype=np.uint64)
    if src.ndim != 1 or dst.ndim != 1 or len(src) < 1 or len(dst) < 1:
        raise ValueError("unit boundary arrays must hold n_units+1 values")
    out = C.c_void_p()
    _check(lib().ew_plan_migrate(assignment, dp, len(src) - 1, src.ctypes.data, len(dst) - 1, dst.ctypes.data, n_move,
                                 C.byref(out)), "ew_plan_migrate")
    return Plan(out.value)


def ew_partition_layers(t, mem, cap):
    """t[p][a][b], mem[a][b], cap[p] (array-likes).  Returns (cost, bounds) with bounds[p] = number of
    layers on stages 0..p; raises EwError(EW_EINFEASIBLE) if nothing fits."""
    t = np.ascontiguousarray(t, dtype=np.float64)
    mem = np.ascontiguousarray(mem, dtype=np.float64)
    cap = np.ascontiguousarray(cap, dtype=np.float64)
    if t.ndim != 3 or t.shape[1] != t.shape[2] or mem.shape != t.shape[1:] or cap.shape != (t.shape[0],):
        raise ValueError("expected t[P][L][L], mem[L][L], cap[P]")
    P, L = t.shape[0], t.shape[1]
    bounds = np.zeros(max(P - 1, 1), dtype=np.uint32)
    cost = C.c_double()
    _check(lib().ew_partition_layers(L, P, t.ctypes.data, mem.ctypes.data, cap.ctypes.data, bounds.ctypes.data,
                                     C.byref(cost)), "ew_partition_layers")
    return cost.value, [int(x) for x in bounds[:P - 1]]


def ew_tile_of_workgroup(workgroup: int, n_workgroups: int, group: int) -> int:
    return int(lib().ew_tile_of_workgroup(workgroup, n_workgroups, group))


def ew_plan_upload(plan: Plan, tile_elems: int = 0, stream=None):
    _check(lib().ew_plan_upload(plan.handle, tile_elems, _stream(stream)), "ew_plan_upload")


def _check_sources(plan: Plan, old_shards, snapshots, elem_size):
    for name, bufs in (("old shard", old_shards), ("snapshot", snapshots)):
        if bufs is None:
            continue
        for j, b in enumerate(bufs):
            n = _nbytes(b) if b is not None else None
            if n is not None and n < plan.old_shard_len(j) * elem_size:
                raise ValueError(f"{name} {j} holds {n} bytes, plan needs {plan.old_shard_len(j) * elem_size}")


def ew_pack(plan: Plan, old_shards, snapshots, stage, elem_size: int, stream=None):
    _check_sources(plan, old_shards, snapshots, elem_size)
    n = _nbytes(stage)
    if n is not None and n < plan.stage_len * elem_size:
        raise ValueError(f"staging arena holds {n} bytes, plan needs {plan.stage_len * elem_size}")
    D = plan.old_dp
    _check(lib().ew_pack(plan.handle, _ptr_array(old_shards, D), _ptr_array(snapshots, D), _ptr(stage),
                         elem_size, _stream(stream)), "ew_pack")


def ew_unpack(plan: Plan, stage, old_shards, snapshots, new_shards, elem_size: int, stream=None):
    _check_sources(plan, old_shards, snapshots, elem_size)
    n = _nbytes(stage)
    if n is not None and n < plan.stage_len * elem_size:
        raise ValueError(f"staging arena holds {n} bytes, plan needs {plan.stage_len * elem_size}")
    for k, b in enumerate(new_shards):
        n = _nbytes(b) if b is not None else None
        if n is not None and n < plan.new_shard_len(k) * elem_size:
            raise ValueError(f"new shard {k} holds {n} bytes, plan needs {plan.new_shard_len(k) * elem_size}")
    _check(lib().ew_unpack(plan.handle, _ptr(stage), _ptr_array(old_shards, plan.old_dp),
                           _ptr_array(snapshots, plan.old_dp), _ptr_array(new_shards, plan.new_dp),
                           elem_size, _stream(stream)), "ew_unpack")


def ew_unpack_snapshot(plan: Plan, stage, old_shards, snapshots, new_shards, new_snapshots, new_cksums,
                       elem_size: int, stream=None):
    _check_sources(plan, old_shards, snapshots, elem_size)
    n = _nbytes(stage)
    if n is not None and n < plan.stage_len * elem_size:
        raise ValueError(f"staging arena holds {n} bytes, plan needs {plan.stage_len * elem_size}")
    for k in range(plan.new_dp):
        need = plan.new_shard_len(k) * elem_size
        for name, bufs, want in (("new shard", new_shards, need), ("new snapshot", new_snapshots, need),
                                 ("new checksum array", new_cksums, 16 * num_blocks(need))):
            n = _nbytes(bufs[k]) if bufs[k] is not None else None
            if n is not None and n < want:
                raise ValueError(f"{name} {k} holds {n} bytes, plan needs {want}")
    D = plan.new_dp
    _check(lib().ew_unpack_snapshot(plan.handle, _ptr(stage), _ptr_array(old_shards, plan.old_dp),
                                    _ptr_array(snapshots, plan.old_dp), _ptr_array(new_shards, D),
                                    _ptr_array(new_snapshots, D), _ptr_array(new_cksums, D), elem_size,
                                    _stream(stream)), "ew_unpack_snapshot")


def _check_new(plan, new_shards, new_snapshots, new_cksums, elem_size):
    for k in range(plan.new_dp):
        need = plan.new_shard_len(k) * elem_size
        for name, bufs, want in (("new shard", new_shards, need), ("new snapshot", new_snapshots, need),
                                 ("new checksum array", new_cksums, 16 * num_blocks(need))):
            if bufs is None:
                continue
            n = _nbytes(bufs[k]) if bufs[k] is not None else None
            if n is not None and n < want:
                raise ValueError(f"{name} {k} holds {n} bytes, plan needs {want}")


def ew_reshard(plan: Plan, old_shards, snapshots, new_shards, elem_size: int, stream=None):
    _check_sources(plan, old_shards, snapshots, elem_size)
    _check_new(plan, new_shards, None, None, elem_size)
    _check(lib().ew_reshard(plan.handle, _ptr_array(old_shards, plan.old_dp), _ptr_array(snapshots, plan.old_dp),
                            _ptr_array(new_shards, plan.new_dp), elem_size, _stream(stream)), "ew_reshard")


def ew_reshard_snapshot(plan: Plan, old_shards, snapshots, new_shards, new_snapshots, new_cksums, elem_size: int,
                        stream=None):
    _check_sources(plan, old_shards, snapshots, elem_size)
    _check_new(plan, new_shards, new_snapshots, new_cksums, elem_size)
    D = plan.new_dp
    _check(lib().ew_reshard_snapshot(plan.handle, _ptr_array(old_shards, plan.old_dp),
                                     _ptr_array(snapshots, plan.old_dp), _ptr_array(new_shards, D),
                                     _ptr_array(new_snapshots, D), _ptr_array(new_cksums, D), elem_size,
                                     _stream(stream)), "ew_reshard_snapshot")


def num_blocks(nbytes: int) -> int:
    return -(-int(nbytes) // EW_CKSUM_BLOCK)


def ew_snapshot(src, dst, nbytes: int, cksums, stream=None):
    for name, b, need in (("src", src, nbytes), ("dst", dst, nbytes), ("cksums", cksums, 16 * num_blocks(nbytes))):
        n = _nbytes(b)
        if n is not None and n < need:
            raise ValueError(f"{name} holds {n} bytes, call needs {need}")
    _check(lib().ew_snapshot(_ptr(src), _ptr(dst), nbytes, _ptr(cksums), _stream(stream)), "ew_snapshot")


def ew_snapshot_noalloc(src, dst, nbytes: int, cksums, stream=None):
    for name, b, need in (("src", src, nbytes), ("dst", dst, nbytes), ("cksums", cksums, 16 * num_blocks(nbytes))):
        n = _nbytes(b)
        if n is not None and n < need:
            raise ValueError(f"{name} holds {n} bytes, call needs {need}")
    _check(lib().ew_snapshot_noalloc(_ptr(src), _ptr(dst), nbytes, _ptr(cksums), _stream(stream)),
           "ew_snapshot_noalloc")


def ew_scratch_release(stream=None):
    _check(lib().ew_scratch_release(_stream(stream)), "ew_scratch_release")


def ew_verify(buf, nbytes: int, expect, got, n_bad, bad_blocks, diffs, cap: int, stream=None):
    nb = num_blocks(nbytes)
    for name, b, need in (("buf", buf, nbytes), ("expect", expect, 16 * nb), ("got", got, 16 * nb),
                          ("n_bad", n_bad, 8), ("bad_blocks", bad_blocks, 8 * cap), ("diffs", diffs, 16 * cap)):
        n = _nbytes(b)
        if n is not None and n < need:
            raise ValueError(f"{name} holds {n} bytes, call needs {need}")
    _check(lib().ew_verify(_ptr(buf), nbytes, _ptr(expect), _ptr(got), _ptr(n_bad), _ptr(bad_blocks), _ptr(diffs),
                           cap, _stream(stream)), "ew_verify")


def ew_single_bit_flip(sum_diff: int, xor_diff: int):
    """(lane, direction) if the differences of one bad block are those of one flipped bit, else None."""
    rec = (C.c_uint64 * 2)(sum_diff & ((1 << 64) - 1), xor_diff & ((1 << 64) - 1))
    lane, direction = C.c_uint32(), C.c_int32()
    if lib().ew_single_bit_flip(C.addressof(rec), C.byref(lane), C.byref(direction)):
        return lane.value, direction.value
    return None


class AdamHyper(C.Structure):
    """ew_adam_t: the nine fp32 scalars of one optimizer step."""
    _fields_ = [(n, C.c_float) for n in ("lr", "beta1", "beta2", "omb1", "omb2", "eps", "wd", "bias1", "bias2")]


def ew_adam_hyper(lr, beta1, beta2, eps, weight_decay, step: int) -> AdamHyper:
    h = AdamHyper()
    _check(lib().ew_adam_hyper(lr, beta1, beta2, eps, weight_decay, step, C.byref(h)), "ew_adam_hyper")
    return h


def _check_len(name, buf, need):
    n = _nbytes(buf)
    if n is not None and n < need:
        raise ValueError(f"{name} holds {n} bytes, call needs {need}")


def ew_adam_step(p, w, m, v, grad, grad_elem_size: int, n: int, h: AdamHyper, stream=None):
    """Device buffers (tensors or raw addresses)."""
    for name, b, need in (("p", p, 2 * n), ("w", w, 4 * n), ("m", m, 4 * n), ("v", v, 4 * n),
                          ("grad", grad, grad_elem_size * n)):
        _check_len(name, b, need)
    _check(lib().ew_adam_step(_ptr(p), _ptr(w), _ptr(m), _ptr(v), _ptr(grad), grad_elem_size, n, C.byref(h),
                              _stream(stream)), "ew_adam_step")


def ew_adam_replay_host(p, w, m, v, grad, grad_elem_size: int, n: int, h: AdamHyper, n_threads: int = 0):
    """Host buffers: CPU tensors or numpy arrays (updated in place)."""
    for name, b, need in (("p", p, 2 * n), ("w", w, 4 * n), ("m", m, 4 * n), ("v", v, 4 * n),
                          ("grad", grad, grad_elem_size * n)):
        _check_len(name, b, need)
    _check(lib().ew_adam_replay_host(_host_ptr(p), _host_ptr(w), _host_ptr(m), _host_ptr(v), _host_ptr(grad),
                                     grad_elem_size, n, C.byref(h), n_threads), "ew_adam_replay_host")


def ew_grad_ship(grad_dev, peer_dev, host_buf, nbytes: int, stream=None):
    for name, b in (("grad", grad_dev), ("peer buffer", peer_dev), ("host buffer", host_buf)):
        if b is not None:
            _check_len(name, b, nbytes)
    _check(lib().ew_grad_ship(_ptr(grad_dev), _ptr(peer_dev), _host_ptr(host_buf) if host_buf is not None else 0,
                              nbytes, _stream(stream)), "ew_grad_ship")


def ew_checksum_host(buf, nbytes: int, n_threads: int = 0) -> np.ndarray:
    """Block checksums of a host buffer as a CKSUM_DTYPE array."""
    _check_len("buf", buf, nbytes)
    out = np.zeros(num_blocks(nbytes), CKSUM_DTYPE)
    _check(lib().ew_checksum_host(_host_ptr(buf), nbytes, out.ctypes.data, n_threads), "ew_checksum_host")
    return out


def _host_ptr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, np.ndarray):
        return int(x.ctypes.data)
    if hasattr(x, "data_ptr"):
        if getattr(x, "is_cuda", False):
            raise ValueError("expected a host buffer, got a device tensor")
        return int(x.data_ptr())
    return int(x)


def ew_memcpy(src, dst, nbytes: int, stream=None):
    for name, b in (("src", src), ("dst", dst)):
        n = _nbytes(b)
        if n is not None and n < nbytes:
            raise ValueError(f"{name} holds {n} bytes, call needs {nbytes}")
    _check(lib().ew_memcpy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "ew_memcpy")


def ew_set_param(name: str, value: int):
    _check(lib().ew_set_param(name.encode(), int(value)), f"ew_set_param({name})")


def ew_get_param(name: str) -> int:
    return int(lib().ew_get_param(name.encode()))


def ew_strerror(code: int) -> str:
    return lib().ew_strerror(code).decode()


def ew_version() -> str:
    return lib().ew_version().decode()
