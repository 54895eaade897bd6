"""MI355X-native reshard + snapshot/checksum path of ElasWave (arXiv 2510.00606).

  binding   ctypes wrappers with the names of include/elaswave.h (the product path)
  build     compiles csrc/ into libelaswave.so for gfx950
  synth     seeded synthetic inputs (no arithmetic of the method)
  configs   the benchmark/test workloads (shapes, DP changes, unit boundaries)
"""
from .binding import (  # noqa: F401
    EW_ASSIGN_CONTIGUOUS, EW_ASSIGN_INTERLEAVED, EW_CKSUM_BLOCK, EW_EHIP, EW_EINFEASIBLE, EW_EINVAL, EW_ENOMEM, EW_ETOOBIG, EW_EUNRECOVERABLE, EW_GRANULE, EW_MAX_DP, EW_NOALLOC_MAX_BYTES, EW_NO_STAGE, EW_OK,
    EW_SEG_LOCAL, EW_SEG_SNAPSHOT, CKSUM_DTYPE, SEG_DTYPE, TILE_DTYPE, AdamHyper, EwError, Plan, ew_adam_hyper, ew_adam_replay_host, ew_adam_step, ew_checksum_host, ew_grad_ship, ew_get_param, ew_memcpy, ew_pack, ew_partition_layers, ew_plan,
    ew_plan_bounds, ew_plan_migrate, ew_plan_upload, ew_reshard, ew_reshard_snapshot, ew_set_param, ew_single_bit_flip, ew_scratch_release, ew_snapshot, ew_snapshot_noalloc, ew_strerror, ew_tile_of_workgroup, ew_unpack, ew_unpack_snapshot, ew_verify, ew_version,
    num_blocks,
)
