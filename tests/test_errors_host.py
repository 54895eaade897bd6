"""Error reporting of the C ABI on a machine without a GPU: a failing HIP call must come back as
EW_EHIP with the failing call's name and the runtime's message behind ew_strerror, argument checks
must precede any HIP call, and nothing may throw or abort."""
import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew

no_gpu = pytest.mark.skipif(torch.cuda.device_count() > 0, reason="forces HIP failures by having no GPU")


@no_gpu
def test_hip_failure_text_reaches_strerror():
    a = np.zeros(64, np.uint8)
    with pytest.raises(ew.EwError) as e:
        ew.ew_grad_ship(a.ctypes.data, a.ctypes.data + 32, None, 16, None)
    assert e.value.code == ew.EW_EHIP
    msg = ew.ew_strerror(ew.EW_EHIP)
    assert "hipMemcpyAsync" in msg and msg in str(e.value)
    with pytest.raises(ew.EwError) as e:        # host-to-device leg, reported under its own name
        ew.ew_grad_ship(a.ctypes.data, None, a, 16, None)
    assert e.value.code == ew.EW_EHIP and "hipMemcpyDeviceToHost" in ew.ew_strerror(ew.EW_EHIP)
    with pytest.raises(ew.EwError) as e:        # a kernel launch that cannot happen
        ew.ew_memcpy(a.ctypes.data & ~15, (a.ctypes.data & ~15) + 32, 16, None)
    assert e.value.code == ew.EW_EHIP and "no HIP error recorded" not in ew.ew_strerror(ew.EW_EHIP)


def test_argument_checks_come_before_any_hip_call():
    a = np.zeros(64, np.uint8)
    for call in (lambda: ew.ew_snapshot_noalloc(a.ctypes.data, a.ctypes.data + 32, ew.EW_NOALLOC_MAX_BYTES + 1, a.ctypes.data, None),):
        with pytest.raises(ew.EwError) as e:
            call()
        assert e.value.code == ew.EW_ETOOBIG and "too big" in ew.ew_strerror(ew.EW_ETOOBIG)
    with pytest.raises(ew.EwError) as e:
        ew.ew_snapshot_noalloc(None, a.ctypes.data, 16, a.ctypes.data, None)
    assert e.value.code == ew.EW_EINVAL
    ew.ew_snapshot_noalloc(None, None, 0, None, None)      # zero bytes: nothing to do, no error
    with pytest.raises(ew.EwError) as e:
        ew.ew_memcpy(a.ctypes.data, a.ctypes.data + 32, 24, None)
    assert e.value.code == ew.EW_EINVAL


def test_statistics_knob_can_only_be_reset():
    assert ew.ew_get_param("scratch_max_concurrent") >= 0
    ew.ew_set_param("scratch_max_concurrent", 0)
    assert ew.ew_get_param("scratch_max_concurrent") == 0
    with pytest.raises(ew.EwError):
        ew.ew_set_param("scratch_max_concurrent", 3)
    with pytest.raises(ew.EwError):
        ew.ew_set_param("fused_mode", 2)
    assert ew.ew_get_param("fused_mode") == 0


def test_host_replay_uses_every_requested_thread_count():
    """The thread pool behind the host replay and the host checksum gives the same bits for any
    number of threads, including more threads than items."""
    rng = np.random.default_rng(3)
    buf = rng.integers(0, 256, 5 * (1 << 20) + 77, dtype=np.uint8)
    ref = ew.ew_checksum_host(buf, buf.nbytes, 1)
    for n in (2, 3, 7, 64):
        assert np.array_equal(ew.ew_checksum_host(buf, buf.nbytes, n), ref)
