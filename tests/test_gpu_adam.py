"""Gradient-shipping snapshot on the GPU (Sec. 5.1, Fig. 6): the owner's Adam step (ew_adam_step)
against the oracle, and the whole loop -- step on the live shard, ship the gradient shard device to
device to host, replay on the host snapshot -- keeping snapshot and live state identical to the bit."""
import numpy as np
import pytest
import torch

import paper_2510_00606_amd as ew
from oracle import adam
from paper_2510_00606_amd import synth

from gpu_util import DEV, stream

pytestmark = pytest.mark.gpu
F = np.float32


def dev_f32(a, shift=0):
    """Device copy of a float32 array; shift > 0 places it `shift` elements into a larger buffer."""
    t = torch.zeros(len(a) + shift + 8, dtype=torch.float32, device=DEV)
    t[shift:shift + len(a)] = torch.from_numpy(a)
    return t, t[shift:shift + len(a)]


@pytest.mark.parametrize("grad_bits", [32, 16])
@pytest.mark.parametrize("n,shift", [(1, 0), (3, 0), (4, 0), (1023, 0), (1024, 0), (4099, 0), (100003, 1), (100003, 2), (1 << 21, 0)])
def test_device_step_is_bit_exact(n, shift, grad_bits):
    rng = np.random.default_rng(n + shift + grad_bits)
    ow = (rng.standard_normal(n) * 0.02).astype(F)
    om, ov = np.zeros(n, F), np.zeros(n, F)
    wb, w = dev_f32(ow, shift)
    mb, m = dev_f32(om, shift)
    vb, v = dev_f32(ov, shift)
    pb = torch.full((n + 16,), 0x5A5A, dtype=torch.int16, device=DEV)
    p = pb[:n]
    for t in range(1, 5):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, n)).astype(F)
        if grad_bits == 16:
            g = (g.view(np.uint32) >> 16).astype(np.uint16)
            gd = torch.from_numpy(g.view(np.int16)).to(DEV)
        else:
            gd = torch.from_numpy(g).to(DEV)
        args = (3e-4, 0.9, 0.95, 1e-8, 0.1, t)
        ow, om, ov, op = adam.step(ow, om, ov, g, adam.hyper(*args))
        ew.ew_adam_step(p, w, m, v, gd, grad_bits // 8, n, ew.ew_adam_hyper(*args), stream())
        torch.cuda.synchronize()
        for name, got, want in (("w", w, ow), ("m", m, om), ("v", v, ov)):
            assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"{name} differs at step {t}"
        assert np.array_equal(p.cpu().numpy().view(np.uint16), op), f"bf16 copy differs at step {t}"
    assert bool((pb[n:] == 0x5A5A).all()) and bool((wb[shift + n:] == 0).all()) and bool((wb[:shift] == 0).all())


@pytest.mark.parametrize("group", [1, 3, 64, 256, 1 << 24])
def test_device_step_with_workgroups_dealt_to_xcds_in_runs(group):
    """Runs of consecutive chunks per XCD permute which workgroup updates which 256 elements, never the
    result: run lengths that do not divide the launch, a ragged tail, runs longer than the launch."""
    saved = ew.ew_get_param("adam_xcd_group")
    ew.ew_set_param("adam_xcd_group", group)
    try:
        test_device_step_is_bit_exact(300_001, 0, 32)
        test_device_step_is_bit_exact(1 << 21, 0, 16)
        test_device_step_is_bit_exact(4099, 0, 32)
    finally:
        ew.ew_set_param("adam_xcd_group", saved)


@pytest.mark.parametrize("wgs", [0, 1, 5, 12, 32])
def test_device_step_with_occupancy_caps(wgs):
    """The cap on resident workgroups changes the launch only, never the result."""
    saved = ew.ew_get_param("adam_wgs_per_cu")
    ew.ew_set_param("adam_wgs_per_cu", wgs)
    try:
        test_device_step_is_bit_exact(300_001, 0, 32)
    finally:
        ew.ew_set_param("adam_wgs_per_cu", saved)


def test_device_step_special_values():
    w = np.array([0.0, -0.0, 1e-40, 1e38, -1e38, 1.0, 3e-39, 1.0], F)
    m = np.array([0.0, 1e-45, -1e-40, 1e30, 0.0, 1e-42, 0.0, 0.5], F)
    v = np.array([0.0, 0.0, 1e-45, 1e38, 0.0, 1e-44, 1e-39, 1e-30], F)
    g = np.array([0.0, 1e-30, -1e-20, 1e19, -3e38, 1e-25, 1e-22, 1e-12], F)
    args = (1e-3, 0.9, 0.999, 1e-8, 0.01, 2)
    ow, om, ov, op = adam.step(w.copy(), m.copy(), v.copy(), g, adam.hyper(*args))
    dw, dm, dv, dg = (torch.from_numpy(x.copy()).to(DEV) for x in (w, m, v, g))
    dp = torch.zeros(8, dtype=torch.int16, device=DEV)
    ew.ew_adam_step(dp, dw, dm, dv, dg, 4, 8, ew.ew_adam_hyper(*args), stream())
    torch.cuda.synchronize()
    assert np.array_equal(dw.cpu().numpy().view(np.uint32), ow.view(np.uint32))
    assert np.array_equal(dm.cpu().numpy().view(np.uint32), om.view(np.uint32))
    assert np.array_equal(dv.cpu().numpy().view(np.uint32), ov.view(np.uint32))
    assert np.array_equal(dp.cpu().numpy().view(np.uint16), op)


@pytest.mark.parametrize("grad_bits", [32, 16])
def test_snapshot_by_gradient_shipping_tracks_the_live_state(grad_bits):
    """Worker i+1 updates its live shard; worker i receives only the gradient shard (D2D, then D2H)
    and replays the update on its host snapshot.  After every step the two are identical, which the
    block checksums confirm without moving the state; a flipped bit in the snapshot is located."""
    n = 3 * (1 << 20) + 4099
    seed = 0x25100606
    live = {a: synth.fill(seed, 1, a, 0, n, DEV) for a in ("W", "M", "V")}
    live["V"] = live["V"].abs()                       # second moments are non-negative
    live["P"] = live["W"].to(torch.bfloat16)
    snap = {a: live[a].cpu().clone() for a in live}   # the snapshot starts as a copy (step 0)
    ges = grad_bits // 8
    gdt = torch.float32 if ges == 4 else torch.bfloat16
    peer = torch.empty(n, dtype=gdt, device=DEV)      # receive buffer on the snapshot holder's device
    host_g = torch.empty(n, dtype=gdt).pin_memory()
    st = stream()
    for t in range(1, 5):
        g = (synth.fill(seed + t, 7, "M", 0, n, DEV) * 0.05).to(gdt)
        h = ew.ew_adam_hyper(3e-4, 0.9, 0.95, 1e-8, 0.1, t)
        ew.ew_grad_ship(g, peer, host_g, n * ges, st)                                   # Grad D2D, D2H
        ew.ew_adam_step(live["P"], live["W"], live["M"], live["V"], g, ges, n, h, st)   # Step
        torch.cuda.synchronize()
        ew.ew_adam_replay_host(snap["P"], snap["W"], snap["M"], snap["V"], host_g, ges, n, h, 0)   # Update Param
        for a in ("W", "M", "V"):
            assert torch.equal(live[a].cpu().view(torch.int32), snap[a].view(torch.int32)), f"{a} differs at step {t}"
        assert torch.equal(live["P"].cpu().view(torch.int16), snap["P"].view(torch.int16))
    # online verification: host checksums of the snapshot against the live shard's bytes
    for a in ("W", "P"):
        nbytes = n * live[a].element_size()
        ck = torch.from_numpy(ew.ew_checksum_host(snap[a], nbytes).view(np.uint64).view(np.int64).reshape(-1, 2)).to(DEV)
        got = torch.zeros_like(ck)
        n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
        bad = torch.full((4,), -1, dtype=torch.int64, device=DEV)
        diffs = torch.zeros((4, 2), dtype=torch.int64, device=DEV)
        ew.ew_verify(live[a], nbytes, ck, got, n_bad, bad, diffs, 4, st)
        assert int(n_bad.item()) == 0
        o = nbytes // 2 + 5
        snap[a].view(torch.uint8)[o] ^= 0x08
        ck = torch.from_numpy(ew.ew_checksum_host(snap[a], nbytes).view(np.uint64).view(np.int64).reshape(-1, 2)).to(DEV)
        ew.ew_verify(live[a], nbytes, ck, got, n_bad, bad, diffs, 4, st)
        assert int(n_bad.item()) == 1 and int(bad[0].item()) == o >> 20
