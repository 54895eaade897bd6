"""Host side of the gradient-shipping snapshot (CPU only): ew_adam_replay_host and ew_checksum_host
against the oracle, bit for bit."""
import numpy as np
import pytest

import paper_2510_00606_amd as ew
from oracle import adam, checksum

F = np.float32


def same_hyper(h, o):
    return all(np.float32(getattr(h, k)) == o[k] for k in ("lr", "beta1", "beta2", "omb1", "omb2", "eps", "wd", "bias1", "bias2"))


def test_hyper_matches_oracle():
    for args in ((1e-3, 0.9, 0.999, 1e-8, 0.0, 1), (3e-4, 0.9, 0.95, 1e-8, 0.1, 7), (1e-2, 0.5, 0.25, 1e-6, 0.01, 1000),
                 (1.0, 0.0, 0.0, 0.0, 0.0, 2)):
        assert same_hyper(ew.ew_adam_hyper(*args), adam.hyper(*args))
    with pytest.raises(ew.EwError):
        ew.ew_adam_hyper(1e-3, 0.9, 0.999, 1e-8, 0.0, 0)
    with pytest.raises(ew.EwError):
        ew.ew_adam_hyper(1e-3, 1.0, 0.999, 1e-8, 0.0, 1)


@pytest.mark.parametrize("grad_bits", [32, 16])
@pytest.mark.parametrize("n,threads", [(1, 1), (7, 3), (4096, 1), (100003, 5), (1 << 20, 0)])
def test_replay_is_bit_exact(n, threads, grad_bits):
    rng = np.random.default_rng(n + grad_bits)
    w = (rng.standard_normal(n) * 0.02).astype(F)
    m = np.zeros(n, F)
    v = np.zeros(n, F)
    p = np.zeros(n, np.uint16)
    ow, om, ov = w.copy(), m.copy(), v.copy()
    for t in range(1, 6):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, n)).astype(F)
        if t == 3:
            g[:: max(1, n // 7)] = 0.0
        if grad_bits == 16:
            g = (g.view(np.uint32) >> 16).astype(np.uint16)
        args = (3e-4, 0.9, 0.95, 1e-8, 0.1, t)
        ow, om, ov, op = adam.step(ow, om, ov, g, adam.hyper(*args))
        ew.ew_adam_replay_host(p, w, m, v, g, grad_bits // 8, n, ew.ew_adam_hyper(*args), threads)
        assert np.array_equal(w.view(np.uint32), ow.view(np.uint32)), f"w differs at step {t}"
        assert np.array_equal(m.view(np.uint32), om.view(np.uint32)) and np.array_equal(v.view(np.uint32), ov.view(np.uint32))
        assert np.array_equal(p, op)


def test_replay_special_values():
    # zeros, denormals, huge values, infinities and NaNs go through the same operations on both sides
    w = np.array([0.0, -0.0, 1e-40, 1e38, -1e38, np.inf, np.nan, 1.0], F)
    m = np.array([0.0, 1e-45, -1e-40, 1e30, 0.0, 0.0, 0.0, np.nan], F)
    v = np.array([0.0, 0.0, 1e-45, 1e38, 0.0, 0.0, 1.0, 1.0], F)
    g = np.array([0.0, 1e-30, -1e-20, 1e19, -3e38, 1.0, 1.0, np.inf], F)
    p = np.zeros(8, np.uint16)
    args = (1e-3, 0.9, 0.999, 1e-8, 0.01, 2)
    ow, om, ov, op = adam.step(w.copy(), m.copy(), v.copy(), g, adam.hyper(*args))
    ew.ew_adam_replay_host(p, w, m, v, g, 4, 8, ew.ew_adam_hyper(*args), 1)
    fin = ~np.isnan(ow)
    assert np.array_equal(np.isnan(w), np.isnan(ow)) and np.array_equal(w[fin].view(np.uint32), ow[fin].view(np.uint32))
    assert np.array_equal(np.isnan(m), np.isnan(om)) and np.array_equal(np.isnan(v), np.isnan(ov))
    assert np.array_equal(p[fin], op[fin]) and all((int(x) & 0x7F80) == 0x7F80 and int(x) & 0x7F for x in p[~fin])


@pytest.mark.parametrize("nbytes", [0, 1, 8, 9, (1 << 20) - 3, 1 << 20, (1 << 20) + 8, 5 * (1 << 20) + 12345])
def test_host_checksums(nbytes):
    raw = np.random.default_rng(nbytes).integers(0, 256, nbytes, dtype=np.uint8)
    for threads in (1, 3, 0):
        got = ew.ew_checksum_host(raw, nbytes, threads)
        want = checksum.block_checksums(raw)
        assert np.array_equal(got["sum"], want[:, 0]) and np.array_equal(got["xr"], want[:, 1])
