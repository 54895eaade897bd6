"""Pins for oracle/adam.py (CPU only): closed forms, a float64 evaluation of the same formula, and
torch.optim.AdamW as the library routine."""
import numpy as np
import torch

from oracle import adam

F = np.float32


def test_first_step_closed_form():
    # zero state, t = 1: m_hat = g, v_hat = g*g, so the update is lr * g / (|g| + eps)
    h = adam.hyper(1e-3, 0.9, 0.999, 1e-8, 0.0, 1)
    g = np.array([0.5, -2.0, 1e-3, 3.0], F)
    w0 = np.array([1.0, 1.0, -1.0, 0.0], F)
    w, m, v, p = adam.step(w0, np.zeros(4, F), np.zeros(4, F), g, h)
    assert np.allclose(m, 0.1 * g, rtol=1e-6) and np.allclose(v, 0.001 * g * g, rtol=1e-4)
    assert np.allclose(w, w0 - 1e-3 * np.sign(g), rtol=0, atol=2e-7)


def test_zero_gradient_decays_moments_and_applies_weight_decay_only():
    h = adam.hyper(1e-2, 0.9, 0.99, 1e-8, 0.1, 5)
    w0, m0, v0 = np.array([2.0, -4.0], F), np.zeros(2, F), np.zeros(2, F)
    w, m, v, _ = adam.step(w0, m0, v0, np.zeros(2, F), h)
    assert (m == 0).all() and (v == 0).all()
    assert np.allclose(w, w0 * (1 - 1e-2 * 0.1), rtol=1e-6)      # decoupled decay: w -= lr * wd * w
    m1 = np.array([1.0, -1.0], F)
    _, m, v, _ = adam.step(w0, m1, np.ones(2, F), np.zeros(2, F), adam.hyper(1e-2, 0.5, 0.25, 1e-8, 0, 3))
    assert (m == F(0.5) * m1).all() and (v == F(0.25)).all()


def test_against_float64_and_torch_adamw():
    rng = np.random.default_rng(0)
    n = 4096
    w = (rng.standard_normal(n) * 0.02).astype(F)
    m, v = np.zeros(n, F), np.zeros(n, F)
    w64, m64, v64 = w.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    tw = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.AdamW([tw], lr=3e-4, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    for t in range(1, 21):
        g = (rng.standard_normal(n) * 1e-3).astype(F)
        h = adam.hyper(3e-4, 0.9, 0.95, 1e-8, 0.1, t)
        w, m, v, p = adam.step(w, m, v, g, h)
        b1, b2 = float(F(0.9)), float(F(0.95))
        m64 = b1 * m64 + (1 - b1) * g
        v64 = b2 * v64 + (1 - b2) * g.astype(np.float64) ** 2
        w64 = w64 - 3e-4 * ((m64 / (1 - b1 ** t)) / (np.sqrt(v64 / (1 - b2 ** t)) + 1e-8) + 0.1 * w64)
        tw.grad = torch.from_numpy(g.copy())
        opt.step()
    assert np.allclose(w, w64, rtol=0, atol=5e-7)
    assert np.allclose(m, m64, rtol=1e-5, atol=1e-9) and np.allclose(v, v64, rtol=1e-5, atol=1e-12)
    # torch's AdamW orders the operations differently (decay first, bias corrections folded into
    # the step size), so agreement is to rounding, not to the bit
    assert np.allclose(w, tw.detach().numpy(), rtol=0, atol=2e-6)
    # bf16 copy = torch's own rounding of the new master weights
    assert np.array_equal(p, torch.from_numpy(w).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_bf16_gradient_widens_exactly():
    bits = np.array([0x3F80, 0xBF00, 0x0000, 0x3DCC], np.uint16)          # 1.0, -0.5, 0, ~0.0996
    g = adam.grad_to_f32(bits)
    assert g.tolist()[:3] == [1.0, -0.5, 0.0] and abs(g[3] - 0.0996) < 1e-3
    h = adam.hyper(1e-3, 0.9, 0.999, 1e-8, 0.0, 1)
    a = adam.step(np.ones(4, F), np.zeros(4, F), np.zeros(4, F), bits, h)
    b = adam.step(np.ones(4, F), np.zeros(4, F), np.zeros(4, F), g, h)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_hyper_scalars():
    h = adam.hyper(1e-3, 0.9, 0.999, 1e-8, 0.01, 10)
    assert h["omb1"] == F(1.0 - float(F(0.9))) and abs(float(h["bias1"]) - 1 / (1 - 0.9 ** 10)) < 1e-6
    assert abs(float(h["bias2"]) - 1 / (1 - 0.999 ** 10)) < 1e-3 * float(h["bias2"])
