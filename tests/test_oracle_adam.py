"""Pins for oracle/adam.py (CPU only): closed forms, a float64 evaluation of the same formula,
torch.optim.AdamW as the library routine, and -- for the bf16 copy of the master weights -- a
hand-worked table of bit patterns plus an integer-only statement of round-to-nearest-even, neither of
which calls the conversion routine the oracle uses."""
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


# fp32 bit pattern -> bf16 bit pattern under round to nearest, ties to even (the upper 16 bits are
# kept; the lower 16 decide: above 0x8000 up, below down, exactly 0x8000 to the even neighbour).
# Worked by hand; sign-magnitude, so "up" means away from zero for either sign.
BF16_BY_HAND = [
    (0x00000000, 0x0000), (0x80000000, 0x8000),      # +0, -0
    (0x3F800000, 0x3F80), (0xC0490FDB, 0xC049),      # 1.0 exact; -pi: lower half 0x0FDB < 0x8000, down
    (0x3F808000, 0x3F80),                            # tie, kept half even: stays
    (0x3F818000, 0x3F82),                            # tie, kept half odd: up to the even neighbour
    (0x3F808001, 0x3F81), (0x3F807FFF, 0x3F80),      # just above / just below the half
    (0x3F817FFF, 0x3F81), (0x3F818001, 0x3F82),
    (0xBF808000, 0xBF80), (0xBF818000, 0xBF82),      # the same ties with the sign bit set
    (0x3F7FFFFF, 0x3F80),                            # 0.99999994: the carry runs through the mantissa into the exponent
    (0x3FFFFFFF, 0x4000),                            # 1.9999999 -> 2.0
    (0x3FFF8000, 0x4000),                            # tie at an all-ones mantissa (odd): up, exponent changes
    (0x7F7F7FFF, 0x7F7F),                            # stays the largest finite bf16
    (0x7F7F8000, 0x7F80),                            # tie at the largest finite bf16 (odd): up is infinity
    (0x7F7FFFFF, 0x7F80), (0xFF7FFFFF, 0xFF80),      # largest finite fp32 -> +-infinity
    (0x7F800000, 0x7F80), (0xFF800000, 0xFF80),      # infinities stay
    (0x00000001, 0x0000), (0x00007FFF, 0x0000),      # fp32 denormals below half of the smallest bf16 denormal
    (0x00008000, 0x0000),                            # tie between 0 and the smallest bf16 denormal: even is 0
    (0x00008001, 0x0001), (0x00018000, 0x0002),      # just above it; tie at an odd denormal: up
    (0x007FFFFF, 0x0080),                            # largest fp32 denormal -> smallest normal bf16
    (0x80008001, 0x8001),
]


def rne_bits_integer(u: int):
    """Round to nearest even stated on integers alone; None for NaNs."""
    if (u & 0x7FFFFFFF) > 0x7F800000:
        return None
    kept, rest = u >> 16, u & 0xFFFF
    if rest > 0x8000 or (rest == 0x8000 and kept & 1):
        kept += 1
    return kept


def test_bf16_rounding_by_hand():
    bits = np.array([b for b, _ in BF16_BY_HAND], np.uint32)
    got = adam.bf16_bits(bits.view(F))
    assert got.dtype == np.uint16
    assert got.tolist() == [w for _, w in BF16_BY_HAND]
    for b, w in BF16_BY_HAND:        # the table agrees with the integer rule (guards the table itself)
        assert rne_bits_integer(b) == w
    # NaNs stay NaNs (exponent all ones, mantissa not zero), whatever their payload
    nans = np.array([0x7FC00000, 0x7F800001, 0xFFC00000, 0x7FFFFFFF], np.uint32)
    for g in adam.bf16_bits(nans.view(F)).tolist():
        assert (g & 0x7F80) == 0x7F80 and (g & 0x007F) != 0


def test_bf16_rounding_matches_integer_rule_on_random_bits():
    rng = np.random.default_rng(16)
    bits = rng.integers(0, 1 << 32, 200_000, dtype=np.uint64).astype(np.uint32)
    # plenty of exact ties and near-ties, which uniform bits hit with probability 2^-16 only
    ties = (rng.integers(0, 1 << 16, 50_000, dtype=np.uint64).astype(np.uint32) << np.uint32(16)) | np.uint32(0x8000)
    near = ties + rng.integers(-1, 2, len(ties)).astype(np.int64).astype(np.uint32)
    bits = np.concatenate([bits, ties, near])
    got = adam.bf16_bits(bits.view(F)).tolist()
    n = 0
    for b, g in zip(bits.tolist(), got):
        w = rne_bits_integer(b)
        if w is not None:
            assert g == w, hex(b)
            n += 1
    assert n > 290_000
