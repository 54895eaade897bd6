"""Mixed-precision Adam step in plain numpy fp32 (CPU oracle for the gradient-shipping snapshot).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Sec. 5.1 keeps the snapshot of a neighbour's optimizer partition up to date by shipping the
neighbour's GRADIENT shard and replaying the optimizer update on the copy, instead of copying the
(at least four times larger) Adam state.  That only works if the replay gives the same bits as the
update the owner applied to its live state, so the step is pinned down to single IEEE fp32
operations in a fixed order, each rounded on its own (no fused multiply-add):

    m   <- beta1*m + (1-beta1)*g
    v   <- beta2*v + (1-beta2)*(g*g)
    den <- sqrt(v * bias2) + eps          bias1 = 1/(1-beta1^t), bias2 = 1/(1-beta2^t), rounded to fp32
    w   <- w - lr * ((m * bias1) / den + weight_decay * w)
    p   <- bf16(w), round to nearest even

(the textbook Adam of Kingma & Ba with bias correction and decoupled weight decay).  numpy's
float32 add, multiply, divide and sqrt are single correctly rounded IEEE operations, which is what
makes this file a definition rather than an approximation.
"""
from __future__ import annotations

import numpy as np
import torch

F = np.float32


def hyper(lr, beta1, beta2, eps, weight_decay, step: int):
    """The nine fp32 scalars of one step, derived in float64 and rounded once."""
    return {
        "lr": F(lr), "beta1": F(beta1), "beta2": F(beta2), "omb1": F(1.0 - float(F(beta1))),
        "omb2": F(1.0 - float(F(beta2))), "eps": F(eps), "wd": F(weight_decay),
        "bias1": F(1.0 / (1.0 - float(F(beta1)) ** step)), "bias2": F(1.0 / (1.0 - float(F(beta2)) ** step)),
    }


def grad_to_f32(g: np.ndarray) -> np.ndarray:
    """fp32 gradients pass through; bf16 gradients (uint16 bit patterns) widen exactly."""
    if g.dtype == np.float32:
        return g
    if g.dtype == np.uint16:
        return (g.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise TypeError("gradient must be float32 or bf16 bits as uint16")


def bf16_bits(w: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 through torch's conversion routine (pinned by a hand-worked
    table of bit patterns and an integer-only rule in the tests, not by calling torch again)."""
    return torch.from_numpy(np.ascontiguousarray(w)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def step(w, m, v, g, h):
    """One update of (w, m, v) float32 arrays (returned, not in place) and the bf16 bits of w."""
    g = grad_to_f32(g)
    with np.errstate(all="ignore"):
        m = F(h["beta1"]) * m + F(h["omb1"]) * g
        v = F(h["beta2"]) * v + F(h["omb2"]) * (g * g)
        den = np.sqrt(v * F(h["bias2"])) + F(h["eps"])
        upd = (m * F(h["bias1"])) / den
        w = w - F(h["lr"]) * (upd + F(h["wd"]) * w)
    assert m.dtype == v.dtype == w.dtype == np.float32
    return w, m, v, bf16_bits(w)
