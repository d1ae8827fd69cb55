"""Pins for the hidden-state read-out oracle (oracle/lm_head_oracle.py).

As in oracle_pins.py every check takes the oracle *module*, so the same checks run on broken copies.
Nothing here re-types the oracle: brute force with exact summation on tiny shapes, closed forms, torch's
float64 linear + cross-entropy and autograd, finite differences, and invariances of the softmax.
"""
from __future__ import annotations

import math

import numpy as np
import torch

RNG = np.random.default_rng(20260514)


def _case(R=5, D=3, V=7, seed=0, p_valid=0.8):
    rng = np.random.default_rng(seed)
    h = rng.normal(0, 1.0, size=(R, D))
    w = rng.normal(0, 1.0, size=(V, D))
    y = rng.integers(0, V, size=R)
    valid = rng.random(R) < p_valid
    valid[0] = True
    g = rng.normal(0, 1.0, size=R)
    return h, w, y, valid, g


def pin_brute_force(L):
    """Plain definition with Python floats and exact summation; D != V != R so a transposed operand cannot pass."""
    h, w, y, _, _ = _case(R=4, D=3, V=6, seed=1)
    logp, lse = L.token_logprob(h, w, y)
    for n in range(4):
        z = [math.fsum(h[n, d] * w[v, d] for d in range(3)) for v in range(6)]
        s = math.fsum(math.exp(v) for v in z)
        assert abs(lse[n] - math.log(s)) < 1e-12
        assert abs(logp[n] - math.log(math.exp(z[y[n]]) / s)) < 1e-12


def pin_square_shapes_orientation(L):
    """With D == V a product taken against W instead of W^T has the right shape but the wrong values."""
    rng = np.random.default_rng(2)
    h = rng.normal(size=(3, 4))
    w = rng.normal(size=(4, 4))
    z = L.logits(h, w)
    for n in range(3):
        for v in range(4):
            assert abs(z[n, v] - math.fsum(h[n, d] * w[v, d] for d in range(4))) < 1e-12


def pin_closed_forms(L):
    """Equal rows of W give the uniform law; a unit hidden vector reads out one column of W."""
    rng = np.random.default_rng(3)
    V, D = 9, 4
    w = np.tile(rng.normal(size=(1, D)), (V, 1))
    h = rng.normal(size=(5, D))
    y = rng.integers(0, V, size=5)
    logp, lse = L.token_logprob(h, w, y)
    np.testing.assert_allclose(logp, -math.log(V), rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, h @ w[0] + math.log(V), rtol=0, atol=1e-12)
    w = rng.normal(size=(V, D))
    e = np.zeros((1, D))
    e[0, 2] = 1.0
    col = w[:, 2]
    logp, lse = L.token_logprob(e, w, [5])
    assert abs(lse[0] - math.log(math.fsum(math.exp(c) for c in col))) < 1e-12
    assert abs(logp[0] - (col[5] - lse[0])) < 1e-12


def pin_library_cross_entropy(L):
    """torch float64: cross_entropy(linear(h, W) / T) is -log pi(y)."""
    h, w, y, valid, _ = _case(R=8, D=5, V=13, seed=4)
    for inv_t in (1.0, 0.7, 1.9):
        logp, lse = L.token_logprob(h, w, y, valid, inv_t)
        zt = torch.nn.functional.linear(torch.from_numpy(h), torch.from_numpy(w)) * inv_t
        ce = torch.nn.functional.cross_entropy(zt, torch.from_numpy(y), reduction="none").numpy()
        np.testing.assert_allclose(logp[valid], -ce[valid], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[valid], torch.logsumexp(zt, dim=1).numpy()[valid], rtol=0, atol=1e-12)
        assert np.all(logp[~valid] == 0.0) and np.all(lse[~valid] == 0.0)


def pin_invariances(L):
    """Adding one vector to every row of W shifts all logits of a row equally: log-probs unchanged, lse shifted
    by <h, c>.  Probabilities sum to one."""
    h, w, y, _, _ = _case(R=6, D=4, V=10, seed=5)
    c = RNG.normal(size=4)
    logp0, lse0 = L.token_logprob(h, w, y)
    logp1, lse1 = L.token_logprob(h, w + c, y)
    np.testing.assert_allclose(logp1, logp0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse1 - lse0, h @ c, rtol=0, atol=1e-12)
    total = np.zeros(6)
    for v in range(10):
        total += np.exp(L.token_logprob(h, w, np.full(6, v))[0])
    np.testing.assert_allclose(total, 1.0, rtol=0, atol=1e-12)


def pin_grads_autograd(L):
    """float64 autograd of L = -sum_t g_t log pi(y_t) over valid rows."""
    h, w, y, valid, g = _case(R=7, D=4, V=9, seed=6)
    for inv_t in (1.0, 1.6):
        ht = torch.from_numpy(h).requires_grad_(True)
        wt = torch.from_numpy(w).requires_grad_(True)
        lp = torch.log_softmax(torch.nn.functional.linear(ht, wt) * inv_t, dim=1)[torch.arange(7), torch.from_numpy(y)]
        loss = -(torch.from_numpy(g) * lp)[torch.from_numpy(valid)].sum()
        loss.backward()
        dh, dw = L.grads(h, w, y, g, valid, inv_t)
        np.testing.assert_allclose(dh, ht.grad.numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=0, atol=1e-12)
        assert np.all(dh[~valid] == 0.0)


def pin_grads_finite_difference(L):
    """Central differences of the scalar objective built from the oracle's own forward (chain-rule check that
    does not rely on torch)."""
    h, w, y, valid, g = _case(R=4, D=3, V=5, seed=7)
    inv_t = 1.3

    def objective(hh, ww):
        lp, _ = L.token_logprob(hh, ww, y, valid, inv_t)
        return -float((g * lp)[valid].sum())

    dh, dw = L.grads(h, w, y, g, valid, inv_t)
    eps = 1e-6
    for (n, d) in [(0, 0), (1, 2), (3, 1)]:
        hp, hm = h.copy(), h.copy()
        hp[n, d] += eps
        hm[n, d] -= eps
        fd = (objective(hp, w) - objective(hm, w)) / (2 * eps)
        assert abs(fd - dh[n, d]) < 1e-7
    for (v, d) in [(0, 0), (2, 1), (4, 2), (int(y[0]), 1)]:
        wp, wm = w.copy(), w.copy()
        wp[v, d] += eps
        wm[v, d] -= eps
        fd = (objective(h, wp) - objective(h, wm)) / (2 * eps)
        assert abs(fd - dw[v, d]) < 1e-7


def pin_gradient_structure(L):
    """Each row of dL/dz sums to zero; dL/dh of a row is g/T times (expected embedding - embedding of y)."""
    h, w, y, _, g = _case(R=5, D=4, V=8, seed=8)
    inv_t = 0.8
    dz = L.dlogits(h, w, y, g, None, inv_t)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, rtol=0, atol=1e-12)
    dh, _ = L.grads(h, w, y, g, None, inv_t)
    for n in range(5):
        probs = np.array([math.exp(L.token_logprob(h[n:n + 1], w, [v], None, inv_t)[0][0]) for v in range(8)])
        expect = g[n] * inv_t * (probs @ w - w[y[n]])
        np.testing.assert_allclose(dh[n], expect, rtol=0, atol=1e-12)


ALL_PINS = [
    pin_brute_force,
    pin_square_shapes_orientation,
    pin_closed_forms,
    pin_library_cross_entropy,
    pin_invariances,
    pin_grads_autograd,
    pin_grads_finite_difference,
    pin_gradient_structure,
]
