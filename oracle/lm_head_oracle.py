"""CPU fp64 oracle for the log-probability step taken straight from the last hidden states.
TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the CPU-baseline leg of the benchmark may
call it; the GPU library shares no code with it and never imports it.

Alg. 1 ("Adaptive Coefficient Estimation") needs log pi_train(o_t) for every generated token.  In the
models the paper trains, the distribution over the vocabulary is the softmax of a linear read-out of the
final hidden state h_t with the output-embedding matrix W (one row per vocabulary entry):

    z_t[v]   = sum_d h_t[d] W[v, d]                       (logits)
    log pi(v | .) = z_t[v] / T - log sum_u exp(z_t[u] / T)

The functions below are that definition written out in numpy float64, with a library matrix product as
the contraction step.  The gradient functions apply the chain rule to
L = - sum_t g_t log pi(y_t | .) with g held constant, which is the form the AIS-GRPO loss takes once the
per-row coefficient g (clip gate, advantage, rectification weight, 1/|o_i|, 1/B of Eq. 19) is known:

    dL/dz_t[v] = (g_t / T) (pi(v) - 1[v = y_t])
    dL/dh_t    = sum_v dL/dz_t[v] W[v, :]
    dL/dW[v,:] = sum_t dL/dz_t[v] h_t

Readings: rows with valid == 0 are not evaluated (log-prob and lse reported as 0, zero gradient);
temperature divides the logits before the softmax.

Pins: tests/lm_head_pins.py (brute force with exact summation, closed forms, a library cross-entropy,
float64 autograd, finite differences, invariances).
"""
from __future__ import annotations

import numpy as np


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def logits(hidden, weight):
    """The read-out that produces the logits of Alg. 1 ("Compute full-precision log-probs"; the model families of
    Sec. 4.1): z[t, v] = <h_t, W[v, :]> ; hidden [R, D], weight [V, D] -> [R, V]."""
    h = _f64(hidden)
    w = _f64(weight)
    assert h.ndim == 2 and w.ndim == 2 and h.shape[1] == w.shape[1]
    return h @ w.T


def token_logprob(hidden, weight, y, valid=None, inv_temperature: float = 1.0):
    """(log pi(y_t), lse_t) per row from hidden states and the output embedding: the log-probs of Alg. 1 ("Compute
    full-precision log-probs") with the logits formed on the way."""
    z = logits(hidden, weight)
    R = z.shape[0]
    y = np.asarray(y, dtype=np.int64)
    valid = np.ones(R, dtype=bool) if valid is None else np.asarray(valid).astype(bool)
    logp = np.zeros(R)
    lse = np.zeros(R)
    for n in range(R):
        if not valid[n]:
            continue
        row = z[n] * inv_temperature
        m = row.max()
        lse[n] = m + np.log(np.exp(row - m).sum())
        logp[n] = row[y[n]] - lse[n]
    return logp, lse


def dlogits(hidden, weight, y, g, valid=None, inv_temperature: float = 1.0):
    """dL/dz for L = -sum_t g_t log pi(y_t), the form Eq. 19 takes once the per-token coefficients g_t are fixed (Alg. 1,
    "Policy Update"): (g_t / T)(softmax - onehot); zero rows where not valid."""
    z = logits(hidden, weight)
    R = z.shape[0]
    y = np.asarray(y, dtype=np.int64)
    g = _f64(g)
    valid = np.ones(R, dtype=bool) if valid is None else np.asarray(valid).astype(bool)
    dz = np.zeros_like(z)
    for n in range(R):
        if not valid[n]:
            continue
        row = z[n] * inv_temperature
        m = row.max()
        prob = np.exp(row - m)
        prob /= prob.sum()
        prob[int(y[n])] -= 1.0
        dz[n] = (g[n] * inv_temperature) * prob
    return dz


def grads(hidden, weight, y, g, valid=None, inv_temperature: float = 1.0):
    """(dL/dhidden [R, D], dL/dweight [V, D]): the gradient of Eq. 19 carried through the read-out z = H W^T by the chain
    rule."""
    dz = dlogits(hidden, weight, y, g, valid, inv_temperature)
    d_hidden = dz @ _f64(weight)
    d_weight = dz.T @ _f64(hidden)
    return d_hidden, d_weight
