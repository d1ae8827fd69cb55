"""CPU fp64 oracle for the AIS-GRPO hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the path computes, written from
the paper's equations in their order and notation, in numpy float64.  It exists
so that the GPU library can be checked against something that can be read side
by side with the paper.  It shares no code with the HIP path and must never be
imported by it: only the test-suite, the smoke check and the CPU-baseline leg of
the benchmark may call anything in here.

Steps (each function cites the passage it follows):

  O1  token log-probability         log pi_train(o_t)         Alg. 1 "full-precision log-probs"
  O2  sampler-trainer ratio         rho, w_bar = min(rho, C)  Eq. 7, Eq. 10, Alg. 1
  O3  group-relative advantage      A_i = r_i - mean_j r_j    Eq. 3
  O4  three diagnostics and alpha   Eq. 12-17
  O5  rectification weight          w_tilde = 1 + alpha (w_bar - 1)   Eq. 18, Alg. 1
  O6  AIS-GRPO loss                 Eq. 19 (sign flipped: a loss to minimise)
  O7  gradient of O6 w.r.t. logits  chain rule through log-softmax, alpha / w_tilde / A held constant
                                    (App. "Low-bit Rollout and AIS": signals come from detached tensors)

Readings where the paper is silent:
  * CV and std are population statistics (ddof = 0) over *valid token positions*;
    only ddof = 0 makes the two sides of Eq. 12 equal.
  * alpha is one scalar per batch (Eq. 17 carries no sample index).
  * beta in Eq. 17 has no published value: it is a parameter (default 1).
  * |o_i| is the number of evaluated positions of response i; a response with none contributes 0.
  * the 1/G sum and the expectation over prompts become 1/B with B = all responses passed.
  * log pi_old absent  =>  rho_on = 1 (first update after the rollout, theta = theta_old).
  * log pi_old given (theta has moved on from theta_old): the sampler-trainer ratio, the diagnostics and
    alpha are taken at theta_old, as Alg. 1 writes them, so w_bar = min(exp(log pi_old - log pi_roll), C)
    does not move during optimisation; only rho_on = exp(log pi_theta - log pi_old) does (Sec. 3.2: the two
    ratios are orthogonal).
  * the KL term of Eq. 19 names no estimator; the optional term here is the per-token
    k3 form exp(q) - q - 1 with q = log pi_ref - log pi_theta, averaged like the surrogate.
    Parity unpinned by the paper for that term (pinned here only by its own closed forms).
  * temperature: logits are multiplied by inv_temperature before the softmax.
  * quotients that are 0 / 0 for degenerate batches are read as 0: CV^2 when every truncated ratio is exactly 0,
    Delta-sigma and the normalised advantage when eps_std = 0 and the advantages (rewards of a group) are all equal.

Parity pins for every function are in tests/oracle_pins.py; numeric values of alpha
for a given input are not printed anywhere in the paper, so they are pinned by closed
forms worked out by hand from Eq. 12-17 for two-point weight distributions.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class Params:
    """Hyper-parameters; defaults from App. "AIS hyperparameters" and the hyper-parameter table."""

    C: float = 5.0            # IS truncation threshold, C >= 1 (Eq. 10)
    delta: float = 0.02       # saturation threshold of alpha_mis (Eq. 14)
    gamma: float = 1.2        # variance tolerance (Eq. 16)
    eps_std: float = 1e-6     # numerical stabiliser in Delta-sigma (Eq. 15)
    beta_var: float = 1.0     # beta of Eq. 17 (no published value)
    clip_eps: float = 0.2     # PPO clipping range (Eq. 19)
    adv_mode: int = 0         # 0: r - mean (Eq. 3); 1: (r - mean) / (pstd + eps_std)
    alpha_override: float = -1.0   # < 0: adaptive (Eq. 17); in [0,1]: forced (0 = GRPO, 1 = TIS, Eq. 8)
    inv_temperature: float = 1.0
    beta_kl: float = 0.0      # weight of the KL term of Eq. 19 (0 = omitted)


def _f64(x):
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------- O1
def token_logprob(z, y, valid=None, inv_temperature: float = 1.0):
    """log pi_train(o_t) for every evaluated row (Alg. 1, "Compute full-precision log-probs").

    z [R, V] logits (any float dtype, widened exactly to fp64), y [R] token ids,
    valid [R] (None = all rows).  Returns (logp [R], lse [R]) with 0 on rows that
    are not evaluated.  lse is the log-sum-exp of the temperature-scaled row; an
    evaluated row whose token id is outside [0, V) raises.
    """
    z = _f64(z)
    R, V = z.shape
    y = np.asarray(y).astype(np.int64)
    valid = np.ones(R, dtype=bool) if valid is None else np.asarray(valid).astype(bool)
    logp = np.zeros(R)
    lse = np.zeros(R)
    for n in range(R):
        if not valid[n]:
            continue
        if not (0 <= y[n] < V):
            raise ValueError(f"row {n}: token id {y[n]} outside [0, {V})")
        row = z[n] * inv_temperature
        m = row.max()
        lse[n] = m + np.log(np.exp(row - m).sum())
        logp[n] = row[y[n]] - lse[n]
    return logp, lse


# --------------------------------------------------------------------------- O2
def importance_weights(logp_train, logp_roll, C: float):
    """d = log pi_train - log pi_roll, rho = exp(d) (Eq. 7, Alg. 1), w_bar = min(rho, C) (Eq. 10)."""
    d = _f64(logp_train) - _f64(logp_roll)
    with np.errstate(over="ignore"):
        rho = np.exp(d)
    wbar = np.minimum(rho, C)
    return d, rho, wbar


# --------------------------------------------------------------------------- O3
def group_advantages(rewards, group_size: int, adv_mode: int = 0, eps_std: float = 1e-6):
    """A_i = r_i - mean of the G rewards of its prompt (Eq. 3, the unnormalised form the paper uses).
    adv_mode 1 divides by (population std of the group + eps_std)."""
    r = _f64(rewards)
    if r.size % group_size:
        raise ValueError("number of responses is not a multiple of the group size")
    g = r.reshape(-1, group_size)
    adv = g - g.mean(axis=1, keepdims=True)
    if adv_mode == 1:
        den = g.std(axis=1, keepdims=True) + eps_std
        # eps_std = 0 and a group with equal rewards: 0 / 0, read as 0 (the numerator is exactly 0)
        adv = np.where(den > 0.0, adv / np.where(den > 0.0, den, 1.0), 0.0)
    return adv.reshape(-1)


def rows_to_responses(cu_rows, n_rows: int):
    """seq[n] = index of the response that owns row n (the o_i of Eq. 19 that token position n belongs to)."""
    cu = np.asarray(cu_rows).astype(np.int64)
    seq = np.zeros(n_rows, dtype=np.int64)
    for i in range(cu.size - 1):
        seq[cu[i]:cu[i + 1]] = i
    return seq


# --------------------------------------------------------------------------- O4
def diagnostics(logp_train, logp_roll, valid, cu_rows, adv, p: Params):
    """The three signals and the mixing coefficient over the valid token positions of the batch.

    alpha_ess (Eq. 12), d_bar (Eq. 13), alpha_mis (Eq. 14), Delta-sigma (Eq. 15),
    alpha_var (Eq. 16), alpha (Eq. 17).  Returns a dict that also carries the
    logged statistics (mean/var of w_bar, CV^2, ESS ratio, share of truncated
    ratios) and count[i] = number of valid rows of response i.
    """
    logp_train = _f64(logp_train)
    R = logp_train.size
    valid = np.ones(R, dtype=bool) if valid is None else np.asarray(valid).astype(bool)
    cu = np.asarray(cu_rows).astype(np.int64)
    B = cu.size - 1
    seq = rows_to_responses(cu, R)
    d, rho, wbar = importance_weights(logp_train, logp_roll, p.C)
    count = np.array([int(valid[cu[i]:cu[i + 1]].sum()) for i in range(B)], dtype=np.int64)
    N = int(valid.sum())
    out = dict(n_valid=N, count=count)
    if N == 0:
        out.update(mean_w=0.0, var_w=0.0, cv2=0.0, ess_ratio=1.0, dbar=0.0, std_a=0.0, std_aw=0.0,
                   dsigma=0.0, alpha_ess=1.0, alpha_mis=0.0, alpha_var=0.0, clip_frac=0.0, alpha=0.0,
                   kl_roll_train=0.0, mean_abs_dp=0.0)
        if p.alpha_override >= 0:
            out["alpha"] = float(p.alpha_override)
        return out
    w = wbar[valid]
    a = _f64(adv)[seq][valid]                       # A broadcast to its tokens
    mean_w = w.mean()
    var_w = ((w - mean_w) ** 2).mean()              # population variance
    # every truncated ratio exactly 0 (exp underflow, a trainer hundreds of nats away from the sampler): CV^2 is
    # 0 / 0; read as 0, i.e. equal weights and alpha_ess = 1, the same convention as the empty batch above
    cv2 = (np.sqrt(var_w) / mean_w) ** 2 if mean_w > 0.0 else 0.0    # (std / mean)^2: mean^2 alone may underflow
    alpha_ess = (1.0 + cv2) ** -0.5                 # Eq. 12
    dbar = np.abs(d[valid]).mean()                  # Eq. 13
    alpha_mis = min(1.0, dbar / p.delta)            # Eq. 14
    std_a = a.std()
    std_aw = (a * w).std()
    # Eq. 15; with eps_std = 0 and all advantages equal the ratio is 0 / 0: nothing to amplify, read as 0
    dsigma = std_aw / (std_a + p.eps_std) if std_a + p.eps_std > 0.0 else 0.0
    alpha_var = max(0.0, (dsigma - p.gamma) / p.gamma)          # Eq. 16
    alpha = min(1.0, max(0.0, alpha_ess - p.beta_var * alpha_var)) * alpha_mis   # Eq. 17
    if p.alpha_override >= 0:
        alpha = float(p.alpha_override)
    out.update(mean_w=mean_w, var_w=var_w, cv2=cv2, ess_ratio=1.0 / (1.0 + cv2), dbar=dbar,
               std_a=std_a, std_aw=std_aw, dsigma=dsigma, alpha_ess=alpha_ess, alpha_mis=alpha_mis,
               alpha_var=alpha_var, clip_frac=float((rho[valid] > p.C).mean()), alpha=alpha)
    # the two mismatch metrics the paper plots next to the ESS ratio (Sec. 3.1, first paragraph):
    # KL(pi_roll || pi_train), estimated on the tokens the rollout policy sampled as the mean of
    # log pi_roll - log pi_train, and the mean absolute probability gap E|Delta p| of those tokens
    out["kl_roll_train"] = float((-d[valid]).mean())
    out["mean_abs_dp"] = float(np.abs(np.exp(logp_train[valid]) - np.exp(_f64(logp_roll)[valid])).mean())
    return out


# --------------------------------------------------------------------------- O5
def mixed_weights(wbar, alpha: float, valid=None):
    """w_tilde = 1 + alpha (w_bar - 1) (Eq. 18 / Alg. 1 "Rectification weight"); 0 on rows not evaluated."""
    wt = 1.0 + alpha * (_f64(wbar) - 1.0)
    if valid is not None:
        wt = np.where(np.asarray(valid).astype(bool), wt, 0.0)
    return wt


# --------------------------------------------------------------------------- O6
def row_terms(logp, logp_old, logp_ref, wtilde, a, p: Params):
    """Per-row surrogate s, old-new ratio rho_on, and d(row objective)/d(logp) before the 1/(B|o_i|) weight.

    s = min(rho_on A, clip(rho_on, 1 -+ eps) A) (Eq. 19).  The derivative of
    w_tilde * s w.r.t. logp is w_tilde * A * rho_on where the unclipped branch is
    the minimum (ties go to the unclipped branch) and 0 otherwise.  With a KL
    weight, k3 = exp(q) - q - 1, q = logp_ref - logp, is subtracted from the
    objective; d k3 / d logp = 1 - exp(q).
    """
    logp = _f64(logp)
    rho_on = np.ones_like(logp) if logp_old is None else np.exp(logp - _f64(logp_old))
    unclipped = rho_on * a
    clipped = np.clip(rho_on, 1.0 - p.clip_eps, 1.0 + p.clip_eps) * a
    s = np.minimum(unclipped, clipped)
    active = (unclipped <= clipped).astype(np.float64)
    obj = wtilde * s
    dobj = wtilde * a * rho_on * active
    if p.beta_kl != 0.0 and logp_ref is not None:
        q = _f64(logp_ref) - logp
        obj = obj - p.beta_kl * (np.exp(q) - q - 1.0)
        dobj = dobj - p.beta_kl * (1.0 - np.exp(q))
    return obj, dobj, rho_on, s


def loss_and_row_coeff(logp, logp_roll, logp_old, logp_ref, valid, cu_rows, adv, count, alpha, p: Params):
    """loss = -(1/B) sum_i (1/|o_i|) sum_{t valid} [ w_tilde s - beta_kl k3 ]  (Eq. 19, negated),
    w_tilde [R] and g [R] with  d loss / d z[n, v] = g_n (softmax(z_n)_v - 1[v = y_n]) * inv_temperature.
    The rectification weight comes from the sampler-trainer ratio at the checkpoint that generated the
    rollout (Alg. 1, "Sampler-Trainer ratio"): log pi_old where it is given, the current log-probs otherwise."""
    logp = _f64(logp)
    R = logp.size
    valid = np.ones(R, dtype=bool) if valid is None else np.asarray(valid).astype(bool)
    cu = np.asarray(cu_rows).astype(np.int64)
    B = cu.size - 1
    seq = rows_to_responses(cu, R)
    logp_at_rollout = logp if logp_old is None else _f64(logp_old)
    _, _, wbar = importance_weights(logp_at_rollout, logp_roll, p.C)
    wtilde = mixed_weights(wbar, alpha, valid)
    a = _f64(adv)[seq]
    obj, dobj, _, _ = row_terms(logp, logp_old, logp_ref, wtilde, a, p)
    cnt = _f64(count)[seq]
    with np.errstate(divide="ignore", invalid="ignore"):
        wgt = np.where(valid & (cnt > 0), 1.0 / (B * cnt), 0.0)
    loss = 0.0
    for i in range(B):                    # response by response, as Eq. 19 is written
        lo, hi = cu[i], cu[i + 1]
        loss -= float((wgt[lo:hi] * obj[lo:hi])[valid[lo:hi]].sum())
    g = np.where(valid, wgt * dobj, 0.0)
    return loss, wtilde, g


# --------------------------------------------------------------------------- O7
def dlogits_rows(z, lse, y, g, inv_temperature: float = 1.0):
    """d loss / d z for a block of rows, the chain rule on Eq. 19 through log pi = z_y / T - lse (Alg. 1, "Policy
    Update"): g_n inv_T (exp(inv_T z - lse) - onehot(y_n)); rows with g_n = 0 are 0."""
    z = _f64(z)
    R, V = z.shape
    g = _f64(g)
    dz = np.zeros((R, V))
    for n in range(R):
        if g[n] == 0.0:
            continue
        prob = np.exp(z[n] * inv_temperature - lse[n])
        prob[int(y[n])] -= 1.0
        dz[n] = (g[n] * inv_temperature) * prob
    return dz


# ----------------------------------------------------------------- whole path
def ais_grpo(z, y, valid, cu_rows, logp_roll, rewards, group_size: int, p: Optional[Params] = None,
             logp_old=None, logp_ref=None, want_dz: bool = True):
    """O1 ... O7 on one batch: Alg. 1 from "Compute full-precision log-probs" through "Policy Update" (Eq. 3, 7, 10,
    12-19) in the paper's order.  Returns a dict with every intermediate."""
    p = p or Params()
    logp, lse = token_logprob(z, y, valid, p.inv_temperature)
    adv = group_advantages(rewards, group_size, p.adv_mode, p.eps_std)
    # "Adaptive Coefficient Estimation" of Alg. 1 works on log pi_train(. | theta_old)
    diag = diagnostics(logp if logp_old is None else logp_old, logp_roll, valid, cu_rows, adv, p)
    loss, wtilde, g = loss_and_row_coeff(logp, logp_roll, logp_old, logp_ref, valid, cu_rows, adv,
                                         diag["count"], diag["alpha"], p)
    out = dict(logp=logp, lse=lse, adv=adv, diag=diag, loss=loss, wtilde=wtilde, g=g)
    if want_dz:
        out["dz"] = dlogits_rows(z, lse, y, g, p.inv_temperature)
    return out
