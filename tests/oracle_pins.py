"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

Every function takes the oracle *module* as its argument, so that the same
checks can be run on deliberately broken copies of the oracle (see
test_oracle_mutants.py): a pin that no plausible mistake can trip is not a pin.

None of these checks re-types an oracle formula.  They use closed forms worked
out by hand from Eq. 12-19, library routines (scipy's logsumexp, torch's float64
autograd), brute force on tiny vocabularies, finite differences, and the
invariants the paper states (Prop. 2, Prop. 3, the two end-points alpha = 0 / 1), and
exact enumeration of the expectation that the appendix's analysis is about.
"""
from __future__ import annotations

import math

import numpy as np
import torch
from scipy.special import logsumexp as scipy_logsumexp

RNG = np.random.default_rng(20260513)


def _rand_batch(B=4, G=2, V=11, lo=1, hi=6, seed=0, p_valid=0.8):
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi + 1, size=B)
    cu = np.concatenate([[0], np.cumsum(lens)])
    R = int(cu[-1])
    z = rng.normal(0, 2.0, size=(R, V))
    y = rng.integers(0, V, size=R)
    valid = rng.random(R) < p_valid
    logp_roll = rng.normal(0, 0.3, size=R)  # filled in by callers that need a consistent value
    rewards = (rng.random(B) < 0.5).astype(np.float64)
    if G > 1:  # make sure at least one group is mixed so that gradients are not all zero
        rewards[0], rewards[1] = 1.0, 0.0
    return z, y, valid, cu, logp_roll, rewards


# --------------------------------------------------------------------------- O1
def pin_logprob_library(O):
    """log-softmax agrees with scipy's logsumexp and with torch float64 log_softmax."""
    z = RNG.normal(0, 3, size=(7, 33))
    y = RNG.integers(0, 33, size=7)
    logp, lse = O.token_logprob(z, y)
    np.testing.assert_allclose(lse, scipy_logsumexp(z, axis=1), rtol=0, atol=1e-12)
    ref = torch.log_softmax(torch.from_numpy(z), dim=1).numpy()[np.arange(7), y]
    np.testing.assert_allclose(logp, ref, rtol=0, atol=1e-12)


def pin_logprob_brute_force(O):
    """Tiny vocabularies: probability from the plain definition exp(z_y) / sum_v exp(z_v) with exact summation."""
    for V in (1, 2, 3, 8):
        z = RNG.normal(0, 1.5, size=(5, V))
        y = RNG.integers(0, V, size=5)
        logp, _ = O.token_logprob(z, y)
        for n in range(5):
            prob = math.exp(z[n, y[n]]) / math.fsum(math.exp(v) for v in z[n])
            assert abs(logp[n] - math.log(prob)) < 1e-12


def pin_logprob_invariants(O):
    """Rows exponentiate and sum to 1; adding a constant to a row changes nothing; a flat row gives -ln V;
    huge logits do not overflow."""
    z = RNG.normal(0, 4, size=(6, 50))
    _, lse = O.token_logprob(z, np.zeros(6, dtype=int))
    assert np.all(np.abs(np.exp(z - lse[:, None]).sum(1) - 1.0) < 1e-12)
    y = RNG.integers(0, 50, size=6)
    lp0, _ = O.token_logprob(z, y)
    lp1, _ = O.token_logprob(z + 123.456, y)
    np.testing.assert_allclose(lp0, lp1, atol=1e-10)
    flat = np.full((2, 37), 3.25)
    lp, _ = O.token_logprob(flat, np.array([0, 36]))
    np.testing.assert_allclose(lp, -math.log(37), atol=1e-14)
    big = np.array([[1000.0, 999.0, -1000.0]])
    lp, lse = O.token_logprob(big, np.array([1]))
    assert np.isfinite(lp).all() and abs(lp[0] - (-1.0 - math.log1p(math.exp(-1.0)))) < 1e-12


def pin_logprob_mask_and_temperature(O):
    """Rows that are not evaluated return exactly 0 and never touch their token id; temperature scales logits."""
    z = RNG.normal(0, 2, size=(4, 9))
    y = np.array([3, -1, 10 ** 9, 8])
    valid = np.array([1, 0, 0, 1], dtype=np.uint8)
    lp, lse = O.token_logprob(z, y, valid)
    assert lp[1] == 0 and lp[2] == 0 and lse[1] == 0 and lse[2] == 0
    lp_t, _ = O.token_logprob(z, y, valid, inv_temperature=1 / 0.9)
    ref, _ = O.token_logprob(z / 0.9, y, valid)
    np.testing.assert_allclose(lp_t, ref, atol=1e-12)
    try:
        O.token_logprob(z, np.array([3, 0, 0, 9]), valid)
    except ValueError:
        pass
    else:
        raise AssertionError("out-of-range token on an evaluated row must be rejected")


# --------------------------------------------------------------------------- O2
def pin_ratio_identity_and_truncation(O):
    """Identical policies give rho = w_bar = 1 bit-exactly (Prop. 3); rho above C is cut to exactly C (Eq. 10);
    rho below C is untouched; an enormous gap does not produce inf or nan in w_bar."""
    lp = RNG.normal(-2, 1, size=100)
    d, rho, wbar = O.importance_weights(lp, lp.copy(), 5.0)
    assert np.all(d == 0) and np.all(rho == 1.0) and np.all(wbar == 1.0)
    d, rho, wbar = O.importance_weights(np.array([0.0, 0.0, 0.0, 0.0]),
                                        np.array([-math.log(7.0), -math.log(2.0), math.log(4.0), -800.0]), 5.0)
    np.testing.assert_allclose(rho[:3], [7.0, 2.0, 0.25], rtol=1e-14)
    np.testing.assert_allclose(wbar, [5.0, 2.0, 0.25, 5.0], rtol=1e-14)
    assert wbar[0] == 5.0 and wbar[3] == 5.0


# --------------------------------------------------------------------------- O3
def pin_advantages(O):
    """Eq. 3: advantages of a group sum to zero; with k ones among G Bernoulli rewards they are
    1 - k/G and -k/G; the optional normalised form has unit population std."""
    r = np.array([1, 0, 0, 1, 1, 1, 0, 0, 0, 0, 0, 0], dtype=float)   # two groups of 6: k = 4 and k = 0
    a = O.group_advantages(r, 6)
    np.testing.assert_allclose(a[:6], [1 / 3, -2 / 3, -2 / 3, 1 / 3, 1 / 3, 1 / 3], atol=1e-15)
    assert np.all(a[6:] == 0)
    assert abs(a[:6].sum()) < 1e-15
    r2 = RNG.normal(size=24)
    a2 = O.group_advantages(r2, 8)
    assert np.all(np.abs(a2.reshape(3, 8).sum(1)) < 1e-14)
    # group boundaries are consecutive blocks of G, not strided
    np.testing.assert_allclose(a2[:8], r2[:8] - r2[:8].mean(), atol=1e-15)
    a3 = O.group_advantages(r2, 8, adv_mode=1, eps_std=0.0)
    np.testing.assert_allclose(a3.reshape(3, 8).std(axis=1), 1.0, atol=1e-12)
    # eps_std = 0 and a group whose rewards are all equal: 0/0 is read as 0, the other group is unaffected
    a4 = O.group_advantages(r, 6, adv_mode=1, eps_std=0.0)
    assert np.all(a4[6:] == 0) and np.all(np.isfinite(a4)) and abs(a4[:6].std() - 1.0) < 1e-12


# --------------------------------------------------------------------------- O4
def _two_point(O, d_plus, d_minus, n_half=6, **kw):
    """Half the tokens have A = +1 and log-ratio d_plus, half have A = -1 and log-ratio d_minus."""
    p = O.Params(**kw)
    N = 2 * n_half
    lp_roll = RNG.normal(-1, 0.5, size=N)
    d = np.array([d_plus, d_minus] * n_half)
    lp_train = lp_roll + d
    cu = np.arange(N + 1)                 # N responses of one row each, advantages alternate
    adv = np.array([1.0, -1.0] * n_half)
    return O.diagnostics(lp_train, lp_roll, None, cu, adv, p), p


def pin_diag_two_point_closed_form(O):
    """Hand-worked case (defaults C=5, delta=0.02, gamma=1.2, eps=1e-6, beta=1):
    half the tokens A=+1, w_bar=1; half A=-1, w_bar=3.
      mean_w = 2, var_w = 1, CV^2 = 1/4           => alpha_ess = 1/sqrt(1.25)         (Eq. 12)
      ESS ratio = (sum w)^2 / (N sum w^2) = 0.8
      d_bar = ln(3)/2 > delta                      => alpha_mis = 1                    (Eq. 13-14)
      A w_bar in {1, -3}: pstd = 2; pstd(A) = 1    => Delta-sigma = 2/(1+1e-6)         (Eq. 15)
      alpha_var = (Delta-sigma - 1.2)/1.2                                              (Eq. 16)
      alpha = alpha_ess - alpha_var                                                    (Eq. 17)
    """
    out, p = _two_point(O, 0.0, math.log(3.0))
    assert out["n_valid"] == 12
    assert abs(out["mean_w"] - 2.0) < 1e-12 and abs(out["var_w"] - 1.0) < 1e-12
    assert abs(out["cv2"] - 0.25) < 1e-12
    assert abs(out["alpha_ess"] - 1 / math.sqrt(1.25)) < 1e-12
    assert abs(out["ess_ratio"] - 0.8) < 1e-12
    assert abs(out["dbar"] - 0.5 * math.log(3.0)) < 1e-12
    assert out["alpha_mis"] == 1.0
    dsig = 2.0 / (1.0 + 1e-6)
    assert abs(out["dsigma"] - dsig) < 1e-12
    assert abs(out["alpha_var"] - (dsig - 1.2) / 1.2) < 1e-12
    assert abs(out["alpha"] - (1 / math.sqrt(1.25) - (dsig - 1.2) / 1.2)) < 1e-12
    assert abs(out["alpha"] - 0.2277621909982) < 1e-9        # the same number, written out
    assert out["clip_frac"] == 0.0


def pin_diag_small_mismatch_closed_form(O):
    """d = +-0.01: w_bar = e^{+-0.01}; mean = cosh, pvar = sinh^2 => CV^2 = tanh^2(0.01);
    d_bar = 0.01 = delta/2 => alpha_mis = 1/2 (Eq. 14, the linear branch);
    A w_bar in {e^.01, -e^-.01}: pstd = cosh(0.01) => Delta-sigma < gamma => alpha_var = 0 (Eq. 16);
    alpha = alpha_ess / 2 (Eq. 17)."""
    out, _ = _two_point(O, 0.01, -0.01)
    t2 = math.tanh(0.01) ** 2
    assert abs(out["cv2"] - t2) < 1e-12
    assert abs(out["alpha_mis"] - 0.5) < 1e-12
    assert abs(out["dsigma"] - math.cosh(0.01) / (1 + 1e-6)) < 1e-12
    assert out["alpha_var"] == 0.0
    assert abs(out["alpha"] - 0.5 / math.sqrt(1 + t2)) < 1e-12


def pin_diag_beta_and_clip(O):
    """Eq. 17: beta scales the variance penalty; the reliability gate is clipped at 0 before the product.
    Two-point case with w_bar in {1, 5} (rho = 9 truncated at C = 5), A in {+1, -1}:
      mean 3, pvar 4 => CV^2 = 4/9, alpha_ess = 1/sqrt(13/9); A w in {1,-5}: pstd 3 => Delta-sigma ~ 3
      alpha_var = (3/(1+1e-6) - 1.2)/1.2 ~ 1.5 > alpha_ess => alpha = 0 for beta = 1, alpha_ess - 0.1 alpha_var for beta = 0.1."""
    out, _ = _two_point(O, 0.0, math.log(9.0))
    assert abs(out["alpha_ess"] - 1 / math.sqrt(13 / 9)) < 1e-12
    av = (3.0 / (1 + 1e-6) - 1.2) / 1.2
    assert abs(out["alpha_var"] - av) < 1e-12
    assert out["alpha"] == 0.0
    assert abs(out["clip_frac"] - 0.5) < 1e-15
    out2, _ = _two_point(O, 0.0, math.log(9.0), beta_var=0.1)
    assert abs(out2["alpha"] - (1 / math.sqrt(13 / 9) - 0.1 * av)) < 1e-12
    out3, _ = _two_point(O, 0.0, math.log(9.0), alpha_override=0.3)
    assert out3["alpha"] == 0.3 and abs(out3["alpha_ess"] - out["alpha_ess"]) < 1e-15


def pin_diag_ess_identity_and_ranges(O):
    """Eq. 12 states two expressions for alpha_ess; the second is evaluated independently here as
    sum(w) / sqrt(N sum(w^2)).  alpha and the three signals stay in their ranges on random inputs;
    masked rows and response boundaries are honoured (count, n_valid)."""
    for seed in range(8):
        z, y, valid, cu, _, rewards = _rand_batch(B=6, G=3, seed=seed, hi=9)
        R = z.shape[0]
        rng = np.random.default_rng(100 + seed)
        lp_roll = rng.normal(-2, 1, size=R)
        lp_train = lp_roll + rng.normal(0, 0.5 * (seed + 1) / 4, size=R)
        adv = O.group_advantages(rewards, 3)
        p = O.Params()
        out = O.diagnostics(lp_train, lp_roll, valid, cu, adv, p)
        w = np.minimum(np.exp(lp_train - lp_roll), p.C)[valid]
        ess_sqrt = w.sum() / math.sqrt(w.size * (w ** 2).sum())
        assert abs(out["alpha_ess"] - ess_sqrt) < 1e-12
        assert abs(out["ess_ratio"] - ess_sqrt ** 2) < 1e-12
        assert 0.0 <= out["alpha"] <= 1.0 and 0.0 < out["alpha_ess"] <= 1.0
        assert 0.0 <= out["alpha_mis"] <= 1.0 and out["alpha_var"] >= 0.0
        assert out["n_valid"] == int(valid.sum())
        assert list(out["count"]) == [int(valid[cu[i]:cu[i + 1]].sum()) for i in range(6)]
        # token-level statistics: A is broadcast to the tokens of its response (std over tokens, not responses)
        a_tok = np.repeat(adv, np.diff(cu))[valid]
        assert abs(out["std_a"] - np.sqrt(np.mean((a_tok - a_tok.mean()) ** 2))) < 1e-12
        aw = a_tok * w
        assert abs(out["std_aw"] - np.sqrt(np.mean(aw ** 2) - np.mean(aw) ** 2)) < 1e-9


def pin_diag_degenerate(O):
    """Uniform weights => alpha_ess = 1 exactly; identical policies => d_bar = 0 => alpha = 0 (Eq. 14, 17);
    all rewards equal => std(A) = 0 => Delta-sigma = 0/(0+eps) = 0 => alpha_var = 0; no valid rows => alpha = 0."""
    lp = RNG.normal(-1, 1, size=10)
    cu = np.array([0, 5, 10])
    p = O.Params()
    out = O.diagnostics(lp, lp, None, cu, np.array([0.5, -0.5]), p)
    assert out["alpha_ess"] == 1.0 and out["dbar"] == 0.0 and out["alpha_mis"] == 0.0 and out["alpha"] == 0.0
    # w_bar == 1 everywhere: Delta-sigma = std(A)/(std(A)+eps) < 1 < gamma
    assert out["alpha_var"] == 0.0 and abs(out["dsigma"] - 0.5 / (0.5 + 1e-6)) < 1e-12
    out = O.diagnostics(lp + 0.3, lp, None, cu, np.array([0.0, 0.0]), p)
    assert out["dsigma"] == 0.0 and out["alpha_var"] == 0.0 and out["alpha_mis"] == 1.0
    assert abs(out["alpha"] - 1.0) < 1e-12          # constant ratio: CV = 0
    out = O.diagnostics(lp, lp, np.zeros(10, dtype=bool), cu, np.array([0.5, -0.5]), p)
    assert out["n_valid"] == 0 and out["alpha"] == 0.0 and list(out["count"]) == [0, 0]
    # eps_std = 0 and all advantages equal: Delta-sigma is 0/0, read as 0 (nothing to amplify), alpha stays finite
    import dataclasses
    p0 = dataclasses.replace(p, eps_std=0.0)
    out = O.diagnostics(lp + 0.3, lp, None, cu, np.array([0.0, 0.0]), p0)
    assert out["dsigma"] == 0.0 and out["alpha_var"] == 0.0 and abs(out["alpha"] - 1.0) < 1e-12


def pin_diag_vanishing_weights(O):
    """A trainer far below the sampler on every token.  Ratios of 1e-98 are still numbers: CV^2 is scale-invariant,
    so it equals the CV^2 of the same log-ratios shifted back by a constant (which sit near 1).  Beyond the range of
    exp every ratio is exactly 0 and CV^2 is 0/0: read as 0, alpha_ess = 1, and nothing is NaN."""
    lp_roll = RNG.normal(-2, 1, size=12)
    jitter = RNG.normal(0, 0.3, size=12)
    cu = np.array([0, 6, 12])
    adv = np.array([0.5, -0.5])
    p = O.Params()
    near = O.diagnostics(lp_roll + jitter - 0.5, lp_roll, None, cu, adv, p)      # ratios around e^-0.5: none truncated
    far = O.diagnostics(lp_roll + jitter - 225.0, lp_roll, None, cu, adv, p)     # the same ratios times e^-224.5
    assert far["mean_w"] < 1e-90 and abs(far["cv2"] - near["cv2"]) < 1e-9 * near["cv2"]
    assert abs(far["alpha_ess"] - near["alpha_ess"]) < 1e-12
    gone = O.diagnostics(lp_roll + jitter - 2000.0, lp_roll, None, cu, adv, p)
    assert gone["mean_w"] == 0.0 and gone["cv2"] == 0.0 and gone["alpha_ess"] == 1.0 and gone["ess_ratio"] == 1.0
    assert gone["alpha_mis"] == 1.0 and gone["alpha"] == 1.0 and all(np.isfinite(float(v)) for k, v in gone.items()
                                                                      if k != "count")


def pin_mismatch_metrics(O):
    """The two logged mismatch metrics (Sec. 3.1, the training-dynamics figure).  Closed form: every token has
    pi_roll = 0.1; half of them pi_train = 0.3, half 0.1  =>  mean(log pi_roll - log pi_train) = -ln(3)/2 and
    E|dp| = 0.1.  Statistically: on tokens drawn from pi_roll the KL estimate converges to the exact
    KL(pi_roll || pi_train) of two small categorical distributions."""
    n = 10
    lr = np.full(n, math.log(0.1))
    lt = np.where(np.arange(n) % 2 == 0, math.log(0.3), math.log(0.1))
    out = O.diagnostics(lt, lr, None, np.array([0, n]), np.array([0.0]), O.Params())
    assert abs(out["kl_roll_train"] + 0.5 * math.log(3.0)) < 1e-12
    assert abs(out["mean_abs_dp"] - 0.1) < 1e-12
    rng = np.random.default_rng(7)
    p_roll = np.array([0.4, 0.25, 0.15, 0.1, 0.07, 0.03])
    p_train = np.array([0.3, 0.3, 0.2, 0.05, 0.1, 0.05])
    exact = float(np.sum(p_roll * np.log(p_roll / p_train)))
    tok = rng.choice(6, size=200_000, p=p_roll)
    out = O.diagnostics(np.log(p_train)[tok], np.log(p_roll)[tok], None, np.array([0, tok.size]), np.array([0.0]),
                        O.Params())
    sd = float(np.sqrt(np.sum(p_roll * np.log(p_roll / p_train) ** 2) - exact ** 2) / math.sqrt(tok.size))
    assert exact > 0.01 and abs(out["kl_roll_train"] - exact) < 5 * sd
    exact_dp = float(np.sum(p_roll * np.abs(p_train - p_roll)))
    assert abs(out["mean_abs_dp"] - exact_dp) < 2e-3


# --------------------------------------------------------------------------- O5
def pin_mixed_weight_bounds(O):
    """Prop. 2: 0 <= 1 - alpha + alpha w_bar <= 1 + alpha (C - 1); alpha = 0 gives 1, alpha = 1 gives w_bar (Eq. 9)."""
    C = 5.0
    wbar = np.minimum(np.exp(RNG.normal(0, 2, size=1000)), C)
    for alpha in (0.0, 0.25, 1.0):
        wt = O.mixed_weights(wbar, alpha)
        assert np.all(wt >= 1 - alpha - 1e-15) and np.all(wt <= 1 + alpha * (C - 1) + 1e-12)
    assert np.all(O.mixed_weights(wbar, 0.0) == 1.0)
    np.testing.assert_allclose(O.mixed_weights(wbar, 1.0), wbar, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(O.mixed_weights(wbar, 0.4), 0.6 + 0.4 * wbar, rtol=1e-12)
    assert np.all(O.mixed_weights(wbar, 0.4, valid=np.zeros(1000)) == 0.0)


# ------------------------------------------------------------------------ O6/O7
def _torch_objective(z, y, valid, cu, wtilde, adv, B, clip_eps, logp_old=None, inv_t=1.0,
                     logp_ref=None, beta_kl=0.0):
    """Eq. 19 typed independently in torch float64 (weights are constants), negated.  Used with autograd."""
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    logp_all = torch.log_softmax(zt * inv_t, dim=1)
    total = torch.zeros((), dtype=torch.float64)
    for i in range(B):
        rows = [n for n in range(cu[i], cu[i + 1]) if valid[n]]
        if not rows:
            continue
        acc = torch.zeros((), dtype=torch.float64)
        for n in rows:
            lp = logp_all[n, int(y[n])]
            ratio = torch.exp(lp - (lp.detach() if logp_old is None else logp_old[n]))
            A = float(adv[i])
            surr = torch.minimum(ratio * A, torch.clamp(ratio, 1 - clip_eps, 1 + clip_eps) * A)
            term = float(wtilde[n]) * surr
            if beta_kl:
                q = float(logp_ref[n]) - lp
                term = term - beta_kl * (torch.exp(q) - q - 1)
            acc = acc + term
        total = total + acc / len(rows)
    loss = -total / B
    loss.backward()
    return float(loss.detach()), zt.grad.numpy()


def pin_grad_autograd(O):
    """loss and dlogits against float64 autograd of an independently typed Eq. 19, with rho_on == 1,
    with a stale log pi_old on both sides of the clip range, with temperature, and with the KL term."""
    for case in range(5):
        z, y, valid, cu, _, rewards = _rand_batch(B=4, G=2, V=7, seed=40 + case)
        R = z.shape[0]
        y[~valid] = -1
        p = O.Params(clip_eps=0.2)
        kw = {}
        if case == 2:
            p.inv_temperature = 1 / 0.9
        logp, _ = O.token_logprob(z, y, valid, p.inv_temperature)
        rng = np.random.default_rng(case)
        logp_roll = logp + rng.normal(0, 0.4, size=R)
        logp_old = logp_ref = None
        if case in (1, 3):
            logp_old = logp + rng.normal(0, 0.25, size=R)     # ratios on both sides of 1 +- 0.2
            kw["logp_old"] = logp_old
        if case in (3, 4):
            p.beta_kl = 0.05
            logp_ref = logp + rng.normal(0, 0.3, size=R)
            kw["logp_ref"] = logp_ref
        out = O.ais_grpo(z, y, valid, cu, logp_roll, rewards, 2, p, **kw)
        ref_loss, ref_grad = _torch_objective(z, y, valid, cu, out["wtilde"], out["adv"], 4, p.clip_eps,
                                              logp_old, p.inv_temperature, logp_ref, p.beta_kl)
        assert abs(out["loss"] - ref_loss) < 1e-12 * max(1.0, abs(ref_loss))
        np.testing.assert_allclose(out["dz"], ref_grad, rtol=1e-9, atol=1e-13)
        assert np.abs(out["dz"]).max() > 0
        assert np.all(out["dz"][~valid] == 0)
        assert np.all(np.abs(out["dz"].sum(axis=1)) < 1e-12)           # sum_v (p_v - 1[v=y]) = 0


def pin_grad_finite_difference(O):
    """Central differences of the loss in z with alpha, w_tilde and A frozen (they come from detached tensors)."""
    z, y, valid, cu, _, rewards = _rand_batch(B=4, G=2, V=5, seed=77, hi=3)
    R, V = z.shape
    y[~valid] = 0
    p = O.Params()
    logp0, _ = O.token_logprob(z, y, valid)
    rng = np.random.default_rng(5)
    logp_roll = logp0 + rng.normal(0, 0.5, size=R)
    logp_old = logp0 + rng.normal(0, 0.15, size=R)
    out = O.ais_grpo(z, y, valid, cu, logp_roll, rewards, 2, p, logp_old=logp_old)
    alpha, count, adv = out["diag"]["alpha"], out["diag"]["count"], out["adv"]
    seq = O.rows_to_responses(cu, R)

    def frozen_loss(zz):
        lp, _ = O.token_logprob(zz, y, valid)
        obj, _, _, _ = O.row_terms(lp, logp_old, None, out["wtilde"], adv[seq], p)
        tot = 0.0
        for i in range(4):
            rows = [n for n in range(cu[i], cu[i + 1]) if valid[n]]
            if rows:
                tot += sum(obj[n] for n in rows) / len(rows)
        return -tot / 4

    h = 1e-6
    for n in range(R):
        for v in range(V):
            zp, zm = z.copy(), z.copy()
            zp[n, v] += h
            zm[n, v] -= h
            fd = (frozen_loss(zp) - frozen_loss(zm)) / (2 * h)
            assert abs(fd - out["dz"][n, v]) < 2e-8, (n, v, fd, out["dz"][n, v])


def pin_endpoints_and_on_policy(O):
    """alpha = 0 is vanilla GRPO and alpha = 1 is token-level truncated IS (Eq. 8, Eq. 9, text after Eq. 19),
    each coded here from its own formula; with identical policies every alpha gives the same gradient (Prop. 3)."""
    z, y, valid, cu, _, rewards = _rand_batch(B=4, G=2, V=9, seed=9)
    R, V = z.shape
    y[~valid] = 0
    logp, _ = O.token_logprob(z, y, valid)
    logp_roll = logp + np.random.default_rng(1).normal(0, 0.8, size=R)
    prob = np.exp(z - scipy_logsumexp(z, axis=1, keepdims=True))
    onehot = np.zeros((R, V))
    onehot[np.arange(R), y] = 1
    adv = rewards.reshape(2, 2) - rewards.reshape(2, 2).mean(1, keepdims=True)
    a_row = np.repeat(adv.reshape(-1), np.diff(cu))
    cnt = np.array([valid[cu[i]:cu[i + 1]].sum() for i in range(4)])
    per_row = np.where(valid, 1.0 / (4 * np.maximum(np.repeat(cnt, np.diff(cu)), 1)), 0.0)
    grpo = (per_row * a_row)[:, None] * (prob - onehot)                       # d/dz of -(1/B) sum (1/|o|) sum A log p
    tis_w = np.minimum(np.exp(logp - logp_roll), 5.0)
    tis = (per_row * a_row * tis_w)[:, None] * (prob - onehot)                # Eq. 8 with the GRPO normalisation
    o0 = O.ais_grpo(z, y, valid, cu, logp_roll, rewards, 2, O.Params(alpha_override=0.0))
    o1 = O.ais_grpo(z, y, valid, cu, logp_roll, rewards, 2, O.Params(alpha_override=1.0))
    np.testing.assert_allclose(o0["dz"], grpo, rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(o1["dz"], tis, rtol=1e-10, atol=1e-15)
    assert np.abs(grpo - tis).max() > 1e-4
    # interpolation (Eq. 9): the alpha-gradient is the convex combination of the two end-points
    oh = O.ais_grpo(z, y, valid, cu, logp_roll, rewards, 2, O.Params(alpha_override=0.3))
    np.testing.assert_allclose(oh["dz"], 0.7 * grpo + 0.3 * tis, rtol=1e-10, atol=1e-15)
    # loss value at the end-points: -(1/B) sum_i mean_t (w A)
    l1 = -sum(np.mean((tis_w * a_row)[cu[i]:cu[i + 1]][valid[cu[i]:cu[i + 1]]]) for i in range(4) if cnt[i]) / 4
    assert abs(o1["loss"] - l1) < 1e-12
    same = [O.ais_grpo(z, y, valid, cu, logp, rewards, 2, O.Params(alpha_override=a))["dz"] for a in (0.0, 0.3, 1.0)]
    assert np.array_equal(same[0], same[1]) and np.array_equal(same[0], same[2])
    adaptive = O.ais_grpo(z, y, valid, cu, logp, rewards, 2)
    assert adaptive["diag"]["alpha"] == 0.0 and np.array_equal(adaptive["dz"], same[0])


def pin_exact_expectation_is_policy_gradient(O):
    """Appendix, Prop. 1's set-up, by exact enumeration.  One prompt, one position, a group that holds every token of a
    small vocabulary once.  Weighting response x by pi_roll(x) turns the batch sum into the expectation under the
    rollout policy, so: with alpha = 1 and C above every ratio the estimate *is* the on-policy gradient
    grad_z E_{x ~ pi_train}[A(x)] = pi * (A - <pi, A>) (a softmax Jacobian applied to A, coded from that
    formula); with alpha = 0 it is the same expression under pi_roll's sampling, i.e. sum_x pi_roll(x) A(x) (e_x - pi),
    whose distance from the first is the mismatch bias b_0; a general alpha interpolates the two."""
    V = 7
    rng = np.random.default_rng(77)
    z_row = rng.normal(0, 1.5, size=V)
    pi_train = np.exp(z_row - scipy_logsumexp(z_row))
    z_roll = z_row + rng.normal(0, 0.7, size=V)
    pi_roll = np.exp(z_roll - scipy_logsumexp(z_roll))
    rewards = np.array([1.0, 0.0, 0.0, 1.0, 1.0, 0.0, 1.0])
    A = rewards - rewards.mean()                                    # Eq. 3 over the one group
    z = np.tile(z_row, (V, 1))                                      # every response sees the same context
    y = np.arange(V)
    cu = np.arange(V + 1)
    valid = np.ones(V, dtype=bool)
    eye = np.eye(V)

    def expectation(alpha, C):
        out = O.ais_grpo(z, y, valid, cu, np.log(pi_roll), rewards, V, O.Params(alpha_override=alpha, C=C))
        # the loss is -(1/B) sum_i (...): undo the sign and the 1/B, weight response x by pi_roll(x)
        return -(V * pi_roll[:, None] * out["dz"]).sum(axis=0)

    C_big = 2.0 * (pi_train / pi_roll).max()
    g_true = pi_train * (A - pi_train @ A)
    g0 = (pi_roll * A) @ (eye - pi_train[None, :])
    np.testing.assert_allclose(expectation(1.0, C_big), g_true, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(expectation(0.0, C_big), g0, rtol=1e-12, atol=1e-15)
    assert np.abs(g0 - g_true).max() > 1e-2                         # the bias b_0 is really there
    np.testing.assert_allclose(expectation(0.4, C_big), 0.6 * g0 + 0.4 * g_true, rtol=1e-12, atol=1e-15)
    # truncation (Eq. 10) leaves a residual bias b_1: ratios above C are cut, so the estimate moves off g_true
    C_small = 1.0 + 0.5 * ((pi_train / pi_roll).max() - 1.0)
    g1 = (pi_roll * np.minimum(pi_train / pi_roll, C_small) * A) @ (eye - pi_train[None, :])
    np.testing.assert_allclose(expectation(1.0, C_small), g1, rtol=1e-12, atol=1e-15)
    assert np.abs(g1 - g_true).max() > 1e-4
    # the score function has mean zero under its own policy: a constant advantage carries no gradient
    assert np.abs(pi_train @ (eye - pi_train[None, :])).max() < 1e-15


def pin_sampler_trainer_ratio_at_rollout_checkpoint(O):
    """Alg. 1 takes the sampler-trainer ratio at theta_old and Sec. 3.2 calls the two ratios orthogonal: with a
    stale log pi_old, (a) a rollout engine without precision gap (log pi_roll = log pi_old) gives w_tilde = 1 for
    any theta and any alpha, i.e. plain GRPO with its old-new ratio; (b) w_tilde, alpha and every diagnostic do not
    move when theta does; (c) w_tilde equals 1 + alpha (min(exp(log pi_old - log pi_roll), C) - 1) row by row."""
    z, y, valid, cu, _, rewards = _rand_batch(B=4, G=2, V=9, seed=91)
    R = z.shape[0]
    y[~valid] = 0
    rng = np.random.default_rng(91)
    logp0, _ = O.token_logprob(z, y, valid)
    logp_old = logp0 + rng.normal(0, 0.3, size=R)
    for alpha in (0.3, 1.0, -1.0):
        p = O.Params(alpha_override=alpha)
        out = O.ais_grpo(z, y, valid, cu, logp_old.copy(), rewards, 2, p, logp_old=logp_old)      # (a)
        assert np.all(out["wtilde"][valid] == 1.0)
        ref = O.ais_grpo(z, y, valid, cu, logp_old.copy(), rewards, 2, O.Params(alpha_override=0.0), logp_old=logp_old)
        np.testing.assert_allclose(out["dz"], ref["dz"], rtol=1e-13, atol=1e-16)
        assert np.abs(ref["dz"]).max() > 0
    logp_roll = logp_old + rng.normal(0, 0.5, size=R)
    p = O.Params()
    a = O.ais_grpo(z, y, valid, cu, logp_roll, rewards, 2, p, logp_old=logp_old)
    b = O.ais_grpo(z + rng.normal(0, 0.7, size=z.shape), y, valid, cu, logp_roll, rewards, 2, p, logp_old=logp_old)   # (b)
    assert np.array_equal(a["wtilde"], b["wtilde"]) and a["diag"]["alpha"] == b["diag"]["alpha"] > 0
    for k in ("mean_w", "cv2", "dbar", "dsigma", "alpha_ess", "alpha_mis", "alpha_var", "kl_roll_train"):
        assert a["diag"][k] == b["diag"][k], k
    assert not np.allclose(a["dz"], b["dz"])
    want = 1.0 + a["diag"]["alpha"] * (np.minimum(np.exp(logp_old - logp_roll), p.C) - 1.0)              # (c)
    np.testing.assert_allclose(a["wtilde"][valid], want[valid], rtol=1e-14)
    assert np.abs(want[valid] - 1.0).max() > 0.05


def pin_clip_region(O):
    """Tokens whose old-new ratio left the trust region on the penalised side get no gradient (Eq. 19):
    A > 0 and rho_on > 1 + eps, or A < 0 and rho_on < 1 - eps; on the other side the gradient is rho_on A w."""
    p = O.Params(clip_eps=0.2)
    logp = np.zeros(4)
    logp_old = -np.log(np.array([1.5, 1.5, 0.5, 0.5]))            # rho_on = 1.5, 1.5, 0.5, 0.5
    a = np.array([1.0, -1.0, 1.0, -1.0])
    wt = np.array([1.0, 2.0, 3.0, 4.0])
    obj, dobj, rho_on, s = O.row_terms(logp, logp_old, None, wt, a, p)
    np.testing.assert_allclose(rho_on, [1.5, 1.5, 0.5, 0.5], rtol=1e-14)
    np.testing.assert_allclose(s, [1.2, -1.5, 0.5, -0.8], rtol=1e-14)
    np.testing.assert_allclose(obj, [1.2, -3.0, 1.5, -3.2], rtol=1e-14)
    np.testing.assert_allclose(dobj, [0.0, -3.0, 1.5, 0.0], rtol=1e-14)


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
