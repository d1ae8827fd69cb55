"""The per-row scalar kernels (plan, two-level diagnostics reduction, row coefficients, loss) at sizes the
logits-based parity tests cannot reach: millions of rows, tens of thousands of responses, responses that span
thousands of tiles, empty responses.  They need no logits: seeded log-probs go straight into ais_diagnostics and
ais_grpo_row_scale and are compared with the CPU oracle (exact inputs, so the relative tolerance applies as is)."""
import numpy as np
import pytest
import torch

import oracle.ais_oracle as O
from paper_2605_13907_amd import binding as B
from tests import parity as P

pytestmark = pytest.mark.gpu

CASES = {
    # name: (responses, group size, length recipe, share of valid rows)
    "long_responses": (64, 8, ("lognormal", 9.5, 0.8), 1.0),          # ~13 k rows each, up to ~100 tiles
    "one_huge_response": (1, 1, ("fixed", 2_000_000), 0.6),            # ~2,000 tiles of one response
    "many_short": (20_000, 8, ("uniform", 0, 5), 0.8),                 # empty responses included
    "mixed": (512, 4, ("lognormal", 6.0, 1.5), 0.5),
}


def lengths(recipe, n, rng):
    if recipe[0] == "fixed":
        return np.full(n, recipe[1], dtype=np.int64)
    if recipe[0] == "uniform":
        return rng.integers(recipe[1], recipe[2] + 1, size=n).astype(np.int64)
    return np.minimum(np.floor(rng.lognormal(recipe[1], recipe[2], size=n)), 300_000).astype(np.int64)


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("stale", [False, True])
def test_scalars_at_scale(name, stale):
    n_resp, G, recipe, p_valid = CASES[name]
    rng = np.random.default_rng(sum(map(ord, name)) + (7 if stale else 0))
    L = lengths(recipe, n_resp, rng)
    cu = np.concatenate([[0], np.cumsum(L)]).astype(np.int64)
    R = int(cu[-1])
    valid = (rng.random(R) < p_valid).astype(np.uint8)
    logp_roll = -np.abs(rng.normal(2.0, 1.5, size=R)).astype(np.float32)
    logp_train = (logp_roll + rng.normal(0.0, 0.05, size=R) + (rng.random(R) < 0.01) * rng.normal(0, 2.0, size=R)).astype(np.float32)
    logp_train = np.minimum(logp_train, 0.0).astype(np.float32)
    logp_train[valid == 0] = 0.0
    logp_roll[valid == 0] = 0.0
    rewards = (rng.random(n_resp) < 0.4).astype(np.float32)
    kw = dict(beta_kl=0.04, clip_eps=0.2) if stale else {}
    p = B.default_params(**kw)
    logp_old = logp_ref = None
    if stale:
        logp_old = (logp_train + rng.normal(0, 0.15, size=R)).astype(np.float32)
        logp_ref = (logp_train + rng.normal(0, 0.1, size=R)).astype(np.float32)
    print(f"{name}: rows {R}, responses {n_resp}, longest {int(L.max())}, empty {int((L == 0).sum())}", flush=True)

    op = P.oracle_params(p)
    adv_ref = O.group_advantages(rewards.astype(np.float64), G, op.adv_mode, op.eps_std)
    rd = O.diagnostics(logp_train, logp_roll, valid, cu, adv_ref, op)
    loss_ref, wt_ref, g_ref = O.loss_and_row_coeff(logp_train.astype(np.float64), logp_roll.astype(np.float64),
                                                   None if logp_old is None else logp_old.astype(np.float64),
                                                   None if logp_ref is None else logp_ref.astype(np.float64),
                                                   valid, cu, adv_ref, rd["count"], rd["alpha"], op)

    ctx = B.AisContext()
    t = lambda a: None if a is None else torch.from_numpy(a).cuda()
    adv, count, diag = ctx.diagnostics(t(logp_train), t(logp_roll), t(valid), t(cu), t(rewards), G, p)
    loss, wtilde, g = ctx.grpo_row_scale(t(logp_train), t(logp_roll), t(valid), t(cu), adv, count, diag, p,
                                         logp_old=t(logp_old), logp_ref=t(logp_ref))
    torch.cuda.synchronize()
    d = ctx.read_diag(diag)
    assert ctx.status() == 0
    ctx.close()

    assert d["n_valid"] == rd["n_valid"] == int(valid.sum())
    assert count.cpu().tolist() == [int(c) for c in rd["count"]]
    np.testing.assert_allclose(P.to_np64(adv), adv_ref, rtol=0, atol=1e-6)
    for k in ("mean_w", "var_w", "cv2", "ess_ratio", "dbar", "std_a", "std_aw", "dsigma", "alpha_ess", "alpha_mis",
              "clip_frac", "mean_abs_dp", "alpha_var", "alpha"):
        P.rel_close(d[k], rd[k], rel=1e-9 if k in ("clip_frac",) else 1e-6, floor=1e-9, what=k)
    P.rel_close(d["kl_roll_train"], rd["kl_roll_train"], rel=1e-6, floor=rd["dbar"], what="kl_roll_train")
    np.testing.assert_allclose(P.to_np64(wtilde), wt_ref, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(P.to_np64(g), g_ref * op.inv_temperature, rtol=2e-6, atol=1e-30)
    scale = float(np.sum(np.abs(adv_ref)) / n_resp) + op.beta_kl
    assert abs(float(loss.item()) - loss_ref) <= 1e-6 * max(abs(loss_ref), scale, 1e-12), (float(loss.item()), loss_ref)


@pytest.mark.parametrize("shift", [-40.0, -0.3125, 0.0, 0.078125, 9.0])     # dyadic: the sum below is exact
@pytest.mark.parametrize("n_resp,length", [(2, 3), (8, 700), (64, 5_000)])
def test_equal_weights_have_no_spread(shift, n_resp, length):
    """Every valid row has the same ratio (all truncated at C for shift = 9, all exp(shift) otherwise) and the valid
    rows sit in responses of equal advantage: the spread statistics are those of a constant.  The variance of equal
    numbers is 0 whatever the way the rows were cut into tiles, and the advantage-weighted spread of Eq. 15 is
    0 / (0 + eps): rounding noise divided by the 1e-6 stabiliser would show up here as a spurious amplification."""
    rng = np.random.default_rng(n_resp * 1000 + length)
    cu = (np.arange(n_resp + 1) * length).astype(np.int64)
    R = int(cu[-1])
    logp_roll = -np.abs(rng.normal(2.0, 1.0, size=R)).astype(np.float32)
    logp_roll = np.round(logp_roll * 64) / 64 - 50.0                  # multiples of 1/64: adding `shift` is exact in fp32
    logp_train = (logp_roll + np.float32(shift)).astype(np.float32)
    assert np.all(logp_train.astype(np.float64) - logp_roll.astype(np.float64) == float(np.float32(shift)))
    rewards = np.tile(np.array([1.0, 0.0], dtype=np.float32), n_resp // 2)
    valid = np.zeros(R, dtype=np.uint8)
    for i in range(0, n_resp, 2):                                     # only the rewarded responses are evaluated
        valid[cu[i]:cu[i + 1]] = rng.random(length) < 0.7
    valid[0] = 1
    p = B.default_params()
    op = P.oracle_params(p)
    adv_ref = O.group_advantages(rewards.astype(np.float64), 2, op.adv_mode, op.eps_std)
    rd = O.diagnostics(logp_train, logp_roll.astype(np.float32), valid, cu, adv_ref, op)
    ctx = B.AisContext()
    t = lambda a: torch.from_numpy(a).cuda()
    adv, count, diag = ctx.diagnostics(t(logp_train), t(logp_roll.astype(np.float32)), t(valid), t(cu), t(rewards), 2, p)
    torch.cuda.synchronize()
    d = ctx.read_diag(diag)
    assert ctx.status() == 0
    ctx.close()
    w = min(np.exp(float(np.float32(shift))), 5.0)
    print(f"shift {shift}: w_bar {w:.4g}, gpu var_w {d['var_w']:.3e} std_aw {d['std_aw']:.3e} dsigma {d['dsigma']:.3e}; "
          f"oracle {rd['var_w']:.3e} {rd['std_aw']:.3e} {rd['dsigma']:.3e}", flush=True)
    assert d["n_valid"] == rd["n_valid"] == int(valid.sum())
    P.rel_close(d["mean_w"], w, rel=1e-12, what="mean_w")
    assert d["var_w"] == 0.0 and d["cv2"] == 0.0 and d["alpha_ess"] == 1.0
    assert d["std_a"] == 0.0 and d["std_aw"] == 0.0 and d["dsigma"] == 0.0 and d["alpha_var"] == 0.0
    # the oracle's two-pass forms agree up to the rounding of its own mean
    assert rd["var_w"] <= 1e-28 * w * w and rd["std_aw"] <= 1e-14 * w and rd["dsigma"] <= 1e-8 * w
    P.rel_close(d["alpha"], rd["alpha"], rel=1e-9, floor=1e-12, what="alpha")
