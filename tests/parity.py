"""Shared machinery of the GPU parity tests: run the HIP path and the CPU oracle on the same bits and
compare element by element.

Tolerances (the bar this repository holds itself to):
  * log-prob, lse        |gpu - oracle| <= 2e-3 absolute on evaluated rows; exactly 0 on the others
  * n_valid, count[i], status, the set of rows with non-zero output: exact
  * mean_w, cv2, ess_ratio, dbar, std_a, std_aw, dsigma, alpha_ess, alpha_mis: relative 1e-3
  * kl_roll_train (a signed mean that cancels): |d| <= 1e-3 * max(|ref|, dbar); mean_abs_dp: relative 1e-3
  * alpha_var, alpha (hard-thresholded, may sit at 0): |d| <= 1e-3 * max(|ref|, 1e-3)
  * loss: |d| <= 1e-3 * max(|ref|, floor), floor = (1/B) sum_i |A_i| mean_t(w_tilde) — the size of the terms
    whose cancellation (sum of a group's advantages is 0) produces the loss
  * advantages: 1e-6 absolute (they are stored in fp32)
  * w_tilde: relative 1e-3
  * strict mode (the five named workloads, at reduced and at full size): exactly the bounds above and nothing else
  * otherwise (random and adversarial configurations): every bound above that depends on the log-probs also admits
    what the observed log-prob error E (<= 2e-3, of the order of 1e-6 on the workloads) can do to the quantity;
    compare_scalars derives each such term
  * dlogits: |d| <= 1e-2 |ref| + 1e-2 * 2^-8 * max_v |ref[n, :]| + 2^-126 (one bf16 half-ulp of the row maximum as
    absolute cushion; the same bound is used for fp32 logits; 2^-126 is the smallest normal number of both output
    types: an fp64 oracle resolves probabilities of 1e-100 on a sharply peaked row, fp32 arithmetic flushes them
    to 0), and exactly 0 on rows whose coefficient is 0.  Strict mode keeps only the first two terms.  Otherwise, on top
    of that, the oracle's own rounding floor,
    |g_n| * 8 * 2^-52 * max(1, |lse_n|): the oracle follows the definitions (logp = z_y - lse, p_y - 1 by
    subtraction), and both cancel when the sampled token's probability approaches 1, leaving an error of a few ulps
    of lse in fp64; the HIP path evaluates the same quantities through log1p / expm1 and keeps their relative
    accuracy, so on a row whose whole gradient is of that size the oracle is the less accurate side.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle.ais_oracle as O
from paper_2605_13907_amd import binding as B

from tests.tolerances import (DZ_CUSHION, DZ_ORACLE_ULPS, DZ_REL, DZ_TINY, LOGP_ATOL, REL, dz_tolerance,  # noqa: F401
                              oracle_floor)


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_params(p: B.AisParams) -> O.Params:
    return O.Params(C=float(p.C), delta=float(p.delta), gamma=float(p.gamma), eps_std=float(p.eps_std),
                    beta_var=float(p.beta_var), clip_eps=float(p.clip_eps), adv_mode=int(p.adv_mode),
                    alpha_override=float(p.alpha_override), inv_temperature=float(p.inv_temperature),
                    beta_kl=float(p.beta_kl))


def run_oracle(batch, p: B.AisParams, logp_old=None, logp_ref=None, row_chunk=256):
    """Oracle on the batch's bits.  dlogits are produced chunk by chunk by the returned generator."""
    op = oracle_params(p)
    valid = batch.valid.cpu().numpy()
    y = batch.token_ids.cpu().numpy()
    cu = batch.cu_rows.cpu().numpy()
    R = batch.n_rows
    logp = np.zeros(R)
    lse = np.zeros(R)
    for r0 in range(0, R, row_chunk):
        r1 = min(R, r0 + row_chunk)
        logp[r0:r1], lse[r0:r1] = O.token_logprob(to_np64(batch.logits[r0:r1]), y[r0:r1], valid[r0:r1],
                                                  op.inv_temperature)
    adv = O.group_advantages(to_np64(batch.rewards), batch.shape.group_size, op.adv_mode, op.eps_std)
    lp_roll = to_np64(batch.logp_roll)
    lo = None if logp_old is None else to_np64(logp_old)
    lr = None if logp_ref is None else to_np64(logp_ref)
    # Alg. 1: the coefficient is estimated from log pi_train at the checkpoint that generated the rollout
    diag = O.diagnostics(logp if lo is None else lo, lp_roll, valid, cu, adv, op)
    loss, wtilde, g = O.loss_and_row_coeff(logp, lp_roll, lo, lr, valid, cu, adv, diag["count"], diag["alpha"], op)
    # how strongly a row's coefficient reacts to its own log-prob through the KL term: d/dlogp of beta_kl (1 - e^q) / (B |o_i|)
    kl_sens = np.zeros(R)
    if lr is not None and op.beta_kl > 0:
        seq = O.rows_to_responses(cu, R)
        cnt = np.maximum(diag["count"][seq], 1)
        kl_sens = np.where(valid.astype(bool), op.beta_kl * np.exp(lr - logp) / (len(cu) - 1) / cnt, 0.0)

    def dz_chunks():
        for r0 in range(0, R, row_chunk):
            r1 = min(R, r0 + row_chunk)
            yield r0, r1, O.dlogits_rows(to_np64(batch.logits[r0:r1]), lse[r0:r1], y[r0:r1], g[r0:r1],
                                         op.inv_temperature)

    return dict(logp=logp, lse=lse, adv=adv, diag=diag, loss=loss, wtilde=wtilde, g=g, dz_chunks=dz_chunks, params=op,
                kl_sens=kl_sens, g_slack=np.zeros(R))


def rel_close(got, ref, rel=REL, floor=0.0, what=""):
    tol = rel * max(abs(ref), floor)
    assert abs(got - ref) <= tol, f"{what}: gpu {got!r} oracle {ref!r} tol {tol:.3e}"


def compare_scalars(ctx, out, ref, batch, strict=False):
    """Scalars of the path against the oracle.  strict: the stated tolerances alone (the five named workloads).
    Otherwise every bound is the stated relative tolerance plus what the observed
    log-prob error E = max |logp_gpu - logp_oracle| (itself held to LOGP_ATOL) can do to the quantity: a truncated
    ratio moves by at most C E, and the diagnostics inherit that through their formulas.  With E of the order of
    1e-6, as on the workloads, the extra terms vanish against the relative tolerance; they matter on inputs where
    lse is in the hundreds (fp32 resolves it to 1e-4) or where a statistic is exactly 0 in the oracle."""
    valid = batch.valid.cpu().numpy().astype(bool)
    logp = to_np64(out["logp"])
    lse = to_np64(out["lse"])
    assert np.all(logp[~valid] == 0) and np.all(lse[~valid] == 0), "rows that are not evaluated must be exactly 0"
    E = float(np.max(np.abs(logp - ref["logp"]), initial=0))
    assert E <= LOGP_ATOL, E
    assert np.max(np.abs(lse - ref["lse"]), initial=0) <= LOGP_ATOL
    d = ctx.read_diag(out["diag"])
    rd = ref["diag"]
    op = ref["params"]
    assert d["n_valid"] == rd["n_valid"]
    assert out["count"].cpu().tolist() == [int(c) for c in rd["count"]]
    np.testing.assert_allclose(to_np64(out["adv"]), ref["adv"], rtol=0, atol=1e-6)
    Ew = 0.0 if strict else op.C * E                     # bound on the change of one truncated ratio
    a_max = float(np.max(np.abs(ref["adv"]), initial=0))
    worst = {"logp": E / LOGP_ATOL, "lse": float(np.max(np.abs(lse - ref["lse"]), initial=0)) / LOGP_ATOL}
    E_log = E                                            # kept for the report
    if strict:
        E = 0.0                                          # no propagated slack below
    if rd["n_valid"] > 0:
        mean_w, var_w = rd["mean_w"], rd["var_w"]
        t_var = 4.0 * (np.sqrt(var_w) * Ew + Ew * Ew)
        t_cv2 = (t_var + 2.0 * var_w * Ew / max(mean_w, 1e-300)) / max(mean_w * mean_w, 1e-300) if mean_w > 0 else 0.0
        den = rd["std_a"] + op.eps_std
        t_dsig = 2.0 * a_max * Ew / den if den > 0 else 0.0
        # a ratio within E of the truncation level may fall on either side of it: each such token moves the
        # truncated share by 1 / N
        d_ref = ref["logp"] - to_np64(batch.logp_roll)
        on_edge = 0 if strict else int(np.sum(valid & (np.abs(d_ref - np.log(op.C)) <= 2.0 * E + 1e-12)))
        extra = dict(mean_w=Ew, var_w=t_var, cv2=t_cv2, ess_ratio=t_cv2, alpha_ess=t_cv2, dbar=E, std_a=0.0,
                     std_aw=2.0 * a_max * Ew, dsigma=t_dsig, alpha_mis=E / op.delta,
                     clip_frac=on_edge / rd["n_valid"], mean_abs_dp=E)
        # weights below 1e-140 have squares at the bottom of the fp64 range: the oracle's own variance is made of
        # denormals there and says nothing; only finiteness and range are checked for the spread statistics
        skip = ("var_w", "cv2", "ess_ratio", "alpha_ess") if 0.0 < mean_w < 1e-140 else ()
        if skip:
            assert np.isfinite(d["cv2"]) and d["cv2"] >= 0.0 and 0.0 < d["alpha_ess"] <= 1.0
        for k in ("mean_w", "var_w", "cv2", "ess_ratio", "dbar", "std_a", "std_aw", "dsigma", "alpha_ess", "alpha_mis",
                  "clip_frac", "mean_abs_dp"):
            if k in skip:
                continue
            # quantities that are exactly 0 in the oracle (e.g. std of all-equal advantages) get a tiny floor
            tol = REL * max(abs(rd[k]), 1e-9) + extra[k]
            assert abs(d[k] - rd[k]) <= tol, f"{k}: gpu {d[k]!r} oracle {rd[k]!r} tol {tol:.3e} (E = {E_log:.1e})"
            worst[k] = abs(d[k] - rd[k]) / (REL * max(abs(rd[k]), 1e-9))
        # the signed mean of d cancels: its natural scale is the mean of |d|
        rel_close(d["kl_roll_train"], rd["kl_roll_train"], floor=rd["dbar"] + E / REL, what="kl_roll_train")
        worst["kl_roll_train"] = abs(d["kl_roll_train"] - rd["kl_roll_train"]) / (REL * max(abs(rd["kl_roll_train"]), rd["dbar"], 1e-300))
        t_avar = t_dsig / op.gamma
        t_alpha = t_cv2 + op.beta_var * t_avar + E / op.delta
    else:
        t_avar = t_alpha = 0.0
    assert abs(d["alpha_var"] - rd["alpha_var"]) <= REL * max(abs(rd["alpha_var"]), 1e-3) + t_avar, "alpha_var"
    worst["alpha_var"] = abs(d["alpha_var"] - rd["alpha_var"]) / (REL * max(abs(rd["alpha_var"]), 1e-3))
    worst["alpha"] = abs(d["alpha"] - rd["alpha"]) / (REL * max(abs(rd["alpha"]), 1e-3))
    if op.alpha_override < 0 and rd["n_valid"] > 0 and 0.0 < rd["mean_w"] < 1e-140:
        assert 0.0 <= d["alpha"] <= 1.0
    elif op.alpha_override < 0:
        assert abs(d["alpha"] - rd["alpha"]) <= REL * max(abs(rd["alpha"]), 1e-3) + t_alpha, \
            f"alpha: gpu {d['alpha']!r} oracle {rd['alpha']!r}"
    else:
        assert abs(d["alpha"] - rd["alpha"]) <= 1e-12
    t_alpha = 0.0 if op.alpha_override >= 0 else t_alpha
    wt = to_np64(out["wtilde"])
    assert np.all(wt[~valid] == 0)
    # w_tilde = 1 + alpha (w_bar - 1): moves by alpha C E through its ratio and by |w_bar - 1| through alpha
    np.testing.assert_allclose(wt, ref["wtilde"], rtol=REL,
                               atol=0.0 if strict else 1e-7 + Ew + t_alpha * max(1.0, op.C - 1.0))
    worst["wtilde"] = float(np.max(np.abs(wt - ref["wtilde"])[valid] /
                                   (REL * np.maximum(np.abs(ref["wtilde"][valid]), 1e-300)), initial=0))
    B_ = batch.shape.n_resp
    cnt = rd["count"]
    cu = batch.cu_rows.cpu().numpy()
    mean_wt = [ref["wtilde"][cu[i]:cu[i + 1]][valid[cu[i]:cu[i + 1]]].mean() if cnt[i] else 0.0 for i in range(B_)]
    floor = float(np.sum(np.abs(ref["adv"]) * np.array(mean_wt)) / B_)
    # the loss is a sum of terms of size `floor`, each of which inherits the relative error of w_tilde and of the
    # on-policy ratio (2 E); the KL term adds beta_kl times an error of the same size
    t_loss = (floor + op.beta_kl) * (2.0 * E + Ew + t_alpha * max(1.0, op.C - 1.0))
    loss_floor = max(abs(ref["loss"]), floor) if strict else max(abs(ref["loss"]), floor, 1e-12)
    assert abs(float(out["loss"].item()) - ref["loss"]) <= REL * loss_floor + t_loss, \
        f"loss: gpu {float(out['loss'].item())!r} oracle {ref['loss']!r} floor {floor:.3e} E {E_log:.1e}"
    worst["loss"] = abs(float(out["loss"].item()) - ref["loss"]) / (REL * max(loss_floor, 1e-300))
    worst["loss_rel_to_value"] = abs(float(out["loss"].item()) - ref["loss"]) / max(abs(ref["loss"]), 1e-300)
    d["_E"] = E_log
    d["_t_alpha"] = t_alpha
    d["_worst"] = worst          # observed error of every quantity as a fraction of its plain stated bound
    # what E can do to a row's gradient coefficient: through w_tilde and the on-policy ratio (relative), and through
    # the KL term (absolute, and the whole of it on rows whose advantage is 0 and whose q is close to 0)
    ref["g_slack"] = np.abs(ref["g"]) * (2.0 * E + Ew + t_alpha * max(1.0, op.C - 1.0)) + ref["kl_sens"] * E
    return d


def compare_dlogits(out, ref, batch, strict=False):
    dz = out["dlogits"]
    V = batch.shape.vocab
    worst = 0.0
    for r0, r1, ref_dz in ref["dz_chunks"]():
        got = to_np64(dz[r0:r1, :V])
        zero_rows = ref["g"][r0:r1] == 0
        assert np.all(got[zero_rows] == 0), "rows without gradient must be exactly 0"
        rowmax = np.abs(ref_dz).max(axis=1, keepdims=True)
        tol = dz_tolerance(ref_dz, ref["g"][r0:r1], ref["lse"][r0:r1], strict, ref["g_slack"][r0:r1],
                           ref["params"].inv_temperature)
        err = np.abs(got - ref_dz)
        bad = err > tol
        assert not bad.any(), (f"dlogits mismatch in rows {r0}:{r1}: {int(bad.sum())} elements, worst "
                               f"{float((err - tol).max()):.3e} over tolerance at {np.argwhere(bad)[0]}")
        nz = ~zero_rows
        if nz.any():
            # rows that carry gradient must actually be written (guards against a silently skipped row)
            live = nz & (rowmax[:, 0] > 1e-30)          # V = 1 gives p - 1 = 0 even where the coefficient is not 0
            assert np.all(np.abs(got[live]).max(axis=1) > 0)
            worst = max(worst, float((err[nz] / (tol[nz] + 1e-300)).max()))
    return worst


def run_both(ctx, batch, p=None, logp_old=None, logp_ref=None, in_place=False):
    p = p or B.default_params()
    ref = run_oracle(batch, p, logp_old, logp_ref)         # before the GPU call: in-place runs overwrite the logits
    if in_place:
        ref["_dz"] = [(r0, r1, c) for r0, r1, c in ref["dz_chunks"]()]
        ref["dz_chunks"] = lambda: iter(ref["_dz"])
    out = ctx.step(batch, p, logp_old, logp_ref, in_place=in_place)
    torch.cuda.synchronize()
    return out, ref


def check(ctx, batch, p=None, logp_old=None, logp_ref=None, in_place=False, expect_status=0, strict=False):
    out, ref = run_both(ctx, batch, p, logp_old, logp_ref, in_place)
    d = compare_scalars(ctx, out, ref, batch, strict)
    d["_worst"]["dlogits"] = compare_dlogits(out, ref, batch, strict)
    assert ctx.status() == expect_status
    return out, ref, d
