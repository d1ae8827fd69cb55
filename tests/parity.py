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
  * dlogits: |d| <= 1e-2 |ref| + 1e-2 * 2^-8 * max_v |ref[n, :]| (one bf16 half-ulp of the row maximum as
    absolute cushion; the same bound is used for fp32 logits), and exactly 0 on rows whose coefficient is 0
"""
from __future__ import annotations

import numpy as np
import torch

import oracle.ais_oracle as O
from paper_2605_13907_amd import binding as B

LOGP_ATOL = 2e-3
REL = 1e-3
DZ_REL = 1e-2
DZ_CUSHION = 1e-2 * 2.0 ** -8


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
    diag = O.diagnostics(logp, lp_roll, valid, cu, adv, op)
    lo = None if logp_old is None else to_np64(logp_old)
    lr = None if logp_ref is None else to_np64(logp_ref)
    loss, wtilde, g = O.loss_and_row_coeff(logp, lp_roll, lo, lr, valid, cu, adv, diag["count"], diag["alpha"], op)

    def dz_chunks():
        for r0 in range(0, R, row_chunk):
            r1 = min(R, r0 + row_chunk)
            yield r0, r1, O.dlogits_rows(to_np64(batch.logits[r0:r1]), lse[r0:r1], y[r0:r1], g[r0:r1],
                                         op.inv_temperature)

    return dict(logp=logp, lse=lse, adv=adv, diag=diag, loss=loss, wtilde=wtilde, g=g, dz_chunks=dz_chunks, params=op)


def rel_close(got, ref, rel=REL, floor=0.0, what=""):
    tol = rel * max(abs(ref), floor)
    assert abs(got - ref) <= tol, f"{what}: gpu {got!r} oracle {ref!r} tol {tol:.3e}"


def compare_scalars(ctx, out, ref, batch):
    valid = batch.valid.cpu().numpy().astype(bool)
    logp = to_np64(out["logp"])
    lse = to_np64(out["lse"])
    assert np.all(logp[~valid] == 0) and np.all(lse[~valid] == 0), "rows that are not evaluated must be exactly 0"
    assert np.max(np.abs(logp - ref["logp"]), initial=0) <= LOGP_ATOL, np.max(np.abs(logp - ref["logp"]))
    assert np.max(np.abs(lse - ref["lse"]), initial=0) <= LOGP_ATOL
    d = ctx.read_diag(out["diag"])
    rd = ref["diag"]
    assert d["n_valid"] == rd["n_valid"]
    assert out["count"].cpu().tolist() == [int(c) for c in rd["count"]]
    np.testing.assert_allclose(to_np64(out["adv"]), ref["adv"], rtol=0, atol=1e-6)
    if rd["n_valid"] > 0:
        for k in ("mean_w", "cv2", "ess_ratio", "dbar", "std_a", "std_aw", "dsigma", "alpha_ess", "alpha_mis"):
            # quantities that are exactly 0 in the oracle (e.g. std of all-equal advantages) get a tiny floor
            rel_close(d[k], rd[k], floor=1e-9, what=k)
        rel_close(d["var_w"], rd["var_w"], floor=1e-9, what="var_w")
        rel_close(d["clip_frac"], rd["clip_frac"], floor=1e-9, what="clip_frac")
        # the signed mean of d cancels: its natural scale is the mean of |d|
        rel_close(d["kl_roll_train"], rd["kl_roll_train"], floor=rd["dbar"], what="kl_roll_train")
        rel_close(d["mean_abs_dp"], rd["mean_abs_dp"], floor=1e-9, what="mean_abs_dp")
    rel_close(d["alpha_var"], rd["alpha_var"], floor=1e-3, what="alpha_var")
    rel_close(d["alpha"], rd["alpha"], floor=1e-3, what="alpha")
    wt = to_np64(out["wtilde"])
    assert np.all(wt[~valid] == 0)
    np.testing.assert_allclose(wt, ref["wtilde"], rtol=REL, atol=1e-7)
    B_ = batch.shape.n_resp
    cnt = rd["count"]
    cu = batch.cu_rows.cpu().numpy()
    mean_wt = [ref["wtilde"][cu[i]:cu[i + 1]][valid[cu[i]:cu[i + 1]]].mean() if cnt[i] else 0.0 for i in range(B_)]
    floor = float(np.sum(np.abs(ref["adv"]) * np.array(mean_wt)) / B_)
    rel_close(float(out["loss"].item()), ref["loss"], floor=max(floor, 1e-12), what="loss")
    return d


def compare_dlogits(out, ref, batch):
    dz = out["dlogits"]
    V = batch.shape.vocab
    worst = 0.0
    for r0, r1, ref_dz in ref["dz_chunks"]():
        got = to_np64(dz[r0:r1, :V])
        zero_rows = ref["g"][r0:r1] == 0
        assert np.all(got[zero_rows] == 0), "rows without gradient must be exactly 0"
        rowmax = np.abs(ref_dz).max(axis=1, keepdims=True)
        tol = DZ_REL * np.abs(ref_dz) + DZ_CUSHION * rowmax
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


def check(ctx, batch, p=None, logp_old=None, logp_ref=None, in_place=False, expect_status=0):
    out, ref = run_both(ctx, batch, p, logp_old, logp_ref, in_place)
    d = compare_scalars(ctx, out, ref, batch)
    compare_dlogits(out, ref, batch)
    assert ctx.status() == expect_status
    return out, ref, d
