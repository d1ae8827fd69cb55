"""GPU parity of the one-sweep variant (each logits row read once; direction s = softmax - onehot plus a
per-row scale g) against the CPU oracle.  g[n] * s[n, :] must reproduce the oracle's dlogits."""
import numpy as np
import pytest
import torch

import oracle.ais_oracle as O
from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.AisContext()
    yield c
    c.close()


def check_one_sweep(ctx, batch, p=None, logp_old=None, logp_ref=None, in_place=False, strict=False):
    p = p or B.default_params()
    ref = P.run_oracle(batch, p, logp_old, logp_ref)
    valid = batch.valid.cpu().numpy().astype(bool)
    y = batch.token_ids.cpu().numpy()
    V = batch.shape.vocab
    inv_t = float(p.inv_temperature)
    # oracle direction and gradient, chunk by chunk, before an in-place run overwrites the logits
    chunks = []
    for r0, r1, dz in ref["dz_chunks"]():
        s_ref = O.dlogits_rows(P.to_np64(batch.logits[r0:r1]), ref["lse"][r0:r1], y[r0:r1],
                               valid[r0:r1].astype(np.float64), inv_t) / inv_t
        chunks.append((r0, r1, dz, s_ref))
    out = ctx.step_one_sweep(batch, p, logp_old, logp_ref, in_place=in_place)
    torch.cuda.synchronize()
    d = P.compare_scalars(ctx, out, ref, batch, strict)
    g = P.to_np64(out["g"])
    g_ref = ref["g"] * inv_t
    assert np.all(g[g_ref == 0] == 0)
    # the coefficient carries w_tilde, the on-policy ratio and the KL term: what the observed log-prob error E can do
    # to them (parity.compare_scalars leaves the per-row bound in ref["g_slack"]) is added to the relative tolerance
    assert np.all(np.abs(g - g_ref) <= P.REL * np.abs(g_ref) + (0.0 if strict else 1e-12 + ref["g_slack"] * inv_t)), \
        f"g: worst {float(np.max(np.abs(g - g_ref)))!r}"

    for r0, r1, dz_ref, s_ref in chunks:
        s = P.to_np64(out["sgrad"][r0:r1, :V])
        assert np.all(s[~valid[r0:r1]] == 0), "rows that are not evaluated must have a zero direction"
        tol = P.dz_tolerance(s_ref, valid[r0:r1].astype(np.float64), ref["lse"][r0:r1], strict)
        bad = np.abs(s - s_ref) > tol
        assert not bad.any(), f"direction mismatch rows {r0}:{r1} at {np.argwhere(bad)[0]}"
        prod = g[r0:r1, None] * s
        tol = P.dz_tolerance(dz_ref, ref["g"][r0:r1], ref["lse"][r0:r1], strict, ref["g_slack"][r0:r1], inv_t)
        bad = np.abs(prod - dz_ref) > tol
        assert not bad.any(), f"g * s differs from dlogits in rows {r0}:{r1} at {np.argwhere(bad)[0]}"
    assert ctx.status() == 0
    return out, ref, d


@pytest.mark.parametrize("k,len_div", [(2, 64), (3, 16), (4, 64), (5, 128)])
def test_full_vocab(ctx, k, len_div):
    """Real row geometry: 151,936 (19 vector slots per lane, all in registers), 126,464 (16), and 248,320
    (31 slots: 22 in registers, 9 in LDS)."""
    shape = W.config(k).scaled(len_div=len_div, n_prompts=2 if k == 3 else None)
    check_one_sweep(ctx, W.generate(shape, "cuda", row_chunk=128), strict=True)


def test_tiny_fp32(ctx):
    check_one_sweep(ctx, W.generate(W.config(1), "cuda"), strict=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("vocab", [1, 5, 1003, 8200, 40_001, 98_312, 110_597, 122_881, 127_000, 132_501, 140_000])
def test_odd_vocabularies(ctx, vocab, dtype):
    shape = W.RolloutShape("odd", n_prompts=2, group_size=4, vocab=vocab, logits_dtype=dtype, sigma=2.5, boost=4.0,
                           layout="padded", max_len=6, length_dist=("uniform", 1, 6), reward_p=0.5, seed=vocab)
    # fp32: 98,312 needs 25 slots per lane (18 + 9 in LDS), 110,597 needs 28 (20 + 9), 122,881 needs 31 (22 + 9, only
    # one vector of the last slot exists), 127,000 needs 32 and 132,501 needs 33 (24 + 9), 140,000 needs 35 and
    # takes the two-pass route; bf16 rows of these widths stay in registers
    batch = W.generate(shape, "cuda")
    batch.rewards[:] = torch.tensor([1, 0, 0, 1, 0, 0, 1, 0], dtype=torch.float32)
    check_one_sweep(ctx, batch)


@pytest.mark.parametrize("vocab", [200_003, 230_011, 248_327, 262_147, 268_001, 270_336, 270_337, 280_001])
def test_wide_bf16_rows(ctx, vocab):
    """bf16 rows of 25 to 33 vectors per lane (the last 9 in LDS), the widest row that fits (270,336), and the first
    widths that do not and take the two-pass route."""
    shape = W.RolloutShape("wide", n_prompts=1, group_size=4, vocab=vocab, logits_dtype="bf16", sigma=2.5, boost=4.0,
                           layout="padded", max_len=5, length_dist=("uniform", 2, 5), reward_p=0.5, seed=vocab)
    batch = W.generate(shape, "cuda")
    batch.rewards[:] = torch.tensor([1, 0, 0, 1], dtype=torch.float32)
    check_one_sweep(ctx, batch)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("vocab", [1, 5, 7, 264, 1003, 9001])
@pytest.mark.parametrize("inv_t", [0.3, 0.6])
def test_high_temperature_short_rows(ctx, vocab, dtype, inv_t):
    """Temperatures above 1 on rows so short that most lanes hold nothing but excluded elements (positions past
    the end of the row, the sampled token's own term): those must add exactly 0 whatever the multiplier inside the
    exponent."""
    shape = W.RolloutShape("hot", n_prompts=2, group_size=4, vocab=vocab, logits_dtype=dtype, sigma=2.5, boost=4.0,
                           layout="padded", max_len=9, length_dist=("uniform", 3, 9), reward_p=0.5, seed=vocab + 17)
    batch = W.generate(shape, "cuda")
    batch.rewards[:] = torch.tensor([1, 0, 0, 1, 0, 0, 1, 0], dtype=torch.float32)
    check_one_sweep(ctx, batch, p=B.default_params(inv_temperature=inv_t))


def test_pitch_misalignment_and_in_place(ctx):
    shape = W.RolloutShape("pitch", n_prompts=1, group_size=4, vocab=3003, logits_dtype="bf16", sigma=3.0, boost=0.0,
                           layout="packed", max_len=30, length_dist=("uniform", 5, 30), reward_p=0.5, seed=7)
    batch = W.generate(shape, "cuda")
    batch.rewards[:] = torch.tensor([1, 0, 0, 1], dtype=torch.float32)
    R, V = batch.logits.shape
    wide = torch.full((R, 3016), 8192.0, dtype=torch.bfloat16, device="cuda")
    wide[:, :V] = batch.logits
    batch.logits = wide[:, :V]                       # row pitch > vocab: register path with a scalar tail
    check_one_sweep(ctx, batch, in_place=True)
    assert bool((wide[:, V:] == 8192.0).all())
    flat = torch.empty(R * V + 1, dtype=torch.bfloat16, device="cuda")
    batch2 = W.generate(shape, "cuda")
    batch2.rewards[:] = batch.rewards
    flat[1:] = batch2.logits.reshape(-1)
    batch2.logits = flat[1:].view(R, V)              # misaligned base: two-pass element-wise route
    check_one_sweep(ctx, batch2)


def test_modes(ctx):
    shape = W.config(2).scaled(vocab=20_008, len_div=32, seed=5)
    batch = W.generate(shape, "cuda")
    p = B.default_params(beta_kl=0.03, inv_temperature=1 / 0.9, adv_mode=1)
    lp = torch.log_softmax(batch.logits.float() * p.inv_temperature, 1)
    lp = lp.gather(1, batch.token_ids.long().unsqueeze(1)).squeeze(1)
    g = torch.Generator(device="cuda").manual_seed(2)
    logp_old = lp + 0.2 * torch.randn(lp.shape, device="cuda", generator=g)
    rho = torch.exp(lp - logp_old)
    logp_old = torch.where(((rho - 0.8).abs() < 1e-3) | ((rho - 1.2).abs() < 1e-3), lp, logp_old)
    logp_ref = lp + 0.3 * torch.randn(lp.shape, device="cuda", generator=g)
    check_one_sweep(ctx, batch, p, logp_old=logp_old, logp_ref=logp_ref)
    check_one_sweep(ctx, batch, B.default_params(alpha_override=1.0))


def test_masked_rows_bad_token_and_reproducibility(ctx):
    shape = W.config(3).scaled(vocab=5000, len_div=8, n_prompts=2, seed=3)
    batch = W.generate(shape, "cuda")
    a = ctx.step_one_sweep(batch)
    b = ctx.step_one_sweep(batch)
    torch.cuda.synchronize()
    for k in ("logp", "lse", "sgrad", "g", "loss", "diag"):
        assert torch.equal(a[k], b[k]), k
    # same log-probs as the two-call path, bit for bit is not required but the tolerance is
    logp, lse = ctx.token_logprob(batch.logits, batch.token_ids, batch.valid)
    assert float((logp - a["logp"]).abs().max()) <= 1e-5
    first = int(batch.valid.nonzero()[0])
    batch.token_ids[first] = 5000
    out = ctx.step_one_sweep(batch)
    torch.cuda.synchronize()
    assert ctx.status() & B.STATUS_BAD_TOKEN and out["logp"][first].item() == 0
    assert torch.isfinite(out["sgrad"].float()).all()


@pytest.mark.parametrize("vocab", [4_107, 151_936])
def test_vocabulary_masked_with_minus_infinity(ctx, vocab):
    """Banned tokens (-inf logits) through the register-resident kernel: probability and direction exactly 0 there,
    no NaN; whole vectors, the ragged tail and a row that keeps only its sampled token."""
    shape = W.config(2).scaled(vocab=vocab, len_div=64 if vocab < 10_000 else 256, seed=78)
    batch = W.generate(shape, "cuda", row_chunk=128)
    R, V = batch.logits.shape
    g = torch.Generator(device="cuda")
    g.manual_seed(6)
    ban = torch.rand(R, V, generator=g, device="cuda") < 0.33
    ban[:, V - 11:] = True
    ban[:, 64:96] = True
    ban[3] = True
    ban[torch.arange(R, device="cuda"), batch.token_ids.long().clamp(min=0)] = False
    batch.logits[ban] = float("-inf")
    out, ref, d = check_one_sweep(ctx, batch)
    assert torch.isfinite(out["logp"]).all() and torch.isfinite(out["sgrad"].float()).all()
    assert bool((out["sgrad"][ban] == 0).all())


def test_extreme_logit_magnitudes(ctx):
    """Logits thousands of units apart through the register-resident kernel: sampled tokens whose probability
    underflows a double still get a finite log-prob."""
    batch = W.generate(W.config(2).scaled(vocab=4_104, len_div=64, seed=79), "cuda")
    batch.logits.mul_(1000.0)
    out, ref, d = check_one_sweep(ctx, batch)
    assert torch.isfinite(out["logp"]).all() and float(out["logp"].min()) < -1000.0
