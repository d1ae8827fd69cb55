"""GPU parity: the HIP path (through the C ABI) against the CPU fp64 oracle on the same seeded inputs.
Tolerances are defined in tests/parity.py."""
import os
import time
from dataclasses import replace as dataclasses_replace

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


def gen(shape, **kw):
    return W.generate(shape, "cuda", **kw)


# ------------------------------------------------------------------ the five workloads, at oracle-sized scale
def test_config1_tiny_full_size(ctx):
    """Workload 1 as specified: fp32 logits, padded layout, V = 1024."""
    batch = gen(W.config(1))
    assert batch.logits.dtype == torch.float32 and batch.n_rows == 8 * 64
    out, ref, d = P.check(ctx, batch, strict=True)
    assert 0 < d["n_valid"] < batch.n_rows


@pytest.mark.parametrize("k,len_div", [(2, 64), (3, 16), (4, 64), (5, 128)])
def test_configs_full_vocab_fewer_rows(ctx, k, len_div):
    """Workloads 2-5 at their real vocabulary (the kernels' real row geometry, many unrolled iterations plus
    the ragged tail), with response lengths divided so that the oracle finishes in seconds."""
    n_prompts = 2 if k == 3 else None
    shape = W.config(k).scaled(len_div=len_div, n_prompts=n_prompts)
    batch = gen(shape, row_chunk=128)
    out, ref, d = P.check(ctx, batch, strict=True)
    assert d["n_valid"] > 100
    if k == 5:      # extra rollout noise: mismatch far above delta, correction fully engaged on the necessity side
        assert d["alpha_mis"] == 1.0


@pytest.mark.parametrize("k,vocab,len_div", [(2, 20_008, 8), (3, 4_104, 2), (4, 33_000, 8), (5, 8_200, 16)])
def test_configs_many_rows_smaller_vocab(ctx, k, vocab, len_div):
    """The same structures with more rows (several reduction tiles per response, more responses than one tile row)."""
    shape = W.config(k).scaled(vocab=vocab, len_div=len_div)
    batch = gen(shape)
    out, ref, d = P.check(ctx, batch, strict=True)
    assert batch.n_rows > 2000


# ------------------------------------------------------------------ adversarial shapes
@pytest.mark.parametrize("vocab", [1, 5, 255, 1003, 2056, 8191])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_odd_vocabularies(ctx, vocab, dtype):
    """Vocabularies below one workgroup, not a multiple of the vector width, or with a row pitch that is not
    16-byte aligned (element-wise path)."""
    shape = W.RolloutShape("odd", n_prompts=2, group_size=4, vocab=vocab, logits_dtype=dtype, sigma=2.5, boost=4.0,
                           layout="padded", max_len=12, length_dist=("uniform", 1, 12), reward_p=0.5, seed=vocab)
    batch = gen(shape)
    batch.rewards[:] = torch.tensor([1, 0, 0, 1, 0, 0, 1, 0], dtype=torch.float32)
    P.check(ctx, batch)


# every instantiation of the gradient sweep: 4 / 8 / 12 and each of 13 .. 20 vectors per lane in one burst, two and
# three bursts of 16, and the run-time loop over bursts beyond that (a lane's vector holds 8 bf16 or 4 fp32
# elements); around 19 x 1,024 vectors also a row that fills its last vector slot exactly, one element more (a
# scalar tail), and one vector more (the next class, with a single lane in its last slot)
BURST_VOCABS = {"bf16": [40_001, 90_007, 100_003, 110_001, 120_011, 126_464, 135_007, 143_003, 150_001, 155_648, 155_649,
                         155_656, 160_003, 250_007, 300_017, 450_029],
                "f32": [20_011, 45_007, 50_001, 55_001, 60_013, 63_233, 67_501, 71_503, 75_011, 77_824, 77_825, 77_828,
                        80_021, 125_003, 150_011, 230_003]}


@pytest.mark.parametrize("dtype,vocab", [(d, v) for d in ("bf16", "f32") for v in BURST_VOCABS[d]])
def test_every_row_width_class(ctx, dtype, vocab):
    shape = W.RolloutShape("width", n_prompts=1, group_size=4, vocab=vocab, logits_dtype=dtype, sigma=3.0, boost=6.0,
                           layout="padded", max_len=6, length_dist=("uniform", 2, 6), reward_p=0.5, seed=vocab)
    batch = gen(shape)
    batch.rewards[:] = torch.tensor([1, 0, 0, 1], dtype=torch.float32)
    P.check(ctx, batch)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_padded_pitch_and_misaligned_base(ctx, dtype):
    """row_stride > vocab (a column slice of a wider matrix): vector body plus scalar tail; and a base pointer
    that is not 16-byte aligned: element-wise path."""
    shape = W.RolloutShape("pitch", n_prompts=1, group_size=4, vocab=3003, logits_dtype=dtype, sigma=3.0, boost=0.0,
                           layout="packed", max_len=40, length_dist=("uniform", 5, 40), reward_p=0.5, seed=77)
    batch = gen(shape)
    batch.rewards[:] = torch.tensor([1, 0, 0, 1], dtype=torch.float32)
    R, V = batch.logits.shape
    wide = torch.full((R, 3008 + 8), 8192.0, dtype=batch.logits.dtype, device="cuda")    # poison outside the row
    wide[:, :V] = batch.logits
    batch.logits = wide[:, :V]
    assert batch.logits.stride(0) == 3016
    out, _, _ = P.check(ctx, batch)
    assert bool((wide[:, V:] == 8192.0).all()), "columns beyond vocab must not be touched"
    # misaligned base: shift by one element
    flat = torch.empty(R * V + 1, dtype=batch.logits.dtype, device="cuda")
    flat[1:] = batch.logits.reshape(-1)
    batch.logits = flat[1:].view(R, V)
    assert batch.logits.data_ptr() % 16 != 0
    P.check(ctx, batch)


def test_degenerate_batches(ctx):
    shape = W.RolloutShape("deg", n_prompts=2, group_size=4, vocab=520, logits_dtype="bf16", sigma=3.0, boost=0.0,
                           layout="padded", max_len=16, length_dist=("uniform", 1, 16), reward_p=0.5, seed=5)
    # a response with no valid row, and a prompt whose rewards are all equal
    batch = gen(shape)
    batch.valid.view(8, 16)[2] = 0
    batch.token_ids.view(8, 16)[2] = -1
    batch.rewards[:] = torch.tensor([1, 0, 1, 1, 1, 1, 1, 1], dtype=torch.float32)
    out, ref, d = P.check(ctx, batch)
    assert out["count"][2].item() == 0
    # all rewards equal everywhere: advantages 0, loss 0, gradient identically 0
    batch.rewards[:] = 1.0
    out, ref, d = P.check(ctx, batch)
    assert float(out["loss"].item()) == 0.0 and not bool(out["dlogits"].any())
    assert d["alpha_var"] == 0.0 and d["dsigma"] == 0.0
    # nothing valid at all
    batch.valid[:] = 0
    batch.token_ids[:] = -1
    batch.rewards[:] = torch.tensor([1, 0, 1, 1, 0, 0, 1, 0], dtype=torch.float32)
    out, ref, d = P.check(ctx, batch)
    assert d["n_valid"] == 0 and d["alpha"] == 0.0 and not bool(out["dlogits"].any())


def test_single_row_and_empty(ctx):
    shape = W.RolloutShape("one", n_prompts=1, group_size=1, vocab=777, logits_dtype="bf16", sigma=3.0, boost=0.0,
                           layout="packed", max_len=1, length_dist=("uniform", 1, 1), reward_p=1.0, seed=9)
    batch = gen(shape)
    P.check(ctx, batch)              # one response alone in its group: advantage 0
    # zero rows: every call must accept it and launch nothing harmful
    z = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    tok = torch.empty(0, dtype=torch.int32, device="cuda")
    logp, lse = ctx.token_logprob(z, tok)
    cu = torch.zeros(3, dtype=torch.int64, device="cuda")
    rewards = torch.tensor([1.0, 0.0], device="cuda")
    adv, count, diag = ctx.diagnostics(logp, logp, None, cu, rewards, 2)
    loss, wt, dz = ctx.grpo_loss_grad(z, tok, None, cu, logp, lse, logp, adv, count, diag)
    torch.cuda.synchronize()
    assert ctx.read_diag(diag)["n_valid"] == 0 and float(loss.item()) == 0.0
    assert adv.tolist() == [0.5, -0.5] and count.tolist() == [0, 0]


def test_many_short_responses(ctx):
    """More responses than threads in the planning workgroup (each thread scans a chunk of responses), many of
    them one or two rows long, several empty, plus a few longer than one reduction tile."""
    rng = np.random.default_rng(3)
    G, n_prompts, V = 4, 300, 264
    B_ = G * n_prompts
    lens = rng.integers(0, 4, size=B_)
    lens[rng.integers(0, B_, size=40)] = 0
    lens[[7, 500, 1199]] = [1500, 2300, 1025]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    R = int(cu[-1])
    shape = W.RolloutShape("short", n_prompts=n_prompts, group_size=G, vocab=V, logits_dtype="bf16", sigma=3.0,
                           boost=0.0, layout="packed", max_len=1, length_dist=("fixed",), reward_p=0.5, seed=12)
    base = gen(dataclasses_replace(shape, n_prompts=1, group_size=1, max_len=R))    # R rows of logits / tokens
    gcpu = torch.Generator().manual_seed(4)
    batch = W.RolloutBatch(shape=shape, logits=base.logits, token_ids=base.token_ids,
                           valid=(torch.rand(R, generator=gcpu) < 0.9).to(torch.uint8).cuda(),
                           cu_rows=torch.from_numpy(cu).cuda(), logp_roll=base.logp_roll,
                           rewards=(torch.rand(B_, generator=gcpu) < 0.5).float().cuda(),
                           lengths=torch.from_numpy(lens))
    out, ref, d = P.check(ctx, batch)
    assert d["n_valid"] == int(batch.valid.sum().item()) and (out["count"] == 0).sum().item() >= 40


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_vocabulary_masked_with_minus_infinity(ctx, dtype):
    """Logits processors ban tokens by setting their logit to -inf.  A third of every row's vocabulary is banned
    (never the sampled token), whole 16-byte vectors and the ragged tail included; one row keeps only its sampled
    token.  Banned entries must get probability 0 and gradient exactly 0, with no NaN anywhere."""
    shape = dataclasses_replace(W.config(2).scaled(vocab=4_107, len_div=64, seed=77), logits_dtype=dtype)
    batch = gen(shape)
    R, V = batch.logits.shape
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    ban = torch.rand(R, V, generator=g) < 0.33
    ban[:, 4096:] = True                                   # the tail past the last full vector
    ban[:, 64:96] = True                                   # whole vectors
    ban[3] = True                                          # a row with nothing but its sampled token
    ban = ban.cuda()
    ban[torch.arange(R, device="cuda"), batch.token_ids.long().clamp(min=0)] = False
    batch.logits[ban] = float("-inf")
    out, ref, d = P.check(ctx, batch)
    assert torch.isfinite(out["logp"]).all() and torch.isfinite(out["dlogits"].float()).all()
    assert bool((out["dlogits"][ban] == 0).all())
    assert abs(float(out["logp"][3])) < 1e-6


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("vocab", [1, 5, 7, 264, 1003])
@pytest.mark.parametrize("inv_t", [0.3, 0.6])
def test_high_temperature_short_rows(ctx, vocab, dtype, inv_t):
    """Temperatures above 1 (a multiplier below 1 inside the exponent) on rows so short that most lanes see nothing
    but excluded elements, and whose sampled token often sits in the scalar tail: an excluded element must add
    exactly 0 whatever the multiplier."""
    shape = W.RolloutShape("hot", n_prompts=2, group_size=4, vocab=vocab, logits_dtype=dtype, sigma=2.5, boost=4.0,
                           layout="padded", max_len=9, length_dist=("uniform", 3, 9), reward_p=0.5, seed=vocab + 17)
    batch = gen(shape)
    batch.rewards[:] = torch.tensor([1, 0, 0, 1, 0, 0, 1, 0], dtype=torch.float32)
    out, ref, d = P.check(ctx, batch, B.default_params(inv_temperature=inv_t))
    assert torch.isfinite(out["logp"]).all() and torch.isfinite(out["dlogits"].float()).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_sampled_token_among_banned_neighbours(ctx, dtype):
    """Every row keeps only its sampled token and one other entry; everything else, the sampled token's whole
    16-byte vector included, is -inf.  With a temperature of 2 the lane that holds the sampled token sees nothing
    but excluded and banned elements."""
    shape = dataclasses_replace(W.config(2).scaled(vocab=4_107, len_div=64, seed=78), logits_dtype=dtype)
    batch = gen(shape)
    R, V = batch.logits.shape
    y = batch.token_ids.long().clamp(min=0)
    other = (y + 1777) % V
    keep = torch.zeros(R, V, dtype=torch.bool, device="cuda")
    rows = torch.arange(R, device="cuda")
    keep[rows, y] = True
    keep[rows, other] = True
    batch.logits[~keep] = float("-inf")
    out, ref, d = P.check(ctx, batch, B.default_params(inv_temperature=0.5))
    assert torch.isfinite(out["logp"]).all() and torch.isfinite(out["dlogits"].float()).all()
    assert bool((out["dlogits"][~keep] == 0).all())


@pytest.mark.parametrize("dtype,factor", [("bf16", 1000.0), ("f32", 3000.0)])
def test_extreme_logit_magnitudes(ctx, dtype, factor):
    """Logits thousands of units apart: the soft-max is one-hot to working precision, lse is of order 1e4, and
    nothing may overflow (the running maximum is subtracted before every exponential)."""
    shape = dataclasses_replace(W.config(2).scaled(vocab=4_104, len_div=64, seed=79), logits_dtype=dtype)
    batch = gen(shape)
    batch.logits.mul_(factor)
    out, ref, d = P.check(ctx, batch)
    assert torch.isfinite(out["lse"]).all() and float(out["lse"].abs().max()) > 3000.0
    assert torch.isfinite(out["dlogits"].float()).all()


@pytest.mark.parametrize("drift", [40.0, 225.0, 2000.0])
def test_vanishing_weights(ctx, drift):
    """The trainer puts all of its mass on a token the sampler did not choose, `drift` logit units above the rest:
    ratios of about 4e-18, 1e-98, and 0 (beyond the range of exp).  Mean and spread of the weights must survive as
    long as the ratios are numbers, and the 0/0 of the last case is read as CV^2 = 0; alpha stays finite."""
    shape = W.config(2).scaled(vocab=1032, len_div=64, seed=23)
    batch = gen(shape)
    R, V = batch.logits.shape
    rows = torch.arange(R, device="cuda")
    other = (batch.token_ids.long().clamp(min=0) + 1) % V
    batch.logits[rows, other] = batch.logits.float().amax(dim=1).to(batch.logits.dtype) + drift
    out, ref, d = P.check(ctx, batch)
    assert np.isfinite(d["alpha"]) and np.isfinite(d["cv2"]) and d["alpha_mis"] == 1.0
    if drift > 1000:
        assert d["mean_w"] == 0.0 and d["cv2"] == 0.0 and d["alpha_ess"] == 1.0
    else:
        assert 0.0 < d["mean_w"] < 1e-12 and d["cv2"] > 0.0


def test_zero_stabiliser_and_equal_rewards(ctx):
    """eps_std = 0 with every reward equal: Delta-sigma is 0/0 and is read as 0; alpha, loss and gradient stay
    finite (the gradient is exactly 0: every advantage is 0)."""
    shape = W.config(2).scaled(vocab=1032, len_div=64, seed=25)
    batch = gen(shape)
    batch.rewards[:] = 1.0
    out, ref, d = P.check(ctx, batch, B.default_params(eps_std=0.0))
    assert d["dsigma"] == 0.0 and d["alpha_var"] == 0.0 and np.isfinite(d["alpha"])
    assert float(out["loss"].item()) == 0.0 and not bool(out["dlogits"].any())
    # normalised advantages: 0 / (0 + 0) per group is read as 0 as well
    out, ref, d = P.check(ctx, batch, B.default_params(eps_std=0.0, adv_mode=1))
    assert not bool(out["adv"].any()) and np.isfinite(d["alpha"]) and float(out["loss"].item()) == 0.0


def test_all_ratios_truncated(ctx):
    """rho > C on every token: w_bar == C, CV = 0, alpha_ess = 1, clip_frac = 1."""
    shape = W.config(2).scaled(vocab=1032, len_div=64, seed=21)
    batch = gen(shape)
    batch.logp_roll -= 5.0
    out, ref, d = P.check(ctx, batch)
    assert d["clip_frac"] == 1.0 and abs(d["mean_w"] - 5.0) < 1e-12 and d["alpha_ess"] == 1.0


# ------------------------------------------------------------------ modes of the objective
@pytest.mark.parametrize("mode", ["grpo", "tis", "alpha_0.37", "adv_norm", "temperature", "beta_var", "C2"])
def test_modes(ctx, mode):
    shape = W.config(5).scaled(vocab=2600, len_div=256, seed=31)
    batch = gen(shape)
    kw = {"grpo": dict(alpha_override=0.0), "tis": dict(alpha_override=1.0), "alpha_0.37": dict(alpha_override=0.37),
          "adv_norm": dict(adv_mode=1), "temperature": dict(inv_temperature=1 / 0.9), "beta_var": dict(beta_var=0.25),
          "C2": dict(C=2.0)}[mode]
    out, ref, d = P.check(ctx, batch, B.default_params(**kw))
    if mode == "grpo":
        assert bool((out["wtilde"][batch.valid.bool()] == 1).all())


@pytest.mark.parametrize("with_kl", [False, True])
def test_stale_old_policy_and_kl(ctx, with_kl):
    """log pi_old != log pi_train: ratios on both sides of the clip range; optionally the KL term."""
    shape = W.config(4).scaled(vocab=3000, len_div=32, seed=41)
    batch = gen(shape)
    # inputs of the method must not come from the path under test: torch's own log_softmax stands in for the
    # trainer's log-probs when building the stale old-policy and reference log-probs
    logp = torch.log_softmax(batch.logits.float(), dim=1).gather(1, batch.token_ids.long().unsqueeze(1)).squeeze(1)
    g = torch.Generator(device="cuda").manual_seed(3)
    logp_old = logp + 0.25 * torch.randn(logp.shape, device="cuda", generator=g)
    # keep ratios away from the clip edges so that fp32 vs fp64 log-probs cannot flip a branch
    rho = torch.exp(logp - logp_old)
    near = ((rho - 0.8).abs() < 1e-3) | ((rho - 1.2).abs() < 1e-3)
    logp_old = torch.where(near, logp, logp_old)
    p = B.default_params(beta_kl=0.04 if with_kl else 0.0)
    logp_ref = logp + 0.3 * torch.randn(logp.shape, device="cuda", generator=g) if with_kl else None
    out, ref, d = P.check(ctx, batch, p, logp_old=logp_old, logp_ref=logp_ref)
    rho = np.exp(ref["logp"] - P.to_np64(logp_old))
    assert (rho > 1.2).any() and (rho < 0.8).any()


@pytest.mark.parametrize("mode", ["tis", "grpo", "clipped_kl_norm_temp"])
def test_baseline_modes_full_vocab(ctx, mode):
    """The paper's comparison configurations on the real row geometry (V = 151,936): token-level truncated IS
    (alpha forced to 1, Eq. 8), uncorrected GRPO (alpha forced to 0), and the general clipped surrogate of
    Eq. 19 with a stale old policy, the KL term, normalised advantages and a sampling temperature together."""
    shape = W.config(2).scaled(len_div=96, seed=91)
    batch = gen(shape, row_chunk=128)
    if mode == "tis":
        P.check(ctx, batch, B.default_params(alpha_override=1.0))
    elif mode == "grpo":
        out, ref, d = P.check(ctx, batch, B.default_params(alpha_override=0.0))
        assert d["alpha"] == 0.0
    else:
        p = B.default_params(beta_kl=0.02, adv_mode=1, inv_temperature=1 / 0.9)
        lp = torch.log_softmax(batch.logits.float() * p.inv_temperature, dim=1)
        lp = lp.gather(1, batch.token_ids.long().unsqueeze(1)).squeeze(1)
        g = torch.Generator(device="cuda").manual_seed(5)
        logp_old = lp + 0.2 * torch.randn(lp.shape, device="cuda", generator=g)
        rho = torch.exp(lp - logp_old)
        logp_old = torch.where(((rho - 0.8).abs() < 1e-3) | ((rho - 1.2).abs() < 1e-3), lp, logp_old)
        logp_ref = lp + 0.3 * torch.randn(lp.shape, device="cuda", generator=g)
        P.check(ctx, batch, p, logp_old=logp_old, logp_ref=logp_ref)


def test_in_place_gradient(ctx):
    shape = W.config(2).scaled(vocab=4104, len_div=32, seed=51)
    batch = gen(shape)
    ptr = batch.logits.data_ptr()
    out, ref, d = P.check(ctx, batch, in_place=True)
    assert out["dlogits"].data_ptr() == ptr


# ------------------------------------------------------------------ reproducibility and device-detected faults
def test_bit_reproducible(ctx):
    shape = W.config(3).scaled(vocab=5000, len_div=4, n_prompts=2, seed=61)
    batch = gen(shape)
    a = ctx.step(batch)
    b = ctx.step(batch)
    torch.cuda.synchronize()
    for k in ("logp", "lse", "adv", "count", "diag", "loss", "wtilde", "dlogits"):
        assert torch.equal(a[k], b[k]), k


def test_bad_token_is_flagged_not_dereferenced(ctx):
    shape = W.config(2).scaled(vocab=1000, len_div=128, seed=71)
    batch = gen(shape)
    batch.token_ids[3] = 1000          # == vocab
    batch.token_ids[7] = -5
    batch.token_ids[9] = 2 ** 30
    out = ctx.step(batch)
    torch.cuda.synchronize()
    assert ctx.status() & B.STATUS_BAD_TOKEN
    assert out["logp"][3].item() == 0 and out["logp"][7].item() == 0 and out["logp"][9].item() == 0
    assert torch.isfinite(out["dlogits"].float()).all()
    assert ctx.status() == 0           # reading cleared it


def test_bad_cu_rows_is_flagged(ctx):
    shape = W.config(2).scaled(vocab=512, len_div=128, seed=81)
    batch = gen(shape)
    cu = batch.cu_rows.clone()
    cu[3], cu[4] = cu[4].item(), cu[3].item()          # not monotone
    cu[-1] = batch.n_rows + 1000                        # beyond the rows
    logp, lse = ctx.token_logprob(batch.logits, batch.token_ids, batch.valid)
    adv, count, diag = ctx.diagnostics(logp, batch.logp_roll, batch.valid, cu, batch.rewards, 8)
    torch.cuda.synchronize()
    assert ctx.status() & B.STATUS_BAD_CU
    assert int(count.max().item()) <= batch.n_rows and int(count.min().item()) >= 0   # ranges were clamped


def _bits(t):
    """Raw values of a device tensor as numpy: bf16 as uint16 bit patterns, fp32 as it is."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def _report(k, line):
    """Progress and results of the whole-batch test, for the run log (pytest swallows stdout of passing tests)."""
    where = os.environ.get("AIS_PARITY_REPORT_DIR")
    if where and os.path.isdir(where):
        with open(os.path.join(where, f"full_size_parity_cfg{k}.log"), "a") as f:
            f.write(line + "\n")
    print(line, flush=True)


@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_full_size_whole_batch(ctx, k):
    """Workloads 2-5 at full size, the very bits and launch configuration the benchmark times: EVERY row goes
    through the oracle (spread over the host's cores), and the comparison is the strict one: log-probs and lse of
    every row at 2e-3, counts exact, every diagnostic, alpha and the loss at plain relative 1e-3, w_tilde per row,
    and the gradient element by element for every row, for the three-call path (dlogits) and the one-sweep path
    (g * s)."""
    from tests import full_size as F

    batch = gen(W.config(k), row_chunk=512)
    p = B.default_params()
    op = P.oracle_params(p)
    t_start = time.perf_counter()
    out = ctx.step(batch, p)
    one = ctx.step_one_sweep(batch, p)
    torch.cuda.synchronize()
    assert ctx.status() == 0
    R, V = batch.logits.shape
    dtype = batch.shape.logits_dtype
    valid = batch.valid.cpu().numpy()
    y = batch.token_ids.cpu().numpy()
    cu = batch.cu_rows.cpu().numpy()
    seg_rows, chunk = 2048, 32
    segs = [(a, min(R, a + seg_rows)) for a in range(0, R, seg_rows)]
    seg_bytes = seg_rows * V * batch.logits.element_size()
    w = F.Workers()
    try:
        keep_z = w.free_bytes() > R * V * batch.logits.element_size() + 8 * seg_bytes
        _report(k, f"cfg {k}: R={R} V={V} workers={w.n} segments={len(segs)} keep_logits_files={keep_z}")

        def cuts(a, b):
            return [(r0, min(b, r0 + chunk)) for r0 in range(a, b, chunk)]

        # ---- pass 1: log-probs of every row (O1)
        logp, lse = np.zeros(R), np.zeros(R)
        zfiles = {}
        pending = []

        def collect1():
            a, b, zpath, futs = pending.pop(0)
            for (r0, r1), f in zip(cuts(a, b), futs):
                logp[r0:r1], lse[r0:r1] = f.result()
            if not keep_z:
                w.drop(zpath)

        for a, b in segs:
            zpath = w.put(f"z{a}", _bits(batch.logits[a:b]))
            zfiles[a] = zpath
            futs = [w.pool.submit(F.logprob_task, (zpath, r0 - a, r1 - a, dtype, y[r0:r1], valid[r0:r1],
                                                   op.inv_temperature)) for r0, r1 in cuts(a, b)]
            pending.append((a, b, zpath, futs))
            if len(pending) > 1:
                collect1()
        while pending:
            collect1()
        t1 = time.perf_counter()
        # ---- per-row scalars (O2-O6)
        adv = O.group_advantages(P.to_np64(batch.rewards), batch.shape.group_size, op.adv_mode, op.eps_std)
        lp_roll = P.to_np64(batch.logp_roll)
        diag = O.diagnostics(logp, lp_roll, valid, cu, adv, op)
        loss, wtilde, g = O.loss_and_row_coeff(logp, lp_roll, None, None, valid, cu, adv, diag["count"], diag["alpha"], op)
        ref = dict(logp=logp, lse=lse, adv=adv, diag=diag, loss=loss, wtilde=wtilde, g=g, params=op,
                   kl_sens=np.zeros(R), g_slack=np.zeros(R))
        d = P.compare_scalars(ctx, out, ref, batch, strict=True)
        d1 = P.compare_scalars(ctx, one, ref, batch, strict=True)
        g_gpu = P.to_np64(one["g"])
        g_ref = g * op.inv_temperature
        assert np.all(g_gpu[g_ref == 0] == 0)
        assert np.all(np.abs(g_gpu - g_ref) <= P.REL * np.abs(g_ref)), "one-sweep row coefficient"
        _report(k, f"cfg {k}: alpha gpu {d['alpha']!r} oracle {diag['alpha']!r}; loss gpu {float(out['loss'].item())!r} "
                   f"oracle {loss!r}; n_valid {d['n_valid']}; max|dlogp| {d['_E']:.3e}; pass 1 {t1 - t_start:.1f} s")
        # ---- pass 2: the gradient of every row (O7) against dlogits and against g * s
        stats = []
        pending2 = []

        def collect2():
            paths, futs = pending2.pop(0)
            stats.extend(f.result() for f in futs)
            w.drop(*paths)

        for a, b in segs:
            zpath = zfiles[a] if keep_z else w.put(f"z{a}", _bits(batch.logits[a:b]))
            dzpath = w.put(f"dz{a}", _bits(out["dlogits"][a:b, :V]))
            spath = w.put(f"s{a}", _bits(one["sgrad"][a:b, :V]))
            futs = [w.pool.submit(F.gradient_task, (zpath, dzpath, spath, r0 - a, r1 - a, dtype, lse[r0:r1], y[r0:r1],
                                                    g[r0:r1], g_gpu[r0:r1], op.inv_temperature, True))
                    for r0, r1 in cuts(a, b)]
            pending2.append(((zpath, dzpath, spath), futs))
            if len(pending2) > 1:
                collect2()
        while pending2:
            collect2()
    finally:
        w.close()
    t2 = time.perf_counter()
    assert sum(s_["rows"] for s_ in stats) == R
    firsts = [s_["first_bad"] for s_ in stats if s_["first_bad"] is not None]
    n_bad_dz, n_bad_gs = sum(s_["dz_bad"] for s_ in stats), sum(s_["gs_bad"] for s_ in stats)
    worst_dz, worst_gs = max(s_["dz_worst"] for s_ in stats), max(s_["gs_worst"] for s_ in stats)
    worst = {q: round(v, 4) for q, v in d["_worst"].items()}
    _report(k, f"cfg {k}: dlogits worst error / bound {worst_dz:.4f} ({n_bad_dz} over), g*s {worst_gs:.4f} ({n_bad_gs} over); "
               f"pass 2 {t2 - t1:.1f} s; scalars as fractions of their bounds {worst}; one-sweep alpha {d1['alpha']!r}")
    assert n_bad_dz == 0 and n_bad_gs == 0, firsts[:3]
    assert all(s_["dz_zero_rows_exact"] and s_["gs_zero_rows_exact"] for s_ in stats)
    assert all(s_["dz_live_rows_written"] and s_["gs_live_rows_written"] for s_ in stats)
    assert sum(s_["abs_sum"] for s_ in stats) > 0 and d["alpha"] > 0
    where = os.environ.get("AIS_PARITY_REPORT_DIR")
    if where and os.path.isdir(where):
        import json
        with open(os.path.join(where, f"full_size_parity_cfg{k}.json"), "w") as f:
            json.dump(dict(workload=k, rows=R, valid_rows=int(d["n_valid"]), vocab=V, alpha_gpu=d["alpha"],
                           alpha_oracle=diag["alpha"], loss_gpu=float(out["loss"].item()), loss_oracle=loss,
                           max_abs_dlogp=d["_E"], worst_over_bound=dict(d["_worst"], dlogits=worst_dz, one_sweep_g_s=worst_gs),
                           seconds=t2 - t_start), f)
