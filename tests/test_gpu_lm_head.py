"""GPU parity of the hidden-state read-out (ais_lm_head_logprob) against the CPU oracle
(oracle/lm_head_oracle.py) on the same seeded bits.

Tolerance: the bar of the log-prob step, |gpu - oracle| <= 2e-3 absolute on evaluated rows and exactly 0 on
the others.  The inputs are bf16, so every product is exact in fp32 and the only error against the fp64
oracle is the fp32 accumulation over d_model terms (about sqrt(d_model) * 2^-24 * |z|, 1e-5 at d_model = 4096)
plus the fp32 exp/log of the soft-max; the observed maximum is printed by each test."""
import os

import numpy as np
import pytest
import torch

import oracle.lm_head_oracle as L
from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W

pytestmark = pytest.mark.gpu
LOGP_ATOL = 2e-3


@pytest.fixture(scope="module")
def ctx():
    c = B.AisContext()
    yield c
    c.close()


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def compare(ctx, hidden, weight, y, valid, inv_t=1.0, rows=None):
    """Runs the GPU path on everything, the oracle on `rows` (all rows if None)."""
    logp, lse = ctx.lm_head_logprob(hidden, weight, y, valid, inv_t)
    torch.cuda.synchronize()
    status = ctx.status()
    R = hidden.shape[0]
    sel = np.arange(R) if rows is None else np.asarray(rows)
    v_np = np.ones(R, bool) if valid is None else valid.cpu().numpy().astype(bool)
    y_np = y.cpu().numpy().astype(np.int64)
    y_ok = (y_np >= 0) & (y_np < weight.shape[0])
    ref_logp, ref_lse = L.token_logprob(f64(hidden[torch.from_numpy(sel).to(hidden.device)]), f64(weight),
                                        np.where(y_ok, y_np, 0)[sel], v_np[sel], inv_t)
    got_logp, got_lse = logp.cpu().numpy()[sel], lse.cpu().numpy()[sel]
    ev = v_np[sel]
    assert np.all(got_logp[~ev] == 0.0) and np.all(got_lse[~ev] == 0.0)
    err_lse = np.abs(got_lse[ev] - ref_lse[ev]).max() if ev.any() else 0.0
    good = ev & y_ok[sel]
    err_lp = np.abs(got_logp[good] - ref_logp[good]).max() if good.any() else 0.0
    print(f"max |dlogp| {err_lp:.2e}  max |dlse| {err_lse:.2e}  rows {len(sel)}", flush=True)
    assert err_lse <= LOGP_ATOL and err_lp <= LOGP_ATOL
    bad = ev & ~y_ok[sel]
    assert np.all(got_logp[bad] == 0.0)
    assert bool(status & 1) == bool((v_np & ~y_ok).any())
    return logp, lse


def make(R, D, V, seed, p_valid=1.0, scale=1.0, device="cuda"):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    hidden = (torch.randn(R, D, generator=g) * scale).to(torch.bfloat16).to(device)
    weight = (torch.randn(V, D, generator=g) / np.sqrt(D) * 3.0).to(torch.bfloat16).to(device)
    y = torch.randint(0, V, (R,), generator=g, dtype=torch.int32).to(device)
    valid = None
    if p_valid < 1.0:
        valid = (torch.rand(R, generator=g) < p_valid).to(torch.uint8).to(device)
    return hidden, weight, y, valid


# several tiles in both directions, ragged tails in rows, vocabulary and d_model, and the degenerate sizes.
# d_model a multiple of 32 takes the streaming kernel (32: a single step per tile, fewer steps than LDS stages),
# any other multiple of 8 the register-staged one.
SHAPES = [
    (1, 8, 1), (1, 64, 1000), (3, 8, 2), (5, 32, 100), (256, 64, 256), (257, 64, 257), (300, 72, 1000),
    (64, 40, 300), (300, 96, 600), (513, 128, 2049), (1000, 200, 700), (640, 512, 5000), (255, 64, 70_000),
    (700, 32, 1300),
]


@pytest.mark.parametrize("R,D,V", SHAPES)
def test_shapes(ctx, R, D, V):
    hidden, weight, y, valid = make(R, D, V, seed=R * 7 + D + V, p_valid=0.8 if R > 3 else 1.0)
    compare(ctx, hidden, weight, y, valid)


@pytest.mark.parametrize("seed", range(int(os.environ.get("AIS_RANDOM_CASES", "40"))))
def test_random_shapes(ctx, seed):
    """Seeded random draws of rows, model width (both kernels), vocabulary, mask density, temperature, operand scale
    and row pitches."""
    rng = np.random.default_rng(500 + seed)
    R = int(rng.choice([1, 2, 31, 255, 256, 257, 300, 511, 513, 700, 1025]))
    D = int(rng.choice([8, 16, 24, 32, 40, 64, 72, 96, 128, 160, 200, 256, 320]))
    V = int(rng.choice([1, 2, 7, 255, 256, 257, 511, 1000, 2049, 5000, 12_345, 33_333]))
    p_valid = float(rng.choice([1.0, 0.9, 0.5, 0.1]))
    inv_t = float(rng.choice([0.3, 0.7, 1.0, 1.0, 1.9]))
    scale = float(rng.choice([0.05, 1.0, 1.0, 6.0, 40.0]))
    pad_h, pad_w = int(rng.choice([0, 8, 24])), int(rng.choice([0, 8, 40]))
    print(f"case {seed}: R={R} D={D} V={V} p_valid={p_valid} inv_t={inv_t} scale={scale} pads={pad_h},{pad_w}", flush=True)
    hidden, weight, y, valid = make(R, D, V, seed=900 + seed, p_valid=p_valid, scale=scale)
    if pad_h:
        hs = torch.full((R, D + pad_h), float("nan"), dtype=torch.bfloat16, device="cuda")
        hs[:, :D] = hidden
        hidden = hs[:, :D]
    if pad_w:
        ws = torch.full((V, D + pad_w), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws[:, :D] = weight
        weight = ws[:, :D]
    logp, lse = compare(ctx, hidden, weight, y, valid, inv_t)
    assert torch.isfinite(logp).all() and torch.isfinite(lse).all()


@pytest.mark.parametrize("inv_t", [0.5, 1.0, 1.7])
def test_temperature_and_peaked_rows(ctx, inv_t):
    hidden, weight, y, valid = make(400, 256, 3000, seed=11, scale=4.0)
    # make half of the rows sharply peaked on their sampled token
    w_y = weight[y[:200].long()].float()
    hidden[:200] = (hidden[:200].float() + 6.0 * w_y / (w_y * w_y).sum(1, keepdim=True)).to(torch.bfloat16)
    compare(ctx, hidden, weight, y, valid, inv_t)


def test_large_logits(ctx):
    """Hidden states a hundred times larger: logits hundreds of units apart, sampled tokens with probabilities far
    below fp32 range; the running maximum keeps every exponential in range and the log-prob stays finite."""
    hidden, weight, y, valid = make(300, 128, 3000, seed=18, scale=100.0)
    logp, lse = compare(ctx, hidden, weight, y, valid)
    assert torch.isfinite(logp).all() and float(logp.min()) < -200.0


def test_deep_contraction(ctx):
    """d_model = 4096: the accumulation length of the real workloads."""
    hidden, weight, y, valid = make(512, 4096, 4096, seed=12, p_valid=0.9)
    compare(ctx, hidden, weight, y, valid)


def test_strided_operands(ctx):
    hidden, weight, y, valid = make(300, 64, 900, seed=13)
    hs = torch.zeros(300, 96, dtype=torch.bfloat16, device="cuda")
    ws = torch.full((900, 136), float("nan"), dtype=torch.bfloat16, device="cuda")
    hs[:, :64] = hidden
    ws[:, :64] = weight
    a = compare(ctx, hs[:, :64], ws[:, :64], y, valid)
    b = ctx.lm_head_logprob(hidden, weight, y, valid)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_bad_tokens_and_masked_rows(ctx):
    hidden, weight, y, valid = make(300, 64, 500, seed=14, p_valid=0.7)
    y = y.clone()
    y[5] = 500
    y[17] = -3
    valid[5] = 1
    valid[17] = 1
    hidden[torch.nonzero(valid == 0)[0]] = float("nan")          # rows that are not evaluated may hold anything
    compare(ctx, hidden, weight, y, valid)
    assert ctx.status() == 0                                      # reading the status cleared it


@pytest.mark.parametrize("p_valid", [0.03, 0.3, 0.97])
def test_masked_rows_are_gathered(ctx, p_valid):
    """Only evaluated rows are read and computed: every other row holds NaN, the first and last rows are masked,
    and the evaluated rows straddle several token blocks."""
    hidden, weight, y, _ = make(3000, 128, 2000, seed=21)
    g = torch.Generator(device="cpu")
    g.manual_seed(22)
    valid = (torch.rand(3000, generator=g) < p_valid).to(torch.uint8)
    valid[0] = valid[-1] = 0
    valid[1500] = 1
    valid = valid.cuda()
    hidden[valid == 0] = float("nan")
    y = torch.where(valid.bool(), y, torch.full_like(y, -1))
    compare(ctx, hidden, weight, y, valid)


def test_all_rows_masked(ctx):
    hidden, weight, y, _ = make(70, 64, 300, seed=15)
    valid = torch.zeros(70, dtype=torch.uint8, device="cuda")
    logp, lse = ctx.lm_head_logprob(hidden, weight, y, valid)
    torch.cuda.synchronize()
    assert not logp.any() and not lse.any() and ctx.status() == 0


def test_empty_batch(ctx):
    hidden, weight, y, _ = make(4, 64, 300, seed=16)
    logp, lse = ctx.lm_head_logprob(hidden[:0], weight, y[:0], None)
    assert logp.numel() == 0 and lse.numel() == 0


def test_reproducible(ctx):
    hidden, weight, y, valid = make(700, 128, 3000, seed=17)
    a = ctx.lm_head_logprob(hidden, weight, y, valid)
    b = ctx.lm_head_logprob(hidden, weight, y, valid)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_workload_1(ctx):
    batch = W.generate_readout(W.config(1), device="cuda")
    compare(ctx, batch.hidden, batch.weight, batch.token_ids, batch.valid)


def test_workload_3_masked_full_vocab(ctx):
    """The masked-diffusion workload (about half of the positions evaluated) at its full vocabulary and model width,
    on a slice of its rows; the oracle evaluates a sample."""
    shape = W.config(3)
    batch = W.generate_readout(shape, device="cuda", n_rows=6000)
    v = batch.valid.cpu().numpy().astype(bool)
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([np.flatnonzero(v)[[0, 1, 255, 256, -1]], rng.integers(0, 6000, 30)]))
    compare(ctx, batch.hidden, batch.weight, batch.token_ids, batch.valid, rows=rows)


def test_workload_4_widest_vocabulary(ctx):
    """The widest vocabulary of the workloads (248,320 = 970 tiles) on 1,024 of its rows: few token blocks, so the
    device-side decomposition uses its largest chunk counts."""
    batch = W.generate_readout(W.config(4), device="cuda", n_rows=1024)
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, 255, 256, 1023], rng.integers(0, 1024, 20)]))
    compare(ctx, batch.hidden, batch.weight, batch.token_ids, batch.valid, rows=rows)


def test_full_size_sampled(ctx):
    """Workload 2 at full size (41,643 rows, d_model 4096, vocabulary 151,936) in the launch configuration the
    benchmark times; the oracle evaluates a sample of rows that covers the first and last token block and the
    block boundaries."""
    shape = W.config(2)
    batch = W.generate_readout(shape, device="cuda")
    R = batch.hidden.shape[0]
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, R - 257, R - 256, R - 1], rng.integers(0, R, 40)]))
    compare(ctx, batch.hidden, batch.weight, batch.token_ids, batch.valid, rows=rows)


def test_hidden_state_path_end_to_end(ctx):
    """The path without materialised logits: log-probs from hidden states, then the diagnostics and the per-row
    gradient coefficient.  The oracle forms the logits in fp64 and runs its own steps on them; what comes out of the
    three calls (alpha, loss, w_tilde, g) must agree to the tolerances of the logits-based path."""
    import oracle.ais_oracle as O
    from tests import parity as P
    R, D, V, G, n_resp = 640, 128, 3000, 4, 8
    hidden, weight, y, _ = make(R, D, V, seed=71)
    g = torch.Generator(device="cpu")
    g.manual_seed(72)
    valid = (torch.rand(R, generator=g) < 0.85).to(torch.uint8)
    cu = torch.arange(n_resp + 1, dtype=torch.int64) * (R // n_resp)
    rewards = torch.tensor([1, 0, 0, 1, 0, 1, 1, 0], dtype=torch.float32)
    inv_t = 1.0 / 0.9
    p = B.default_params(inv_temperature=inv_t, beta_kl=0.04)
    z = L.logits(f64(hidden), f64(weight))
    lp_ref, lse_ref = O.token_logprob(z, y.cpu().numpy(), valid.numpy(), inv_t)
    rng = np.random.default_rng(73)
    logp_roll = np.where(valid.numpy() != 0, lp_ref + rng.normal(0, 0.05, size=R), 0.0).astype(np.float32)
    logp_ref_policy = np.where(valid.numpy() != 0, lp_ref + rng.normal(0, 0.1, size=R), 0.0).astype(np.float32)
    op = P.oracle_params(p)
    adv_ref = O.group_advantages(rewards.double().numpy(), G, op.adv_mode, op.eps_std)
    rd = O.diagnostics(lp_ref, logp_roll, valid.numpy(), cu.numpy(), adv_ref, op)
    loss_ref, wt_ref, g_ref = O.loss_and_row_coeff(lp_ref, logp_roll.astype(np.float64), None,
                                                   logp_ref_policy.astype(np.float64), valid.numpy(), cu.numpy(),
                                                   adv_ref, rd["count"], rd["alpha"], op)

    dev = lambda a: torch.from_numpy(a).cuda() if isinstance(a, np.ndarray) else a.cuda()
    logp, lse = ctx.lm_head_logprob(hidden, weight, y, dev(valid), inv_t)
    adv, count, diag = ctx.diagnostics(logp, dev(logp_roll), dev(valid), dev(cu), dev(rewards), G, p)
    loss, wtilde, gcoef = ctx.grpo_row_scale(logp, dev(logp_roll), dev(valid), dev(cu), adv, count, diag, p,
                                             logp_ref=dev(logp_ref_policy))
    torch.cuda.synchronize()
    d = ctx.read_diag(diag)
    E = float(np.abs(logp.cpu().numpy() - lp_ref).max())
    print(f"max |dlogp| {E:.2e}", flush=True)
    assert E <= LOGP_ATOL and ctx.status() == 0
    assert d["n_valid"] == rd["n_valid"] and count.cpu().tolist() == [int(c) for c in rd["count"]]
    for k in ("mean_w", "cv2", "dbar", "dsigma", "alpha_ess", "alpha_mis", "alpha"):
        P.rel_close(d[k], rd[k], floor=1e-6 + 10 * E, what=k)
    np.testing.assert_allclose(wtilde.cpu().numpy(), wt_ref, rtol=P.REL, atol=1e-6 + 10 * E)
    np.testing.assert_allclose(gcoef.cpu().numpy(), g_ref * inv_t, rtol=P.REL,
                               atol=(1e-6 + 10 * E) * float(np.abs(g_ref).max()))
    scale = float(np.sum(np.abs(adv_ref)) / n_resp) + op.beta_kl
    assert abs(float(loss.item()) - loss_ref) <= (P.REL + 10 * E) * max(abs(loss_ref), scale)
