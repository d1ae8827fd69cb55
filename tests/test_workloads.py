"""The synthetic-input generator: FP8 E4M3 round trip against the format's definition, determinism,
layout structure of the five workloads.  CPU only."""
import math

import numpy as np
import pytest
import torch

from paper_2605_13907_amd import workloads as W


def e4m3_table():
    """All finite values of OCP FP8 E4M3 'fn' from the format definition: sign, 4 exponent bits (bias 7),
    3 mantissa bits, subnormals at exponent 0, S.1111.111 is NaN, no infinities (Sec. 2.1 cites the format)."""
    vals = []
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 0xF, code & 7
        if e == 15 and m == 7:
            continue
        mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        vals.append(-mag if s else mag)
    return sorted(set(vals))


def nearest_even(x, table, mant_even):
    best = min(table, key=lambda t: (abs(t - x), 0 if mant_even[t] else 1))
    return best


def test_e4m3_round_trip_matches_format_definition():
    table = e4m3_table()
    assert max(table) == 448.0 and min(v for v in table if v > 0) == 2.0 ** -9 and len(table) == 253
    # parity of the mantissa code decides ties
    mant_even = {}
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 0xF, code & 7
        if e == 15 and m == 7:
            continue
        mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        mant_even[-mag if s else mag] = (m % 2 == 0)
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.normal(0, 100, 2000), rng.normal(0, 1, 2000), rng.normal(0, 0.01, 500),
                         [0.0, 448.0, -448.0, 447.0, 464.0, 1e6, -1e6, 2.0 ** -10, 3 * 2.0 ** -10, 17.0, 19.0, 21.0]])
    xs = xs.astype(np.float32)
    got = W.e4m3_round_trip(torch.from_numpy(xs)).numpy()
    for x, g in zip(xs, got):
        xc = min(448.0, max(-448.0, float(x)))
        assert g == nearest_even(xc, table, mant_even), (x, g)
    # representable values are fixed points
    t = torch.tensor(table, dtype=torch.float32)
    assert torch.equal(W.e4m3_round_trip(t), t)


def test_rollout_logits_row_scale():
    z = torch.randn(5, 300) * 3
    zr = W.fp8_rollout_logits(z)
    # the row abs-max maps to +-448 and is reproduced to fp32 rounding; relative step of e4m3 is at most 2^-4
    idx = z.abs().argmax(dim=1)
    assert torch.allclose(zr[torch.arange(5), idx], z[torch.arange(5), idx], rtol=1e-6)
    big = z.abs() > z.abs().amax(dim=1, keepdim=True) * 2.0 ** -6 * 8 / 448     # above the subnormal range
    rel = ((zr - z).abs() / z.abs())[big]
    assert rel.max() <= 2.0 ** -4 + 1e-6
    assert torch.equal(W.fp8_rollout_logits(torch.zeros(2, 8)), torch.zeros(2, 8))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_layout_structure(k):
    shape = W.config(k)
    lengths, valid, cu, rewards = W.layout_of(shape)
    B = shape.n_resp
    assert cu.numel() == B + 1 and cu[0] == 0 and bool((cu[1:] >= cu[:-1]).all())
    assert valid.numel() == int(cu[-1]) and rewards.numel() == B
    assert set(rewards.tolist()) <= {0.0, 1.0}
    if shape.layout == "packed":
        assert bool((valid == 1).all()) and torch.equal(cu[1:] - cu[:-1], lengths)
    if shape.layout == "padded":
        v = valid.view(B, shape.max_len)
        assert torch.equal(v.sum(1).to(torch.int64), lengths)
        assert bool((v[:, :16] == 1).all())
    if shape.length_dist[0] == "uniform":
        assert int(lengths.min()) >= shape.length_dist[1] and int(lengths.max()) <= shape.length_dist[2]
    if shape.length_dist[0] == "lognormal":
        assert int(lengths.min()) >= 64 and int(lengths.max()) <= shape.max_len
    # same seed, same structure
    l2, v2, c2, r2 = W.layout_of(shape)
    assert torch.equal(lengths, l2) and torch.equal(valid, v2) and torch.equal(cu, c2) and torch.equal(rewards, r2)
    # every full-size workload must have at least one prompt with mixed rewards, else all gradients vanish
    g = rewards.view(shape.n_prompts, shape.group_size)
    assert bool(((g.sum(1) > 0) & (g.sum(1) < shape.group_size)).any())


def test_generate_small_is_deterministic_and_consistent():
    shape = W.config(2).scaled(vocab=520, len_div=64, seed=5)
    a = W.generate(shape, "cpu", row_chunk=37)
    b = W.generate(shape, "cpu", row_chunk=37)
    for f in ("logits", "token_ids", "valid", "cu_rows", "logp_roll", "rewards"):
        assert torch.equal(getattr(a, f), getattr(b, f)), f
    assert a.logits.dtype == torch.bfloat16 and a.logits.shape == (a.n_rows, 520)
    assert int(a.token_ids.min()) >= 0 and int(a.token_ids.max()) < 520
    # the boosted arg-max dominates the row: it is the row abs-max, so FP8 keeps it (nearly) exactly
    z = a.logits.float()
    assert float((z.amax(1) - z.median(1).values).min()) > 8.0
    # logp_roll is a log-probability of the perturbed row, close to but not equal to the trainer's
    lp_train = torch.log_softmax(z, 1).gather(1, a.token_ids.long().unsqueeze(1)).squeeze(1)
    assert bool((a.logp_roll <= 0).all())
    gap = (lp_train - a.logp_roll).abs()
    assert 0 < float(gap.mean()) < 1.0


def test_generate_masked_rows_carry_no_token():
    shape = W.config(3).scaled(vocab=264, len_div=16, n_prompts=2, seed=11)
    b = W.generate(shape, "cpu")
    off = b.valid == 0
    assert int(off.sum()) > 0 and int((~off).sum()) > 0
    assert bool((b.token_ids[off] == -1).all()) and bool((b.logp_roll[off] == 0).all())
    assert bool((b.token_ids[~off] >= 0).all())


def test_sampled_tokens_follow_rollout_softmax():
    """Gumbel-max draws from softmax(z_r): on a tiny vocabulary the empirical frequencies match."""
    shape = W.RolloutShape("freq", n_prompts=1, group_size=2, vocab=4, logits_dtype="f32", sigma=0.0, boost=0.0,
                           layout="packed", max_len=4000, length_dist=("uniform", 4000, 4000), reward_p=0.5, seed=3)
    b = W.generate(shape, "cpu", row_chunk=8000)
    # sigma = 0: all logits equal, the distribution is uniform over 4 tokens
    freq = torch.bincount(b.token_ids.long(), minlength=4).double() / b.n_rows
    assert float((freq - 0.25).abs().max()) < 0.03
    assert torch.allclose(b.logp_roll, torch.full_like(b.logp_roll, -math.log(4)), atol=1e-6)


def test_readout_generator_structure_and_determinism():
    """Hidden states and output embeddings of the read-out: shapes, dtypes, row structure shared with the rollout
    batch of the same workload, masked rows without a token, the preferred token dominating sharp rows."""
    shape = W.config(1)
    a = W.generate_readout(shape)
    b = W.generate_readout(shape)
    assert torch.equal(a.hidden, b.hidden) and torch.equal(a.weight, b.weight) and torch.equal(a.token_ids, b.token_ids)
    _, valid, _, _ = W.layout_of(shape)
    assert a.hidden.shape == (valid.numel(), W.D_MODEL["tiny"]) and a.weight.shape == (shape.vocab, W.D_MODEL["tiny"])
    assert a.hidden.dtype == torch.bfloat16 and a.weight.dtype == torch.bfloat16
    assert torch.equal(a.valid, valid)
    assert bool((a.token_ids[valid == 0] == -1).all())
    tid = a.token_ids[valid != 0]
    assert int(tid.min()) >= 0 and int(tid.max()) < shape.vocab
    # rows are neither flat nor all one-hot: the largest probability of a row spreads over (0, 1)
    z = a.hidden.double() @ a.weight.double().t()
    pmax = torch.softmax(z, dim=1).max(dim=1).values
    assert float(pmax.min()) < 0.2 and float(pmax.max()) > 0.9
    # a slice of the rows is the leading part of the same batch structure
    c = W.generate_readout(shape, n_rows=100)
    assert c.hidden.shape[0] == 100 and torch.equal(c.valid, valid[:100])


def test_oracle_pool_equals_the_oracle_in_one_process():
    """The worker pool of the CPU-baseline timing only moves data: its results are those of the plain oracle."""
    import numpy as np
    import oracle.ais_oracle as O
    from oracle.pool import OraclePool, widen

    rng = np.random.default_rng(5)
    R, V, G = 96, 300, 4
    z32 = rng.normal(0, 3, size=(R, V)).astype(np.float32)
    bits = (z32.view(np.uint32) >> 16).astype(np.uint16)             # bf16 bit patterns (truncated fp32)
    z = widen(bits, "bf16")
    assert np.array_equal(z, ((bits.astype(np.uint32) << 16).view(np.float32)).astype(np.float64))
    y = rng.integers(0, V, size=R)
    valid = (rng.random(R) < 0.8).astype(np.uint8)
    cu = np.arange(G + 1, dtype=np.int64) * (R // G)
    lp_roll = rng.normal(-3, 0.5, size=R)
    rewards = np.array([1.0, 0.0, 0.0, 1.0])
    ref = O.ais_grpo(z, y, valid, cu, lp_roll, rewards, G, O.Params())
    pool = OraclePool(2)
    try:
        path = pool.share(bits)
        out = pool.whole_path(path, R, "bf16", y, valid, cu, lp_roll, rewards, G, O.Params(), row_chunk=20)
    finally:
        pool.close()
    import os
    assert not os.path.exists(path)                                  # the shared file is gone after close()
    assert np.array_equal(out["logp"], ref["logp"]) and np.array_equal(out["lse"], ref["lse"])
    assert out["loss"] == ref["loss"] and np.array_equal(out["g"], ref["g"])
    assert abs(out["abs_sum"] - np.abs(ref["dz"]).sum()) <= 1e-12 * np.abs(ref["dz"]).sum()
