"""GPU parity on seeded random configurations: every case draws its own vocabulary width, batch structure,
dtype, hyper-parameters, temperature, optional stale / reference policies, banned (-inf) tokens, logit magnitude
and memory layout, and runs the three-call path and the one-sweep path against the CPU oracle with the same
tolerances as the other parity tests.  The draws are functions of the seed alone, so a failure names its case."""
import os

import numpy as np
import pytest
import torch

from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W
from tests import parity as P
from tests.test_gpu_one_sweep import check_one_sweep

pytestmark = pytest.mark.gpu

# widths around the boundaries of the kernels' row-width classes and vector sizes, and ordinary ones
VOCABS = [1, 2, 3, 7, 8, 9, 31, 64, 255, 256, 257, 1000, 1023, 1024, 1025, 2047, 4097, 8191, 8192, 8200, 12_289,
          16_385, 20_481, 33_001, 40_961, 66_000, 98_312, 131_073, 151_936, 200_003, 262_147]


@pytest.fixture(scope="module")
def ctx():
    c = B.AisContext()
    yield c
    c.close()


def draw_case(seed):
    rng = np.random.default_rng(10_000 + seed)
    vocab = int(rng.choice(VOCABS))
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    group_size = int(rng.choice([1, 2, 4, 8]))
    n_prompts = int(rng.integers(1, 4))
    layout = str(rng.choice(["packed", "padded", "masked"]))
    max_len = int(rng.integers(1, 4 if vocab > 90_000 else 13 if vocab > 20_000 else 40))
    lo = int(rng.integers(1, max_len + 1))
    shape = W.RolloutShape(f"random{seed}", n_prompts=n_prompts, group_size=group_size, vocab=vocab,
                           logits_dtype=dtype, sigma=float(rng.uniform(0.5, 4.0)),
                           boost=float(rng.choice([0.0, 4.0, 8.0])), layout=layout, max_len=max_len,
                           length_dist=("uniform", lo, max_len), reward_p=float(rng.uniform(0.2, 0.8)),
                           rollout_noise=float(rng.choice([0.0, 0.0, 0.5])), seed=int(rng.integers(1, 1 << 30)))
    params = dict(C=float(rng.choice([1.0, 2.0, 5.0, 20.0])), delta=float(rng.choice([0.005, 0.02, 0.3])),
                  gamma=float(rng.choice([0.3, 1.2, 3.0])), beta_var=float(rng.choice([0.0, 0.25, 1.0])),
                  clip_eps=float(rng.choice([0.0, 0.1, 0.2, 0.5])), adv_mode=int(rng.integers(0, 2)),
                  alpha_override=float(rng.choice([-1.0, -1.0, -1.0, 0.0, 0.37, 1.0])),
                  inv_temperature=float(rng.choice([0.25, 0.6, 1.0, 1.0, 1.0 / 0.9, 2.5])),
                  beta_kl=float(rng.choice([0.0, 0.0, 0.04, 0.5])), eps_std=float(rng.choice([1e-6, 1e-6, 0.0])))
    extras = dict(stale=bool(rng.random() < 0.4), ban=float(rng.choice([0.0, 0.0, 0.3, 0.9])),
                  factor=float(rng.choice([1.0, 1.0, 1.0, 30.0, 0.01])), in_place=bool(rng.random() < 0.3),
                  pad=int(rng.choice([0, 0, 8, 24])), mixed_rewards=bool(rng.random() < 0.8))
    return shape, params, extras, rng


def build_case(seed):
    shape, params, extras, rng = draw_case(seed)
    batch = W.generate(shape, "cuda")
    R, V = batch.logits.shape
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    if extras["factor"] != 1.0:
        batch.logits.mul_(extras["factor"])
    if extras["ban"] > 0 and V > 1 and R > 0:
        ban = (torch.rand(R, V, generator=g) < extras["ban"]).cuda()
        ban[torch.arange(R, device="cuda"), batch.token_ids.long().clamp(min=0)] = False
        batch.logits[ban] = float("-inf")
    if extras["mixed_rewards"] and shape.group_size > 1:
        batch.rewards[::2] = 1.0                       # no group with all-equal rewards: every row carries gradient
        batch.rewards[1::2] = 0.0
    if extras["pad"] and R > 0:
        wide = torch.full((R, V + extras["pad"]), 77.0, dtype=batch.logits.dtype, device="cuda")
        wide[:, :V] = batch.logits
        batch.logits = wide[:, :V]                     # row pitch larger than the vocabulary
    p = B.default_params(**params)
    logp_old = logp_ref = None
    if R > 0 and (extras["stale"] or params["beta_kl"] > 0):
        # inputs of the method must not come from the path under test: torch's own soft-max stands in for a policy
        z = batch.logits.float() * params["inv_temperature"]
        lp = torch.log_softmax(z, dim=1)[torch.arange(R, device="cuda"), batch.token_ids.long().clamp(min=0)]
        lp = torch.where(batch.valid.bool(), lp, torch.zeros_like(lp))
        if extras["stale"]:
            logp_old = (lp + 0.25 * torch.randn(R, generator=g).cuda()).contiguous()
        if params["beta_kl"] > 0:
            logp_ref = (lp + 0.1 * torch.randn(R, generator=g).cuda()).contiguous()
    return batch, p, logp_old, logp_ref, extras


# more cases, or another range of seeds, for an occasional long run
FIRST = int(os.environ.get("AIS_RANDOM_FIRST", "0"))
SEEDS = list(range(FIRST, FIRST + int(os.environ.get("AIS_RANDOM_CASES", "160"))))


@pytest.mark.parametrize("seed", SEEDS)
def test_three_call_path(ctx, seed):
    batch, p, logp_old, logp_ref, extras = build_case(seed)
    print("case", seed, batch.shape, extras, flush=True)
    if batch.n_rows == 0:
        pytest.skip("the draw produced an empty batch")
    out, ref, d = P.check(ctx, batch, p, logp_old, logp_ref, in_place=extras["in_place"])
    assert torch.isfinite(out["logp"]).all() and torch.isfinite(out["dlogits"].float()[:, :batch.shape.vocab]).all()
    if extras["pad"] and not extras["in_place"]:
        pass                                           # the output has its own buffer; the padding is not touched
    elif extras["pad"]:
        R, V = batch.logits.shape
        assert bool((batch.logits.as_strided((R, extras["pad"]), batch.logits.stride(), V) == 77.0).all())


@pytest.mark.parametrize("seed", SEEDS)
def test_one_sweep_path(ctx, seed):
    batch, p, logp_old, logp_ref, extras = build_case(seed)
    print("case", seed, batch.shape, extras, flush=True)
    if batch.n_rows == 0:
        pytest.skip("the draw produced an empty batch")
    check_one_sweep(ctx, batch, p, logp_old, logp_ref, in_place=extras["in_place"])
