"""Every kernel that holds or bursts a whole row picks an instantiation by the number of 16-byte vectors per lane,
k = ceil(V / (1024 N)) (N = 8 bf16 or 4 fp32 elements per vector), and skips the bounds check for vectors that the
class guarantees.  This file walks the widths around every class boundary — V = 1024 N k - 1, exactly 1024 N k,
+ 1 (a scalar tail), + N (one more vector: the next class with a single lane in its last slot) — through both
paths and the FP8 kernels, on a few rows each."""
import numpy as np
import pytest
import torch

from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W
from tests import parity as P
from tests.test_gpu_fp8 import check_quant
from tests.test_gpu_one_sweep import check_one_sweep

pytestmark = pytest.mark.gpu

K = [1, 4, 5, 8, 9, 12, 13, 14, 15, 16, 17, 18, 19, 20, 21, 23, 24, 25, 27, 28, 29, 30, 31, 32, 33, 34, 48, 49]


@pytest.fixture(scope="module")
def ctx():
    c = B.AisContext()
    yield c
    c.close()


def widths(k, n):
    edge = 1024 * n * k
    return [edge - 1, edge, edge + 1, edge + n]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("k", K)
def test_paths_at_class_boundaries(ctx, k, dtype):
    n = 8 if dtype == "bf16" else 4
    for vocab in widths(k, n):
        shape = W.RolloutShape("edge", n_prompts=1, group_size=2, vocab=vocab, logits_dtype=dtype, sigma=2.5, boost=4.0,
                               layout="padded", max_len=2, length_dist=("uniform", 1, 2), reward_p=0.5,
                               seed=vocab % 100_003)
        batch = W.generate(shape, "cuda")
        batch.rewards[:] = torch.tensor([1, 0], dtype=torch.float32)
        print("vocab", vocab, flush=True)
        P.check(ctx, batch)
        check_one_sweep(ctx, batch)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("k", K)
def test_fp8_at_class_boundaries(ctx, k, dtype):
    n = 8 if dtype == "bf16" else 4
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for vocab in widths(k, n):
        g = torch.Generator(device="cuda")
        g.manual_seed(vocab)
        z = (torch.randn(3, vocab, generator=g, device="cuda") * 3.0).to(dt)
        z[1, vocab - 1] = -47.0                      # the abs-max in the last element (the tail, or the last vector)
        print("vocab", vocab, flush=True)
        check_quant(ctx, z)
