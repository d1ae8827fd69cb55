"""The path recorded into a HIP graph and replayed: serving loops and trainers that capture their step must get the
bits of the eager calls.  After one eager warm-up (which sizes the context's workspace) the calls only launch kernels:
no allocation, no synchronisation, no memset node.  Every replay runs on new input values, with eager work and
synchronisations between the replays, and is compared bit for bit with the eager path on the same values."""
import numpy as np
import pytest
import torch

from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.AisContext()
    yield c
    c.close()


def same_bits(a: torch.Tensor, b: torch.Tensor) -> bool:
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def perturb(batch, k: int):
    """New values in the same buffers (the graph holds their addresses)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 + k)
    noise = torch.randn(batch.logits.shape[1], generator=gen, device="cuda", dtype=torch.float32) * 0.5
    batch.logits.copy_((batch.logits.float() + noise).to(batch.logits.dtype))
    live = batch.valid.bool()
    batch.logp_roll.add_(torch.where(live, torch.randn(batch.logp_roll.shape, generator=gen, device="cuda") * 0.02,
                                     torch.zeros_like(batch.logp_roll)))
    batch.rewards.copy_((torch.rand(batch.rewards.shape, generator=gen, device="cuda") < 0.5).float())


@pytest.mark.parametrize("which", ["three_call", "one_sweep"])
@pytest.mark.parametrize("cfg,vocab,len_div", [(1, None, 1), (2, 20_008, 64), (3, 9_000, 8)])
def test_replays_equal_eager(ctx, which, cfg, vocab, len_div):
    shape = W.config(cfg) if vocab is None else W.config(cfg).scaled(vocab=vocab, len_div=len_div, seed=77)
    batch = W.generate(shape, device="cuda")
    p = B.default_params()
    run = (lambda: ctx.step(batch, p)) if which == "three_call" else (lambda: ctx.step_one_sweep(batch, p))
    run()                                        # warm-up: workspace, kernel attributes
    torch.cuda.synchronize()
    assert ctx.status() == 0
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = run()
    keys = [k for k, v in out.items() if isinstance(v, torch.Tensor)]
    alphas = []
    for k in range(4):
        perturb(batch, k)
        ref = run()                              # eager, between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in keys:
            assert same_bits(out[name], ref[name]), f"replay {k}: {name} differs from the eager call"
        alphas.append(ctx.read_diag(out["diag"])["alpha"])
        assert ctx.status() == 0
    assert len(set(alphas)) > 1, "the replays must have seen different inputs"


def test_static_diagnostics_replays(ctx):
    """The diagnostics call that allocates nothing, recorded without any warm-up of its own size."""
    shape = W.config(5).scaled(vocab=512, len_div=16, seed=5)
    batch = W.generate(shape, device="cuda")
    p = B.default_params()
    logp, _ = ctx.token_logprob(batch.logits, batch.token_ids, batch.valid)
    torch.cuda.synchronize()
    args = (logp, batch.logp_roll, batch.valid, batch.cu_rows, batch.rewards, shape.group_size, p)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        adv, count, diag = ctx.diagnostics(*args, static_scratch=True)
    for k in range(3):
        batch.logp_roll.add_(0.01 * (k + 1) * batch.valid.float())
        ref = ctx.diagnostics(*args)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert same_bits(adv, ref[0]) and same_bits(count, ref[1]) and same_bits(diag, ref[2])
    assert ctx.status() == 0
