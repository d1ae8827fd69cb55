"""Contexts and streams.  Two contexts on two streams of one GPU, their calls interleaved from the host: each context
owns its workspace, so the results must be bit-identical to running the same batches one after the other.  And a
context that is destroyed gives back everything it allocated."""
import pytest
import torch

from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W

pytestmark = pytest.mark.gpu


def step(ctx, batch, p):
    return ctx.step(batch, p)


def test_two_contexts_two_streams():
    shapes = [W.config(2).scaled(vocab=20_008, len_div=16, seed=61), W.config(3).scaled(vocab=4_104, len_div=2, seed=62)]
    batches = [W.generate(s, "cuda") for s in shapes]
    p = B.default_params()
    ref_ctx = B.AisContext()
    ref = [step(ref_ctx, b, p) for b in batches]
    torch.cuda.synchronize()
    ref_ctx.close()

    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    ctxs = [B.AisContext(), B.AisContext()]
    outs = [None, None]
    for rep in range(3):                                          # interleaved: a, b, a, b, ... without waiting
        for k in (0, 1):
            with torch.cuda.stream(streams[k]):
                outs[k] = step(ctxs[k], batches[k], p)
    for s in streams:
        s.synchronize()
    for k in (0, 1):
        for name in ("logp", "lse", "wtilde", "dlogits", "adv", "count"):
            assert torch.equal(outs[k][name], ref[k][name]), (k, name)
        assert float(outs[k]["loss"].item()) == float(ref[k]["loss"].item())
        assert ctxs[k].status() == 0
        ctxs[k].close()


def test_context_lifetimes_release_their_memory():
    """Creating a context, running every entry point once and destroying it leaves no device memory behind."""
    shape = W.config(1)
    batch = W.generate(shape, "cuda")
    rb = W.generate_readout(shape, device="cuda")
    p = B.default_params()

    def one_lifetime():
        ctx = B.AisContext()
        ctx.step(batch, p)
        ctx.step_one_sweep(batch, p)
        ctx.lm_head_logprob(rb.hidden, rb.weight, rb.token_ids, rb.valid)
        ctx.profile(True)
        ctx.step(batch, p)
        ctx.profile_read(B.AIS_K_LOGPROB)
        ctx.profile(False)
        assert ctx.status() == 0
        ctx.close()

    for _ in range(3):                                            # torch's caching allocator reaches its steady state
        one_lifetime()
    torch.cuda.synchronize()
    free_before, held_before = torch.cuda.mem_get_info()[0], torch.cuda.memory_reserved()
    for _ in range(100):
        one_lifetime()
    torch.cuda.synchronize()
    free_after, held_after = torch.cuda.mem_get_info()[0], torch.cuda.memory_reserved()
    # what torch's own caching allocator took in the meantime is not the library's
    leaked = (free_before - free_after) - (held_after - held_before)
    assert leaked < 32 << 20, (free_before, free_after, held_before, held_after)
