"""The three calls are capturable in a HIP graph: they allocate nothing once the workspace exists, never
synchronise, and clear nothing with memset nodes.  Every replay is checked against the eager result, with
eager work and synchronisations between replays and new input values each time."""
import pytest
import torch

from paper_2605_13907_amd import binding as B
from paper_2605_13907_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    ctx = B.AisContext()
    shape = W.config(3).scaled(vocab=4104, len_div=4, n_prompts=2, seed=23)
    batch = W.generate(shape, "cuda")
    p = B.default_params()
    dz = torch.empty_like(batch.logits)
    logits0 = batch.logits.clone()

    def step(dlogits):
        logp, lse = ctx.token_logprob(batch.logits, batch.token_ids, batch.valid)
        adv, count, diag = ctx.diagnostics(logp, batch.logp_roll, batch.valid, batch.cu_rows, batch.rewards,
                                           shape.group_size, p)
        loss, wt, out = ctx.grpo_loss_grad(batch.logits, batch.token_ids, batch.valid, batch.cu_rows, logp, lse,
                                           batch.logp_roll, adv, count, diag, p, dlogits=dlogits)
        return logp, diag, loss, wt, out

    step(dz)                                   # warm-up: sizes the context's workspace outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            g_logp, g_diag, g_loss, g_wt, g_dz = step(dz)
    torch.cuda.synchronize()
    for it in range(4):
        # new inputs in the captured buffers
        batch.logits.copy_(logits0 * (1.0 + 0.05 * it))
        batch.logp_roll.add_(0.01 * it * batch.valid.float())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (g_logp, g_diag, g_loss, g_wt, g_dz)]
        ref = step(torch.empty_like(dz))       # eager, into a different output buffer
        torch.cuda.synchronize()
        for a, b, name in zip(got, ref, ("logp", "diag", "loss", "wtilde", "dlogits")):
            assert torch.equal(a, b), f"replay {it}: {name} differs from the eager result"
    assert ctx.status() == 0
    ctx.close()


def test_lm_head_graph_replays_match_eager():
    """The hidden-state log-prob call under capture: its set-up kernel decides the decomposition on the device, so
    a replay with a different mask (a different number of evaluated rows) must still match the eager result."""
    ctx = B.AisContext()
    g = torch.Generator(device="cpu")
    g.manual_seed(31)
    R, D, V = 1500, 128, 3000
    hidden = torch.randn(R, D, generator=g).to(torch.bfloat16).cuda()
    weight = (torch.randn(V, D, generator=g) / D ** 0.5 * 3).to(torch.bfloat16).cuda()
    y = torch.randint(0, V, (R,), generator=g, dtype=torch.int32).cuda()
    valid = (torch.rand(R, generator=g) < 0.6).to(torch.uint8).cuda()
    ctx.lm_head_logprob(hidden, weight, y, valid)          # warm-up: sizes the workspace outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            g_logp, g_lse = ctx.lm_head_logprob(hidden, weight, y, valid)
    torch.cuda.synchronize()
    for it, p_valid in enumerate((0.6, 0.05, 1.0, 0.3)):
        valid.copy_((torch.rand(R, generator=g) < p_valid).to(torch.uint8))
        hidden.mul_(1.0 + 0.1 * it)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (g_logp.clone(), g_lse.clone())
        ref = ctx.lm_head_logprob(hidden, weight, y, valid)
        torch.cuda.synchronize()
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1]), f"replay {it} differs from the eager result"
    assert ctx.status() == 0
    ctx.close()


def test_one_sweep_and_fp8_graph_replays_match_eager():
    """The one-sweep path and the three FP8 kernels under capture, at two row-width classes, replayed on new
    inputs."""
    ctx = B.AisContext()
    p = B.default_params(inv_temperature=1.0 / 0.9)
    for vocab in (21_512, 4104):
        shape = W.config(2).scaled(vocab=vocab, len_div=64, seed=29)
        batch = W.generate(shape, "cuda")
        logits0 = batch.logits.clone()

        def step():
            out = ctx.step_one_sweep(batch, p)
            codes, scale = ctx.fp8_quantize_rows(batch.logits)
            zr = ctx.fp8_dequantize_rows(codes, scale, dtype=batch.logits.dtype)
            lpr = ctx.fp8_rollout_logprob(batch.logits, batch.token_ids, batch.valid)
            return [out[k] for k in ("logp", "lse", "diag", "loss", "wtilde", "sgrad", "g")] + [codes, scale, zr, lpr]

        names = ("logp", "lse", "diag", "loss", "wtilde", "sgrad", "g", "codes", "scale", "dequantised", "logp_roll")
        step()                                 # warm-up: sizes the context's workspace outside the capture
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                held = step()
        torch.cuda.synchronize()
        for it in range(3):
            batch.logits.copy_(logits0 * (1.0 - 0.07 * it))
            batch.logp_roll.sub_(0.02 * it * batch.valid.float())
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = [t.clone() for t in held]
            ref = step()
            torch.cuda.synchronize()
            for a, b, name in zip(got, ref, names):
                assert torch.equal(a, b), f"vocab {vocab}, replay {it}: {name} differs from the eager result"
        del graph, held
    assert ctx.status() == 0
    ctx.close()


@pytest.fixture(scope="module")
def ctx():
    c = B.AisContext()
    yield c
    c.close()


# ---- the same on the named workloads' shapes, for both forms of the path and the call that allocates nothing: bit
# equality of every output tensor, new values before every replay

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
