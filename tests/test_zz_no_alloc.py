"""The diagnostics call that allocates nothing (static device scratch) against the ordinary one, through the C ABI:
same kernels, so every output must be bit-identical.  Two calls in a row, the second on a smaller batch (the
scratch array keeps the first call's contents), then a larger one again; run alone in a fresh process and after the
other tests."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_13907_amd import binding as B

pytestmark = pytest.mark.gpu


def _batch(n_resp, G, max_len, seed, p_valid=0.85):
    rng = np.random.default_rng(seed)
    L = rng.integers(0, max_len + 1, size=n_resp)
    L[rng.integers(0, n_resp)] = 0                                  # an empty response
    cu = np.concatenate([[0], np.cumsum(L)]).astype(np.int64)
    R = int(cu[-1])
    valid = (rng.random(R) < p_valid).astype(np.uint8)
    logp_roll = -np.abs(rng.normal(2.0, 1.5, size=R)).astype(np.float32)
    logp_train = np.minimum(logp_roll + rng.normal(0.0, 0.3, size=R).astype(np.float32), 0.0).astype(np.float32)
    rewards = (rng.random(n_resp) < 0.4).astype(np.float32)
    t = lambda a: torch.from_numpy(a).cuda()
    return dict(lt=t(logp_train), lr=t(logp_roll), valid=t(valid), cu=t(cu), rewards=t(rewards), G=G, R=R, B=n_resp)


def _raw_call(lib, fn_name, h, b, p, adv, count, diag):
    """Straight through the C ABI: pointers and sizes only."""
    fn = getattr(lib, fn_name)
    return fn(h, C.c_void_p(b["lt"].data_ptr()), C.c_void_p(b["lr"].data_ptr()), C.c_void_p(b["valid"].data_ptr()),
              b["R"], C.c_void_p(b["cu"].data_ptr()), b["B"], b["G"], C.c_void_p(b["rewards"].data_ptr()), C.byref(p),
              C.c_void_p(adv.data_ptr()), C.c_void_p(count.data_ptr()), C.c_void_p(diag.data_ptr()))


def test_static_scratch_matches_workspace_path():
    ctx = B.AisContext()
    lib = B._lib()
    p = B.default_params()
    # a large batch (many tiles and responses), then a much smaller one, then a mid-sized one with other parameters
    cases = [(_batch(256, 8, 9000, 1), p), (_batch(8, 4, 40, 2), p), (_batch(64, 8, 3000, 3), B.default_params(C=2.0, adv_mode=1))]
    for it, (b, params) in enumerate(cases):
        outs = {}
        for name in ("ais_diagnostics", "ais_diagnostics_static"):
            adv = torch.full((b["B"],), -7.0, dtype=torch.float32, device="cuda")
            count = torch.full((b["B"],), -7, dtype=torch.int32, device="cuda")
            diag = torch.full((C.sizeof(B.AisDiag),), 0xAB, dtype=torch.uint8, device="cuda")
            ctx._sync_stream()
            free_before = torch.cuda.mem_get_info()[0]
            rc = _raw_call(lib, name, ctx._h, b, params, adv, count, diag)
            assert rc == 0, (name, rc)
            torch.cuda.synchronize()
            if name == "ais_diagnostics_static":
                assert torch.cuda.mem_get_info()[0] == free_before, "the static entry point must not allocate"
            outs[name] = (adv.clone(), count.clone(), diag.clone())
        for x, y, what in zip(outs["ais_diagnostics"], outs["ais_diagnostics_static"], ("adv", "count", "diag")):
            assert torch.equal(x, y), f"call {it}: {what} differs between the two entry points"
        d = ctx.read_diag(outs["ais_diagnostics_static"][2])
        assert d["n_valid"] == int(b["valid"].sum().item()) and 0.0 < d["alpha"] <= 1.0
        assert outs["ais_diagnostics_static"][1].sum().item() == d["n_valid"]
    assert ctx.status() == 0
    # beyond the limit: a clear error, nothing launched
    big = _batch(8, 4, 40, 4)
    big["B"] = 1 << 20
    big["G"] = 1
    adv = torch.zeros(1, device="cuda")
    assert _raw_call(lib, "ais_diagnostics_static", ctx._h, big, p, adv, adv, adv) == -10
    # the step that follows it must not take the static call's tiling for its own: whole path after a static call
    b = cases[2][0]
    adv, count, diag = ctx.diagnostics(b["lt"], b["lr"], b["valid"], b["cu"], b["rewards"], b["G"], p)
    ctx.diagnostics(cases[1][0]["lt"], cases[1][0]["lr"], cases[1][0]["valid"], cases[1][0]["cu"], cases[1][0]["rewards"],
                    cases[1][0]["G"], p, static_scratch=True)
    loss_a, wt_a, g_a = ctx.grpo_row_scale(b["lt"], b["lr"], b["valid"], b["cu"], adv, count, diag, p)
    adv2, count2, diag2 = ctx.diagnostics(b["lt"], b["lr"], b["valid"], b["cu"], b["rewards"], b["G"], p)
    loss_b, wt_b, g_b = ctx.grpo_row_scale(b["lt"], b["lr"], b["valid"], b["cu"], adv2, count2, diag2, p)
    torch.cuda.synchronize()
    assert torch.equal(loss_a, loss_b) and torch.equal(wt_a, wt_b) and torch.equal(g_a, g_b)
    ctx.close()
