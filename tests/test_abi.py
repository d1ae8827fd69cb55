"""The C ABI without a GPU: the library loads, exports every function include/ais.h declares, fills in
the paper's defaults, and rejects bad arguments on the host before touching any device."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

from paper_2605_13907_amd import binding as B
from tests.test_golden import read_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "ais.h")).read()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int|void|char\s*\*)\s*\*?\s*(ais_\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    lib = C.CDLL(B.LIB_PATH)
    names = declared_functions()
    assert {"ais_token_logprob", "ais_diagnostics", "ais_grpo_loss_grad", "ais_create", "ais_destroy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B.SYMBOLS), "binding and header disagree on the set of functions"


def test_every_compute_entry_point_cites_the_passage_it_implements():
    """The comment in front of each declaration that computes something names the section, equation or algorithm of
    the paper that defines the operation; the entry point that allocates nothing names the callers it is for."""
    import re
    text = HEADER
    helpers = {"ais_create", "ais_destroy", "ais_set_stream", "ais_params_default", "ais_strerror",
               "ais_last_hip_error", "ais_status", "ais_version", "ais_profile", "ais_profile_read", "ais_copy"}
    for name in declared_functions():
        if name in helpers:
            continue
        at = re.search(r"^[a-z].*\b%s\(" % name, text, re.M).start()
        comment = text[text.rfind("/*", 0, at):at]
        assert text.rfind("*/", 0, at) > text.rfind("/*", 0, at), name
        if name == "ais_diagnostics_static":
            assert "cannot" in comment and "allocate" in comment, name
        else:
            assert re.search(r"\b(Alg\.|Eq\.|Sec\.)", comment), f"{name}: no citation in its comment"


def test_struct_sizes_match_header_layout():
    assert C.sizeof(B.AisParams) == 40          # 9 floats + 1 int
    assert C.sizeof(B.AisDiag) == 8 + 15 * 8 + 8


def test_defaults_are_the_papers():
    g = read_golden("hyperparameters.txt")
    p = B.default_params()
    for k in ("C", "delta", "gamma", "eps_std", "clip_eps"):
        assert getattr(p, k) == pytest.approx(g[k], rel=1e-7), k
    assert p.adv_mode == 0 and p.alpha_override < 0 and p.inv_temperature == 1.0 and p.beta_kl == 0.0
    assert p.beta_var == 1.0


def test_strerror_and_version():
    lib = B._lib()
    assert lib.ais_version() >= 1000
    for code in range(0, -11, -1):
        assert len(lib.ais_strerror(code)) > 0
    assert lib.ais_strerror(0) == b"ok"


FAKE = C.c_void_p(0x1000)       # never dereferenced: validation fails (or ctx is NULL) before any launch


def call_logprob(**kw):
    a = dict(ctx=None, logits=FAKE, dtype=B.AIS_BF16, n_rows=4, vocab=64, stride=64, tok=FAKE, valid=None,
             inv_t=1.0, logp=FAKE, lse=FAKE)
    a.update(kw)
    return B._lib().ais_token_logprob(a["ctx"], a["logits"], a["dtype"], a["n_rows"], a["vocab"], a["stride"],
                                      a["tok"], a["valid"], a["inv_t"], a["logp"], a["lse"])


def test_token_logprob_argument_checks():
    assert call_logprob() == -1                                  # everything fine except the NULL context
    assert call_logprob(logits=None) == -1
    assert call_logprob(tok=None) == -1
    assert call_logprob(n_rows=-1) == -2
    assert call_logprob(vocab=0) == -2
    assert call_logprob(vocab=2 ** 31) == -2
    assert call_logprob(stride=63) == -3
    assert call_logprob(dtype=7) == -7
    assert call_logprob(logits=C.c_void_p(0x1001)) == -4
    assert call_logprob(inv_t=0.0) == -5
    assert call_logprob(inv_t=float("nan")) == -5
    assert call_logprob(n_rows=0, logits=None, tok=None, logp=None, lse=None) == -1   # only the context is missing


def call_diag(params=None, **kw):
    p = params or B.default_params()
    a = dict(ctx=None, lt=FAKE, lr=FAKE, valid=None, n_rows=10, cu=FAKE, n_resp=8, G=4, rewards=FAKE,
             adv=FAKE, count=FAKE, diag=FAKE)
    a.update(kw)
    return B._lib().ais_diagnostics(a["ctx"], a["lt"], a["lr"], a["valid"], a["n_rows"], a["cu"], a["n_resp"],
                                    a["G"], a["rewards"], C.byref(p), a["adv"], a["count"], a["diag"])


def test_diagnostics_argument_checks():
    assert call_diag() == -1
    assert call_diag(n_resp=0) == -2
    assert call_diag(G=0) == -2
    assert call_diag(n_resp=9) == -6
    assert call_diag(cu=None) == -1
    assert call_diag(diag=None) == -1
    for bad in (dict(C=0.5), dict(delta=0.0), dict(gamma=-1.0), dict(eps_std=-1e-3), dict(alpha_override=1.5),
                dict(adv_mode=2), dict(clip_eps=1.0), dict(inv_temperature=0.0), dict(beta_kl=-1.0),
                dict(beta_var=float("nan"))):
        assert call_diag(params=B.default_params(**bad)) == -5, bad


def test_static_diagnostics_argument_checks_and_size_limit():
    """The entry point that allocates nothing: the argument checks of ais_diagnostics, and a documented error for
    batches beyond what the static scratch array holds (checked before the context, so no GPU is needed)."""
    lib = B._lib()
    p = B.default_params()

    def call(**kw):
        a = dict(ctx=None, lt=FAKE, lr=FAKE, valid=None, n_rows=10, cu=FAKE, n_resp=8, G=4, rewards=FAKE,
                 adv=FAKE, count=FAKE, diag=FAKE)
        a.update(kw)
        return lib.ais_diagnostics_static(a["ctx"], a["lt"], a["lr"], a["valid"], a["n_rows"], a["cu"], a["n_resp"],
                                          a["G"], a["rewards"], C.byref(p), a["adv"], a["count"], a["diag"])

    assert call() == -1                                   # everything fine except the NULL context
    assert call(n_resp=0) == -2 and call(n_resp=9) == -6 and call(cu=None) == -1 and call(diag=None) == -1
    assert call(n_rows=18_000_000, n_resp=512) == -1      # the header's examples fit ...
    assert call(n_rows=1_000_000, n_resp=16_000) == -1
    assert call(n_rows=19_000_000, n_resp=512) == -10     # ... and these do not
    assert call(n_rows=1_000_000, n_resp=17_500) == -10
    assert call(n_rows=0, n_resp=1 << 20) == -10
    assert b"static scratch" in lib.ais_strerror(-10)
    assert B.STATIC_SCRATCH_BYTES == int(re.search(r"#define AIS_STATIC_SCRATCH_BYTES \(1 << (\d+)\)", HEADER).group(1)) ** 0 << 20


def test_loss_grad_argument_checks():
    lib = B._lib()
    p = B.default_params()

    def call(**kw):
        a = dict(ctx=None, logits=FAKE, dtype=B.AIS_BF16, n_rows=4, vocab=64, stride=64, tok=FAKE, valid=None,
                 cu=FAKE, n_resp=2, lt=FAKE, lse=FAKE, lr=FAKE, lo=None, lref=None, adv=FAKE, count=FAKE,
                 diag=FAKE, wt=None, loss=FAKE, dz=FAKE)
        a.update(kw)
        return lib.ais_grpo_loss_grad(a["ctx"], a["logits"], a["dtype"], a["n_rows"], a["vocab"], a["stride"],
                                      a["tok"], a["valid"], a["cu"], a["n_resp"], a["lt"], a["lse"], a["lr"],
                                      a["lo"], a["lref"], a["adv"], a["count"], a["diag"], C.byref(p), a["wt"],
                                      a["loss"], a["dz"])

    assert call() == -1
    assert call(dz=None) == -1
    assert call(loss=None) == -1
    assert call(stride=8) == -3
    assert call(n_resp=0) == -2
    assert call(dz=C.c_void_p(0x2001)) == -4
    assert call(dtype=3) == -7


def test_lm_head_logprob_argument_checks():
    lib = B._lib()

    def call(**kw):
        a = dict(ctx=None, hidden=C.c_void_p(0x1000), ld_h=64, weight=C.c_void_p(0x2000), ld_w=64, dtype=B.AIS_BF16,
                 n_rows=4, d=64, vocab=100, tok=FAKE, valid=None, inv_t=1.0, logp=FAKE, lse=FAKE)
        a.update(kw)
        return lib.ais_lm_head_logprob(a["ctx"], a["hidden"], a["ld_h"], a["weight"], a["ld_w"], a["dtype"],
                                       a["n_rows"], a["d"], a["vocab"], a["tok"], a["valid"], a["inv_t"],
                                       a["logp"], a["lse"])

    assert call() == -1                                          # everything fine except the NULL context
    assert call(dtype=B.AIS_F32) == -7
    assert call(n_rows=-1) == -2
    assert call(vocab=0) == -2
    assert call(d=0) == -2
    assert call(d=12) == -2                                      # not a multiple of 8
    assert call(ld_h=56) == -3
    assert call(ld_w=8) == -3
    assert call(ld_h=68) == -4                                   # rows would not stay 16-byte aligned
    assert call(hidden=C.c_void_p(0x1008)) == -4
    assert call(weight=C.c_void_p(0x2002)) == -4
    assert call(weight=None) == -1
    assert call(hidden=None) == -1
    assert call(lse=None) == -1
    assert call(inv_t=-1.0) == -5
    assert call(n_rows=0, hidden=None, tok=None, logp=None, lse=None) == -1


def test_one_sweep_argument_checks():
    lib = B._lib()
    p = B.default_params()

    def sweep(**kw):
        a = dict(ctx=None, logits=FAKE, dtype=B.AIS_F32, n_rows=4, vocab=64, stride=72, tok=FAKE, valid=None,
                 inv_t=1.0, logp=FAKE, lse=FAKE, sgrad=FAKE)
        a.update(kw)
        return lib.ais_token_logprob_softmax_grad(a["ctx"], a["logits"], a["dtype"], a["n_rows"], a["vocab"],
                                                  a["stride"], a["tok"], a["valid"], a["inv_t"], a["logp"],
                                                  a["lse"], a["sgrad"])

    assert sweep() == -1                                         # everything fine except the NULL context
    assert sweep(sgrad=None) == -1
    assert sweep(lse=None) == -1
    assert sweep(sgrad=C.c_void_p(0x3002)) == -4                 # fp32 output on a 2-byte boundary
    assert sweep(dtype=B.AIS_BF16, sgrad=C.c_void_p(0x3002)) == -1   # fine for bf16: only the context is missing
    assert sweep(stride=63) == -3
    assert sweep(vocab=0) == -2
    assert sweep(dtype=-1) == -7
    assert sweep(inv_t=float("inf")) == -5
    assert sweep(n_rows=0, logits=None, tok=None, logp=None, lse=None, sgrad=None) == -1

    def scale(params=p, **kw):
        a = dict(ctx=None, lt=FAKE, lr=FAKE, lo=None, lref=None, valid=None, n_rows=10, cu=FAKE, n_resp=8, adv=FAKE,
                 count=FAKE, diag=FAKE, wt=None, loss=FAKE, g=FAKE)
        a.update(kw)
        return lib.ais_grpo_row_scale(a["ctx"], a["lt"], a["lr"], a["lo"], a["lref"], a["valid"], a["n_rows"],
                                      a["cu"], a["n_resp"], a["adv"], a["count"], a["diag"],
                                      C.byref(params) if params is not None else None, a["wt"], a["loss"], a["g"])

    assert scale() == -1
    assert scale(g=None) == -1
    assert scale(lr=None) == -1
    assert scale(adv=None) == -1
    assert scale(params=None) == -1
    assert scale(n_rows=-3) == -2
    assert scale(n_resp=0) == -2
    assert scale(n_resp=(1 << 24) + 1) == -2
    assert scale(params=B.default_params(C=float("inf"))) == -5
    assert scale(params=B.default_params(clip_eps=-0.1)) == -5
    assert scale(n_rows=0, lt=None, lr=None, g=None) == -1       # an empty batch needs no per-row arrays


def test_fp8_argument_checks():
    lib = B._lib()

    def quant(**kw):
        a = dict(ctx=None, logits=FAKE, dtype=B.AIS_BF16, n_rows=3, vocab=100, stride=104, codes=FAKE, cstride=100,
                 scale=FAKE)
        a.update(kw)
        return lib.ais_fp8_quantize_rows(a["ctx"], a["logits"], a["dtype"], a["n_rows"], a["vocab"], a["stride"],
                                         a["codes"], a["cstride"], a["scale"])

    assert quant() == -1
    assert quant(codes=None) == -1
    assert quant(scale=None) == -1
    assert quant(cstride=99) == -3
    assert quant(stride=99) == -3
    assert quant(dtype=2) == -7
    assert quant(n_rows=2 ** 31) == -2
    assert quant(logits=C.c_void_p(0x1003)) == -4

    def dequant(**kw):
        a = dict(ctx=None, codes=FAKE, cstride=100, scale=FAKE, n_rows=3, vocab=100, out=FAKE, dtype=B.AIS_F32,
                 ostride=100)
        a.update(kw)
        return lib.ais_fp8_dequantize_rows(a["ctx"], a["codes"], a["cstride"], a["scale"], a["n_rows"], a["vocab"],
                                           a["out"], a["dtype"], a["ostride"])

    assert dequant() == -1
    assert dequant(codes=None) == -1
    assert dequant(out=None) == -1
    assert dequant(cstride=64) == -3
    assert dequant(ostride=64) == -3
    assert dequant(out=C.c_void_p(0x1002)) == -4                 # fp32 output on a 2-byte boundary
    assert dequant(dtype=9) == -7
    assert dequant(vocab=-5) == -2

    def roll(**kw):
        a = dict(ctx=None, logits=FAKE, dtype=B.AIS_BF16, n_rows=3, vocab=100, stride=100, tok=FAKE, valid=None,
                 out=FAKE)
        a.update(kw)
        return lib.ais_fp8_rollout_logprob(a["ctx"], a["logits"], a["dtype"], a["n_rows"], a["vocab"], a["stride"],
                                           a["tok"], a["valid"], a["out"])

    assert roll() == -1
    assert roll(tok=None) == -1
    assert roll(out=None) == -1
    assert roll(stride=10) == -3
    assert roll(dtype=5) == -7
    assert roll(n_rows=-1) == -2


def test_context_and_utility_argument_checks():
    lib = B._lib()
    one, f = C.c_int(0), C.c_float(0.0)
    assert lib.ais_create(None, 0, None) == -1
    assert lib.ais_destroy(None) == 0                            # destroying nothing is not an error
    assert lib.ais_set_stream(None, None) == -1
    assert lib.ais_last_hip_error(None) == 0
    assert lib.ais_status(None, C.byref(one), 0) == -1
    assert lib.ais_profile(None, 1) == -1
    assert lib.ais_profile_read(None, 0, C.byref(f), C.byref(one)) == -1
    assert lib.ais_copy(None, FAKE, C.c_void_p(0x2000), 64) == -1       # only the context is missing
    assert lib.ais_copy(None, FAKE, C.c_void_p(0x2000), 8) == -2        # whole 16-byte vectors only
    assert lib.ais_copy(None, FAKE, C.c_void_p(0x2000), -16) == -2
    assert lib.ais_copy(None, None, C.c_void_p(0x2000), 64) == -1
    assert lib.ais_copy(None, C.c_void_p(0x1008), C.c_void_p(0x2000), 64) == -4
    assert lib.ais_copy(None, FAKE, C.c_void_p(0x2004), 64) == -4


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        B._lib()


def test_header_is_plain_c_and_links(tmp_path):
    """include/ais.h compiles as strict C99 and a C program can call the library."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    exe = tmp_path / "c_abi_check"
    src = os.path.join(ROOT, "tests", "c_abi_check.c")
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    src, "-o", str(exe), B.LIB_PATH, f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert out.stdout.strip() == "0"


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
    assert not r.stdout.strip().startswith("{")              # no result line for a run that did not happen


def test_lm_head_grad_argument_checks():
    lib = B._lib()

    def call(**kw):
        a = dict(ctx=None, hidden=FAKE, ld_h=64, weight=FAKE, ld_w=64, dtype=B.AIS_BF16, n_rows=4, d=64, vocab=100,
                 tok=FAKE, lse=FAKE, logp=FAKE, coeff=FAKE, inv_t=1.0, chunk=0, live=-1, dh=FAKE, dw=FAKE)
        a.update(kw)
        return lib.ais_lm_head_grad(a["ctx"], a["hidden"], a["ld_h"], a["weight"], a["ld_w"], a["dtype"], a["n_rows"],
                                    a["d"], a["vocab"], a["tok"], a["lse"], a["logp"], a["coeff"], a["inv_t"],
                                    a["chunk"], a["live"], a["dh"], a["dw"])

    assert call() == -1                                   # everything fine except the NULL context
    assert call(dtype=B.AIS_F32) == -7
    assert call(d=40) == -2 and call(d=16) == -2          # the gradient call needs d_model % 32 == 0
    assert call(chunk=100) == -2 and call(chunk=255) == -2 and call(chunk=512) == -1
    assert call(vocab=0) == -2 and call(n_rows=-1) == -2
    assert call(ld_h=32) == -3 and call(ld_w=60) == -3
    assert call(weight=None) == -1 and call(dw=None) == -1 and call(lse=None) == -1 and call(coeff=None) == -1
    assert call(hidden=C.c_void_p(0x1008)) == -4 and call(ld_w=68) == -4
    assert call(inv_t=0.0) == -5 and call(inv_t=float("inf")) == -5
    assert call(live=0) == -1 and call(live=3) == -1 and call(live=10 ** 12) == -1      # any bound is a valid argument


def test_binding_rejects_host_tensors_before_any_launch():
    """A host (or foreign-device) tensor handed to a kernel would be a GPU memory fault, not an error code: the
    binding must refuse every large buffer that is not on the context's GPU before it allocates or launches
    anything.  No GPU is needed: the context object below has no library handle, so reaching a launch would raise
    AttributeError instead of the expected ValueError."""
    import torch

    ctx = object.__new__(B.AisContext)
    ctx.device = torch.device("cuda", 0)
    ctx._h = None
    ctx._lib = None
    z = torch.zeros(4, 64, dtype=torch.bfloat16)
    tok = torch.zeros(4, dtype=torch.int32)
    f = torch.zeros(4)
    with pytest.raises(ValueError, match="logits is on cpu"):
        ctx.token_logprob(z, tok)
    with pytest.raises(ValueError, match="logits is on cpu"):
        ctx.token_logprob_softmax_grad(z, tok)
    with pytest.raises(ValueError, match="logits is on cpu"):
        ctx.grpo_loss_grad(z, tok, None, torch.zeros(3, dtype=torch.int64), f, f, f, torch.zeros(2),
                           torch.zeros(2, dtype=torch.int32), torch.zeros(C.sizeof(B.AisDiag), dtype=torch.uint8))
    with pytest.raises(ValueError, match="logits is on cpu"):
        ctx.fp8_quantize_rows(z)
    with pytest.raises(ValueError, match="logits is on cpu"):
        ctx.fp8_rollout_logprob(z, tok)
    with pytest.raises(ValueError, match="codes is on cpu"):
        ctx.fp8_dequantize_rows(torch.zeros(4, 64, dtype=torch.uint8), f)
    with pytest.raises(ValueError, match="hidden is on cpu"):
        ctx.lm_head_logprob(z, torch.zeros(100, 64, dtype=torch.bfloat16), tok)
    with pytest.raises(ValueError, match="hidden is on cpu"):
        ctx.lm_head_grad(z, torch.zeros(100, 64, dtype=torch.bfloat16), tok, f, f, f)
    with pytest.raises(ValueError, match="dst is on cpu"):
        ctx.copy(torch.zeros(16), torch.zeros(16))
    with pytest.raises(ValueError):                         # the geometry helper itself, with and without a device
        B._logits_geometry(torch.zeros(4, 8, 2), None)
    assert B._logits_geometry(z, None) == (4, 64, 64)
