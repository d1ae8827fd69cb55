#!/usr/bin/env python3
"""Benchmark of the fused log-prob + AIS + gradient path on one MI355X.

A step is one pass of the whole path over one synthetic batch already resident in HBM:
ais_token_logprob -> ais_diagnostics -> ais_grpo_loss_grad, back to back on one stream.
Prints one JSON line (tokens/s = valid token rows per second), with the HBM roofline figures of the
dominant kernel (the gradient sweep) and the CPU oracle timed on a bounded sample of the same batch.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # dense bf16 MFMA, MI355X
HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, vendor figure


def measured_traffic(kernel: str, workload: int):
    """HBM bytes per launch from the hardware-counter summaries under profiles/, or None when there is no
    summary for this kernel and workload or the kernel sources have changed since the counters were taken."""
    import glob
    import hashlib
    import re
    csrc = os.path.join(ROOT, "paper_2605_13907_amd", "csrc")
    for path in glob.glob(os.path.join(ROOT, "profiles", "pmc_hbm_traffic_*.txt")):
        text = open(path).read()
        stamped = re.findall(r"^(\S+) sha256=([0-9a-f]{64})$", text, flags=re.M)
        if not stamped:
            continue
        if any(hashlib.sha256(open(os.path.join(csrc, f), "rb").read()).hexdigest() != h for f, h in stamped):
            continue
        m = re.search(rf"^{kernel} workload={workload} traffic_bytes_per_launch=(\d+)", text, flags=re.M)
        if m:
            return int(m.group(1))
    return None


def cpu_baseline(batch, params, sample_rows: int):
    """The CPU oracle, as it stands, on the leading whole prompt groups of the timed batch: their own response
    boundaries, mask, tokens, rollout log-probs and rewards.  As many groups as fit in `sample_rows` rows, at least
    one, so every step of the path runs on a part of the very batch the GPU is timed on."""
    import numpy as np
    import oracle.ais_oracle as O
    from oracle.pool import OraclePool, widen

    shape = batch.shape
    G = shape.group_size
    cu_all = batch.cu_rows.cpu().numpy().astype(np.int64)
    n_groups_all = (len(cu_all) - 1) // G
    n_groups = max(1, int(np.searchsorted(cu_all[G::G], sample_rows, side="right")))
    n_groups = min(n_groups, n_groups_all)
    n_resp = n_groups * G
    n = int(cu_all[n_resp])
    cu = cu_all[:n_resp + 1]
    z = batch.logits[:n]
    dtype = shape.logits_dtype
    bits = (z.view(__import__("torch").int16).cpu().numpy().view(np.uint16) if dtype == "bf16"
            else z.cpu().numpy())
    y = batch.token_ids[:n].cpu().numpy()
    valid = batch.valid[:n].cpu().numpy()
    lp_roll = batch.logp_roll[:n].double().cpu().numpy()
    rewards = batch.rewards[:n_resp].double().cpu().numpy()
    workers = min(16, len(os.sched_getaffinity(0)))
    pool = OraclePool(workers)
    try:
        path = pool.share(bits)                      # inputs resident in host memory before the clock starts
        t0 = time.perf_counter()
        pool.whole_path(path, n, dtype, y, valid, cu, lp_roll, rewards, G, O.Params(**params))
        dt = time.perf_counter() - t0
    finally:
        pool.close()
    n_valid = int(valid.astype(bool).sum())
    # the same oracle in this process alone, on the leading rows of each response of the first group (a sixteenth of
    # the sample at most), for a per-core figure
    m_per = max(1, min(int(np.diff(cu[:G + 1]).min()), max(1, n // (16 * G))))
    rows = np.concatenate([np.arange(cu[i], cu[i] + m_per) for i in range(G)])
    zs = widen(bits[rows], dtype)
    t0 = time.perf_counter()
    O.ais_grpo(zs, y[rows], valid[rows], np.arange(G + 1, dtype=np.int64) * m_per, lp_roll[rows], rewards[:G], G,
               O.Params(**params))
    dt1 = time.perf_counter() - t0
    return {"value": n_valid / dt, "unit": "tokens/s", "cores": workers, "kind": "oracle",
            "sample": f"the first {n_groups} of {n_groups_all} prompt groups of the timed batch ({n_resp} responses, {n} rows, "
                      f"{n_valid} valid, their own boundaries and rewards), numpy fp64 oracle over {workers} worker "
                      f"processes, {dt:.2f} s wall",
            "single_core": {"value": int(valid[rows].astype(bool).sum()) / dt1, "unit": "tokens/s",
                            "sample": f"the leading {m_per} rows of each response of the first group in one process, "
                                      f"{dt1:.2f} s wall"}}


def burst_class(vocab: int, esize: int) -> str:
    """Name of the gradient-sweep instantiation that the library's launcher picks for 16-byte aligned rows of this
    width (reporting only; mirrors the table in csrc/sweeps.hip: vectors per lane and burst, bursts, vectors that
    surely exist)."""
    per_vec = 16 // esize
    need = (vocab // per_vec + 1023) // 1024
    t = "bf16" if esize == 2 else "float"
    if need <= 12:
        nv = 4 * ((max(need, 1) + 3) // 4)
        return f"dlogits_burst_kernel<{t}, {nv}, 1, {nv - 4}>"
    if need <= 20:
        return f"dlogits_burst_kernel<{t}, {need}, 1, {need - 1}>"
    if need <= 32:
        return f"dlogits_burst_kernel<{t}, 16, 2, 20>"
    if need <= 48:
        return f"dlogits_burst_kernel<{t}, 16, 3, 32>"
    return f"dlogits_burst_kernel<{t}, 16, 0, 0>"


def time_workload(torch, binding, workloads, ctx, k, steps, warmup, mode="ais", stale_old=False, in_place=False):
    """Generates workload k, runs `warmup` untimed and `steps` timed passes of the three-call path over it, and
    returns (summary dict, batch, params, output buffer, step function, logp_old)."""
    shape = workloads.config(k)
    t0 = time.perf_counter()
    batch = workloads.generate(shape, "cuda", row_chunk=512)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t0
    R, V = batch.logits.shape
    N = batch.n_valid
    e = batch.logits.element_size()
    p = binding.default_params(alpha_override={"ais": -1.0, "tis": 1.0, "grpo": 0.0}[mode])
    dz = batch.logits if in_place else torch.empty_like(batch.logits)
    logp_old = None
    if stale_old:       # torch's log_softmax stands in for the trainer's earlier log-probs (not timed)
        logp_old = torch.empty(R, dtype=torch.float32, device="cuda")
        gen_old = torch.Generator(device="cuda").manual_seed(17)
        for r0 in range(0, R, 512):
            z = batch.logits[r0:r0 + 512].float()
            tok = batch.token_ids[r0:r0 + 512].long().clamp(min=0).unsqueeze(1)
            logp_old[r0:r0 + 512] = torch.log_softmax(z, 1).gather(1, tok).squeeze(1)
        logp_old += 0.2 * torch.randn(R, device="cuda", generator=gen_old)

    def step():
        logp, lse = ctx.token_logprob(batch.logits, batch.token_ids, batch.valid, p.inv_temperature)
        adv, count, diag = ctx.diagnostics(logp if logp_old is None else logp_old, batch.logp_roll, batch.valid,
                                           batch.cu_rows, batch.rewards, shape.group_size, p)
        return ctx.grpo_loss_grad(batch.logits, batch.token_ids, batch.valid, batch.cu_rows, logp, lse,
                                  batch.logp_roll, adv, count, diag, p, logp_old=logp_old, dlogits=dz), diag

    if in_place:
        keep = batch.logits.clone()
    for _ in range(warmup):
        step()
        if in_place:
            batch.logits.copy_(keep)
    torch.cuda.synchronize()
    ctx.profile(True)
    t_total = 0.0
    if in_place:                 # the logits have to be restored between steps: time each step on its own
        for _ in range(steps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            (loss, _, _), diag = step()
            torch.cuda.synchronize()
            t_total += time.perf_counter() - t0
            batch.logits.copy_(keep)
    else:                        # exactly K steps between two synchronisations
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            (loss, _, _), diag = step()
        torch.cuda.synchronize()
        t_total = time.perf_counter() - t0
    ms_fwd, n_fwd = ctx.profile_read(binding.AIS_K_LOGPROB)
    ms_bwd, n_bwd = ctx.profile_read(binding.AIS_K_DLOGITS)
    ctx.profile(False)
    d = ctx.read_diag(diag)
    assert ctx.status() == 0
    ms_step = t_total / steps * 1e3
    # The same step recorded once into a HIP graph and replayed: what a caller whose batches are small enough to be
    # bound by launches gains (reported beside the eager figure, which stays the headline).
    ms_graph = None
    if not in_place:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) / steps * 1e3
        del graph
        assert ctx.status() == 0
    fwd_bytes = e * V * N                                   # one read of every valid row
    bwd_bytes = 2 * e * V * N + e * V * (R - N)             # read + write of valid rows, zero-fill of the others
    fwd_gbps = fwd_bytes / (ms_fwd / n_fwd * 1e-3) / 1e9
    bwd_gbps = bwd_bytes / (ms_bwd / n_bwd * 1e-3) / 1e9
    path_gbps = (fwd_bytes + bwd_bytes) / (ms_step * 1e-3) / 1e9
    summary = {
        "k": k, "workload": f"config {k}: {shape.name}", "vocab": V, "rows": R, "valid_rows": N, "responses": shape.n_resp,
        "group_size": shape.group_size, "logits": shape.logits_dtype, "layout": shape.layout,
        "ms_per_step": ms_step, "tokens_per_s": N / (ms_step * 1e-3), "ms_per_step_hip_graph": ms_graph,
        "path_hbm": {"GB/s": path_gbps, "frac": path_gbps / HBM_PEAK_GBPS, "bytes_per_step": fwd_bytes + bwd_bytes},
        "dominant_kernel": {"name": burst_class(V, e), "avg_ms": ms_bwd / n_bwd, "bytes_per_launch": bwd_bytes,
                            "GB/s": bwd_gbps, "frac": bwd_gbps / HBM_PEAK_GBPS,
                            "zero_filled_rows": R - N},
        "token_logprob": {"avg_ms": ms_fwd / n_fwd, "GB/s": fwd_gbps, "frac": fwd_gbps / HBM_PEAK_GBPS},
        "diag": {q: d[q] for q in ("alpha", "alpha_ess", "alpha_mis", "alpha_var", "dbar", "ess_ratio")},
        "loss": float(loss.item()), "gen_s": t_gen,
    }
    return summary, batch, p, dz, logp_old


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="headline workload 1..5 (2 = Qwen3-8B-shaped, V = 151,936)")
    ap.add_argument("--others", type=str, default="1,3,4,5",
                    help="workloads also timed and listed under `workloads` (comma-separated, empty = none)")
    ap.add_argument("--cpu-rows", type=int, default=24000,
                    help="the CPU oracle is timed on the leading whole prompt groups within this many rows, at least one (0 = skip)")
    ap.add_argument("--in-place", action="store_true", help="write the gradient over the logits")
    ap.add_argument("--extras", action="store_true",
                    help="also time the FP8 rollout-perturbation kernels on the same batch (reported under next_rows)")
    ap.add_argument("--mode", choices=["ais", "tis", "grpo"], default="ais",
                    help="ais: adaptive alpha (the paper's method); tis: alpha forced to 1; grpo: alpha forced to 0")
    ap.add_argument("--stale-old", action="store_true",
                    help="pass a perturbed log pi_old so that the clipped surrogate's gate is exercised")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no inter-GPU step; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_13907_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    ctx = binding.AisContext()

    # the other workloads first (each generated, timed and released), the headline workload last so that its batch
    # is the one the extras and the CPU baseline work on
    others = []
    for k in [int(x) for x in args.others.split(",") if x.strip()]:
        if k == args.config:
            continue
        summary, batch, p, dz, _ = time_workload(torch, binding, workloads, ctx, k, args.steps, args.warmup, args.mode)
        others.append(summary)
        del batch, dz
        torch.cuda.empty_cache()

    head, batch, p, dz, logp_old = time_workload(torch, binding, workloads, ctx, args.config, args.steps, args.warmup,
                                                 args.mode, args.stale_old, args.in_place)
    shape = batch.shape
    R, V = batch.logits.shape
    N = head["valid_rows"]
    e = batch.logits.element_size()
    ms_step = head["ms_per_step"]

    # plain copy of the logits: what this device's HBM sustains for a read+write stream
    ctx.profile(True)
    scratch = dz if not args.in_place else torch.empty_like(batch.logits)
    for _ in range(3):
        ctx.copy(scratch, batch.logits)
    ms_copy, n_copy = ctx.profile_read(binding.AIS_K_COPY)
    ctx.profile(False)
    copy_gbps = 2.0 * R * V * e / (ms_copy / n_copy * 1e-3) / 1e9

    dom = head["dominant_kernel"]
    result = {
        "metric": "fused_logprob_ais_grad_tokens_per_s", "value": head["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.logits_dtype, "arithmetic": "f32 on the logits' storage type; f64 in the batch reductions",
        "data": "synthetic",
        "config": {"workload": head["workload"], "vocab": V, "rows": R, "valid_rows": N,
                   "responses": shape.n_resp, "group_size": shape.group_size, "logits": shape.logits_dtype,
                   "layout": shape.layout, "in_place": bool(args.in_place), "mode": args.mode,
                   "stale_old_policy": bool(args.stale_old)},
        "roofline": {"bound": "hbm", "kernel": dom["name"], "achieved": dom["GB/s"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": dom["frac"],
                     "traffic": measured_traffic("dlogits_burst_kernel", args.config),
                     "avg_ms": dom["avg_ms"], "bytes_per_launch": dom["bytes_per_launch"]},
        "kernels": {"token_logprob": head["token_logprob"],
                    "dlogits": {q: dom[q] for q in ("avg_ms", "GB/s", "frac")},
                    "copy_yardstick": {"avg_ms": ms_copy / n_copy, "GB/s": copy_gbps}},
        "path_hbm": head["path_hbm"], "ms_per_step_hip_graph": head["ms_per_step_hip_graph"],
        "diag": head["diag"], "loss": head["loss"], "gen_s": head["gen_s"],
        "workloads": [dict(w, dominant_kernel=dict(w["dominant_kernel"],
                                                    traffic=measured_traffic("dlogits_burst_kernel", w["k"])))
                      for w in others],
    }
    if args.extras:
        ctx.profile(True)
        for _ in range(3):
            codes, scale = ctx.fp8_quantize_rows(batch.logits)
            ctx.fp8_dequantize_rows(codes, scale, batch.logits.dtype)
            ctx.fp8_rollout_logprob(batch.logits, batch.token_ids, batch.valid)
        extras = {}
        for name, which, nbytes in (("fp8_quantize_rows", binding.AIS_K_FP8_QUANT, (e + 1) * V * R),
                                    ("fp8_dequantize_rows", binding.AIS_K_FP8_DEQUANT, (e + 1) * V * R),
                                    ("fp8_rollout_logprob", binding.AIS_K_FP8_LOGPROB, e * V * N)):
            ms, n = ctx.profile_read(which)
            extras[name] = {"avg_ms": ms / n, "algorithmic_bytes": nbytes, "GB/s": nbytes / (ms / n * 1e-3) / 1e9,
                            "frac": nbytes / (ms / n * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        ctx.profile(False)
        del codes, scale
        # one-sweep variant (direction + per-row scale): each row read once, 2 e V bytes per valid token
        def one_sweep():
            logp, lse, sg = ctx.token_logprob_softmax_grad(batch.logits, batch.token_ids, batch.valid,
                                                           p.inv_temperature, sgrad=dz)
            adv, count, diag = ctx.diagnostics(logp, batch.logp_roll, batch.valid, batch.cu_rows, batch.rewards,
                                               shape.group_size, p)
            return ctx.grpo_row_scale(logp, batch.logp_roll, batch.valid, batch.cu_rows, adv, count, diag, p,
                                      logp_old)
        for _ in range(2):
            one_sweep()
        torch.cuda.synchronize()
        ctx.profile(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_sweep()
        torch.cuda.synchronize()
        ms_os = (time.perf_counter() - t0) / args.steps * 1e3
        ms_k, n_k = ctx.profile_read(binding.AIS_K_FUSED)
        ctx.profile(False)
        os_bytes = 2 * e * V * N + e * V * (R - N)
        extras["one_sweep_path"] = {"ms_per_step": ms_os, "tokens/s": N / (ms_os * 1e-3),
                                    "algorithmic_bytes": os_bytes, "GB/s": os_bytes / (ms_os * 1e-3) / 1e9,
                                    "frac": os_bytes / (ms_os * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                    "fused_kernel_avg_ms": (ms_k / n_k) if n_k else None,
                                    "speedup_vs_three_call_path": ms_step / ms_os}
        # log-probs straight from hidden states (matrix cores): the same rows and vocabulary, d_model of the family
        rb = workloads.generate_readout(shape, device="cuda")
        Dm = rb.hidden.shape[1]
        for _ in range(2):
            ctx.lm_head_logprob(rb.hidden, rb.weight, rb.token_ids, rb.valid, p.inv_temperature)
        ctx.profile(True)
        for _ in range(5):
            ctx.lm_head_logprob(rb.hidden, rb.weight, rb.token_ids, rb.valid, p.inv_temperature)
        ms, n = ctx.profile_read(binding.AIS_K_LM_HEAD)
        ctx.profile(False)
        flops = 2.0 * R * V * Dm
        tf = flops / (ms / n * 1e-3) / 1e12
        # yardstick: the library GEMM that materialises the bf16 logits, followed by the streaming log-prob sweep
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        z = torch.empty(R, V, dtype=torch.bfloat16, device="cuda")
        for _ in range(2):
            torch.matmul(rb.hidden, rb.weight.t(), out=z)
        ev0.record()
        for _ in range(5):
            torch.matmul(rb.hidden, rb.weight.t(), out=z)
        ev1.record()
        torch.cuda.synchronize()
        ms_gemm = ev0.elapsed_time(ev1) / 5
        extras["lm_head_logprob"] = {
            "avg_ms": ms / n, "d_model": Dm, "flops": flops,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
            "library_gemm_yardstick": {"avg_ms": ms_gemm, "TFLOP/s": flops / (ms_gemm * 1e-3) / 1e12,
                                       "note": "torch.matmul to bf16 logits; the materialised route adds the "
                                               "token_logprob sweep above to this"}}
        # gradient w.r.t. hidden states and output embedding without materialised logits (recompute on the matrix
        # cores, chunk by chunk, + two library GEMMs per chunk), against the route that materialises the logits
        # (library GEMM, the two sweeps of this library, two library GEMMs on the [R, V] dlogits)
        logp_h, lse_h = ctx.lm_head_logprob(rb.hidden, rb.weight, rb.token_ids, rb.valid, p.inv_temperature)
        gen_c = torch.Generator(device="cuda").manual_seed(23)
        coeff = torch.randn(R, device="cuda", generator=gen_c) * 1e-5 * (rb.valid != 0)
        ctx.lm_head_grad(rb.hidden, rb.weight, rb.token_ids, lse_h, logp_h, coeff, p.inv_temperature)
        ctx.profile(True)
        ev0.record()
        for _ in range(3):
            dh, dw = ctx.lm_head_grad(rb.hidden, rb.weight, rb.token_ids, lse_h, logp_h, coeff, p.inv_temperature)
        ev1.record()
        torch.cuda.synchronize()
        ms_grad = ev0.elapsed_time(ev1) / 3
        ms_rec, n_rec = ctx.profile_read(binding.AIS_K_LM_HEAD_GRAD)
        ctx.profile(False)
        del dh, dw
        # a batch with a mask: the loader knows how many positions are evaluated; with that bound the call gathers them
        n_live = int((rb.valid != 0).sum().item())
        ms_bound = None
        if n_live < R:
            ctx.lm_head_grad(rb.hidden, rb.weight, rb.token_ids, lse_h, logp_h, coeff, p.inv_temperature, n_live_max=n_live)
            ev0.record()
            for _ in range(3):
                dh, dw = ctx.lm_head_grad(rb.hidden, rb.weight, rb.token_ids, lse_h, logp_h, coeff, p.inv_temperature,
                                          n_live_max=n_live)
            ev1.record()
            torch.cuda.synchronize()
            ms_bound = ev0.elapsed_time(ev1) / 3
            assert ctx.status() == 0
            del dh, dw
        dh16 = torch.empty(R, Dm, dtype=torch.bfloat16, device="cuda")
        dw16 = torch.empty(V, Dm, dtype=torch.bfloat16, device="cuda")
        for it in range(4):
            if it == 1:
                ev0.record()
            torch.matmul(z, rb.weight, out=dh16)              # dhidden = dlogits W      (z stands in for dlogits)
            torch.matmul(z.t(), rb.hidden, out=dw16)          # dweight = dlogits^T H
        ev1.record()
        torch.cuda.synchronize()
        ms_two = ev0.elapsed_time(ev1) / 3
        k_fwd, k_bwd = result["kernels"]["token_logprob"]["avg_ms"], result["kernels"]["dlogits"]["avg_ms"]
        extras["lm_head_grad"] = {
            "avg_ms": ms_grad, "avg_ms_with_row_bound": ms_bound, "rows_with_gradient": n_live,
            "recompute_kernel_ms": ms_rec / 3, "chunks": n_rec // 3, "flops": 3 * flops,
            "TFLOP/s": 3 * flops / (ms_grad * 1e-3) / 1e12, "frac_of_mfma_peak": 3 * flops / (ms_grad * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "dlogits_bytes_held": 2 * R * 8192, "logits_bytes_of_materialised_route": 2 * R * V,
            "materialised_route": {"ms": ms_gemm + k_fwd + k_bwd + ms_two, "logits_gemm_ms": ms_gemm,
                                   "two_sweeps_ms": k_fwd + k_bwd, "two_gradient_gemms_ms": ms_two,
                                   "note": "library GEMMs with bf16 outputs; the sweeps are this library's"}}
        del z, rb, dh16, dw16
        result["next_rows"] = extras
    if args.cpu_rows > 0:
        params = dict(C=p.C, delta=p.delta, gamma=p.gamma, eps_std=p.eps_std, beta_var=p.beta_var,
                      clip_eps=p.clip_eps)
        result["cpu_baseline"] = cpu_baseline(batch, params, args.cpu_rows)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
