#!/usr/bin/env python3
"""Benchmark of the decoder-stage hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: M x mls_stage_forward, then one
mls_stage_backward over the M stashed micro-batches in overwrite mode, which writes the fp32 gradients of the step
(nothing is zeroed beforehand and the gradient buffer is never read).  Default: the 7B-shaped stage, 4 layers, 4
micro-batches of 4096 tokens.  Prints ONE JSON line.  Inputs are resident in HBM before the timed region starts.
Model FLOPs: 3 x (dense GEMMs + causal-halved attention), recompute not credited.  The timed process imports the
library, the input generator and torch only; the CPU oracle is loaded by the cpu_baseline leg alone, after the
timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
# HBM bytes per GEMM launch (average over all gemm16_kernel and gemm_dma_kernel dispatches of a step), from the rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/stage_7b_4x4_hbm_traffic.txt:
# (2.0 * 364308 KiB fetched + 1.0 * 85181 KiB written) * 1024.  Only valid for the default workload.
PROFILED_GEMM_TRAFFIC = {"7b": 8.33e8}


def cpu_baseline(sh):
    """The CPU oracle as it stands on a bounded sample: ONE layer x ONE micro-batch at the full shape
    (the work is exactly linear in layers x micro-batches), forward + backward in fp64."""
    import numpy as np
    import synth
    from oracle import stage as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    one = sh.with_(layers=1, microbatches=1)
    _, p64 = synth.make_params(one, 1001)
    W = [synth.split_params(one, p64, 0)]
    _, x = synth.make_x(one, 2001, 0)
    _, dy = synth.make_dy(one, 3001, 0)
    t0 = time.perf_counter()
    y, caches = O.stage_forward(x, W, one)
    O.stage_backward(dy, W, caches, one)
    dt = time.perf_counter() - t0
    flops = one.model_flops_layer_mb()
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 layer x 1 micro-batch of the same shape, fwd+bwd, fp64 numpy, {dt:.1f} s",
            "tokens_per_s": one.tokens / dt}


def plan_sweep(a):
    print(json.dumps(run_plan_sweep(None, a.steps)))


def run_plan_sweep(plans, steps):
    """The straggler-shaped plan sweep: 16 seeded (layers, micro-batches) plans on the 7B layer shape at seq 2048;
    checks the paper's cost model (Sec. 4.2: stage time = l * tau(b) per micro-batch, step ~ m * l * tau(b)) by a
    least-squares fit t = alpha + c * l * m and reports the largest relative residual."""
    import numpy as np
    import torch
    import synth
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["sweep"]
    plans = plans or synth.plan_sweep()
    sh = sh.with_(layers=max(k for k, _ in plans), microbatches=max(m for _, m in plans))
    st = mls.Stage.from_shape(sh, seed=1004)           # one handle serves every plan
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    mmax = max(m for _, m in plans)
    xs = [synth.to_device(synth.make_x(sh, 2004, mb)[0], sh.dtype) for mb in range(mmax)]
    dy = torch.stack([synth.to_device(synth.make_dy(sh, 3004, mb)[0], sh.dtype) for mb in range(mmax)])
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(mmax)]
    dx = torch.empty_like(dy)
    grads = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    times = []
    for k, m in plans:
        def step():     # the library's step form: the backward call writes the gradients, no zeroing pass
            for mb in range(m):
                st.forward(xs[mb], k, ys[mb])
            st.backward(dy[:m], grads, m, dx[:m], overwrite=True)
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3 / steps)
    km = np.array([k * m for k, m in plans], dtype=np.float64)
    t = np.array(times)
    A = np.stack([np.ones_like(km), km], axis=1)
    (alpha, c), *_ = np.linalg.lstsq(A, t, rcond=None)
    fit = alpha + c * km
    resid = np.abs(t - fit) / t
    flops_unit = sh.model_flops_layer_mb()
    out = {"metric": "stage fwd+bwd TFLOP/s (bf16)", "value": flops_unit / (c * 1e-3) / 1e12, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": steps, "warmup": 1, "ms_per_step": float(t.mean()), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "plan sweep: 7B layer shape, seq 2048, 16 seeded plans (layers 2..9, micro-batches 1..16)"},
           "tau_ms_per_layer_microbatch": float(c), "alpha_ms": float(alpha),
           "max_relative_residual": float(resid.max()),
           "r2": float(1 - np.sum((t - fit) ** 2) / np.sum((t - t.mean()) ** 2)),
           "plans": [{"layers": k, "microbatches": m, "ms": float(ms)} for (k, m), ms in zip(plans, times)]}
    # Close the loop of Sec. 4.2: the measured tau(b) feeds the planner's lower level.  Orchestration of the paper's
    # 110B case study (Sec. 7.3, Table 4: 80 layers, 64 micro-batches, two pipelines of 8 and 6 stages), group rates
    # taken as inversely proportional to the group size (1, 2, 4 or 8 GPUs).
    import timeit
    pipes = [[1.0, 1.0, 1.0, 0.25, 0.25, 0.25, 0.125, 0.125], [0.5, 0.5, 0.5, 0.125, 0.125, 0.125]]
    ls, ms, est = mls.plan_lower_level(pipes, 80, 64, float(c))
    solve_us = min(timeit.repeat(lambda: mls.plan_lower_level(pipes, 80, 64, float(c)), number=200, repeat=3)) / 200 * 1e6
    out["plan_example"] = {"pipelines": pipes, "layers": ls, "microbatches": ms, "estimated_step_ms": est,
                           "solve_us_incl_binding": solve_us}
    st.close()
    return out


def run_ends(steps, warmup, n_mb=4):
    """The non-uniform layers of the first and last stage at the 7B shape (hidden 4096, vocabulary 32000, 4096 tokens
    per micro-batch): embedding forward, head forward (final RMSNorm, LM head, cross-entropy), head backward and
    embedding backward over n_mb micro-batches per step.  Not the headline metric: reported beside it."""
    import numpy as np
    import torch
    import synth
    import paper_2410_13333_amd as mls
    sh = synth.ENDS_CONFIGS["7b"].with_(microbatches=n_mb)
    en = mls.Ends.from_shape(sh, seed=1101, max_inflight=n_mb)
    toks = [torch.from_numpy(synth.make_tokens(sh, 2100, mb).reshape(-1)).cuda() for mb in range(n_mb)]
    tgts = [torch.from_numpy(synth.make_targets(sh, 2200, mb).reshape(-1)).cuda() for mb in range(n_mb)]
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [torch.empty(shape, dtype=en.tdtype, device="cuda") for _ in range(n_mb)]
    ys = [torch.randn(shape, device="cuda").to(en.tdtype) for _ in range(n_mb)]
    dy = torch.empty((n_mb,) + shape, dtype=en.tdtype, device="cuda")
    dx = torch.randn((n_mb,) + shape, device="cuda").to(en.tdtype)
    loss = torch.zeros(n_mb, dtype=torch.float32, device="cuda")
    grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")

    def step():
        grads.zero_()
        for mb in range(n_mb):
            en.embed_forward(toks[mb], xs[mb])
        for mb in range(n_mb):
            en.head_forward(ys[mb], tgts[mb], 1.0 / n_mb, loss[mb:mb + 1])
        en.head_backward(grads, n_mb, dy)
        en.embed_backward(dx, grads, n_mb)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flops = sh.model_flops_mb() * n_mb
    out = {"metric": "first/last-stage layers fwd+bwd TFLOP/s (bf16)", "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"embedding + final RMSNorm + LM head + cross-entropy, hidden 4096, vocabulary 32000, "
                                  f"{n_mb} micro-batches of 4096 tokens"},
           "ms_per_microbatch": ms / n_mb, "mean_loss": float(loss.mean())}
    en.close()
    return out


def run_optim(steps, warmup):
    """AdamW step on the parameters of the 7B-shaped 4-layer stage (809.5 M parameters, bf16 storage, fp32 master
    weights and moments): one HBM-bound kernel, 30 B per parameter."""
    import torch
    import synth
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["7b"]
    n = sh.layers * synth.layer_param_elems(sh)
    p = (0.02 * torch.randn(n, device="cuda")).to(torch.bfloat16)
    g = torch.randn(n, device="cuda", dtype=torch.float32)
    opt = mls.Optim(p)
    for _ in range(warmup):
        opt.step(g, p, lr=1e-4)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        opt.step(g, p, lr=1e-4)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    gbs = n * 30 / (ms * 1e-3) / 1e9
    out = {"metric": "AdamW step GB/s", "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic", "config": {"workload": f"AdamW on {n} parameters (7B-shaped stage, 4 layers), bf16 storage"},
           "roofline": {"bound": "hbm", "kernel": "adamw_kernel", "achieved": gbs, "peak": 8000.0, "unit": "GB/s",
                        "frac": gbs / 8000.0, "traffic": None}}
    opt.close()
    return out


def run_model(steps, warmup, n_mb=4):
    """A complete training step of a 4-layer model of the 7B layer shape on one GPU: token embedding, the decoder
    stage, final RMSNorm + LM head + loss, their backwards over n_mb accumulated micro-batches, and the AdamW update of
    all parameters (stage: 809.5 M, embedding + head: 262.1 M).  Reported beside the headline stage metric."""
    import torch
    import synth
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["7b"].with_(microbatches=n_mb)
    esh = synth.ENDS_CONFIGS["7b"].with_(microbatches=n_mb)
    st = mls.Stage.from_shape(sh, seed=1001)
    en = mls.Ends.from_shape(esh, seed=1101)
    ps, pe = st.get_params(), en.get_params()
    os_, oe_ = mls.Optim(ps), mls.Optim(pe)
    toks = [torch.from_numpy(synth.make_tokens(esh, 2100, mb).reshape(-1)).cuda() for mb in range(n_mb)]
    tgts = [torch.from_numpy(synth.make_targets(esh, 2200, mb).reshape(-1)).cuda() for mb in range(n_mb)]
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    x = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(n_mb)]
    y = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(n_mb)]
    dy = torch.empty((n_mb,) + shape, dtype=st.tdtype, device="cuda")
    dx = torch.empty_like(dy)
    loss = torch.zeros(n_mb, dtype=torch.float32, device="cuda")
    gs = torch.empty(st.grad_elems, dtype=torch.float32, device="cuda")
    ge = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
    losses = []

    def step():
        ge.zero_()
        for mb in range(n_mb):
            en.embed_forward(toks[mb], x[mb])
            st.forward(x[mb], sh.layers, y[mb])
            en.head_forward(y[mb], tgts[mb], 1.0 / n_mb, loss[mb:mb + 1])
        en.head_backward(ge, n_mb, dy)
        st.backward(dy, gs, n_mb, dx, overwrite=True)
        en.embed_backward(dx, ge, n_mb)
        os_.step(gs, ps, lr=3e-4)
        oe_.step(ge, pe, lr=3e-4)
        st.set_params(ps)
        en.set_params(pe)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
        losses.append(loss.mean())
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flops = (sh.model_flops_layer_mb() * sh.layers + esh.model_flops_mb()) * n_mb
    out = {"metric": "model step fwd+bwd+update TFLOP/s (bf16)", "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"4-layer model of the 7B layer shape (vocabulary 32000), {n_mb} micro-batches of 4096 "
                                  f"tokens, AdamW on all 1.07 G parameters"},
           "tokens_per_s": n_mb * sh.tokens / (ms * 1e-3),
           "loss_first_last": [float(losses[0]), float(losses[-1])]}
    for h in (os_, oe_, st, en):
        h.close()
    return out


def run_gemm(steps, warmup, data):
    """The twelve contractions of one 7B layer x micro-batch through the stand-alone entry point mls_gemm (weight
    gradients over the 4 micro-batches of the headline step), on operands of a chosen value distribution: the rate of
    the same kernel depends on how many bits its operands toggle (the chip's power limit sets the shader clock)."""
    import torch
    import paper_2410_13333_amd as mls
    T = 4096
    # (mode, M, N, K): as the stage runs them, the forward products in the NT form against transposed weight copies
    groups = {"forward (NT on W^T)": [(1, T, 12288, 4096), (1, T, 4096, 4096), (1, T, 22016, 4096), (1, T, 4096, 11008)],
              "data gradient (NT on W)": [(1, T, 11008, 4096), (1, T, 4096, 22016), (1, T, 4096, 4096), (1, T, 4096, 12288)],
              "weight gradient (TN)": [(2, 11008, 4096, 4 * T), (2, 4096, 22016, 4 * T), (2, 4096, 4096, 4 * T),
                                       (2, 4096, 12288, 4 * T)]}
    g = torch.Generator(device="cuda").manual_seed(5)

    def operand(r, c):  # row-padded like the library's internal layout
        ld = c + 64 if c % 256 == 0 else c
        if data == "randn":
            t = torch.randn(r, ld, device="cuda", generator=g)
        elif data == "zeros":
            t = torch.zeros(r, ld, device="cuda")
        elif data == "ones":
            t = torch.ones(r, ld, device="cuda")
        elif data == "bits":
            t = (torch.rand(r, ld, device="cuda", generator=g) < 0.5).float()
        else:
            raise SystemExit("--data must be randn, zeros, ones or bits")
        return t.to(torch.bfloat16)[:, :c]
    per_mode, tot_ms, tot_fl = {}, 0.0, 0.0
    for name, shapes in groups.items():
        ms_mode = fl_mode = 0.0
        for (mode, M, N, K) in shapes:
            a = operand(M, K) if mode != 2 else operand(K, M)
            b = operand(K, N) if mode != 1 else operand(N, K)
            c = torch.zeros(M, N + 64, device="cuda", dtype=torch.float32 if mode == 2 else torch.bfloat16)[:, :N]
            for _ in range(warmup):
                mls.gemm(mode, a, b, c)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(steps):
                mls.gemm(mode, a, b, c)
            e1.record()
            torch.cuda.synchronize()
            ms_mode += e0.elapsed_time(e1) / steps
            fl_mode += 2.0 * M * N * K
        per_mode[name] = {"ms": ms_mode, "tflops": fl_mode / (ms_mode * 1e-3) / 1e12}
        tot_ms += ms_mode
        tot_fl += fl_mode
    tf = tot_fl / (tot_ms * 1e-3) / 1e12
    return {"metric": "bf16 GEMM TFLOP/s (stand-alone)", "value": tf, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
            "warmup": warmup, "ms_per_step": tot_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": f"synthetic ({data})",
            "config": {"workload": "the 12 contractions of one 7B layer x micro-batch, 4096 tokens, stand-alone launches"},
            "roofline": {"bound": "mfma", "kernel": "gemm16_kernel", "achieved": tf, "peak": PEAK_BF16_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS, "traffic": None},
            "per_mode": per_mode}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b", help="7b (headline), 13b, 70b_tp4, tiny, sweep (16-plan linearity check), ends (first/last-stage layers), optim (AdamW step), model (embedding + stage + head + update), gemm (the layer's contractions stand-alone, --data)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--data", default="randn", help="gemm workload only: operand values, randn | zeros | ones | bits")
    ap.add_argument("--recompute", action="store_true", help="activation recomputation: keep only the layer inputs")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    if a.workload == "sweep":
        return plan_sweep(a)
    if a.workload == "ends":
        print(json.dumps(run_ends(a.steps, a.warmup)))
        return
    if a.workload == "model":
        print(json.dumps(run_model(a.steps, a.warmup)))
        return
    if a.workload == "gemm":
        print(json.dumps(run_gemm(a.steps, a.warmup, a.data)))
        return
    if a.workload == "optim":
        print(json.dumps(run_optim(a.steps, a.warmup)))
        return

    import torch
    import synth
    import paper_2410_13333_amd as mls

    sh = synth.CONFIGS[a.workload]
    K, M = sh.layers, sh.microbatches
    torch.cuda.set_device(0)
    st = mls.Stage.from_shape(sh, seed=1001, recompute=a.recompute)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [synth.to_device(synth.make_x(sh, 2001, mb)[0], sh.dtype) for mb in range(M)]
    dy = torch.stack([synth.to_device(synth.make_dy(sh, 3001, mb)[0], sh.dtype) for mb in range(M)])
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(M)]
    dx = torch.empty_like(dy)
    grads = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")

    def step():
        # one backward call per step: it writes the gradients (MLS_BWD_OVERWRITE) instead of adding to a vector the
        # harness would have to zero first; the result is bit-identical to zeroing and accumulating
        for mb in range(M):
            st.forward(xs[mb], K, ys[mb])
        st.backward(dy, grads, M, dx, overwrite=True)

    for _ in range(a.warmup):
        step()
    # the events mark the step boundaries on the stream the library launches on (torch's current stream, which the
    # handle was created with); they are read after the timed region
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(a.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(a.steps))
    ms_median = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])

    # per-kernel-class durations from HIP events on the stage's stream, over the same K-step region again
    st.timing(True)
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    tm = st.timing_read()
    st.timing(False)
    classes = {k: {"ms_per_step": v[0] / a.steps, "launches_per_step": v[1] // a.steps} for k, v in tm.items()}

    flops_step = sh.model_flops_layer_mb() * K * M
    tflops = flops_step / (ms * 1e-3) / 1e12
    # dominant kernel: the bf16 MFMA GEMM (per layer: 8 launches per micro-batch + 4 weight-gradient launches)
    gemm_ms = sum(tm[k][0] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad"))
    gemm_n = sum(tm[k][1] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad"))
    # algorithmic FLOPs of all GEMM launches of the timed steps / their summed duration; per launch = / launches
    gemm_flops = 3 * 2 * sh.tokens * sh.matrix_params() * K * M * a.steps
    if a.recompute:  # the backward re-runs every forward contraction but the last one of the layer
        gemm_flops += 2 * sh.tokens * (sh.matrix_params() - sh.ffn * sh.hidden) * K * M * a.steps
    gemm_flops_launch = gemm_flops / gemm_n
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
    out = {
        "metric": "stage fwd+bwd TFLOP/s (bf16)", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}-shaped stage: {K} layers x {M} micro-batches, hidden {sh.hidden}, "
                               f"{sh.n_q_heads}/{sh.n_kv_heads} heads x {sh.head_dim}, ffn {sh.ffn}, seq {sh.seq}, "
                               f"micro-batch {sh.micro_batch}" + (", activation recomputation" if a.recompute else ""),
                   "layers": K, "microbatches": M},
        "ms_per_step_median": ms_median, "ms_per_step_min": per_step[0],
        "tokens_per_s": M * sh.tokens / (ms * 1e-3),
        "frac_of_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "tau_ms_per_layer_microbatch": ms / (K * M),
        "model_flops_per_step": flops_step,
        "roofline": {"bound": "mfma", "kernel": "gemm16_kernel (256x256 tiles) + gemm_dma_kernel (column remainders)", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": PROFILED_GEMM_TRAFFIC.get(a.workload),
                     "flops_per_launch": gemm_flops_launch, "avg_launch_ms": gemm_ms / gemm_n},
        "kernel_classes": classes,
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(sh)
    st.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
