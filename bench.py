#!/usr/bin/env python3
"""Benchmark of the SMoE MLP hot path (routing + Alg. 3 forward + backward) on one MI355X.

One "step" = top-k gate, routing sort, SMoE MLP forward and backward over one synthetic
batch that is already resident in HBM.  Prints ONE JSON line:
  metric/value  GEMM TFLOP/s of fwd+bwd (6 grouped GEMMs, 2*Tk*d_model*(d_h+d_expert)*3 flop)
  roofline      the dominant kernel of the step (the first ParallelLinear's scatter2scatter, with the SwiGLU
                epilogue it has inside the step) timed with HIP events on the launch stream, against the
                roofline that bounds it (dense bf16 MFMA peak or HBM bandwidth), the other one alongside
  forward_hbm   the whole forward pass against its algorithmic HBM bytes
  cpu_baseline  the fp64 CPU oracle timed on sampled tokens of the same workload, one thread and all threads
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak (published)
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E (published)


def _events(n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


class _F64Experts:
    """float64 copies of the expert matrices, made once per expert before the clock starts (the oracle converts
    whatever it is handed to float64; handing it float64 keeps that conversion out of the timed region)."""

    def __init__(self, w32: np.ndarray, experts):
        self.shape = w32.shape
        self.m = {int(e): w32[int(e)].astype(np.float64) for e in experts}

    def __getitem__(self, e):
        return self.m[int(e)]


def cpu_baseline(case, cfg, budget_s: float):
    """Times the oracle as it stands (per-token fp64 forward + analytic backward, Sec. 3.1's naive loop) on a
    bounded random sample of the workload's tokens: half the budget with the BLAS pool limited to one thread,
    half with the pool as the box gives it.  Routing comes from the oracle's own top-k, not from the GPU."""
    import oracle
    import smoe_inputs as si
    from threadpoolctl import threadpool_info, threadpool_limits
    pool = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    rng = np.random.default_rng(0)
    cand = rng.permutation(cfg.T)[:256]
    logits = case["logits"].numpy()
    ei, g = oracle.topk_gate(logits[cand], cfg.k)
    g = g.astype(np.float32).astype(np.float64)
    # tokens whose experts are among the few whose matrices are converted up front (bounds host memory and set-up time)
    per_expert_bytes = 8.0 * cfg.d_model * (cfg.d_h + cfg.d_expert)
    n_keep = int(max(cfg.k, min(cfg.E, 8e9 // per_expert_bytes)))
    counts = np.bincount(ei.reshape(-1), minlength=cfg.E)
    keep = set(np.argsort(-counts, kind="stable")[:n_keep].tolist())
    rows = [i for i in range(len(cand)) if set(ei[i].tolist()) <= keep]
    X = si.as_f32(case["X"]); dY = si.as_f32(case["dY"])
    W1 = _F64Experts(si.as_f32(case["W1"]), keep)
    W2 = _F64Experts(si.as_f32(case["W2"]), keep)
    flops_per_token = 3.0 * cfg.gemm_flops_fwd() / cfg.T

    def leg(seconds, start):
        t0, c0 = time.perf_counter(), time.process_time()
        n = 0
        while True:
            i = rows[(start + n) % len(rows)]
            t = cand[i]
            oracle.mlp_token_fwd(X[t], ei[i], g[i], W1, W2, cfg.act)
            oracle.mlp_token_bwd(X[t], dY[t], ei[i], g[i], W1, W2, cfg.act)
            n += 1
            dt = time.perf_counter() - t0
            if dt > seconds or n >= 4096:
                return n, dt, (time.process_time() - c0) / dt

    with threadpool_limits(limits=1):
        n1, dt1, busy1 = leg(budget_s / 2, 0)
    nN, dtN, busyN = leg(budget_s / 2, n1)
    return {
        "value": nN * flops_per_token / dtN / 1e12, "unit": "TFLOP/s", "cores": max(1, int(round(busyN))), "kind": "oracle",
        "tokens_per_s": nN / dtN, "blas_pool_threads": int(pool), "cores_busy": busyN,
        "single_thread": {"value": n1 * flops_per_token / dt1 / 1e12, "unit": "TFLOP/s", "tokens_per_s": n1 / dt1,
                          "cores_busy": busy1},
        "sample": f"{n1} + {nN} randomly sampled tokens of {cfg.name} (one-thread leg {dt1:.1f} s, then all-thread leg "
                  f"{dtN:.1f} s; `cores` = process CPU time / wall time of the all-thread leg): per-token fp64 forward + "
                  f"analytic backward (activation/input gradients; weight-gradient outer products not formed), the "
                  f"experts' matrices converted to float64 before the clock starts",
    }


def granularity_sweep(args):
    """Sec. 4.2: throughput of the SMoE MLP for k in {1,2,4,8,16} (E = 8k, d_expert = d_ff/k) relative to the
    dense MLP with the same active parameters, run through the same library as one expert with k = 1.
    Inputs are drawn on the GPU (timing only; parity at these shapes is covered by the GPU tests)."""
    import smoe_inputs as si
    import paper_2403_08245_amd as smoe

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)

    def draw(shape, std, dtype=torch.bfloat16):
        return (torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32) * std).to(dtype)

    def run(cfg):
        X, dY = draw((cfg.T, cfg.d_model), 1.0), draw((cfg.T, cfg.d_model), 1.0)
        W1, W2 = draw((cfg.E, cfg.d_model, cfg.d_h), 0.02), draw((cfg.E, cfg.d_expert, cfg.d_model), 0.02)
        logits = draw((cfg.T, cfg.E), 1.0, torch.float32)
        buf = smoe.MLPBuffers(cfg.T, cfg.k, cfg.E, cfg.d_model, cfg.d_expert, cfg.act, torch.bfloat16, dev,
                              training=True)

        def fwd():
            ei, gates = smoe.topk_gate(logits, cfg.k)
            r = smoe.route(ei, cfg.E)
            smoe.mlp_fwd(X, W1, W2, r, cfg.k, gates, cfg.act, buf)
            return r, gates

        def fwd_bwd():
            r, gates = fwd()
            smoe.mlp_bwd(dY, X, W1, W2, r, cfg.k, gates, cfg.act, buf)

        out = {}
        for name, fn in (("inference", fwd), ("training", fwd_bwd)):
            for _ in range(args.warmup):
                fn()
            ev = _events(args.steps + 1)
            ev[0].record(stream)
            for i in range(args.steps):
                fn()
                ev[i + 1].record(stream)
            torch.cuda.synchronize()
            ts = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)])
            flops = cfg.gemm_flops_fwd() * (1.0 if name == "inference" else 3.0)
            out[name] = {"ms_median": float(np.median(ts)), "ms_p5": float(np.percentile(ts, 5)),
                         "ms_p95": float(np.percentile(ts, 95)), "tflops": flops / (np.median(ts) * 1e-3) / 1e12,
                         "tokens_per_s": cfg.T / (np.median(ts) * 1e-3)}
        del X, dY, W1, W2, buf
        torch.cuda.empty_cache()
        return out

    sparsity = args.sweep == "sparsity"
    dense = run(si.CONFIGS["S-dense" if sparsity else "G-dense"])

    def vendor_dense():
        """The same dense MLP with the vendor's GEMM (torch.matmul) and torch's GELU, for context only."""
        cfg = si.CONFIGS["G-dense"]
        X, dY = draw((cfg.T, cfg.d_model), 1.0), draw((cfg.T, cfg.d_model), 1.0)
        W1, W2 = draw((cfg.d_model, cfg.d_expert), 0.02), draw((cfg.d_expert, cfg.d_model), 0.02)

        def fwd():
            hpre = X @ W1
            return hpre, torch.nn.functional.gelu(hpre)

        def fwd_only():
            return fwd()[1] @ W2

        def fwd_bwd():
            hpre, hh = fwd()
            _ = hh @ W2
            dh = dY @ W2.t()
            _ = hh.t() @ dY
            t = hpre.float()
            dhpre = (dh.float() * (0.5 * (1 + torch.erf(t * 0.7071067811865476))
                                   + t * torch.exp(-0.5 * t * t) * 0.3989422804014327)).to(torch.bfloat16)
            _ = X.t() @ dhpre
            _ = dhpre @ W1.t()

        out = {}
        for name, fn in (("inference", fwd_only), ("training", fwd_bwd)):
            for _ in range(args.warmup):
                fn()
            ev = _events(args.steps + 1)
            ev[0].record(stream)
            for i in range(args.steps):
                fn()
                ev[i + 1].record(stream)
            torch.cuda.synchronize()
            ts = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)])
            flops = cfg.gemm_flops_fwd() * (1.0 if name == "inference" else 3.0)
            out[name] = {"ms_median": float(np.median(ts)), "tflops": flops / (np.median(ts) * 1e-3) / 1e12}
        return out

    vendor = None if sparsity else vendor_dense()
    torch.cuda.empty_cache()
    rows = []
    for k in (si.SPARSITY_KS if sparsity else si.GRANULARITY_KS):
        cfg = si.CONFIGS[f"S{k}" if sparsity else f"G{k}"]
        res = run(cfg)
        rows.append({"k": k, "E": cfg.E, "d_expert": cfg.d_expert, **res,
                     "relative_throughput_training": dense["training"]["ms_median"] / res["training"]["ms_median"],
                     "relative_throughput_inference": dense["inference"]["ms_median"] / res["inference"]["ms_median"]})
    if sparsity:
        head = next(r for r in rows if r["k"] == 8)
        print(json.dumps({
            "metric": "SMoE MLP fwd+bwd GEMM throughput per layer, E=64 k=8 d_expert=1024 (Sec. 4.3 sweep)",
            "value": head["training"]["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": head["training"]["ms_median"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "sparsity sweep: T=61440 d_model=4096 E=64 d_expert=1024 act=gelu, uniform router, "
                                   "k in (1,2,4,8,16,30); dense = one expert of 65536 hidden units"},
            "dense_all_parameters": dense, "sweep": rows}))
        return
    head = next(r for r in rows if r["k"] == 4)
    print(json.dumps({
        "metric": "SMoE MLP fwd+bwd GEMM throughput per layer, unit-benchmark shape E=32 k=4 (Sec. 4.1)",
        "value": head["training"]["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["training"]["ms_median"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "granularity sweep: T=61440 d_model=4096 d_ff=8192 d_expert=d_ff/k E=8k act=gelu, "
                               "uniform router"},
        "dense_equal_active_parameters": dense, "dense_vendor_gemm_context": vendor, "sweep": rows}))


def bench_momha(args):
    """SMoE multi-head attention layer (Alg. 4) at the C5 shape: top-k + routing + layer forward + backward."""
    import smoe_inputs as si
    import paper_2403_08245_amd as smoe

    if args.workload == "C5":
        m = si.MOA_C5
        B, T, d_model, E, k, d_out = 2, m["T"] // 2, m["d_model"], m["E"], m["k"], m["d_out"]
        label = "C5"
    else:   # Sec. 4.4 shapes: d_model 4096, d_head 128, 16 sequences of 2048, 32 active heads, h_expert = 32 / k, E = 8k
        k = int(args.workload.split("-k")[1])
        B, T, d_model, E, d_out = 16, 2048, 4096, 8 * k, (32 // k) * 128
        label = f"MoA-k{k} (Sec. 4.4 shape)"
    h, d_head = d_out // 128, 128
    N, Tk = B * T, B * T * k
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    draw = lambda shape, std, dt=torch.bfloat16: (torch.randn(*shape, generator=gen, device=dev) * std).to(dt)
    X, dO = draw((N, d_model), 1.0), draw((N, d_model), 1.0)
    W_K, W_V = draw((d_model, d_out), 0.02), draw((d_model, d_out), 0.02)
    W_Q, W_O = draw((E, d_model, d_out), 0.02), draw((E, d_out, d_model), 0.02)
    logits = draw((N, E), 1.0, torch.float32)

    def fwd():
        ei, gates = smoe.topk_gate(logits, k)
        r = smoe.route(ei, E)
        O, buf = smoe.momha_fwd(X, W_K, W_V, W_Q, W_O, r, k, gates, B, T, h, d_head)
        return r, gates, buf

    def step():
        r, gates, buf = fwd()
        smoe.momha_bwd(dO, X, W_K, W_V, W_Q, W_O, r, k, gates, B, T, h, d_head, buf)
        return buf

    def timed(fn, reps):
        for _ in range(args.warmup):
            out = fn()
        ev = _events(reps + 1)
        ev[0].record(stream)
        for i in range(reps):
            fn()
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        return np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]), out

    ts_f, _ = timed(fwd, args.steps)
    t0 = time.perf_counter()
    ts, buf = timed(step, args.steps)
    Qh = buf.Q.view(B, T, k, h, d_head)
    Kh, Vh = buf.K.view(B, T, h, d_head), buf.V.view(B, T, h, d_head)
    ts_a, (Oh, L) = timed(lambda: smoe.attention_fwd(Qh, Kh, Vh), args.kernel_reps)
    ts_ab, _ = timed(lambda: smoe.attention_bwd(Oh, Qh, Kh, Vh, Oh, L), args.kernel_reps)
    pl = 2.0 * Tk * d_model * d_out * 2          # query and output ParallelLinears
    dense = 2.0 * N * d_model * d_out * 2        # key and value projections
    attn = 2.0 * 2.0 * B * h * (T * k) * ((T + 1) / 2.0) * d_head       # QK^T and PV over the causal half
    flops = 3.0 * (pl + dense) + 3.5 * attn      # backward: two products per forward GEMM, five per attention pair
    ms = float(np.median(ts))
    ach = attn / (np.median(ts_a) * 1e-3) / 1e12
    print(json.dumps({
        "metric": "SMoE multi-head attention layer (Alg. 4) fwd+bwd throughput (routing + layer forward + backward)",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{label}: B={B} T={T} d_model={d_model} E={E} k={k} h_expert={h} d_head={d_head}, "
                               "both ParallelLinears scattered->scattered, causal attention"},
        "tokens_per_s": N / (ms * 1e-3),
        "phases_ms": {"forward_with_routing": float(np.median(ts_f)), "attention_fwd": float(np.median(ts_a)),
                      "attention_bwd": float(np.median(ts_ab))},
        "flop": {"parallel_linears_fwd": pl, "dense_kv_fwd": dense, "attention_fwd": attn},
        "roofline": {"bound": "mfma", "kernel": "attn_fwd_kernel (causal grouped-query attention)", "achieved": ach,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                     "ms_per_launch": float(np.median(ts_a)), "flop_per_launch": attn, "traffic": None}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget for the oracle baseline (0 = skip)")
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB elementwise copy kernel (reference for the HBM byte counters)")
    ap.add_argument("--tile-group", type=int, default=0,
                    help="M-tiles per group of the persistent kernels' tile order (measurement aid; default: the library's 4)")
    ap.add_argument("--sweep", choices=["granularity", "sparsity"], default=None,
                    help="run the Sec. 4.2 granularity sweep or the Sec. 4.3 sparsity sweep instead of one workload "
                         "(one JSON line with all points)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (data-parallel sharding is a design note); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        return granularity_sweep(args)
    if args.workload == "C5" or args.workload.startswith("MoA-k"):
        return bench_momha(args)

    import smoe_inputs as si
    import paper_2403_08245_amd as smoe

    cfg = si.CONFIGS[args.workload]
    td = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    if args.tile_group:
        torch.cuda.set_device(0)
        smoe.set_tile_group(args.tile_group)
    case = si.mlp_case(cfg, args.seed)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    logits, X, W1, W2, dY = (case[n].to(dev) for n in ("logits", "X", "W1", "W2", "dY"))
    buf = smoe.MLPBuffers(cfg.T, cfg.k, cfg.E, cfg.d_model, cfg.d_expert, cfg.act, td, dev, training=True)
    stream = torch.cuda.current_stream()

    def step():
        ei, gates = smoe.topk_gate(logits, cfg.k)
        r = smoe.route(ei, cfg.E)
        smoe.mlp_fwd(X, W1, W2, r, cfg.k, gates, cfg.act, buf)
        smoe.mlp_bwd(dY, X, W1, W2, r, cfg.k, gates, cfg.act, buf)
        return ei, gates, r

    for _ in range(args.warmup):
        ei, gates, r = step()
    torch.cuda.synchronize()
    ev = _events(args.steps + 1)
    t0 = time.perf_counter()
    ev[0].record(stream)
    for i in range(args.steps):
        step()
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_step = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)])
    ms = wall * 1e3 / args.steps

    flops = 3.0 * cfg.gemm_flops_fwd()
    tflops = flops / (ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS

    # phases, each timed with events on the launch stream
    def timed(fn, reps):
        fn(); torch.cuda.synchronize()
        e = _events(2)
        e[0].record(stream)
        for _ in range(reps):
            fn()
        e[1].record(stream)
        torch.cuda.synchronize()
        return e[0].elapsed_time(e[1]) / reps

    reps = args.kernel_reps
    ms_route = timed(lambda: smoe.route(smoe.topk_gate(logits, cfg.k)[0], cfg.E), reps)
    ms_fwd = timed(lambda: smoe.mlp_fwd(X, W1, W2, r, cfg.k, gates, cfg.act, buf), reps)
    ms_bwd = timed(lambda: smoe.mlp_bwd(dY, X, W1, W2, r, cfg.k, gates, cfg.act, buf), reps)

    # Dominant kernel of the step: the first ParallelLinear (scattered -> grouped).  For bf16 SwiGLU it runs with the
    # activation in its epilogue; smoe_plinear_act_fwd launches exactly that kernel (and nothing else), writing into
    # the step's own Hpre / H buffers.  Other activations / fp32: the plain product through smoe_plinear_fwd.
    import ctypes
    rc = r.c()
    d_h = cfg.d_h
    dt_code = smoe.BF16 if cfg.dtype == "bf16" else smoe.F32
    fused = cfg.act == si.ACT_SWIGLU and cfg.dtype == "bf16" and cfg.d_model % 32 == 0 and cfg.d_model >= 96 and cfg.E <= 256
    decode = cfg.dtype == "bf16" and cfg.Tk <= 32 * cfg.E and cfg.d_model % 32 == 0
    static4 = "true" if cfg.d_model % 128 == 0 else "false"
    if fused:
        ws_act = smoe._ws(smoe.lib.smoe_plinear_act_fwd_workspace_bytes(dt_code, cfg.act, cfg.T, cfg.k, cfg.d_model,
                                                                     cfg.d_expert, 1), dev)

        def s2s_once():
            smoe.plinear_act_fwd(X, W1, r, cfg.k, cfg.act, out=(buf.H, buf.Hpre), ws=ws_act)

        kname = (f"s2s_stream_kernel<false,false,1,{static4}> (ParallelLinear #1 scattered->grouped with SwiGLU in its "
                 "epilogue, as launched inside the step)")
        if decode:
            kname = "s2s_decode_kernel<1,false> (ParallelLinear #1 with SwiGLU, small batch)"
    else:
        def s2s_once():
            smoe._check(smoe.lib.smoe_plinear_fwd(smoe.ctx(), stream.cuda_stream, dt_code, X.data_ptr(), cfg.T, cfg.d_model,
                                                  W1.data_ptr(), d_h, ctypes.byref(rc), cfg.k, None, 0, 0, 1,
                                                  buf.Hpre.data_ptr(), None), "smoe_plinear_fwd")

        kname = (f"s2s_stream_kernel<false,false,0,{static4}>" if cfg.dtype == "bf16" else "s2s_plain_kernel") + \
                " (ParallelLinear #1, scattered->grouped)"

    ms_s2s = timed(s2s_once, reps)
    s2s_flops = 2.0 * cfg.Tk * cfg.d_model * d_h
    achieved = s2s_flops / (ms_s2s * 1e-3) / 1e12

    # Clock the compute units ran at during one more launch of that kernel (the persistent kernels can report the
    # shader-clock cycles and the 100 MHz real-time ticks each block saw: smoe_set_clock_probe).
    clock = None
    if cfg.dtype == "bf16" and not decode:
        probe = torch.zeros(512, dtype=torch.int64, device=dev)
        smoe.set_clock_probe(probe)
        try:
            for _ in range(3):   # back to back, so the launch that is read runs in the state the timed launches ran in
                s2s_once()
            torch.cuda.synchronize()
        finally:
            smoe.set_clock_probe(None)
        pr = probe.cpu().numpy().reshape(256, 2).astype(np.float64)
        ok = pr[:, 1] > 0
        if ok.any():
            mhz = np.where(ok, pr[:, 0] / np.maximum(pr[:, 1], 1) * 100.0, np.nan)
            clock = {"mean": float(np.nanmean(mhz)), "min": float(np.nanmin(mhz)), "max": float(np.nanmax(mhz)),
                     "per_xcd": [float(np.nanmean(mhz[x::8])) for x in range(8)],
                     "block_us_min": float(pr[ok, 1].min() / 100.0), "block_us_max": float(pr[ok, 1].max() / 100.0),
                     "needed_over_elapsed_cycles": float(s2s_flops / (peak * 1e12 / 2.4e9 / 256.0) / pr[ok, 0].sum())}

    if args.calibrate_copy:   # known traffic: reads 1 GiB, writes 1 GiB per launch
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"s2s_fwd1_{cfg.name}_hbm_traffic.json")
    if os.path.exists(tpath):   # bytes per launch measured with rocprofv3 --pmc (see the file for the commands)
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")

    # Algorithmic bytes of that launch: each used expert's W1 once, one gathered X row per routed row, and what the
    # launch writes (pre-activation, plus H when the activation is fused).
    rows = np.diff(r.expert_offsets.cpu().numpy())
    esz = 2 if cfg.dtype == "bf16" else 4
    used = int((rows > 0).sum())
    s2s_bytes = float(esz) * (used * cfg.d_model * d_h + cfg.Tk * cfg.d_model + cfg.Tk * d_h +
                              (cfg.Tk * cfg.d_expert if fused else 0))
    t_mfma, t_hbm = s2s_flops / (peak * 1e12), s2s_bytes / (PEAK_HBM_GBS * 1e9)
    gbs = s2s_bytes / (ms_s2s * 1e-3) / 1e9
    by_hbm = {"bound": "hbm", "kernel": kname, "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
              "frac": gbs / PEAK_HBM_GBS, "ms_per_launch": ms_s2s, "bytes_per_launch": s2s_bytes, "traffic": traffic}
    by_mfma = {"bound": "mfma", "kernel": kname, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
               "frac": achieved / peak, "ms_per_launch": ms_s2s, "flop_per_launch": s2s_flops, "traffic": traffic}
    # the roofline that bounds the launch is the one with the longer minimum time; the other one rides along
    roofline, other = (by_hbm, by_mfma) if t_hbm > t_mfma else (by_mfma, by_hbm)
    roofline["min_ms_mfma"], roofline["min_ms_hbm"] = t_mfma * 1e3, t_hbm * 1e3
    roofline["other_roofline"] = {k_: other[k_] for k_ in ("bound", "achieved", "peak", "unit", "frac")}
    if clock:      # the published peak assumes 2.4 GHz; this is the clock the kernel actually got
        roofline["shader_clock_mhz"] = clock
        # cycle for cycle: compute-unit cycles the launch's flop needs at the peak rate (2500 TFLOP/s = 256 CUs x 2.4 GHz x
        # 4069 flop per cycle) over the shader-clock cycles its blocks were resident (one block per compute unit),
        # whatever clock those cycles ran at
        roofline["frac_of_peak_at_measured_clock"] = clock.pop("needed_over_elapsed_cycles")

    # Whole forward pass against HBM: algorithmic bytes with the activation counted as its own pass (each used expert's
    # W1 and W2 once, gathered X rows, Hpre written and read, H written and read, Yhat written and read, Y written).
    fwd_bytes = float(esz) * (used * cfg.d_model * (d_h + cfg.d_expert) + cfg.Tk * cfg.d_model + 2 * cfg.Tk * d_h +
                              2 * cfg.Tk * cfg.d_expert + 2 * cfg.Tk * cfg.d_model + cfg.T * cfg.d_model)
    fwd_gbs = fwd_bytes / (ms_fwd * 1e-3) / 1e9
    forward_hbm = {"algorithmic_bytes": fwd_bytes, "ms": ms_fwd, "achieved": fwd_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                   "frac": fwd_gbs / PEAK_HBM_GBS, "min_ms_hbm": fwd_bytes / (PEAK_HBM_GBS * 1e9) * 1e3,
                   "min_ms_mfma": cfg.gemm_flops_fwd() / (peak * 1e12) * 1e3,
                   "tflops": cfg.gemm_flops_fwd() / (ms_fwd * 1e-3) / 1e12}

    out = {
        "metric": "SMoE MLP fwd+bwd GEMM throughput per layer (routing + Alg. 3 forward + backward)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d_model={cfg.d_model} d_expert={cfg.d_expert} E={cfg.E} "
                               f"k={cfg.k} act={'swiglu' if cfg.act == 2 else 'gelu'} zipf_s={cfg.zipf_s}",
                   "global_batch": cfg.T, "expert_rows": rows.tolist()},
        "tokens_per_s": cfg.T / (ms * 1e-3),
        "frac_mfma_peak": tflops / peak,
        "ms_event_median": float(np.median(per_step)), "ms_event_p5": float(np.percentile(per_step, 5)),
        "ms_event_p95": float(np.percentile(per_step, 95)),
        "phases_ms": {"routing": ms_route, "mlp_fwd": ms_fwd, "mlp_bwd": ms_bwd},
        "roofline": roofline,
        "forward_hbm": forward_hbm,
    }
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(case, cfg, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
