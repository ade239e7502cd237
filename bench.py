#!/usr/bin/env python3
"""Benchmark of the prob-sparse self-attention forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload conformer_s] [--variant log|ratio|indices|mhsa]

One "step" is one call of probsparse_attn_fwd (measure, select, attend and
fill: two or three kernels) on one batch of the seeded synthetic workload.
Inputs are resident in device memory before the timed region; the timed loop
rotates over enough independent copies of the batch that each step finds its
tensors in HBM rather than in the 256 MB last-level cache (a back-to-back
"warm" figure on a single copy is reported beside it).  The K steps are captured
once into a HIP graph and replayed, so the figure is the GPU's time for the
steps, not the interpreter's time to issue them (that one is `eager_latency_us`).

`--variant ratio` times the paper's own configuration instead (u = 0.5 n kept
queries, v_i for the others: Sec. 3.2, Sec. 4.2, Eq. 12), `--variant indices`
the layers that reuse a given index set (Sec. 4.4: no measure, no selection),
`--variant mhsa` the whole multi-head module (projections, attention, output
matrix: Sec. 3.1, Sec. 2.2); each prints the same kind of line for the whole call.

Prints ONE JSON line: whole-call throughput in queries/s (B*H*L_Q per step),
the roofline of the dominant kernel (timed alone, live, with events on the
launch stream), and the float64 CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
FP64_MFMA_PEAK_TFLOPS = 78.6     # dense float64 matrix
BF16_MFMA_PEAK_TFLOPS = 2500.0   # dense bfloat16 matrix


def algorithmic_bytes(cfg, stage):
    """Bytes each stage must move if every tensor crossed HBM exactly once."""
    s = 4 if cfg.dtype == "f32" else 2
    nq = cfg.B * cfg.H * cfg.L
    d = 64
    u = cfg.U                                   # u = U at every named workload
    if stage == "measure":                      # Q, K, V once, sample_idx, M out
        return 3 * nq * d * s + nq * cfg.U * 4 + nq * 4
    if stage == "select":
        return nq * 4 + cfg.B * cfg.H * u * 4
    if stage == "attend":                       # K, V once, selected Q rows, every output row written once
        return cfg.B * cfg.H * (2 * cfg.L * d * s + u * d * s) + nq * d * s
    raise ValueError(stage)


def attend_flops(cfg):
    return 4 * cfg.B * cfg.H * cfg.U * cfg.L * 64


def variant_line(args, cfg, w, sets, n_sets, psa):
    """Whole-call timing of the two variants the paper itself describes."""
    import ctypes
    import torch
    from paper_2106_09236_amd import workloads as W_
    shape = psa.make_shape(cfg.B, cfg.H, cfg.L, cfg.U, psa.PSA_F32 if cfg.dtype == "f32" else psa.PSA_BF16)
    lib = psa.load()
    s = 4 if cfg.dtype == "f32" else 2
    nq = cfg.B * cfg.H * cfg.L
    if args.variant == "ratio":
        rs = args.r_sparse
        opt = psa.PsaOptions(psa.U_RATIO, psa.FILL_VALUE, rs)
        need = lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(shape), ctypes.byref(opt))
        wss = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(n_sets)]
        u = math.ceil(rs * cfg.L)

        def step(i):
            (Q, K, V, lengths, idx), out, _ = sets[i % n_sets]
            psa.probsparse_attn_fwd_opt(Q, K, V, lengths, idx, psa.U_RATIO, rs, psa.FILL_VALUE, out=out,
                                        workspace=wss[i % n_sets], taps=False)
        alg_bytes = 4 * nq * 64 * s + nq * cfg.U * 4          # Q, K, V in, out, sample_idx
        what = f"u = ceil({rs:g} n) = {u} kept queries per head, v_i fill"
        plan = plan_words(shape, opt)
    elif args.variant == "mhsa":
        raw = W_.make_mhsa_inputs(cfg.B, cfg.L, cfg.H, cfg.dtype, seed=1)

        def dev(a):
            x = torch.from_numpy(a)
            if cfg.dtype == "bf16":
                x = x.view(torch.int16).view(torch.bfloat16)
            return x.cuda()
        d = {k: dev(v) for k, v in raw.items()}
        weights = psa.make_weights(d["Wq"], d["Wk"], d["Wv"], d["Wo"], d["bq"], d["bk"], d["bv"], d["bo"])
        opt = psa.PsaOptions(psa.U_LOG, psa.FILL_MEAN, cfg.c)
        need = lib.probsparse_mhsa_workspace_bytes(ctypes.byref(shape), ctypes.byref(opt))
        n_x = max(2, math.ceil(768e6 / (need + 2 * d["X"].numel() * d["X"].element_size())))
        Xs = [d["X"].clone() for _ in range(n_x)]
        Ys = [torch.empty_like(d["X"]) for _ in range(n_x)]
        wss = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(n_x)]
        n_sets = n_x
        dm = cfg.H * 64
        u = cfg.U

        def step(i):
            (_, _, _, lengths, idx), _, _ = sets[i % len(sets)]
            psa.probsparse_mhsa_fwd(Xs[i % n_x], weights, lengths, idx, psa.U_LOG, cfg.c, psa.FILL_MEAN,
                                    Y=Ys[i % n_x], workspace=wss[i % n_x])
        # X in, Y out, weights, sample_idx; Q, K, V, A written once and read once each
        alg_bytes = 2 * nq * 64 * s + 4 * dm * dm * s + nq * cfg.U * 4 + 2 * 4 * nq * 64 * s
        what = f"projections + attention + output matrix, d_model = {dm}"
        plan = plan_words(shape, opt)
        extra_flops = 4 * 2 * cfg.B * cfg.L * dm * dm
    else:
        um = psa.u_max(shape, cfg.c)
        need = lib.probsparse_attn_with_indices_workspace_bytes(ctypes.byref(shape), um)
        wss = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(n_sets)]
        (Q, K, V, lengths, idx), out, ws = sets[0]
        _, _, sel, ub = psa.probsparse_attn_fwd_debug(Q, K, V, lengths, idx, cfg.c, out=out, workspace=ws)
        u = cfg.U

        def step(i):
            (Q, K, V, lengths, idx), out, _ = sets[i % n_sets]
            psa.probsparse_attn_fwd_with_indices(Q, K, V, lengths, sel, ub, psa.FILL_MEAN, out=out,
                                                 workspace=wss[i % n_sets])
        alg_bytes = 2 * nq * 64 * s + cfg.B * cfg.H * u * 64 * s + nq * 64 * s   # K, V, kept Q rows in, out
        what = f"index sets of the full forward reused (u = {u}), mean fill"
        plan = plan_words(shape, None, um)
    for i in range(max(n_sets, args.warmup)):
        step(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(args.steps):
            step(i)
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    flops = 4 * cfg.B * cfg.H * u * cfg.L * 64
    if args.variant == "mhsa":
        flops += extra_flops                                  # the four d_model x d_model products
    peak = FP64_MFMA_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS
    tf, gbs = flops / (ms * 1e-3) / 1e12, alg_bytes / (ms * 1e-3) / 1e9
    # (the module mixes float32/bfloat16 GEMM flops with the attention's: no single matrix peak applies, so its
    # line is priced against HBM by algorithmic bytes)
    if args.variant != "mhsa" and tf / peak > gbs / HBM_PEAK_GBS:
        roofline = {"kernel": "whole call", "bound": "mfma", "achieved": round(tf, 3), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(tf / peak, 4), "traffic": None}
    else:
        roofline = {"kernel": "whole call", "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None}
    print(json.dumps({
        "metric": "prob-sparse MHSA fwd latency (us) & queries/s; % HBM/MFMA roofline",
        "value": round(nq / (ms * 1e-3), 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 6), "latency_us": round(ms * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if cfg.dtype == "f32" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} H={cfg.H} L={cfg.L} d=64 {cfg.dtype} U={cfg.U}",
                   "variant": f"{args.variant}: {what}", "queries_per_step": nq, "input_copies_rotated": n_sets,
                   "launch": "hip graph replay", "kernel_plan": plan},
        "roofline": roofline, "cpu_baseline": None,
        "whole_call": {"alg_bytes": alg_bytes, "GBps": round(gbs, 1), "flops": flops, "TFLOPs": round(tf, 3)},
    }))


def plan_words(shape, opt=None, u_stride=0):
    """Which kernels the call launches (the host's choice), as a short string for the JSON line."""
    from paper_2106_09236_amd import binding as psa
    d = psa.probsparse_describe_plan(shape, opt, u_stride)
    return " ".join(f"{k}={d[k]}" for k in ("measure", "select", "attend", "key_splits", "merge"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="conformer_s")
    ap.add_argument("--variant", default="log", choices=["log", "ratio", "indices", "mhsa"])
    ap.add_argument("--r-sparse", type=float, default=0.5,
                    help="share of the queries kept by --variant ratio (Sec. 3.2; the paper uses 0.35 .. 0.5)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy a few times, so that a rocprofv3 --pmc run "
                         "of this command has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 "
              "(the path shards over (batch, head) pairs with no communication between them)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2106_09236_amd import binding as psa
    from paper_2106_09236_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.workload]
    w = W.make_workload(cfg)

    def dev(a):
        x = torch.from_numpy(a)
        if cfg.dtype == "bf16":
            x = x.view(torch.int16).view(torch.bfloat16)
        return x.cuda()

    base = (dev(w.Q), dev(w.K), dev(w.V), None if w.lengths is None else torch.from_numpy(w.lengths).cuda(),
            torch.from_numpy(w.sample_idx).cuda())
    shape = psa.make_shape(cfg.B, cfg.H, cfg.L, cfg.U, psa.PSA_F32 if cfg.dtype == "f32" else psa.PSA_BF16)
    ws_bytes = psa.workspace_bytes(shape, cfg.c)
    set_bytes = sum(t.numel() * t.element_size() for t in base if t is not None) + base[0].numel() * base[0].element_size() + ws_bytes
    n_sets = max(2, math.ceil(768e6 / set_bytes))          # > 3x the 256 MB last-level cache
    sets = []
    for i in range(n_sets):
        ts = tuple(None if t is None else t.clone() for t in base)
        sets.append((ts, torch.empty_like(base[0]), torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")))

    def step(i, mask=psa.STAGE_ALL):
        (Q, K, V, lengths, idx), out, ws = sets[i % n_sets]
        psa.probsparse_attn_fwd_stages(Q, K, V, lengths, idx, cfg.c, out, ws, mask)

    if args.variant != "log":
        return variant_line(args, cfg, w, sets, n_sets, psa)

    def dense_step(i):
        (Q, K, V, lengths, idx), out, ws = sets[i % n_sets]
        psa.dense_attn_fwd(Q, K, V, lengths, out=out, workspace=ws)

    def ms_between(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def eager_ms(n_steps, fn=step, **kw):
        return ms_between(lambda: [fn(i, **kw) for i in range(n_steps)]) / n_steps

    def graph_ms(n_steps, fn=step, **kw):
        """The same K launches captured once into a HIP graph and replayed: the
        GPU time of the launches without the Python/ctypes cost of issuing them."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n_steps):
                fn(i, **kw)
        g.replay()                                        # untimed: graph upload
        torch.cuda.synchronize()
        return ms_between(g.replay) / n_steps

    if args.pmc_calibration:
        src = torch.zeros(256 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)                                 # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # fill every workspace with valid intermediates, then warm up
    for i in range(n_sets):
        step(i)
    for i in range(args.warmup):
        step(i)
    dense_step(0)
    torch.cuda.synchronize()

    # ---- the timed region: exactly K whole-path steps (graph replay), rotating inputs
    t0 = time.perf_counter()
    ms_per_step = graph_ms(args.steps)
    queries = cfg.B * cfg.H * cfg.L
    value = queries / (ms_per_step * 1e-3)
    eager = eager_ms(args.steps)                           # same steps issued call by call from Python
    warm = graph_ms(args.steps, fn=lambda i, **kw: step(0))  # one input set: cache-resident

    # ---- per-stage durations (each stage launched alone K times, same rotation)
    stages = {"measure": psa.STAGE_MEASURE, "attend": psa.STAGE_ATTEND}
    if cfg.L * 64 * (4 if cfg.dtype == "f32" else 2) > 128 * 1024:      # K of a head beyond the measure kernel's LDS
        stages["select"] = psa.STAGE_SELECT
    stage_us = {k: graph_ms(args.steps, mask=m) * 1e3 for k, m in stages.items()}
    dense_us = graph_ms(max(20, args.steps // 4), fn=lambda i, **kw: dense_step(i)) * 1e3
    dom = max(stage_us, key=stage_us.get)
    kernels = {}
    for k in stages:
        by = algorithmic_bytes(cfg, k)
        kernels[k] = {"us": round(stage_us[k], 3), "alg_bytes": by,
                      "GBps": round(by / (stage_us[k] * 1e-6) / 1e9, 1),
                      "hbm_frac": round(by / (stage_us[k] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    fl = attend_flops(cfg)
    mfma_peak = FP64_MFMA_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS
    kernels["attend"]["TFLOPs"] = round(fl / (stage_us["attend"] * 1e-6) / 1e12, 3)
    kernels["attend"]["mfma_frac"] = round(fl / (stage_us["attend"] * 1e-6) / 1e12 / mfma_peak, 4)
    kernels["attend"]["mfma_dtype"] = "f64" if cfg.dtype == "f32" else "bf16"

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{cfg.name}.json")
    if os.path.exists(tpath):                              # HBM bytes per launch from rocprofv3 --pmc runs
        traffic = json.load(open(tpath)).get(dom)
    if dom == "attend" and kernels["attend"]["mfma_frac"] > kernels["attend"]["hbm_frac"]:
        ach = kernels["attend"]["TFLOPs"]
        roofline = {"kernel": "attend", "bound": "mfma", "achieved": ach, "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": round(ach / mfma_peak, 4), "traffic": traffic}
    else:
        ach = kernels[dom]["GBps"]
        roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic}

    # ---- CPU oracle on the host cores (float64 NumPy, as it stands)
    cpu = None
    if not args.no_cpu:
        from oracle import probsparse_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        except Exception:
            cores = 1
        nb = max(1, min(cfg.B, int(round(cfg.B * 65536 / max(queries, 1)))))    # about 64K queries of CPU work
        Qs, Ks, Vs = (w.as_f64(n)[:nb] for n in ("Q", "K", "V"))
        ls = None if w.lengths is None else w.lengths[:nb]
        times = []
        busy0 = time.process_time()
        while sum(times) < 10.0 and len(times) < 100:        # about 10 s of CPU work
            t0 = time.perf_counter()
            O.probsparse_attn_fwd(Qs, Ks, Vs, ls, w.sample_idx[:nb], cfg.c)
            times.append(time.perf_counter() - t0)
        # threads it actually kept busy: CPU time of the process over wall time (the library pool is larger)
        used = max(1, int(round((time.process_time() - busy0) / max(sum(times), 1e-9))))
        dt = sorted(times)[len(times) // 2]
        cpu = {"value": round(nb * cfg.H * cfg.L / dt, 1), "unit": "queries/s", "cores": min(used, cores), "kind": "oracle",
               "sample": f"first {nb} of {cfg.B} batch items ({nb * cfg.H * cfg.L} queries), "
                         f"median of {len(times)} runs, {dt:.2f} s each; library thread pool of {cores}"}
        # the paper's own setting is one CPU thread (Sec. 4.6): the same sample with the library pools held to one
        try:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                t1 = []
                while sum(t1) < 4.0 and len(t1) < 20:
                    t0 = time.perf_counter()
                    O.probsparse_attn_fwd(Qs, Ks, Vs, ls, w.sample_idx[:nb], cfg.c)
                    t1.append(time.perf_counter() - t0)
            cpu["one_thread_value"] = round(nb * cfg.H * cfg.L / sorted(t1)[len(t1) // 2], 1)
        except Exception:
            pass

    line = {
        "metric": "prob-sparse MHSA fwd latency (us) & queries/s; % HBM/MFMA roofline",
        "value": round(value, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "latency_us": round(ms_per_step * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if cfg.dtype == "f32" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} H={cfg.H} L={cfg.L} d=64 {cfg.dtype} c={cfg.c:g} U={cfg.U}",
                   "queries_per_step": queries, "input_copies_rotated": n_sets, "launch": "hip graph replay",
                   "kernel_plan": plan_words(shape, psa.PsaOptions(psa.U_LOG, psa.FILL_MEAN, cfg.c))},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "dense_baseline": {"us": round(dense_us, 3), "speedup_vs_dense": round(dense_us / (ms_per_step * 1e3), 2),
                           "TFLOPs": round(4 * cfg.B * cfg.H * cfg.L * cfg.L * 64 / (dense_us * 1e-6) / 1e12, 2)},
        "frames_per_s": round(float(w.lengths_or_full().sum()) / (ms_per_step * 1e-3), 1),
        "eager_latency_us": round(eager * 1e3, 3),
        "warm_latency_us": round(warm * 1e3, 3),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
