#!/usr/bin/env python3
"""Benchmark of the prob-sparse self-attention forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|<name>] [--replays R]
                    [--variant log|ratio|indices|mhsa|bwd]

One "step" is one call of probsparse_attn_fwd (measure, select, attend and
fill: two to four kernels) on one batch of a seeded synthetic workload.
Inputs are resident in device memory before the timed region; the timed steps
rotate over enough independent copies of the batch that each step finds its
tensors in HBM rather than in the 256 MB last-level cache (a back-to-back
"warm" figure on a single copy is reported beside it).  The K steps are captured
once into a HIP graph; the graph is replayed R + 1 times back to back with an
event between replays, the first replay is dropped and the MEDIAN of the other
R intervals is the figure (minimum and maximum beside it), so the number is the
GPU's time for K steps, not the interpreter's time to issue them.

By default all five benchmark workloads are run.  The headline fields (`value`,
`ms_per_step`, `config`, `roofline`, `cpu_baseline`) are those of the largest
one, `longform`; the key `configs` carries the same block for every workload.

`--variant ratio` times the paper's own configuration instead (u = 0.5 n kept
queries, v_i for the others: Sec. 3.2, Sec. 4.2, Eq. 12), `--variant indices`
the layers that reuse a given index set (Sec. 4.4: no measure, no selection),
`--variant mhsa` the whole multi-head module (projections, attention, output
matrix: Sec. 3.1, Sec. 2.2), `--variant bwd` the gradients of the attention and
fill steps for the forward's index sets (Sec. 4.2 retraining); each prints the same kind of line for the whole
call at ONE workload (`--workload`, default conformer_s).

Prints ONE JSON line.  The CPU legs (the float64 oracle on one thread and on all
host cores, the dense float64 reference where affordable) run first, before the
process touches the GPU.
"""
from __future__ import annotations

import argparse
import hashlib
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
# what a CU's vector-memory path returns: 64 B per clock and CU, 256 CUs, 2.4 GHz
L1_RETURN_PEAK_GBS = 64 * 256 * 2.4
HEADLINE = "longform"
ORDER = ["tiny", "conformer_s", "ragged", "conformer_l", "longform"]
METRIC = "prob-sparse MHSA fwd latency (us) & queries/s; % HBM/MFMA roofline"


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


def ideal_bytes(cfg):
    """Whole call with every tensor moved once: Q, K, V in, sample_idx in, out."""
    s = 4 if cfg.dtype == "f32" else 2
    nq = cfg.B * cfg.H * cfg.L
    return 3 * nq * 64 * s + nq * cfg.U * 4 + nq * 64 * s


def attend_flops(cfg):
    return 4 * cfg.B * cfg.H * cfg.U * cfg.L * 64


def workload_label(cfg):
    return f"{cfg.name}: B={cfg.B} H={cfg.H} L={cfg.L} d=64 {cfg.dtype} c={cfg.c:g} U={cfg.U}"


# the sources that define the kernels of stages a1 .. a4 and the host plan that shapes their launches
STAGE_SOURCES = ("psa_api.cpp", "psa_attend.hip", "psa_attend_common.h", "psa_device.h", "psa_internal.h",
                 "psa_measure.hip", "psa_select.h", "psa_select.hip", "psa_tile.h", "psa_trace.h")


def sources_digest():
    """Digest of the stage kernels' sources: a stored HBM-traffic figure is only quoted for the sources it was measured on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2106_09236_amd", "csrc")
    for f in STAGE_SOURCES:
        h.update(f.encode())
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(name):
    """HBM bytes per launch of each kernel from the committed rocprofv3 --pmc runs (profiles/traffic_<name>.json),
    or None when the kernel sources have changed since they were measured."""
    tpath = os.path.join(ROOT, "profiles", f"traffic_{name}.json")
    if not os.path.exists(tpath):
        return None
    d = json.load(open(tpath))
    if d.get("sources") != sources_digest():
        return None
    return d


# ---------------------------------------------------------------------------------------------------------
# CPU legs: the oracle as it stands, before anything touches the GPU
# ---------------------------------------------------------------------------------------------------------
_CPU_W = None          # the workload the pool's workers inherit by fork


def _cpu_head(task):
    """Oracle for one (batch, head) pair; run inside a worker with the math library held to one thread."""
    from oracle import probsparse_oracle as O
    b, h = task
    w = _CPU_W
    n = w.cfg.L if w.lengths is None else int(w.lengths[b])
    Q, K, V = (w.as_f64_head(name, b, h) for name in ("Q", "K", "V"))
    O.probsparse_head(Q, K, V, w.sample_idx[b, h], n, w.cfg.c)
    return n


class _HeadView:
    """The arrays of a Workload with per-head float64 widening (so that a worker converts only its own head)."""
    def __init__(self, w):
        self.cfg, self.lengths, self.sample_idx, self._w = w.cfg, w.lengths, w.sample_idx, w

    def as_f64_head(self, name, b, h):
        import numpy as np
        from paper_2106_09236_amd import workloads as W
        a = getattr(self._w, name)[b, h]
        if self.cfg.dtype == "bf16":
            a = W.bf16_bits_to_f32(a)
        return a.astype(np.float64)


def cpu_legs(w, budget_s=6.0):
    """Times the float64 oracle on this workload: one thread (the paper's own setting, Sec. 4.6), all host
    cores parallel over (batch, head), and the dense float64 reference where it is affordable."""
    global _CPU_W
    import multiprocessing as mp
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import probsparse_oracle as O
    cfg = w.cfg
    queries = cfg.B * cfg.H * cfg.L
    tasks = [(b, h) for b in range(cfg.B) for h in range(cfg.H)]
    try:
        host_cores = len(os.sched_getaffinity(0))
    except AttributeError:
        host_cores = os.cpu_count() or 1
    workers = max(1, min(host_cores, 16, len(tasks)))      # a one-GPU machine's CPU share is 16 cores
    view = _HeadView(w)
    _CPU_W = view

    def median_time(fn, cap):
        ts = []
        while len(ts) < 3 or (sum(ts) < cap and len(ts) < 9):
            t0 = time.perf_counter()
            fn()
            ts.append(time.perf_counter() - t0)
            if sum(ts) > 3 * cap:
                break
        return sorted(ts)[len(ts) // 2], len(ts)

    with threadpool_limits(limits=1):
        t1, n1 = median_time(lambda: [_cpu_head(t) for t in tasks], budget_s / 2)
    ctx = mp.get_context("fork")

    def init_worker():
        threadpool_limits(limits=1)
    with ctx.Pool(workers, initializer=init_worker) as pool:
        pool.map(_cpu_head, tasks[:workers])               # start-up outside the timing
        chunk = max(1, len(tasks) // (4 * workers))
        tn, nn = median_time(lambda: pool.map(_cpu_head, tasks, chunksize=chunk), budget_s / 2)
    out = {"value": round(queries / tn, 1), "unit": "queries/s", "cores": workers, "kind": "oracle",
           "sample": f"the whole workload ({queries} queries, {len(tasks)} (batch, head) pairs over {workers} worker "
                     f"processes of one thread each, host shows {host_cores} cores), median of {nn} runs, {tn:.2f} s each",
           "one_thread_value": round(queries / t1, 1),
           "one_thread_sample": f"the whole workload on one thread, median of {n1} runs, {t1:.2f} s each"}
    # dense float64 attention on the CPU (Eq. 6): whole workload where that is seconds, one head at conformer_l,
    # skipped at longform (550 GFLOP)
    dense_flops = 4 * cfg.B * cfg.H * cfg.L * cfg.L * 64
    if dense_flops <= 2e10:
        heads, what = tasks, "the whole workload"
    elif 4 * cfg.L * cfg.L * 64 <= 2e10:
        heads, what = tasks[:1], "one (batch, head) pair of the workload"
    else:
        heads, what = [], ""
    if heads:
        def dense():
            for b, h in heads:
                n = cfg.L if w.lengths is None else int(w.lengths[b])
                O.attention_rows(view.as_f64_head("Q", b, h)[:n], view.as_f64_head("K", b, h)[:n],
                                 view.as_f64_head("V", b, h)[:n])
        td, nd = median_time(dense, 2.0)
        out["dense_cpu"] = {"queries_per_s": round(len(heads) * cfg.L / td, 1), "sample": f"{what}, library threads as "
                            f"they come, median of {nd} runs, {td:.2f} s each"}
    else:
        out["dense_cpu"] = None                            # skipped: too many flops for the CPU leg
    _CPU_W = None
    return out


# ---------------------------------------------------------------------------------------------------------
# GPU side
# ---------------------------------------------------------------------------------------------------------
def plan_words(shape, opt=None, u_stride=0):
    """Which kernels the call launches (the host's choice), as a short string for the JSON line."""
    from paper_2106_09236_amd import binding as psa
    d = psa.probsparse_describe_plan(shape, opt, u_stride)
    return " ".join(f"{k}={d[k]}" for k in ("measure", "select", "attend", "key_splits", "merge"))


class Timer:
    """Median / min / max over R back-to-back replays of a graph of K steps (events on the launch stream)."""
    def __init__(self, steps, replays):
        self.steps, self.replays = steps, replays

    def graph_us(self, fn, n_steps=None):
        import torch
        n_steps = self.steps if n_steps is None else n_steps
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n_steps):
                fn(i)
        g.replay()                                        # untimed: graph upload
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(self.replays + 2)]
        ev[0].record()
        for r in range(self.replays + 1):
            g.replay()
            ev[r + 1].record()
        torch.cuda.synchronize()
        dt = sorted(ev[r].elapsed_time(ev[r + 1]) * 1e3 / n_steps for r in range(1, self.replays + 1))   # first dropped
        del g
        return {"median": dt[len(dt) // 2], "min": dt[0], "max": dt[-1]}

    def eager_us(self, fn):
        import torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(self.steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / self.steps


def device_sets(cfg, w, ws_bytes):
    """Enough independent copies of the batch (inputs, out, workspace) to exceed 3x the last-level cache."""
    import torch

    def dev(a):
        x = torch.from_numpy(a)
        if cfg.dtype == "bf16":
            x = x.view(torch.int16).view(torch.bfloat16)
        return x.cuda()
    base = (dev(w.Q), dev(w.K), dev(w.V), None if w.lengths is None else torch.from_numpy(w.lengths).cuda(),
            torch.from_numpy(w.sample_idx).cuda())
    set_bytes = (sum(t.numel() * t.element_size() for t in base if t is not None)
                 + base[0].numel() * base[0].element_size() + ws_bytes)
    n_sets = max(2, math.ceil(768e6 / set_bytes))          # > 3x the 256 MB last-level cache
    sets = []
    for _ in range(n_sets):
        ts = tuple(None if t is None else t.clone() for t in base)
        sets.append((ts, torch.empty_like(base[0]), torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")))
    return sets


def gpu_block(cfg, w, args, timer):
    """Whole-call and per-kernel timing of one workload; returns its block of the JSON line."""
    import torch
    from paper_2106_09236_amd import binding as psa
    shape = psa.make_shape(cfg.B, cfg.H, cfg.L, cfg.U, psa.PSA_F32 if cfg.dtype == "f32" else psa.PSA_BF16)
    ws_bytes = psa.workspace_bytes(shape, cfg.c)
    sets = device_sets(cfg, w, ws_bytes)
    n_sets = len(sets)

    def step(i, mask=psa.STAGE_ALL):
        (Q, K, V, lengths, idx), out, ws = sets[i % n_sets]
        psa.probsparse_attn_fwd_stages(Q, K, V, lengths, idx, cfg.c, out, ws, mask)

    def dense_step(i):
        (Q, K, V, lengths, idx), out, ws = sets[i % n_sets]
        psa.dense_attn_fwd(Q, K, V, lengths, out=out, workspace=ws)

    # fill every workspace with valid intermediates, then warm up
    for i in range(n_sets):
        step(i)
    for i in range(args.warmup):
        step(i)
    dense_step(0)
    torch.cuda.synchronize()

    # ---- the timed region: graphs of exactly K whole-path steps, rotating inputs
    whole = timer.graph_us(step)
    us = whole["median"]
    queries = cfg.B * cfg.H * cfg.L
    eager = timer.eager_us(step)                           # same steps issued call by call from Python
    warm = timer.graph_us(lambda i: step(0))               # one input set: cache-resident

    # ---- per-stage durations (each stage launched alone K times, same rotation)
    plan = psa.probsparse_describe_plan(shape, psa.PsaOptions(psa.U_LOG, psa.FILL_MEAN, cfg.c))
    stages = {"measure": psa.STAGE_MEASURE, "attend": psa.STAGE_ATTEND}
    if plan["select"] in ("kernel", "segments"):
        stages["select"] = psa.STAGE_SELECT
    stage_us = {k: timer.graph_us(lambda i, m=m: step(i, m)) for k, m in stages.items()}
    # the dense baseline is up to a millisecond per call: about 20 ms of it per replay
    dense_est_us = 4.0 * cfg.B * cfg.H * cfg.L * cfg.L * 64 / (40e12 if cfg.dtype == "f32" else 500e12) * 1e6
    dense_steps = max(5, min(timer.steps, int(2e4 / max(1.0, dense_est_us))))
    dense = timer.graph_us(dense_step, n_steps=dense_steps)
    traffic = stored_traffic(cfg.name)
    kernels = {}
    for k in stages:
        by = algorithmic_bytes(cfg, k)
        t = stage_us[k]["median"]
        kernels[k] = {"us": round(t, 3), "us_min": round(stage_us[k]["min"], 3), "us_max": round(stage_us[k]["max"], 3),
                      "alg_bytes": by, "GBps": round(by / (t * 1e-6) / 1e9, 1),
                      "hbm_frac": round(by / (t * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                      "traffic": None if traffic is None else traffic.get(k)}
    fl = attend_flops(cfg)
    mfma_peak = FP64_MFMA_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS
    ta = stage_us["attend"]["median"]
    kernels["attend"]["TFLOPs"] = round(fl / (ta * 1e-6) / 1e12, 3)
    kernels["attend"]["mfma_frac"] = round(fl / (ta * 1e-6) / 1e12 / mfma_peak, 4)
    kernels["attend"]["mfma_dtype"] = "f64" if cfg.dtype == "f32" else "bf16"
    # the measure stage is a gather: its second bound is what the CUs' vector-memory path can return
    # (every sampled key row crosses it once), beside the HBM bound of the compulsory bytes
    if plan["measure"] == "stream":
        gb = queries * cfg.U * 64 * (4 if cfg.dtype == "f32" else 2)
        tm = stage_us["measure"]["median"]
        kernels["measure"]["gather_bytes"] = gb
        kernels["measure"]["l1_return_frac"] = round(gb / (tm * 1e-6) / 1e9 / L1_RETURN_PEAK_GBS, 4)

    dom = max(stage_us, key=lambda k: stage_us[k]["median"])
    if dom == "attend" and kernels["attend"]["mfma_frac"] > kernels["attend"]["hbm_frac"]:
        ach = kernels["attend"]["TFLOPs"]
        roofline = {"kernel": "attend", "bound": "mfma", "achieved": ach, "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": round(ach / mfma_peak, 4), "traffic": kernels["attend"]["traffic"]}
    else:
        ach = kernels[dom]["GBps"]
        roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": kernels[dom]["traffic"]}
    del sets
    torch.cuda.empty_cache()
    ib = ideal_bytes(cfg)
    return {
        "workload": workload_label(cfg),
        "latency_us": round(us, 3), "latency_us_min": round(whole["min"], 3), "latency_us_max": round(whole["max"], 3),
        "queries_per_s": round(queries / (us * 1e-6), 1),
        "frames_per_s": round(float(w.lengths_or_full().sum()) / (us * 1e-6), 1),
        "queries_per_step": queries, "input_copies_rotated": n_sets,
        "tensor_dtype": cfg.dtype, "accumulate_dtype": "f64" if cfg.dtype == "f32" else "f32",
        "kernel_plan": " ".join(f"{k}={plan[k]}" for k in ("measure", "select", "attend", "key_splits", "merge")),
        "whole_call_hbm_frac": round(ib / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "ideal_bytes": ib,
        "roofline": roofline, "kernels": kernels,
        "dense_baseline": {"us": round(dense["median"], 3), "us_min": round(dense["min"], 3),
                           "us_max": round(dense["max"], 3), "steps": dense_steps,
                           "speedup_vs_dense": round(dense["median"] / us, 2),
                           "TFLOPs": round(4 * cfg.B * cfg.H * cfg.L * cfg.L * 64 / (dense["median"] * 1e-6) / 1e12, 2),
                           "arithmetic": ("float64 MFMA, parity-holding (the same arithmetic as the prob-sparse path)"
                                          if cfg.dtype == "f32" else "bfloat16 MFMA, float32 accumulation")},
        "eager_latency_us": round(eager, 3), "warm_latency_us": round(warm["median"], 3),
    }


def variant_line(args, cfg, w, timer):
    """Whole-call timing of the two variants the paper itself describes, and of the whole module."""
    import ctypes
    import torch
    from paper_2106_09236_amd import binding as psa
    from paper_2106_09236_amd import workloads as W_
    shape = psa.make_shape(cfg.B, cfg.H, cfg.L, cfg.U, psa.PSA_F32 if cfg.dtype == "f32" else psa.PSA_BF16)
    lib = psa.load()
    sets = device_sets(cfg, w, psa.workspace_bytes(shape, cfg.c))
    n_sets = len(sets)
    s = 4 if cfg.dtype == "f32" else 2
    nq = cfg.B * cfg.H * cfg.L
    extra_flops = 0
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
        dm = cfg.H * 64
        u = cfg.U

        def step(i):
            (_, _, _, lengths, idx), _, _ = sets[i % n_sets]
            psa.probsparse_mhsa_fwd(Xs[i % n_x], weights, lengths, idx, psa.U_LOG, cfg.c, psa.FILL_MEAN,
                                    Y=Ys[i % n_x], workspace=wss[i % n_x])
        n_sets = n_x
        # X in, Y out, weights, sample_idx; Q, K, V, A written once and read once each
        alg_bytes = 2 * nq * 64 * s + 4 * dm * dm * s + nq * cfg.U * 4 + 2 * 4 * nq * 64 * s
        what = f"projections + attention + output matrix, d_model = {dm}"
        plan = plan_words(shape, opt)
        extra_flops = 4 * 2 * cfg.B * cfg.L * dm * dm
    elif args.variant == "bwd":
        um = psa.u_max(shape, cfg.c)
        need = lib.probsparse_attn_bwd_workspace_bytes(ctypes.byref(shape), um)
        wss = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(n_sets)]
        (Q, K, V, lengths, idx), out, ws = sets[0]
        _, _, sel, ub = psa.probsparse_attn_fwd_debug(Q, K, V, lengths, idx, cfg.c, out=out, workspace=ws)
        u = cfg.U
        grads = [tuple(torch.empty_like(Q) for _ in range(3)) for _ in range(n_sets)]
        Gs = [torch.randn(Q.shape, device="cuda").to(Q.dtype) for _ in range(n_sets)]

        def step(i):
            (Q, K, V, lengths, idx), _, _ = sets[i % n_sets]
            dQ, dK, dV = grads[i % n_sets]
            shape_ = shape
            rc = lib.probsparse_attn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                         None if lengths is None else lengths.data_ptr(), sel.data_ptr(), ub.data_ptr(),
                                         um, psa.FILL_MEAN, Gs[i % n_sets].data_ptr(), dQ.data_ptr(), dK.data_ptr(),
                                         dV.data_ptr(), ctypes.byref(shape_), wss[i % n_sets].data_ptr(), need,
                                         torch.cuda.current_stream().cuda_stream)
            assert rc == 0, rc
        # Q, K, V, dOut in; dQ, dK, dV out
        alg_bytes = 7 * nq * 64 * s
        what = f"gradients of the attention and fill steps for the forward's own index sets (u = {u}), mean fill, float64 arithmetic"
        plan = "stats + dq + dkv (+ dq reduce)"
        extra_flops = 4 * 4 * cfg.B * cfg.H * u * cfg.L * 64 - 4 * cfg.B * cfg.H * u * cfg.L * 64     # five products, two of them twice
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
    t = timer.graph_us(step)
    us = t["median"]
    flops = 4 * cfg.B * cfg.H * u * cfg.L * 64 + extra_flops     # (+ the four d_model x d_model products)
    peak = FP64_MFMA_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS
    tf, gbs = flops / (us * 1e-6) / 1e12, alg_bytes / (us * 1e-6) / 1e9
    # (the module mixes float32/bfloat16 GEMM flops with the attention's: no single matrix peak applies, so its
    # line is priced against HBM by algorithmic bytes)
    if args.variant == "bwd":
        peak = FP64_MFMA_PEAK_TFLOPS                          # float64 MFMA for both tensor types
    if args.variant != "mhsa" and tf / peak > gbs / HBM_PEAK_GBS:
        roofline = {"kernel": "whole call", "bound": "mfma", "achieved": round(tf, 3), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(tf / peak, 4), "traffic": None}
    else:
        roofline = {"kernel": "whole call", "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None}
    print(json.dumps({
        "metric": METRIC,
        "value": round(nq / (us * 1e-6), 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(us * 1e-3, 6), "latency_us": round(us, 3),
        "latency_us_min": round(t["min"], 3), "latency_us_max": round(t["max"], 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if (cfg.dtype == "f32" or args.variant == "bwd") else "f32", "data": "synthetic",
        "config": {"workload": workload_label(cfg), "tensor_dtype": cfg.dtype,
                   "variant": f"{args.variant}: {what}", "queries_per_step": nq, "input_copies_rotated": n_sets,
                   "launch": f"hip graph of {args.steps} steps, median of {timer.replays} replays", "kernel_plan": plan},
        "roofline": roofline, "cpu_baseline": None,
        "whole_call": {"alg_bytes": alg_bytes, "GBps": round(gbs, 1), "flops": flops, "TFLOPs": round(tf, 3)},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--replays", type=int, default=11, help="timed replays of the graph of K steps (median reported)")
    ap.add_argument("--workload", default=None, help="all (default), or one of " + ", ".join(ORDER))
    ap.add_argument("--variant", default="log", choices=["log", "ratio", "indices", "mhsa", "bwd"])
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
    if args.replays < 3:
        args.replays = 3

    from paper_2106_09236_amd import workloads as W
    if args.variant != "log":
        names = [args.workload or "conformer_s"]
    elif args.workload in (None, "all"):
        names = ORDER
    else:
        names = [args.workload]
    for n in names:
        if n not in W.CONFIGS:
            print(f"bench.py: unknown workload {n!r}", file=sys.stderr)
            sys.exit(2)
    head_name = HEADLINE if HEADLINE in names else names[-1]

    # ---- CPU legs first: the worker processes are forked before this process touches the GPU
    made = {}
    cpu = {}
    if args.variant == "log" and not args.no_cpu:
        for n in names:
            made[n] = W.make_workload(W.CONFIGS[n])
            cpu[n] = cpu_legs(made[n], budget_s=8.0 if n == head_name else 3.0)
            print(f"bench.py: cpu legs of {n} done", file=sys.stderr, flush=True)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    timer = Timer(args.steps, args.replays)

    if args.variant != "log":
        cfg = W.CONFIGS[names[0]]
        return variant_line(args, cfg, W.make_workload(cfg), timer)

    if args.pmc_calibration:
        src = torch.zeros(256 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)                                 # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    blocks = {}
    for n in names:
        cfg = W.CONFIGS[n]
        w = made.pop(n, None) or W.make_workload(cfg)
        blocks[n] = gpu_block(cfg, w, args, timer)
        blocks[n]["cpu_baseline"] = cpu.get(n)
        del w
        print(f"bench.py: {n} timed: {blocks[n]['latency_us']} us", file=sys.stderr, flush=True)

    h = blocks[head_name]
    hcfg = W.CONFIGS[head_name]
    line = {
        "metric": METRIC,
        "value": h["queries_per_s"], "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(h["latency_us"] * 1e-3, 6), "latency_us": h["latency_us"],
        "latency_us_min": h["latency_us_min"], "latency_us_max": h["latency_us_max"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if hcfg.dtype == "f32" else "f32", "data": "synthetic",
        "config": {"workload": h["workload"], "tensor_dtype": h["tensor_dtype"], "accumulate_dtype": h["accumulate_dtype"],
                   "queries_per_step": h["queries_per_step"], "input_copies_rotated": h["input_copies_rotated"],
                   "launch": f"hip graph of {args.steps} steps, median of {args.replays} back-to-back replays "
                             "(the first one dropped)",
                   "kernel_plan": h["kernel_plan"]},
        "roofline": h["roofline"],
        "cpu_baseline": h["cpu_baseline"],
        "kernels": h["kernels"],
        "dense_baseline": h["dense_baseline"],
        "frames_per_s": h["frames_per_s"],
        "eager_latency_us": h["eager_latency_us"],
        "warm_latency_us": h["warm_latency_us"],
        "whole_call_hbm_frac": h["whole_call_hbm_frac"],
        "configs": {n: b for n, b in blocks.items() if n != head_name},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
