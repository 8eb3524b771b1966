#!/usr/bin/env python3
"""Benchmark of the fused RMSNorm -> FFN-SwiGLU hot path on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--no-cpu]

A "step" is one pass of the whole hot path over one batch of synthetic input
(`bb_rmsnorm_swiglu_ffn`, or `bb_layernorm_matmul` for c5) with every input
already resident in HBM.  Prints ONE JSON line.  The primary workload is the
prefill shape c3 (M=2048, D=4096, F=11008; TFLOP/s against the bf16 matrix-core
peak); the decode shape c2 (M=16; GB/s against the HBM peak) is measured in the
same run and reported in the "decode" object with its own roofline.  The fp64
oracle is timed on the host cores on a bounded sample ("cpu_baseline") and the
same sample gives the parity figure.  The unfused kernel sequence is timed
beside the fused one.
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

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this same script (profiles/hbm_traffic_c1_c2_c3_ffn.txt, attention: profiles/hbm_traffic_c2_c3_attention.txt;
# FETCH_SIZE scaled by 2.0, WRITE_SIZE by 1.0 as
# calibrated against bb_calib_copy).  Counters cannot be read from inside a timed run, so the
# figures are carried here (the line says so in "traffic_source"); workloads without a counter run report null.
TRAFFIC_SOURCE = ("carried from profiles/hbm_traffic_c1_c2_c3_ffn.txt and hbm_traffic_c2_c3_attention.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE "
                  "runs of this script, scaled by a copy of known size); not measured in this run")
MEASURED_TRAFFIC_BYTES = {
    ("c1", "ffn_nest"): 4.45e6 + 0.03e6,
    ("c2", "ffn_stream"): 280.4e6 + 16.2e6,
    ("c2", "ffn_stream_t"): 275.0e6 + 0.7e6,
    ("c3", "gemm_gateup"): 588.0e6 + 45.1e6,
    ("c3", "gemm_gateup_prescaled"): 587.6e6 + 45.1e6,
    ("attention", "attention"): 100.9e6 + 33.6e6,
    ("attention", "attention_decode"): 67.6e6 + 0.3e6,
}


def parity_block(y, ref, rows_checked):
    import bb_parity
    row, elem = bb_parity.errors(y, ref)
    return {"max_row_rel_err": row, "max_elem_err": elem, "rows_checked": rows_checked,
            "tolerance": bb_parity.TOL_ROW, "tolerance_elem": bb_parity.TOL_ELEM,
            "ok": bool(row <= bb_parity.TOL_ROW and elem <= bb_parity.TOL_ELEM)}


def roofline_block(kernel, bound, work, ms, traffic, step_work=None, step_ms=None):
    """roofline object of one kernel: `work` algorithmic flops (mfma) or bytes (hbm) per launch, `ms` its
    average launch duration; with step_work/step_ms also the whole step's fraction of the same peak"""
    if bound == "mfma":
        achieved, peak, unit, scale = work / (ms * 1e-3) / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s", 1e12
    else:
        achieved, peak, unit, scale = work / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s", 1e9
    r = {"kernel": kernel, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
         "traffic": traffic, "traffic_unit": "bytes per launch", "traffic_source": TRAFFIC_SOURCE if traffic else None,
         "algorithmic": work, "algorithmic_unit": "flop per launch" if bound == "mfma" else "bytes per launch",
         "kernel_ms": ms}
    if step_work is not None:
        a = step_work / (step_ms * 1e-3) / scale
        r["whole_step"] = {"achieved": a, "unit": unit, "frac": a / peak, "ms": step_ms,
                           "note": "all kernels of one step, launch gaps included: the figure the metric names"}
    return r


# The chip leaves its idle power state gradually: measured on c3 after 1 s without work, ten-step averages
# read 0.59, 0.57, 0.53, 0.51, 0.50, 0.49 ms and then stay at 0.486 ms, i.e. the first ~30 ms of any burst of
# work run up to 20 % slow.  Between two measurements of this script the GPU idles (inputs are generated on
# the CPU, the oracle is timed), and `--warmup 5` is 3 ms of work.  So every timed region is preceded by
# PRECONDITION_MS of a calibration kernel (not a step of the workload, nothing of it is cached or skipped) that
# brings the clocks to the state sustained work runs in: a matrix-instruction loop (bb_calib_mfma_data) before
# matrix-bound workloads, a streaming read of 1 GiB (bb_calib_read) before bandwidth-bound ones; then the W
# warm-up steps, then the K timed steps.
PRECONDITION_MS = 100.0
_precond = {}


def precondition(torch, bb, kind="mfma"):
    if not _precond:
        g = torch.Generator(device="cpu"); g.manual_seed(1)
        _precond["ops"] = torch.randn(16384, generator=g).to(torch.bfloat16).cuda()
        _precond["sink"] = torch.zeros(4096, dtype=torch.float32, device="cuda")
        _precond["buf"] = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        fns = {"mfma": lambda: bb.bb_calib_mfma_data(_precond["ops"], 1024, 500, _precond["sink"]),
               "hbm": lambda: bb.bb_calib_read(_precond["buf"], _precond["sink"])}
        _precond["fn"] = fns
        for k, fn in fns.items():
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn()
            torch.cuda.synchronize()
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            _precond["reps_" + k] = max(1, int(PRECONDITION_MS / max(e0.elapsed_time(e1), 1e-3)))
    for _ in range(_precond["reps_" + kind]):
        _precond["fn"][kind]()


def flops_of(cfg):
    return (6.0 if cfg.op == "ffn" else 2.0) * cfg.M * cfg.D * cfg.F


def bytes_of(cfg):
    if cfg.op == "ffn":
        return 2.0 * (3 * cfg.D * cfg.F + 2 * cfg.M * cfg.D + cfg.D)
    return 2.0 * (cfg.M * cfg.D + cfg.D * cfg.F + cfg.M * cfg.F + 2 * cfg.D)


def dominant_kernel(cfg, variant_stream):
    """name in the library's per-kernel profile, algorithmic work of one launch, bound"""
    if cfg.op == "ln":
        return "gemm_ln", 2.0 * cfg.M * cfg.D * cfg.F, "mfma"
    if variant_stream:
        return "ffn_stream", bytes_of(cfg), "hbm"
    return "gemm_gateup", 4.0 * cfg.M * cfg.D * cfg.F, "mfma"


def run_workload(name, steps, warmup, with_cpu, torch, bb, bb_inputs, orc, np, cpu_seconds=15.0):
    cfg = bb_inputs.CONFIGS[name]
    cpu = bb_inputs.make_config(name)
    stream_variant = cfg.op == "ffn" and cfg.M <= 16
    # decode: rotate weight sets so that the 256 MB memory-side cache cannot hold them
    nsets = 3 if stream_variant else 1
    dev_sets = []
    for s in range(nsets):
        src = cpu if s == 0 else bb_inputs.make_config(name, seed=s)
        d = [t.cuda() for t in src]
        if s > 0:                      # same activations, different weights
            d[0], d[1] = dev_sets[0][0], dev_sets[0][1]
        dev_sets.append(d)
    out = torch.empty((cfg.M, cfg.D if cfg.op == "ffn" else cfg.F), dtype=torch.bfloat16, device="cuda")

    def step(i, unfused=False):
        d = dev_sets[i % nsets]
        if cfg.op == "ffn":
            bb.bb_rmsnorm_swiglu_ffn(*d, cfg.eps, Y=out, unfused=unfused)
        else:
            bb.bb_layernorm_matmul(*d, cfg.eps, Y=out, unfused=unfused)

    pkind = "hbm" if stream_variant else "mfma"

    def timed(unfused=False):
        precondition(torch, bb, pkind)
        for i in range(warmup):
            step(i, unfused)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            step(i, unfused)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return max(wall, e0.elapsed_time(e1)) / steps, e0.elapsed_time(e1) / steps

    ms_step, ms_step_events = timed(False)
    # result of the fused path on weight set 0, kept for the parity figure
    step(0, False)
    torch.cuda.synchronize()
    y_fused = out.clone()

    # per-kernel durations: HIP events recorded by the library on the launch stream around every kernel of
    # `steps` back-to-back calls (at most 64 are kept), read after the run
    precondition(torch, bb, pkind)
    bb.bb_profile_enable(True)
    per = {}
    for i in range(min(steps, 64)):
        step(i, False)
    for call in bb.bb_profile_history():
        for kname, ms in call:
            per.setdefault(kname, []).append(ms)
    bb.bb_profile_enable(False)
    kernels_ms = {k: float(np.mean(v)) for k, v in per.items()}

    ms_unfused, _ = timed(True)
    # the program with the statistics inside the product loop (nothing but the hidden materialised)
    ms_snapshot1 = None
    if not stream_variant:
        bb.bb_set_variant(bb.VARIANT_SNAPSHOT1)
        try:
            ms_snapshot1, _ = timed(False)
        finally:
            bb.bb_set_variant(bb.VARIANT_AUTO)

    # the last snapshot (fully fused nest, one block of output columns: ONE launch, the hidden never leaves the
    # compute unit) where the model dimension allows it; its output is kept for a parity figure of its own
    nest = None
    if cfg.op == "ffn" and cfg.D <= 512:
        bb.bb_set_variant(bb.VARIANT_NEST)
        try:
            ms_nest, _ = timed(False)
            bb.bb_profile_enable(True)
            step(0, False)
            launches = [k for k, _ in bb.bb_profile_last()]
            bb.bb_profile_enable(False)
            torch.cuda.synchronize()
            nest = {"ms_per_step": ms_nest, "launches": launches, "y": out.clone()}
        finally:
            bb.bb_set_variant(bb.VARIANT_AUTO)

    # the same operator through the transposed-weight entry points (W^T layouts), timed the same way
    ms_transposed = None
    if not stream_variant:
        d0 = dev_sets[0]
        if cfg.op == "ffn":
            dt = [d0[0], d0[1]] + [w.t().contiguous() for w in d0[2:]]
            stept = lambda: bb.bb_rmsnorm_swiglu_ffn_t(*dt, cfg.eps, Y=out)
        else:
            dt = [d0[0], d0[1], d0[2], d0[3].t().contiguous()]
            stept = lambda: bb.bb_layernorm_matmul_t(*dt, cfg.eps, Y=out)
        precondition(torch, bb)
        for _ in range(warmup):
            stept()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            stept()
        e1.record()
        torch.cuda.synchronize()
        ms_transposed = e0.elapsed_time(e1) / steps
        del dt

    # decode: the same operator on transposed weights (W1^T, W3^T [F,D], W2^T [D,F]) runs the streaming
    # kernel of that layout; timed like the primary, on rotating transposed weight sets
    t_stream = None
    if stream_variant:
        tsets = [[d[0], d[1]] + [w.t().contiguous() for w in d[2:]] for d in dev_sets]
        def stept(i):
            bb.bb_rmsnorm_swiglu_ffn_t(*tsets[i % nsets], cfg.eps, Y=out)
        precondition(torch, bb, pkind)
        for i in range(warmup):
            stept(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            stept(i)
        e1.record()
        torch.cuda.synchronize()
        ms_t = e0.elapsed_time(e1) / steps
        bb.bb_profile_enable(True)
        for i in range(min(steps, 64)):
            stept(i)
        kt = [ms for call in bb.bb_profile_history() for kname, ms in call if kname == "ffn_stream_t"]
        bb.bb_profile_enable(False)
        stept(0)
        torch.cuda.synchronize()
        y_t = out.clone()
        k_ms = float(np.mean(kt)) if kt else None
        t_stream = {"ms_per_step": ms_t, "gbs": bytes_of(cfg) / (ms_t * 1e-3) / 1e9, "kernel_ms": k_ms, "y": y_t}
        del tsets

    # the FFN with the decoder block's residual connection fused into the last kernel's epilogue
    ms_residual = None
    if cfg.op == "ffn":
        def stepr(i):
            d = dev_sets[i % nsets]
            bb.bb_rmsnorm_swiglu_ffn_residual(*d, d[0], cfg.eps, Y=out)
        precondition(torch, bb, pkind)
        for i in range(warmup):
            stepr(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            stepr(i)
        e1.record()
        torch.cuda.synchronize()
        ms_residual = e0.elapsed_time(e1) / steps

    dom, work, bound = dominant_kernel(cfg, stream_variant)
    if dom + "_prescaled" in kernels_ms:
        dom = dom + "_prescaled"             # AUTO ran the statistics loop as a kernel of its own
    if dom not in kernels_ms:                # (a program of one launch reports under its own name)
        dom = max(kernels_ms, key=kernels_ms.get)
    # A step of ONE kernel: its average launch duration is the step time of the back-to-back timed region
    # (HIP events on the launch stream); the per-call events above bracket a launch that starts on an idle
    # chip and read longer than that.
    dom_ms = ms_step_events if len(kernels_ms) == 1 else kernels_ms[dom]
    res = {
        "workload": name, "op": cfg.op, "M": cfg.M, "D": cfg.D, "F_or_N": cfg.F,
        "variant": "stream" if stream_variant else "nest" if dom == "ffn_nest" else (
            "prescale" if dom.endswith("_prescaled") else "snapshot1"),
        "ms_per_step": ms_step, "ms_per_step_events": ms_step_events,
        "tflops": flops_of(cfg) / (ms_step * 1e-3) / 1e12,
        "gbs": bytes_of(cfg) / (ms_step * 1e-3) / 1e9,
        "kernels_ms": kernels_ms,
        "unfused_ms_per_step": ms_unfused,
        "snapshot1_ms_per_step": ms_snapshot1,
        "fully_fused_nest": nest,
        "transposed_weights_ms_per_step": ms_transposed,
        "residual_ms_per_step": ms_residual,
        "roofline": roofline_block(dom, bound, work, dom_ms, MEASURED_TRAFFIC_BYTES.get((name, dom)),
                                   flops_of(cfg) if bound == "mfma" else bytes_of(cfg), ms_step_events),
    }

    if with_cpu:
        # bounded oracle sample: first a few rows to size the sample, then ~15 s of work
        rows_all = list(range(cfg.M))
        probe = rows_all[:: max(1, cfg.M // 16)][:16]
        t0 = time.perf_counter()
        _oracle(orc, cfg, cpu, probe)
        per_row = (time.perf_counter() - t0) / len(probe)
        n = int(min(cfg.M, max(16, cpu_seconds / max(per_row, 1e-9))))
        rng = np.random.default_rng(0)
        edges = {r for t0 in range(0, cfg.M, 128) for r in (t0, min(cfg.M, t0 + 128) - 1)}   # every row tile's edges
        rows = sorted(set(rng.choice(cfg.M, size=n, replace=False).tolist()) | edges)
        reps, t_total, ref = 0, 0.0, None
        while t_total < cpu_seconds * 2 / 3 and reps < 64:       # small configs: repeat to reach the sample time
            t0 = time.perf_counter()
            ref = _oracle(orc, cfg, cpu, rows)
            t_total += time.perf_counter() - t0
            reps += 1
        sec_per_row = t_total / (reps * len(rows))
        row_work = flops_of(cfg) / cfg.M
        res["parity"] = parity_block(y_fused[rows], ref, len(rows))
        if t_stream is not None:
            t_stream["parity"] = parity_block(t_stream["y"][rows], ref, len(rows))
        if nest is not None:
            nest["parity"] = parity_block(nest["y"][rows], ref, len(rows))
        cpu_tflops = row_work / sec_per_row / 1e12
        res["cpu_baseline"] = {
            "value": cpu_tflops if bound == "mfma" else bytes_of(cfg) / (sec_per_row * cfg.M) / 1e9,
            "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
            "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{len(rows)} of {cfg.M} rows of {name}, all output columns, x{reps} repeats, "
                      f"{t_total:.1f} s; whole-workload time extrapolated as seconds_per_row * M",
            "seconds_full_workload_extrapolated": sec_per_row * cfg.M,
        }
    if nest is not None:
        nest.pop("y")
    if t_stream is not None:
        t_stream.pop("y")
        k_ms = t_stream.pop("kernel_ms")
        if k_ms:
            t_stream["kernels_ms"] = {"ffn_stream_t": k_ms}
            t_stream["roofline"] = roofline_block("ffn_stream_t", "hbm", bytes_of(cfg), t_stream["ms_per_step"],
                                                  MEASURED_TRAFFIC_BYTES.get((name, "ffn_stream_t")))
        res["transposed_weights"] = t_stream
    del dev_sets
    torch.cuda.empty_cache()
    return res


ATTN_WORKLOAD = dict(B=32, M=4096, N=4096, d=128, dv=128)   # 32 heads, 4096 x 4096, head dimension 128


def run_attention(steps, warmup, with_cpu, torch, bb, bb_inputs, orc, np):
    """bb_attention on ATTN_WORKLOAD (synthetic N(0,1) Q, K, V): time per call from
    HIP events on the launch stream, roofline against the bf16 matrix peak with
    4 B M N d useful flops, and parity on sampled query rows against the oracle."""
    w = ATTN_WORKLOAD
    cpu = bb_inputs.make_attn(w["B"], w["M"], w["N"], w["d"], w["dv"], seed=0)
    Q, K, V = [t.cuda() for t in cpu]
    O = torch.empty((w["B"], w["M"], w["dv"]), dtype=torch.bfloat16, device="cuda")
    precondition(torch, bb)
    for _ in range(warmup):
        bb.bb_attention(Q, K, V, O)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        bb.bb_attention(Q, K, V, O)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    bb.bb_profile_enable(True)
    for _ in range(min(steps, 64)):
        bb.bb_attention(Q, K, V, O)
    per = [dict(call)["attention"] for call in bb.bb_profile_history()]
    bb.bb_profile_enable(False)
    k_ms = float(np.mean(per))
    flops = 2.0 * w["B"] * w["M"] * w["N"] * (w["d"] + w["dv"])
    res = {
        "workload": "attention B=%(B)d M=%(M)d N=%(N)d d=%(d)d dv=%(dv)d" % w, "op": "attention",
        "ms_per_step": ms, "tflops": flops / (ms * 1e-3) / 1e12, "kernels_ms": {"attention": k_ms},
        "roofline": roofline_block("attention", "mfma", flops, k_ms, MEASURED_TRAFFIC_BYTES.get(("attention", "attention"))),
    }
    if with_cpu:
        rng = np.random.default_rng(0)
        rows = sorted(set(int(r) for r in rng.integers(0, w["B"] * w["M"], size=65536)))
        t0 = time.perf_counter()
        ref = orc.attention(*cpu, rows=rows)
        sec = time.perf_counter() - t0
        res["parity"] = parity_block(O.reshape(-1, w["dv"])[rows], ref, len(rows))
        row_flops = flops / (w["B"] * w["M"])
        res["cpu_baseline"] = {"value": row_flops * len(rows) / sec / 1e12, "unit": "TFLOP/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"{len(rows)} of {w['B'] * w['M']} query rows, {sec:.2f} s"}
    del Q, K, V, O
    # few queries (decoding): one query per head against the same keys, keys split over workgroups;
    # bandwidth-bound: K and V are read once
    wd = dict(w, M=1)
    cpu_d = bb_inputs.make_attn(wd["B"], 1, wd["N"], wd["d"], wd["dv"], seed=1)
    Qd, Kd, Vd = [t.cuda() for t in cpu_d]
    Od = torch.empty((wd["B"], 1, wd["dv"]), dtype=torch.bfloat16, device="cuda")
    precondition(torch, bb, "hbm")
    for _ in range(warmup):
        bb.bb_attention(Qd, Kd, Vd, Od)
    torch.cuda.synchronize()
    # one kernel per call: its average launch duration is the time per call of back-to-back launches
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        bb.bb_attention(Qd, Kd, Vd, Od)
    e1.record()
    torch.cuda.synchronize()
    d_ms = e0.elapsed_time(e1) / steps
    d_bytes = 2.0 * wd["B"] * (wd["N"] * (wd["d"] + wd["dv"]) + wd["d"] + wd["dv"])
    refd = orc.attention(*cpu_d)
    res["decode"] = {
        "workload": "attention B=%(B)d M=1 N=%(N)d d=%(d)d dv=%(dv)d (one-query streaming kernel: keys split over workgroups, added by the last to finish)" % wd,
        "kernels_ms": {"attention": d_ms},
        "roofline": roofline_block("attention_decode_kernel", "hbm", d_bytes, d_ms,
                                   MEASURED_TRAFFIC_BYTES.get(("attention", "attention_decode"))),
        "parity": parity_block(Od.reshape(-1, wd["dv"]), refd, wd["B"]),
    }
    del Qd, Kd, Vd, Od
    torch.cuda.empty_cache()
    return res


def run_selection(torch, bb, bb_inputs):
    """Measured selection between the candidate programs (bb_*_tune) over the row counts between
    decode and prefill for the Llama-shaped FFN, and for the c5 LN->matmul shape."""
    names = {bb.VARIANT_STREAM: "stream", bb.VARIANT_SNAPSHOT1: "snapshot1", bb.VARIANT_UNFUSED: "unfused",
             bb.VARIANT_PRESCALE: "prescale"}
    out = []
    full = [t.cuda() for t in bb_inputs.make_ffn(2048, 4096, 11008, seed=0)]
    for M in (8, 16, 32, 64, 128, 256, 512, 1024, 2048):
        X = full[0][:M].contiguous()
        chosen, ms = bb.bb_rmsnorm_swiglu_ffn_tune(X, *full[1:], 1e-5, reps=10)
        out.append({"op": "ffn", "M": M, "D": 4096, "F": 11008, "chosen": names[chosen],
                    "ms": {names[v]: t for v, t in ms.items()}})
    del full
    c5 = bb_inputs.CONFIGS["c5"]
    ln = [t.cuda() for t in bb_inputs.make_config("c5")]
    chosen, ms = bb.bb_layernorm_matmul_tune(*ln, c5.eps, reps=10)
    out.append({"op": "ln", "M": c5.M, "D": c5.D, "N": c5.F, "chosen": names[chosen],
                "ms": {names[v]: t for v, t in ms.items()}})
    del ln
    bb.bb_tune_clear()
    torch.cuda.empty_cache()
    return out


def _oracle(orc, cfg, cpu, rows):
    if cfg.op == "ffn":
        return orc.rmsnorm_swiglu_ffn(*cpu, cfg.eps, rows=rows)
    return orc.layernorm_matmul(*cpu, cfg.eps, rows=rows)


def calibrate(torch, bb):
    """measured streaming-read and matrix-core peaks (context for the spec-sheet denominators)"""
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
    def t(fn, n):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    ms_r = t(lambda: bb.bb_calib_read(buf, sink), 10)
    half = buf.numel() // 2          # plain copy of known size: the reference for HBM byte counters
    ms_c = t(lambda: bb.bb_calib_copy(buf[:half], buf[half:]), 5)
    iters, wgs = 4000, 1024
    ms_m = t(lambda: bb.bb_calib_mfma(wgs, iters, sink), 3)
    # the same matrix-instruction stream on random N(0,1) operands: the clock the chip sustains
    # depends on the operand data, so this is the rate attainable on real data
    g = torch.Generator(device="cpu"); g.manual_seed(1)
    ops = torch.randn(16384, generator=g).to(torch.bfloat16).cuda()
    ms_d = t(lambda: bb.bb_calib_mfma_data(ops, wgs, iters, sink), 3)
    return {"mfma_bf16_tflops_random_operands": wgs * 4 * iters * 16 * 32768.0 / (ms_d * 1e-3) / 1e12,
            "read_gbs": buf.numel() / (ms_r * 1e-3) / 1e9,
            "copy_gbs_read_plus_write": 2 * half / (ms_c * 1e-3) / 1e9,
            "mfma_bf16_tflops": wgs * 4 * iters * 16 * 32768.0 / (ms_m * 1e-3) / 1e12}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed steps first; the chip needs ~50 ms of work to reach its sustained clocks "
                         "(the first 50 steps after 10 warm-up steps run ~7 %% slower)")
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--also", default="c2,c1,c4,c5", help="comma list of further workloads reported in 'others' "
                    "(the decode shape c2 is reported as 'decode')")
    ap.add_argument("--no-attention", action="store_true", help="skip the attention workload")
    ap.add_argument("--no-selection", action="store_true", help="skip the measured-selection table")
    ap.add_argument("--attention-only", action="store_true",
                    help="time only the attention workload and print its block as the line (for profiler runs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing / parity sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import bb_inputs
    import paper_2505_07829_amd as bb
    from oracle import oracle as orc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    bb.load()          # fails loudly if the HIP library has not been built

    if args.attention_only:
        attn = run_attention(args.steps, args.warmup, not args.no_cpu, torch, bb, bb_inputs, orc, np)
        bb.bb_shutdown()
        print(json.dumps({"metric": "attention TFLOP/s", "value": attn["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": attn["ms_per_step"],
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
                          "data": "synthetic", "config": {"workload": attn["workload"]},
                          "roofline": attn["roofline"], "cpu_baseline": attn.get("cpu_baseline"),
                          "parity": attn.get("parity"), "decode": attn.get("decode")}))
        return
    # Measured peaks first: context for the spec-sheet denominators, and about 0.2 s of matrix and memory work
    # that takes the chip from idle to the clocks it sustains (it needs ~50 ms of work for that) before
    # anything is timed.
    peaks = calibrate(torch, bb)
    primary = run_workload(args.workload, args.steps, args.warmup, not args.no_cpu, torch, bb, bb_inputs, orc, np)
    others = {}
    for name in [w for w in args.also.split(",") if w and w != args.workload]:
        # (the large configurations take milliseconds per step: fewer steps keep the default run short)
        big = bb_inputs.CONFIGS[name].M >= 4096
        others[name] = run_workload(name, min(args.steps, 20) if big else args.steps,
                                    min(args.warmup, 10) if big else args.warmup, not args.no_cpu, torch, bb,
                                    bb_inputs, orc, np, cpu_seconds=6.0)
    attn = None if args.no_attention else run_attention(args.steps, args.warmup, not args.no_cpu, torch, bb,
                                                        bb_inputs, orc, np)
    selection = None if args.no_selection else run_selection(torch, bb, bb_inputs)
    bb.bb_shutdown()

    mfma_bound = primary["roofline"]["bound"] == "mfma"
    line = {
        "metric": "fused RMSNorm+SwiGLU FFN TFLOP/s (% bf16 MFMA peak); decode HBM GB/s",
        "value": primary["tflops"] if mfma_bound else primary["gbs"],
        "unit": "TFLOP/s" if mfma_bound else "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": primary["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "precondition": f"{PRECONDITION_MS:.0f} ms of a calibration kernel (bb_calib_mfma_data; bb_calib_read before "
                        "bandwidth-bound workloads) before the warm-up steps of every timed region (the chip leaves "
                        "its idle power state over the first ~30 ms of work)",
        "config": {"workload": f"{args.workload}: {primary['op']} M={primary['M']} D={primary['D']} "
                               f"F_or_N={primary['F_or_N']} ({primary['variant']})"},
        "roofline": primary["roofline"],
        "cpu_baseline": primary.get("cpu_baseline"),
        "parity": primary.get("parity"),
        "kernels_ms": primary["kernels_ms"],
        "unfused_ms_per_step": primary["unfused_ms_per_step"],
        "snapshot1_ms_per_step": primary["snapshot1_ms_per_step"],
        "fully_fused_nest": primary.get("fully_fused_nest"),
        "transposed_weights_ms_per_step": primary["transposed_weights_ms_per_step"],
        "residual_ms_per_step": primary["residual_ms_per_step"],
        "measured_peaks": peaks,
    }
    if "c2" in others:
        d = others.pop("c2")
        line["decode"] = {
            "workload": "c2: ffn M=16 D=4096 F=11008 (stream), 3 rotating weight sets",
            "value": d["gbs"], "unit": "GB/s", "ms_per_step": d["ms_per_step"],
            "roofline": d["roofline"], "cpu_baseline": d.get("cpu_baseline"), "parity": d.get("parity"),
            "kernels_ms": d["kernels_ms"], "unfused_ms_per_step": d["unfused_ms_per_step"],
            "residual_ms_per_step": d["residual_ms_per_step"],
            "transposed_weights": d.get("transposed_weights"),
        }
    if attn is not None:
        line["attention"] = attn
    if selection is not None:
        line["selection"] = selection
    if others:
        line["others"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
