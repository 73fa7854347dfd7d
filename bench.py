#!/usr/bin/env python3
"""Benchmark of the Streamlined-Inference hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
GroupNorm statistics, every slice of the sliced block forward (slice-in,
proj_in, LN+QKV, attention, out-proj, GEGLU FFN, proj_out + residual into the
preallocated output) and the Step Rehash similarity test of the new output
against a cached one.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: whole-step throughput in algorithmic TFLOP/s, the
roofline record of the dominant kernel (per-launch duration from HIP events
recorded by the library around each launch), and the CPU oracle timed on a
bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
PEAK_F32_VALU_TFLOPS = 157.3


def stage_work(spec, stage, M, window_tokens_per_seq=None):
    """Algorithmic work of one launch of `stage` on a window of M tokens.

    Returns (kind, amount): kind "flop" for contractions (2mnk; attention
    4*Nq*Nk*d per head), "byte" for HBM-bound stages."""
    import si_workloads as wl
    C, D = spec.C, spec.D
    es = 4 if spec.dtype == "f32" else 2
    P = spec.H * spec.W
    gemm = {
        "proj_in": 2.0 * M * C * D, "qkv": 2.0 * M * D * 3 * D, "attn_out": 2.0 * M * D * D,
        "q2": 2.0 * M * D * D, "cross_out": 2.0 * M * D * D,
        "ff1_geglu": 2.0 * M * D * 8 * D, "ff2": 2.0 * M * 4 * D * D, "proj_out": 2.0 * M * D * C,
        "ctx_kv": 2.0 * spec.B * spec.ctx_tokens * spec.ctx_dim * 2 * D,
    }
    if stage in gemm:
        return "flop", gemm[stage]
    if stage == "self_attn":
        nk = spec.F if spec.kind == wl.TEMPORAL else P
        return "flop", 4.0 * M * nk * D
    if stage == "cross_attn":
        return "flop", 4.0 * M * spec.ctx_tokens * D
    if stage == "attn_half_fused":      # proj_in, q/k/v, attention over F frames
        return "flop", 2.0 * M * (C * D + 3 * D * D) + 4.0 * M * spec.F * D
    if stage == "ffn_half_fused":       # attention out-projection, W1, W2, proj_out
        return "flop", 2.0 * M * (D * D + 8 * D * D + 4 * D * D + D * C)
    if stage == "pre_attn_fused":       # proj_in and the q / k / v projections
        return "flop", 2.0 * M * (C * D + 3 * D * D)
    if stage == "post_attn_fused":      # self-attention out-projection, query projection, context attention and
        # its out-projection, W1, W2, proj_out
        return "flop", 2.0 * M * (3 * D * D + 8 * D * D + 4 * D * D + D * C) + 4.0 * M * spec.ctx_tokens * D
    if stage == "temporal_block_fused":  # the whole operator group of a window in one kernel
        return "flop", 2.0 * M * (C * D + 3 * D * D + D * D + 8 * D * D + 4 * D * D + D * C) + 4.0 * M * spec.F * D
    if stage == "gn_stats":
        return "byte", float(spec.tokens * C * es)
    if stage == "gn_stats_cosine":      # statistics pass that also reduces x against the rehash anchor
        return "byte", 2.0 * spec.tokens * C * es
    if stage == "cache_handback":       # device copy of the cached output
        return "byte", 2.0 * spec.tokens * C * es
    if stage == "cache_update":         # device copies of x and out into the anchor
        return "byte", 4.0 * spec.tokens * C * es
    if stage == "slice_in":
        return "byte", 2.0 * M * C * es
    if stage in ("ln1", "ln2", "ln3"):
        return "byte", M * D * (4.0 + es)
    if stage == "cosine_partial":
        return "byte", 2.0 * spec.tokens * C * es
    return "none", 0.0


def _blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([i.get("num_threads", 1) for i in threadpool_info()] or [1]))
    except Exception:
        return len(os.sched_getaffinity(0))


def _oracle_sample(spec, max_positions=1152):
    """A bounded sample of a block workload for the oracle: positions of a temporal block (all
    frames; GroupNorm over the sample), one frame of a spatial block."""
    import si_workloads as wl
    if spec.kind == wl.TEMPORAL:
        npos = min(spec.H * spec.W, max_positions)
        return wl.scaled(spec, H=1, W=npos), f"{spec.name}: {npos} of {spec.H * spec.W} positions (all {spec.F} frames, B={spec.B})"
    return wl.scaled(spec, F=1), f"{spec.name}: 1 of {spec.F} frames (B={spec.B})"


def _time_oracle(sub):
    import oracle
    import si_workloads as wl
    x, w, ctx = wl.make_x(sub), wl.make_weights(sub), wl.make_context(sub)
    t0 = time.perf_counter()
    oracle.block_forward_ref(x, w, sub, ctx)
    return time.perf_counter() - t0


def cpu_baseline(specs):
    """The fp64 NumPy oracle, as it stands, timed on this host: a bounded sample of the headline
    workload (the reported baseline), the whole cfg2 tensor, and single-thread figures."""
    import si_workloads as wl
    threads = _blas_threads()
    flop, secs, what = 0.0, 0.0, []
    for spec in specs:
        sub, desc = _oracle_sample(spec)
        secs += _time_oracle(sub)
        flop += sub.flops()
        what.append(desc)
    rec = {"value": flop / secs / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
           "sample": "; ".join(what) + f"; fp64 NumPy, one pass each, {secs:.1f} s",
           "host_cpus": len(os.sched_getaffinity(0))}
    cfg2 = wl.CONFIGS["cfg2"]
    dt = _time_oracle(cfg2)
    rec["cfg2_whole_tensor"] = {"value": cfg2.flops() / dt / 1e12, "unit": "TFLOP/s", "seconds": round(dt, 2), "cores": threads}
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            single = {}
            for name, sub in (("cfg1", wl.CONFIGS["cfg1"]), ("cfg2", wl.scaled(cfg2, H=1, W=96))):
                dt = _time_oracle(sub)
                single[name] = {"value": sub.flops() / dt / 1e12, "unit": "TFLOP/s", "seconds": round(dt, 2),
                                "sample": "whole tensor" if name == "cfg1" else "96 of 4096 positions"}
        rec["single_thread"] = single
    except Exception as e:                                   # threadpoolctl missing: no single-thread figure
        rec["single_thread"] = {"error": repr(e)}
    return rec


def res_stage_work(spec, stage, M):
    """Algorithmic work of one launch of a ResBlock stage on a window of M tokens."""
    C, Co = spec.C, spec.C_out or spec.C
    if stage == "conv1":
        return "flop", 2.0 * M * 9 * C * Co
    if stage == "conv2":
        return "flop", 2.0 * M * 9 * Co * Co
    if stage == "conv_skip":
        return "flop", 2.0 * M * C * Co
    if stage == "gn_stats":
        return "byte", float(spec.tokens * C * 2)
    if stage in ("slice_in", "slice_in_raw"):
        return "byte", 2.0 * M * C * 2
    C = Co                              # the stages after conv1 work on the output width
    if stage == "gn2_stats":            # one read of the fp16 intermediate
        return "byte", 2.0 * M * C
    if stage == "gn2_silu":             # fp16 in, fp16 out
        return "byte", 4.0 * M * C
    return "none", 0.0


def main_resblock(args):
    """Spatial ResBlock operator group sliced along frames (the second spatial group workload)."""
    import numpy as np
    import torch
    import paper_2411_01171_amd as si
    import si_workloads as wl
    from paper_2411_01171_amd.devio import device_res_weights, to_dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    spec = wl.RES_CONFIGS[args.workload]
    slice_len = args.slice_len or spec.slice_len
    x_np = wl.make_x(spec)
    x = to_dev(x_np, spec.dtype)
    temb_np = wl.make_temb(spec)
    temb = None if temb_np is None else to_dev(temb_np, spec.dtype)
    w_np = wl.make_res_weights(spec)
    wts = device_res_weights(spec, w_np)
    ws_bytes = si.si_resblock_workspace_bytes(x, wts, slice_len)
    live_sliced = si.si_resblock_live_activation_bytes(x, wts, slice_len)
    live_unsliced = si.si_resblock_live_activation_bytes(x, wts, spec.F)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    out = torch.empty((spec.B, spec.C_out or spec.C, spec.F, spec.H, spec.W), dtype=x.dtype, device="cuda")

    def step():
        si.si_resblock_forward(x, wts, temb, out, slice_len, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    flops = spec.flops()
    value = flops / (ms_per_step * 1e-3) / 1e12

    si.si_stage_timing_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    stages = si.si_stage_timing_read()
    si.si_stage_timing_enable(False)
    n_slices = -(-spec.F // slice_len)
    M_slice = spec.B * min(slice_len, spec.F) * spec.H * spec.W
    stage_report = {}
    for name, (ms, cnt) in stages.items():
        avg_ms = ms / cnt
        kind, work = res_stage_work(spec, name, M_slice)
        rec = {"avg_us": round(avg_ms * 1e3, 2), "launches_per_step": cnt / args.steps, "ms_per_step": round(ms / args.steps, 4)}
        if kind == "flop":
            rec["TFLOP/s"] = round(work / (avg_ms * 1e-3) / 1e12, 2)
        elif kind == "byte":
            rec["GB/s"] = round(work / (avg_ms * 1e-3) / 1e9, 1)
        stage_report[name] = rec
    conv_ms = stages["conv1"][0] + stages["conv2"][0]
    conv_cnt = stages["conv1"][1] + stages["conv2"][1]
    d_work = 0.5 * (res_stage_work(spec, "conv1", M_slice)[1] + res_stage_work(spec, "conv2", M_slice)[1])
    ach = d_work / (conv_ms / conv_cnt * 1e-3) / 1e12
    roof = {"bound": "mfma", "kernel": "conv3x3 (conv1 + conv2 launches)", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
            "avg_launch_us": conv_ms / conv_cnt * 1e3, "algorithmic_flop_per_launch": d_work}
    result = {
        "metric": "sliced block-forward TFLOP/s (% MFMA peak) + peak live activation bytes vs unsliced",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 operands from bf16 storage, f32 accumulation", "data": "synthetic",
        "config": {"workload": f"{args.workload}: Spatial ResBlock group x[B={spec.B},C={spec.C}->{spec.C_out or spec.C},F={spec.F},H={spec.H},W={spec.W}], "
                               f"embedding width {spec.temb_dim}, sliced along frames in windows of {slice_len} ({n_slices} slices)",
                   "algorithmic_flop_per_step": flops, "tokens": spec.tokens},
        "frac_mfma_peak": value / PEAK_BF16_TFLOPS,
        "live_activation_bytes": {"sliced": live_sliced, "unsliced_same_kernels": live_unsliced,
                                  "ratio": live_sliced / live_unsliced, "workspace_bytes": ws_bytes,
                                  "x_bytes": x.numel() * x.element_size()},
        "roofline": roof,
        "stages": stage_report,
    }
    if not args.no_cpu_baseline:
        import oracle
        sub = wl.scaled(spec, F=1)
        xs = x_np[:, :, :1]
        t0 = time.perf_counter()
        oracle.resblock_forward_ref(xs, w_np, sub, temb_np)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            threads = len(os.sched_getaffinity(0))
        result["cpu_baseline"] = {"value": sub.flops() / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
                                  "sample": f"1 of {spec.F} frames (B={spec.B}); fp64 NumPy; 1 pass in {dt:.1f} s"}
    print(json.dumps(result))


def main_resample(args):
    """Spatial Down/UpSample of the ResBlock group on the ResBlock workloads' features (down4, up4b)."""
    import numpy as np
    import torch
    import paper_2411_01171_amd as si
    import si_workloads as wl
    from paper_2411_01171_amd.devio import to_dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    kind = "down" if args.workload.startswith("down") else "up"
    spec = wl.RES_CONFIGS["res4" if kind == "down" else "res4b"]
    slice_len = args.slice_len or spec.slice_len
    x_np = wl.make_x(spec)
    x = to_dev(x_np, "bf16")
    rng = np.random.default_rng(spec.seed + 50)
    w_np = wl.round_to_storage(0.02 * rng.standard_normal((spec.C, spec.C, 3, 3), dtype=np.float32), "bf16")
    w = to_dev(w_np, "bf16")
    k = si.SI_RESAMPLE_DOWN if kind == "down" else si.SI_RESAMPLE_UP
    Ho, Wo = ((spec.H + 1) // 2, (spec.W + 1) // 2) if kind == "down" else (2 * spec.H, 2 * spec.W)
    out = torch.empty((spec.B, spec.C, spec.F, Ho, Wo), dtype=torch.bfloat16, device="cuda")
    ws_bytes = si.si_resample_workspace_bytes(x, k, slice_len)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def step():
        si.si_resample_forward(x, k, w, None, out, slice_len, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    M_out = spec.B * spec.F * Ho * Wo
    flops = 2.0 * M_out * 9 * spec.C * spec.C
    si.si_stage_timing_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    stages = si.si_stage_timing_read()
    si.si_stage_timing_enable(False)
    conv = "conv_down" if kind == "down" else "conv_up"
    n_slices = -(-spec.F // slice_len)
    w_flops = 2.0 * (M_out // spec.F) * min(slice_len, spec.F) * 9 * spec.C * spec.C
    stage_report = {n: {"avg_us": round(ms / c * 1e3, 2), "launches_per_step": c / args.steps, "ms_per_step": round(ms / args.steps, 4)}
                    for n, (ms, c) in stages.items()}
    c_ms, c_cnt = stages[conv]
    ach = w_flops / (c_ms / c_cnt * 1e-3) / 1e12
    stage_report[conv]["TFLOP/s"] = round(ach, 2)
    value = flops / (ms_per_step * 1e-3) / 1e12
    print(json.dumps({
        "metric": "sliced block-forward TFLOP/s (% MFMA peak) + peak live activation bytes vs unsliced",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: Spatial {kind}-sample (3x3 convolution) of x[B={spec.B},C={spec.C},F={spec.F},H={spec.H},"
                               f"W={spec.W}] -> {Ho}x{Wo}, sliced along frames in windows of {slice_len} ({n_slices} slices)",
                   "algorithmic_flop_per_step": flops},
        "frac_mfma_peak": value / PEAK_BF16_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": conv, "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / PEAK_BF16_TFLOPS, "traffic": None, "avg_launch_us": c_ms / c_cnt * 1e3,
                     "algorithmic_flop_per_launch": w_flops},
        "stages": stage_report}))


def source_hash():
    """Hash of the kernel sources the library is built from; a counter summary under profiles/ is
    tied to the build it was measured on through this value."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2411_01171_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def traffic_record(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter runs summarised under profiles/
    (separate runs of this command; never measured inside this process).  Returned only when the
    summary was taken on this very build of the kernels; else None and the reason."""
    tpath = os.path.join(ROOT, "profiles", "traffic_per_launch.txt")
    try:
        doc = json.load(open(tpath))
    except Exception:
        return None, "no counter summary under profiles/"
    rec = doc.get(workload, {}).get(kernel)
    if not rec:
        return None, f"no counter run of {kernel} at {workload} under profiles/"
    if doc.get("_source_hash") != source_hash():
        return None, (f"profiles/traffic_per_launch.txt was measured on kernel sources {doc.get('_source_hash')}, "
                      f"this build is {source_hash()}: stale, not reported")
    return rec, f"separate rocprofv3 --pmc runs, {rec.get('source', tpath)}"


class BlockRun:
    """Device tensors of one block workload and its launch configuration."""

    def __init__(self, spec, slice_len=None, x=None):
        import torch
        import paper_2411_01171_amd as si
        import si_workloads as wl
        from paper_2411_01171_amd.devio import AXIS, device_weights, to_dev
        self.spec = spec
        self.slice_len = slice_len or spec.slice_len
        self.axis = AXIS[spec.slice_axis]
        self.extent = spec.F if spec.slice_axis == wl.AXIS_F else spec.H * spec.W
        self.x = to_dev(wl.make_x(spec), spec.dtype) if x is None else x
        ctx_np = wl.make_context(spec)
        self.ctx = None if ctx_np is None else to_dev(ctx_np, spec.dtype)
        self.wts = device_weights(spec, wl.make_weights(spec))
        self.ws_bytes = si.si_workspace_bytes(self.x, self.wts, self.ctx, self.axis, self.slice_len)
        self.live_sliced = si.si_live_activation_bytes(self.x, self.wts, self.ctx, self.axis, self.slice_len)
        self.live_unsliced = si.si_live_activation_bytes(self.x, self.wts, self.ctx, self.axis, self.extent)
        self.lanes = si.si_windows_in_flight(self.x, self.wts, self.ctx, self.axis, self.slice_len)
        self.out = torch.empty_like(self.x)
        self.ws = None

    def forward(self, flags=0):
        import paper_2411_01171_amd as si
        si.si_block_forward_ex(self.x, self.wts, self.ctx, self.out, self.axis, self.slice_len, self.ws, flags)


def measure(name, blocks, args, headline=False):
    """Times one workload: `blocks` run back to back (each block's output is the next one's input),
    then the Step Rehash test of the last output against a cached one.  Returns the record."""
    import numpy as np
    import torch
    import paper_2411_01171_amd as si
    import si_workloads as wl

    specs = [wl.CONFIGS[b] for b in blocks]
    runs = []
    for i, spec in enumerate(specs):
        sl = args.slice_len if (args.slice_len and len(specs) == 1) else None
        runs.append(BlockRun(spec, sl, x=None if i == 0 else runs[-1].out))
    # one workspace serves the blocks of a pair in turn (each call re-lays-out its weights)
    ws_bytes = max(r.ws_bytes for r in runs)
    before = torch.cuda.memory_allocated()
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    ws_alloc = torch.cuda.memory_allocated() - before
    for r in runs:
        r.ws = ws
    last = runs[-1]
    x0 = runs[0].x
    scratch = torch.empty(si.si_rehash_scratch_bytes(x0.numel()), dtype=torch.uint8, device="cuda")
    cos = torch.zeros(1, dtype=torch.float64, device="cuda")
    dec = torch.zeros(1, dtype=torch.int32, device="cuda")
    gamma = wl.CFG5_GAMMA
    flags = si.SI_FWD_WEIGHTS_PACKED if (args.weights_packed and len(runs) == 1) else 0

    # cached feature: the output for a drifted earlier input (what a previous key step would have stored)
    from paper_2411_01171_amd.devio import to_dev
    x_keep = x0.clone()
    x_prev = to_dev(wl.cfg5_step_input(wl.make_x(specs[0]), 5, specs[0].dtype), specs[0].dtype)
    x0.copy_(x_prev)
    del x_prev
    for r in runs:
        r.forward()
    cached = last.out.clone()
    x0.copy_(x_keep)
    del x_keep
    torch.cuda.synchronize()

    def step():
        for r in runs:
            r.forward(flags)
        si.si_rehash_check(last.out, cached, gamma, cos, dec, scratch)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    mem0 = torch.cuda.memory_allocated()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    hidden_alloc = torch.cuda.max_memory_allocated() - mem0     # nothing may be allocated during the steps

    # distribution over repetitions, each bracketed by its own event pair
    reps = args.reps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    rep_ms = np.array([a.elapsed_time(b) for a, b in evs])

    flops = sum(s.flops() for s in specs)
    value = flops / (ms_per_step * 1e-3) / 1e12

    # per-kernel durations: every launch between its own HIP event pair on the stream it runs on,
    # windows one at a time; one block at a time so that stage names stay per block
    block_reports, dominant = {}, None
    for r in runs:
        si.si_stage_timing_enable(True)
        for _ in range(args.steps):
            r.forward(flags)
            if r is last:
                si.si_rehash_check(last.out, cached, gamma, cos, dec, scratch)
        torch.cuda.synchronize()
        stages = si.si_stage_timing_read()
        si.si_stage_timing_enable(False)
        spec = r.spec
        M_slice = spec.tokens // r.extent * min(r.slice_len, r.extent)
        rep = {}
        for sname, (ms, cnt) in stages.items():
            avg_ms = ms / cnt
            kind, work = stage_work(spec, sname, M_slice)
            rec = {"avg_us": round(avg_ms * 1e3, 2), "launches_per_step": cnt / args.steps,
                   "ms_per_step": round(ms / args.steps, 4)}
            if kind == "flop":
                rec["TFLOP/s"] = round(work / (avg_ms * 1e-3) / 1e12, 1)
                rec["frac_mfma_peak"] = round(work / (avg_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
            elif kind == "byte":
                rec["GB/s"] = round(work / (avg_ms * 1e-3) / 1e9, 1)
                rec["frac_hbm_peak"] = round(work / (avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
            rep[sname] = rec
            if dominant is None or ms > dominant[3]:
                dominant = (spec, sname, M_slice, ms, cnt)
        n_slices = -(-r.extent // r.slice_len)
        block_reports[spec.name] = {
            "slice_axis": spec.slice_axis, "slice_len": r.slice_len, "slices": n_slices, "windows_in_flight": r.lanes,
            "live_activation_bytes": {"sliced": r.live_sliced, "unsliced_same_kernels": r.live_unsliced,
                                      "ratio": r.live_sliced / r.live_unsliced,
                                      "unsliced_op_by_op": 13 * spec.tokens * spec.C * r.x.element_size(),
                                      "ratio_op_by_op": r.live_sliced / (13 * spec.tokens * spec.C * r.x.element_size())},
            "kernel_ms_per_step": round(sum(v["ms_per_step"] for v in rep.values()), 4),
            "stages": rep}

    d_spec, d_name, d_M, d_ms, d_cnt = dominant
    d_kind, d_work = stage_work(d_spec, d_name, d_M)
    avg_s = d_ms / d_cnt * 1e-3
    if d_kind == "flop":
        peak = PEAK_BF16_TFLOPS if d_spec.dtype == "bf16" else PEAK_F32_VALU_TFLOPS
        ach = d_work / avg_s / 1e12
        roof = {"bound": "mfma" if d_spec.dtype == "bf16" else "alu", "kernel": f"{d_spec.name}/{d_name}", "achieved": ach,
                "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "algorithmic_flop_per_launch": d_work}
    else:
        ach = d_work / avg_s / 1e9
        roof = {"bound": "hbm", "kernel": f"{d_spec.name}/{d_name}", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "algorithmic_bytes_per_launch": d_work}
    roof["avg_launch_us"] = avg_s * 1e6
    trec, tnote = traffic_record(d_spec.name, d_name)
    roof["traffic"] = trec["total_bytes"] if trec else None
    roof["traffic_source"] = tnote
    if trec:
        roof["traffic_detail"] = trec

    x_bytes = x0.numel() * x0.element_size()
    rec = {
        "workload": name, "blocks": blocks, "ms_per_step": ms_per_step,
        "ms_reps": {"n": reps, "median": float(np.median(rep_ms)), "mean": float(rep_ms.mean()), "min": float(rep_ms.min())},
        "TFLOP/s": value, "frac_mfma_peak": value / PEAK_BF16_TFLOPS,
        "algorithmic_flop_per_step": flops, "tokens": specs[0].tokens,
        "live_activation_bytes": {"sliced": max(r.live_sliced for r in runs),
                                  "unsliced_same_kernels": max(r.live_unsliced for r in runs),
                                  "ratio": max(r.live_sliced for r in runs) / max(r.live_unsliced for r in runs),
                                  "workspace_bytes": ws_bytes, "x_bytes": x_bytes},
        # the library allocates nothing: torch's allocator grows by exactly the workspace the caller
        # made and by nothing during the timed steps
        "memory_check": {"workspace_bytes": ws_bytes, "torch_allocated_for_workspace": ws_alloc,
                         "allocated_during_steps": hidden_alloc},
        # 3 reads + 1 write of the feature per block at the very least
        "hbm_floor_check": {"GB/s_if_4x_feature_per_block": 4 * x_bytes * len(runs) / (ms_per_step * 1e-3) / 1e9,
                            "peak": PEAK_HBM_GBS},
        "rehash": {"cos": float(cos.item()), "decision": int(dec.item())},
        "roofline": roof,
        "per_block": block_reports,
    }
    return rec


WORKLOADS = {
    "cfg2": ["cfg2"], "cfg3": ["cfg3"], "cfg4s": ["cfg4s"], "cfg4t": ["cfg4t"], "cfg4": ["cfg4s", "cfg4t"],
    "cfg5s": ["cfg5s"], "cfg5t": ["cfg5t"], "cfg5": ["cfg5s", "cfg5t"], "cfg1": ["cfg1"],
}
HEADLINE = "cfg4"     # the largest single-GPU workload: the SVD-XT-shaped spatial + temporal pair


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--reps", type=int, default=50, help="repetitions behind the median / mean / min figures")
    ap.add_argument("--workload", default="all",
                    help="all (default): the headline workload cfg4 (SVD-XT-shaped spatial + temporal pair) plus one record "
                         "for every other configuration; or one of cfg1, cfg2, cfg3, cfg4s, cfg4t, cfg4, cfg5s, cfg5t, cfg5; "
                         "res4, res4b, res4c (Spatial ResBlock group); down4, up4b (its Down/UpSample)")
    ap.add_argument("--slice-len", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--weights-packed", action="store_true",
                    help="steady-state serving: the timed steps promise unchanged weights (SI_FWD_WEIGHTS_PACKED), so "
                         "the per-call weight re-layout is skipped; the default re-lays-out the weights in every step")
    ap.add_argument("--rehash-in-place", action="store_true",
                    help="with --rehash-probe: the result is taken in the anchor's output buffer (out == cache.y_key), "
                         "so a reused step copies nothing and a computed step copies only x")
    ap.add_argument("--rehash-probe", choices=["reuse", "compute"], default=None,
                    help="time si_block_forward_rehash instead of forward + output check: the anchor is the input "
                         "itself (reuse: the cached output is handed back) or a drifted input restored before every "
                         "step (compute: test fails, full forward, anchor update)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of the feature (known bytes) so that hardware byte counters "
                         "collected around this command can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path would shard over slices and batch entries "
              "without changing a kernel); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload.startswith("res"):
        return main_resblock(args)
    if args.workload in ("down4", "up4b"):
        return main_resample(args)
    if args.rehash_probe:
        return main_rehash_probe(args)

    import torch
    import si_workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    head_name = HEADLINE if args.workload == "all" else args.workload
    if args.calibration_copy:
        from paper_2411_01171_amd.devio import to_dev
        xc = to_dev(wl.make_x(wl.CONFIGS[WORKLOADS[head_name][0]]), "bf16")
        torch.empty_like(xc).copy_(xc)       # reads and writes xc.numel() * element_size bytes
        torch.cuda.synchronize()
        del xc
    head = measure(head_name, WORKLOADS[head_name], args, headline=True)
    specs = [wl.CONFIGS[b] for b in WORKLOADS[head_name]]
    desc = " then ".join(
        f"{s.kind} block x[B={s.B},C={s.C},F={s.F},H={s.H},W={s.W}], {s.heads} heads x {s.dim_head}, sliced along "
        f"{s.slice_axis} in windows of {head['per_block'][s.name]['slice_len']} ({head['per_block'][s.name]['slices']} slices)"
        for s in specs)
    result = {
        "metric": "sliced block-forward TFLOP/s (% MFMA peak) + peak live activation bytes vs unsliced",
        "value": head["TFLOP/s"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": specs[0].dtype, "data": "synthetic",
        "config": {"workload": f"{head_name}: {desc} + rehash check of the output (threshold {wl.CFG5_GAMMA})"
                               + ("; weights re-laid-out once, not per step" if args.weights_packed else "")
                               + ("; headline = the largest single-GPU workload of the five configurations" if args.workload == "all" else ""),
                   "algorithmic_flop_per_step": head["algorithmic_flop_per_step"], "tokens": head["tokens"]},
        "frac_mfma_peak": head["frac_mfma_peak"],
        "ms_reps": head["ms_reps"],
        "live_activation_bytes": head["live_activation_bytes"],
        "memory_check": head["memory_check"], "hbm_floor_check": head["hbm_floor_check"],
        "rehash": head["rehash"],
        "roofline": head["roofline"],
        "per_block": head["per_block"],
        "kernel_source_hash": source_hash(),
    }
    if args.workload == "all":
        # one record per configuration, each timed like the headline (same steps / warm-up)
        configs = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4s", "cfg4t", "cfg5s", "cfg5t"):
            torch.cuda.empty_cache()
            configs[name] = measure(name, WORKLOADS[name], args)
        result["configs"] = configs
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(specs)
    print(json.dumps(result))


def main_rehash_probe(args):
    """Cost of one si_block_forward_rehash step that reuses / recomputes (one block workload)."""
    import numpy as np
    import torch
    import paper_2411_01171_amd as si
    import si_workloads as wl
    from paper_2411_01171_amd.devio import to_dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    name = "cfg2" if args.workload == "all" else args.workload
    spec = wl.CONFIGS[name]
    r = BlockRun(spec, args.slice_len)
    r.ws = torch.empty(r.ws_bytes, dtype=torch.uint8, device="cuda")
    x_np = wl.make_x(spec)
    gamma = wl.CFG5_GAMMA
    cache = si.RehashCache(r.x)
    far = to_dev(wl.round_to_storage(x_np + np.float32(0.5) * wl.make_x(spec, seed=spec.seed + 77), spec.dtype), spec.dtype)
    si.si_block_forward_rehash(r.x, r.wts, r.ctx, r.out, r.axis, r.slice_len, r.ws, cache, gamma)   # fills the anchor
    probe = {}

    def step():
        if args.rehash_probe == "compute":
            cache.x_key.copy_(far)
        dst = cache.y_key if args.rehash_in_place else r.out
        probe["reused"], probe["cos"] = si.si_block_forward_rehash(r.x, r.wts, r.ctx, dst, r.axis, r.slice_len, r.ws, cache, gamma)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    si.si_stage_timing_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    stages = si.si_stage_timing_read()
    si.si_stage_timing_enable(False)
    value = spec.flops() / (ms_per_step * 1e-3) / 1e12
    print(json.dumps({
        "metric": "sliced block-forward TFLOP/s (% MFMA peak) + peak live activation bytes vs unsliced",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": f"{name}: one-pass rehash on the input, probe '{args.rehash_probe}' (value counts the forward's "
                               f"FLOPs whether computed or handed back)", "algorithmic_flop_per_step": spec.flops()},
        "rehash": {"probe": args.rehash_probe, "reused": bool(probe["reused"]), "cos": probe["cos"]},
        "stages": {n: {"avg_us": round(ms / c * 1e3, 2), "launches_per_step": c / args.steps, "ms_per_step": round(ms / args.steps, 4)}
                   for n, (ms, c) in stages.items()}}))


if __name__ == "__main__":
    main()
