"""Benchmark of the SNIP quantized linear-layer hot path on one MI355X.

A step is one pass of the whole path over one Llama-shaped transformer block's seven linear
layers: every quantization the plan calls for (each distinct (tensor, format, axis) once; a
tensor wanted in both orientations gets them from one call and one read) with the statistics
pass fused into it (the same call returns the squared norms of the tensor and of its
quantization error for both candidate formats and both block directions: the complete Step-1
record, no stand-alone statistics launch), and the 21 GEMMs (fwd, dgrad, wgrad per linear).
A tensor that no two-orientation call covers gets its record from the stand-alone statistics
call.  Inputs are resident in HBM before timing starts.  Prints one JSON line.
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

import numpy as np
import torch

PEAK = {"fp4": 10.1e15, "fp8": 5.0e15, "hbm": 8.0e12}
# L2-miss-side bytes per launch (FETCH_SIZE + WRITE_SIZE, calibrated against a copy kernel) of the dominant kernel.
# Not measured by this run: counters need rocprofv3.  The figure is copied from the profile summary named beside
# it, taken with this command on this kernel; a (config, plan, kernel) without such a profile reports null.
MEASURED_TRAFFIC = {(4, "mix50", "gemm_fast_kernel<fp4,fp4>"): 546.6e6}
TRAFFIC_SOURCE = "profiles/hbm_traffic_config4_mix50.md"
KERNEL_NAME = {(0, 0): "gemm_fast_kernel<fp8,fp8>", (1, 1): "gemm_fast_kernel<fp4,fp4>",
               (0, 1): "gemm_fast_kernel<fp8,fp4>", (1, 0): "gemm_fast_kernel<fp4,fp8>"}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=10)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--config", type=int, default=4, help="workload configuration 1..5 (default: Llama-7B-shaped layer)")
    p.add_argument("--plan", type=str, default=None, help="fp4 | fp8 | mixNN | tensor (default: the config's mixed plan)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    p.add_argument("--no-next-rows", action="store_true",
                   help="skip the measurements made after the timed region: per-variant rates of the streaming kernels, "
                        "stochastic rounding, the paper's own recipe, the AdamW sensitivity")
    p.add_argument("--output-norms", action="store_true",
                   help="use the GEMM variants that also return the squared Frobenius norm of Y, dX, dW")
    p.add_argument("--separate-quantize", action="store_true",
                   help="one quantize call per orientation (two reads of a tensor wanted in both) instead of snip_quantize_both")
    p.add_argument("--library-reference", action="store_true",
                   help="time the vendor library's GEMMs beside snip_gemm_fwd on the 7B shapes, print JSON and exit")
    p.add_argument("--microbench", nargs="?", const="default", default=None, choices=["default", "hbm-sweep", "lds", "mfma-lds"],
                   help="run the device microbenchmarks (measured MFMA / HBM / L2 rates; `hbm-sweep`: copy / read / write "
                        "rates over launch shapes, loads in flight, access widths and non-temporal hints) and exit")
    return p.parse_args()


class Layer:
    """Device tensors, pre-allocated outputs and the launch list of one step."""

    def __init__(self, cfg, plan, snip, wl, output_norms=False, separate_quantize=False):
        self.cfg, self.plan, self.snip = cfg, plan, snip
        self.output_norms = output_norms
        dev = "cuda"

        def up(bits):
            return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

        t0 = time.time()
        self.src = {}
        for l in cfg.linears:
            if ("X", l.x_group) not in self.src:
                self.src[("X", l.x_group)] = up(wl.make_tensor(cfg, "X", l.x_group))
            self.src[("W", l.name)] = up(wl.make_tensor(cfg, "W", l.name))
            self.src[("dY", l.name)] = up(wl.make_tensor(cfg, "dY", l.name))
        self.gen_seconds = time.time() - t0

        max_r = max(t.shape[0] for t in self.src.values())
        max_c = max(t.shape[1] for t in self.src.values())
        self.ws = snip.alloc_workspace(max_r, max_c)
        self.qjobs, self.q = [], {}       # distinct (src key, fmt, axis)
        self.gjobs = []

        def need(key, fmt, axis):
            k = (key, fmt, axis)
            if k not in self.q:
                t = self.src[key]
                sr, sc = (t.shape[0], t.shape[1]) if axis == snip.ROW else (t.shape[1], t.shape[0])
                self.q[k] = snip.alloc_qtensor(sr, sc, fmt)
                self.qjobs.append((k, snip.alloc_stats()))
            return self.q[k]

        M = cfg.M
        for l, e in zip(cfg.linears, plan):
            pc = snip.make_plan(e)
            kx, kw, kdy = ("X", l.x_group), ("W", l.name), ("dY", l.name)
            self.gjobs.append(("fwd", pc, need(kx, e[0], snip.ROW), need(kw, e[1], snip.ROW),
                               torch.empty((M, l.N), dtype=torch.bfloat16, device=dev), 2 * M * l.N * l.K, (e[0], e[1])))
            self.gjobs.append(("dgrad", pc, need(kdy, e[2], snip.ROW), need(kw, e[3], snip.COL),
                               torch.empty((M, l.K), dtype=torch.bfloat16, device=dev), 2 * M * l.N * l.K, (e[2], e[3])))
            self.gjobs.append(("wgrad", pc, need(kdy, e[4], snip.COL), need(kx, e[5], snip.COL),
                               torch.empty((l.N, l.K), dtype=torch.bfloat16, device=dev), 2 * M * l.N * l.K, (e[4], e[5])))
        # Quantize calls: a tensor wanted with blocks along its rows and down its columns gets both from one call
        # (the formats may differ); whatever is left over (a second format in one orientation) goes alone.
        self.qcalls, left = [], list(self.qjobs)
        while left:
            j = left.pop(0)
            mate = next((o for o in left if o[0][0] == j[0][0] and o[0][2] != j[0][2]), None) if not separate_quantize else None
            if mate is None:
                self.qcalls.append((j,))
            else:
                left.remove(mate)
                self.qcalls.append((j, mate) if j[0][2] == snip.ROW else (mate, j))
        self.qcalls.sort(key=lambda call: call[0][0][0][0] != "W")        # weights first (stable): their time is reported apart
        # statistics pass: both block directions and both formats of every distinct tensor, one read each
        self.sjobs = [(key, snip.alloc_stats(), snip.alloc_stats()) for key in self.src]
        covered = {c[0][0][0] for c in self.qcalls if len(c) == 2}
        self.sjobs_uncovered = [j for j in self.sjobs if j[0] not in covered]
        if output_norms:
            self.gws = torch.empty(max(snip.gemm_workspace_bytes(j[4].shape[0], j[4].shape[1]) for j in self.gjobs),
                                   dtype=torch.uint8, device=dev)
            self.gnorm = [torch.empty(1, dtype=torch.float64, device=dev) for _ in self.gjobs]
        self.flops = sum(j[5] for j in self.gjobs)
        # algorithmic bytes of the quantize calls: one read of the source per call, codes + scales per output
        self.q_bytes = sum(self.src[call[0][0][0]].numel() * (2 + sum((1.0 if k[1] == snip.FP8 else 0.5) + 1 / 32 for k, _ in call))
                           for call in self.qcalls)
        self.s_bytes = sum(self.src[key].numel() * 2 for key, _, _ in self.sjobs)        # one read per tensor

    def step(self, ev=None, fused_statistics=True):
        snip = self.snip
        fn = {"fwd": snip.snip_gemm_fwd, "dgrad": snip.snip_gemm_dgrad, "wgrad": snip.snip_gemm_wgrad}

        # One HIP event in front of every GEMM call, one wherever the kind of call changes (weight quantizations,
        # other quantizations, statistics) and one behind the last call: a GEMM's duration, and a group's, is the
        # distance to the next event, on the stream the kernels are launched on.
        last = [None]

        def timed(tag, f):
            if ev is not None and (tag[0] == "g" or tag != last[0]):
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                ev.append((tag, e))
            last[0] = tag
            f()

        for job in self.qcalls:
            if len(job) == 2:           # both orientations of one tensor from one read
                ((key, fr, _), st_r), ((_, fc, _), st_c) = job
                timed(("q", key[0] == "W"), lambda: snip.snip_quantize_both(
                    self.src[key], fr, fc, out_row=self.q[(key, fr, snip.ROW)], out_col=self.q[(key, fc, snip.COL)],
                    stats_row=st_r, stats_col=st_c, workspace=self.ws, both_formats=fused_statistics))
            else:
                ((key, fmt, axis), st), = job
                timed(("q", key[0] == "W"), lambda: snip.snip_quantize(self.src[key], fmt, axis, out=self.q[(key, fmt, axis)],
                                                                      stats=st, workspace=self.ws))
        fn_norm = {"fwd": snip.snip_gemm_fwd_norm, "dgrad": snip.snip_gemm_dgrad_norm, "wgrad": snip.snip_gemm_wgrad_norm}
        for gi, (name, pc, a, b, out, fl, fmts) in enumerate(self.gjobs):
            if self.output_norms:
                timed(("g", fmts, fl), lambda: fn_norm[name](pc, a, b, out=out, sum_sq=self.gnorm[gi], workspace=self.gws))
            else:
                timed(("g", fmts, fl), lambda: fn[name](pc, a, b, out=out))
        # fused_statistics: a tensor's two-orientation quantize call has delivered its complete record already;
        # only tensors without such a call (none in configurations 2-5) need the stand-alone statistics call
        for key, st_row, st_col in (self.sjobs_uncovered if fused_statistics else self.sjobs):
            timed(("s",), lambda: snip.snip_quant_error_stats_both(self.src[key], out_row=st_row, out_col=st_col,
                                                                   workspace=self.ws))
        if ev is not None:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            ev.append((("end",), e))


def graph_replay(layer, steps, warmup):
    """The same step captured once into a HIP graph and replayed: what the launch gaps of the ~150 kernel
    launches of a step cost.  Reported beside `value` (which times ordinary launches with per-call events)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.step()                                   # everything the step touches exists before capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.step()
    for _ in range(max(1, warmup)):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    return {"ms_per_step": ms, "value": layer.flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s"}


def kernel_variants(cfg, layer, snip, warm=10, reps=50):
    """Algorithmic GB/s of every streaming-kernel variant on the output gradient of this configuration's largest
    linear (larger than the 256 MB Infinity Cache for configs 4 and 5): median of `reps` event-to-event intervals
    after `warm` untimed calls.  Measured after the timed region; not part of `value`."""
    lin = max(cfg.linears, key=lambda l: l.N * l.K)
    x = layer.src[("dY", lin.name)]
    R, C = x.shape
    n = x.numel()

    def med_gbps(f, nbytes):
        for _ in range(warm):
            f()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            f()
            ev[i + 1].record()
        torch.cuda.synchronize()
        t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
        return round(nbytes / (t[reps // 2] * 1e-3) / 1e9, 1)

    code = {snip.FP8: 1.0, snip.FP4: 0.5}
    name = {snip.FP8: "fp8", snip.FP4: "fp4"}
    out = {"tensor": f"dY of '{lin.name}' [{R} x {C}]", "unit": "GB/s of algorithmic bytes", "hbm_peak_gbps": PEAK["hbm"] / 1e9}
    st, st2 = snip.alloc_stats(), snip.alloc_stats()
    for fmt in (snip.FP8, snip.FP4):
        q = {snip.ROW: snip.alloc_qtensor(R, C, fmt), snip.COL: snip.alloc_qtensor(C, R, fmt)}
        one = n * (2 + code[fmt] + 1 / 32)
        for axis, tag in ((snip.ROW, "row"), (snip.COL, "col")):
            out[f"quantize_{tag}_{name[fmt]}"] = med_gbps(lambda: snip.snip_quantize(x, fmt, axis, out=q[axis]), one)
            out[f"quantize_{tag}_{name[fmt]}_stats"] = med_gbps(
                lambda: snip.snip_quantize(x, fmt, axis, out=q[axis], stats=st, workspace=layer.ws), one)
        both = n * (2 + 2 * (code[fmt] + 1 / 32))
        out[f"quantize_both_{name[fmt]}"] = med_gbps(
            lambda: snip.snip_quantize_both(x, fmt, fmt, out_row=q[snip.ROW], out_col=q[snip.COL]), both)
        out[f"quantize_both_{name[fmt]}_stats"] = med_gbps(
            lambda: snip.snip_quantize_both(x, fmt, fmt, out_row=q[snip.ROW], out_col=q[snip.COL], stats_row=st, stats_col=st2,
                                            workspace=layer.ws), both)
        out[f"quantize_both_{name[fmt]}_stats_both_formats"] = med_gbps(
            lambda: snip.snip_quantize_both(x, fmt, fmt, out_row=q[snip.ROW], out_col=q[snip.COL], stats_row=st, stats_col=st2,
                                            workspace=layer.ws, both_formats=True), both)
        del q
    for axis, tag in ((snip.ROW, "row"), (snip.COL, "col")):
        out[f"stats_{tag}"] = med_gbps(lambda: snip.snip_quant_error_stats(x, axis, out=st, workspace=layer.ws), n * 2)
    out["stats_both"] = med_gbps(lambda: snip.snip_quant_error_stats_both(x, out_row=st, out_col=st2, workspace=layer.ws), n * 2)
    return out


def next_rows(cfg, layer, snip, wl, reps=10):
    """Throughput of the variants beyond the core path, on this configuration's largest linear: FP4
    quantization with stochastic rounding of its output gradient (both axes) and the AdamW sensitivity
    reduction over its weight's optimizer state.  Measured after the timed region; not part of `value`."""
    lin = max(cfg.linears, key=lambda l: l.N * l.K)
    dy = layer.src[("dY", lin.name)]

    def rate(f, nbytes):
        for _ in range(2):
            f()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return nbytes / (a.elapsed_time(b) * 1e-3 / reps) / 1e9

    out = {"linear": lin.name}
    qbytes = dy.numel() * (2 + 0.5 + 1 / 32)
    for axis, tag in ((snip.ROW, "row"), (snip.COL, "col")):
        sr, sc = (dy.shape[0], dy.shape[1]) if axis == snip.ROW else (dy.shape[1], dy.shape[0])
        q = snip.alloc_qtensor(sr, sc, snip.FP4)
        out[f"sr_quantize_{tag}_gbps"] = rate(lambda: snip.snip_quantize_sr_fp4(dy, axis, seed=1, out=q), qbytes)
        out[f"rne_quantize_{tag}_gbps"] = rate(lambda: snip.snip_quantize(dy, snip.FP4, axis, out=q), qbytes)
        del q
    # the paper's own recipe: 1x128 tiles with real-valued scales on the same gradient, both axes, FP4 and FP8;
    # its statistics; and the software-scaled GEMM (tiles x 128x128 blocks) on the first linear's forward shapes
    T, B = snip.TILE_1x128, snip.BLOCK_128x128
    pws = torch.empty(int(snip._lib().snip_paper_workspace_bytes(dy.shape[0], dy.shape[1])), dtype=torch.uint8, device="cuda")
    pst = snip.alloc_stats()
    for axis, tag in ((snip.ROW, "row"), (snip.COL, "col")):
        out[f"paper_tile_quantize_fp4_{tag}_gbps"] = rate(lambda: snip.snip_quantize_paper(dy, snip.FP4, axis, T), qbytes)
        out[f"paper_tile_stats_{tag}_gbps"] = rate(lambda: snip.snip_quant_error_stats_paper(dy, axis, T, out=pst, workspace=pws),
                                                   dy.numel() * 2)
    l0 = cfg.linears[0]
    x0, w0 = layer.src[("X", l0.x_group)], layer.src[("W", l0.name)]
    y0 = torch.empty((cfg.M, l0.N), dtype=torch.bfloat16, device="cuda")
    for fmt, tag in ((snip.FP8, "fp8"), (snip.FP4, "fp4")):
        qa, qb = snip.snip_quantize_paper(x0, fmt, snip.ROW, T), snip.snip_quantize_paper(w0, fmt, snip.ROW, B)
        out[f"paper_gemm_{tag}_tflops"] = rate(lambda: snip.snip_gemm_paper(*qa, fmt, T, *qb, fmt, B, out=y0),
                                              2.0 * cfg.M * l0.N * l0.K) / 1e3
    m, v, g = (torch.from_numpy(t).cuda().reshape(-1) for t in wl.make_optimizer_state(cfg, lin.name))
    o = torch.empty(1, dtype=torch.float64, device="cuda")
    out["adamw_sensitivity_gbps"] = rate(lambda: snip.snip_adamw_sensitivity(m, v, g, 0.9, 0.999, 1e-8, out=o, workspace=layer.ws),
                                         m.numel() * 12)
    return out


def library_reference(snip, reps=20):
    """Context, not part of the path: the GEMMs of the vendor's library (hipBLASLt through torch.mm and
    torch._scaled_mm) on the 7B-shaped problems with N(0,1) operands, beside this repository's block-scaled kernels
    on the same shapes and data.  A kind the installed library does not support is reported as null."""
    torch.manual_seed(0)

    def tflops(f, flop):
        try:
            for _ in range(3):
                f()
        except Exception:
            return None
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return round(flop / (a.elapsed_time(b) * 1e-3 / reps) / 1e12, 1)

    rows = []
    for M, N, K in ((16384, 4096, 4096), (16384, 11008, 4096), (4096, 4096, 16384), (16384, 4096, 11008)):
        flop = 2.0 * M * N * K
        x, w = torch.randn(M, K, device="cuda"), torch.randn(N, K, device="cuda")
        xb, wb = x.bfloat16(), w.bfloat16()
        r = {"M": M, "N": N, "K": K, "unit": "TFLOP/s"}
        r["library_bf16"] = tflops(lambda: torch.mm(xb, wb.t()), flop)
        x8, w8 = x.to(torch.float8_e4m3fn), w.to(torch.float8_e4m3fn)
        one = torch.ones((), device="cuda")
        r["library_fp8_one_scale_per_tensor"] = tflops(
            lambda: torch._scaled_mm(x8, w8.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16), flop)
        try:
            e8 = torch.float8_e8m0fnu
            sa = torch.full((M, K // 32), 127, dtype=torch.uint8, device="cuda").view(e8)
            sb = torch.full((N, K // 32), 127, dtype=torch.uint8, device="cuda").view(e8)
            r["library_fp8_e8m0_blocks_of_32"] = tflops(
                lambda: torch._scaled_mm(x8, w8.t(), scale_a=sa, scale_b=sb, out_dtype=torch.bfloat16), flop)
            x4 = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda").view(torch.float4_e2m1fn_x2)
            w4 = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda").view(torch.float4_e2m1fn_x2)
            r["library_fp4_e8m0_blocks_of_32"] = tflops(
                lambda: torch._scaled_mm(x4, w4.t(), scale_a=sa, scale_b=sb, out_dtype=torch.bfloat16), flop)
        except Exception:
            r["library_fp8_e8m0_blocks_of_32"] = r["library_fp4_e8m0_blocks_of_32"] = None
        y = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        for fmt, tag in ((snip.FP8, "fp8"), (snip.FP4, "fp4")):
            xq, wq = snip.snip_quantize(xb, fmt, snip.ROW), snip.snip_quantize(wb, fmt, snip.ROW)
            plan = snip.make_plan((fmt,) * 6)
            r[f"snip_gemm_{tag}_e8m0_blocks_of_32"] = tflops(lambda: snip.snip_gemm_fwd(plan, xq, wq, out=y), flop)
        rows.append(r)
    return rows


def cpu_baseline(cfg, wl):
    """The oracle, as it stands, on bounded samples of this configuration (a baseline for context):
    GEMM: the first 256 tokens of the first linear, all three GEMMs with their quantizations (fake-quant + fp64
    product); the full-layer time is EXTRAPOLATED from that slab.  Quantize and statistics: the oracle's
    quantize (FP4, row blocks) and statistics (both formats, row blocks) in full on the largest tensor."""
    import oracle
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    lin = cfg.linears[0]
    ms = min(256, cfg.M)
    X = wl.make_tensor(cfg, "X", lin.x_group, 0, ms)
    dY = wl.make_tensor(cfg, "dY", lin.name, 0, ms)
    W = wl.make_tensor(cfg, "W", lin.name)
    t0 = time.time()
    y = oracle.gemm_fwd(oracle.fake_quant(X, oracle.FP4, oracle.ROW), oracle.fake_quant(W, oracle.FP4, oracle.ROW))
    dx = oracle.gemm_dgrad(oracle.fake_quant(dY, oracle.FP4, oracle.ROW), oracle.fake_quant(W, oracle.FP4, oracle.COL))
    dw = oracle.gemm_wgrad(oracle.fake_quant(dY, oracle.FP4, oracle.COL), oracle.fake_quant(X, oracle.FP4, oracle.COL))
    dt = time.time() - t0
    assert y.shape[0] == ms and dx.shape[0] == ms and dw.shape[0] == lin.N
    flops = 3 * 2 * ms * lin.N * lin.K
    layer_flop = sum(3 * 2 * cfg.M * l.N * l.K for l in cfg.linears)
    # quantize + statistics in full on the largest source tensor of the configuration
    big = max(cfg.linears, key=lambda l: l.N * l.K)
    T = wl.make_tensor(cfg, "dY", big.name)
    t1 = time.time()
    oracle.quantize(T, oracle.FP4, oracle.ROW)
    dq = time.time() - t1
    t1 = time.time()
    oracle.stats(T, oracle.ROW)
    ds = time.time() - t1
    n = T.size
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"first {ms} tokens of linear '{lin.name}' ({lin.N}x{lin.K}): 3 fake-quant GEMMs in fp64, "
                      f"{flops:.3g} FLOP in {dt:.2f} s",
            "gemm_full_layer_seconds_extrapolated": dt * layer_flop / flops,
            "quantize_gbps": n * (2 + 0.5 + 1 / 32) / dq / 1e9, "quantize_seconds": dq,
            "stats_gbps": n * 2 / ds / 1e9, "stats_seconds": ds,
            "quantize_stats_sample": f"dY of '{big.name}' [{T.shape[0]} x {T.shape[1]}] in full: oracle.quantize (FP4, row blocks; "
                                     f"GB/s of 2 B read + codes + scales written) and oracle.stats (both formats, row blocks; "
                                     f"GB/s of 2 B read)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.microbench:
        import subprocess
        exe = os.path.join(ROOT, "paper_2602_01410_amd", "snip_microbench")
        sys.exit(subprocess.run([exe] + ([] if args.microbench == "default" else [args.microbench])).returncode)
    from paper_2602_01410_amd import snip, workloads as wl
    if args.library_reference:
        snip._lib()
        print(json.dumps({"library_reference": library_reference(snip)}))
        return
    snip._lib()
    cfg = wl.CONFIGS[args.config]
    plan_name = args.plan or next((p for p in cfg.plans if p.startswith("mix")), cfg.plans[0])
    plan = wl.make_plan(cfg, plan_name)
    torch.cuda.set_device(0)
    layer = Layer(cfg, plan, snip, wl, args.output_norms, args.separate_quantize)

    for _ in range(args.warmup):
        layer.step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layer.step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # per-kernel figures from the HIP events recorded on the launch stream inside the timed region
    agg = {"qw": [0.0, 0, 0.0]}
    for (tag, a), (_, b) in zip(events[:-1], events[1:]):
        if tag[0] == "end":
            continue
        sec = a.elapsed_time(b) * 1e-3
        d = agg.setdefault(tag[0] if tag[0] != "g" else ("g", tag[1]), [0.0, 0, 0.0])
        d[0] += sec
        d[1] += 1
        if tag[0] == "g":
            d[2] += tag[2]
        if tag[0] == "q" and tag[1]:
            agg["qw"][0] += sec
    gem = {k[1]: v for k, v in agg.items() if isinstance(k, tuple)}
    dom = max(gem, key=lambda k: gem[k][0])
    dsec, dn, dfl = gem[dom]
    peak = PEAK["fp4"] if dom == (1, 1) else PEAK["fp8"]
    achieved = dfl / dsec
    gemm_sec = sum(v[0] for v in gem.values()) / args.steps
    q_sec = agg["q"][0] / args.steps
    s_sec = agg.get("s", [0.0])[0] / args.steps     # stand-alone statistics calls inside the step (none in configs 2-5)
    qw_sec = agg["qw"][0] / args.steps          # quantizations of weights (change once per optimizer step)
    plan_peak = wl.plan_peak_flops(cfg, plan, PEAK["fp4"], PEAK["fp8"])
    value = layer.flops / (ms_per_step * 1e-3) / 1e12
    traffic = MEASURED_TRAFFIC.get((cfg.index, plan_name, KERNEL_NAME[dom]))

    out = {
        "metric": "TFLOP/s of mixed FP4/FP8 fwd+bwd linear GEMMs incl. quantize (% of MFMA peak)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4_e2m1+fp8_e4m3 (fp32 accumulate, bf16 out)", "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}, {cfg.M} tokens, 7 linears x (fwd, dgrad, wgrad) "
                               f"+ all quantizations with the statistics pass fused into them", "plan": plan_name,
                   "fp4_flop_fraction": wl.plan_fp4_fraction(cfg, plan), "layer_flop": layer.flops,
                   "output_norms": bool(args.output_norms)},
        "pct_of_plan_peak": 100.0 * value * 1e12 / plan_peak,
        "gemm_only_tflops": layer.flops / gemm_sec / 1e12,
        "gemm_only_pct_of_plan_peak": 100.0 * layer.flops / gemm_sec / plan_peak,
        # quantize calls with the complete statistics record fused in; algorithmic bytes = one read of the source
        # plus the codes and scales written
        "quantize_gbps": layer.q_bytes / q_sec / 1e9, "quantize_pct_hbm": 100.0 * layer.q_bytes / q_sec / PEAK["hbm"],
        "ms_gemm": gemm_sec * 1e3, "ms_quantize_with_statistics": q_sec * 1e3, "ms_standalone_statistics": s_sec * 1e3,
        "quantized_tensors": len(layer.qjobs), "quantize_calls": len(layer.qcalls),
        # the two accountings of "incl. quantize"
        "gemm_plus_quantize_tflops": layer.flops / (gemm_sec + q_sec) / 1e12,
        "gemm_plus_quantize_w_amortised_tflops": layer.flops / (gemm_sec + q_sec - qw_sec) / 1e12,
        "input_generation_s": layer.gen_seconds,
        "roofline": {"bound": "mfma", "kernel": KERNEL_NAME[dom], "achieved": achieved / 1e12, "peak": peak / 1e12,
                     "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
                     "traffic_source": TRAFFIC_SOURCE if traffic is not None else None,
                     "launches": dn, "avg_launch_us": dsec / dn * 1e6, "avg_flop_per_launch": dfl / dn},
    }
    # the same step launched the ordinary way without the per-call events of the timed region (on the small
    # configurations creating and recording ~60 events per step costs more than the kernels take)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        layer.step()
    torch.cuda.synchronize()
    ms_plain = (time.perf_counter() - t1) / args.steps * 1e3
    out["no_events"] = {"ms_per_step": ms_plain, "value": layer.flops / (ms_plain * 1e-3) / 1e12, "unit": "TFLOP/s"}
    # Not `value`: the same outputs with the statistics as a pass of its own (every quantize call returns the error of
    # the format it writes, a stand-alone call per tensor reads it again for both formats and both block directions).
    sep_ev = []
    for _ in range(2):
        layer.step(fused_statistics=False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        layer.step(fused_statistics=False)
    torch.cuda.synchronize()
    ms_f = (time.perf_counter() - t1) / args.steps * 1e3
    # a second set of steps with one event per call, only to split the time between quantize and statistics calls
    # (recording that many events slows the small configurations down, so the step time above is taken without)
    for _ in range(args.steps):
        layer.step(sep_ev, fused_statistics=False)
    torch.cuda.synchronize()
    sq = ss = 0.0
    for (tag, a), (_, b) in zip(sep_ev[:-1], sep_ev[1:]):
        if tag[0] == "q":
            sq += a.elapsed_time(b) * 1e-3
        elif tag[0] == "s":
            ss += a.elapsed_time(b) * 1e-3
    sq /= args.steps
    ss /= args.steps
    out["statistics_as_separate_pass"] = {
        "ms_per_step": ms_f, "value": layer.flops / (ms_f * 1e-3) / 1e12, "unit": "TFLOP/s",
        "ms_quantize": sq * 1e3, "quantize_gbps": layer.q_bytes / sq / 1e9 if sq else None,
        "ms_stats": ss * 1e3, "stats_gbps": layer.s_bytes / ss / 1e9 if ss else None,
        "stats_pct_hbm": 100.0 * layer.s_bytes / ss / PEAK["hbm"] if ss else None}
    if not args.no_graph:
        out["hip_graph"] = graph_replay(layer, args.steps, args.warmup)
    if not args.no_next_rows:
        out["kernel_variants"] = kernel_variants(cfg, layer, snip)
        out["next_rows"] = next_rows(cfg, layer, snip, wl)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
