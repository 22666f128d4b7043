"""The library's calls only enqueue kernels on the caller's stream, so a sequence of them can be captured
into a HIP graph.  Replays (several, with ordinary work and synchronisation in between) must reproduce the
eager results bit for bit."""
import numpy as np
import pytest
import torch

from paper_2602_01410_amd import workloads as wl

from gpu_util import require_gpu, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("gemm_tile")]


def test_graph_replay_matches_eager():
    snip = require_gpu()
    cfg = wl.CONFIGS[1]
    lay = wl.make_layer(cfg)
    lin = cfg.linears[0]
    X, W, dY = (to_dev(t) for t in (lay.X[lin.x_group], lay.W[lin.name], lay.dY[lin.name]))
    entry = (1, 1, 0, 0, 1, 0)
    plan = snip.make_plan(entry)
    M, N, K = cfg.M, lin.N, lin.K

    def alloc():
        return {
            "xr": snip.alloc_qtensor(M, K, entry[0]), "wr": snip.alloc_qtensor(N, K, entry[1]),
            "dyr": snip.alloc_qtensor(M, N, entry[2]), "wc": snip.alloc_qtensor(K, N, entry[3]),
            "dyc": snip.alloc_qtensor(N, M, entry[4]), "xc": snip.alloc_qtensor(K, M, entry[5]),
            "y": torch.empty((M, N), dtype=torch.bfloat16, device="cuda"),
            "dx": torch.empty((M, K), dtype=torch.bfloat16, device="cuda"),
            "dw": torch.empty((N, K), dtype=torch.bfloat16, device="cuda"),
            "st": [snip.alloc_stats() for _ in range(3)], "ndw": torch.empty(1, dtype=torch.float64, device="cuda"),
            "ws": snip.alloc_workspace(max(M, N), max(N, K)),
            "gws": torch.empty(snip.gemm_workspace_bytes(max(M, N), max(N, K)), dtype=torch.uint8, device="cuda"),
        }

    def step(b):
        snip.snip_quantize(X, entry[0], snip.ROW, out=b["xr"], stats=b["st"][0], workspace=b["ws"])
        snip.snip_quantize(W, entry[1], snip.ROW, out=b["wr"])
        snip.snip_quantize_sr_fp4(dY, snip.ROW, seed=9, out=b["dyr"]) if entry[2] == snip.FP4 else \
            snip.snip_quantize(dY, entry[2], snip.ROW, out=b["dyr"])
        snip.snip_quantize(W, entry[3], snip.COL, out=b["wc"])
        snip.snip_quantize_sr_fp4(dY, snip.COL, seed=10, out=b["dyc"])
        snip.snip_quantize(X, entry[5], snip.COL, out=b["xc"], stats=b["st"][1], workspace=b["ws"])
        snip.snip_gemm_fwd(plan, b["xr"], b["wr"], out=b["y"])
        snip.snip_gemm_dgrad(plan, b["dyr"], b["wc"], out=b["dx"])
        snip.snip_gemm_wgrad_norm(plan, b["dyc"], b["xc"], out=b["dw"], sum_sq=b["ndw"], workspace=b["gws"])
        snip.snip_quant_error_stats(dY, snip.COL, out=b["st"][2], workspace=b["ws"])

    def snapshot(b):
        torch.cuda.synchronize()
        return [t.clone() for t in (b["y"], b["dx"], b["dw"], b["ndw"], *b["st"], b["xr"].codes, b["dyc"].codes,
                                    b["dyc"].scales, b["wc"].scales_g4)]

    eager = alloc()
    step(eager)
    want = snapshot(eager)

    g = alloc()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(g)                                        # warm-up outside capture, as torch asks for
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(g)
    for rep in range(4):
        for t in (g["y"], g["dx"], g["dw"]):
            t.zero_()                                  # eager work between replays; results must come from the replay
        g["ndw"].fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot(g)
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), rep
