"""GPU: calls on different streams overlap safely when their outputs and workspaces differ (the header's
re-entrancy rule), and every call honours the stream it is given."""
import numpy as np
import pytest
import torch

from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu, to_dev

pytestmark = pytest.mark.gpu


def test_two_streams_with_their_own_workspaces():
    snip = require_gpu()
    rng = np.random.default_rng(77)
    xs = [to_dev(wl.f32_to_bf16_bits(rng.standard_normal((2048, 2048)).astype(np.float32))) for _ in range(2)]
    # serial reference on the current stream
    ref = []
    for x in xs:
        sr, sc = snip.alloc_stats(), snip.alloc_stats()
        qr, qc = snip.snip_quantize_both(x, snip.FP4, snip.FP8, stats_row=sr, stats_col=sc, both_formats=True)
        y = snip.snip_gemm_fwd(snip.make_plan((snip.FP4, snip.FP4, 0, 0, 0, 0)), qr, qr)
        ref.append((qr, qc, sr, sc, y))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [None, None]
    keep = []                                  # nothing is freed while kernels that use it may still run
    for rep in range(5):                       # interleave the two streams' launches
        for i, (x, st) in enumerate(zip(xs, streams)):
            ws = snip.alloc_workspace(2048, 2048)
            sr, sc = snip.alloc_stats(), snip.alloc_stats()
            with torch.cuda.stream(st):
                qr, qc = snip.snip_quantize_both(x, snip.FP4, snip.FP8, stats_row=sr, stats_col=sc, workspace=ws,
                                                 both_formats=True, stream=st)
                y = snip.snip_gemm_fwd(snip.make_plan((snip.FP4, snip.FP4, 0, 0, 0, 0)), qr, qr, stream=st)
            got[i] = (qr, qc, sr, sc, y, ws)
            keep.append(got[i])
    for st in streams:
        st.synchronize()
    for g, r in zip(got, ref):
        assert torch.equal(g[0].codes, r[0].codes) and torch.equal(g[1].codes, r[1].codes)
        assert torch.equal(g[0].scales, r[0].scales) and torch.equal(g[1].scales, r[1].scales)
        assert host(g[2]).tobytes() == host(r[2]).tobytes() and host(g[3]).tobytes() == host(r[3]).tobytes()
        assert torch.equal(g[4], r[4])


def test_temporaries_belong_to_the_stream_of_the_call():
    """A call on a side stream that lets the wrapper allocate its workspace and outputs: the temporaries are taken
    from that stream's pool (so the current stream's work cannot be handed the workspace while the side stream's
    kernels still use it), and a raw handle of a foreign stream is refused when a buffer would have to be allocated."""
    snip = require_gpu()
    rng = np.random.default_rng(78)
    x = to_dev(wl.f32_to_bf16_bits(rng.standard_normal((1024, 1024)).astype(np.float32)))
    ref = snip.snip_quant_error_stats(x, snip.COL)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    outs = []
    for _ in range(8):
        outs.append(snip.snip_quant_error_stats(x, snip.COL, stream=side))       # workspace + output allocated inside
        torch.empty(1 << 22, dtype=torch.uint8, device="cuda").fill_(0xFF)      # current-stream work wanting memory
    side.synchronize()
    torch.cuda.synchronize()
    for o in outs:
        assert host(o).tobytes() == host(ref).tobytes()
    with pytest.raises(ValueError):
        snip.snip_quant_error_stats(x, snip.COL, stream=side.cuda_stream)        # raw handle, would allocate
    ws, out = snip.alloc_workspace(1024, 1024), snip.alloc_stats()
    side.wait_stream(torch.cuda.current_stream())
    snip.snip_quant_error_stats(x, snip.COL, out=out, workspace=ws, stream=side.cuda_stream)   # raw handle, nothing to allocate
    side.synchronize()
    assert host(out).tobytes() == host(ref).tobytes()
