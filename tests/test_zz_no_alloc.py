"""GPU: the entry point that allocates nothing (its workspace is an array resident in the library's device
image) against snip_quant_error_stats, which takes the caller's workspace: same kernels, same launch shapes,
so the results must agree bit for bit; two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared array is there when the second one runs."""
import numpy as np
import pytest
import torch

from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu, to_dev

pytestmark = pytest.mark.gpu


def both(snip, bits, axis, rule):
    x = to_dev(bits)
    L = bits.shape[0] if axis == snip.ROW else bits.shape[1]
    want_lines = torch.empty((L, 3), dtype=torch.float32, device="cuda")
    want = snip.snip_quant_error_stats(x, axis, rule, per_line=want_lines)
    got = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    got_lines = torch.full((L, 3), -1.0, dtype=torch.float32, device="cuda")
    snip.snip_quant_error_stats_noalloc(x, axis, rule, out=got, per_line=got_lines)
    torch.cuda.synchronize()
    return host(got), host(got_lines), host(want), host(want_lines)


@pytest.mark.parametrize("axis", [0, 1])
def test_noalloc_matches_workspace_call_twice(axis):
    snip = require_gpu()
    rng = np.random.default_rng(90 + axis)
    for rows, cols in ((1504, 4128), (352, 1056)):          # the second call is smaller than the first
        a = rng.standard_t(3, size=(rows, cols)) * 10.0 ** rng.integers(-3, 3, size=(rows, 1))
        bits = wl.f32_to_bf16_bits(a.astype(np.float32))
        got, got_lines, want, want_lines = both(snip, bits, axis, snip.NO_OVERFLOW)
        assert got.tobytes() == want.tobytes()
        assert got_lines.tobytes() == want_lines.tobytes()
        assert np.all(np.isfinite(got)) and got[0] > 0


def test_noalloc_against_oracle_and_limits():
    import ctypes
    import oracle
    snip = require_gpu()
    rng = np.random.default_rng(92)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((256, 768)).astype(np.float32))
    for axis in (oracle.ROW, oracle.COL):
        got, got_lines, _, _ = both(snip, bits, axis, snip.OCP_FLOOR)
        want, want_lines = oracle.stats(bits, axis, oracle.FLOOR, per_line=True)
        np.testing.assert_allclose(got, want, rtol=1e-5)
        np.testing.assert_allclose(got_lines, want_lines, rtol=1e-5, atol=0)
    # wider than the resident array allows: rejected on the host, nothing launched
    L = snip._lib()
    limit = int(L.snip_noalloc_max_cols())
    fake = ctypes.c_void_p(0x1000)
    assert L.snip_quant_error_stats_noalloc(fake, 32, limit + 32, limit + 32, 0, 0, fake, None, None) == 5
    assert L.snip_quant_error_stats_noalloc(fake, 32, 48, 48, 0, 0, fake, None, None) == 2
    # empty input: zeros, as the workspace call
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    snip.snip_quant_error_stats_noalloc(x, snip.ROW, snip.NO_OVERFLOW, out=out)
    torch.cuda.synchronize()
    assert host(out).tolist() == [0.0, 0.0, 0.0]
