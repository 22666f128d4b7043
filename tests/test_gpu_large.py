"""GPU parity at the largest sizes: tensors of more than 2^31 elements (byte and element offsets beyond 32 bits in
every kernel), checked against the CPU oracle on slabs at the start, across the 2^31-element boundary and at the
end.  The tensor is a seeded [2112 x 32768] block repeated 32 times down the rows; 2112 does not divide 65536, so a
position computed modulo 2^32 bytes or 2^31 elements lands on different content."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, host_bf16_as_f64, rel_fro, require_gpu, to_dev

pytestmark = pytest.mark.gpu

BASE_ROWS, REPEAT, COLS = 2112, 32, 32768
ROWS = BASE_ROWS * REPEAT                      # 67584 rows x 32768 columns = 2.2e9 elements, 4.4 GB of bf16
ROW_SLABS = [(0, 32), (65504, 65568), (ROWS - 32, ROWS)]       # the middle one straddles element 2^31
COL_SLABS = [(0, 2), (16382, 16386), (COLS - 2, COLS)]


@pytest.fixture(scope="module")
def big():
    require_gpu()
    rng = np.random.default_rng(4242)
    base = rng.standard_normal((BASE_ROWS, COLS), dtype=np.float32)
    base *= np.exp2(rng.integers(-6, 7, size=(BASE_ROWS, COLS // 32))).repeat(32, axis=1).astype(np.float32)
    bits = wl.f32_to_bf16_bits(base)
    x = to_dev(bits).repeat(REPEAT, 1)
    assert x.shape == (ROWS, COLS) and x.numel() > 2 ** 31
    yield bits, x
    del x
    torch.cuda.empty_cache()


def rows_of(bits, lo, hi):
    return bits[np.arange(lo, hi) % BASE_ROWS]


def cols_of(bits, lo, hi):
    return np.ascontiguousarray(np.tile(bits[:, lo:hi], (REPEAT, 1)))


def check_row_output(q, bits, fmt):
    for lo, hi in ROW_SLABS:
        c, s = oracle.quantize(rows_of(bits, lo, hi), fmt, oracle.ROW)
        assert np.array_equal(host(q.codes[lo:hi]), c), (lo, hi)
        assert np.array_equal(host(q.scales[lo:hi]), s), (lo, hi)
        g4 = host(q.scales_g4[:, lo:hi, :])                   # [group][row][4] holds the same bytes
        assert np.array_equal(g4.transpose(1, 0, 2).reshape(hi - lo, -1), s), (lo, hi)


def check_col_output(q, bits, fmt):
    for lo, hi in COL_SLABS:
        c, s = oracle.quantize(cols_of(bits, lo, hi), fmt, oracle.COL)
        assert np.array_equal(host(q.codes[lo:hi]), c), (lo, hi)
        assert np.array_equal(host(q.scales[lo:hi]), s), (lo, hi)
        g4 = host(q.scales_g4[:, lo:hi, :])
        assert np.array_equal(g4.transpose(1, 0, 2).reshape(hi - lo, -1), s), (lo, hi)


def test_quantize_both_beyond_2_31_elements(big):
    snip = require_gpu()
    bits, x = big
    print("snip_quantize_both", tuple(x.shape), flush=True)
    qr, qc = snip.snip_quantize_both(x, snip.FP4, snip.FP8)
    torch.cuda.synchronize()
    check_row_output(qr, bits, oracle.FP4)
    check_col_output(qc, bits, oracle.FP8)


@pytest.mark.parametrize("fmt", [oracle.FP8, oracle.FP4])
def test_single_orientation_quantize_beyond_2_31_elements(big, fmt):
    snip = require_gpu()
    bits, x = big
    print("snip_quantize ROW", tuple(x.shape), fmt, flush=True)
    q = snip.snip_quantize(x, fmt, snip.ROW)
    torch.cuda.synchronize()
    check_row_output(q, bits, fmt)
    del q
    print("snip_quantize COL", tuple(x.shape), fmt, flush=True)
    q = snip.snip_quantize(x, fmt, snip.COL)
    torch.cuda.synchronize()
    check_col_output(q, bits, fmt)


def test_statistics_beyond_2_31_elements(big):
    snip = require_gpu()
    bits, x = big
    print("snip_quant_error_stats ROW per line", tuple(x.shape), flush=True)
    lines = torch.empty((ROWS, 3), dtype=torch.float32, device="cuda")
    tot_r = snip.snip_quant_error_stats(x, snip.ROW, per_line=lines)
    torch.cuda.synchronize()
    for lo, hi in ROW_SLABS:
        _, want = oracle.stats(rows_of(bits, lo, hi), oracle.ROW, per_line=True)
        np.testing.assert_allclose(host(lines[lo:hi]), want, rtol=1e-5)
    # the tensor is 32 copies of the block: every sum is 32 times the block's
    want_tot = REPEAT * oracle.stats(bits, oracle.ROW)
    np.testing.assert_allclose(host(tot_r), want_tot, rtol=1e-5)
    print("snip_quant_error_stats COL per line", flush=True)
    clines = torch.empty((COLS, 3), dtype=torch.float32, device="cuda")
    tot_c = snip.snip_quant_error_stats(x, snip.COL, per_line=clines)
    torch.cuda.synchronize()
    for lo, hi in COL_SLABS:
        _, want = oracle.stats(cols_of(bits, lo, hi), oracle.COL, per_line=True)
        np.testing.assert_allclose(host(clines[lo:hi]), want, rtol=1e-5)
    print("snip_quant_error_stats_both", flush=True)
    both_r, both_c = snip.snip_quant_error_stats_both(x)
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(both_r), want_tot, rtol=1e-5)
    np.testing.assert_allclose(host(both_c), host(tot_c), rtol=1e-5)
    np.testing.assert_allclose(host(both_c), host(clines).astype(np.float64).sum(axis=0), rtol=1e-5)


@pytest.mark.parametrize("fmt,R", [(oracle.FP4, 256), (oracle.FP8, 96)])
def test_gemm_output_beyond_2_31_elements(big, fmt, R):
    """Output [67584 x 32800] (2.2e9 elements): the large-tile kernel (R = 256, FP4) and the general one (R = 96)."""
    snip = require_gpu()
    bits, x = big
    J = 32800
    rng = np.random.default_rng(99)
    b_bits = wl.f32_to_bf16_bits(rng.standard_normal((J, R), dtype=np.float32) * 0.05)
    a_src = x[:, :R]                                       # strided source, ld = 32768
    print("gemm", ROWS, J, R, fmt, flush=True)
    aq = snip.snip_quantize(a_src, fmt, snip.ROW)
    bq = snip.snip_quantize(to_dev(b_bits), fmt, snip.ROW)
    plan = snip.make_plan((fmt,) * 6)
    ws = torch.empty(snip.gemm_workspace_bytes(ROWS, J), dtype=torch.uint8, device="cuda")
    nrm = torch.empty(1, dtype=torch.float64, device="cuda")
    y, _ = snip.snip_gemm_fwd_norm(plan, aq, bq, sum_sq=nrm, workspace=ws)
    torch.cuda.synchronize()
    assert y.shape == (ROWS, J) and y.numel() > 2 ** 31
    bh = oracle.fake_quant(b_bits, fmt, oracle.ROW)
    for lo, hi in [(0, 4), (65470, 65476), (ROWS - 4, ROWS)]:          # element 2^31 lies in row 65472
        want = oracle.gemm_fwd(oracle.fake_quant(np.ascontiguousarray(rows_of(bits, lo, hi)[:, :R]), fmt, oracle.ROW), bh)
        assert rel_fro(host_bf16_as_f64(y[lo:hi]), want) <= 2e-3, (lo, hi)
    # norm of the stored output: chunked sum of squares in double on the device as the reference
    stored = sum(float((y[i:i + 4096].double() ** 2).sum()) for i in range(0, ROWS, 4096))
    assert float(host(nrm)[0]) == pytest.approx(stored, rel=5e-6)


@pytest.mark.parametrize("g_bf16", [False, True])
def test_adamw_sensitivity_beyond_2_31_elements(g_bf16):
    """n = 2048 copies of a 1048584-element state plus a 5-element tail (2.1475e9 elements): the sum is 2048 times
    the block's plus the tail's."""
    snip = require_gpu()
    B, R, T = 1048584, 2048, 5
    b1, b2, eps = float(np.float32(0.9)), float(np.float32(0.999)), float(np.float32(1e-8))
    rng = np.random.default_rng(4343)
    g = (1e-3 * rng.standard_normal(B)).astype(np.float32)
    m = (0.3e-3 * rng.standard_normal(B)).astype(np.float32)
    v = (1e-6 * (0.5 + rng.random(B))).astype(np.float32)
    if g_bf16:
        g = torch.from_numpy(g).to(torch.bfloat16).float().numpy()
    want = R * oracle.adamw_sensitivity_sq(m, v, g, b1, b2, eps) + oracle.adamw_sensitivity_sq(m[:T], v[:T], g[:T], b1, b2, eps)

    def big(a, dtype):
        t = torch.from_numpy(a).cuda().to(dtype)
        return torch.cat([t.repeat(R), t[:T]])

    n = R * B + T
    assert n > 2 ** 31
    print("snip_adamw_sensitivity", n, "bf16 g" if g_bf16 else "fp32 g", flush=True)
    out = snip.snip_adamw_sensitivity(big(m, torch.float32), big(v, torch.float32),
                                      big(g, torch.bfloat16 if g_bf16 else torch.float32), b1, b2, eps)
    torch.cuda.synchronize()
    assert float(host(out)[0]) == pytest.approx(want, rel=1e-5)


def test_stochastic_rounding_positions_beyond_2_31(big):
    """Random bytes are drawn by stored position: the last stored row of either orientation lies beyond element
    2^31.  The oracle's per-element functions are composed here for sampled blocks of that row (its whole-tensor
    routine would need the whole tensor); scales equal those of nearest-even quantization."""
    snip = require_gpu()
    bits, x = big
    seed = 0x1234567887654321
    for axis, sr, sc in ((snip.ROW, ROWS, COLS), (snip.COL, COLS, ROWS)):
        print("snip_quantize_sr_fp4", axis, flush=True)
        q = snip.snip_quantize_sr_fp4(x, axis, seed=seed)
        torch.cuda.synchronize()
        r = sr - 1
        line = rows_of(bits, r, r + 1)[0] if axis == snip.ROW else cols_of(bits, r, r + 1)[:, 0]
        assert line.shape == (sc,) and r * sc > 2 ** 31
        _, want_s = oracle.quantize(line[None, :], oracle.FP4, oracle.ROW)
        assert np.array_equal(host(q.scales[r]), want_s[0])
        codes = host(q.codes[r])
        for b in (0, 1, sc // 64, sc // 32 - 1):
            scale = 2.0 ** (int(want_s[0, b]) - 127)
            for k in range(32):
                c = b * 32 + k
                v = oracle.bf16_to_f64(int(line[c])) / scale
                want = oracle.encode_sr_fp4(v, oracle.sr_byte(seed, r * sc + c))
                got = (int(codes[c // 2]) >> (4 * (c % 2))) & 0xF
                assert got == want, (axis, c)
        del q
