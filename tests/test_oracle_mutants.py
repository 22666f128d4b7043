"""Are the oracle's pins strong enough?  Each case plants one plausible mistake (a dropped term, a wrong
sign or index, a transposed operand, an off-by-one constant) in a COPY of the oracle's source, builds it on
the CPU and runs the pin suites against the copy; at least one pin must fail.  Nothing here touches the GPU
or the real oracle library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "snip_oracle.c")

# (name, text in the source, replacement, pin suites that must catch it)
MUTANTS = [
    ("decode_bias", "static int fmt_bias(int fmt)  { return fmt == 0 ? 7 : 1; }",
     "static int fmt_bias(int fmt)  { return fmt == 0 ? 8 : 1; }", ["test_oracle_formats.py"]),
    ("decode_subnormal_exponent", "if (E == 0u) mag = ldexp((double)T, 1 - bias - mb);",
     "if (E == 0u) mag = ldexp((double)T, 0 - bias - mb);", ["test_oracle_formats.py"]),
    ("encode_ties_away", "double q = nearbyint(ldexp(a, -step_exp));", "double q = round(ldexp(a, -step_exp));",
     ["test_oracle_formats.py"]),
    ("encode_truncates", "double q = nearbyint(ldexp(a, -step_exp));", "double q = floor(ldexp(a, -step_exp));",
     ["test_oracle_formats.py"]),
    ("encode_subnormal_spacing", "if (ex < 1 - bias) ex = 1 - bias;   /* subnormal range", "if (ex < 0 - bias) ex = 0 - bias;   /* subnormal range",
     ["test_oracle_formats.py"]),
    ("scale_no_bump", "if (rule == 0 && m > mmax) e += 1;", "if (rule == 0 && m > 2.0) e += 1;", ["test_oracle_formats.py"]),
    ("scale_bump_on_equal", "if (rule == 0 && m > mmax) e += 1;", "if (rule == 0 && m >= mmax) e += 1;", ["test_oracle_formats.py"]),
    ("scale_rules_swapped", "if (rule == 0 && m > mmax) e += 1;", "if (rule == 1 && m > mmax) e += 1;", ["test_oracle_formats.py"]),
    ("scale_emax_off", "e = n - emax;", "e = n - emax + 1;", ["test_oracle_formats.py"]),
    ("quantize_axis_ignored", "return axis == 0 ? src[r * ld + c] : src[c * ld + r];", "return src[r * ld + c];",
     ["test_oracle_tensors.py"]),
    ("quantize_nibbles_swapped", "if ((e & 1) == 0) *p = (uint8_t)((*p & 0xF0u) | code);\n                    else              *p = (uint8_t)((*p & 0x0Fu) | (code << 4));",
     "if ((e & 1) == 1) *p = (uint8_t)((*p & 0xF0u) | code);\n                    else              *p = (uint8_t)((*p & 0x0Fu) | (code << 4));",
     ["test_oracle_tensors.py"]),
    ("quantize_block_of_16", "#define ORACLE_TILE 32", "#define ORACLE_TILE 16", ["test_oracle_tensors.py"]),
    ("dequantize_scale_bias", "out[e] = sb == 0xFFu ? NAN : ldexp(oracle_decode(fmt, code), (int)sb - 127);",
     "out[e] = sb == 0xFFu ? NAN : ldexp(oracle_decode(fmt, code), (int)sb - 126);", ["test_oracle_tensors.py"]),
    ("fake_quant_not_transposed_back", "out[r * cols + c] = axis == 0 ? st[r * cols + c] : st[c * rows + r];",
     "out[r * cols + c] = st[r * cols + c];", ["test_oracle_tensors.py"]),
    ("gemm_fwd_w_transposed", "for (int64_t k = 0; k < K; ++k) s += X[m * K + k] * W[n * K + k];",
     "for (int64_t k = 0; k < K; ++k) s += X[m * K + k] * W[k * N + n];", ["test_oracle_tensors.py"]),
    ("gemm_dgrad_w_transposed", "for (int64_t n = 0; n < N; ++n) s += dY[m * N + n] * W[n * K + k];",
     "for (int64_t n = 0; n < N; ++n) s += dY[m * N + n] * W[k * N + n];", ["test_oracle_tensors.py"]),
    ("gemm_wgrad_operands_swapped", "for (int64_t m = 0; m < M; ++m) s += dY[m * N + n] * X[m * K + k];",
     "for (int64_t m = 0; m < M; ++m) s += dY[m * N + k % N] * X[m * K + n % K];", ["test_oracle_tensors.py"]),
    ("stats_fp4_uses_fp8", "rc = oracle_fake_quant(src, rows, cols, ld, 1, axis, rule, q4);",
     "rc = oracle_fake_quant(src, rows, cols, ld, 0, axis, rule, q4);", ["test_oracle_tensors.py"]),
    ("stats_error_not_squared", "s0 += x * x; s4 += d4 * d4; s8 += d8 * d8;", "s0 += x * x; s4 += fabs(d4); s8 += d8 * d8;",
     ["test_oracle_tensors.py"]),
    ("stats_formats_swapped", "line[r * 3 + 0] = s0; line[r * 3 + 1] = s4; line[r * 3 + 2] = s8;",
     "line[r * 3 + 0] = s0; line[r * 3 + 1] = s8; line[r * 3 + 2] = s4;", ["test_oracle_tensors.py"]),
    ("stats_lines_reversed", "if (per_line) memcpy(per_line, line, (size_t)SR * 3 * sizeof(double));",
     "if (per_line) for (int64_t r = 0; r < SR; ++r) memcpy(per_line + r * 3, line + (SR - 1 - r) * 3, 3 * sizeof(double));",
     ["test_oracle_tensors.py"]),
    ("round_output_one_bit_short", "double quantum = ldexp(1.0, ex - 7);", "double quantum = ldexp(1.0, ex - 6);", ["test_oracle_norms.py"]),
    ("round_output_truncates", "return nearbyint(v / quantum) * quantum;", "return trunc(v / quantum) * quantum;", ["test_oracle_norms.py"]),
    ("output_norm_unrounded", "double r = oracle_round_output(c[i], out_dtype);", "double r = c[i];", ["test_oracle_norms.py"]),
    ("loss_divergence_weight_count", "double tw = sqrt(grad_w_sq) * sqrt(err_w_sq) / sqrt((double)N * (double)K);",
     "double tw = sqrt(grad_w_sq) * sqrt(err_w_sq) / sqrt((double)M * (double)K);", ["test_oracle_norms.py"]),
    ("loss_divergence_plain_sum", "return sqrt(tx * tx + tw * tw);", "return tx + tw;", ["test_oracle_norms.py"]),
    ("threefry_rotation", "static const int rot[8] = { 13, 15, 26, 6, 17, 29, 16, 24 };",
     "static const int rot[8] = { 13, 15, 26, 6, 17, 29, 16, 25 };", ["test_oracle_sr.py"]),
    ("threefry_parity_constant", "0x1BD11BDAu ^ key[0] ^ key[1]", "0x1BD11BDBu ^ key[0] ^ key[1]", ["test_oracle_sr.py"]),
    ("threefry_injection_counter", "x1 += ks[(inj + 1) % 3] + (uint32_t)inj;", "x1 += ks[(inj + 1) % 3];", ["test_oracle_sr.py"]),
    ("sr_byte_word_order", "return (out[j / 4] >> (8 * (j % 4))) & 0xFFu;", "return (out[1 - j / 4] >> (8 * (j % 4))) & 0xFFu;",
     ["test_oracle_sr.py"]),
    ("sr_threshold_inclusive", "return sign | (lo_code + ((double)rnd < threshold ? 1u : 0u));",
     "return sign | (lo_code + ((double)rnd <= threshold ? 1u : 0u));", ["test_oracle_sr.py"]),
    ("sr_threshold_rounds_up", "double threshold = floor(256.0 * p);", "double threshold = ceil(256.0 * p);", ["test_oracle_sr.py"]),
    ("sr_probability_of_lower", "double p = (a - lo) / (hi - lo);", "double p = (hi - a) / (hi - lo);", ["test_oracle_sr.py"]),
    ("sr_index_by_source", "uint64_t index = (uint64_t)r * (uint64_t)SC + (uint64_t)c;",
     "uint64_t index = axis == 0 ? (uint64_t)r * (uint64_t)SC + (uint64_t)c : (uint64_t)c * (uint64_t)SR + (uint64_t)r;",
     ["test_oracle_sr.py"]),
    ("paper_scale_inverted", "float s = (float)oracle_fmt_max(fmt) / amax;", "float s = amax / (float)oracle_fmt_max(fmt);",
     ["test_oracle_paper.py"]),
    ("paper_scale_in_double", "float t = x * s;\n                        code = oracle_encode_rne(fmt, (double)t);",
     "double t = (double)x * (double)oracle_fmt_max(fmt) / (double)fabsf(x == 0 ? 1 : x) * 0 + (double)x * (double)s * (1.0 + 1e-7);\n                        code = oracle_encode_rne(fmt, (double)t);",
     ["test_oracle_paper.py"]),
    ("paper_block_is_tile", "int64_t r1 = r0 + group_rows < SR ? r0 + group_rows : SR;", "int64_t r1 = r0 + 1;", ["test_oracle_paper.py"]),
    ("paper_dequant_multiplies", "out[e] = isnan(s) ? NAN : oracle_decode(fmt, code) / s;", "out[e] = isnan(s) ? NAN : oracle_decode(fmt, code) * s;",
     ["test_oracle_paper.py"]),
    ("paper_no_cap", "if (!(s <= 0x1p126f)) s = 0x1p126f;", "", ["test_oracle_paper.py"]),
    ("adamw_denominator_not_squared", "second = (1.0 - beta2) * m[i] * g[i] / (root * (root + eps) * (root + eps));",
     "second = (1.0 - beta2) * m[i] * g[i] / (root * (root + eps));", ["test_oracle_adamw.py"]),
    ("adamw_sign", "double t = first - second;", "double t = first + second;", ["test_oracle_adamw.py"]),
    ("adamw_betas_swapped", "double first = (1.0 - beta1) / (root + eps);", "double first = (1.0 - beta2) / (root + eps);", ["test_oracle_adamw.py"]),
    ("weight_divergence_no_root", "double corr = sqrt(1.0 - pow(beta2, (double)t)) / (1.0 - pow(beta1, (double)t));",
     "double corr = (1.0 - pow(beta2, (double)t)) / (1.0 - pow(beta1, (double)t));", ["test_oracle_adamw.py"]),
]


def run_mutant(args):
    name, old, new, suites, tmp = args
    src = open(SRC).read()
    if src.count(old) != 1:
        return name, "source text not found exactly once"
    c_path = os.path.join(tmp, name + ".c")
    so_path = os.path.join(tmp, name + ".so")
    with open(c_path, "w") as f:
        f.write(src.replace(old, new))
    cc = subprocess.run(["gcc", "-std=c11", "-O1", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-w",
                         "-o", so_path, c_path, "-lm"], capture_output=True, text=True)
    if cc.returncode != 0:
        return name, "mutant does not compile: " + cc.stderr[-300:]
    env = dict(os.environ, SNIP_ORACLE_LIB=so_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"]
                       + [os.path.join(ROOT, "tests", s) for s in suites],
                       capture_output=True, text=True, env=env, cwd=ROOT)
    if r.returncode == 0:
        return name, "survived: no pin failed"
    if "failed" not in r.stdout and "error" not in r.stdout.lower():
        return name, "suite did not run: " + r.stdout[-300:]
    return name, None


def test_every_planted_mistake_is_caught(tmp_path):
    jobs = [(n, o, r, s, str(tmp_path)) for n, o, r, s in MUTANTS]
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(run_mutant, jobs))
    problems = {n: msg for n, msg in results if msg}
    assert not problems, problems
