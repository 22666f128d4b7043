"""Seeded synthetic workloads: Llama-shaped linear layers, their tensors and precision plans.

This module holds no arithmetic of the method (no quantization, no GEMM, no statistics).
It only names shapes, draws seeded random tensors and rounds them to bf16 bit patterns, and
draws seeded precision plans.  Both the CPU oracle's tests and the GPU path read their
inputs from here so that they see the same bits.

The tensors stand in for the activations X [M, K], weights W [N, K] and output gradients
dY [M, N] of the seven linear layers of a Llama-style transformer block (q, k, v, o, gate,
up, down; SNIP Sec. 2.1), which the paper trains on real corpora that are not needed here.
Distribution parameters are standard deviations.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

FP8, FP4 = 0, 1
GEMMS = ("fwd", "dgrad", "wgrad")
_CHUNK_ROWS_ELEMS = 1 << 22      # elements per independently seeded chunk


@dataclass(frozen=True)
class Linear:
    name: str
    N: int          # output features
    K: int          # input features
    x_group: str    # linears with the same group read the same activation tensor


@dataclass(frozen=True)
class Config:
    index: int                  # 1-based, as in the configuration list
    name: str
    M: int                      # tokens
    linears: Tuple[Linear, ...]
    x_dist: str                 # "normal" | "student_t3" | "normal_outliers"
    w_std: float
    dy_std: float
    plans: Tuple[str, ...]      # plan names runnable on this config

    def flops(self) -> int:
        """2*M*N*K for each of the three GEMMs of every linear."""
        return sum(3 * 2 * self.M * l.N * l.K for l in self.linears)


def _llama(hidden: int, kv: int, inter: int) -> Tuple[Linear, ...]:
    return (
        Linear("q", hidden, hidden, "attn_in"),
        Linear("k", kv, hidden, "attn_in"),
        Linear("v", kv, hidden, "attn_in"),
        Linear("o", hidden, hidden, "o_in"),
        Linear("gate", inter, hidden, "mlp_in"),
        Linear("up", inter, hidden, "mlp_in"),
        Linear("down", hidden, inter, "down_in"),
    )


CONFIGS: Dict[int, Config] = {
    1: Config(1, "single-512", 256, (Linear("lin", 512, 512, "x"),), "normal", 0.02, 1e-3,
              ("fp8",)),
    2: Config(2, "llama-1b-layer", 4096, _llama(2048, 2048, 8192), "normal", 0.02, 1e-4,
              ("fp4",)),
    3: Config(3, "llama-3b-layer", 8192, _llama(3072, 1024, 8192), "normal_outliers", 0.02, 1e-4,
              ("mix60",)),
    4: Config(4, "llama-7b-layer", 16384, _llama(4096, 4096, 11008), "student_t3", 0.02, 1e-5,
              ("fp4", "fp8", "mix50")),
    5: Config(5, "llama-70b-layer", 8192, _llama(8192, 1024, 28672), "normal", 0.02, 1e-4,
              ("mix50",)),
}

TENSOR_ID = {"X": 0, "W": 1, "dY": 2}


def tensor_seed(config: int, linear_index: int, tensor: str) -> int:
    return 1000 * config + 10 * linear_index + TENSOR_ID[tensor]


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = ((u + (0x7FFF + ((u >> 16) & 1))) >> 16).astype(np.uint16)
    r[nan] = 0x7FC0
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _draw_chunk(seed: int, chunk: int, rows: int, cols: int, dist: str, std: float) -> np.ndarray:
    rng = np.random.default_rng([seed, chunk])
    if dist == "student_t3":
        a = rng.standard_t(3.0, size=(rows, cols)).astype(np.float32)
    else:
        a = rng.standard_normal(size=(rows, cols), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def draw_bf16(seed: int, rows: int, cols: int, dist: str = "normal", std: float = 1.0,
              row_start: int = 0, row_stop: int | None = None, workers: int = 8) -> np.ndarray:
    """Seeded [rows, cols] tensor as bf16 bits.  The tensor is drawn in row chunks, each from
    its own stream (seed, chunk), so that any row range [row_start, row_stop) can be produced
    without drawing the rest and chunks can be drawn in parallel.

    dist "normal_outliers": N(0, std) with a seeded 1% of the columns multiplied by 20.
    """
    row_stop = rows if row_stop is None else row_stop
    rows_per_chunk = max(1, _CHUNK_ROWS_ELEMS // max(cols, 1))
    base = "normal" if dist == "normal_outliers" else dist
    first, last = row_start // rows_per_chunk, (max(row_stop, row_start + 1) - 1) // rows_per_chunk
    jobs = []
    for c in range(first, last + 1):
        r0 = c * rows_per_chunk
        jobs.append((c, min(rows_per_chunk, rows - r0)))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        parts = list(pool.map(lambda j: _draw_chunk(seed, j[0], j[1], cols, base, std), jobs))
    a = np.concatenate(parts, axis=0) if len(parts) > 1 else parts[0]
    off = first * rows_per_chunk
    a = a[row_start - off: row_stop - off]
    if dist == "normal_outliers":
        crng = np.random.default_rng([seed, 1 << 30])
        n_out = max(1, cols // 100)
        out_cols = crng.choice(cols, size=n_out, replace=False)
        a = a.copy()
        a[:, out_cols] *= np.float32(20.0)
    return f32_to_bf16_bits(a)


@dataclass
class LayerTensors:
    """bf16 bit patterns of one configuration's tensors."""
    config: Config
    X: Dict[str, np.ndarray] = field(default_factory=dict)    # by x_group, [M, K]
    W: Dict[str, np.ndarray] = field(default_factory=dict)    # by linear name, [N, K]
    dY: Dict[str, np.ndarray] = field(default_factory=dict)   # by linear name, [M, N]


def x_seed(cfg: Config, group: str) -> int:
    """An activation tensor shared by several linears takes the seed of the first of them."""
    for i, l in enumerate(cfg.linears):
        if l.x_group == group:
            return tensor_seed(cfg.index, i, "X")
    raise KeyError(group)


def make_tensor(cfg: Config, kind: str, key: str, row_start: int = 0,
                row_stop: int | None = None) -> np.ndarray:
    """One tensor of a configuration (or a row range of it): kind 'X' (key = x_group),
    'W' or 'dY' (key = linear name)."""
    if kind == "X":
        lin = next(l for l in cfg.linears if l.x_group == key)
        return draw_bf16(x_seed(cfg, key), cfg.M, lin.K, cfg.x_dist, 1.0, row_start, row_stop)
    idx = next(i for i, l in enumerate(cfg.linears) if l.name == key)
    lin = cfg.linears[idx]
    if kind == "W":
        return draw_bf16(tensor_seed(cfg.index, idx, "W"), lin.N, lin.K, "normal", cfg.w_std,
                         row_start, row_stop)
    if kind == "dY":
        return draw_bf16(tensor_seed(cfg.index, idx, "dY"), cfg.M, lin.N, "normal", cfg.dy_std,
                         row_start, row_stop)
    raise KeyError(kind)


def make_optimizer_state(cfg: Config, name: str, beta1: float = 0.9, beta2: float = 0.999):
    """Synthetic AdamW state of one linear's weight after an update: (m, v, g) as float32 [N, K].

    g ~ N(0, s) with s = dy_std * sqrt(M) (the scale of dW = dY^T X for unit-variance inputs); the previous
    moments are those of a stationary run with the same gradient scale, m' ~ N(0, s sqrt((1-b1)/(1+b1))),
    v' = s^2 (1 + 0.05 N(0,1)) kept positive; m and v are the moments after this step's update.  A recipe
    for inputs only: it stands in for the optimizer state of the paper's training runs."""
    idx = next(i for i, l in enumerate(cfg.linears) if l.name == name)
    lin = cfg.linears[idx]
    rng = np.random.default_rng([tensor_seed(cfg.index, idx, "W"), 4242])
    s = cfg.dy_std * float(np.sqrt(cfg.M))
    shape = (lin.N, lin.K)
    g = (s * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    m_prev = (s * np.sqrt((1 - beta1) / (1 + beta1)) * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    v_prev = (s * s * np.maximum(1.0 + 0.05 * rng.standard_normal(shape, dtype=np.float32), 0.05)).astype(np.float32)
    m = (beta1 * m_prev + (1 - beta1) * g).astype(np.float32)
    v = (beta2 * v_prev + (1 - beta2) * g * g).astype(np.float32)
    return m, v, g


def make_layer(cfg: Config) -> LayerTensors:
    t = LayerTensors(cfg)
    for l in cfg.linears:
        if l.x_group not in t.X:
            t.X[l.x_group] = make_tensor(cfg, "X", l.x_group)
        t.W[l.name] = make_tensor(cfg, "W", l.name)
        t.dY[l.name] = make_tensor(cfg, "dY", l.name)
    return t


# ---- precision plans -----------------------------------------------------------------
# A plan gives, for every linear, the element format of each operand of each GEMM:
# (fwd_x, fwd_w, dgrad_dy, dgrad_w, wgrad_dy, wgrad_x).  The measured plans choose one
# format per (linear, GEMM) for both operands, so "FP4 FLOPs" is well defined
# (SNIP Sec. 4.1: efficiency = fraction of linear-layer FLOPs run in FP4).

PlanEntry = Tuple[int, int, int, int, int, int]


def make_plan(cfg: Config, name: str) -> List[PlanEntry]:
    n = len(cfg.linears)
    if name == "fp4":
        return [(FP4,) * 6] * n
    if name == "fp8":
        return [(FP8,) * 6] * n
    if name.startswith("mix"):
        p_fp4 = int(name[3:]) / 100.0
        rng = np.random.default_rng(7000 + cfg.index)
        u = rng.random(size=(n, 3))
        plan = []
        for i in range(n):
            f = [FP4 if u[i, g] < p_fp4 else FP8 for g in range(3)]
            plan.append((f[0], f[0], f[1], f[1], f[2], f[2]))
        return plan
    if name.startswith("tensor"):
        # the paper's per-tensor option (Sec. 4.2): one format each for inputs, weights and
        # gradients, shared by the GEMMs that read them; operands of one GEMM may differ
        rng = np.random.default_rng(7100 + cfg.index)
        u = rng.random(size=(n, 3))
        plan = []
        for i in range(n):
            fx, fw, fg = (FP4 if u[i, j] < 0.5 else FP8 for j in range(3))
            plan.append((fx, fw, fg, fw, fg, fx))
        return plan
    raise KeyError(name)


def gemm_flops(cfg: Config, lin: Linear) -> int:
    return 2 * cfg.M * lin.N * lin.K


def plan_fp4_fraction(cfg: Config, plan: List[PlanEntry]) -> float:
    """Fraction of the layer's GEMM FLOPs whose two operands are both FP4."""
    tot = fp4 = 0
    for lin, e in zip(cfg.linears, plan):
        f = gemm_flops(cfg, lin)
        for g in range(3):
            tot += f
            if e[2 * g] == FP4 and e[2 * g + 1] == FP4:
                fp4 += f
    return fp4 / tot


def plan_peak_flops(cfg: Config, plan: List[PlanEntry], peak_fp4: float, peak_fp8: float) -> float:
    """FLOP-weighted harmonic mean of the per-GEMM matrix-core peaks: a GEMM runs at the
    FP4 rate only when both of its operands are FP4."""
    tot = t = 0.0
    for lin, e in zip(cfg.linears, plan):
        f = gemm_flops(cfg, lin)
        for g in range(3):
            both4 = e[2 * g] == FP4 and e[2 * g + 1] == FP4
            tot += f
            t += f / (peak_fp4 if both4 else peak_fp8)
    return tot / t
