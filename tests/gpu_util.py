"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import pytest
import torch


def require_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_01410_amd import snip
    snip._lib()          # raises if the HIP library has not been built: no fallback
    return snip


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns (uint16) -> CUDA bf16 tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def host_bf16_as_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    d = np.linalg.norm(got.astype(np.float64) - want)
    n = np.linalg.norm(want)
    return float(d / n) if n > 0 else float(d)
