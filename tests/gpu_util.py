"""Helpers shared by the GPU parity tests: host<->device conversion and the parity metric."""
import numpy as np
import torch

import oracle
from conftest import rel_err

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}   # relative-error bars: fp32 arithmetic, bf16 storage


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def padded(a: np.ndarray, ld: int, dtype, fill=0.0) -> torch.Tensor:
    """Device matrix [n, ld] of `dtype` holding `a` in its first columns (pad = fill)."""
    n, f = a.shape
    t = torch.full((n, ld), fill, dtype=dtype, device="cuda")
    t[:, :f] = torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)
    return t


def host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def as_stored(a: np.ndarray, dtype) -> np.ndarray:
    """float64 copy of `a` holding exactly the values the device stores for `dtype`."""
    x = np.array(a, dtype=np.float32).astype(np.float64)
    return oracle.round_bf16(np.ascontiguousarray(x)) if dtype == torch.bfloat16 else x


def check(got, want, dtype, what="", calls=1):
    """Parity bar of one kernel call; `calls` > 1 when the compared value went through that many
    chained calls, each with its own rounding (whole-model tests)."""
    e = rel_err(got, want)
    assert e <= TOL[dtype] * calls, f"{what}: rel err {e:.3e} > {TOL[dtype] * calls:.0e}"
    return e
