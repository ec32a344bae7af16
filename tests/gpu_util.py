"""Helpers shared by the GPU parity tests: host<->device conversion and the parity metric."""
import os

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
    if os.environ.get("GNN_PARITY_REPORT"):      # survey mode: print every figure, judge nothing
        print(f"PARITY {what}: rel err {e:.3e} (bar {TOL[dtype] * calls:.0e})", flush=True)
        return e
    assert e <= TOL[dtype] * calls, f"{what}: rel err {e:.3e} > {TOL[dtype] * calls:.0e}"
    return e


def backward_at_the_oracles_point(m, om, dims, dtype, labels_dev):
    """Whole-model backward parity, element by element.

    A ReLU unit whose pre-activation is zero to within the forward rounding error may come out on either side of zero
    on the GPU (fp32 / bf16 accumulation) and in the oracle (fp64): its gradient then differs by the unit's WHOLE
    upstream gradient, and with a fraction f of such units a weight-gradient element is off by about sqrt(2 f) of its
    rms - 5 % for f = 1e-3, which is what bf16 storage gives - although every kernel is exact to rounding.  The
    decision "is this unit active" therefore has to be taken alike on both sides: the GPU model's stored activations
    (A_l, H_l; for the residual model also the pre-activations) are overwritten with the ORACLE's, rounded to the
    storage type, the loss gradient is recomputed from the oracle's logits, and only then the GPU runs its backward
    pass.  Forward parity is checked before, on the GPU's own activations.  Nothing of the GPU flows into the oracle."""
    import paper_2311_06837_amd as P
    L = m.L
    with torch.no_grad():
        for l in range(1, L + 1):
            rows = torch.from_numpy(np.asarray(om.rows_of_layer(l), dtype=np.int64)).cuda()
            m.H[l][rows, : dims[l]] = dev(as_stored(om.H[l][om.rows_of_layer(l)], dtype), dtype)
            A = getattr(m, "A", None)
            if A is not None and l < len(A) and A[l] is not None and not getattr(m, "recompute", False):
                A[l][rows, : dims[l - 1]] = dev(as_stored(om.A[l][om.rows_of_layer(l)], dtype), dtype)
            T = getattr(m, "T", None)
            if T is not None and l >= 2 and l < len(T) and T[l] is not None and not getattr(m, "recompute", False):
                prev = torch.from_numpy(np.asarray(om.rows_of_layer(l - 1), dtype=np.int64)).cuda()
                T[l][prev, : dims[l - 1]] = dev(as_stored(om.T[l][om.rows_of_layer(l - 1)], dtype), dtype)
    nt = m.n_rows_of_layer(L)
    dlogits = m.dH[L] if isinstance(m.dH, list) and len(m.dH) > L else m.dlogits
    P.gnn_softmax_ce(m.rows, nt, m.H[L], dims[L], labels_dev, dlogits, m.loss, ws=m.ws)
    m.backward()
    torch.cuda.synchronize()
