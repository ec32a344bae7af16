"""Pins of the oracle's per-step arithmetic: dense brute force (a textbook matmul), closed
forms and library routines.  Section 2.1 (layer equation)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle


def _dense(g):
    return g.to_scipy().toarray().astype(np.float64)      # A[v,u] = 1 iff v aggregates u


@pytest.mark.parametrize("seed", [0, 1])
@pytest.mark.parametrize("directed", [False, True])
def test_spmm_fwd_equals_dense_matmul(seed, directed):
    n, F = 150, 7
    g = gg.random_directed(n, 4.0, seed) if directed else gg.erdos_renyi(n, 5.0, seed)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F))
    rs, cs = rng.random(n) + 0.5, rng.random(n) + 0.5
    rows = np.sort(rng.choice(n, size=60, replace=False)).astype(np.int32)
    Y = np.full((n, F), 777.0)
    oracle.spmm_fwd(g.row_ptr, g.col_idx, rows, X, Y, F, rs, cs)
    want = np.diag(rs) @ _dense(g) @ np.diag(cs) @ X
    assert np.allclose(Y[rows], want[rows], rtol=1e-13, atol=1e-13)
    mask = np.ones(n, dtype=bool)
    mask[rows] = False
    assert (Y[mask] == 777.0).all()                       # masked rows are not written
    # no scale vectors = plain sum
    Y2 = np.zeros((n, F))
    oracle.spmm_fwd(g.row_ptr, g.col_idx, None, X, Y2, F)
    assert np.allclose(Y2, _dense(g) @ X, rtol=1e-13, atol=1e-13)


def test_spmm_partial_width_and_leading_dimension():
    n = 40
    g = gg.erdos_renyi(n, 4.0, 3)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((n, 10))
    Y = np.full((n, 12), -5.0)
    oracle.spmm_fwd(g.row_ptr, g.col_idx, None, X, Y, 6)   # only 6 of X's 10 columns
    assert np.allclose(Y[:, :6], _dense(g) @ X[:, :6])
    assert (Y[:, 6:] == -5.0).all()


def test_sum_of_ones_is_the_row_length():
    g = gg.chung_lu(300, 8.0, 2.1, 5)
    Y = np.zeros((300, 3))
    oracle.spmm_fwd(g.row_ptr, g.col_idx, None, np.ones((300, 3)), Y, 3)
    assert np.array_equal(Y, np.repeat(g.degrees()[:, None], 3, axis=1).astype(np.float64))


def test_mean_preserves_constants_and_empty_rows_give_zero():
    g = gg.random_directed(200, 1.5, 6)                   # has empty rows
    deg = g.degrees()
    assert (deg == 0).any()
    rs = oracle.norm_scales("mean", deg)
    X = np.tile(np.array([3.25, -1.5]), (200, 1))
    Y = np.full((200, 2), np.nan)
    oracle.spmm_fwd(g.row_ptr, g.col_idx, None, X, Y, 2, rs, None)
    assert np.allclose(Y[deg > 0], X[deg > 0], rtol=1e-14)
    assert (Y[deg == 0] == 0.0).all()


def test_norm_scales_closed_form():
    deg = np.array([0, 1, 4, 9, 16], dtype=np.int32)
    assert np.array_equal(oracle.norm_scales("mean", deg), [0, 1, 0.25, 1 / 9, 1 / 16])
    assert np.allclose(oracle.norm_scales("sym", deg), [0, 1, 0.5, 1 / 3, 0.25], rtol=1e-15)


@pytest.mark.parametrize("seed", [0, 1])
def test_spmm_bwd_is_the_adjoint(seed):
    # <Y, dY> over the active rows == <X, dX>  for the linear map X -> Y
    n, F = 90, 5
    g = gg.random_directed(n, 3.0, seed)
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(n, size=40, replace=False)).astype(np.int32)
    rs, cs = rng.random(n) + 0.5, rng.random(n) + 0.5
    X, dY = rng.standard_normal((n, F)), rng.standard_normal((n, F))
    Y = np.zeros((n, F))
    oracle.spmm_fwd(g.row_ptr, g.col_idx, rows, X, Y, F, rs, cs)
    dX = np.zeros((n, F))
    oracle.spmm_bwd(g.row_ptr, g.col_idx, rows, dY, dX, F, rs, cs)
    assert np.isclose((Y[rows] * dY[rows]).sum(), (X * dX).sum(), rtol=1e-12)
    # and equals the dense transpose with the row mask
    M = np.zeros(n)
    M[rows] = 1
    want = (np.diag(M) @ np.diag(rs) @ _dense(g) @ np.diag(cs)).T @ dY
    assert np.allclose(dX, want, rtol=1e-12, atol=1e-12)
    # accumulates
    oracle.spmm_bwd(g.row_ptr, g.col_idx, rows, dY, dX, F, rs, cs)
    assert np.allclose(dX, 2 * want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("sage", [False, True])
@pytest.mark.parametrize("relu", [False, True])
def test_linear_fwd_equals_numpy_matmul(sage, relu):
    rng = np.random.default_rng(7)
    n, K, N = 50, 9, 6
    A, Xs = rng.standard_normal((n, K)), rng.standard_normal((n, K))
    Wn, Ws, b = rng.standard_normal((K, N)), rng.standard_normal((K, N)), rng.standard_normal(N)
    rows = np.array([3, 4, 10, 49, 0], dtype=np.int32)
    H = np.full((n, N), 9.0)
    oracle.linear_fwd(rows, A, Xs if sage else None, K, Wn, Ws if sage else None, b, H, relu)
    want = A @ Wn + b + (Xs @ Ws if sage else 0)
    if relu:
        want = np.maximum(want, 0)
    assert np.allclose(H[rows], want[rows], rtol=1e-13, atol=1e-13)
    rest = np.setdiff1d(np.arange(n), rows)
    assert (H[rest] == 9.0).all()


@pytest.mark.parametrize("relu", [False, True])
def test_linear_bwd_equals_numpy_matmul(relu):
    rng = np.random.default_rng(8)
    n, K, N = 40, 7, 5
    A, Xs = rng.standard_normal((n, K)), rng.standard_normal((n, K))
    Wn, Ws = rng.standard_normal((K, N)), rng.standard_normal((K, N))
    H = rng.standard_normal((n, N))
    dH = rng.standard_normal((n, N))
    rows = np.sort(rng.choice(n, size=17, replace=False)).astype(np.int32)
    dA, dXs = np.full((n, K), 5.0), np.full((n, K), 5.0)
    dWn, dWs, db = oracle.linear_bwd(rows, dH, H if relu else None, relu, A, Xs, K, Wn, Ws, dA, dXs)
    dZ = dH[rows] * (H[rows] > 0) if relu else dH[rows]
    assert np.allclose(dWn, A[rows].T @ dZ) and np.allclose(dWs, Xs[rows].T @ dZ)
    assert np.allclose(db, dZ.sum(0))
    assert np.allclose(dA[rows], dZ @ Wn.T) and np.allclose(dXs[rows], dZ @ Ws.T)
    rest = np.setdiff1d(np.arange(n), rows)
    assert (dA[rest] == 5.0).all() and (dXs[rest] == 5.0).all()


def test_softmax_ce_equals_library_cross_entropy():
    rng = np.random.default_rng(9)
    n, Cn = 30, 11
    Z = rng.standard_normal((n, Cn)) * 4
    rows = np.sort(rng.choice(n, size=12, replace=False)).astype(np.int32)
    y = rng.integers(0, Cn, size=12).astype(np.int32)
    dZ = np.full((n, Cn), 3.0)
    loss = oracle.softmax_ce(rows, Z, Cn, y, dZ)
    zt = torch.tensor(Z[rows], dtype=torch.float64, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(y, dtype=torch.int64))
    lt.backward()
    assert np.isclose(loss, lt.item(), rtol=1e-13)
    assert np.allclose(dZ[rows], zt.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert (dZ[np.setdiff1d(np.arange(n), rows)] == 3.0).all()
    # closed form: uniform logits -> log C
    assert np.isclose(oracle.softmax_ce(None, np.zeros((4, Cn)), Cn, np.zeros(4, dtype=np.int32)), np.log(Cn))


def test_bf16_rounding_equals_library_conversion_and_ties_to_even():
    rng = np.random.default_rng(10)
    x = np.concatenate([rng.standard_normal(5000) * np.exp(rng.uniform(-20, 20, 5000)),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 3.3895313892515355e38]])
    want = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_bf16(x.astype(np.float32).astype(np.float64))
    assert np.array_equal(got, want)
    # 1 + 2^-8 lies half-way between 1 and 1 + 2^-7: even mantissa wins -> 1.0 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_bf16(np.array([1.00390625]))[0] == 1.0
    assert oracle.round_bf16(np.array([1.01171875]))[0] == 1.015625
