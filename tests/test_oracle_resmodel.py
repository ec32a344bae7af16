"""Pins of the oracle's deep residual GraphSAGE (ResSAGE+ of section 8.1: GraphSAGE layers with residual connections
and pre-activation): the pre-activation against torch's layer_norm / relu and autograd on the CPU (a library routine),
the whole model against a dense numpy re-derivation and central finite differences, and the paper's invariant that the
masked model gives the targets the unmasked / unpartitioned result."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

import graphgen as gg
import oracle


def test_pre_activation_against_torch_layer_norm_and_autograd():
    rng = np.random.default_rng(0)
    n, F = 50, 13
    X = rng.standard_normal((n, F)) * 2 + 0.5
    gamma, beta = 1 + 0.3 * rng.standard_normal(F), 0.2 * rng.standard_normal(F)
    rows = np.sort(rng.choice(n, 31, replace=False)).astype(np.int32)
    Y = np.full((n, F), np.nan)
    oracle.ln_relu_fwd(rows, X, F, gamma, beta, Y)
    xt = torch.tensor(X[rows], dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(beta, dtype=torch.float64, requires_grad=True)
    yt = torch.relu(torch.nn.functional.layer_norm(xt, (F,), gt, bt, eps=oracle.LN_EPS))
    assert np.allclose(Y[rows], yt.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.isnan(Y[np.setdiff1d(np.arange(n), rows)]).all()
    dY = rng.standard_normal((n, F))
    yt.backward(torch.tensor(dY[rows]))
    dX = np.full((n, F), np.nan)
    dg, db = oracle.ln_relu_bwd(rows, dY, Y, X, F, gamma, dX)
    assert np.allclose(dX[rows], xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dg, gt.grad.numpy(), rtol=1e-10, atol=1e-12) and np.allclose(db, bt.grad.numpy(), rtol=1e-10, atol=1e-12)
    # closed forms: a constant row normalises to zero -> ReLU(beta); the output does not change under x -> a*x + c
    Xc = np.full((3, F), 7.0)
    Yc = np.zeros((3, F))
    oracle.ln_relu_fwd(None, Xc, F, gamma, beta, Yc)
    assert np.allclose(Yc, np.maximum(beta, 0)[None, :])
    Y2 = np.zeros((n, F))
    oracle.ln_relu_fwd(None, 3.0 * X + 11.0, F, gamma, beta, Y2, eps=0.0)
    Y1 = np.zeros((n, F))
    oracle.ln_relu_fwd(None, X, F, gamma, beta, Y1, eps=0.0)
    assert np.allclose(Y1, Y2, rtol=1e-9, atol=1e-11)


def _dense_forward(g, T, params, H0, y, masked=True):
    n, L = g.n_rows, len(params)
    A = g.to_scipy().toarray().astype(np.float64)
    deg = A.sum(1)
    Ahat = np.where(deg > 0, 1 / np.maximum(deg, 1), 0)[:, None] * A
    dist = np.full(n, -1)
    dist[T] = 0
    reach = dist >= 0
    for j in range(1, L + 1):
        new = ((A.T @ reach.astype(np.float64)) > 0) & ~reach
        dist[new] = j
        reach |= new
    H = np.array(H0, dtype=np.float64)
    for l in range(1, L + 1):
        p = {k: np.asarray(v, dtype=np.float64) for k, v in params[l - 1].items()}
        M = ((dist >= 0) & (dist <= L - l)).astype(np.float64) if masked else np.ones(n)
        if l == 1:
            t = H
        else:
            mu = H.mean(1, keepdims=True)
            var = ((H - mu) ** 2).mean(1, keepdims=True)
            t = np.maximum(0, (H - mu) / np.sqrt(var + oracle.LN_EPS) * p["ln_gamma"] + p["ln_beta"])
        Z = (Ahat @ t) @ p["W_neigh"] + t @ p["W_self"] + p["bias"]
        H = M[:, None] * (H + Z if 1 < l < L else Z)
    logits = H[T]
    return logits, float(np.mean(logsumexp(logits, axis=1) - logits[np.arange(T.size), y]))


def _setup(seed, n=70, dims=(6, 5, 5, 5, 3), directed=False):
    g = gg.random_directed(n, 2.5, seed) if directed else gg.erdos_renyi(n, 3.0, seed)
    rng = np.random.default_rng(seed)
    T = np.sort(rng.choice(n, 6, replace=False)).astype(np.int32)
    params = gg.res_layer_weights(list(dims), seed)
    H0 = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], T.size).astype(np.int32)
    return g, T, params, H0, y


@pytest.mark.parametrize("directed", [False, True])
@pytest.mark.parametrize("dims", [(6, 5, 3), (6, 5, 5, 3), (6, 5, 5, 5, 5, 3)])
def test_forward_equals_dense_rederivation(directed, dims):
    g, T, params, H0, y = _setup(3 + len(dims), dims=dims, directed=directed)
    m = oracle.ResModel(g.row_ptr, g.col_idx, T, params)
    loss = m.forward(H0, y)
    logits, want = _dense_forward(g, T, params, H0, y)
    assert np.allclose(m.H[-1][T], logits, rtol=1e-11, atol=1e-12) and np.isclose(loss, want, rtol=1e-11)


@pytest.mark.parametrize("directed", [False, True])
def test_backward_equals_central_finite_differences(directed):
    g, T, params, H0, y = _setup(9, n=40, directed=directed)
    m = oracle.ResModel(g.row_ptr, g.col_idx, T, params)
    m.forward(H0, y)
    grads = m.backward()
    rng = np.random.default_rng(1)
    eps = 1e-6
    names = {"dW_neigh": "W_neigh", "dW_self": "W_self", "dbias": "bias", "dln_gamma": "ln_gamma", "dln_beta": "ln_beta"}
    for l in range(len(params)):
        assert set(grads[l]) == {"d" + k for k in params[l]}
        for name, G in grads[l].items():
            for _ in range(4):
                idx = tuple(rng.integers(0, s) for s in G.shape)
                vals = []
                for sgn in (+1, -1):
                    q = [{k: np.array(v, dtype=np.float64) for k, v in p.items()} for p in params]
                    q[l][names[name]][idx] += sgn * eps
                    vals.append(_dense_forward(g, T, q, H0, y)[1])
                fd = (vals[0] - vals[1]) / (2 * eps)
                assert abs(fd - G[idx]) <= 2e-6 * max(1.0, abs(fd)), (l, name, idx, fd, G[idx])


def test_masked_equals_unmasked_equals_global():
    n, dims = 400, (5, 4, 4, 4, 3)
    L = len(dims) - 1
    g = gg.erdos_renyi(n, 3.0, 21)
    rng = np.random.default_rng(21)
    Tg = np.sort(rng.choice(n, 9, replace=False)).astype(np.int64)
    params = gg.res_layer_weights(list(dims), 21)
    H0 = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], Tg.size).astype(np.int32)
    full = oracle.ResModel(g.row_ptr, g.col_idx, Tg, params, all_rows=True)
    loss_full = full.forward(H0, y)
    part = gg.halo_partition(g, Tg, L)
    assert part.graph.n_rows < n
    H0l = H0[part.local_to_global]
    mk = oracle.ResModel(part.graph.row_ptr, part.graph.col_idx, part.targets, params)
    um = oracle.ResModel(part.graph.row_ptr, part.graph.col_idx, part.targets, params, all_rows=True)
    assert np.isclose(mk.forward(H0l, y), loss_full, rtol=1e-12) and np.isclose(um.forward(H0l, y), loss_full, rtol=1e-12)
    gf, gm, gu = full.backward(), mk.backward(), um.backward()
    for a, b, c in zip(gf, gm, gu):
        for k in a:
            assert np.allclose(a[k], b[k], rtol=1e-9, atol=1e-13), k
            assert np.allclose(a[k], c[k], rtol=1e-9, atol=1e-13), k
