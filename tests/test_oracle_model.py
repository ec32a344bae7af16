"""Pins of the oracle's whole masked forward/backward (sections 2.1 and 6):
dense-adjacency brute force with diagonal masks, central finite differences, and the paper's
invariant that masked outputs on the targets equal the unmasked / unpartitioned result."""
import numpy as np
import pytest
from scipy.special import logsumexp

import graphgen as gg
import oracle


def _setup(kind, seed, n=80, L=3, dims=(6, 5, 4, 3), directed=False):
    g = gg.random_directed(n, 2.5, seed) if directed else gg.erdos_renyi(n, 3.0, seed)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    rng = np.random.default_rng(seed)
    T = np.sort(rng.choice(n, size=6, replace=False)).astype(np.int32)
    params = gg.layer_weights(list(dims[: L + 1]), kind == "sage", seed)
    H0 = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[L], size=T.size).astype(np.int32)
    return g, T, params, H0, y


def _dense_forward(g, T, kind, params, H0, y, masked=True):
    """H_l = M_l sigma(M_l (Ahat H_{l-1} W_n [+ H_{l-1} W_s]) + b), M_l = diag[dist <= L - l]."""
    n, L = g.n_rows, len(params)
    A = g.to_scipy().toarray().astype(np.float64)
    deg = A.sum(1)
    if kind == "gcn":
        s = np.where(deg > 0, 1 / np.sqrt(np.maximum(deg, 1)), 0)
        Ahat = s[:, None] * A * s[None, :]
    else:
        Ahat = np.where(deg > 0, 1 / np.maximum(deg, 1), 0)[:, None] * A
    # hop distance by repeated boolean products
    dist = np.full(n, -1)
    dist[T] = 0
    reach = dist >= 0
    for j in range(1, L + 1):
        new = ((A.T @ reach.astype(np.float64)) > 0) & ~reach
        dist[new] = j
        reach |= new
    H = np.array(H0, dtype=np.float64)
    for l in range(1, L + 1):
        p = params[l - 1]
        M = ((dist >= 0) & (dist <= L - l)).astype(np.float64) if masked else np.ones(n)
        Z = (Ahat @ H) @ p["W_neigh"].astype(np.float64) + p["bias"].astype(np.float64)
        if kind == "sage":
            Z = Z + H @ p["W_self"].astype(np.float64)
        H = M[:, None] * (np.maximum(Z, 0) if l < L else Z)
    logits = H[T]
    loss = float(np.mean(logsumexp(logits, axis=1) - logits[np.arange(T.size), y]))
    return logits, loss


@pytest.mark.parametrize("kind", ["gcn", "sage"])
@pytest.mark.parametrize("directed", [False, True])
@pytest.mark.parametrize("L", [1, 2, 3])
def test_forward_equals_dense_brute_force(kind, directed, L):
    g, T, params, H0, y = _setup(kind, 11 + L, L=L, directed=directed)
    m = oracle.Model(g.row_ptr, g.col_idx, T, kind, params)
    loss = m.forward(H0, y)
    logits, want = _dense_forward(g, T, kind, params, H0, y)
    assert np.allclose(m.H[-1][T], logits, rtol=1e-12, atol=1e-12)
    assert np.isclose(loss, want, rtol=1e-12)


@pytest.mark.parametrize("kind", ["gcn", "sage"])
def test_masked_equals_unmasked_equals_global(kind):
    """Section 6, step 5: the targets' logits use the exact dependency."""
    n, L = 400, 3
    g = gg.erdos_renyi(n, 3.0, 21)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    rng = np.random.default_rng(21)
    Tg = np.sort(rng.choice(n, size=9, replace=False)).astype(np.int64)
    params = gg.layer_weights([5, 4, 4, 3], kind == "sage", 21)
    H0 = rng.standard_normal((n, 5))
    y = rng.integers(0, 3, size=Tg.size).astype(np.int32)
    # (a) no partition at all: whole graph, every row computed
    full = oracle.Model(g.row_ptr, g.col_idx, Tg, kind, params, all_rows=True)
    loss_full = full.forward(H0, y)
    # (b) the partition (targets + 3-hop halo), masked and (c) unmasked
    part = gg.halo_partition(g, Tg, L)
    assert part.graph.n_rows < n
    H0l = H0[part.local_to_global]
    mk = oracle.Model(part.graph.row_ptr, part.graph.col_idx, part.targets, kind, params, part.global_degree)
    um = oracle.Model(part.graph.row_ptr, part.graph.col_idx, part.targets, kind, params, part.global_degree,
                      all_rows=True)
    loss_mk, loss_um = mk.forward(H0l, y), um.forward(H0l, y)
    assert np.allclose(mk.H[-1][part.targets], full.H[-1][Tg], rtol=1e-12, atol=1e-13)
    assert np.allclose(um.H[-1][part.targets], full.H[-1][Tg], rtol=1e-12, atol=1e-13)
    assert np.isclose(loss_mk, loss_full, rtol=1e-12) and np.isclose(loss_um, loss_full, rtol=1e-12)
    # weight gradients agree too (the masked rows carry no gradient to the targets' loss)
    gf, gm, gu = full.backward(), mk.backward(), um.backward()
    for a, b, c in zip(gf, gm, gu):
        for k in a:
            assert np.allclose(a[k], b[k], rtol=1e-10, atol=1e-13), k
            assert np.allclose(a[k], c[k], rtol=1e-10, atol=1e-13), k


def test_masked_rows_are_never_read():
    # rows outside R_l hold NaN in the oracle's buffers; a finite loss proves nothing read them
    g, T, params, H0, y = _setup("sage", 31)
    m = oracle.Model(g.row_ptr, g.col_idx, T, "sage", params)
    assert np.isfinite(m.forward(H0, y))
    assert np.isnan(m.H[-1]).sum() == (g.n_rows - T.size) * params[-1]["bias"].size
    for gr in m.backward():
        for v in gr.values():
            assert np.isfinite(v).all()


@pytest.mark.parametrize("kind", ["gcn", "sage"])
@pytest.mark.parametrize("directed", [False, True])
def test_backward_equals_central_finite_differences(kind, directed):
    g, T, params, H0, y = _setup(kind, 41, n=40, L=3, directed=directed)
    m = oracle.Model(g.row_ptr, g.col_idx, T, kind, params)
    m.forward(H0, y)
    grads = m.backward()
    eps = 1e-6
    rng = np.random.default_rng(0)
    for l, p in enumerate(params):
        for name, arr in p.items():
            gname = {"W_neigh": "dW_neigh", "W_self": "dW_self", "bias": "dbias"}[name]
            flat = np.array(arr, dtype=np.float64).reshape(-1)
            idx = rng.choice(flat.size, size=min(flat.size, 12), replace=False)
            for i in idx:
                vals = []
                for sgn in (+1, -1):
                    q = [{k: np.array(v, dtype=np.float64) for k, v in pp.items()} for pp in params]
                    q[l][name].reshape(-1)[i] += sgn * eps
                    vals.append(_dense_forward(g, T, kind, q, H0, y)[1])
                fd = (vals[0] - vals[1]) / (2 * eps)
                an = grads[l][gname].reshape(-1)[i]
                assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) , (l, name, i, fd, an)


def test_bf16_model_stays_close_to_fp64_model():
    g, T, params, H0, y = _setup("sage", 51)
    a = oracle.Model(g.row_ptr, g.col_idx, T, "sage", params)
    b = oracle.Model(g.row_ptr, g.col_idx, T, "sage", params, bf16=True)
    la, lb = a.forward(H0, y), b.forward(H0, y)
    assert abs(la - lb) < 2e-2 * abs(la)
    ga, gb = a.backward(), b.backward()
    for x, z in zip(ga, gb):
        for k in x:
            assert np.linalg.norm(x[k] - z[k]) <= 5e-2 * np.linalg.norm(x[k])
    # every stored activation is a bf16 value
    for H in b.H:
        fin = H[np.isfinite(H)]
        assert np.array_equal(oracle.round_bf16(fin.copy()), fin)


@pytest.mark.parametrize("directed", [False, True])
def test_first_layer_in_the_exchanged_order_is_the_same_layer(directed):
    """Section 2.1's layer is linear in front of the activation, so a first layer may multiply by its weights before it
    aggregates: Agg(H_0 W_n) + H_0 W_s + b = Agg(H_0) W_n + H_0 W_s + b, and then dW_n = H_0^T Agg^T(dZ_1).  The exchanged
    order written out with dense matrices against the oracle's aggregate-first model; dZ_1 comes from central
    differences of the dense brute-force loss (a shift of Z_1[v, c] is emulated by a one-hot extra input column that
    only the self weights of column c see)."""
    g, T, params, H0, y = _setup("sage", 71, n=48, L=3, dims=(9, 5, 4, 3), directed=directed)
    m = oracle.Model(g.row_ptr, g.col_idx, T, "sage", params)
    m.forward(H0, y)
    grads = m.backward()
    n = g.n_rows
    A = g.to_scipy().toarray().astype(np.float64)
    deg = A.sum(1)
    Ahat = np.where(deg > 0, 1 / np.maximum(deg, 1), 0)[:, None] * A
    R1 = m.rows_of_layer(1)
    base = [{k: np.array(v, dtype=np.float64) for k, v in pp.items()} for pp in params]
    Wn, Ws, b = base[0]["W_neigh"], base[0]["W_self"], base[0]["bias"]
    N1 = Wn.shape[1]
    # forward
    H1 = np.maximum(Ahat @ (H0 @ Wn) + H0 @ Ws + b, 0)
    assert np.allclose(H1[R1], m.H[1][R1], rtol=1e-12, atol=1e-12)

    # backward: dZ_1 by central differences
    def loss_with_shift(v, c, d):
        H0x = np.concatenate([H0, np.zeros((n, 1))], axis=1)
        H0x[v, -1] = d
        col = np.zeros((1, N1))
        col[0, c] = 1.0
        q = [dict(pp) for pp in base]
        q[0] = {"W_neigh": np.concatenate([Wn, np.zeros_like(col)]), "W_self": np.concatenate([Ws, col]), "bias": b}
        return _dense_forward(g, T, "sage", q, H0x, y)[1]

    eps = 1e-6
    dZ1 = np.zeros((n, N1))
    for v in R1:
        for c in range(N1):
            dZ1[v, c] = (loss_with_shift(v, c, eps) - loss_with_shift(v, c, -eps)) / (2 * eps)
    dP = Ahat.T @ dZ1                                         # what reaches the transformed rows: Agg^T(dZ_1)
    for name, want in (("dW_neigh", H0.T @ dP), ("dW_self", H0.T @ dZ1), ("dbias", dZ1.sum(0))):
        got = grads[0][name]
        assert np.abs(got - want).max() <= 1e-7 * max(1.0, np.abs(want).max()), name
