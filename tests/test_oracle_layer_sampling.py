"""Pins of the oracle's layer-wise sampling as per-layer masking (section 5.2: for layer-wise sampling methods the
maskings are generated per layer and the layer aggregates through them): the mask rules against a Python big-integer
re-derivation and counting properties, reductions to the unmasked functions (everything kept) and to the boundary
sampler's selection, the masked aggregation against a dense matrix product, its backward against the adjoint identity
and finite differences of the whole model, and the transposed mask against a dictionary of edges."""
import numpy as np
import pytest
from scipy.special import logsumexp

import graphgen as gg
import oracle

M64 = (1 << 64) - 1


def _py_key(seed, v, u, layer):
    def mix(x):
        x = (x + 0x9E3779B97F4A7C15) & M64
        x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & M64
        x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & M64
        return x ^ (x >> 31)
    return mix(mix(mix((seed + layer) & M64) ^ v) ^ u)


@pytest.mark.parametrize("rule,par", [("threshold", oracle.keep_threshold(0.4)), ("fanout", 3)])
def test_mask_equals_python_rederivation(rule, par):
    g = gg.chung_lu(300, 8.0, 2.1, 5)
    rows = np.arange(0, 300, 3, dtype=np.int32)
    seed, layer = 12345, 2
    keep, kept_len = oracle.layer_edge_mask(g.row_ptr, g.col_idx, rows, rule, layer, seed, fanout=par if rule == "fanout" else 0,
                                            threshold=par if rule == "threshold" else M64)
    want = np.zeros(g.nnz, dtype=np.uint8)
    for v in rows:
        s, e = g.row_ptr[v], g.row_ptr[v + 1]
        keys = [(_py_key(seed, int(v), int(g.col_idx[p]), layer), int(g.col_idx[p]), p) for p in range(s, e)]
        if rule == "threshold":
            for k, u, p in keys:
                want[p] = k <= par
        else:
            for k, u, p in sorted(keys)[:par]:
                want[p] = 1
    assert np.array_equal(keep, want)
    assert np.array_equal(kept_len[rows], np.add.reduceat(np.concatenate([want, [0]]), g.row_ptr[rows])[: len(rows)] * (np.diff(g.row_ptr)[rows] > 0))
    others = np.setdiff1d(np.arange(300), rows)
    assert not kept_len[others].any()


def test_counting_properties_and_seeds():
    g = gg.chung_lu(4000, 20.0, 2.1, 6)
    deg = np.diff(g.row_ptr)
    for f in (1, 5, 25):
        keep, kept_len = oracle.layer_edge_mask(g.row_ptr, g.col_idx, None, "fanout", 1, 7, fanout=f)
        assert np.array_equal(kept_len, np.minimum(deg, f)) and keep.sum() == kept_len.sum()
    # a threshold keeps about p of the edges, independently per layer and seed
    p = 0.3
    k1, _ = oracle.layer_edge_mask(g.row_ptr, g.col_idx, None, "threshold", 1, 7, threshold=oracle.keep_threshold(p))
    k2, _ = oracle.layer_edge_mask(g.row_ptr, g.col_idx, None, "threshold", 2, 7, threshold=oracle.keep_threshold(p))
    k3, _ = oracle.layer_edge_mask(g.row_ptr, g.col_idx, None, "threshold", 1, 8, threshold=oracle.keep_threshold(p))
    n = g.nnz
    for k in (k1, k2, k3):
        assert abs(k.mean() - p) < 4 * np.sqrt(p * (1 - p) / n)
    for a, b in ((k1, k2), (k1, k3)):
        assert abs((a & b).mean() - p * p) < 4 * np.sqrt(p * p * (1 - p * p) / n)     # independent masks
    again, _ = oracle.layer_edge_mask(g.row_ptr, g.col_idx, None, "threshold", 1, 7, threshold=oracle.keep_threshold(p))
    assert np.array_equal(k1, again)


def test_fanout_rule_selects_what_the_boundary_sampler_selects():
    """With no vertex inside the target set the boundary sampler thins every row to its `fanout` smallest (key, id):
    the same selection, by a function that is pinned on its own (layer = 1 is the sampler's hop)."""
    n = 2000
    g = gg.chung_lu(n, 14.0, 2.1, 8)
    rows = np.arange(0, n, 2, dtype=np.int32)
    keep, kept_len = oracle.layer_edge_mask(g.row_ptr, g.col_idx, rows, "fanout", 1, 99, fanout=4)
    srp, sci = oracle.sample_boundary(g.row_ptr, g.col_idx, np.zeros(n, dtype=np.uint8), rows, 4, 99)
    for i, v in enumerate(rows):
        s, e = g.row_ptr[v], g.row_ptr[v + 1]
        assert np.array_equal(g.col_idx[s:e][keep[s:e] == 1], sci[srp[i]:srp[i + 1]])


@pytest.mark.parametrize("kind", ["gcn", "sage"])
def test_everything_kept_is_the_unmasked_model(kind):
    g = gg.erdos_renyi(200, 4.0, 2)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    rng = np.random.default_rng(2)
    T = np.sort(rng.choice(200, 12, replace=False)).astype(np.int32)
    params = gg.layer_weights([5, 4, 3], kind == "sage", 2)
    H0 = rng.standard_normal((200, 5))
    y = rng.integers(0, 3, T.size).astype(np.int32)
    plain = oracle.Model(g.row_ptr, g.col_idx, T, kind, params)
    for ls in (("threshold", M64, 3), ("fanout", 10**6, 3)):
        m = oracle.Model(g.row_ptr, g.col_idx, T, kind, params, layer_sampling=ls)
        assert m.forward(H0, y) == plain.forward(H0, y)
        for a, b in zip(m.backward(), plain.backward()):
            for k in a:
                assert np.array_equal(a[k], b[k])


def _dense_forward(g, T, kind, params, H0, y, keeps):
    """H_l = M_l sigma(M_l ((Ahat o K_l) H_{l-1} W_n [+ H_{l-1} W_s]) + b): a dense matrix product per layer."""
    n, L = g.n_rows, len(params)
    rows_of = np.repeat(np.arange(n), np.diff(g.row_ptr))
    deg = np.diff(g.row_ptr).astype(np.float64)
    A_full = g.to_scipy().toarray().astype(np.float64)
    dist = np.full(n, -1)
    dist[T] = 0
    reach = dist >= 0
    for j in range(1, L + 1):
        new = ((A_full.T @ reach.astype(np.float64)) > 0) & ~reach
        dist[new] = j
        reach |= new
    H = np.array(H0, dtype=np.float64)
    for l in range(1, L + 1):
        p = params[l - 1]
        Kl = np.zeros((n, n))
        Kl[rows_of, g.col_idx] = keeps[l]
        A = A_full * Kl
        if kind == "gcn":
            s = np.where(deg > 0, 1 / np.sqrt(np.maximum(deg, 1)), 0)
            Ahat = s[:, None] * A * s[None, :]
        else:
            kept = A.sum(1)
            Ahat = np.where(kept > 0, 1 / np.maximum(kept, 1), 0)[:, None] * A
        M = ((dist >= 0) & (dist <= L - l)).astype(np.float64)
        Z = (Ahat @ H) @ p["W_neigh"].astype(np.float64) + p["bias"].astype(np.float64)
        if kind == "sage":
            Z = Z + H @ p["W_self"].astype(np.float64)
        H = M[:, None] * (np.maximum(Z, 0) if l < L else Z)
    logits = H[T]
    return logits, float(np.mean(logsumexp(logits, axis=1) - logits[np.arange(T.size), y]))


@pytest.mark.parametrize("kind", ["gcn", "sage"])
@pytest.mark.parametrize("ls", [("threshold", oracle.keep_threshold(0.6), 4), ("fanout", 2, 9)])
def test_forward_equals_dense_brute_force_and_backward_equals_finite_differences(kind, ls):
    n, L = 60, 3
    g = gg.erdos_renyi(n, 3.5, 17)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    rng = np.random.default_rng(17)
    T = np.sort(rng.choice(n, 6, replace=False)).astype(np.int32)
    params = gg.layer_weights([5, 4, 4, 3], kind == "sage", 17)
    H0 = rng.standard_normal((n, 5))
    y = rng.integers(0, 3, T.size).astype(np.int32)
    m = oracle.Model(g.row_ptr, g.col_idx, T, kind, params, layer_sampling=ls)
    loss = m.forward(H0, y)
    logits, want = _dense_forward(g, T, kind, params, H0, y, m.keep)
    assert np.allclose(m.H[-1][T], logits, rtol=1e-12, atol=1e-12) and np.isclose(loss, want, rtol=1e-12)
    assert any(k.sum() < np.count_nonzero(k >= 0) for k in m.keep[1:])           # something was dropped
    grads = m.backward()
    eps = 1e-6
    for l in range(L):
        for name, G in grads[l].items():
            key = {"dW_neigh": "W_neigh", "dW_self": "W_self", "dbias": "bias"}[name]
            for _ in range(4):
                idx = tuple(rng.integers(0, s) for s in G.shape)
                vals = []
                for sgn in (+1, -1):
                    q = [{k: np.array(v, dtype=np.float64) for k, v in p.items()} for p in params]
                    q[l][key][idx] += sgn * eps
                    vals.append(_dense_forward(g, T, kind, q, H0, y, m.keep)[1])
                fd = (vals[0] - vals[1]) / (2 * eps)
                assert abs(fd - G[idx]) <= 1e-6 * max(1.0, abs(fd)), (l, name, idx, fd, G[idx])


def test_masked_aggregation_adjoint_identity():
    g = gg.random_directed(500, 5.0, 3)
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(500, 200, replace=False)).astype(np.int32)
    keep, kept_len = oracle.layer_edge_mask(g.row_ptr, g.col_idx, rows, "threshold", 1, 5, threshold=oracle.keep_threshold(0.5))
    rs, cs = rng.random(500), rng.random(500)
    X, dY = rng.standard_normal((500, 7)), rng.standard_normal((500, 7))
    Y = np.zeros((500, 7))
    oracle.spmm_fwd_em(g.row_ptr, g.col_idx, keep, rows, X, Y, 7, rs, cs)
    dX = np.zeros((500, 7))
    oracle.spmm_bwd_em(g.row_ptr, g.col_idx, keep, rows, dY, dX, 7, rs, cs)
    assert np.isclose((Y[rows] * dY[rows]).sum(), (X * dX).sum(), rtol=1e-12)


def test_transposed_mask_against_an_edge_dictionary():
    g = gg.random_directed(700, 4.0, 4)
    gt = gg.transpose(g)
    keep, _ = oracle.layer_edge_mask(g.row_ptr, g.col_idx, None, "threshold", 3, 11, threshold=oracle.keep_threshold(0.5))
    kt = oracle.transpose_mask(g.row_ptr, g.col_idx, keep, gt.row_ptr, gt.col_idx)
    rows_of = np.repeat(np.arange(700), np.diff(g.row_ptr))
    d = {(int(v), int(u)): int(k) for v, u, k in zip(rows_of, g.col_idx, keep)}
    rows_t = np.repeat(np.arange(700), np.diff(gt.row_ptr))
    want = np.array([d[(int(v), int(u))] for u, v in zip(rows_t, gt.col_idx)], dtype=np.uint8)
    assert np.array_equal(kt, want) and kt.sum() == keep.sum()
