"""Pins of the oracle's boundary-only sampler (section 5.3.1 with the hash rule):
published hash vectors, an independent big-integer re-derivation, counting properties,
brute force on tiny graphs and a uniformity test."""
import os

import numpy as np
import pytest

import graphgen as gg
import oracle

M64 = 2**64 - 1
GOLD = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed0.txt")


def _mix_py(x):
    x = (x + 0x9E3779B97F4A7C15) & M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & M64
    return x ^ (x >> 31)


def _key_py(seed, v, u, hop):
    return _mix_py(_mix_py(_mix_py((seed + hop) & M64) ^ v) ^ u)


def test_mix64_published_vectors():
    want = [int(l, 16) for l in open(GOLD) if not l.startswith("#") and l.strip()]
    got = [oracle.mix64((k * 0x9E3779B97F4A7C15) & M64) for k in range(3)]
    assert got == want


def test_edge_key_against_big_integer_arithmetic():
    rng = np.random.default_rng(0)
    for _ in range(200):
        seed, v, u = (int(x) for x in rng.integers(0, 2**63, size=3))
        hop = int(rng.integers(1, 4))
        assert oracle.edge_key(seed, v, u, hop) == _key_py(seed, v, u, hop)
    assert oracle.edge_key(M64, 10**7, 3, 1) == _key_py(M64, 10**7, 3, 1)     # wrap-around of seed + hop
    assert oracle.edge_key(1, 2, 3, 1) != oracle.edge_key(1, 3, 2, 1)          # direction matters


def _setup(seed, n=300, avg=12.0):
    g = gg.chung_lu(n, avg, 2.1, seed)
    pid = gg.bfs_partition(g, 4, seed)
    T = np.flatnonzero(pid == 0).astype(np.int32)
    is_t = np.zeros(n, dtype=np.uint8)
    is_t[T] = 1
    return g, T, is_t


@pytest.mark.parametrize("f", [0, 1, 3, 5])
def test_row_counts_and_inner_edges_untouched(f):
    g, T, is_t = _setup(1)
    rp, ci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, f, 99)
    for i, v in enumerate(T):
        row = g.col_idx[g.row_ptr[v]:g.row_ptr[v + 1]]
        kept = ci[rp[i]:rp[i + 1]]
        inner, ext = row[is_t[row] == 1], row[is_t[row] == 0]
        assert kept.size == inner.size + min(f, ext.size)
        assert (np.diff(kept) > 0).all()
        assert np.array_equal(kept[is_t[kept] == 1], inner)          # inner dependencies bit-identical
        assert np.isin(kept[is_t[kept] == 0], ext).all()


def test_large_fanout_keeps_everything():
    g, T, is_t = _setup(2)
    rp, ci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, int(g.degrees().max()), 5)
    want = np.concatenate([g.col_idx[g.row_ptr[v]:g.row_ptr[v + 1]] for v in T])
    assert np.array_equal(ci, want)


def test_brute_force_python_rederivation():
    g, T, is_t = _setup(3, n=120, avg=10.0)
    f, seed = 2, 0xABCDEF0123456789
    rp, ci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, f, seed)
    out = []
    for v in T:
        row = [int(u) for u in g.col_idx[g.row_ptr[v]:g.row_ptr[v + 1]]]
        ext = sorted((_key_py(seed, int(v), u, 1), u) for u in row if not is_t[u])[:f]
        out.append(sorted([u for u in row if is_t[u]] + [u for _, u in ext]))
    assert ci.tolist() == [u for r in out for u in r]
    assert rp.tolist() == np.concatenate([[0], np.cumsum([len(r) for r in out])]).tolist()


def test_seed_dependence_and_independence_from_target_order():
    g, T, is_t = _setup(4)
    a = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, 2, 7)
    b = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, 2, 7)
    c = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, 2, 8)
    assert np.array_equal(a[1], b[1]) and not np.array_equal(a[1], c[1])
    perm = np.random.default_rng(0).permutation(T.size)
    rp, ci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T[perm], 2, 7)
    for j, i in enumerate(perm):                                     # row content depends on (seed, v, u) only
        assert np.array_equal(ci[rp[j]:rp[j + 1]], a[1][a[0][i]:a[0][i + 1]])


def test_each_outside_neighbour_is_kept_with_probability_f_over_d():
    # a star: centre 0 is the only target, d outside leaves, fanout f; over many seeds each leaf is kept ~ f/d
    d, f, trials = 12, 3, 4000
    und = [(0, i) for i in range(1, d + 1)]
    g = gg.csr_from_edges(d + 1, d + 1, np.array([a for a, b in und] + [b for a, b in und]),
                          np.array([b for a, b in und] + [a for a, b in und]))
    is_t = np.zeros(d + 1, dtype=np.uint8)
    is_t[0] = 1
    hits = np.zeros(d + 1)
    for s in range(trials):
        _, ci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, np.array([0], dtype=np.int32), f, s)
        assert ci.size == f
        hits[ci] += 1
    exp = trials * f / d
    chi2 = ((hits[1:] - exp) ** 2 / exp).sum()
    assert chi2 < 40.0, chi2        # 11 degrees of freedom: P(chi2 > 40) < 4e-5


def test_sampled_local_graph_is_symmetric_and_keeps_inner_rows():
    g, T, is_t = _setup(5)
    rp, ci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, 2, 11)
    l2g, er, ec = oracle.sampled_local_edges(T, rp, ci)
    part = gg.partition_from_edges(g.n_rows, l2g, er, ec, T, g.degrees())
    assert gg.is_symmetric(part.graph)
    assert np.array_equal(part.local_to_global[part.targets], T)
    # every target's local row maps back to exactly its kept row
    for i, t in enumerate(part.targets):
        loc = part.graph.col_idx[part.graph.row_ptr[t]:part.graph.row_ptr[t + 1]]
        assert np.array_equal(part.local_to_global[loc], ci[rp[i]:rp[i + 1]])
    # halo rows hold only reverse edges into the target set
    halo = np.setdiff1d(np.arange(part.graph.n_rows), part.targets)
    for h in halo[:50]:
        loc = part.graph.col_idx[part.graph.row_ptr[h]:part.graph.row_ptr[h + 1]]
        assert loc.size >= 1 and np.isin(loc, part.targets).all()
