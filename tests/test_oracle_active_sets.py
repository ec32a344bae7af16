"""Pins of the oracle's active-set construction (section 6, steps 1 and 4):
closed forms on textbook graphs and dense boolean reachability."""
import numpy as np
import pytest

import graphgen as gg
import oracle


def _csr(n, edges):
    r = np.array([e[0] for e in edges], dtype=np.int64)
    c = np.array([e[1] for e in edges], dtype=np.int64)
    return gg.csr_from_edges(n, n, r, c)


def _sym(n, und):
    return _csr(n, und + [(b, a) for a, b in und])


def test_path_graph_rings_have_two_vertices():
    n = 21
    g = _sym(n, [(i, i + 1) for i in range(n - 1)])
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, [10], 4)
    assert list(np.diff(off)) == [1, 2, 2, 2, 2]
    assert np.array_equal(dist, np.where(np.abs(np.arange(n) - 10) <= 4, np.abs(np.arange(n) - 10), -1))
    assert list(ring) == [10, 9, 11, 8, 12, 7, 13, 6, 14]


def test_star_from_leaf_and_from_hub():
    n = 9
    g = _sym(n, [(0, i) for i in range(1, n)])
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, [3], 2)
    assert dist[3] == 0 and dist[0] == 1 and all(dist[i] == 2 for i in range(1, n) if i != 3)
    assert list(np.diff(off)) == [1, 1, n - 2]
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, [0], 3)
    assert list(np.diff(off)) == [1, n - 1, 0, 0]      # L larger than the eccentricity: empty late rings


def test_complete_graph_everything_at_distance_one():
    n = 12
    g = _sym(n, [(i, j) for i in range(n) for j in range(i + 1, n)])
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, [2, 5], 3)
    assert (dist[[2, 5]] == 0).all() and (np.delete(dist, [2, 5]) == 1).all()
    assert list(off) == [0, 2, n, n, n]


def test_unreachable_component_is_minus_one_and_absent():
    g = _sym(8, [(0, 1), (1, 2), (2, 3), (4, 5), (5, 6), (6, 7)])
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, [0], 5)
    assert list(dist) == [0, 1, 2, 3, -1, -1, -1, -1]
    assert list(ring) == [0, 1, 2, 3]


def test_direction_follows_rows_not_columns():
    # row v lists what v aggregates: 0 <- 1 <- 2 (row 0 = {1}, row 1 = {2})
    g = _csr(3, [(0, 1), (1, 2)])
    dist, _, _ = oracle.active_sets(g.row_ptr, g.col_idx, [0], 2)
    assert list(dist) == [0, 1, 2]
    dist, _, _ = oracle.active_sets(g.row_ptr, g.col_idx, [2], 2)
    assert list(dist) == [-1, -1, 0]


def test_duplicate_targets_are_a_set():
    g = _sym(5, [(0, 1), (1, 2), (2, 3), (3, 4)])
    a = oracle.active_sets(g.row_ptr, g.col_idx, [2, 2, 2], 1)
    b = oracle.active_sets(g.row_ptr, g.col_idx, [2], 1)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("directed", [False, True])
def test_equals_dense_boolean_reachability(seed, directed):
    n, L = 120, 4
    g = gg.random_directed(n, 2.0, seed) if directed else gg.erdos_renyi(n, 2.5, seed)
    rng = np.random.default_rng(seed)
    T = rng.choice(n, size=7, replace=False)
    A = g.to_scipy().toarray().astype(bool)            # A[v,u]: v aggregates u
    reach = np.zeros(n, dtype=bool)
    reach[T] = True
    want = np.where(reach, 0, -1)
    x = reach.copy()
    for j in range(1, L + 1):
        x = (A.T.astype(np.int64) @ x.astype(np.int64)) > 0    # everything some reached vertex aggregates
        new = x & ~reach
        want[new] = j
        reach |= new
        x = reach.copy()
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, T, L)
    assert np.array_equal(dist, want)
    # R_L = T, rings disjoint and sorted, sizes add up
    assert sorted(ring[off[0]:off[1]]) == sorted(T)
    assert len(set(ring.tolist())) == len(ring) == int((want >= 0).sum())
    for j in range(L + 1):
        seg = ring[off[j]:off[j + 1]]
        assert (dist[seg] == j).all() and (np.diff(seg) > 0).all()


def test_generator_partition_is_the_L_hop_ball():
    # cross-check of the input generator: the halo it cut holds exactly the reachable ball
    w = gg.make_workload("cfg0", scale=0.05)
    g, p = w.global_graph, w.partition
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, w.targets_global, w.n_layers)
    assert np.array_equal(np.flatnonzero(dist >= 0), p.local_to_global)
    dl, _, _ = oracle.active_sets(p.graph.row_ptr, p.graph.col_idx, p.targets, w.n_layers)
    assert np.array_equal(dl, dist[p.local_to_global])
