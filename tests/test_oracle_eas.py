"""Pins of the oracle's expansion-aware traversal (section 5.3.1: at most h hops from the inner vertices, at most f
new vertices per traversed vertex, many-connections-first): a hand-worked example, reductions to functions that are
pinned elsewhere (plain breadth-first rings when nothing is dropped; the boundary sampler for the hash rule and one
hop), an independent re-derivation with Python sets, and structural invariants."""
import numpy as np
import pytest

import graphgen as gg
import oracle


def _sym(n, und):
    r = np.array([a for a, b in und] + [b for a, b in und], dtype=np.int64)
    c = np.array([b for a, b in und] + [a for a, b in und], dtype=np.int64)
    return gg.csr_from_edges(n, n, r, c)


def test_hand_worked_example_h2_f1():
    """Inner vertices {0, 1}.  0 sees the outside vertices 2 and 3, 1 sees 3 and 4.
    Connections to unselected vertices when hop 1 starts: 2 -> {5} = 1, 3 -> {5, 6, 7} = 3, 4 -> {6} = 1.
    f = 1: vertex 0 keeps 3 (3 > 1), vertex 1 keeps 3 (3 > 1)          -> hop 1 = {3}.
    Hop 2 from 3: candidates 5, 6, 7 (0 and 1 are selected).  Unselected now: 2, 4, 5, 6, 7.
    5 -> {2} = 1 (3 is selected), 6 -> {4, 7} = 2, 7 -> {6} = 1          -> hop 2 = {6}."""
    g = _sym(8, [(0, 1), (0, 2), (0, 3), (1, 3), (1, 4), (2, 5), (3, 5), (3, 6), (3, 7), (4, 6), (6, 7)])
    dist, ring, off = oracle.eas_traverse(g.row_ptr, g.col_idx, [0, 1], 2, 1, "degree")
    assert list(ring) == [0, 1, 3, 6] and list(off) == [0, 2, 3, 4]
    assert list(dist) == [0, 0, -1, 1, -1, -1, 2, -1]
    # f = 2: 0 keeps 3 and 2 (tie 2 vs nothing else), 1 keeps 3 and 4; hop 2 from {2, 3, 4}: 2 -> 5; 3 -> 5, 6, 7 minus
    # nothing selected: connections 5 -> {} = 0, 6 -> {7} = 1, 7 -> {6} = 1: keeps 6 and 7 (tie: smaller id first); 4 -> 6
    dist, ring, off = oracle.eas_traverse(g.row_ptr, g.col_idx, [0, 1], 2, 2, "degree")
    assert list(ring) == [0, 1, 2, 3, 4, 5, 6, 7] and list(off) == [0, 2, 5, 8]


@pytest.mark.parametrize("rule", ["degree", "hash"])
@pytest.mark.parametrize("hops", [1, 3])
def test_nothing_dropped_is_plain_breadth_first(rule, hops):
    g = gg.chung_lu(3000, 9.0, 2.1, 3)
    T = np.sort(np.random.default_rng(hops).choice(3000, 25, replace=False))
    dist, ring, off = oracle.eas_traverse(g.row_ptr, g.col_idx, T, hops, 10**6, rule, seed=5)
    d2, r2, o2 = oracle.active_sets(g.row_ptr, g.col_idx, T, hops)
    assert np.array_equal(dist, d2) and np.array_equal(ring, r2) and np.array_equal(off, o2)
    dist0, ring0, off0 = oracle.eas_traverse(g.row_ptr, g.col_idx, T, hops, 0, rule, seed=5)
    assert np.array_equal(ring0, T) and list(np.diff(off0)) == [len(T)] + [0] * hops


@pytest.mark.parametrize("fanout", [1, 3, 8])
def test_hash_rule_one_hop_selects_what_the_boundary_sampler_keeps(fanout):
    n = 5000
    g = gg.chung_lu(n, 12.0, 2.1, 4)
    T = np.sort(np.random.default_rng(fanout).choice(n, 500, replace=False))
    dist, ring, off = oracle.eas_traverse(g.row_ptr, g.col_idx, T, 1, fanout, "hash", seed=77)
    is_t = np.zeros(n, dtype=np.uint8)
    is_t[T] = 1
    srp, sci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, fanout, 77)
    outside = np.unique(sci[is_t[sci] == 0])
    assert np.array_equal(ring[off[1]:], outside)


def _python_eas(g, T, hops, fanout):
    """Independent re-derivation of the degree rule with sets and sorted()."""
    rows = [set(g.col_idx[g.row_ptr[v]:g.row_ptr[v + 1]].tolist()) for v in range(g.n_rows)]
    selected = set(int(t) for t in T)
    rings = [sorted(selected)]
    for _ in range(hops):
        before = set(selected)
        new = set()
        for v in rings[-1]:
            cand = [u for u in rows[v] if u not in before]
            cand.sort(key=lambda u: (-len(rows[u] - before), u))
            new.update(cand[:fanout])
        rings.append(sorted(new))
        selected |= new
    return rings


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_degree_rule_equals_python_rederivation(seed):
    g = gg.chung_lu(600, 7.0, 2.1, 10 + seed)
    T = np.sort(np.random.default_rng(seed).choice(600, 30, replace=False))
    for hops, fanout in ((1, 2), (2, 3), (3, 1)):
        dist, ring, off = oracle.eas_traverse(g.row_ptr, g.col_idx, T, hops, fanout, "degree")
        want = _python_eas(g, T, hops, fanout)
        got = [list(ring[off[j]:off[j + 1]]) for j in range(hops + 1)]
        assert got == want


def test_structure_of_the_traversal():
    n, hops, f = 4000, 3, 4
    g = gg.chung_lu(n, 10.0, 2.1, 6)
    T = np.sort(np.random.default_rng(6).choice(n, 100, replace=False))
    for rule in ("degree", "hash"):
        dist, ring, off = oracle.eas_traverse(g.row_ptr, g.col_idx, T, hops, f, rule, seed=1)
        sizes = np.diff(off)
        assert all(sizes[j + 1] <= f * sizes[j] for j in range(hops))        # at most f new vertices per traversed vertex
        assert len(set(ring.tolist())) == ring.size                          # rings are disjoint
        d_bfs, _, _ = oracle.active_sets(g.row_ptr, g.col_idx, T, hops)
        sel = dist >= 0
        assert np.all(d_bfs[sel] >= 0) and np.all(d_bfs[sel] <= dist[sel])   # selected within its hop budget
        for j in range(1, hops + 1):                                         # every ring-j vertex hangs on ring j-1
            prev = set(ring[off[j - 1]:off[j]].tolist())
            for u in ring[off[j]:off[j + 1]][:200]:
                assert prev & set(g.col_idx[g.row_ptr[u]:g.row_ptr[u + 1]].tolist())
