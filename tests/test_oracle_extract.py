"""Pins of the oracle's partition extraction (section 6, step 1; section 5.3.1: the sub-graph of the traversed
vertices, renumbered by (distance, id)): closed forms on a path graph, the edge set against an independent
construction (graphgen.halo_partition: boolean masks + scipy slicing, ascending-id numbering), structural
invariants, and the paper's own invariant - training on the extracted graph gives the unpartitioned result."""
import numpy as np
import pytest

import graphgen as gg
import oracle


def _sym(n, und):
    r = np.array([a for a, b in und] + [b for a, b in und], dtype=np.int64)
    c = np.array([b for a, b in und] + [a for a, b in und], dtype=np.int64)
    return gg.csr_from_edges(n, n, r, c)


def test_path_graph_closed_form():
    """Targets {10} on a path of 21 vertices, L = 3: local order is 10 | 9 11 | 8 12 | 7 13, i.e. local ids
    0 | 1 2 | 3 4 | 5 6, and the path's edges become 0-1, 0-2, 1-3, 2-4, 3-5, 4-6."""
    g = _sym(21, [(i, i + 1) for i in range(20)])
    rp, ci, l2g, off, dl = oracle.extract_partition(g.row_ptr, g.col_idx, [10], 3)
    assert list(l2g) == [10, 9, 11, 8, 12, 7, 13]
    assert list(off) == [0, 1, 3, 5, 7]
    assert list(dl) == [0, 1, 1, 2, 2, 3, 3]
    rows = [list(ci[rp[i]:rp[i + 1]]) for i in range(7)]
    assert rows == [[1, 2], [0, 3], [0, 4], [1, 5], [2, 6], [3], [4]]     # the outermost ring loses its outward edge


def test_star_and_unreached_vertices():
    g = _sym(9, [(0, i) for i in range(1, 7)] + [(7, 8)])                 # 7-8 is a separate component
    rp, ci, l2g, off, dl = oracle.extract_partition(g.row_ptr, g.col_idx, [3], 2)
    assert list(l2g) == [3, 0, 1, 2, 4, 5, 6]                             # 7 and 8 are never traversed
    assert rp[-1] == 12 and list(ci[rp[1]:rp[2]]) == [0, 2, 3, 4, 5, 6]   # the hub's row, in local ids, ascending


@pytest.mark.parametrize("directed", [False, True])
@pytest.mark.parametrize("L", [1, 2, 4])
def test_edge_set_equals_independent_construction(directed, L):
    n = 3000
    g = gg.random_directed(n, 4.0, 5) if directed else gg.chung_lu(n, 8.0, 2.1, 5)
    rng = np.random.default_rng(L)
    T = np.sort(rng.choice(n, size=40, replace=False)).astype(np.int64)
    rp, ci, l2g, off, dl = oracle.extract_partition(g.row_ptr, g.col_idx, T, L)
    part = gg.halo_partition(g, T, L, symmetric=not directed)
    # same vertex set
    assert np.array_equal(np.sort(l2g), part.local_to_global)
    # same edges, compared in global ids
    rows = np.repeat(np.arange(rp.size - 1), np.diff(rp))
    mine = set(zip(l2g[rows].tolist(), l2g[ci].tolist()))
    prow = np.repeat(np.arange(part.graph.n_rows), np.diff(part.graph.row_ptr))
    theirs = set(zip(part.local_to_global[prow].tolist(), part.local_to_global[part.graph.col_idx].tolist()))
    assert len(mine) == ci.size and mine == theirs
    # every kept edge is an edge of the graph, and no edge between two traversed vertices is missing
    A = g.to_scipy()
    assert all(A[a, b] != 0 for a, b in list(mine)[:500])
    held = np.zeros(n, dtype=bool)
    held[l2g] = True
    gr = np.repeat(np.arange(n), np.diff(g.row_ptr))
    assert int((held[gr] & held[g.col_idx]).sum()) == ci.size


def test_structure_prefixes_sorted_columns_and_distances():
    n, L = 5000, 3
    g = gg.chung_lu(n, 10.0, 2.1, 9)
    T = np.sort(np.random.default_rng(1).choice(n, size=60, replace=False)).astype(np.int64)
    rp, ci, l2g, off, dl = oracle.extract_partition(g.row_ptr, g.col_idx, T, L)
    assert np.array_equal(l2g[: off[1]], T)                                # targets first, ascending id
    for j in range(L + 1):                                                 # each ring ascending in global id
        assert np.all(np.diff(l2g[off[j]:off[j + 1]]) > 0)
    for i in range(rp.size - 1):                                           # columns ascending, no repeats
        assert np.all(np.diff(ci[rp[i]:rp[i + 1]]) > 0)
    # the local numbering IS the ring order: active sets of the local graph from targets 0..|T|-1 are prefixes
    d2, ring2, off2 = oracle.active_sets(rp, ci, np.arange(off[1], dtype=np.int32), L)
    assert np.array_equal(ring2, np.arange(l2g.size)) and np.array_equal(off2, off) and np.array_equal(d2, dl)
    # a row of ring j only reaches rings j-1, j, j+1 (symmetric graph)
    rows = np.repeat(np.arange(rp.size - 1), np.diff(rp))
    assert np.all(np.abs(dl[rows] - dl[ci]) <= 1)


@pytest.mark.parametrize("kind", ["gcn", "sage"])
def test_training_on_the_extracted_graph_equals_the_unpartitioned_result(kind):
    """Section 6, step 5 on top of step 1: logits, loss and weight gradients of the targets."""
    n, L = 500, 3
    g = gg.erdos_renyi(n, 3.0, 31)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    rng = np.random.default_rng(31)
    T = np.sort(rng.choice(n, size=11, replace=False)).astype(np.int64)
    params = gg.layer_weights([6, 5, 4, 3], kind == "sage", 31)
    H0 = rng.standard_normal((n, 6))
    y = rng.integers(0, 3, size=T.size).astype(np.int32)
    full = oracle.Model(g.row_ptr, g.col_idx, T, kind, params, all_rows=True)
    loss_full = full.forward(H0, y)
    rp, ci, l2g, off, dl = oracle.extract_partition(g.row_ptr, g.col_idx, T, L)
    assert l2g.size < n
    t_local = np.arange(T.size, dtype=np.int32)
    m = oracle.Model(rp, ci, t_local, kind, params, g.degrees()[l2g] if kind == "gcn" else None)
    loss = m.forward(H0[l2g], y)
    assert np.isclose(loss, loss_full, rtol=1e-12)
    assert np.allclose(m.H[-1][t_local], full.H[-1][T], rtol=1e-12, atol=1e-13)
    assert [m.rows_of_layer(l).size for l in range(1, L + 1)] == [int(off[L - l + 1]) for l in range(1, L + 1)]
    for a, b in zip(full.backward(), m.backward()):
        for k in a:
            assert np.allclose(a[k], b[k], rtol=1e-10, atol=1e-13), k


# ---- extraction after boundary sampling (section 5.3.1) ------------------------------------------------------

def _sampled(g, T, fanout, seed):
    is_t = np.zeros(g.n_rows, dtype=np.uint8)
    is_t[T] = 1
    return oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, fanout, seed)


def test_sampled_extraction_closed_form():
    """Path 0-1-2-3-4-5 plus the chord 2-5, targets {2, 3}, everything kept (fanout 9): outside vertices 1, 4, 5;
    local order 2 3 | 1 4 5 -> ids 0 1 | 2 3 4; kept edges 2-3, 2-1, 2-5, 3-4 and their reverses; no 4-5 edge."""
    g = _sym(6, [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5), (2, 5)])
    T = np.array([2, 3])
    srp, sci = _sampled(g, T, 9, 1)
    rp, ci, l2g, off, dl = oracle.extract_sampled(6, T, srp, sci)
    assert list(l2g) == [2, 3, 1, 4, 5] and list(off) == [0, 2, 5] and list(dl) == [0, 0, 1, 1, 1]
    rows = [list(ci[rp[i]:rp[i + 1]]) for i in range(5)]
    assert rows == [[1, 2, 4], [0, 3], [0], [1], [0]]


@pytest.mark.parametrize("fanout", [0, 2, 5, 1000])
def test_sampled_extraction_equals_edge_list_construction(fanout):
    """Against the edge-list construction used since the first sampler tests (oracle.sampled_local_edges + scipy
    assembly in graphgen.partition_from_edges, ascending-id numbering), compared in global ids."""
    n = 4000
    g = gg.chung_lu(n, 12.0, 2.1, 71)
    T = np.sort(np.random.default_rng(fanout).choice(n, 400, replace=False)).astype(np.int64)
    srp, sci = _sampled(g, T, fanout, 99)
    rp, ci, l2g, off, dl = oracle.extract_sampled(n, T, srp, sci)
    l2g_ref, er, ec = oracle.sampled_local_edges(T, srp, sci)
    assert np.array_equal(np.sort(l2g), l2g_ref) and np.array_equal(l2g[: len(T)], T)
    rows = np.repeat(np.arange(rp.size - 1), np.diff(rp))
    mine = set(zip(l2g[rows].tolist(), l2g[ci].tolist()))
    assert len(mine) == ci.size and mine == set(zip(er.tolist(), ec.tolist()))
    part = gg.partition_from_edges(n, l2g_ref, er, ec, T, g.degrees())
    assert part.graph.nnz == ci.size
    # structure: symmetric, target rows = kept rows, outside rows only reach targets, columns ascending
    assert mine == {(b, a) for a, b in mine}
    assert np.array_equal(np.diff(rp)[: len(T)], np.diff(srp))
    assert np.all(ci[rp[len(T)]:] < len(T))
    for i in range(rp.size - 1):
        assert np.all(np.diff(ci[rp[i]:rp[i + 1]]) > 0)
    if fanout == 0:
        assert l2g.size == len(T)                                          # nothing outside survives
    if fanout == 1000:                                                     # nothing is dropped: the one-hop halo, minus outside-outside edges
        rp1, ci1, l2g1, off1, _ = oracle.extract_partition(g.row_ptr, g.col_idx, T, 1)
        assert np.array_equal(l2g1, l2g)
        r1 = np.repeat(np.arange(rp1.size - 1), np.diff(rp1))
        keep = (r1 < len(T)) | (ci1 < len(T))
        assert np.array_equal(r1[keep], rows) and np.array_equal(ci1[keep], ci)


def test_sampled_extraction_rejects_unsorted_targets():
    g = _sym(4, [(0, 1), (1, 2), (2, 3)])
    srp, sci = _sampled(g, np.array([1, 2]), 3, 0)
    with pytest.raises(ValueError):
        oracle.extract_sampled(4, np.array([2, 1]), srp, sci)
