"""GPU parity: gnn_build_active_sets against the oracle, bit-exact (section 6, steps 1 and 4)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _run(g, targets, L, with_transpose):
    import paper_2311_06837_amd as P
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    GT = None
    if with_transpose:
        t = gg.transpose(g)
        GT = P.Graph.from_numpy(t.row_ptr, t.col_idx)
    t = dev(np.asarray(targets, dtype=np.int32))
    dist, ring, off, hop = P.gnn_build_active_sets(G, t, L, gt=GT)
    torch.cuda.synchronize()
    return dist.cpu().numpy(), ring.cpu().numpy(), off.cpu().numpy(), hop


def _compare(g, targets, L):
    """Both forms of the call - every level from the frontier, and with the transposed graph (levels may then run from
    the unreached vertices) - against the oracle's plain breadth-first levels."""
    valid = np.asarray(targets, dtype=np.int64)
    valid = valid[(valid >= 0) & (valid < g.n_rows)]
    od, oring, ooff = oracle.active_sets(g.row_ptr, g.col_idx, valid.astype(np.int32), L)
    for with_transpose in (False, True):
        print(f"active sets: n={g.n_rows} nnz={g.nnz} |T|={len(targets)} L={L} transposed graph given: {with_transpose}", flush=True)
        dist, ring, off, hop = _run(g, targets, L, with_transpose)
        assert np.array_equal(off, ooff) and list(hop) == list(ooff)
        assert np.array_equal(dist, od)
        assert np.array_equal(ring[: ooff[-1]], oring)


def _sym(n, und):
    r = np.array([a for a, b in und] + [b for a, b in und], dtype=np.int64)
    c = np.array([b for a, b in und] + [a for a, b in und], dtype=np.int64)
    return gg.csr_from_edges(n, n, r, c)


def test_closed_form_graphs():
    _compare(_sym(21, [(i, i + 1) for i in range(20)]), [10], 4)
    _compare(_sym(9, [(0, i) for i in range(1, 9)]), [0], 3)            # empty late rings
    _compare(_sym(8, [(0, 1), (1, 2), (2, 3), (4, 5), (5, 6), (6, 7)]), [0], 5)   # unreachable part
    _compare(_sym(12, [(i, j) for i in range(12) for j in range(i + 1, 12)]), [2, 5], 3)


@pytest.mark.parametrize("seed", [0, 1])
def test_random_graphs_directed_and_symmetric(seed):
    rng = np.random.default_rng(seed)
    g = gg.erdos_renyi(20000, 6.0, seed)
    _compare(g, rng.choice(20000, 300, replace=False), 3)
    d = gg.random_directed(30011, 3.0, seed)                              # ragged bitmap tail
    _compare(d, rng.choice(30011, 500, replace=False), 5)


def test_power_law_with_hub_rows():
    g = gg.chung_lu(60000, 60.0, 2.1, 7)                                  # max degree ~ 1900
    assert g.degrees().max() > 1024
    _compare(g, np.arange(0, 60000, 97), 2)
    big = gg.chung_lu(20000, 1500.0, 2.1, 8)                              # rows above the 4096 hub split
    assert big.degrees().max() > 4096
    _compare(big, np.arange(0, 20000, 501), 2)


def test_edge_cases():
    g = gg.erdos_renyi(500, 4.0, 3)
    _compare(g, [], 2)                                                    # no targets
    _compare(g, [7, 7, 7, 3, 3], 2)                                       # repeated targets
    _compare(g, [5, -1, 500, 10**6, 9], 2)                                # out-of-range ids are ignored
    _compare(g, np.arange(500), 1)                                        # everything is a target
    empty = gg.CSR(64, 64, np.zeros(65, dtype=np.int32), np.zeros(0, dtype=np.int32))
    _compare(empty, [1, 2, 3], 3)                                         # no edges
    _compare(g, [0], 40)                                                  # far more levels than the diameter


def test_deep_shrinking_sets_like_cfg3():
    w = gg.make_workload("cfg3", scale=0.03)
    p = w.partition
    _compare(p.graph, p.targets, w.n_layers)


def test_levels_that_run_from_the_unreached_vertices():
    """Graphs on which the direction switch picks the pull form: a frontier that is most of the graph (dense power
    law), directed edges (the transposed rows differ from the rows), a long transposed row that is still unreached
    when the switch happens (its own workgroup), and unreached vertices that no frontier vertex reaches."""
    g = gg.chung_lu(50000, 200.0, 2.1, 17)                                # ring 1 is most of the graph
    _compare(g, np.arange(0, 50000, 9), 3)
    d = gg.random_directed(40000, 40.0, 5)
    _compare(d, np.arange(0, 40000, 7), 4)
    # Long transposed rows that are still unreached when a level pulls (a workgroup each): the centre of a star in a
    # component the targets do not touch (no entry is in the frontier), and a vertex that 3000 vertices of the dense
    # part aggregate from while it aggregates from nobody (reached by the pull, through one of them).
    na = 30000
    dense = gg.chung_lu(na, 100.0, 2.1, 3)
    centre, leaves = na, np.arange(na + 1, na + 5001)
    h = na + 5001
    n = h + 1
    fans = np.arange(1, na, 10)[:3000]                                    # no target among them (targets are multiples of 10)
    rows = np.concatenate([np.repeat(np.arange(na), np.diff(dense.row_ptr)), np.full(5000, centre), leaves, fans])
    cols = np.concatenate([dense.col_idx.astype(np.int64), leaves, np.full(5000, centre), np.full(3000, h)])
    g2 = gg.csr_from_edges(n, n, rows, cols)
    assert np.diff(gg.transpose(g2).row_ptr)[[centre, h]].min() >= 3000
    _compare(g2, np.arange(0, na, 10), 3)
    iso = gg.csr_from_edges(n, n, np.repeat(np.arange(n // 2), 60),
                            np.random.default_rng(0).integers(0, n // 2, 60 * (n // 2)))   # half the graph is unreachable
    _compare(iso, np.arange(0, n // 2, 5), 3)
