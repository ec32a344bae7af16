"""GPU parity: gnn_eas_traverse against the oracle's expansion-aware traversal, bit-exact (section 5.3.1: at most h
hops from the inner vertices, at most f kept neighbours per traversed vertex; best-connected-first or seeded hash),
and the sub-graph of the traversed vertices (gnn_extract_partition on the traversal's outputs)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _compare(g, targets, hops, fanout, rule, seed=0):
    import paper_2311_06837_amd as P
    print(f"eas traverse: n={g.n_rows} nnz={g.nnz} |T|={len(targets)} h={hops} f={fanout} rule={rule} seed={seed}", flush=True)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    t = dev(np.asarray(targets, dtype=np.int32))
    dist, ring, off, hop = P.gnn_eas_traverse(G, t, hops, fanout, rule, seed)
    torch.cuda.synchronize()
    od, oring, ooff = oracle.eas_traverse(g.row_ptr, g.col_idx, np.asarray(targets, dtype=np.int32), hops, fanout, rule, seed)
    assert list(hop) == list(ooff) and np.array_equal(off.cpu().numpy(), ooff)
    assert np.array_equal(dist.cpu().numpy(), od)
    assert np.array_equal(ring.cpu().numpy()[: ooff[-1]], oring)
    return G, dist, ring, hop


def _sym(n, und):
    r = np.array([a for a, b in und] + [b for a, b in und], dtype=np.int64)
    c = np.array([b for a, b in und] + [a for a, b in und], dtype=np.int64)
    return gg.csr_from_edges(n, n, r, c)


def test_hand_worked_example():
    g = _sym(8, [(0, 1), (0, 2), (0, 3), (1, 3), (1, 4), (2, 5), (3, 5), (3, 6), (3, 7), (4, 6), (6, 7)])
    _, dist, ring, hop = _compare(g, [0, 1], 2, 1, "degree")
    assert ring.cpu().numpy()[:4].tolist() == [0, 1, 3, 6] and list(hop) == [0, 2, 3, 4]
    _compare(g, [0, 1], 2, 2, "degree")
    _compare(g, [1, 0], 2, 1, "hash", seed=3)


@pytest.mark.parametrize("rule", ["degree", "hash"])
@pytest.mark.parametrize("hops,fanout", [(1, 15), (1, 25), (2, 15), (2, 25), (3, 15), (3, 25),     # the paper's sensitivity grid (section 8.5)
                                         (1, 5), (2, 3), (2, 1)])
def test_power_law_graph(rule, hops, fanout):
    g = gg.chung_lu(40000, 18.0, 2.1, 11)
    T = np.sort(np.random.default_rng(hops * 100 + fanout).choice(40000, 700, replace=False))
    _compare(g, T, hops, fanout, rule, seed=12345 + fanout)


@pytest.mark.parametrize("rule", ["degree", "hash"])
def test_long_rows_and_ragged_sizes(rule):
    g = gg.chung_lu(30011, 120.0, 2.1, 5)                       # rows far longer than 16 lanes x fanout
    assert g.degrees().max() > 1000
    T = np.arange(0, 30011, 211)
    _compare(g, T, 2, 7, rule, seed=9)
    d = gg.random_directed(10007, 6.0, 2)                       # directed: rows are what a vertex aggregates
    _compare(d, np.arange(0, 10007, 37), 3, 2, rule, seed=4)
    big = gg.chung_lu(20000, 1500.0, 2.1, 8)                    # rows with more candidates than a wavefront lists in LDS
    assert big.degrees().max() > 4096
    _compare(big, np.arange(0, 20000, 501), 2, 30, rule, seed=2)
    _compare(big, np.arange(0, 20000, 501), 1, 1500, rule, seed=3)     # a fanout above the list size


@pytest.mark.parametrize("rule", ["degree", "hash"])
def test_edge_cases(rule):
    g = gg.erdos_renyi(700, 5.0, 3)
    _compare(g, [], 2, 3, rule)                                 # no inner vertices
    _compare(g, [5, 9, 11], 2, 0, rule)                         # fanout 0: nothing is selected
    _compare(g, [5, 9, 11], 4, 10**6, rule)                     # nothing dropped: plain breadth-first rings
    _compare(g, np.arange(700), 2, 3, rule)                     # everything is inner
    _compare(g, [3, 3, 8, 8, 8], 2, 2, rule)                    # repeated inner vertices
    empty = gg.CSR(70, 70, np.zeros(71, dtype=np.int32), np.zeros(0, dtype=np.int32))
    _compare(empty, [1, 2], 2, 3, rule)


def test_induced_subgraph_of_the_traversed_vertices():
    """Section 5.3.1: the local graph is the sub-graph on the vertices the traversal reached - the extraction call takes
    the traversal's outputs as it takes those of the plain active sets."""
    import paper_2311_06837_amd as P
    g = gg.chung_lu(20000, 15.0, 2.1, 6)
    T = np.sort(np.random.default_rng(1).choice(20000, 2500, replace=False))
    hops, fanout = 2, 4
    G, dist, ring, hop = _compare(g, T, hops, fanout, "degree")
    n_local = hop[-1]
    local, new_id = P.gnn_extract_partition(G, ring, n_local, dist, hops)
    torch.cuda.synchronize()
    od, oring, ooff = oracle.eas_traverse(g.row_ptr, g.col_idx, T.astype(np.int32), hops, fanout, "degree")
    orp, oci = oracle.extract_from_ring(g.row_ptr, g.col_idx, oring)
    assert np.array_equal(local.row_ptr.cpu().numpy(), orp)
    assert np.array_equal(local.col_idx.cpu().numpy()[: orp[-1]], oci)
