"""GPU parity: gnn_sample_boundary and gnn_make_bitmap against the oracle, bit-exact
(section 5.3 with the seeded hash rule)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _compare(g, T, fanout, seed):
    import paper_2311_06837_amd as P
    print(f"sampling: n={g.n_rows} nnz={g.nnz} |T|={len(T)} f={fanout} seed={seed:#x}", flush=True)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = dev(np.asarray(T, dtype=np.int32))
    bits = P.gnn_make_bitmap(Td, g.n_rows)
    rp, ci = P.gnn_sample_boundary(G, bits, Td, fanout, seed)
    torch.cuda.synchronize()
    is_t = np.zeros(g.n_rows, dtype=np.uint8)
    is_t[T] = 1
    want_bits = np.packbits(is_t.astype(bool), bitorder="little")
    got_bits = bits.cpu().numpy().view(np.uint8)[: want_bits.size]
    assert np.array_equal(got_bits, want_bits)
    orp, oci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, fanout, seed)
    assert np.array_equal(rp.cpu().numpy(), orp)
    assert np.array_equal(ci.cpu().numpy(), oci)


@pytest.mark.parametrize("fanout", [0, 1, 5, 15])
def test_power_law_partition(fanout):
    g = gg.chung_lu(40000, 15.0, 2.1, 31)
    pid = gg.bfs_partition(g, 8, 31)
    T = np.flatnonzero(pid == 0).astype(np.int32)
    _compare(g, T, fanout, 0x5EED0004)


def test_hub_rows_and_large_fanout_and_seed_range():
    g = gg.chung_lu(8000, 300.0, 2.1, 32)                 # rows far longer than one wavefront
    assert g.degrees().max() > 1200
    T = np.arange(0, 8000, 3).astype(np.int32)
    _compare(g, T, 5, 1)
    _compare(g, T, 70, 2**64 - 1)                         # fanout above the wavefront width; seed + hop wraps
    _compare(g, T, int(g.degrees().max()), 3)             # keeps everything


def test_unsorted_targets_and_edge_cases():
    g = gg.erdos_renyi(3000, 8.0, 33)
    rng = np.random.default_rng(0)
    T = rng.permutation(3000)[:1025].astype(np.int32)     # ragged count, arbitrary order
    _compare(g, T, 2, 9)
    _compare(g, np.zeros(0, dtype=np.int32), 2, 9)        # no targets
    _compare(g, np.arange(3000, dtype=np.int32), 2, 9)    # no outside neighbours at all


def test_row_lengths_around_the_sixteen_lane_limit():
    """Rows of 63 / 64 / 65 entries (the last one leaves its sixteen lanes for a workgroup), of 1023 / 1024 / 1025 (one step
    of that workgroup's sweep, then two) and an empty one, targets and outside vertices mixed in every row."""
    rng = np.random.default_rng(35)
    n = 5000
    lens = [63, 64, 65, 0, 1023, 1024, 1025, 1, 256, 257]
    rows, cols = [], []
    for r, ln in enumerate(lens):
        c = rng.choice(n, size=ln, replace=False)
        rows.append(np.full(ln, r, dtype=np.int64))
        cols.append(c.astype(np.int64))
    g = gg.csr_from_edges(n, n, np.concatenate(rows), np.concatenate(cols))
    assert list(g.degrees()[: len(lens)]) == lens
    T = np.concatenate([np.arange(len(lens)), np.arange(100, n, 2)]).astype(np.int32)   # about half of every row is inside
    for fanout in (0, 3, 40, 600):
        _compare(g, T, fanout, 0xABCDEF)
