"""GPU parity: gnn_masked_spmm_fwd / _bwd against the oracle (section 2.1 aggregation under
the section 6 mask).  fp32: 1e-4, bf16 storage: 2e-2 (see gpu_util.TOL)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import as_stored, check, dev, host64, padded

pytestmark = pytest.mark.gpu

SENTINEL = 12345.0


def _used_blocked_route(ws):
    """The size query reports 0 bytes when the column-blocked route does not apply, so the workspace stays minimal."""
    return ws is not None and ws.buf is not None and ws.buf.numel() > 256


def _fwd_case(g, F, ld, dtype, rows, scales, seed, ws=None):
    import paper_2311_06837_amd as P
    print(f"spmm fwd: n={g.n_rows} nnz={g.nnz} F={F} ld={ld} {dtype} rows={'list' if rows is not None else 'all'} "
          f"scales={scales}", flush=True)
    rng = np.random.default_rng(seed)
    n = g.n_rows
    X = as_stored(rng.standard_normal((n, F)), dtype)
    rs = (rng.random(n) + 0.5).astype(np.float32) if scales else None
    cs = (rng.random(n) + 0.5).astype(np.float32) if scales else None
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Xd = padded(X, ld, dtype, fill=float("nan") if ld > F else 0.0)       # pad columns must never matter
    if ld > F and ld - F >= 1:
        Xd[:, F:] = float("nan")
    Yd = torch.full((n, ld), SENTINEL, dtype=dtype, device="cuda")
    rows_d = dev(rows) if rows is not None else None
    n_active = len(rows) if rows is not None else n
    P.gnn_masked_spmm_fwd(G, rows_d, n_active, Xd, Yd, F, dev(rs) if scales else None, dev(cs) if scales else None, ws=ws)
    torch.cuda.synchronize()
    want = np.full((n, F), SENTINEL)
    oracle.spmm_fwd(g.row_ptr, g.col_idx, rows, X, want, F, rs, cs)
    got = host64(Yd)
    sel = np.asarray(rows if rows is not None else np.arange(n))
    check(got[sel, :F], want[sel], dtype, "active rows")
    rest = np.setdiff1d(np.arange(n), sel)
    assert (got[rest] == host64(torch.tensor(SENTINEL, dtype=dtype))).all(), "masked rows were written"
    if ld > F:
        assert (got[:, F:] == host64(torch.tensor(SENTINEL, dtype=dtype))).all(), "pad columns were written"


def _fwd_add_case(g, F, ld, dtype, rows, relu, seed, ws=None, bias=False):
    """gnn_masked_spmm_fwd_add: Y = act(Y + aggregation).  The oracle aggregates into a zeroed matrix; the sum with
    the self term and the ReLU are written out here (in the storage precision of the self term).  bias: the form
    without a self term - the listed rows start from a bias vector, whatever the output matrix held."""
    import paper_2311_06837_amd as P
    print(f"spmm fwd_add: n={g.n_rows} nnz={g.nnz} F={F} ld={ld} {dtype} rows={'list' if rows is not None else 'all'} relu={relu}",
          flush=True)
    rng = np.random.default_rng(seed)
    n = g.n_rows
    X = as_stored(rng.standard_normal((n, F)), dtype)
    S = as_stored(rng.standard_normal((n, F)), dtype)
    rs = (1.0 / np.maximum(g.degrees(), 1)).astype(np.float32)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Xd = padded(X, ld, dtype)
    Yd = torch.full((n, ld), SENTINEL, dtype=dtype, device="cuda")
    Yd[:, :F] = padded(S, F, dtype)
    rows_d = dev(rows) if rows is not None else None
    n_active = len(rows) if rows is not None else n
    b = (rng.standard_normal(F) * 0.5).astype(np.float32) if bias else None
    P.gnn_masked_spmm_fwd_add(G, rows_d, n_active, Xd, Yd, F, dev(rs), None, relu=relu, ws=ws, bias=dev(b) if bias else None)
    torch.cuda.synchronize()
    agg = np.zeros((n, F))
    oracle.spmm_fwd(g.row_ptr, g.col_idx, rows, X, agg, F, rs, None)
    start = np.broadcast_to(as_stored(b.astype(np.float64), dtype), (n, F)) if bias else S
    want = start + agg
    if relu:
        want = np.maximum(want, 0.0)
    got = host64(Yd)
    sel = np.asarray(rows if rows is not None else np.arange(n))
    check(got[sel, :F], want[sel], dtype, "active rows")
    if relu:
        assert (got[sel, :F] >= 0).all()
        # a row without neighbours still gets its activation
        empty = sel[g.degrees()[sel] == 0]
        assert np.array_equal(got[empty, :F], np.maximum(start[empty], 0.0))
    rest = np.setdiff1d(np.arange(n), sel)
    assert np.array_equal(got[rest, :F], S[rest]), "masked rows were written"
    if ld > F:
        assert (got[:, F:] == host64(torch.tensor(SENTINEL, dtype=dtype))).all(), "pad columns were written"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("relu", [False, True])
def test_fwd_add_on_top_of_the_self_term(dtype, relu):
    g = gg.chung_lu(3000, 6.0, 2.1, 13)
    assert (g.degrees() == 0).any()
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(3000, 1777, replace=False)).astype(np.int32)
    _fwd_add_case(g, 256, 256, dtype, None, relu, 51)
    _fwd_add_case(g, 100, 104, dtype, rows, relu, 52)
    _fwd_add_case(g, 7, 7, dtype, rows, relu, 53)            # element-wise lanes
    _fwd_add_case(g, 16, 16, dtype, rows, relu, 54)          # narrow rows
    _fwd_add_case(g, 41, 48, dtype, None, relu, 55)
    _fwd_add_case(g, 47, 48, dtype, rows, relu, 56, bias=True)     # no self term: the rows start from the bias
    _fwd_add_case(g, 256, 256, dtype, None, relu, 57, bias=True)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("F,ld", [(64, 64), (100, 100), (128, 128), (256, 256), (602, 608), (602, 602), (7, 7), (1, 8),
                                  (300, 304), (1000, 1000), (16, 16), (32, 32), (41, 44), (47, 48)])
def test_fwd_widths(dtype, F, ld):
    g = gg.chung_lu(3000, 20.0, 2.1, 11)
    rng = np.random.default_rng(F)
    rows = np.sort(rng.choice(3000, 1777, replace=False)).astype(np.int32)
    _fwd_case(g, F, ld, dtype, rows, True, F)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fwd_hub_rows_empty_rows_and_all_rows(dtype):
    g = gg.chung_lu(12000, 150.0, 2.1, 12)                                # hub rows > 1024 neighbours
    assert g.degrees().max() > 1024
    _fwd_case(g, 128, 128, dtype, None, True, 1)
    _fwd_case(g, 602, 608, dtype, None, False, 2)
    d = gg.random_directed(5000, 1.5, 13)                                 # many empty rows
    assert (d.degrees() == 0).any()
    _fwd_case(d, 64, 64, dtype, None, True, 3)
    rows = np.random.default_rng(0).permutation(5000)[:3001].astype(np.int32)     # unsorted row list, ragged count
    _fwd_case(d, 100, 100, dtype, rows, False, 4)


def test_fwd_sum_of_ones_is_degree_exactly():
    import paper_2311_06837_amd as P
    g = gg.chung_lu(20000, 80.0, 2.1, 14)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    X = torch.ones(20000, 64, device="cuda")
    Y = torch.zeros(20000, 64, device="cuda")
    P.gnn_masked_spmm_fwd(G, None, 20000, X, Y, 64)
    assert torch.equal(Y[:, 0].cpu(), torch.from_numpy(g.degrees()).float())     # integers < 2^24 are exact in fp32
    assert torch.equal(Y, Y[:, :1].expand(-1, 64))


def test_fwd_is_bitwise_reproducible():
    import paper_2311_06837_amd as P
    g = gg.chung_lu(12000, 150.0, 2.1, 12)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    X = torch.randn(12000, 256, device="cuda", generator=torch.Generator("cuda").manual_seed(0))
    outs = []
    for _ in range(3):
        Y = torch.zeros(12000, 256, device="cuda")
        P.gnn_masked_spmm_fwd(G, None, 12000, X, Y, 256)
        outs.append(Y)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def _bwd_case(g, F, ld, dtype, L, lyr, accumulate, seed, ws=None, relu=False):
    """Backward of layer `lyr` of an L-layer model: forward rows R_lyr, outputs for R_{lyr-1}.  relu: the call also
    undoes the ReLU of the layer in front (what it stores is zeroed where that layer's activations are <= 0)."""
    import paper_2311_06837_amd as P
    print(f"spmm bwd: n={g.n_rows} nnz={g.nnz} F={F} ld={ld} {dtype} L={L} layer={lyr} acc={accumulate} relu={relu}", flush=True)
    rng = np.random.default_rng(seed)
    n = g.n_rows
    T = np.sort(rng.choice(n, max(1, n // 50), replace=False)).astype(np.int32)
    dist, ring, off = oracle.active_sets(g.row_ptr, g.col_idx, T, L)
    rows_f = ring[: off[L - lyr + 1]]                 # R_lyr
    rows_o = ring[: off[L - lyr + 2]]                 # R_{lyr-1}
    gt = gg.transpose(g)
    dY = as_stored(rng.standard_normal((n, F)), dtype)
    rs = (rng.random(n) + 0.5).astype(np.float32)
    cs = (rng.random(n) + 0.5).astype(np.float32)
    init = as_stored(rng.standard_normal((n, F)), dtype) if accumulate else np.full((n, F), SENTINEL)
    GT = P.Graph.from_numpy(gt.row_ptr, gt.col_idx)
    dYd = padded(dY, ld, dtype)
    dXd = padded(init, ld, dtype, fill=SENTINEL)
    Hact = as_stored(np.maximum(rng.standard_normal((n, F)), 0), dtype) if relu else None     # about half of it is zero
    P.gnn_masked_spmm_bwd(GT, dev(rows_o), len(rows_o), dev(dist), L - lyr, dYd, dXd, F, dev(rs), dev(cs), accumulate=accumulate,
                          ws=ws, relu_H=padded(Hact, ld, dtype, fill=float("nan") if ld > F else 0.0) if relu else None)
    torch.cuda.synchronize()
    want = np.zeros((n, F))
    oracle.spmm_bwd(g.row_ptr, g.col_idx, rows_f, dY, want, F, rs, cs)
    # everything the adjoint touches lies inside R_{lyr-1}
    outside = np.setdiff1d(np.arange(n), rows_o)
    assert not want[outside].any()
    if accumulate:
        want = want + init
    if relu:
        want = want * (Hact > 0)
    got = host64(dXd)
    check(got[rows_o, :F], want[rows_o], dtype, "bwd rows")
    assert (got[outside, :F] == host64(padded(init, ld, dtype, fill=SENTINEL))[outside, :F]).all(), "rows outside were written"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("accumulate", [False, True])
def test_bwd_directed_graph_with_filter(dtype, accumulate):
    g = gg.random_directed(8000, 6.0, 21)
    _bwd_case(g, 128, 128, dtype, 3, 3, accumulate, 5)
    _bwd_case(g, 256, 256, dtype, 3, 2, accumulate, 6)
    _bwd_case(g, 602, 608, dtype, 2, 2, accumulate, 7)
    _bwd_case(g, 16, 16, dtype, 3, 2, accumulate, 8)                     # narrow rows: 4 / 8 lanes per row
    _bwd_case(g, 41, 48, dtype, 3, 3, accumulate, 9)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("accumulate", [False, True])
def test_bwd_that_undoes_the_relu_in_front(dtype, accumulate):
    g = gg.random_directed(8000, 6.0, 22)
    _bwd_case(g, 128, 128, dtype, 3, 3, accumulate, 15, relu=True)
    _bwd_case(g, 602, 608, dtype, 2, 2, accumulate, 16, relu=True)
    _bwd_case(g, 100, 100, dtype, 2, 2, accumulate, 17, relu=True)       # unaligned for bf16: element route
    _bwd_case(g, 7, 7, dtype, 2, 2, accumulate, 18, relu=True)
    h = gg.chung_lu(12000, 150.0, 2.1, 12)                                # hub rows: reduced through LDS, then masked
    _bwd_case(h, 64, 64, dtype, 2, 2, accumulate, 19, relu=True)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_bwd_power_law_hubs(dtype):
    g = gg.chung_lu(12000, 150.0, 2.1, 12)
    _bwd_case(g, 64, 64, dtype, 2, 2, False, 8)
    _bwd_case(g, 100, 100, dtype, 3, 2, True, 9)
    _bwd_case(g, 16, 16, dtype, 2, 2, True, 10, relu=True)               # hub rows reduced by 64 narrow lane groups
    _bwd_case(g, 32, 32, dtype, 2, 2, False, 11)


def test_empty_calls_are_noops():
    import paper_2311_06837_amd as P
    g = gg.erdos_renyi(100, 3.0, 1)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    with pytest.raises(P.GnnError):             # a source prefix is -1 (none) or a vertex count
        z = torch.zeros(100, 8, device="cuda")
        P.gnn_masked_spmm_bwd(G, None, 100, None, 0, z, torch.zeros_like(z), 8, src_prefix=-2)
    X = torch.randn(100, 8, device="cuda")
    Y = torch.full((100, 8), 3.0, device="cuda")
    P.gnn_masked_spmm_fwd(G, None, 0, X, Y, 8)
    P.gnn_masked_spmm_fwd(G, None, 100, X, Y, 0)
    torch.cuda.synchronize()
    assert (Y == 3.0).all()


# ---- column-blocked route (dense graph + workspace) ------------------------------------------

_DENSE = {}


def _dense_graph():
    """70k vertices (a 256-byte feature slab of 17.9 MB), average row length 90, plus one vertex adjacent to
    20k others, so that one of its column blocks alone is longer than the hub threshold."""
    if "g" not in _DENSE:
        n = 70000
        base = gg.erdos_renyi(n, 88.0, 31)
        rng = np.random.default_rng(32)
        nb = rng.choice(n - 1, 20000, replace=False).astype(np.int64) + 1      # neighbours of vertex 0
        r = np.repeat(np.arange(n, dtype=np.int64), np.diff(base.row_ptr))
        c = base.col_idx.astype(np.int64)
        z = np.zeros_like(nb)
        _DENSE["g"] = gg.csr_from_edges(n, n, np.concatenate([r, z, nb]), np.concatenate([c, nb, z]))
    return _DENSE["g"]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_blocked_route_forward(dtype):
    import paper_2311_06837_amd as P
    g = _dense_graph()
    assert g.nnz / g.n_rows >= 64 and g.degrees()[0] > 8 * 1024
    ws = P.Workspace()
    _fwd_case(g, 200, 200, dtype, None, True, 41, ws=ws)                  # 4 (fp32) / 2 (bf16) slabs, ragged last slab
    assert _used_blocked_route(ws)
    rows = np.random.default_rng(5).permutation(g.n_rows)[:40001].astype(np.int32)   # unsorted list, ragged count
    if 0 not in rows:
        rows[17] = 0
    _fwd_case(g, 602, 608, dtype, rows, False, 42, ws=ws)
    _fwd_case(g, 64, 64, dtype, rows, True, 43, ws=ws)                    # a single slab


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_blocked_route_forward_add(dtype):
    import paper_2311_06837_amd as P
    g = _dense_graph()
    ws = P.Workspace()
    _fwd_add_case(g, 200, 200, dtype, None, True, 44, ws=ws)
    assert _used_blocked_route(ws)
    rows = np.random.default_rng(6).permutation(g.n_rows)[:40001].astype(np.int32)
    _fwd_add_case(g, 256, 256, dtype, rows, False, 45, ws=ws)
    _fwd_add_case(g, 90, 96, dtype, rows, True, 46, ws=ws)
    _fwd_add_case(g, 200, 200, dtype, rows, True, 47, ws=ws, bias=True)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("accumulate", [False, True])
def test_blocked_route_backward_with_filter(dtype, accumulate):
    import paper_2311_06837_amd as P
    g = _dense_graph()
    ws = P.Workspace()
    _bwd_case(g, 136, 136, dtype, 2, 2, accumulate, 44, ws=ws)            # forward rows = targets only: most neighbours filtered out
    assert _used_blocked_route(ws)
    _bwd_case(g, 136, 136, dtype, 2, 2, accumulate, 45, ws=ws, relu=True)  # the plane sum undoes the ReLU in front


def test_blocked_route_falls_back_without_promise_or_density():
    """Unsorted columns (no GNN_CSR_SORTED_COLUMNS promise) or a sparse graph: the size query reports 0 and the
    call gathers whole rows."""
    import paper_2311_06837_amd as P
    g = _dense_graph()
    ws = P.Workspace()
    G = P.Graph(dev(g.row_ptr), dev(g.col_idx), sorted_columns=False)
    X = torch.randn(g.n_rows, 64, device="cuda")
    Y1, Y2 = torch.zeros_like(X), torch.zeros_like(X)
    P.gnn_masked_spmm_fwd(G, None, g.n_rows, X, Y1, 64, ws=ws)
    assert not _used_blocked_route(ws)
    Gs = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    assert Gs.sorted_columns
    P.gnn_masked_spmm_fwd(Gs, None, g.n_rows, X, Y2, 64, ws=ws)
    assert _used_blocked_route(ws)
    assert (Y1 - Y2).abs().max() <= 1e-4 * Y1.abs().max()                 # the two routes differ by rounding order only
    sparse = gg.chung_lu(80000, 12.0, 2.1, 33)
    ws2 = P.Workspace()
    _fwd_case(sparse, 128, 128, torch.float32, None, True, 45, ws=ws2)
    assert not _used_blocked_route(ws2)


def test_blocked_route_backward_with_prefix_active_sources():
    """After a (distance, id) renumbering the forward rows are a PREFIX of the id range: every kept neighbour falls
    into the first stretch of ids.  The route balances its column blocks over the active vertices; results as ever."""
    import paper_2311_06837_amd as P
    g = _dense_graph()
    n, F = g.n_rows, 96
    rng = np.random.default_rng(77)
    n_fwd = 9000                                                          # forward rows 0 .. 8999
    dist = np.where(np.arange(n) < n_fwd, 0, 1).astype(np.int32)
    dY = as_stored(rng.standard_normal((n, F)), torch.float32)
    rs = (rng.random(n) + 0.5).astype(np.float32)
    cs = (rng.random(n) + 0.5).astype(np.float32)
    GT = P.Graph.from_numpy(g.row_ptr, g.col_idx)                         # symmetric
    ws = P.Workspace()
    dX = torch.full((n, F), SENTINEL, device="cuda")
    P.gnn_masked_spmm_bwd(GT, None, n, dev(dist), 0, dev(dY).float(), dX, F, dev(rs), dev(cs), accumulate=False, ws=ws)
    torch.cuda.synchronize()
    assert _used_blocked_route(ws)
    want = np.zeros((n, F))
    oracle.spmm_bwd(g.row_ptr, g.col_idx, np.arange(n_fwd, dtype=np.int32), dY, want, F, rs, cs)
    check(host64(dX), want, torch.float32, "prefix-active backward")


def _prefix_case(g, n_fwd, F, dtype, seed, sorted_promise=True, ws=None, accumulate=False, relu=False, out_rows=None):
    """Backward aggregation whose forward rows were the ids 0 .. n_fwd-1, told through src_prefix instead of a
    distance array.  The oracle gets the same thing as an explicit row list."""
    import paper_2311_06837_amd as P
    print(f"spmm bwd src_prefix: n={g.n_rows} nnz={g.nnz} n_fwd={n_fwd} F={F} {dtype} sorted={sorted_promise} acc={accumulate} "
          f"relu={relu}", flush=True)
    rng = np.random.default_rng(seed)
    n = g.n_rows
    gt = gg.transpose(g)
    dY = as_stored(rng.standard_normal((n, F)), dtype)
    rs = (rng.random(n) + 0.5).astype(np.float32)
    cs = (rng.random(n) + 0.5).astype(np.float32)
    init = as_stored(rng.standard_normal((n, F)), dtype) if accumulate else np.full((n, F), SENTINEL)
    Hact = as_stored(np.maximum(rng.standard_normal((n, F)), 0), dtype) if relu else None
    GT = P.Graph.from_numpy(gt.row_ptr, gt.col_idx)
    assert GT.sorted_columns
    if not sorted_promise:
        GT = P.Graph(GT.row_ptr, GT.col_idx, None, sorted_columns=False)     # same arrays, no promise: tested entry by entry
    rows_o = np.arange(n, dtype=np.int32) if out_rows is None else out_rows
    dXd = padded(init, F, dtype)
    P.gnn_masked_spmm_bwd(GT, None if out_rows is None else dev(rows_o), len(rows_o), None, 0, padded(dY, F, dtype), dXd, F, dev(rs),
                          dev(cs), accumulate=accumulate, ws=ws, relu_H=padded(Hact, F, dtype) if relu else None, src_prefix=n_fwd)
    torch.cuda.synchronize()
    want = np.zeros((n, F))
    oracle.spmm_bwd(g.row_ptr, g.col_idx, np.arange(n_fwd, dtype=np.int32), dY, want, F, rs, cs)
    if accumulate:
        want = want + init
    if relu:
        want = want * (Hact > 0)
    got = host64(dXd)
    check(got[rows_o], want[rows_o], dtype, "bwd rows")
    outside = np.setdiff1d(np.arange(n), rows_o)
    assert (got[outside] == host64(padded(init, F, dtype))[outside]).all(), "rows outside were written"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("sorted_promise", [True, False])
def test_bwd_source_prefix(dtype, sorted_promise):
    g = gg.random_directed(8000, 6.0, 23)
    _prefix_case(g, 1500, 128, dtype, 31, sorted_promise)
    _prefix_case(g, 1, 64, dtype, 32, sorted_promise, accumulate=True)                 # a single forward row
    _prefix_case(g, 0, 64, dtype, 33, sorted_promise)                                  # none: every row sums to zero
    _prefix_case(g, 8000, 64, dtype, 34, sorted_promise, relu=True)                    # all: no cut at all
    _prefix_case(g, 7999, 100, dtype, 35, sorted_promise, accumulate=True, relu=True)
    rows = np.random.default_rng(36).permutation(8000)[:3001].astype(np.int32)
    _prefix_case(g, 4000, 7, dtype, 37, sorted_promise, out_rows=rows)
    h = gg.chung_lu(12000, 150.0, 2.1, 12)                                             # hub rows, cut inside the hub
    assert h.degrees().max() > 1200                                                    # (hub rows: longer than 1024)
    _prefix_case(h, 11000, 64, dtype, 38, sorted_promise, relu=True)                   # still hubs after the cut
    _prefix_case(h, 11000, 16, dtype, 40, sorted_promise)
    _prefix_case(h, 6000, 64, dtype, 39, sorted_promise)                               # hubs that stop being hubs after the cut


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_blocked_route_backward_with_source_prefix(dtype):
    """The column-blocked route cuts its blocks out of [0, src_prefix) only."""
    import paper_2311_06837_amd as P
    g = _dense_graph()
    ws = P.Workspace()
    _prefix_case(g, 68001, 96, dtype, 78, ws=ws, relu=True)          # 68001 * 256 B is still above the route's threshold
    assert _used_blocked_route(ws)
    _prefix_case(g, 66000, 200, dtype, 79, ws=ws, accumulate=True)
    ws2 = P.Workspace()
    _prefix_case(g, 9000, 96, dtype, 80, ws=ws2)                     # a short prefix fits the caches: one launch
    assert not _used_blocked_route(ws2)


def test_die_mapping_probe_and_the_route_that_depends_on_it():
    """Workgroup i on compute die i mod 8: the probe's raw ids are checked here on the CPU, and the size query of a call the
    column-blocked route is made for offers the route exactly when the pattern holds."""
    import paper_2311_06837_amd as P
    ids, holds = P.gnn_die_mapping()
    print("die ids of the probe grid:", ids, flush=True)
    assert len(ids) == 64 and all(0 <= i < 8 for i in ids)
    pattern = len(set(ids[:8])) == 8 and all(ids[i] == ids[i % 8] for i in range(64))
    assert holds == pattern
    g = gg.chung_lu(80_000, 160.0, 2.1, 17)       # dense enough: 20 entries of a row per column block, an 20 MB slab
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    X = torch.zeros(g.n_rows, 64, device="cuda")
    need = P.binding.spmm_workspace_bytes(G, g.n_rows, X, X.clone(), 64)
    assert (need > 0) == pattern
