"""GPU parity at the FULL sizes of the benchmark workloads, through the same calls and launch
configuration bench.py times.  The oracle cannot recompute whole layers here in seconds, so:
integer outputs (active sets, sampled rows) are compared in full, bit-exact; floating-point kernels
are compared on seeded samples of output rows / columns that the oracle computes one by one from the
same seeded inputs (never from GPU results), plus properties that hold at any size.
fp32: 1e-4, bf16: 2e-2 (gpu_util.TOL)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import as_stored, check, dev, host64, padded

pytestmark = pytest.mark.gpu


_WS = {}


def _ws():
    """One workspace for the aggregation calls, as the model passes one (on cfg1 that selects the column-blocked route)."""
    import paper_2311_06837_amd as P
    if "ws" not in _WS:
        _WS["ws"] = P.Workspace()
    return _WS["ws"]


@pytest.fixture(scope="module")
def cfg1():
    print("generating cfg1 at full size", flush=True)
    return gg.make_workload("cfg1")


@pytest.fixture(scope="module")
def cfg3():
    print("generating cfg3 at full size", flush=True)
    return gg.make_workload("cfg3")


def _graph(part):
    import paper_2311_06837_amd as P
    return P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)


def _sample_rows(part, rows_all, k, seed):
    """Seeded sample of the active rows that always contains the longest and some empty/short rows."""
    rng = np.random.default_rng(seed)
    deg = np.diff(part.graph.row_ptr)[rows_all]
    order = np.argsort(deg)
    pick = np.concatenate([order[:8], order[-24:], rng.choice(rows_all.size, size=min(k, rows_all.size), replace=False)])
    return np.unique(rows_all[pick]).astype(np.int32)


def _active_sets_full(w):
    import paper_2311_06837_amd as P
    part = w.partition
    print(f"{w.name}: active sets n={part.graph.n_rows} nnz={part.graph.nnz} L={w.n_layers}", flush=True)
    G = _graph(part)
    od, oring, ooff = oracle.active_sets(part.graph.row_ptr, part.graph.col_idx, part.targets, w.n_layers)
    # every level from the frontier, then with the transposed graph (the workloads are symmetric: the graph itself),
    # the form the model calls, whose levels may run from the unreached vertices
    for gt in (None, G):
        dist, ring, off, hop = P.gnn_build_active_sets(G, dev(part.targets), w.n_layers, gt=gt)
        assert list(hop) == list(ooff)
        assert np.array_equal(dist.cpu().numpy(), od)
        assert np.array_equal(ring.cpu().numpy()[: ooff[-1]], oring)
    return G, od, oring, ooff


def _rows_arg(rows_all, as_prefix):
    """The row list as the call gets it: the id list, or NULL when the rows are the id prefix 0 .. m-1 of a (distance,
    id)-numbered partition (the form bench.py's model passes)."""
    if as_prefix:
        assert np.array_equal(rows_all, np.arange(rows_all.size))
        return None
    return dev(rows_all)


def _spmm_fwd_sampled(w, G, rows_all, F, dtype, kind, seed, n_sample=1500, as_prefix=False):
    """The forward aggregation over ALL of rows_all on the GPU; the oracle recomputes a sample of them."""
    import paper_2311_06837_amd as P
    part = w.partition
    n = part.graph.n_rows
    ld = P.row_stride(F, dtype)                       # the layout the model (and so bench.py) uses
    print(f"{w.name}: spmm fwd rows={rows_all.size} F={F} {dtype} {kind}", flush=True)
    X = as_stored(gg.features(n, F, seed), dtype)
    length = np.diff(part.graph.row_ptr).astype(np.int32)
    if kind == "sage":
        rs, cs = oracle.norm_scales("mean", length), None
        rs_d = P.gnn_norm_scales(P.GNN_NORM_MEAN, n, row_ptr=G.row_ptr)
        cs_d = None
    else:
        s = oracle.norm_scales("sym", part.global_degree)
        rs, cs = s, s
        rs_d = P.gnn_norm_scales(P.GNN_NORM_SYM, n, length=dev(part.global_degree))
        cs_d = rs_d
    Xd = padded(X, ld, dtype)
    Yd = torch.zeros(n, ld, dtype=dtype, device="cuda")
    P.gnn_masked_spmm_fwd(G, _rows_arg(rows_all, as_prefix), rows_all.size, Xd, Yd, F, rs_d, cs_d, ws=_ws())
    torch.cuda.synchronize()
    sample = _sample_rows(part, rows_all, n_sample, seed)
    want = np.zeros((n, F))
    oracle.spmm_fwd(part.graph.row_ptr, part.graph.col_idx, sample, X, want, F, rs, cs)
    got = host64(Yd[dev(sample).long()])[:, :F]
    check(got, want[sample], dtype, "sampled rows of the aggregation")
    return X, Xd, Yd, (rs, cs, rs_d, cs_d)


def _spmm_fwd_add_sampled(w, G, F, dtype, seed, n_sample=600, n_rows=None, kind="sage", relu=True):
    """The add-on-top form of the forward aggregation (a layer that multiplies by its weights first) over the id prefix
    0 .. n_rows-1 (default: every vertex); the oracle recomputes the plain aggregation of a sample, the sum with the
    self term (GraphSAGE) or the bias (GCN: no self term, the rows start from the bias) and the ReLU are written out here."""
    import paper_2311_06837_amd as P
    part = w.partition
    n = part.graph.n_rows
    m = n if n_rows is None else n_rows
    ld = P.row_stride(F, dtype)
    print(f"{w.name}: spmm fwd_add rows={m} F={F} {dtype} {kind}", flush=True)
    X = as_stored(gg.features(n, F, seed), dtype)
    S = as_stored(gg.features(n, F, seed + 300), dtype)
    bias, cs, cs_d = None, None, None
    if kind == "sage":
        rs = oracle.norm_scales("mean", np.diff(part.graph.row_ptr).astype(np.int32))
        rs_d = P.gnn_norm_scales(P.GNN_NORM_MEAN, n, row_ptr=G.row_ptr)
    else:
        rs = cs = oracle.norm_scales("sym", part.global_degree)
        rs_d = cs_d = P.gnn_norm_scales(P.GNN_NORM_SYM, n, length=dev(part.global_degree))
        bias = np.random.default_rng(seed).standard_normal(F).astype(np.float32)
    Yd = padded(S, ld, dtype)
    P.gnn_masked_spmm_fwd_add(G, None, m, padded(X, ld, dtype), Yd, F, rs_d, cs_d, relu=relu, ws=_ws(),
                              bias=None if bias is None else dev(bias))
    torch.cuda.synchronize()
    sample = _sample_rows(part, np.arange(m, dtype=np.int32), n_sample, seed)
    agg = np.zeros((n, F))
    oracle.spmm_fwd(part.graph.row_ptr, part.graph.col_idx, sample, X, agg, F, rs, cs)
    start = S[sample] if bias is None else as_stored(np.broadcast_to(bias.astype(np.float64), (sample.size, F)), dtype)
    want = start + agg[sample]
    if relu:
        want = np.maximum(want, 0.0)
    check(host64(Yd[dev(sample).long()])[:, :F], want, dtype, "sampled rows of the aggregation on top of the self term / bias")
    if m < n:       # rows past the prefix keep what they held
        tail = np.arange(m, min(n, m + 1000))
        assert np.array_equal(host64(Yd[dev(tail.astype(np.int32)).long()])[:, :F], S[tail])


def _spmm_bwd_sampled(w, G, dist, rows_out, max_dist, F, dtype, scales, seed, n_sample=1500, whole=False, src_prefix=-1,
                      as_prefix=False, accumulate=False, relu=False):
    """Backward aggregation for every row of rows_out; the oracle recomputes a sample in gather form over
    the (symmetric) graph with the activity filter folded into the per-neighbour scale.
    whole: the form the model uses when every vertex was a forward row - no row list, no filter, and the call undoes
    the ReLU of the layer in front (relu_H).
    src_prefix >= 0: the contributing rows are the ids below it, told through src_prefix instead of the distances
    (the form of the call on a (distance, id)-numbered partition; any graph will do to check it).
    With src_prefix: as_prefix - the output rows are an id prefix and no list is passed; accumulate - the sums are added
    onto what the rows hold (the self half of a GraphSAGE layer's input gradient); relu - the stored rows are masked by
    a seeded activation matrix (relu_H)."""
    import paper_2311_06837_amd as P
    part = w.partition
    n = part.graph.n_rows
    rs, cs, rs_d, cs_d = scales
    if src_prefix >= 0:
        dist = np.where(np.arange(n) < src_prefix, 0, max_dist + 1).astype(np.int32)
    ld = P.row_stride(F, dtype)                       # the layout the model (and so bench.py) uses
    print(f"{w.name}: spmm bwd rows={rows_out.size} F={F} {dtype} max_dist={max_dist}", flush=True)
    dY = as_stored(gg.features(n, F, seed + 100), dtype)
    dYd = padded(dY, ld, dtype)
    dXd = torch.zeros(n, ld, dtype=dtype, device="cuda")
    Hact, dX0 = None, None
    if accumulate:
        dX0 = as_stored(gg.features(n, F, seed + 400), dtype)
        dXd = padded(dX0, ld, dtype)
    if relu and not whole:
        Hact = as_stored(np.maximum(gg.features(n, F, seed + 200), 0), dtype)
    if whole:
        assert rows_out.size == n and np.array_equal(rows_out, np.arange(n)) and ((dist >= 0) & (dist <= max_dist)).all()
        Hact = as_stored(np.maximum(gg.features(n, F, seed + 200), 0), dtype)
        P.gnn_masked_spmm_bwd(G, None, n, None, max_dist, dYd, dXd, F, rs_d, cs_d, accumulate=False, ws=_ws(), relu_H=padded(Hact, ld, dtype))
    elif src_prefix >= 0:
        P.gnn_masked_spmm_bwd(G, _rows_arg(rows_out, as_prefix), rows_out.size, None, max_dist, dYd, dXd, F, rs_d, cs_d,
                              accumulate=accumulate, ws=_ws(), src_prefix=src_prefix if src_prefix < n else -1,
                              relu_H=padded(Hact, ld, dtype) if relu else None)
    else:
        P.gnn_masked_spmm_bwd(G, dev(rows_out), rows_out.size, dev(dist), max_dist, dYd, dXd, F, rs_d, cs_d, accumulate=False, ws=_ws())
    torch.cuda.synchronize()
    sample = _sample_rows(part, rows_out, n_sample, seed + 1)
    active = ((dist >= 0) & (dist <= max_dist)).astype(np.float64)
    nbr = active * (rs if rs is not None else 1.0)           # per contributing row v: rs[v] * [v active]
    want = np.zeros((n, F))
    oracle.spmm_fwd(part.graph.row_ptr, part.graph.col_idx, sample, dY, want, F, cs, nbr)   # symmetric: gT = g
    if accumulate:
        want[sample] += dX0[sample]
    if whole or relu:
        want = want * (Hact > 0)
    got = host64(dXd[dev(sample).long()])[:, :F]
    check(got, want[sample], dtype, "sampled rows of the backward aggregation")


def _linear_sampled(w, rows_all, K, N, dtype, sage, seed, n_sample=2000, n_cols=8, in_place=False):
    """Forward + backward feature transform over ALL rows on the GPU.  The oracle recomputes sampled output
    rows (forward, dA, dX_self) and, for the weight gradients, n_cols whole columns of dW / dbias
    (a column of dW depends on that column of dZ only).
    in_place: the form the model uses on a (distance, id)-numbered partition - no row list (rows_all must be
    0 .. m-1) and, in the backward call, no activation to undo (the gradient arrives masked)."""
    import paper_2311_06837_amd as P
    n = w.partition.graph.n_rows
    if in_place:
        n = rows_all.size            # an id prefix: the matrices need no more rows than that
    ld_in, ld_out = P.row_stride(K, dtype), P.row_stride(N, dtype)
    print(f"{w.name}: linear rows={rows_all.size} K={K} N={N} {dtype} sage={sage}", flush=True)
    params = gg.layer_weights([K, N], sage, seed)[0]
    A = as_stored(gg.features(n, K, seed + 1), dtype)
    Xs = as_stored(gg.features(n, K, seed + 2), dtype) if sage else None
    Wn = as_stored(params["W_neigh"], dtype)
    Ws = as_stored(params["W_self"], dtype) if sage else None
    b = params["bias"]
    Ad, Xd = padded(A, ld_in, dtype), (padded(Xs, ld_in, dtype) if sage else None)
    Wnd, Wsd = dev(Wn, dtype), (dev(Ws, dtype) if sage else None)
    Hd = torch.zeros(n, ld_out, dtype=dtype, device="cuda")
    rows_d = dev(rows_all)
    relu_b = True
    if in_place:
        assert np.array_equal(rows_all, np.arange(rows_all.size))
        rows_d, relu_b = None, False
    P.gnn_linear_fwd(rows_d, rows_all.size, Ad, Xd, K, Wnd, Wsd, dev(b), Hd, True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(seed)
    sample = np.unique(rows_all[rng.choice(rows_all.size, size=min(n_sample, rows_all.size), replace=False)]).astype(np.int32)
    H = np.zeros((n, N))
    oracle.linear_fwd(sample, A, Xs, K, Wn, Ws, b.astype(np.float64), H, True)
    check(host64(Hd[dev(sample).long()])[:, :N], H[sample], dtype, "sampled rows of H")

    # backward with the GPU-independent inputs: H is replaced by a seeded stand-in so both sides mask alike
    Hs = as_stored(gg.features(n, N, seed + 3), dtype)
    dH = as_stored(gg.features(n, N, seed + 4), dtype)
    dWn_d = torch.zeros(K, N, device="cuda")
    dWs_d = torch.zeros(K, N, device="cuda") if sage else None
    db_d = torch.zeros(N, device="cuda")
    dA_d = torch.zeros(n, ld_in, dtype=dtype, device="cuda")
    dX_d = torch.zeros(n, ld_in, dtype=dtype, device="cuda") if sage else None
    P.gnn_linear_bwd(rows_d, rows_all.size, padded(dH, ld_out, dtype), padded(Hs, ld_out, dtype) if relu_b else None, relu_b, Ad, Xd, K,
                     Wnd, Wsd, dWn_d, dWs_d, db_d, dA_d, dX_d)
    torch.cuda.synchronize()
    # (a) input gradients on sampled rows
    dA = np.zeros((n, K))
    dX = np.zeros((n, K)) if sage else None
    oracle.linear_bwd(sample, dH, Hs if relu_b else None, relu_b, A, Xs, K, Wn, Ws, dA, dX)
    check(host64(dA_d[dev(sample).long()])[:, :K], dA[sample], dtype, "sampled rows of dA")
    if sage:
        check(host64(dX_d[dev(sample).long()])[:, :K], dX[sample], dtype, "sampled rows of dX_self")
    # (b) n_cols full columns of the weight and bias gradients, reduced over ALL rows by the oracle
    cols = np.sort(rng.choice(N, size=min(n_cols, N), replace=False))
    dWn, dWs, db = oracle.linear_bwd(rows_all, np.ascontiguousarray(dH[:, cols]), np.ascontiguousarray(Hs[:, cols]) if relu_b else None, relu_b, A, Xs, K,
                                     np.ascontiguousarray(Wn[:, cols]), np.ascontiguousarray(Ws[:, cols]) if sage else None)
    check(host64(dWn_d)[:, cols], dWn, dtype, "columns of dW_neigh")
    check(host64(db_d)[cols], db, dtype, "entries of dbias")
    if sage:
        check(host64(dWs_d)[:, cols], dWs, dtype, "columns of dW_self")


def test_cfg1_full_size(cfg1):
    """configs[1] (the benchmark workload): fp32, 3-layer GraphSAGE-mean, 602-256-256-41."""
    w = cfg1
    G, dist, ring, off = _active_sets_full(w)
    L = w.n_layers
    R1, R2, R3 = ring[: off[L]], ring[: off[L - 1]], ring[: off[L - 2]]
    _, _, _, sc = _spmm_fwd_sampled(w, G, R1, 602, torch.float32, "sage", 11, n_sample=600)
    _spmm_fwd_sampled(w, G, R3, 256, torch.float32, "sage", 12, n_sample=600)
    _spmm_bwd_sampled(w, G, dist, R1, L - 2, 256, torch.float32, sc, 13, n_sample=600)      # backward of layer 2
    _spmm_bwd_sampled(w, G, dist, R2, L - 3, 256, torch.float32, sc, 14, n_sample=600)      # backward of layer 3
    _linear_sampled(w, R1, 602, 256, torch.float32, True, 15, n_sample=1500, n_cols=4)
    _linear_sampled(w, R3, 256, 41, torch.float32, True, 16, n_sample=1500, n_cols=8)
    # the forms the model uses where every vertex is a row (layers 1 and 2 here): no row list, no filter, the ReLU in
    # front undone by the aggregation, the gradient read in place by the feature transform
    n = w.partition.graph.n_rows
    assert R1.size == n
    allrows = np.arange(n, dtype=np.int32)
    _spmm_bwd_sampled(w, G, dist, allrows, L - 2, 256, torch.float32, sc, 17, n_sample=600, whole=True)
    _spmm_fwd_add_sampled(w, G, 256, torch.float32, 19)
    _spmm_bwd_sampled(w, G, dist, allrows, 0, 256, torch.float32, sc, 20, n_sample=600, src_prefix=29125)      # one launch, rows cut
    _spmm_bwd_sampled(w, G, dist, allrows, 0, 256, torch.float32, sc, 21, n_sample=600, src_prefix=200001)     # column-blocked route
    _linear_sampled(w, allrows, 256, 256, torch.float32, True, 18, n_sample=1500, n_cols=4, in_place=True)


def test_cfg1_sum_of_ones_is_degree_at_full_size(cfg1):
    import paper_2311_06837_amd as P
    part = cfg1.partition
    n = part.graph.n_rows
    G = _graph(part)
    X = torch.ones(n, 64, device="cuda")
    Y = torch.zeros(n, 64, device="cuda")
    P.gnn_masked_spmm_fwd(G, None, n, X, Y, 64, ws=_ws())
    assert _ws().buf.numel() > 256 or not P.gnn_die_mapping()[1]     # the column-blocked route: sums of ones stay exact
    assert torch.equal(Y[:, 0].cpu(), torch.from_numpy(part.graph.degrees()).float())
    assert torch.equal(Y, Y[:, :1].expand(-1, 64))


def test_cfg3_full_size_bf16(cfg3):
    """configs[3]: bf16 storage, 8-layer GraphSAGE-mean, hidden 128; active sets shrink layer by layer."""
    w = cfg3
    G, dist, ring, off = _active_sets_full(w)
    L = w.n_layers
    R1, R7, R8 = ring[: off[L]], ring[: off[2]], ring[: off[1]]
    _, _, _, sc = _spmm_fwd_sampled(w, G, R1, 128, torch.bfloat16, "sage", 21)
    _spmm_fwd_sampled(w, G, R8, 128, torch.bfloat16, "sage", 22)
    _spmm_bwd_sampled(w, G, dist, R7, 0, 128, torch.bfloat16, sc, 23)                       # backward of layer 8
    _spmm_bwd_sampled(w, G, dist, R1, L - 2, 128, torch.bfloat16, sc, 24)                   # backward of layer 2
    _linear_sampled(w, R1, 128, 128, torch.bfloat16, True, 25)
    _linear_sampled(w, R8, 128, 16, torch.bfloat16, True, 26)
    n = w.partition.graph.n_rows
    assert R1.size == n
    allrows = np.arange(n, dtype=np.int32)
    _spmm_bwd_sampled(w, G, dist, allrows, L - 2, 128, torch.bfloat16, sc, 27, whole=True)
    _linear_sampled(w, allrows, 128, 128, torch.bfloat16, True, 28, in_place=True)


@pytest.fixture(scope="module")
def cfg4_sampled():
    """configs[4] through sampling and extraction on the GPU and in the oracle, once for the tests below (the 10M-vertex
    graph takes a minute to generate).  Everything the later tests use on the host side is the ORACLE's."""
    import paper_2311_06837_amd as P
    print("generating cfg4 at full size", flush=True)
    w = gg.make_workload("cfg4")
    g, T = w.global_graph, w.targets_global.astype(np.int32)
    print(f"cfg4: sampling n={g.n_rows} nnz={g.nnz} |T|={T.size} fanout={w.fanout}", flush=True)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = dev(T)
    rp, ci = P.gnn_sample_boundary(G, P.gnn_make_bitmap(Td, g.n_rows), Td, w.fanout, w.sample_seed)
    torch.cuda.synchronize()
    is_t = np.zeros(g.n_rows, dtype=np.uint8)
    is_t[T] = 1
    orp, oci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, w.fanout, w.sample_seed)
    print("cfg4: extraction of the sampled partition", flush=True)
    local, l2g_d, hop = P.gnn_extract_sampled_partition(G, Td, rp, ci)
    torch.cuda.synchronize()
    xrp, xci, xl2g, xoff, _ = oracle.extract_sampled(g.n_rows, T, orp, oci)
    del G
    return dict(w=w, g=g, T=T, gpu=(rp.cpu().numpy(), ci.cpu().numpy(), [int(x) for x in hop], l2g_d.cpu().numpy(),
                                    local.row_ptr.cpu().numpy(), local.col_idx.cpu().numpy()),
                oracle=(orp, oci, xrp, xci, xl2g, xoff), local=local)


def test_cfg4_sampling_and_extraction_full_size(cfg4_sampled):
    """configs[4]: boundary sampling over the 10M-vertex graph and the extraction of the sampled partition, both
    bit-exact in full; then the active sets of the sampled partition."""
    c = cfg4_sampled
    rp, ci, hop, l2g_gpu, lrp, lci = c["gpu"]
    orp, oci, xrp, xci, xl2g, xoff = c["oracle"]
    assert np.array_equal(rp, orp)
    assert np.array_equal(ci, oci)
    assert hop == [int(x) for x in xoff]
    assert np.array_equal(l2g_gpu, xl2g)
    assert np.array_equal(lrp, xrp)
    assert np.array_equal(lci, xci)
    w, g, T = c["w"], c["g"], c["T"]
    l2g, er, ec = oracle.sampled_local_edges(T, orp, oci)
    w.partition = gg.partition_from_edges(g.n_rows, l2g, er, ec, T, g.degrees())
    _active_sets_full(w)


def _cfg4_local_partition(c):
    """The extracted partition as a host workload (the oracle's extraction, which the GPU's equals bit for bit)."""
    w, g, T = c["w"], c["g"], c["T"]
    orp, oci, xrp, xci, xl2g, xoff = c["oracle"]
    n_loc, nt = int(xoff[-1]), int(T.size)
    lg = gg.CSR(n_loc, n_loc, xrp, xci)
    w.partition = gg.Partition(lg, lg, xl2g.astype(np.int64), np.arange(nt, dtype=np.int32), g.degrees()[xl2g].astype(np.int32))
    return w, n_loc, nt


def test_cfg4_aggregations_full_size(cfg4_sampled):
    """The aggregation calls of the step on the extracted partition of configs[4], in the forms bench.py's model issues
    them: bf16, rows as id prefixes (no lists), the backward filter as a source prefix, 128 / 256 / 32 columns."""
    w, n_loc, nt = _cfg4_local_partition(cfg4_sampled)
    local = cfg4_sampled["local"]
    allrows = np.arange(n_loc, dtype=np.int32)
    bf = torch.bfloat16
    _, _, _, sc = _spmm_fwd_sampled(w, local, allrows, 128, bf, "sage", 41, n_sample=1200, as_prefix=True)     # layer 1
    _spmm_fwd_sampled(w, local, allrows, 256, bf, "sage", 42, n_sample=1200, as_prefix=True)                    # layer 2 (dominant call)
    _spmm_fwd_add_sampled(w, local, 32, bf, 43, n_sample=1200, n_rows=nt, relu=False)                           # layer 3, exchanged order
    # backward of layer 3 in the exchanged order: the targets' gradient aggregated to every vertex, 32 columns
    _spmm_bwd_sampled(w, local, None, allrows, 0, 32, bf, sc, 44, n_sample=1200, src_prefix=nt, as_prefix=True)
    # backward of layer 2: every vertex was a forward row, sums added onto the self half, ReLU of layer 1 undone
    _spmm_bwd_sampled(w, local, None, allrows, 0, 256, bf, sc, 45, n_sample=1200, src_prefix=n_loc, as_prefix=True,
                      accumulate=True, relu=True)


def test_cfg4_feature_transforms_full_size(cfg4_sampled):
    """The feature transforms of configs[4] on the extracted partition: bf16, 128 -> 256, 256 -> 256, 256 -> 32."""
    w, n_loc, nt = _cfg4_local_partition(cfg4_sampled)
    cfg4_sampled["local"] = None        # the device copy of the graph is not needed any more
    allrows, trows = np.arange(n_loc, dtype=np.int32), np.arange(nt, dtype=np.int32)
    bf = torch.bfloat16
    _linear_sampled(w, allrows, 128, 256, bf, True, 46, n_sample=1000, n_cols=4, in_place=True)
    _linear_sampled(w, allrows, 256, 256, bf, True, 47, n_sample=1000, n_cols=4, in_place=True)
    _linear_sampled(w, trows, 256, 32, bf, True, 48, n_sample=1000, n_cols=4, in_place=True)


@pytest.fixture(scope="module")
def cfg2():
    print("generating cfg2 at full size", flush=True)
    return gg.make_workload("cfg2")


def test_cfg2_full_size_gcn(cfg2):
    """configs[2]: fp32, 3-layer GCN 100-256-256-47 with the symmetric normalisation over the GLOBAL degrees, 2.45M
    vertices; the last layer in the exchanged order (47 columns gathered, the rows start from the bias)."""
    w = cfg2
    G, dist, ring, off = _active_sets_full(w)
    L = w.n_layers
    R1, R2, R3 = ring[: off[L]], ring[: off[L - 1]], ring[: off[L - 2]]
    f32 = torch.float32
    _, _, _, sc = _spmm_fwd_sampled(w, G, R1, 100, f32, "gcn", 51, n_sample=1000)
    _spmm_fwd_sampled(w, G, R2, 256, f32, "gcn", 52, n_sample=1000)
    _spmm_fwd_sampled(w, G, R3, 47, f32, "gcn", 53, n_sample=1000)
    _spmm_bwd_sampled(w, G, dist, R1, L - 2, 256, f32, sc, 54, n_sample=1000)       # backward of layer 2
    _spmm_bwd_sampled(w, G, dist, R2, L - 3, 47, f32, sc, 55, n_sample=1000)        # backward of layer 3 (exchanged order: 47 wide)
    _spmm_bwd_sampled(w, G, dist, R2, L - 3, 256, f32, sc, 56, n_sample=1000)       # backward of layer 3 (the paper's order)
    _linear_sampled(w, R1, 100, 256, f32, False, 57, n_sample=1000, n_cols=4)
    _linear_sampled(w, R2, 256, 256, f32, False, 58, n_sample=1000, n_cols=4)
    _linear_sampled(w, R3, 256, 47, f32, False, 59, n_sample=1000, n_cols=6)


def test_more_than_2_31_elements():
    """One aggregation and one feature transform on a matrix of more than 2^31 elements (4.3M x 512 fp32, 8.8 GB): every
    element address must be formed in 64 bits.  Inputs are made on the device by torch's seeded generator (too large
    to come from the host in reasonable time); the oracle gets exactly the rows it needs, copied back: it recomputes
    output rows near the END of the matrix, where a 32-bit offset would have wrapped."""
    import paper_2311_06837_amd as P
    n, F, N = 4_300_000, 512, 64
    assert n * F > 2 ** 31
    print(f"2^31: n={n} F={F}", flush=True)
    g = gg.erdos_renyi(n, 4.0, 77)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    Xd = torch.randn(n, F, device="cuda", generator=gen)
    Yd = torch.zeros(n, F, device="cuda")
    rs_d = P.gnn_norm_scales(P.GNN_NORM_MEAN, n, row_ptr=G.row_ptr)
    P.gnn_masked_spmm_fwd(G, None, n, Xd, Yd, F, rs_d, None)
    torch.cuda.synchronize()
    rng = np.random.default_rng(77)
    sample = np.unique(np.concatenate([np.arange(n - 300, n), rng.choice(n, 300, replace=False), np.arange(200)])).astype(np.int32)
    # sub-problem for the oracle: the sampled rows with their neighbours renumbered 0 .. k-1
    starts, ends = g.row_ptr[sample], g.row_ptr[sample + 1]
    nb = np.concatenate([g.col_idx[s:e] for s, e in zip(starts, ends)])
    uniq, inv = np.unique(nb, return_inverse=True)
    sub_rp = np.concatenate([[0], np.cumsum(ends - starts)]).astype(np.int32)
    Xsub = Xd[torch.from_numpy(uniq).cuda().long()].double().cpu().numpy()
    want = np.zeros((sample.size, F))
    rs_sub = oracle.norm_scales("mean", (ends - starts).astype(np.int32))
    oracle.spmm_fwd(sub_rp, inv.astype(np.int32), np.arange(sample.size, dtype=np.int32), Xsub, want, F, rs_sub, None)
    check(host64(Yd[dev(sample).long()]), want, torch.float32, "aggregation rows of a matrix with more than 2^31 elements")
    del Yd
    # feature transform: H = relu(X W + b) over all rows, then the input gradient dX = dZ W^T back into an 8.8 GB matrix
    p = gg.layer_weights([F, N], False, 77)[0]
    Wd, bd = dev(p["W_neigh"]), dev(p["bias"])
    Hd = torch.zeros(n, N, device="cuda")
    P.gnn_linear_fwd(None, n, Xd, None, F, Wd, None, bd, Hd, True)
    torch.cuda.synchronize()
    Xs = Xd[dev(sample).long()].double().cpu().numpy()
    H = np.zeros((sample.size, N))
    oracle.linear_fwd(np.arange(sample.size, dtype=np.int32), Xs, None, F, p["W_neigh"].astype(np.float64), None,
                      p["bias"].astype(np.float64), H, True)
    check(host64(Hd[dev(sample).long()]), H, torch.float32, "transform rows of a matrix with more than 2^31 elements")
    dZd = torch.randn(n, N, device="cuda", generator=gen)
    dXd = torch.zeros(n, F, device="cuda")
    del Xd
    P.gnn_linear_bwd_input(None, n, dZd, N, Wd, F, 0, None, dXd)
    torch.cuda.synchronize()
    dZs = dZd[dev(sample).long()].double().cpu().numpy()
    want_dx = dZs @ p["W_neigh"].astype(np.float64).T        # a textbook product (numpy), rows taken one by one
    check(host64(dXd[dev(sample).long()]), want_dx, torch.float32, "input-gradient rows of a matrix with more than 2^31 elements")


def test_blocked_route_two_passes():
    """The column-blocked route with MORE THAN ONE pass over the neighbour-id range (16 column blocks: a gathered matrix
    of more than 262144 rows on a graph dense enough for it): forward, filtered backward (distances), backward with a
    source prefix, and the bf16 form with its per-edge scale.  The benchmark workloads all need one pass only."""
    import paper_2311_06837_amd as P
    g = gg.chung_lu(300_000, 140.0, 2.1, 91)
    part = gg.halo_partition(g, np.arange(0, g.n_rows, 7, dtype=np.int64), 2)
    n = part.graph.n_rows
    print(f"two-pass blocked route: n={n} nnz={part.graph.nnz}", flush=True)
    assert n > 290_000
    w = gg.Workload("twopass", "sage", "f32", [64, 64, 8], 2, part, g, None)
    G = _graph(part)
    assert G.sorted_columns
    # the size query says whether (and the workspace size how) the route applies: 16 blocks -> 17 cut points per row
    X = torch.zeros(n, 64, device="cuda")
    need = P.binding.spmm_workspace_bytes(G, n, X, X.clone(), 64)
    if not P.gnn_die_mapping()[1]:
        pytest.skip("workgroups are not dealt round-robin to the compute dies here: the library does not take the route")
    assert need >= n * 17 * 4 + 8 * n * 64 * 4, "the two-pass column-blocked route was expected to apply"
    od, oring, ooff = oracle.active_sets(part.graph.row_ptr, part.graph.col_idx, part.targets, 2)
    allrows = np.arange(n, dtype=np.int32)
    for dtype, seed in ((torch.float32, 92), (torch.bfloat16, 93)):
        _, _, _, sc = _spmm_fwd_sampled(w, G, allrows, 64, dtype, "sage", seed, n_sample=500, as_prefix=True)
        _spmm_bwd_sampled(w, G, od, allrows, 1, 64, dtype, sc, seed + 10, n_sample=500)                 # distance filter
        _spmm_bwd_sampled(w, G, od, allrows, 0, 64, dtype, sc, seed + 20, n_sample=500, src_prefix=n - 15_000)
    # GCN scales: a neighbour scale in the forward call (fp32: scaled copy of the matrix, bf16: a factor per edge)
    _spmm_fwd_sampled(w, G, allrows, 64, torch.bfloat16, "gcn", 95, n_sample=500)
    _spmm_fwd_sampled(w, G, allrows, 64, torch.float32, "gcn", 96, n_sample=500)
