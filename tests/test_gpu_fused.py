"""GPU parity: gnn_fused_layer_fwd (aggregation and feature transform of a layer in one kernel, section 2.1) against the
oracle's two steps - orc_spmm_fwd, the aggregate rounded to the storage type (where the two-call path stores it), then
orc_linear_fwd.  fp32: 1e-4, bf16: 2e-2."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import as_stored, check, dev, host64, padded

pytestmark = pytest.mark.gpu

SENT = 333.0


def _case(g, rows, n_active, K, N, dtype, kind, relu, seed, global_degree=None):
    import paper_2311_06837_amd as P
    n = g.n_rows
    print(f"fused layer: n={n} nnz={g.nnz} rows={'list' if rows is not None else 'prefix'} active={n_active} K={K} N={N} {dtype} "
          f"{kind} relu={relu}", flush=True)
    sage = kind == "sage"
    rng = np.random.default_rng(seed)
    p = gg.layer_weights([K, N], sage, seed)[0]
    Wn = as_stored(p["W_neigh"], dtype)
    Ws = as_stored(p["W_self"], dtype) if sage else None
    b = p["bias"]
    X = as_stored(rng.standard_normal((n, K)), dtype)
    length = np.diff(g.row_ptr).astype(np.int32)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    if sage:
        rs, cs = oracle.norm_scales("mean", length), None
        rs_d, cs_d = P.gnn_norm_scales(P.GNN_NORM_MEAN, n, row_ptr=G.row_ptr), None
    else:
        deg = length if global_degree is None else global_degree
        rs = cs = oracle.norm_scales("sym", deg)
        rs_d = cs_d = P.gnn_norm_scales(P.GNN_NORM_SYM, n, length=dev(deg.astype(np.int32)))
    ld_in, ld_out = P.row_stride(K, dtype), P.row_stride(N, dtype)
    Xd = padded(X, ld_in, dtype, fill=float("nan") if ld_in > K else 0.0)      # pad columns must never reach a sum
    Hd = torch.full((n, ld_out), SENT, dtype=dtype, device="cuda")
    P.gnn_fused_layer_fwd(G, dev(rows) if rows is not None else None, n_active, Xd, K, rs_d, cs_d, dev(Wn, dtype),
                          dev(Ws, dtype) if sage else None, dev(b), Hd, relu)
    torch.cuda.synchronize()
    sel = rows[:n_active] if rows is not None else np.arange(n_active, dtype=np.int32)
    A = np.zeros((n, K))
    oracle.spmm_fwd(g.row_ptr, g.col_idx, sel, X, A, K, rs, cs)
    A = as_stored(A, dtype)                                                       # the aggregate in the storage type
    H = np.zeros((n, N))
    oracle.linear_fwd(sel, A, X if sage else None, K, Wn, Ws, b.astype(np.float64), H, relu)
    got = host64(Hd)
    check(got[sel, :N], H[sel], dtype, "H")
    sent = host64(torch.tensor(SENT, dtype=dtype))
    rest = np.setdiff1d(np.arange(n), sel)
    assert (got[rest] == sent).all() and (got[:, N:] == sent).all(), "the fused layer wrote outside its rows / columns"


@pytest.mark.parametrize("K,N", [(128, 128), (256, 256), (256, 32), (128, 16), (128, 256), (64, 64), (200, 100), (72, 41)])
def test_bf16_shapes(K, N):
    g = gg.chung_lu(6000, 12.0, 2.1, 41)
    rng = np.random.default_rng(K + N)
    rows = rng.permutation(g.n_rows)[:3333].astype(np.int32)
    _case(g, None, 6000, K, N, torch.bfloat16, "sage", True, K * 7 + N)
    _case(g, rows, 3333, K, N, torch.bfloat16, "sage", False, K * 7 + N + 1)


@pytest.mark.parametrize("K,N", [(64, 64), (128, 128), (100, 47), (32, 8), (96, 128)])
def test_fp32_shapes_and_gcn(K, N):
    g = gg.add_self_loops(gg.chung_lu(5000, 10.0, 2.1, 42))
    rng = np.random.default_rng(K + N)
    rows = rng.permutation(g.n_rows)[:1999].astype(np.int32)
    _case(g, rows, 1999, K, N, torch.float32, "sage", True, K * 5 + N)
    _case(g, None, 4097, K, N, torch.float32, "gcn", True, K * 5 + N + 1, global_degree=np.diff(g.row_ptr) + 3)
    _case(g, None, 5000, K, N, torch.bfloat16 if K * 2 >= 128 else torch.float32, "gcn", False, K * 5 + N + 2)


def test_hub_rows_empty_rows_and_ragged_tiles():
    """Rows of thousands of entries (shared by the whole workgroup), rows without entries, a last tile of one row."""
    g = gg.chung_lu(4000, 150.0, 2.1, 43)
    assert g.degrees().max() > 600          # beyond the 512 entries a lane group takes alone
    for dtype in (torch.float32, torch.bfloat16):
        _case(g, None, 4000, 128, 64, dtype, "sage", True, 431)
        _case(g, None, 65, 128, 64, dtype, "sage", True, 432)
    iso = gg.csr_from_edges(300, 300, np.array([0, 0, 5, 299]), np.array([5, 299, 0, 0]))      # almost every row is empty
    _case(iso, None, 300, 64, 32, torch.float32, "sage", False, 433)
    _case(iso, np.array([299, 5, 7, 0], dtype=np.int32), 4, 128, 128, torch.bfloat16, "sage", True, 434)
    _case(iso, None, 0, 128, 128, torch.bfloat16, "sage", True, 435)                             # nothing to do


def test_shapes_outside_the_limits_are_refused():
    import paper_2311_06837_amd as P
    g = gg.erdos_renyi(500, 6.0, 44)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    for K, N, dtype in ((602, 256, torch.float32), (16, 16, torch.float32), (128, 256, torch.float32), (512, 64, torch.bfloat16),
                        (32, 32, torch.bfloat16)):
        assert not P.binding.fused_layer_supported(K, N, dtype)
        X = torch.zeros(500, P.row_stride(K, dtype), dtype=dtype, device="cuda")
        H = torch.zeros(500, P.row_stride(N, dtype), dtype=dtype, device="cuda")
        W = torch.zeros(K, N, dtype=dtype, device="cuda")
        with pytest.raises(P.GnnError) as ei:
            P.gnn_fused_layer_fwd(G, None, 500, X, K, None, None, W, None, None, H, False)
        assert ei.value.status == 4
    assert P.binding.fused_layer_supported(128, 128, torch.bfloat16) and P.binding.fused_layer_supported(100, 47, torch.float32)
