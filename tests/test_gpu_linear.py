"""GPU parity: gnn_linear_fwd / _bwd (MFMA GEMMs) and gnn_softmax_ce against the oracle
(section 2.1 feature transform; section 8.1 task).  fp32: 1e-4, bf16: 2e-2."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import as_stored, check, dev, host64, padded

pytestmark = pytest.mark.gpu

SENT = 777.0


def _pad(n, m):
    return (n + m - 1) // m * m


def _case(M_total, n_active, K, N, dtype, sage, relu, use_rows, aligned, seed, need_in=True):
    import paper_2311_06837_amd as P
    print(f"linear: n={M_total} active={n_active} K={K} N={N} {dtype} sage={sage} relu={relu} rows={use_rows} "
          f"aligned={aligned}", flush=True)
    rng = np.random.default_rng(seed)
    mult = (4 if dtype == torch.float32 else 8) if aligned else 1
    ld_in, ld_out = _pad(K, mult), _pad(N, mult)
    A = as_stored(rng.standard_normal((M_total, K)), dtype)
    Xs = as_stored(rng.standard_normal((M_total, K)), dtype) if sage else None
    Wn = as_stored(rng.standard_normal((K, N)) / np.sqrt(K), dtype)
    Ws = as_stored(rng.standard_normal((K, N)) / np.sqrt(K), dtype) if sage else None
    b = rng.standard_normal(N).astype(np.float32)
    rows = np.sort(rng.choice(M_total, n_active, replace=False)).astype(np.int32) if use_rows else None
    sel = rows if use_rows else np.arange(n_active)
    rest = np.setdiff1d(np.arange(M_total), sel)

    Ad = padded(A, ld_in, dtype, fill=float("nan") if ld_in > K else 0.0)
    Xd = padded(Xs, ld_in, dtype, fill=float("nan") if ld_in > K else 0.0) if sage else None
    Wnd, Wsd = dev(Wn, dtype), (dev(Ws, dtype) if sage else None)
    Hd = torch.full((M_total, ld_out), SENT, dtype=dtype, device="cuda")
    P.gnn_linear_fwd(dev(rows) if use_rows else None, n_active, Ad, Xd, K, Wnd, Wsd, dev(b), Hd, relu)
    torch.cuda.synchronize()
    H = np.full((M_total, N), SENT)
    oracle.linear_fwd(rows if use_rows else np.arange(n_active, dtype=np.int32), A, Xs, K, Wn, Ws, b.astype(np.float64), H, relu)
    got = host64(Hd)
    check(got[sel, :N], H[sel], dtype, "H")
    sent = host64(torch.tensor(SENT, dtype=dtype))
    assert (got[rest] == sent).all() and (got[:, N:] == sent).all(), "forward wrote outside its rows/columns"

    # backward, fed with the oracle's own H (rounded to storage) so both sides mask the same entries
    Hs = as_stored(H, dtype)
    dH = as_stored(rng.standard_normal((M_total, N)), dtype)
    dWn_d = torch.full((K, N), SENT, device="cuda")
    dWs_d = torch.full((K, N), SENT, device="cuda") if sage else None
    db_d = torch.full((N,), SENT, device="cuda")
    dA_d = torch.full((M_total, ld_in), SENT, dtype=dtype, device="cuda") if need_in else None
    dX_d = torch.full((M_total, ld_in), SENT, dtype=dtype, device="cuda") if (need_in and sage) else None
    P.gnn_linear_bwd(dev(rows) if use_rows else None, n_active, padded(dH, ld_out, dtype, fill=float("nan") if ld_out > N else 0.0),
                     padded(Hs, ld_out, dtype) if relu else None, relu, Ad, Xd, K, Wnd, Wsd, dWn_d, dWs_d, db_d, dA_d, dX_d)
    torch.cuda.synchronize()
    dA = np.full((M_total, K), SENT)
    dX = np.full((M_total, K), SENT) if sage else None
    dWn, dWs, db = oracle.linear_bwd(rows if use_rows else np.arange(n_active, dtype=np.int32), dH, Hs if relu else None, relu,
                                     A, Xs, K, Wn, Ws, dA if need_in else None, dX if (need_in and sage) else None)
    check(host64(dWn_d), dWn, dtype, "dW_neigh")
    check(host64(db_d), db, dtype, "dbias")
    if sage:
        check(host64(dWs_d), dWs, dtype, "dW_self")
    if need_in:
        g = host64(dA_d)
        check(g[sel, :K], dA[sel], dtype, "dA")
        assert (g[rest] == sent).all() and (g[:, K:] == sent).all(), "dA wrote outside its rows/columns"
        if sage:
            g = host64(dX_d)
            check(g[sel, :K], dX[sel], dtype, "dX_self")
            assert (g[rest] == sent).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K,N", [(64, 64), (64, 8), (602, 256), (100, 256), (256, 47), (128, 16), (256, 41), (33, 5), (128, 128),
                                 (256, 256), (128, 256), (96, 160), (608, 256), (512, 512), (192, 128), (64, 256)])
def test_shapes_of_the_workloads(dtype, K, N):
    _case(3000, 1777, K, N, dtype, sage=(K != 100 and K != 64), relu=(N > 50), use_rows=True, aligned=True, seed=K + N)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_prefix_rows_ragged_counts_and_unaligned_leading_dimensions(dtype):
    _case(700, 700, 64, 64, dtype, sage=True, relu=True, use_rows=False, aligned=True, seed=1)
    _case(700, 129, 48, 40, dtype, sage=False, relu=False, use_rows=False, aligned=True, seed=2)
    _case(300, 1, 64, 64, dtype, sage=True, relu=True, use_rows=True, aligned=True, seed=3)
    _case(500, 257, 602, 41, dtype, sage=True, relu=False, use_rows=True, aligned=False, seed=4)     # ld = 602 / 41
    _case(500, 333, 100, 256, dtype, sage=False, relu=True, use_rows=True, aligned=True, seed=5, need_in=False)


def test_large_row_count_many_splits():
    _case(70000, 65537, 256, 256, torch.float32, sage=True, relu=True, use_rows=True, aligned=True, seed=6)
    _case(70000, 65537, 128, 128, torch.bfloat16, sage=True, relu=True, use_rows=True, aligned=True, seed=7)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_backward_without_activation_and_row_list_reads_the_gradient_in_place(dtype):
    """No ReLU to undo and rows = NULL: no compact copy of the gradient is made and the bias gradient is summed inside
    the weight-gradient kernel (many row splits, ragged last tile, narrow and unaligned widths)."""
    _case(70000, 65537, 256, 256, dtype, sage=True, relu=False, use_rows=False, aligned=True, seed=21)
    _case(9000, 8999, 128, 128, dtype, sage=True, relu=False, use_rows=False, aligned=True, seed=22)
    _case(5000, 4097, 100, 256, dtype, sage=False, relu=False, use_rows=False, aligned=True, seed=23)
    _case(5000, 3000, 256, 41, dtype, sage=True, relu=False, use_rows=False, aligned=True, seed=24)
    _case(3000, 1234, 64, 16, dtype, sage=True, relu=False, use_rows=False, aligned=True, seed=25)
    _case(900, 31, 64, 64, dtype, sage=False, relu=False, use_rows=False, aligned=True, seed=26)       # fewer rows than a tile
    _case(500, 257, 602, 41, dtype, sage=True, relu=False, use_rows=False, aligned=False, seed=27)     # unaligned: copies after all


def test_zero_active_rows_zeroes_the_weight_gradients():
    import paper_2311_06837_amd as P
    K, N = 16, 8
    A = torch.randn(10, K, device="cuda")
    W = torch.randn(K, N, device="cuda")
    dW = torch.full((K, N), 5.0, device="cuda")
    db = torch.full((N,), 5.0, device="cuda")
    P.gnn_linear_bwd(None, 0, torch.randn(10, N, device="cuda"), None, False, A, None, K, W, None, dW, None, db)
    H = torch.full((10, N), 5.0, device="cuda")
    P.gnn_linear_fwd(None, 0, A, None, K, W, None, None, H, False)
    torch.cuda.synchronize()
    assert not dW.any() and not db.any() and (H == 5.0).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("C", [8, 41, 47, 16, 32, 100])
def test_softmax_cross_entropy(dtype, C):
    import paper_2311_06837_amd as P
    rng = np.random.default_rng(C)
    n, nt = 5000, 2111
    Z = as_stored(rng.standard_normal((n, C)) * 3, dtype)
    rows = np.sort(rng.choice(n, nt, replace=False)).astype(np.int32)
    y = rng.integers(0, C, nt).astype(np.int32)
    ld = _pad(C, 8)
    Zd = padded(Z, ld, dtype, fill=float("nan") if ld > C else 0.0)
    dZd = torch.full((n, ld), SENT, dtype=dtype, device="cuda")
    loss = torch.zeros(1, device="cuda")
    P.gnn_softmax_ce(dev(rows), nt, Zd, C, dev(y), dZd, loss)
    torch.cuda.synchronize()
    dZ = np.full((n, C), SENT)
    want = oracle.softmax_ce(rows, Z, C, y, dZ)
    assert abs(loss.item() - want) <= 1e-4 * abs(want)
    got = host64(dZd)
    check(got[rows, :C], dZ[rows], dtype, "dZ")
    rest = np.setdiff1d(np.arange(n), rows)
    sent = host64(torch.tensor(SENT, dtype=dtype))
    assert (got[rest] == sent).all() and (got[:, C:] == sent).all()


def test_softmax_cross_entropy_many_rows_and_tiny_class_counts():
    """More rows than one sweep of the launch covers; class counts below the lane-group width and C = 1."""
    import paper_2311_06837_amd as P
    for C, nt, dtype in ((32, 300001, torch.bfloat16), (5, 70001, torch.float32), (1, 100, torch.float32), (64, 3, torch.float32)):
        print(f"softmax-ce: C={C} rows={nt} {dtype}", flush=True)
        rng = np.random.default_rng(C + nt)
        Z = as_stored(rng.standard_normal((nt, C)) * 2, dtype)
        y = rng.integers(0, C, nt).astype(np.int32)
        ld = _pad(C, 8)
        Zd = padded(Z, ld, dtype, fill=float("nan") if ld > C else 0.0)
        dZd = torch.full((nt, ld), SENT, dtype=dtype, device="cuda")
        loss = torch.zeros(1, device="cuda")
        P.gnn_softmax_ce(None, nt, Zd, C, dev(y), dZd, loss)
        torch.cuda.synchronize()
        dZ = np.zeros((nt, C))
        want = oracle.softmax_ce(np.arange(nt, dtype=np.int32), Z, C, y, dZ)
        assert abs(loss.item() - want) <= 1e-4 * max(abs(want), 1e-6)
        got = host64(dZd)
        check(got[:, :C], dZ, dtype, "dZ")
        assert (got[:, C:] == host64(torch.tensor(SENT, dtype=dtype))).all()


def test_norm_scales():
    import paper_2311_06837_amd as P
    deg = np.array([0, 1, 2, 3, 4, 9, 490, 10520], dtype=np.int32)
    for mode, code in (("mean", P.GNN_NORM_MEAN), ("sym", P.GNN_NORM_SYM)):
        got = P.gnn_norm_scales(code, len(deg), length=dev(deg)).cpu().numpy().astype(np.float64)
        want = oracle.norm_scales(mode, deg)
        assert np.allclose(got, want, rtol=2e-7, atol=0)
    rp = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    got = P.gnn_norm_scales(P.GNN_NORM_MEAN, len(deg), row_ptr=dev(rp)).cpu().numpy()
    assert np.allclose(got, oracle.norm_scales("mean", deg), rtol=2e-7)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N,ld", [(47, 48), (256, 256), (7, 7), (100, 104)])
def test_bias_grad(dtype, N, ld):
    """gnn_bias_grad: column sums of the listed rows (the definition, summed in fp64 here)."""
    import paper_2311_06837_amd as P
    rng = np.random.default_rng(N)
    n = 5000
    dZ = as_stored(rng.standard_normal((n, N)), dtype)
    rows = rng.permutation(n)[:3333].astype(np.int32)
    for rws, cnt in ((rows, len(rows)), (None, 4097), (rows, 1), (None, 0)):
        print(f"bias_grad: N={N} ld={ld} {dtype} rows={'list' if rws is not None else 'prefix'} n={cnt}", flush=True)
        db = torch.full((N,), 9.0, device="cuda")
        P.gnn_bias_grad(dev(rws) if rws is not None else None, cnt, padded(dZ, ld, dtype, fill=float("nan")), N, db)
        torch.cuda.synchronize()
        sel = rws[:cnt] if rws is not None else np.arange(cnt)
        want = dZ[sel].sum(0)
        got = db.double().cpu().numpy()
        assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(dZ[sel]).sum(0).max()), (got, want)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K,N", [(256, 41), (256, 32), (128, 16), (256, 256), (96, 47), (40, 7), (512, 128), (128, 64)])
def test_input_gradient_product_with_sum_and_mask_in_its_store(dtype, K, N):
    """gnn_linear_bwd_input: dX = [H > 0] * (dZ W^T + dX on the first n_accumulate listed rows).  The product comes from
    the oracle's feature-transform backward, the sum and the mask are written out here."""
    import paper_2311_06837_amd as P
    rng = np.random.default_rng(K * 1000 + N)
    n = 3000
    params = gg.layer_weights([K, N], False, K + N)[0]
    W = as_stored(params["W_neigh"], dtype)
    dZ = as_stored(rng.standard_normal((n, N)), dtype)
    old = as_stored(rng.standard_normal((n, K)), dtype)
    H = as_stored(np.maximum(rng.standard_normal((n, K)), 0), dtype)
    rows = rng.permutation(n)[:1777].astype(np.int32)
    ld_in, ld_out = P.row_stride(K, dtype), P.row_stride(N, dtype)
    for rws, cnt, n_acc, mask in ((rows, len(rows), 600, True), (None, 2049, 2049, True), (rows, len(rows), 0, True), (rows, 129, 0, False)):
        print(f"linear_bwd_input: K={K} N={N} {dtype} rows={'list' if rws is not None else 'prefix'} n={cnt} n_acc={n_acc} mask={mask}", flush=True)
        dXd = padded(old, ld_in, dtype, fill=SENT)
        P.gnn_linear_bwd_input(dev(rws) if rws is not None else None, cnt, padded(dZ, ld_out, dtype), N, dev(W).to(dtype), K, n_acc,
                               padded(H, ld_in, dtype) if mask else None, dXd)
        torch.cuda.synchronize()
        sel = rws[:cnt] if rws is not None else np.arange(cnt, dtype=np.int32)
        prod = np.zeros((n, K))
        oracle.linear_bwd(sel, dZ, None, False, np.zeros((n, K)), None, K, W, None, prod, None)
        want = old.copy()
        t = prod[sel]
        t[:n_acc] += old[sel[:n_acc]]
        want[sel] = t * (H[sel] > 0) if mask else t
        got = host64(dXd)
        check(got[sel, :K], want[sel], dtype, "listed rows")
        rest = np.setdiff1d(np.arange(n), sel)
        assert np.array_equal(got[rest, :K], old[rest]), "rows outside the list were written"
        if ld_in > K:
            assert (got[:, K:] == host64(torch.tensor(SENT, dtype=dtype))).all()
    # rows to accumulate need the activations of the ReLU they are summed in front of; counts must fit
    with pytest.raises(P.GnnError):
        P.gnn_linear_bwd_input(None, 10, padded(dZ, ld_out, dtype), N, dev(W).to(dtype), K, 5, None, padded(old, ld_in, dtype))
    with pytest.raises(P.GnnError):
        P.gnn_linear_bwd_input(None, 10, padded(dZ, ld_out, dtype), N, dev(W).to(dtype), K, 11, padded(H, ld_in, dtype), padded(old, ld_in, dtype))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K,N", [(128, 128), (256, 256), (256, 41), (128, 16), (96, 47), (40, 7), (602, 256), (512, 256), (128, 192)])
def test_input_gradient_from_the_aggregated_gradient(dtype, K, N):
    """gnn_linear_bwd_input2: dX = [H > 0] * (dG W_neigh^T + dZ W_self^T on the first n_self listed rows).  Both products
    come from the oracle's feature-transform backward; the sum, the row limit and the mask are written out here.  The rows
    of dZ past n_self hold NaN: they are fetched by the kernel and must not reach the result."""
    import paper_2311_06837_amd as P
    rng = np.random.default_rng(K * 1000 + N + 7)
    n = 3000
    params = gg.layer_weights([K, N], True, K + N)[0]
    Wn, Ws = as_stored(params["W_neigh"], dtype), as_stored(params["W_self"], dtype)
    dG = as_stored(rng.standard_normal((n, N)), dtype)
    dZ = as_stored(rng.standard_normal((n, N)), dtype)
    H = as_stored(np.maximum(rng.standard_normal((n, K)), 0), dtype)
    rows = rng.permutation(n)[:1777].astype(np.int32)
    ld_in, ld_out = P.row_stride(K, dtype), P.row_stride(N, dtype)
    # (row list or prefix, listed rows, rows with a self half, mask): limits inside a 128-row tile, at a tile edge, none, all
    for rws, cnt, n_self, mask in ((rows, len(rows), 600, True), (None, 2049, 2049, True), (rows, len(rows), 0, True),
                                   (None, 1500, 1280, False), (rows, 130, 1, True), (None, 700, 129, True)):
        print(f"linear_bwd_input2: K={K} N={N} {dtype} rows={'list' if rws is not None else 'prefix'} n={cnt} n_self={n_self} "
              f"mask={mask}", flush=True)
        sel = rws[:cnt] if rws is not None else np.arange(cnt, dtype=np.int32)
        dZ_poisoned = dZ.copy()
        no_self = np.setdiff1d(np.arange(n), sel[:n_self])
        dZd = padded(dZ_poisoned, ld_out, dtype)
        dZd[dev(no_self.astype(np.int64))] = float("nan")
        dXd = torch.full((n, ld_in), SENT, dtype=dtype, device="cuda")
        P.gnn_linear_bwd_input2(dev(rws) if rws is not None else None, cnt, padded(dG, ld_out, dtype), dev(Wn).to(dtype), dZd,
                                dev(Ws).to(dtype), n_self, N, K, padded(H, ld_in, dtype) if mask else None, dXd)
        torch.cuda.synchronize()
        p1, p2 = np.zeros((n, K)), np.zeros((n, K))
        oracle.linear_bwd(sel, dG, None, False, np.zeros((n, K)), None, K, Wn, None, p1, None)
        if n_self:
            oracle.linear_bwd(sel[:n_self], dZ, None, False, np.zeros((n, K)), None, K, Ws, None, p2, None)
        want = p1[sel] + p2[sel]
        if mask:
            want = want * (H[sel] > 0)
        got = host64(dXd)
        check(got[sel, :K], want, dtype, "listed rows")
        rest = np.setdiff1d(np.arange(n), sel)
        sent = host64(torch.tensor(SENT, dtype=dtype))
        assert (got[rest] == sent).all(), "rows outside the list were written"
        if ld_in > K:
            assert (got[:, K:] == sent).all()
    with pytest.raises(P.GnnError):      # more rows with a self half than rows
        P.gnn_linear_bwd_input2(None, 10, padded(dG, ld_out, dtype), dev(Wn).to(dtype), padded(dZ, ld_out, dtype), dev(Ws).to(dtype), 11,
                                N, K, None, torch.zeros(n, ld_in, dtype=dtype, device="cuda"))
