"""GPU parity of the whole masked forward/backward against the oracle model (sections 2.1, 6)
on scaled-down versions of the five workloads, plus the masking invariants on the GPU."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import TOL, as_stored, backward_at_the_oracles_point, check, dev, host64, padded

pytestmark = pytest.mark.gpu


def _gpu_model(part, kind, params, dtype, transform_first="auto", grad_first="auto"):
    import paper_2311_06837_amd as P
    G = P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
    same = part.graph_t is part.graph
    GT = G if same else P.Graph.from_numpy(part.graph_t.row_ptr, part.graph_t.col_idx)
    dparams = [{k: dev(v) for k, v in p.items()} for p in params]
    return P.MaskedGNN(G, GT, dev(part.targets), kind, dparams, dtype=dtype,
                       global_degree=dev(part.global_degree) if kind == "gcn" else None, transform_first=transform_first,
                       grad_first=grad_first)


def _parity(name, part, kind, dims, dtype, seed, transform_first="auto", grad_first="auto"):
    """transform_first: the order of the first layer's halves on the GPU ("auto": weights first where the layer narrows
    its input).  The oracle always aggregates first; the two orders are the same sums up to rounding."""
    print(f"model {name}: n={part.graph.n_rows} nnz={part.graph.nnz} |T|={len(part.targets)} {kind} dims={dims} {dtype} "
          f"transform_first={transform_first}", flush=True)
    import paper_2311_06837_amd as P
    L = len(dims) - 1
    params = gg.layer_weights(dims, kind == "sage", seed)
    n = part.graph.n_rows
    H0 = as_stored(gg.features(n, dims[0], seed), dtype)
    y = gg.labels(len(part.targets), dims[-1], seed)
    bf16 = dtype == torch.bfloat16

    om = oracle.Model(part.graph.row_ptr, part.graph.col_idx, part.targets, kind, params,
                      part.global_degree if kind == "gcn" else None, bf16=bf16)
    loss_o = om.forward(H0, y)
    grads_o = om.backward()

    m = _gpu_model(part, kind, params, dtype, transform_first, grad_first)
    if transform_first != "auto":
        narrowing = {l for l in range(1, len(dims)) if dims[l - 1] > dims[l]}
        assert m.tf_layers == (narrowing if transform_first else set())
    hop = m.build_active_sets()
    assert list(hop) == list(om.hop_offsets)
    assert np.array_equal(m.dist.cpu().numpy(), om.dist)
    assert np.array_equal(m.ring_ids.cpu().numpy()[: hop[-1]], om.ring_ids)
    m.set_input(padded(H0, P.row_stride(dims[0], dtype), dtype))
    loss = m.forward(dev(y))
    m.backward()
    torch.cuda.synchronize()

    tol = TOL[dtype]
    assert abs(loss.item() - loss_o) <= tol * abs(loss_o), (loss.item(), loss_o)
    for l in range(1, L + 1):
        rows = om.rows_of_layer(l)
        if m.A[l] is not None:          # (the exchanged order never forms the aggregate of the input features)
            check(host64(m.A[l])[rows, : dims[l - 1]], om.A[l][rows], dtype, f"{name} A_{l}", calls=l)
        check(host64(m.H[l])[rows, : dims[l]], om.H[l][rows], dtype, f"{name} H_{l}", calls=l)
    # every gradient element by element: the backward pass again from the oracle's forward point (gpu_util explains why)
    backward_at_the_oracles_point(m, om, dims, dtype, dev(y))
    for l in range(L):
        for k, want in grads_o[l].items():
            check(host64(m.grads[l][k]), want, dtype, f"{name} layer {l + 1} {k}", calls=L - l)
    return m, om


@pytest.mark.parametrize("transform_first", [False, True])
def test_cfg0_full_size(transform_first):
    w = gg.make_workload("cfg0")
    _parity("cfg0", w.partition, w.model, w.dims, torch.float32, 0, transform_first)      # GCN 64-64-8: the last layer narrows


@pytest.mark.parametrize("transform_first", [False, True])
def test_cfg1_scaled(transform_first):
    w = gg.make_workload("cfg1", scale=0.02)
    assert w.dims[0] > w.dims[1]
    _parity("cfg1@0.02", w.partition, w.model, w.dims, torch.float32, 1, transform_first)


@pytest.mark.parametrize("dims", [[96, 64, 64, 7], [40, 12], [64, 48, 32, 16, 5], [16, 32, 8]])
def test_transform_first_bf16_and_single_layer(dims):
    """Layers in the exchanged order in both storage types: first and last layer with a plain one between, the only
    layer (its output is the logits: no ReLU, the gradient comes straight from the loss), every layer (their input
    gradients hand over masked from one to the next), only the last."""
    g = gg.chung_lu(5000, 9.0, 2.2, 61)
    T = np.sort(np.random.default_rng(61).choice(5000, 300, replace=False)).astype(np.int64)
    part = gg.halo_partition(g, T, len(dims) - 1)
    _parity("narrowing", part, "sage", dims, torch.bfloat16, 61, True)
    _parity("narrowing", part, "sage", dims, torch.float32, 62, True)


@pytest.mark.parametrize("transform_first", [False, True])
def test_cfg2_scaled(transform_first):
    w = gg.make_workload("cfg2", scale=0.01)
    _parity("cfg2@0.01", w.partition, w.model, w.dims, torch.float32, 2, transform_first)  # GCN 100-256-256-47


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gcn_every_layer_in_the_exchanged_order(dtype):
    """GCN layers have no self term: the aggregation starts from the bias, the bias gradient is summed on its own."""
    g = gg.add_self_loops(gg.chung_lu(5000, 9.0, 2.2, 63))
    T = np.sort(np.random.default_rng(63).choice(5000, 300, replace=False)).astype(np.int64)
    part = gg.halo_partition(g, T, 3)
    _parity("gcn narrowing", part, "gcn", [64, 48, 24, 6], dtype, 63, True)


def test_cfg3_scaled_deep_bf16():
    w = gg.make_workload("cfg3", scale=0.02)
    _parity("cfg3@0.02", w.partition, w.model, w.dims, torch.bfloat16, 3)


def test_cfg4_scaled_sampled_bf16():
    import paper_2311_06837_amd as P
    w = gg.make_workload("cfg4", scale=0.004)
    g, T = w.global_graph, w.targets_global.astype(np.int32)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = dev(T)
    rp, ci = P.gnn_sample_boundary(G, P.gnn_make_bitmap(Td, g.n_rows), Td, w.fanout, w.sample_seed)
    is_t = np.zeros(g.n_rows, dtype=np.uint8)
    is_t[T] = 1
    orp, oci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, w.fanout, w.sample_seed)
    assert np.array_equal(rp.cpu().numpy(), orp) and np.array_equal(ci.cpu().numpy(), oci)
    # the local one-hop graph of the sampled partition (host-side extraction from the kept rows)
    l2g, er, ec = oracle.sampled_local_edges(T, orp, oci)
    part = gg.partition_from_edges(g.n_rows, l2g, er, ec, T, g.degrees())
    _parity("cfg4@0.004", part, w.model, w.dims, torch.bfloat16, 4)


def test_directed_graph_uses_the_transpose():
    g = gg.random_directed(6000, 5.0, 41)
    T = np.sort(np.random.default_rng(41).choice(6000, 200, replace=False)).astype(np.int64)
    part = gg.halo_partition(g, T, 3, symmetric=False)
    assert part.graph_t is not part.graph
    _parity("directed", part, "sage", [32, 24, 16, 5], torch.float32, 41, False)
    _parity("directed", part, "sage", [32, 24, 16, 5], torch.float32, 41, True)    # every layer aggregates backward through gT


def test_masked_equals_unmasked_on_targets_on_the_gpu():
    """Section 6, step 5, checked on the device alone: computing every row at every layer
    (targets = the whole partition gives dist = 0 everywhere) leaves the targets' logits unchanged."""
    import paper_2311_06837_amd as P
    w = gg.make_workload("cfg0", scale=0.3)
    part = w.partition
    params = gg.layer_weights(w.dims, False, 5)
    H0 = padded(gg.features(part.graph.n_rows, w.dims[0], 5), w.dims[0], torch.float32)
    y = dev(gg.labels(len(part.targets), w.dims[-1], 5))
    masked = _gpu_model(part, "gcn", params, torch.float32)
    masked.build_active_sets()
    masked.set_input(H0)
    masked.forward(y)
    G = masked.g
    every = torch.arange(part.graph.n_rows, dtype=torch.int32, device="cuda")
    full = P.MaskedGNN(G, G, every, "gcn", [{k: dev(v) for k, v in p.items()} for p in params],
                       global_degree=dev(part.global_degree))
    full.build_active_sets()
    full.set_input(H0)
    full.forward(dev(gg.labels(part.graph.n_rows, w.dims[-1], 5)))
    torch.cuda.synchronize()
    t = dev(part.targets).long()
    a, b = masked.H[-1][t][:, : w.dims[-1]], full.H[-1][t][:, : w.dims[-1]]
    assert torch.allclose(a, b, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("F,ld", [(256, 256), (100, 104), (41, 44), (7, 7)])
def test_add_rows_masked(dtype, F, ld):
    """gnn_add_rows_masked: the two input gradients of a layer in the exchanged order meet in front of a ReLU.
    Elementwise, so the expected values are the definition written out (one rounding of the sum in storage precision)."""
    import paper_2311_06837_amd as P
    SENT = 777.0
    rng = np.random.default_rng(F)
    n = 2000
    rows = rng.permutation(n)[:1234].astype(np.int32)
    n_add = 400
    X, Y = as_stored(rng.standard_normal((n, F)), dtype), as_stored(rng.standard_normal((n, F)), dtype)
    H = as_stored(np.maximum(rng.standard_normal((n, F)), 0), dtype)
    for rws, n_act, n_a in ((rows, len(rows), n_add), (None, 1500, 1500), (rows, len(rows), 0)):
        print(f"add_rows_masked: F={F} ld={ld} {dtype} rows={'list' if rws is not None else 'prefix'} n={n_act} n_add={n_a}", flush=True)
        Yd = padded(Y, ld, dtype, fill=SENT)
        Xd = padded(X, ld, dtype, fill=float("nan")) if n_a else None
        P.gnn_add_rows_masked(dev(rws) if rws is not None else None, n_act, Xd, n_a, Yd, F, padded(H, ld, dtype, fill=float("nan")))
        torch.cuda.synchronize()
        sel = rws if rws is not None else np.arange(n_act)
        want = Y.copy()
        t = Y[sel].copy()
        t[:n_a] += X[sel[:n_a]]
        want[sel] = as_stored(t, dtype) * (H[sel] > 0)
        got = host64(Yd)
        assert np.array_equal(got[:, :F], want)
        assert (got[:, F:] == host64(torch.tensor(SENT, dtype=dtype))).all()
    with pytest.raises(P.GnnError):
        P.gnn_add_rows_masked(None, 10, padded(X, ld, dtype), 11, padded(Y, ld, dtype), F, padded(H, ld, dtype))


@pytest.mark.parametrize("kind,dims", [("sage", [96, 64, 64, 7]), ("gcn", [64, 48, 24, 6]), ("sage", [16, 32, 32, 8])])
def test_side_stream_changes_nothing(kind, dims):
    """The weight-gradient products run on a second stream by default; with everything on one stream the step gives the
    same bits (same kernels, same inputs - only the order in time differs)."""
    import paper_2311_06837_amd as P
    g = gg.chung_lu(6000, 9.0, 2.2, 71)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    T = np.sort(np.random.default_rng(71).choice(6000, 400, replace=False)).astype(np.int64)
    part = gg.halo_partition(g, T, 3)
    params = gg.layer_weights(dims, kind == "sage", 71)
    H0 = padded(gg.features(part.graph.n_rows, dims[0], 71), P.row_stride(dims[0], torch.float32), torch.float32)
    y = dev(gg.labels(len(part.targets), dims[-1], 71))
    out = []
    for side in (True, False):
        G = P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
        m = P.MaskedGNN(G, G, dev(part.targets), kind, [{k: dev(v) for k, v in p.items()} for p in params],
                        global_degree=dev(part.global_degree) if kind == "gcn" else None, transform_first=True, side_stream=side)
        m.set_input(H0)
        for _ in range(2):                      # twice: the second step reuses every buffer while the side stream may still run
            loss = m.step(y)
        torch.cuda.synchronize()
        out.append((loss.item(), [{k: v.clone() for k, v in gr.items()} for gr in m.grads]))
    assert out[0][0] == out[1][0]
    for ga, gb in zip(out[0][1], out[1][1]):
        for k in ga:
            assert torch.equal(ga[k], gb[k]), k


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("transform_first", [False, True])
def test_backward_in_the_chain_rules_order(dtype, transform_first):
    """grad_first=False: input gradients per half (dA = dZ W_neigh^T, aggregated onto dZ W_self^T) instead of the default
    one product from the aggregated output gradient; a widening layer keeps this order under "auto" as well."""
    g = gg.chung_lu(5000, 9.0, 2.2, 71)
    T = np.sort(np.random.default_rng(71).choice(5000, 300, replace=False)).astype(np.int64)
    part = gg.halo_partition(g, T, 3)
    m, _ = _parity("chain-rule order", part, "sage", [64, 48, 48, 6], dtype, 71, transform_first, grad_first=False)
    assert not m.gf_layers
    m, _ = _parity("widening", part, "sage", [32, 48, 64, 6], dtype, 72, transform_first)
    assert m.gf_layers == {3}


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fused_forward_layers(dtype):
    """fused_forward=True: the layers of a shape the one-kernel layer takes keep no aggregate; their weight gradient comes
    from the aggregated output gradient.  Same results as the two-call path up to rounding."""
    g = gg.chung_lu(6000, 10.0, 2.2, 73)
    T = np.sort(np.random.default_rng(73).choice(6000, 400, replace=False)).astype(np.int64)
    part = gg.halo_partition(g, T, 3)
    dims = [64, 64, 64, 6]
    print(f"fused model: {dtype}", flush=True)
    import paper_2311_06837_amd as P
    params = gg.layer_weights(dims, True, 73)
    n = part.graph.n_rows
    H0 = as_stored(gg.features(n, dims[0], 73), dtype)
    y = gg.labels(len(part.targets), dims[-1], 73)
    om = oracle.Model(part.graph.row_ptr, part.graph.col_idx, part.targets, "sage", params, None, bf16=dtype == torch.bfloat16)
    loss_o = om.forward(H0, y)
    grads_o = om.backward()
    G = P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
    m = P.MaskedGNN(G, G, dev(part.targets), "sage", [{k: dev(v) for k, v in p.items()} for p in params], dtype=dtype,
                    transform_first=False, fused_forward=True)
    assert m.fused_layers == {2, 3} and m.A[2] is None and m.A[3] is None and m.A[1] is not None
    m.set_input(padded(H0, P.row_stride(dims[0], dtype), dtype))
    loss = m.step(dev(y))
    torch.cuda.synchronize()
    assert abs(loss.item() - loss_o) <= TOL[dtype] * abs(loss_o)
    for l in range(1, 4):
        rows = om.rows_of_layer(l)
        check(host64(m.H[l])[rows, : dims[l]], om.H[l][rows], dtype, f"fused H_{l}", calls=l)
    backward_at_the_oracles_point(m, om, dims, dtype, dev(y))
    for l in range(3):
        for k, want in grads_o[l].items():
            check(host64(m.grads[l][k]), want, dtype, f"fused layer {l + 1} {k}", calls=3 - l)
