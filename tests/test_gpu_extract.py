"""GPU parity: gnn_extract_partition and gnn_gather_rows against the oracle (section 6 step 1: the one-hop graph
of the traversed vertices, renumbered by (distance, id)).  Integer outputs are compared bit-exact."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from gpu_util import TOL, backward_at_the_oracles_point, check, dev

pytestmark = pytest.mark.gpu


def _extract_case(g, T, L, what):
    import paper_2311_06837_amd as P
    print(f"extract: {what} n={g.n_rows} nnz={g.nnz} |T|={len(T)} L={L}", flush=True)
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    ws = P.Workspace()
    dist, ring, hop_d, hop = P.gnn_build_active_sets(G, dev(np.asarray(T, dtype=np.int32)), L, ws=ws)
    n_local = int(hop[-1])
    local, new_id = P.gnn_extract_partition(G, ring, n_local, dist, L, ws=ws)
    torch.cuda.synchronize()
    rp, ci, l2g, off, dl = oracle.extract_partition(g.row_ptr, g.col_idx, T, L)
    assert n_local == l2g.size and list(hop) == list(off)
    assert np.array_equal(ring.cpu().numpy()[:n_local], l2g)
    assert np.array_equal(local.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(local.col_idx.cpu().numpy(), ci)
    want_new = np.full(g.n_rows, -1, dtype=np.int32)
    want_new[l2g] = np.arange(l2g.size, dtype=np.int32)
    assert np.array_equal(new_id.cpu().numpy(), want_new)
    assert local.sorted_columns and local.n_rows == n_local and local.nnz == ci.size
    return local, ring, hop, (rp, ci, l2g, off, dl)


@pytest.mark.parametrize("L", [1, 2, 3])
def test_power_law_graph_with_hubs(L):
    g = gg.chung_lu(30000, 40.0, 2.1, 51)                     # hub rows of > 1000 entries
    T = np.sort(np.random.default_rng(L).choice(30000, 300, replace=False))
    _extract_case(g, T, L, "chung-lu")


def test_directed_graph_deep_and_unreached_vertices():
    g = gg.random_directed(20000, 1.5, 52)                    # many empty rows, most vertices never reached
    T = np.sort(np.random.default_rng(2).choice(20000, 50, replace=False))
    local, ring, hop, (rp, ci, l2g, off, dl) = _extract_case(g, T, 8, "directed")
    assert l2g.size < 20000


def test_whole_graph_is_traversed_and_degenerate_sizes():
    import paper_2311_06837_amd as P
    g = gg.erdos_renyi(5000, 12.0, 53)
    _extract_case(g, np.arange(0, 5000, 7), 4, "everything reached")
    _extract_case(g, np.array([17]), 1, "one target")
    # n_local = 0: an empty graph comes back
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    dist = torch.full((5000,), -1, dtype=torch.int32, device="cuda")
    ring = torch.zeros(1, dtype=torch.int32, device="cuda")
    local, new_id = P.gnn_extract_partition(G, ring, 0, dist, 2)
    assert local.n_rows == 0 and local.nnz == 0 and int(local.row_ptr[0]) == 0 and bool((new_id == -1).all())


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("F,ld_src,ld_dst", [(64, 64, 64), (602, 608, 608), (100, 100, 128), (7, 7, 9)])
def test_gather_rows(dtype, F, ld_src, ld_dst):
    import paper_2311_06837_amd as P
    rng = np.random.default_rng(F)
    n_src, n = 4000, 2501
    src = torch.randn(n_src, ld_src, device="cuda").to(dtype)
    ids = rng.integers(0, n_src, size=n).astype(np.int32)
    dst = torch.full((n, ld_dst), 7.0, dtype=dtype, device="cuda")
    P.gnn_gather_rows(src, dev(ids), F, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst[:, :F], src[torch.from_numpy(ids).cuda().long(), :F])
    if ld_dst > F:
        assert bool((dst[:, F:] == 7.0).all()), "pad columns were written"


@pytest.mark.parametrize("kind,dtype", [("sage", torch.float32), ("gcn", torch.float32), ("sage", torch.bfloat16)])
def test_training_step_on_the_extracted_graph(kind, dtype):
    """The whole chain on the GPU - active sets of the unpartitioned graph, extraction, feature gather, one training
    step with prefix row sets - against the oracle's model on the oracle's extraction."""
    import paper_2311_06837_amd as P
    n, L, dims = 20000, 3, [48, 32, 32, 7]
    g = gg.chung_lu(n, 14.0, 2.1, 61)
    if kind == "gcn":
        g = gg.add_self_loops(g)
    rng = np.random.default_rng(61)
    T = np.sort(rng.choice(n, 150, replace=False))
    local, ring, hop, (rp, ci, l2g, off, dl) = _extract_case(g, T, L, f"model {kind}")
    n_local = l2g.size
    assert n_local < n
    params = gg.layer_weights(dims, kind == "sage", 61)
    H0g = gg.features(n, dims[0], 61)
    y = gg.labels(len(T), dims[-1], 61)

    bf16 = dtype == torch.bfloat16
    H0o = oracle.round_bf16(H0g.astype(np.float64)) if bf16 else H0g.astype(np.float64)
    om = oracle.Model(rp, ci, np.arange(len(T), dtype=np.int32), kind, params, g.degrees()[l2g] if kind == "gcn" else None, bf16=bf16)
    loss_o = om.forward(H0o[l2g], y)
    grads_o = om.backward()

    ld0 = P.row_stride(dims[0], dtype)
    H0d = torch.zeros(n_local, ld0, dtype=dtype, device="cuda")
    P.gnn_gather_rows(dev(H0g).to(dtype), ring[:n_local], dims[0], H0d)
    m = P.MaskedGNN(local, local, torch.arange(len(T), dtype=torch.int32, device="cuda"), kind,
                    [{k: dev(v) for k, v in p.items()} for p in params], dtype=dtype,
                    global_degree=dev(g.degrees()[l2g].astype(np.int32)) if kind == "gcn" else None,
                    prefix_numbered=True,     # the extraction numbers by (distance, id): the calls get rows = NULL
                    transform_first=kind == "sage")   # and the narrowing GraphSAGE layers run in the exchanged order
    m.set_input(H0d)
    loss = m.step(dev(y))
    torch.cuda.synchronize()
    assert list(m.hop) == list(off)
    assert torch.equal(m.ring_ids[:n_local].cpu(), torch.arange(n_local, dtype=torch.int32))   # the numbering IS the ring order
    tol = TOL[dtype] * 2 * L
    assert abs(loss.item() - loss_o) <= tol * abs(loss_o), (loss.item(), loss_o)
    backward_at_the_oracles_point(m, om, dims, dtype, dev(y))     # same ReLU decisions on both sides, then element by element
    for l, gr in enumerate(grads_o):
        for k, want in gr.items():
            check(m.grads[l][k].double().cpu().numpy(), want, dtype, f"layer {l + 1} {k}", calls=L - l)


# ---- extraction after boundary sampling ----------------------------------------------------------------------

def _sampled_case(g, T, fanout, seed, what):
    import paper_2311_06837_amd as P
    print(f"extract sampled: {what} n={g.n_rows} nnz={g.nnz} |T|={len(T)} fanout={fanout}", flush=True)
    n = g.n_rows
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = dev(np.asarray(T, dtype=np.int32))
    bits = P.gnn_make_bitmap(Td, n)
    ws = P.Workspace()
    srp, sci = P.gnn_sample_boundary(G, bits, Td, fanout, seed, ws=ws)
    local, l2g_d, hop = P.gnn_extract_sampled_partition(G, Td, srp, sci, ws=ws)      # symmetric graph: gT = g
    torch.cuda.synchronize()
    is_t = np.zeros(n, dtype=np.uint8)
    is_t[T] = 1
    osrp, osci = oracle.sample_boundary(g.row_ptr, g.col_idx, is_t, T, fanout, seed)
    rp, ci, l2g, off, dl = oracle.extract_sampled(n, T, osrp, osci)
    assert list(hop) == list(off)
    assert np.array_equal(l2g_d.cpu().numpy(), l2g)
    assert np.array_equal(local.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(local.col_idx.cpu().numpy(), ci)
    return local, l2g_d, (rp, ci, l2g, off, dl)


@pytest.mark.parametrize("fanout", [0, 3, 5, 100000])
def test_sampled_extraction_power_law(fanout):
    g = gg.chung_lu(40000, 15.0, 2.1, 81)
    pid = gg.bfs_partition(g, 8, 81)
    T = np.flatnonzero(pid == 0)
    _sampled_case(g, T, fanout, 0x5EED, "one of 8 parts")


def test_sampled_extraction_hub_outside_vertex_and_tiny_sets():
    n = 30000
    base = gg.erdos_renyi(n, 6.0, 82)
    rng = np.random.default_rng(82)
    T = np.sort(rng.choice(np.arange(1, n), 6000, replace=False))
    r = np.repeat(np.arange(n, dtype=np.int64), np.diff(base.row_ptr))
    c = base.col_idx.astype(np.int64)
    z = np.zeros(T.size, dtype=np.int64)
    g = gg.csr_from_edges(n, n, np.concatenate([r, z, T]), np.concatenate([c, T, z]))   # vertex 0 (outside) adjacent to every target
    local, l2g, (rp, ci, l2g_o, off, dl) = _sampled_case(g, T, 4, 7, "outside hub")
    k = int(np.searchsorted(l2g_o[len(T):], 0)) + len(T)
    assert l2g_o[k] == 0 and rp[k + 1] - rp[k] > 1024                     # a long reverse row
    _sampled_case(g, np.array([5]), 2, 1, "one target")


def test_training_step_after_sampling_and_extraction():
    """configs[4]'s chain at small size, all on the GPU: sample, extract, gather features, one bf16 training step."""
    import paper_2311_06837_amd as P
    n, dims, dtype = 40000, [64, 48, 48, 5], torch.bfloat16
    g = gg.chung_lu(n, 15.0, 2.1, 83)
    T = np.flatnonzero(gg.bfs_partition(g, 8, 83) == 0)
    local, l2g_d, (rp, ci, l2g, off, dl) = _sampled_case(g, T, 5, 0xABC, "model")
    n_local, L = l2g.size, 3
    params = gg.layer_weights(dims, True, 83)
    H0g = gg.features(n, dims[0], 83)
    y = gg.labels(len(T), dims[-1], 83)
    H0o = oracle.round_bf16(H0g.astype(np.float64))
    om = oracle.Model(rp, ci, np.arange(len(T), dtype=np.int32), "sage", params, bf16=True)
    loss_o = om.forward(H0o[l2g], y)
    grads_o = om.backward()
    H0d = torch.zeros(n_local, P.row_stride(dims[0], dtype), dtype=dtype, device="cuda")
    P.gnn_gather_rows(dev(H0g).to(dtype), l2g_d, dims[0], H0d)
    m = P.MaskedGNN(local, local, torch.arange(len(T), dtype=torch.int32, device="cuda"), "sage",
                    [{k: dev(v) for k, v in p.items()} for p in params], dtype=dtype, prefix_numbered=True,
                    transform_first=True)
    m.set_input(H0d)
    loss = m.step(dev(y))
    torch.cuda.synchronize()
    assert [int(x) for x in m.hop] == [0, len(T), n_local, n_local, n_local]      # dist is 0 or 1: every later ring is empty
    tol = TOL[dtype] * 2 * L
    assert abs(loss.item() - loss_o) <= tol * abs(loss_o), (loss.item(), loss_o)
    backward_at_the_oracles_point(m, om, dims, dtype, dev(y))     # same ReLU decisions on both sides, then element by element
    for l, gr in enumerate(grads_o):
        for k, want in gr.items():
            check(m.grads[l][k].double().cpu().numpy(), want, dtype, f"layer {l + 1} {k}", calls=L - l)
