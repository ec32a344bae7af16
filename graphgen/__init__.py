"""Seeded synthetic inputs for the masked GNN-layer hot path.

This module only *makes inputs*: graphs, partitions, feature/weight/label
arrays.  It holds none of the method's arithmetic (no aggregation, no active
sets, no normalisation factors, no sampling hash); the CPU oracle and the HIP
library each implement those on their own and both read the arrays made here.

Graph convention (one-hop graph, paper section 6): CSR row ``v`` lists the
vertices ``u`` whose hidden vectors ``v`` aggregates.  ``row_ptr`` and
``col_idx`` are int32, columns of a row strictly ascending (no duplicates).

The shapes stand in for the datasets of the paper's Table 3 (Reddit,
ogbn-products, IGB) which are not available here; see ``WORKLOADS``.
"""
from __future__ import annotations

import dataclasses
import numpy as np
import scipy.sparse as sp


# --------------------------------------------------------------------------
# CSR plumbing
# --------------------------------------------------------------------------
@dataclasses.dataclass
class CSR:
    n_rows: int
    n_cols: int
    row_ptr: np.ndarray  # int32 [n_rows+1]
    col_idx: np.ndarray  # int32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])

    def to_scipy(self) -> sp.csr_matrix:
        data = np.ones(self.col_idx.shape[0], dtype=np.int8)
        return sp.csr_matrix((data, self.col_idx, self.row_ptr), shape=(self.n_rows, self.n_cols))

    def degrees(self) -> np.ndarray:
        return np.diff(self.row_ptr).astype(np.int32)


def _from_scipy(m: sp.spmatrix) -> CSR:
    m = m.tocsr()
    m.sum_duplicates()
    m.sort_indices()
    if m.nnz >= 2**31:
        raise ValueError("nnz does not fit int32 row_ptr")
    return CSR(m.shape[0], m.shape[1], m.indptr.astype(np.int32), m.indices.astype(np.int32))


def csr_from_edges(n_rows: int, n_cols: int, rows: np.ndarray, cols: np.ndarray) -> CSR:
    """CSR with one entry per distinct (row, col) pair, columns ascending."""
    data = np.ones(rows.shape[0], dtype=np.int8)
    m = sp.coo_matrix((data, (rows, cols)), shape=(n_rows, n_cols)).tocsr()
    return _from_scipy(m)


def transpose(g: CSR) -> CSR:
    return _from_scipy(g.to_scipy().T)


def add_self_loops(g: CSR) -> CSR:
    """Insert (v, v) into every row that lacks it (graph structure only)."""
    assert g.n_rows == g.n_cols
    m = g.to_scipy().astype(np.int8) + sp.identity(g.n_rows, dtype=np.int8, format="csr")
    return _from_scipy(m)


def is_symmetric(g: CSR) -> bool:
    t = transpose(g)
    return np.array_equal(t.row_ptr, g.row_ptr) and np.array_equal(t.col_idx, g.col_idx)


# --------------------------------------------------------------------------
# random graphs
# --------------------------------------------------------------------------
def _symmetric_from_pairs(n: int, a: np.ndarray, b: np.ndarray) -> sp.csr_matrix:
    keep = a != b
    a, b = a[keep], b[keep]
    data = np.ones(a.shape[0], dtype=np.int8)
    m = sp.coo_matrix((data, (a, b)), shape=(n, n)).tocsr()
    m = m + m.T
    m.data[:] = 1
    return m


def erdos_renyi(n: int, avg_deg: float, seed: int) -> CSR:
    """Symmetric G(n, m) graph with about ``avg_deg`` neighbours per vertex."""
    rng = np.random.default_rng([seed, 0x45525F])
    want = int(round(n * avg_deg))  # directed entries
    m = None
    for _ in range(8):
        have = 0 if m is None else m.nnz
        if have >= want * 0.995:
            break
        k = max(16, int((want - have) * 0.5) + 1)
        a = rng.integers(0, n, size=k, dtype=np.int64)
        b = rng.integers(0, n, size=k, dtype=np.int64)
        add = _symmetric_from_pairs(n, a, b)
        m = add if m is None else m + add
        m.data[:] = 1
    return _from_scipy(m)


def _powerlaw_weights(n: int, avg_deg: float, gamma: float) -> np.ndarray:
    """Expected degrees w_i ~ i^(-1/(gamma-1)), capped so w_i*w_j <= sum(w)."""
    total = n * avg_deg
    cap = min(np.sqrt(total), n - 1.0)
    shape = np.arange(1, n + 1, dtype=np.float64) ** (-1.0 / (gamma - 1.0))
    lo, hi = 0.0, total * 64
    for _ in range(200):
        c = 0.5 * (lo + hi)
        s = np.minimum(cap, c * shape).sum()
        if s < total:
            lo = c
        else:
            hi = c
    return np.minimum(cap, hi * shape)


def chung_lu(n: int, avg_deg: float, gamma: float, seed: int) -> CSR:
    """Symmetric power-law graph (Chung-Lu, edge-sampling form).

    Endpoints of each undirected edge are drawn independently with
    probability proportional to the expected-degree weights; self-loops and
    repeated pairs are dropped and the loss topped up, so the realised
    number of directed entries is within 1 % of ``n*avg_deg``.  Vertex
    labels are randomly permuted so that hubs are spread over the id range.
    """
    rng = np.random.default_rng([seed, 0x434C5F])
    w = _powerlaw_weights(n, avg_deg, gamma)
    perm = rng.permutation(n).astype(np.int64)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    want = int(round(n * avg_deg))
    m = None
    for _ in range(12):
        have = 0 if m is None else m.nnz
        if have >= want * 0.99:
            break
        k = max(16, int((want - have) * 0.5) + 1)
        a = perm[np.searchsorted(cdf, rng.random(k), side="right").clip(0, n - 1)]
        b = perm[np.searchsorted(cdf, rng.random(k), side="right").clip(0, n - 1)]
        add = _symmetric_from_pairs(n, a, b)
        m = add if m is None else m + add
        m.data[:] = 1
    return _from_scipy(m)


def random_directed(n: int, avg_deg: float, seed: int) -> CSR:
    """Directed (non-symmetric) random graph; used by tests of the transposed path."""
    rng = np.random.default_rng([seed, 0x444952])
    k = int(round(n * avg_deg))
    a = rng.integers(0, n, size=k, dtype=np.int64)
    b = rng.integers(0, n, size=k, dtype=np.int64)
    keep = a != b
    return csr_from_edges(n, n, a[keep], b[keep])


# --------------------------------------------------------------------------
# partitions and halos (which vertices a GPU holds; not how they are used)
# --------------------------------------------------------------------------
def _neighbours_of(g: CSR, frontier: np.ndarray) -> np.ndarray:
    """Concatenated rows of ``frontier`` (with repeats)."""
    if frontier.size == 0:
        return np.zeros(0, dtype=np.int32)
    start = g.row_ptr[frontier].astype(np.int64)
    cnt = (g.row_ptr[frontier + 1] - g.row_ptr[frontier]).astype(np.int64)
    tot = int(cnt.sum())
    if tot == 0:
        return np.zeros(0, dtype=np.int32)
    off = np.repeat(start - np.concatenate(([0], np.cumsum(cnt)[:-1])), cnt)
    return g.col_idx[off + np.arange(tot, dtype=np.int64)]


def bfs_partition(g: CSR, n_parts: int, seed: int) -> np.ndarray:
    """Stand-in for a min-cut partitioner: seeded breadth-first region growing.

    ``n_parts`` random roots grow in round-robin, one BFS level at a time,
    each part claiming unassigned vertices (lowest id first) up to
    ceil(n/n_parts); what is left when every frontier is exhausted is dealt
    out by lowest id to the parts that still have room.  Returns int32 part
    ids.
    """
    n = g.n_rows
    cap = -(-n // n_parts)
    rng = np.random.default_rng([seed, 0x504152])
    part = np.full(n, -1, dtype=np.int32)
    roots = rng.choice(n, size=n_parts, replace=False)
    size = np.zeros(n_parts, dtype=np.int64)
    frontiers = []
    for p, r in enumerate(roots):
        part[r] = p
        size[p] = 1
        frontiers.append(np.array([r], dtype=np.int64))
    active = True
    while active:
        active = False
        for p in range(n_parts):
            f = frontiers[p]
            if f.size == 0 or size[p] >= cap:
                frontiers[p] = f[:0]
                continue
            cand = np.unique(_neighbours_of(g, f))
            cand = cand[part[cand] < 0]
            room = cap - size[p]
            cand = cand[:room]
            part[cand] = p
            size[p] += cand.size
            frontiers[p] = cand.astype(np.int64)
            if cand.size:
                active = True
    rest = np.flatnonzero(part < 0)
    pos = 0
    for p in range(n_parts):
        room = int(cap - size[p])
        take = rest[pos:pos + room]
        part[take] = p
        pos += take.size
    assert pos == rest.size
    return part


@dataclasses.dataclass
class Partition:
    """One GPU's share: target vertices plus every vertex within ``hops`` of them.

    Local ids are the positions in ``local_to_global`` (ascending global id),
    so the local numbering carries no information about hop distance.
    ``graph`` is the sub-graph induced on the local vertices;
    ``global_degree[v]`` is the row length of local vertex ``v`` in the
    *global* graph (rows of the outermost vertices are cut short locally).
    """
    graph: CSR
    graph_t: CSR
    local_to_global: np.ndarray  # int64 [n_local]
    targets: np.ndarray          # int32 local ids, ascending
    global_degree: np.ndarray    # int32 [n_local]


def halo_partition(g: CSR, targets_global: np.ndarray, hops: int, symmetric: bool = True) -> Partition:
    n = g.n_rows
    held = np.zeros(n, dtype=bool)
    held[targets_global] = True
    frontier = np.unique(targets_global).astype(np.int64)
    for _ in range(hops):
        nb = np.unique(_neighbours_of(g, frontier))
        nb = nb[~held[nb]]
        if nb.size == 0:
            break
        held[nb] = True
        frontier = nb.astype(np.int64)
    l2g = np.flatnonzero(held).astype(np.int64)
    deg = g.degrees()[l2g]
    if l2g.size == n:
        local = g
    else:
        m = g.to_scipy()[l2g][:, l2g]
        local = _from_scipy(m)
    g2l = np.full(n, -1, dtype=np.int64)
    g2l[l2g] = np.arange(l2g.size)
    t_local = np.sort(g2l[np.unique(targets_global)]).astype(np.int32)
    local_t = local if symmetric else transpose(local)
    return Partition(local, local_t, l2g, t_local, deg.astype(np.int32))


def partition_from_edges(n_global: int, local_to_global: np.ndarray, rows_g: np.ndarray, cols_g: np.ndarray,
                         targets_global: np.ndarray, global_degree_of: np.ndarray) -> Partition:
    """Partition over an explicit (already chosen) local edge list in global ids."""
    g2l = np.full(n_global, -1, dtype=np.int64)
    g2l[local_to_global] = np.arange(local_to_global.size)
    local = csr_from_edges(local_to_global.size, local_to_global.size, g2l[rows_g], g2l[cols_g])
    t_local = np.sort(g2l[np.unique(targets_global)]).astype(np.int32)
    return Partition(local, transpose(local), local_to_global.astype(np.int64), t_local,
                     global_degree_of[local_to_global].astype(np.int32))


# --------------------------------------------------------------------------
# dense inputs
# --------------------------------------------------------------------------
def features(n: int, f: int, seed: int, ld: int | None = None) -> np.ndarray:
    """fp32 N(0,1) features, row-major with leading dimension ``ld`` (pad = 0)."""
    rng = np.random.default_rng([seed, 0x464541])
    ld = f if ld is None else ld
    out = np.zeros((n, ld), dtype=np.float32)
    block = max(1, (1 << 24) // max(f, 1))
    for s in range(0, n, block):
        e = min(n, s + block)
        out[s:e, :f] = rng.standard_normal((e - s, f), dtype=np.float32)
    return out


def layer_weights(dims: list[int], sage: bool, seed: int) -> list[dict]:
    """Per layer: W_neigh [K,N] (+ W_self for GraphSAGE) ~ N(0, 1/K), bias ~ N(0, 0.01)."""
    rng = np.random.default_rng([seed, 0x574549])
    out = []
    for k, n in zip(dims[:-1], dims[1:]):
        p = {"W_neigh": (rng.standard_normal((k, n)) / np.sqrt(k)).astype(np.float32)}
        if sage:
            p["W_self"] = (rng.standard_normal((k, n)) / np.sqrt(k)).astype(np.float32)
        p["bias"] = (0.1 * rng.standard_normal(n)).astype(np.float32)
        out.append(p)
    return out


def res_layer_weights(dims: list[int], seed: int) -> list[dict]:
    """Parameters of the deep residual GraphSAGE: layer_weights(sage) plus, from the second layer on, the scale and
    shift of the layer normalisation in front of it (ln_gamma ~ 1 + N(0, 0.01), ln_beta ~ N(0, 0.01), float32)."""
    out = layer_weights(dims, True, seed)
    rng = np.random.default_rng([seed, 0x4C4E])
    for l in range(1, len(out)):
        k = dims[l]
        out[l]["ln_gamma"] = (1.0 + 0.1 * rng.standard_normal(k)).astype(np.float32)
        out[l]["ln_beta"] = (0.1 * rng.standard_normal(k)).astype(np.float32)
    return out


def labels(n: int, n_classes: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 0x4C4142])
    return rng.integers(0, n_classes, size=n, dtype=np.int32)


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    name: str
    model: str            # "gcn" | "sage"
    dtype: str            # "f32" | "bf16"
    dims: list            # [F_in, hidden..., classes]
    n_layers: int
    partition: Partition | None = None
    global_graph: CSR | None = None
    targets_global: np.ndarray | None = None
    fanout: int = 0
    seed: int = 0
    sample_seed: int = 0


WORKLOADS = {
    # name: (stands in for, generator description)
    "cfg0": "toy: Erdos-Renyi n=10000 avg deg 10; 2-layer GCN 64-64-8 fp32; targets 0..1999, 2-hop halo",
    "cfg1": "Reddit-like: Chung-Lu gamma 2.1 n=233000 avg deg ~490; 3-layer SAGE-mean 602-256-256-41 fp32; "
            "targets random n/8, 3-hop halo",
    "cfg2": "products-like: Chung-Lu n=2.45M avg deg ~50; 3-layer GCN 100-256-256-47 fp32; targets = part 0 of "
            "8-way BFS-grown partition, 3-hop halo",
    "cfg3": "deep: Chung-Lu n=1M avg deg 20; 8-layer SAGE-mean 128-(128x7)-16 bf16; targets = 1/16 partition, 8-hop halo",
    "cfg4": "IGB-medium-like: Chung-Lu n=10M avg deg 15; 3-layer SAGE-mean 128-256-256-32 bf16; targets = 1/8 "
            "partition; boundary edges sampled at fanout 5 (done by the method, not here)",
}


def _cache_path(name: str, scale: float, seed) -> str | None:
    import os
    d = os.environ.get("GRAPHGEN_CACHE")
    if not d:
        return None
    os.makedirs(d, exist_ok=True)
    return os.path.join(d, f"{name}_s{scale:g}_seed{'d' if seed is None else seed}.npz")


def _save_workload(path: str, w: Workload) -> None:
    """Plain arrays only (numpy's own container, no pickled objects)."""
    a = {"meta": np.array([w.n_layers, w.fanout, w.seed, w.sample_seed, 1 if w.partition is not None else 0], dtype=np.int64),
         "dims": np.array(w.dims, dtype=np.int64), "g_rp": w.global_graph.row_ptr, "g_ci": w.global_graph.col_idx,
         "g_shape": np.array([w.global_graph.n_rows, w.global_graph.n_cols], dtype=np.int64), "tg": w.targets_global}
    if w.partition is not None:
        p = w.partition
        sym = p.graph_t is p.graph
        a.update({"p_rp": p.graph.row_ptr, "p_ci": p.graph.col_idx, "p_l2g": p.local_to_global, "p_t": p.targets,
                  "p_deg": p.global_degree, "p_sym": np.array([1 if sym else 0], dtype=np.int64)})
        if p.graph is w.global_graph:           # the halo is the whole graph: keep one copy
            a.pop("p_rp"), a.pop("p_ci")
            a["p_same"] = np.array([1], dtype=np.int64)
        if not sym:
            a.update({"pt_rp": p.graph_t.row_ptr, "pt_ci": p.graph_t.col_idx})
    tmp = path + ".tmp.npz"
    np.savez(tmp, **a)
    import os
    os.replace(tmp, path)


def _load_workload(path: str, name: str, model: str, dtype: str) -> Workload:
    z = np.load(path, allow_pickle=False)
    n_layers, fanout, seed, sample_seed, has_part = (int(x) for x in z["meta"])
    g = CSR(int(z["g_shape"][0]), int(z["g_shape"][1]), z["g_rp"], z["g_ci"])
    part = None
    if has_part:
        if "p_same" in z.files:
            lg = g
        else:
            n_loc = z["p_l2g"].shape[0]
            lg = CSR(n_loc, n_loc, z["p_rp"], z["p_ci"])
        lt = lg if int(z["p_sym"][0]) else CSR(lg.n_rows, lg.n_cols, z["pt_rp"], z["pt_ci"])
        part = Partition(lg, lt, z["p_l2g"], z["p_t"], z["p_deg"])
    return Workload(name, model, dtype, [int(d) for d in z["dims"]], n_layers, part, g, z["tg"], fanout=fanout, seed=seed,
                    sample_seed=sample_seed)


_MODEL_OF = {"cfg0": ("gcn", "f32"), "cfg1": ("sage", "f32"), "cfg2": ("gcn", "f32"), "cfg3": ("sage", "bf16"), "cfg4": ("sage", "bf16")}


def make_workload(name: str, scale: float = 1.0, seed: int | None = None) -> Workload:
    """Build the named workload; ``scale`` < 1 shrinks the vertex count (tests).

    For cfg4 only the global graph and the target list are made here: the
    local partition depends on the method's boundary sampling.

    With the environment variable GRAPHGEN_CACHE naming a directory, the
    arrays of a workload are kept there after the first build and read back
    on later calls (the generators are deterministic, so this only saves time).
    """
    import os
    path = _cache_path(name, scale, seed)
    if path and os.path.exists(path):
        return _load_workload(path, name, *_MODEL_OF[name])
    w = _make_workload(name, scale, seed)
    if path:
        _save_workload(path, w)
    return w


def _make_workload(name: str, scale: float = 1.0, seed: int | None = None) -> Workload:
    if name == "cfg0":
        s = 0 if seed is None else seed
        n = max(50, int(10_000 * scale))
        g = add_self_loops(erdos_renyi(n, 10, s))
        tg = np.arange(max(1, n // 5), dtype=np.int64)
        part = halo_partition(g, tg, 2)
        return Workload(name, "gcn", "f32", [64, 64, 8], 2, part, g, tg, seed=s)
    if name == "cfg1":
        s = 1 if seed is None else seed
        n = max(64, int(233_000 * scale))
        avg = min(490.0, max(4.0, (n - 1) / 3))
        g = chung_lu(n, avg, 2.1, s)
        rng = np.random.default_rng([s, 0x544752])
        tg = np.sort(rng.choice(n, size=max(1, n // 8), replace=False)).astype(np.int64)
        part = halo_partition(g, tg, 3)
        return Workload(name, "sage", "f32", [602, 256, 256, 41], 3, part, g, tg, seed=s)
    if name == "cfg2":
        s = 2 if seed is None else seed
        n = max(64, int(2_450_000 * scale))
        g = add_self_loops(chung_lu(n, min(50.0, (n - 1) / 3), 2.1, s))
        pid = bfs_partition(g, 8, s)
        tg = np.flatnonzero(pid == 0).astype(np.int64)
        part = halo_partition(g, tg, 3)
        return Workload(name, "gcn", "f32", [100, 256, 256, 47], 3, part, g, tg, seed=s)
    if name == "cfg3":
        s = 3 if seed is None else seed
        n = max(64, int(1_000_000 * scale))
        g = chung_lu(n, min(20.0, (n - 1) / 3), 2.1, s)
        pid = bfs_partition(g, 16, s)
        tg = np.flatnonzero(pid == 0).astype(np.int64)
        part = halo_partition(g, tg, 8)
        return Workload(name, "sage", "bf16", [128] * 8 + [16], 8, part, g, tg, seed=s)
    if name == "cfg4":
        s = 4 if seed is None else seed
        n = max(64, int(10_000_000 * scale))
        g = chung_lu(n, min(15.0, (n - 1) / 3), 2.1, s)
        pid = bfs_partition(g, 8, s)
        tg = np.flatnonzero(pid == 0).astype(np.int64)
        return Workload(name, "sage", "bf16", [128, 256, 256, 32], 3, None, g, tg, fanout=5, seed=s,
                        sample_seed=0x5EED0000 + s)
    raise KeyError(name)
