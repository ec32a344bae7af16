"""CPU oracle (test infrastructure only) - ctypes binding of ``gnn_oracle.c`` plus
the model-level forward/backward written as the paper's definitions.

Nothing in the product package imports this.  Only ``tests/``, the smoke check
and the CPU-baseline leg of ``bench.py`` do.  All arithmetic is float64; the
bf16 variants round *stored* tensors to bfloat16 and keep accumulating in
float64.

Sections followed: 2.1 (layer equation), 5.3 (expansion-aware sampling),
6 (one-hop graph masking, figure 7c).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gnn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_mix64.restype = C.c_uint64
        _lib.orc_mix64.argtypes = [C.c_uint64]
        _lib.orc_edge_key.restype = C.c_uint64
        _lib.orc_edge_key.argtypes = [C.c_uint64] * 4
        _lib.orc_softmax_ce.restype = C.c_double
        _lib.orc_sample_boundary.restype = C.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def n_threads() -> int:
    """Threads the OpenMP loops of the oracle use (OMP_NUM_THREADS or all cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    return int(v) if v else (os.cpu_count() or 1)


# ------------------------------------------------------------------ steps
def mix64(x: int) -> int:
    return int(lib().orc_mix64(C.c_uint64(x & (2**64 - 1))))


def edge_key(seed: int, v: int, u: int, hop: int) -> int:
    return int(lib().orc_edge_key(C.c_uint64(seed), C.c_uint64(v), C.c_uint64(u), C.c_uint64(hop)))


def active_sets(row_ptr, col_idx, targets, L):
    """-> dist int32[n], ring_ids int32[n_reached], hop_offsets int64[L+2]."""
    row_ptr, col_idx, targets = _i32(row_ptr), _i32(col_idx), _i32(targets)
    n = row_ptr.shape[0] - 1
    dist = np.empty(n, dtype=np.int32)
    ring = np.empty(n, dtype=np.int32)
    off = np.empty(L + 2, dtype=np.int64)
    rc = lib().orc_active_sets(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(targets), C.c_int32(targets.shape[0]),
                               C.c_int32(L), _p(dist), _p(ring), _p(off))
    if rc != 0:
        raise ValueError("target id out of range")
    return dist, ring[: off[-1]].copy(), off


def norm_scales(mode: str, length) -> np.ndarray:
    length = _i32(length)
    out = np.empty(length.shape[0], dtype=np.float64)
    lib().orc_norm_scales(C.c_int32({"mean": 1, "sym": 2}[mode]), _p(length), C.c_int32(length.shape[0]), _p(out))
    return out


def spmm_fwd(row_ptr, col_idx, rows, X, Y, F, rs=None, cs=None):
    """In place on Y (float64 2-D, C-contiguous); rows None -> all rows of the CSR."""
    row_ptr, col_idx, rows = _i32(row_ptr), _i32(col_idx), _i32(rows)
    assert X.dtype == np.float64 and Y.dtype == np.float64 and X.flags.c_contiguous and Y.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else row_ptr.shape[0] - 1
    rs, cs = _f64(rs), _f64(cs)
    lib().orc_spmm_fwd(_p(row_ptr), _p(col_idx), _p(rows), C.c_int32(n_active), _p(X), C.c_int64(X.shape[1]),
                       _p(Y), C.c_int64(Y.shape[1]), C.c_int32(F), _p(rs), _p(cs))
    return Y


def spmm_bwd(row_ptr, col_idx, rows, dY, dX, F, rs=None, cs=None):
    """Adjoint of spmm_fwd over the same CSR and row list; accumulates into dX."""
    row_ptr, col_idx, rows = _i32(row_ptr), _i32(col_idx), _i32(rows)
    assert dY.dtype == np.float64 and dX.dtype == np.float64 and dY.flags.c_contiguous and dX.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else row_ptr.shape[0] - 1
    rs, cs = _f64(rs), _f64(cs)
    lib().orc_spmm_bwd(_p(row_ptr), _p(col_idx), _p(rows), C.c_int32(n_active), _p(dY), C.c_int64(dY.shape[1]),
                       _p(dX), C.c_int64(dX.shape[1]), C.c_int32(F), _p(rs), _p(cs))
    return dX


def linear_fwd(rows, A, X_self, K, W_neigh, W_self, bias, H, relu):
    rows = _i32(rows)
    n_active = rows.shape[0] if rows is not None else A.shape[0]
    W_neigh, W_self, bias = _f64(W_neigh), _f64(W_self), _f64(bias)
    N = W_neigh.shape[1]
    assert A.dtype == np.float64 and A.flags.c_contiguous and H.dtype == np.float64 and H.flags.c_contiguous
    if X_self is not None:
        assert X_self.dtype == np.float64 and X_self.flags.c_contiguous and X_self.shape[1] == A.shape[1]
    lib().orc_linear_fwd(_p(rows), C.c_int32(n_active), _p(A), _p(X_self), C.c_int64(A.shape[1]), C.c_int32(K),
                         _p(W_neigh), _p(W_self), _p(bias), C.c_int32(N), _p(H), C.c_int64(H.shape[1]),
                         C.c_int32(1 if relu else 0))
    return H


def linear_bwd(rows, dH, H, relu, A, X_self, K, W_neigh, W_self, dA=None, dX_self=None):
    """-> dW_neigh, dW_self (or None), dbias; writes rows of dA / dX_self if given."""
    rows = _i32(rows)
    n_active = rows.shape[0] if rows is not None else A.shape[0]
    W_neigh, W_self = _f64(W_neigh), _f64(W_self)
    N = W_neigh.shape[1]
    dWn = np.zeros((K, N))
    dWs = np.zeros((K, N)) if W_self is not None else None
    db = np.zeros(N)
    ld_din = dA.shape[1] if dA is not None else (dX_self.shape[1] if dX_self is not None else 0)
    for t in (dH, A) + ((H,) if H is not None else ()) + ((dA,) if dA is not None else ()) + \
            ((dX_self,) if dX_self is not None else ()) + ((X_self,) if X_self is not None else ()):
        assert t.dtype == np.float64 and t.flags.c_contiguous
    lib().orc_linear_bwd(_p(rows), C.c_int32(n_active), _p(dH), C.c_int64(dH.shape[1]),
                         _p(H), C.c_int64(H.shape[1] if H is not None else 0), C.c_int32(1 if relu else 0),
                         _p(A), _p(X_self), C.c_int64(A.shape[1]), C.c_int32(K), _p(W_neigh), _p(W_self), C.c_int32(N),
                         _p(dWn), _p(dWs), _p(db), _p(dA), _p(dX_self), C.c_int64(ld_din))
    return dWn, dWs, db


def softmax_ce(rows, Z, n_classes, labels, dZ=None) -> float:
    rows, labels = _i32(rows), _i32(labels)
    assert Z.dtype == np.float64 and Z.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else Z.shape[0]
    assert labels.shape[0] == n_active
    return float(lib().orc_softmax_ce(_p(rows), C.c_int32(n_active), _p(Z), C.c_int64(Z.shape[1]),
                                      C.c_int32(n_classes), _p(labels), _p(dZ),
                                      C.c_int64(dZ.shape[1] if dZ is not None else 0)))


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round a float64 array (in place) to the nearest bfloat16 values."""
    assert x.dtype == np.float64 and x.flags.c_contiguous
    lib().orc_round_bf16(_p(x), C.c_int64(x.size))
    return x


def sample_boundary(row_ptr, col_idx, is_target, targets, fanout, seed):
    """-> (out_row_ptr int32[n_targets+1], out_col_idx int32[kept]) in global ids."""
    row_ptr, col_idx, targets = _i32(row_ptr), _i32(col_idx), _i32(targets)
    is_target = np.ascontiguousarray(is_target, dtype=np.uint8)
    n = row_ptr.shape[0] - 1
    orp = np.empty(targets.shape[0] + 1, dtype=np.int32)
    args = [C.c_int32(n), _p(row_ptr), _p(col_idx), _p(is_target), _p(targets), C.c_int32(targets.shape[0]),
            C.c_int32(fanout), C.c_uint64(seed), _p(orp)]
    kept = lib().orc_sample_boundary(*args, None)
    if kept < 0:
        raise ValueError("bad argument")
    oci = np.empty(kept, dtype=np.int32)
    lib().orc_sample_boundary(*args, _p(oci))
    return orp, oci


def sampled_local_edges(targets, out_row_ptr, out_col_idx):
    """Section 5.3.1, last step: the sub-graph of the traversed vertices.

    Local vertices = targets + every kept outside neighbour; edges = the kept
    rows of the targets plus the reverse (u, v) of every kept outside edge, so
    that the local one-hop graph stays symmetric.  Returns
    (local_to_global ascending, edge rows, edge cols) in global ids.
    """
    targets = np.asarray(targets, dtype=np.int64)
    rows = np.repeat(targets, np.diff(out_row_ptr).astype(np.int64))
    cols = out_col_idx.astype(np.int64)
    is_t = np.zeros(max(int(targets.max(initial=0)), int(cols.max(initial=0))) + 1, dtype=bool)
    is_t[targets] = True
    ext = ~is_t[cols]
    l2g = np.union1d(targets, cols)
    er = np.concatenate([rows, cols[ext]])
    ec = np.concatenate([cols, rows[ext]])
    return l2g, er, ec


def eas_traverse(row_ptr, col_idx, targets, hops, fanout, rule, seed=0):
    """Section 5.3.1 traversal.  rule: "degree" (the paper's: best-connected candidates first) or
    "hash" (seeded).  -> dist int32[n] (hop of selection or -1), ring_ids, hop_offsets int64[hops+2]."""
    row_ptr, col_idx, targets = _i32(row_ptr), _i32(col_idx), _i32(targets)
    n = row_ptr.shape[0] - 1
    dist = np.empty(n, dtype=np.int32)
    ring = np.empty(max(n, 1), dtype=np.int32)
    off = np.empty(hops + 2, dtype=np.int64)
    rc = lib().orc_eas_traverse(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(targets), C.c_int32(targets.shape[0]), C.c_int32(hops),
                                C.c_int32(fanout), C.c_int32({"hash": 0, "degree": 1}[rule]), C.c_uint64(seed & (2**64 - 1)),
                                _p(dist), _p(ring), _p(off))
    if rc != 0:
        raise ValueError("bad argument")
    return dist, ring[: off[-1]].copy(), off


def keep_threshold(p: float) -> int:
    """The 64-bit threshold that keeps an edge with probability p under the rule key <= threshold (p = 1: all ones)."""
    assert 0.0 < p <= 1.0
    return min((1 << 64) - 1, int(p * (1 << 64)) - 1) if p < 1.0 else (1 << 64) - 1


def layer_edge_mask(row_ptr, col_idx, rows, rule, layer, seed=0, fanout=0, threshold=(1 << 64) - 1):
    """Section 5.2: the mask of one layer over the one-hop graph.  rule "threshold" (every edge on its own, kept
    iff its key <= threshold) or "fanout" (a row keeps its `fanout` entries with the smallest (key, id)).
    -> keep uint8[nnz] (0 outside the listed rows), kept_len int32[n] (0 outside the listed rows)."""
    row_ptr, col_idx, rows = _i32(row_ptr), _i32(col_idx), _i32(rows)
    n = row_ptr.shape[0] - 1
    n_active = rows.shape[0] if rows is not None else n
    keep = np.zeros(max(col_idx.shape[0], 1), dtype=np.uint8)
    kept_len = np.zeros(n, dtype=np.int32)
    rc = lib().orc_layer_edge_mask(_p(row_ptr), _p(col_idx), _p(rows), C.c_int32(n_active), C.c_int32({"threshold": 0, "fanout": 1}[rule]),
                                   C.c_int32(fanout), C.c_uint64(threshold), C.c_uint64(seed & (2**64 - 1)), C.c_int32(layer),
                                   _p(keep), _p(kept_len))
    if rc != 0:
        raise ValueError("bad argument")
    return keep[: col_idx.shape[0]], kept_len


def transpose_mask(row_ptr, col_idx, keep, rpT, ciT):
    """keep (positions of the graph) -> the same mask in the positions of the transposed graph."""
    row_ptr, col_idx, rpT, ciT = _i32(row_ptr), _i32(col_idx), _i32(rpT), _i32(ciT)
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    out = np.zeros(max(ciT.shape[0], 1), dtype=np.uint8)
    lib().orc_transpose_mask(_p(row_ptr), _p(col_idx), _p(keep), C.c_int32(rpT.shape[0] - 1), _p(rpT), _p(ciT), _p(out))
    return out[: ciT.shape[0]]


def spmm_fwd_em(row_ptr, col_idx, keep, rows, X, Y, F, rs=None, cs=None):
    """spmm_fwd through a layer's edge mask (keep uint8[nnz])."""
    row_ptr, col_idx, rows = _i32(row_ptr), _i32(col_idx), _i32(rows)
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    assert X.dtype == np.float64 and Y.dtype == np.float64 and X.flags.c_contiguous and Y.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else row_ptr.shape[0] - 1
    rs, cs = _f64(rs), _f64(cs)
    lib().orc_spmm_fwd_em(_p(row_ptr), _p(col_idx), _p(keep), _p(rows), C.c_int32(n_active), _p(X), C.c_int64(X.shape[1]),
                          _p(Y), C.c_int64(Y.shape[1]), C.c_int32(F), _p(rs), _p(cs))
    return Y


def spmm_bwd_em(row_ptr, col_idx, keep, rows, dY, dX, F, rs=None, cs=None):
    """Adjoint of spmm_fwd_em; accumulates into dX."""
    row_ptr, col_idx, rows = _i32(row_ptr), _i32(col_idx), _i32(rows)
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    assert dY.dtype == np.float64 and dX.dtype == np.float64 and dY.flags.c_contiguous and dX.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else row_ptr.shape[0] - 1
    rs, cs = _f64(rs), _f64(cs)
    lib().orc_spmm_bwd_em(_p(row_ptr), _p(col_idx), _p(keep), _p(rows), C.c_int32(n_active), _p(dY), C.c_int64(dY.shape[1]),
                          _p(dX), C.c_int64(dX.shape[1]), C.c_int32(F), _p(rs), _p(cs))
    return dX


def extract_from_ring(row_ptr, col_idx, ring):
    """The sub-graph induced by the listed vertices, renumbered in list order (section 5.3.1: a sub-graph is
    generated from the traversed vertices).  -> (local_row_ptr, local_col_idx)."""
    row_ptr, col_idx, ring = _i32(row_ptr), _i32(col_idx), _i32(ring)
    n = row_ptr.shape[0] - 1
    n_local = ring.shape[0]
    new_id = np.empty(max(n, 1), dtype=np.int32)
    rp = np.empty(n_local + 1, dtype=np.int32)
    f = lib().orc_extract_partition
    f.restype = C.c_int64
    nnz = f(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(ring), C.c_int32(n_local), _p(new_id), _p(rp), None)
    ci = np.empty(max(int(nnz), 1), dtype=np.int32)
    f(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(ring), C.c_int32(n_local), _p(new_id), _p(rp), _p(ci))
    return rp, ci[: int(nnz)]


def extract_partition(row_ptr, col_idx, targets, L):
    """Section 6 step 1: the one-hop graph of everything within L hops of the targets, vertices renumbered by
    (distance, id).  -> (local_row_ptr, local_col_idx, local_to_global, hop_offsets, dist_local);
    layer l's rows are the local ids 0 .. hop_offsets[L-l+1]-1."""
    _, ring, off = active_sets(row_ptr, col_idx, targets, L)
    rp, ci = extract_from_ring(row_ptr, col_idx, ring)
    dist_local = np.repeat(np.arange(L + 1, dtype=np.int32), np.diff(off).astype(np.int64))
    return rp, ci, ring, off, dist_local


def extract_sampled(n, targets, s_row_ptr, s_col_idx):
    """Section 5.3.1: the one-hop graph of the targets and the outside vertices they kept, renumbered by
    (distance, id).  targets ascending.  -> (local_row_ptr, local_col_idx, local_to_global, hop_offsets, dist_local)."""
    targets, s_row_ptr, s_col_idx = _i32(targets), _i32(s_row_ptr), _i32(s_col_idx)
    nt = targets.shape[0]
    new_id = np.empty(n, dtype=np.int32)
    l2g = np.empty(max(n, 1), dtype=np.int32)
    rp = np.empty(n + 1, dtype=np.int32)
    n_local = C.c_int32(0)
    f = lib().orc_extract_sampled
    f.restype = C.c_int64
    args = [C.c_int32(n), _p(targets), C.c_int32(nt), _p(s_row_ptr), _p(s_col_idx), _p(new_id), _p(l2g), C.byref(n_local), _p(rp)]
    nnz = f(*args, None)
    if nnz < 0:
        raise ValueError("targets must be ascending, without repeats, inside [0, n)")
    ci = np.empty(max(int(nnz), 1), dtype=np.int32)
    f(*args, _p(ci))
    nl = int(n_local.value)
    off = np.array([0, nt, nl], dtype=np.int64)
    dist_local = np.repeat(np.arange(2, dtype=np.int32), np.diff(off))
    return rp[: nl + 1].copy(), ci[: int(nnz)], l2g[:nl].copy(), off, dist_local


def _row_entries(row_ptr, col_idx, rows):
    """All column entries of the listed rows, concatenated."""
    start = row_ptr[rows].astype(np.int64)
    cnt = (row_ptr[rows + 1] - row_ptr[rows]).astype(np.int64)
    tot = int(cnt.sum())
    if tot == 0:
        return np.zeros(0, dtype=np.int32)
    shift = np.repeat(start - (np.cumsum(cnt) - cnt), cnt)
    return col_idx[shift + np.arange(tot, dtype=np.int64)]


# ------------------------------------------------------------- the model
class Model:
    """L-layer GCN or GraphSAGE-mean over one partition under one-hop masking.

    graph        (row_ptr, col_idx) of the one-hop graph, reused by every layer
    targets      local ids of the inner vertices
    kind         "gcn": Z = (rs * G (cs * H)) W + b with rs = cs = deg^-1/2
                 "sage": Z = H W_self + mean_G(H) W_neigh + b
    params       list of dicts W_neigh [K,N], W_self (sage), bias [N]
    bf16         round every stored tensor (inputs, A_l, H_l, W, and the
                 gradients dZ, dA, dH) to bfloat16
    all_rows     compute every row at every layer (the unmasked variant)
    layer_sampling  None, or (rule, parameter, seed): layer-wise sampling as per-layer masking (section 5.2) -
                 ("threshold", t, seed) or ("fanout", f, seed); layer l aggregates through layer_edge_mask(..., layer=l)
                 over its rows R_l, and the mean is taken over the kept neighbours
    """

    def __init__(self, row_ptr, col_idx, targets, kind, params, global_degree=None, bf16=False, all_rows=False,
                 layer_sampling=None):
        self.row_ptr, self.col_idx = _i32(row_ptr), _i32(col_idx)
        self.n = self.row_ptr.shape[0] - 1
        self.targets = _i32(targets)
        self.kind = kind
        self.L = len(params)
        self.bf16 = bf16
        self.params = []
        for p in params:
            q = {k: np.array(v, dtype=np.float64) for k, v in p.items()}
            if bf16:
                for k in ("W_neigh", "W_self"):
                    if k in q:
                        round_bf16(q[k])
            self.params.append(q)
        self.dist, self.ring_ids, self.hop_offsets = active_sets(self.row_ptr, self.col_idx, self.targets, self.L)
        length = np.diff(self.row_ptr)
        if kind == "gcn":
            s = norm_scales("sym", global_degree if global_degree is not None else length)
            self.rs, self.cs = s, s
        else:
            self.rs, self.cs = norm_scales("mean", length), None
        self.all_rows = all_rows
        self.keep, self.rs_l = None, None
        if layer_sampling is not None:
            rule, par, seed = layer_sampling
            self.keep, self.rs_l = [None], [None]
            for l in range(1, self.L + 1):
                keep, kept_len = layer_edge_mask(self.row_ptr, self.col_idx, self.rows_of_layer(l), rule, l, seed,
                                                 fanout=par if rule == "fanout" else 0,
                                                 threshold=par if rule == "threshold" else (1 << 64) - 1)
                self.keep.append(keep)
                self.rs_l.append(self.rs if kind == "gcn" else norm_scales("mean", kept_len))

    def rows_of_layer(self, l: int) -> np.ndarray:
        """R_l = {dist <= L - l} as ring-sorted ids (l = 0 is the input set)."""
        if self.all_rows:
            return np.arange(self.n, dtype=np.int32)
        return self.ring_ids[: self.hop_offsets[self.L - l + 1]]

    def _store(self, x):
        return round_bf16(x) if self.bf16 else x

    def forward(self, H0, labels):
        """labels[i] belongs to targets[i].  Returns loss; keeps A_l, H_l for backward."""
        H = self._store(np.array(H0, dtype=np.float64, order="C"))
        self.H = [H]
        self.A = [None]
        for l in range(1, self.L + 1):
            p = self.params[l - 1]
            K, N = p["W_neigh"].shape
            rows = self.rows_of_layer(l)
            if not self.all_rows:
                # every row read by layer l was produced by layer l-1 (or is an input row)
                need = _row_entries(self.row_ptr, self.col_idx, rows)
                assert (self.dist[need] >= 0).all() and (self.dist[need] <= self.L - l + 1).all()
            A = np.full((self.n, K), np.nan)
            assert self.H[l - 1].shape[1] == K
            if self.keep is None:
                spmm_fwd(self.row_ptr, self.col_idx, rows, self.H[l - 1], A, K, self.rs, self.cs)
            else:
                spmm_fwd_em(self.row_ptr, self.col_idx, self.keep[l], rows, self.H[l - 1], A, K, self.rs_l[l], self.cs)
            self._store(A)
            Hn = np.full((self.n, N), np.nan)
            Xs = self.H[l - 1] if self.kind == "sage" else None
            linear_fwd(rows, A, Xs, K, p["W_neigh"], p.get("W_self"), p["bias"], Hn, relu=(l < self.L))
            self._store(Hn)
            self.A.append(A)
            self.H.append(Hn)
        self.labels = _i32(labels)
        C_ = self.params[-1]["W_neigh"].shape[1]
        self.dlogits = np.zeros((self.n, C_))
        self.loss = softmax_ce(self.targets, self.H[-1], C_, self.labels, self.dlogits)
        return self.loss

    def backward(self):
        """Returns list of dicts dW_neigh, dW_self, dbias (layer 1 first)."""
        grads = [None] * self.L
        dH = self._store(self.dlogits.copy())
        for l in range(self.L, 0, -1):
            p = self.params[l - 1]
            K, N = p["W_neigh"].shape
            rows = self.rows_of_layer(l)
            relu = l < self.L
            need_in = l > 1
            dA = np.zeros((self.n, K)) if need_in else None
            dXs = np.zeros((self.n, K)) if (need_in and self.kind == "sage") else None
            Xs = self.H[l - 1] if self.kind == "sage" else None
            dWn, dWs, db = linear_bwd(rows, dH, self.H[l] if relu else None, relu, self.A[l], Xs, K,
                                      p["W_neigh"], p.get("W_self"), dA, dXs)
            g = {"dW_neigh": dWn, "dbias": db}
            if dWs is not None:
                g["dW_self"] = dWs
            grads[l - 1] = g
            if need_in:
                self._store(dA)
                dprev = dXs if dXs is not None else np.zeros((self.n, K))
                if self.keep is None:
                    spmm_bwd(self.row_ptr, self.col_idx, rows, dA, dprev, K, self.rs, self.cs)
                else:
                    spmm_bwd_em(self.row_ptr, self.col_idx, self.keep[l], rows, dA, dprev, K, self.rs_l[l], self.cs)
                dH = self._store(dprev)
        return grads


LN_EPS = 1e-5


def ln_relu_fwd(rows, X, F, gamma, beta, Y, eps=LN_EPS):
    """Y[rows] = ReLU(LayerNorm(X[rows])) over the first F columns; in place on Y."""
    rows = _i32(rows)
    gamma, beta = _f64(gamma), _f64(beta)
    assert X.dtype == np.float64 and Y.dtype == np.float64 and X.flags.c_contiguous and Y.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else X.shape[0]
    lib().orc_ln_relu_fwd(_p(rows), C.c_int32(n_active), _p(X), C.c_int64(X.shape[1]), C.c_int32(F), _p(gamma), _p(beta),
                          C.c_double(eps), _p(Y), C.c_int64(Y.shape[1]))
    return Y


def ln_relu_bwd(rows, dY, T, X, F, gamma, dX, eps=LN_EPS):
    """-> (dgamma, dbeta); dX[rows] is overwritten.  T = the stored forward output (ReLU mask)."""
    rows = _i32(rows)
    gamma = _f64(gamma)
    for a in (dY, T, X, dX):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    n_active = rows.shape[0] if rows is not None else X.shape[0]
    dg, db = np.zeros(F), np.zeros(F)
    lib().orc_ln_relu_bwd(_p(rows), C.c_int32(n_active), _p(dY), C.c_int64(dY.shape[1]), _p(T), C.c_int64(T.shape[1]),
                          _p(X), C.c_int64(X.shape[1]), C.c_int32(F), _p(gamma), C.c_double(eps), _p(dX), C.c_int64(dX.shape[1]),
                          _p(dg), _p(db))
    return dg, db


class ResModel:
    """The deep residual GraphSAGE the paper calls ResSAGE+ (section 8.1; residual connections and pre-activation):
        h_1 = SAGE_1(h_0)
        h_l = h_{l-1} + SAGE_l(ReLU(LN_l(h_{l-1})))      1 < l < L     (all hidden widths equal)
        out = SAGE_L(ReLU(LN_L(h_{L-1})))
    with SAGE_l(t)[v] = t[v] W_self + mean_{u in row(v)} t[u] W_neigh + b, under one-hop masking: layer l produces the
    rows R_l, its pre-activation runs over R_{l-1}.  params[l-1]: W_neigh, W_self, bias and, for l > 1, ln_gamma, ln_beta.
    bf16: every stored tensor is rounded (h_0, t_l, A_l, the layer's transform before the residual is added, h_l, W,
    and the gradients)."""

    def __init__(self, row_ptr, col_idx, targets, params, bf16=False, all_rows=False):
        self.row_ptr, self.col_idx = _i32(row_ptr), _i32(col_idx)
        self.n = self.row_ptr.shape[0] - 1
        self.targets = _i32(targets)
        self.L = len(params)
        self.bf16 = bf16
        self.params = []
        for p in params:
            q = {k: np.array(v, dtype=np.float64) for k, v in p.items()}
            if bf16:
                round_bf16(q["W_neigh"]), round_bf16(q["W_self"])
            self.params.append(q)
        self.dist, self.ring_ids, self.hop_offsets = active_sets(self.row_ptr, self.col_idx, self.targets, self.L)
        self.rs = norm_scales("mean", np.diff(self.row_ptr))
        self.all_rows = all_rows

    def rows_of_layer(self, l):
        if self.all_rows:
            return np.arange(self.n, dtype=np.int32)
        return self.ring_ids[: self.hop_offsets[self.L - l + 1]]

    def _store(self, x):
        return round_bf16(x) if self.bf16 else x

    def forward(self, H0, labels):
        self.H = [self._store(np.array(H0, dtype=np.float64, order="C"))]
        self.T, self.A = [None, None], [None]
        for l in range(1, self.L + 1):
            p = self.params[l - 1]
            K, N = p["W_neigh"].shape
            rows = self.rows_of_layer(l)
            if l == 1:
                src = self.H[0]
            else:
                src = np.full((self.n, K), np.nan)
                ln_relu_fwd(self.rows_of_layer(l - 1), self.H[l - 1], K, p["ln_gamma"], p["ln_beta"], src)
                self._store(src)
                self.T.append(src)
            A = np.full((self.n, K), np.nan)
            spmm_fwd(self.row_ptr, self.col_idx, rows, src, A, K, self.rs, None)
            self._store(A)
            Z = np.full((self.n, N), np.nan)
            linear_fwd(rows, A, src, K, p["W_neigh"], p["W_self"], p["bias"], Z, relu=False)
            self._store(Z)
            if 1 < l < self.L:
                Z[rows] = Z[rows] + self.H[l - 1][rows]
                self._store(Z)
            self.A.append(A)
            self.H.append(Z)
        self.labels = _i32(labels)
        C_ = self.params[-1]["W_neigh"].shape[1]
        self.dlogits = np.zeros((self.n, C_))
        self.loss = softmax_ce(self.targets, self.H[-1], C_, self.labels, self.dlogits)
        return self.loss

    def backward(self):
        grads = [None] * self.L
        dH = self._store(self.dlogits.copy())
        for l in range(self.L, 0, -1):
            p = self.params[l - 1]
            K, N = p["W_neigh"].shape
            rows = self.rows_of_layer(l)
            need_in = l > 1
            src = self.H[0] if l == 1 else self.T[l]
            dA = np.zeros((self.n, K)) if need_in else None
            dT = np.zeros((self.n, K)) if need_in else None
            dWn, dWs, db = linear_bwd(rows, dH, None, False, self.A[l], src, K, p["W_neigh"], p["W_self"], dA, dT)
            g = {"dW_neigh": dWn, "dW_self": dWs, "dbias": db}
            if need_in:
                self._store(dA)
                self._store(dT)       # the self part is stored before the aggregated part is added to it
                spmm_bwd(self.row_ptr, self.col_idx, rows, dA, dT, K, self.rs, None)
                self._store(dT)
                rows_prev = self.rows_of_layer(l - 1)
                dprev = np.zeros((self.n, K))
                g["dln_gamma"], g["dln_beta"] = ln_relu_bwd(rows_prev, dT, self.T[l], self.H[l - 1], K, p["ln_gamma"], dprev)
                if l < self.L:
                    dprev[rows] += dH[rows]          # the residual connection
                dH = self._store(dprev)
            grads[l - 1] = g
        return grads
