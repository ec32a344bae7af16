"""ctypes binding of libgnnhot.so: the same entry points as include/gnnhot.h, taking torch
tensors.  Argument marshalling and host-side shape checks only - every step of the path runs
in the HIP kernels behind the C ABI.  torch supplies device memory and the current stream.

There is no CPU fallback: importing works without a GPU (so that the symbols can be
inspected), but every call needs the built library and CUDA/HIP tensors.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgnnhot.so")

GNN_F32, GNN_BF16 = 0, 1
GNN_NORM_MEAN, GNN_NORM_SYM = 1, 2
GNN_CSR_SORTED_COLUMNS = 1
STATUS = {0: "GNN_OK", 1: "GNN_ERR_INVALID_ARG", 2: "GNN_ERR_SHAPE", 3: "GNN_ERR_WORKSPACE",
          4: "GNN_ERR_UNSUPPORTED", 5: "GNN_ERR_HIP"}

EXPORTS = ["gnn_version", "gnn_last_error", "gnn_build_active_sets", "gnn_norm_scales", "gnn_masked_spmm_fwd", "gnn_masked_spmm_fwd_add",
           "gnn_masked_spmm_bwd", "gnn_linear_fwd", "gnn_linear_bwd", "gnn_softmax_ce", "gnn_make_bitmap",
           "gnn_sample_boundary", "gnn_extract_partition", "gnn_gather_rows", "gnn_expand_row_ptr",
           "gnn_extract_sampled_partition", "gnn_eas_traverse", "gnn_layer_edge_mask", "gnn_transpose_edge_mask",
           "gnn_layer_edge_mask_transposed", "gnn_layer_norm_relu_fwd", "gnn_layer_norm_relu_bwd", "gnn_add_rows", "gnn_add_rows_masked", "gnn_bias_grad", "gnn_linear_bwd_input",
           "gnn_linear_fwd_static", "gnn_linear_bwd_input2", "gnn_die_mapping", "gnn_fused_layer_fwd"]


class GnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


class gnn_csr(C.Structure):
    _fields_ = [("n_rows", C.c_int32), ("n_cols", C.c_int32), ("nnz", C.c_int64),
                ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("flags", C.c_int32), ("edge_keep", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2311_06837_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with paper_2311_06837_amd.build.build_library(); "
                               "there is no fallback path")
        _lib = C.CDLL(LIB_PATH)
        _lib.gnn_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("gnn_last_error",):
                getattr(_lib, name).restype = C.c_int32
    return _lib


def _check(status: int):
    if status != 0:
        raise GnnError(status, lib().gnn_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    assert isinstance(t, torch.Tensor) and t.is_cuda, "device tensor expected"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GNN_F32
    if t.dtype == torch.bfloat16:
        return GNN_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _i32(t, name):
    assert t is None or (t.dtype == torch.int32 and t.is_contiguous()), f"{name}: contiguous int32 expected"
    return t


def _mat(t, name):
    assert t.dim() == 2 and t.stride(1) == 1, f"{name}: row-major 2-D tensor expected"
    return t


class Graph:
    """Device CSR (int32) of a one-hop graph plus the host struct handed to the C ABI."""

    def __init__(self, row_ptr: torch.Tensor, col_idx: torch.Tensor, n_cols: int | None = None, sorted_columns: bool = False,
                 edge_keep: torch.Tensor | None = None):
        """sorted_columns: the caller's promise that every row lists its columns in ascending order.
        edge_keep: optional int32 device tensor, one bit per entry of col_idx: the aggregation calls skip the
        entries whose bit is 0 (per-layer mask of layer-wise sampling)."""
        _i32(row_ptr, "row_ptr"), _i32(col_idx, "col_idx")
        assert row_ptr.is_cuda and col_idx.is_cuda
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.n_rows = row_ptr.numel() - 1
        self.n_cols = self.n_rows if n_cols is None else n_cols
        self.nnz = col_idx.numel()
        self.sorted_columns = bool(sorted_columns)
        self.edge_keep = edge_keep
        if edge_keep is not None:
            assert edge_keep.is_cuda and edge_keep.dtype == torch.int32 and edge_keep.numel() * 32 >= self.nnz
        self.c = gnn_csr(self.n_rows, self.n_cols, self.nnz, row_ptr.data_ptr(), col_idx.data_ptr() if self.nnz else None,
                         GNN_CSR_SORTED_COLUMNS if sorted_columns else 0,
                         edge_keep.data_ptr() if edge_keep is not None else None)

    def with_edge_keep(self, edge_keep: torch.Tensor | None) -> "Graph":
        """The same graph (arrays shared) seen through a layer's edge mask."""
        return Graph(self.row_ptr, self.col_idx, self.n_cols, self.sorted_columns, edge_keep)

    @staticmethod
    def from_numpy(row_ptr, col_idx, device="cuda", n_cols=None) -> "Graph":
        """Copies host arrays to the device; whether the rows are column-sorted is checked here, on the host."""
        import numpy as np
        ok = True
        if col_idx.size > 1:
            falls = np.flatnonzero(col_idx[1:] < col_idx[:-1]) + 1          # positions lower than their predecessor
            ok = bool(np.isin(falls, row_ptr[:-1]).all())                   # fine only where a new row starts
        return Graph(torch.from_numpy(row_ptr).to(device), torch.from_numpy(col_idx).to(device), n_cols, sorted_columns=ok)


class Workspace:
    """Grow-only scratch buffer handed to the calls that take (ws, ws_bytes)."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes: int) -> torch.Tensor:
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        return self.buf


_default_ws = Workspace()


def _with_ws(fn, args_before, args_after, ws: Workspace | None):
    """Run the (ws, ws_bytes) protocol: query the size, then call with a buffer of that size."""
    ws = ws or _default_ws
    need = C.c_size_t(0)
    _check(fn(*args_before, None, C.byref(need), *args_after))
    buf = ws.get(need.value)
    have = C.c_size_t(buf.numel())
    _check(fn(*args_before, _ptr(buf), C.byref(have), *args_after))


def gnn_version() -> int:
    return int(lib().gnn_version())


def gnn_build_active_sets(g: Graph, targets: torch.Tensor, L: int, sync: bool = True, ws: Workspace | None = None,
                          gt: Graph | None = None):
    """-> dist int32[n], ring_ids int32[n] (first hop_offsets[L+1] valid), hop_offsets int64[L+2] (device),
    and the host copy of hop_offsets as a list (None when sync is False).  gt: the transposed graph (optional)."""
    _i32(targets, "targets")
    dev = g.row_ptr.device
    dist = torch.empty(g.n_rows, dtype=torch.int32, device=dev)
    ring = torch.empty(max(g.n_rows, 1), dtype=torch.int32, device=dev)
    off = torch.empty(L + 2, dtype=torch.int64, device=dev)
    host = (C.c_int64 * (L + 2))() if sync else None
    _with_ws(lib().gnn_build_active_sets,
             (C.byref(g.c), C.byref(gt.c) if gt is not None else None, _ptr(targets) if targets.numel() else None, C.c_int32(targets.numel()), C.c_int32(L),
              _ptr(dist) if g.n_rows else None, _ptr(ring), _ptr(off), host),
             (_stream(),), ws)
    return dist, ring, off, (list(host) if sync else None)


def gnn_eas_traverse(g: Graph, targets: torch.Tensor, hops: int, fanout: int, rule: str = "degree", seed: int = 0,
                     sync: bool = True, ws: Workspace | None = None):
    """rule: "degree" (best-connected candidates first, the paper's rule) or "hash" (seeded).  Outputs as for
    gnn_build_active_sets with L = hops."""
    _i32(targets, "targets")
    dev = g.row_ptr.device
    dist = torch.empty(g.n_rows, dtype=torch.int32, device=dev)
    ring = torch.empty(max(g.n_rows, 1), dtype=torch.int32, device=dev)
    off = torch.empty(hops + 2, dtype=torch.int64, device=dev)
    host = (C.c_int64 * (hops + 2))() if sync else None
    _with_ws(lib().gnn_eas_traverse,
             (C.byref(g.c), _ptr(targets) if targets.numel() else None, C.c_int32(targets.numel()), C.c_int32(hops),
              C.c_int32(fanout), C.c_int32({"hash": 0, "degree": 1}[rule]), C.c_uint64(seed & (2 ** 64 - 1)),
              _ptr(dist) if g.n_rows else None, _ptr(ring), _ptr(off), host),
             (_stream(),), ws)
    return dist, ring, off, (list(host) if sync else None)


def gnn_layer_edge_mask(g: Graph, rows, n_active: int, rule: str, layer: int, seed: int = 0, fanout: int = 0,
                        threshold: int = (1 << 64) - 1, with_thresholds: bool = False):
    """rule "threshold" (an entry is kept iff its key <= threshold) or "fanout" (a row keeps its `fanout` entries with
    the smallest (key, id)).  -> edge_keep int32[ceil(nnz / 32)] (bit p = entry p), kept_len int32[n_rows] (0 for rows
    that are not listed) and, with_thresholds, the per-row threshold pairs (int64 keys, int32 ids)."""
    dev = g.row_ptr.device
    keep = torch.empty(max((g.nnz + 31) // 32, 1), dtype=torch.int32, device=dev)
    kept_len = torch.zeros(max(g.n_rows, 1), dtype=torch.int32, device=dev)
    thr_k = torch.empty(max(g.n_rows, 1), dtype=torch.int64, device=dev) if with_thresholds else None
    thr_u = torch.empty(max(g.n_rows, 1), dtype=torch.int32, device=dev) if with_thresholds else None
    assert rows is None or rows.numel() >= n_active
    _check(lib().gnn_layer_edge_mask(C.byref(g.c), _ptr(_i32(rows, "rows")), C.c_int32(n_active),
                                     C.c_int32({"threshold": 0, "fanout": 1}[rule]), C.c_int32(fanout), C.c_uint64(threshold),
                                     C.c_uint64(seed & (2 ** 64 - 1)), C.c_int32(layer), _ptr(keep), _ptr(kept_len),
                                     _ptr(thr_k), _ptr(thr_u), _stream()))
    if with_thresholds:
        return keep, kept_len[: g.n_rows], thr_k, thr_u
    return keep, kept_len[: g.n_rows]


def gnn_layer_edge_mask_transposed(gT: Graph, thr_k: torch.Tensor, thr_u: torch.Tensor, layer: int, seed: int = 0) -> torch.Tensor:
    """The layer's mask as a bit per entry of gT, from the threshold pairs of gnn_layer_edge_mask(with_thresholds=True)."""
    assert thr_k.dtype == torch.int64 and thr_u.dtype == torch.int32 and thr_k.numel() >= gT.n_cols and thr_u.numel() >= gT.n_cols
    keep_t = torch.empty(max((gT.nnz + 31) // 32, 1), dtype=torch.int32, device=thr_k.device)
    _check(lib().gnn_layer_edge_mask_transposed(C.byref(gT.c), _ptr(thr_k), _ptr(thr_u), C.c_uint64(seed & (2 ** 64 - 1)),
                                                C.c_int32(layer), _ptr(keep_t), _stream()))
    return keep_t


def gnn_transpose_edge_mask(g: Graph, gT: Graph, keep: torch.Tensor) -> torch.Tensor:
    """keep (bit per entry of g) -> the same mask as a bit per entry of gT."""
    assert keep.dtype == torch.int32 and keep.numel() * 32 >= g.nnz
    keep_t = torch.empty(max((gT.nnz + 31) // 32, 1), dtype=torch.int32, device=keep.device)
    _check(lib().gnn_transpose_edge_mask(C.byref(g.c), C.byref(gT.c), _ptr(keep), _ptr(keep_t), _stream()))
    return keep_t


def gnn_norm_scales(norm: int, n: int, length: torch.Tensor | None = None, row_ptr: torch.Tensor | None = None) -> torch.Tensor:
    src = length if length is not None else row_ptr
    out = torch.empty(n, dtype=torch.float32, device=src.device)
    _check(lib().gnn_norm_scales(C.c_int32(norm), _ptr(_i32(length, "len")), _ptr(_i32(row_ptr, "row_ptr")), C.c_int32(n),
                                 _ptr(out), _stream()))
    return out


def _with_optional_ws(fn, args_before, args_after, ws: Workspace | None):
    """ws None: the call runs without a workspace (ws_bytes = NULL); else the usual size query + call."""
    if ws is None:
        _check(fn(*args_before, None, None, *args_after))
    else:
        _with_ws(fn, args_before, args_after, ws)


def gnn_masked_spmm_fwd(g: Graph, rows, n_active: int, X: torch.Tensor, Y: torch.Tensor, F: int,
                        row_scale=None, col_scale=None, ws: Workspace | None = None):
    _mat(X, "X"), _mat(Y, "Y")
    assert X.dtype == Y.dtype and X.shape[0] >= g.n_cols and Y.shape[0] >= g.n_rows
    assert rows is None or rows.numel() >= n_active
    _with_optional_ws(lib().gnn_masked_spmm_fwd, (
        C.byref(g.c), _ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0)), _ptr(Y),
        C.c_int64(Y.stride(0)), C.c_int32(F), C.c_int32(_dtype_code(X)), _ptr(row_scale), _ptr(col_scale)), (_stream(),), ws)


def gnn_masked_spmm_fwd_add(g: Graph, rows, n_active: int, X: torch.Tensor, Y: torch.Tensor, F: int,
                            row_scale=None, col_scale=None, relu: bool = False, ws: Workspace | None = None, bias=None):
    """Y[rows] = act(Y[rows] + aggregation of X): the transform-before-aggregate order of a layer.  bias (float [F]):
    no self term - the rows start from bias instead of what Y holds."""
    _mat(X, "X"), _mat(Y, "Y")
    assert X.dtype == Y.dtype and X.shape[0] >= g.n_cols and Y.shape[0] >= g.n_rows
    assert rows is None or rows.numel() >= n_active
    _with_optional_ws(lib().gnn_masked_spmm_fwd_add, (
        C.byref(g.c), _ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0)), _ptr(Y),
        C.c_int64(Y.stride(0)), C.c_int32(F), C.c_int32(_dtype_code(X)), _ptr(row_scale), _ptr(col_scale), _ptr(bias),
        C.c_int32(1 if relu else 0)), (_stream(),), ws)


def spmm_workspace_bytes(g: Graph, n_active: int, X: torch.Tensor, Y: torch.Tensor, F: int) -> int:
    """Size query of gnn_masked_spmm_fwd: what a workspace would have to hold; 0 = the call gathers whole rows
    in one launch, > 0 = it takes the column-blocked route."""
    need = C.c_size_t(0)
    _check(lib().gnn_masked_spmm_fwd(
        C.byref(g.c), None, C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0)), _ptr(Y), C.c_int64(Y.stride(0)), C.c_int32(F),
        C.c_int32(_dtype_code(X)), None, None, None, C.byref(need), None))
    return int(need.value)


def gnn_masked_spmm_bwd(gT: Graph, out_rows, n_out: int, dist, max_active_dist: int, dY: torch.Tensor, dX: torch.Tensor,
                        F: int, row_scale=None, col_scale=None, accumulate: bool = False, ws: Workspace | None = None,
                        relu_H: torch.Tensor | None = None, src_prefix: int = -1):
    """relu_H: activations of the layer whose gradient dX is; the stored rows are zeroed where relu_H <= 0.
    src_prefix: >= 0: only the entries v < src_prefix of a row of gT are gathered (the forward rows of a (distance, id)-
    numbered partition)."""
    _mat(dY, "dY"), _mat(dX, "dX")
    if relu_H is not None:
        _mat(relu_H, "relu_H")
        assert relu_H.dtype == dX.dtype and relu_H.shape[0] >= gT.n_rows
    assert dY.dtype == dX.dtype and dY.shape[0] >= gT.n_cols and dX.shape[0] >= gT.n_rows
    assert out_rows is None or out_rows.numel() >= n_out
    _with_optional_ws(lib().gnn_masked_spmm_bwd, (
        C.byref(gT.c), _ptr(_i32(out_rows, "out_rows")), C.c_int32(n_out), _ptr(_i32(dist, "dist")),
        C.c_int32(max_active_dist), C.c_int32(src_prefix), _ptr(dY), C.c_int64(dY.stride(0)), _ptr(dX), C.c_int64(dX.stride(0)), C.c_int32(F),
        C.c_int32(_dtype_code(dY)), _ptr(row_scale), _ptr(col_scale), C.c_int32(1 if accumulate else 0), _ptr(relu_H),
        C.c_int64(relu_H.stride(0) if relu_H is not None else 0)), (_stream(),), ws)


def gnn_linear_fwd(rows, n_active: int, A_neigh: torch.Tensor, X_self, K: int, W_neigh: torch.Tensor, W_self, bias,
                   H_out: torch.Tensor, relu: bool, ws: Workspace | None = None):
    _mat(A_neigh, "A_neigh"), _mat(H_out, "H_out")
    N = W_neigh.shape[1]
    assert W_neigh.shape == (K, N) and W_neigh.is_contiguous() and W_neigh.dtype == A_neigh.dtype == H_out.dtype
    if X_self is not None:
        _mat(X_self, "X_self")
        assert X_self.stride(0) == A_neigh.stride(0) and X_self.dtype == A_neigh.dtype
        assert W_self.shape == (K, N) and W_self.is_contiguous() and W_self.dtype == W_neigh.dtype
    assert bias is None or (bias.dtype == torch.float32 and bias.numel() == N)
    _with_ws(lib().gnn_linear_fwd,
             (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(A_neigh), _ptr(X_self), C.c_int64(A_neigh.stride(0)),
              C.c_int32(K), _ptr(W_neigh), _ptr(W_self), _ptr(bias), C.c_int32(N), _ptr(H_out), C.c_int64(H_out.stride(0)),
              C.c_int32(1 if relu else 0), C.c_int32(_dtype_code(A_neigh))),
             (_stream(),), ws)


def gnn_linear_fwd_static(rows, n_active: int, A_neigh: torch.Tensor, X_self, K: int, W_neigh: torch.Tensor, W_self, bias,
                          H_out: torch.Tensor, relu: bool):
    """gnn_linear_fwd without a workspace: the library's own static device array takes its place (no allocation)."""
    _mat(A_neigh, "A_neigh"), _mat(H_out, "H_out")
    N = W_neigh.shape[1]
    assert W_neigh.shape == (K, N) and W_neigh.is_contiguous() and W_neigh.dtype == A_neigh.dtype == H_out.dtype
    if X_self is not None:
        _mat(X_self, "X_self")
        assert X_self.stride(0) == A_neigh.stride(0) and X_self.dtype == A_neigh.dtype
        assert W_self.shape == (K, N) and W_self.is_contiguous() and W_self.dtype == W_neigh.dtype
    assert bias is None or (bias.dtype == torch.float32 and bias.numel() == N)
    _check(lib().gnn_linear_fwd_static(
        _ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(A_neigh), _ptr(X_self), C.c_int64(A_neigh.stride(0)),
        C.c_int32(K), _ptr(W_neigh), _ptr(W_self), _ptr(bias), C.c_int32(N), _ptr(H_out), C.c_int64(H_out.stride(0)),
        C.c_int32(1 if relu else 0), C.c_int32(_dtype_code(A_neigh)), _stream()))


def gnn_linear_bwd(rows, n_active: int, dH_out: torch.Tensor, H_out, relu: bool, A_neigh: torch.Tensor, X_self, K: int,
                   W_neigh: torch.Tensor, W_self, dW_neigh: torch.Tensor, dW_self, dbias: torch.Tensor,
                   dA_neigh=None, dX_self=None, ws: Workspace | None = None):
    _mat(dH_out, "dH_out"), _mat(A_neigh, "A_neigh")
    N = W_neigh.shape[1]
    assert W_neigh.shape == (K, N) and W_neigh.is_contiguous()
    assert dW_neigh.dtype == torch.float32 and dW_neigh.shape == (K, N) and dW_neigh.is_contiguous()
    assert dbias.dtype == torch.float32 and dbias.numel() == N
    if H_out is not None:
        assert H_out.stride(0) == dH_out.stride(0) and H_out.dtype == dH_out.dtype
    if X_self is not None:
        assert X_self.stride(0) == A_neigh.stride(0)
        assert dW_self is not None and dW_self.dtype == torch.float32 and dW_self.shape == (K, N) and dW_self.is_contiguous()
    ld_din = 0
    for t in (dA_neigh, dX_self):
        if t is not None:
            _mat(t, "dA/dX")
            assert ld_din in (0, t.stride(0)) and t.dtype == A_neigh.dtype
            ld_din = t.stride(0)
    _with_ws(lib().gnn_linear_bwd,
             (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(dH_out), _ptr(H_out), C.c_int64(dH_out.stride(0)),
              C.c_int32(1 if relu else 0), _ptr(A_neigh), _ptr(X_self), C.c_int64(A_neigh.stride(0)), C.c_int32(K),
              _ptr(W_neigh), _ptr(W_self), C.c_int32(N), _ptr(dW_neigh), _ptr(dW_self), _ptr(dbias), _ptr(dA_neigh),
              _ptr(dX_self), C.c_int64(ld_din), C.c_int32(_dtype_code(A_neigh))),
             (_stream(),), ws)


def gnn_softmax_ce(rows, n_active: int, Z: torch.Tensor, n_classes: int, labels: torch.Tensor, dZ, loss: torch.Tensor,
                   ws: Workspace | None = None):
    _mat(Z, "Z")
    assert loss.dtype == torch.float32 and loss.numel() == 1 and labels.numel() >= n_active
    _with_ws(lib().gnn_softmax_ce,
             (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(Z), C.c_int64(Z.stride(0)), C.c_int32(n_classes),
              _ptr(_i32(labels, "labels")), _ptr(dZ), C.c_int64(dZ.stride(0) if dZ is not None else 0),
              C.c_int32(_dtype_code(Z)), _ptr(loss)),
             (_stream(),), ws)


def gnn_make_bitmap(ids: torch.Tensor, n: int) -> torch.Tensor:
    bitmap = torch.empty((n + 31) // 32, dtype=torch.int32, device=ids.device)
    _check(lib().gnn_make_bitmap(_ptr(_i32(ids, "ids")) if ids.numel() else None, C.c_int32(ids.numel()), C.c_int32(n),
                                 _ptr(bitmap) if n else None, _stream()))
    return bitmap


def gnn_sample_boundary(g: Graph, target_bitmap: torch.Tensor, targets: torch.Tensor, fanout: int, seed: int, hops: int = 1,
                        ws: Workspace | None = None):
    """Count pass + fill pass.  -> out_row_ptr int32[n_targets+1], out_col_idx int32[kept] (global ids)."""
    _i32(targets, "targets")
    nt = targets.numel()
    dev = g.row_ptr.device
    out_rp = torch.empty(nt + 1, dtype=torch.int32, device=dev)
    nnz_dev = torch.empty(1, dtype=torch.int64, device=dev)
    nnz_host = C.c_int64(0)
    common = (C.byref(g.c), _ptr(target_bitmap), _ptr(targets) if nt else None, C.c_int32(nt), C.c_int32(fanout),
              C.c_int32(hops), C.c_uint64(seed & (2**64 - 1)), _ptr(out_rp))
    _with_ws(lib().gnn_sample_boundary, common + (None, C.c_int64(0), _ptr(nnz_dev), C.byref(nnz_host)), (_stream(),), ws)
    kept = int(nnz_host.value)
    out_ci = torch.empty(max(kept, 1), dtype=torch.int32, device=dev)
    _with_ws(lib().gnn_sample_boundary, common + (_ptr(out_ci), C.c_int64(kept), _ptr(nnz_dev), None), (_stream(),), ws)
    return out_rp, out_ci[:kept]


def gnn_extract_partition(g: Graph, ring_ids: torch.Tensor, n_local: int, dist: torch.Tensor, L: int, ws: Workspace | None = None):
    """Count pass + fill pass.  -> (local Graph with sorted columns if g has them, new_id int32[g.n_rows])."""
    _i32(ring_ids, "ring_ids"), _i32(dist, "dist")
    assert ring_ids.numel() >= n_local and dist.numel() >= g.n_rows
    dev = g.row_ptr.device
    new_id = torch.empty(max(g.n_rows, 1), dtype=torch.int32, device=dev)
    out_rp = torch.empty(n_local + 1, dtype=torch.int32, device=dev)
    nnz_dev = torch.empty(1, dtype=torch.int64, device=dev)
    nnz_host = C.c_int64(0)
    common = (C.byref(g.c), _ptr(ring_ids) if n_local else None, C.c_int32(n_local), _ptr(dist), C.c_int32(L), _ptr(new_id), _ptr(out_rp))
    _with_ws(lib().gnn_extract_partition, common + (None, C.c_int64(0), _ptr(nnz_dev), C.byref(nnz_host)), (_stream(),), ws)
    nnz = int(nnz_host.value)
    out_ci = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    _with_ws(lib().gnn_extract_partition, common + (_ptr(out_ci), C.c_int64(nnz), _ptr(nnz_dev), None), (_stream(),), ws)
    return Graph(out_rp, out_ci[:nnz], n_cols=n_local, sorted_columns=g.sorted_columns), new_id[: g.n_rows]


def gnn_expand_row_ptr(n: int, ids: torch.Tensor, list_row_ptr: torch.Tensor, ws: Workspace | None = None) -> torch.Tensor:
    """-> int32[n + 1]: row ids[i] has the length of listed row i, all other rows are empty."""
    _i32(ids, "ids"), _i32(list_row_ptr, "list_row_ptr")
    assert list_row_ptr.numel() == ids.numel() + 1
    out = torch.empty(n + 1, dtype=torch.int32, device=ids.device)
    _with_ws(lib().gnn_expand_row_ptr, (C.c_int32(n), _ptr(ids) if ids.numel() else None, C.c_int32(ids.numel()), _ptr(list_row_ptr),
                                        _ptr(out)), (_stream(),), ws)
    return out


def gnn_extract_sampled_partition(gT: Graph, targets: torch.Tensor, kept_row_ptr: torch.Tensor, kept_col_idx: torch.Tensor,
                                  ws: Workspace | None = None):
    """The whole chain after gnn_sample_boundary (targets ASCENDING, as they were given to the sampler): kept rows as a
    CSR over the full id range, its two rings, extraction.  -> (local Graph, local_to_global int32[n_local], hop)."""
    n = gT.n_rows
    gs_rp = gnn_expand_row_ptr(n, targets, kept_row_ptr, ws=ws)
    gs = Graph(gs_rp, kept_col_idx.contiguous(), n_cols=n, sorted_columns=True)
    dist, ring, _, hop = gnn_build_active_sets(gs, targets, 1, ws=ws)
    n_local = int(hop[-1])
    dev = gT.row_ptr.device
    new_id = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    out_rp = torch.empty(n_local + 1, dtype=torch.int32, device=dev)
    nnz_dev = torch.empty(1, dtype=torch.int64, device=dev)
    nnz_host = C.c_int64(0)
    common = (C.byref(gT.c), C.byref(gs.c), _ptr(ring) if n_local else None, C.c_int32(n_local), _ptr(dist), _ptr(new_id), _ptr(out_rp))
    _with_ws(lib().gnn_extract_sampled_partition, common + (None, C.c_int64(0), _ptr(nnz_dev), C.byref(nnz_host)), (_stream(),), ws)
    nnz = int(nnz_host.value)
    out_ci = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    _with_ws(lib().gnn_extract_sampled_partition, common + (_ptr(out_ci), C.c_int64(nnz), _ptr(nnz_dev), None), (_stream(),), ws)
    return Graph(out_rp, out_ci[:nnz], n_cols=n_local, sorted_columns=True), ring[:n_local], hop


def gnn_gather_rows(src: torch.Tensor, ids: torch.Tensor, F: int, dst: torch.Tensor):
    """dst[i, :F] = src[ids[i], :F]."""
    _mat(src, "src"), _mat(dst, "dst"), _i32(ids, "ids")
    assert src.dtype == dst.dtype and dst.shape[0] >= ids.numel()
    _check(lib().gnn_gather_rows(_ptr(src), C.c_int64(src.stride(0)), C.c_int32(src.shape[0]), _ptr(ids), C.c_int32(ids.numel()),
                                 C.c_int32(F), C.c_int32(_dtype_code(src)), _ptr(dst), C.c_int64(dst.stride(0)), _stream()))


LN_EPS = 1e-5


def gnn_layer_norm_relu_fwd(rows, n_active: int, X: torch.Tensor, F: int, gamma: torch.Tensor, beta: torch.Tensor, Y: torch.Tensor,
                            eps: float = LN_EPS):
    """Y[rows, :F] = ReLU(LayerNorm(X[rows, :F]) * gamma + beta)."""
    _mat(X, "X"), _mat(Y, "Y")
    assert X.dtype == Y.dtype and gamma.dtype == torch.float32 and beta.dtype == torch.float32 and gamma.numel() == F == beta.numel()
    _check(lib().gnn_layer_norm_relu_fwd(_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0)), C.c_int32(F),
                                         _ptr(gamma), _ptr(beta), C.c_float(eps), _ptr(Y), C.c_int64(Y.stride(0)),
                                         C.c_int32(_dtype_code(X)), _stream()))


def gnn_layer_norm_relu_bwd(rows, n_active: int, dY: torch.Tensor, T: torch.Tensor, X: torch.Tensor, F: int, gamma: torch.Tensor,
                            dRes, n_res: int, dX: torch.Tensor, dgamma: torch.Tensor, dbeta: torch.Tensor, eps: float = LN_EPS,
                            ws: Workspace | None = None):
    """dX[rows] = LN-backward(dY where T > 0) (+ dRes for the first n_res listed rows); dgamma, dbeta overwritten."""
    for t, nm in ((dY, "dY"), (T, "T"), (X, "X"), (dX, "dX")):
        _mat(t, nm)
        assert t.dtype == X.dtype
    assert dgamma.dtype == torch.float32 and dbeta.dtype == torch.float32 and dgamma.numel() == F == dbeta.numel()
    if dRes is not None:
        _mat(dRes, "dRes")
        assert dRes.dtype == X.dtype
    _with_ws(lib().gnn_layer_norm_relu_bwd,
             (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(dY), C.c_int64(dY.stride(0)), _ptr(T), C.c_int64(T.stride(0)),
              _ptr(X), C.c_int64(X.stride(0)), C.c_int32(F), _ptr(gamma), C.c_float(eps), _ptr(dRes),
              C.c_int64(dRes.stride(0) if dRes is not None else 0), C.c_int32(n_res), _ptr(dX), C.c_int64(dX.stride(0)),
              _ptr(dgamma), _ptr(dbeta), C.c_int32(_dtype_code(X))),
             (_stream(),), ws)


def gnn_add_rows(rows, n_active: int, X: torch.Tensor, Y: torch.Tensor, F: int):
    """Y[rows, :F] += X[rows, :F]."""
    _mat(X, "X"), _mat(Y, "Y")
    assert X.dtype == Y.dtype
    _check(lib().gnn_add_rows(_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0)), _ptr(Y),
                              C.c_int64(Y.stride(0)), C.c_int32(F), C.c_int32(_dtype_code(X)), _stream()))


def gnn_add_rows_masked(rows, n_active: int, X, n_add: int, Y: torch.Tensor, F: int, H: torch.Tensor):
    """Y[rows, :F] = (Y[rows, :F] + X[rows, :F] for the first n_add listed rows) where H > 0, else 0."""
    _mat(Y, "Y"), _mat(H, "H")
    assert H.dtype == Y.dtype
    assert rows is None or rows.numel() >= n_active
    if X is not None:
        _mat(X, "X")
        assert X.dtype == Y.dtype
    else:
        assert n_add == 0
    _check(lib().gnn_add_rows_masked(_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0) if X is not None else 0),
                                     C.c_int32(n_add), _ptr(Y), C.c_int64(Y.stride(0)), C.c_int32(F), _ptr(H), C.c_int64(H.stride(0)),
                                     C.c_int32(_dtype_code(Y)), _stream()))


def gnn_bias_grad(rows, n_active: int, dZ: torch.Tensor, N: int, dbias: torch.Tensor, ws: Workspace | None = None):
    """dbias[:N] = sum of dZ[rows, :N]."""
    _mat(dZ, "dZ")
    assert dbias.dtype == torch.float32 and dbias.numel() >= N and dbias.is_contiguous()
    assert rows is None or rows.numel() >= n_active
    _with_ws(lib().gnn_bias_grad, (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(dZ), C.c_int64(dZ.stride(0)), C.c_int32(N),
                                   C.c_int32(_dtype_code(dZ)), _ptr(dbias)), (_stream(),), ws)


def gnn_linear_bwd_input(rows, n_active: int, dZ: torch.Tensor, N: int, W: torch.Tensor, K: int, n_accumulate: int, relu_H, dX: torch.Tensor,
                         ws: Workspace | None = None):
    """dX[rows] = (dZ[rows] W^T + dX[rows] for the first n_accumulate listed rows) where relu_H > 0, else 0."""
    _mat(dZ, "dZ"), _mat(dX, "dX")
    assert W.shape == (K, N) and W.is_contiguous() and W.dtype == dZ.dtype == dX.dtype
    assert rows is None or rows.numel() >= n_active
    if relu_H is not None:
        _mat(relu_H, "relu_H")
        assert relu_H.dtype == dX.dtype
    _with_ws(lib().gnn_linear_bwd_input,
             (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(dZ), C.c_int64(dZ.stride(0)), C.c_int32(N), _ptr(W), C.c_int32(K),
              C.c_int32(n_accumulate), _ptr(relu_H), C.c_int64(relu_H.stride(0) if relu_H is not None else 0), _ptr(dX),
              C.c_int64(dX.stride(0)), C.c_int32(_dtype_code(dZ))), (_stream(),), ws)


def gnn_linear_bwd_input2(rows, n_active: int, dG: torch.Tensor, W_neigh: torch.Tensor, dZ, W_self, n_self: int, N: int, K: int,
                          relu_H, dX: torch.Tensor, ws: Workspace | None = None):
    """dX[rows] = (dG[rows] W_neigh^T + dZ[rows] W_self^T for the first n_self listed rows) where relu_H > 0, else 0."""
    _mat(dG, "dG"), _mat(dX, "dX")
    assert W_neigh.shape == (K, N) and W_neigh.is_contiguous() and W_neigh.dtype == dG.dtype == dX.dtype
    assert rows is None or rows.numel() >= n_active
    if n_self > 0:
        _mat(dZ, "dZ")
        assert dZ.dtype == dG.dtype and dZ.stride(0) == dG.stride(0) and dZ.shape[0] >= dG.shape[0]
        assert W_self.shape == (K, N) and W_self.is_contiguous() and W_self.dtype == dG.dtype
    if relu_H is not None:
        _mat(relu_H, "relu_H")
        assert relu_H.dtype == dX.dtype
    _with_ws(lib().gnn_linear_bwd_input2,
             (_ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(dG), _ptr(W_neigh), _ptr(dZ) if n_self > 0 else None,
              _ptr(W_self) if n_self > 0 else None, C.c_int32(n_self), C.c_int64(dG.stride(0)), C.c_int32(N), C.c_int32(K),
              _ptr(relu_H), C.c_int64(relu_H.stride(0) if relu_H is not None else 0), _ptr(dX), C.c_int64(dX.stride(0)),
              C.c_int32(_dtype_code(dG))), (_stream(),), ws)


def gnn_die_mapping():
    """-> (list of the compute-die ids the 64 workgroups of the probe grid ran on, whether workgroup i ran on die i mod 8)."""
    ids = (C.c_int32 * 64)()
    holds = C.c_int32(0)
    _check(lib().gnn_die_mapping(ids, C.c_int32(64), C.byref(holds)))
    return list(ids), bool(holds.value)


def fused_layer_supported(K: int, N: int, dtype) -> bool:
    """Shapes gnn_fused_layer_fwd takes: input rows of 128 to 512 bytes (K rounded up to 32 bytes), output rows up to 512."""
    es = torch.empty(0, dtype=dtype).element_size()
    kp = (K * es + 31) // 32 * 32
    return 128 <= kp <= 512 and N * es <= 512


def gnn_fused_layer_fwd(g: Graph, rows, n_active: int, X: torch.Tensor, K: int, row_scale, col_scale, W_neigh: torch.Tensor,
                        W_self, bias, H_out: torch.Tensor, relu: bool, ws: Workspace | None = None):
    """H_out[rows] = act(aggregate(X)[rows] W_neigh (+ X[rows] W_self) + bias) in one kernel; the aggregate stays on chip."""
    _mat(X, "X"), _mat(H_out, "H_out")
    N = W_neigh.shape[1]
    assert W_neigh.shape == (K, N) and W_neigh.is_contiguous() and W_neigh.dtype == X.dtype == H_out.dtype
    assert X.shape[0] >= g.n_cols and H_out.shape[0] >= g.n_rows
    assert W_self is None or (W_self.shape == (K, N) and W_self.is_contiguous() and W_self.dtype == X.dtype)
    assert bias is None or (bias.dtype == torch.float32 and bias.numel() == N)
    assert rows is None or rows.numel() >= n_active
    _with_ws(lib().gnn_fused_layer_fwd,
             (C.byref(g.c), _ptr(_i32(rows, "rows")), C.c_int32(n_active), _ptr(X), C.c_int64(X.stride(0)), C.c_int32(K),
              _ptr(row_scale), _ptr(col_scale), _ptr(W_neigh), _ptr(W_self), _ptr(bias), C.c_int32(N), _ptr(H_out),
              C.c_int64(H_out.stride(0)), C.c_int32(1 if relu else 0), C.c_int32(_dtype_code(X))), (_stream(),), ws)
