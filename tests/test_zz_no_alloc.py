"""GPU: gnn_linear_fwd_static (the forward feature transform for callers that cannot allocate) against
gnn_linear_fwd on the same inputs, through the C ABI.  Same kernels, so the bar is bit equality (inside the
fp32 1e-4 / bf16 2e-2 bars by construction); also checked against the oracle once.  Two calls in a row share the
library's static device array; the second one is smaller, so stale contents of the first must not matter."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from gpu_util import as_stored, check, dev, host64, padded
from paper_2311_06837_amd import binding as B

pytestmark = pytest.mark.gpu

SENT = 555.0


def _call(fn_static, rows, n_active, A, X, K, Wn, Ws, bias, H, relu):
    """The C symbol itself, with raw pointers (no workspace arguments exist for the static form)."""
    p = lambda t: None if t is None else C.c_void_p(t.data_ptr())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    dt = B.GNN_F32 if A.dtype == torch.float32 else B.GNN_BF16
    common = (p(rows), C.c_int32(n_active), p(A), p(X), C.c_int64(A.stride(0)), C.c_int32(K), p(Wn), p(Ws), p(bias),
              C.c_int32(Wn.shape[1]), p(H), C.c_int64(H.stride(0)), C.c_int32(1 if relu else 0), C.c_int32(dt))
    lib = B.lib()
    if fn_static:
        st = lib.gnn_linear_fwd_static(*common, stream)
        assert st == 0, lib.gnn_last_error()
        return
    need = C.c_size_t(0)
    assert lib.gnn_linear_fwd(*common, None, C.byref(need), stream) == 0
    ws = torch.empty(max(need.value, 256), dtype=torch.uint8, device="cuda")
    have = C.c_size_t(ws.numel())
    st = lib.gnn_linear_fwd(*common, C.c_void_p(ws.data_ptr()), C.byref(have), stream)
    assert st == 0, lib.gnn_last_error()
    torch.cuda.synchronize()


def _one(M, n_active, K, N, dtype, sage, relu, use_rows, seed, with_oracle=False):
    print(f"static linear fwd: M={M} active={n_active} K={K} N={N} {dtype} sage={sage} rows={use_rows}", flush=True)
    rng = np.random.default_rng(seed)
    mult = 4 if dtype == torch.float32 else 8
    ld_in, ld_out = (K + mult - 1) // mult * mult, (N + mult - 1) // mult * mult
    A = as_stored(rng.standard_normal((M, K)), dtype)
    Xs = as_stored(rng.standard_normal((M, K)), dtype) if sage else None
    Wn = as_stored(rng.standard_normal((K, N)) / np.sqrt(K), dtype)
    Ws = as_stored(rng.standard_normal((K, N)) / np.sqrt(K), dtype) if sage else None
    b = rng.standard_normal(N).astype(np.float32)
    rows = np.sort(rng.choice(M, n_active, replace=False)).astype(np.int32) if use_rows else None
    Ad = padded(A, ld_in, dtype)
    Xd = padded(Xs, ld_in, dtype) if sage else None
    Wnd, Wsd, bd = dev(Wn, dtype), (dev(Ws, dtype) if sage else None), dev(b)
    rd = dev(rows) if use_rows else None
    H_ws = torch.full((M, ld_out), SENT, dtype=dtype, device="cuda")
    H_st = torch.full((M, ld_out), SENT, dtype=dtype, device="cuda")
    _call(False, rd, n_active, Ad, Xd, K, Wnd, Wsd, bd, H_ws, relu)
    _call(True, rd, n_active, Ad, Xd, K, Wnd, Wsd, bd, H_st, relu)
    torch.cuda.synchronize()
    assert torch.equal(H_ws.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       H_st.view(torch.int16 if dtype == torch.bfloat16 else torch.int32)), "static form differs from gnn_linear_fwd"
    if with_oracle:
        sel = rows if use_rows else np.arange(n_active)
        H = np.zeros((M, N))
        oracle.linear_fwd(sel.astype(np.int32), A, Xs, K, Wn, Ws, b.astype(np.float64), H, relu)
        check(host64(H_st)[sel, :N], H[sel], dtype, "H (static form)")


def test_two_calls_in_a_row_second_one_smaller():
    # larger first: both weight slots of the static array are filled to 602 x 256 floats; then a smaller GCN-shaped call
    # (one slot, fewer columns) must not see what the first one left behind
    _one(3000, 2500, 602, 256, torch.float32, True, True, True, 1, with_oracle=True)
    _one(700, 700, 100, 47, torch.float32, False, False, False, 2, with_oracle=True)
    _one(2000, 1999, 256, 128, torch.bfloat16, True, True, False, 3, with_oracle=True)
    _one(300, 17, 33, 5, torch.bfloat16, False, True, True, 4, with_oracle=True)


def test_setup_call_and_size_limit():
    lib = B.lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # n_active == 0: set-up only (address lookup), nothing is read
    assert lib.gnn_linear_fwd_static(None, 0, None, None, C.c_int64(64), 64, None, None, None, 64, None, C.c_int64(64), 0, 0, stream) == 0
    # 2048 x 1024 floats = 8 MiB per matrix: beyond the 4 MiB the static array has per matrix
    st = lib.gnn_linear_fwd_static(None, 0, None, None, C.c_int64(2048), 2048, None, None, None, 1024, None, C.c_int64(1024), 0, 0, stream)
    assert st == 4 and b"static array" in lib.gnn_last_error()
    # the same shape in bf16 is exactly at the limit: accepted
    assert lib.gnn_linear_fwd_static(None, 0, None, None, C.c_int64(2048), 2048, None, None, None, 1024, None, C.c_int64(1024), 0, 1, stream) == 0
