"""Sequencing of the C-ABI calls for one partition: active sets once, then per training step
forward (aggregation + transform per layer), loss, backward.  Host orchestration only; all
arithmetic happens behind include/gnnhot.h.

Paper section 6, figure 7c: (1) multi-hop dependency from the inner vertices, (3)-(4) every
layer reuses the same one-hop graph and a per-layer mask, (5) logits of the inner vertices.
"""
from __future__ import annotations

import torch

from . import binding as B


def row_stride(width: int, dtype) -> int:
    """Leading dimension (in elements) the model gives a matrix of `width` columns: rows start on 128-byte
    boundaries, so a 256-byte stretch of a gathered row touches two cache lines, never three."""
    mult = 128 // torch.empty(0, dtype=dtype).element_size()
    return (width + mult - 1) // mult * mult


class MaskedGNN:
    """L-layer GCN ("gcn") or GraphSAGE-mean ("sage") over one partition under one-hop masking.

    graph, graph_t   B.Graph of the one-hop graph and of its transpose (same object if symmetric)
    targets          int32 device tensor of inner-vertex ids
    params           list of dicts with float32 device tensors W_neigh [K,N], W_self (sage), bias [N]
    dtype            torch.float32 or torch.bfloat16 (storage of activations and weights)
    global_degree    int32 device tensor: row lengths in the unpartitioned graph (GCN normalisation)
    prefix_numbered  the caller's promise that the vertices are numbered by (distance from the targets, id), as
                     gnn_extract_partition numbers them: every R_l is then the id range 0 .. |R_l|-1 and the calls
                     get rows = NULL instead of an id list (checked once, when the active sets are first built)
    layer_sampling   None, or (rule, parameter, seed): layer-wise sampling as per-layer masking - layer l aggregates
                     through gnn_layer_edge_mask(rule, layer = l) over its rows, forward and backward; rule
                     "threshold" (parameter = 64-bit key threshold) or "fanout" (parameter = neighbours kept per row).
                     The masks are rebuilt in every step (a training run changes the seed per epoch).
    transform_first  the order of a layer's two halves.  The paper's order: aggregate the layer's input, then multiply by
                     the weights.  Exchanged: multiply first, P = H_{l-1} W_neigh, then aggregate P on top of the self
                     term (gnn_masked_spmm_fwd_add) - the same sum, gathered dims[l] instead of dims[l-1] columns wide;
                     the backward pass aggregates the layer's output gradient (dP = Agg^T(dZ), dims[l] wide) and gets
                     dW_neigh = H_{l-1}^T dP and the input gradient dP W_neigh^T + dZ W_self^T (two products; the
                     second one adds onto the first and masks in front of the previous ReLU: gnn_linear_bwd_input).  A GCN layer has no self term: its sum starts
                     from the bias, its bias gradient comes from gnn_bias_grad.  True: every layer that narrows its
                     input (dims[l-1] > dims[l]); "auto" (default): those of them whose input rows are at
                     least 512 bytes long (shorter rows are gathered at a rate set by their number, not their bytes:
                     narrowing them further buys nothing and the two extra products cost); False: none; or a
                     collection of layer numbers.
    grad_first       the order of the two linear steps of a GraphSAGE layer's neighbour half in the BACKWARD pass.  The
                     chain rule gives dA_l = dZ W_neigh^T, then the backward aggregation of dA_l added onto dZ W_self^T.
                     True ("auto": where dims[l] <= dims[l-1], the default): aggregate the output gradient first,
                     G = Agg^T(dZ) (dims[l] columns, plain store), then ONE product dH_{l-1} = mask(G W_neigh^T + dZ W_self^T)
                     (gnn_linear_bwd_input2) - one pass over dZ and one over dH_{l-1} fewer.  False: the chain rule's order.
    fused_forward    True: the GraphSAGE layers whose backward pass aggregates first (grad_first), in the paper's order and
                     of a shape the kernel takes run their forward pass as ONE kernel (gnn_fused_layer_fwd): the aggregate
                     A_l stays on chip and is never stored; the backward pass then gets dW_neigh = H_{l-1}^T Agg^T(dZ) from
                     the aggregated gradient it forms anyway.  False (default): two calls per layer.
    side_stream      True (default): the weight-gradient products of the backward pass - nothing in the step waits for
                     them - are enqueued on a second HIP stream (default priority, a workspace of its own), so they
                     run beside the backward aggregations, which leave the matrix cores idle; the step's stream
                     waits for that stream when the backward pass ends.  False: everything on the caller's stream.
    """

    def __init__(self, graph: B.Graph, graph_t: B.Graph, targets: torch.Tensor, kind: str, params: list,
                 dtype=torch.float32, global_degree: torch.Tensor | None = None, prefix_numbered: bool = False,
                 layer_sampling=None, transform_first="auto", side_stream: bool = True, grad_first="auto",
                 fused_forward: bool = False):
        assert kind in ("gcn", "sage")
        self.layer_sampling = layer_sampling
        self.prefix_numbered, self._prefix_checked = prefix_numbered, False
        self.rs = self.cs = None
        self.g, self.gt, self.targets, self.kind, self.dtype = graph, graph_t, targets, kind, dtype
        self.n = graph.n_rows
        self.L = len(params)
        self.ws = B.Workspace()
        self.side = torch.cuda.Stream(device=targets.device) if side_stream else None
        self.ws_side = B.Workspace()
        self.dims = [params[0]["W_neigh"].shape[0]] + [p["W_neigh"].shape[1] for p in params]
        self.params = []
        for p in params:
            q = {"W_neigh": p["W_neigh"].to(dtype).contiguous(), "bias": p["bias"].float().contiguous()}
            if kind == "sage":
                q["W_self"] = p["W_self"].to(dtype).contiguous()
            self.params.append(q)
        self.global_degree = global_degree
        self.ld = [row_stride(d, dtype) for d in self.dims]
        dev = targets.device
        if transform_first is True or (isinstance(transform_first, str) and transform_first == "auto"):
            es = 4 if dtype == torch.float32 else 2
            min_bytes = 0 if transform_first is True else 512
            self.tf_layers = frozenset(l for l in range(1, self.L + 1) if self.dims[l - 1] > self.dims[l]
                                       and self.dims[l - 1] * es >= min_bytes)
        elif transform_first is False:
            self.tf_layers = frozenset()
        else:
            self.tf_layers = frozenset(int(l) for l in transform_first)
            assert all(1 <= l <= self.L for l in self.tf_layers)
        if kind != "sage" or grad_first is False:
            self.gf_layers = frozenset()
        else:
            self.gf_layers = frozenset(l for l in range(2, self.L + 1)
                                       if grad_first is True or self.dims[l] <= self.dims[l - 1])
        self.fused_layers = frozenset(l for l in self.gf_layers if fused_forward and l not in self.tf_layers and layer_sampling is None
                                      and B.fused_layer_supported(self.dims[l - 1], self.dims[l], dtype))
        # activations A_l, H_l and their gradients; rows outside the active sets are never touched
        self.A = [None] + [None if (l in self.tf_layers or l in self.fused_layers)
                           else torch.zeros(self.n, self.ld[l - 1], dtype=dtype, device=dev) for l in range(1, self.L + 1)]
        # a layer in the exchanged order keeps no aggregate of its input; instead its transformed rows P_l and the
        # gradient dP_l that reaches them
        self.P = {l: torch.zeros(self.n, self.ld[l], dtype=dtype, device=dev) for l in self.tf_layers}
        self.dP = {l: torch.zeros(self.n, self.ld[l], dtype=dtype, device=dev) for l in self.tf_layers}
        self._dbias_unused = torch.zeros(max(self.dims), dtype=torch.float32, device=dev)
        self.H = [None] + [torch.zeros(self.n, self.ld[l], dtype=dtype, device=dev) for l in range(1, self.L + 1)]
        self.dH = [None] + [torch.zeros(self.n, self.ld[l], dtype=dtype, device=dev) for l in range(1, self.L + 1)]
        self.dA = [None, None] + [None if (l in self.tf_layers or l in self.gf_layers)
                                  else torch.zeros(self.n, self.ld[l - 1], dtype=dtype, device=dev) for l in range(2, self.L + 1)]
        # the output gradient of a layer aggregated backwards (layers whose backward pass aggregates first)
        self.dG = {l: torch.zeros(self.n, self.ld[l], dtype=dtype, device=dev) for l in self.gf_layers if l not in self.tf_layers}
        self.grads = []
        for p in self.params:
            gdict = {"dW_neigh": torch.zeros_like(p["W_neigh"], dtype=torch.float32), "dbias": torch.zeros_like(p["bias"])}
            if kind == "sage":
                gdict["dW_self"] = torch.zeros_like(p["W_self"], dtype=torch.float32)
            self.grads.append(gdict)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.hop = None
        self.trace = None   # when a list: (name, start_event, end_event) per C-ABI call, for the benchmark

    def _call(self, name, fn, *args, **kw):
        """Run one C-ABI call; with tracing on, bracket it by events on the stream it is launched on."""
        if self.trace is None:
            return fn(*args, **kw)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        out = fn(*args, **kw)
        b.record()
        self.trace.append((name, a, b))
        return out

    def _call_beside(self, name, fn, *args, **kw):
        """A call whose inputs are final by now and whose outputs nobody reads before the backward pass ends (weight
        and bias gradients): on the side stream, after everything enqueued so far on the step's stream."""
        if self.side is None:
            return self._call(name, fn, *args, ws=self.ws, **kw)
        ready = torch.cuda.Event()
        ready.record()
        with torch.cuda.stream(self.side):
            self.side.wait_event(ready)
            return self._call(name, fn, *args, ws=self.ws_side, **kw)

    def _join_side(self):
        if self.side is not None:
            torch.cuda.current_stream().wait_stream(self.side)

    # -- step a1 -------------------------------------------------------------------------
    def build_active_sets(self):
        self.dist, self.ring_ids, self.hop_offsets, self.hop = self._call(
            "active_sets", B.gnn_build_active_sets, self.g, self.targets, self.L, ws=self.ws, gt=self.gt)
        if self.rs is None:      # the normalisation factors depend on the graph alone: made once, not per step
            if self.kind == "gcn":
                s = B.gnn_norm_scales(B.GNN_NORM_SYM, self.n, length=self.global_degree,
                                      row_ptr=None if self.global_degree is not None else self.g.row_ptr)
                self.rs, self.cs = s, s
            else:
                self.rs, self.cs = B.gnn_norm_scales(B.GNN_NORM_MEAN, self.n, row_ptr=self.g.row_ptr), None
        if self.prefix_numbered and not self._prefix_checked:
            n_all = int(self.hop[-1])
            ident = torch.arange(n_all, dtype=torch.int32, device=self.ring_ids.device)
            if not torch.equal(self.ring_ids[:n_all], ident):
                raise ValueError("prefix_numbered was promised but the ring-sorted ids are not 0 .. n-1")
            self._prefix_checked = True
        self.rows = None if self.prefix_numbered else self.ring_ids
        return self.hop

    def build_layer_masks(self):
        """Per-layer edge masks of layer-wise sampling: the graph seen through layer l's mask (forward), its transpose
        seen through the same mask (backward), and the mean over the kept neighbours."""
        rule, par, seed = self.layer_sampling
        self.g_l, self.gt_l, self.rs_l, self.kept_l = [None], [None], [None], [None]
        for l in range(1, self.L + 1):
            nl = self.n_rows_of_layer(l)
            # layer 1 has no backward aggregation in the paper's order: its threshold pairs are not needed then
            need_t = l > 1 or l in self.tf_layers
            out = self._call(f"layer_mask_{l}", B.gnn_layer_edge_mask, self.g, self.rows, nl, rule, l, seed,
                             fanout=par if rule == "fanout" else 0, threshold=par if rule == "threshold" else (1 << 64) - 1,
                             with_thresholds=need_t)
            keep, kept_len = out[0], out[1]
            self.g_l.append(self.g.with_edge_keep(keep))
            self.kept_l.append(kept_len)
            if need_t:
                keep_t = self._call(f"layer_mask_t_{l}", B.gnn_layer_edge_mask_transposed, self.gt, out[2], out[3], l, seed)
                self.gt_l.append(self.gt.with_edge_keep(keep_t))
            else:
                self.gt_l.append(None)
            self.rs_l.append(self.rs if self.kind == "gcn" else B.gnn_norm_scales(B.GNN_NORM_MEAN, self.n, length=kept_len))

    def n_rows_of_layer(self, l: int) -> int:
        """|R_l|, R_l = {dist <= L - l}: a prefix of the ring-sorted ids."""
        return int(self.hop[self.L - l + 1])

    @property
    def transform_first(self) -> bool:
        return bool(self.tf_layers)

    def agg_width(self, l: int) -> int:
        """Columns of the matrix that layer l's forward aggregation gathers."""
        return self.dims[l] if l in self.tf_layers else self.dims[l - 1]

    def set_input(self, H0: torch.Tensor):
        """H0: [n, row_stride(F0, dtype)] of the model dtype, row-major; used in place."""
        assert H0.dtype == self.dtype and H0.shape[0] == self.n and H0.stride(0) == self.ld[0]
        self.H[0] = H0

    # -- steps a2, a3, a4 ----------------------------------------------------------------
    def forward(self, labels: torch.Tensor) -> torch.Tensor:
        for l in range(1, self.L + 1):
            p = self.params[l - 1]
            K = self.dims[l - 1]
            nl = self.n_rows_of_layer(l)
            g_l, rs_l = (self.g, self.rs) if self.layer_sampling is None else (self.g_l[l], self.rs_l[l])
            if l in self.tf_layers:
                n_prev = self.n_rows_of_layer(l - 1)    # every row of R_{l-1} can be a neighbour of a row of R_l
                self._call(f"linear_pre_{l}", B.gnn_linear_fwd, self.rows, n_prev, self.H[l - 1], None, K, p["W_neigh"], None, None,
                           self.P[l], relu=False, ws=self.ws)
                if self.kind == "sage":
                    self._call(f"linear_fwd_{l}", B.gnn_linear_fwd, self.rows, nl, self.H[l - 1], None, K, p["W_self"], None, p["bias"],
                               self.H[l], relu=False, ws=self.ws)
                self._call(f"spmm_fwd_{l}", B.gnn_masked_spmm_fwd_add, g_l, self.rows, nl, self.P[l], self.H[l], self.dims[l], rs_l,
                           self.cs, relu=(l < self.L), ws=self.ws, bias=None if self.kind == "sage" else p["bias"])
                continue
            if l in self.fused_layers:
                self._call(f"fused_fwd_{l}", B.gnn_fused_layer_fwd, g_l, self.rows, nl, self.H[l - 1], K, rs_l, self.cs, p["W_neigh"],
                           p["W_self"], p["bias"], self.H[l], relu=(l < self.L), ws=self.ws)
                continue
            self._call(f"spmm_fwd_{l}", B.gnn_masked_spmm_fwd, g_l, self.rows, nl, self.H[l - 1], self.A[l], K, rs_l, self.cs, ws=self.ws)
            self._call(f"linear_fwd_{l}", B.gnn_linear_fwd, self.rows, nl, self.A[l], self.H[l - 1] if self.kind == "sage" else None, K,
                             p["W_neigh"], p.get("W_self"), p["bias"], self.H[l], relu=(l < self.L), ws=self.ws)
        nt = self.n_rows_of_layer(self.L)
        self._call("softmax_ce", B.gnn_softmax_ce, self.rows, nt, self.H[self.L], self.dims[self.L], labels, self.dH[self.L], self.loss, ws=self.ws)
        return self.loss

    # -- steps a5, a6 --------------------------------------------------------------------
    def backward(self):
        L = self.L
        for l in range(L, 0, -1):
            p, gr = self.params[l - 1], self.grads[l - 1]
            K = self.dims[l - 1]
            nl = self.n_rows_of_layer(l)
            sage = self.kind == "sage"
            need_in = l > 1
            if l in self.tf_layers:
                self._backward_transform_first(l)
                continue
            # dH_l arrives with the ReLU of layer l already undone: the call that wrote it last masked it
            N = self.dims[l]
            if l in self.gf_layers:
                # weight and bias gradients beside the rest (they need A_l, H_{l-1} and dZ only); the input gradient from the
                # aggregated output gradient: G = Agg^T(dZ) over every row of R_{l-1}, then one product for both halves
                fused = l in self.fused_layers
                if fused:   # no A_l: the self half's gradients from dZ now, the neighbour half's from the aggregated gradient below
                    self._call_beside(f"linear_bwd_{l}", B.gnn_linear_bwd, self.rows, nl, self.dH[l], None, False, self.H[l - 1], None, K,
                                      p["W_self"], None, gr["dW_self"], None, gr["dbias"], None, None)
                else:
                    self._call_beside(f"linear_bwd_{l}", B.gnn_linear_bwd, self.rows, nl, self.dH[l], None, False, self.A[l],
                                      self.H[l - 1], K, p["W_neigh"], p["W_self"], gr["dW_neigh"], gr["dW_self"], gr["dbias"], None, None)
                n_prev = self.n_rows_of_layer(l - 1)
                gt_l, rs_l = (self.gt, self.rs) if self.layer_sampling is None else (self.gt_l[l], self.rs_l[l])
                dist_l, pre_l = self._source_filter(nl)
                self._call(f"spmm_bwd_{l}", B.gnn_masked_spmm_bwd, gt_l, self.rows, n_prev, dist_l, L - l, self.dH[l], self.dG[l], N,
                           rs_l, self.cs, accumulate=False, ws=self.ws if 4 * nl >= self.n else None, src_prefix=pre_l)
                if fused:
                    self._call_beside(f"linear_bwd_{l}_neigh", B.gnn_linear_bwd, self.rows, n_prev, self.dG[l], None, False, self.H[l - 1],
                                      None, K, p["W_neigh"], None, gr["dW_neigh"], None, self._dbias_unused[:N], None, None)
                self._call(f"linear_bwd_{l}_input", B.gnn_linear_bwd_input2, self.rows, n_prev, self.dG[l], p["W_neigh"], self.dH[l],
                           p["W_self"], nl, N, K, self.H[l - 1], self.dH[l - 1], ws=self.ws)
                continue
            if need_in and self.side is not None:
                # weight and bias gradients beside the rest; the input gradients, which the aggregation waits for, here
                self._call_beside(f"linear_bwd_{l}", B.gnn_linear_bwd, self.rows, nl, self.dH[l], None, False, self.A[l],
                                  self.H[l - 1] if sage else None, K, p["W_neigh"], p.get("W_self"),
                                  gr["dW_neigh"], gr.get("dW_self"), gr["dbias"], None, None)
                self._call(f"linear_bwd_{l}_input", B.gnn_linear_bwd_input, self.rows, nl, self.dH[l], N, p["W_neigh"], K, 0, None,
                           self.dA[l], ws=self.ws)
                if sage:
                    self._call(f"linear_bwd_{l}_input_self", B.gnn_linear_bwd_input, self.rows, nl, self.dH[l], N, p["W_self"], K, 0,
                               None, self.dH[l - 1], ws=self.ws)
            else:
                self._call(f"linear_bwd_{l}", B.gnn_linear_bwd, self.rows, nl, self.dH[l], None, False, self.A[l],
                           self.H[l - 1] if sage else None, K, p["W_neigh"], p.get("W_self"),
                           gr["dW_neigh"], gr.get("dW_self"), gr["dbias"],
                           self.dA[l] if need_in else None, self.dH[l - 1] if (need_in and sage) else None, ws=self.ws)
            if need_in:
                n_prev = self.n_rows_of_layer(l - 1)
                # The backward gather only keeps the neighbours that were rows of the forward call.  When those are
                # few (the last layers: R_l is close to T), the column-blocked route would spend more on preparing
                # every edge than the gathers cost: no workspace -> the one-launch route.
                ws_bwd = self.ws if 4 * nl >= self.n else None
                gt_l, rs_l = (self.gt, self.rs) if self.layer_sampling is None else (self.gt_l[l], self.rs_l[l])
                # when the forward call computed every vertex of the partition the filter keeps everything: leave it out
                dist_l, pre_l = self._source_filter(nl)
                relu_h = self.H[l - 1]      # layer l-1 ends in a ReLU (l-1 < L): its gradient leaves the aggregation masked
                if sage:
                    # rows of R_l already hold dZ W_self^T: add the aggregated part; the next ring starts from zero
                    self._call(f"spmm_bwd_{l}", B.gnn_masked_spmm_bwd, gt_l, self.rows, nl, dist_l, L - l, self.dA[l], self.dH[l - 1], K,
                                          rs_l, self.cs, accumulate=True, ws=ws_bwd, relu_H=relu_h, src_prefix=pre_l)
                    if n_prev > nl:
                        self._call(f"spmm_bwd_{l}_ring", B.gnn_masked_spmm_bwd, gt_l, self.ring_ids[nl:], n_prev - nl, dist_l, L - l, self.dA[l],
                                              self.dH[l - 1], K, rs_l, self.cs, accumulate=False, ws=ws_bwd, relu_H=relu_h, src_prefix=pre_l)
                else:
                    self._call(f"spmm_bwd_{l}", B.gnn_masked_spmm_bwd, gt_l, self.rows, n_prev, dist_l, L - l, self.dA[l], self.dH[l - 1], K,
                                          rs_l, self.cs, accumulate=False, ws=ws_bwd, relu_H=relu_h, src_prefix=pre_l)
        self._join_side()
        return self.grads

    def _source_filter(self, n_fwd: int):
        """(dist, src_prefix) of a backward aggregation whose forward call computed the first n_fwd ring-sorted vertices:
        nothing when those are all vertices, the id prefix on a (distance, id)-numbered partition, else the distances."""
        if n_fwd == self.n:
            return None, -1
        if self.prefix_numbered:
            return None, n_fwd
        return self.dist, -1

    def _backward_transform_first(self, l: int):
        """Layer l in the exchanged order, Z = rs * Agg(H_{l-1} W_neigh) + H_{l-1} W_self + b: the self half takes dZ as
        it is, the neighbour half takes dP = Agg^T(rs * dZ) (one backward aggregation, dims[l] wide); the two input
        gradients meet in front of the previous layer's ReLU."""
        L, p, gr, K, N = self.L, self.params[l - 1], self.grads[l - 1], self.dims[l - 1], self.dims[l]
        nl, n_prev = self.n_rows_of_layer(l), self.n_rows_of_layer(l - 1)
        need_in = l > 1
        gt_l, rs_l = (self.gt, self.rs) if self.layer_sampling is None else (self.gt_l[l], self.rs_l[l])
        dist_l, pre_l = self._source_filter(nl)
        sage = self.kind == "sage"
        # the gradients of the self half (or, GCN, of the bias) need dZ only: beside the backward aggregation
        if sage:
            self._call_beside(f"linear_bwd_{l}", B.gnn_linear_bwd, self.rows, nl, self.dH[l], None, False, self.H[l - 1], None, K,
                              p["W_self"], None, gr["dW_self"], None, gr["dbias"], None, None)
            if need_in and l not in self.gf_layers:
                self._call(f"linear_bwd_{l}_input_self", B.gnn_linear_bwd_input, self.rows, nl, self.dH[l], N, p["W_self"], K, 0, None,
                           self.dH[l - 1], ws=self.ws)
        else:
            self._call_beside(f"linear_bwd_{l}", B.gnn_bias_grad, self.rows, nl, self.dH[l], N, gr["dbias"])
        self._call(f"spmm_bwd_{l}", B.gnn_masked_spmm_bwd, gt_l, self.rows, n_prev, dist_l, L - l, self.dH[l], self.dP[l], N,
                   rs_l, self.cs, accumulate=False, ws=self.ws if 4 * nl >= self.n else None, src_prefix=pre_l)
        self._call_beside(f"linear_bwd_{l}_neigh", B.gnn_linear_bwd, self.rows, n_prev, self.dP[l], None, False, self.H[l - 1], None, K,
                          p["W_neigh"], None, gr["dW_neigh"], None, self._dbias_unused[:N], None, None)
        if need_in and l in self.gf_layers:
            # both halves in one product: dP W_neigh^T for every row of R_{l-1} plus dZ W_self^T for the rows of R_l, masked in
            # front of layer l-1's ReLU in the store
            self._call(f"linear_bwd_{l}_input", B.gnn_linear_bwd_input2, self.rows, n_prev, self.dP[l], p["W_neigh"], self.dH[l],
                       p["W_self"], nl, N, K, self.H[l - 1], self.dH[l - 1], ws=self.ws)
        elif need_in:
            # dP W_neigh^T for every row of R_{l-1}, added (GraphSAGE) to the dZ W_self^T that the rows of R_l already
            # hold and masked in front of layer l-1's ReLU, all in the product's store: dH_{l-1} leaves masked
            self._call(f"linear_bwd_{l}_input", B.gnn_linear_bwd_input, self.rows, n_prev, self.dP[l], N, p["W_neigh"], K,
                       nl if sage else 0, self.H[l - 1], self.dH[l - 1], ws=self.ws)

    def step(self, labels: torch.Tensor):
        """One pass of the whole hot path: active sets, forward, loss, backward."""
        self.build_active_sets()
        if self.layer_sampling is not None:
            self.build_layer_masks()
        self.forward(labels)
        self.backward()
        return self.loss

    def product_costs(self) -> dict:
        """call name -> (layer, direction, flops, operand bytes with every operand read or written once) of each
        feature-transform product of a step, in the order this model runs them (host-side bookkeeping for the benchmark's
        rooflines; the bias-only calls are left out)."""
        es = torch.empty(0, dtype=self.dtype).element_size()
        sage = self.kind == "sage"
        srcs = 2 if sage else 1
        out = {}

        def put(name, l, direction, flops, nbytes):
            out[name] = {"layer": l, "direction": direction, "flops": float(flops), "bytes": float(nbytes) * es}

        for l in range(1, self.L + 1):
            K, N = self.dims[l - 1], self.dims[l]
            nl = self.n_rows_of_layer(l)
            n_prev = self.n_rows_of_layer(l - 1) if l > 1 else self.n
            need_in = l > 1
            one = lambda m: (2.0 * m * K * N, m * (K + N))      # one product over m rows: flops, elements moved
            both_in = (2.0 * N * K * (n_prev + (nl if sage else 0)),          # the two-source input gradient: G and dZ in,
                       n_prev * N + (nl * N if sage else 0) + 2 * n_prev * K)   # the ReLU mask in, dH_{l-1} out
            if l in self.tf_layers:
                put(f"linear_pre_{l}", l, "fwd", *one(n_prev))
                if sage:
                    put(f"linear_fwd_{l}", l, "fwd", *one(nl))
                    put(f"linear_bwd_{l}", l, "bwd", *one(nl))
                    if need_in and l not in self.gf_layers:
                        put(f"linear_bwd_{l}_input_self", l, "bwd", *one(nl))
                put(f"linear_bwd_{l}_neigh", l, "bwd", *one(n_prev))
                if need_in and l in self.gf_layers:
                    put(f"linear_bwd_{l}_input", l, "bwd", *both_in)
                elif need_in:
                    put(f"linear_bwd_{l}_input", l, "bwd", 2.0 * n_prev * N * K, n_prev * (N + 2 * K) + (nl * K if sage else 0))
                continue
            if l not in self.fused_layers:
                put(f"linear_fwd_{l}", l, "fwd", 2.0 * nl * K * N * srcs, nl * (K * srcs + N))
            if l in self.gf_layers:
                if l in self.fused_layers:
                    put(f"linear_bwd_{l}", l, "bwd", *one(nl))
                    put(f"linear_bwd_{l}_neigh", l, "bwd", *one(n_prev))
                else:
                    put(f"linear_bwd_{l}", l, "bwd", 2.0 * nl * K * N * srcs, nl * (N + K * srcs))
                put(f"linear_bwd_{l}_input", l, "bwd", *both_in)
            elif need_in and self.side is not None:
                put(f"linear_bwd_{l}", l, "bwd", 2.0 * nl * K * N * srcs, nl * (N + K * srcs))
                put(f"linear_bwd_{l}_input", l, "bwd", *one(nl))
                if sage:
                    put(f"linear_bwd_{l}_input_self", l, "bwd", *one(nl))
            else:
                f = 2.0 * nl * K * N * srcs
                put(f"linear_bwd_{l}", l, "bwd", f * (2 if need_in else 1), nl * (N + K * srcs) + (nl * K * srcs if need_in else 0))
        return out

    def aggregated_edges(self) -> dict:
        """Edges visited per layer by the forward and the backward aggregation of the paper's order (host-side
        bookkeeping from row_ptr; used by the benchmark's edges/s metric).  A first layer in the exchanged order aggregates
        backward as well; that is NOT counted: the exchanged order must not raise the metric by doing more, narrower sums."""
        rp = self.g.row_ptr.long()
        ring = self.ring_ids.long()
        out = {}
        for l in range(1, self.L + 1):
            rows = ring[: self.n_rows_of_layer(l)]
            if self.layer_sampling is not None:      # only the entries the layer's mask keeps are aggregated
                fwd = int(self.kept_l[l][rows].sum().item())
            else:
                fwd = int((rp[rows + 1] - rp[rows]).sum().item())
            bwd = 0
            if l > 1:
                # transposed rows of R_{l-1}; entries v with dist(v) <= L - l are exactly the forward edges of R_l
                bwd = fwd
            out[l] = {"fwd": fwd, "bwd": bwd}
        return out


class ResSAGEPlus:
    """The deep residual GraphSAGE of the paper's evaluation (ResSAGE+: GraphSAGE layers, residual connections,
    pre-activation by layer normalisation and ReLU) over one partition under one-hop masking:
        h_1 = SAGE_1(h_0);   h_l = h_{l-1} + SAGE_l(ReLU(LN_l(h_{l-1})))  (1 < l < L);   out = SAGE_L(ReLU(LN_L(h_{L-1})))
    Layer l produces the rows R_l, its pre-activation runs over R_{l-1}.  Call order only; every step runs in the
    library's kernels.

    params       per layer W_neigh, W_self [K,N], bias [N]; from the second layer on ln_gamma, ln_beta [K]
    recompute    activation recomputation: the forward pass keeps only h_l (one matrix per layer); the backward pass
                 makes the pre-activation t_l and the aggregate A_l of a layer again (one more normalisation and one
                 more forward aggregation per layer) in two buffers shared by all layers, instead of 3 matrices per layer
    """

    def __init__(self, graph: B.Graph, graph_t: B.Graph, targets: torch.Tensor, params: list, dtype=torch.float32,
                 prefix_numbered: bool = False, recompute: bool = False):
        self.g, self.gt, self.targets, self.dtype = graph, graph_t, targets, dtype
        self.n, self.L = graph.n_rows, len(params)
        self.prefix_numbered, self.recompute = prefix_numbered, recompute
        self._prefix_checked, self.rs = False, None
        self.ws = B.Workspace()
        self.dims = [params[0]["W_neigh"].shape[0]] + [p["W_neigh"].shape[1] for p in params]
        assert all(d == self.dims[1] for d in self.dims[1:-1]), "the residual connection needs equal hidden widths"
        self.params = []
        for l, p in enumerate(params):
            q = {"W_neigh": p["W_neigh"].to(dtype).contiguous(), "W_self": p["W_self"].to(dtype).contiguous(),
                 "bias": p["bias"].float().contiguous()}
            if l > 0:
                q["ln_gamma"], q["ln_beta"] = p["ln_gamma"].float().contiguous(), p["ln_beta"].float().contiguous()
            self.params.append(q)
        self.ld = [row_stride(d, dtype) for d in self.dims]
        dev, n, L = targets.device, self.n, self.L
        z = lambda w: torch.zeros(n, w, dtype=dtype, device=dev)
        self.H = [None] + [z(self.ld[l]) for l in range(1, L + 1)]
        n_buf = min(2, L) if recompute else L        # with recomputation all layers share the buffers of layers 1 and 2
        self.T = [None, None] + [z(self.ld[l - 1]) for l in range(2, n_buf + 1)]
        self.A = [None] + [z(self.ld[l - 1]) for l in range(1, n_buf + 1)]
        hid = self.ld[1] if L > 1 else self.ld[0]
        # gradients: dH ping-pong (hidden width), the logits' gradient, dA and dT (shared by all layers)
        self.dH = [z(hid), z(hid)]
        self.dlogits = z(self.ld[L])
        self.dA, self.dT = (z(hid), z(hid)) if L > 1 else (None, None)
        self.grads = []
        for l, p in enumerate(self.params):
            gdict = {"dW_neigh": torch.zeros_like(p["W_neigh"], dtype=torch.float32), "dW_self": torch.zeros_like(p["W_self"], dtype=torch.float32),
                     "dbias": torch.zeros_like(p["bias"])}
            if l > 0:
                gdict["dln_gamma"], gdict["dln_beta"] = torch.zeros_like(p["ln_gamma"]), torch.zeros_like(p["ln_beta"])
            self.grads.append(gdict)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.trace = None

    _call = MaskedGNN._call

    def build_active_sets(self):
        self.dist, self.ring_ids, self.hop_offsets, self.hop = self._call("active_sets", B.gnn_build_active_sets, self.g, self.targets, self.L, ws=self.ws, gt=self.gt)
        if self.rs is None:      # depends on the graph alone: made once, not per step
            self.rs = B.gnn_norm_scales(B.GNN_NORM_MEAN, self.n, row_ptr=self.g.row_ptr)
        if self.prefix_numbered and not self._prefix_checked:
            self._prefix_checked = True
            n_all = int(self.hop[-1])
            if not torch.equal(self.ring_ids[:n_all], torch.arange(n_all, dtype=torch.int32, device=self.ring_ids.device)):
                raise ValueError("prefix_numbered was promised but the ring-sorted ids are not 0 .. n-1")
        self.rows = None if self.prefix_numbered else self.ring_ids
        return self.hop

    def n_rows_of_layer(self, l: int) -> int:
        return int(self.hop[self.L - l + 1])

    def set_input(self, H0: torch.Tensor):
        assert H0.dtype == self.dtype and H0.shape[0] == self.n and H0.stride(0) == self.ld[0]
        self.H[0] = H0

    def _slot(self, l):
        """index of the buffers that hold t_l / A_l"""
        return l if not self.recompute else min(l, 2)

    def _pre_and_aggregate(self, l, tag):
        """t_l = ReLU(LN_l(h_{l-1})) over R_{l-1} (layer 1: the input itself), A_l = mean aggregation of t_l over R_l."""
        p, K, nl = self.params[l - 1], self.dims[l - 1], self.n_rows_of_layer(l)
        if l == 1:
            src = self.H[0]
        else:
            src = self.T[self._slot(l)]
            self._call(f"ln_fwd_{l}{tag}", B.gnn_layer_norm_relu_fwd, self.rows, self.n_rows_of_layer(l - 1), self.H[l - 1], K,
                       p["ln_gamma"], p["ln_beta"], src)
        A = self.A[self._slot(l)]
        self._call(f"spmm_fwd_{l}{tag}", B.gnn_masked_spmm_fwd, self.g, self.rows, nl, src, A, K, self.rs, None, ws=self.ws)
        return src, A

    def forward(self, labels: torch.Tensor) -> torch.Tensor:
        for l in range(1, self.L + 1):
            p, K, nl = self.params[l - 1], self.dims[l - 1], self.n_rows_of_layer(l)
            src, A = self._pre_and_aggregate(l, "")
            self._call(f"linear_fwd_{l}", B.gnn_linear_fwd, self.rows, nl, A, src, K, p["W_neigh"], p["W_self"], p["bias"], self.H[l],
                       relu=False, ws=self.ws)
            if 1 < l < self.L:
                self._call(f"residual_{l}", B.gnn_add_rows, self.rows, nl, self.H[l - 1], self.H[l], self.dims[l])
        nt = self.n_rows_of_layer(self.L)
        self._call("softmax_ce", B.gnn_softmax_ce, self.rows, nt, self.H[self.L], self.dims[self.L], labels, self.dlogits, self.loss, ws=self.ws)
        return self.loss

    def backward(self):
        L = self.L
        dH = self.dlogits
        for l in range(L, 0, -1):
            p, gr, K, nl = self.params[l - 1], self.grads[l - 1], self.dims[l - 1], self.n_rows_of_layer(l)
            need_in = l > 1
            if self.recompute and l > 1:
                src, A = self._pre_and_aggregate(l, "_again")
            else:
                src, A = (self.H[0] if l == 1 else self.T[self._slot(l)]), self.A[self._slot(l)]
            self._call(f"linear_bwd_{l}", B.gnn_linear_bwd, self.rows, nl, dH, None, False, A, src, K, p["W_neigh"], p["W_self"],
                       gr["dW_neigh"], gr["dW_self"], gr["dbias"], self.dA if need_in else None, self.dT if need_in else None, ws=self.ws)
            if not need_in:
                break
            n_prev = self.n_rows_of_layer(l - 1)
            # every vertex was a forward row: the filter keeps everything; on a (distance, id)-numbered partition the
            # forward rows are an id prefix; else their distances decide
            dist_l, pre_l = (None, -1) if nl == self.n else ((None, nl) if self.prefix_numbered else (self.dist, -1))
            # rows of R_l already hold dZ W_self^T: add the aggregated part; the next ring starts from zero
            self._call(f"spmm_bwd_{l}", B.gnn_masked_spmm_bwd, self.gt, self.rows, nl, dist_l, L - l, self.dA, self.dT, K,
                       self.rs, None, accumulate=True, ws=None, src_prefix=pre_l)
            if n_prev > nl:
                self._call(f"spmm_bwd_{l}_ring", B.gnn_masked_spmm_bwd, self.gt, self.ring_ids[nl:], n_prev - nl, dist_l, L - l, self.dA,
                           self.dT, K, self.rs, None, accumulate=False, ws=None, src_prefix=pre_l)
            out = self.dH[l % 2]
            self._call(f"ln_bwd_{l}", B.gnn_layer_norm_relu_bwd, self.rows, n_prev, self.dT, src, self.H[l - 1], K, p["ln_gamma"],
                       dH if l < L else None, nl if l < L else 0, out, gr["dln_gamma"], gr["dln_beta"], ws=self.ws)
            dH = out
        return self.grads

    def step(self, labels: torch.Tensor):
        self.build_active_sets()
        self.forward(labels)
        self.backward()
        return self.loss

    def aggregated_edges(self) -> dict:
        """Edges visited per layer by the forward and the backward aggregation (and by the recomputed forward)."""
        rp = self.g.row_ptr.long()
        ring = self.ring_ids.long()
        out = {}
        for l in range(1, self.L + 1):
            rows = ring[: self.n_rows_of_layer(l)]
            fwd = int((rp[rows + 1] - rp[rows]).sum().item())
            out[l] = {"fwd": fwd, "bwd": fwd if l > 1 else 0, "again": fwd if (self.recompute and l > 1) else 0}
        return out

    def activation_bytes(self) -> int:
        """Bytes of the per-layer activation and gradient buffers this model holds (the memory the recomputation saves)."""
        ts = [t for lst in (self.H[1:], self.T, self.A, self.dH, [self.dlogits, self.dA, self.dT]) for t in lst if t is not None]
        return sum(t.numel() * t.element_size() for t in ts)
