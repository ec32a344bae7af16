/*
 * gnnhot - one GPU's share of a full-neighbourhood GNN training step under one-hop graph
 * masking, for AMD MI355X (gfx950).  C ABI; every kernel behind it is hand-written HIP.
 *
 * The problem (paper sections 2.1, 5.3 and 6).  A partition holds its target ("inner")
 * vertices T and a preloaded multi-hop halo.  ONE one-hop graph is reused by all L layers;
 * row v of its CSR lists the vertices u whose hidden vectors v aggregates.  With
 * dist(v) = hops from T to v along rows, layer l (l = 1..L) only produces the rows
 *     R_l = { v : dist(v) <= L - l },       R_L = T,
 * because nothing else can reach the targets' outputs (the per-layer mask of section 6,
 * figure 7c steps 4-5).  Every layer is the two halves of the equation of section 2.1:
 *     A_l[v]  = rs[v] * sum_{u in row(v)} cs[u] * H_{l-1}[u]          (aggregation)
 *     H_l[v]  = sigma( A_l[v] W_neigh [+ H_{l-1}[v] W_self] + b )     (feature transform)
 * followed, for training, by the matching backward pass.
 *
 * General rules of this interface
 *   - Pointers are DEVICE pointers unless the name ends in _host.  The gnn_csr struct itself
 *     is read on the host; the arrays it points to are on the device.
 *   - The caller owns every buffer.  The library allocates nothing and keeps no state
 *     between calls.  Calls that need scratch take (ws, ws_bytes): with ws == NULL the call
 *     only writes the number of bytes it needs to *ws_bytes and returns GNN_OK; otherwise
 *     *ws_bytes is the size of ws, which must be 256-byte aligned.  ws contents are
 *     meaningless between calls.
 *   - `stream` is a hipStream_t (NULL = the default stream).  All work is enqueued on it and
 *     nothing synchronises, except where a *_host output is requested (documented below).
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS (int64).
 *     dtype GNN_F32: float storage and arithmetic.  dtype GNN_BF16: bfloat16 storage,
 *     float accumulation; weight and bias gradients are float in both cases.
 *   - Rows that a call is not asked to produce are neither read nor written.
 *   - Every function returns a gnn_status.  Nothing throws, aborts or prints.
 *     gnn_last_error() gives a message for the calling thread's last failure.
 *   - Index type is int32; nnz must be < 2^31.  Addresses are formed in 64 bits.
 */
#ifndef GNNHOT_H
#define GNNHOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gnn_status {
    GNN_OK = 0,
    GNN_ERR_INVALID_ARG = 1, /* null where not allowed, negative size, misaligned ws, L < 1, fanout < 0 */
    GNN_ERR_SHAPE = 2,       /* leading dimension smaller than the width, inconsistent sizes */
    GNN_ERR_WORKSPACE = 3,   /* *ws_bytes smaller than required */
    GNN_ERR_UNSUPPORTED = 4, /* unknown dtype, nnz >= 2^31, hops != 1, width over the limit */
    GNN_ERR_HIP = 5          /* a HIP runtime call or kernel launch failed */
} gnn_status;

typedef enum gnn_dtype { GNN_F32 = 0, GNN_BF16 = 1 } gnn_dtype;

typedef enum gnn_norm { GNN_NORM_MEAN = 1, GNN_NORM_SYM = 2 } gnn_norm;

/* Properties of a graph that the caller guarantees (gnn_csr.flags). */
typedef enum gnn_csr_flags {
    GNN_CSR_SORTED_COLUMNS = 1 /* within every row the columns are in ascending order (repeats allowed) */
} gnn_csr_flags;

/* One-hop graph in CSR form.  Columns of a row may be in any order unless flags says otherwise;
 * a repeated column counts as often as it appears. */
typedef struct gnn_csr {
    int32_t n_rows;
    int32_t n_cols;
    int64_t nnz;
    const int32_t *row_ptr; /* device, [n_rows + 1], row_ptr[0] = 0, row_ptr[n_rows] = nnz */
    const int32_t *col_idx; /* device, [nnz], each in [0, n_cols) */
    int32_t flags;          /* OR of gnn_csr_flags; 0 promises nothing.  A promise that does not hold
                               gives wrong sums (never an out-of-bounds access). */
    const uint32_t *edge_keep; /* device, nullable: one bit per entry of col_idx (bit p % 32 of word p / 32);
                               entries whose bit is 0 are skipped by the aggregation calls - the per-layer mask of
                               layer-wise sampling (section 5.2).  Read by gnn_masked_spmm_fwd / _bwd only. */
} gnn_csr;

int32_t gnn_version(void);
const char *gnn_last_error(void);

/*
 * Per-layer active vertex sets (section 6: step 1 extracts the multi-hop dependency starting
 * from the inner vertices; step 4 generates the per-layer mask).  Level-synchronous frontier
 * expansion from T over CSR rows, L levels deep.
 *   gt               nullable: the transpose of g (same sizes; entry (u, v) for every entry (v, u) of g;
 *                    g itself for a symmetric graph).  With it a level may run from the unreached
 *                    vertices instead of from the frontier (each looks through its row of gt for a
 *                    frontier vertex and stops at the first), chosen on the device per level from
 *                    the exact edge counts of the two directions.  The outputs are the same with and
 *                    without it; a gt that is not the transpose gives wrong sets (never an
 *                    out-of-bounds access).
 *   targets          [n_targets] vertex ids; repeats are allowed (set semantics);
 *                    ids outside [0, n_rows) are ignored
 *   dist             out [n_rows]: hop distance, -1 if farther than L hops or unreachable
 *   ring_ids         out [n_rows] capacity: vertices ordered by (dist, id); only the first
 *                    hop_offsets[L+1] entries are written
 *   hop_offsets      out [L+2], device: ring j = ring_ids[hop_offsets[j] .. hop_offsets[j+1]);
 *                    the rows of layer l are the prefix ring_ids[0 .. hop_offsets[L-l+1])
 *   hop_offsets_host optional host copy of hop_offsets; when non-NULL the call waits for the
 *                    stream before returning
 * Requires g->n_rows == g->n_cols.  All outputs are bit-exact functions of the inputs.
 */
int32_t gnn_build_active_sets(const gnn_csr *g, const gnn_csr *gt, const int32_t *targets, int32_t n_targets,
                              int32_t L, int32_t *dist, int32_t *ring_ids, int64_t *hop_offsets,
                              int64_t *hop_offsets_host, void *ws, size_t *ws_bytes, void *stream);

/*
 * Normalisation factors for the aggregation of the two models the paper trains (section 8.1):
 * GNN_NORM_MEAN  out[v] = 1 / len[v], 0 for an empty row   (GraphSAGE mean aggregator)
 * GNN_NORM_SYM   out[v] = len[v]^(-1/2), 0 if len[v] = 0   (GCN; len counts the self loop)
 * len[v] is taken from `len` when non-NULL, else row_ptr[v+1] - row_ptr[v].
 */
int32_t gnn_norm_scales(int32_t norm, const int32_t *len, const int32_t *row_ptr, int32_t n, float *out,
                        void *stream);

/*
 * Masked aggregation, forward (section 2.1, first half of the layer equation; section 6 mask):
 *     Y[v, 0:F] = row_scale[v] * sum_{u in row(v)} col_scale[u] * X[u, 0:F]     for v in rows
 *   rows        [n_active] row ids, or NULL for rows 0 .. n_active-1
 *   X           [g->n_cols, ldx], Y [g->n_rows, ldy]; X and Y must not overlap
 *   row_scale, col_scale   float vectors or NULL (= 1)
 * An empty row gives 0.  Columns F..ldy of Y are not written.  Results do not depend on launch
 * order (no floating-point atomics): the same call gives the same bits.  Row ids in `rows` must
 * lie in [0, g->n_rows); they are not checked.
 *
 * Workspace (optional).  ws_bytes == NULL: no workspace, one kernel launch that gathers whole rows.
 * With a workspace the call may take the column-blocked route for dense graphs whose gathered
 * matrix is far larger than a cache (on average at least 8 entries of a row per column block, columns sorted:
 * GNN_CSR_SORTED_COLUMNS, 16-byte aligned operands): the neighbour-id range is cut into 8 blocks
 * per pass, workgroup i works on block i mod 8 (the compute die it runs on), so each die's L2
 * only ever holds one eighth of a 256-byte-wide feature slab; the per-block partial sums (float)
 * go to ws and are added in block order.  The size query (ws == NULL) reports 0 when the route
 * does not apply; the sums of the two routes differ by float rounding only.
 */
int32_t gnn_masked_spmm_fwd(const gnn_csr *g, const int32_t *rows, int32_t n_active,
                            const void *X, int64_t ldx, void *Y, int64_t ldy, int32_t F, int32_t dtype,
                            const float *row_scale, const float *col_scale,
                            void *ws, size_t *ws_bytes, void *stream);

/*
 * (Helper; no passage of the paper.)  The compute die (XCC id, 0..7) that each of the first n_ids <= 64 workgroups of a
 * 16 x 4 probe grid ran on, in dispatch order (x fastest), to xcc_ids_host (HOST memory); *holds_host (nullable, host) = 1
 * if workgroup i ran on the die of workgroup i mod 8 and the first eight dies are all different - the dispatch order the
 * column-blocked route of the aggregation calls is built on.  The library asks the same question once per device before
 * it takes that route for the first time (the size query then reports 0 if the answer is no).  Launches on the null
 * stream and waits.
 */
int32_t gnn_die_mapping(int32_t *xcc_ids_host, int32_t n_ids, int32_t *holds_host);

/*
 * Masked aggregation added onto the output (section 2.1's layer equation with the neighbour sum and the weight
 * product exchanged: sum_u (x_u W) instead of (sum_u x_u) W, the cheaper order when the layer narrows its input):
 *     Y[v, 0:F] = act( Y[v, 0:F] + row_scale[v] * sum_{u in row(v)} col_scale[u] * X[u, 0:F] )     for v in rows
 *   X     the already transformed rows (x_u W_neigh), Y on entry the self term (x_v W_self + bias) of the same rows
 *   bias  float [F] or NULL.  Non-NULL: the layer has no self term (GCN); what Y holds on entry is ignored and the
 *         listed rows start from bias instead
 *   relu  1: act = max(., 0), 0: identity
 * Everything else (row list, scales, determinism, workspace, errors) as in gnn_masked_spmm_fwd; a row without
 * entries still gets its activation.
 */
int32_t gnn_masked_spmm_fwd_add(const gnn_csr *g, const int32_t *rows, int32_t n_active,
                                const void *X, int64_t ldx, void *Y, int64_t ldy, int32_t F, int32_t dtype,
                                const float *row_scale, const float *col_scale, const float *bias, int32_t relu,
                                void *ws, size_t *ws_bytes, void *stream);

/*
 * Masked aggregation, backward = the adjoint of the forward map, in gather form over the
 * TRANSPOSED graph gT (row u of gT lists every v that aggregates u; for a symmetric graph pass
 * the same arrays):
 *     dX[u, 0:F] (+)= col_scale[u] * sum_{v in rowT(u), active(v)} row_scale[v] * dY[v, 0:F]   for u in out_rows
 *   active(v)   (dist == NULL or 0 <= dist[v] <= max_active_dist) and (src_prefix < 0 or v < src_prefix): v was a
 *               row of the forward call.  src_prefix is the form of the test for a partition numbered by (distance,
 *               id) (gnn_extract_partition): the forward rows were the ids 0 .. src_prefix-1, so dist can stay NULL;
 *               when gT promises GNN_CSR_SORTED_COLUMNS every row is simply cut at its first entry >= src_prefix
 *               (a binary search per row instead of a test per entry), otherwise the entries are tested one by one.
 *               -1: no such test.
 *   accumulate  0: overwrite dX rows, 1: add to them
 *   relu_H      nullable: the activations H of the layer whose gradient dX is (same rows, F columns, leading
 *               dimension ld_relu).  What is stored (after the addition of accumulate) is zeroed where H <= 0, i.e. dX
 *               leaves the call as the gradient in front of that layer's ReLU (the chain rule's next factor), and
 *               gnn_linear_bwd of that layer is then called with relu = 0.  The call that writes a row LAST must be the
 *               one that masks it.
 * Same determinism and the same optional workspace as the forward call.
 */
int32_t gnn_masked_spmm_bwd(const gnn_csr *gT, const int32_t *out_rows, int32_t n_out,
                            const int32_t *dist, int32_t max_active_dist, int32_t src_prefix,
                            const void *dY, int64_t lddy, void *dX, int64_t lddx, int32_t F, int32_t dtype,
                            const float *row_scale, const float *col_scale, int32_t accumulate,
                            const void *relu_H, int64_t ld_relu,
                            void *ws, size_t *ws_bytes, void *stream);

/*
 * Feature transform, forward (section 2.1, second half: weights, then the activation):
 *     Z[v] = A_neigh[v, 0:K] W_neigh (+ X_self[v, 0:K] W_self) + bias,   H_out[v, 0:N] = relu ? max(Z, 0) : Z
 * for v in rows (NULL = 0 .. n_active-1).
 *   A_neigh, X_self  [*, ld_in]; X_self and W_self both NULL for a GCN layer
 *   W_neigh, W_self  [K, N] dense row-major, same dtype as the activations
 *   bias             float [N] or NULL
 * MFMA GEMM (fp32 or bf16 inputs, float accumulation).  K, N <= 4096.
 */
int32_t gnn_linear_fwd(const int32_t *rows, int32_t n_active,
                       const void *A_neigh, const void *X_self, int64_t ld_in, int32_t K,
                       const void *W_neigh, const void *W_self, const float *bias, int32_t N,
                       void *H_out, int64_t ld_out, int32_t relu, int32_t dtype,
                       void *ws, size_t *ws_bytes, void *stream);

/*
 * A layer's forward pass in ONE kernel (section 2.1, both halves of the layer equation; the mask of section 6 through the
 * row list): the aggregate of a tile of rows is formed in on-chip memory and multiplied by the weights there,
 *     H_out[v, 0:N] = act( (row_scale[v] * sum_{u in row(v)} col_scale[u] * X[u, 0:K]) W_neigh (+ X[v, 0:K] W_self) + bias )
 * for v in rows, so the aggregate A_l of gnn_masked_spmm_fwd is neither written nor read back.  The aggregate is rounded
 * to `dtype` before the product, exactly as if it had been stored: the result equals that of the two calls up to the
 * order of additions.  Arguments as in gnn_masked_spmm_fwd and gnn_linear_fwd (W_self NULL: no self term).
 * Limits: input rows of 128 to 512 bytes (K rounded up to 32 bytes), output rows of at most 512 bytes, X rows 16-byte
 * aligned, no per-layer edge mask; anything else returns GNN_ERR_UNSUPPORTED (use the two calls).
 * A backward pass cannot rely on A_l then: dW_neigh = X^T Agg^T(dZ) (gnn_masked_spmm_bwd of dZ, then gnn_linear_bwd with X).
 * Workspace: (ws, ws_bytes) protocol (transposed, zero-padded weights).
 */
int32_t gnn_fused_layer_fwd(const gnn_csr *g, const int32_t *rows, int32_t n_active, const void *X, int64_t ldx, int32_t K,
                            const float *row_scale, const float *col_scale, const void *W_neigh, const void *W_self,
                            const float *bias, int32_t N, void *H_out, int64_t ld_out, int32_t relu, int32_t dtype,
                            void *ws, size_t *ws_bytes, void *stream);

/*
 * gnn_linear_fwd for callers that cannot allocate device memory and so have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * (ws, ws_bytes), same kernels, same bits.  The two transposed weight copies go to an array that the library
 * holds in device memory on every GPU it runs on until the process ends (8 MiB); no hipMalloc / hipFree or other
 * allocating call is made.
 *   limit      N * round_up(K, 16 bytes) * element size <= 4 MiB per weight matrix (1024 x 1024 floats,
 *              2048 x 1024 bf16); beyond it GNN_ERR_UNSUPPORTED - use gnn_linear_fwd
 *   set-up     the first call on a device looks up the array's address on that device (the device must be
 *              current, as for every call); a call with n_active == 0 does only that and can serve as set-up
 *              before a capture starts
 *   sharing    all calls on one GPU use the same array: calls that overlap there (two streams, two threads)
 *              race; calls on one stream are ordered and safe.  Nothing has to be cleared between calls: every
 *              call rewrites what it reads.
 */
int32_t gnn_linear_fwd_static(const int32_t *rows, int32_t n_active,
                              const void *A_neigh, const void *X_self, int64_t ld_in, int32_t K,
                              const void *W_neigh, const void *W_self, const float *bias, int32_t N,
                              void *H_out, int64_t ld_out, int32_t relu, int32_t dtype, void *stream);

/*
 * Feature transform, backward (chain rule of the above), for v in rows:
 *     dZ[v]    = relu ? dH_out[v] * [H_out[v] > 0] : dH_out[v]
 *     dW_neigh = sum_v A_neigh[v]^T dZ[v]      dW_self = sum_v X_self[v]^T dZ[v]      dbias = sum_v dZ[v]
 *     dA_neigh[v, 0:K] = dZ[v] W_neigh^T       dX_self[v, 0:K] = dZ[v] W_self^T
 *   dH_out, H_out     [*, ld_out]; H_out may be NULL when relu == 0
 *   dW_neigh, dW_self float [K, N], overwritten; dbias float [N], overwritten
 *   dA_neigh, dX_self [*, ld_din], rows in the list overwritten; either may be NULL to skip it
 *                     (the first layer needs no input gradient)
 * Reductions over rows use a fixed split and order (no atomics).
 */
int32_t gnn_linear_bwd(const int32_t *rows, int32_t n_active,
                       const void *dH_out, const void *H_out, int64_t ld_out, int32_t relu,
                       const void *A_neigh, const void *X_self, int64_t ld_in, int32_t K,
                       const void *W_neigh, const void *W_self, int32_t N,
                       float *dW_neigh, float *dW_self, float *dbias,
                       void *dA_neigh, void *dX_self, int64_t ld_din, int32_t dtype,
                       void *ws, size_t *ws_bytes, void *stream);

/*
 * Input gradient of one half of a layer in the exchanged order, finished in the product's own store:
 *     dX[v, 0:K] = [relu_H[v, 0:K] > 0] * ( dZ[v, 0:N] W^T  +  (i < n_accumulate ? dX[v, 0:K] : 0) )      v = rows[i]
 * (the neighbour half dP W_neigh^T reaches every row of R_{l-1}; the rows of R_l, listed first, already hold the self
 * half dZ W_self^T; relu_H = H_{l-1} puts the sum in front of the previous layer's ReLU).
 *   W        [K, N] as in gnn_linear_fwd;  relu_H NULL: no mask, then n_accumulate must be 0
 * Rounding with bf16 storage: the product is rounded to bf16, added to the stored dX in float and the sum rounded again -
 * the bits that storing the two halves separately and adding them would give (gnn_linear_bwd_input2 below forms both
 * halves in one float accumulator and rounds once).
 * Workspace: (ws, ws_bytes) size-query protocol.
 */
int32_t gnn_linear_bwd_input(const int32_t *rows, int32_t n_active, const void *dZ, int64_t lddz, int32_t N, const void *W,
                             int32_t K, int32_t n_accumulate, const void *relu_H, int64_t ld_relu, void *dX, int64_t lddx,
                             int32_t dtype, void *ws, size_t *ws_bytes, void *stream);

/*
 * Input gradient of a GraphSAGE layer from its AGGREGATED output gradient (chain rule of section 2.1's layer equation
 * with the linear steps of the neighbour half exchanged: Agg^T(dZ W_neigh^T) = Agg^T(dZ) W_neigh^T), one product:
 *     dX[v, 0:K] = [relu_H[v, 0:K] > 0] * ( dG[v, 0:N] W_neigh^T  +  (i < n_self ? dZ[v, 0:N] W_self^T : 0) )     v = rows[i]
 *   dG       the layer's output gradient aggregated backwards (gnn_masked_spmm_bwd of dZ): one row for every vertex of
 *            R_{l-1}, listed in `rows`
 *   dZ       the layer's output gradient itself; only the first n_self listed rows (those of R_l) have one.  dG and dZ
 *            share the leading dimension ldd; the rows of dZ past the first n_self listed ones must be addressable
 *            (they are fetched and discarded)
 *   W_neigh, W_self   [K, N] as in gnn_linear_fwd;  n_self == 0: no self half (dZ, W_self may be NULL)
 *   relu_H   nullable: no mask
 * Against gnn_linear_bwd's two input gradients plus an accumulating backward aggregation this saves one product pass
 * over dZ, the aggregation's re-read of dX, and gathers N instead of K columns.  Workspace: (ws, ws_bytes) protocol.
 */
int32_t gnn_linear_bwd_input2(const int32_t *rows, int32_t n_active, const void *dG, const void *W_neigh, const void *dZ,
                              const void *W_self, int32_t n_self, int64_t ldd, int32_t N, int32_t K, const void *relu_H,
                              int64_t ld_relu, void *dX, int64_t lddx, int32_t dtype, void *ws, size_t *ws_bytes, void *stream);

/*
 * Bias gradient alone (chain rule of section 2.1's layer equation, the bias term):
 * dbias[0:N] = sum over the listed rows of dZ[v, 0:N] (fixed order, no atomics) - for a layer in
 * the exchanged order without a self term, whose gnn_linear_bwd call runs on another matrix (dP) than dZ.
 * Workspace: (ws, ws_bytes) size-query protocol.  N <= 4096.
 */
int32_t gnn_bias_grad(const int32_t *rows, int32_t n_active, const void *dZ, int64_t lddz, int32_t N, int32_t dtype,
                      float *dbias, void *ws, size_t *ws_bytes, void *stream);

/*
 * Node-classification loss on the targets (section 8.1): mean softmax cross-entropy.
 *     loss = mean_i -log softmax(Z[rows[i]])[labels[i]],   dZ[rows[i]] = (softmax - onehot) / n_active
 *   Z, dZ   [*, ldz] / [*, lddz] of `dtype`; dZ may be NULL; C <= 1024 classes
 *   loss    float, device, overwritten
 */
int32_t gnn_softmax_ce(const int32_t *rows, int32_t n_active, const void *Z, int64_t ldz, int32_t C,
                       const int32_t *labels, void *dZ, int64_t lddz, int32_t dtype, float *loss,
                       void *ws, size_t *ws_bytes, void *stream);

/*
 * (Helper; no passage of the paper.)  Bitmap of a vertex set: bit (v & 31) of word v >> 5 is set iff v is in `ids`.
 * bitmap has (n + 31) / 32 words and is overwritten.
 */
int32_t gnn_make_bitmap(const int32_t *ids, int32_t n_ids, int32_t n, uint32_t *bitmap, void *stream);

/*
 * Expansion-aware sampling, boundary only (section 5.3): dependencies between targets are kept
 * whole; of the neighbours OUTSIDE the target set each target keeps at most `fanout`, chosen
 * by a seeded counter-based hash so that the result depends on (seed, v, u) alone:
 *     key(v, u) = mix64(mix64(mix64(seed + hop) ^ v) ^ u),  hop = 1,
 *     mix64 = splitmix64's output function; keep the `fanout` smallest (key, u).
 * For targets[i] the kept neighbours (global ids, ascending) are
 * out_col_idx[out_row_ptr[i] .. out_row_ptr[i+1]).
 * Two calls:
 *   count pass  out_col_idx == NULL: writes out_row_ptr[0..n_targets] and *out_nnz (device);
 *               out_nnz_host, if non-NULL, receives the same number (the call then waits).
 *   fill pass   out_col_idx != NULL: reads out_row_ptr as written by the count pass with the
 *               same arguments and writes the kept ids; entries at or beyond out_capacity
 *               are not written.
 * hops must be 1.  Rows must not repeat a column (a repeated outside neighbour would be counted once per
 * appearance by the count pass but share one key in the fill pass: the two passes would disagree).
 * Bit-exact and independent of the order of `targets`.
 */
int32_t gnn_sample_boundary(const gnn_csr *g, const uint32_t *target_bitmap,
                            const int32_t *targets, int32_t n_targets,
                            int32_t fanout, int32_t hops, uint64_t seed,
                            int32_t *out_row_ptr, int32_t *out_col_idx, int64_t out_capacity,
                            int64_t *out_nnz, int64_t *out_nnz_host,
                            void *ws, size_t *ws_bytes, void *stream);

/*
 * Traversal of expansion-aware sampling (section 5.3.1): from the inner vertices (targets, hop 0) at
 * most `hops` hops outwards; in hop j every vertex selected in hop j-1 keeps at most `fanout` of its
 * neighbours that had not been selected when the hop started - those with the smallest (key, id):
 *   GNN_EAS_DEGREE  the paper's rule, the best-connected candidates (towards the unselected part) first:
 *                   key(u) = -(entries of row u that were unselected when the hop started)
 *   GNN_EAS_HASH    key(v, u) = mix64(mix64(mix64(seed + j) ^ v) ^ u), as in gnn_sample_boundary
 * A vertex is selected in hop j if some vertex of hop j-1 kept it.  Outputs as for
 * gnn_build_active_sets with L = hops ("distance" = hop of selection): dist, ring_ids (selected
 * vertices sorted by (hop, id)), hop_offsets [hops+2] (device), hop_offsets_host (optional; waits).
 * gnn_extract_partition(g, ring_ids, n, dist, hops) then gives the sub-graph of the traversed
 * vertices.  Rows must not repeat a column.  Bit-exact, independent of the order of `targets`.
 */
typedef enum gnn_eas_rule { GNN_EAS_HASH = 0, GNN_EAS_DEGREE = 1 } gnn_eas_rule;

int32_t gnn_eas_traverse(const gnn_csr *g, const int32_t *targets, int32_t n_targets, int32_t hops,
                         int32_t fanout, int32_t rule, uint64_t seed,
                         int32_t *dist, int32_t *ring_ids, int64_t *hop_offsets, int64_t *hop_offsets_host,
                         void *ws, size_t *ws_bytes, void *stream);

/*
 * Layer-wise sampling as a per-layer edge mask (section 5.2: for layer-wise sampling methods the maskings are
 * generated per layer and the layer aggregates through them).  The one-hop graph stays as it is; layer `layer`
 * keeps a subset of the entries of every listed row:
 *   GNN_LAYER_MASK_THRESHOLD  entry (v <- u) is kept iff key(v, u) <= threshold (each edge on its own: a keep
 *                             probability p is threshold = floor(p * 2^64) - 1; all ones keeps everything)
 *   GNN_LAYER_MASK_FANOUT     a row keeps its min(fanout, length) entries with the smallest (key, id)
 * key(v, u) = mix64(mix64(mix64(seed + layer) ^ v) ^ u), the seeded edge hash of gnn_sample_boundary.
 * Outputs: edge_keep (ceil(nnz / 32) words, all written: bit p belongs to the entry at position p of col_idx, the
 * bits of rows that are not listed are 0), kept_len[v] (entries kept in row v, listed rows only;
 * gnn_norm_scales(GNN_NORM_MEAN, kept_len) gives the mean over the kept neighbours); optionally the threshold pair
 * of every row (row_thr_key, row_thr_id: [n_rows] each, both or neither; an entry of row v is kept iff
 * (key, id) <= (row_thr_key[v], row_thr_id[v]); rows that are not listed get a pair that keeps nothing), from
 * which gnn_layer_edge_mask_transposed makes the backward mask.
 * rows NULL => 0 .. n_active-1.  Rows must not repeat a column.  Bit-exact, independent of launch geometry.
 */
typedef enum gnn_layer_mask_rule { GNN_LAYER_MASK_THRESHOLD = 0, GNN_LAYER_MASK_FANOUT = 1 } gnn_layer_mask_rule;

int32_t gnn_layer_edge_mask(const gnn_csr *g, const int32_t *rows, int32_t n_active, int32_t rule, int32_t fanout,
                            uint64_t threshold, uint64_t seed, int32_t layer, uint32_t *edge_keep, int32_t *kept_len,
                            uint64_t *row_thr_key, int32_t *row_thr_id, void *stream);

/*
 * The mask gnn_layer_edge_mask made for (seed, layer), in the positions of the transposed graph gT (the backward
 * aggregation gathers over gT): entry (row u, column v) of gT is the forward entry (v <- u), kept iff
 * (key(v, u), u) <= (row_thr_key[v], row_thr_id[v]).  keep_t: ceil(gT.nnz / 32) words, all written.  Same result
 * as gnn_transpose_edge_mask on that mask, without the search.
 */
int32_t gnn_layer_edge_mask_transposed(const gnn_csr *gT, const uint64_t *row_thr_key, const int32_t *row_thr_id,
                                       uint64_t seed, int32_t layer, uint32_t *keep_t, void *stream);

/*
 * The same mask in the positions of the transposed graph, for the backward aggregation: bit q of keep_t (entry v
 * of row u of gT) = bit p of keep, p = the position of u in row v of g.  g needs GNN_CSR_SORTED_COLUMNS
 * (only g's is used) and rows without repeated columns; an entry of gT that g does not have gets 0.  keep_t: ceil(gT.nnz / 32) words,
 * all written.
 */
int32_t gnn_transpose_edge_mask(const gnn_csr *g, const gnn_csr *gT, const uint32_t *keep, uint32_t *keep_t, void *stream);

/*
 * Pre-activation of the deep residual GraphSAGE (ResSAGE+, section 8.1; the paper's related-work section: residual
 * connections and pre-activation): for the listed rows, over the first F columns (1 <= F <= 1024),
 *   Y[v] = max(0, (X[v] - mean) / sqrt(var + eps) * gamma + beta),   mean / var over the row (var = mean of squares
 *   of the deviations).  gamma, beta: float [F], device.  Rows that are not listed are neither read nor written.
 */
int32_t gnn_layer_norm_relu_fwd(const int32_t *rows, int32_t n_active, const void *X, int64_t ldx, int32_t F,
                                const float *gamma, const float *beta, float eps, void *Y, int64_t ldy, int32_t dtype,
                                void *stream);

/*
 * Its backward.  T = the forward output as stored (the ReLU passes the gradient where T > 0), X = the forward input.
 *   dX[v] = LayerNorm-backward(dY[v] where T[v] > 0)  (+ dRes[v] for the first n_res listed rows: the gradient that
 *   arrives over the residual connection; dRes NULL: none).  dX is overwritten for the listed rows only.
 *   dgamma, dbeta: float [F], overwritten with the sums over the listed rows (fixed order: bit-reproducible).
 * Workspace: (ws, ws_bytes) size-query protocol.
 */
int32_t gnn_layer_norm_relu_bwd(const int32_t *rows, int32_t n_active, const void *dY, int64_t lddy, const void *T,
                                int64_t ldt, const void *X, int64_t ldx, int32_t F, const float *gamma, float eps,
                                const void *dRes, int64_t ldr, int32_t n_res, void *dX, int64_t lddx, float *dgamma,
                                float *dbeta, int32_t dtype, void *ws, size_t *ws_bytes, void *stream);

/* Y[v, 0:F] += X[v, 0:F] for the listed rows: the residual connection of the same model (section 8.1, ResSAGE+), forward. */
int32_t gnn_add_rows(const int32_t *rows, int32_t n_active, const void *X, int64_t ldx, void *Y, int64_t ldy, int32_t F,
                     int32_t dtype, void *stream);

/*
 * Two gradient contributions meet in front of a ReLU (backward of a layer in the exchanged order of
 * gnn_masked_spmm_fwd_add: the neighbour half reaches every listed row, the self half only the first n_add of them):
 *     Y[v, 0:F] = [H[v, 0:F] > 0] * (Y[v, 0:F] + (i < n_add ? X[v, 0:F] : 0))      v = rows[i], i < n_active
 *   H   the activations behind that ReLU (same rows and columns, leading dimension ldh), not NULL
 *   X   may be NULL when n_add == 0
 */
int32_t gnn_add_rows_masked(const int32_t *rows, int32_t n_active, const void *X, int64_t ldx, int32_t n_add, void *Y,
                            int64_t ldy, int32_t F, const void *H, int64_t ldh, int32_t dtype, void *stream);

/*
 * Extraction of the partition's one-hop graph (section 6, figure 7c step 1; section 5.3.1: the sub-graph
 * on the vertices a traversal from the partition's own vertices reached).  g is the UNPARTITIONED graph (square); ring_ids[0 .. n_local) and dist are
 * what gnn_build_active_sets wrote for it (traversed vertices sorted by (distance, id)).  The
 * traversed vertices become the local vertices 0 .. n_local-1 in that order - so the rows of layer l
 * are the PREFIX 0 .. hop_offsets[L-l+1]-1 of the local numbering, targets first - and the local
 * graph keeps every edge of g between two traversed vertices, in local ids, each row ascending
 * (the result satisfies GNN_CSR_SORTED_COLUMNS if g does).
 *   new_id       out [g->n_rows]: local id of every vertex, -1 if not traversed (written by the
 *                count pass, read by the fill pass)
 * Two calls, as for gnn_sample_boundary:
 *   count pass   out_col_idx == NULL: writes new_id, out_row_ptr[0 .. n_local] and *out_nnz (device);
 *                out_nnz_host, if non-NULL, receives the same number (the call then waits)
 *   fill pass    out_col_idx != NULL: writes the local column ids; entries at or beyond out_capacity
 *                are not written
 * Ids in ring_ids outside [0, g->n_rows) give empty rows.  L <= 30.  Bit-exact.
 */
int32_t gnn_extract_partition(const gnn_csr *g, const int32_t *ring_ids, int32_t n_local,
                              const int32_t *dist, int32_t L, int32_t *new_id,
                              int32_t *out_row_ptr, int32_t *out_col_idx, int64_t out_capacity,
                              int64_t *out_nnz, int64_t *out_nnz_host,
                              void *ws, size_t *ws_bytes, void *stream);

/*
 * (Helper; no passage of the paper.)  out_row_ptr[0 .. n] over the full id range from a row list: row ids[i] gets the length
 * list_row_ptr[i+1] - list_row_ptr[i] of listed row i, every other row is empty.  With ids ascending,
 * (out_row_ptr, the list's col_idx) is the row list as an n-row CSR - this is how the kept rows of
 * gnn_sample_boundary become the graph `gs` below.  Ids outside [0, n) are ignored.
 */
int32_t gnn_expand_row_ptr(int32_t n, const int32_t *ids, int32_t n_ids, const int32_t *list_row_ptr,
                           int32_t *out_row_ptr, void *ws, size_t *ws_bytes, void *stream);

/*
 * Extraction after boundary sampling (section 5.3.1: the local graph is built on what the sampler's
 * traversal reached, and no edge between two inner vertices is dropped).
 *   gs   the kept rows as an n-row CSR (rows of non-targets empty, columns ascending)
 *   gT   the transposed unpartitioned graph (the same arrays as the graph itself if it is symmetric)
 *   ring_ids, dist   gnn_build_active_sets(gs, targets, L = 1): targets (distance 0), then every
 *        outside vertex some target kept (distance 1), each group ascending
 * Local vertices = ring order (targets first).  Local rows: a target keeps its kept row; an outside
 * vertex u gets the reverse of the kept edges that reach it, { v target : u in kept row of v } (so the
 * local graph is symmetric); there are no edges between two outside vertices.  Rows ascending in
 * local id.  new_id and the two passes are as for gnn_extract_partition.  Bit-exact.
 */
int32_t gnn_extract_sampled_partition(const gnn_csr *gT, const gnn_csr *gs, const int32_t *ring_ids,
                                      int32_t n_local, const int32_t *dist, int32_t *new_id,
                                      int32_t *out_row_ptr, int32_t *out_col_idx, int64_t out_capacity,
                                      int64_t *out_nnz, int64_t *out_nnz_host,
                                      void *ws, size_t *ws_bytes, void *stream);

/*
 * (Helper; no passage of the paper: section 6 only says that a partition holds the features of its vertices.)
 * Row gather (the features of the extracted vertices, in local order):
 *     dst[i, 0:F] = src[ids[i], 0:F]    for i in [0, n);  rows with ids[i] outside [0, n_src) are skipped
 * src [n_src, ld_src], dst [n, ld_dst] of `dtype`; columns F..ld_dst of dst are not written.
 */
int32_t gnn_gather_rows(const void *src, int64_t ld_src, int32_t n_src, const int32_t *ids, int32_t n,
                        int32_t F, int32_t dtype, void *dst, int64_t ld_dst, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GNNHOT_H */
