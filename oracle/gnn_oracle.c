/*
 * CPU oracle for the masked full-neighbourhood GNN layer path.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain loops, double precision, written from the
 * paper's definitions; it shares no code with the HIP library and must never
 * be called from the product path (only tests, the smoke check and the CPU
 * baseline leg of the benchmark use it).
 *
 * What it follows:
 *   - layer equation of section 2.1:  h_N(v) = AGGREGATE({h_u : u in N(v)}),
 *     h_v = F(h_v, h_N(v)), AGGREGATE a (scaled) sum, F = weights then sigma;
 *   - one-hop graph masking of section 6 (figure 7c, steps 1-5): ONE one-hop
 *     graph is reused by every layer, and layer l only produces the vertices
 *     that the targets' exact dependency still needs;
 *   - expansion-aware sampling of section 5.3: inner dependencies are kept
 *     whole, only edges that leave the target set are thinned, at most
 *     `fanout` per boundary vertex;
 *   - the traversal of expansion-aware sampling itself (section 5.3.1): from
 *     the inner vertices, at most h hops outwards, at most f new vertices per
 *     traversed vertex and hop, high-degree-first with respect to the part of
 *     the graph not yet selected;
 *   - layer-wise sampling as per-layer masking (section 5.2): the one-hop
 *     graph stays whole and every layer aggregates through its own edge mask;
 *   - the deep residual model the paper trains (ResSAGE+, section 8.1): GraphSAGE layers with residual
 *     connections and pre-activation (layer normalisation, then ReLU);
 *   - extraction of the partition (section 6, step 1; section 5.3.1 "a
 *     subgraph is generated from the traversed vertices"): the vertices the
 *     traversal reached and every edge of the graph between two of them.
 *
 * Conventions.  L layers numbered l = 1..L.  T = target (inner) vertices.
 * Row v of the CSR lists the vertices u that v aggregates.  dist(v) = number
 * of hops from T to v following rows (dist = 0 on T).  Layer l computes the
 * rows R_l = {v : dist(v) <= L - l}; R_L = T.
 *
 * Every pin of this file (dense brute force, finite differences, closed forms,
 * the published splitmix64 vector) lives in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------------- */
/* Active sets: breadth-first levels from T over rows, capped at L.        */
/* Section 6, step 1 ("extract the multi-hop dependency starting from the  */
/* inner vertices") and step 4 (per-layer mask).                           */
/*   dist[v]      hop distance, -1 if v is farther than L hops or unreachable */
/*   ring_ids     vertices sorted by (dist, id); ring j = vertices at dist j  */
/*   hop_offsets  [L+2]; ring j is ring_ids[hop_offsets[j] .. hop_offsets[j+1]) */
/* ---------------------------------------------------------------------- */
int orc_active_sets(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                    const int32_t *targets, int32_t n_targets, int32_t L,
                    int32_t *dist, int32_t *ring_ids, int64_t *hop_offsets)
{
    for (int32_t v = 0; v < n; ++v) dist[v] = -1;
    for (int32_t i = 0; i < n_targets; ++i) {
        if (targets[i] < 0 || targets[i] >= n) return 1;
        dist[targets[i]] = 0;                 /* duplicates: set semantics */
    }
    for (int32_t j = 0; j < L; ++j) {
        /* every vertex at distance j opens its row; unseen entries get j+1 */
        for (int32_t v = 0; v < n; ++v) {
            if (dist[v] != j) continue;
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                int32_t u = col_idx[e];
                if (dist[u] < 0) dist[u] = j + 1;
            }
        }
    }
    int64_t pos = 0;
    for (int32_t j = 0; j <= L; ++j) {
        hop_offsets[j] = pos;
        for (int32_t v = 0; v < n; ++v)
            if (dist[v] == j) ring_ids[pos++] = v;
    }
    hop_offsets[L + 1] = pos;
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Normalisation factors (section 2.1 leaves the aggregator open beyond a   */
/* sum; these are the two named models').  mode 1: mean, 1/len (0 if empty).*/
/* mode 2: symmetric GCN, len^-1/2 (len counts the self loop in the graph).*/
/* ---------------------------------------------------------------------- */
void orc_norm_scales(int32_t mode, const int32_t *len, int32_t n, double *out)
{
    for (int32_t v = 0; v < n; ++v) {
        if (len[v] <= 0) out[v] = 0.0;
        else if (mode == 1) out[v] = 1.0 / (double)len[v];
        else out[v] = 1.0 / sqrt((double)len[v]);
    }
}

/* ---------------------------------------------------------------------- */
/* Masked aggregation, forward (section 2.1 equation, first half):         */
/*   Y[v,:] = rs[v] * sum_{u in row(v)} cs[u] * X[u,:]   for v in rows     */
/* rows == NULL means 0..n_active-1.  rs/cs NULL means 1.  Rows outside    */
/* the list are not touched (masked vertices are never read afterwards).   */
/* ---------------------------------------------------------------------- */
void orc_spmm_fwd(const int32_t *row_ptr, const int32_t *col_idx,
                  const int32_t *rows, int32_t n_active,
                  const double *X, int64_t ldx, double *Y, int64_t ldy, int32_t F,
                  const double *rs, const double *cs)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int32_t i = 0; i < n_active; ++i) {
        int32_t v = rows ? rows[i] : i;
        double *y = Y + (int64_t)v * ldy;
        for (int32_t f = 0; f < F; ++f) y[f] = 0.0;
        for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            int32_t u = col_idx[e];
            double w = cs ? cs[u] : 1.0;
            const double *x = X + (int64_t)u * ldx;
            for (int32_t f = 0; f < F; ++f) y[f] += w * x[f];
        }
        if (rs)
            for (int32_t f = 0; f < F; ++f) y[f] *= rs[v];
    }
}

/* ---------------------------------------------------------------------- */
/* Masked aggregation, backward = adjoint of the forward map, written as   */
/* the scatter the chain rule gives over the SAME (forward) CSR:           */
/*   for v in rows, u in row(v):  dX[u,:] += cs[u] * rs[v] * dY[v,:]       */
/* dX is accumulated into (caller zeroes it).  Threads split the feature   */
/* columns, so no two threads touch the same element.                      */
/* ---------------------------------------------------------------------- */
void orc_spmm_bwd(const int32_t *row_ptr, const int32_t *col_idx,
                  const int32_t *rows, int32_t n_active,
                  const double *dY, int64_t lddy, double *dX, int64_t lddx, int32_t F,
                  const double *rs, const double *cs)
{
    const int32_t CB = 16;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t f0 = 0; f0 < F; f0 += CB) {
        int32_t f1 = f0 + CB < F ? f0 + CB : F;
        for (int32_t i = 0; i < n_active; ++i) {
            int32_t v = rows ? rows[i] : i;
            const double *dy = dY + (int64_t)v * lddy;
            double wv = rs ? rs[v] : 1.0;
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                int32_t u = col_idx[e];
                double w = wv * (cs ? cs[u] : 1.0);
                double *dx = dX + (int64_t)u * lddx;
                for (int32_t f = f0; f < f1; ++f) dx[f] += w * dy[f];
            }
        }
    }
}

/* ---------------------------------------------------------------------- */
/* Feature transform, forward (section 2.1 equation, second half):         */
/*   Z[v,:] = A[v,:] W_neigh (+ X_self[v,:] W_self) + bias                 */
/*   H[v,:] = relu ? max(Z,0) : Z          for v in rows                   */
/* A, X_self: [*, K] with leading dimension ld_in; W: [K, N] row-major.    */
/* ---------------------------------------------------------------------- */
void orc_linear_fwd(const int32_t *rows, int32_t n_active,
                    const double *A, const double *X_self, int64_t ld_in, int32_t K,
                    const double *W_neigh, const double *W_self, const double *bias, int32_t N,
                    double *H, int64_t ld_out, int32_t relu)
{
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n_active; ++i) {
        int32_t v = rows ? rows[i] : i;
        double *h = H + (int64_t)v * ld_out;
        for (int32_t j = 0; j < N; ++j) h[j] = bias ? bias[j] : 0.0;
        const double *a = A + (int64_t)v * ld_in;
        for (int32_t k = 0; k < K; ++k)
            for (int32_t j = 0; j < N; ++j) h[j] += a[k] * W_neigh[(int64_t)k * N + j];
        if (X_self) {
            const double *x = X_self + (int64_t)v * ld_in;
            for (int32_t k = 0; k < K; ++k)
                for (int32_t j = 0; j < N; ++j) h[j] += x[k] * W_self[(int64_t)k * N + j];
        }
        if (relu)
            for (int32_t j = 0; j < N; ++j) h[j] = h[j] > 0.0 ? h[j] : 0.0;
    }
}

/* ---------------------------------------------------------------------- */
/* Feature transform, backward (chain rule of the above):                  */
/*   dZ = relu ? dH * [H > 0] : dH                                          */
/*   dW_neigh = A[rows]^T dZ,  dW_self = X_self[rows]^T dZ,  dbias = sum dZ */
/*   dA[v,:] = dZ W_neigh^T,   dX_self[v,:] = dZ W_self^T   (v in rows)     */
/* dW_*, dbias are overwritten.  dA / dX_self rows in the list are         */
/* overwritten; either may be NULL to skip.  H may be NULL when relu == 0.  */
/* ---------------------------------------------------------------------- */
void orc_linear_bwd(const int32_t *rows, int32_t n_active,
                    const double *dH, int64_t ld_dh, const double *H, int64_t ld_h, int32_t relu,
                    const double *A, const double *X_self, int64_t ld_in, int32_t K,
                    const double *W_neigh, const double *W_self, int32_t N,
                    double *dW_neigh, double *dW_self, double *dbias,
                    double *dA, double *dX_self, int64_t ld_din)
{
    double *dz = (double *)malloc(sizeof(double) * (size_t)N);
    memset(dW_neigh, 0, sizeof(double) * (size_t)K * N);
    if (dW_self) memset(dW_self, 0, sizeof(double) * (size_t)K * N);
    memset(dbias, 0, sizeof(double) * (size_t)N);
    for (int32_t i = 0; i < n_active; ++i) {
        int32_t v = rows ? rows[i] : i;
        const double *dh = dH + (int64_t)v * ld_dh;
        for (int32_t j = 0; j < N; ++j) {
            double g = dh[j];
            if (relu && !(H[(int64_t)v * ld_h + j] > 0.0)) g = 0.0;
            dz[j] = g;
            dbias[j] += g;
        }
        const double *a = A + (int64_t)v * ld_in;
        for (int32_t k = 0; k < K; ++k)
            for (int32_t j = 0; j < N; ++j) dW_neigh[(int64_t)k * N + j] += a[k] * dz[j];
        if (X_self && dW_self) {
            const double *x = X_self + (int64_t)v * ld_in;
            for (int32_t k = 0; k < K; ++k)
                for (int32_t j = 0; j < N; ++j) dW_self[(int64_t)k * N + j] += x[k] * dz[j];
        }
        if (dA) {
            double *da = dA + (int64_t)v * ld_din;
            for (int32_t k = 0; k < K; ++k) {
                double s = 0.0;
                for (int32_t j = 0; j < N; ++j) s += dz[j] * W_neigh[(int64_t)k * N + j];
                da[k] = s;
            }
        }
        if (dX_self && W_self) {
            double *dx = dX_self + (int64_t)v * ld_din;
            for (int32_t k = 0; k < K; ++k) {
                double s = 0.0;
                for (int32_t j = 0; j < N; ++j) s += dz[j] * W_self[(int64_t)k * N + j];
                dx[k] = s;
            }
        }
    }
    free(dz);
}

/* ---------------------------------------------------------------------- */
/* Node-classification loss on the targets (section 8.1, task):            */
/*   loss = mean_{v in T} -log softmax(Z[v])[y_v];  dZ = (softmax - onehot)/|T| */
/* labels[i] belongs to rows[i].  Rows outside the list are not written.   */
/* ---------------------------------------------------------------------- */
double orc_softmax_ce(const int32_t *rows, int32_t n_active,
                      const double *Z, int64_t ldz, int32_t C, const int32_t *labels,
                      double *dZ, int64_t lddz)
{
    double loss = 0.0;
    for (int32_t i = 0; i < n_active; ++i) {
        int32_t v = rows ? rows[i] : i;
        const double *z = Z + (int64_t)v * ldz;
        double m = z[0];
        for (int32_t c = 1; c < C; ++c) if (z[c] > m) m = z[c];
        double s = 0.0;
        for (int32_t c = 0; c < C; ++c) s += exp(z[c] - m);
        loss += -(z[labels[i]] - m - log(s));
        if (dZ) {
            double *d = dZ + (int64_t)v * lddz;
            for (int32_t c = 0; c < C; ++c)
                d[c] = (exp(z[c] - m) / s - (c == labels[i] ? 1.0 : 0.0)) / (double)n_active;
        }
    }
    return n_active > 0 ? loss / (double)n_active : 0.0;
}

/* ---------------------------------------------------------------------- */
/* bf16 storage: round a value to the nearest bfloat16 (ties to even),     */
/* taken from its float32 value.  NaN stays NaN.                           */
/* ---------------------------------------------------------------------- */
void orc_round_bf16(double *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        float f = (float)x[i];
        uint32_t b;
        memcpy(&b, &f, 4);
        if ((b & 0x7fffffffu) > 0x7f800000u) { x[i] = NAN; continue; }
        uint32_t lsb = (b >> 16) & 1u;
        b += 0x7fffu + lsb;
        b &= 0xffff0000u;
        memcpy(&f, &b, 4);
        x[i] = (double)f;
    }
}

/* ---------------------------------------------------------------------- */
/* Expansion-aware sampling, one hop (section 5.3.1 with the selection     */
/* rule replaced by a seeded counter-based hash: every edge (v,u) gets a   */
/* 64-bit key that depends on (seed, v, u, hop) only).                     */
/*                                                                         */
/* mix64 is the splitmix64 output function (Steele, Lea, Flood 2014;       */
/* Vigna's public-domain constants): add the golden-ratio increment, then  */
/* two xor-shift-multiply rounds and a final xor-shift.                    */
/* ---------------------------------------------------------------------- */
uint64_t orc_mix64(uint64_t x)
{
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

uint64_t orc_edge_key(uint64_t seed, uint64_t v, uint64_t u, uint64_t hop)
{
    return orc_mix64(orc_mix64(orc_mix64(seed + hop) ^ v) ^ u);
}

typedef struct { uint64_t key; int32_t u; } orc_cand;

static int orc_cand_cmp(const void *a, const void *b)
{
    const orc_cand *x = (const orc_cand *)a, *y = (const orc_cand *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return (x->u > y->u) - (x->u < y->u);
}

static int orc_i32_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * For every target v (in the order given): keep every neighbour that is a
 * target (section 5.3: only the boundary is sampled); of the neighbours outside T
 * keep the min(fanout, count) with the smallest (key, id).  The kept row is
 * emitted in ascending id order.  Two-call use: out_col_idx == NULL only
 * fills out_row_ptr[0..n_targets] (so the caller can size the second call).
 * Returns the number of kept entries, or -1 on a bad argument.
 */
int64_t orc_sample_boundary(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                            const uint8_t *is_target, const int32_t *targets, int32_t n_targets,
                            int32_t fanout, uint64_t seed,
                            int32_t *out_row_ptr, int32_t *out_col_idx)
{
    if (fanout < 0) return -1;
    int64_t pos = 0;
    orc_cand *cand = NULL;
    int32_t cap = 0;
    for (int32_t i = 0; i < n_targets; ++i) {
        int32_t v = targets[i];
        if (v < 0 || v >= n) { free(cand); return -1; }
        int32_t len = row_ptr[v + 1] - row_ptr[v];
        if (len > cap) { cap = len; cand = (orc_cand *)realloc(cand, sizeof(orc_cand) * (size_t)cap); }
        out_row_ptr[i] = (int32_t)pos;
        int32_t n_ext = 0;
        int64_t row_start = pos;
        for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            int32_t u = col_idx[e];
            if (is_target[u]) {
                if (out_col_idx) out_col_idx[pos] = u;
                ++pos;
            } else {
                cand[n_ext].key = orc_edge_key(seed, (uint64_t)v, (uint64_t)u, 1);
                cand[n_ext].u = u;
                ++n_ext;
            }
        }
        qsort(cand, (size_t)n_ext, sizeof(orc_cand), orc_cand_cmp);
        int32_t keep = n_ext < fanout ? n_ext : fanout;
        for (int32_t k = 0; k < keep; ++k) {
            if (out_col_idx) out_col_idx[pos] = cand[k].u;
            ++pos;
        }
        if (out_col_idx) qsort(out_col_idx + row_start, (size_t)(pos - row_start), sizeof(int32_t), orc_i32_cmp);
    }
    out_row_ptr[n_targets] = (int32_t)pos;
    free(cand);
    return pos;
}

/* ---------------------------------------------------------------------- */
/* Extraction of the partition's one-hop graph (section 6, step 1; section  */
/* 5.3.1): the traversed vertices = ring_ids (all vertices within L hops of */
/* the targets, sorted by (distance, id), as orc_active_sets returns them)  */
/* become the local vertices 0 .. n_local-1 in that order, so that every    */
/* per-layer active set is a prefix of the local numbering; the local graph */
/* keeps exactly the edges of the graph whose two ends were both traversed  */
/* (vertex-induced sub-graph).  Local rows list their columns in ascending  */
/* local id.                                                                */
/*   new_id       scratch [n]: local id of every vertex, -1 if not traversed */
/*   out_col_idx  NULL: only count (out_row_ptr is still written)            */
/* Returns the number of local edges.                                       */
/* ---------------------------------------------------------------------- */
int64_t orc_extract_partition(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                              const int32_t *ring_ids, int32_t n_local, int32_t *new_id,
                              int32_t *out_row_ptr, int32_t *out_col_idx)
{
    for (int32_t v = 0; v < n; ++v) new_id[v] = -1;
    for (int32_t i = 0; i < n_local; ++i) new_id[ring_ids[i]] = i;
    int64_t pos = 0;
    for (int32_t i = 0; i < n_local; ++i) {
        const int32_t v = ring_ids[i];
        out_row_ptr[i] = (int32_t)pos;
        const int64_t first = pos;
        for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            const int32_t u = new_id[col_idx[e]];
            if (u < 0) continue;              /* the other end was not traversed */
            if (out_col_idx) out_col_idx[pos] = u;
            ++pos;
        }
        if (out_col_idx) qsort(out_col_idx + first, (size_t)(pos - first), sizeof(int32_t), orc_i32_cmp);
    }
    out_row_ptr[n_local] = (int32_t)pos;
    return pos;
}

/* ---------------------------------------------------------------------- */
/* Extraction after boundary sampling (section 5.3.1: the sub-graph is      */
/* built on the vertices the traversal reached; edges between two inner     */
/* vertices are never dropped).                                             */
/* Traversed vertices = the targets (distance 0) and every outside vertex   */
/* that some target kept (distance 1); local numbering by (distance, id):   */
/* targets first.  Edges: the kept row of every target, plus the reverse    */
/* (u, v) of every kept edge (v, u) that leaves the target set, so that the */
/* local one-hop graph stays symmetric; no edges between two outside        */
/* vertices.  Local rows list their columns in ascending local id.          */
/*   targets        ascending, no repeats (else -1 is returned)             */
/*   s_row_ptr/s_col_idx  kept rows as orc_sample_boundary writes them      */
/*   new_id         scratch [n]                                             */
/*   local_to_global  out, room for n                                       */
/*   out_row_ptr    out, room for n + 1;  out_col_idx NULL: only count      */
/* Returns the number of local edges; *n_local_out = local vertices.        */
/* ---------------------------------------------------------------------- */
int64_t orc_extract_sampled(int32_t n, const int32_t *targets, int32_t n_targets,
                            const int32_t *s_row_ptr, const int32_t *s_col_idx,
                            int32_t *new_id, int32_t *local_to_global, int32_t *n_local_out,
                            int32_t *out_row_ptr, int32_t *out_col_idx)
{
    for (int32_t v = 0; v < n; ++v) new_id[v] = -1;
    for (int32_t i = 0; i < n_targets; ++i) {
        if (targets[i] < 0 || targets[i] >= n) return -1;
        if (i > 0 && targets[i] <= targets[i - 1]) return -1;
        new_id[targets[i]] = i;
        local_to_global[i] = targets[i];
    }
    /* outside vertices that were kept by somebody, in ascending id */
    for (int32_t e = 0; e < s_row_ptr[n_targets]; ++e)
        if (new_id[s_col_idx[e]] == -1) new_id[s_col_idx[e]] = -2;
    int32_t n_local = n_targets;
    for (int32_t v = 0; v < n; ++v)
        if (new_id[v] == -2) { new_id[v] = n_local; local_to_global[n_local] = v; ++n_local; }
    *n_local_out = n_local;
    /* row lengths: a target keeps its sampled row; an outside vertex gets one entry per target that kept it */
    for (int32_t i = 0; i <= n_local; ++i) out_row_ptr[i] = 0;
    for (int32_t i = 0; i < n_targets; ++i) {
        out_row_ptr[i + 1] += s_row_ptr[i + 1] - s_row_ptr[i];
        for (int32_t e = s_row_ptr[i]; e < s_row_ptr[i + 1]; ++e) {
            int32_t u = new_id[s_col_idx[e]];
            if (u >= n_targets) out_row_ptr[u + 1] += 1;
        }
    }
    for (int32_t i = 0; i < n_local; ++i) out_row_ptr[i + 1] += out_row_ptr[i];
    const int64_t nnz = out_row_ptr[n_local];
    if (!out_col_idx) return nnz;
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_local + 1));
    for (int32_t i = 0; i < n_local; ++i) cursor[i] = out_row_ptr[i];
    for (int32_t i = 0; i < n_targets; ++i) {              /* ascending i: reverse rows come out ascending */
        for (int32_t e = s_row_ptr[i]; e < s_row_ptr[i + 1]; ++e) {
            int32_t u = new_id[s_col_idx[e]];
            out_col_idx[cursor[i]++] = u;
            if (u >= n_targets) out_col_idx[cursor[u]++] = i;
        }
        qsort(out_col_idx + out_row_ptr[i], (size_t)(out_row_ptr[i + 1] - out_row_ptr[i]), sizeof(int32_t), orc_i32_cmp);
    }
    free(cursor);
    return nnz;
}

/* ---------------------------------------------------------------------- */
/* Traversal of expansion-aware sampling (section 5.3.1).  From the inner   */
/* vertices (targets, hop 0) go at most `hops` hops outwards; in hop j      */
/* every vertex v selected in hop j-1 looks at its neighbours that have not */
/* been selected before this hop started and keeps at most `fanout` of them */
/* - those with the smallest (key, id):                                     */
/*   rule 1 (the paper's): key = -(entries of row u that were unselected    */
/*           when the hop started), i.e. the best-connected candidate first;*/
/*   rule 0 (seeded hash, as in orc_sample_boundary): key = orc_edge_key(   */
/*           seed, v, u, j).                                                */
/* A vertex is selected in hop j if some v kept it.  Outputs are those of   */
/* orc_active_sets with "distance" = the hop of selection:                  */
/*   dist[v]      hop in which v was selected, -1 if never                  */
/*   ring_ids     selected vertices sorted by (hop, id)                     */
/*   hop_offsets  [hops+2]                                                  */
/* ---------------------------------------------------------------------- */
typedef struct { uint64_t key; int32_t u; } orc_eas_cand;

static int orc_eas_cmp(const void *a, const void *b)
{
    const orc_eas_cand *x = (const orc_eas_cand *)a, *y = (const orc_eas_cand *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return (x->u > y->u) - (x->u < y->u);
}

int orc_eas_traverse(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                     const int32_t *targets, int32_t n_targets, int32_t hops, int32_t fanout,
                     int32_t rule, uint64_t seed,
                     int32_t *dist, int32_t *ring_ids, int64_t *hop_offsets)
{
    if (fanout < 0 || hops < 1 || (rule != 0 && rule != 1)) return 1;
    for (int32_t v = 0; v < n; ++v) dist[v] = -1;
    for (int32_t i = 0; i < n_targets; ++i) {
        if (targets[i] < 0 || targets[i] >= n) return 1;
        dist[targets[i]] = 0;
    }
    int64_t pos = 0;
    hop_offsets[0] = 0;
    for (int32_t v = 0; v < n; ++v) if (dist[v] == 0) ring_ids[pos++] = v;
    hop_offsets[1] = pos;
    uint8_t *was_selected = (uint8_t *)malloc((size_t)n + 1);
    int32_t *conn = (int32_t *)malloc(sizeof(int32_t) * ((size_t)n + 1));
    orc_eas_cand *cand = NULL;
    int32_t cap = 0;
    for (int32_t j = 1; j <= hops; ++j) {
        /* state when the hop starts */
        for (int32_t v = 0; v < n; ++v) was_selected[v] = dist[v] >= 0;
        for (int32_t u = 0; u < n; ++u) {
            int32_t c = 0;
            for (int32_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) c += !was_selected[col_idx[e]];
            conn[u] = c;
        }
        for (int64_t q = hop_offsets[j - 1]; q < hop_offsets[j]; ++q) {
            const int32_t v = ring_ids[q];
            const int32_t len = row_ptr[v + 1] - row_ptr[v];
            if (len > cap) { cap = len; cand = (orc_eas_cand *)realloc(cand, sizeof(orc_eas_cand) * (size_t)cap); }
            int32_t nc = 0;
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                const int32_t u = col_idx[e];
                if (was_selected[u]) continue;
                cand[nc].u = u;
                cand[nc].key = rule == 1 ? (uint64_t)(0xffffffffu - (uint32_t)conn[u])
                                         : orc_edge_key(seed, (uint64_t)v, (uint64_t)u, (uint64_t)j);
                ++nc;
            }
            qsort(cand, (size_t)nc, sizeof(orc_eas_cand), orc_eas_cmp);
            const int32_t keep = nc < fanout ? nc : fanout;
            for (int32_t k = 0; k < keep; ++k)
                if (dist[cand[k].u] < 0) dist[cand[k].u] = j;
        }
        for (int32_t v = 0; v < n; ++v) if (dist[v] == j) ring_ids[pos++] = v;
        hop_offsets[j + 1] = pos;
    }
    free(cand); free(conn); free(was_selected);
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Layer-wise sampling as per-layer masking (section 5.2: "for layer-wise   */
/* samplings the maskings are generated per layer to conduct layer-wise     */
/* aggregation of them").  The one-hop graph stays whole; layer `layer`     */
/* aggregates only through the entries a rule keeps:                        */
/*   rule 0  every entry (v <- u) on its own: kept iff key <= threshold     */
/*   rule 1  a row keeps its min(fanout, length) entries with the smallest  */
/*           (key, id)                                                      */
/* with key = orc_edge_key(seed, v, u, layer).                              */
/*   keep[e]      1/0 for every entry e of a listed row (others untouched)  */
/*   kept_len[v]  kept entries of listed row v (others untouched)           */
/* ---------------------------------------------------------------------- */
int orc_layer_edge_mask(const int32_t *row_ptr, const int32_t *col_idx,
                        const int32_t *rows, int32_t n_active, int32_t rule, int32_t fanout,
                        uint64_t threshold, uint64_t seed, int32_t layer,
                        uint8_t *keep, int32_t *kept_len)
{
    if ((rule != 0 && rule != 1) || fanout < 0) return 1;
    orc_cand *cand = NULL;
    int32_t cap = 0;
    for (int32_t i = 0; i < n_active; ++i) {
        const int32_t v = rows ? rows[i] : i;
        const int32_t s = row_ptr[v], e = row_ptr[v + 1], len = e - s;
        int32_t kept = 0;
        if (rule == 0) {
            for (int32_t p = s; p < e; ++p) {
                keep[p] = orc_edge_key(seed, (uint64_t)v, (uint64_t)col_idx[p], (uint64_t)layer) <= threshold;
                kept += keep[p];
            }
        } else {
            if (len > cap) { cap = len; cand = (orc_cand *)realloc(cand, sizeof(orc_cand) * (size_t)cap); }
            for (int32_t p = s; p < e; ++p) {
                cand[p - s].key = orc_edge_key(seed, (uint64_t)v, (uint64_t)col_idx[p], (uint64_t)layer);
                cand[p - s].u = col_idx[p];
                keep[p] = 0;
            }
            qsort(cand, (size_t)len, sizeof(orc_cand), orc_cand_cmp);
            kept = len < fanout ? len : fanout;
            for (int32_t k = 0; k < kept; ++k)
                for (int32_t p = s; p < e; ++p)
                    if (col_idx[p] == cand[k].u) keep[p] = 1;
        }
        kept_len[v] = kept;
    }
    free(cand);
    return 0;
}

/* The mask in the positions of the transposed graph: entry q of row u of   */
/* (rpT, ciT) is the vertex v whose row lists u; keep_t[q] = keep[p] with p */
/* the position of u in row v (0 if row v does not list u).                 */
void orc_transpose_mask(const int32_t *row_ptr, const int32_t *col_idx, const uint8_t *keep,
                        int32_t n_t, const int32_t *rpT, const int32_t *ciT, uint8_t *keep_t)
{
    for (int32_t u = 0; u < n_t; ++u)
        for (int32_t q = rpT[u]; q < rpT[u + 1]; ++q) {
            const int32_t v = ciT[q];
            keep_t[q] = 0;
            for (int32_t p = row_ptr[v]; p < row_ptr[v + 1]; ++p)
                if (col_idx[p] == u) { keep_t[q] = keep[p]; break; }
        }
}

/* orc_spmm_fwd / orc_spmm_bwd through a mask: the entries with keep[e] == 0 */
/* do not exist for this layer.                                             */
void orc_spmm_fwd_em(const int32_t *row_ptr, const int32_t *col_idx, const uint8_t *keep,
                     const int32_t *rows, int32_t n_active,
                     const double *X, int64_t ldx, double *Y, int64_t ldy, int32_t F,
                     const double *rs, const double *cs)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int32_t i = 0; i < n_active; ++i) {
        int32_t v = rows ? rows[i] : i;
        double *y = Y + (int64_t)v * ldy;
        for (int32_t f = 0; f < F; ++f) y[f] = 0.0;
        for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            if (!keep[e]) continue;
            int32_t u = col_idx[e];
            double w = cs ? cs[u] : 1.0;
            const double *x = X + (int64_t)u * ldx;
            for (int32_t f = 0; f < F; ++f) y[f] += w * x[f];
        }
        if (rs)
            for (int32_t f = 0; f < F; ++f) y[f] *= rs[v];
    }
}

void orc_spmm_bwd_em(const int32_t *row_ptr, const int32_t *col_idx, const uint8_t *keep,
                     const int32_t *rows, int32_t n_active,
                     const double *dY, int64_t lddy, double *dX, int64_t lddx, int32_t F,
                     const double *rs, const double *cs)
{
    const int32_t CB = 16;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t f0 = 0; f0 < F; f0 += CB) {
        int32_t f1 = f0 + CB < F ? f0 + CB : F;
        for (int32_t i = 0; i < n_active; ++i) {
            int32_t v = rows ? rows[i] : i;
            const double *dy = dY + (int64_t)v * lddy;
            double wv = rs ? rs[v] : 1.0;
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                if (!keep[e]) continue;
                int32_t u = col_idx[e];
                double w = wv * (cs ? cs[u] : 1.0);
                double *dx = dX + (int64_t)u * lddx;
                for (int32_t f = f0; f < f1; ++f) dx[f] += w * dy[f];
            }
        }
    }
}

/* ---------------------------------------------------------------------- */
/* Pre-activation of the deep residual model (section 8.1 names ResSAGE+;   */
/* the related-work section describes it as residual connections plus       */
/* pre-activation): t = ReLU(LayerNorm(x)) per vertex, over its F features: */
/*   mu = mean(x), var = mean((x - mu)^2), xhat = (x - mu) / sqrt(var + eps) */
/*   t  = max(0, xhat * gamma + beta)                                        */
/* Only the listed rows are read and written.                               */
/* ---------------------------------------------------------------------- */
void orc_ln_relu_fwd(const int32_t *rows, int32_t n_active, const double *X, int64_t ldx, int32_t F,
                     const double *gamma, const double *beta, double eps, double *Y, int64_t ldy)
{
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n_active; ++i) {
        const int32_t v = rows ? rows[i] : i;
        const double *x = X + (int64_t)v * ldx;
        double *y = Y + (int64_t)v * ldy;
        double mu = 0.0, var = 0.0;
        for (int32_t f = 0; f < F; ++f) mu += x[f];
        mu /= (double)F;
        for (int32_t f = 0; f < F; ++f) var += (x[f] - mu) * (x[f] - mu);
        var /= (double)F;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int32_t f = 0; f < F; ++f) {
            const double t = (x[f] - mu) * rstd * gamma[f] + beta[f];
            y[f] = t > 0.0 ? t : 0.0;
        }
    }
}

/* Backward of orc_ln_relu_fwd by the chain rule.  Tmask = the forward      */
/* output as it was stored (the ReLU passes gradient where it is > 0).      */
/*   g = dY where Tmask > 0, else 0;  dgamma += sum_rows g * xhat;          */
/*   dbeta += sum_rows g;  gx = g * gamma;                                   */
/*   dX = rstd * (gx - mean(gx) - xhat * mean(gx * xhat))   (overwrites)     */
/* dgamma, dbeta are accumulated into (caller zeroes them).                 */
void orc_ln_relu_bwd(const int32_t *rows, int32_t n_active, const double *dY, int64_t lddy,
                     const double *Tmask, int64_t ldt, const double *X, int64_t ldx, int32_t F,
                     const double *gamma, double eps, double *dX, int64_t lddx,
                     double *dgamma, double *dbeta)
{
    double *xhat = (double *)malloc(sizeof(double) * (size_t)(F > 0 ? F : 1));
    double *gx = (double *)malloc(sizeof(double) * (size_t)(F > 0 ? F : 1));
    for (int32_t i = 0; i < n_active; ++i) {
        const int32_t v = rows ? rows[i] : i;
        const double *x = X + (int64_t)v * ldx;
        const double *dy = dY + (int64_t)v * lddy;
        const double *tm = Tmask + (int64_t)v * ldt;
        double *dx = dX + (int64_t)v * lddx;
        double mu = 0.0, var = 0.0;
        for (int32_t f = 0; f < F; ++f) mu += x[f];
        mu /= (double)F;
        for (int32_t f = 0; f < F; ++f) var += (x[f] - mu) * (x[f] - mu);
        var /= (double)F;
        const double rstd = 1.0 / sqrt(var + eps);
        double m1 = 0.0, m2 = 0.0;
        for (int32_t f = 0; f < F; ++f) {
            xhat[f] = (x[f] - mu) * rstd;
            const double g = tm[f] > 0.0 ? dy[f] : 0.0;
            dgamma[f] += g * xhat[f];
            dbeta[f] += g;
            gx[f] = g * gamma[f];
            m1 += gx[f];
            m2 += gx[f] * xhat[f];
        }
        m1 /= (double)F;
        m2 /= (double)F;
        for (int32_t f = 0; f < F; ++f) dx[f] = rstd * (gx[f] - m1 - xhat[f] * m2);
    }
    free(xhat); free(gx);
}
