/*
 * CPU oracle for the embed-and-aggregate step of lazy message passing.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to say what the GPU library must
 * compute; it is deliberately plain and slow, shares no code with the GPU
 * path, and nothing in the product imports or links it.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg call it.
 *
 * What is defined here and where it comes from:
 *
 *  - One GNN layer is Q^m_v = f( COMBINE( Q^{m-1}_v , AGGR_{u in N(v)} Q^{m-1}_u ) ),
 *    Q^0 = the raw features (Eq. 1 of the paper, section "Architecture of
 *    Classical GNNs").  f is a fully connected layer followed by ReLU,
 *    COMBINE is concatenation (the gloss under Eq. 1).
 *  - Lazy message passing (section "Lazy Message Passing") freezes a trained
 *    layer, evaluates it for every node and then performs one aggregation
 *    over the graph; the very first aggregation is over the raw features.
 *    So one round is  Z = act(H W + b)  (or Z = H for the first round)
 *    followed by AGGR over the graph.
 *  - The graph is undirected (section "Edge-partitioned Distributed Setup"),
 *    so every pair {u,v} contributes the two directed entries (u,v), (v,u).
 *  - The paper names its three model families (GCN, GraphSAGE, GAT) but does
 *    not print their aggregators.  They are taken in their standard forms:
 *      mean      out_v = (1/deg v) sum_{u in N(v)} z_u
 *      sum       out_v = sum_{u in N(v)} z_u
 *      gcn_sym   out_v = sum_{u in N~(v)} z_u / sqrt(d~_v d~_u), N~ contains v
 *                itself through an explicit self-loop entry, d~ = row length
 *      gat       per head h:  e_uv = LeakyReLU(<a_src_h, z_u,h> + <a_dst_h, z_v,h>),
 *                alpha_uv = softmax over u in N(v) of e_uv,
 *                out_v,h = sum_u alpha_uv z_u,h
 *      max       out_v = element-wise max over u in N(v) of z_u — the "max-pooling
 *                layer" the gloss under Eq. 1 gives as GraphSAGE's AGGR (the pooling
 *                network in front of it is the round's dense transform)
 *    An empty neighbourhood gives a zero aggregate in every mode.
 *
 * Everything accumulates in double and consumes the float inputs exactly.
 * The one float quantity is dinv[v] = 1/sqrt(deg v), which is DEFINED as the
 * correctly rounded single-precision sqrt followed by the correctly rounded
 * single-precision divide, so that it can be compared bit for bit.
 *
 * oracle_aggregate_backward differentiates these aggregations (chain rule
 * written out above the function); it is needed when a layer whose AGGR has
 * trainable parameters is trained with the aggregation in the loop.
 *
 * No worked numeric example exists in the paper.  The pins that tie these
 * functions to something other than themselves (dense-matrix brute force,
 * closed forms on regular graphs, hand-computed values, invariants) live in
 * tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_MEAN = 0, ORACLE_SUM = 1, ORACLE_GCN_SYM = 2, ORACLE_GAT_SOFTMAX = 3, ORACLE_MAX = 4 };

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * CSR of the undirected simple graph given by raw pairs.
 *   - each pair (u,v), u != v, yields entries (row u, col v) and (row v, col u)
 *   - pairs with u == v are dropped
 *   - if add_self_loops, exactly one entry (v,v) is then added for every v
 *   - repeated entries are kept once; columns ascend inside a row
 * row_ptr has N+1 entries; col_idx must have room for 2*n_pairs + N entries.
 * Returns nnz, or -1 if a node id is outside [0,N), -2 if out of memory.
 */
int64_t oracle_csr_from_coo(int64_t n_pairs, const int32_t *src, const int32_t *dst,
                            int64_t N, int add_self_loops,
                            int64_t *row_ptr, int32_t *col_idx)
{
    int64_t *start = (int64_t *)calloc((size_t)N + 1, sizeof(int64_t));
    if (!start) return -2;
    for (int64_t e = 0; e < n_pairs; ++e) {
        if (src[e] < 0 || src[e] >= N || dst[e] < 0 || dst[e] >= N) { free(start); return -1; }
        if (src[e] == dst[e]) continue;
        start[src[e] + 1]++;
        start[dst[e] + 1]++;
    }
    if (add_self_loops)
        for (int64_t v = 0; v < N; ++v) start[v + 1]++;
    for (int64_t v = 0; v < N; ++v) start[v + 1] += start[v];
    int64_t total = start[N];
    int32_t *raw = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
    int64_t *fill = (int64_t *)malloc(((size_t)N + 1) * sizeof(int64_t));
    if (!raw || !fill) { free(start); free(raw); free(fill); return -2; }
    memcpy(fill, start, ((size_t)N + 1) * sizeof(int64_t));
    for (int64_t e = 0; e < n_pairs; ++e) {
        int32_t u = src[e], v = dst[e];
        if (u == v) continue;
        raw[fill[u]++] = v;
        raw[fill[v]++] = u;
    }
    if (add_self_loops)
        for (int64_t v = 0; v < N; ++v) raw[fill[v]++] = (int32_t)v;
    /* sort every row, then copy it out without repeats */
    int64_t nnz = 0;
    row_ptr[0] = 0;
    for (int64_t v = 0; v < N; ++v) {
        int64_t lo = start[v], hi = start[v + 1];
        qsort(raw + lo, (size_t)(hi - lo), sizeof(int32_t), cmp_i32);
        for (int64_t k = lo; k < hi; ++k)
            if (k == lo || raw[k] != raw[k - 1]) col_idx[nnz++] = raw[k];
        row_ptr[v + 1] = nnz;
    }
    free(start); free(raw); free(fill);
    return nnz;
}

/* deg[v] = row length; dinv[v] = 1/sqrt(deg v) in correctly rounded float
 * arithmetic, 0 for an empty row. */
void oracle_degree(int64_t N, const int64_t *row_ptr, int32_t *deg, float *dinv)
{
    for (int64_t v = 0; v < N; ++v) {
        int64_t d = row_ptr[v + 1] - row_ptr[v];
        deg[v] = (int32_t)d;
        if (d > 0) {
            volatile float s = sqrtf((float)d);
            volatile float r = 1.0f / s;
            dinv[v] = r;
        } else {
            dinv[v] = 0.0f;
        }
    }
}

/*
 * Z[i,:] = act( H[rows[i],:] W + b ) for i < n_rows (rows == NULL: rows[i] = i).
 * H is [*, ldh] floats of which the first D_in columns are used, W is
 * [D_in, D_out] row-major, b is [D_out] or NULL, act is ReLU when relu != 0.
 * Z is [n_rows, D_out] doubles.
 */
void oracle_transform(int64_t n_rows, const int64_t *rows, int64_t D_in, int64_t D_out,
                      const float *H, int64_t ldh, const float *W, const float *b,
                      int relu, double *Z)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t r = rows ? rows[i] : i;
        for (int64_t j = 0; j < D_out; ++j) {
            double acc = b ? (double)b[j] : 0.0;
            for (int64_t k = 0; k < D_in; ++k)
                acc += (double)H[r * ldh + k] * (double)W[k * D_out + j];
            if (relu && acc < 0.0) acc = 0.0;
            Z[i * D_out + j] = acc;
        }
    }
}

static double leaky(double x, double slope) { return x > 0.0 ? x : slope * x; }

/*
 * out[i,:] = aggregate of row rows[i] (rows == NULL: all rows, n_rows == N).
 * Z is [N, ldz] floats, first F columns used.  For gat, F = heads * Dh,
 * a_src and a_dst are [heads, Dh].  dinv (gcn_sym only) is the float array
 * oracle_degree produced.  With self_concat the output row is 2F wide: the
 * node's own Z row first, its aggregate second; otherwise F wide.
 * out is doubles, row pitch F or 2F.
 */
void oracle_aggregate(int mode, int64_t n_rows, const int64_t *rows,
                      const int64_t *row_ptr, const int32_t *col_idx, const float *dinv,
                      int64_t F, int heads, const float *Z, int64_t ldz,
                      const float *a_src, const float *a_dst, double slope,
                      int self_concat, double *out)
{
    const int64_t pitch = self_concat ? 2 * F : F;
    const int64_t Dh = (mode == ORACLE_GAT_SOFTMAX) ? F / heads : F;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t v = rows ? rows[i] : i;
        double *o = out + i * pitch;
        if (self_concat) {
            for (int64_t j = 0; j < F; ++j) o[j] = (double)Z[v * ldz + j];
            o += F;
        }
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
        const int64_t deg = hi - lo;
        for (int64_t j = 0; j < F; ++j) o[j] = 0.0;
        if (deg == 0) continue;

        if (mode == ORACLE_SUM || mode == ORACLE_MEAN) {
            for (int64_t j = 0; j < F; ++j) {
                double s = 0.0;
                for (int64_t e = lo; e < hi; ++e) s += (double)Z[(int64_t)col_idx[e] * ldz + j];
                o[j] = (mode == ORACLE_MEAN) ? s / (double)deg : s;
            }
        } else if (mode == ORACLE_MAX) {
            for (int64_t j = 0; j < F; ++j) {
                double m = (double)Z[(int64_t)col_idx[lo] * ldz + j];
                for (int64_t e = lo + 1; e < hi; ++e) {
                    const double z = (double)Z[(int64_t)col_idx[e] * ldz + j];
                    if (z > m) m = z;
                }
                o[j] = m;
            }
        } else if (mode == ORACLE_GCN_SYM) {
            for (int64_t j = 0; j < F; ++j) {
                double s = 0.0;
                for (int64_t e = lo; e < hi; ++e) {
                    int64_t u = col_idx[e];
                    s += (double)dinv[v] * (double)dinv[u] * (double)Z[u * ldz + j];
                }
                o[j] = s;
            }
        } else { /* ORACLE_GAT_SOFTMAX */
            double *score = (double *)malloc((size_t)deg * sizeof(double));
            for (int h = 0; h < heads; ++h) {
                const float *as = a_src + (int64_t)h * Dh, *ad = a_dst + (int64_t)h * Dh;
                double er = 0.0;
                for (int64_t d = 0; d < Dh; ++d) er += (double)ad[d] * (double)Z[v * ldz + h * Dh + d];
                double m = -INFINITY;
                for (int64_t e = lo; e < hi; ++e) {
                    int64_t u = col_idx[e];
                    double el = 0.0;
                    for (int64_t d = 0; d < Dh; ++d) el += (double)as[d] * (double)Z[u * ldz + h * Dh + d];
                    score[e - lo] = leaky(el + er, slope);
                    if (score[e - lo] > m) m = score[e - lo];
                }
                double denom = 0.0;
                for (int64_t e = lo; e < hi; ++e) {
                    score[e - lo] = exp(score[e - lo] - m);
                    denom += score[e - lo];
                }
                for (int64_t d = 0; d < Dh; ++d) {
                    double s = 0.0;
                    for (int64_t e = lo; e < hi; ++e)
                        s += score[e - lo] * (double)Z[(int64_t)col_idx[e] * ldz + h * Dh + d];
                    o[h * Dh + d] = s / denom;
                }
            }
            free(score);
        }
    }
}

void oracle_gat_alpha(int64_t v, int h, const int64_t *row_ptr, const int32_t *col_idx,
                      int64_t F, int heads, const float *Z, int64_t ldz,
                      const float *a_src, const float *a_dst, double slope, double *alpha);

/*
 * The size of the terms behind every output element of oracle_aggregate: with
 * out[v,j] = sum_u c_vu z_uj (c_vu = 1, 1/deg v, dinv_v dinv_u or alpha_vu), this returns
 *     mag[v,j] = sum_u |c_vu z_uj|
 * (the self half under self_concat and the max aggregator have a single term, |z|).
 * It is the yardstick of the condition-aware error measure of the parity tests: a float32
 * evaluation of a sum can only be expected to be accurate relative to the size of its terms,
 * not relative to a result that cancels to nearly zero.  Same arguments and layout as
 * oracle_aggregate.
 */
void oracle_aggregate_abs(int mode, int64_t n_rows, const int64_t *rows,
                          const int64_t *row_ptr, const int32_t *col_idx, const float *dinv,
                          int64_t F, int heads, const float *Z, int64_t ldz,
                          const float *a_src, const float *a_dst, double slope,
                          int self_concat, double *mag)
{
    const int64_t pitch = self_concat ? 2 * F : F;
    const int64_t Dh = (mode == ORACLE_GAT_SOFTMAX) ? F / heads : F;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t v = rows ? rows[i] : i;
        double *o = mag + i * pitch;
        if (self_concat) {
            for (int64_t j = 0; j < F; ++j) o[j] = fabs((double)Z[v * ldz + j]);
            o += F;
        }
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
        const int64_t deg = hi - lo;
        for (int64_t j = 0; j < F; ++j) o[j] = 0.0;
        if (deg == 0) continue;
        const int n_blocks = (mode == ORACLE_GAT_SOFTMAX) ? heads : 1;     /* column blocks sharing coefficients */
        double *alpha = (mode == ORACLE_GAT_SOFTMAX) ? (double *)malloc((size_t)deg * sizeof(double)) : NULL;
        for (int h = 0; h < n_blocks; ++h) {
            if (alpha) oracle_gat_alpha(v, h, row_ptr, col_idx, F, heads, Z, ldz, a_src, a_dst, slope, alpha);
            for (int64_t j = h * Dh; j < (h + 1) * Dh; ++j) {
                double s = 0.0, top = -INFINITY;
                for (int64_t e = lo; e < hi; ++e) {
                    const int64_t u = col_idx[e];
                    const double z = (double)Z[u * ldz + j];
                    double c = 1.0;
                    if (mode == ORACLE_MEAN) c = 1.0 / (double)deg;
                    else if (mode == ORACLE_GCN_SYM) c = (double)dinv[v] * (double)dinv[u];
                    else if (mode == ORACLE_GAT_SOFTMAX) c = alpha[e - lo];
                    s += fabs(c * z);
                    if (z > top) top = z;
                }
                o[j] = (mode == ORACLE_MAX) ? fabs(top) : s;
            }
        }
        free(alpha);
    }
}

/*
 * Attention coefficients alpha_uv of one row and one head, in CSR entry
 * order (deg doubles).  Same formula as above, exposed so that a test can
 * look at the weights themselves.
 */
void oracle_gat_alpha(int64_t v, int h, const int64_t *row_ptr, const int32_t *col_idx,
                      int64_t F, int heads, const float *Z, int64_t ldz,
                      const float *a_src, const float *a_dst, double slope, double *alpha)
{
    const int64_t Dh = F / heads, lo = row_ptr[v], hi = row_ptr[v + 1];
    const float *as = a_src + (int64_t)h * Dh, *ad = a_dst + (int64_t)h * Dh;
    double er = 0.0, m = -INFINITY, denom = 0.0;
    for (int64_t d = 0; d < Dh; ++d) er += (double)ad[d] * (double)Z[v * ldz + h * Dh + d];
    for (int64_t e = lo; e < hi; ++e) {
        int64_t u = col_idx[e];
        double el = 0.0;
        for (int64_t d = 0; d < Dh; ++d) el += (double)as[d] * (double)Z[u * ldz + h * Dh + d];
        alpha[e - lo] = leaky(el + er, slope);
        if (alpha[e - lo] > m) m = alpha[e - lo];
    }
    for (int64_t e = lo; e < hi; ++e) { alpha[e - lo] = exp(alpha[e - lo] - m); denom += alpha[e - lo]; }
    for (int64_t e = lo; e < hi; ++e) alpha[e - lo] /= denom;
}

/* ---------------------------------------------------------------------------
 * Backward of the aggregation (needed to train a layer whose AGGR has
 * trainable parameters — the gloss under Eq. 1 allows that, and GAT's
 * attention vectors are such parameters — with the aggregation inside the
 * local training loop).  Given G = dL/d(out) this returns dL/dZ and, for gat,
 * dL/da_src and dL/da_dst, by the chain rule through the definitions above.
 *
 * Every CSR entry (v,u) of the forward pass carries a coefficient c_vu with
 * out_v = sum_u c_vu z_u:   mean 1/deg v,  sum 1,  gcn_sym dinv_v dinv_u,
 * gat alpha_vu (per head).  The direct term is dL/dz_u += c_vu G_v.
 * For gat the coefficients themselves depend on Z, a_src, a_dst:
 *      dL/dalpha_vu = <G_v, z_u>                               (out_v is linear in alpha)
 *      dL/de_vu     = alpha_vu ( dL/dalpha_vu - sum_w alpha_vw dL/dalpha_vw )   (softmax)
 *      dL/dp_vu     = dL/de_vu * (p_vu > 0 ? 1 : slope),  p_vu = <a_src,z_u> + <a_dst,z_v>
 *      dL/dz_u += dL/dp_vu a_src,   dL/dz_v += dL/dp_vu a_dst,
 *      dL/da_src += dL/dp_vu z_u,   dL/da_dst += dL/dp_vu z_v        (all per head)
 * With self_concat the forward output was [z_v | aggregate], G is 2F wide and
 * its first F columns flow straight into dL/dz_v.
 *
 * Nothing here assumes that the graph is symmetric: the entries that point at
 * a node u are found through an explicit transpose of the CSR.
 *
 * rows == NULL: dZ is [N, F] and da_src / da_dst ([F] each, gat only) are
 * filled.  rows given: only those rows of dZ ([n_rows, F]); da_* untouched.
 * max has no backward here (returns -1).  Returns 0 on success.
 */
static int aggregate_backward_impl(int mode, int64_t N, int64_t n_rows, const int64_t *rows,
                                   const int64_t *row_ptr, const int32_t *col_idx, const float *dinv,
                                   int64_t F, int heads, const float *Z, int64_t ldz,
                                   const float *a_src, const float *a_dst, double slope,
                                   const float *G, int64_t ldg, int self_concat,
                                   double *dZ, double *da_src, double *da_dst,
                                   double kink_rel, double *slack)
{
    if (mode == ORACLE_MAX) return -1;
    const int gat = mode == ORACLE_GAT_SOFTMAX;
    if (!gat) heads = 1;
    const int64_t Dh = F / heads, nnz = row_ptr[N];
    const float *Ga = G + (self_concat ? F : 0);      /* gradient of the aggregate half */

    /* transpose: for every node u the entries e (and their rows v) with col_idx[e] == u */
    int64_t *t_ptr = (int64_t *)calloc((size_t)N + 2, sizeof(int64_t));
    int64_t *t_ent = (int64_t *)malloc((size_t)(nnz ? nnz : 1) * sizeof(int64_t));
    int32_t *t_row = (int32_t *)malloc((size_t)(nnz ? nnz : 1) * sizeof(int32_t));
    for (int64_t e = 0; e < nnz; ++e) t_ptr[col_idx[e] + 2]++;
    for (int64_t u = 0; u < N; ++u) t_ptr[u + 2] += t_ptr[u + 1];
    for (int64_t v = 0; v < N; ++v)
        for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            const int64_t k = t_ptr[col_idx[e] + 1]++;
            t_ent[k] = e;
            t_row[k] = (int32_t)v;
        }
    /* now t_ptr[u] .. t_ptr[u+1] delimit node u's incoming entries */

    /* which rows' entry coefficients are needed, and where they are kept */
    unsigned char *need = (unsigned char *)calloc((size_t)N + 1, 1);
    int64_t *off = (int64_t *)malloc(((size_t)N + 1) * sizeof(int64_t));
    if (rows) {
        for (int64_t i = 0; i < n_rows; ++i) {
            const int64_t u = rows[i];
            need[u] = 1;
            for (int64_t k = t_ptr[u]; k < t_ptr[u + 1]; ++k) need[t_row[k]] = 1;
        }
    } else {
        memset(need, 1, (size_t)N);
    }
    int64_t kept = 0;
    for (int64_t v = 0; v < N; ++v) {
        off[v] = kept;
        if (need[v]) kept += row_ptr[v + 1] - row_ptr[v];
    }
    double *coef = (double *)malloc((size_t)(kept ? kept : 1) * heads * sizeof(double));  /* c_vu  */
    double *dp = (double *)calloc((size_t)(kept ? kept : 1) * heads, sizeof(double));     /* dL/dp */
    /* |change of dL/dp| if the entry's score p were taken on the other side of the LeakyReLU kink (slack only) */
    double *ks = (slack && gat) ? (double *)calloc((size_t)(kept ? kept : 1) * heads, sizeof(double)) : NULL;

    /* step 1: coefficient and score gradient of every needed entry */
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t v = 0; v < N; ++v) {
        if (!need[v]) continue;
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1], deg = hi - lo;
        double *cv = coef + off[v] * heads, *dv = dp + off[v] * heads;
        if (!gat) {
            for (int64_t e = lo; e < hi; ++e)
                cv[e - lo] = mode == ORACLE_MEAN ? 1.0 / (double)deg
                           : mode == ORACLE_SUM  ? 1.0
                           : (double)dinv[v] * (double)dinv[col_idx[e]];
            continue;
        }
        if (deg == 0) continue;
        double *p = (double *)malloc((size_t)deg * sizeof(double));
        double *da = (double *)malloc((size_t)deg * sizeof(double));
        double *pmag = (double *)malloc((size_t)deg * sizeof(double));   /* size of the terms of p (slack only) */
        for (int h = 0; h < heads; ++h) {
            const float *as = a_src + (int64_t)h * Dh, *ad = a_dst + (int64_t)h * Dh;
            const float *zv = Z + v * ldz + h * Dh, *gv = Ga + v * ldg + h * Dh;
            double er = 0.0, er_mag = 0.0, m = -INFINITY, denom = 0.0, mean_da = 0.0;
            for (int64_t d = 0; d < Dh; ++d) {
                er += (double)ad[d] * (double)zv[d];
                er_mag += fabs((double)ad[d] * (double)zv[d]);
            }
            for (int64_t e = lo; e < hi; ++e) {
                const float *zu = Z + (int64_t)col_idx[e] * ldz + h * Dh;
                double el = 0.0, g = 0.0, el_mag = 0.0;
                for (int64_t d = 0; d < Dh; ++d) {
                    el += (double)as[d] * (double)zu[d];
                    el_mag += fabs((double)as[d] * (double)zu[d]);
                    g += (double)gv[d] * (double)zu[d];
                }
                pmag[e - lo] = el_mag + er_mag;
                p[e - lo] = el + er;
                da[e - lo] = g;
                if (leaky(p[e - lo], slope) > m) m = leaky(p[e - lo], slope);
            }
            for (int64_t j = 0; j < deg; ++j) denom += exp(leaky(p[j], slope) - m);
            for (int64_t j = 0; j < deg; ++j) {
                cv[j * heads + h] = exp(leaky(p[j], slope) - m) / denom;
                mean_da += cv[j * heads + h] * da[j];
            }
            for (int64_t j = 0; j < deg; ++j) {
                dv[j * heads + h] = cv[j * heads + h] * (da[j] - mean_da) * (p[j] > 0.0 ? 1.0 : slope);
                if (ks && fabs(p[j]) <= kink_rel * pmag[j])
                    ks[(off[v] + j) * heads + h] = fabs(cv[j * heads + h] * (da[j] - mean_da) * (1.0 - slope));
            }
        }
        free(p);
        free(da);
        free(pmag);
    }

    /* step 2: collect what flows into each requested node */
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t u = rows ? rows[i] : i;
        double *o = dZ + i * F;
        for (int64_t j = 0; j < F; ++j) o[j] = self_concat ? (double)G[u * ldg + j] : 0.0;
        for (int64_t k = t_ptr[u]; k < t_ptr[u + 1]; ++k) {       /* entries (v,u) */
            const int64_t e = t_ent[k], v = t_row[k];
            const int64_t q = (off[v] + (e - row_ptr[v])) * heads;
            for (int h = 0; h < heads; ++h)
                for (int64_t d = 0; d < Dh; ++d) {
                    o[h * Dh + d] += coef[q + h] * (double)Ga[v * ldg + h * Dh + d];
                    if (gat) o[h * Dh + d] += dp[q + h] * (double)a_src[h * Dh + d];
                }
        }
        if (gat)
            for (int64_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) {   /* u's own entries (u,w) */
                const int64_t q = (off[u] + (e - row_ptr[u])) * heads;
                for (int h = 0; h < heads; ++h)
                    for (int64_t d = 0; d < Dh; ++d) o[h * Dh + d] += dp[q + h] * (double)a_dst[h * Dh + d];
            }
        if (slack) {
            double *sl = slack + i * F;
            for (int64_t j = 0; j < F; ++j) sl[j] = 0.0;
            if (ks) {
                for (int64_t k = t_ptr[u]; k < t_ptr[u + 1]; ++k) {
                    const int64_t e = t_ent[k], v = t_row[k];
                    const int64_t q = (off[v] + (e - row_ptr[v])) * heads;
                    for (int h = 0; h < heads; ++h)
                        for (int64_t d = 0; d < Dh; ++d) sl[h * Dh + d] += ks[q + h] * fabs((double)a_src[h * Dh + d]);
                }
                for (int64_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) {
                    const int64_t q = (off[u] + (e - row_ptr[u])) * heads;
                    for (int h = 0; h < heads; ++h)
                        for (int64_t d = 0; d < Dh; ++d) sl[h * Dh + d] += ks[q + h] * fabs((double)a_dst[h * Dh + d]);
                }
            }
        }
    }

    /* step 3: gradients of the attention vectors (sums over every entry of the graph) */
    if (gat && !rows && da_src && da_dst) {
        for (int64_t j = 0; j < F; ++j) { da_src[j] = 0.0; da_dst[j] = 0.0; }
        for (int64_t v = 0; v < N; ++v)
            for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                const int64_t q = (off[v] + (e - row_ptr[v])) * heads, u = col_idx[e];
                for (int h = 0; h < heads; ++h)
                    for (int64_t d = 0; d < Dh; ++d) {
                        da_src[h * Dh + d] += dp[q + h] * (double)Z[u * ldz + h * Dh + d];
                        da_dst[h * Dh + d] += dp[q + h] * (double)Z[v * ldz + h * Dh + d];
                    }
            }
    }
    free(coef); free(dp); free(ks); free(need); free(off); free(t_ptr); free(t_ent); free(t_row);
    return 0;
}

int oracle_aggregate_backward(int mode, int64_t N, int64_t n_rows, const int64_t *rows,
                              const int64_t *row_ptr, const int32_t *col_idx, const float *dinv,
                              int64_t F, int heads, const float *Z, int64_t ldz,
                              const float *a_src, const float *a_dst, double slope,
                              const float *G, int64_t ldg, int self_concat,
                              double *dZ, double *da_src, double *da_dst)
{
    return aggregate_backward_impl(mode, N, n_rows, rows, row_ptr, col_idx, dinv, F, heads, Z, ldz, a_src, a_dst,
                                   slope, G, ldg, self_concat, dZ, da_src, da_dst, 0.0, NULL);
}

/*
 * The same gradient, plus how much each element of dZ depends on a decision no float32 evaluation can
 * be held to: the derivative of LeakyReLU jumps from slope to 1 at p = 0, and an entry whose score
 * p_vu = <a_src,z_u> + <a_dst,z_v> lies within rounding of zero can land on either side.  Both values
 * are then correct results of the method (the forward pass is continuous there).  An entry counts as
 * undecided when |p_vu| <= kink_rel * (sum_d |a_src,d z_u,d| + sum_d |a_dst,d z_v,d|), i.e. within
 * kink_rel of the size of the terms p is the sum of; taking the other side changes dL/dp_vu by
 * (1 - slope) |alpha_vu (dL/dalpha_vu - c_v)|, which reaches dZ_u through |a_src| and dZ_v through |a_dst|.
 * slack[i, :] (n_rows x F) receives the sum of those magnitudes for row rows[i]; it is zero for a row
 * that no undecided entry touches, and zero everywhere for the modes without a kink.
 */
int oracle_aggregate_backward_slack(int mode, int64_t N, int64_t n_rows, const int64_t *rows,
                                    const int64_t *row_ptr, const int32_t *col_idx, const float *dinv,
                                    int64_t F, int heads, const float *Z, int64_t ldz,
                                    const float *a_src, const float *a_dst, double slope,
                                    const float *G, int64_t ldg, int self_concat,
                                    double *dZ, double *da_src, double *da_dst,
                                    double kink_rel, double *slack)
{
    return aggregate_backward_impl(mode, N, n_rows, rows, row_ptr, col_idx, dinv, F, heads, Z, ldz, a_src, a_dst,
                                   slope, G, ldg, self_concat, dZ, da_src, da_dst, kink_rel, slack);
}

/* ---------------------------------------------------------------------------
 * The random draws of dropout.  Both sides of a parity test must draw the same
 * mask, so the mask is a pure function of (seed, draw, node, unit) through a
 * counter-based generator: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror,
 * Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC 2011).  One block
 * gives four 32-bit words:
 *      counter = (node, unit / 4, low word of draw, high word of draw)
 *      key     = (low word of seed, high word of seed)
 * and unit j takes word j % 4.  The unit is dropped when its word is below
 * floor(p * 2^32) (p is a float, so the product is exact in double) and kept
 * otherwise: p = 0 keeps everything.
 * A round multiplies counter words 0 and 2 by two fixed odd constants, swaps the
 * halves of the products into place and mixes the other two words and the key in;
 * the key grows by two fixed increments between rounds.
 * ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;      /* golden ratio */
            k1 += 0xBB67AE85u;      /* sqrt(3) - 1 */
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* keep[v * H + j] = 1 if unit j of node v survives the dropout of probability p_drop */
void oracle_dropout_keep(int64_t N, int64_t H, float p_drop, uint64_t seed, uint64_t draw, uint8_t *keep)
{
    const uint32_t threshold = (uint32_t)((double)p_drop * 4294967296.0);
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int64_t v = 0; v < N; ++v)
        for (int64_t q = 0; 4 * q < H; ++q) {
            const uint32_t counter[4] = {(uint32_t)v, (uint32_t)q, (uint32_t)draw, (uint32_t)(draw >> 32)};
            uint32_t w[4];
            oracle_philox4x32_10(counter, key, w);
            for (int64_t k = 0; k < 4 && 4 * q + k < H; ++k) keep[v * H + 4 * q + k] = w[k] >= threshold;
        }
}

/* ---------------------------------------------------------------------------
 * Local training of one layer (section "Lazy Message Passing": a layer is
 * trained by itself on its fixed aggregated inputs, with a temporary
 * classification layer C added on top, using stochastic gradient descent; the
 * appendix sizes C as an H_m x H_K linear map).  Read here as
 *      A      = ReLU(X W1 + b1)                       the layer's f (Eq. 1)
 *      logits = A Wc + bc                             the temporary classifier
 *      loss   = mean over labelled nodes of  -log softmax(logits)[label]
 * and, when H == 0, the layer is the final classification function itself:
 *      logits = X W1 + b1   (W1 is [D_in, C]).
 * A node with label < 0 is not a training node and contributes nothing.
 * This function returns the loss and its gradient with respect to every
 * parameter, all in double:  gW1 [D_in, H or C], gb1, gWc [H, C], gbc [C];
 * and, when gX is not NULL, with respect to the layer's input, gX [N, D_in]
 * (zero rows for nodes that are not training nodes) — what flows back into an
 * aggregation with trainable parameters that produced X.
 * With no labelled node the loss and all gradients are zero.
 *
 * Dropout (the appendix on hyper-parameters trains with dropout 0.3 or 0.5; where it
 * sits is not said, it is taken on the layer's output A, in front of the temporary
 * classifier): with keep != NULL, keep[v * H + j] in {0, 1},
 *      A_vj = keep_vj ? scale * ReLU(X W1 + b1)_vj : 0,      scale = 1 / (1 - p),
 * and the gradients are those of the loss with this fixed mask.  keep == NULL is the
 * step without dropout.  oracle_dropout_keep below draws the mask.
 */
double oracle_layer_grad(int64_t N, int64_t D_in, int64_t H, int64_t C,
                         const float *X, int64_t ldx, const int32_t *labels,
                         const float *W1, const float *b1, const float *Wc, const float *bc,
                         double *gW1, double *gb1, double *gWc, double *gbc, double *gX,
                         const uint8_t *keep, double scale)
{
    const int64_t W1cols = H > 0 ? H : C;
    if (gX) for (int64_t i = 0; i < N * D_in; ++i) gX[i] = 0.0;
    for (int64_t i = 0; i < D_in * W1cols; ++i) gW1[i] = 0.0;
    for (int64_t i = 0; i < W1cols; ++i) gb1[i] = 0.0;
    if (H > 0) {
        for (int64_t i = 0; i < H * C; ++i) gWc[i] = 0.0;
        for (int64_t i = 0; i < C; ++i) gbc[i] = 0.0;
    }
    int64_t n_lab = 0;
    for (int64_t v = 0; v < N; ++v) n_lab += labels[v] >= 0;
    if (n_lab == 0) return 0.0;

    double *a = (double *)malloc((size_t)(H > 0 ? H : 1) * sizeof(double));
    double *z = (double *)malloc((size_t)C * sizeof(double));
    double *da = (double *)malloc((size_t)(H > 0 ? H : 1) * sizeof(double));
    double loss = 0.0;
    for (int64_t v = 0; v < N; ++v) {
        const int32_t y = labels[v];
        if (y < 0) continue;
        const float *x = X + v * ldx;
        if (H > 0) {
            for (int64_t j = 0; j < H; ++j) {
                double s = (double)b1[j];
                for (int64_t k = 0; k < D_in; ++k) s += (double)x[k] * (double)W1[k * H + j];
                a[j] = s > 0.0 ? s : 0.0;
                if (keep) a[j] = keep[v * H + j] ? scale * a[j] : 0.0;
            }
            for (int64_t c = 0; c < C; ++c) {
                double s = (double)bc[c];
                for (int64_t j = 0; j < H; ++j) s += a[j] * (double)Wc[j * C + c];
                z[c] = s;
            }
        } else {
            for (int64_t c = 0; c < C; ++c) {
                double s = (double)b1[c];
                for (int64_t k = 0; k < D_in; ++k) s += (double)x[k] * (double)W1[k * C + c];
                z[c] = s;
            }
        }
        double m = z[0];
        for (int64_t c = 1; c < C; ++c) if (z[c] > m) m = z[c];
        double den = 0.0;
        for (int64_t c = 0; c < C; ++c) den += exp(z[c] - m);
        loss += -(z[y] - m - log(den));
        /* z becomes d loss / d logits for this node */
        for (int64_t c = 0; c < C; ++c) z[c] = (exp(z[c] - m) / den - (c == y ? 1.0 : 0.0)) / (double)n_lab;
        if (H > 0) {
            for (int64_t c = 0; c < C; ++c) gbc[c] += z[c];
            for (int64_t j = 0; j < H; ++j) {
                double s = 0.0;
                for (int64_t c = 0; c < C; ++c) {
                    gWc[j * C + c] += a[j] * z[c];
                    s += z[c] * (double)Wc[j * C + c];
                }
                /* a_j > 0 exactly when the unit is active and kept */
                da[j] = a[j] > 0.0 ? (keep ? scale * s : s) : 0.0;
            }
            for (int64_t j = 0; j < H; ++j) gb1[j] += da[j];
            for (int64_t k = 0; k < D_in; ++k) {
                const double xk = (double)x[k];
                double gx = 0.0;
                for (int64_t j = 0; j < H; ++j) {
                    gW1[k * H + j] += xk * da[j];
                    gx += da[j] * (double)W1[k * H + j];
                }
                if (gX) gX[v * D_in + k] = gx;
            }
        } else {
            for (int64_t c = 0; c < C; ++c) gb1[c] += z[c];
            for (int64_t k = 0; k < D_in; ++k) {
                const double xk = (double)x[k];
                double gx = 0.0;
                for (int64_t c = 0; c < C; ++c) {
                    gW1[k * C + c] += xk * z[c];
                    gx += z[c] * (double)W1[k * C + c];
                }
                if (gX) gX[v * D_in + k] = gx;
            }
        }
    }
    free(a); free(z); free(da);
    return loss / (double)n_lab;
}

/*
 * Parameter gradients of the dense transform Z = H W + b given dZ = dL/dZ:
 *      gW[k, j] = sum_v H[v, k] dZ[v, j],    gb[j] = sum_v dZ[v, j]
 * (the transform in front of an aggregation is trained through the
 * aggregation's backward, which supplies dZ).
 */
void oracle_transform_backward(int64_t N, int64_t D_in, int64_t D_out, const float *H, int64_t ldh,
                               const float *dZ, int64_t lddz, double *gW, double *gb)
{
    for (int64_t j = 0; j < D_out; ++j) {
        double s = 0.0;
        for (int64_t v = 0; v < N; ++v) s += (double)dZ[v * lddz + j];
        gb[j] = s;
    }
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < D_in; ++k)
        for (int64_t j = 0; j < D_out; ++j) {
            double s = 0.0;
            for (int64_t v = 0; v < N; ++v) s += (double)H[v * ldh + k] * (double)dZ[v * lddz + j];
            gW[k * D_out + j] = s;
        }
}

/* The loss alone (same formula), used by the tests to difference numerically. */
double oracle_layer_loss(int64_t N, int64_t D_in, int64_t H, int64_t C,
                         const float *X, int64_t ldx, const int32_t *labels,
                         const double *W1, const double *b1, const double *Wc, const double *bc,
                         const uint8_t *keep, double scale)
{
    int64_t n_lab = 0;
    double loss = 0.0;
    double *a = (double *)malloc((size_t)(H > 0 ? H : 1) * sizeof(double));
    double *z = (double *)malloc((size_t)C * sizeof(double));
    for (int64_t v = 0; v < N; ++v) {
        const int32_t y = labels[v];
        if (y < 0) continue;
        ++n_lab;
        const float *x = X + v * ldx;
        if (H > 0) {
            for (int64_t j = 0; j < H; ++j) {
                double s = b1[j];
                for (int64_t k = 0; k < D_in; ++k) s += (double)x[k] * W1[k * H + j];
                a[j] = s > 0.0 ? s : 0.0;
                if (keep) a[j] = keep[v * H + j] ? scale * a[j] : 0.0;
            }
            for (int64_t c = 0; c < C; ++c) {
                double s = bc[c];
                for (int64_t j = 0; j < H; ++j) s += a[j] * Wc[j * C + c];
                z[c] = s;
            }
        } else {
            for (int64_t c = 0; c < C; ++c) {
                double s = b1[c];
                for (int64_t k = 0; k < D_in; ++k) s += (double)x[k] * W1[k * C + c];
                z[c] = s;
            }
        }
        double m = z[0];
        for (int64_t c = 1; c < C; ++c) if (z[c] > m) m = z[c];
        double den = 0.0;
        for (int64_t c = 0; c < C; ++c) den += exp(z[c] - m);
        loss += -(z[y] - m - log(den));
    }
    free(a); free(z);
    return n_lab ? loss / (double)n_lab : 0.0;
}
