/*
 * CPU oracle for the broadcast-based GNN layer step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker, not the product: it is called from tests, from the
 * smoke check and from the benchmark's CPU-baseline leg, and from nowhere else.
 * It shares no code, header, table or helper with the GPU library.
 *
 * The paper states that pushing each source's embedding along its out-edges is,
 * per layer, semantically equal to every destination pulling from its
 * in-neighbours (Sec. 3.1, "Broadcast Execution Model", Fig. 2).  So the oracle
 * is the plain definition written out as a pull: for every destination, walk
 * its in-neighbour list and accumulate in fp64.  No chunks, no counters, no
 * atomics.  Integer side products (pending counts, completion chunk, the
 * degree ordering) are derived from the in-neighbour lists directly, never by
 * simulating the message stream.
 *
 * Layer definitions:
 *   mean aggregation / SAGE: Sec. 3.4 (layer formula with 1/|N(v)| mean), and
 *       Sec. 4.3 for the concatenation of a vertex's own embedding;
 *   GCN: symmetric normalisation of Kipf & Welling (the paper's "GraphConv",
 *       Sec. 4.1, gives no formula) with D = in-degree of the graph as given;
 *   GAT: the textbook attention layer (the paper only names it as adoptable,
 *       Sec. 3.9), plain two-pass softmax over the in-neighbour multiset;
 *   GIN: the sum-aggregation layer of Xu et al. that the paper evaluates as
 *       "GINConv" (Sec. 4.1, no formula given): y_v = ((1+eps) x_v + sum x_u) W + b,
 *       with a single linear map standing for the layer's MLP;
 *   SGC hop: one application of the symmetric-normalised adjacency without a
 *       weight matrix (Wu et al.; named as adoptable in Sec. 3.9);
 *   completion: a vertex is complete when it has received d_in(v) messages
 *       (Sec. 3.8, k_v(t) = d_in(v)).
 *
 * Multi-edges count with multiplicity everywhere.  fp64 throughout; inputs are
 * the already-rounded storage values (passed as float).  Storage formats: fp32,
 * bf16 and IEEE half precision (the paper's largest feature set is stored in
 * FP16, Sec. 4.1), each a single round-to-nearest-even of the fp64 result.
 *
 * Pins: tests/test_oracle_pins.py (dense adjacency brute force, the Fig. 2 worked
 * example, closed forms, permutation invariance, counter invariants) and
 * tests/test_oracle_subset_pins.py (the same functions called on a subset of the
 * destinations with renumbered ids, against the dense brute force; the placement
 * of the activation in a chain of layers; planted slips that the pins must catch).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ao_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* indeg[v] = number of edges whose destination is v. */
void ao_in_degree(int64_t n, int64_t num_edges, const int32_t *col, int64_t *indeg) {
    for (int64_t v = 0; v < n; ++v) indeg[v] = 0;
    for (int64_t e = 0; e < num_edges; ++e) indeg[col[e]] += 1;
}

/* In-neighbour lists from a CSR by source.  Sources appear in ascending order
 * (with multiplicity) inside each destination's list. */
void ao_build_in_lists(int64_t n, const int64_t *off, const int32_t *col,
                       int64_t *in_off, int32_t *in_src) {
    int64_t num_edges = off[n];
    for (int64_t v = 0; v <= n; ++v) in_off[v] = 0;
    for (int64_t e = 0; e < num_edges; ++e) in_off[col[e] + 1] += 1;
    for (int64_t v = 0; v < n; ++v) in_off[v + 1] += in_off[v];
    int64_t *cur = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    for (int64_t v = 0; v < n; ++v) cur[v] = in_off[v];
    for (int64_t u = 0; u < n; ++u)
        for (int64_t e = off[u]; e < off[u + 1]; ++e) in_src[cur[col[e]]++] = (int32_t)u;
    free(cur);
}

/* S[i][:] = sum over in-neighbours u of destination i of scale[u] * X[u][:]
 * (scale == NULL means 1). */
void ao_neighbor_sum(int64_t n_dst, const int64_t *in_off, const int32_t *in_src,
                     const float *X, int64_t d, const double *scale, double *S) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_dst; ++i) {
        double *s = S + i * d;
        for (int64_t k = 0; k < d; ++k) s[k] = 0.0;
        for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p) {
            int64_t u = in_src[p];
            const float *x = X + u * d;
            double g = scale ? scale[u] : 1.0;
            for (int64_t k = 0; k < d; ++k) s[k] += g * (double)x[k];
        }
    }
}

/* Y[i][:] = A[i][:] * W + b, A is n x K (fp64), W is K x dout row-major. */
void ao_affine(int64_t n, const double *A, int64_t K, const double *W, const double *b,
               int64_t dout, double *Y) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *y = Y + i * dout;
        for (int64_t j = 0; j < dout; ++j) y[j] = b ? b[j] : 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = A[i * K + k];
            const double *w = W + k * dout;
            for (int64_t j = 0; j < dout; ++j) y[j] += a * w[j];
        }
    }
}

static int64_t dst_id(const int64_t *dst_ids, int64_t i) { return dst_ids ? dst_ids[i] : i; }

/* GraphSAGE-mean: y_v = [x_v || mean_{u in N(v)} x_u] * W + b, W is 2d x dout.
 * The mean of an empty neighbourhood is 0.  Destination i is vertex
 * dst_ids[i] (or i); in_off / in_src are indexed by i. */
void ao_sage_mean(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off,
                  const int32_t *in_src, const float *X, int64_t d, const double *W,
                  const double *b, int64_t dout, double *Y) {
    double *S = (double *)malloc((size_t)(n_dst > 0 ? n_dst : 1) * d * sizeof(double));
    double *A = (double *)malloc((size_t)(n_dst > 0 ? n_dst : 1) * 2 * d * sizeof(double));
    ao_neighbor_sum(n_dst, in_off, in_src, X, d, NULL, S);
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        int64_t deg = in_off[i + 1] - in_off[i];
        for (int64_t k = 0; k < d; ++k) {
            A[i * 2 * d + k] = (double)X[v * d + k];
            A[i * 2 * d + d + k] = deg > 0 ? S[i * d + k] / (double)deg : 0.0;
        }
    }
    ao_affine(n_dst, A, 2 * d, W, b, dout, Y);
    free(S);
    free(A);
}

/* GCN: y_v = (sum_{u in N(v)} x_u / sqrt(D_u D_v)) * W + b with D = indeg of the
 * graph as given (the caller has already added one self-edge per vertex).
 * indeg is indexed by vertex id and covers all n vertices. */
void ao_gcn(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off, const int32_t *in_src,
            int64_t n, const int64_t *indeg, const float *X, int64_t d, const double *W,
            const double *b, int64_t dout, double *Y) {
    double *S = (double *)malloc((size_t)(n_dst > 0 ? n_dst : 1) * d * sizeof(double));
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        double *s = S + i * d;
        for (int64_t k = 0; k < d; ++k) s[k] = 0.0;
        for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p) {
            int64_t u = in_src[p];
            double g = 1.0 / sqrt((double)indeg[u] * (double)indeg[v]);
            for (int64_t k = 0; k < d; ++k) s[k] += g * (double)X[u * d + k];
        }
    }
    (void)n;
    ao_affine(n_dst, S, d, W, b, dout, Y);
    free(S);
}

/* GIN: y_v = ((1 + eps) x_v + sum_{u in N(v)} x_u) * W + b, W is d x dout. */
void ao_gin(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off, const int32_t *in_src,
            const float *X, int64_t d, double eps, const double *W, const double *b, int64_t dout,
            double *Y) {
    double *S = (double *)malloc((size_t)(n_dst > 0 ? n_dst : 1) * d * sizeof(double));
    ao_neighbor_sum(n_dst, in_off, in_src, X, d, NULL, S);
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        for (int64_t k = 0; k < d; ++k) S[i * d + k] += (1.0 + eps) * (double)X[v * d + k];
    }
    ao_affine(n_dst, S, d, W, b, dout, Y);
    free(S);
}

/* SGC hop: y_v = sum_{u in N(v)} x_u / sqrt(D_u D_v), D = in-degree of the graph as
 * given (self-edges already added by the caller); no weights, Y is n_dst x d. */
void ao_sym_propagate(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off,
                      const int32_t *in_src, const int64_t *indeg, const float *X, int64_t d,
                      double *Y) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        double *y = Y + i * d;
        for (int64_t k = 0; k < d; ++k) y[k] = 0.0;
        for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p) {
            int64_t u = in_src[p];
            double g = 1.0 / sqrt((double)indeg[u] * (double)indeg[v]);
            for (int64_t k = 0; k < d; ++k) y[k] += g * (double)X[u * d + k];
        }
    }
}

/* Z[r][:] = X[r][:] * W for the listed rows r (row_ids == NULL: all n_rows
 * rows); Z is indexed by vertex id like X.  Used for the GAT transform. */
void ao_linear_rows(int64_t n_rows, const int64_t *row_ids, const float *X, int64_t d,
                    const double *W, int64_t dout, double *Z) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t r = row_ids ? row_ids[i] : i;
        double *z = Z + r * dout;
        for (int64_t j = 0; j < dout; ++j) z[j] = 0.0;
        for (int64_t k = 0; k < d; ++k) {
            double a = (double)X[r * d + k];
            const double *w = W + k * dout;
            for (int64_t j = 0; j < dout; ++j) z[j] += a * w[j];
        }
    }
}

/* GAT attention over already-transformed rows Z (n x heads*dh, by vertex id):
 *   s_uv^k = LeakyReLU(a_src^k . z_u^k + a_dst^k . z_v^k)
 *   alpha  = softmax over the in-neighbour multiset of v (two passes)
 *   y_v    = concat_k sum_u alpha_uv^k z_u^k + b ;  empty neighbourhood: y_v = b. */
void ao_gat_attend(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off,
                   const int32_t *in_src, const double *Z, const double *a_src,
                   const double *a_dst, int64_t heads, int64_t dh, double slope,
                   const double *b, double *Y) {
    int64_t dout = heads * dh;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        double *y = Y + i * dout;
        for (int64_t h = 0; h < heads; ++h) {
            const double *as = a_src + h * dh, *ad = a_dst + h * dh;
            double er = 0.0;
            for (int64_t k = 0; k < dh; ++k) er += ad[k] * Z[v * dout + h * dh + k];
            double smax = -INFINITY;
            for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p) {
                const double *zu = Z + (int64_t)in_src[p] * dout + h * dh;
                double el = 0.0;
                for (int64_t k = 0; k < dh; ++k) el += as[k] * zu[k];
                double s = el + er;
                s = s > 0.0 ? s : slope * s;
                if (s > smax) smax = s;
            }
            double denom = 0.0;
            for (int64_t k = 0; k < dh; ++k) y[h * dh + k] = 0.0;
            for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p) {
                const double *zu = Z + (int64_t)in_src[p] * dout + h * dh;
                double el = 0.0;
                for (int64_t k = 0; k < dh; ++k) el += as[k] * zu[k];
                double s = el + er;
                s = s > 0.0 ? s : slope * s;
                double w = exp(s - smax);
                denom += w;
                for (int64_t k = 0; k < dh; ++k) y[h * dh + k] += w * zu[k];
            }
            for (int64_t k = 0; k < dh; ++k)
                y[h * dh + k] = (denom > 0.0 ? y[h * dh + k] / denom : 0.0) + (b ? b[h * dh + k] : 0.0);
        }
    }
}

/* In-place activation: 0 none, 1 ReLU, 2 ELU (alpha = 1). */
void ao_activation(int64_t count, double *Y, int kind) {
    for (int64_t i = 0; i < count; ++i) {
        double y = Y[i];
        if (kind == 1) Y[i] = y > 0.0 ? y : 0.0;
        else if (kind == 2) Y[i] = y > 0.0 ? y : expm1(y);
    }
}

/* Round to the storage format, round-to-nearest-even: 0 = fp32, 1 = bf16
 * (8 significant bits, fp32 exponent range; subnormal results go through fp32). */
void ao_round_storage(int64_t count, double *Y, int fmt) {
    for (int64_t i = 0; i < count; ++i) {
        double y = Y[i];
        if (fmt == 0) { Y[i] = (double)(float)y; continue; }
        if (y == 0.0 || !isfinite(y)) continue;
        if (fmt == 2) {   /* IEEE binary16: 11-bit significand, normals from 2^-14, subnormals in steps of 2^-24 */
            int e16;
            double m16 = frexp(y, &e16);
            if (fabs(y) >= 65520.0) { Y[i] = y > 0 ? INFINITY : -INFINITY; continue; }   /* halfway to 2^16 rounds up */
            if (e16 >= -13) Y[i] = ldexp(nearbyint(m16 * 2048.0), e16 - 11);
            else Y[i] = ldexp(nearbyint(ldexp(y, 24)), -24);
            continue;
        }
        int e;
        double m = frexp(y, &e);              /* y = m * 2^e, 0.5 <= |m| < 1 */
        if (e < -120) { Y[i] = 0.0; continue; }
        Y[i] = ldexp(nearbyint(m * 256.0), e - 8);
    }
}

/* completion_chunk[i] = floor(max(in-neighbours of v, and v itself when the
 * model sends a self message) / C) for destination i = vertex v = dst_ids[i]
 * (or i); -1 when that set is empty (complete at layer start).  Source ids in
 * in_src are the ids the chunks are streamed in. */
void ao_completion_chunk(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off,
                         const int32_t *in_src, int selfmsg, int64_t C, int64_t *cc) {
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        int64_t last = selfmsg ? v : -1;
        for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p)
            if (in_src[p] > last) last = in_src[p];
        cc[i] = last < 0 ? -1 : last / C;
    }
}

/* pending of destination i (vertex v = dst_ids[i] or i) after all sources < bound
 * have been broadcast:
 * d_in(v) + selfmsg - #{in-neighbours u < bound} - [selfmsg and v < bound]. */
void ao_pending_after(int64_t n_dst, const int64_t *dst_ids, const int64_t *in_off,
                      const int32_t *in_src, int selfmsg, int64_t bound, int64_t *pending) {
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t v = dst_id(dst_ids, i);
        int64_t got = 0;
        for (int64_t p = in_off[i]; p < in_off[i + 1]; ++p) got += in_src[p] < bound;
        if (selfmsg && v < bound) got += 1;
        pending[i] = (in_off[i + 1] - in_off[i]) + (selfmsg ? 1 : 0) - got;
    }
}

/* old_of_new = vertex ids sorted by in-degree descending, ties by smaller id
 * first; new_of_old is its inverse.  Plain insertion into degree buckets. */
void ao_reorder_indegree_desc(int64_t n, const int64_t *indeg, int32_t *new_of_old,
                              int32_t *old_of_new) {
    int64_t maxd = 0;
    for (int64_t v = 0; v < n; ++v) if (indeg[v] > maxd) maxd = indeg[v];
    int64_t *start = (int64_t *)calloc((size_t)maxd + 2, sizeof(int64_t));
    for (int64_t v = 0; v < n; ++v) start[maxd - indeg[v] + 1] += 1;   /* bucket 0 = largest degree */
    for (int64_t k = 0; k <= maxd; ++k) start[k + 1] += start[k];
    for (int64_t v = 0; v < n; ++v) {
        int64_t pos = start[maxd - indeg[v]]++;
        old_of_new[pos] = (int32_t)v;
    }
    for (int64_t i = 0; i < n; ++i) new_of_old[old_of_new[i]] = (int32_t)i;
    free(start);
}

/* The paper's greedy ordering score (Sec. 3.8):
 * Score(u) = (sum_{v in Out(u)} 1/d_in(v)) / d_out(u); 0 for d_out(u) = 0. */
void ao_order_score(int64_t n, const int64_t *off, const int32_t *col, const int64_t *indeg,
                    double *score) {
    for (int64_t u = 0; u < n; ++u) {
        double s = 0.0;
        for (int64_t e = off[u]; e < off[u + 1]; ++e) s += 1.0 / (double)indeg[col[e]];
        int64_t dout = off[u + 1] - off[u];
        score[u] = dout > 0 ? s / (double)dout : 0.0;
    }
}
