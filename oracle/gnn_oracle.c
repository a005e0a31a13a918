/*
 * CPU oracle for graph message passing -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C loops over the COO edge list in its given
 * order, with double accumulators rounded to float once at the end.  It is the
 * definition the GPU library is checked against and shares no code with it.
 * Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
 * call it; the product never does.
 *
 * What is computed follows the paper's description of message passing
 * (section 3, "Message Passing"): a per-edge message built from the source
 * node's features x_j and the edge's own data e_(j->i) (apply_edges), followed
 * by a reduction of the messages over each destination node's neighbourhood
 * (aggregate_neighbors); propagate is the two combined and must give the same
 * result.  The paper only names the layers (GCNConv, GAT, GIN, GlobalPool:
 * section 3, "Graph Convolutional Layers" and "Training Example") and prints no
 * formulas, so the layer arithmetic below is the textbook definition of each;
 * every choice the paper leaves open is listed next to the function.
 *
 * Conventions: nodes 0..N-1, edges 0..E-1; edge k carries a message from
 * j = src[k] to i = dst[k] and is reduced at i.  Features are row-major
 * [N x F] float.  Multi-edges and self-loops count with multiplicity.
 * A node without incoming edges gets 0 for sum, mean and max alike.
 * Inputs are finite by contract (behaviour on NaN/Inf: parity unpinned).
 *
 * Every function returns 0 on success, 1 for an index out of range,
 * 2 for a bad size/enum, 3 if memory could not be obtained.
 *
 * Optional output `sabs` (may be NULL) receives, per output element, the sum of
 * the absolute values of the terms that were added up to produce it -- the
 * condition number the tests scale their floating-point tolerance with.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { MSG_COPY_XJ = 0, MSG_E_MUL_XJ = 1, MSG_XJ_SUB_XI = 2, MSG_XI_DOT_XJ = 3 };
enum { AGGR_SUM = 0, AGGR_MEAN = 1, AGGR_MAX = 2, AGGR_MIN = 3, AGGR_PROD = 4 };

static int check_edges(const int32_t *src, const int32_t *dst, int64_t E, int32_t N)
{
    for (int64_t k = 0; k < E; ++k) {
        if (src && (src[k] < 0 || src[k] >= N)) return 1;
        if (dst && (dst[k] < 0 || dst[k] >= N)) return 1;
    }
    return 0;
}

/* IEEE-754 "maximum" on finite floats: the larger value; +0 beats -0. */
static float max_f32(float a, float b)
{
    if (a > b) return a;
    if (b > a) return b;
    uint32_t ua, ub;
    memcpy(&ua, &a, 4);
    memcpy(&ub, &b, 4);
    ua &= ub;                       /* equal values: only the zero pair differs in encoding */
    memcpy(&a, &ua, 4);
    return a;
}

/* IEEE-754 "minimum" on finite floats: the smaller value; -0 is below +0. */
static float min_f32(float a, float b)
{
    if (a < b) return a;
    if (b < a) return b;
    uint32_t ua, ub;
    memcpy(&ua, &a, 4);
    memcpy(&ub, &b, 4);
    ua |= ub;
    memcpy(&a, &ua, 4);
    return a;
}

/* The product of an edge datum and a feature, rounded to float as one operation. */
static float mul_f32(float a, float b)
{
    volatile float p = a * b;
    return p;
}

/*
 * COO -> CSR by destination (the sparse form of the same topology; section 3,
 * "Graph Data Structures").  Counting sort: rows list their edges in increasing
 * original edge index, so perm/colidx are unique even with duplicate edges.
 *   rowptr[N+1], colidx[E] = src[perm[p]], perm[E], indeg[N].
 */
int oracle_build_csr(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                     int32_t *rowptr, int32_t *colidx, int32_t *perm, int32_t *indeg)
{
    if (N <= 0 || E < 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    for (int32_t i = 0; i < N; ++i) indeg[i] = 0;
    for (int64_t k = 0; k < E; ++k) indeg[dst[k]]++;
    rowptr[0] = 0;
    for (int32_t i = 0; i < N; ++i) rowptr[i + 1] = rowptr[i] + indeg[i];
    int32_t *cursor = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    if (!cursor) return 3;
    for (int32_t i = 0; i < N; ++i) cursor[i] = rowptr[i];
    for (int64_t k = 0; k < E; ++k) {
        int32_t p = cursor[dst[k]]++;
        colidx[p] = src[k];
        perm[p] = (int32_t)k;
    }
    free(cursor);
    return 0;
}

/*
 * The message of edge k = (j -> i) at feature f, from the target's features x_i, the source's
 * features x_j and the edge's own data (section 3, "Message Passing": the message function takes
 * xi, xj and e):
 *   copy_xj  : x[j,f]
 *   e_mul_xj : float(e[k, f or 0] * x[j,f])       (e_dim = F or 1)
 *   xj_sub_xi: float(x[j,f] - x[i,f])
 */
static float message_value(int32_t msg, const float *x, int32_t F, int64_t i, int64_t j, const float *e,
                           int32_t e_dim, int64_t k, int32_t f)
{
    float v = x[j * F + f];
    if (msg == MSG_E_MUL_XJ) v = mul_f32(e[k * e_dim + (e_dim == 1 ? 0 : f)], v);
    if (msg == MSG_XJ_SUB_XI) { volatile float d = v - x[i * F + f]; v = d; }
    return v;
}

/* One step of a neighbourhood reduction: message v joins element q of a row that held cnt messages. */
static void reduce_step(int32_t aggr, double *acc, double *sa, int64_t q, int64_t cnt, float v)
{
    if (aggr == AGGR_MAX) {
        acc[q] = (cnt == 0) ? (double)v : (double)max_f32((float)acc[q], v);
        sa[q] = fabs(acc[q]);
    } else if (aggr == AGGR_MIN) {
        acc[q] = (cnt == 0) ? (double)v : (double)min_f32((float)acc[q], v);
        sa[q] = fabs(acc[q]);
    } else if (aggr == AGGR_PROD) {
        acc[q] = (cnt == 0) ? (double)v : acc[q] * (double)v;
        sa[q] = fabs(acc[q]) * (double)(cnt + 1);   /* one rounding per factor in any float evaluation */
    } else {
        acc[q] += (double)v;
        sa[q] += fabs((double)v);
    }
}

/*
 * apply_edges: one message row per edge, [E x F]; for xi_dot_xj one scalar per edge, [E x 1]:
 *   xi_dot_xj: m[k] = float(sum_f x[i,f] x[j,f]).
 * dst may be NULL for the messages that do not use the target.  sabs (may be NULL) is filled for
 * xi_dot_xj only (sum of |x_i x_j|).
 */
int oracle_apply_edges(const int32_t *src, const int32_t *dst, int64_t E, int32_t N, const float *x, int32_t F,
                       const float *e, int32_t e_dim, int32_t msg, float *m, double *sabs)
{
    if (N <= 0 || E < 0 || F <= 0) return 2;
    if (msg < MSG_COPY_XJ || msg > MSG_XI_DOT_XJ) return 2;
    if (msg == MSG_E_MUL_XJ && e_dim != 1 && e_dim != F) return 2;
    if ((msg == MSG_XJ_SUB_XI || msg == MSG_XI_DOT_XJ) && !dst && E > 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    for (int64_t k = 0; k < E; ++k) {
        int64_t j = src[k], i = dst ? dst[k] : 0;
        if (msg == MSG_XI_DOT_XJ) {
            double d = 0.0, a = 0.0;
            for (int32_t f = 0; f < F; ++f) {
                double t = (double)x[i * F + f] * (double)x[j * F + f];
                d += t;
                a += fabs(t);
            }
            m[k] = (float)d;
            if (sabs) sabs[k] = a;
        } else {
            for (int32_t f = 0; f < F; ++f) m[k * F + f] = message_value(msg, x, F, i, j, e, e_dim, k, f);
        }
    }
    return 0;
}

/* Shared finishing step of a neighbourhood reduction held in double. */
static void finish_rows(int32_t N, int32_t F, int32_t aggr, const double *acc, const int64_t *cnt,
                        double *sabs_acc, float *out, double *sabs)
{
    for (int32_t i = 0; i < N; ++i)
        for (int32_t f = 0; f < F; ++f) {
            int64_t q = (int64_t)i * F + f;
            double v = 0.0, s = sabs_acc ? sabs_acc[q] : 0.0;
            if (cnt[i] > 0) {
                v = acc[q];
                if (aggr == AGGR_MEAN) { v /= (double)cnt[i]; s /= (double)cnt[i]; }
            }
            out[q] = (float)v;
            if (sabs) sabs[q] = (cnt[i] > 0) ? s : 0.0;
        }
}

/*
 * aggregate_neighbors: reduce the message rows m[E x F] onto their destinations with
 * sum, mean, max, min or prod.  mean divides by the number of incoming edges (not by any sum of
 * weights); a node without incoming edges gets 0 under every reduction.
 */
int oracle_aggregate_neighbors(const int32_t *dst, int64_t E, int32_t N, const float *m, int32_t F,
                               int32_t aggr, float *out, double *sabs)
{
    if (N <= 0 || E < 0 || F <= 0) return 2;
    if (aggr < AGGR_SUM || aggr > AGGR_PROD) return 2;
    if (check_edges(NULL, dst, E, N)) return 1;
    size_t nf = (size_t)N * F;
    double *acc = (double *)calloc(nf, sizeof(double));
    double *sa = (double *)calloc(nf, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)N, sizeof(int64_t));
    if (!acc || !sa || !cnt) { free(acc); free(sa); free(cnt); return 3; }
    for (int64_t k = 0; k < E; ++k) {
        int64_t i = dst[k];
        for (int32_t f = 0; f < F; ++f) reduce_step(aggr, acc, sa, i * F + f, cnt[i], m[k * F + f]);
        cnt[i]++;
    }
    finish_rows(N, F, aggr, acc, cnt, sa, out, sabs);
    free(acc); free(sa); free(cnt);
    return 0;
}

/*
 * The reduction of propagate on a graph whose sources and destinations may be different node sets
 * (a relation of a heterogeneous graph, section 3 "Graph Data Structures": x has N_src rows, the result
 * N_dst rows), left in double: out64 / sabs64 [N_dst x F].
 */
static int propagate_core(const int32_t *src, const int32_t *dst, int64_t E, int32_t N_src, int32_t N_dst,
                          const float *x, int32_t F, const float *e, int32_t e_dim, int32_t msg, int32_t aggr,
                          double *out64, double *sabs64)
{
    if (N_src <= 0 || N_dst <= 0 || E < 0 || F <= 0) return 2;
    if (msg < MSG_COPY_XJ || msg > MSG_XJ_SUB_XI) return 2;
    if (msg == MSG_XJ_SUB_XI && N_src != N_dst) return 2;       /* x_i is a row of the same array */
    if (aggr < AGGR_SUM || aggr > AGGR_PROD) return 2;
    if (msg == MSG_E_MUL_XJ && e_dim != 1 && e_dim != F) return 2;
    for (int64_t k = 0; k < E; ++k)
        if (src[k] < 0 || src[k] >= N_src || dst[k] < 0 || dst[k] >= N_dst) return 1;
    size_t nf = (size_t)N_dst * F;
    double *acc = (double *)calloc(nf, sizeof(double));
    double *sa = (double *)calloc(nf, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)N_dst, sizeof(int64_t));
    if (!acc || !sa || !cnt) { free(acc); free(sa); free(cnt); return 3; }
    for (int64_t k = 0; k < E; ++k) {
        int64_t i = dst[k], j = src[k];
        for (int32_t f = 0; f < F; ++f)
            reduce_step(aggr, acc, sa, i * F + f, cnt[i], message_value(msg, x, F, i, j, e, e_dim, k, f));
        cnt[i]++;
    }
    for (int32_t i = 0; i < N_dst; ++i)
        for (int32_t f = 0; f < F; ++f) {
            int64_t q = (int64_t)i * F + f;
            double v = 0.0, sv = 0.0;
            if (cnt[i] > 0) {
                v = acc[q];
                sv = sa[q];
                if (aggr == AGGR_MEAN) { v /= (double)cnt[i]; sv /= (double)cnt[i]; }
            }
            out64[q] = v;
            if (sabs64) sabs64[q] = sv;
        }
    free(acc); free(sa); free(cnt);
    return 0;
}

/*
 * propagate = apply_edges then aggregate_neighbors, without storing the
 * [E x F] messages (same values, same order of edges).  xi_dot_xj (a message of another width)
 * is not a propagate message.
 */
int oracle_propagate(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                     const float *x, int32_t F, const float *e, int32_t e_dim,
                     int32_t msg, int32_t aggr, float *out, double *sabs)
{
    if (N <= 0 || F <= 0) return 2;
    size_t nf = (size_t)N * F;
    double *o64 = (double *)malloc(nf * sizeof(double));
    if (!o64) return 3;
    int rc = propagate_core(src, dst, E, N, N, x, F, e, e_dim, msg, aggr, o64, sabs);
    if (rc == 0)
        for (size_t q = 0; q < nf; ++q) out[q] = (float)o64[q];
    free(o64);
    return rc;
}

/*
 * propagate once more, for the timing of a CPU baseline on all host cores: the rows of the by-destination
 * sparse form (oracle_build_csr) are dealt to OpenMP threads, each row reducing its own messages in
 * increasing edge index -- per element the very additions oracle_propagate makes in the very same order, so
 * the result is the same bit for bit (a test checks this).  *threads_used receives the team size.
 */
int oracle_propagate_all_cores(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                               const float *x, int32_t F, const float *e, int32_t e_dim,
                               int32_t msg, int32_t aggr, float *out, int32_t *threads_used)
{
    if (N <= 0 || E < 0 || F <= 0) return 2;
    if (msg < MSG_COPY_XJ || msg > MSG_XJ_SUB_XI) return 2;
    if (aggr < AGGR_SUM || aggr > AGGR_PROD) return 2;
    if (msg == MSG_E_MUL_XJ && e_dim != 1 && e_dim != F) return 2;
    int32_t *rowptr = (int32_t *)malloc(((size_t)N + 1) * sizeof(int32_t));
    int32_t *colidx = (int32_t *)malloc((size_t)(E > 0 ? E : 1) * sizeof(int32_t));
    int32_t *perm = (int32_t *)malloc((size_t)(E > 0 ? E : 1) * sizeof(int32_t));
    int32_t *indeg = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    int rc = 3, failed = 0, team = 1;
    if (!rowptr || !colidx || !perm || !indeg) goto done;
    rc = oracle_build_csr(src, dst, E, N, rowptr, colidx, perm, indeg);
    if (rc) goto done;
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)F * sizeof(double));
        double *sa = (double *)malloc((size_t)F * sizeof(double));
        if (!acc || !sa) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp single
        team = omp_get_num_threads();
#pragma omp for schedule(dynamic, 64)
        for (int32_t i = 0; i < N; ++i) {
            if (!acc || !sa) continue;
            for (int32_t f = 0; f < F; ++f) { acc[f] = 0.0; sa[f] = 0.0; }
            int64_t cnt = 0;
            for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p, ++cnt)
                for (int32_t f = 0; f < F; ++f)
                    reduce_step(aggr, acc, sa, f, cnt, message_value(msg, x, F, i, colidx[p], e, e_dim, perm[p], f));
            for (int32_t f = 0; f < F; ++f) {
                double v = cnt > 0 ? acc[f] : 0.0;
                if (aggr == AGGR_MEAN && cnt > 0) v /= (double)cnt;
                out[(int64_t)i * F + f] = (float)v;
            }
        }
        free(acc); free(sa);
    }
    if (failed) rc = 3;
    if (threads_used) *threads_used = team;
done:
    free(rowptr); free(colidx); free(perm); free(indeg);
    return rc;
}

/*
 * One relation of a heterogeneous graph: edges from a source node type (N_src nodes, features x) to a
 * destination node type (N_dst nodes).  The result is ADDED, in double, to out64 / sabs64 [N_dst x F]:
 * the caller sums the relations that end in one node type and rounds once.
 */
int oracle_propagate_relation_add(const int32_t *src, const int32_t *dst, int64_t E, int32_t N_src, int32_t N_dst,
                                  const float *x, int32_t F, const float *e, int32_t e_dim, int32_t msg,
                                  int32_t aggr, double *out64, double *sabs64)
{
    if (N_dst <= 0 || F <= 0) return 2;
    size_t nf = (size_t)N_dst * F;
    double *o = (double *)malloc(nf * sizeof(double)), *sa = (double *)malloc(nf * sizeof(double));
    if (!o || !sa) { free(o); free(sa); return 3; }
    int rc = propagate_core(src, dst, E, N_src, N_dst, x, F, e, e_dim, msg, aggr, o, sa);
    if (rc == 0)
        for (size_t q = 0; q < nf; ++q) { out64[q] += o[q]; sabs64[q] += sa[q]; }
    free(o); free(sa);
    return rc;
}

/*
 * Backward of propagate (reverse-mode derivative of the forward definition above; the paper's
 * training example differentiates through its layers, section 3 "Training Example").
 * Given g = dL/d out [N x F]:
 *   sum : dL/dx[j,f] = sum_{k: src[k]=j} w[k,f] g[dst[k],f],   w = 1 (copy_xj) or e (e_mul_xj)
 *         dL/de[k]   = sum_f x[src[k],f] g[dst[k],f]  (e_dim = 1)  or  x[src[k],f] g[dst[k],f]  (e_dim = F)
 *   mean: the same with g[i,:] divided by the number of incoming edges of i
 *   max : only the winning edge of each output element carries gradient; the winner of (i,f) is
 *         the FIRST edge in increasing edge index whose message equals out[i,f] (with +0 above -0).
 * grad_x [N x F] and grad_e [E x e_dim] may each be NULL.  argmax_out [N x F] (may be NULL, max
 * only) receives the winning edge index or -1.  sabs_x / sabs_e (may be NULL) receive the sums of
 * absolute values of the terms behind each element.
 */
int oracle_propagate_backward(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                              const float *x, int32_t F, const float *e, int32_t e_dim,
                              int32_t msg, int32_t aggr, const float *grad_out,
                              float *grad_x, float *grad_e, int32_t *argmax_out,
                              double *sabs_x, double *sabs_e)
{
    if (N <= 0 || E < 0 || F <= 0) return 2;
    if (msg != MSG_COPY_XJ && msg != MSG_E_MUL_XJ) return 2;
    if (aggr < AGGR_SUM || aggr > AGGR_MAX) return 2;
    if (msg == MSG_E_MUL_XJ && e_dim != 1 && e_dim != F) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    const int has_e = (msg == MSG_E_MUL_XJ);
    size_t nf = (size_t)N * F;
    size_t ne = has_e ? (size_t)E * e_dim : 0;
    double *gx = (double *)calloc(nf, sizeof(double));
    double *sx = (double *)calloc(nf, sizeof(double));
    double *ge = (double *)calloc(ne ? ne : 1, sizeof(double));
    double *se = (double *)calloc(ne ? ne : 1, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)N, sizeof(int64_t));
    float *best = NULL;
    int64_t *win = NULL;
    int rc = 3;
    if (!gx || !sx || !ge || !se || !cnt) goto done;
    for (int64_t k = 0; k < E; ++k) cnt[dst[k]]++;
    if (aggr == AGGR_MAX) {
        best = (float *)malloc(nf * sizeof(float));
        win = (int64_t *)malloc(nf * sizeof(int64_t));
        if (!best || !win) goto done;
        for (size_t q = 0; q < nf; ++q) win[q] = -1;
        for (int64_t k = 0; k < E; ++k)
            for (int32_t f = 0; f < F; ++f) {
                float v = x[(int64_t)src[k] * F + f];
                if (has_e) v = mul_f32(e[k * e_dim + (e_dim == 1 ? 0 : f)], v);
                int64_t q = (int64_t)dst[k] * F + f;
                /* strictly better than the current winner (+0 is better than -0): replaces it;
                   equal: the earlier edge stays */
                if (win[q] < 0 || v > best[q] || (v == best[q] && signbit(best[q]) && !signbit(v))) {
                    best[q] = v;
                    win[q] = k;
                }
            }
    }
    for (int64_t k = 0; k < E; ++k) {
        int64_t i = dst[k], j = src[k];
        for (int32_t f = 0; f < F; ++f) {
            int64_t qi = i * F + f, qj = j * F + f;
            double g = (double)grad_out[qi];
            if (aggr == AGGR_MEAN) g /= (double)cnt[i];
            if (aggr == AGGR_MAX && win[qi] != k) continue;
            double wv = has_e ? (double)e[k * e_dim + (e_dim == 1 ? 0 : f)] : 1.0;
            gx[qj] += wv * g;
            sx[qj] += fabs(wv * g);
            if (has_e) {
                int64_t qe = k * e_dim + (e_dim == 1 ? 0 : f);
                ge[qe] += (double)x[qj] * g;
                se[qe] += fabs((double)x[qj] * g);
            }
        }
    }
    for (size_t q = 0; q < nf; ++q) {
        if (grad_x) grad_x[q] = (float)gx[q];
        if (sabs_x) sabs_x[q] = sx[q];
        if (argmax_out) argmax_out[q] = (aggr == AGGR_MAX) ? (int32_t)win[q] : -1;
    }
    for (size_t q = 0; q < ne; ++q) {
        if (grad_e) grad_e[q] = (float)ge[q];
        if (sabs_e) sabs_e[q] = se[q];
    }
    rc = 0;
done:
    free(gx); free(sx); free(ge); free(se); free(cnt); free(best); free(win);
    return rc;
}

/* Z = X W and Zabs = |X| |W| in double, [N x f_out]. */
static int dense_xw(const float *x, int32_t N, int32_t f_in, const float *w, int32_t f_out,
                    double **z_out, double **zabs_out)
{
    double *z = (double *)calloc((size_t)N * f_out, sizeof(double));
    double *za = (double *)calloc((size_t)N * f_out, sizeof(double));
    if (!z || !za) { free(z); free(za); return 3; }
    for (int32_t i = 0; i < N; ++i)
        for (int32_t k = 0; k < f_in; ++k) {
            double xv = (double)x[(int64_t)i * f_in + k];
            for (int32_t o = 0; o < f_out; ++o) {
                double t = xv * (double)w[(int64_t)k * f_out + o];
                z[(int64_t)i * f_out + o] += t;
                za[(int64_t)i * f_out + o] += fabs(t);
            }
        }
    *z_out = z;
    *zabs_out = za;
    return 0;
}

/*
 * GCNConv forward: out = D^-1/2 (A [+ I]) D^-1/2 X W + b.
 * Choices the paper leaves open: d_i is the in-degree of i in the edge list
 * (after one self-loop per node has been appended when add_self_loops != 0, with
 * no de-duplication) and is used for both endpoints, so an edge j->i carries the
 * coefficient 1/sqrt(d_i d_j); a node with d = 0 (possible only without
 * self-loops) contributes the coefficient 0; bias is added last; no activation.
 * sabs = sum over edges of coefficient * (|X||W|)[j] + |b|.
 */
int oracle_gcnconv(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                   const float *x, int32_t f_in, const float *w, const float *bias, int32_t f_out,
                   int32_t add_self_loops, float *out, double *sabs)
{
    if (N <= 0 || E < 0 || f_in <= 0 || f_out <= 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    int64_t E2 = E + (add_self_loops ? N : 0);
    int32_t *s2 = (int32_t *)malloc((size_t)(E2 > 0 ? E2 : 1) * sizeof(int32_t));
    int32_t *d2 = (int32_t *)malloc((size_t)(E2 > 0 ? E2 : 1) * sizeof(int32_t));
    double *deg = (double *)calloc((size_t)N, sizeof(double));
    double *acc = (double *)calloc((size_t)N * f_out, sizeof(double));
    double *sa = (double *)calloc((size_t)N * f_out, sizeof(double));
    double *z = NULL, *za = NULL;
    int rc = 3;
    if (!s2 || !d2 || !deg || !acc || !sa) goto done;
    for (int64_t k = 0; k < E; ++k) { s2[k] = src[k]; d2[k] = dst[k]; }
    if (add_self_loops)
        for (int32_t i = 0; i < N; ++i) { s2[E + i] = i; d2[E + i] = i; }
    for (int64_t k = 0; k < E2; ++k) deg[d2[k]] += 1.0;
    if (dense_xw(x, N, f_in, w, f_out, &z, &za)) goto done;
    for (int64_t k = 0; k < E2; ++k) {
        int64_t i = d2[k], j = s2[k];
        double dd = deg[i] * deg[j];
        double c = dd > 0.0 ? 1.0 / sqrt(dd) : 0.0;
        for (int32_t o = 0; o < f_out; ++o) {
            acc[i * f_out + o] += c * z[j * f_out + o];
            sa[i * f_out + o] += c * za[j * f_out + o];
        }
    }
    for (int32_t i = 0; i < N; ++i)
        for (int32_t o = 0; o < f_out; ++o) {
            double b = bias ? (double)bias[o] : 0.0;
            out[(int64_t)i * f_out + o] = (float)(acc[(int64_t)i * f_out + o] + b);
            if (sabs) sabs[(int64_t)i * f_out + o] = sa[(int64_t)i * f_out + o] + fabs(b);
        }
    rc = 0;
done:
    free(s2); free(d2); free(deg); free(acc); free(sa); free(z); free(za);
    return rc;
}

/*
 * Backward of the GCNConv forward above.  With Ahat = D^-1/2 (A [+ I]) D^-1/2, Z = X W and
 * G = dL/d out [N x f_out]:
 *   T = Ahat^T G,   dL/dX = T W^T,   dL/dW = X^T T,   dL/db[o] = sum_i G[i,o].
 * Any output may be NULL.  sabs_* (may be NULL) are the sums of absolute values of the terms.
 */
int oracle_gcnconv_backward(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                            const float *x, int32_t f_in, const float *w, int32_t f_out,
                            int32_t add_self_loops, const float *grad_out,
                            float *grad_x, float *grad_w, float *grad_b,
                            double *sabs_x, double *sabs_w, double *sabs_b)
{
    if (N <= 0 || E < 0 || f_in <= 0 || f_out <= 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    double *deg = (double *)calloc((size_t)N, sizeof(double));
    double *t = (double *)calloc((size_t)N * f_out, sizeof(double));
    double *ta = (double *)calloc((size_t)N * f_out, sizeof(double));
    if (!deg || !t || !ta) { free(deg); free(t); free(ta); return 3; }
    for (int64_t k = 0; k < E; ++k) deg[dst[k]] += 1.0;
    if (add_self_loops)
        for (int32_t i = 0; i < N; ++i) deg[i] += 1.0;
    /* T[j,:] += c(i,j) G[i,:] for every edge j -> i (and every self-loop) */
    for (int64_t k = 0; k < E + (add_self_loops ? N : 0); ++k) {
        int64_t i = k < E ? dst[k] : k - E, j = k < E ? src[k] : k - E;
        double dd = deg[i] * deg[j];
        double c = dd > 0.0 ? 1.0 / sqrt(dd) : 0.0;
        for (int32_t o = 0; o < f_out; ++o) {
            double g = (double)grad_out[i * f_out + o];
            t[j * f_out + o] += c * g;
            ta[j * f_out + o] += c * fabs(g);
        }
    }
    if (grad_x || sabs_x)
        for (int32_t i = 0; i < N; ++i)
            for (int32_t q = 0; q < f_in; ++q) {
                double a = 0.0, sa = 0.0;
                for (int32_t o = 0; o < f_out; ++o) {
                    a += t[(int64_t)i * f_out + o] * (double)w[(int64_t)q * f_out + o];
                    sa += ta[(int64_t)i * f_out + o] * fabs((double)w[(int64_t)q * f_out + o]);
                }
                if (grad_x) grad_x[(int64_t)i * f_in + q] = (float)a;
                if (sabs_x) sabs_x[(int64_t)i * f_in + q] = sa;
            }
    if (grad_w || sabs_w)
        for (int32_t q = 0; q < f_in; ++q)
            for (int32_t o = 0; o < f_out; ++o) {
                double a = 0.0, sa = 0.0;
                for (int32_t i = 0; i < N; ++i) {
                    a += (double)x[(int64_t)i * f_in + q] * t[(int64_t)i * f_out + o];
                    sa += fabs((double)x[(int64_t)i * f_in + q]) * ta[(int64_t)i * f_out + o];
                }
                if (grad_w) grad_w[(int64_t)q * f_out + o] = (float)a;
                if (sabs_w) sabs_w[(int64_t)q * f_out + o] = sa;
            }
    if (grad_b || sabs_b)
        for (int32_t o = 0; o < f_out; ++o) {
            double a = 0.0, sa = 0.0;
            for (int32_t i = 0; i < N; ++i) {
                a += (double)grad_out[(int64_t)i * f_out + o];
                sa += fabs((double)grad_out[(int64_t)i * f_out + o]);
            }
            if (grad_b) grad_b[o] = (float)a;
            if (sabs_b) sabs_b[o] = sa;
        }
    free(deg); free(t); free(ta);
    return 0;
}

/*
 * Segment softmax over each destination's incoming edges, per head:
 *   alpha[k,h] = exp(s[k,h] - mx[i,h]) / sum_{q: dst[q]=i} exp(s[q,h] - mx[i,h]),  i = dst[k],
 * with mx the segment maximum (so the denominator is >= 1 and needs no epsilon).
 * Input and output are [E x H] in the caller's edge order.
 */
int oracle_segment_softmax(const int32_t *dst, int64_t E, int32_t N, const float *s, int32_t H,
                           float *alpha)
{
    if (N <= 0 || E < 0 || H <= 0) return 2;
    if (check_edges(NULL, dst, E, N)) return 1;
    size_t nh = (size_t)N * H;
    double *mx = (double *)malloc(nh * sizeof(double));
    double *den = (double *)calloc(nh, sizeof(double));
    if (!mx || !den) { free(mx); free(den); return 3; }
    for (size_t q = 0; q < nh; ++q) mx[q] = -INFINITY;
    for (int64_t k = 0; k < E; ++k)
        for (int32_t h = 0; h < H; ++h) {
            double v = (double)s[k * H + h];
            if (v > mx[(int64_t)dst[k] * H + h]) mx[(int64_t)dst[k] * H + h] = v;
        }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t h = 0; h < H; ++h)
            den[(int64_t)dst[k] * H + h] += exp((double)s[k * H + h] - mx[(int64_t)dst[k] * H + h]);
    for (int64_t k = 0; k < E; ++k)
        for (int32_t h = 0; h < H; ++h) {
            int64_t q = (int64_t)dst[k] * H + h;
            alpha[k * H + h] = (float)(exp((double)s[k * H + h] - mx[q]) / den[q]);
        }
    free(mx); free(den);
    return 0;
}

/*
 * GAT-style attention layer (multi-head, heads concatenated, no bias, no
 * activation, self-loops only if the edge list holds them):
 *   h = float(X W)                      [N x heads*ch], rounded once (a stored tensor)
 *   sl[j,hd] = sum_c a_src[hd,c] h[j,hd,c],  sr[i,hd] = sum_c a_dst[hd,c] h[i,hd,c]
 *   s[k,hd]  = lrelu(sl[src[k],hd] + sr[dst[k],hd]),  lrelu(v) = v > 0 ? v : slope * v
 *   alpha    = segment softmax of s over each destination
 *   out[i,hd,:] = sum_{k: dst[k]=i} alpha[k,hd] * h[src[k],hd,:]
 * sabs = sum_k alpha[k,hd] * (|X||W|)[src[k]].
 */
int oracle_gatconv(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                   const float *x, int32_t f_in, const float *w,
                   const float *a_src, const float *a_dst, int32_t heads, int32_t ch,
                   float negative_slope, float *out, double *sabs)
{
    if (N <= 0 || E < 0 || f_in <= 0 || heads <= 0 || ch <= 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    int32_t fo = heads * ch;
    size_t nh = (size_t)N * heads;
    double *z = NULL, *za = NULL;
    double *sl = (double *)calloc(nh, sizeof(double));
    double *sr = (double *)calloc(nh, sizeof(double));
    double *mx = (double *)malloc(nh * sizeof(double));
    double *den = (double *)calloc(nh, sizeof(double));
    double *acc = (double *)calloc((size_t)N * fo, sizeof(double));
    double *sa = (double *)calloc((size_t)N * fo, sizeof(double));
    int rc = 3;
    if (!sl || !sr || !mx || !den || !acc || !sa) goto done;
    if (dense_xw(x, N, f_in, w, fo, &z, &za)) goto done;
    for (size_t q = 0; q < (size_t)N * fo; ++q) z[q] = (double)(float)z[q];
    for (int32_t i = 0; i < N; ++i)
        for (int32_t hd = 0; hd < heads; ++hd)
            for (int32_t c = 0; c < ch; ++c) {
                double hv = z[(int64_t)i * fo + hd * ch + c];
                sl[(int64_t)i * heads + hd] += (double)a_src[hd * ch + c] * hv;
                sr[(int64_t)i * heads + hd] += (double)a_dst[hd * ch + c] * hv;
            }
    double slope = (double)negative_slope;
#define SCORE(k, hd, v) do { (v) = sl[(int64_t)src[k] * heads + (hd)] + sr[(int64_t)dst[k] * heads + (hd)]; \
                             if (!((v) > 0.0)) (v) *= slope; } while (0)
    for (size_t q = 0; q < nh; ++q) mx[q] = -INFINITY;
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            double v; SCORE(k, hd, v);
            if (v > mx[(int64_t)dst[k] * heads + hd]) mx[(int64_t)dst[k] * heads + hd] = v;
        }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            double v; SCORE(k, hd, v);
            den[(int64_t)dst[k] * heads + hd] += exp(v - mx[(int64_t)dst[k] * heads + hd]);
        }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            double v; SCORE(k, hd, v);
            int64_t q = (int64_t)dst[k] * heads + hd;
            double alpha = exp(v - mx[q]) / den[q];
            for (int32_t c = 0; c < ch; ++c) {
                acc[(int64_t)dst[k] * fo + hd * ch + c] += alpha * z[(int64_t)src[k] * fo + hd * ch + c];
                sa[(int64_t)dst[k] * fo + hd * ch + c] += alpha * za[(int64_t)src[k] * fo + hd * ch + c];
            }
        }
#undef SCORE
    for (size_t q = 0; q < (size_t)N * fo; ++q) {
        out[q] = (float)acc[q];
        if (sabs) sabs[q] = sa[q];
    }
    rc = 0;
done:
    free(z); free(za); free(sl); free(sr); free(mx); free(den); free(acc); free(sa);
    return rc;
}

/*
 * Backward of the segment softmax (the Jacobian of a softmax, per destination segment):
 *   gs[k,h] = alpha[k,h] * (galpha[k,h] - sum_{k': dst[k']=dst[k]} alpha[k',h] galpha[k',h]).
 * alpha is the forward result, galpha = dL/d alpha.  sabs = alpha (|galpha| + sum alpha |galpha|).
 */
int oracle_segment_softmax_backward(const int32_t *dst, int64_t E, int32_t N, const float *alpha,
                                    const float *galpha, int32_t H, float *gs, double *sabs)
{
    if (N <= 0 || E < 0 || H <= 0) return 2;
    for (int64_t k = 0; k < E; ++k)
        if (dst[k] < 0 || dst[k] >= N) return 1;
    size_t nh = (size_t)N * H;
    double *t = (double *)calloc(nh, sizeof(double));
    double *ta = (double *)calloc(nh, sizeof(double));
    if (!t || !ta) { free(t); free(ta); return 3; }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t h = 0; h < H; ++h) {
            double p = (double)alpha[k * H + h] * (double)galpha[k * H + h];
            t[(int64_t)dst[k] * H + h] += p;
            ta[(int64_t)dst[k] * H + h] += fabs(p);
        }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t h = 0; h < H; ++h) {
            int64_t q = (int64_t)dst[k] * H + h;
            double a = (double)alpha[k * H + h], g = (double)galpha[k * H + h];
            gs[k * H + h] = (float)(a * (g - t[q]));
            if (sabs) sabs[k * H + h] = fabs(a) * (fabs(g) + ta[q]);
        }
    free(t); free(ta);
    return 0;
}

/*
 * Backward of the attention layer above, by the chain rule through its steps in reverse
 * (G = dL/d out; the rounding of h to float is treated as the identity):
 *   dalpha[k,hd] = sum_c G[dst[k],hd,c] h[src[k],hd,c]
 *   ds[k,hd]     = alpha (dalpha - sum_{k' into dst[k]} alpha' dalpha')          (softmax Jacobian)
 *   dv[k,hd]     = ds * (v > 0 ? 1 : slope),  v = sl[src[k],hd] + sr[dst[k],hd]  (lrelu', slope at v = 0
 *                                                                                  as in the forward's branch)
 *   dsl[j,hd] = sum_{k: src[k]=j} dv,   dsr[i,hd] = sum_{k: dst[k]=i} dv
 *   dh[j,hd,c] = sum_{k: src[k]=j} alpha[k,hd] G[dst[k],hd,c] + dsl[j,hd] a_src[hd,c] + dsr[j,hd] a_dst[hd,c]
 *   d a_src[hd,c] = sum_j dsl[j,hd] h[j,hd,c],   d a_dst[hd,c] = sum_i dsr[i,hd] h[i,hd,c]
 *   dW = X^T dh,   dX = dh W^T.
 * The sabs outputs carry the same recurrences on absolute values (|h| replaced by |X||W|).
 */
int oracle_gatconv_backward(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                            const float *x, int32_t f_in, const float *w,
                            const float *a_src, const float *a_dst, int32_t heads, int32_t ch,
                            float negative_slope, const float *gout,
                            float *gx, float *gw, float *ga_src, float *ga_dst,
                            double *sabs_x, double *sabs_w, double *sabs_as, double *sabs_ad)
{
    if (N <= 0 || E < 0 || f_in <= 0 || heads <= 0 || ch <= 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    int32_t fo = heads * ch;
    size_t nh = (size_t)N * heads, nfo = (size_t)N * fo, eh = (size_t)(E > 0 ? E : 1) * heads;
    double *z = NULL, *za = NULL;
    double *sl = (double *)calloc(nh, sizeof(double)), *sr = (double *)calloc(nh, sizeof(double));
    double *mx = (double *)malloc(nh * sizeof(double)), *den = (double *)calloc(nh, sizeof(double));
    double *t = (double *)calloc(nh, sizeof(double)), *tb = (double *)calloc(nh, sizeof(double));
    double *dsl = (double *)calloc(nh, sizeof(double)), *dslb = (double *)calloc(nh, sizeof(double));
    double *dsr = (double *)calloc(nh, sizeof(double)), *dsrb = (double *)calloc(nh, sizeof(double));
    double *al = (double *)calloc(eh, sizeof(double)), *pre = (double *)calloc(eh, sizeof(double));
    double *da = (double *)calloc(eh, sizeof(double)), *dab = (double *)calloc(eh, sizeof(double));
    double *dh = (double *)calloc(nfo, sizeof(double)), *dhb = (double *)calloc(nfo, sizeof(double));
    double *acc_as = (double *)calloc((size_t)fo, sizeof(double)), *acc_ad = (double *)calloc((size_t)fo, sizeof(double));
    double *abs_as = (double *)calloc((size_t)fo, sizeof(double)), *abs_ad = (double *)calloc((size_t)fo, sizeof(double));
    double *acc_w = (double *)calloc((size_t)f_in * fo, sizeof(double));
    double *abs_w = (double *)calloc((size_t)f_in * fo, sizeof(double));
    int rc = 3;
    if (!sl || !sr || !mx || !den || !t || !tb || !dsl || !dslb || !dsr || !dsrb || !al || !pre || !da || !dab ||
        !dh || !dhb || !acc_as || !acc_ad || !abs_as || !abs_ad || !acc_w || !abs_w)
        goto done;
    if (dense_xw(x, N, f_in, w, fo, &z, &za)) goto done;
    for (size_t q = 0; q < nfo; ++q) z[q] = (double)(float)z[q];
    for (int32_t i = 0; i < N; ++i)
        for (int32_t hd = 0; hd < heads; ++hd)
            for (int32_t c = 0; c < ch; ++c) {
                double hv = z[(int64_t)i * fo + hd * ch + c];
                sl[(int64_t)i * heads + hd] += (double)a_src[hd * ch + c] * hv;
                sr[(int64_t)i * heads + hd] += (double)a_dst[hd * ch + c] * hv;
            }
    double slope = (double)negative_slope;
    /* forward: pre-activations, scores, attention weights */
    for (size_t q = 0; q < nh; ++q) mx[q] = -INFINITY;
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            double v = sl[(int64_t)src[k] * heads + hd] + sr[(int64_t)dst[k] * heads + hd];
            pre[k * heads + hd] = v;
            double sc = v > 0.0 ? v : v * slope;
            if (sc > mx[(int64_t)dst[k] * heads + hd]) mx[(int64_t)dst[k] * heads + hd] = sc;
        }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            double v = pre[k * heads + hd], sc = v > 0.0 ? v : v * slope;
            al[k * heads + hd] = exp(sc - mx[(int64_t)dst[k] * heads + hd]);
            den[(int64_t)dst[k] * heads + hd] += al[k * heads + hd];
        }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) al[k * heads + hd] /= den[(int64_t)dst[k] * heads + hd];
    /* d alpha and the per-destination sums of alpha * d alpha */
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            double d = 0.0, db = 0.0;
            for (int32_t c = 0; c < ch; ++c) {
                double g = (double)gout[(int64_t)dst[k] * fo + hd * ch + c];
                d += g * z[(int64_t)src[k] * fo + hd * ch + c];
                db += fabs(g) * za[(int64_t)src[k] * fo + hd * ch + c];
            }
            da[k * heads + hd] = d;
            dab[k * heads + hd] = db;
            t[(int64_t)dst[k] * heads + hd] += al[k * heads + hd] * d;
            tb[(int64_t)dst[k] * heads + hd] += al[k * heads + hd] * db;
        }
    /* through the softmax and the leaky ReLU; reductions onto both endpoints; the alpha * G part of dh */
    for (int64_t k = 0; k < E; ++k)
        for (int32_t hd = 0; hd < heads; ++hd) {
            int64_t qi = (int64_t)dst[k] * heads + hd, qj = (int64_t)src[k] * heads + hd;
            double a = al[k * heads + hd];
            double slopek = pre[k * heads + hd] > 0.0 ? 1.0 : slope;
            double dv = a * (da[k * heads + hd] - t[qi]) * slopek;
            double dvb = a * (dab[k * heads + hd] + tb[qi]) * fabs(slopek);
            dsl[qj] += dv; dslb[qj] += dvb;
            dsr[qi] += dv; dsrb[qi] += dvb;
            for (int32_t c = 0; c < ch; ++c) {
                double g = (double)gout[(int64_t)dst[k] * fo + hd * ch + c];
                dh[(int64_t)src[k] * fo + hd * ch + c] += a * g;
                dhb[(int64_t)src[k] * fo + hd * ch + c] += a * fabs(g);
            }
        }
    /* d a_src, d a_dst: sums over the nodes, accumulated node by node */
    for (int32_t i = 0; i < N; ++i)
        for (int32_t hd = 0; hd < heads; ++hd)
            for (int32_t c = 0; c < ch; ++c) {
                int64_t q = (int64_t)i * fo + hd * ch + c;
                acc_as[hd * ch + c] += dsl[(int64_t)i * heads + hd] * z[q];
                acc_ad[hd * ch + c] += dsr[(int64_t)i * heads + hd] * z[q];
                abs_as[hd * ch + c] += dslb[(int64_t)i * heads + hd] * za[q];
                abs_ad[hd * ch + c] += dsrb[(int64_t)i * heads + hd] * za[q];
            }
    for (int32_t q = 0; q < fo; ++q) {
        ga_src[q] = (float)acc_as[q];
        ga_dst[q] = (float)acc_ad[q];
        if (sabs_as) sabs_as[q] = abs_as[q];
        if (sabs_ad) sabs_ad[q] = abs_ad[q];
    }
    for (int32_t i = 0; i < N; ++i)
        for (int32_t hd = 0; hd < heads; ++hd)
            for (int32_t c = 0; c < ch; ++c) {
                int64_t q = (int64_t)i * fo + hd * ch + c;
                dh[q] += dsl[(int64_t)i * heads + hd] * (double)a_src[hd * ch + c] +
                         dsr[(int64_t)i * heads + hd] * (double)a_dst[hd * ch + c];
                dhb[q] += dslb[(int64_t)i * heads + hd] * fabs((double)a_src[hd * ch + c]) +
                          dsrb[(int64_t)i * heads + hd] * fabs((double)a_dst[hd * ch + c]);
            }
    /* dW = X^T dh (accumulated node by node), dX = dh W^T */
    for (int32_t i = 0; i < N; ++i)
        for (int32_t k = 0; k < f_in; ++k) {
            double xv = (double)x[(int64_t)i * f_in + k];
            for (int32_t o = 0; o < fo; ++o) {
                acc_w[(int64_t)k * fo + o] += xv * dh[(int64_t)i * fo + o];
                abs_w[(int64_t)k * fo + o] += fabs(xv) * dhb[(int64_t)i * fo + o];
            }
        }
    for (int64_t q = 0; q < (int64_t)f_in * fo; ++q) {
        gw[q] = (float)acc_w[q];
        if (sabs_w) sabs_w[q] = abs_w[q];
    }
    for (int32_t i = 0; i < N; ++i)
        for (int32_t k = 0; k < f_in; ++k) {
            double s1 = 0.0, b1 = 0.0;
            for (int32_t o = 0; o < fo; ++o) {
                s1 += dh[(int64_t)i * fo + o] * (double)w[(int64_t)k * fo + o];
                b1 += dhb[(int64_t)i * fo + o] * fabs((double)w[(int64_t)k * fo + o]);
            }
            gx[(int64_t)i * f_in + k] = (float)s1;
            if (sabs_x) sabs_x[(int64_t)i * f_in + k] = b1;
        }
    rc = 0;
done:
    free(z); free(za); free(sl); free(sr); free(mx); free(den); free(t); free(tb); free(dsl); free(dslb);
    free(dsr); free(dsrb); free(al); free(pre); free(da); free(dab); free(dh); free(dhb);
    free(acc_as); free(acc_ad); free(abs_as); free(abs_ad); free(acc_w); free(abs_w);
    return rc;
}

/*
 * Dense layer of the paper's example model (section 3, "Training Example": Dense(64, 1)):
 *   out = act(X W + b),  X [N x k], W [k x n] row-major, b [n] or NULL, act = identity or relu.
 * sabs = sum_k |x||w| + |b|.
 */
int oracle_dense(const float *x, int32_t N, int32_t k, const float *w, int32_t n, const float *bias,
                 int32_t relu, float *out, double *sabs)
{
    if (N < 0 || k <= 0 || n <= 0) return 2;
    for (int32_t i = 0; i < N; ++i)
        for (int32_t o = 0; o < n; ++o) {
            double a = bias ? (double)bias[o] : 0.0, b = fabs(a);
            for (int32_t q = 0; q < k; ++q) {
                double t = (double)x[(int64_t)i * k + q] * (double)w[(int64_t)q * n + o];
                a += t;
                b += fabs(t);
            }
            if (relu && a < 0.0) a = 0.0;
            out[(int64_t)i * n + o] = (float)a;
            if (sabs) sabs[(int64_t)i * n + o] = b;
        }
    return 0;
}

/*
 * Batch normalisation across the node dimension (the example model's BatchNorm(64), "normalize
 * across node dimension"), followed by an optional relu:
 *   mean[f] = (1/N) sum_i x[i,f],   var[f] = (1/N) sum_i (x[i,f] - mean[f])^2      (biased variance)
 *   out[i,f] = act(gamma[f] * (x[i,f] - mean[f]) / sqrt(var[f] + eps) + beta[f]).
 * With use_given != 0 the statistics are read from mean_io / var_io (inference with stored
 * statistics) instead of being computed from the batch and written there.
 * gamma / beta may be NULL (1 and 0).  Returns 2 for N <= 0.
 */
int oracle_batchnorm(const float *x, int32_t N, int32_t F, const float *gamma, const float *beta, float eps,
                     int32_t relu, int32_t use_given, float *mean_io, float *var_io, float *out)
{
    if (N <= 0 || F <= 0) return 2;
    for (int32_t f = 0; f < F; ++f) {
        double mu, var;
        if (use_given) {
            mu = (double)mean_io[f];
            var = (double)var_io[f];
        } else {
            double s = 0.0;
            for (int32_t i = 0; i < N; ++i) s += (double)x[(int64_t)i * F + f];
            mu = s / (double)N;
            double q = 0.0;
            for (int32_t i = 0; i < N; ++i) {
                double d = (double)x[(int64_t)i * F + f] - mu;
                q += d * d;
            }
            var = q / (double)N;
            if (mean_io) mean_io[f] = (float)mu;
            if (var_io) var_io[f] = (float)var;
        }
        double g = gamma ? (double)gamma[f] : 1.0, b = beta ? (double)beta[f] : 0.0;
        double inv = 1.0 / sqrt(var + (double)eps);
        for (int32_t i = 0; i < N; ++i) {
            double y = g * ((double)x[(int64_t)i * F + f] - mu) * inv + b;
            if (relu && y < 0.0) y = 0.0;
            out[(int64_t)i * F + f] = (float)y;
        }
    }
    return 0;
}

/*
 * bfloat16 storage of features (16-bit codes = sign, 8 exponent bits, 7 fraction bits: the upper half of
 * the IEEE binary32 encoding).  Finite inputs are rounded to the nearest representable value, ties to
 * the code with an even last bit; this is written out by cases rather than as an integer trick:
 *   lower = the float with the low 16 bits cleared (truncation towards zero), upper = the next code
 *   away from zero; the one nearer to x wins, a tie goes to the even code.
 * codes (may be NULL) receives the 16-bit codes, widened (may be NULL) the rounded values as floats.
 */
int oracle_round_bf16(const float *x, int64_t n, uint16_t *codes, float *widened)
{
    if (n < 0) return 2;
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &x[i], 4);
        uint32_t lo_bits = u & 0xffff0000u, hi_bits = lo_bits + 0x10000u;   /* same sign, next magnitude */
        float lo, hi;
        memcpy(&lo, &lo_bits, 4);
        memcpy(&hi, &hi_bits, 4);
        double hv = isinf(hi) ? copysign(ldexp(1.0, 128), (double)hi) : (double)hi;   /* the value the code after the
                                                                                          largest finite one would have */
        double dl = fabs((double)x[i] - (double)lo), dh = fabs(hv - (double)x[i]);
        uint32_t pick = lo_bits;
        if (dh < dl) pick = hi_bits;
        else if (dh == dl && ((lo_bits >> 16) & 1u)) pick = hi_bits;
        if (codes) codes[i] = (uint16_t)(pick >> 16);
        if (widened) memcpy(&widened[i], &pick, 4);
    }
    return 0;
}

/*
 * Rounding of finite floats to IEEE 754 binary16 ("half": 1 sign, 5 exponent, 10 fraction bits; the 16-bit
 * feature storage named next to bfloat16 among the next steps), round to nearest, ties to even, written
 * from the definition: inside the binade 2^e <= |x| < 2^(e+1) (e clamped to -14, the subnormal range) the
 * representable values are n * 2^(e-10) for whole n; |x| / 2^(e-10) is exact in double, its two whole neighbours
 * are compared by distance, a tie goes to the even n.  |x| >= 65520 (half way from the largest finite value
 * 65504 to 2^16) gives infinity.  codes / widened may be NULL.
 */
int oracle_round_f16(const float *x, int64_t n_values, uint16_t *codes, float *widened)
{
    if (n_values < 0) return 2;
    for (int64_t i = 0; i < n_values; ++i) {
        const double v = (double)x[i], a = fabs(v);
        const uint16_t sign = signbit(x[i]) ? 0x8000u : 0u;
        uint16_t code;
        double back;
        if (a >= 65520.0) {
            code = 0x7C00u;
            back = INFINITY;
        } else {
            int e = -14;
            if (a >= ldexp(1.0, -14)) {
                (void)frexp(a, &e);   /* a = f * 2^e with 0.5 <= f < 1 */
                e -= 1;
            }
            const double q = ldexp(1.0, e - 10), k = a / q;
            double lo = floor(k);
            const double frac = k - lo;
            if (frac > 0.5 || (frac == 0.5 && fmod(lo, 2.0) == 1.0)) lo += 1.0;
            int64_t nn = (int64_t)lo;   /* 0 .. 2048 */
            if (nn == 2048) {
                nn = 1024;
                e += 1;
            }
            back = (double)nn * ldexp(1.0, e - 10);
            if (nn < 1024) code = (uint16_t)nn;                                   /* subnormal or zero (e = -14) */
            else code = (uint16_t)(((e + 15) << 10) | (int)(nn - 1024));
        }
        if (codes) codes[i] = (uint16_t)(sign | code);
        if (widened) widened[i] = (float)(sign ? -back : back);
    }
    return 0;
}

/*
 * Backward passes of the example model's dense-side layers (the training example differentiates the
 * whole chain, section 3 "Training Example").  All in double, rounded once per output.
 *
 * oracle_dense_backward: out = X W + b (no activation; a relu is differentiated by masking gy first)
 *   gx = gy W^T [N x k],  gw = X^T gy [k x n],  gb = column sums of gy [n].   Each output may be NULL.
 */
int oracle_dense_backward(const float *x, int32_t N, int32_t k, const float *w, int32_t n, const float *gy,
                          float *gx, float *gw, float *gb)
{
    if (N < 0 || k <= 0 || n <= 0) return 2;
    if (gx)
        for (int32_t i = 0; i < N; ++i)
            for (int32_t q = 0; q < k; ++q) {
                double a = 0.0;
                for (int32_t o = 0; o < n; ++o) a += (double)gy[(int64_t)i * n + o] * (double)w[(int64_t)q * n + o];
                gx[(int64_t)i * k + q] = (float)a;
            }
    if (gw) {
        double *acc = (double *)calloc((size_t)k * n, sizeof(double));
        if (!acc) return 3;
        for (int32_t i = 0; i < N; ++i)
            for (int32_t q = 0; q < k; ++q)
                for (int32_t o = 0; o < n; ++o)
                    acc[(int64_t)q * n + o] += (double)x[(int64_t)i * k + q] * (double)gy[(int64_t)i * n + o];
        for (int64_t q = 0; q < (int64_t)k * n; ++q) gw[q] = (float)acc[q];
        free(acc);
    }
    if (gb)
        for (int32_t o = 0; o < n; ++o) {
            double a = 0.0;
            for (int32_t i = 0; i < N; ++i) a += (double)gy[(int64_t)i * n + o];
            gb[o] = (float)a;
        }
    return 0;
}

/*
 * oracle_batchnorm_backward: y = gamma * xhat + beta with xhat = (x - mean) / sqrt(var + eps) and batch
 * statistics (mean and biased variance depend on x).  With gy = dL/dy (already masked if a relu followed):
 *   gbeta[f] = sum_i gy[i,f],   ggamma[f] = sum_i gy[i,f] xhat[i,f],
 *   gx[i,f]  = gamma[f] / sqrt(var[f] + eps) * (gy[i,f] - gbeta[f] / N - xhat[i,f] * ggamma[f] / N).
 * mean / var are recomputed from x.  gamma may be NULL (1).
 */
int oracle_batchnorm_backward(const float *x, int32_t N, int32_t F, const float *gamma, float eps, const float *gy,
                              float *gx, float *ggamma, float *gbeta)
{
    if (N <= 0 || F <= 0) return 2;
    for (int32_t f = 0; f < F; ++f) {
        double s = 0.0;
        for (int32_t i = 0; i < N; ++i) s += (double)x[(int64_t)i * F + f];
        double mu = s / (double)N, q = 0.0;
        for (int32_t i = 0; i < N; ++i) {
            double d = (double)x[(int64_t)i * F + f] - mu;
            q += d * d;
        }
        double inv = 1.0 / sqrt(q / (double)N + (double)eps);
        double gb = 0.0, gg = 0.0;
        for (int32_t i = 0; i < N; ++i) {
            double g = (double)gy[(int64_t)i * F + f];
            gb += g;
            gg += g * ((double)x[(int64_t)i * F + f] - mu) * inv;
        }
        double gm = gamma ? (double)gamma[f] : 1.0;
        if (gx)
            for (int32_t i = 0; i < N; ++i) {
                double xh = ((double)x[(int64_t)i * F + f] - mu) * inv;
                gx[(int64_t)i * F + f] =
                    (float)(gm * inv * ((double)gy[(int64_t)i * F + f] - gb / (double)N - xh * gg / (double)N));
            }
        if (ggamma) ggamma[f] = (float)gg;
        if (gbeta) gbeta[f] = (float)gb;
    }
    return 0;
}

/*
 * oracle_pool_backward: graph-level readout by sum or mean; gx[i,:] = gout[g(i),:] (divided by the node
 * count of graph g(i) for the mean).
 */
int oracle_pool_backward(const int32_t *gi, int32_t N, int32_t G, const float *gout, int32_t F, int32_t aggr,
                         float *gx)
{
    if (N < 0 || G <= 0 || F <= 0) return 2;
    if (aggr != AGGR_SUM && aggr != AGGR_MEAN) return 2;
    int64_t *cnt = (int64_t *)calloc((size_t)G, sizeof(int64_t));
    if (!cnt) return 3;
    for (int32_t i = 0; i < N; ++i) {
        if (gi[i] < 0 || gi[i] >= G) { free(cnt); return 1; }
        cnt[gi[i]]++;
    }
    for (int32_t i = 0; i < N; ++i)
        for (int32_t f = 0; f < F; ++f) {
            double v = (double)gout[(int64_t)gi[i] * F + f];
            if (aggr == AGGR_MEAN) v /= (double)cnt[gi[i]];
            gx[(int64_t)i * F + f] = (float)v;
        }
    free(cnt);
    return 0;
}

/*
 * One Adam step on a parameter array (the example's optimiser, Adam(1e-4)):
 *   m = b1 m + (1 - b1) g,  v = b2 v + (1 - b2) g^2,
 *   p = p - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),      t = step count starting at 1.
 * p, m, v are updated in place (each rounded to float once).
 */
int oracle_adam_step(float *p, float *m, float *v, const float *g, int64_t n, float lr, float b1, float b2,
                     float eps, int32_t t)
{
    if (n < 0 || t <= 0) return 2;
    double c1 = 1.0 - pow((double)b1, (double)t), c2 = 1.0 - pow((double)b2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double mi = (double)b1 * (double)m[i] + (1.0 - (double)b1) * (double)g[i];
        double vi = (double)b2 * (double)v[i] + (1.0 - (double)b2) * (double)g[i] * (double)g[i];
        m[i] = (float)mi;
        v[i] = (float)vi;
        p[i] = (float)((double)p[i] - (double)lr * (mi / c1) / (sqrt(vi / c2) + (double)eps));
    }
    return 0;
}

/*
 * GIN-style node update without the MLP:  out[i,:] = (1 + eps) x[i,:] + sum_{j->i} x[j,:].
 */
int oracle_gin_update(const int32_t *src, const int32_t *dst, int64_t E, int32_t N,
                      const float *x, int32_t F, float eps, float *out, double *sabs)
{
    if (N <= 0 || E < 0 || F <= 0) return 2;
    if (check_edges(src, dst, E, N)) return 1;
    size_t nf = (size_t)N * F;
    double *acc = (double *)calloc(nf, sizeof(double));
    double *sa = (double *)calloc(nf, sizeof(double));
    if (!acc || !sa) { free(acc); free(sa); return 3; }
    double scale = 1.0 + (double)eps;
    for (size_t q = 0; q < nf; ++q) { acc[q] = scale * (double)x[q]; sa[q] = fabs(acc[q]); }
    for (int64_t k = 0; k < E; ++k)
        for (int32_t f = 0; f < F; ++f) {
            double v = (double)x[(int64_t)src[k] * F + f];
            acc[(int64_t)dst[k] * F + f] += v;
            sa[(int64_t)dst[k] * F + f] += fabs(v);
        }
    for (size_t q = 0; q < nf; ++q) { out[q] = (float)acc[q]; if (sabs) sabs[q] = sa[q]; }
    free(acc); free(sa);
    return 0;
}

/*
 * Graph-level readout of a batch of graphs:  pooled[g,:] = AGG_{i: gi[i]=g} x[i,:]
 * (sum, mean over the graph's node count, or max); a graph without nodes gives 0.
 * gi must lie in [0, G); it is what batching produces, one graph id per node.
 */
int oracle_graph_pool(const int32_t *gi, int32_t N, int32_t G, const float *x, int32_t F,
                      int32_t aggr, float *out, double *sabs)
{
    if (N < 0 || G <= 0 || F <= 0) return 2;
    if (aggr < AGGR_SUM || aggr > AGGR_MAX) return 2;
    for (int32_t i = 0; i < N; ++i)
        if (gi[i] < 0 || gi[i] >= G) return 1;
    size_t gf = (size_t)G * F;
    double *acc = (double *)calloc(gf, sizeof(double));
    double *sa = (double *)calloc(gf, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)G, sizeof(int64_t));
    if (!acc || !sa || !cnt) { free(acc); free(sa); free(cnt); return 3; }
    for (int32_t i = 0; i < N; ++i) {
        int64_t g = gi[i];
        for (int32_t f = 0; f < F; ++f) {
            float v = x[(int64_t)i * F + f];
            int64_t q = g * F + f;
            if (aggr == AGGR_MAX) {
                acc[q] = (cnt[g] == 0) ? (double)v : (double)max_f32((float)acc[q], v);
                sa[q] = fabs(acc[q]);
            } else {
                acc[q] += (double)v;
                sa[q] += fabs((double)v);
            }
        }
        cnt[g]++;
    }
    finish_rows(G, F, aggr, acc, cnt, sa, out, sabs);
    free(acc); free(sa); free(cnt);
    return 0;
}
