/*
 * CPU oracle: full-graph GCN / GraphSAGE-mean forward, softmax cross-entropy and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or import this
 * file; it exists so that tests, the smoke check and the bench's CPU-baseline leg have an
 * independent statement of what the partition-wise GPU path must compute.
 *
 * The paper's method processes the graph partition by partition but states that it leaves
 * the training algorithm untouched (Introduction, last paragraph; Evaluation, accuracy
 * check in the appendix), so the result it must reach is the ordinary full-graph one.  This
 * file is therefore that plain definition, with no partitions anywhere in it:
 *
 *   forward  (Background, "Forward Pass"): aggregate source features along the edges, then
 *            multiply by the shared weight matrix, then normalise/activate;
 *   backward (Background, "Backward Pass"): the dependency flow is inverted and gradients
 *            are scatter-accumulated onto the source vertices.
 *
 * All arithmetic is fp64.  The only parallelism is an OpenMP "parallel for" over
 * independent output elements (rows, or column blocks for the scatter); every sum is taken
 * in one fixed order, so the result does not depend on the thread count.
 *
 * Graph input: CSR by destination.  Row v lists the sources u of edges u -> v, ascending,
 * no duplicates.
 *
 * GCN layer l:   A~ = A + I (one self-loop per vertex, not doubled when already present),
 *                deg(v) = row length of A~,
 *                Z[v]  = sum_{u in row v of A~}  A^{l-1}[u] / sqrt(deg(u) deg(v)),
 *                Y     = Z W^l + b^l,     A^l = relu(Y) for l < L,  A^L = Y.
 * SAGE-mean l:   no self-loops added, Z[v] = mean_{u in row v} A^{l-1}[u]  (0 if empty),
 *                Y     = Z W_n^l + A^{l-1} W_s^l + b^l,   same activation rule.
 * Loss:          mean over the train mask of -log softmax(A^L[v])[y_v].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_GCN = 0, ORACLE_SAGE = 1 };

typedef struct {
    int64_t n;
    int64_t *rowptr; /* n+1 */
    int32_t *col;    /* nnz */
    double *w;       /* per-entry weight of the aggregation operator */
} agg_op;

static void agg_free(agg_op *op)
{
    free(op->rowptr);
    free(op->col);
    free(op->w);
    memset(op, 0, sizeof *op);
}

/* Build the aggregation operator S (so that Z = S A) with explicit per-entry weights. */
static int agg_build(int model, int64_t n, const int64_t *rowptr, const int32_t *colidx,
                     agg_op *op)
{
    memset(op, 0, sizeof *op);
    op->n = n;
    op->rowptr = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    if (!op->rowptr) return -1;
    if (model == ORACLE_GCN) {
        /* rows of A~ : insert v into row v unless it is there already */
        int64_t nnz = 0;
        for (int64_t v = 0; v < n; ++v) {
            int has_self = 0;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
                if (colidx[e] == v) has_self = 1;
            nnz += (rowptr[v + 1] - rowptr[v]) + (has_self ? 0 : 1);
            op->rowptr[v + 1] = nnz;
        }
        op->col = (int32_t *)malloc((size_t)(nnz ? nnz : 1) * sizeof(int32_t));
        op->w = (double *)malloc((size_t)(nnz ? nnz : 1) * sizeof(double));
        if (!op->col || !op->w) return -1;
        for (int64_t v = 0; v < n; ++v) {
            int64_t o = op->rowptr[v];
            int placed = 0;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int32_t u = colidx[e];
                if (u == v) placed = 1;
                if (!placed && u > v) {
                    op->col[o++] = (int32_t)v;
                    placed = 1;
                }
                op->col[o++] = u;
            }
            if (!placed) op->col[o++] = (int32_t)v;
        }
        /* deg(v) = row length of A~, used for both end points of an edge */
        for (int64_t v = 0; v < n; ++v) {
            double dv = (double)(op->rowptr[v + 1] - op->rowptr[v]);
            for (int64_t e = op->rowptr[v]; e < op->rowptr[v + 1]; ++e) {
                int64_t u = op->col[e];
                double du = (double)(op->rowptr[u + 1] - op->rowptr[u]);
                op->w[e] = 1.0 / sqrt(du * dv);
            }
        }
    } else {
        int64_t nnz = rowptr[n];
        op->col = (int32_t *)malloc((size_t)(nnz ? nnz : 1) * sizeof(int32_t));
        op->w = (double *)malloc((size_t)(nnz ? nnz : 1) * sizeof(double));
        if (!op->col || !op->w) return -1;
        memcpy(op->rowptr, rowptr, ((size_t)n + 1) * sizeof(int64_t));
        memcpy(op->col, colidx, (size_t)nnz * sizeof(int32_t));
        for (int64_t v = 0; v < n; ++v) {
            int64_t deg = rowptr[v + 1] - rowptr[v];
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) op->w[e] = 1.0 / (double)deg;
        }
    }
    return 0;
}

/* Z = S X   (X, Z are [n, d] row-major) */
static void agg_apply(const agg_op *op, int64_t d, const double *X, double *Z)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < op->n; ++v) {
        double *z = Z + v * d;
        for (int64_t c = 0; c < d; ++c) z[c] = 0.0;
        for (int64_t e = op->rowptr[v]; e < op->rowptr[v + 1]; ++e) {
            const double *x = X + (int64_t)op->col[e] * d;
            double w = op->w[e];
            for (int64_t c = 0; c < d; ++c) z[c] += w * x[c];
        }
    }
}

/* G += S^T Q : every entry (v <- u, w) sends w * Q[v] to G[u].  Threads own column blocks,
   so no two threads touch the same element and the order of additions is fixed. */
static void agg_apply_transpose_add(const agg_op *op, int64_t d, const double *Q, double *G)
{
    const int64_t blk = 8;
    const int64_t nblk = (d + blk - 1) / blk;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nblk; ++b) {
        int64_t c0 = b * blk, c1 = c0 + blk < d ? c0 + blk : d;
        for (int64_t v = 0; v < op->n; ++v) {
            const double *q = Q + v * d;
            for (int64_t e = op->rowptr[v]; e < op->rowptr[v + 1]; ++e) {
                double *g = G + (int64_t)op->col[e] * d;
                double w = op->w[e];
                for (int64_t c = c0; c < c1; ++c) g[c] += w * q[c];
            }
        }
    }
}

/* C[n, q] (+)= A[n, p] B[p, q] */
static void matmul_nn(int64_t n, int64_t p, int64_t q, const double *A, const double *B,
                      double *C, int accumulate)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *c = C + i * q;
        if (!accumulate)
            for (int64_t j = 0; j < q; ++j) c[j] = 0.0;
        for (int64_t t = 0; t < p; ++t) {
            double a = A[i * p + t];
            const double *b = B + t * q;
            for (int64_t j = 0; j < q; ++j) c[j] += a * b[j];
        }
    }
}

/* C[n, p] (+)= A[n, q] B[p, q]^T */
static void matmul_nt(int64_t n, int64_t q, int64_t p, const double *A, const double *B,
                      double *C, int accumulate)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t t = 0; t < p; ++t) {
            double s = 0.0;
            for (int64_t j = 0; j < q; ++j) s += A[i * q + j] * B[t * q + j];
            if (accumulate)
                C[i * p + t] += s;
            else
                C[i * p + t] = s;
        }
    }
}

/* C[p, q] = A[n, p]^T B[n, q] */
static void matmul_tn(int64_t n, int64_t p, int64_t q, const double *A, const double *B,
                      double *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < p; ++t) {
        double *c = C + t * q;
        for (int64_t j = 0; j < q; ++j) c[j] = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double a = A[i * p + t];
            const double *b = B + i * q;
            for (int64_t j = 0; j < q; ++j) c[j] += a * b[j];
        }
    }
}

/* Z = S X for one layer width; exported so tests can pin the aggregation alone. */
int oracle_aggregate(int model, int64_t n, const int64_t *rowptr, const int32_t *colidx,
                     int64_t d, const double *X, double *Z)
{
    agg_op op;
    if (agg_build(model, n, rowptr, colidx, &op)) {
        agg_free(&op);
        return -1;
    }
    agg_apply(&op, d, X, Z);
    agg_free(&op);
    return 0;
}

/* G = S^T Q */
int oracle_aggregate_transpose(int model, int64_t n, const int64_t *rowptr,
                               const int32_t *colidx, int64_t d, const double *Q, double *G)
{
    agg_op op;
    if (agg_build(model, n, rowptr, colidx, &op)) {
        agg_free(&op);
        return -1;
    }
    memset(G, 0, (size_t)(n * d) * sizeof(double));
    agg_apply_transpose_add(&op, d, Q, G);
    agg_free(&op);
    return 0;
}

/* Mean softmax cross-entropy over the mask; optionally its gradient w.r.t. the logits. */
double oracle_loss(int64_t n, int64_t C, const double *logits, const int32_t *labels,
                   const uint8_t *mask, double *grad /* [n, C] or NULL */)
{
    int64_t cnt = 0;
    for (int64_t v = 0; v < n; ++v) cnt += mask[v] ? 1 : 0;
    double total = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        const double *x = logits + v * C;
        double *g = grad ? grad + v * C : NULL;
        if (!mask[v]) {
            if (g)
                for (int64_t c = 0; c < C; ++c) g[c] = 0.0;
            continue;
        }
        double mx = x[0];
        for (int64_t c = 1; c < C; ++c)
            if (x[c] > mx) mx = x[c];
        double se = 0.0;
        for (int64_t c = 0; c < C; ++c) se += exp(x[c] - mx);
        double lse = mx + log(se);
        total += lse - x[labels[v]];
        if (g)
            for (int64_t c = 0; c < C; ++c)
                g[c] = (exp(x[c] - lse) - (c == labels[v] ? 1.0 : 0.0)) / (double)cnt;
    }
    return cnt ? total / (double)cnt : 0.0;
}

/*
 * Forward through L layers.
 *
 * dims[0..L]           layer widths d_0 .. d_L
 * X        [n, d_0]    input features A^0
 * W[l]     [d_l, d_{l+1}]   (GCN weight, or SAGE neighbour weight W_n)      l = 0..L-1
 * Ws[l]    [d_l, d_{l+1}]   SAGE self weight (ignored for GCN; may be NULL)
 * b[l]     [d_{l+1}]        bias (may be NULL = no bias)
 * drop[l]  [n, d_{l+1}]     optional (NULL array or NULL entries): dropout multipliers of hidden
 *                           layer l+1, each 0 or 1/(1-p), applied after the activation (training
 *                           with the dropout rates of the datasets table); the random draws are
 *                           an input, made by the caller
 * act[l]   [n, d_{l+1}]     out: A^{l+1}
 * zagg[l]  [n, d_l]         out: aggregated input Z of layer l+1
 * Returns 0, or -1 when memory runs out.
 */
int oracle_forward(int model, int64_t n, const int64_t *rowptr, const int32_t *colidx, int L,
                   const int32_t *dims, const double *X, const double *const *W,
                   const double *const *Ws, const double *const *b, const double *const *drop,
                   double *const *act, double *const *zagg)
{
    agg_op op;
    if (agg_build(model, n, rowptr, colidx, &op)) {
        agg_free(&op);
        return -1;
    }
    for (int l = 0; l < L; ++l) {
        int64_t din = dims[l], dout = dims[l + 1];
        const double *Ain = l == 0 ? X : act[l - 1];
        agg_apply(&op, din, Ain, zagg[l]);
        double *Y = act[l];
        matmul_nn(n, din, dout, zagg[l], W[l], Y, 0);
        if (model == ORACLE_SAGE) matmul_nn(n, din, dout, Ain, Ws[l], Y, 1);
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < n; ++v)
            for (int64_t c = 0; c < dout; ++c) {
                double y = Y[v * dout + c] + (b && b[l] ? b[l][c] : 0.0);
                if (l < L - 1 && !(y > 0.0)) y = 0.0;
                if (l < L - 1 && drop && drop[l]) y *= drop[l][v * dout + c];
                Y[v * dout + c] = y;
            }
    }
    agg_free(&op);
    return 0;
}

/*
 * Loss and backward, given the forward results.
 *
 * act, zagg            as returned by oracle_forward
 * relu_on[l] [n, d_{l+1}]   optional (NULL array or NULL entries): the activation decision of
 *                      hidden layer l+1 as 0/1 bytes.  By default the decision is act > 0.  A
 *                      test that compares against an fp32 implementation passes the other
 *                      side's decision for the few elements whose pre-activation lies within
 *                      rounding distance of zero, where either choice is a correct result.
 * drop                 the multipliers the forward pass used (or NULL)
 * gW, gWs, gb          out: gradients, same shapes as W, Ws, b (NULL entries skipped)
 * gact[l]  [n, d_{l+1}]     out: dLoss/dA^{l+1}  (NULL array or NULL entries skipped)
 * gX       [n, d_0]         out (optional): dLoss/dA^0.  The training pass does not need it
 *                           (the backward loop of the overall-procedure algorithm stops at
 *                           layer 2); tests ask for it so that finite differences on the
 *                           inputs can check the whole backward chain.
 * Returns 0, or -1 when memory runs out.
 */
int oracle_backward(int model, int64_t n, const int64_t *rowptr, const int32_t *colidx, int L,
                    const int32_t *dims, const double *X, const double *const *W,
                    const double *const *Ws, const double *const *act, const double *const *zagg,
                    const int32_t *labels, const uint8_t *mask, const uint8_t *const *relu_on,
                    const double *const *drop, double *loss, double *const *gW, double *const *gWs, double *const *gb,
                    double *const *gact, double *gX)
{
    agg_op op;
    int rc = -1;
    double *G = NULL, *dY = NULL, *dZ = NULL, *Gprev = NULL;
    int64_t dmax = 0;
    for (int l = 0; l <= L; ++l)
        if (dims[l] > dmax) dmax = dims[l];
    if (agg_build(model, n, rowptr, colidx, &op)) goto done;
    size_t gsz = (size_t)(n * dmax > 0 ? n * dmax : 1) * sizeof(double);
    G = (double *)malloc(gsz);
    dY = (double *)malloc(gsz);
    dZ = (double *)malloc(gsz);
    Gprev = (double *)malloc(gsz);
    if (!G || !dY || !dZ || !Gprev) goto done;
    *loss = oracle_loss(n, dims[L], act[L - 1], labels, mask, G);

    for (int l = L - 1; l >= 0; --l) {
        int64_t din = dims[l], dout = dims[l + 1];
        const double *Ain = l == 0 ? X : act[l - 1];
        const uint8_t *on = (relu_on && l < L - 1) ? relu_on[l] : NULL;
        if (gact && gact[l]) memcpy(gact[l], G, (size_t)(n * dout) * sizeof(double));
        /* through the activation: relu on hidden layers, identity on the last */
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n * dout; ++i) {
            int pass = 1;
            if (l < L - 1) pass = on ? (on[i] != 0) : (act[l][i] > 0.0);
            dY[i] = pass ? G[i] : 0.0;
            if (l < L - 1 && drop && drop[l]) dY[i] *= drop[l][i];
        }
        if (gb && gb[l])
            for (int64_t c = 0; c < dout; ++c) {
                double s = 0.0;
                for (int64_t v = 0; v < n; ++v) s += dY[v * dout + c];
                gb[l][c] = s;
            }
        if (gW && gW[l]) matmul_tn(n, din, dout, zagg[l], dY, gW[l]);
        if (model == ORACLE_SAGE && gWs && gWs[l]) matmul_tn(n, din, dout, Ain, dY, gWs[l]);
        if (l >= 1 || gX) {
            matmul_nt(n, dout, din, dY, W[l], dZ, 0);
            memset(Gprev, 0, (size_t)(n * din) * sizeof(double));
            agg_apply_transpose_add(&op, din, dZ, Gprev);
            if (model == ORACLE_SAGE) matmul_nt(n, dout, din, dY, Ws[l], Gprev, 1);
            double *t = G;
            G = Gprev;
            Gprev = t;
        }
    }
    if (gX) memcpy(gX, G, (size_t)(n * dims[0]) * sizeof(double));
    rc = 0;
done:
    free(G);
    free(dY);
    free(dZ);
    free(Gprev);
    agg_free(&op);
    return rc;
}

#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int t) { omp_set_num_threads(t); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int t) { (void)t; }
#endif
