/*
 * CPU oracle for one GCN / GAT layer and the sparse-dense primitives it is
 * composed of.  TEST INFRASTRUCTURE ONLY: it is called by the tests, by the
 * smoke check and by the benchmark's cpu_baseline leg, never by the product
 * path, and it shares no code with the HIP library.
 *
 * Everything is the plain definition, single threaded, evaluated in fp64 on
 * the fp32 input bits, with no blocking, fusion or reordering:
 *   - g-SpMM with (+,x)                     : Background, Eq. 1
 *   - g-SDDMM with k = 1                    : Background, Eq. 2
 *   - GCN layer                             : Case study GCN, Eq. 3 (== Eq. 4)
 *   - GAT layer                             : Case study GAT, Eq. 5-6
 *   - backward of both layers (training)    : chain rule on Eq. 3 and Eq. 5-6
 * Readings where the paper is silent (degree clamp, score function, softmax
 * over the stored entries of a row) are stated at each function.
 *
 * Pins (tests/test_oracle_*.py): dense brute force on small graphs, closed
 * forms (self-loop graph, regular ring, complete graph, star), softmax
 * invariants, agreement of every re-association, library routines on special
 * cases.  The row-sampled entry points (*_rows) are pinned against the full
 * ones.  The backward functions are pinned against central finite
 * differences of the forward functions, dense linear algebra and closed forms
 * (tests/test_oracle_backward.py).
 *
 * Build: gcc -O2 -shared -fPIC sensei_oracle.c -o liboracle.so -lm
 *        (-fopenmp -DORC_OMP builds the row-parallel timing variant of the
 *         same source; rows are independent, so results are identical.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORC_OMP
#include <omp.h>
#define ORC_PAR _Pragma("omp parallel for schedule(dynamic, 64)")
int orc_threads(void) { return omp_get_max_threads(); }
#else
#define ORC_PAR
int orc_threads(void) { return 1; }
#endif

/* ---------------------------------------------------------------- a0 */

/* Degrees of the stored pattern (which already holds the self edges):
 * deg_row[i] = entries in row i, deg_col[j] = entries in column j.
 * Case study GCN: D~ is the degree of the nodes in A~. */
void orc_degrees(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                 int32_t *deg_row, int32_t *deg_col) {
    for (int32_t j = 0; j < n_cols; ++j) deg_col[j] = 0;
    for (int32_t i = 0; i < n_rows; ++i) {
        deg_row[i] = row_ptr[i + 1] - row_ptr[i];
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) deg_col[col_idx[k]] += 1;
    }
}

/* D~^(-1/2) as a vector.  Reading: a zero degree (an unused column of a
 * sampled block) is clamped to 1 so the factor is finite. */
void orc_inv_sqrt_deg(const int32_t *deg, int64_t n, double *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = 1.0 / sqrt((double)(deg[i] < 1 ? 1 : deg[i]));
}

/* ------------------------------------------------------- primitives */

/* Eq. 1 with (+,x): C[i,:] = sum_j a_ij * B[j,:]; val == NULL means a_ij = 1
 * on the pattern (the value-less SpMM of the candidate->primitive rules). */
void orc_spmm(int32_t n_rows, const int32_t *row_ptr, const int32_t *col_idx, const double *val,
              const double *B, int64_t ldb, int32_t F, double *C, int64_t ldc) {
    ORC_PAR
    for (int32_t i = 0; i < n_rows; ++i) {
        double *c = C + (int64_t)i * ldc;
        for (int32_t f = 0; f < F; ++f) c[f] = 0.0;
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            const double a = val ? val[k] : 1.0;
            const double *b = B + (int64_t)col_idx[k] * ldb;
            for (int32_t f = 0; f < F; ++f) c[f] += a * b[f];
        }
    }
}

/* Eq. 2 with k = 1 and (+,x): d_ij = a_ij * (b_i * c_j) on the pattern; the
 * two diagonal matrices enter as dense vectors.  a == NULL means a_ij = 1. */
void orc_sddmm_mul(int32_t n_rows, const int32_t *row_ptr, const int32_t *col_idx, const double *a,
                   const double *b, const double *c, double *d) {
    for (int32_t i = 0; i < n_rows; ++i)
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k)
            d[k] = (a ? a[k] : 1.0) * (b[i] * c[col_idx[k]]);
}

/* Attention logits on the pattern: t = s_l[i] + s_r[j] (Eq. 2 with the inner
 * operator taken as +, k = 1), then LeakyReLU with the given negative slope.
 * Reading: i = CSR row = destination, j = column = in-neighbour. */
void orc_gat_scores(int32_t n_rows, const int32_t *row_ptr, const int32_t *col_idx, const double *s_l,
                    const double *s_r, double slope, double *e) {
    for (int32_t i = 0; i < n_rows; ++i)
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            double t = s_l[i] + s_r[col_idx[k]];
            e[k] = t > 0.0 ? t : slope * t;
        }
}

/* Softmax over the stored entries of each row (self edge included):
 * alpha_ij = exp(e_ij - m_i) / sum_j' exp(e_ij' - m_i), m_i = max_j e_ij.
 * An empty row has no entries to write. */
void orc_edge_softmax(int32_t n_rows, const int32_t *row_ptr, const double *e, double *alpha) {
    for (int32_t i = 0; i < n_rows; ++i) {
        int32_t lo = row_ptr[i], hi = row_ptr[i + 1];
        if (lo == hi) continue;
        double m = e[lo];
        for (int32_t k = lo + 1; k < hi; ++k) if (e[k] > m) m = e[k];
        double s = 0.0;
        for (int32_t k = lo; k < hi; ++k) s += exp(e[k] - m);
        for (int32_t k = lo; k < hi; ++k) alpha[k] = exp(e[k] - m) / s;
    }
}

/* Row broadcast: Y[i,:] = s[i] * X[i,:]. */
void orc_row_broadcast(int64_t n, int32_t F, const double *s, const double *X, int64_t ldx, double *Y, int64_t ldy) {
    for (int64_t i = 0; i < n; ++i)
        for (int32_t f = 0; f < F; ++f) Y[i * ldy + f] = s[i] * X[i * ldx + f];
}

/* Dense update Y = A.W, textbook triple loop. */
void orc_gemm(int64_t n, int32_t K, int32_t M, const double *A, int64_t lda, const double *W, int64_t ldw,
              double *Y, int64_t ldy) {
    ORC_PAR
    for (int64_t i = 0; i < n; ++i)
        for (int32_t m = 0; m < M; ++m) {
            double s = 0.0;
            for (int32_t k = 0; k < K; ++k) s += A[i * lda + k] * W[(int64_t)k * ldw + m];
            Y[i * ldy + m] = s;
        }
}

/* y = A.v for a dense matrix and a vector. */
void orc_gemv(int64_t n, int32_t K, const double *A, int64_t lda, const double *v, double *y) {
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int32_t k = 0; k < K; ++k) s += A[i * lda + k] * v[k];
        y[i] = s;
    }
}

/* activation: 0 = identity, 1 = ReLU */
void orc_activation(int64_t n, int act, double *y) {
    if (act == 1) for (int64_t i = 0; i < n; ++i) if (y[i] < 0.0) y[i] = 0.0;
}

/* ------------------------------------------------ GCN layer, Eq. 3 / 4 */

/* Y[i,k] = act( sum_{j in row i} r_i c_j sum_f X[j,f] W[f,k] ),
 * r = deg_row^(-1/2), c = deg_col^(-1/2) counted on the stored pattern.
 * Order: Z = X.W first, then the normalised neighbour sum.  No bias. */
int orc_gcn_layer(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                  const float *X, int64_t ldx, int32_t F_in, const float *W, int64_t ldw, int32_t F_out,
                  int act, double *Y) {
    int32_t *dr = (int32_t *)malloc((size_t)(n_rows + 1) * sizeof(int32_t));
    int32_t *dc = (int32_t *)malloc((size_t)(n_cols + 1) * sizeof(int32_t));
    double *r = (double *)malloc((size_t)(n_rows + 1) * sizeof(double));
    double *c = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    double *Z = (double *)malloc((size_t)n_cols * (size_t)F_out * sizeof(double) + 8);
    if (!dr || !dc || !r || !c || !Z) { free(dr); free(dc); free(r); free(c); free(Z); return 1; }
    orc_degrees(n_rows, n_cols, row_ptr, col_idx, dr, dc);
    orc_inv_sqrt_deg(dr, n_rows, r);
    orc_inv_sqrt_deg(dc, n_cols, c);
    ORC_PAR
    for (int32_t j = 0; j < n_cols; ++j)
        for (int32_t m = 0; m < F_out; ++m) {
            double s = 0.0;
            for (int32_t f = 0; f < F_in; ++f) s += (double)X[(int64_t)j * ldx + f] * (double)W[(int64_t)f * ldw + m];
            Z[(int64_t)j * F_out + m] = s;
        }
    ORC_PAR
    for (int32_t i = 0; i < n_rows; ++i) {
        double *y = Y + (int64_t)i * F_out;
        for (int32_t m = 0; m < F_out; ++m) y[m] = 0.0;
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            int32_t j = col_idx[k];
            double w = r[i] * c[j];
            for (int32_t m = 0; m < F_out; ++m) y[m] += w * Z[(int64_t)j * F_out + m];
        }
        if (act == 1) for (int32_t m = 0; m < F_out; ++m) if (y[m] < 0.0) y[m] = 0.0;
    }
    free(dr); free(dc); free(r); free(c); free(Z);
    return 0;
}

/* Selected output rows of the same layer, for sizes where Z = X.W for every
 * node is out of reach on the host.  Uses linearity of the neighbour sum:
 * sum_j w_ij (x_j W) = (sum_j w_ij x_j) W, exact up to fp64 rounding order.
 * Y is n_sel x F_out. */
int orc_gcn_layer_rows(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                       const float *X, int64_t ldx, int32_t F_in, const float *W, int64_t ldw, int32_t F_out,
                       int act, const int32_t *rows, int32_t n_sel, double *Y) {
    int32_t *dr = (int32_t *)malloc((size_t)(n_rows + 1) * sizeof(int32_t));
    int32_t *dc = (int32_t *)malloc((size_t)(n_cols + 1) * sizeof(int32_t));
    double *c = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    if (!dr || !dc || !c) { free(dr); free(dc); free(c); return 1; }
    orc_degrees(n_rows, n_cols, row_ptr, col_idx, dr, dc);
    orc_inv_sqrt_deg(dc, n_cols, c);
    ORC_PAR
    for (int32_t t = 0; t < n_sel; ++t) {
        int32_t i = rows[t];
        double *u = (double *)calloc((size_t)F_in + 1, sizeof(double));
        double ri = 1.0 / sqrt((double)(dr[i] < 1 ? 1 : dr[i]));
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            int32_t j = col_idx[k];
            double w = ri * c[j];
            for (int32_t f = 0; f < F_in; ++f) u[f] += w * (double)X[(int64_t)j * ldx + f];
        }
        for (int32_t m = 0; m < F_out; ++m) {
            double s = 0.0;
            for (int32_t f = 0; f < F_in; ++f) s += u[f] * (double)W[(int64_t)f * ldw + m];
            if (act == 1 && s < 0.0) s = 0.0;
            Y[(int64_t)t * F_out + m] = s;
        }
        free(u);
    }
    free(dr); free(dc); free(c);
    return 0;
}

/* ------------------------------------------------ GAT layer, Eq. 5 / 6 */

/* Theta = X.W; s_l = Theta.a_l, s_r = Theta.a_r; e_ij = LeakyReLU(s_l[i] +
 * s_r[j]) on the pattern; alpha = row softmax of e; Y = act(alpha.Theta).
 * Single head, no bias.  An empty row gives act(0) = 0. */
int orc_gat_layer(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                  const float *X, int64_t ldx, int32_t F_in, const float *W, int64_t ldw, int32_t F_out,
                  const float *a_l, const float *a_r, double slope, int act, double *Y) {
    /* destinations are the first n_rows source nodes (square graph: all of them) */
    if (n_rows > n_cols) return 2;
    double *T = (double *)malloc((size_t)n_cols * (size_t)F_out * sizeof(double) + 8);
    double *sl = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    double *sr = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    if (!T || !sl || !sr) { free(T); free(sl); free(sr); return 1; }
    ORC_PAR
    for (int32_t j = 0; j < n_cols; ++j) {
        for (int32_t m = 0; m < F_out; ++m) {
            double s = 0.0;
            for (int32_t f = 0; f < F_in; ++f) s += (double)X[(int64_t)j * ldx + f] * (double)W[(int64_t)f * ldw + m];
            T[(int64_t)j * F_out + m] = s;
        }
        double pl = 0.0, pr = 0.0;
        for (int32_t m = 0; m < F_out; ++m) {
            pl += T[(int64_t)j * F_out + m] * (double)a_l[m];
            pr += T[(int64_t)j * F_out + m] * (double)a_r[m];
        }
        sl[j] = pl; sr[j] = pr;
    }
    ORC_PAR
    for (int32_t i = 0; i < n_rows; ++i) {
        double *y = Y + (int64_t)i * F_out;
        for (int32_t m = 0; m < F_out; ++m) y[m] = 0.0;
        int32_t lo = row_ptr[i], hi = row_ptr[i + 1];
        if (lo == hi) continue;
        double *e = (double *)malloc((size_t)(hi - lo) * sizeof(double));
        double mx = -INFINITY;
        for (int32_t k = lo; k < hi; ++k) {
            double t = sl[i] + sr[col_idx[k]];
            e[k - lo] = t > 0.0 ? t : slope * t;
            if (e[k - lo] > mx) mx = e[k - lo];
        }
        double den = 0.0;
        for (int32_t k = lo; k < hi; ++k) den += exp(e[k - lo] - mx);
        for (int32_t k = lo; k < hi; ++k) {
            double al = exp(e[k - lo] - mx) / den;
            const double *th = T + (int64_t)col_idx[k] * F_out;
            for (int32_t m = 0; m < F_out; ++m) y[m] += al * th[m];
        }
        if (act == 1) for (int32_t m = 0; m < F_out; ++m) if (y[m] < 0.0) y[m] = 0.0;
        free(e);
    }
    free(T); free(sl); free(sr);
    return 0;
}

/* Selected output rows of the GAT layer.  Uses (X.W).a = X.(W.a) for the two
 * score vectors and sum_j alpha_ij (x_j W) = (sum_j alpha_ij x_j) W for the
 * aggregate, both exact up to fp64 rounding order.  Y is n_sel x F_out. */
int orc_gat_layer_rows(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                       const float *X, int64_t ldx, int32_t F_in, const float *W, int64_t ldw, int32_t F_out,
                       const float *a_l, const float *a_r, double slope, int act,
                       const int32_t *rows, int32_t n_sel, double *Y) {
    if (n_rows > n_cols) return 2;
    double *vl = (double *)calloc((size_t)F_in + 1, sizeof(double));
    double *vr = (double *)calloc((size_t)F_in + 1, sizeof(double));
    double *sl = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    double *sr = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    if (!vl || !vr || !sl || !sr) { free(vl); free(vr); free(sl); free(sr); return 1; }
    for (int32_t f = 0; f < F_in; ++f)
        for (int32_t m = 0; m < F_out; ++m) {
            vl[f] += (double)W[(int64_t)f * ldw + m] * (double)a_l[m];
            vr[f] += (double)W[(int64_t)f * ldw + m] * (double)a_r[m];
        }
    ORC_PAR
    for (int32_t j = 0; j < n_cols; ++j) {
        double pl = 0.0, pr = 0.0;
        for (int32_t f = 0; f < F_in; ++f) {
            pl += (double)X[(int64_t)j * ldx + f] * vl[f];
            pr += (double)X[(int64_t)j * ldx + f] * vr[f];
        }
        sl[j] = pl; sr[j] = pr;
    }
    ORC_PAR
    for (int32_t t = 0; t < n_sel; ++t) {
        int32_t i = rows[t];
        int32_t lo = row_ptr[i], hi = row_ptr[i + 1];
        double *y = Y + (int64_t)t * F_out;
        for (int32_t m = 0; m < F_out; ++m) y[m] = 0.0;
        if (lo == hi) continue;
        double *e = (double *)malloc((size_t)(hi - lo) * sizeof(double));
        double *u = (double *)calloc((size_t)F_in + 1, sizeof(double));
        double mx = -INFINITY;
        for (int32_t k = lo; k < hi; ++k) {
            double s = sl[i] + sr[col_idx[k]];
            e[k - lo] = s > 0.0 ? s : slope * s;
            if (e[k - lo] > mx) mx = e[k - lo];
        }
        double den = 0.0;
        for (int32_t k = lo; k < hi; ++k) den += exp(e[k - lo] - mx);
        for (int32_t k = lo; k < hi; ++k) {
            double al = exp(e[k - lo] - mx) / den;
            const float *x = X + (int64_t)col_idx[k] * ldx;
            for (int32_t f = 0; f < F_in; ++f) u[f] += al * (double)x[f];
        }
        for (int32_t m = 0; m < F_out; ++m) {
            double s = 0.0;
            for (int32_t f = 0; f < F_in; ++f) s += u[f] * (double)W[(int64_t)f * ldw + m];
            if (act == 1 && s < 0.0) s = 0.0;
            y[m] = s;
        }
        free(e); free(u);
    }
    free(vl); free(vr); free(sl); free(sr);
    return 0;
}

/* ------------------------------------------- training: gradients of a layer
 *
 * The evaluation section trains the models (forward + backward per
 * iteration); the paper leaves the backward pass to the framework's automatic
 * differentiation.  Reading: the backward of a layer is the gradient of the
 * scalar  L = sum_{i,k} dY[i,k] * Y[i,k]  with respect to the layer's inputs,
 * written out by the chain rule on the plain forward definition above, in
 * fp64.  The ReLU mask is taken from the forward output the caller passes
 * (Y[i,k] > 0), so that both sides of a comparison take that decision on the
 * same fp32 values.
 * Pins (tests/test_oracle_backward.py): central finite differences of the
 * forward oracle, closed forms (self-loop graph = dense linear layer; zero
 * attention vectors = mean aggregation), linearity in dY. */

/* col_ptr / row_of: the stored entries grouped by column (the transposed
 * pattern), entries of one column in ascending row order; pos[k] = place of
 * entry k in that order. */
static int orc_transpose(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                         int32_t **col_ptr_out, int32_t **row_of_out, int32_t **pos_out) {
    const int64_t nnz = row_ptr[n_rows];
    int32_t *col_ptr = (int32_t *)calloc((size_t)n_cols + 2, sizeof(int32_t));
    int32_t *row_of = (int32_t *)malloc(((size_t)nnz + 1) * sizeof(int32_t));
    int32_t *pos = (int32_t *)malloc(((size_t)nnz + 1) * sizeof(int32_t));
    if (!col_ptr || !row_of || !pos) { free(col_ptr); free(row_of); free(pos); return 1; }
    for (int64_t k = 0; k < nnz; ++k) col_ptr[col_idx[k] + 1]++;
    for (int32_t j = 0; j < n_cols; ++j) col_ptr[j + 1] += col_ptr[j];
    int32_t *fill = (int32_t *)malloc(((size_t)n_cols + 1) * sizeof(int32_t));
    if (!fill) { free(col_ptr); free(row_of); free(pos); return 1; }
    memcpy(fill, col_ptr, (size_t)n_cols * sizeof(int32_t));
    for (int32_t i = 0; i < n_rows; ++i)
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            int32_t p = fill[col_idx[k]]++;
            row_of[p] = i;
            pos[k] = p;
        }
    free(fill);
    *col_ptr_out = col_ptr; *row_of_out = row_of; *pos_out = pos;
    return 0;
}

/* GCN layer, Y = act(P), P = R A~ C (X W):
 *   dP = dY (.) [Y > 0]            (identity activation: dP = dY)
 *   dZ[j,:] = c_j sum_{i : (i,j) stored} r_i dP[i,:]        (Z = X W)
 *   dW = X^T dZ ,  dX = dZ W^T.
 * Y may be NULL when act == 0.  dX: n_cols x F_in, dW: F_in x F_out (fp64).
 * sel / n_sel: when sel != NULL only the rows sel[0..n_sel) of dX are computed
 * (dX is n_sel x F_in) and dW is not touched unless want_dw != 0.  dZ_out (optional,
 * n_cols x F_out, needs the full dZ: sel == NULL or want_dw) receives dZ, whose products with X are the
 * terms of the reduction over nodes in dW. */
int orc_gcn_backward(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                     const float *X, int64_t ldx, int32_t F_in, const float *W, int64_t ldw, int32_t F_out,
                     const float *Y, int64_t ldy, const float *dY, int64_t lddy, int act,
                     const int32_t *sel, int32_t n_sel, int want_dw, double *dX, double *dW, double *dZ_out) {
    int32_t *dr = (int32_t *)malloc((size_t)(n_rows + 1) * sizeof(int32_t));
    int32_t *dc = (int32_t *)malloc((size_t)(n_cols + 1) * sizeof(int32_t));
    double *r = (double *)malloc((size_t)(n_rows + 1) * sizeof(double));
    double *c = (double *)malloc((size_t)(n_cols + 1) * sizeof(double));
    int32_t *col_ptr = NULL, *row_of = NULL, *pos = NULL;
    if (!dr || !dc || !r || !c || orc_transpose(n_rows, n_cols, row_ptr, col_idx, &col_ptr, &row_of, &pos)) {
        free(dr); free(dc); free(r); free(c); return 1;
    }
    orc_degrees(n_rows, n_cols, row_ptr, col_idx, dr, dc);
    orc_inv_sqrt_deg(dr, n_rows, r);
    orc_inv_sqrt_deg(dc, n_cols, c);
    const int full = (sel == NULL);
    const int32_t n_out = full ? n_cols : n_sel;
    int rc = 0;
    double *dZ = NULL;
    if (full || want_dw) {
        dZ = (double *)malloc((size_t)n_cols * (size_t)F_out * sizeof(double) + 8);
        if (!dZ) rc = 1;
    }
    if (rc == 0 && dZ) {
        ORC_PAR
        for (int32_t j = 0; j < n_cols; ++j) {
            double *z = dZ + (int64_t)j * F_out;
            for (int32_t m = 0; m < F_out; ++m) z[m] = 0.0;
            for (int32_t p = col_ptr[j]; p < col_ptr[j + 1]; ++p) {
                const int32_t i = row_of[p];
                for (int32_t m = 0; m < F_out; ++m) {
                    double g = (double)dY[(int64_t)i * lddy + m];
                    if (act == 1 && !(Y[(int64_t)i * ldy + m] > 0.0f)) g = 0.0;
                    z[m] += r[i] * g;
                }
            }
            for (int32_t m = 0; m < F_out; ++m) z[m] *= c[j];
        }
        if (dZ_out) memcpy(dZ_out, dZ, (size_t)n_cols * (size_t)F_out * sizeof(double));
        if (full || want_dw) {
            ORC_PAR
            for (int32_t f = 0; f < F_in; ++f)
                for (int32_t m = 0; m < F_out; ++m) {
                    double s = 0.0;
                    for (int32_t j = 0; j < n_cols; ++j) s += (double)X[(int64_t)j * ldx + f] * dZ[(int64_t)j * F_out + m];
                    dW[(int64_t)f * F_out + m] = s;
                }
        }
    }
    if (rc == 0) {
        ORC_PAR
        for (int32_t t = 0; t < n_out; ++t) {
            const int32_t j = full ? t : sel[t];
            double *z = (double *)calloc((size_t)F_out + 1, sizeof(double));
            if (dZ) {
                memcpy(z, dZ + (int64_t)j * F_out, (size_t)F_out * sizeof(double));
            } else {
                for (int32_t p = col_ptr[j]; p < col_ptr[j + 1]; ++p) {
                    const int32_t i = row_of[p];
                    for (int32_t m = 0; m < F_out; ++m) {
                        double g = (double)dY[(int64_t)i * lddy + m];
                        if (act == 1 && !(Y[(int64_t)i * ldy + m] > 0.0f)) g = 0.0;
                        z[m] += r[i] * g;
                    }
                }
                for (int32_t m = 0; m < F_out; ++m) z[m] *= c[j];
            }
            for (int32_t f = 0; f < F_in; ++f) {
                double s = 0.0;
                for (int32_t m = 0; m < F_out; ++m) s += z[m] * (double)W[(int64_t)f * ldw + m];
                dX[(int64_t)t * F_in + f] = s;
            }
            free(z);
        }
    }
    free(dr); free(dc); free(r); free(c); free(col_ptr); free(row_of); free(pos); free(dZ);
    return rc;
}

/* GAT layer, Y = act(P), P = alpha Theta, Theta = X W, s_l = Theta a_l, s_r = Theta a_r,
 * t_ij = s_l[i] + s_r[j], e_ij = LeakyReLU(t_ij), alpha = row softmax of e:
 *   dP = dY (.) [Y > 0]
 *   dalpha_ij = <dP[i,:], Theta[j,:]>
 *   de_ij = alpha_ij (dalpha_ij - sum_j' alpha_ij' dalpha_ij')        (softmax)
 *   dt_ij = de_ij * (t_ij > 0 ? 1 : slope)
 *   ds_l[i] = sum_j dt_ij ,  ds_r[j] = sum_i dt_ij
 *   dTheta[j,:] = sum_i alpha_ij dP[i,:] + ds_l[j] a_l + ds_r[j] a_r
 *   da_l = Theta^T ds_l , da_r = Theta^T ds_r , dW = X^T dTheta , dX = dTheta W^T.
 * Square pattern only (destinations = the first n_rows sources, as in the
 * forward).  Outputs fp64: dX n_cols x F_in, dW F_in x F_out, da_l, da_r F_out; dTh_out (optional,
 * n_cols x F_out) receives dTheta; ds_out (optional, 2 n_cols) receives ds_l then ds_r. */
int orc_gat_backward(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                     const float *X, int64_t ldx, int32_t F_in, const float *W, int64_t ldw, int32_t F_out,
                     const float *a_l, const float *a_r, double slope,
                     const float *Y, int64_t ldy, const float *dY, int64_t lddy, int act,
                     double *dX, double *dW, double *da_l, double *da_r, double *dTh_out, double *ds_out) {
    if (n_rows > n_cols) return 2;
    const int64_t nnz = row_ptr[n_rows];
    double *Th = (double *)malloc((size_t)n_cols * (size_t)F_out * sizeof(double) + 8);
    double *dTh = (double *)calloc((size_t)n_cols * (size_t)F_out + 1, sizeof(double));
    double *sl = (double *)calloc((size_t)n_cols + 1, sizeof(double));
    double *sr = (double *)calloc((size_t)n_cols + 1, sizeof(double));
    double *dsl = (double *)calloc((size_t)n_cols + 1, sizeof(double));
    double *dsr = (double *)calloc((size_t)n_cols + 1, sizeof(double));
    double *alpha = (double *)malloc(((size_t)nnz + 1) * sizeof(double));
    double *dt = (double *)malloc(((size_t)nnz + 1) * sizeof(double));
    double *dP = (double *)malloc((size_t)n_rows * (size_t)F_out * sizeof(double) + 8);
    if (!Th || !dTh || !sl || !sr || !dsl || !dsr || !alpha || !dt || !dP) {
        free(Th); free(dTh); free(sl); free(sr); free(dsl); free(dsr); free(alpha); free(dt); free(dP);
        return 1;
    }
    ORC_PAR
    for (int32_t j = 0; j < n_cols; ++j) {
        for (int32_t m = 0; m < F_out; ++m) {
            double s = 0.0;
            for (int32_t f = 0; f < F_in; ++f) s += (double)X[(int64_t)j * ldx + f] * (double)W[(int64_t)f * ldw + m];
            Th[(int64_t)j * F_out + m] = s;
        }
        double a = 0.0, b = 0.0;
        for (int32_t m = 0; m < F_out; ++m) {
            a += Th[(int64_t)j * F_out + m] * (double)a_l[m];
            b += Th[(int64_t)j * F_out + m] * (double)a_r[m];
        }
        sl[j] = a; sr[j] = b;
    }
    ORC_PAR
    for (int32_t i = 0; i < n_rows; ++i)
        for (int32_t m = 0; m < F_out; ++m) {
            double g = (double)dY[(int64_t)i * lddy + m];
            if (act == 1 && !(Y[(int64_t)i * ldy + m] > 0.0f)) g = 0.0;
            dP[(int64_t)i * F_out + m] = g;
        }
    /* per destination row: alpha, dalpha, softmax and LeakyReLU backward */
    ORC_PAR
    for (int32_t i = 0; i < n_rows; ++i) {
        const int32_t b = row_ptr[i], e = row_ptr[i + 1];
        if (b == e) continue;
        double mx = -INFINITY;
        for (int32_t k = b; k < e; ++k) {
            double t = sl[i] + sr[col_idx[k]];
            double v = t > 0.0 ? t : slope * t;
            if (v > mx) mx = v;
        }
        double z = 0.0;
        for (int32_t k = b; k < e; ++k) {
            double t = sl[i] + sr[col_idx[k]];
            double v = t > 0.0 ? t : slope * t;
            alpha[k] = exp(v - mx);
            z += alpha[k];
        }
        double dot = 0.0;
        for (int32_t k = b; k < e; ++k) {
            alpha[k] /= z;
            const int32_t j = col_idx[k];
            double da = 0.0;
            for (int32_t m = 0; m < F_out; ++m) da += dP[(int64_t)i * F_out + m] * Th[(int64_t)j * F_out + m];
            dt[k] = da;  /* dalpha for now */
            dot += alpha[k] * da;
        }
        double acc = 0.0;
        for (int32_t k = b; k < e; ++k) {
            double t = sl[i] + sr[col_idx[k]];
            double de = alpha[k] * (dt[k] - dot);
            dt[k] = de * (t > 0.0 ? 1.0 : slope);
            acc += dt[k];
        }
        dsl[i] = acc;
    }
    /* the transposed sums, one source node j at a time over the entries of column j (ascending rows) */
    {
        int32_t *col_ptr = NULL, *row_of = NULL, *pos = NULL;
        int32_t *entry = (int32_t *)malloc(((size_t)nnz + 1) * sizeof(int32_t));  /* entry[p]: the stored entry at transposed place p */
        if (!entry || orc_transpose(n_rows, n_cols, row_ptr, col_idx, &col_ptr, &row_of, &pos)) {
            free(entry);
            free(Th); free(dTh); free(sl); free(sr); free(dsl); free(dsr); free(alpha); free(dt); free(dP);
            return 1;
        }
        for (int64_t k = 0; k < nnz; ++k) entry[pos[k]] = (int32_t)k;
        ORC_PAR
        for (int32_t j = 0; j < n_cols; ++j)
            for (int32_t p = col_ptr[j]; p < col_ptr[j + 1]; ++p) {
                const int32_t i = row_of[p], k = entry[p];
                dsr[j] += dt[k];
                for (int32_t m = 0; m < F_out; ++m) dTh[(int64_t)j * F_out + m] += alpha[k] * dP[(int64_t)i * F_out + m];
            }
        free(col_ptr); free(row_of); free(pos); free(entry);
    }
    for (int32_t m = 0; m < F_out; ++m) { da_l[m] = 0.0; da_r[m] = 0.0; }
    for (int32_t j = 0; j < n_cols; ++j)
        for (int32_t m = 0; m < F_out; ++m) {
            da_l[m] += Th[(int64_t)j * F_out + m] * dsl[j];
            da_r[m] += Th[(int64_t)j * F_out + m] * dsr[j];
            dTh[(int64_t)j * F_out + m] += dsl[j] * (double)a_l[m] + dsr[j] * (double)a_r[m];
        }
    if (dTh_out) memcpy(dTh_out, dTh, (size_t)n_cols * (size_t)F_out * sizeof(double));
    if (ds_out) {
        memcpy(ds_out, dsl, (size_t)n_cols * sizeof(double));
        memcpy(ds_out + n_cols, dsr, (size_t)n_cols * sizeof(double));
    }
    ORC_PAR
    for (int32_t f = 0; f < F_in; ++f)
        for (int32_t m = 0; m < F_out; ++m) {
            double s = 0.0;
            for (int32_t j = 0; j < n_cols; ++j) s += (double)X[(int64_t)j * ldx + f] * dTh[(int64_t)j * F_out + m];
            dW[(int64_t)f * F_out + m] = s;
        }
    ORC_PAR
    for (int32_t j = 0; j < n_cols; ++j)
        for (int32_t f = 0; f < F_in; ++f) {
            double s = 0.0;
            for (int32_t m = 0; m < F_out; ++m) s += dTh[(int64_t)j * F_out + m] * (double)W[(int64_t)f * ldw + m];
            dX[(int64_t)j * F_in + f] = s;
        }
    free(Th); free(dTh); free(sl); free(sr); free(dsl); free(dsr); free(alpha); free(dt); free(dP);
    return 0;
}
