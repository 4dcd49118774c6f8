/*
 * sensei.h - C ABI of the MI355X (gfx950) library that runs one GCN or GAT
 * layer as a chosen composition of sparse and dense primitives, after the
 * input-sensitive re-association method of SENSEi (arXiv 2306.15155).
 *
 * Conventions for every entry point
 *   - Pointers named in a struct or argument as "device" are device (HBM)
 *     addresses owned by the caller; the library never allocates, frees or
 *     keeps them past the call.  Everything else is host memory.
 *   - Dense matrices are row-major fp32 with an explicit leading dimension
 *     (ld >= cols, in elements).  Indices are int32.  A sparse matrix is CSR:
 *     rows are destination nodes, columns are source (in-neighbour) nodes,
 *     row_ptr[0] == 0, columns strictly ascending within a row, all in
 *     [0, n_cols).  Well-formed CSR is a precondition; it is not validated on
 *     the device.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work and return; only sensei_select in timed mode and
 *     sensei_calibrate synchronise.
 *   - `workspace` is device memory of at least the size the matching
 *     *_workspace query returns, aligned to 256 bytes; its contents are
 *     scratch.  Outputs must not alias inputs or the workspace.
 *   - Return value: a sensei_status.  No exception or abort crosses the ABI.
 *     Arguments are checked on the host before anything is launched; a failed
 *     check launches nothing.
 */
#ifndef SENSEI_H
#define SENSEI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SENSEI_OK = 0,
    SENSEI_INVALID_ARGUMENT = 1,   /* null pointer, negative size, ld < cols, shape mismatch, aliasing */
    SENSEI_INVALID_COMPOSITION = 2,
    SENSEI_WORKSPACE_TOO_SMALL = 3,
    SENSEI_HIP_ERROR = 4,          /* a HIP runtime call or a launch failed */
    SENSEI_UNSUPPORTED = 5,
    SENSEI_SCRATCH_TOO_SMALL = 6   /* sensei_spmm_static: the input needs more than SENSEI_STATIC_SCRATCH_BYTES */
} sensei_status;

typedef struct sensei_ctx sensei_ctx; /* opaque: device id and cost-model calibration only */

typedef struct sensei_panels sensei_panels; /* opaque host object: column-panel copy of a pattern, see below */
typedef struct sensei_tiles sensei_tiles;   /* opaque host object: dense-tile split of a pattern, see below */

typedef struct {
    int32_t n_rows, n_cols;
    int64_t nnz;
    const int32_t *row_ptr; /* device, n_rows + 1 */
    const int32_t *col_idx; /* device, nnz */
    const float *val;       /* device, nnz, or NULL: unweighted, only the positions are used
                               (matrix attribute table: sparse weighted / unweighted) */
    const sensei_panels *panels; /* host, optional (NULL: none): made by sensei_panels_create for this very pattern */
    const sensei_tiles *tiles;   /* host, optional (NULL: none): made by sensei_tiles_create for this very pattern */
} sensei_csr;

typedef struct {
    const float *ptr; /* device */
    int64_t rows, cols, ld;
} sensei_mat;

enum { SENSEI_ACT_NONE = 0, SENSEI_ACT_RELU = 1 };
enum { SENSEI_KIND_GCN = 0, SENSEI_KIND_GAT = 1 };

/* GCN compositions (case study GCN).  AGG = aggregate then update (GEMM last), UPD = update then
 * aggregate (GEMM first).  DYN = normalisation by two row broadcasts around a value-less SpMM
 * (Eq. 3); DYNF = the same scalings applied inside the SpMM; PRE = weighted SpMM over the
 * precomputed N~ (Eq. 4; the caller passes N~ as A->val, see sensei_gcn_precompute). */
enum {
    SENSEI_GCN_DYN_AGG = 0, SENSEI_GCN_DYN_UPD = 1, SENSEI_GCN_DYNF_AGG = 2,
    SENSEI_GCN_DYNF_UPD = 3, SENSEI_GCN_PRE_AGG = 4, SENSEI_GCN_PRE_UPD = 5
};
/* GAT compositions (case study GAT).  REUSE aggregates the updated embeddings Theta (Eq. 6);
 * RECOMP aggregates the input embeddings and applies W afterwards (Eq. 7).  *_FOLD obtain the
 * two score vectors as X.(W.a) instead of (X.W).a. */
enum { SENSEI_GAT_REUSE = 0, SENSEI_GAT_RECOMP = 1, SENSEI_GAT_RECOMP_FOLD = 2, SENSEI_GAT_REUSE_FOLD = 3 };

/* SpMM flavours (sensei_spmm `mode`) */
enum {
    SENSEI_SPMM_PATTERN = 0, /* C[i,:] = sum_j B[j,:]                 value-less SpMM                */
    SENSEI_SPMM_WEIGHTED = 1,/* C[i,:] = sum_j val[i,j] B[j,:]        Eq. 1 with (+,x)               */
    SENSEI_SPMM_SCALED = 2   /* C[i,:] = r[i] sum_j c[j] B[j,:]       Eq. 3's scalings inside the sum */
};

/* ------------------------------------------------------------------ context */

/* Creates a context bound to HIP device `device` (host pointer out). */
int sensei_create(sensei_ctx **out, int device);
int sensei_destroy(sensei_ctx *ctx);

/* Measures the few device rates the additive cost model uses (streaming and gather bandwidth,
 * GEMM rate, launch latency) with small kernels on `stream`; synchronises.  Optional: without it
 * sensei_select uses built-in MI355X defaults.  `workspace` >= 64 MiB. */
int sensei_calibrate(sensei_ctx *ctx, void *workspace, size_t ws_bytes, void *stream);

/* Optional instrumentation for benchmarks.  While enabled, every launch of the SpMM kernel and of the
 * GEMM kernel made through this context is bracketed by a pair of HIP events on the launch stream (at most
 * 4096 launches of each per recording; enabling starts a new recording).  sensei_profile_read waits for
 * the recorded events of one kernel and writes the elapsed milliseconds of each launch, in launch order,
 * to ms_out (host, `capacity` floats); count_out (host) receives the number of recorded launches. */
enum { SENSEI_PROFILE_SPMM = 0, SENSEI_PROFILE_GEMM = 1 };
int sensei_profile_enable(sensei_ctx *ctx, int enable);
int sensei_profile_read(sensei_ctx *ctx, int kernel, float *ms_out, int capacity, int *count_out);

int sensei_num_compositions(int kind);
const char *sensei_composition_name(int kind, int comp_id);
const char *sensei_status_string(int status);

/* Optional, once per graph: a copy of the pattern cut into column panels (columns [q*w, (q+1)*w) of panel q
 * stored contiguously, with the position of every entry in the original pattern).  When a sensei_csr carries
 * it, wide SpMMs (at least `min_width` floats per gathered row, 128 by default) run one panel after the other and add the partial results, so the
 * neighbour rows of the live panel stay resident in the L2s; results are the same up to fp32 summation order.
 * Not a step of the paper's method: a graph-dependent layout choice in the spirit of its input-sensitive
 * selection.  n_panels = 0 lets the library choose from the graph features (it may choose 1 = no panels, in
 * which case the object is ignored by the layer calls); 1..8 forces a count.
 *   sensei_panels_bytes : device bytes sensei_panels_create needs for this pattern (host pointers).
 *   sensei_panels_create: builds the copy in `device_buf` (caller-owned device memory, must stay alive and
 *                         unmodified as long as the object is used); A->row_ptr / A->col_idx must stay
 *                         unchanged too.  Synchronises `stream` once.  *out is a host object.
 *   sensei_panels_count : number of panels of the object.
 *   sensei_panels_set_min_width: narrowest SpMM (floats per gathered row, after the internal padding of
 *                         intermediates to a multiple of 32) that uses the panels; min_width >= 1.
 *   sensei_panels_destroy frees the host object only.
 * Measured choice (the analytic guess cannot see how skewed the column degrees are: the Reddit-shaped R-MAT
 * graph is fastest with 2 panels from width 128 on, a uniform graph of the same density with 4 from width 64 on):
 *   sensei_panels_tune_bytes: device scratch bytes sensei_panels_tune needs (256 when the graph features
 *                         alone rule panels out).
 *   sensei_panels_tune  : times the value-less SpMM of width 256 over the pattern with 1, 2, 3, 4, 6, 8 panels
 *                         (stopping once times rise again) on scratch operands, then width 64 with and without
 *                         the best count.  Returns the count (1 = keep the single pass; a gain under 3 % does
 *                         not count) and the min_width to set (64 or 128).  ms_per_count: optional host array of
 *                         2 * (SENSEI_PANELS_MAX + 1) floats, [q] = ms of the width-256 SpMM with q panels,
 *                         [SENSEI_PANELS_MAX + 1 + q] = ms of the width-64 SpMM, -1 where not tried.  `scratch`: caller-owned device memory, 256-byte aligned, free to reuse
 *                         afterwards.  Synchronises `stream` repeatedly; must not run under stream capture. */
int sensei_panels_bytes(const sensei_csr *A, int n_panels, size_t *device_bytes);
int sensei_panels_create(sensei_ctx *ctx, const sensei_csr *A, int n_panels, void *device_buf, size_t bytes, void *stream,
                         sensei_panels **out);
int sensei_panels_count(const sensei_panels *panels);
int sensei_panels_set_min_width(sensei_panels *panels, int min_width);
int sensei_panels_destroy(sensei_panels *panels);
#define SENSEI_PANELS_MAX 8
int sensei_panels_tune_bytes(const sensei_csr *A, size_t *bytes);
int sensei_panels_tune(sensei_ctx *ctx, const sensei_csr *A, void *scratch, size_t bytes, void *stream, int *n_panels_out,
                       int *min_width_out, float *ms_per_count);

/* Backward of the GAT layer (training; chain rule on Eq. 5-6).  With Theta = X.W, t_ij = s_l[i] + s_r[j],
 * e = LeakyReLU(t), alpha = row softmax(e), P = alpha.Theta, Y = act(P) and dP = dY (.) [Y > 0]:
 *     dalpha_ij = <dP[i,:], Theta[j,:]>                         (g-SDDMM, Eq. 2 with a dot product)
 *     de_ij = alpha_ij (dalpha_ij - sum_j' alpha_ij' dalpha_ij'),  dt_ij = de_ij * (t_ij > 0 ? 1 : slope)
 *     ds_l[i] = sum_j dt_ij,  ds_r[j] = sum_i dt_ij
 *     dTheta = alpha^T.dP + ds_l a_l^T + ds_r a_r^T,  da_l = Theta^T ds_l,  da_r = Theta^T ds_r
 *     dW = X^T.dTheta,  dX = dTheta.W^T  (skipped when dX is NULL).
 * Theta, the logits and the softmax statistics are recomputed from X, W, a_l, a_r (nothing is kept from the
 * forward call).  At: the transposed pattern (A itself when symmetric); t_pos: nnz int32 (device), the place of
 * each stored entry of A in At, from sensei_transpose_positions.  n_rows <= n_cols as in the forward.
 *   sensei_transpose_positions: fills t_pos; synchronises `stream`; INVALID_ARGUMENT if At is not the transpose
 *   of A (an entry of A has no counterpart).  Columns must be ascending within each row of At.
 *   Dense-tile splits (sensei_tiles_create, below) are used where attached: one on A serves the dalpha products of the
 *   entries inside its tiles (from F_out = 128), one on At the product alpha^T.dP.  The workspace query takes both patterns
 *   as the layer call will get them (At may be NULL there if it carries no split). */
int sensei_transpose_positions(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, int32_t *t_pos, void *workspace,
                               size_t ws_bytes, void *stream);
int sensei_gat_backward_workspace(const sensei_csr *A, const sensei_csr *At, int f_in, int f_out, size_t *bytes);
int sensei_gat_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W,
                        const float *a_l, const float *a_r, float neg_slope, const float *Y, int64_t ldy, sensei_mat dY, int activation,
                        float *dX, int64_t lddx, float *dW, int64_t lddw, float *da_l, float *da_r, void *workspace, size_t ws_bytes,
                        void *stream);

/* Backward of the multi-head layer sensei_gat_layer_heads (heads concatenated; they share only the input): head h is the single-head
 * layer on columns [h d, (h + 1) d) of W, a_l, a_r and Y, d = f_out / n_heads, so dW, da_l and da_r hold the heads' gradients in the
 * same columns and dX is the sum over the heads; the products with X and W are formed once for all heads.  Arguments, aliasing rules
 * and error codes as for sensei_gat_backward; n_heads must divide f_out. */
int sensei_gat_backward_heads_workspace(const sensei_csr *A, const sensei_csr *At, int f_in, int f_out, int n_heads, size_t *bytes);
int sensei_gat_backward_heads(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W,
                              const float *a_l, const float *a_r, int n_heads, float neg_slope, const float *Y, int64_t ldy, sensei_mat dY,
                              int activation, float *dX, int64_t lddx, float *dW, int64_t lddw, float *da_l, float *da_r, void *workspace,
                              size_t ws_bytes, void *stream);

/* Backward of the layer sensei_gatv2_layer (the GATv2 variant named with the attention variants of the paper's discussion; training as in
 * its evaluation section).  With dP = dY (.) [Y > 0], Theta_l = X_dst W_l, Theta_r = X W_r, U_ij = Theta_l[i] + Theta_r[j],
 * e_ij = att . LeakyReLU(U_ij) and alpha the row softmax of e (Eq. 5 with this score):
 *   dalpha_ij = <dP_i, Theta_r[j]>,   de_ij = alpha_ij (dalpha_ij - sum_k alpha_ik dalpha_ik),
 *   datt = sum_ij de_ij LeakyReLU(U_ij),
 *   dTheta_l[i] = att (.) sum_j de_ij LeakyReLU'(U_ij),   dTheta_r[j] = sum_i alpha_ij dP_i + att (.) sum_i de_ij LeakyReLU'(U_ij),
 *   dW_l = X_dst^T dTheta_l (f_in x f_out, lddwl),   dW_r = X^T dTheta_r (lddwr),   datt (f_out floats),
 *   dX = dTheta_r W_r^T, plus dTheta_l W_l^T on the first n_rows rows (n_cols x f_in, lddx; skipped when dX is NULL).
 * With one shared weight matrix (W_l = W_r in the forward) its gradient is dW_l + dW_r.  At, t_pos: the transposed pattern and the
 * place of every stored entry in it (sensei_transpose_positions), as for sensei_gat_backward; the other arguments, aliasing rules and
 * error codes as there.  Column panels and tile splits attached to the patterns are not used by this call. */
int sensei_gatv2_backward_workspace(const sensei_csr *A, int f_in, int f_out, size_t *bytes);
int sensei_gatv2_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W_l,
                          sensei_mat W_r, const float *att, float neg_slope, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX,
                          int64_t lddx, float *dW_l, int64_t lddwl, float *dW_r, int64_t lddwr, float *datt, void *workspace, size_t ws_bytes,
                          void *stream);

/* Backward of the layer sensei_dotgat_layer (key-query attention; training as in the paper's evaluation section).  With
 * dP = dY (.) [Y > 0], Q = X_dst W_q, K = X W_k, V = X W_v, e_ij = scale <Q_i, K_j> and alpha the row softmax of e:
 *   dV_j = sum_i alpha_ij dP_i,   dalpha_ij = <dP_i, V_j>,   de_ij = alpha_ij (dalpha_ij - sum_k alpha_ik dalpha_ik),
 *   dQ_i = scale sum_j de_ij K_j,   dK_j = scale sum_i de_ij Q_i,
 *   dW_q = X_dst^T dQ (f_in x d_k, lddwq),   dW_k = X^T dK (lddwk),   dW_v = X^T dV (f_in x f_out, lddwv),
 *   dX = dK W_k^T + dV W_v^T, plus dQ W_q^T on the first n_rows rows (n_cols x f_in, lddx; skipped when dX is NULL).
 * At, t_pos and the other arguments, aliasing rules and error codes as for sensei_gat_backward.  Column panels and tile splits attached
 * to the patterns are not used by this call. */
int sensei_dotgat_backward_workspace(const sensei_csr *A, int f_in, int d_k, int f_out, size_t *bytes);
int sensei_dotgat_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W_q,
                           sensei_mat W_k, sensei_mat W_v, float scale, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX,
                           int64_t lddx, float *dW_q, int64_t lddwq, float *dW_k, int64_t lddwk, float *dW_v, int64_t lddwv, void *workspace,
                           size_t ws_bytes, void *stream);

/* ------------------------------------------------- primitives (steps of a layer) */

/* Degrees of the stored pattern, which holds the self edges (case study GCN: D~ is the degree
 * of the nodes of A~).  deg_row[i] = entries of row i; deg_col[j] = entries of column j.
 * Outputs: device int32, n_rows and n_cols entries.  Exact integer work. */
int sensei_degrees(sensei_ctx *ctx, const sensei_csr *A, int32_t *deg_row, int32_t *deg_col, void *stream);

/* out[i] = 1 / sqrt(max(deg[i], 1)) in fp32 with correctly rounded sqrt and divide: the vector
 * form of D~^(-1/2) (Eq. 3).  deg, out: device, n entries. */
int sensei_norm_vectors(sensei_ctx *ctx, const int32_t *deg, int64_t n, float *out, void *stream);

/* Stored entries per chunk (= per 64-lane wavefront) that every sparse kernel uses on a pattern of `nnz` entries: 64, 128, 256
 * or 512, growing with nnz (small graphs are latency bound and get more, shorter wavefronts).  Host arithmetic; 0 if nnz < 0. */
int sensei_chunk_nnz(int64_t nnz);

/* Which matrix-core kernel sensei_gemm (and the GEMM inside the layers) takes for an n x k by k x m product: the fp32 instruction,
 * or, for large products, the bf16 instruction on three exact bf16 pieces per fp32 operand element with six piece products per
 * term (what is left out is below 2^-23 of a term: the result is as accurate as the fp32 instruction's, at several times its
 * rate).  Host arithmetic; for reports that price the kernel against the right matrix-core peak. */
enum { SENSEI_GEMM_FP32 = 0, SENSEI_GEMM_BF16_PIECES = 1 };
int sensei_gemm_kernel(int64_t n, int k, int m);

/* Upper bound, in bytes, on the workspace any sparse primitive below needs for this matrix at
 * feature width `f` (host pointers). */
int sensei_sparse_workspace(const sensei_csr *A, int f, size_t *bytes);

/* N~ = D_r^(-1/2) . A~ . D_c^(-1/2) as an SDDMM whose two dense operands are the diagonal
 * matrices taken as vectors (Eq. 4; first candidate->primitive rule): val_out[e] = r[i] * c[j]
 * for the e-th stored entry (i,j).  r: n_rows, c: n_cols, val_out: nnz, all device. */
int sensei_gcn_precompute(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, float *val_out,
                          void *workspace, size_t ws_bytes, void *stream);

/* Row broadcast (Eq. 3): Y[i,:] = s[i] * X[i,:], s device with X.rows entries.  Y may equal X.ptr. */
int sensei_row_broadcast(sensei_ctx *ctx, const float *s, sensei_mat X, float *Y, int64_t ldy, void *stream);

/* g-SpMM with (+,x) (Eq. 1) in the three flavours above, followed by the activation.  B has
 * A->n_cols rows; C is n_rows x B.cols with leading dimension ldc.  r / c are used by
 * SENSEI_SPMM_SCALED only (NULL otherwise); A->val by SENSEI_SPMM_WEIGHTED only. */
int sensei_spmm(sensei_ctx *ctx, const sensei_csr *A, int mode, const float *r, const float *c, sensei_mat B,
                float *C, int64_t ldc, int activation, void *workspace, size_t ws_bytes, void *stream);

/* sensei_spmm for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result and same kernels as sensei_spmm without the
 * workspace pair: the chunk plan and the carry slots live in a static device array of SENSEI_STATIC_SCRATCH_BYTES that each
 * GPU the library runs on holds until the process ends (its address is resolved by sensei_create).  The call allocates
 * nothing, creates no events and uses no second stream; A->panels and A->tiles are ignored and B is gathered as it is
 * (row-major).  Inputs that need more scratch (about 4 bytes per 512 stored entries for the plan plus
 * ceil(nnz / chunk) * (pad32(B.cols) + 256) * 4 bytes of carry slots, chunk = 64..512 entries by nnz) are rejected with
 * SENSEI_SCRATCH_TOO_SMALL and launch nothing.  Every call on a GPU shares that GPU's array: calls that overlap in time on
 * one GPU (different streams, or graphs replayed concurrently) race on it; calls in stream order are safe.  `stream` must
 * belong to the context's device. */
#define SENSEI_STATIC_SCRATCH_BYTES (32u << 20)
int sensei_spmm_static(sensei_ctx *ctx, const sensei_csr *A, int mode, const float *r, const float *c, sensei_mat B, float *C,
                       int64_t ldc, int activation, void *stream);

/* Dense update Y = act(A . W) on the matrix cores, fp32 in and out at fp32 accuracy (background: dense primitives; which
 * instruction a shape takes: sensei_gemm_kernel).
 * A: n x k, W: k x m, Y: n x m with leading dimension ldy. */
int sensei_gemm(sensei_ctx *ctx, sensei_mat A, sensei_mat W, float *Y, int64_t ldy, int activation, void *stream);

/* Two matrix-vector products in one pass over A: y1 = A.v1, y2 = A.v2 (v*: A.cols entries,
 * y*: A.rows entries, device).  Used for the attention projections s_l, s_r of Eq. 5. */
int sensei_gemv2(sensei_ctx *ctx, sensei_mat A, const float *v1, const float *v2, float *y1, float *y2, void *stream);

/* Attention logits on the pattern (g-SDDMM, Eq. 2, with k = 1 and + as the inner operator):
 * e[(i,j)] = LeakyReLU_slope(s_l[i] + s_r[j]); s_l: n_rows, s_r: n_cols, e_out: nnz (device). */
int sensei_sddmm_score(sensei_ctx *ctx, const sensei_csr *A, const float *s_l, const float *s_r, float neg_slope,
                       float *e_out, void *workspace, size_t ws_bytes, void *stream);

/* Softmax over the stored entries of each row: alpha = exp(e - m_i) / sum_row exp(e - m_i),
 * m_i the row maximum.  e, alpha_out: nnz (device); alpha_out may equal e. */
int sensei_edge_softmax(sensei_ctx *ctx, const sensei_csr *A, const float *e, float *alpha_out,
                        void *workspace, size_t ws_bytes, void *stream);

/* ----------------------------------------------------------------------- layers */

int sensei_gcn_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes);

/* One GCN layer, Y = act( D_r^(-1/2) A~ D_c^(-1/2) X W ) (Eq. 3 / Eq. 4), evaluated in the
 * order composition `comp_id` prescribes.  A holds the self edges already.  r: n_rows and
 * c: n_cols are the D~^(-1/2) vectors (sensei_norm_vectors of the row / column degrees); for
 * PRE_* compositions A->val must hold N~ and r, c may be NULL; for the others A->val is ignored.
 * X: n_cols x f_in, W: f_in x f_out, Y: n_rows x f_out. */
int sensei_gcn_layer(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, sensei_mat X, sensei_mat W,
                     float *Y, int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream);

/* GATv2 layer (the attention variant the paper's discussion names): Theta_l = X W_l over the destinations, Theta_r = X W_r
 * over the sources, e_ij = sum_m att[m] LeakyReLU(Theta_l[i, m] + Theta_r[j, m]) on every stored entry (Eq. 2 in its general
 * form: a vector per entry, reduced after a non-linearity), alpha = row softmax of e as in the GAT layer,
 * Y = act( sum_j alpha_ij Theta_r[j, :] ).  W_l and W_r are f_in x f_out; passing the same matrix twice shares the weights
 * (one GEMM on a square pattern).  att has f_out entries.  Destinations are the first n_rows sources (n_rows <= n_cols).
 *   comp_id 0 (reuse):     aggregate Theta_r at width f_out;
 *   comp_id 1 (recompute): aggregate X at width f_in, then one more GEMM with W_r (pays when f_in < f_out). */
int sensei_gatv2_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes);
int sensei_gatv2_layer(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W_l, sensei_mat W_r, const float *att, float neg_slope,
                       float *Y, int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream);

/* Key-query attention layer: the score function of GaAN-style layers (named with GATv2 among the attention variants the paper's
 * discussion lists), Eq. 2 with a dot product as the inner operator: Q = X W_q over the destinations, K = X W_k over the sources,
 * e_ij = scale <Q[i,:], K[j,:]> on every stored entry (scale is typically 1 / sqrt(d_k)), alpha = row softmax of e as in the GAT layer,
 * Y = act( sum_j alpha_ij (X W_v)[j,:] ).  W_q, W_k: f_in x d_k; W_v: f_in x f_out.  Destinations are the first n_rows sources
 * (n_rows <= n_cols).  Single head; GaAN's per-head gates are not part of it.
 *   comp_id 0 (reuse):     aggregate the value projections X W_v at width f_out;
 *   comp_id 1 (recompute): aggregate X at width f_in, then the GEMM with W_v (pays when f_in < f_out). */
int sensei_dotgat_workspace(const sensei_csr *A, int f_in, int d_k, int f_out, int comp_id, size_t *bytes);
int sensei_dotgat_layer(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W_q, sensei_mat W_k, sensei_mat W_v, float scale, float *Y,
                        int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream);

/* Dense-tile split of a pattern (layout, not a step of the paper; Section 3.2: which primitive is cheap depends on the input).
 * On a skewed graph the rows and columns of the highest degree meet in a region that is nearly full: with the nodes in
 * order of descending degree, tiles of 128 x 128 ranks (among the first 65,536 ranks of either side) that hold at least
 * min_density * 16384 entries are kept as bit masks and multiplied on the matrix cores (sparse unweighted . dense
 * evaluated as a block-sparse GEMM), the SpMM runs over the CSR remainder of the entries outside such tiles, and a last
 * pass joins the two sums and applies the row scaling and the activation.  The tiles use the bf16 matrix instruction at
 * fp32 accuracy: a mask entry is 0 or 1, and every fp32 operand element is cut exactly into three bf16 pieces (the attention
 * weights as well: six piece products per term, what is left out is below 2^-23 of a term).  Where a step uses the object's
 * own stream (the GAT layer's tile statistics, the backward), the fork and join are event dependencies between the two
 * streams, so the call stays asynchronous and can be captured into a graph.  These steps use the split when `tiles` is set
 * in the sensei_csr:
 * the value-less SpMM on an internal slice-major operand of at most max_width columns (a multiple of 32; what the
 * GCN, SGC and TAGCN layers and the GCN backward run on graphs whose rows are gathered often); the attention
 * aggregation of the GAT layer (reuse compositions: every head whose width is a whole number of 32-column slices;
 * recompute compositions: when the layer gathers from its slice-major copy of X), where the tiles form the softmax
 * weights from the attention projections themselves; and two steps of the
 * GAT backward (see there).  Every other call ignores it.  Results differ from the unsplit path only in the order of
 * summation.  Whether the split pays depends on the graph: attach it when a good part of the entries lies in kept tiles
 * (sensei_tiles_info; measured: 64 % of the entries: SpMM call -44 %; 20 %: +2 %, so leave it off there).
 * min_density: 0 < min_density <= 1; 0.05 .. 0.09 measured best on a
 * 233,000-node power-law graph (0.07: 64 % of the entries in 22,334 tiles, step time 16.9 -> 9.65 ms).
 *   sensei_tiles_bytes   device bytes sensei_tiles_create needs (an upper bound taken before the tiles are counted);
 *   sensei_tiles_create  builds the split in device_buf (256-byte aligned, caller-owned, must outlive the object);
 *                        ranks the nodes on the host, so it synchronises the stream several times: a set-up call;
 *   sensei_tiles_info    kept tiles, entries inside them, entries in the remainder;
 *   sensei_tiles_set_min_width  narrowest SpMM (columns) that takes the split; 64 unless set (the attention aggregation
 *                        takes it from half that width);
 *   sensei_tiles_destroy frees the host object only.
 * The object keeps buffers for the operand in rank order and for the tiles' product, and its stream: calls that use one
 * object at the same time on different streams race on them.
 * The remainder itself may be kept a second time in panel-major order (its entries column panel by column panel, two or three panels), which the
 * forward SpMM calls of 64 columns or more then walk in one launch, one raw partial row per (panel, row), joined by the last pass: the part
 * of the gathered matrix in use at one time then fits the L2s.  Chosen automatically (a 128-byte slice of the gathered matrix of 12 MB or
 * more, 128 or more entries per row; three panels from 24 MB on); sensei_tiles_remainder_panels overrides the choice for the objects created afterwards in this
 * process (0: automatic, 1: never, 2..8: that many panels whatever the graph; returns the previous setting; a tuning and testing knob -
 * set it before sensei_tiles_bytes, which sizes the buffer for it). */
int sensei_tiles_remainder_panels(int n_panels);
int sensei_tiles_bytes(const sensei_csr *A, float min_density, int max_width, size_t *device_bytes);
int sensei_tiles_create(sensei_ctx *ctx, const sensei_csr *A, float min_density, int max_width, void *device_buf, size_t bytes, void *stream,
                        sensei_tiles **out);
int sensei_tiles_info(const sensei_tiles *tiles, int *n_tiles_kept, int64_t *nnz_dense, int64_t *nnz_sparse);
int sensei_tiles_set_min_width(sensei_tiles *tiles, int min_width);
int sensei_tiles_destroy(sensei_tiles *tiles);

/* K-hop simplified graph convolution (SGC, one of the GCN variants the paper names as further targets of the same
 * re-association): Y = act( A^^k X W ) with A^ = D_r^(-1/2) A~ D_c^(-1/2) on a square pattern, k_hops >= 1.
 *   comp_id 0: aggregate first, ((A^^k X) W): k SpMMs at width f_in, then the GEMM (the choice for f_in <= f_out);
 *   comp_id 1: update first, (A^^k (X W)): the GEMM, then k SpMMs at width f_out (f_in >= f_out).
 * Inner hops stay in the slice-major layout (the SpMM writes what the next SpMM gathers) with the factor r_i c_i
 * of two adjacent scalings applied in the epilogue.  k_hops = 1 is the GCN layer. */
int sensei_sgc_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes);
int sensei_sgc_layer(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, sensei_mat X, sensei_mat W, int k_hops, float *Y,
                     int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream);

/* Topology-adaptive graph convolution (TAGCN, the other K-hop variant the paper names): Y = act( sum_{k=0..k_hops} A^^k X W_k ),
 * W = [W_0; W_1; ...; W_k_hops] stacked by hop, (k_hops + 1) * f_in rows by f_out columns; square pattern, k_hops >= 1.
 *   comp_id 0: aggregate first: the hops H_k = A^ H_(k-1) at width f_in, then one GEMM over all hops, [H_0 .. H_K] W;
 *   comp_id 1: update first, Horner form at width f_out: T_K = X W_K, T_k = X W_k + A^ T_(k+1), Y = act(T_0).
 * Both do k_hops SpMMs and (k_hops + 1) n f_in f_out multiply-adds of GEMM work; they differ in the SpMM width, as in
 * the GCN layer. */
int sensei_tagcn_workspace(const sensei_csr *A, int f_in, int f_out, int k_hops, int comp_id, size_t *bytes);
int sensei_tagcn_layer(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, sensei_mat X, sensei_mat W, int k_hops, float *Y,
                       int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream);

/* Backward of the GCN layer (the paper's evaluation trains the models: one forward and one backward per
 * iteration; the backward is the gradient of the forward by the chain rule, with the same freedom of
 * association): given dY = dL/dY it computes
 *     dP = dY (.) [Y > 0]  (ReLU; dP = dY without activation),
 *     dW = X^T D_c^(-1/2) A~^T D_r^(-1/2) dP     (f_in x f_out),
 *     dX = D_c^(-1/2) A~^T D_r^(-1/2) dP W^T     (n_cols x f_in; skipped when dX is NULL).
 * bwd_id chooses where the transposed aggregation runs:
 *     SENSEI_GCN_BWD_AGG: G = D_c^(-1/2) A~^T D_r^(-1/2) dP at width f_out, dW = X^T G, dX = G W^T
 *                         (the choice for f_out <= f_in, the mirror of the update-first forward);
 *     SENSEI_GCN_BWD_UPD: dW = U^T dP with U = D_r^(-1/2) A~ D_c^(-1/2) X (taken from `U_saved` if given, else
 *                         recomputed by one SpMM at width f_in), dX = D_c^(-1/2) A~^T D_r^(-1/2) (dP W^T) at
 *                         width f_in (the choice for f_in < f_out).
 * At: the transposed pattern (n_cols x n_rows, CSR); for a symmetric pattern pass A itself.  Y: the forward
 * output (n_rows x f_out, ldy), needed only with SENSEI_ACT_RELU.  U_saved: optional n_rows x f_in, ldu.
 * Outputs must not alias inputs or the workspace.  Results equal the plain chain rule up to fp32 summation
 * order; dW is reduced over the nodes in fixed slabs, so it does not depend on scheduling. */
enum { SENSEI_GCN_BWD_AGG = 0, SENSEI_GCN_BWD_UPD = 1 };
int sensei_gcn_backward_workspace(const sensei_csr *A, int f_in, int f_out, int bwd_id, size_t *bytes);
int sensei_gcn_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const float *r, const float *c, sensei_mat X,
                        sensei_mat W, const float *Y, int64_t ldy, sensei_mat dY, int activation, const float *U_saved, int64_t ldu,
                        float *dX, int64_t lddx, float *dW, int64_t lddw, int bwd_id, void *workspace, size_t ws_bytes, void *stream);

/* Backward of the K-hop layer sensei_sgc_layer, Y = act( A^^k X W ) on a square pattern: dP = dY (.) [Y > 0], G = (A^^T)^k dP,
 * dW = X^T G, dX = G W^T (skipped when dX is NULL), with the two associations of sensei_gcn_backward applied to the k hops:
 *     SENSEI_GCN_BWD_AGG: the k transposed hops run on dP at width f_out, then dW = X^T G and dX = G W^T;
 *     SENSEI_GCN_BWD_UPD: dW = U^T dP with U = A^^k X recomputed (k hops at width f_in), dX = (A^^T)^k (dP W^T) at width f_in.
 * Hops keep their intermediate results in the slice-major layout the next hop gathers from, as in the forward.  k_hops = 1 is
 * sensei_gcn_backward without a saved U.  Arguments as there. */
int sensei_sgc_backward_workspace(const sensei_csr *A, int f_in, int f_out, int k_hops, int bwd_id, size_t *bytes);
int sensei_sgc_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const float *r, const float *c, sensei_mat X, sensei_mat W,
                        int k_hops, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX, int64_t lddx, float *dW, int64_t lddw,
                        int bwd_id, void *workspace, size_t ws_bytes, void *stream);

/* Backward of the layer sensei_tagcn_layer, Y = act( sum_{k=0..K} A^^k X W_k ) on a square pattern (the K-hop variant with a weight
 * block per hop, among the further GNN variants the paper's discussion names; training as in its evaluation section): with
 * dP = dY (.) [Y > 0],   dW_k = (A^^k X)^T dP = X^T (A^^T)^k dP   (stacked by rows like W)   and   dX = sum_k (A^^T)^k dP W_k^T
 * (skipped when dX is NULL).  The two ways of writing dW_k are the two associations:
 *     SENSEI_GCN_BWD_AGG: the gradient goes through the hops at width f_out, Q_k = A^^T Q_(k-1) from Q_0 = dP (K transposed
 *                         aggregations), dW_k = X^T Q_k, dX = [Q_0 .. Q_K] [W_0^T; ..; W_K^T] as one product of depth (K+1) f_out;
 *     SENSEI_GCN_BWD_UPD: the input goes forward at width f_in, H_k = A^^ H_(k-1) from H_0 = X (K aggregations), dW_k = H_k^T dP,
 *                         and dX comes back in Horner form, R_K = dP W_K^T, R_k = dP W_k^T + A^^T R_(k+1), dX = R_0 (K transposed
 *                         aggregations at width f_in).
 * k_hops >= 0 (0: a dense layer).  W and dW: (k_hops + 1) f_in x f_out.  Other arguments, aliasing rules and error codes as for
 * sensei_gcn_backward; with no rows dW is set to zero. */
int sensei_tagcn_backward_workspace(const sensei_csr *A, int f_in, int f_out, int k_hops, int bwd_id, size_t *bytes);
int sensei_tagcn_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const float *r, const float *c, sensei_mat X, sensei_mat W,
                          int k_hops, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX, int64_t lddx, float *dW, int64_t lddw,
                          int bwd_id, void *workspace, size_t ws_bytes, void *stream);

/* Which association of the GCN backward is predicted faster for this graph and these sizes (the additive
 * per-primitive cost model of sensei_select, host arithmetic only).  have_saved_u: the forward kept
 * U = D_r^(-1/2) A~ D_c^(-1/2) X; want_dx: the input gradient is needed.  est_ms: optional, 2 entries. */
int sensei_select_gcn_backward(sensei_ctx *ctx, const sensei_csr *A, int f_in, int f_out, int have_saved_u, int want_dx,
                               int *bwd_id_out, float *est_ms);
/* The same for the backward of the K-hop layers (the selection of Section 3.5 applied to their two associations): per_hop_weights = 0
 * prices sensei_sgc_backward, 1 sensei_tagcn_backward.  Every hop adds one aggregation at the width the association carries through
 * the hops (f_out for SENSEI_GCN_BWD_AGG; f_in, forward and - with want_dx - back again, for SENSEI_GCN_BWD_UPD). */
int sensei_select_khop_backward(sensei_ctx *ctx, const sensei_csr *A, int f_in, int f_out, int k_hops, int per_hop_weights, int want_dx,
                                int *bwd_id_out, float *est_ms);

int sensei_gat_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes);

/* One single-head GAT layer (Eq. 5-7): Theta = X.W; s_l = Theta.a_l, s_r = Theta.a_r;
 * e_ij = LeakyReLU(s_l[i] + s_r[j]) on the pattern; alpha = row softmax; Y = act(alpha.Theta),
 * in the order composition `comp_id` prescribes.  Destination node i is source node i
 * (n_rows <= n_cols).  a_l, a_r: f_out entries (device). */
int sensei_gat_layer(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W, const float *a_l,
                     const float *a_r, float neg_slope, float *Y, int64_t ldy, int activation, int comp_id,
                     void *workspace, size_t ws_bytes, void *stream);

/* Which form the attention part (scores, softmax, aggregation) of sensei_gat_layer / sensei_gat_layer_heads takes for this
 * input (host arithmetic on the sizes and on what A carries; -1 on invalid arguments):
 *   TWO_PASS  one pass forms the logits and the row statistics (max, sum of exp), the aggregation applies exp(e - max) / sum;
 *   ONE_WALK  score, running-maximum softmax and weighted sum in a single walk of each row, nothing stored per entry: taken where
 *             the aggregation is 32 columns wide at most and rows average 16 entries or more, or 64 columns and 128 entries;
 *   TILES     the dense-tile split attached to A serves statistics and aggregation; PANELS: two passes over the column panels. */
enum { SENSEI_GAT_PATH_TWO_PASS = 0, SENSEI_GAT_PATH_ONE_WALK = 1, SENSEI_GAT_PATH_TILES = 2, SENSEI_GAT_PATH_PANELS = 3 };
int sensei_gat_attention_path(const sensei_csr *A, int f_in, int f_out, int n_heads, int comp_id);

/* Multi-head GAT layer, heads concatenated: W is f_in x (n_heads * d) with head h in columns [h d, (h + 1) d), a_l and
 * a_r hold n_heads * d entries laid out the same way, Y is n_rows x (n_heads * d).  Every head is the single-head layer
 * above on its d columns of Theta = X.W (its own logits, softmax and aggregation); Theta is formed by one GEMM for all
 * heads.  comp_id as for sensei_gat_layer; the workspace is that of sensei_gat_workspace for f_out = n_heads * d.
 * n_heads must divide W.cols. */
int sensei_gat_layer_heads(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W, const float *a_l, const float *a_r,
                           int n_heads, float neg_slope, float *Y, int64_t ldy, int activation, int comp_id, void *workspace,
                           size_t ws_bytes, void *stream);

/* --------------------------------------------------------------------- selector */

enum { SENSEI_SELECT_MODEL = 0, SENSEI_SELECT_TIMED = 1, SENSEI_SELECT_LEARNED = 2, SENSEI_SELECT_AUTO = 3 };

/* Bytes sensei_select needs in timed mode (it runs every candidate once on scratch operands); learned mode needs
 * 256 bytes. */
int sensei_select_workspace(int kind, const sensei_csr *A, int f_in, int f_out, size_t *bytes);

/* Chooses a composition for (graph, f_in, f_out) (online stage; code generation of promoted
 * candidates).  First the embedding-size conditions drop the candidates annotated for the other
 * scenario; then
 *   mode MODEL: cost(id) = sum of the predicted times of its primitives from the graph features
 *               (rows, columns, non-zeros, density) and the sizes; smallest cost wins, ties to
 *               the lowest id.  Host arithmetic only, nothing is launched, workspace unused.
 *   mode TIMED: every remaining candidate is run once on scratch operands in `workspace` and the fastest is kept (the
 *               "run all once, keep the best" strategy); a candidate that takes under 0.5 ms is run a second time and the second
 *               figure kept, so that no candidate is judged on a cold first run where that could decide; synchronises `stream`.
 *   mode AUTO:  MODEL first; if more than one candidate lies within 15 % of the cheapest prediction and `workspace` holds
 *               sensei_select_workspace bytes, those candidates alone go through the TIMED trial (others cannot win; their
 *               est_ms stays the prediction).  With one clear candidate, or without the workspace, it is MODEL.
 *   mode LEARNED: as MODEL, but the SpMM and GEMM times come from gradient-boosted regression trees fitted to
 *               timings of these primitives on MI355X over a grid of synthetic graphs (the learned per-primitive
 *               cost models of Section 3.5; tables generated by paper_2306_15155_amd/costmodel/train.py).
 *   In MODEL, LEARNED and AUTO the value-less and attention SpMMs are priced on the path they will take: a dense-tile split
 *   attached to A (made for this very pattern) takes its share of the gathers off those calls.  The graph
 *               feature extractor adds two measures of skew read from row_ptr by one small kernel (largest row,
 *               second moment of the row lengths): needs 256 bytes of `workspace`, synchronises `stream`.
 * comp_id_out: host int.  est_ms (host, nullable): sensei_num_compositions(kind) floats,
 * predicted or measured ms per id, negative for ids the conditions dropped. */
int sensei_select(sensei_ctx *ctx, int kind, const sensei_csr *A, int f_in, int f_out, int mode, int *comp_id_out,
                  float *est_ms, void *workspace, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SENSEI_H */
