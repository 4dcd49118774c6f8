// C ABI of libsensei_hip: argument checks, workspace layout, the composition
// executors for the GCN and GAT layer, and the composition selector.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <new>

#include "sensei_internal.h"

using namespace sensei;

// Rates the additive cost model is built from; defaults are MI355X measurements and can be
// replaced by sensei_calibrate.
struct sensei_ctx {
    int device;
    double launch_us;      // fixed cost of one kernel launch in a stream
    double stream_bps;     // achieved bandwidth of a streaming (read + write) kernel
    double gather_l2_bps;  // row-gather bandwidth when the gathered slice fits the L2s
    double gather_far_bps; // row-gather bandwidth when it does not (Infinity Cache / HBM)
    double gemm_flops;     // achieved rate of fp32 multiply-adds of the GEMM on large products
    double l2_slice_bytes; // feature-slice footprint at which 88 % of the gathers are served by the L2s
    Timers timers;         // optional per-launch timing of the SpMM and GEMM kernels
    void *scratch;         // device address of the static scratch array on this context's GPU (sensei_spmm_static)
};

// Scratch memory of sensei_spmm_static (chunk plan + carry slots): a file-scope device array, so every GPU the library is
// loaded on holds its own copy at its own address until the process ends.  In host code the name is only a stand-in for the
// symbol: the device address comes from hipGetSymbolAddress (sensei_create, once per device) and is what the kernels get.
static __device__ __align__(256) unsigned char scratch[SENSEI_STATIC_SCRATCH_BYTES];

// Column-panel copy of a pattern (host descriptor; the arrays live in the caller's device buffer).
struct sensei_panels {
    int n_panels, width;
    int32_t n_rows, n_cols;
    int64_t nnz;
    const int32_t *src_row_ptr, *src_col_idx;  // the pattern it was built from
    int chunk_nnz;                             // every panel uses the chunk size of the whole pattern
    int64_t nnz_q[SENSEI_MAX_PANELS];
    int32_t *row_ptr_q[SENSEI_MAX_PANELS], *col_q[SENSEI_MAX_PANELS], *chunk_row_q[SENSEI_MAX_PANELS];
    int32_t *position;                         // position[k]: where original entry k sits in the panel copy
    int32_t off_q[SENSEI_MAX_PANELS + 1];      // first entry of each panel in the copy
    int n_chunks_q[SENSEI_MAX_PANELS];
    int min_width = 128;                       // narrowest SpMM (floats per gathered row) that goes panel by panel
};

// Dense-tile split of a pattern: bit masks of the kept 128 x 128 tiles (in degree-rank order), the CSR of everything else.
struct sensei_tiles {
    int32_t n_rows, n_cols;
    int64_t nnz;
    const int32_t *src_row_ptr, *src_col_idx;  // the pattern it was built from
    sensei::TileSplit T;
    int64_t nnz_rem;                           // entries left in the sparse remainder
    const int32_t *row_ptr_rem, *col_rem;
    const int32_t *dst_rem;                    // nnz: place of each original entry in the remainder, -1 for the entries inside tiles
    sensei::ChunkPlan plan_rem;
    float *Bh;                                 // room for the gathered matrix in rank order, max_width columns
    int max_width;
    hipStream_t side = nullptr;                // the tiles are multiplied on this stream while the caller's runs the sparse remainder
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int min_width = 64;                        // narrowest SpMM that takes the split
    // Panel-major copy of the remainder (rem_panels > 1): its entries run column panel by column panel, so that the part of the
    // gathered matrix in use at one time fits the L2s; read as one CSR over the segments (panel q, row i) -> q * n_rows + i.
    int rem_panels = 1;
    const int32_t *seg_ptr = nullptr;          // rem_panels * n_rows + 1 row pointers of the segments
    const int32_t *col_pm = nullptr;           // nnz_rem columns, panel-major
    const int32_t *pos_pm = nullptr;           // nnz_rem: place of remainder entry d in the panel-major order
    sensei::ChunkPlan plan_pm;
    float *part_pm = nullptr;                  // rem_panels * n_rows x max_width raw partial rows, slice-major
    float2 *stats_pm = nullptr;                // rem_panels copies of the per-row softmax statistics
};

namespace {

const char *kGcnNames[] = {"DYN_AGG", "DYN_UPD", "DYNF_AGG", "DYNF_UPD", "PRE_AGG", "PRE_UPD"};
const char *kGatNames[] = {"REUSE", "RECOMP", "RECOMP_FOLD", "REUSE_FOLD"};
constexpr int kNumGcn = 6, kNumGat = 4;

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` per GPU, resolved by the first sensei_create on that GPU

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline int hip_status(hipError_t e) { return e == hipSuccess ? SENSEI_OK : SENSEI_HIP_ERROR; }

bool csr_ok(const sensei_csr *A, bool need_val) {
    if (!A || A->n_rows < 0 || A->n_cols < 0 || A->nnz < 0) return false;
    if (A->nnz > 2147483647LL - 4096) return false;
    if (!A->row_ptr) return false;
    if (A->nnz > 0 && !A->col_idx) return false;
    if (need_val && A->nnz > 0 && !A->val) return false;
    return true;
}
bool mat_ok(const sensei_mat &M) { return M.rows >= 0 && M.cols >= 0 && M.ld >= M.cols && (M.ptr || M.rows == 0 || M.cols == 0); }

bool overlap(const void *a, size_t na, const void *b, size_t nb) {
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
}
size_t mat_bytes(const float *, int64_t rows, int64_t cols, int64_t ld) {
    if (rows <= 0 || cols <= 0) return 0;
    return (size_t)((rows - 1) * ld + cols) * sizeof(float);
}

// carves 256-byte aligned pieces out of the caller's workspace
struct Carver {
    char *base;
    size_t used, cap;
    Carver(void *p, size_t n) : base(static_cast<char *>(p)), used(0), cap(n) {}
    template <class T> T *take(size_t count) {
        const size_t bytes = align_up(count * sizeof(T), 256);
        T *p = reinterpret_cast<T *>(base + used);
        used += bytes;
        return p;
    }
};

bool relayout_pays(const sensei_csr &A);

// room for a slice-major copy of the gathered matrix of the stand-alone SpMM, where it pays
size_t spmm_copy_bytes(const sensei_csr &A, int f) {
    return (relayout_pays(A) && f >= 32) ? align_up((size_t)A.n_cols * pad32(f) * sizeof(float), 256) : 0;
}

size_t sparse_ws(const sensei_csr &A, int f) {
    return plan_bytes(A.nnz) + spmm_carry_bytes(A.nnz, f) + softmax_ws_bytes(A) + spmm_copy_bytes(A, f) + 256;
}

ChunkPlan make_plan(const sensei_csr &A, Carver &cv) {
    ChunkPlan p;
    p.chunk_nnz = choose_chunk_nnz(A.nnz);
    p.n_chunks = A.nnz <= 0 ? 1 : (int)((A.nnz + p.chunk_nnz - 1) / p.chunk_nnz);
    p.chunk_row = cv.take<int32_t>((size_t)p.n_chunks + 1);
    return p;
}

bool gcn_is_agg(int id) { return id == SENSEI_GCN_DYN_AGG || id == SENSEI_GCN_DYNF_AGG || id == SENSEI_GCN_PRE_AGG; }

// A slice-major copy of a user matrix the SpMM gathers from costs one pass over it (8 bytes per element); it pays
// once every row is gathered many times.
bool relayout_pays(const sensei_csr &A) { return A.nnz >= 16 * (int64_t)A.n_cols; }  // declared above

size_t gcn_ws(const sensei_csr &A, int f_in, int f_out, int id) {
    const int fs = gcn_is_agg(id) ? pad4(f_in) : pad32(f_out);
    size_t b = plan_bytes(A.nnz) + spmm_carry_bytes(A.nnz, fs);
    if (gcn_is_agg(id)) {
        b += align_up((size_t)A.n_rows * fs * sizeof(float), 256);                                    // U
        b += align_up((size_t)A.n_cols * pad32(f_in) * sizeof(float), 256);                           // c (x) X, or the slice-major copy of X
    } else {
        b += align_up((size_t)A.n_cols * fs * sizeof(float), 256);                                    // Z = X.W
    }
    return b + 256;
}

bool gat_is_reuse(int id) { return id == SENSEI_GAT_REUSE || id == SENSEI_GAT_REUSE_FOLD; }

size_t gat_ws(const sensei_csr &A, int f_in, int f_out, int id) {
    const int fo = pad32(f_out), fi = pad4(f_in);
    size_t b = plan_bytes(A.nnz) + softmax_ws_bytes(A);
    b += 2 * align_up((size_t)A.n_cols * sizeof(float), 256);                  // s_l, s_r
    b += align_up((size_t)(A.nnz > 0 ? A.nnz : 1) * sizeof(float), 256);       // attention logits
    b += 2 * align_up((size_t)fi * sizeof(float), 256);                        // W.a_l, W.a_r
    if (id != SENSEI_GAT_RECOMP_FOLD) b += align_up((size_t)A.n_cols * fo * sizeof(float), 256);  // Theta
    if (gat_is_reuse(id)) {
        b += spmm_carry_bytes(A.nnz, fo);
    } else {
        b += spmm_carry_bytes(A.nnz, fi);
        b += align_up((size_t)A.n_rows * fi * sizeof(float), 256);             // U = alpha.X
        b += align_up((size_t)A.n_cols * pad32(f_in) * sizeof(float), 256);    // slice-major copy of X
    }
    return b + 256;
}

#define SENSEI_TRY(expr)                                  \
    do {                                                  \
        hipError_t e__ = (expr);                          \
        if (e__ != hipSuccess) return SENSEI_HIP_ERROR;   \
    } while (0)

int auto_panels(const sensei_csr &A) {
    const double slice = (double)A.n_cols * 128.0;  // one 128-byte feature slice of the gathered matrix
    const double avg = A.n_rows > 0 ? (double)A.nnz / A.n_rows : 0.0;
    if (slice < 12e6 || avg < 128.0) return 1;
    // two panels measured best at a 30 MB slice (6.7 ms against 6.8 with three, 7.2 with four, 7.5 without);
    // larger slices get one panel more per 40 MB
    const int q = 2 + (int)(slice / 40e6);
    return q > 4 ? 4 : q;
}

bool panels_usable(const sensei_csr &A, int f) {
    const sensei_panels *p = A.panels;
    return p && p->n_panels > 1 && f >= p->min_width && p->src_row_ptr == A.row_ptr && p->src_col_idx == A.col_idx && p->nnz == A.nnz &&
           p->n_rows == A.n_rows && p->n_cols == A.n_cols;
}

// The dense-tile split serves the value-less SpMM on a slice-major operand (what the layers use on graphs whose rows are
// gathered often); everything else takes the ordinary paths.
struct AttnVectors {  // what the softmax mode of the dense tiles needs besides the row statistics
    const float *s_l, *s_r;
    float slope;
    bool gathered;  // the operand already sits in the split's buffer in rank order (the caller ran launch_tiles_gather)
    bool tiles_done = false;  // the caller has also multiplied the tiles already, with the tile-local shift (launch_dense_tiles, local_shift)
};

bool tiles_usable(const sensei_csr &A, int mode, int f, bool b_sliced, bool attn = false) {
    const sensei_tiles *D = A.tiles;
    const bool mode_ok = (mode == SENSEI_SPMM_PATTERN) || (mode == kSpmmSoftmax && attn);
    // the attention mode has more to gain per column (its entries also skip the stored logits): half the width suffices
    // (measured: 8 heads of 32 columns on a 233,000-node power-law graph, 13.9 -> 11.8 ms)
    if (!D || !mode_ok || !b_sliced || D->T.n_slots <= 0) return false;
    const int need = attn ? D->min_width / 2 : D->min_width;
    if (pad32(f) > D->max_width || f < need) return false;
    return D->n_rows == A.n_rows && D->n_cols == A.n_cols && D->nnz == A.nnz && D->src_row_ptr == A.row_ptr && D->src_col_idx == A.col_idx;
}

// The remainder of a usable split runs panel-major from 64 columns on (narrower calls are short either way)
bool remainder_panels_usable(const sensei_tiles &D, int f) { return D.rem_panels > 1 && pad32(f) >= 64; }

// SpMM over the whole pattern, or panel after panel when the matrix carries a usable panel copy.  Values
// (WEIGHTED, kSpmmSoftmax) can only follow the panels if they are stored in panel order (val_in_panel_order);
// values in the order of the original pattern use the single pass.
hipError_t spmm_any(const sensei_csr &A, int mode, const float *r, const float *c, const float *B, int64_t ldb, int f, float *C,
                    int64_t ldc, int f_store, int act, const ChunkPlan &plan, float *carry, hipStream_t s, KernelTimer *kt,
                    bool val_in_panel_order = false, const float2 *mz = nullptr, bool b_sliced = false, bool c_sliced = false,
                    const AttnVectors *attn = nullptr) {
    // attn: softmax mode on a pattern with a dense-tile split; A.val then holds the logits of the remainder, in its order
    const bool has_val = (mode == SENSEI_SPMM_WEIGHTED || mode == kSpmmSoftmax);
    if (tiles_usable(A, mode, f, b_sliced, attn != nullptr)) {
        // The hub tiles go to the matrix cores, the sparse remainder runs as an SpMM; a last pass joins the two raw sums and
        // applies scale and activation.
        const sensei_tiles &D = *A.tiles;
        hipEvent_t t0 = kt ? kt->next() : nullptr, t1 = t0 ? kt->next() : nullptr;
        if (t1 && hipEventRecord(t0, s) != hipSuccess) return hipErrorUnknown;
        // The tiles run before the sparse remainder, on the same stream.  On a second stream beside it they gain nothing: the
        // tile kernels keep most of a compute unit's registers, and beside them the remainder loses more time than the tiles
        // take alone (233,000-node power-law graph, 256 columns: 3.44 ms together, 3.28 ms one after the other); the attention
        // tiles, eight wavefronts and 36 KB of LDS a workgroup, find no room beside the remainder and run after it anyway.
        const bool tiles_done = attn && attn->tiles_done;
        const float *tile_shift = tiles_done ? D.T.rank_vec + (size_t)D.T.nt_r * 128 : nullptr;
        hipError_t e = tiles_done ? hipSuccess
                                  : launch_dense_tiles(D.T, B, A.n_cols, pad32(f), D.Bh, s, attn ? attn->s_l : nullptr, attn ? attn->s_r : nullptr,
                                                       attn ? mz : nullptr, attn ? attn->slope : 0.f, false, attn && attn->gathered);
        if (e != hipSuccess) return e;
        sensei_csr Ar = A;
        Ar.nnz = D.nnz_rem; Ar.row_ptr = D.row_ptr_rem; Ar.col_idx = D.col_rem; Ar.panels = nullptr; Ar.tiles = nullptr;
        if (remainder_panels_usable(D, f)) {
            // Panel-major remainder: one launch over the segments (panel, row), whose chunks run panel by panel, so what the
            // wavefronts in flight gather from is one column panel of one 32-column slice per L2 (measured on the 233,000-node
            // power-law graph at 256 columns: L2 hit rate of the remainder 44 -> 82 %, bytes over the fabric 25 -> 7.5 GB per call).
            // Every segment leaves a raw partial row; the join below adds a row's segments.  Values (the remainder's logits in
            // attention mode) are in panel-major order: the caller wrote them through pos_pm.
            Ar.n_rows = D.rem_panels * A.n_rows; Ar.row_ptr = D.seg_ptr; Ar.col_idx = D.col_pm;
            const float2 *mz_seg = mz;
            if (mode == kSpmmSoftmax) {  // the kernel reads the row maximum by segment number
                e = launch_replicate_stats(mz, A.n_rows, D.rem_panels, D.stats_pm, s);
                mz_seg = D.stats_pm;
            }
            const int fp = pad32(f);
            if (e == hipSuccess)
                e = launch_spmm(Ar, mode, nullptr, c, B, ldb, fp, D.part_pm, 32, fp, SENSEI_ACT_NONE, D.plan_pm, carry, s, nullptr, false, false, mz_seg,
                                b_sliced, 1, true, true);
            if (e == hipSuccess)
                e = launch_tiles_combine_pm(D.T, C, A.n_rows, f_store, ldc, c_sliced, fp, mode == kSpmmSoftmax ? nullptr : r,
                                            mode == kSpmmSoftmax ? mz : nullptr, act, s, D.part_pm, D.rem_panels, D.seg_ptr, D.plan_pm.chunk_nnz, carry, fp,
                                            tile_shift);
            if (e != hipSuccess) return e;
            if (t1 && hipEventRecord(t1, s) != hipSuccess) return hipErrorUnknown;
            return hipSuccess;
        }
        // the SpMM leaves its carry slots to the combine pass, which visits every row anyway
        e = launch_spmm(Ar, mode, nullptr, c, B, ldb, f, C, ldc, f_store, SENSEI_ACT_NONE, D.plan_rem, carry, s, nullptr, false, false, mz, b_sliced, 1,
                        c_sliced, true);
        if (e == hipSuccess)
            e = launch_tiles_combine(D.T, C, A.n_rows, f_store, ldc, c_sliced, pad32(f), mode == kSpmmSoftmax ? nullptr : r,
                                     mode == kSpmmSoftmax ? mz : nullptr, act, s, D.row_ptr_rem, D.plan_rem.chunk_nnz, carry, pad32(f), tile_shift);
        if (e != hipSuccess) return e;
        if (t1 && hipEventRecord(t1, s) != hipSuccess) return hipErrorUnknown;
        return hipSuccess;
    }
    if (!panels_usable(A, f) || (has_val && !val_in_panel_order))
        return launch_spmm(A, mode, r, c, B, ldb, f, C, ldc, f_store, act, plan, carry, s, kt, false, true, mz, b_sliced, 1, c_sliced);
    const sensei_panels &P = *A.panels;
    hipEvent_t t0 = kt ? kt->next() : nullptr, t1 = t0 ? kt->next() : nullptr;
    if (t1 && hipEventRecord(t0, s) != hipSuccess) return hipErrorUnknown;
    for (int q = 0; q < P.n_panels; ++q) {
        sensei_csr Aq = A;
        Aq.nnz = P.nnz_q[q];
        Aq.row_ptr = P.row_ptr_q[q];
        Aq.col_idx = P.col_q[q];
        if (Aq.val) Aq.val = A.val + P.off_q[q];
        ChunkPlan pq;
        pq.chunk_nnz = P.chunk_nnz;
        pq.n_chunks = P.n_chunks_q[q];
        pq.chunk_row = P.chunk_row_q[q];
        const hipError_t e = launch_spmm(Aq, mode, r, c, B, ldb, f, C, ldc, f_store, act, pq, carry, s, nullptr, q > 0, q == P.n_panels - 1, mz, b_sliced, 1, c_sliced);
        if (e != hipSuccess) return e;
    }
    if (t1 && hipEventRecord(t1, s) != hipSuccess) return hipErrorUnknown;
    return hipSuccess;
}

int run_gcn(const sensei_csr &A, const float *r, const float *c, const sensei_mat &X, const sensei_mat &W, float *Y,
            int64_t ldy, int act, int id, void *ws, size_t ws_bytes, hipStream_t s, Timers *tm) {
    KernelTimer *kt = tm ? &tm->spmm : nullptr, *gt = tm ? &tm->gemm : nullptr;
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv);
    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    const int mode = (id == SENSEI_GCN_DYN_AGG || id == SENSEI_GCN_DYN_UPD) ? SENSEI_SPMM_PATTERN
                     : (id == SENSEI_GCN_DYNF_AGG || id == SENSEI_GCN_DYNF_UPD) ? SENSEI_SPMM_SCALED
                                                                                 : SENSEI_SPMM_WEIGHTED;
    if (gcn_is_agg(id)) {
        const int fs = pad4(f_in);
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fs) / sizeof(float));
        float *U = cv.take<float>((size_t)A.n_rows * fs);
        // The SpMM gathers from c (x) X (DYN_AGG, Eq. 3) or from X itself; either way from a slice-major copy when the
        // rows are gathered often enough to pay for writing it.
        const float *src = X.ptr;
        int64_t ld_src = X.ld;
        const bool sliced = relayout_pays(A);
        if (sliced || id == SENSEI_GCN_DYN_AGG) {
            float *T = cv.take<float>((size_t)A.n_cols * pad32(f_in));
            const float *scale = (id == SENSEI_GCN_DYN_AGG) ? c : nullptr;
            if (sliced) SENSEI_TRY(launch_to_slices(scale, X.ptr, X.ld, A.n_cols, f_in, T, s));
            else SENSEI_TRY(launch_row_broadcast(scale, X.ptr, X.ld, A.n_cols, f_in, T, fs, SENSEI_ACT_NONE, s));
            src = T;
            ld_src = fs;
        }
        const bool scaled = (mode == SENSEI_SPMM_SCALED);
        SENSEI_TRY(spmm_any(A, mode, scaled ? r : nullptr, scaled ? c : nullptr, src, ld_src, f_in, U, fs, f_in, SENSEI_ACT_NONE, plan, carry, s, kt,
                            false, nullptr, sliced));
        if (id == SENSEI_GCN_DYN_AGG) SENSEI_TRY(launch_row_broadcast(r, U, fs, A.n_rows, f_in, U, fs, SENSEI_ACT_NONE, s));
        SENSEI_TRY(launch_gemm(U, fs, W.ptr, W.ld, Y, ldy, A.n_rows, f_in, f_out, f_out, act, s, nullptr, gt));
    } else {
        const int fs = pad32(f_out);
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fs) / sizeof(float));
        float *Z = cv.take<float>((size_t)A.n_cols * fs);
        // DYNF_UPD: the column scaling is a row broadcast on Z = X.W, fused into the GEMM epilogue; the row
        // scaling and the activation are fused into the SpMM epilogue, so the SpMM itself is value-less.
        const float *z_scale = (id == SENSEI_GCN_DYNF_UPD) ? c : nullptr;
        // Z is only ever gathered by the SpMM, so the GEMM writes it slice-major (the in-place row broadcast of
        // DYN_UPD keeps the row-major form)
        const bool sliced = (id != SENSEI_GCN_DYN_UPD);
        SENSEI_TRY(launch_gemm(X.ptr, X.ld, W.ptr, W.ld, Z, fs, A.n_cols, f_in, f_out, fs, SENSEI_ACT_NONE, s, z_scale, gt, sliced));
        if (id == SENSEI_GCN_DYN_UPD) {
            SENSEI_TRY(launch_row_broadcast(c, Z, fs, A.n_cols, fs, Z, fs, SENSEI_ACT_NONE, s));
            SENSEI_TRY(spmm_any(A, mode, nullptr, nullptr, Z, fs, fs, Y, ldy, f_out, SENSEI_ACT_NONE, plan, carry, s, kt));
            SENSEI_TRY(launch_row_broadcast(r, Y, ldy, A.n_rows, f_out, Y, ldy, act, s));
        } else if (id == SENSEI_GCN_DYNF_UPD) {
            SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, r, nullptr, Z, fs, fs, Y, ldy, f_out, act, plan, carry, s, kt, false, nullptr, true));
        } else {
            SENSEI_TRY(spmm_any(A, mode, nullptr, nullptr, Z, fs, fs, Y, ldy, f_out, act, plan, carry, s, kt, false, nullptr, true));
        }
    }
    return SENSEI_OK;
}

// ---- K-hop simplified graph convolution: Y = act(A^^K X W), A^ = R A~ C, square pattern
size_t sgc_ws(const sensei_csr &A, int f_in, int f_out, int id) {
    const int f = (id == 0) ? f_in : f_out;
    size_t b = plan_bytes(A.nnz) + spmm_carry_bytes(A.nnz, pad32(f)) + 512;
    b += 2 * align_up((size_t)A.n_cols * pad32(f) * sizeof(float), 256);  // the two slice-major hop buffers
    b += align_up((size_t)A.n_rows * sizeof(float), 256);                 // r (.) c
    if (id == 0) b += align_up((size_t)A.n_rows * pad4(f_in) * sizeof(float), 256);  // U = A^^K X
    return b;
}

int run_sgc(const sensei_csr &A, const float *r, const float *c, const sensei_mat &X, const sensei_mat &W, int k_hops, float *Y, int64_t ldy,
            int act, int id, void *ws, size_t ws_bytes, hipStream_t s, Timers *tm) {
    KernelTimer *kt = tm ? &tm->spmm : nullptr, *gt = tm ? &tm->gemm : nullptr;
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    const int f = (id == 0) ? f_in : f_out, fp = pad32(f);
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv);
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fp) / sizeof(float));
    float *buf[2] = {cv.take<float>((size_t)A.n_cols * fp), cv.take<float>((size_t)A.n_cols * fp)};
    float *rc = cv.take<float>((size_t)A.n_rows);
    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    // between two hops the row scaling of one and the column scaling of the next meet: one factor r_i c_i per node
    SENSEI_TRY(launch_row_broadcast(r, c, 1, A.n_rows, 1, rc, 1, SENSEI_ACT_NONE, s));
    // hop input 0, slice-major with the column scaling applied: c (x) X, or c (x) (X.W) straight from the GEMM epilogue
    if (id == 0) SENSEI_TRY(launch_to_slices(c, X.ptr, X.ld, A.n_cols, f_in, buf[0], s));
    else SENSEI_TRY(launch_gemm(X.ptr, X.ld, W.ptr, W.ld, buf[0], fp, A.n_cols, f_in, f_out, fp, SENSEI_ACT_NONE, s, c, gt, true));
    for (int k = 0; k + 1 < k_hops; ++k)  // inner hops stay slice-major: the SpMM writes what the next one gathers
        SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, rc, nullptr, buf[k & 1], fp, fp, buf[(k + 1) & 1], fp, fp, SENSEI_ACT_NONE, plan, carry, s, kt,
                            false, nullptr, true, true));
    const float *last = buf[(k_hops - 1) & 1];
    if (id == 0) {
        float *U = cv.take<float>((size_t)A.n_rows * pad4(f_in));
        SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, r, nullptr, last, fp, f_in, U, pad4(f_in), f_in, SENSEI_ACT_NONE, plan, carry, s, kt, false,
                            nullptr, true));
        SENSEI_TRY(launch_gemm(U, pad4(f_in), W.ptr, W.ld, Y, ldy, A.n_rows, f_in, f_out, f_out, act, s, nullptr, gt));
    } else {
        SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, r, nullptr, last, fp, fp, Y, ldy, f_out, act, plan, carry, s, kt, false, nullptr, true));
    }
    return SENSEI_OK;
}

// ---- TAGCN: Y = act(sum_{k=0..K} A^^k X W_k), W = [W_0; ...; W_K] stacked by hop
size_t tagcn_ws(const sensei_csr &A, int f_in, int f_out, int k_hops, int id) {
    const int f = (id == 0) ? f_in : f_out, fp = pad32(f);
    size_t b = plan_bytes(A.nnz) + spmm_carry_bytes(A.nnz, fp) + 512;
    b += align_up((size_t)A.n_rows * sizeof(float), 256);  // r (.) c, or nothing to merge for id 1 (kept for one layout)
    if (id == 0) {
        b += align_up((size_t)(k_hops + 1) * A.n_cols * fp * sizeof(float), 256);           // c (x) H_0 .. c (x) H_K, slice-major, side by side
        b += align_up((size_t)A.n_rows * sizeof(float), 256);                               // 1 / c
        b += align_up((size_t)(k_hops + 1) * fp * pad4(f_out) * sizeof(float), 256);        // W with each hop's block padded to the slices
    } else {
        b += 2 * align_up((size_t)A.n_cols * fp * sizeof(float), 256);                      // T and the aggregated term
    }
    return b;
}

int run_tagcn(const sensei_csr &A, const float *r, const float *c, const sensei_mat &X, const sensei_mat &W, int k_hops, float *Y, int64_t ldy,
              int act, int id, void *ws, size_t ws_bytes, hipStream_t s, Timers *tm) {
    KernelTimer *kt = tm ? &tm->spmm : nullptr, *gt = tm ? &tm->gemm : nullptr;
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    const int f = (id == 0) ? f_in : f_out, fp = pad32(f);
    const int64_t n = A.n_rows;
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv);
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fp) / sizeof(float));
    float *rc = cv.take<float>((size_t)n);
    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    if (id == 0) {
        // hops at width f_in, kept as G_k = c (x) H_k (what the next SpMM gathers); the one GEMM over all hops undoes the
        // scaling per row: sum_k H_k W_k = diag(1/c) [G_0 .. G_K] [W_0; ..; W_K]
        const size_t hop = (size_t)n * fp;
        float *G = cv.take<float>((size_t)(k_hops + 1) * hop);
        float *inv_c = cv.take<float>((size_t)n);
        const int ldws = pad4(f_out);
        float *Wst = cv.take<float>((size_t)(k_hops + 1) * fp * ldws);
        SENSEI_TRY(launch_row_broadcast(r, c, 1, n, 1, rc, 1, SENSEI_ACT_NONE, s));
        SENSEI_TRY(launch_reciprocal(c, n, inv_c, s));
        SENSEI_TRY(launch_stack_weights(W.ptr, W.ld, k_hops + 1, f_in, f_out, Wst, ldws, s));
        SENSEI_TRY(launch_to_slices(c, X.ptr, X.ld, n, f_in, G, s));
        for (int k = 1; k <= k_hops; ++k)
            SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, rc, nullptr, G + (k - 1) * hop, fp, fp, G + k * hop, fp, fp, SENSEI_ACT_NONE, plan, carry, s, kt,
                                false, nullptr, true, true));
        SENSEI_TRY(launch_gemm(G, 32, Wst, ldws, Y, ldy, n, (k_hops + 1) * fp, f_out, f_out, act, s, inv_c, gt, false, true));
        return SENSEI_OK;
    }
    // Horner form at width f_out: T_K = X W_K, T_k = X W_k + A^ T_{k+1}; T is kept as c (x) T_k, slice-major
    float *T = cv.take<float>((size_t)n * fp), *P = cv.take<float>((size_t)n * fp);
    auto w_block = [&](int k) { return W.ptr + (size_t)k * f_in * W.ld; };
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, w_block(k_hops), W.ld, T, fp, n, f_in, f_out, fp, SENSEI_ACT_NONE, s, c, gt, true));
    for (int k = k_hops - 1; k >= 0; --k) {
        SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, r, nullptr, T, fp, fp, P, fp, fp, SENSEI_ACT_NONE, plan, carry, s, kt, false, nullptr, true, true));
        if (k > 0) SENSEI_TRY(launch_gemm(X.ptr, X.ld, w_block(k), W.ld, T, fp, n, f_in, f_out, fp, SENSEI_ACT_NONE, s, c, gt, true, false, P));
        else SENSEI_TRY(launch_gemm(X.ptr, X.ld, w_block(0), W.ld, Y, ldy, n, f_in, f_out, f_out, act, s, nullptr, gt, false, false, P));
    }
    return SENSEI_OK;
}

// ---- backward of the GCN layer
size_t gcn_bwd_ws(const sensei_csr &A, int f_in, int f_out, int id, int k_hops = 1) {
    const int64_t nnz = A.nnz;
    size_t b = 2 * plan_bytes(nnz) + 256;
    if (k_hops > 1) {  // K-hop layer: a second slice-major hop buffer per chain of hops, and the merged scaling r (.) c
        b += align_up((size_t)A.n_rows * sizeof(float), 256);
        b += (id == SENSEI_GCN_BWD_AGG ? 1 : 3) * align_up((size_t)A.n_cols * pad32(id == SENSEI_GCN_BWD_AGG ? f_out : f_in) * sizeof(float), 256);
    }
    b += align_up((size_t)pad4(f_in) * pad4(f_out) * sizeof(float), 256);                             // W^T
    if (id == SENSEI_GCN_BWD_AGG) {
        b += spmm_carry_bytes(nnz, pad32(f_out));
        b += align_up((size_t)A.n_rows * pad32(f_out) * sizeof(float), 256);                          // r (x) dP
        b += align_up((size_t)A.n_cols * pad4(f_out) * sizeof(float), 256);                           // G
        b += gemm_tn_bytes(A.n_cols, f_in, f_out);
    } else {
        b += spmm_carry_bytes(nnz, pad32(f_in));
        b += align_up((size_t)A.n_rows * pad4(f_out) * sizeof(float), 256);                           // dP
        b += align_up((size_t)A.n_cols * pad32(f_in) * sizeof(float), 256);                           // c (x) X
        b += align_up((size_t)A.n_rows * pad4(f_in) * sizeof(float), 256);                            // U
        b += align_up((size_t)A.n_rows * pad32(f_in) * sizeof(float), 256);                           // r (x) dP.W^T
        b += gemm_tn_bytes(A.n_rows, f_in, f_out);
    }
    return b;
}

int run_gcn_backward(const sensei_csr &A, const sensei_csr &At, const float *r, const float *c, const sensei_mat &X, const sensei_mat &W,
                     const float *Y, int64_t ldy, const sensei_mat &dY, int act, const float *U_saved, int64_t ldu, float *dX, int64_t lddx,
                     float *dW, int64_t lddw, int id, void *ws, size_t ws_bytes, hipStream_t s, int k_hops = 1) {
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    const float *mask = (act == SENSEI_ACT_RELU) ? Y : nullptr;
    Carver cv(ws, ws_bytes);
    ChunkPlan plan_t = make_plan(At, cv);
    SENSEI_TRY(launch_chunk_rows(At, plan_t, s));
    // K-hop layer (square pattern): every chain of hops keeps its intermediate results slice-major, one buffer written while the
    // other is gathered from, with the adjacent scalings of two hops merged into r (.) c, as in the forward
    float *rc = nullptr;
    if (k_hops > 1) {
        rc = cv.take<float>((size_t)A.n_rows);
        SENSEI_TRY(launch_row_broadcast(r, c, 1, A.n_rows, 1, rc, 1, SENSEI_ACT_NONE, s));
    }
    if (id == SENSEI_GCN_BWD_AGG) {
        const int fo4 = pad4(f_out);
        float *carry = cv.take<float>(spmm_carry_bytes(At.nnz, pad32(f_out)) / sizeof(float));
        float *T = cv.take<float>((size_t)A.n_rows * pad32(f_out));
        float *G = cv.take<float>((size_t)A.n_cols * fo4);
        double *part = cv.take<double>(gemm_tn_bytes(A.n_cols, f_in, f_out) / sizeof(double));
        // T = r (x) (dY (.) mask), slice-major when the transposed SpMM gathers each row often enough (always between hops)
        const bool sliced = relayout_pays(At) || k_hops > 1;
        if (sliced) SENSEI_TRY(launch_to_slices(r, dY.ptr, dY.ld, A.n_rows, f_out, T, s, mask, ldy));
        else SENSEI_TRY(launch_row_broadcast(r, dY.ptr, dY.ld, A.n_rows, f_out, T, fo4, SENSEI_ACT_NONE, s, mask, ldy));
        const float *last = T;
        if (k_hops > 1) {  // inner hops: T <- (r (.) c) (x) (A~^T T)
            float *T2 = cv.take<float>((size_t)A.n_cols * pad32(f_out));
            float *buf[2] = {T, T2};
            for (int k = 0; k + 1 < k_hops; ++k)
                SENSEI_TRY(spmm_any(At, SENSEI_SPMM_PATTERN, rc, nullptr, buf[k & 1], pad32(f_out), pad32(f_out), buf[(k + 1) & 1], pad32(f_out),
                                    pad32(f_out), SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false, nullptr, true, true));
            last = buf[(k_hops - 1) & 1];
        }
        // G = c (x) (A~^T T)
        SENSEI_TRY(spmm_any(At, SENSEI_SPMM_PATTERN, c, nullptr, last, fo4, f_out, G, fo4, f_out, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false,
                            nullptr, sliced));
        SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, G, fo4, A.n_cols, f_in, f_out, dW, lddw, part, s));
        if (dX) {
            float *Wt = cv.take<float>((size_t)f_out * pad4(f_in));
            SENSEI_TRY(launch_transpose(W.ptr, W.ld, f_in, f_out, Wt, pad4(f_in), s));
            SENSEI_TRY(launch_gemm(G, fo4, Wt, pad4(f_in), dX, lddx, A.n_cols, f_out, f_in, f_in, SENSEI_ACT_NONE, s));
        }
    } else {
        const int fo4 = pad4(f_out), fi4 = pad4(f_in), fi32 = pad32(f_in);
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fi32) / sizeof(float));
        float *dP = cv.take<float>((size_t)A.n_rows * fo4);
        double *part = cv.take<double>(gemm_tn_bytes(A.n_rows, f_in, f_out) / sizeof(double));
        SENSEI_TRY(launch_row_broadcast(nullptr, dY.ptr, dY.ld, A.n_rows, f_out, dP, fo4, SENSEI_ACT_NONE, s, mask, ldy));
        const float *U = U_saved;
        int64_t ld_u = ldu;
        if (!U) {  // recompute U = r (x) (A~ (c (x) X)), the aggregate-first half of the forward
            ChunkPlan plan = make_plan(A, cv);
            SENSEI_TRY(launch_chunk_rows(A, plan, s));
            float *T = cv.take<float>((size_t)A.n_cols * fi32);
            float *Uw = cv.take<float>((size_t)A.n_rows * fi4);
            const bool sliced = relayout_pays(A) || k_hops > 1;
            if (sliced) SENSEI_TRY(launch_to_slices(c, X.ptr, X.ld, A.n_cols, f_in, T, s));
            else SENSEI_TRY(launch_row_broadcast(c, X.ptr, X.ld, A.n_cols, f_in, T, fi4, SENSEI_ACT_NONE, s));
            const float *last = T;
            if (k_hops > 1) {  // the inner hops of the forward: T <- (r (.) c) (x) (A~ T)
                float *T2 = cv.take<float>((size_t)A.n_cols * fi32);
                float *buf[2] = {T, T2};
                for (int k = 0; k + 1 < k_hops; ++k)
                    SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, rc, nullptr, buf[k & 1], fi32, fi32, buf[(k + 1) & 1], fi32, fi32, SENSEI_ACT_NONE, plan,
                                        carry, s, nullptr, false, nullptr, true, true));
                last = buf[(k_hops - 1) & 1];
            }
            SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, r, nullptr, last, fi4, f_in, Uw, fi4, f_in, SENSEI_ACT_NONE, plan, carry, s, nullptr, false,
                                nullptr, sliced));
            U = Uw;
            ld_u = fi4;
        }
        SENSEI_TRY(launch_gemm_tn(U, ld_u, dP, fo4, A.n_rows, f_in, f_out, dW, lddw, part, s));
        if (dX) {
            float *Wt = cv.take<float>((size_t)f_out * fi4);
            float *V = cv.take<float>((size_t)A.n_rows * fi32);
            SENSEI_TRY(launch_transpose(W.ptr, W.ld, f_in, f_out, Wt, fi4, s));
            // V = r (x) (dP W^T), written slice-major by the GEMM epilogue; dX = c (x) (A~^T V)
            const bool sliced = relayout_pays(At) || k_hops > 1;
            SENSEI_TRY(launch_gemm(dP, fo4, Wt, fi4, V, sliced ? fi32 : fi4, A.n_rows, f_out, f_in, sliced ? fi32 : f_in, SENSEI_ACT_NONE, s, r,
                                   nullptr, sliced));
            const float *last = V;
            if (k_hops > 1) {  // inner hops of the transposed chain
                float *V2 = cv.take<float>((size_t)A.n_cols * fi32);
                float *buf[2] = {V, V2};
                for (int k = 0; k + 1 < k_hops; ++k)
                    SENSEI_TRY(spmm_any(At, SENSEI_SPMM_PATTERN, rc, nullptr, buf[k & 1], fi32, fi32, buf[(k + 1) & 1], fi32, fi32, SENSEI_ACT_NONE, plan_t,
                                        carry, s, nullptr, false, nullptr, true, true));
                last = buf[(k_hops - 1) & 1];
            }
            SENSEI_TRY(spmm_any(At, SENSEI_SPMM_PATTERN, c, nullptr, last, fi4, f_in, dX, lddx, f_in, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false,
                                nullptr, sliced));
        }
    }
    return SENSEI_OK;
}

// ---- backward of the TAGCN layer Y = act(sum_k A^^k X W_k): with dP = dY (.) [Y > 0],
//   dW_k = (A^^k X)^T dP = X^T (A^^T)^k dP   and   dX = sum_k (A^^T)^k dP W_k^T.
// The two forms of dW_k are the two associations: bwd_id AGG carries the gradient through the hops at width f_out (Q_k = (A^^T)^k dP,
// K transposed propagations, dW_k = X^T Q_k, dX = [Q_0 .. Q_K] [W_0^T; ..; W_K^T] as one GEMM); bwd_id UPD carries the input forward at
// width f_in (H_k = A^^k X, K propagations, dW_k = H_k^T dP) and dX back in Horner form, R_K = dP W_K^T, R_k = dP W_k^T + A^^T R_(k+1).
// Between hops the operand stays slice-major with the scaling of the next gather already applied; the row-major copy of every hop's
// result is what the weight gradient reads.
size_t tagcn_bwd_ws(const sensei_csr &A, int f_in, int f_out, int k_hops, int id) {
    const int fo4 = pad4(f_out), fi4 = pad4(f_in);
    const size_t n = (size_t)A.n_rows;
    size_t b = 2 * plan_bytes(A.nnz) + 512;
    if (id == SENSEI_GCN_BWD_AGG) {
        b += spmm_carry_bytes(A.nnz, pad32(f_out));
        b += align_up(n * (size_t)(k_hops + 1) * fo4 * sizeof(float), 256);          // Q_0 .. Q_K side by side, row-major
        b += align_up(n * pad32(f_out) * sizeof(float), 256);                        // r (x) Q_k, slice-major
        b += align_up((size_t)(k_hops + 1) * fo4 * fi4 * sizeof(float), 256);        // W_k^T stacked
        b += gemm_tn_bytes(A.n_rows, f_in, f_out);
    } else {
        b += spmm_carry_bytes(A.nnz, pad32(f_in));
        b += align_up(n * fo4 * sizeof(float), 256);                                 // dP
        b += align_up(n * fi4 * sizeof(float), 256);                                 // H_k, row-major
        b += 2 * align_up(n * pad32(f_in) * sizeof(float), 256);                     // slice-major operand of a hop and its result
        b += align_up((size_t)(k_hops + 1) * fo4 * fi4 * sizeof(float), 256);        // W_k^T, block after block
        b += gemm_tn_bytes(A.n_rows, f_in, f_out);
    }
    return b;
}

int run_tagcn_backward(const sensei_csr &A, const sensei_csr &At, const float *r, const float *c, const sensei_mat &X, const sensei_mat &W,
                       int k_hops, const float *Y, int64_t ldy, const sensei_mat &dY, int act, float *dX, int64_t lddx, float *dW, int64_t lddw,
                       int id, void *ws, size_t ws_bytes, hipStream_t s) {
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    const int fo4 = pad4(f_out), fi4 = pad4(f_in), fo32 = pad32(f_out), fi32 = pad32(f_in);
    const int64_t n = A.n_rows;
    const float *mask = (act == SENSEI_ACT_RELU) ? Y : nullptr;
    Carver cv(ws, ws_bytes);
    ChunkPlan plan_t = make_plan(At, cv);
    SENSEI_TRY(launch_chunk_rows(At, plan_t, s));
    auto w_block = [&](int k) { return W.ptr + (size_t)k * f_in * W.ld; };
    auto dw_block = [&](int k) { return dW + (size_t)k * f_in * lddw; };
    if (id == SENSEI_GCN_BWD_AGG) {
        const int64_t ldq = (int64_t)(k_hops + 1) * fo4;
        float *carry = cv.take<float>(spmm_carry_bytes(At.nnz, fo32) / sizeof(float));
        float *Q = cv.take<float>((size_t)n * ldq);
        float *S = cv.take<float>((size_t)n * fo32);
        float *Wst = cv.take<float>((size_t)ldq * fi4);
        double *part = cv.take<double>(gemm_tn_bytes(n, f_in, f_out) / sizeof(double));
        if (fo4 != f_out) SENSEI_TRY(launch_zero_matrix(Q, n, (int)ldq, ldq, false, s));   // the pad columns enter the GEMM below
        SENSEI_TRY(launch_row_broadcast(nullptr, dY.ptr, dY.ld, n, f_out, Q, ldq, SENSEI_ACT_NONE, s, mask, ldy));
        for (int k = 1; k <= k_hops; ++k) {   // Q_k = c (x) (A~^T (r (x) Q_(k-1)))
            SENSEI_TRY(launch_to_slices(r, Q + (size_t)(k - 1) * fo4, ldq, n, f_out, S, s));
            SENSEI_TRY(spmm_any(At, SENSEI_SPMM_PATTERN, c, nullptr, S, fo32, f_out, Q + (size_t)k * fo4, ldq, f_out, SENSEI_ACT_NONE, plan_t, carry, s,
                                nullptr, false, nullptr, true));
        }
        for (int k = 0; k <= k_hops; ++k)
            SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, Q + (size_t)k * fo4, ldq, n, f_in, f_out, dw_block(k), lddw, part, s));
        if (dX) {
            SENSEI_TRY(launch_zero_matrix(Wst, ldq, fi4, fi4, false, s));
            for (int k = 0; k <= k_hops; ++k) SENSEI_TRY(launch_transpose(w_block(k), W.ld, f_in, f_out, Wst + (size_t)k * fo4 * fi4, fi4, s));
            SENSEI_TRY(launch_gemm(Q, ldq, Wst, fi4, dX, lddx, n, (int)ldq, f_in, f_in, SENSEI_ACT_NONE, s));
        }
        return SENSEI_OK;
    }
    ChunkPlan plan = make_plan(A, cv);
    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fi32) / sizeof(float));
    float *dP = cv.take<float>((size_t)n * fo4);
    float *H = cv.take<float>((size_t)n * fi4);
    float *T = cv.take<float>((size_t)n * fi32), *P = cv.take<float>((size_t)n * fi32);
    float *Wt = cv.take<float>((size_t)(k_hops + 1) * fo4 * fi4);
    double *part = cv.take<double>(gemm_tn_bytes(n, f_in, f_out) / sizeof(double));
    SENSEI_TRY(launch_row_broadcast(nullptr, dY.ptr, dY.ld, n, f_out, dP, fo4, SENSEI_ACT_NONE, s, mask, ldy));
    // weight gradients, hop after hop: H_k = r (x) (A~ (c (x) H_(k-1)))
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dP, fo4, n, f_in, f_out, dw_block(0), lddw, part, s));
    for (int k = 1; k <= k_hops; ++k) {
        SENSEI_TRY(launch_to_slices(c, k == 1 ? X.ptr : H, k == 1 ? X.ld : fi4, n, f_in, T, s));
        SENSEI_TRY(spmm_any(A, SENSEI_SPMM_PATTERN, r, nullptr, T, fi32, f_in, H, fi4, f_in, SENSEI_ACT_NONE, plan, carry, s, nullptr, false, nullptr,
                            true));
        SENSEI_TRY(launch_gemm_tn(H, fi4, dP, fo4, n, f_in, f_out, dw_block(k), lddw, part, s));
    }
    if (dX) {
        for (int k = 0; k <= k_hops; ++k) SENSEI_TRY(launch_transpose(w_block(k), W.ld, f_in, f_out, Wt + (size_t)k * fo4 * fi4, fi4, s));
        auto wt_block = [&](int k) { return Wt + (size_t)k * fo4 * fi4; };
        if (k_hops == 0) {
            SENSEI_TRY(launch_gemm(dP, fo4, wt_block(0), fi4, dX, lddx, n, f_out, f_in, f_in, SENSEI_ACT_NONE, s));
        } else {
            // T holds r (x) R_k, slice-major: what the transposed propagation gathers
            SENSEI_TRY(launch_gemm(dP, fo4, wt_block(k_hops), fi4, T, fi32, n, f_out, f_in, fi32, SENSEI_ACT_NONE, s, r, nullptr, true));
            for (int k = k_hops - 1; k >= 0; --k) {
                SENSEI_TRY(spmm_any(At, SENSEI_SPMM_PATTERN, c, nullptr, T, fi32, fi32, P, fi32, fi32, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false,
                                    nullptr, true, true));
                if (k > 0) SENSEI_TRY(launch_gemm(dP, fo4, wt_block(k), fi4, T, fi32, n, f_out, f_in, fi32, SENSEI_ACT_NONE, s, r, nullptr, true, false, P));
                else SENSEI_TRY(launch_gemm(dP, fo4, wt_block(0), fi4, dX, lddx, n, f_out, f_in, f_in, SENSEI_ACT_NONE, s, nullptr, nullptr, false, false, P));
            }
        }
    }
    return SENSEI_OK;
}

// n_heads > 1: W holds the heads side by side (head h = columns [h d, (h + 1) d), d = f_out / n_heads), a_l / a_r likewise,
// Y is their concatenation; Theta = X.W is formed by one GEMM for all heads, everything after it runs head by head on the
// head's columns (its own logits, statistics and aggregation), reusing the same buffers.
// How the attention part of a GAT layer call runs (sensei_gat_attention_path reports it):
//   tiles: statistics and aggregation split into dense tiles and remainder; panels: two passes, the logits stored in panel order;
//   one walk: score, running-maximum softmax and weighted sum fused in the aggregation kernel (no stored logits, no statistics
//   pass) - where the aggregation is one 32-column slice wide and rows average at least 16 entries, or two slices and 128
//   entries (measured, 32 / 64 columns, layer time against the two-pass form: 233,000-node power-law graph -19 % / -7 %,
//   98,000 nodes with 1,021 entries per row -26 % / -17 %, 2.45 M nodes with 52 per row -12 % / +6 %, road-shaped graph with 3
//   per row +6 % / +13 %: each further slice repeats the score work, and short rows pay the per-row merge);
//   two passes otherwise.
enum { kAttnTwoPass = SENSEI_GAT_PATH_TWO_PASS, kAttnOneWalk = SENSEI_GAT_PATH_ONE_WALK, kAttnTiles = SENSEI_GAT_PATH_TILES,
       kAttnPanels = SENSEI_GAT_PATH_PANELS };
int attention_path(const sensei_csr &A, int f_gather, bool operand_sliced) {
    if (operand_sliced && tiles_usable(A, kSpmmSoftmax, f_gather, true, true)) return kAttnTiles;
    if (panels_usable(A, f_gather)) return kAttnPanels;
    const double mean_row = A.n_rows > 0 ? (double)A.nnz / A.n_rows : 0.0;
    const int slices = pad32(f_gather) / 32;
    if ((slices == 1 && mean_row >= 16.0) || (slices == 2 && mean_row >= 128.0)) return kAttnOneWalk;
    return kAttnTwoPass;
}

int run_gat(const sensei_csr &A, const sensei_mat &X, const sensei_mat &W, const float *a_l, const float *a_r,
            float slope, float *Y, int64_t ldy, int act, int id, void *ws, size_t ws_bytes, hipStream_t s, Timers *tm, int n_heads = 1) {
    KernelTimer *kt = tm ? &tm->spmm : nullptr, *gt = tm ? &tm->gemm : nullptr;
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    const int fo = pad32(f_out), fi = pad4(f_in);
    const int d = f_out / n_heads;
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv);
    float2 *stats = cv.take<float2>((size_t)A.n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    float *s_l = cv.take<float>((size_t)A.n_cols);
    float *s_r = cv.take<float>((size_t)A.n_cols);
    float *logits = cv.take<float>((size_t)(A.nnz > 0 ? A.nnz : 1));
    float *v_l = cv.take<float>((size_t)fi);
    float *v_r = cv.take<float>((size_t)fi);
    float *theta = nullptr;
    if (id != SENSEI_GAT_RECOMP_FOLD) theta = cv.take<float>((size_t)A.n_cols * fo);

    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    const bool fold = (id == SENSEI_GAT_RECOMP_FOLD || id == SENSEI_GAT_REUSE_FOLD);
    const bool reuse = gat_is_reuse(id);
    // Theta is slice-major when the SpMM gathers from it (reuse) and a head's columns are whole 32-column slices; the
    // recompute id only projects it
    const bool theta_sliced = reuse && (n_heads == 1 || d % 32 == 0);
    if (theta) SENSEI_TRY(launch_gemm(X.ptr, X.ld, W.ptr, W.ld, theta, fo, A.n_cols, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, gt, theta_sliced));
    // recompute ids gather from X: slice-major copy once for all heads when its rows are gathered often enough
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, reuse ? fo : fi) / sizeof(float));
    float *U = nullptr;
    const float *x_src = X.ptr;
    bool x_sliced = false;
    if (!reuse) {
        U = cv.take<float>((size_t)A.n_rows * fi);
        x_sliced = relayout_pays(A);
        if (x_sliced) {
            float *T = cv.take<float>((size_t)A.n_cols * pad32(f_in));
            SENSEI_TRY(launch_to_slices(nullptr, X.ptr, X.ld, A.n_cols, f_in, T, s));
            x_src = T;
        }
    }
    const int f_gather = reuse ? (n_heads == 1 ? fo : d) : f_in;  // width of the aggregation of one head
    // dense-tile split (the gathered operand, Theta or X, must be slice-major): the tiles form their weights from s_l, s_r
    // themselves, only the remainder's logits are stored
    const int path = attention_path(A, f_gather, reuse ? theta_sliced : x_sliced);
    const bool by_tiles = path == kAttnTiles, by_panel = path == kAttnPanels, fused = path == kAttnOneWalk;
    for (int h = 0; h < n_heads; ++h) {
        const float *al = a_l + (size_t)h * d, *ar = a_r + (size_t)h * d;
        const float *theta_h = !theta ? nullptr : theta_sliced ? theta + (size_t)h * (d / 32) * (size_t)A.n_cols * 32 : theta + (size_t)h * d;
        if (!fold) {  // the two projections of the head's columns of Theta
            SENSEI_TRY(launch_gemv2(theta_h, fo, A.n_cols, d, al, ar, s_l, s_r, s, theta_sliced));
        } else {      // (X.W).a = X.(W.a)
            SENSEI_TRY(launch_gemv2(W.ptr + (size_t)h * d, W.ld, f_in, d, al, ar, v_l, v_r, s));
            SENSEI_TRY(launch_gemv2(X.ptr, X.ld, A.n_cols, f_in, v_l, v_r, s_l, s_r, s));
        }
        // One pass computes the logits and the per-row softmax statistics; the aggregation then weighs each neighbour
        // by exp(e - max) and scales the row by 1 / sum, so the attention weights themselves are never stored.  With a
        // panel copy the logits are written straight in panel order and the SpMM follows the panels.
        if (by_tiles) {
            // the entries inside kept tiles: (max, sum) per row and segment of tiles from the bit masks and the two vectors in rank
            // order, on the split's stream; the remainder: the ordinary pass over its CSR, which leaves its logits in its own order;
            // then the pairs of every row are merged
            const sensei_tiles &D = *A.tiles;
            SENSEI_TRY(hipEventRecord(D.ev_fork, s));
            SENSEI_TRY(hipStreamWaitEvent(D.side, D.ev_fork, 0));
            SENSEI_TRY(launch_tile_stats(D.T, s_l, s_r, slope, D.side));
            // the rows the tiles will multiply, in rank order: known since the GEMM, so gathered here, beside the remainder's pass; and
            // the tiles themselves, with the maximum over a row's tile entries as its shift (the join rescales their product to the
            // row's own maximum): the remainder's pass asks little of the matrix cores, so the two share the chip better than
            // the tiles and the aggregation of the remainder would (233,000-node power-law graph, 256 columns: layer 4.94 -> 4.78 ms)
            SENSEI_TRY(launch_tiles_gather(D.T, reuse ? theta_h : x_src, A.n_cols, pad32(f_gather), D.Bh, D.side));
            SENSEI_TRY(launch_dense_tiles(D.T, nullptr, A.n_cols, pad32(f_gather), D.Bh, D.side, s_l, s_r, nullptr, slope, false, true, true));
            SENSEI_TRY(hipEventRecord(D.ev_join, D.side));
            sensei_csr Ar = A;
            Ar.nnz = D.nnz_rem; Ar.row_ptr = D.row_ptr_rem; Ar.col_idx = D.col_rem; Ar.panels = nullptr; Ar.tiles = nullptr;
            // the aggregation reads the remainder's logits in the order it walks the remainder: panel-major where that copy is used
            SENSEI_TRY(launch_attention_stats(Ar, s_l, s_r, slope, logits, remainder_panels_usable(D, f_gather) ? D.pos_pm : nullptr, D.plan_rem, stats,
                                              carry_stats, s));
            SENSEI_TRY(hipStreamWaitEvent(s, D.ev_join, 0));
            SENSEI_TRY(launch_tile_stats_merge(D.T, stats, A.n_rows, s));
        } else if (!fused) {
            SENSEI_TRY(launch_attention_stats(A, s_l, s_r, slope, logits, by_panel ? A.panels->position : nullptr, plan, stats, carry_stats, s));
        }
        const AttnVectors attn = {s_l, s_r, slope, by_tiles, by_tiles};
        sensei_csr Aw = A;
        Aw.val = logits;
        float *Y_h = Y + (size_t)h * d;
        if (fused) {
            const AttnFusedArgs fa = {s_l, s_r, slope, stats, carry_stats};
            hipEvent_t t0 = kt ? kt->next() : nullptr, t1 = t0 ? kt->next() : nullptr;   // the whole call, fix-up included
            if (t1) SENSEI_TRY(hipEventRecord(t0, s));
            if (reuse) {
                SENSEI_TRY(launch_spmm(A, kSpmmAttnFused, nullptr, nullptr, theta_h, fo, f_gather, Y_h, ldy, d, act, plan, carry, s, nullptr, false, true,
                                       nullptr, theta_sliced, 1, false, false, &fa));
                if (t1) SENSEI_TRY(hipEventRecord(t1, s));
            } else {
                SENSEI_TRY(launch_spmm(A, kSpmmAttnFused, nullptr, nullptr, x_src, X.ld, f_in, U, fi, f_in, SENSEI_ACT_NONE, plan, carry, s, nullptr, false,
                                       true, nullptr, x_sliced, 1, false, false, &fa));
                if (t1) SENSEI_TRY(hipEventRecord(t1, s));
                SENSEI_TRY(launch_gemm(U, fi, W.ptr + (size_t)h * d, W.ld, Y_h, ldy, A.n_rows, f_in, d, d, act, s, nullptr, gt));
            }
        } else if (reuse) {
            SENSEI_TRY(spmm_any(Aw, kSpmmSoftmax, nullptr, nullptr, theta_h, fo, f_gather, Y_h, ldy, d, act, plan, carry, s, kt, by_panel, stats,
                                theta_sliced, false, by_tiles ? &attn : nullptr));
        } else {
            SENSEI_TRY(spmm_any(Aw, kSpmmSoftmax, nullptr, nullptr, x_src, X.ld, f_in, U, fi, f_in, SENSEI_ACT_NONE, plan, carry, s, kt, by_panel, stats,
                                x_sliced, false, by_tiles ? &attn : nullptr));
            SENSEI_TRY(launch_gemm(U, fi, W.ptr + (size_t)h * d, W.ld, Y_h, ldy, A.n_rows, f_in, d, d, act, s, nullptr, gt));
        }
    }
    return SENSEI_OK;
}

// ---- GATv2: e_ij = a . LeakyReLU(W_l x_i + W_r x_j), Y = act(sum_j alpha_ij W_r x_j)
size_t gatv2_ws(const sensei_csr &A, int f_in, int f_out, int id, bool shared) {
    const int fo = pad32(f_out), fi = pad4(f_in);
    size_t b = plan_bytes(A.nnz) + softmax_ws_bytes(A) + 512;
    b += align_up((size_t)(A.nnz > 0 ? A.nnz : 1) * sizeof(float), 256);       // logits, then the attention weights in place
    b += align_up((size_t)fo * sizeof(float), 256);                            // a, padded
    b += align_up((size_t)A.n_cols * fo * sizeof(float), 256);                 // Theta_r (slice-major)
    if (!shared) b += align_up((size_t)A.n_rows * fo * sizeof(float), 256);    // Theta_l (slice-major)
    if (id == 0) {
        b += spmm_carry_bytes(A.nnz, fo);
    } else {
        b += spmm_carry_bytes(A.nnz, pad32(f_in));
        b += align_up((size_t)A.n_rows * fi * sizeof(float), 256);             // U = alpha.X
        b += align_up((size_t)A.n_cols * pad32(f_in) * sizeof(float), 256);    // slice-major copy of X
    }
    return b;
}

int run_gatv2(const sensei_csr &A, const sensei_mat &X, const sensei_mat &Wl, const sensei_mat &Wr, const float *att, float slope, float *Y,
              int64_t ldy, int act, int id, void *ws, size_t ws_bytes, hipStream_t s, Timers *tm) {
    KernelTimer *kt = tm ? &tm->spmm : nullptr, *gt = tm ? &tm->gemm : nullptr;
    const int f_in = (int)X.cols, f_out = (int)Wr.cols;
    const int fo = pad32(f_out), fi = pad4(f_in);
    const bool shared = (Wl.ptr == Wr.ptr && Wl.ld == Wr.ld);
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv);
    float2 *stats = cv.take<float2>((size_t)A.n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    float *logits = cv.take<float>((size_t)(A.nnz > 0 ? A.nnz : 1));
    float *att_pad = cv.take<float>((size_t)fo);
    float *theta_r = cv.take<float>((size_t)A.n_cols * fo);
    // the destinations are the first n_rows sources: with one shared weight matrix their projections are rows of Theta_r,
    // but a slice of Theta_r holds n_cols rows and a slice of Theta_l n_rows, so the slices coincide only on a square pattern
    float *theta_l = (shared && A.n_rows == A.n_cols) ? theta_r : cv.take<float>((size_t)A.n_rows * fo);
    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    SENSEI_TRY(launch_to_slices(nullptr, att, f_out, 1, f_out, att_pad, s));
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wr.ptr, Wr.ld, theta_r, fo, A.n_cols, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, gt, true));
    if (theta_l != theta_r)
        SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wl.ptr, Wl.ld, theta_l, fo, A.n_rows, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, gt, true));
    SENSEI_TRY(launch_score_v2(A, theta_l, theta_r, f_out, att_pad, slope, logits, plan, s));
    SENSEI_TRY(launch_softmax(A, logits, logits, plan, stats, carry_stats, s));
    sensei_csr Aw = A;
    Aw.val = logits;
    if (id == 0) {  // reuse: aggregate the projected features at width f_out
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fo) / sizeof(float));
        SENSEI_TRY(spmm_any(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, theta_r, fo, fo, Y, ldy, f_out, act, plan, carry, s, kt, false, nullptr, true));
    } else {        // recompute: aggregate the inputs at width f_in, then project once more
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, pad32(f_in)) / sizeof(float));
        float *U = cv.take<float>((size_t)A.n_rows * fi);
        const float *x_src = X.ptr;
        const bool x_sliced = relayout_pays(A);
        if (x_sliced) {
            float *T = cv.take<float>((size_t)A.n_cols * pad32(f_in));
            SENSEI_TRY(launch_to_slices(nullptr, X.ptr, X.ld, A.n_cols, f_in, T, s));
            x_src = T;
        }
        SENSEI_TRY(spmm_any(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, x_src, X.ld, f_in, U, fi, f_in, SENSEI_ACT_NONE, plan, carry, s, kt, false,
                            nullptr, x_sliced));
        SENSEI_TRY(launch_gemm(U, fi, Wr.ptr, Wr.ld, Y, ldy, A.n_rows, f_in, f_out, f_out, act, s, nullptr, gt));
    }
    return SENSEI_OK;
}

// ---- backward of the GATv2 layer.  With dP = dY (.) [Y > 0], U_ij = Theta_l[i] + Theta_r[j], e_ij = att . LeakyReLU(U_ij):
//   dalpha_ij = <dP_i, Theta_r[j]>,  de_ij = alpha_ij (dalpha_ij - sum_k alpha_ik dalpha_ik)          (as in the GAT backward, no outer LeakyReLU)
//   dTheta_l[i] = att (.) sum_j de_ij LeakyReLU'(U_ij)                                                 (row sums over the pattern)
//   dTheta_r[j] = sum_i alpha_ij dP_i + att (.) sum_i de_ij LeakyReLU'(U_ij)                           (row sums over the transposed pattern)
//   datt        = sum_i sum_j de_ij LeakyReLU(U_ij)
//   dW_l = X_dst^T dTheta_l,  dW_r = X^T dTheta_r,  dX = dTheta_r W_r^T + [dTheta_l W_l^T on the first n_rows rows]
// The three sums with a vector per entry are SpMM walks whose gathered row meets a vector of the output row (kSpmmSignSum / kSpmmLreluSum).
size_t gatv2_bwd_ws(const sensei_csr &A, int f_in, int f_out) {
    const size_t nz = (size_t)(A.nnz > 0 ? A.nnz : 1), fo = pad32(f_out), fo4 = pad4(f_out), fi4 = pad4(f_in);
    const int t = choose_chunk_nnz(A.nnz);
    const size_t n_chunks = A.nnz <= 0 ? 1 : (size_t)((A.nnz + t - 1) / t);
    size_t b = 2 * plan_bytes(A.nnz) + softmax_ws_bytes(A) + 1024;
    b += 2 * align_up(nz * sizeof(float), 256) + align_up(nz * sizeof(float2), 256);   // logits, dalpha / de, (alpha, de) transposed
    b += align_up((size_t)(A.n_rows + 1) * sizeof(float), 256) + align_up(n_chunks * sizeof(float), 256);   // row dots and their carry
    b += 2 * align_up(fo * sizeof(float), 256);                                        // att padded, a scratch vector
    b += align_up((size_t)A.n_cols * fo * sizeof(float), 256);                         // Theta_r (slice-major)
    b += 3 * align_up((size_t)A.n_rows * fo * sizeof(float), 256);                     // Theta_l, dP, the LeakyReLU sums (slice-major)
    b += align_up((size_t)A.n_cols * 2 * fo4 * sizeof(float), 256);                    // [dTheta_r | dTheta_l]
    b += align_up((size_t)A.n_cols * fo4 * sizeof(float), 256);                        // the sign sums over the transposed pattern
    b += align_up((size_t)A.n_rows * sizeof(float), 256);                              // ones
    b += spmm_carry_bytes(A.nnz, (int)fo);
    b += align_up(2 * fo4 * fi4 * sizeof(float), 256);                                 // [W_r^T; W_l^T]
    b += gemm_tn_bytes(A.n_cols, f_in, f_out) + theta_t_vec_bytes(A.n_rows, f_out);
    return b;
}

int run_gatv2_backward(const sensei_csr &A_in, const sensei_csr &At_in, const int32_t *t_pos, const sensei_mat &X, const sensei_mat &Wl,
                       const sensei_mat &Wr, const float *att, float slope, const float *Y, int64_t ldy, const sensei_mat &dY, int act, float *dX,
                       int64_t lddx, float *dWl, int64_t lddwl, float *dWr, int64_t lddwr, float *datt, void *ws, size_t ws_bytes, hipStream_t s) {
    sensei_csr A = A_in, At = At_in;   // plain walks: no column panels, no tile split
    A.panels = nullptr; A.tiles = nullptr; At.panels = nullptr; At.tiles = nullptr;
    const int f_in = (int)X.cols, f_out = (int)Wr.cols;
    const int fo = pad32(f_out), fo4 = pad4(f_out), fi4 = pad4(f_in);
    const int64_t ldd = 2 * (int64_t)fo4;
    const size_t nz = (size_t)(A.nnz > 0 ? A.nnz : 1);
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv), plan_t = make_plan(At, cv);
    float2 *stats = cv.take<float2>((size_t)A.n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    float *logits = cv.take<float>(nz);
    float *de = cv.take<float>(nz);
    float2 *ade_t = cv.take<float2>(nz);            // (alpha, de) in the order of the transposed pattern
    float *rowdot = cv.take<float>((size_t)A.n_rows + 1);
    float *sum_carry = cv.take<float>((size_t)plan.n_chunks);
    float *att_pad = cv.take<float>((size_t)fo);
    float *vec_scratch = cv.take<float>((size_t)fo);
    float *theta_r = cv.take<float>((size_t)A.n_cols * fo);
    float *theta_l = cv.take<float>((size_t)A.n_rows * fo);
    float *dPs = cv.take<float>((size_t)A.n_rows * fo);
    float *Rs = cv.take<float>((size_t)A.n_rows * fo);
    float *Dcat = cv.take<float>((size_t)A.n_cols * ldd);
    float *GR = cv.take<float>((size_t)A.n_cols * fo4);
    float *ones = cv.take<float>((size_t)A.n_rows);
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fo) / sizeof(float));
    float *Wcat = cv.take<float>((size_t)ldd * fi4);
    double *part = cv.take<double>(gemm_tn_bytes(A.n_cols, f_in, f_out) / sizeof(double));
    double *part_a = cv.take<double>(theta_t_vec_bytes(A.n_rows, f_out) / sizeof(double));
    float *dThR = Dcat, *dThL = Dcat + fo4;

    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    SENSEI_TRY(launch_chunk_rows(At, plan_t, s));
    // forward quantities: both projections (slice-major), the logits and the row statistics
    SENSEI_TRY(launch_to_slices(nullptr, att, f_out, 1, f_out, att_pad, s));
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wr.ptr, Wr.ld, theta_r, fo, A.n_cols, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, nullptr, true));
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wl.ptr, Wl.ld, theta_l, fo, A.n_rows, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, nullptr, true));
    SENSEI_TRY(launch_score_v2(A, theta_l, theta_r, f_out, att_pad, slope, logits, plan, s));
    SENSEI_TRY(launch_softmax(A, logits, de, plan, stats, carry_stats, s));   // the weights it writes are not kept: de is overwritten below
    SENSEI_TRY(launch_to_slices(nullptr, dY.ptr, dY.ld, A.n_rows, f_out, dPs, s, act == SENSEI_ACT_RELU ? Y : nullptr, ldy));
    // per stored entry: dalpha and its weighted row sums, then the softmax backward; alpha and de also in transposed order
    SENSEI_TRY(launch_gat_dalpha(A, theta_r, dPs, f_out, logits, stats, de, rowdot, plan, sum_carry, s));
    SENSEI_TRY(launch_gat_dt(A, logits, de, rowdot, stats, t_pos, 1.f, de, ade_t, plan, s));
    // [dTheta_r | dTheta_l], zero where nothing is written (pad columns; the rows of dTheta_l past the destinations)
    SENSEI_TRY(launch_zero_matrix(Dcat, A.n_cols, (int)ldd, ldd, false, s));
    SENSEI_TRY(launch_zero_matrix(Wcat, ldd, fi4, fi4, false, s));
    sensei_csr Aw = At;
    Aw.val = reinterpret_cast<const float *>(ade_t);
    SENSEI_TRY(launch_spmm(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, dPs, fo, f_out, dThR, ldd, f_out, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false,
                           true, nullptr, true, 2));
    SelfSumArgs self_l = {theta_l, slope}, self_r = {theta_r, slope};
    sensei_csr Ae = A;
    Ae.val = de;
    SENSEI_TRY(launch_spmm(Ae, kSpmmSignSum, nullptr, nullptr, theta_r, fo, f_out, dThL, ldd, f_out, SENSEI_ACT_NONE, plan, carry, s, nullptr, false, true,
                           nullptr, true, 1, false, false, nullptr, &self_l));
    SENSEI_TRY(launch_spmm(Ae, kSpmmLreluSum, nullptr, nullptr, theta_r, fo, fo, Rs, fo, fo, SENSEI_ACT_NONE, plan, carry, s, nullptr, false, true, nullptr,
                           true, 1, true, false, nullptr, &self_l));
    Aw.val = reinterpret_cast<const float *>(ade_t) + 1;
    SENSEI_TRY(launch_spmm(Aw, kSpmmSignSum, nullptr, nullptr, theta_l, fo, f_out, GR, fo4, f_out, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false, true,
                           nullptr, true, 2, false, false, nullptr, &self_r));
    SENSEI_TRY(launch_scale_cols(dThL, ldd, dThL, ldd, att, A.n_rows, f_out, false, s));
    SENSEI_TRY(launch_scale_cols(dThR, ldd, GR, fo4, att, A.n_cols, f_out, true, s));
    // datt: column sums of the LeakyReLU sums
    SENSEI_TRY(launch_fill_f32(ones, A.n_rows, 1.f, s));
    SENSEI_TRY(launch_theta_t_vec(Rs, A.n_rows, f_out, ones, A.n_rows, ones, datt, vec_scratch, part_a, s));
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dThL, ldd, A.n_rows, f_in, f_out, dWl, lddwl, part, s));
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dThR, ldd, A.n_cols, f_in, f_out, dWr, lddwr, part, s));
    if (dX) {
        SENSEI_TRY(launch_transpose(Wr.ptr, Wr.ld, f_in, f_out, Wcat, fi4, s));
        SENSEI_TRY(launch_transpose(Wl.ptr, Wl.ld, f_in, f_out, Wcat + (size_t)fo4 * fi4, fi4, s));
        SENSEI_TRY(launch_gemm(Dcat, ldd, Wcat, fi4, dX, lddx, A.n_cols, (int)ldd, f_in, f_in, SENSEI_ACT_NONE, s));
    }
    return SENSEI_OK;
}

// ---- key-query attention (the score function of GaAN-style layers): e_ij = scale <W_q x_i, W_k x_j>, Y = act(sum_j alpha_ij W_v x_j)
size_t dotgat_ws(const sensei_csr &A, int f_in, int d_k, int f_out, int id) {
    const int dk = pad32(d_k), fo = pad32(f_out), fi = pad4(f_in);
    size_t b = plan_bytes(A.nnz) + softmax_ws_bytes(A) + 512;
    b += align_up((size_t)(A.nnz > 0 ? A.nnz : 1) * sizeof(float), 256);       // logits, then the attention weights in place
    b += align_up((size_t)A.n_rows * dk * sizeof(float), 256);                 // queries (slice-major)
    b += align_up((size_t)A.n_cols * dk * sizeof(float), 256);                 // keys (slice-major)
    if (id == 0) {
        b += align_up((size_t)A.n_cols * fo * sizeof(float), 256);             // values (slice-major)
        b += spmm_carry_bytes(A.nnz, fo);
    } else {
        b += spmm_carry_bytes(A.nnz, pad32(f_in));
        b += align_up((size_t)A.n_rows * fi * sizeof(float), 256);             // U = alpha.X
        b += align_up((size_t)A.n_cols * pad32(f_in) * sizeof(float), 256);    // slice-major copy of X
    }
    return b;
}

int run_dotgat(const sensei_csr &A, const sensei_mat &X, const sensei_mat &Wq, const sensei_mat &Wk, const sensei_mat &Wv, float scale, float *Y,
               int64_t ldy, int act, int id, void *ws, size_t ws_bytes, hipStream_t s, Timers *tm) {
    KernelTimer *kt = tm ? &tm->spmm : nullptr, *gt = tm ? &tm->gemm : nullptr;
    const int f_in = (int)X.cols, d_k = (int)Wq.cols, f_out = (int)Wv.cols;
    const int dk = pad32(d_k), fo = pad32(f_out), fi = pad4(f_in);
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv);
    float2 *stats = cv.take<float2>((size_t)A.n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    float *logits = cv.take<float>((size_t)(A.nnz > 0 ? A.nnz : 1));
    float *Q = cv.take<float>((size_t)A.n_rows * dk);
    float *K = cv.take<float>((size_t)A.n_cols * dk);
    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    // both projections slice-major with zero pad columns, the layout the per-entry dot product walks (one launch per 32-column slice)
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wq.ptr, Wq.ld, Q, dk, A.n_rows, f_in, d_k, dk, SENSEI_ACT_NONE, s, nullptr, gt, true));
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wk.ptr, Wk.ld, K, dk, A.n_cols, f_in, d_k, dk, SENSEI_ACT_NONE, s, nullptr, gt, true));
    SENSEI_TRY(launch_gat_dalpha(A, K, Q, d_k, nullptr, nullptr, logits, nullptr, plan, nullptr, s, scale));
    SENSEI_TRY(launch_softmax(A, logits, logits, plan, stats, carry_stats, s));
    sensei_csr Aw = A;
    Aw.val = logits;
    if (id == 0) {  // reuse: aggregate the value projections at width f_out
        float *V = cv.take<float>((size_t)A.n_cols * fo);
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fo) / sizeof(float));
        SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wv.ptr, Wv.ld, V, fo, A.n_cols, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, gt, true));
        SENSEI_TRY(spmm_any(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, V, fo, fo, Y, ldy, f_out, act, plan, carry, s, kt, false, nullptr, true));
    } else {        // recompute: aggregate the inputs at width f_in, then project
        float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, pad32(f_in)) / sizeof(float));
        float *U = cv.take<float>((size_t)A.n_rows * fi);
        const float *x_src = X.ptr;
        const bool x_sliced = relayout_pays(A);
        if (x_sliced) {
            float *T = cv.take<float>((size_t)A.n_cols * pad32(f_in));
            SENSEI_TRY(launch_to_slices(nullptr, X.ptr, X.ld, A.n_cols, f_in, T, s));
            x_src = T;
        }
        SENSEI_TRY(spmm_any(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, x_src, X.ld, f_in, U, fi, f_in, SENSEI_ACT_NONE, plan, carry, s, kt, false,
                            nullptr, x_sliced));
        SENSEI_TRY(launch_gemm(U, fi, Wv.ptr, Wv.ld, Y, ldy, A.n_rows, f_in, f_out, f_out, act, s, nullptr, gt));
    }
    return SENSEI_OK;
}

// ---- backward of the key-query attention layer.  With dP = dY (.) [Y > 0], e_ij = scale <Q_i, K_j>, alpha the row softmax of e:
//   dV_j = sum_i alpha_ij dP_i,  dalpha_ij = <dP_i, V_j>,  de_ij = alpha_ij (dalpha_ij - sum_k alpha_ik dalpha_ik),
//   dQ_i = scale sum_j de_ij K_j,  dK_j = scale sum_i de_ij Q_i,
//   dW_q = X_dst^T dQ,  dW_k = X^T dK,  dW_v = X^T dV,  dX = dK W_k^T + dV W_v^T + [dQ W_q^T on the first n_rows rows].
// Every step is a kernel the other layers already use: the per-entry dot products and the softmax backward of the GAT backward, weighted
// SpMMs over the pattern (dQ) and its transpose (dK, dV).
size_t dotgat_bwd_ws(const sensei_csr &A, int f_in, int d_k, int f_out) {
    const size_t nz = (size_t)(A.nnz > 0 ? A.nnz : 1), dk = pad32(d_k), fo = pad32(f_out), dk4 = pad4(d_k), fo4 = pad4(f_out), fi4 = pad4(f_in);
    const int t = choose_chunk_nnz(A.nnz);
    const size_t n_chunks = A.nnz <= 0 ? 1 : (size_t)((A.nnz + t - 1) / t);
    const size_t ldd = 2 * dk4 + fo4;
    size_t b = 2 * plan_bytes(A.nnz) + softmax_ws_bytes(A) + 1024;
    b += 2 * align_up(nz * sizeof(float), 256) + align_up(nz * sizeof(float2), 256);   // logits, dalpha / de, (alpha, de) transposed
    b += align_up((size_t)(A.n_rows + 1) * sizeof(float), 256) + align_up(n_chunks * sizeof(float), 256);   // row dots and their carry
    b += align_up((size_t)A.n_rows * dk * sizeof(float), 256) + align_up((size_t)A.n_cols * dk * sizeof(float), 256);   // Q, K (slice-major)
    b += align_up((size_t)A.n_cols * fo * sizeof(float), 256) + align_up((size_t)A.n_rows * fo * sizeof(float), 256);   // V, dP (slice-major)
    b += align_up((size_t)A.n_cols * ldd * sizeof(float), 256);                        // [dK | dV | dQ]
    b += align_up(dk * sizeof(float), 256);                                            // the scale, once per column
    b += spmm_carry_bytes(A.nnz, (int)(fo > dk ? fo : dk));
    b += align_up(ldd * fi4 * sizeof(float), 256);                                     // [W_k^T; W_v^T; W_q^T]
    b += gemm_tn_bytes(A.n_cols, f_in, f_out > d_k ? f_out : d_k);
    return b;
}

int run_dotgat_backward(const sensei_csr &A_in, const sensei_csr &At_in, const int32_t *t_pos, const sensei_mat &X, const sensei_mat &Wq,
                        const sensei_mat &Wk, const sensei_mat &Wv, float scale, const float *Y, int64_t ldy, const sensei_mat &dY, int act,
                        float *dX, int64_t lddx, float *dWq, int64_t lddwq, float *dWk, int64_t lddwk, float *dWv, int64_t lddwv, void *ws,
                        size_t ws_bytes, hipStream_t s) {
    sensei_csr A = A_in, At = At_in;   // plain walks: no column panels, no tile split
    A.panels = nullptr; A.tiles = nullptr; At.panels = nullptr; At.tiles = nullptr;
    const int f_in = (int)X.cols, d_k = (int)Wq.cols, f_out = (int)Wv.cols;
    const int dk = pad32(d_k), fo = pad32(f_out), dk4 = pad4(d_k), fo4 = pad4(f_out), fi4 = pad4(f_in);
    const int64_t ldd = 2 * (int64_t)dk4 + fo4;
    const size_t nz = (size_t)(A.nnz > 0 ? A.nnz : 1);
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv), plan_t = make_plan(At, cv);
    float2 *stats = cv.take<float2>((size_t)A.n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    float *logits = cv.take<float>(nz);
    float *de = cv.take<float>(nz);
    float2 *ade_t = cv.take<float2>(nz);
    float *rowdot = cv.take<float>((size_t)A.n_rows + 1);
    float *sum_carry = cv.take<float>((size_t)plan.n_chunks);
    float *Q = cv.take<float>((size_t)A.n_rows * dk);
    float *K = cv.take<float>((size_t)A.n_cols * dk);
    float *V = cv.take<float>((size_t)A.n_cols * fo);
    float *dPs = cv.take<float>((size_t)A.n_rows * fo);
    float *Dcat = cv.take<float>((size_t)A.n_cols * ldd);
    float *scale_vec = cv.take<float>((size_t)dk);
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fo > dk ? fo : dk) / sizeof(float));
    float *Wcat = cv.take<float>((size_t)ldd * fi4);
    double *part = cv.take<double>(gemm_tn_bytes(A.n_cols, f_in, f_out > d_k ? f_out : d_k) / sizeof(double));
    float *dK = Dcat, *dV = Dcat + dk4, *dQ = Dcat + dk4 + fo4;

    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    SENSEI_TRY(launch_chunk_rows(At, plan_t, s));
    // forward quantities
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wq.ptr, Wq.ld, Q, dk, A.n_rows, f_in, d_k, dk, SENSEI_ACT_NONE, s, nullptr, nullptr, true));
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wk.ptr, Wk.ld, K, dk, A.n_cols, f_in, d_k, dk, SENSEI_ACT_NONE, s, nullptr, nullptr, true));
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, Wv.ptr, Wv.ld, V, fo, A.n_cols, f_in, f_out, fo, SENSEI_ACT_NONE, s, nullptr, nullptr, true));
    SENSEI_TRY(launch_gat_dalpha(A, K, Q, d_k, nullptr, nullptr, logits, nullptr, plan, nullptr, s, scale));
    SENSEI_TRY(launch_softmax(A, logits, de, plan, stats, carry_stats, s));   // the weights it writes are not kept: de is overwritten below
    SENSEI_TRY(launch_to_slices(nullptr, dY.ptr, dY.ld, A.n_rows, f_out, dPs, s, act == SENSEI_ACT_RELU ? Y : nullptr, ldy));
    // per stored entry: dalpha and its weighted row sums, then the softmax backward; alpha and de also in transposed order
    SENSEI_TRY(launch_gat_dalpha(A, V, dPs, f_out, logits, stats, de, rowdot, plan, sum_carry, s));
    SENSEI_TRY(launch_gat_dt(A, logits, de, rowdot, stats, t_pos, 1.f, de, ade_t, plan, s));
    SENSEI_TRY(launch_zero_matrix(Dcat, A.n_cols, (int)ldd, ldd, false, s));   // pad columns; the rows of dQ past the destinations
    SENSEI_TRY(launch_zero_matrix(Wcat, ldd, fi4, fi4, false, s));
    sensei_csr Aw = At;
    Aw.val = reinterpret_cast<const float *>(ade_t);
    SENSEI_TRY(launch_spmm(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, dPs, fo, f_out, dV, ldd, f_out, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false, true,
                           nullptr, true, 2));
    Aw.val = reinterpret_cast<const float *>(ade_t) + 1;
    SENSEI_TRY(launch_spmm(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, Q, dk, d_k, dK, ldd, d_k, SENSEI_ACT_NONE, plan_t, carry, s, nullptr, false, true,
                           nullptr, true, 2));
    sensei_csr Ae = A;
    Ae.val = de;
    SENSEI_TRY(launch_spmm(Ae, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, K, dk, d_k, dQ, ldd, d_k, SENSEI_ACT_NONE, plan, carry, s, nullptr, false, true,
                           nullptr, true, 1));
    SENSEI_TRY(launch_fill_f32(scale_vec, d_k, scale, s));
    SENSEI_TRY(launch_scale_cols(dK, ldd, dK, ldd, scale_vec, A.n_cols, d_k, false, s));
    SENSEI_TRY(launch_scale_cols(dQ, ldd, dQ, ldd, scale_vec, A.n_rows, d_k, false, s));
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dK, ldd, A.n_cols, f_in, d_k, dWk, lddwk, part, s));
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dV, ldd, A.n_cols, f_in, f_out, dWv, lddwv, part, s));
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dQ, ldd, A.n_rows, f_in, d_k, dWq, lddwq, part, s));
    if (dX) {
        SENSEI_TRY(launch_transpose(Wk.ptr, Wk.ld, f_in, d_k, Wcat, fi4, s));
        SENSEI_TRY(launch_transpose(Wv.ptr, Wv.ld, f_in, f_out, Wcat + (size_t)dk4 * fi4, fi4, s));
        SENSEI_TRY(launch_transpose(Wq.ptr, Wq.ld, f_in, d_k, Wcat + (size_t)(dk4 + fo4) * fi4, fi4, s));
        SENSEI_TRY(launch_gemm(Dcat, ldd, Wcat, fi4, dX, lddx, A.n_cols, (int)ldd, f_in, f_in, SENSEI_ACT_NONE, s));
    }
    return SENSEI_OK;
}

// ---- backward of the GAT layer
// The per-entry dot products of the attention backward can use the dense-tile split of A: same pattern, wide enough, and
// every tile cell addressable by the (negative) codes in dst_rem.  Below 128 columns the extra pass that merges the two
// sources costs more than the matrix cores save.
constexpr int kDalphaTilesMinWidth = 128;
bool tiles_serve_dalpha(const sensei_csr &A, int f_out) {
    const sensei_tiles *D = A.tiles;
    if (!D || D->T.n_slots <= 0 || D->T.n_slots > kMaxCellSlots || f_out < kDalphaTilesMinWidth) return false;
    return D->n_rows == A.n_rows && D->n_cols == A.n_cols && D->nnz == A.nnz && D->src_row_ptr == A.row_ptr && D->src_col_idx == A.col_idx;
}

// alpha^T . dP of the attention backward can use a dense-tile split of the transposed pattern: the coefficients of the entries inside
// kept tiles are formed on the fly from s_l, s_r and the row statistics, the others are copied into the order of the remainder.
bool tiles_serve_transposed(const sensei_csr &At, int f_out) {
    const sensei_tiles *D = At.tiles;
    if (!D || D->T.n_slots <= 0 || pad32(f_out) > D->max_width || f_out < D->min_width) return false;
    return D->n_rows == At.n_rows && D->n_cols == At.n_cols && D->nnz == At.nnz && D->src_row_ptr == At.row_ptr && D->src_col_idx == At.col_idx;
}

size_t gat_bwd_ws(const sensei_csr &A, const sensei_csr *At, int f_in, int f_out) {
    const size_t nz = (size_t)(A.nnz > 0 ? A.nnz : 1), fo32 = pad32(f_out), fo4 = pad4(f_out), fi4 = pad4(f_in);
    const int t = choose_chunk_nnz(A.nnz);
    const size_t n_chunks = A.nnz <= 0 ? 1 : (size_t)((A.nnz + t - 1) / t);
    size_t b = 2 * plan_bytes(A.nnz) + softmax_ws_bytes(A) + 512;
    b += 2 * align_up((size_t)A.n_cols * sizeof(float), 256);        // s_l, s_r
    b += align_up((size_t)A.n_cols * fo32 * sizeof(float), 256);     // Theta (slice-major)
    b += align_up((size_t)A.n_rows * fo32 * sizeof(float), 256);     // dP (slice-major)
    b += 4 * align_up(nz * sizeof(float), 256);                      // logits, dalpha / dt, alpha^T, dt^T
    b += align_up((size_t)(A.n_rows + 1) * sizeof(float), 256);      // row dots
    b += align_up(n_chunks * sizeof(float), 256);                    // carry of the row sums
    b += 2 * align_up((size_t)(A.n_cols + 1) * sizeof(float), 256);  // ds_l, ds_r
    b += align_up((size_t)A.n_cols * fo4 * sizeof(float), 256);      // dTheta
    b += spmm_carry_bytes(A.nnz, (int)fo32);
    b += align_up(fo4 * fi4 * sizeof(float), 256);                   // W^T
    b += gemm_tn_bytes(A.n_cols, f_in, f_out) + theta_t_vec_bytes(A.n_cols, f_out);
    if (tiles_serve_dalpha(A, f_out)) {  // dense-tile split: the tiles' dot products, the two operands in rank order, the remainder's dalpha
        const sensei_tiles &D = *A.tiles;
        b += align_up((size_t)D.T.n_slots * 128 * 128 * sizeof(float), 256);
        b += align_up((size_t)D.T.nt_r * 128 * fo32 * sizeof(float), 256) + align_up((size_t)D.T.nt_c * 128 * fo32 * sizeof(float), 256);
        b += align_up((size_t)(D.nnz_rem > 0 ? D.nnz_rem : 1) * sizeof(float), 256);
    }
    if (At && tiles_serve_transposed(*At, f_out)) b += align_up((size_t)(At->tiles->nnz_rem > 0 ? At->tiles->nnz_rem : 1) * sizeof(float), 256);
    return b;
}

int run_gat_backward(const sensei_csr &A, const sensei_csr &At, const int32_t *t_pos, const sensei_mat &X, const sensei_mat &W,
                     const float *a_l, const float *a_r, float slope, const float *Y, int64_t ldy, const sensei_mat &dY, int act, float *dX,
                     int64_t lddx, float *dW, int64_t lddw, float *da_l, float *da_r, void *ws, size_t ws_bytes, hipStream_t s,
                     float *dtheta_out = nullptr, int64_t ld_dtheta = 0) {
    // dtheta_out (one head of a multi-head layer): dTheta is left there (row-major, ld_dtheta) and the products with X and W, which the
    // caller forms once for all heads, are skipped
    const int f_in = (int)X.cols, f_out = (int)W.cols;
    const int fo32 = pad32(f_out), fo4 = pad4(f_out), fi4 = pad4(f_in);
    const size_t nz = (size_t)(A.nnz > 0 ? A.nnz : 1);
    Carver cv(ws, ws_bytes);
    ChunkPlan plan = make_plan(A, cv), plan_t = make_plan(At, cv);
    float2 *stats = cv.take<float2>((size_t)A.n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    float *s_l = cv.take<float>((size_t)A.n_cols);
    float *s_r = cv.take<float>((size_t)A.n_cols);
    float *theta = cv.take<float>((size_t)A.n_cols * fo32);
    float *T = cv.take<float>((size_t)A.n_rows * fo32);
    float *logits = cv.take<float>(nz);
    float *dt = cv.take<float>(nz);
    float2 *adt_t = cv.take<float2>(nz);  // (alpha, dt) in the order of the transposed pattern
    float *rowdot = cv.take<float>((size_t)A.n_rows + 1);
    float *sum_carry = cv.take<float>((size_t)plan.n_chunks);
    float *ds_l = cv.take<float>((size_t)A.n_cols + 1);
    float *ds_r = cv.take<float>((size_t)A.n_cols + 1);
    float *dTheta_own = cv.take<float>((size_t)A.n_cols * fo4);
    float *dTheta = dtheta_out ? dtheta_out : dTheta_own;
    const int64_t ldt = dtheta_out ? ld_dtheta : fo4;
    float *carry = cv.take<float>(spmm_carry_bytes(A.nnz, fo32) / sizeof(float));
    float *Wt = cv.take<float>((size_t)fo4 * fi4);
    double *part = cv.take<double>(gemm_tn_bytes(A.n_cols, f_in, f_out) / sizeof(double));
    double *part_a = cv.take<double>(theta_t_vec_bytes(A.n_cols, f_out) / sizeof(double));

    SENSEI_TRY(launch_chunk_rows(A, plan, s));
    SENSEI_TRY(launch_chunk_rows(At, plan_t, s));
    // forward quantities: Theta (slice-major: the edge kernel gathers its rows), projections, logits, row statistics
    SENSEI_TRY(launch_gemm(X.ptr, X.ld, W.ptr, W.ld, theta, fo32, A.n_cols, f_in, f_out, fo32, SENSEI_ACT_NONE, s, nullptr, nullptr, true));
    SENSEI_TRY(launch_gemv2(theta, fo32, A.n_cols, f_out, a_l, a_r, s_l, s_r, s, true));
    SENSEI_TRY(launch_attention_stats(A, s_l, s_r, slope, logits, nullptr, plan, stats, carry_stats, s));
    // dP = dY (.) [Y > 0], slice-major
    SENSEI_TRY(launch_to_slices(nullptr, dY.ptr, dY.ld, A.n_rows, f_out, T, s, act == SENSEI_ACT_RELU ? Y : nullptr, ldy));
    // per stored entry: dalpha, then softmax and LeakyReLU backward; alpha and dt also in transposed order
    // With a tile split on the transposed pattern, the tiles' share of alpha^T . dP needs only s_l, s_r, the row statistics and dP, all
    // known by now: it runs on that split's own stream beside the per-entry work below and is joined where dTheta is put together.
    const bool split_t = tiles_serve_transposed(At, f_out);
    auto fork_transposed_tiles = [&]() -> hipError_t {
        const sensei_tiles &D = *At.tiles;
        hipError_t e = hipEventRecord(D.ev_fork, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(D.side, D.ev_fork, 0);
        if (e == hipSuccess) e = launch_dense_tiles(D.T, T, At.n_cols, fo32, D.Bh, D.side, s_l, s_r, stats, slope, true);
        if (e == hipSuccess) e = hipEventRecord(D.ev_join, D.side);
        return e;
    };
    if (tiles_serve_dalpha(A, f_out)) {
        // entries inside kept tiles: one 128 x 128 x F product per tile on the matrix cores, on the split's own stream; the rest: the
        // slice-by-slice kernel over the remainder on this stream; then one pass puts both in the order of the pattern and forms the
        // row sums
        const sensei_tiles &D = *A.tiles;
        float *Dt = cv.take<float>((size_t)D.T.n_slots * 128 * 128);
        float *Lh = cv.take<float>((size_t)D.T.nt_r * 128 * fo32);
        float *Rh = cv.take<float>((size_t)D.T.nt_c * 128 * fo32);
        float *dalpha_rem = cv.take<float>((size_t)(D.nnz_rem > 0 ? D.nnz_rem : 1));
        SENSEI_TRY(hipEventRecord(D.ev_fork, s));
        SENSEI_TRY(hipStreamWaitEvent(D.side, D.ev_fork, 0));
        SENSEI_TRY(launch_tiles_sddmm(D.T, T, A.n_rows, theta, A.n_cols, fo32, Lh, Rh, Dt, D.side));
        SENSEI_TRY(hipEventRecord(D.ev_join, D.side));
        sensei_csr Ar = A;
        Ar.nnz = D.nnz_rem; Ar.row_ptr = D.row_ptr_rem; Ar.col_idx = D.col_rem; Ar.panels = nullptr; Ar.tiles = nullptr;
        SENSEI_TRY(launch_gat_dalpha(Ar, theta, T, f_out, nullptr, nullptr, dalpha_rem, nullptr, D.plan_rem, sum_carry, s));
        SENSEI_TRY(hipStreamWaitEvent(s, D.ev_join, 0));
        if (split_t) SENSEI_TRY(fork_transposed_tiles());  // the side stream goes on while this one merges
        SENSEI_TRY(launch_gat_dalpha_merge(A, D.dst_rem, dalpha_rem, Dt, logits, stats, dt, rowdot, plan, sum_carry, s));
    } else {
        if (split_t) SENSEI_TRY(fork_transposed_tiles());
        SENSEI_TRY(launch_gat_dalpha(A, theta, T, f_out, logits, stats, dt, rowdot, plan, sum_carry, s));
    }
    SENSEI_TRY(launch_gat_dt(A, logits, dt, rowdot, stats, t_pos, slope, dt, adt_t, plan, s));
    SENSEI_TRY(launch_row_sum(A, dt, 1, ds_l, plan, sum_carry, s));
    SENSEI_TRY(launch_row_sum(At, reinterpret_cast<const float *>(adt_t) + 1, 2, ds_r, plan_t, sum_carry, s));
    // dTheta = alpha^T.dP + ds_l a_l^T + ds_r a_r^T
    if (split_t) {
        // the remainder of the transposed pattern with its coefficients copied into its own order; the tiles' share was started above
        const sensei_tiles &D = *At.tiles;
        float *alpha_rem = cv.take<float>((size_t)(D.nnz_rem > 0 ? D.nnz_rem : 1));
        const bool pm = remainder_panels_usable(D, f_out);   // the panel-major copy of the remainder, as in the forward aggregation
        SENSEI_TRY(launch_compact_values(At.nnz, D.dst_rem, reinterpret_cast<const float *>(adt_t), 2, alpha_rem, s, pm ? D.pos_pm : nullptr));
        sensei_csr Ar = At;
        Ar.nnz = D.nnz_rem; Ar.row_ptr = D.row_ptr_rem; Ar.col_idx = D.col_rem; Ar.val = alpha_rem; Ar.panels = nullptr; Ar.tiles = nullptr;
        if (pm) {
            Ar.n_rows = D.rem_panels * At.n_rows; Ar.row_ptr = D.seg_ptr; Ar.col_idx = D.col_pm;
            SENSEI_TRY(launch_spmm(Ar, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, T, fo32, fo32, D.part_pm, 32, fo32, SENSEI_ACT_NONE, D.plan_pm, carry, s,
                                   nullptr, false, false, nullptr, true, 1, true, true));
            SENSEI_TRY(hipStreamWaitEvent(s, D.ev_join, 0));
            SENSEI_TRY(launch_tiles_combine_pm(D.T, dTheta, At.n_rows, f_out, ldt, false, fo32, nullptr, nullptr, SENSEI_ACT_NONE, s, D.part_pm,
                                               D.rem_panels, D.seg_ptr, D.plan_pm.chunk_nnz, carry, fo32));
        } else {
            SENSEI_TRY(launch_spmm(Ar, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, T, fo32, f_out, dTheta, ldt, f_out, SENSEI_ACT_NONE, D.plan_rem, carry, s,
                                   nullptr, false, false, nullptr, true, 1, false, true));
            SENSEI_TRY(hipStreamWaitEvent(s, D.ev_join, 0));
            SENSEI_TRY(launch_tiles_combine(D.T, dTheta, At.n_rows, f_out, ldt, false, fo32, nullptr, nullptr, SENSEI_ACT_NONE, s, D.row_ptr_rem,
                                            D.plan_rem.chunk_nnz, carry, fo32));
        }
    } else {
        sensei_csr Aw = At;
        Aw.val = reinterpret_cast<const float *>(adt_t);
        Aw.panels = nullptr;  // the values follow the order of At itself
        SENSEI_TRY(launch_spmm(Aw, SENSEI_SPMM_WEIGHTED, nullptr, nullptr, T, fo32, f_out, dTheta, ldt, f_out, SENSEI_ACT_NONE, plan_t, carry, s, nullptr,
                               false, true, nullptr, true, 2));
    }
    SENSEI_TRY(launch_rank1_add(dTheta, ldt, A.n_cols, f_out, ds_l, A.n_rows, ds_r, a_l, a_r, s));
    SENSEI_TRY(launch_theta_t_vec(theta, A.n_cols, f_out, ds_l, A.n_rows, ds_r, da_l, da_r, part_a, s));
    if (dtheta_out) return SENSEI_OK;
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dTheta, ldt, A.n_cols, f_in, f_out, dW, lddw, part, s));
    if (dX) {
        SENSEI_TRY(launch_transpose(W.ptr, W.ld, f_in, f_out, Wt, fi4, s));
        SENSEI_TRY(launch_gemm(dTheta, ldt, Wt, fi4, dX, lddx, A.n_cols, f_out, f_in, f_in, SENSEI_ACT_NONE, s));
    }
    return SENSEI_OK;
}

// Multi-head layer: the heads share only the input.  Every head runs the single-head backward on its columns and leaves its dTheta
// beside the others'; dW = X^T [dTheta_0 .. dTheta_(H-1)] and dX = [dTheta_0 ..] W^T are then one product each for all heads.
size_t gat_bwd_heads_ws(const sensei_csr &A, const sensei_csr *At, int f_in, int f_out, int n_heads) {
    const size_t fo4 = pad4(f_out), fi4 = pad4(f_in);
    return gat_bwd_ws(A, At, f_in, f_out / n_heads) + align_up((size_t)A.n_cols * fo4 * sizeof(float), 256) + align_up(fo4 * fi4 * sizeof(float), 256) +
           gemm_tn_bytes(A.n_cols, f_in, f_out) + 256;
}

int run_gat_backward_heads(const sensei_csr &A, const sensei_csr &At, const int32_t *t_pos, const sensei_mat &X, const sensei_mat &W,
                           const float *a_l, const float *a_r, int n_heads, float slope, const float *Y, int64_t ldy, const sensei_mat &dY, int act,
                           float *dX, int64_t lddx, float *dW, int64_t lddw, float *da_l, float *da_r, void *ws, size_t ws_bytes, hipStream_t s) {
    const int f_in = (int)X.cols, f_out = (int)W.cols, d = f_out / n_heads;
    const int fo4 = pad4(f_out), fi4 = pad4(f_in);
    Carver cv(ws, ws_bytes);
    float *dTh = cv.take<float>((size_t)A.n_cols * fo4);
    float *Wt = cv.take<float>((size_t)fo4 * fi4);
    double *part = cv.take<double>(gemm_tn_bytes(A.n_cols, f_in, f_out) / sizeof(double));
    void *ws_head = cv.base + cv.used;
    const size_t ws_head_bytes = ws_bytes - cv.used;
    for (int h = 0; h < n_heads; ++h) {
        sensei_mat W_h = W, dY_h = dY;
        W_h.ptr = W.ptr + (size_t)h * d; W_h.cols = d;
        dY_h.ptr = dY.ptr + (size_t)h * d; dY_h.cols = d;
        const int rc = run_gat_backward(A, At, t_pos, X, W_h, a_l + (size_t)h * d, a_r + (size_t)h * d, slope, Y ? Y + (size_t)h * d : nullptr, ldy,
                                        dY_h, act, nullptr, 0, nullptr, 0, da_l + (size_t)h * d, da_r + (size_t)h * d, ws_head, ws_head_bytes, s,
                                        dTh + (size_t)h * d, fo4);
        if (rc != SENSEI_OK) return rc;
    }
    SENSEI_TRY(launch_gemm_tn(X.ptr, X.ld, dTh, fo4, A.n_cols, f_in, f_out, dW, lddw, part, s));
    if (dX) {
        SENSEI_TRY(launch_transpose(W.ptr, W.ld, f_in, f_out, Wt, fi4, s));
        SENSEI_TRY(launch_gemm(dTh, fo4, Wt, fi4, dX, lddx, A.n_cols, f_out, f_in, f_in, SENSEI_ACT_NONE, s));
    }
    return SENSEI_OK;
}

// ------------------------------------------------------------------ cost model

struct Features {
    double n_rows, n_cols, nnz, density;
    double max_row = 0.0, sum_sq_row = 0.0;  // learned models only: largest row, sum of squared row lengths
    bool learned = false;                    // price SpMM and GEMM with the gradient-boosted trees
    double tile_share = 0.0;                 // share of the stored entries inside kept dense tiles (0: no split attached)
    int tile_min_width = 0, tile_max_width = 0;
};

// ---- learned per-primitive models (Section 3.5): gradient-boosted regression trees over graph features and sizes
struct GbtNode {
    int feat, left, right;  // feat < 0: leaf
    float thr, val;
};
#include "learned_model.inc"

template <size_t NR>
double gbt_predict(const GbtNode *nodes, const int (&roots)[NR], float base, const double *x) {
    double y = base;
    for (size_t t = 0; t < NR; ++t) {
        int k = roots[t];
        while (nodes[k].feat >= 0) k = x[nodes[k].feat] <= (double)nodes[k].thr ? nodes[k].left : nodes[k].right;
        y += nodes[k].val;
    }
    return y;
}

// seconds; the features and the unit of work mirror costmodel/train.py entry by entry
double t_spmm_learned(const Features &g, double f, int flavour) {
    const double nnz = std::fmax(g.nnz, 1.0), rows = std::fmax(g.n_rows, 1.0), cols = std::fmax(g.n_cols, 1.0), mean = nnz / rows;
    double x[12] = {std::log2(rows), std::log2(cols), std::log2(nnz), std::log2(mean), std::log2(nnz / (rows * cols)),
                    std::log2(std::fmax(f, 1.0)), std::log2(std::fmax(g.max_row, 1.0) / mean),
                    std::log2(std::fmax(g.sum_sq_row, 1.0) / rows / (mean * mean)), 0.0, 0.0, 0.0, 0.0};
    x[8 + flavour] = 1.0;  // pattern, weighted, scaled, softmax
    const double log_ms = gbt_predict(kSpmmNodes, kSpmmRoots, kSpmmBase, x) + std::log2(nnz * std::fmax(f, 1.0));
    return 1e-3 * std::exp2(log_ms);
}

double t_gemm_learned(double n, double k, double m) {
    n = std::fmax(n, 1.0); k = std::fmax(k, 1.0); m = std::fmax(m, 1.0);
    const double x[3] = {std::log2(n), std::log2(k), std::log2(m)};
    return 1e-3 * std::exp2(gbt_predict(kGemmNodes, kGemmRoots, kGemmBase, x) + std::log2(n * k * m));
}

double t_stream(const sensei_ctx &c, double bytes) { return c.launch_us * 1e-6 + bytes / c.stream_bps; }

double t_gemm_learned(double n, double k, double m);

double t_gemm(const sensei_ctx &c, double n, double k, double m, bool learned = false) {
    if (learned) return t_gemm_learned(n, k, m);
    const double flops = 2.0 * n * k * m, bytes = 4.0 * (n * k + k * m + n * m);
    // narrow outputs leave part of each MFMA tile idle
    const double rate = c.gemm_flops * (m >= 128 ? 1.0 : m >= 64 ? 0.8 : 0.5);
    return c.launch_us * 1e-6 + std::fmax(flops / rate, bytes / c.stream_bps);
}

enum { kSpmmPattern = 0, kSpmmWeighted = 1, kSpmmScaled = 2, kSpmmSoftmaxCost = 3 };

// SpMM.  The neighbour rows are gathered at a rate between the L2-resident and the far
// (memory-side cache / HBM) rate; the share served by the L2s falls with the size of one 128-byte
// feature slice of the gathered matrix (n_cols lines), fitted on the two R-MAT workloads.  The
// index stream is read once per feature tile; weights double it; gathering c[j] per non-zero
// (SCALED) costs about a third on top of the row gather.
double t_spmm_learned(const Features &g, double f, int flavour);

double t_spmm_unsplit(const sensei_ctx &c, const Features &g, double f, int flavour);

// What the call costs on the path it will take: a pattern that carries a usable dense-tile split runs its value-less and
// attention aggregations as tiles + remainder, which removes the tiles' share of the gathers but leaves the cold entries
// (measured on the 233,000-node power-law graph, 64 % of the entries in tiles: 0.57 of the unsplit call at 256 columns,
// 3.26 against 5.74 ms).  Weighted and scaled SpMMs do not take the split.
double t_spmm(const sensei_ctx &c, const Features &g, double f, int flavour) {
    const double t = t_spmm_unsplit(c, g, f, flavour);
    const bool takes_split = (flavour == kSpmmPattern || flavour == kSpmmSoftmaxCost) && g.tile_share > 0.0;
    const double need = flavour == kSpmmSoftmaxCost ? g.tile_min_width / 2.0 : g.tile_min_width;
    if (!takes_split || f < need || std::ceil(f / 32.0) * 32.0 > g.tile_max_width) return t;
    return t * (1.0 - 0.65 * g.tile_share);
}

double t_spmm_unsplit(const sensei_ctx &c, const Features &g, double f, int flavour) {
    if (g.learned) return t_spmm_learned(g, f, flavour);
    if (flavour == kSpmmSoftmaxCost) flavour = kSpmmWeighted;  // same streams: one value per entry
    const double tiles = std::ceil(f / 32.0);
    const double idx_bytes = g.nnz * (flavour == kSpmmWeighted ? 8.0 : 4.0) * tiles;
    const double out_bytes = 4.0 * f * g.n_rows;
    const double slice = std::fmax(g.n_cols * 128.0, 1.0);
    const double hit = std::fmin(0.9, 0.88 * std::pow(c.l2_slice_bytes / slice, 0.7));
    const double bw = 1.0 / (hit / c.gather_l2_bps + (1.0 - hit) / c.gather_far_bps);
    double gather = g.nnz * 4.0 * f / bw;
    if (flavour == kSpmmScaled) gather *= 1.33;
    const double compulsory = (4.0 * f * g.n_cols + out_bytes + idx_bytes) / c.stream_bps;
    return 3.0 * c.launch_us * 1e-6 + std::fmax(gather + idx_bytes / c.stream_bps, compulsory);
}

double gcn_cost(const sensei_ctx &c, const Features &g, int f_in, int f_out, int id) {
    const bool agg = gcn_is_agg(id);
    const double fs = agg ? f_in : f_out;
    const double gemm_rows = agg ? g.n_rows : g.n_cols;
    double t = c.launch_us * 1e-6 + t_gemm(c, gemm_rows, f_in, f_out, g.learned);
    Features gs = g;  // the split needs a slice-major operand: not DYN_UPD's row-major Z, not a user matrix that is gathered as it is
    if (id == SENSEI_GCN_DYN_UPD || (agg && g.nnz < 16.0 * g.n_cols)) gs.tile_share = 0.0;
    switch (id) {
        case SENSEI_GCN_DYN_AGG: case SENSEI_GCN_DYN_UPD:
            t += t_spmm(c, gs, fs, kSpmmPattern) + t_stream(c, 8.0 * g.n_cols * fs) + t_stream(c, 8.0 * g.n_rows * fs);
            break;
        case SENSEI_GCN_DYNF_AGG:
            t += t_spmm(c, g, fs, kSpmmScaled);
            if (g.nnz >= 16.0 * g.n_cols) t += t_stream(c, 8.0 * g.n_cols * fs);  // slice-major copy of X
            break;
        case SENSEI_GCN_DYNF_UPD:  // scalings live in the GEMM and SpMM epilogues
            t += t_spmm(c, gs, fs, kSpmmPattern);
            break;
        default:
            t += t_spmm(c, g, fs, kSpmmWeighted);
            if (agg && g.nnz >= 16.0 * g.n_cols) t += t_stream(c, 8.0 * g.n_cols * fs);
            break;
    }
    return t;
}

double gat_cost(const sensei_ctx &c, const Features &g, int f_in, int f_out, int id) {
    const bool fold = (id == SENSEI_GAT_RECOMP_FOLD || id == SENSEI_GAT_REUSE_FOLD);
    double t = c.launch_us * 1e-6;
    // attention: one pass over the pattern for the logits and the row statistics (the normalisation is part of the SpMM),
    // unless the aggregation is narrow enough, and the rows long enough, to run as one walk
    const double f_agg = gat_is_reuse(id) ? f_out : f_in, mean_row = g.n_rows > 0 ? g.nnz / g.n_rows : 0.0;
    const bool one_walk = g.tile_share <= 0.0 && ((f_agg <= 32 && mean_row >= 16.0) || (f_agg <= 64 && mean_row >= 128.0));
    if (!one_walk) t += 2.0 * c.launch_us * 1e-6 + (g.nnz * 8.0 + g.n_rows * 16.0) / c.stream_bps;
    if (fold) t += t_stream(c, 4.0 * f_in * f_out) + t_stream(c, 4.0 * g.n_cols * f_in);
    else t += t_gemm(c, g.n_cols, f_in, f_out, g.learned) + t_stream(c, 4.0 * g.n_cols * f_out);
    if (gat_is_reuse(id)) {
        if (fold) t += t_gemm(c, g.n_cols, f_in, f_out, g.learned);
        t += t_spmm(c, g, f_out, kSpmmSoftmaxCost);
    } else {
        Features gs = g;
        if (g.nnz < 16.0 * g.n_cols) gs.tile_share = 0.0;  // X is gathered row-major: no split
        t += t_spmm(c, gs, f_in, kSpmmSoftmaxCost) + t_gemm(c, g.n_rows, f_in, f_out, g.learned);
        if (g.nnz >= 16.0 * g.n_cols) t += t_stream(c, 8.0 * g.n_cols * f_in);  // slice-major copy of X
    }
    return t;
}

double gcn_bwd_cost(const sensei_ctx &c, const Features &g, int f_in, int f_out, int id, bool saved_u, bool want_dx) {
    Features gt = g;  // the transposed pattern
    gt.n_rows = g.n_cols; gt.n_cols = g.n_rows;
    double t = t_stream(c, 12.0 * g.n_rows * f_out);  // dP = dY (.) mask, scaled / re-laid
    if (id == SENSEI_GCN_BWD_AGG) {
        t += t_spmm(c, gt, f_out, kSpmmPattern) + t_gemm(c, f_in, g.n_cols, f_out, g.learned);
        if (want_dx) t += t_gemm(c, g.n_cols, f_out, f_in, g.learned);
    } else {
        if (!saved_u) t += t_stream(c, 8.0 * g.n_cols * f_in) + t_spmm(c, g, f_in, kSpmmPattern);
        t += t_gemm(c, f_in, g.n_rows, f_out, g.learned);
        if (want_dx) t += t_gemm(c, g.n_rows, f_out, f_in, g.learned) + t_spmm(c, gt, f_in, kSpmmPattern);
    }
    return t;
}

// The K-hop layers: every hop is one more aggregation at the width its association carries through the hops; TAGCN forms one weight
// gradient per hop and, in its update-side association, one product with W_k^T per hop.
double khop_bwd_cost(const sensei_ctx &c, const Features &g, int f_in, int f_out, int k_hops, bool tagcn, int id, bool want_dx) {
    Features gt = g;  // the transposed pattern
    gt.n_rows = g.n_cols; gt.n_cols = g.n_rows;
    const int blocks = tagcn ? k_hops + 1 : 1;
    double t = t_stream(c, 12.0 * g.n_rows * f_out);
    if (id == SENSEI_GCN_BWD_AGG) {
        t += k_hops * (t_spmm(c, gt, f_out, kSpmmPattern) + (tagcn ? t_stream(c, 8.0 * g.n_rows * f_out) : 0.0));
        t += blocks * t_gemm(c, f_in, g.n_cols, f_out, g.learned);
        if (want_dx) t += t_gemm(c, g.n_cols, (double)blocks * f_out, f_in, g.learned);
    } else {
        t += k_hops * (t_stream(c, 8.0 * g.n_cols * f_in) + t_spmm(c, g, f_in, kSpmmPattern));
        t += blocks * t_gemm(c, f_in, g.n_rows, f_out, g.learned);
        if (want_dx) t += blocks * t_gemm(c, g.n_rows, f_out, f_in, g.learned) + k_hops * t_spmm(c, gt, f_in, kSpmmPattern);
    }
    return t;
}

constexpr double kAutoMargin = 0.15;  // AUTO mode: predicted costs this close to the cheapest are settled by measurement

void rule_filter(int kind, int f_in, int f_out, bool *keep) {
    if (kind == SENSEI_KIND_GCN) {
        for (int id = 0; id < kNumGcn; ++id) {
            const bool agg = gcn_is_agg(id);
            keep[id] = (f_in == f_out) || (agg ? f_in < f_out : f_in > f_out);
        }
    } else {
        for (int id = 0; id < kNumGat; ++id) keep[id] = (f_in < f_out) || id == SENSEI_GAT_REUSE;
    }
}

__global__ void k_fill_f32(float *p, long long n, float v) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) p[t] = v * (float)((t % 7) - 3);
}
hipError_t fill(float *p, size_t n, float v, hipStream_t s) {
    if (n) hipLaunchKernelGGL(k_fill_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, (long long)n, v);
    return hipGetLastError();
}

size_t select_scratch_bytes(int kind, const sensei_csr &A, int f_in, int f_out) {
    size_t b = 0;
    b += align_up((size_t)A.n_cols * f_in * sizeof(float), 256);   // X
    b += align_up((size_t)f_in * f_out * sizeof(float), 256);      // W
    b += align_up((size_t)A.n_rows * f_out * sizeof(float), 256);  // Y
    b += 2 * align_up((size_t)(A.n_rows + A.n_cols) * sizeof(float), 256);  // r, c, degrees
    b += align_up((size_t)(A.nnz > 0 ? A.nnz : 1) * sizeof(float), 256);    // N~
    b += 2 * align_up((size_t)f_out * sizeof(float), 256);                  // a_l, a_r
    size_t layer = 0;
    const int n = kind == SENSEI_KIND_GCN ? kNumGcn : kNumGat;
    for (int id = 0; id < n; ++id) {
        const size_t w = kind == SENSEI_KIND_GCN ? gcn_ws(A, f_in, f_out, id) : gat_ws(A, f_in, f_out, id);
        layer = w > layer ? w : layer;
    }
    return b + layer + 1024;
}

}  // namespace

// ------------------------------------------------------------------- C ABI

extern "C" {

int sensei_create(sensei_ctx **out, int device) {
    if (!out) return SENSEI_INVALID_ARGUMENT;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess) return SENSEI_HIP_ERROR;
    if (device < 0 || device >= count) return SENSEI_INVALID_ARGUMENT;
    sensei_ctx *c = new (std::nothrow) sensei_ctx;
    if (!c) return SENSEI_HIP_ERROR;
    c->device = device;
    c->launch_us = 2.5;
    c->stream_bps = 4.5e12;
    c->gather_l2_bps = 19.0e12;
    c->gather_far_bps = 6.5e12;
    c->gemm_flops = 100.0e12;
    c->l2_slice_bytes = 29.8e6;
    // address of this GPU's copy of the static scratch array: resolved once per device, with that device current
    c->scratch = device < kMaxDevices ? g_scratch_ptr[device] : nullptr;
    hipError_t e = hipSuccess;
    if (!c->scratch) {
        int prev = 0;
        e = hipGetDevice(&prev);
        if (e == hipSuccess) e = hipSetDevice(device);
        if (e == hipSuccess) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            const hipError_t e2 = hipSetDevice(prev);
            if (e == hipSuccess) e = e2;
            if (e == hipSuccess) {
                c->scratch = ptr;
                if (device < kMaxDevices) g_scratch_ptr[device] = ptr;
            }
        }
    }
    if (e != hipSuccess || !c->scratch) {
        delete c;
        return SENSEI_HIP_ERROR;
    }
    *out = c;
    return SENSEI_OK;
}

int sensei_destroy(sensei_ctx *ctx) {
    if (ctx) {
        for (hipEvent_t e : ctx->timers.spmm.events) (void)hipEventDestroy(e);
        for (hipEvent_t e : ctx->timers.gemm.events) (void)hipEventDestroy(e);
    }
    delete ctx;
    return SENSEI_OK;
}

int sensei_profile_enable(sensei_ctx *ctx, int enable) {
    if (!ctx) return SENSEI_INVALID_ARGUMENT;
    for (KernelTimer *t : {&ctx->timers.spmm, &ctx->timers.gemm}) {
        t->enabled = enable != 0;
        if (enable) t->used = 0;
    }
    return SENSEI_OK;
}

int sensei_profile_read(sensei_ctx *ctx, int kernel, float *ms_out, int capacity, int *count_out) {
    if (!ctx || !count_out || capacity < 0 || (capacity > 0 && !ms_out)) return SENSEI_INVALID_ARGUMENT;
    if (kernel != SENSEI_PROFILE_SPMM && kernel != SENSEI_PROFILE_GEMM) return SENSEI_INVALID_ARGUMENT;
    KernelTimer &t = kernel == SENSEI_PROFILE_SPMM ? ctx->timers.spmm : ctx->timers.gemm;
    const size_t pairs = t.used / 2;
    *count_out = (int)pairs;
    for (size_t p = 0; p < pairs && p < (size_t)capacity; ++p) {
        if (hipEventSynchronize(t.events[2 * p + 1]) != hipSuccess) return SENSEI_HIP_ERROR;
        if (hipEventElapsedTime(&ms_out[p], t.events[2 * p], t.events[2 * p + 1]) != hipSuccess) return SENSEI_HIP_ERROR;
    }
    return SENSEI_OK;
}

int sensei_num_compositions(int kind) { return kind == SENSEI_KIND_GCN ? kNumGcn : kind == SENSEI_KIND_GAT ? kNumGat : 0; }

const char *sensei_composition_name(int kind, int id) {
    if (kind == SENSEI_KIND_GCN && id >= 0 && id < kNumGcn) return kGcnNames[id];
    if (kind == SENSEI_KIND_GAT && id >= 0 && id < kNumGat) return kGatNames[id];
    return "?";
}

const char *sensei_status_string(int status) {
    switch (status) {
        case SENSEI_OK: return "ok";
        case SENSEI_INVALID_ARGUMENT: return "invalid argument";
        case SENSEI_INVALID_COMPOSITION: return "invalid composition id";
        case SENSEI_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SENSEI_HIP_ERROR: return "HIP error";
        case SENSEI_UNSUPPORTED: return "unsupported";
        case SENSEI_SCRATCH_TOO_SMALL: return "input exceeds the static scratch buffer";
        default: return "unknown status";
    }
}

static size_t panels_layout(const sensei_csr &A, int q_count, size_t *rp_each, size_t *col_bytes, size_t *chunk_each, size_t *temp_bytes) {
    const int t = choose_chunk_nnz(A.nnz);
    *rp_each = align_up(((size_t)A.n_rows + 1) * sizeof(int32_t), 256);
    *col_bytes = align_up((size_t)(A.nnz > 0 ? A.nnz : 1) * sizeof(int32_t), 256);
    *chunk_each = align_up(((size_t)(A.nnz / t) + 3) * sizeof(int32_t), 256);
    *temp_bytes = plan_bytes(A.nnz) + scan_temp_bytes(A.n_rows + 1);
    return (size_t)q_count * (*rp_each + *chunk_each) + 2 * *col_bytes + 256 /* offsets */ + *temp_bytes;
}

int sensei_panels_bytes(const sensei_csr *A, int n_panels, size_t *device_bytes) {
    if (!csr_ok(A, false) || !device_bytes || n_panels < 0 || n_panels > SENSEI_MAX_PANELS) return SENSEI_INVALID_ARGUMENT;
    size_t a, b, c, d;
    *device_bytes = panels_layout(*A, n_panels > 0 ? n_panels : auto_panels(*A), &a, &b, &c, &d);
    return SENSEI_OK;
}

// Builds the panel copy for Q panels into `base` (laid out as panels_layout says) and waits for it.
static int build_panels(sensei_panels *P, const sensei_csr &A, int Q, char *base, hipStream_t s) {
    size_t rp_each, col_bytes, chunk_each, temp_bytes;
    panels_layout(A, Q, &rp_each, &col_bytes, &chunk_each, &temp_bytes);
    P->n_panels = Q;
    P->width = (int)((A.n_cols + Q - 1) / Q);
    if (P->width < 1) P->width = 1;
    P->n_rows = A.n_rows; P->n_cols = A.n_cols; P->nnz = A.nnz;
    P->src_row_ptr = A.row_ptr; P->src_col_idx = A.col_idx;
    P->chunk_nnz = choose_chunk_nnz(A.nnz);
    size_t used = 0;
    for (int q = 0; q < Q; ++q) { P->row_ptr_q[q] = reinterpret_cast<int32_t *>(base + used); used += rp_each; }
    for (int q = 0; q < Q; ++q) { P->chunk_row_q[q] = reinterpret_cast<int32_t *>(base + used); used += chunk_each; }
    int32_t *col_all = reinterpret_cast<int32_t *>(base + used); used += col_bytes;
    int32_t *perm_all = reinterpret_cast<int32_t *>(base + used); used += col_bytes;
    int32_t *off = reinterpret_cast<int32_t *>(base + used); used += 256;
    Carver cv(base + used, temp_bytes);
    ChunkPlan plan = make_plan(A, cv);
    int32_t *scan_temp = cv.take<int32_t>(scan_temp_bytes(A.n_rows + 1) / sizeof(int32_t));
    int32_t off_host[SENSEI_MAX_PANELS + 1] = {0};
    if (launch_chunk_rows(A, plan, s) != hipSuccess ||
        launch_panel_build(A, plan, Q, P->width, P->row_ptr_q, off, col_all, perm_all, scan_temp, s) != hipSuccess ||
        hipMemcpyAsync(off_host, off, (size_t)(Q + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return SENSEI_HIP_ERROR;
    for (int q = 0; q < Q; ++q) {
        P->nnz_q[q] = (int64_t)off_host[q + 1] - off_host[q];
        P->col_q[q] = col_all + off_host[q];
        P->off_q[q] = off_host[q];
        P->n_chunks_q[q] = P->nnz_q[q] <= 0 ? 1 : (int)((P->nnz_q[q] + P->chunk_nnz - 1) / P->chunk_nnz);
        sensei_csr Aq = A;
        Aq.nnz = P->nnz_q[q]; Aq.row_ptr = P->row_ptr_q[q]; Aq.col_idx = P->col_q[q];
        ChunkPlan pq;
        pq.chunk_nnz = P->chunk_nnz; pq.n_chunks = P->n_chunks_q[q]; pq.chunk_row = P->chunk_row_q[q];
        if (launch_chunk_rows(Aq, pq, s) != hipSuccess) return SENSEI_HIP_ERROR;
    }
    P->position = perm_all;
    P->off_q[Q] = off_host[Q];
    if (off_host[Q] != (int32_t)A.nnz) return SENSEI_INVALID_ARGUMENT;  // malformed pattern
    return SENSEI_OK;
}

int sensei_panels_create(sensei_ctx *ctx, const sensei_csr *A, int n_panels, void *device_buf, size_t bytes, void *stream,
                         sensei_panels **out) {
    if (!ctx || !csr_ok(A, false) || !out || !device_buf || n_panels < 0 || n_panels > SENSEI_MAX_PANELS) return SENSEI_INVALID_ARGUMENT;
    if (reinterpret_cast<uintptr_t>(device_buf) % 256 != 0) return SENSEI_INVALID_ARGUMENT;
    const int Q = n_panels > 0 ? n_panels : auto_panels(*A);
    size_t rp_each, col_bytes, chunk_each, temp_bytes;
    if (bytes < panels_layout(*A, Q, &rp_each, &col_bytes, &chunk_each, &temp_bytes)) return SENSEI_WORKSPACE_TOO_SMALL;
    sensei_panels *P = new (std::nothrow) sensei_panels;
    if (!P) return SENSEI_HIP_ERROR;
    const int status = build_panels(P, *A, Q, static_cast<char *>(device_buf), as_stream(stream));
    if (status != SENSEI_OK) { delete P; return status; }
    *out = P;
    return SENSEI_OK;
}

int sensei_panels_set_min_width(sensei_panels *panels, int min_width) {
    if (!panels || min_width < 1) return SENSEI_INVALID_ARGUMENT;
    panels->min_width = min_width;
    return SENSEI_OK;
}

// ---- measured choice of the panel count
namespace {
constexpr int kTuneWide = 256, kTuneNarrow = 64;
constexpr int kTuneCounts[] = {1, 2, 3, 4, 6, 8};

bool tune_worthwhile(const sensei_csr &A) {
    const double slice = (double)A.n_cols * 128.0;
    const double avg = A.n_rows > 0 ? (double)A.nnz / A.n_rows : 0.0;
    return slice >= 6e6 && avg >= 32.0;  // a slice the L2s hold, or rows too short to be visited once per panel
}

struct TuneLayout {
    size_t b_bytes, c_bytes, sparse_bytes, panel_bytes, total;
};
TuneLayout tune_layout(const sensei_csr &A) {
    TuneLayout t;
    t.b_bytes = align_up((size_t)A.n_cols * kTuneWide * sizeof(float), 256);
    t.c_bytes = align_up((size_t)A.n_rows * kTuneWide * sizeof(float), 256);
    t.sparse_bytes = plan_bytes(A.nnz) + spmm_carry_bytes(A.nnz, kTuneWide) + 256;
    size_t a, b, c, d;
    t.panel_bytes = panels_layout(A, SENSEI_MAX_PANELS, &a, &b, &c, &d);
    t.total = t.b_bytes + t.c_bytes + t.sparse_bytes + t.panel_bytes + 256;
    return t;
}
}  // namespace

int sensei_panels_tune_bytes(const sensei_csr *A, size_t *bytes) {
    if (!csr_ok(A, false) || !bytes) return SENSEI_INVALID_ARGUMENT;
    *bytes = tune_worthwhile(*A) ? tune_layout(*A).total : 256;
    return SENSEI_OK;
}

int sensei_panels_tune(sensei_ctx *ctx, const sensei_csr *A, void *scratch, size_t bytes, void *stream, int *n_panels_out,
                       int *min_width_out, float *ms_per_count) {
    if (!ctx || !csr_ok(A, false) || !n_panels_out || !min_width_out) return SENSEI_INVALID_ARGUMENT;
    if (ms_per_count) for (int q = 0; q < 2 * (SENSEI_MAX_PANELS + 1); ++q) ms_per_count[q] = -1.f;
    *n_panels_out = 1;
    *min_width_out = 128;
    if (!tune_worthwhile(*A)) return SENSEI_OK;
    const TuneLayout L = tune_layout(*A);
    if (!scratch || reinterpret_cast<uintptr_t>(scratch) % 256 != 0) return SENSEI_INVALID_ARGUMENT;
    if (bytes < L.total) return SENSEI_WORKSPACE_TOO_SMALL;
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(scratch);
    float *B = reinterpret_cast<float *>(base);
    float *C = reinterpret_cast<float *>(base + L.b_bytes);
    char *sparse = base + L.b_bytes + L.c_bytes;
    char *panel_buf = sparse + L.sparse_bytes;
    if (hipMemsetAsync(B, 0, L.b_bytes, s) != hipSuccess) return SENSEI_HIP_ERROR;
    Carver cv(sparse, L.sparse_bytes);
    ChunkPlan plan = make_plan(*A, cv);
    float *carry = cv.take<float>(spmm_carry_bytes(A->nnz, kTuneWide) / sizeof(float));
    if (launch_chunk_rows(*A, plan, s) != hipSuccess) return SENSEI_HIP_ERROR;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SENSEI_HIP_ERROR;
    if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return SENSEI_HIP_ERROR; }
    sensei_panels P;
    P.min_width = 1;
    // fastest of two timed runs after a warm-up, gathered operand slice-major to the width as the layers' intermediates are;
    // Q = 1 runs the plain single pass
    auto time_spmm = [&](int Q, int f, float *ms) -> int {
        sensei_csr Aq = *A;
        Aq.val = nullptr;
        Aq.panels = Q > 1 ? &P : nullptr;
        float best = 1e30f;
        for (int it = 0; it < 3; ++it) {
            if (hipEventRecord(e0, s) != hipSuccess) return SENSEI_HIP_ERROR;
            if (spmm_any(Aq, SENSEI_SPMM_PATTERN, nullptr, nullptr, B, f, f, C, f, f, SENSEI_ACT_NONE, plan, carry, s, nullptr, false, nullptr, true) != hipSuccess)
                return SENSEI_HIP_ERROR;
            float t = 0.f;
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&t, e0, e1) != hipSuccess)
                return SENSEI_HIP_ERROR;
            if (it > 0 && t < best) best = t;
        }
        *ms = best;
        return SENSEI_OK;
    };
    int status = SENSEI_OK, best_q = 1, built = 0;
    float best_ms = 1e30f, single_ms = 0.f;
    const double slice = (double)A->n_cols * 128.0;
    for (int Q : kTuneCounts) {
        if (Q > 1 && slice / Q < 1e6) break;  // panels far smaller than one L2 gain nothing
        if (Q > 1) {
            status = build_panels(&P, *A, Q, panel_buf, s);
            if (status != SENSEI_OK) break;
            built = Q;
        }
        float ms = 0.f;
        status = time_spmm(Q, kTuneWide, &ms);
        if (status != SENSEI_OK) break;
        if (ms_per_count) ms_per_count[Q] = ms;
        if (Q == 1) single_ms = ms;
        if (ms < 0.98f * best_ms) { best_ms = ms; best_q = Q; }  // one more pass over the rows must buy at least 2 %
        else if (ms > 1.03f * best_ms || best_q == 1) break;     // past the minimum, or two panels gain nothing
    }
    if (status == SENSEI_OK && best_q > 1 && best_ms > 0.97f * single_ms) best_q = 1;  // not worth a second copy of the pattern
    if (status == SENSEI_OK && best_q > 1) {
        // do narrow SpMMs gain as well?
        if (built != best_q) status = build_panels(&P, *A, best_q, panel_buf, s);
        float with_ms = 0.f, without_ms = 0.f;
        if (status == SENSEI_OK) status = time_spmm(best_q, kTuneNarrow, &with_ms);
        if (status == SENSEI_OK) status = time_spmm(1, kTuneNarrow, &without_ms);
        if (status == SENSEI_OK && with_ms < 0.97f * without_ms) *min_width_out = kTuneNarrow;
        if (status == SENSEI_OK && ms_per_count) {
            ms_per_count[SENSEI_MAX_PANELS + 1 + 1] = without_ms;
            ms_per_count[SENSEI_MAX_PANELS + 1 + best_q] = with_ms;
        }
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (status == SENSEI_OK) *n_panels_out = best_q;
    return status;
}

int sensei_panels_count(const sensei_panels *panels) { return panels ? panels->n_panels : 0; }

// ---- dense tiles
namespace {
constexpr int kTileRanksMax = 65536;  // ranks per side that are examined for dense tiles

struct TilesLayout {
    int h_r, h_c, nt_r, nt_c, n_tiles, max_slots, min_count;
    size_t rank_r, rank_c, order_r, order_c, hist, sel_scan, slot_of, slot_ct, slot_rt, rt_ptr, scan_small, plan, bits, pos, scan_large, col_rem,
        dst_rem, row_ptr_rem, plan_rem, bh, seg_first, rt_seg, seg_rt, seg_stats, rank_vec, part, dh, total;
    int max_seg;
    int rem_panels;  // panels of the panel-major copy of the remainder the layout has room for (1: none)
    size_t pm_rp, pm_off, pm_scan, pm_seg_ptr, pm_col, pm_pos, pm_plan, pm_part, pm_stats;
};

// Column panels of the remainder's panel-major copy, from the features known before the split: two where a 128-byte slice of the
// gathered matrix exceeds the L2s several times over (12 MB) and rows are long enough that a part of a row is still a run of
// gathers, three from 24 MB on; none otherwise.  Measured on the 233,000-node power-law graph (slice 29.8 MB, 494 entries per
// row, 41.8 M of 115 M entries in the remainder), whole three-layer step with 2 / 3 / 4 panels: 10.00 / 9.90 / 10.59 ms - the L2
// hit rate of the remainder keeps rising with the panel count (44 % -> 82 % at eight), but every (panel, row) segment costs a
// row end in the kernel and a partial row written and read back.
int g_remainder_panels_override = 0;  // sensei_tiles_remainder_panels: 0 = the rule below
int remainder_panels_for(const sensei_csr &A) {
    if (g_remainder_panels_override > 0) return (int64_t)A.n_rows * g_remainder_panels_override < (1LL << 30) ? g_remainder_panels_override : 1;
    if ((double)A.n_cols * 128.0 < 12e6 || A.nnz < 128 * (int64_t)A.n_rows) return 1;
    const int q = (double)A.n_cols * 128.0 >= 24e6 ? 3 : 2;
    return (int64_t)A.n_rows * q < (1LL << 30) ? q : 1;
}

TilesLayout tiles_layout(const sensei_csr &A, float min_density, int max_width) {
    TilesLayout L;
    L.h_r = A.n_rows < kTileRanksMax ? A.n_rows : kTileRanksMax;
    L.h_c = A.n_cols < kTileRanksMax ? A.n_cols : kTileRanksMax;
    L.nt_r = (L.h_r + 127) / 128;
    L.nt_c = (L.h_c + 127) / 128;
    L.n_tiles = L.nt_r * L.nt_c;
    L.min_count = (int)(min_density * 128.f * 128.f);
    if (L.min_count < 1) L.min_count = 1;
    const int64_t by_count = A.nnz / L.min_count;
    L.max_slots = (int)(by_count < L.n_tiles ? by_count : L.n_tiles);
    size_t off = 0;
    auto put = [&](size_t bytes) { const size_t at = off; off += align_up(bytes > 0 ? bytes : 4, 256); return at; };
    L.rank_r = put((size_t)A.n_rows * 4);
    L.rank_c = put((size_t)A.n_cols * 4);
    L.order_r = put((size_t)L.nt_r * 128 * 4);
    L.order_c = put((size_t)L.nt_c * 128 * 4);
    L.hist = put((size_t)L.n_tiles * 4);
    L.sel_scan = put(((size_t)L.n_tiles + 1) * 4);
    L.slot_of = put((size_t)L.n_tiles * 4);
    L.slot_ct = put((size_t)L.n_tiles * 4);
    L.slot_rt = put((size_t)L.n_tiles * 4);
    L.rt_ptr = put(((size_t)L.nt_r + 1) * 4);
    L.scan_small = put(scan_temp_bytes(L.n_tiles + 1));
    L.plan = put(plan_bytes(A.nnz));
    L.bits = put((size_t)L.max_slots * 128 * 4 * 4);
    L.pos = put(((size_t)A.nnz + 1) * 4);
    L.scan_large = put(scan_large_temp_bytes((long long)A.nnz + 1));
    L.col_rem = put((size_t)A.nnz * 4);
    L.dst_rem = put((size_t)A.nnz * 4);
    L.row_ptr_rem = put(((size_t)A.n_rows + 1) * 4);
    L.plan_rem = put(plan_bytes(A.nnz) + 4096);
    L.bh = put((size_t)L.nt_c * 128 * max_width * 6);   // fp32 rows (attention modes), or three bf16 pieces per element (value-less mode)
    L.max_seg = L.max_slots / kTilesPerSegment + L.nt_r + 1;
    L.seg_first = put(((size_t)L.max_seg + 1) * 4);
    L.rt_seg = put(((size_t)L.nt_r + 1) * 4);
    L.seg_rt = put(((size_t)L.max_seg + 1) * 4);
    L.seg_stats = put((size_t)L.max_seg * 128 * 8);
    L.rank_vec = put((size_t)2 * (L.nt_r + L.nt_c) * 128 * 4);
    L.part = put((size_t)L.max_seg * 128 * max_width * 4);
    L.dh = put((size_t)L.nt_r * 128 * max_width * 4);
    L.rem_panels = remainder_panels_for(A);
    if (L.rem_panels > 1) {
        const size_t P = (size_t)L.rem_panels, n = (size_t)A.n_rows;
        L.pm_rp = put(P * align_up((n + 1) * 4, 256));
        L.pm_off = put(256);
        L.pm_scan = put(scan_temp_bytes(A.n_rows + 1));
        L.pm_seg_ptr = put((P * n + 1) * 4);
        L.pm_col = put((size_t)A.nnz * 4);
        L.pm_pos = put((size_t)A.nnz * 4);
        L.pm_plan = put(plan_bytes(A.nnz) + 4096);
        L.pm_part = put(P * n * (size_t)max_width * 4);
        L.pm_stats = put(P * n * 8);
    }
    L.total = off;
    return L;
}

// nodes in descending order of degree (ties: lower id first): rank of every node (INT_MAX beyond the first h) and the
// node at every rank (-1 in the padding up to whole tiles).  Only the first h places are needed: selection, then a sort
// of those.  Returns the number of entries in the 128 highest-degree rows (or columns), an upper bound for any one tile.
int64_t rank_by_degree(const std::vector<int32_t> &deg, int h, int n_ranks, std::vector<int32_t> *rank, std::vector<int32_t> *order) {
    const int n = (int)deg.size();
    std::vector<int32_t> idx(n);
    for (int i = 0; i < n; ++i) idx[i] = i;
    auto before = [&](int32_t a, int32_t b) { return deg[a] != deg[b] ? deg[a] > deg[b] : a < b; };
    if (h < n) std::nth_element(idx.begin(), idx.begin() + h, idx.end(), before);
    std::sort(idx.begin(), idx.begin() + h, before);
    rank->assign(n, 0x7fffffff);
    order->assign(n_ranks, -1);
    int64_t top = 0;
    for (int q = 0; q < h; ++q) {
        (*rank)[idx[q]] = q;
        (*order)[q] = idx[q];
        if (q < 128) top += deg[idx[q]];
    }
    return top;
}
}  // namespace

int sensei_tiles_bytes(const sensei_csr *A, float min_density, int max_width, size_t *device_bytes) {
    if (!csr_ok(A, false) || !device_bytes || !(min_density > 0.f) || min_density > 1.f || max_width < 32 || max_width % 32 != 0 || max_width > 4096)
        return SENSEI_INVALID_ARGUMENT;
    *device_bytes = tiles_layout(*A, min_density, max_width).total;
    return SENSEI_OK;
}

int sensei_tiles_create(sensei_ctx *ctx, const sensei_csr *A, float min_density, int max_width, void *device_buf, size_t bytes, void *stream,
                        sensei_tiles **out) {
    if (!ctx || !csr_ok(A, false) || !out || !device_buf || !(min_density > 0.f) || min_density > 1.f || max_width < 32 || max_width % 32 != 0 ||
        max_width > 4096)
        return SENSEI_INVALID_ARGUMENT;
    if (reinterpret_cast<uintptr_t>(device_buf) % 256 != 0) return SENSEI_INVALID_ARGUMENT;
    const TilesLayout L = tiles_layout(*A, min_density, max_width);
    if (bytes < L.total) return SENSEI_WORKSPACE_TOO_SMALL;
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(device_buf);
    auto at = [&](size_t off) { return reinterpret_cast<int32_t *>(base + off); };
    sensei_tiles *D = new (std::nothrow) sensei_tiles;
    if (!D) return SENSEI_HIP_ERROR;
    auto fail = [&](int status) { sensei_tiles_destroy(D); return status; };
    D->n_rows = A->n_rows; D->n_cols = A->n_cols; D->nnz = A->nnz;
    D->src_row_ptr = A->row_ptr; D->src_col_idx = A->col_idx;
    D->max_width = max_width;
    D->Bh = reinterpret_cast<float *>(base + L.bh);
    D->T.nt_r = L.nt_r; D->T.nt_c = L.nt_c; D->T.n_slots = 0; D->T.n_seg = 0;
    D->T.seg_first = nullptr; D->T.rt_seg = nullptr; D->T.seg_rt = nullptr; D->T.part = nullptr; D->T.rank_vec = nullptr; D->T.seg_stats = nullptr;
    D->T.dh = nullptr; D->T.rank_r = nullptr;
    D->T.order_r = at(L.order_r); D->T.order_c = at(L.order_c); D->T.rt_ptr = at(L.rt_ptr); D->T.slot_ct = at(L.slot_ct); D->T.slot_rt = at(L.slot_rt);
    D->T.bits = reinterpret_cast<unsigned *>(base + L.bits);
    D->nnz_rem = A->nnz; D->row_ptr_rem = at(L.row_ptr_rem); D->col_rem = at(L.col_rem); D->dst_rem = at(L.dst_rem);
    if (A->n_rows == 0 || A->n_cols == 0 || A->nnz == 0) { *out = D; return SENSEI_OK; }  // nothing to split: never used

    // degrees on the device (the pos area is free until the split), ranking on the host: n log n on a few 10^5..10^6 integers
    int32_t *deg_r_d = at(L.pos), *deg_c_d = at(L.col_rem);
    if (launch_degrees(*A, deg_r_d, deg_c_d, s) != hipSuccess) return fail(SENSEI_HIP_ERROR);
    std::vector<int32_t> deg_r(A->n_rows), deg_c(A->n_cols), rank, order;
    if (hipMemcpyAsync(deg_r.data(), deg_r_d, (size_t)A->n_rows * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(deg_c.data(), deg_c_d, (size_t)A->n_cols * 4, hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);
    const int64_t top_r = rank_by_degree(deg_r, L.h_r, L.nt_r * 128, &rank, &order);
    if (top_r < L.min_count) { *out = D; return SENSEI_OK; }  // not even the 128 longest rows together fill one tile to the threshold
    if (hipMemcpyAsync(at(L.rank_r), rank.data(), rank.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(at(L.order_r), order.data(), order.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);
    const int64_t top_c = rank_by_degree(deg_c, L.h_c, L.nt_c * 128, &rank, &order);
    if (top_c < L.min_count) { *out = D; return SENSEI_OK; }
    if (hipMemcpyAsync(at(L.rank_c), rank.data(), rank.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(at(L.order_c), order.data(), order.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);

    ChunkPlan plan;
    plan.chunk_nnz = choose_chunk_nnz(A->nnz);
    plan.n_chunks = (int)((A->nnz + plan.chunk_nnz - 1) / plan.chunk_nnz);
    plan.chunk_row = at(L.plan);
    if (launch_chunk_rows(*A, plan, s) != hipSuccess) return fail(SENSEI_HIP_ERROR);
    if (launch_tile_select(*A, plan, at(L.rank_r), at(L.rank_c), L.h_r, L.h_c, L.nt_r, L.nt_c, L.min_count, at(L.hist), at(L.sel_scan), at(L.slot_of),
                           at(L.slot_ct), at(L.slot_rt), at(L.rt_ptr), at(L.scan_small), s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);
    int32_t n_slots = 0;
    if (hipMemcpyAsync(&n_slots, at(L.sel_scan) + L.n_tiles, 4, hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);
    if (n_slots < 0 || n_slots > L.max_slots) return fail(SENSEI_HIP_ERROR);
    D->T.n_slots = n_slots;
    if (n_slots == 0) { *out = D; return SENSEI_OK; }  // no tile is dense enough: the pattern stays as it is
    {   // segments of the rows of tiles: the longest rows would otherwise keep one workgroup busy for hundreds of tiles
        std::vector<int32_t> rt_ptr(L.nt_r + 1), seg_first, rt_seg(L.nt_r + 1), seg_rt;
        if (hipMemcpyAsync(rt_ptr.data(), at(L.rt_ptr), rt_ptr.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
            return fail(SENSEI_HIP_ERROR);
        for (int rt = 0; rt < L.nt_r; ++rt) {
            rt_seg[rt] = (int32_t)seg_first.size();
            for (int q = rt_ptr[rt]; q < rt_ptr[rt + 1]; q += kTilesPerSegment) { seg_first.push_back(q); seg_rt.push_back(rt); }
        }
        rt_seg[L.nt_r] = (int32_t)seg_first.size();
        seg_first.push_back(rt_ptr[L.nt_r]);
        seg_rt.push_back(0);
        D->T.n_seg = rt_seg[L.nt_r];
        if (D->T.n_seg > L.max_seg) return fail(SENSEI_HIP_ERROR);
        if (hipMemcpyAsync(at(L.seg_first), seg_first.data(), seg_first.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(at(L.rt_seg), rt_seg.data(), rt_seg.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(at(L.seg_rt), seg_rt.data(), seg_rt.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
            return fail(SENSEI_HIP_ERROR);
        D->T.seg_first = at(L.seg_first); D->T.rt_seg = at(L.rt_seg); D->T.seg_rt = at(L.seg_rt);
        D->T.rank_vec = reinterpret_cast<float *>(base + L.rank_vec);
        D->T.seg_stats = reinterpret_cast<float2 *>(base + L.seg_stats);
        D->T.dh = reinterpret_cast<float *>(base + L.dh);
        D->T.rank_r = at(L.rank_r);
        if (hipStreamCreateWithFlags(&D->side, hipStreamNonBlocking) != hipSuccess || hipEventCreateWithFlags(&D->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&D->ev_join, hipEventDisableTiming) != hipSuccess)
            return fail(SENSEI_HIP_ERROR);
        D->T.part = reinterpret_cast<float *>(base + L.part);
    }
    if (launch_tile_split(*A, plan, at(L.rank_r), at(L.rank_c), L.h_r, L.h_c, L.nt_c, at(L.slot_of), n_slots, reinterpret_cast<unsigned *>(base + L.bits),
                          at(L.pos), at(L.scan_large), at(L.col_rem), at(L.dst_rem), at(L.row_ptr_rem), s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);
    int32_t nnz_rem = 0;
    if (hipMemcpyAsync(&nnz_rem, at(L.pos) + A->nnz, 4, hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return fail(SENSEI_HIP_ERROR);
    if (nnz_rem < 0 || nnz_rem > A->nnz) return fail(SENSEI_HIP_ERROR);
    D->nnz_rem = nnz_rem;
    sensei_csr Ar = *A;
    Ar.nnz = nnz_rem; Ar.row_ptr = D->row_ptr_rem; Ar.col_idx = D->col_rem;
    // the chunk length of the whole pattern: the remainder then never has more chunks than the pattern, and the per-chunk carry
    // buffers that callers size for the pattern hold the remainder's too
    D->plan_rem.chunk_nnz = choose_chunk_nnz(A->nnz);
    D->plan_rem.n_chunks = nnz_rem <= 0 ? 1 : (int)(((int64_t)nnz_rem + D->plan_rem.chunk_nnz - 1) / D->plan_rem.chunk_nnz);
    D->plan_rem.chunk_row = at(L.plan_rem);
    if (launch_chunk_rows(Ar, D->plan_rem, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return fail(SENSEI_HIP_ERROR);
    // (automatic choice: only if the rows of the remainder are still long enough to be cut)
    if (L.rem_panels > 1 && nnz_rem > 0 && (g_remainder_panels_override > 0 || nnz_rem >= 32 * (int64_t)A->n_rows)) {
        const int P = L.rem_panels;
        const int width = (A->n_cols + P - 1) / P;
        int32_t *rp[SENSEI_MAX_PANELS] = {};
        const size_t rp_each = align_up(((size_t)A->n_rows + 1) * 4, 256);
        for (int q = 0; q < P; ++q) rp[q] = reinterpret_cast<int32_t *>(base + L.pm_rp + (size_t)q * rp_each);
        if (launch_panel_build(Ar, D->plan_rem, P, width, rp, at(L.pm_off), at(L.pm_col), at(L.pm_pos), at(L.pm_scan), s) != hipSuccess ||
            launch_panel_segments(rp, at(L.pm_off), A->n_rows, P, at(L.pm_seg_ptr), s) != hipSuccess)
            return fail(SENSEI_HIP_ERROR);
        sensei_csr As = Ar;
        As.n_rows = P * A->n_rows; As.row_ptr = at(L.pm_seg_ptr); As.col_idx = at(L.pm_col);
        D->plan_pm = D->plan_rem;
        D->plan_pm.chunk_row = at(L.pm_plan);
        if (launch_chunk_rows(As, D->plan_pm, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return fail(SENSEI_HIP_ERROR);
        D->rem_panels = P;
        D->seg_ptr = at(L.pm_seg_ptr); D->col_pm = at(L.pm_col); D->pos_pm = at(L.pm_pos);
        D->part_pm = reinterpret_cast<float *>(base + L.pm_part);
        D->stats_pm = reinterpret_cast<float2 *>(base + L.pm_stats);
    }
    *out = D;
    return SENSEI_OK;
}

int sensei_tiles_remainder_panels(int n_panels) {
    const int prev = g_remainder_panels_override;
    if (n_panels >= 0 && n_panels <= SENSEI_MAX_PANELS) g_remainder_panels_override = n_panels;
    return prev;
}

int sensei_tiles_info(const sensei_tiles *tiles, int *n_tiles_kept, int64_t *nnz_dense, int64_t *nnz_sparse) {
    if (!tiles) return SENSEI_INVALID_ARGUMENT;
    if (n_tiles_kept) *n_tiles_kept = tiles->T.n_slots;
    if (nnz_dense) *nnz_dense = tiles->nnz - tiles->nnz_rem;
    if (nnz_sparse) *nnz_sparse = tiles->nnz_rem;
    return SENSEI_OK;
}

int sensei_tiles_set_min_width(sensei_tiles *tiles, int min_width) {
    if (!tiles || min_width < 1) return SENSEI_INVALID_ARGUMENT;
    tiles->min_width = min_width;
    return SENSEI_OK;
}

int sensei_tiles_destroy(sensei_tiles *tiles) {
    if (tiles) {
        if (tiles->ev_fork) (void)hipEventDestroy(tiles->ev_fork);
        if (tiles->ev_join) (void)hipEventDestroy(tiles->ev_join);
        if (tiles->side) (void)hipStreamDestroy(tiles->side);
    }
    delete tiles;
    return SENSEI_OK;
}

int sensei_panels_destroy(sensei_panels *panels) {
    delete panels;
    return SENSEI_OK;
}

int sensei_degrees(sensei_ctx *ctx, const sensei_csr *A, int32_t *deg_row, int32_t *deg_col, void *stream) {
    if (!ctx || !csr_ok(A, false)) return SENSEI_INVALID_ARGUMENT;
    if ((A->n_rows > 0 && !deg_row) || (A->n_cols > 0 && !deg_col)) return SENSEI_INVALID_ARGUMENT;
    return hip_status(launch_degrees(*A, deg_row, deg_col, as_stream(stream)));
}

int sensei_norm_vectors(sensei_ctx *ctx, const int32_t *deg, int64_t n, float *out, void *stream) {
    if (!ctx || n < 0 || (n > 0 && (!deg || !out))) return SENSEI_INVALID_ARGUMENT;
    return hip_status(launch_norm_vectors(deg, n, out, as_stream(stream)));
}

int sensei_chunk_nnz(int64_t nnz) { return nnz < 0 ? 0 : choose_chunk_nnz(nnz); }

int sensei_gemm_kernel(int64_t n, int k, int m) { return (n > 0 && k > 0 && m > 0 && gemm_uses_pieces(n, k, m)) ? SENSEI_GEMM_BF16_PIECES : SENSEI_GEMM_FP32; }

int sensei_sparse_workspace(const sensei_csr *A, int f, size_t *bytes) {
    if (!csr_ok(A, false) || f < 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    *bytes = sparse_ws(*A, pad32(f));
    return SENSEI_OK;
}

int sensei_gcn_precompute(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, float *val_out,
                          void *workspace, size_t ws_bytes, void *stream) {
    if (!ctx || !csr_ok(A, false)) return SENSEI_INVALID_ARGUMENT;
    if (A->nnz > 0 && (!r || !c || !val_out)) return SENSEI_INVALID_ARGUMENT;
    if (!workspace) return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < plan_bytes(A->nnz)) return SENSEI_WORKSPACE_TOO_SMALL;
    Carver cv(workspace, ws_bytes);
    ChunkPlan plan = make_plan(*A, cv);
    SENSEI_TRY(launch_chunk_rows(*A, plan, as_stream(stream)));
    return hip_status(launch_sddmm_norm(*A, r, c, val_out, plan, as_stream(stream)));
}

int sensei_row_broadcast(sensei_ctx *ctx, const float *s, sensei_mat X, float *Y, int64_t ldy, void *stream) {
    if (!ctx || !mat_ok(X) || ldy < X.cols) return SENSEI_INVALID_ARGUMENT;
    if (X.rows > 0 && X.cols > 0 && (!s || !Y)) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > 2147483647LL) return SENSEI_INVALID_ARGUMENT;
    if (Y != X.ptr && overlap(Y, mat_bytes(Y, X.rows, X.cols, ldy), X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld))) return SENSEI_INVALID_ARGUMENT;
    if (Y == X.ptr && ldy != X.ld) return SENSEI_INVALID_ARGUMENT;
    return hip_status(launch_row_broadcast(s, X.ptr, X.ld, X.rows, (int)X.cols, Y, ldy, SENSEI_ACT_NONE, as_stream(stream)));
}

int sensei_spmm(sensei_ctx *ctx, const sensei_csr *A, int mode, const float *r, const float *c, sensei_mat B, float *C,
                int64_t ldc, int activation, void *workspace, size_t ws_bytes, void *stream) {
    if (mode < SENSEI_SPMM_PATTERN || mode > SENSEI_SPMM_SCALED) return SENSEI_INVALID_ARGUMENT;
    if (!ctx || !csr_ok(A, mode == SENSEI_SPMM_WEIGHTED) || !mat_ok(B)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (B.rows != A->n_cols || ldc < B.cols || B.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (mode == SENSEI_SPMM_SCALED && ((A->n_rows > 0 && !r) || (A->n_cols > 0 && !c))) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > 0 && B.cols > 0 && !C) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows == 0 || B.cols == 0) return SENSEI_OK;
    if (!workspace) return SENSEI_INVALID_ARGUMENT;
    const int f = (int)B.cols;
    const size_t cbytes = mat_bytes(C, A->n_rows, f, ldc);
    if (overlap(C, cbytes, B.ptr, mat_bytes(B.ptr, B.rows, f, B.ld)) || overlap(C, cbytes, workspace, ws_bytes) ||
        overlap(B.ptr, mat_bytes(B.ptr, B.rows, f, B.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < plan_bytes(A->nnz) + spmm_carry_bytes(A->nnz, f)) return SENSEI_WORKSPACE_TOO_SMALL;
    Carver cv(workspace, ws_bytes);
    ChunkPlan plan = make_plan(*A, cv);
    float *carry = cv.take<float>(spmm_carry_bytes(A->nnz, f) / sizeof(float));
    SENSEI_TRY(launch_chunk_rows(*A, plan, as_stream(stream)));
    const bool scaled = (mode == SENSEI_SPMM_SCALED);
    // with room in the workspace (sensei_sparse_workspace asks for it) a matrix whose rows are gathered often is first
    // copied slice-major, the layout the layers use for their own intermediates
    const size_t copy_bytes = spmm_copy_bytes(*A, f);
    const float *src = B.ptr;
    bool sliced = false;
    if (copy_bytes > 0 && cv.used + copy_bytes + 256 <= ws_bytes) {
        float *T = cv.take<float>(copy_bytes / sizeof(float));
        SENSEI_TRY(launch_to_slices(nullptr, B.ptr, B.ld, A->n_cols, f, T, as_stream(stream)));
        src = T;
        sliced = true;
    }
    return hip_status(spmm_any(*A, mode, scaled ? r : nullptr, scaled ? c : nullptr, src, B.ld, f, C, ldc, f, activation, plan, carry,
                                  as_stream(stream), &ctx->timers.spmm, false, nullptr, sliced));
}

int sensei_spmm_static(sensei_ctx *ctx, const sensei_csr *A, int mode, const float *r, const float *c, sensei_mat B, float *C,
                       int64_t ldc, int activation, void *stream) {
    if (mode < SENSEI_SPMM_PATTERN || mode > SENSEI_SPMM_SCALED) return SENSEI_INVALID_ARGUMENT;
    if (!ctx || !ctx->scratch || !csr_ok(A, mode == SENSEI_SPMM_WEIGHTED) || !mat_ok(B)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (B.rows != A->n_cols || ldc < B.cols || B.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (mode == SENSEI_SPMM_SCALED && ((A->n_rows > 0 && !r) || (A->n_cols > 0 && !c))) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > 0 && B.cols > 0 && !C) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows == 0 || B.cols == 0) return SENSEI_OK;
    const int f = (int)B.cols;
    if (overlap(C, mat_bytes(C, A->n_rows, f, ldc), B.ptr, mat_bytes(B.ptr, B.rows, f, B.ld))) return SENSEI_INVALID_ARGUMENT;
    // chunk plan + one carry slot per chunk: everything the kernels need beyond inputs and outputs
    if (plan_bytes(A->nnz) + spmm_carry_bytes(A->nnz, f) > (size_t)SENSEI_STATIC_SCRATCH_BYTES) return SENSEI_SCRATCH_TOO_SMALL;
    // Nothing in the array has to start at zero: the plan kernel writes every chunk_row entry, and a carry slot is read by
    // the fix-up pass only for chunks in which a row continues, each of which wrote its slot in this very call.
    Carver cv(ctx->scratch, SENSEI_STATIC_SCRATCH_BYTES);
    ChunkPlan plan = make_plan(*A, cv);
    float *carry = cv.take<float>(spmm_carry_bytes(A->nnz, f) / sizeof(float));
    SENSEI_TRY(launch_chunk_rows(*A, plan, as_stream(stream)));
    const bool scaled = (mode == SENSEI_SPMM_SCALED);
    // the plain single-pass kernel on the caller's row-major operand: no side stream, no events, no copies
    return hip_status(launch_spmm(*A, mode, scaled ? r : nullptr, scaled ? c : nullptr, B.ptr, B.ld, f, C, ldc, f, activation, plan, carry,
                                  as_stream(stream)));
}

int sensei_gemm(sensei_ctx *ctx, sensei_mat A, sensei_mat W, float *Y, int64_t ldy, int activation, void *stream) {
    if (!ctx || !mat_ok(A) || !mat_ok(W) || A.cols != W.rows || ldy < W.cols) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (A.rows > 0 && W.cols > 0 && !Y) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A.rows, W.cols, ldy);
    if (overlap(Y, ybytes, A.ptr, mat_bytes(A.ptr, A.rows, A.cols, A.ld)) || overlap(Y, ybytes, W.ptr, mat_bytes(W.ptr, W.rows, W.cols, W.ld))) return SENSEI_INVALID_ARGUMENT;
    return hip_status(launch_gemm(A.ptr, A.ld, W.ptr, W.ld, Y, ldy, A.rows, (int)A.cols, (int)W.cols, (int)W.cols, activation, as_stream(stream), nullptr,
                                  &ctx->timers.gemm));
}

int sensei_gemv2(sensei_ctx *ctx, sensei_mat A, const float *v1, const float *v2, float *y1, float *y2, void *stream) {
    if (!ctx || !mat_ok(A) || A.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (A.rows > 0 && (!y1 || !y2)) return SENSEI_INVALID_ARGUMENT;
    if (A.rows > 0 && A.cols > 0 && (!v1 || !v2)) return SENSEI_INVALID_ARGUMENT;
    return hip_status(launch_gemv2(A.ptr, A.ld, A.rows, (int)A.cols, v1, v2, y1, y2, as_stream(stream)));
}

int sensei_sddmm_score(sensei_ctx *ctx, const sensei_csr *A, const float *s_l, const float *s_r, float neg_slope,
                       float *e_out, void *workspace, size_t ws_bytes, void *stream) {
    if (!ctx || !csr_ok(A, false)) return SENSEI_INVALID_ARGUMENT;
    if (A->nnz > 0 && (!s_l || !s_r || !e_out)) return SENSEI_INVALID_ARGUMENT;
    if (!workspace) return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < plan_bytes(A->nnz)) return SENSEI_WORKSPACE_TOO_SMALL;
    Carver cv(workspace, ws_bytes);
    ChunkPlan plan = make_plan(*A, cv);
    SENSEI_TRY(launch_chunk_rows(*A, plan, as_stream(stream)));
    return hip_status(launch_score(*A, s_l, s_r, neg_slope, e_out, plan, as_stream(stream)));
}

int sensei_edge_softmax(sensei_ctx *ctx, const sensei_csr *A, const float *e, float *alpha_out, void *workspace,
                        size_t ws_bytes, void *stream) {
    if (!ctx || !csr_ok(A, false)) return SENSEI_INVALID_ARGUMENT;
    if (A->nnz > 0 && (!e || !alpha_out)) return SENSEI_INVALID_ARGUMENT;
    if (!workspace) return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < plan_bytes(A->nnz) + softmax_ws_bytes(*A)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->nnz == 0) return SENSEI_OK;
    Carver cv(workspace, ws_bytes);
    ChunkPlan plan = make_plan(*A, cv);
    float2 *stats = cv.take<float2>((size_t)A->n_rows + 1);
    float2 *carry_stats = cv.take<float2>((size_t)plan.n_chunks);
    SENSEI_TRY(launch_chunk_rows(*A, plan, as_stream(stream)));
    return hip_status(launch_softmax(*A, e, alpha_out, plan, stats, carry_stats, as_stream(stream)));
}

int sensei_gcn_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (comp_id < 0 || comp_id >= kNumGcn) return SENSEI_INVALID_COMPOSITION;
    *bytes = gcn_ws(*A, f_in, f_out, comp_id);
    return SENSEI_OK;
}

int sensei_gcn_layer(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, sensei_mat X, sensei_mat W,
                     float *Y, int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream) {
    if (comp_id < 0 || comp_id >= kNumGcn) return SENSEI_INVALID_COMPOSITION;
    const bool pre = (comp_id == SENSEI_GCN_PRE_AGG || comp_id == SENSEI_GCN_PRE_UPD);
    if (!ctx || !csr_ok(A, pre) || !mat_ok(X) || !mat_ok(W)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0 || ldy < W.cols) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (!X.ptr && A->n_cols > 0) return SENSEI_INVALID_ARGUMENT;
    if (!W.ptr || (!Y && A->n_rows > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (!pre && ((A->n_rows > 0 && !r) || (A->n_cols > 0 && !c))) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A->n_rows, W.cols, ldy);
    if (overlap(Y, ybytes, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(Y, ybytes, W.ptr, mat_bytes(W.ptr, W.rows, W.cols, W.ld)) ||
        overlap(Y, ybytes, workspace, ws_bytes) || overlap(X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gcn_ws(*A, (int)X.cols, (int)W.cols, comp_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return SENSEI_OK;
    return run_gcn(*A, r, c, X, W, Y, ldy, activation, comp_id, workspace, ws_bytes, as_stream(stream), &ctx->timers);
}

int sensei_sgc_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    *bytes = sgc_ws(*A, f_in, f_out, comp_id);
    return SENSEI_OK;
}

int sensei_sgc_layer(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, sensei_mat X, sensei_mat W, int k_hops, float *Y,
                     int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream) {
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !mat_ok(X) || !mat_ok(W)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows != A->n_cols || k_hops < 1 || k_hops > 64) return SENSEI_INVALID_ARGUMENT;  // powers of the pattern need it square
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0 || ldy < W.cols) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W.ptr || (!Y && A->n_rows > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > 0 && (!r || !c)) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A->n_rows, W.cols, ldy);
    if (overlap(Y, ybytes, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(Y, ybytes, W.ptr, mat_bytes(W.ptr, W.rows, W.cols, W.ld)) ||
        overlap(Y, ybytes, workspace, ws_bytes) || overlap(X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < sgc_ws(*A, (int)X.cols, (int)W.cols, comp_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return SENSEI_OK;
    return run_sgc(*A, r, c, X, W, k_hops, Y, ldy, activation, comp_id, workspace, ws_bytes, as_stream(stream), &ctx->timers);
}

int sensei_tagcn_workspace(const sensei_csr *A, int f_in, int f_out, int k_hops, int comp_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || k_hops < 1 || k_hops > 64 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    *bytes = tagcn_ws(*A, f_in, f_out, k_hops, comp_id);
    return SENSEI_OK;
}

int sensei_tagcn_layer(sensei_ctx *ctx, const sensei_csr *A, const float *r, const float *c, sensei_mat X, sensei_mat W, int k_hops, float *Y,
                       int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream) {
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !mat_ok(X) || !mat_ok(W)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows != A->n_cols || k_hops < 1 || k_hops > 64) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols <= 0 || W.cols <= 0 || W.rows != (int64_t)(k_hops + 1) * X.cols || ldy < W.cols) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20) || (int64_t)(k_hops + 1) * pad32((int)X.cols) > (1 << 24)) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W.ptr || (!Y && A->n_rows > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > 0 && (!r || !c)) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A->n_rows, W.cols, ldy);
    if (overlap(Y, ybytes, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(Y, ybytes, W.ptr, mat_bytes(W.ptr, W.rows, W.cols, W.ld)) ||
        overlap(Y, ybytes, workspace, ws_bytes) || overlap(X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld), workspace, ws_bytes) ||
        overlap(W.ptr, mat_bytes(W.ptr, W.rows, W.cols, W.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < tagcn_ws(*A, (int)X.cols, (int)W.cols, k_hops, comp_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return SENSEI_OK;
    return run_tagcn(*A, r, c, X, W, k_hops, Y, ldy, activation, comp_id, workspace, ws_bytes, as_stream(stream), &ctx->timers);
}

int sensei_gcn_backward_workspace(const sensei_csr *A, int f_in, int f_out, int bwd_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (bwd_id != SENSEI_GCN_BWD_AGG && bwd_id != SENSEI_GCN_BWD_UPD) return SENSEI_INVALID_COMPOSITION;
    *bytes = gcn_bwd_ws(*A, f_in, f_out, bwd_id);
    return SENSEI_OK;
}

int sensei_gcn_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const float *r, const float *c, sensei_mat X,
                        sensei_mat W, const float *Y, int64_t ldy, sensei_mat dY, int activation, const float *U_saved, int64_t ldu,
                        float *dX, int64_t lddx, float *dW, int64_t lddw, int bwd_id, void *workspace, size_t ws_bytes, void *stream) {
    if (bwd_id != SENSEI_GCN_BWD_AGG && bwd_id != SENSEI_GCN_BWD_UPD) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W) || !mat_ok(dY)) return SENSEI_INVALID_ARGUMENT;
    if (At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (dY.rows != A->n_rows || dY.cols != W.cols) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W.ptr || (!dY.ptr && A->n_rows > 0) || !dW || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (lddw < W.cols || (dX && lddx < X.cols)) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && ((!Y && A->n_rows > 0) || ldy < W.cols)) return SENSEI_INVALID_ARGUMENT;
    if (U_saved && ldu < X.cols) return SENSEI_INVALID_ARGUMENT;
    if ((A->n_rows > 0 && !r) || (A->n_cols > 0 && !c)) return SENSEI_INVALID_ARGUMENT;
    const size_t dwb = mat_bytes(dW, W.rows, W.cols, lddw), dxb = dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0;
    const size_t xb = mat_bytes(X.ptr, X.rows, X.cols, X.ld), wb = mat_bytes(W.ptr, W.rows, W.cols, W.ld),
                 dyb = mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld);
    if (overlap(dW, dwb, workspace, ws_bytes) || overlap(dW, dwb, X.ptr, xb) || overlap(dW, dwb, W.ptr, wb) || overlap(dW, dwb, dY.ptr, dyb))
        return SENSEI_INVALID_ARGUMENT;
    if (dX && (overlap(dX, dxb, workspace, ws_bytes) || overlap(dX, dxb, X.ptr, xb) || overlap(dX, dxb, W.ptr, wb) ||
               overlap(dX, dxb, dY.ptr, dyb) || overlap(dX, dxb, dW, dwb)))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gcn_bwd_ws(*A, (int)X.cols, (int)W.cols, bwd_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    return run_gcn_backward(*A, *At, r, c, X, W, Y, ldy, dY, activation, U_saved, ldu, dX, lddx, dW, lddw, bwd_id, workspace, ws_bytes,
                            as_stream(stream));
}

int sensei_sgc_backward_workspace(const sensei_csr *A, int f_in, int f_out, int k_hops, int bwd_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || k_hops < 1 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (bwd_id != SENSEI_GCN_BWD_AGG && bwd_id != SENSEI_GCN_BWD_UPD) return SENSEI_INVALID_COMPOSITION;
    *bytes = gcn_bwd_ws(*A, f_in, f_out, bwd_id, k_hops);
    return SENSEI_OK;
}

int sensei_sgc_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const float *r, const float *c, sensei_mat X, sensei_mat W,
                        int k_hops, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX, int64_t lddx, float *dW, int64_t lddw,
                        int bwd_id, void *workspace, size_t ws_bytes, void *stream) {
    if (bwd_id != SENSEI_GCN_BWD_AGG && bwd_id != SENSEI_GCN_BWD_UPD) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W) || !mat_ok(dY) || k_hops < 1) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows != A->n_cols || At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0 || dY.rows != A->n_rows || dY.cols != W.cols) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if ((A->n_rows > 0 && (!r || !c || !X.ptr || !dY.ptr)) || !W.ptr || !dW || lddw < W.cols || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && (!Y || ldy < W.cols)) return SENSEI_INVALID_ARGUMENT;
    if (dX && lddx < X.cols) return SENSEI_INVALID_ARGUMENT;
    const size_t dwb = mat_bytes(dW, W.rows, W.cols, lddw), dxb = dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0;
    if (overlap(dW, dwb, workspace, ws_bytes) || overlap(dX, dxb, workspace, ws_bytes) || overlap(dX, dxb, dW, dwb) ||
        overlap(dX, dxb, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(dX, dxb, dY.ptr, mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld)))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gcn_bwd_ws(*A, (int)X.cols, (int)W.cols, bwd_id, k_hops)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0)   // a sum over no nodes
        return launch_zero_matrix(dW, W.rows, (int)W.cols, lddw, false, as_stream(stream)) == hipSuccess ? SENSEI_OK : SENSEI_HIP_ERROR;
    return run_gcn_backward(*A, *At, r, c, X, W, Y, ldy, dY, activation, nullptr, 0, dX, lddx, dW, lddw, bwd_id, workspace, ws_bytes,
                            as_stream(stream), k_hops);
}

int sensei_tagcn_backward_workspace(const sensei_csr *A, int f_in, int f_out, int k_hops, int bwd_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || k_hops < 0 || k_hops > 64 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (bwd_id != SENSEI_GCN_BWD_AGG && bwd_id != SENSEI_GCN_BWD_UPD) return SENSEI_INVALID_COMPOSITION;
    *bytes = tagcn_bwd_ws(*A, f_in, f_out, k_hops, bwd_id);
    return SENSEI_OK;
}

int sensei_tagcn_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const float *r, const float *c, sensei_mat X, sensei_mat W,
                          int k_hops, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX, int64_t lddx, float *dW, int64_t lddw,
                          int bwd_id, void *workspace, size_t ws_bytes, void *stream) {
    if (bwd_id != SENSEI_GCN_BWD_AGG && bwd_id != SENSEI_GCN_BWD_UPD) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W) || !mat_ok(dY) || k_hops < 0 || k_hops > 64)
        return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows != A->n_cols || At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols <= 0 || W.cols <= 0 || W.rows != (int64_t)(k_hops + 1) * X.cols || dY.rows != A->n_rows || dY.cols != W.cols)
        return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20) || (int64_t)(k_hops + 1) * pad4((int)W.cols) > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if ((A->n_rows > 0 && (!r || !c || !X.ptr || !dY.ptr)) || !W.ptr || !dW || lddw < W.cols || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && A->n_rows > 0 && (!Y || ldy < W.cols)) return SENSEI_INVALID_ARGUMENT;
    if (dX && lddx < X.cols) return SENSEI_INVALID_ARGUMENT;
    const size_t dwb = mat_bytes(dW, W.rows, W.cols, lddw), dxb = dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0;
    const size_t xb = mat_bytes(X.ptr, X.rows, X.cols, X.ld), wb = mat_bytes(W.ptr, W.rows, W.cols, W.ld),
                 dyb = mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld);
    if (overlap(dW, dwb, workspace, ws_bytes) || overlap(dW, dwb, X.ptr, xb) || overlap(dW, dwb, W.ptr, wb) || overlap(dW, dwb, dY.ptr, dyb))
        return SENSEI_INVALID_ARGUMENT;
    if (dX && (overlap(dX, dxb, workspace, ws_bytes) || overlap(dX, dxb, X.ptr, xb) || overlap(dX, dxb, W.ptr, wb) ||
               overlap(dX, dxb, dY.ptr, dyb) || overlap(dX, dxb, dW, dwb)))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < tagcn_bwd_ws(*A, (int)X.cols, (int)W.cols, k_hops, bwd_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return launch_zero_matrix(dW, W.rows, (int)W.cols, lddw, false, as_stream(stream)) == hipSuccess ? SENSEI_OK : SENSEI_HIP_ERROR;
    return run_tagcn_backward(*A, *At, r, c, X, W, k_hops, Y, ldy, dY, activation, dX, lddx, dW, lddw, bwd_id, workspace, ws_bytes, as_stream(stream));
}

int sensei_transpose_positions(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, int32_t *t_pos, void *workspace,
                               size_t ws_bytes, void *stream) {
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || (!t_pos && A->nnz > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz) return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < plan_bytes(A->nnz) + 512) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->nnz == 0) return SENSEI_OK;
    hipStream_t s = as_stream(stream);
    Carver cv(workspace, ws_bytes);
    ChunkPlan plan = make_plan(*A, cv);
    int32_t *miss = cv.take<int32_t>(1);
    int32_t miss_host = 0;
    if (launch_chunk_rows(*A, plan, s) != hipSuccess ||
        launch_transpose_pos(*A, *At, plan, t_pos, miss, s) != hipSuccess ||
        hipMemcpyAsync(&miss_host, miss, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return SENSEI_HIP_ERROR;
    return miss_host == 0 ? SENSEI_OK : SENSEI_INVALID_ARGUMENT;
}

int sensei_gat_backward_workspace(const sensei_csr *A, const sensei_csr *At, int f_in, int f_out, size_t *bytes) {
    if (!csr_ok(A, false) || (At && !csr_ok(At, false)) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    *bytes = gat_bwd_ws(*A, At, f_in, f_out);
    return SENSEI_OK;
}

int sensei_gat_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W,
                        const float *a_l, const float *a_r, float neg_slope, const float *Y, int64_t ldy, sensei_mat dY, int activation,
                        float *dX, int64_t lddx, float *dW, int64_t lddw, float *da_l, float *da_r, void *workspace, size_t ws_bytes,
                        void *stream) {
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W) || !mat_ok(dY)) return SENSEI_INVALID_ARGUMENT;
    if (At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz || A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (dY.rows != A->n_rows || dY.cols != W.cols) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W.ptr || (!dY.ptr && A->n_rows > 0) || !dW || !da_l || !da_r || !a_l || !a_r || !workspace)
        return SENSEI_INVALID_ARGUMENT;
    if (!t_pos && A->nnz > 0) return SENSEI_INVALID_ARGUMENT;
    if (lddw < W.cols || (dX && lddx < X.cols)) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && ((!Y && A->n_rows > 0) || ldy < W.cols)) return SENSEI_INVALID_ARGUMENT;
    const size_t dwb = mat_bytes(dW, W.rows, W.cols, lddw), dxb = dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0;
    const size_t xb = mat_bytes(X.ptr, X.rows, X.cols, X.ld), wb = mat_bytes(W.ptr, W.rows, W.cols, W.ld),
                 dyb = mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld);
    if (overlap(dW, dwb, workspace, ws_bytes) || overlap(dW, dwb, X.ptr, xb) || overlap(dW, dwb, W.ptr, wb) || overlap(dW, dwb, dY.ptr, dyb))
        return SENSEI_INVALID_ARGUMENT;
    if (dX && (overlap(dX, dxb, workspace, ws_bytes) || overlap(dX, dxb, X.ptr, xb) || overlap(dX, dxb, W.ptr, wb) ||
               overlap(dX, dxb, dY.ptr, dyb) || overlap(dX, dxb, dW, dwb)))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gat_bwd_ws(*A, At, (int)X.cols, (int)W.cols)) return SENSEI_WORKSPACE_TOO_SMALL;
    return run_gat_backward(*A, *At, t_pos, X, W, a_l, a_r, neg_slope, Y, ldy, dY, activation, dX, lddx, dW, lddw, da_l, da_r, workspace,
                            ws_bytes, as_stream(stream));
}

int sensei_gat_backward_heads_workspace(const sensei_csr *A, const sensei_csr *At, int f_in, int f_out, int n_heads, size_t *bytes) {
    if (!csr_ok(A, false) || (At && !csr_ok(At, false)) || f_in <= 0 || f_out <= 0 || n_heads < 1 || f_out % n_heads != 0 || !bytes)
        return SENSEI_INVALID_ARGUMENT;
    *bytes = gat_bwd_heads_ws(*A, At, f_in, f_out, n_heads);
    return SENSEI_OK;
}

int sensei_gat_backward_heads(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W,
                              const float *a_l, const float *a_r, int n_heads, float neg_slope, const float *Y, int64_t ldy, sensei_mat dY,
                              int activation, float *dX, int64_t lddx, float *dW, int64_t lddw, float *da_l, float *da_r, void *workspace,
                              size_t ws_bytes, void *stream) {
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W) || !mat_ok(dY)) return SENSEI_INVALID_ARGUMENT;
    if (At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz || A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0 || n_heads < 1 || W.cols % n_heads != 0) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (dY.rows != A->n_rows || dY.cols != W.cols) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W.ptr || (!dY.ptr && A->n_rows > 0) || !dW || !da_l || !da_r || !a_l || !a_r || !workspace)
        return SENSEI_INVALID_ARGUMENT;
    if (!t_pos && A->nnz > 0) return SENSEI_INVALID_ARGUMENT;
    if (lddw < W.cols || (dX && lddx < X.cols)) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && ((!Y && A->n_rows > 0) || ldy < W.cols)) return SENSEI_INVALID_ARGUMENT;
    const size_t dwb = mat_bytes(dW, W.rows, W.cols, lddw), dxb = dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0;
    const size_t xb = mat_bytes(X.ptr, X.rows, X.cols, X.ld), wb = mat_bytes(W.ptr, W.rows, W.cols, W.ld),
                 dyb = mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld);
    if (overlap(dW, dwb, workspace, ws_bytes) || overlap(dW, dwb, X.ptr, xb) || overlap(dW, dwb, W.ptr, wb) || overlap(dW, dwb, dY.ptr, dyb))
        return SENSEI_INVALID_ARGUMENT;
    if (dX && (overlap(dX, dxb, workspace, ws_bytes) || overlap(dX, dxb, X.ptr, xb) || overlap(dX, dxb, W.ptr, wb) ||
               overlap(dX, dxb, dY.ptr, dyb) || overlap(dX, dxb, dW, dwb)))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gat_bwd_heads_ws(*A, At, (int)X.cols, (int)W.cols, n_heads)) return SENSEI_WORKSPACE_TOO_SMALL;
    return run_gat_backward_heads(*A, *At, t_pos, X, W, a_l, a_r, n_heads, neg_slope, Y, ldy, dY, activation, dX, lddx, dW, lddw, da_l, da_r, workspace,
                                  ws_bytes, as_stream(stream));
}

int sensei_gatv2_backward_workspace(const sensei_csr *A, int f_in, int f_out, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    *bytes = gatv2_bwd_ws(*A, f_in, f_out);
    return SENSEI_OK;
}

int sensei_gatv2_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W_l,
                          sensei_mat W_r, const float *att, float neg_slope, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX,
                          int64_t lddx, float *dW_l, int64_t lddwl, float *dW_r, int64_t lddwr, float *datt, void *workspace, size_t ws_bytes,
                          void *stream) {
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W_l) || !mat_ok(W_r) || !mat_ok(dY)) return SENSEI_INVALID_ARGUMENT;
    if (At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz || A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W_r.rows || X.cols != W_l.rows || W_l.cols != W_r.cols || X.cols <= 0 || W_r.cols <= 0)
        return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W_r.cols > (1 << 19)) return SENSEI_INVALID_ARGUMENT;
    if (dY.rows != A->n_rows || dY.cols != W_r.cols) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W_l.ptr || !W_r.ptr || (!dY.ptr && A->n_rows > 0) || !dW_l || !dW_r || !datt || !att || !workspace)
        return SENSEI_INVALID_ARGUMENT;
    if (!t_pos && A->nnz > 0) return SENSEI_INVALID_ARGUMENT;
    if (lddwl < W_l.cols || lddwr < W_r.cols || (dX && lddx < X.cols)) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && ((!Y && A->n_rows > 0) || ldy < W_r.cols)) return SENSEI_INVALID_ARGUMENT;
    const size_t xb = mat_bytes(X.ptr, X.rows, X.cols, X.ld), dyb = mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld);
    const size_t wlb = mat_bytes(W_l.ptr, W_l.rows, W_l.cols, W_l.ld), wrb = mat_bytes(W_r.ptr, W_r.rows, W_r.cols, W_r.ld);
    const size_t dxb = dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0;
    struct Out { const void *p; size_t n; } outs[4] = {{dW_l, mat_bytes(dW_l, W_l.rows, W_l.cols, lddwl)}, {dW_r, mat_bytes(dW_r, W_r.rows, W_r.cols, lddwr)},
                                                     {datt, (size_t)W_r.cols * sizeof(float)}, {dX, dxb}};
    for (int a = 0; a < 4; ++a) {
        const Out &o = outs[a];
        if (overlap(o.p, o.n, workspace, ws_bytes) || overlap(o.p, o.n, X.ptr, xb) || overlap(o.p, o.n, W_l.ptr, wlb) || overlap(o.p, o.n, W_r.ptr, wrb) ||
            overlap(o.p, o.n, dY.ptr, dyb) || overlap(o.p, o.n, att, (size_t)W_r.cols * sizeof(float)))
            return SENSEI_INVALID_ARGUMENT;
        for (int b = a + 1; b < 4; ++b)
            if (overlap(o.p, o.n, outs[b].p, outs[b].n)) return SENSEI_INVALID_ARGUMENT;
    }
    if (ws_bytes < gatv2_bwd_ws(*A, (int)X.cols, (int)W_r.cols)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) {   // no output rows: nothing depends on the inputs
        hipStream_t st = as_stream(stream);
        if (launch_zero_matrix(dW_l, W_l.rows, (int)W_l.cols, lddwl, false, st) != hipSuccess ||
            launch_zero_matrix(dW_r, W_r.rows, (int)W_r.cols, lddwr, false, st) != hipSuccess ||
            launch_zero_matrix(datt, 1, (int)W_r.cols, W_r.cols, false, st) != hipSuccess ||
            (dX && launch_zero_matrix(dX, A->n_cols, (int)X.cols, lddx, false, st) != hipSuccess))
            return SENSEI_HIP_ERROR;
        return SENSEI_OK;
    }
    return run_gatv2_backward(*A, *At, t_pos, X, W_l, W_r, att, neg_slope, Y, ldy, dY, activation, dX, lddx, dW_l, lddwl, dW_r, lddwr, datt, workspace,
                              ws_bytes, as_stream(stream));
}

int sensei_gat_attention_path(const sensei_csr *A, int f_in, int f_out, int n_heads, int comp_id) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || n_heads < 1 || f_out % n_heads != 0 || comp_id < 0 || comp_id >= kNumGat) return -1;
    const bool reuse = gat_is_reuse(comp_id);
    const int d = f_out / n_heads;
    const bool sliced = reuse ? (n_heads == 1 || d % 32 == 0) : relayout_pays(*A);
    return attention_path(*A, reuse ? (n_heads == 1 ? pad32(f_out) : d) : f_in, sliced);
}

int sensei_gat_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (comp_id < 0 || comp_id >= kNumGat) return SENSEI_INVALID_COMPOSITION;
    *bytes = gat_ws(*A, f_in, f_out, comp_id);
    return SENSEI_OK;
}

int sensei_gat_layer_heads(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W, const float *a_l, const float *a_r,
                           int n_heads, float neg_slope, float *Y, int64_t ldy, int activation, int comp_id, void *workspace,
                           size_t ws_bytes, void *stream) {
    if (comp_id < 0 || comp_id >= kNumGat) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !mat_ok(X) || !mat_ok(W)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W.rows || X.cols <= 0 || W.cols <= 0 || ldy < W.cols) return SENSEI_INVALID_ARGUMENT;
    if (n_heads < 1 || W.cols % n_heads != 0) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (!X.ptr && A->n_cols > 0) return SENSEI_INVALID_ARGUMENT;
    if (!W.ptr || !a_l || !a_r || (!Y && A->n_rows > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A->n_rows, W.cols, ldy);
    if (overlap(Y, ybytes, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(Y, ybytes, W.ptr, mat_bytes(W.ptr, W.rows, W.cols, W.ld)) ||
        overlap(Y, ybytes, workspace, ws_bytes) || overlap(X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gat_ws(*A, (int)X.cols, (int)W.cols, comp_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return SENSEI_OK;
    return run_gat(*A, X, W, a_l, a_r, neg_slope, Y, ldy, activation, comp_id, workspace, ws_bytes, as_stream(stream), &ctx->timers, n_heads);
}

int sensei_gat_layer(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W, const float *a_l, const float *a_r,
                     float neg_slope, float *Y, int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes,
                     void *stream) {
    return sensei_gat_layer_heads(ctx, A, X, W, a_l, a_r, 1, neg_slope, Y, ldy, activation, comp_id, workspace, ws_bytes, stream);
}

int sensei_gatv2_workspace(const sensei_csr *A, int f_in, int f_out, int comp_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    *bytes = gatv2_ws(*A, f_in, f_out, comp_id, false);
    return SENSEI_OK;
}

int sensei_gatv2_layer(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W_l, sensei_mat W_r, const float *att, float neg_slope,
                       float *Y, int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream) {
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !mat_ok(X) || !mat_ok(W_l) || !mat_ok(W_r)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols != W_r.rows || X.cols <= 0 || W_r.cols <= 0 || ldy < W_r.cols) return SENSEI_INVALID_ARGUMENT;
    if (W_l.rows != W_r.rows || W_l.cols != W_r.cols) return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W_r.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if (!X.ptr && A->n_cols > 0) return SENSEI_INVALID_ARGUMENT;
    if (!W_l.ptr || !W_r.ptr || !att || (!Y && A->n_rows > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A->n_rows, W_r.cols, ldy);
    if (overlap(Y, ybytes, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(Y, ybytes, W_r.ptr, mat_bytes(W_r.ptr, W_r.rows, W_r.cols, W_r.ld)) ||
        overlap(Y, ybytes, W_l.ptr, mat_bytes(W_l.ptr, W_l.rows, W_l.cols, W_l.ld)) || overlap(Y, ybytes, workspace, ws_bytes) ||
        overlap(X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < gatv2_ws(*A, (int)X.cols, (int)W_r.cols, comp_id, false)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return SENSEI_OK;
    return run_gatv2(*A, X, W_l, W_r, att, neg_slope, Y, ldy, activation, comp_id, workspace, ws_bytes, as_stream(stream), &ctx->timers);
}

int sensei_dotgat_workspace(const sensei_csr *A, int f_in, int d_k, int f_out, int comp_id, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || d_k <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    *bytes = dotgat_ws(*A, f_in, d_k, f_out, comp_id);
    return SENSEI_OK;
}

int sensei_dotgat_layer(sensei_ctx *ctx, const sensei_csr *A, sensei_mat X, sensei_mat W_q, sensei_mat W_k, sensei_mat W_v, float scale, float *Y,
                        int64_t ldy, int activation, int comp_id, void *workspace, size_t ws_bytes, void *stream) {
    if (comp_id != 0 && comp_id != 1) return SENSEI_INVALID_COMPOSITION;
    if (!ctx || !csr_ok(A, false) || !mat_ok(X) || !mat_ok(W_q) || !mat_ok(W_k) || !mat_ok(W_v)) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (A->n_rows > A->n_cols || X.rows != A->n_cols || X.cols <= 0 || W_q.rows != X.cols || W_k.rows != X.cols || W_v.rows != X.cols ||
        W_q.cols <= 0 || W_q.cols != W_k.cols || W_v.cols <= 0 || ldy < W_v.cols)
        return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W_q.cols > (1 << 20) || W_v.cols > (1 << 20)) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W_q.ptr || !W_k.ptr || !W_v.ptr || (!Y && A->n_rows > 0) || !workspace) return SENSEI_INVALID_ARGUMENT;
    const size_t ybytes = mat_bytes(Y, A->n_rows, W_v.cols, ldy);
    if (overlap(Y, ybytes, X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)) || overlap(Y, ybytes, workspace, ws_bytes) ||
        overlap(X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld), workspace, ws_bytes))
        return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < dotgat_ws(*A, (int)X.cols, (int)W_q.cols, (int)W_v.cols, comp_id)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) return SENSEI_OK;
    return run_dotgat(*A, X, W_q, W_k, W_v, scale, Y, ldy, activation, comp_id, workspace, ws_bytes, as_stream(stream), &ctx->timers);
}

int sensei_dotgat_backward_workspace(const sensei_csr *A, int f_in, int d_k, int f_out, size_t *bytes) {
    if (!csr_ok(A, false) || f_in <= 0 || d_k <= 0 || f_out <= 0 || !bytes) return SENSEI_INVALID_ARGUMENT;
    *bytes = dotgat_bwd_ws(*A, f_in, d_k, f_out);
    return SENSEI_OK;
}

int sensei_dotgat_backward(sensei_ctx *ctx, const sensei_csr *A, const sensei_csr *At, const int32_t *t_pos, sensei_mat X, sensei_mat W_q,
                           sensei_mat W_k, sensei_mat W_v, float scale, const float *Y, int64_t ldy, sensei_mat dY, int activation, float *dX,
                           int64_t lddx, float *dW_q, int64_t lddwq, float *dW_k, int64_t lddwk, float *dW_v, int64_t lddwv, void *workspace,
                           size_t ws_bytes, void *stream) {
    if (!ctx || !csr_ok(A, false) || !csr_ok(At, false) || !mat_ok(X) || !mat_ok(W_q) || !mat_ok(W_k) || !mat_ok(W_v) || !mat_ok(dY))
        return SENSEI_INVALID_ARGUMENT;
    if (At->n_rows != A->n_cols || At->n_cols != A->n_rows || At->nnz != A->nnz || A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    if (activation != SENSEI_ACT_NONE && activation != SENSEI_ACT_RELU) return SENSEI_INVALID_ARGUMENT;
    if (X.rows != A->n_cols || X.cols <= 0 || W_q.rows != X.cols || W_k.rows != X.cols || W_v.rows != X.cols || W_q.cols <= 0 ||
        W_q.cols != W_k.cols || W_v.cols <= 0)
        return SENSEI_INVALID_ARGUMENT;
    if (X.cols > (1 << 20) || W_q.cols > (1 << 18) || W_v.cols > (1 << 18)) return SENSEI_INVALID_ARGUMENT;
    if (dY.rows != A->n_rows || dY.cols != W_v.cols) return SENSEI_INVALID_ARGUMENT;
    if ((!X.ptr && A->n_cols > 0) || !W_q.ptr || !W_k.ptr || !W_v.ptr || (!dY.ptr && A->n_rows > 0) || !dW_q || !dW_k || !dW_v || !workspace)
        return SENSEI_INVALID_ARGUMENT;
    if (!t_pos && A->nnz > 0) return SENSEI_INVALID_ARGUMENT;
    if (lddwq < W_q.cols || lddwk < W_k.cols || lddwv < W_v.cols || (dX && lddx < X.cols)) return SENSEI_INVALID_ARGUMENT;
    if (activation == SENSEI_ACT_RELU && ((!Y && A->n_rows > 0) || ldy < W_v.cols)) return SENSEI_INVALID_ARGUMENT;
    struct Buf { const void *p; size_t n; };
    const Buf ins[5] = {{X.ptr, mat_bytes(X.ptr, X.rows, X.cols, X.ld)}, {dY.ptr, mat_bytes(dY.ptr, dY.rows, dY.cols, dY.ld)},
                        {W_q.ptr, mat_bytes(W_q.ptr, W_q.rows, W_q.cols, W_q.ld)}, {W_k.ptr, mat_bytes(W_k.ptr, W_k.rows, W_k.cols, W_k.ld)},
                        {W_v.ptr, mat_bytes(W_v.ptr, W_v.rows, W_v.cols, W_v.ld)}};
    const Buf outs[4] = {{dW_q, mat_bytes(dW_q, W_q.rows, W_q.cols, lddwq)}, {dW_k, mat_bytes(dW_k, W_k.rows, W_k.cols, lddwk)},
                         {dW_v, mat_bytes(dW_v, W_v.rows, W_v.cols, lddwv)}, {dX, dX ? mat_bytes(dX, A->n_cols, X.cols, lddx) : 0}};
    for (int a = 0; a < 4; ++a) {
        if (overlap(outs[a].p, outs[a].n, workspace, ws_bytes)) return SENSEI_INVALID_ARGUMENT;
        for (int b = 0; b < 5; ++b)
            if (overlap(outs[a].p, outs[a].n, ins[b].p, ins[b].n)) return SENSEI_INVALID_ARGUMENT;
        for (int b = a + 1; b < 4; ++b)
            if (overlap(outs[a].p, outs[a].n, outs[b].p, outs[b].n)) return SENSEI_INVALID_ARGUMENT;
    }
    if (ws_bytes < dotgat_bwd_ws(*A, (int)X.cols, (int)W_q.cols, (int)W_v.cols)) return SENSEI_WORKSPACE_TOO_SMALL;
    if (A->n_rows == 0) {   // no output rows: nothing depends on the inputs
        hipStream_t st = as_stream(stream);
        if (launch_zero_matrix(dW_q, W_q.rows, (int)W_q.cols, lddwq, false, st) != hipSuccess ||
            launch_zero_matrix(dW_k, W_k.rows, (int)W_k.cols, lddwk, false, st) != hipSuccess ||
            launch_zero_matrix(dW_v, W_v.rows, (int)W_v.cols, lddwv, false, st) != hipSuccess ||
            (dX && launch_zero_matrix(dX, A->n_cols, (int)X.cols, lddx, false, st) != hipSuccess))
            return SENSEI_HIP_ERROR;
        return SENSEI_OK;
    }
    return run_dotgat_backward(*A, *At, t_pos, X, W_q, W_k, W_v, scale, Y, ldy, dY, activation, dX, lddx, dW_q, lddwq, dW_k, lddwk, dW_v, lddwv,
                               workspace, ws_bytes, as_stream(stream));
}

int sensei_select_workspace(int kind, const sensei_csr *A, int f_in, int f_out, size_t *bytes) {
    if ((kind != SENSEI_KIND_GCN && kind != SENSEI_KIND_GAT) || !csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bytes)
        return SENSEI_INVALID_ARGUMENT;
    *bytes = select_scratch_bytes(kind, *A, f_in, f_out);  // covers the 256 bytes of learned mode
    return SENSEI_OK;
}

int sensei_select_gcn_backward(sensei_ctx *ctx, const sensei_csr *A, int f_in, int f_out, int have_saved_u, int want_dx,
                               int *bwd_id_out, float *est_ms) {
    if (!ctx || !csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !bwd_id_out) return SENSEI_INVALID_ARGUMENT;
    Features g;
    g.n_rows = A->n_rows; g.n_cols = A->n_cols; g.nnz = (double)A->nnz;
    g.density = (A->n_rows > 0 && A->n_cols > 0) ? g.nnz / (g.n_rows * g.n_cols) : 0.0;
    double cost[2];
    for (int id = 0; id < 2; ++id) {
        cost[id] = 1e3 * gcn_bwd_cost(*ctx, g, f_in, f_out, id, have_saved_u != 0, want_dx != 0);
        if (est_ms) est_ms[id] = (float)cost[id];
    }
    *bwd_id_out = cost[SENSEI_GCN_BWD_UPD] < cost[SENSEI_GCN_BWD_AGG] ? SENSEI_GCN_BWD_UPD : SENSEI_GCN_BWD_AGG;
    return SENSEI_OK;
}

int sensei_select_khop_backward(sensei_ctx *ctx, const sensei_csr *A, int f_in, int f_out, int k_hops, int per_hop_weights, int want_dx,
                                int *bwd_id_out, float *est_ms) {
    if (!ctx || !csr_ok(A, false) || f_in <= 0 || f_out <= 0 || k_hops < 0 || k_hops > 64 || !bwd_id_out) return SENSEI_INVALID_ARGUMENT;
    Features g;
    g.n_rows = A->n_rows; g.n_cols = A->n_cols; g.nnz = (double)A->nnz;
    g.density = (A->n_rows > 0 && A->n_cols > 0) ? g.nnz / (g.n_rows * g.n_cols) : 0.0;
    double cost[2];
    for (int id = 0; id < 2; ++id) {
        cost[id] = 1e3 * khop_bwd_cost(*ctx, g, f_in, f_out, k_hops, per_hop_weights != 0, id, want_dx != 0);
        if (est_ms) est_ms[id] = (float)cost[id];
    }
    *bwd_id_out = cost[SENSEI_GCN_BWD_UPD] < cost[SENSEI_GCN_BWD_AGG] ? SENSEI_GCN_BWD_UPD : SENSEI_GCN_BWD_AGG;
    return SENSEI_OK;
}

// The "run every candidate once, keep the fastest" trial over the ids with try_id set: scratch operands in `workspace` (constants
// stand in for the scalings and for N~: their values do not change what a trial costs), one run per candidate bracketed by events.
// A first run is slower than the ones after it (code objects, clocks, cold caches) by tens of microseconds, which decides the
// order of candidates that take a fraction of a millisecond and is noise for the others: a candidate measured under
// kRetimeBelowMs is run and measured a second time and the second figure kept, so every candidate's figure comes from a warm run
// where that matters while a trial of long layers stays at one run per candidate.  measured[id] (ms) is written for the ids tried.
static constexpr float kRetimeBelowMs = 0.5f;
static int timed_trial(int kind, const sensei_csr &A, int f_in, int f_out, const bool *try_id, double *measured, void *workspace,
                       size_t ws_bytes, hipStream_t s) {
    const int n = kind == SENSEI_KIND_GCN ? kNumGcn : kNumGat;
    Carver cv(workspace, ws_bytes);
    float *X = cv.take<float>((size_t)A.n_cols * f_in);
    float *W = cv.take<float>((size_t)f_in * f_out);
    float *Y = cv.take<float>((size_t)A.n_rows * f_out);
    float *r = cv.take<float>((size_t)A.n_rows + A.n_cols);
    float *c = r + A.n_rows;
    (void)cv.take<int32_t>((size_t)A.n_rows + A.n_cols);
    float *nt = cv.take<float>((size_t)(A.nnz > 0 ? A.nnz : 1));
    float *a_l = cv.take<float>((size_t)f_out);
    float *a_r = cv.take<float>((size_t)f_out);
    void *lws = cv.base + cv.used;
    const size_t lws_bytes = ws_bytes - cv.used;
    SENSEI_TRY(fill(X, (size_t)A.n_cols * f_in, 0.25f, s));
    SENSEI_TRY(fill(W, (size_t)f_in * f_out, 0.01f, s));
    SENSEI_TRY(fill(a_l, (size_t)f_out, 0.05f, s));
    SENSEI_TRY(fill(a_r, (size_t)f_out, 0.05f, s));
    SENSEI_TRY(fill(r, (size_t)A.n_rows + A.n_cols, 0.05f, s));
    sensei_csr Aw = A;
    if (kind == SENSEI_KIND_GCN) {
        SENSEI_TRY(fill(nt, (size_t)(A.nnz > 0 ? A.nnz : 1), 0.0025f, s));
        Aw.val = nt;
    }
    sensei_mat Xm = {X, A.n_cols, f_in, f_in}, Wm = {W, f_in, f_out, f_out};
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SENSEI_HIP_ERROR;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SENSEI_HIP_ERROR; }
    int status = SENSEI_OK;
    for (int id = 0; id < n && status == SENSEI_OK; ++id) {
        if (!try_id[id]) continue;
        float ms = 0.f;
        for (int rep = 0; rep < 2 && status == SENSEI_OK; ++rep) {
            if (hipEventRecord(e0, s) != hipSuccess) status = SENSEI_HIP_ERROR;
            if (status == SENSEI_OK)
                status = kind == SENSEI_KIND_GCN
                             ? run_gcn(Aw, r, c, Xm, Wm, Y, f_out, SENSEI_ACT_RELU, id, lws, lws_bytes, s, nullptr)
                             : run_gat(A, Xm, Wm, a_l, a_r, 0.2f, Y, f_out, SENSEI_ACT_RELU, id, lws, lws_bytes, s, nullptr);
            if (status != SENSEI_OK) break;
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
                status = SENSEI_HIP_ERROR;
            if (ms >= kRetimeBelowMs) break;  // a long layer: its first run is representative
        }
        measured[id] = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return status;
}

int sensei_select(sensei_ctx *ctx, int kind, const sensei_csr *A, int f_in, int f_out, int mode, int *comp_id_out,
                  float *est_ms, void *workspace, size_t ws_bytes, void *stream) {
    if (!ctx || (kind != SENSEI_KIND_GCN && kind != SENSEI_KIND_GAT) || !csr_ok(A, false) || f_in <= 0 || f_out <= 0 || !comp_id_out)
        return SENSEI_INVALID_ARGUMENT;
    if (mode != SENSEI_SELECT_MODEL && mode != SENSEI_SELECT_TIMED && mode != SENSEI_SELECT_LEARNED && mode != SENSEI_SELECT_AUTO)
        return SENSEI_INVALID_ARGUMENT;
    if (kind == SENSEI_KIND_GAT && A->n_rows > A->n_cols) return SENSEI_INVALID_ARGUMENT;
    const int n = kind == SENSEI_KIND_GCN ? kNumGcn : kNumGat;
    bool keep[8];
    rule_filter(kind, f_in, f_out, keep);
    double cost[8];
    for (int id = 0; id < n; ++id) cost[id] = -1.0;

    if (mode != SENSEI_SELECT_TIMED) {
        Features g;
        g.n_rows = A->n_rows; g.n_cols = A->n_cols; g.nnz = (double)A->nnz;
        g.density = (A->n_rows > 0 && A->n_cols > 0) ? g.nnz / (g.n_rows * g.n_cols) : 0.0;
        const sensei_tiles *D = A->tiles;  // a split made for this very pattern changes what the value-less and attention SpMMs cost
        if (D && D->T.n_slots > 0 && A->nnz > 0 && D->n_rows == A->n_rows && D->n_cols == A->n_cols && D->nnz == A->nnz &&
            D->src_row_ptr == A->row_ptr && D->src_col_idx == A->col_idx) {
            g.tile_share = (double)(A->nnz - D->nnz_rem) / (double)A->nnz;
            g.tile_min_width = D->min_width;
            g.tile_max_width = D->max_width;
        }
        if (mode == SENSEI_SELECT_LEARNED) {  // graph feature extractor: two exact integer reductions over row_ptr
            if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 8 != 0) return SENSEI_INVALID_ARGUMENT;
            if (ws_bytes < 256) return SENSEI_WORKSPACE_TOO_SMALL;
            hipStream_t s = as_stream(stream);
            unsigned long long *dev2 = static_cast<unsigned long long *>(workspace), host2[2] = {0, 0};
            if (launch_row_moments(*A, dev2, s) != hipSuccess ||
                hipMemcpyAsync(host2, dev2, sizeof(host2), hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
                return SENSEI_HIP_ERROR;
            g.max_row = (double)host2[0];
            g.sum_sq_row = (double)host2[1];
            g.learned = true;
        }
        for (int id = 0; id < n; ++id)
            if (keep[id]) cost[id] = 1e3 * (kind == SENSEI_KIND_GCN ? gcn_cost(*ctx, g, f_in, f_out, id) : gat_cost(*ctx, g, f_in, f_out, id));
        if (mode == SENSEI_SELECT_AUTO) {
            // candidates the model cannot separate (within kAutoMargin of its cheapest) are settled by a timed trial among them
            double best = -1.0;
            for (int id = 0; id < n; ++id)
                if (keep[id] && (best < 0.0 || cost[id] < best)) best = cost[id];
            bool close[8];
            int n_close = 0;
            for (int id = 0; id < n; ++id) {
                close[id] = keep[id] && cost[id] <= best * (1.0 + kAutoMargin);
                n_close += close[id] ? 1 : 0;
            }
            if (n_close > 1 && workspace && ws_bytes >= select_scratch_bytes(kind, *A, f_in, f_out)) {
                double measured[8];
                const int st = timed_trial(kind, *A, f_in, f_out, close, measured, workspace, ws_bytes, as_stream(stream));
                if (st != SENSEI_OK) return st;
                // only the tried ids stay candidates; the others keep their prediction in est_ms but cannot win
                for (int id = 0; id < n; ++id) {
                    if (close[id]) cost[id] = measured[id];
                    else keep[id] = false;
                }
            }
        }
    } else {
        if (!workspace) return SENSEI_INVALID_ARGUMENT;
        if (ws_bytes < select_scratch_bytes(kind, *A, f_in, f_out)) return SENSEI_WORKSPACE_TOO_SMALL;
        const int st = timed_trial(kind, *A, f_in, f_out, keep, cost, workspace, ws_bytes, as_stream(stream));
        if (st != SENSEI_OK) return st;
    }
    int best = -1;
    for (int id = 0; id < n; ++id)
        if (keep[id] && cost[id] >= 0.0 && (best < 0 || cost[id] < cost[best])) best = id;
    if (best < 0) return SENSEI_UNSUPPORTED;
    *comp_id_out = best;
    if (est_ms) for (int id = 0; id < n; ++id) est_ms[id] = (float)cost[id];
    return SENSEI_OK;
}

int sensei_calibrate(sensei_ctx *ctx, void *workspace, size_t ws_bytes, void *stream) {
    if (!ctx || !workspace) return SENSEI_INVALID_ARGUMENT;
    if (ws_bytes < (64u << 20)) return SENSEI_WORKSPACE_TOO_SMALL;
    hipStream_t s = as_stream(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return SENSEI_HIP_ERROR;
    int status = SENSEI_OK;
    float ms = 0.f;
    // streaming rate: scale a 32 MiB matrix into the other half of the workspace
    {
        float *src = static_cast<float *>(workspace);
        float *dst = src + (8u << 20);
        const int64_t rows = 8192, cols = 1024;
        if (launch_row_broadcast(nullptr, src, cols, rows, (int)cols, dst, cols, SENSEI_ACT_NONE, s) != hipSuccess) status = SENSEI_HIP_ERROR;
        (void)hipEventRecord(e0, s);
        for (int it = 0; it < 10 && status == SENSEI_OK; ++it)
            if (launch_row_broadcast(nullptr, src, cols, rows, (int)cols, dst, cols, SENSEI_ACT_NONE, s) != hipSuccess) status = SENSEI_HIP_ERROR;
        (void)hipEventRecord(e1, s);
        if (status == SENSEI_OK && (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) status = SENSEI_HIP_ERROR;
        if (status == SENSEI_OK && ms > 0.f) ctx->stream_bps = 10.0 * 2.0 * rows * cols * 4.0 / (ms * 1e-3);
    }
    // launch latency: empty-sized element-wise launches back to back
    if (status == SENSEI_OK) {
        float *src = static_cast<float *>(workspace);
        (void)hipEventRecord(e0, s);
        for (int it = 0; it < 100 && status == SENSEI_OK; ++it)
            if (launch_row_broadcast(nullptr, src, 4, 64, 4, src + 1024, 4, SENSEI_ACT_NONE, s) != hipSuccess) status = SENSEI_HIP_ERROR;
        (void)hipEventRecord(e1, s);
        if (status == SENSEI_OK && (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) status = SENSEI_HIP_ERROR;
        if (status == SENSEI_OK && ms > 0.f) ctx->launch_us = ms * 1e3 / 100.0;
    }
    // GEMM rate: 16384 x 256 x 256 on scratch
    if (status == SENSEI_OK) {
        float *a = static_cast<float *>(workspace);
        float *w = a + (size_t)16384 * 256;
        float *y = w + (size_t)256 * 256;
        (void)fill(a, (size_t)16384 * 256, 0.1f, s);
        (void)fill(w, (size_t)256 * 256, 0.1f, s);
        (void)launch_gemm(a, 256, w, 256, y, 256, 16384, 256, 256, 256, SENSEI_ACT_NONE, s);
        (void)hipEventRecord(e0, s);
        for (int it = 0; it < 10 && status == SENSEI_OK; ++it)
            if (launch_gemm(a, 256, w, 256, y, 256, 16384, 256, 256, 256, SENSEI_ACT_NONE, s) != hipSuccess) status = SENSEI_HIP_ERROR;
        (void)hipEventRecord(e1, s);
        if (status == SENSEI_OK && (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) status = SENSEI_HIP_ERROR;
        const double t = ms * 1e-3 / 10.0 - ctx->launch_us * 1e-6;
        if (status == SENSEI_OK && t > 0.0) ctx->gemm_flops = 2.0 * 16384 * 256 * 256 / t;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return status;
}

}  // extern "C"
