// Internal declarations shared by the HIP translation units of libsensei_hip.
// Host-side launchers only; every launcher validates nothing (the C ABI layer
// in api.hip does) and returns the hipError_t of its launches.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "sensei.h"

namespace sensei {

// ---- partition of the non-zeros into fixed-size chunks (one wavefront each)

struct ChunkPlan {
    int chunk_nnz;        // T: non-zeros per chunk, multiple of 64
    int n_chunks;         // max(1, ceil(nnz / T))
    int32_t *chunk_row;   // device, n_chunks + 1: first row starting at or after c*T; [n_chunks] = n_rows
};

int choose_chunk_nnz(int64_t nnz);
size_t plan_bytes(int64_t nnz);  // upper bound over all chunk sizes
hipError_t launch_chunk_rows(const sensei_csr &A, const ChunkPlan &p, hipStream_t s);

// ---- optional timing of a kernel's launches with HIP events on the launch stream
struct KernelTimer {
    bool enabled = false;
    size_t used = 0;                 // events handed out since the recording started
    std::vector<hipEvent_t> events;  // start/stop pairs, created on first use, reused afterwards
    static constexpr size_t kMaxEvents = 8192;
    hipEvent_t next() {
        if (!enabled || used >= kMaxEvents) return nullptr;
        if (used == events.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return nullptr;
            events.push_back(e);
        }
        return events[used++];
    }
};

struct Timers {
    KernelTimer spmm, gemm;
};

// ---- SpMM

struct AttnFusedArgs;
struct SpmmShape {
    int vec;      // floats per lane load: 4, 2 or 1
    int lpg;      // lanes per neighbour group: 8, 16, 32 or 64
    int n_tiles;  // feature tiles of vec*lpg floats
    int f_carry;  // n_tiles * vec * lpg
};
SpmmShape spmm_shape(const float *B, int64_t ldb, int f);
size_t spmm_carry_bytes(int64_t nnz, int f);  // upper bound
// C[i, 0:f_store) = act(r_i * sum_j w_ij B[j, 0:f)); f_store <= f.  w_ij = 1 (PATTERN), val (WEIGHTED) or
// c_j (SCALED); the row factor r is applied whenever r is non-null, in every mode.
hipError_t launch_spmm(const sensei_csr &A, int mode, const float *r, const float *c, const float *B, int64_t ldb,
                       int f, float *C, int64_t ldc, int f_store, int act, const ChunkPlan &p, float *carry,
                       hipStream_t s, KernelTimer *timer = nullptr, bool accumulate = false, bool finalize = true,
                       const float2 *mz = nullptr, bool b_sliced = false, int val_stride = 1, bool c_sliced = false, bool defer_fixup = false,
                       const struct AttnFusedArgs *fused = nullptr, const struct SelfSumArgs *self = nullptr);
// b_sliced: B is stored slice-major in tiles of 32 floats, element (j, col) at B[(col / 32) * n_cols * 32 + j * 32 + col % 32]
// (f padded to a multiple of 32, B 128-byte aligned); `ldb` is ignored.  val_stride: floats between consecutive values of A.val.
// c_sliced (needs b_sliced, f a multiple of 32, f_store == f): C is written slice-major too (n_rows x f), `ldc` is ignored.
// defer_fixup (with finalize = false and a slice-major B): the pass that adds the carry slots of rows spanning chunk boundaries is
// left to the caller (launch_tiles_combine does it); the slots are pad32(f) floats apart.
inline size_t sliced_index(int64_t n_rows, int64_t row, int col) { return (size_t)(col >> 5) * (size_t)n_rows * 32 + (size_t)row * 32 + (col & 31); }
// Internal SpMM mode (not part of the C ABI): A.val holds attention logits e_ij, `mz[i]` = (max_j e_ij, sum_j exp(e_ij - max));
// the kernel weighs neighbour j of row i by exp(e_ij - max_i) and scales the finished row by 1 / sum, i.e. it aggregates
// with the softmax weights of Eq. 6 without storing them.
constexpr int kSpmmSoftmax = 3;
// Internal SpMM mode: the attention aggregation of Eq. 5-6 in one walk, nothing stored per entry.  The weight of entry (i, j) is the
// softmax over row i of LeakyReLU(s_l[i] + s_r[j]), formed with a running maximum while the neighbours are gathered.  row_mz
// (n_rows + 1 pairs) and chunk_mz (one pair per chunk) are scratch for the rows that span chunks.  Single pass only (no column
// panels, no deferred fix-up); A.val is not read.
constexpr int kSpmmAttnFused = 4;
struct AttnFusedArgs {
    const float *s_l, *s_r;
    float slope;
    float2 *row_mz, *chunk_mz;
};
// Internal SpMM modes for the backward pass of a score with a vector per entry, e_ij = att . LeakyReLU(U_ij), U_ij = self[i, :] + B[j, :]
// (slice-major self over the rows and B over the columns): C[i, m] = sum_j val_ij LeakyReLU'(U_ij[m]) (kSpmmSignSum: 1 where
// U > 0, else the slope) or sum_j val_ij LeakyReLU(U_ij[m]) (kSpmmLreluSum).  Single pass, slice-major B only.
constexpr int kSpmmSignSum = 5;
constexpr int kSpmmLreluSum = 6;
struct SelfSumArgs {
    const float *self_sliced;
    float slope;
};

// ---- column panels: a copy of the pattern with the columns of each panel contiguous
#define SENSEI_MAX_PANELS SENSEI_PANELS_MAX
size_t scan_temp_bytes(int n);
// rp[q]: n_rows + 1 ints per panel (row pointers of the panel copy on return); off: n_panels + 1 ints (panel starts in
// col_out); perm_out[k] = position of original entry k in the panel copy; `plan` is the chunk plan of A (already computed
// on the stream).
hipError_t launch_panel_build(const sensei_csr &A, const ChunkPlan &plan, int n_panels, int width, int32_t *const *rp, int32_t *off,
                              int32_t *col_out, int32_t *perm_out, int32_t *scan_temp, hipStream_t s);

// seg_ptr (n_panels * n_rows + 1): the panel copy as one CSR over the segments (panel q, row i) -> q * n_rows + i, from the
// per-panel row pointers rp and the panel starts off that launch_panel_build left
hipError_t launch_panel_segments(int32_t *const *rp, const int32_t *off, int n_rows, int n_panels, int32_t *seg_ptr, hipStream_t s);
// dst[q * n + i] = src[i] for q < copies
hipError_t launch_replicate_stats(const float2 *src, int64_t n, int copies, float2 *dst, hipStream_t s);

// ---- element-wise work over the non-zeros, degrees, scalings
hipError_t launch_degrees(const sensei_csr &A, int32_t *deg_row, int32_t *deg_col, hipStream_t s);
hipError_t launch_norm_vectors(const int32_t *deg, int64_t n, float *out, hipStream_t s);
hipError_t launch_sddmm_norm(const sensei_csr &A, const float *r, const float *c, float *val, const ChunkPlan &p,
                             hipStream_t s);
// mask (optional, n x f, ldm): elements whose mask value is not > 0 are written as 0 (backward of ReLU)
hipError_t launch_row_broadcast(const float *s_vec, const float *X, int64_t ldx, int64_t n, int f, float *Y,
                                int64_t ldy, int act, hipStream_t s, const float *mask = nullptr, int64_t ldm = 0);

// Y (slice-major, pad32(f) columns, 128-byte aligned, n * pad32(f) floats) = s_vec (x) X, s_vec optional; pad columns = 0
hipError_t launch_to_slices(const float *s_vec, const float *X, int64_t ldx, int64_t n, int f, float *Y, hipStream_t s,
                            const float *mask = nullptr, int64_t ldm = 0);

// ---- attention: logits, per-row softmax statistics, normalised weights
hipError_t launch_score(const sensei_csr &A, const float *s_l, const float *s_r, float slope, float *e,
                        const ChunkPlan &p, hipStream_t s);
// alpha = row-wise softmax of the logits e (in place allowed); stats[i] = (row max, sum of exp(e - max)) as a by-product.
hipError_t launch_softmax(const sensei_csr &A, const float *e, float *alpha, const ChunkPlan &p, float2 *stats, float2 *carry_stats,
                          hipStream_t s);
// Logits e_ij = LeakyReLU(s_l[i] + s_r[j]) of every stored entry, written to logits[k] (or logits[dst_index[k]]), and the
// statistics stats[i] = (row max, sum of exp(e - max)) that kSpmmSoftmax needs.
// A negative dst_index[k] keeps entry k out of `logits` (it lies in a dense tile); the statistics always cover every entry.
hipError_t launch_attention_stats(const sensei_csr &A, const float *s_l, const float *s_r, float slope, float *logits,
                                  const int32_t *dst_index, const ChunkPlan &p, float2 *stats, float2 *carry_stats, hipStream_t s);
size_t softmax_ws_bytes(const sensei_csr &A);

// ---- backward of the attention layer
// out[i] = sum of val[k * stride] over the entries k of row i; carry: n_chunks floats
hipError_t launch_row_sum(const sensei_csr &A, const float *val, int stride, float *out, const ChunkPlan &p, float *carry, hipStream_t s);
// dalpha[k] = <dP[i,:], Theta[j,:]> per stored entry, rowdot[i] = sum_j alpha_ij dalpha_ij (skipped when rowdot is null); theta, dP slice-major
hipError_t launch_gat_dalpha(const sensei_csr &A, const float *theta, const float *dP, int f, const float *logits, const float2 *mz,
                             float *dalpha, float *rowdot, const ChunkPlan &p, float *carry, hipStream_t s, float scale = 1.f);
// (with rowdot null and a scale it is the key-query score of an attention layer: dalpha[k] = scale <dP[i,:], theta[j,:]>)
// dense-tile split: dalpha[k] from the remainder's values (where[k] >= 0) or the cells of the tiles' product Dt (where[k] < 0), and rowdot
hipError_t launch_gat_dalpha_merge(const sensei_csr &A, const int32_t *where, const float *dalpha_rem, const float *Dt, const float *logits,
                                   const float2 *mz, float *dalpha, float *rowdot, const ChunkPlan &p, float *carry, hipStream_t s);
// dt[k] = alpha (dalpha - rowdot_i) LeakyReLU'(e); dt may be dalpha; adt_t[t_pos[k]] = (alpha, dt)
hipError_t launch_gat_dt(const sensei_csr &A, const float *logits, const float *dalpha, const float *rowdot, const float2 *mz,
                         const int32_t *t_pos, float slope, float *dt, float2 *adt_t, const ChunkPlan &p, hipStream_t s);
// logits[k] = sum_m att[m] LeakyReLU(theta_l[i, m] + theta_r[j, m]) per stored entry (i, j); both matrices slice-major
// (n_rows x pad32(f), n_cols x pad32(f)), att padded with zeros to pad32(f)
hipError_t launch_score_v2(const sensei_csr &A, const float *theta_l, const float *theta_r, int f, const float *att_padded, float slope,
                           float *logits, const ChunkPlan &p, hipStream_t s);
hipError_t launch_rank1_add(float *D, int64_t ldd, int64_t n, int f, const float *ds_l, int64_t n_l, const float *ds_r, const float *a_l,
                            const float *a_r, hipStream_t s);
// out_l = Theta^T v_l (v_l counted for the first n_l rows), out_r = Theta^T v_r; Theta slice-major n x pad32(f); sums in fp64
// D[i, m] = (accumulate ? D[i, m] : 0) + v[m] G[i, m] over n rows and f columns (G may be D)
hipError_t launch_scale_cols(float *D, int64_t ldd, const float *G, int64_t ldg, const float *v, int64_t n, int f, bool accumulate, hipStream_t s);
hipError_t launch_fill_f32(float *p, int64_t n, float v, hipStream_t s);
size_t theta_t_vec_bytes(int64_t n, int f);
hipError_t launch_theta_t_vec(const float *theta_sliced, int64_t n, int f, const float *v_l, int64_t n_l, const float *v_r, float *out_l,
                              float *out_r, double *part, hipStream_t s);
// pos[k] = place of entry k of A in At (binary search in the ascending columns of At); *miss (cleared first) counts entries not found
hipError_t launch_transpose_pos(const sensei_csr &A, const sensei_csr &At, const ChunkPlan &p, int32_t *pos, int32_t *miss, hipStream_t s);

// out[i] = 1 / v[i]
hipError_t launch_reciprocal(const float *v, int64_t n, float *out, hipStream_t s);
// out ((hops * pad32(f_in)) x f_out, ldo): block h holds rows h*f_in .. of W followed by zero rows up to pad32(f_in)
hipError_t launch_stack_weights(const float *W, int64_t ldw, int hops, int f_in, int f_out, float *out, int64_t ldo, hipStream_t s);

// out2[0] = largest row length, out2[1] = sum of squared row lengths (device, 16 bytes)
hipError_t launch_row_moments(const sensei_csr &A, unsigned long long *out2, hipStream_t s);

// ---- dense tiles of the hub region (nodes ranked by degree; tiles of 128 x 128 ranks kept as bit masks)
struct TileSplit {
    int nt_r, nt_c;                    // tiles per side of the tiled region
    int n_slots;                       // kept tiles
    const int32_t *order_r, *order_c;  // device, nt * 128: node at rank, -1 beyond the last node
    const int32_t *rt_ptr, *slot_ct;   // device: first slot of each row of tiles (nt_r + 1), column tile of each slot
    const int32_t *slot_rt;            // device: row of tiles of each slot
    const unsigned *bits;              // device: n_slots x 128 x 4 words
    int n_seg;                         // segments of at most kTilesPerSegment consecutive slots of one row of tiles
    const int32_t *seg_first, *rt_seg; // device: first slot of each segment (n_seg + 1); first segment of each row of tiles (nt_r + 1)
    const int32_t *seg_rt;             // device: row of tiles of each segment
    float *part;                       // device: n_seg x 128 x (widest operand) partial products
    float *rank_vec;                   // device: 2 * (nt_r + nt_c) * 128 floats for the attention vectors in rank order
    float2 *seg_stats;                 // device: n_seg x 128 (max, sum of exp) pairs of the attention logits inside the tiles
    float *dh;                         // device: nt_r * 128 x (widest operand): the tiles' product, by row rank
    const int32_t *rank_r;             // device: rank of every row node (INT_MAX outside the tiled region)
};
constexpr int kTilesPerSegment = 16;
constexpr int kMaxCellSlots = 131071;  // slots whose cells (slot * 16384 + ...) + 1 still fit a positive int32
size_t scan_large_temp_bytes(long long n);
hipError_t launch_exclusive_scan_large(int32_t *data, long long n, int32_t *temp, hipStream_t s);
// histogram of the entries per tile, choice of the tiles with at least min_count entries, slot tables; sel_scan: n_tiles + 1 ints
// (its last element is the number of kept tiles), scan_temp: scan_temp_bytes(n_tiles + 1)
hipError_t launch_tile_select(const sensei_csr &A, const ChunkPlan &p, const int32_t *rank_r, const int32_t *rank_c, int h_r, int h_c,
                              int nt_r, int nt_c, int min_count, int32_t *hist, int32_t *sel_scan, int32_t *slot_of, int32_t *slot_ct,
                              int32_t *slot_rt, int32_t *rt_ptr, int32_t *scan_temp, hipStream_t s);
// bit masks of the kept tiles and the CSR of everything else; pos: nnz + 1 ints of scratch (pos[nnz] = size of the remainder on
// return), scan_temp: scan_large_temp_bytes(nnz + 1); dst_rem[k] = place of entry k of A in the remainder, or, negative,
// -(cell + 1) with cell = (slot * 128 + row in tile) * 128 + column in tile for an entry inside a kept tile (-1 beyond kMaxCellSlots)
hipError_t launch_tile_split(const sensei_csr &A, const ChunkPlan &p, const int32_t *rank_r, const int32_t *rank_c, int h_r, int h_c, int nt_c,
                             const int32_t *slot_of, int n_slots, unsigned *bits, int32_t *pos, int32_t *scan_temp, int32_t *col_rem,
                             int32_t *dst_rem, int32_t *row_ptr_rem, hipStream_t s);
hipError_t launch_zero_matrix(float *C, int64_t n, int f, int64_t ldc, bool sliced, hipStream_t s);
// out[dst_rem[k]] = src[k * stride] for the entries k of the pattern that stay in the sparse remainder (dst_rem[k] >= 0)
hipError_t launch_compact_values(int64_t nnz, const int32_t *dst_rem, const float *src, int stride, float *out, hipStream_t s,
                                 const int32_t *place = nullptr);
// T.dh[rank, 0:f) = (kept tiles of the rank's row of tiles) . B, raw sums; B slice-major with f (a multiple of 32) columns;
// Bh: nt_c * 128 * f floats.  With s_l, s_r, mz (attention mode) entry (i, j) of a tile weighs
// exp(LeakyReLU(s_l[i] + s_r[j]) - mz[i].x) instead of 1.  `transposed` (attention mode only): T holds the tiles of the transposed
// pattern, so its rows are the sources and its columns the destinations: entry (j, i) weighs
// exp(LeakyReLU(s_l[i] + s_r[j]) - mz[i].x) / mz[i].y, the complete coefficient alpha_ij (the division is applied to the rows of B).
hipError_t launch_dense_tiles(const TileSplit &T, const float *B_sliced, int64_t n_cols, int f, float *Bh, hipStream_t s,
                              const float *s_l = nullptr, const float *s_r = nullptr, const float2 *mz = nullptr, float slope = 0.f,
                              bool transposed = false, bool gathered = false, bool local_shift = false);
// local_shift (attention on the pattern itself, after launch_tile_stats on the same stream): the shift of a row is the maximum over its
// tile entries (T.rank_vec + 128 T.nt_r, by row rank), so the tiles can be multiplied before the row statistics of the whole pattern exist;
// the join then rescales their product (tile_shift of the combine launchers).
// the first step of launch_dense_tiles on its own: Bh = rows of B in rank order.  A caller that has other work to wait for can run it
// early and pass gathered = true afterwards (not for the transposed mode, whose rows are scaled while they are gathered).
hipError_t launch_tiles_gather(const TileSplit &T, const float *B_sliced, int64_t n_cols, int f, float *Bh, hipStream_t s);
// Softmax statistics of the attention logits e_ij = LeakyReLU(s_l[i] + s_r[j]) over the entries inside kept tiles: T.seg_stats[seg][row]
// = (max, sum of exp(e - max)) per segment and row of its row of tiles.  launch_tile_stats_merge folds them into stats[i] (which holds
// the pair over the remainder's entries of row i on entry, over all stored entries on return).
hipError_t launch_tile_stats(const TileSplit &T, const float *s_l, const float *s_r, float slope, hipStream_t s);
hipError_t launch_tile_stats_merge(const TileSplit &T, float2 *stats, int64_t n_rows, hipStream_t s);
// Dt[(slot * 128 + i) * 128 + j] = <L[row at rank rt*128+i, 0:f), R[column node at rank ct*128+j, 0:f)> for every kept tile (all
// of its 16384 cells, whether the pattern has them or not; ranks beyond the last node give 0); L and R slice-major with f (a
// multiple of 32) columns; Lh: nt_r * 128 * f floats, Rh: nt_c * 128 * f floats of scratch.
hipError_t launch_tiles_sddmm(const TileSplit &T, const float *L_sliced, int64_t n_rows, const float *R_sliced, int64_t n_cols, int f, float *Lh,
                              float *Rh, float *Dt, hipStream_t s);
// C = act(scale (C + T.dh[rank of the row])) over all rows; scale_i = 1 / mz[i].y if mz, else r[i] if r, else 1
hipError_t launch_tiles_combine(const TileSplit &T, float *C, int64_t n_rows, int f_store, int64_t ldc, bool c_sliced, int f, const float *r,
                                const float2 *mz, int act, hipStream_t s, const int32_t *row_ptr_rem = nullptr, int chunk_nnz = 0,
                                const float *carry = nullptr, int f_carry = 0, const float *tile_shift = nullptr);
// row_ptr_rem, chunk_nnz, carry, f_carry: when the SpMM over the remainder ran with defer_fixup, this pass also adds the carry slots
// (f_carry floats each) of the rows that span chunk boundaries, in chunk order, before anything else.
// The same join when the remainder ran panel-major (its SpMM left one raw partial row per segment (panel q, row i) in `part`,
// slice-major over n_panels * n_rows rows of f floats, fix-up deferred): C = act(scale (sum_q part[q, i] + carries + T.dh[rank])).
hipError_t launch_tiles_combine_pm(const TileSplit &T, float *C, int64_t n_rows, int f_store, int64_t ldc, bool c_sliced, int f, const float *r,
                                   const float2 *mz, int act, hipStream_t s, const float *part, int n_panels, const int32_t *seg_ptr, int chunk_nnz,
                                   const float *carry, int f_carry, const float *tile_shift = nullptr);

// ---- dense
// Y[0:n, 0:m_store) = act(row_scale[i] * (A[n x k] . W[k x m])); columns m..m_store are written as act(0);
// row_scale may be null (no scaling).
bool gemm_uses_pieces(int64_t n, int k, int m_store);   // whether launch_gemm takes the bf16-piece kernel for this shape (ordinary leading dimensions)
hipError_t launch_gemm(const float *A, int64_t lda, const float *W, int64_t ldw, float *Y, int64_t ldy, int64_t n,
                       int k, int m, int m_store, int act, hipStream_t s, const float *row_scale = nullptr,
                       KernelTimer *timer = nullptr, bool y_sliced = false, bool a_sliced = false, const float *add_sliced = nullptr);
// y_sliced / a_sliced: that matrix is stored slice-major in tiles of 32 floats (see launch_spmm); its leading dimension is ignored
// (a slice-major A has k padded to a multiple of 32 in memory; columns k .. are not read).  add_sliced: optional n x pad32(m)
// slice-major matrix added to the product before the row scaling and the activation.
hipError_t launch_gemv2(const float *A, int64_t lda, int64_t n, int k, const float *v1, const float *v2, float *y1,
                        float *y2, hipStream_t s, bool a_sliced = false);

// C[m x n] (row-major, ldc) = A^T . B with A stored k x m and B stored k x n; `part` holds gemm_tn_bytes(k, m, n) bytes.
// The k range is cut into slabs whose partial products are kept and added in fp64, in slab order (deterministic).
size_t gemm_tn_bytes(int64_t k, int m, int n);
hipError_t launch_gemm_tn(const float *A, int64_t lda, const float *B, int64_t ldb, int64_t k, int m, int n, float *C, int64_t ldc,
                          double *part, hipStream_t s);
hipError_t launch_transpose(const float *W, int64_t ldw, int rows, int cols, float *Wt, int64_t ldt, hipStream_t s);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int pad4(int f) { return (f + 3) & ~3; }
// width of an internal matrix that an SpMM gathers from: rows start on 128-byte lines and fill whole feature tiles
inline int pad32(int f) { return (f + 31) & ~31; }

}  // namespace sensei
