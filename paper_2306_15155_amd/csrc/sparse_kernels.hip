// Sparse kernels for gfx950: CSR SpMM (value-less, weighted, scaled), the
// element-wise SDDMM instances, the segmented edge softmax, degree counts.
//
// Work decomposition shared by every kernel that reduces over rows: the
// non-zeros are cut into chunks of T entries and one 64-lane wavefront owns
// one chunk (x one feature tile for SpMM).  A row that lies inside a chunk is
// finished by that wavefront.  A row that crosses a chunk boundary is written
// in pieces - the piece in the chunk where the row starts goes to the output
// row unscaled, each later piece goes to a per-chunk carry slot - and a small
// fix-up kernel adds the carry slots to the row in chunk order.  No float
// atomics: the summation order is fixed, results are reproducible, and a hub
// row of a power-law graph is spread over as many wavefronts as it needs.
#include "sensei_internal.h"

namespace sensei {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kMaxPanels = SENSEI_MAX_PANELS;
constexpr int kShortRowNnz = 12;  // chunks whose rows average fewer non-zeros than this use one neighbour group per row

// ------------------------------------------------------------------ chunk plan

__global__ void k_chunk_rows(const int32_t *__restrict__ row_ptr, int n_rows, int chunk_nnz, int n_chunks,
                             int32_t *__restrict__ chunk_row) {
    int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c > n_chunks) return;
    if (c == n_chunks) { chunk_row[c] = n_rows; return; }
    const long long target = (long long)c * chunk_nnz;
    int lo = 0, hi = n_rows + 1;  // first index in [0, n_rows] with row_ptr[idx] >= target
    while (lo < hi) {
        int mid = (int)(((long long)lo + hi) >> 1);
        if ((long long)row_ptr[mid] < target) lo = mid + 1; else hi = mid;
    }
    chunk_row[c] = lo < n_rows ? lo : n_rows;
}

// ------------------------------------------------------------------------ SpMM

template <int VEC> struct Vec;
template <> struct Vec<1> {
    float v[1];
    __device__ static Vec load(const float *p) { Vec r; r.v[0] = *p; return r; }
    __device__ void store(float *p) const { *p = v[0]; }
};
template <> struct Vec<2> {
    float v[2];
    __device__ static Vec load(const float *p) { float2 t = *reinterpret_cast<const float2 *>(p); Vec r; r.v[0] = t.x; r.v[1] = t.y; return r; }
    __device__ void store(float *p) const { *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]); }
};
template <> struct Vec<4> {
    float v[4];
    __device__ static Vec load(const float *p) { float4 t = *reinterpret_cast<const float4 *>(p); Vec r; r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w; return r; }
    __device__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]); }
};

struct SpmmArgs {
    const int32_t *row_ptr, *col_idx, *chunk_row;
    const float *val, *r, *c, *B;
    const float2 *mz;  // softmax mode: per-row (max logit, sum of exp(logit - max))
    int val_stride;    // floats from the value of one entry to the next (1, or 2 when the values sit in (value, other) pairs)
    long long c_tile;  // floats from feature tile t of C to tile t + 1: VEC*LPG for a row-major C, n_rows * 32 for a slice-major one (ldc = 32)
    int c_tf;          // columns per feature tile (VEC * LPG)
    float *C, *carry;
    long long ldb, ldc;
    long long tile_stride_b;  // bytes from feature tile t of B to tile t + 1: 4*VEC*LPG when rows are contiguous, a whole slice otherwise
    int n_rows, nnz, chunk_nnz, n_chunks;
    int f, f_store, f_carry, n_tiles, act, store_vec_ok;
    int tiles_live, n_groups;  // feature tiles worked on at the same time; chunk groups (blocks per tile)
    int accumulate, finalize;  // column panels: add to what C holds; apply row scale and activation (last panel only)
    // fused attention mode: the two score vectors, the LeakyReLU slope, and where the (max, sum) pairs of row pieces go
    const float *s_l, *s_r;
    float slope;
    float2 *mz_out, *carry_mz;  // per row: pair of a first piece whose row goes on in the next chunk; per chunk: pair of its continued row
    // modes kSpmmSignSum / kSpmmLreluSum: a vector per row, slice-major like C (tile t of row i at self + t * self_tile + i * 32)
    const float *self;
    long long self_tile;
};

// value of `x` held by the lane whose number is byte_lane / 4 (all lanes must be active)
__device__ __forceinline__ int lane_read(int byte_lane, int x) { return __builtin_amdgcn_ds_bpermute(byte_lane, x); }
__device__ __forceinline__ float lane_read(int byte_lane, float x) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(byte_lane, __float_as_int(x)));
}

__device__ __forceinline__ float uni_f(float x) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x))); }
// 1/z of a softmax row; a row without entries (z = 0) gives 0, never inf
__device__ __forceinline__ float inv_z(float z) { return z > 0.f ? 1.f / z : 0.f; }

// One wavefront = one (chunk, feature tile).  The 64 lanes form G = 64/LPG
// neighbour groups of LPG lanes; a group reads VEC*LPG consecutive floats of
// one neighbour row per step (one 128-byte line at the default shape), so G
// neighbours are in flight per step and 4 steps are issued back to back.
// Column indices (and weights) are fetched 64 at a time, one per lane, and
// handed to the groups by cross-lane reads.  The inner loop carries no
// predicates: full steps of G neighbours run unmasked, the ragged end of a row
// piece is one masked step, and lanes past the last feature column read
// column 0 and never store.  With OFF32 the gathered matrix is smaller than
// 4 GiB with fewer than 2^24 rows of fewer than 2^24 bytes, and addresses are
// a uniform base plus a 32-bit byte offset formed by one 24-bit multiply-add.
// Consecutive workgroups go to consecutive XCDs and take consecutive tiles of
// the live tile set, so each XCD's L2 keeps seeing the same 128-byte slice of
// the gathered matrix; the number of live tiles bounds how much of that matrix
// is in use at one time.  B is either row-major (a row holds all its tiles) or
// slice-major (all rows of tile 0, then all rows of tile 1, ...: what an XCD
// gathers from is then one contiguous range, which spreads evenly over the
// memory channels whatever the row pitch).
// MODE kSpmmSoftmax: `val` holds attention logits; the weight of an entry is exp(logit - m_i) and the row is
// scaled by 1/z_i when it is complete, so the normalised attention weights are never stored (Eq. 6).
// MODE kSpmmAttnFused: score, softmax and weighted sum in one walk (Eq. 5-6 with nothing stored per entry): the logit
// LeakyReLU(s_l[i] + s_r[j]) is formed from the two score vectors as the neighbour is gathered, every lane keeps a running
// maximum m, the sum z of exp(logit - m) and its partial row relative to m, rescaling both when the maximum grows; the
// lanes' (m, z, row) triples are merged when the row (piece) ends.  A piece of a row that spans chunks leaves its pair
// beside its partial row (mz_out / carry_mz) and k_spmm_fixup_attn merges the pieces in chunk order.
// MODES kSpmmSignSum, kSpmmLreluSum (slice-major operands, 32-column tiles): the gathered row meets a vector of the output row itself,
// u = self[i, :] + B[j, :], and what is summed is val_ij LeakyReLU'(u) or val_ij LeakyReLU(u), column by column: the reductions
// of the backward pass of a score with a vector per entry.
template <int VEC, int LPG, int MODE, bool OFF32>
__global__ __launch_bounds__(kBlock) void k_spmm(SpmmArgs a) {
    constexpr int G = 64 / LPG;
    constexpr int TF = VEC * LPG;
    constexpr int U = 4;  // steps issued back to back
    const int lane = threadIdx.x & 63;
    // blocks are ordered: tile set (tiles_live tiles each) major, then chunk group, then tile within the set
    const int per_set = a.n_groups * a.tiles_live;
    const int set = blockIdx.x / per_set, in_set = blockIdx.x % per_set;
    const int tile = set * a.tiles_live + in_set % a.tiles_live;
    if (tile >= a.n_tiles) return;
    // wave-uniform by construction; readfirstlane lets the compiler keep the row walk in scalar registers
    const int chunk = (in_set / a.tiles_live) * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (chunk >= a.n_chunks) return;
    const int g = lane / LPG;
    const int f0 = tile * TF + (lane % LPG) * VEC;
    const bool fok = f0 < a.f;
    const char *Bb = reinterpret_cast<const char *>(a.B) + (long long)tile * a.tile_stride_b;
    const unsigned f0_b = fok ? (unsigned)((lane % LPG) * VEC) * 4u : 0u;
    float *c_tile_base = a.C + (size_t)tile * a.c_tile + (lane % LPG) * VEC;  // this lane's columns of row 0 of C
    const unsigned ldb_b32 = (unsigned)(a.ldb * 4);
    const size_t ldb_b64 = (size_t)a.ldb * 4;

    auto gather = [&](int j) -> Vec<VEC> {
        if (OFF32) return Vec<VEC>::load(reinterpret_cast<const float *>(Bb + (__umul24((unsigned)j, ldb_b32) + f0_b)));
        return Vec<VEC>::load(reinterpret_cast<const float *>(Bb + ((size_t)j * ldb_b64 + f0_b)));
    };

    const long long lo_ll = (long long)chunk * a.chunk_nnz;
    const int lo = (int)lo_ll;
    const int hi = (int)((lo_ll + a.chunk_nnz < (long long)a.nnz) ? lo_ll + a.chunk_nnz : (long long)a.nnz);
    const int i0 = a.chunk_row[chunk];
    const int i1 = a.chunk_row[chunk + 1];

    // first row touched: the one crossing `lo` if there is one, else the first owned row
    // (the row walk is wave-uniform; uni() pins its state to scalar registers)
    auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    bool cont = (a.nnz > 0) && (a.row_ptr[i0] > lo);
    int i = uni(cont ? i0 - 1 : i0);
    int re = uni((i < a.n_rows) ? a.row_ptr[i + 1] : 0x7fffffff);
    float m_row = 0.f;  // softmax mode: max logit of row i; fused attention mode: s_l of row i
    if (MODE == kSpmmSoftmax) m_row = uni_f((i < a.n_rows) ? a.mz[i].x : 0.f);
    if (MODE == kSpmmAttnFused) m_row = uni_f((i < a.n_rows) ? a.s_l[i] : 0.f);
    float m_run = -INFINITY, z_run = 0.f;  // fused attention mode: this lane's running maximum and sum of exp(logit - maximum)
    constexpr bool kSelfMode = (MODE == kSpmmSignSum || MODE == kSpmmLreluSum);
    const float *self_lane = nullptr;   // this lane's columns of row 0 of the per-row vector
    Vec<VEC> self_v;
#pragma unroll
    for (int e = 0; e < VEC; ++e) self_v.v[e] = 0.f;
    if (kSelfMode) {
        self_lane = a.self + (size_t)tile * a.self_tile + (fok ? (lane % LPG) * VEC : 0);
        if (i < a.n_rows) self_v = Vec<VEC>::load(self_lane + (size_t)i * 32);
    }

    Vec<VEC> acc;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc.v[e] = 0.f;

    auto accumulate = [&](const Vec<VEC> &b, float ww) {
        if (MODE == kSpmmAttnFused) {  // ww = s_r of the neighbour
            const float t = m_row + ww;
            const float lg = t > 0.f ? t : a.slope * t;
            const float mn = lg > m_run ? lg : m_run;
            const float keep = __expf(m_run - mn);  // 0 on the first neighbour (m_run = -inf), 1 while the maximum stands
            const float p = __expf(lg - mn);
            z_run = fmaf(z_run, keep, p);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc.v[e] = fmaf(acc.v[e], keep, p * b.v[e]);
            m_run = mn;
            return;
        }
        if (kSelfMode) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float u = self_v.v[e] + b.v[e];
                const float d = u > 0.f ? 1.f : a.slope;
                acc.v[e] = fmaf(ww, MODE == kSpmmSignSum ? d : d * u, acc.v[e]);
            }
            return;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (MODE == SENSEI_SPMM_PATTERN) acc.v[e] += b.v[e];
            else acc.v[e] = fmaf(ww, b.v[e], acc.v[e]);
        }
    };

    auto finish_row = [&](bool complete) {
        float m_all = 0.f;
        if (MODE == kSpmmAttnFused) {  // bring every group's partial row to the common maximum of the row piece
            m_all = m_run;
#pragma unroll
            for (int off = LPG; off < 64; off <<= 1) {
                const float o = __shfl_xor(m_all, off, 64);
                m_all = o > m_all ? o : m_all;
            }
            const float sc = m_run > -INFINITY ? __expf(m_run - m_all) : 0.f;  // a group that saw no neighbour holds zeros
            z_run *= sc;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc.v[e] *= sc;
#pragma unroll
            for (int off = LPG; off < 64; off <<= 1) z_run += __shfl_xor(z_run, off, 64);
        }
#pragma unroll
        for (int off = LPG; off < 64; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc.v[e] += __shfl_xor(acc.v[e], off, 64);
        }
        if (MODE == kSpmmAttnFused && lane == 0 && tile == 0) {  // every feature tile of the chunk forms the same pair: one writes it
            if (cont) a.carry_mz[chunk] = make_float2(m_all, z_run);
            else if (!complete) a.mz_out[i] = make_float2(m_all, z_run);
        }
        if (g == 0 && fok) {
            if (cont) {
                acc.store(a.carry + (size_t)chunk * a.f_carry + f0);
            } else {
                float *dst = c_tile_base + (size_t)i * a.ldc;
                const bool vec_store = a.store_vec_ok && f0 + VEC <= a.f_store;
                if (a.accumulate) {  // later column panel: add to what the earlier panels left in C
                    if (vec_store) {
                        const Vec<VEC> old = Vec<VEC>::load(dst);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc.v[e] += old.v[e];
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) if (f0 + e < a.f_store) acc.v[e] += dst[e];
                    }
                }
                if (complete && a.finalize) {
                    const float sc = (MODE == kSpmmAttnFused) ? inv_z(z_run) : (MODE == kSpmmSoftmax) ? inv_z(a.mz[i].y) : (a.r ? a.r[i] : 1.f);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        float y = acc.v[e] * sc;
                        if (a.act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
                        acc.v[e] = y;
                    }
                }
                if (vec_store) {
                    acc.store(dst);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) if (f0 + e < a.f_store) dst[e] = acc.v[e];
                }
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc.v[e] = 0.f;
        m_run = -INFINITY;
        z_run = 0.f;
    };

    // Many short rows in this chunk: walking them one after another would leave most neighbour groups
    // idle and serialise one memory round trip per row.  Give every group a row of its own instead; a
    // group then holds the whole feature slice of its row and needs no cross-lane reduction.
    const int i_first = cont ? i0 - 1 : i0;
    if ((long long)(i1 - i_first) * kShortRowNnz > (long long)(hi - lo)) {
        for (int ib = i_first; ib < i1; ib += G) {
            const int row = ib + g;
            const bool rok = row < i1;
            int rs = 0, rend = 0, row_end = 0;
            float2 mz_g = make_float2(0.f, 0.f);
            if (rok) {
                if (MODE == kSpmmSoftmax) mz_g = a.mz[row];
                rs = a.row_ptr[row];
                row_end = a.row_ptr[row + 1];
                rs = rs > lo ? rs : lo;
                rend = row_end < hi ? row_end : hi;
            }
            Vec<VEC> racc;
#pragma unroll
            for (int e = 0; e < VEC; ++e) racc.v[e] = 0.f;
            float rm = -INFINITY, rz = 0.f;  // fused attention mode: running maximum and sum of the group's row
            const float sl_g = (MODE == kSpmmAttnFused && rok) ? a.s_l[row] : 0.f;
            Vec<VEC> self_g;
#pragma unroll
            for (int e = 0; e < VEC; ++e) self_g.v[e] = 0.f;
            if (kSelfMode && rok) self_g = Vec<VEC>::load(self_lane + (size_t)row * 32);
            for (int k = rs; k < rend; k += U) {
                Vec<VEC> b[U];
                float ww[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const bool valid = k + q < rend;
                    const int kq = valid ? k + q : k;
                    const int j = a.col_idx[kq];
                    float wq = 1.f;
                    if (MODE == SENSEI_SPMM_WEIGHTED || kSelfMode) wq = a.val[(size_t)kq * a.val_stride];
                    if (MODE == SENSEI_SPMM_SCALED) wq = a.c[j];
                    if (MODE == kSpmmSoftmax) wq = __expf(a.val[(size_t)kq * a.val_stride] - mz_g.x);
                    if (MODE == kSpmmAttnFused) {
                        const float t = sl_g + a.s_r[j];
                        wq = valid ? (t > 0.f ? t : a.slope * t) : -INFINITY;  // the logit; an entry past the end weighs exp(-inf) = 0
                        ww[q] = wq;
                    } else {
                        ww[q] = valid ? wq : 0.f;
                    }
                    b[q] = gather(j);
                }
                if (MODE == kSpmmAttnFused) {  // one rescale for the four neighbours of the step
                    float mn = rm;
#pragma unroll
                    for (int q = 0; q < U; ++q) mn = ww[q] > mn ? ww[q] : mn;
                    const float keep = __expf(rm - mn);
                    rz *= keep;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) racc.v[e] *= keep;
#pragma unroll
                    for (int q = 0; q < U; ++q) {
                        ww[q] = __expf(ww[q] - mn);
                        rz += ww[q];
                    }
                    rm = mn;
                }
#pragma unroll
                for (int q = 0; q < U; ++q) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        if (kSelfMode) {
                            const float u = self_g.v[e] + b[q].v[e];
                            const float d = u > 0.f ? 1.f : a.slope;
                            racc.v[e] = fmaf(ww[q], MODE == kSpmmSignSum ? d : d * u, racc.v[e]);
                        } else {
                            racc.v[e] = fmaf(ww[q], b[q].v[e], racc.v[e]);
                        }
                    }
                }
            }
            if (MODE == kSpmmAttnFused && rok && tile == 0 && (lane % LPG) == 0) {
                if (cont && row == i_first) a.carry_mz[chunk] = make_float2(rm, rz);
                else if (row_end > hi) a.mz_out[row] = make_float2(rm, rz);
            }
            if (rok && fok) {
                if (cont && row == i_first) {
                    racc.store(a.carry + (size_t)chunk * a.f_carry + f0);
                } else {
                    float *dst = c_tile_base + (size_t)row * a.ldc;
                    const bool vec_store = a.store_vec_ok && f0 + VEC <= a.f_store;
                    if (a.accumulate) {
                        if (vec_store) {
                            const Vec<VEC> old = Vec<VEC>::load(dst);
#pragma unroll
                            for (int e = 0; e < VEC; ++e) racc.v[e] += old.v[e];
                        } else {
#pragma unroll
                            for (int e = 0; e < VEC; ++e) if (f0 + e < a.f_store) racc.v[e] += dst[e];
                        }
                    }
                    if (row_end <= hi && a.finalize) {
                        const float sc = (MODE == kSpmmAttnFused) ? inv_z(rz) : (MODE == kSpmmSoftmax) ? inv_z(mz_g.y) : (a.r ? a.r[row] : 1.f);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            float y = racc.v[e] * sc;
                            if (a.act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
                            racc.v[e] = y;
                        }
                    }
                    if (vec_store) {
                        racc.store(dst);
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) if (f0 + e < a.f_store) dst[e] = racc.v[e];
                    }
                }
            }
        }
        return;
    }

    int pos = lo;
    for (int base = lo; base < hi; base += 64) {
        const int k = base + lane;
        int col = 0;
        float w = 0.f;
        if (k < hi) {
            col = a.col_idx[k];
            if (MODE == SENSEI_SPMM_WEIGHTED || MODE == kSpmmSoftmax || kSelfMode) w = a.val[(size_t)k * a.val_stride];
            if (MODE == SENSEI_SPMM_SCALED) w = a.c[col];
            if (MODE == kSpmmAttnFused) w = a.s_r[col];
        }
        const int bhi = (base + 64 < hi) ? base + 64 : hi;
        while (pos < bhi) {
            while (re <= pos) {  // rows ending here (or empty): close them and move on
                finish_row(true);
                cont = false;
                i = uni(i + 1);
                re = uni(a.row_ptr[i + 1]);
                if (MODE == kSpmmSoftmax) m_row = uni_f(a.mz[i].x);
                if (MODE == kSpmmAttnFused) m_row = uni_f(a.s_l[i]);
                if (kSelfMode) self_v = Vec<VEC>::load(self_lane + (size_t)i * 32);
            }
            const int seg_hi = uni(re < bhi ? re : bhi);
            const int u0 = uni(pos - base), n = uni(seg_hi - pos);
            const int full = n / G;
            int src4 = (u0 + g) * 4;  // byte-lane address of this group's next neighbour
            int it = 0;
            for (; it + U <= full; it += U) {
                Vec<VEC> b[U];
                float ww[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int j = lane_read(src4 + q * G * 4, col);
                    ww[q] = (MODE == SENSEI_SPMM_PATTERN) ? 1.f : lane_read(src4 + q * G * 4, w);
                    if (MODE == kSpmmSoftmax) ww[q] = __expf(ww[q] - m_row);
                    b[q] = gather(j);
                }
#pragma unroll
                for (int q = 0; q < U; ++q) accumulate(b[q], ww[q]);
                src4 += U * G * 4;
            }
            for (; it < full; ++it) {
                const int j = lane_read(src4, col);
                float ww = (MODE == SENSEI_SPMM_PATTERN) ? 1.f : lane_read(src4, w);
                if (MODE == kSpmmSoftmax) ww = __expf(ww - m_row);
                accumulate(gather(j), ww);
                src4 += G * 4;
            }
            const int rem = n - full * G;
            if (rem > 0) {  // ragged end of the piece: groups g < rem take one more neighbour
                const bool ok = g < rem;
                const int s4 = ok ? src4 : u0 * 4;
                const int j = lane_read(s4, col);
                float ww = (MODE == SENSEI_SPMM_PATTERN) ? 1.f : lane_read(s4, w);
                if (MODE == kSpmmSoftmax) ww = __expf(ww - m_row);
                if (ok) accumulate(gather(j), ww);
            }
            pos = seg_hi;
        }
    }
    // close what is left: the current row if it ends in this chunk, then owned empty rows
    while (i < i1) {
        if (re <= hi) {
            finish_row(true);
            cont = false;
            i = uni(i + 1);
            re = uni((i < a.n_rows) ? a.row_ptr[i + 1] : 0x7fffffff);
        } else {
            finish_row(false);
            break;
        }
    }
}

// Adds the carry slots of a row that spans several chunks to its output row, in chunk order,
// then applies the row scale and the activation.  One wavefront per chunk; only the chunk that
// holds the first continuation of a row does the work for that row.
__global__ __launch_bounds__(kBlock) void k_spmm_fixup(SpmmArgs a) {
    const int c = 1 + blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (c >= a.n_chunks) return;
    const int lane = threadIdx.x & 63;
    const long long lo = (long long)c * a.chunk_nnz;
    const int i0 = a.chunk_row[c];
    if ((long long)a.row_ptr[i0] <= lo) return;  // a row starts exactly at the boundary
    const int i = i0 - 1;
    const long long rs = a.row_ptr[i];
    if (rs < lo - a.chunk_nnz) return;  // the row began before the previous chunk: not its first continuation
    const int re = a.row_ptr[i + 1];
    const int c_last = (re - 1) / a.chunk_nnz;
    const float sc = a.mz ? inv_z(a.mz[i].y) : (a.r ? a.r[i] : 1.f);
    const int tf = a.c_tf;
    // four columns per lane at a time: a hub row spans a hundred chunks, and one chain of dependent adds per column would
    // leave the wavefront waiting for one load after the other; every column still adds its slots in chunk order
    for (int f0 = lane; f0 < a.f_store; f0 += 4 * 64) {
        float acc[4];
        float *dst[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int f = f0 + 64 * q;
            dst[q] = a.C + (size_t)(f / tf) * a.c_tile + (size_t)i * a.ldc + (f % tf);
            acc[q] = f < a.f_store ? *dst[q] : 0.f;
        }
#pragma unroll 4
        for (int cc = c; cc <= c_last; ++cc) {
            const float *slot = a.carry + (size_t)cc * a.f_carry + f0;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (f0 + 64 * q < a.f_store) acc[q] += slot[64 * q];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (f0 + 64 * q >= a.f_store) continue;
            float y = acc[q];
            if (a.finalize) {
                y *= sc;
                if (a.act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
            }
            *dst[q] = y;
        }
    }
}

// The same for the fused attention mode: the pieces of a row come with their (maximum, sum) pairs and are merged like the
// lanes of a wavefront are - everything rescaled to the larger maximum - in chunk order; then 1 / sum and the activation.
__global__ __launch_bounds__(kBlock) void k_spmm_fixup_attn(SpmmArgs a) {
    const int c = 1 + blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (c >= a.n_chunks) return;
    const int lane = threadIdx.x & 63;
    const long long lo = (long long)c * a.chunk_nnz;
    const int i0 = a.chunk_row[c];
    if ((long long)a.row_ptr[i0] <= lo) return;
    const int i = i0 - 1;
    const long long rs = a.row_ptr[i];
    if (rs < lo - a.chunk_nnz) return;
    const int re = a.row_ptr[i + 1];
    const int c_last = (re - 1) / a.chunk_nnz;
    const int tf = a.c_tf;
    const float2 first = a.mz_out[i];
    for (int f = lane; f < a.f_store; f += 64) {
        float *dst = a.C + (size_t)(f / tf) * a.c_tile + (size_t)i * a.ldc + (f % tf);
        float m = first.x, z = first.y, acc = *dst;
        for (int cc = c; cc <= c_last; ++cc) {
            const float2 p = a.carry_mz[cc];
            const float mn = p.x > m ? p.x : m;
            const float k0 = __expf(m - mn), k1 = __expf(p.x - mn);
            acc = acc * k0 + a.carry[(size_t)cc * a.f_carry + f] * k1;
            z = z * k0 + p.y * k1;
            m = mn;
        }
        float y = acc * inv_z(z);
        if (a.act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
        *dst = y;
    }
}

template <int VEC, int LPG, bool OFF32>
hipError_t spmm_dispatch_mode(const SpmmArgs &a, int mode, dim3 grid, hipStream_t s) {
    switch (mode) {
        case SENSEI_SPMM_PATTERN: hipLaunchKernelGGL((k_spmm<VEC, LPG, SENSEI_SPMM_PATTERN, OFF32>), grid, dim3(kBlock), 0, s, a); break;
        case SENSEI_SPMM_WEIGHTED: hipLaunchKernelGGL((k_spmm<VEC, LPG, SENSEI_SPMM_WEIGHTED, OFF32>), grid, dim3(kBlock), 0, s, a); break;
        case kSpmmSoftmax: hipLaunchKernelGGL((k_spmm<VEC, LPG, kSpmmSoftmax, OFF32>), grid, dim3(kBlock), 0, s, a); break;
        case kSpmmAttnFused: hipLaunchKernelGGL((k_spmm<VEC, LPG, kSpmmAttnFused, OFF32>), grid, dim3(kBlock), 0, s, a); break;
        case kSpmmSignSum:
        case kSpmmLreluSum:
            if constexpr (VEC == 4 && LPG == 8) {   // slice-major operands only
                if (mode == kSpmmSignSum) hipLaunchKernelGGL((k_spmm<4, 8, kSpmmSignSum, OFF32>), grid, dim3(kBlock), 0, s, a);
                else hipLaunchKernelGGL((k_spmm<4, 8, kSpmmLreluSum, OFF32>), grid, dim3(kBlock), 0, s, a);
                break;
            } else {
                return hipErrorInvalidValue;
            }
        default: hipLaunchKernelGGL((k_spmm<VEC, LPG, SENSEI_SPMM_SCALED, OFF32>), grid, dim3(kBlock), 0, s, a); break;
    }
    return hipGetLastError();
}

template <int VEC>
hipError_t spmm_dispatch_lpg(const SpmmArgs &a, int mode, int lpg, bool off32, dim3 grid, hipStream_t s) {
    switch (lpg) {
        case 8: return off32 ? spmm_dispatch_mode<VEC, 8, true>(a, mode, grid, s) : spmm_dispatch_mode<VEC, 8, false>(a, mode, grid, s);
        case 16: return off32 ? spmm_dispatch_mode<VEC, 16, true>(a, mode, grid, s) : spmm_dispatch_mode<VEC, 16, false>(a, mode, grid, s);
        case 32: return off32 ? spmm_dispatch_mode<VEC, 32, true>(a, mode, grid, s) : spmm_dispatch_mode<VEC, 32, false>(a, mode, grid, s);
        default: return off32 ? spmm_dispatch_mode<VEC, 64, true>(a, mode, grid, s) : spmm_dispatch_mode<VEC, 64, false>(a, mode, grid, s);
    }
}

// ------------------------------------------------------- element-wise / degrees

__global__ void k_fill_i32(int32_t *p, long long n, int32_t v) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) p[t] = v;
}

__global__ void k_deg_row(const int32_t *__restrict__ row_ptr, int n_rows, int32_t *__restrict__ deg_row) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_rows) deg_row[i] = row_ptr[i + 1] - row_ptr[i];
}

__global__ void k_deg_col(const int32_t *__restrict__ col_idx, long long nnz, int32_t *__restrict__ deg_col) {
    long long k = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < nnz) atomicAdd(&deg_col[col_idx[k]], 1);  // integer atomics: the result is exact in any order
}

// The same count for patterns whose columns fit a few LDS-sized ranges: a workgroup counts the entries of one share of the
// pattern that fall into one range of kDegRange columns in LDS and adds its non-zero counters to deg_col at the end, so the
// global atomics number (shares x columns) instead of one per entry, and the columns that every row refers to no longer
// serialise them.  Workgroup number -> (share, range): the ranges of one share run on one XCD at about the same time
// (workgroups are dealt round-robin to the eight XCDs), so a share is read from memory once and from that L2 afterwards.
constexpr int kDegRange = 32768, kDegThreads = 1024, kDegRangesMax = 16;

__global__ __launch_bounds__(kDegThreads) void k_deg_col_ranges(const int32_t *__restrict__ col_idx, long long nnz, int n_cols, int n_ranges,
                                                                long long per_share, int32_t *__restrict__ deg_col) {
    __shared__ int32_t cnt[kDegRange];
    const int g = blockIdx.x >> 3;
    const int range = g % n_ranges, share = (g / n_ranges) * 8 + (blockIdx.x & 7);
    const int lo_col = range * kDegRange;
    for (int d = threadIdx.x; d < kDegRange; d += kDegThreads) cnt[d] = 0;
    __syncthreads();
    const long long k0 = share * per_share, k1 = k0 + per_share < nnz ? k0 + per_share : nnz;
    long long k = k0 + threadIdx.x;
    for (; k + 3 * kDegThreads < k1; k += 4 * kDegThreads) {
        unsigned d[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) d[u] = (unsigned)(col_idx[k + u * kDegThreads] - lo_col);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (d[u] < (unsigned)kDegRange) atomicAdd(&cnt[d[u]], 1);
    }
    for (; k < k1; k += kDegThreads) {
        const unsigned d = (unsigned)(col_idx[k] - lo_col);
        if (d < (unsigned)kDegRange) atomicAdd(&cnt[d], 1);
    }
    __syncthreads();
    const int width = n_cols - lo_col < kDegRange ? n_cols - lo_col : kDegRange;
    for (int d = threadIdx.x; d < width; d += kDegThreads) {
        const int32_t c = cnt[d];
        if (c) atomicAdd(&deg_col[lo_col + d], c);
    }
}

__global__ void k_norm_vec(const int32_t *__restrict__ deg, long long n, float *__restrict__ out) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) {
        int d = deg[t];
        d = d < 1 ? 1 : d;
        out[t] = 1.0f / sqrtf((float)d);  // IEEE sqrt and divide (hipcc's default), no rsq approximation
    }
}

struct NnzArgs {
    const int32_t *row_ptr, *col_idx, *chunk_row;
    int n_rows, nnz, chunk_nnz, n_chunks;
};

constexpr int kShortRowElem = 16;  // element-wise kernels: chunks whose rows average fewer non-zeros use one lane per row

// Visits every non-zero of one chunk with one wavefront.  per_row(i) is evaluated once per row (piece) and its
// result handed to per_nnz(k, row_data) for each non-zero k of that row inside the chunk.  Long rows: the
// wavefront walks the rows (row data in scalar registers) and its lanes stride over the non-zeros, so loads
// and stores are coalesced.  Short rows: one lane per row.  Either way no per-non-zero row search is needed.
template <class PerRow, class PerNnz>
__device__ __forceinline__ void walk_chunk(const NnzArgs &a, int chunk, int lane, PerRow per_row, PerNnz per_nnz) {
    const long long lo_ll = (long long)chunk * a.chunk_nnz;
    const int lo = (int)lo_ll;
    const int hi = (int)((lo_ll + a.chunk_nnz < (long long)a.nnz) ? lo_ll + a.chunk_nnz : (long long)a.nnz);
    if (lo >= hi) return;
    const int i0 = a.chunk_row[chunk], i1 = a.chunk_row[chunk + 1];
    const int i_first = (a.row_ptr[i0] > lo) ? i0 - 1 : i0;
    if ((long long)(i1 - i_first) * kShortRowElem > (long long)(hi - lo)) {
        for (int ib = i_first; ib < i1; ib += 64) {
            const int row = ib + lane;
            if (row < i1) {
                int rs = a.row_ptr[row], re = a.row_ptr[row + 1];
                rs = rs > lo ? rs : lo;
                re = re < hi ? re : hi;
                if (rs < re) {
                    const auto rd = per_row(row);
#pragma unroll 4
                    for (int k = rs; k < re; ++k) per_nnz(k, rd);
                }
            }
        }
        return;
    }
    int i = __builtin_amdgcn_readfirstlane(i_first);
    int pos = lo;
    while (pos < hi) {
        const int re = __builtin_amdgcn_readfirstlane(a.row_ptr[i + 1]);
        if (re > pos) {
            const int seg_hi = re < hi ? re : hi;
            const auto rd = per_row(i);
#pragma unroll 4
            for (int k = pos + lane; k < seg_hi; k += 64) per_nnz(k, rd);
            pos = seg_hi;
        }
        i = __builtin_amdgcn_readfirstlane(i + 1);
    }
}

// The same walk with the work on a non-zero cut in two: `load(k, row_data)` only reads and returns what it read,
// `apply(k, row_data, loaded)` computes and stores.  The reads of kWalkBatch non-zeros per lane are requested before the
// first store of a trip: a store may alias anything as far as the compiler can tell, so a plain loop waits for one
// memory round trip per non-zero and lane (measured: 12 % off the softmax backward pass of the attention layer).
constexpr int kWalkBatch = 4;
template <class PerRow, class Load, class Apply>
__device__ __forceinline__ void walk_chunk2(const NnzArgs &a, int chunk, int lane, PerRow per_row, Load load, Apply apply) {
    const long long lo_ll = (long long)chunk * a.chunk_nnz;
    const int lo = (int)lo_ll;
    const int hi = (int)((lo_ll + a.chunk_nnz < (long long)a.nnz) ? lo_ll + a.chunk_nnz : (long long)a.nnz);
    if (lo >= hi) return;
    const int i0 = a.chunk_row[chunk], i1 = a.chunk_row[chunk + 1];
    const int i_first = (a.row_ptr[i0] > lo) ? i0 - 1 : i0;
    if ((long long)(i1 - i_first) * kShortRowElem > (long long)(hi - lo)) {
        for (int ib = i_first; ib < i1; ib += 64) {
            const int row = ib + lane;
            if (row < i1) {
                int rs = a.row_ptr[row], re = a.row_ptr[row + 1];
                rs = rs > lo ? rs : lo;
                re = re < hi ? re : hi;
                if (rs < re) {
                    const auto rd = per_row(row);
                    for (int k0 = rs; k0 < re; k0 += kWalkBatch) {
                        decltype(load(k0, rd)) got[kWalkBatch];
#pragma unroll
                        for (int u = 0; u < kWalkBatch; ++u) got[u] = load(k0 + u < re ? k0 + u : rs, rd);
#pragma unroll
                        for (int u = 0; u < kWalkBatch; ++u)
                            if (k0 + u < re) apply(k0 + u, rd, got[u]);
                    }
                }
            }
        }
        return;
    }
    int i = __builtin_amdgcn_readfirstlane(i_first);
    int pos = lo;
    while (pos < hi) {
        const int re = __builtin_amdgcn_readfirstlane(a.row_ptr[i + 1]);
        if (re > pos) {
            const int seg_hi = re < hi ? re : hi;
            const auto rd = per_row(i);
            for (int k0 = pos + lane; k0 < seg_hi; k0 += 64 * kWalkBatch) {
                decltype(load(k0, rd)) got[kWalkBatch];
#pragma unroll
                for (int u = 0; u < kWalkBatch; ++u) got[u] = load(k0 + 64 * u < seg_hi ? k0 + 64 * u : pos, rd);
#pragma unroll
                for (int u = 0; u < kWalkBatch; ++u)
                    if (k0 + 64 * u < seg_hi) apply(k0 + 64 * u, rd, got[u]);
            }
            pos = seg_hi;
        }
        i = __builtin_amdgcn_readfirstlane(i + 1);
    }
}

__device__ __forceinline__ int wave_chunk() {
    return blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
}

__global__ __launch_bounds__(kBlock) void k_sddmm_norm(NnzArgs a, const float *__restrict__ r, const float *__restrict__ c,
                                                        float *__restrict__ val) {
    const int chunk = wave_chunk();
    if (chunk >= a.n_chunks) return;
    walk_chunk(a, chunk, threadIdx.x & 63, [&](int i) { return r[i]; },
               [&](int k, float ri) { val[k] = ri * c[a.col_idx[k]]; });
}

__device__ __forceinline__ float leaky(float t, float slope) { return t > 0.f ? t : slope * t; }

__global__ __launch_bounds__(kBlock) void k_score(NnzArgs a, const float *__restrict__ s_l, const float *__restrict__ s_r, float slope,
                                                   float *__restrict__ e) {
    const int chunk = wave_chunk();
    if (chunk >= a.n_chunks) return;
    walk_chunk(a, chunk, threadIdx.x & 63, [&](int i) { return s_l[i]; },
               [&](int k, float sl) { e[k] = leaky(sl + s_r[a.col_idx[k]], slope); });
}

template <int VEC>
__global__ void k_row_broadcast(const float *__restrict__ s, const float *X, long long ldx, long long n, int f, float *Y,
                                long long ldy, int act, const float *__restrict__ mask, long long ldm) {  // Y may be X (in place)
    const int fv = f / VEC;
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * fv) return;
    const long long i = t / fv;
    const int q = (int)(t % fv) * VEC;
    const float sc = s ? s[i] : 1.f;
    Vec<VEC> x = Vec<VEC>::load(X + i * ldx + q);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        float y = x.v[e] * sc;
        if (act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
        if (mask && !(mask[i * ldm + q + e] > 0.f)) y = 0.f;  // gradient of ReLU: passes where the forward output is positive
        x.v[e] = y;
    }
    x.store(Y + i * ldy + q);
}

__global__ void k_reciprocal(const float *__restrict__ v, long long n, float *__restrict__ out) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = 1.0f / v[i];
}

__global__ void k_stack_weights(const float *__restrict__ W, long long ldw, int hops, int f_in, int fp, int f_out, float *__restrict__ out,
                                long long ldo) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)hops * fp * f_out) return;
    const int m = (int)(i % f_out);
    const long long row = i / f_out;
    const int h = (int)(row / fp), f = (int)(row % fp);
    out[row * ldo + m] = f < f_in ? W[((long long)h * f_in + f) * ldw + m] : 0.f;
}

// Copy of X (n x f, row-major) into slice-major tiles of 32 columns, optionally scaled per row; the pad columns
// up to the next multiple of 32 are written as zeros.  One thread per (row, 4 columns).
__global__ void k_to_slices(const float *__restrict__ s, const float *__restrict__ X, long long ldx, long long n, int f,
                            float *__restrict__ Y, int x_vec_ok, const float *__restrict__ mask, long long ldm) {
    const int fp4 = ((f + 31) & ~31) / 4;
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * fp4) return;
    // consecutive threads walk the rows of one tile: reads are 16-byte pieces 8 to a row, writes are contiguous
    const long long per_tile = n * 8;
    const int tile = (int)(t / per_tile);
    const long long in_tile = t % per_tile;
    const long long i = in_tile >> 3;
    const int q = tile * 32 + (int)(in_tile & 7) * 4;
    const float sc = s ? s[i] : 1.f;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *x = X + i * ldx + q;
    if (x_vec_ok && q + 4 <= f) {
        v = *reinterpret_cast<const float4 *>(x);
    } else {
        if (q < f) v.x = x[0];
        if (q + 1 < f) v.y = x[1];
        if (q + 2 < f) v.z = x[2];
        if (q + 3 < f) v.w = x[3];
    }
    v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
    if (mask) {  // gradient of ReLU: passes where the forward output is positive
        const float *mk = mask + i * ldm + q;
        if (!(q < f && mk[0] > 0.f)) v.x = 0.f;
        if (!(q + 1 < f && mk[1] > 0.f)) v.y = 0.f;
        if (!(q + 2 < f && mk[2] > 0.f)) v.z = 0.f;
        if (!(q + 3 < f && mk[3] > 0.f)) v.w = 0.f;
    }
    *reinterpret_cast<float4 *>(Y + (size_t)tile * (size_t)n * 32 + (size_t)in_tile * 4) = v;
}

// ------------------------------------------------------------- edge softmax

// (m, z) pairs: z = sum of exp(e - m).  Merge keeps m the larger maximum.
__device__ __forceinline__ void mz_add(float &m, float &z, float e) {  // e finite; branch-free: lanes of a wavefront disagree on e > m
    const float mm = e > m ? e : m;
    z = z * __expf(m - mm) + __expf(e - mm);  // m = -inf at the start: exp(-inf) = 0 and z = 0
    m = mm;
}
__device__ __forceinline__ void mz_merge(float &m, float &z, float m2, float z2) {
    const float mm = m > m2 ? m : m2;
    if (mm == -INFINITY) { m = mm; z = 0.f; return; }
    z = z * expf(m - mm) + z2 * expf(m2 - mm);
    m = mm;
}

struct SoftmaxArgs {
    NnzArgs n;
    const float *e, *s_l, *s_r;
    float slope;
    float2 *stats, *carry;
    float *alpha;
    float *logits;             // where the statistics pass parks the logits it computed from s_l, s_r
    const int32_t *dst_index;  // optional: the logit of entry k goes to logits[dst_index[k]] (panel or remainder order), nowhere if negative
};

__device__ __forceinline__ void keep_logit(const SoftmaxArgs &a, int k, float e) {
    if (a.dst_index) {
        const int d = a.dst_index[k];
        if (d >= 0) a.logits[d] = e;  // negative: the entry is not stored (it lies in a dense tile)
    } else {
        a.logits[k] = e;
    }
}

// Row statistics with the same chunk ownership as SpMM: lanes stride over the non-zeros of the
// current row piece, then a wavefront reduction closes the piece.
template <bool FROM_E>
__global__ __launch_bounds__(kBlock) void k_softmax_stats(SoftmaxArgs a) {
    const int chunk = blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (chunk >= a.n.n_chunks) return;
    const int lane = threadIdx.x & 63;
    const long long lo_ll = (long long)chunk * a.n.chunk_nnz;
    const int lo = (int)lo_ll;
    const int hi = (int)((lo_ll + a.n.chunk_nnz < (long long)a.n.nnz) ? lo_ll + a.n.chunk_nnz : (long long)a.n.nnz);
    const int i0 = a.n.chunk_row[chunk], i1 = a.n.chunk_row[chunk + 1];
    bool cont = (a.n.nnz > 0) && (a.n.row_ptr[i0] > lo);
    int i = cont ? i0 - 1 : i0;
    int re = (i < a.n.n_rows) ? a.n.row_ptr[i + 1] : 0x7fffffff;
    float m = -INFINITY, z = 0.f;

    // many short rows: one lane per row, no cross-lane reduction
    const int i_first = cont ? i0 - 1 : i0;
    if ((long long)(i1 - i_first) * kShortRowElem > (long long)(hi - lo)) {
        for (int ib = i_first; ib < i1; ib += 64) {
            const int row = ib + lane;
            if (row >= i1) continue;
            int rs = a.n.row_ptr[row], rend = a.n.row_ptr[row + 1];
            rs = rs > lo ? rs : lo;
            rend = rend < hi ? rend : hi;
            float rm = -INFINITY, rz = 0.f;
            const float sl = FROM_E ? 0.f : a.s_l[row];
#pragma unroll 4
            for (int k = rs; k < rend; ++k) {
                float e;
                if (FROM_E) e = a.e[k];
                else { e = leaky(sl + a.s_r[a.n.col_idx[k]], a.slope); keep_logit(a, k, e); }  // kept for the second pass
                mz_add(rm, rz, e);
            }
            if (cont && row == i_first) a.carry[chunk] = make_float2(rm, rz);
            else a.stats[row] = make_float2(rm, rz);
        }
        return;
    }

    auto finish_row = [&]() {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(m, off, 64), z2 = __shfl_xor(z, off, 64);
            mz_merge(m, z, m2, z2);
        }
        if (lane == 0) {
            if (cont) a.carry[chunk] = make_float2(m, z);
            else a.stats[i] = make_float2(m, z);
        }
        m = -INFINITY; z = 0.f;
    };

    int pos = lo;
    while (pos < hi) {
        while (re <= pos) { finish_row(); cont = false; ++i; re = a.n.row_ptr[i + 1]; }
        const int seg_hi = re < hi ? re : hi;
        float sl = 0.f;
        if (!FROM_E) sl = a.s_l[i];
        if (FROM_E) {
#pragma unroll 4
            for (int k = pos + lane; k < seg_hi; k += 64) mz_add(m, z, a.e[k]);
        } else {
            // four batches of 64 entries per trip, all loads of a trip requested before the first store: a store may alias
            // anything as far as the compiler knows, so a plain loop would wait for one gather chain per 64 entries
            constexpr int UB = 4;
            for (int k0 = pos + lane; k0 < seg_hi; k0 += 64 * UB) {
                int col[UB], dst[UB];
                float sr[UB];
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    const int k = k0 + 64 * u;
                    const int kc = k < seg_hi ? k : pos;
                    col[u] = a.n.col_idx[kc];
                    dst[u] = a.dst_index ? a.dst_index[kc] : kc;
                }
#pragma unroll
                for (int u = 0; u < UB; ++u) sr[u] = a.s_r[col[u]];
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    if (k0 + 64 * u < seg_hi) {
                        const float e = leaky(sl + sr[u], a.slope);
                        if (dst[u] >= 0) a.logits[dst[u]] = e;  // kept for the second pass (negative: the entry lies in a dense tile)
                        mz_add(m, z, e);
                    }
                }
            }
        }
        pos = seg_hi;
    }
    while (i < i1) {
        finish_row();
        if (re <= hi) { cont = false; ++i; re = (i < a.n.n_rows) ? a.n.row_ptr[i + 1] : 0x7fffffff; }
        else break;
    }
}

// merges the carried (m, z) pieces of rows that span several chunks, in chunk order
__global__ void k_softmax_fixup(SoftmaxArgs a) {
    const int c = 1 + blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.n.n_chunks) return;
    const long long lo = (long long)c * a.n.chunk_nnz;
    const int i0 = a.n.chunk_row[c];
    if ((long long)a.n.row_ptr[i0] <= lo) return;
    const int i = i0 - 1;
    if ((long long)a.n.row_ptr[i] < lo - a.n.chunk_nnz) return;
    const int c_last = (a.n.row_ptr[i + 1] - 1) / a.n.chunk_nnz;
    float2 st = a.stats[i];
    for (int cc = c; cc <= c_last; ++cc) {
        const float2 p = a.carry[cc];
        mz_merge(st.x, st.y, p.x, p.y);
    }
    a.stats[i] = st;
}

// alpha = exp(e - m_i) / z_i; `e` may be the alpha array itself (in place)
__global__ __launch_bounds__(kBlock) void k_softmax_alpha(SoftmaxArgs a) {
    const int chunk = wave_chunk();
    if (chunk >= a.n.n_chunks) return;
    walk_chunk2(a.n, chunk, threadIdx.x & 63, [&](int i) { return a.stats[i]; },
                [&](int k, const float2 &) { return a.e[k]; },
                [&](int k, const float2 &st, float e) { a.alpha[k] = expf(e - st.x) / st.y; });
}

// ------------------------------------------------------------ column panels

// first position in [lo, hi) of an ascending index run whose column is >= bound
__device__ __forceinline__ int lower_bound_col(const int32_t *__restrict__ col_idx, int lo, int hi, int bound) {
    while (lo < hi) {
        const int mid = (int)(((long long)lo + hi) >> 1);
        if (col_idx[mid] < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
}

struct PanelPtrs {
    int32_t *rp[kMaxPanels];  // per panel: n_rows + 1 entries (counts, then row pointers after the scan)
};

// cnt[q][i] = entries of row i whose column lies in panel q (panel q = columns [q*width, (q+1)*width))
__global__ void k_panel_count(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, int n_rows, int n_panels,
                              int width, PanelPtrs pp) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_rows) return;
    if (i == n_rows) {
        for (int q = 0; q < n_panels; ++q) pp.rp[q][n_rows] = 0;
        return;
    }
    const int hi = row_ptr[i + 1];
    int prev = row_ptr[i];
    for (int q = 0; q < n_panels; ++q) {
        const int pos = (q + 1 < n_panels) ? lower_bound_col(col_idx, prev, hi, (q + 1) * width) : hi;
        pp.rp[q][i] = pos - prev;
        prev = pos;
    }
}

// exclusive prefix sum over int32, in place: per-block scan, sequential scan of the block totals, add back
constexpr int kScanPerBlock = 2048;
__global__ __launch_bounds__(256) void k_scan_local(int32_t *data, int n, int32_t *block_sums) {
    __shared__ int part[256];
    const int base = blockIdx.x * kScanPerBlock + threadIdx.x * 8;
    int v[8], sum = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[e] = (base + e < n) ? data[base + e] : 0; sum += v[e]; }
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int add = threadIdx.x >= off ? part[threadIdx.x - off] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    int run = part[threadIdx.x] - sum;  // exclusive prefix of this thread within the block
#pragma unroll
    for (int e = 0; e < 8; ++e) { if (base + e < n) data[base + e] = run; run += v[e]; }
    if (threadIdx.x == 255) block_sums[blockIdx.x] = part[255];
}
__global__ void k_scan_sums(int32_t *block_sums, int n_blocks) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int run = 0;
    for (int b = 0; b < n_blocks; ++b) { const int v = block_sums[b]; block_sums[b] = run; run += v; }
}
__global__ __launch_bounds__(256) void k_scan_add(int32_t *data, int n, const int32_t *__restrict__ block_sums) {
    const int add = block_sums[blockIdx.x];
    const int base = blockIdx.x * kScanPerBlock + threadIdx.x * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) if (base + e < n) data[base + e] += add;
}

// off[q] = number of entries in panels before q (start of panel q in the concatenated column / perm arrays); off[n_panels] = nnz
__global__ void k_panel_offsets(PanelPtrs pp, int n_rows, int n_panels, int32_t *off) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int run = 0;
    for (int q = 0; q < n_panels; ++q) { off[q] = run; run += pp.rp[q][n_rows]; }
    off[n_panels] = run;
}

struct PanelRow {
    int pos[kMaxPanels];   // first entry of the row that belongs to panel q (original numbering)
    int base[kMaxPanels];  // where the row's panel-q entries start in the panel copy
};

// copies every entry's column into its panel and records where each original entry went
__global__ __launch_bounds__(kBlock) void k_panel_scatter(NnzArgs a, int n_panels, int width, PanelPtrs pp, const int32_t *__restrict__ off,
                                                           int32_t *__restrict__ col_out, int32_t *__restrict__ perm_out) {
    const int chunk = wave_chunk();
    if (chunk >= a.n_chunks) return;
    walk_chunk(a, chunk, threadIdx.x & 63,
               [&](int i) {
                   PanelRow rd;
                   const int hi = a.row_ptr[i + 1];
                   int prev = a.row_ptr[i];
#pragma unroll
                   for (int q = 0; q < kMaxPanels; ++q) {
                       rd.pos[q] = prev;
                       rd.base[q] = 0;
                       if (q < n_panels) {
                           rd.base[q] = off[q] + pp.rp[q][i];
                           prev = (q + 1 < n_panels) ? lower_bound_col(a.col_idx, prev, hi, (q + 1) * width) : hi;
                       }
                   }
                   return rd;
               },
               [&](int k, const PanelRow &rd) {
                   const int col = a.col_idx[k];
                   int p = rd.pos[0], b = rd.base[0];
#pragma unroll
                   for (int q = 1; q < kMaxPanels; ++q)
                       if (q < n_panels && col >= q * width) { p = rd.pos[q]; b = rd.base[q]; }
                   const int d = b + (k - p);
                   col_out[d] = col;
                   perm_out[k] = d;
               });
}

// One row-pointer array over the segments (panel q, row i) -> q * n_rows + i of a panel copy, in global positions: the panel
// copy read as a single CSR with n_panels * n_rows rows, whose entries run panel by panel
__global__ void k_panel_segments(PanelPtrs pp, const int32_t *__restrict__ off, int n_rows, int n_panels, int32_t *__restrict__ seg_ptr) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)n_panels * n_rows;
    if (t > total) return;
    if (t == total) { seg_ptr[t] = off[n_panels]; return; }
    const int q = (int)(t / n_rows), i = (int)(t % n_rows);
    seg_ptr[t] = off[q] + pp.rp[q][i];
}

__global__ void k_replicate_f2(const float2 *__restrict__ src, long long n, int copies, float2 *__restrict__ dst) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n * copies) dst[t] = src[t % n];
}

// ------------------------------------------------------- dense tiles of the hub region (set-up kernels)
//
// Nodes are ranked by degree (rank 0 = the longest row / the most referenced column).  In rank order the pattern of a
// skewed graph is nearly dense at the top left; tiles of 128 x 128 ranks that hold enough entries are stored as bit
// masks and multiplied on the matrix cores, the entries outside such tiles stay in a (smaller) CSR remainder.
struct TileMapArgs {
    NnzArgs n;
    const int32_t *rank_r, *rank_c;  // rank of every row / column node; ranks >= h_r / h_c lie outside the tiled region
    int h_r, h_c, nt_c;
};

__device__ __forceinline__ int tile_of(const TileMapArgs &a, int rr, int col) {
    if (rr >= a.h_r) return -1;
    const int rc = a.rank_c[col];
    if (rc >= a.h_c) return -1;
    return (rr >> 7) * a.nt_c + (rc >> 7);
}

__global__ __launch_bounds__(kBlock) void k_tile_hist(TileMapArgs a, int32_t *__restrict__ hist) {
    const int chunk = wave_chunk();
    if (chunk >= a.n.n_chunks) return;
    walk_chunk(a.n, chunk, threadIdx.x & 63, [&](int i) { return a.rank_r[i]; },
               [&](int k, int rr) {
                   const int t = tile_of(a, rr, a.n.col_idx[k]);
                   if (t >= 0) atomicAdd(&hist[t], 1);
               });
}

// sel[t] = 1 where tile t holds at least min_count entries (sel[n_tiles] = 0, the slot that receives the total of the scan)
__global__ void k_tile_flags(const int32_t *__restrict__ hist, int n_tiles, int min_count, int32_t *__restrict__ sel) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t <= n_tiles) sel[t] = (t < n_tiles && hist[t] >= min_count) ? 1 : 0;
}

// after the exclusive scan of sel: slot numbers of the kept tiles (row-major, so the slots of one row of tiles are
// consecutive), the column tile of every slot, the first slot of every row of tiles
__global__ void k_tile_slots(const int32_t *__restrict__ hist, const int32_t *__restrict__ sel_scan, int n_tiles, int nt_r, int nt_c,
                             int min_count, int32_t *__restrict__ slot_of, int32_t *__restrict__ slot_ct, int32_t *__restrict__ slot_rt,
                             int32_t *__restrict__ rt_ptr) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n_tiles) {
        const bool kept = hist[t] >= min_count;
        slot_of[t] = kept ? sel_scan[t] : -1;
        if (kept) {
            slot_ct[sel_scan[t]] = t % nt_c;
            slot_rt[sel_scan[t]] = t / nt_c;
        }
    }
    if (t <= nt_r) rt_ptr[t] = sel_scan[(long long)t * nt_c < n_tiles ? t * nt_c : n_tiles];
}

// bit (row, column) of its tile for every entry inside a kept tile; flag[k] = 1 for the entries that stay sparse;
// where[k] = -(cell + 1) for an entry inside a kept tile, cell = (slot * 128 + row in tile) * 128 + column in tile (-1 when that
// does not fit 31 bits; the entries that stay sparse get their place in the remainder later)
__global__ __launch_bounds__(kBlock) void k_tile_mark(TileMapArgs a, const int32_t *__restrict__ slot_of, unsigned *__restrict__ bits,
                                                       int32_t *__restrict__ flag, int32_t *__restrict__ where) {
    const int chunk = wave_chunk();
    if (chunk >= a.n.n_chunks) return;
    walk_chunk(a.n, chunk, threadIdx.x & 63, [&](int i) { return a.rank_r[i]; },
               [&](int k, int rr) {
                   const int col = a.n.col_idx[k];
                   const int t = tile_of(a, rr, col);
                   const int slot = t >= 0 ? slot_of[t] : -1;
                   if (slot >= 0) {
                       const int rc = a.rank_c[col];
                       atomicOr(&bits[((size_t)slot * 128 + (rr & 127)) * 4 + ((rc & 127) >> 5)], 1u << (rc & 31));
                       where[k] = slot < kMaxCellSlots ? -(((slot * 128 + (rr & 127)) * 128 + (rc & 127)) + 1) : -1;
                   }
                   flag[k] = slot >= 0 ? 0 : 1;
               });
}

// pos = exclusive scan of flag over nnz + 1 slots: entry k stays sparse iff pos[k + 1] != pos[k], at place pos[k]
__global__ __launch_bounds__(kBlock) void k_rem_scatter(NnzArgs a, const int32_t *__restrict__ pos, int32_t *__restrict__ col_rem,
                                                         int32_t *__restrict__ dst_rem) {
    const long long k = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= a.nnz) return;
    const int p = pos[k];
    if (pos[k + 1] != p) {  // stays sparse; the others keep the (negative) cell code k_tile_mark gave them
        col_rem[p] = a.col_idx[k];
        dst_rem[k] = p;
    }
}

// values of the entries that stay sparse, moved from the order of the pattern to the order of the remainder (place: to the place of
// every remainder entry in another order of the remainder, its panel-major copy)
__global__ __launch_bounds__(kBlock) void k_compact_values(long long nnz, const int32_t *__restrict__ dst_rem, const float *__restrict__ src, int stride,
                                                            float *__restrict__ out, const int32_t *__restrict__ place) {
    const long long k = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    const int d = dst_rem[k];
    if (d >= 0) out[place ? place[d] : d] = src[k * stride];
}

__global__ void k_rem_rowptr(const int32_t *__restrict__ row_ptr, int n_rows, const int32_t *__restrict__ pos, int32_t *__restrict__ row_ptr_rem) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= n_rows) row_ptr_rem[i] = pos[row_ptr[i]];
}

__global__ void k_zero_f32(float *__restrict__ p, long long n4) {  // n4 groups of four floats, 16-byte aligned
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n4) reinterpret_cast<float4 *>(p)[t] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ void k_zero_rows(float *__restrict__ C, long long n, int f, long long ldc) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n * f) C[(t / f) * ldc + (t % f)] = 0.f;
}

inline unsigned blocks_for(long long n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

// ------------------------------------------------------- backward of the attention layer

// Row walk shared by the row reductions below: one wavefront per chunk; `piece(i, lo, hi)` handles the stored
// entries [lo, hi) of row i and returns this lane's partial sum, `done(i, sum, cont)` receives the wavefront-wide
// sum of a row piece (cont: the row began in an earlier chunk, the sum goes to the chunk's carry slot).
template <class Piece>
__device__ __forceinline__ void reduce_rows(const NnzArgs &a, int chunk, int lane, float *__restrict__ out, float *__restrict__ carry,
                                            Piece piece) {
    const long long lo_ll = (long long)chunk * a.chunk_nnz;
    const int lo = (int)lo_ll;
    const int hi = (int)((lo_ll + a.chunk_nnz < (long long)a.nnz) ? lo_ll + a.chunk_nnz : (long long)a.nnz);
    const int i0 = a.chunk_row[chunk], i1 = a.chunk_row[chunk + 1];
    bool cont = (a.nnz > 0) && (a.row_ptr[i0] > lo);
    int i = __builtin_amdgcn_readfirstlane(cont ? i0 - 1 : i0);
    int re = __builtin_amdgcn_readfirstlane((i < a.n_rows) ? a.row_ptr[i + 1] : 0x7fffffff);
    float acc = 0.f;
    auto finish_row = [&]() {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) {
            if (cont) carry[chunk] = acc;
            else out[i] = acc;
        }
        acc = 0.f;
    };
    int pos = lo;
    while (pos < hi) {
        while (re <= pos) {
            finish_row();
            cont = false;
            i = __builtin_amdgcn_readfirstlane(i + 1);
            re = __builtin_amdgcn_readfirstlane(a.row_ptr[i + 1]);
        }
        const int seg_hi = re < hi ? re : hi;
        acc += piece(i, pos, seg_hi);
        pos = seg_hi;
    }
    while (i < i1) {
        finish_row();
        if (re <= hi) {
            cont = false;
            i = __builtin_amdgcn_readfirstlane(i + 1);
            re = __builtin_amdgcn_readfirstlane((i < a.n_rows) ? a.row_ptr[i + 1] : 0x7fffffff);
        } else {
            break;
        }
    }
}

// adds the carried pieces of rows that span several chunks, in chunk order
__global__ void k_sum_fixup(NnzArgs a, float *__restrict__ out, const float *__restrict__ carry) {
    const int c = 1 + blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.n_chunks) return;
    const long long lo = (long long)c * a.chunk_nnz;
    const int i0 = a.chunk_row[c];
    if ((long long)a.row_ptr[i0] <= lo) return;
    const int i = i0 - 1;
    if ((long long)a.row_ptr[i] < lo - a.chunk_nnz) return;
    const int c_last = (a.row_ptr[i + 1] - 1) / a.chunk_nnz;
    float s = out[i];
    for (int cc = c; cc <= c_last; ++cc) s += carry[cc];
    out[i] = s;
}

// out[i] = sum of val over the stored entries of row i
__global__ __launch_bounds__(kBlock) void k_row_sum(NnzArgs a, const float *__restrict__ val, int stride, float *__restrict__ out,
                                                     float *__restrict__ carry) {
    const int chunk = wave_chunk();
    if (chunk >= a.n_chunks) return;
    const int lane = threadIdx.x & 63;
    reduce_rows(a, chunk, lane, out, carry, [&](int, int lo, int hi) {
        float s = 0.f;
        for (int k = lo + lane; k < hi; k += 64) s += val[(size_t)k * stride];
        return s;
    });
}

// value of x in another lane by a data-parallel-primitive move (no LDS traffic): quad permutations and the mirror of a
// half row of eight lanes; every lane is active where this is used
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

// ---- per-entry reductions over one 32-column slice (the general g-SDDMM of Eq. 2: a vector per stored entry)
//
// acc[k] (+)= sum over the slice's 32 columns of inner(right[j, col]) for the entries k = (i, j) in [lo, hi) of one row,
// `right` slice-major and already offset by this lane's first column (4 * (lane % 4)).  Four lanes take one neighbour:
// lane `sub` of the four reads columns 4 sub .. 4 sub + 3 and 16 + 4 sub .. 16 + 4 sub + 3, so each of the two loads of
// a step covers 64 contiguous bytes of 16 neighbours' lines; four steps make a batch of 64 entries.  The four partial
// sums a lane holds after a batch (one per step) are reduced across the four lanes and scattered at the same time
// (two exchanges: keep the half this lane will own, hand the other half to the partner), after which lane
// (g = lane / 4, sub) owns entry k0 + 16 sub + g: the read-modify-write of acc is one coalesced 256-byte access.
// Two batches are kept in flight: the gathers (and acc values) of the next batch are requested before the current
// one is reduced.  own(k, v, aux) sees every finished entry once (aux = aux_arr[k] when READ_AUX).
struct SliceBatch {
    float4 b[8];
    float v, aux;
};

template <bool READ_AUX, class Inner, class Own>
__device__ __forceinline__ void slice_piece(const int32_t *__restrict__ col_idx, const float *right, float *acc, const float *aux_arr,
                                            bool first, int lane, int lo, int hi, Inner inner, Own own) {
    const int g = lane >> 2, sub = lane & 3;
    const bool up = (sub & 2) != 0, odd = (sub & 1) != 0;
    auto col_at = [&](int k0) {
        const int kl = k0 + lane;
        return col_idx[kl < hi ? kl : lo];
    };
    auto issue = [&](SliceBatch &B, int col, int k0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = lane_read((u * 16 + g) * 4, col);
            const float *src = right + (size_t)j * 32;
            B.b[2 * u] = *reinterpret_cast<const float4 *>(src);
            B.b[2 * u + 1] = *reinterpret_cast<const float4 *>(src + 16);
        }
        const int k_own = k0 + sub * 16 + g;
        B.v = (k_own < hi && !first) ? acc[k_own] : 0.f;
        B.aux = (READ_AUX && k_own < hi) ? aux_arr[k_own] : 0.f;
    };
    auto consume = [&](SliceBatch &B, int k0) {
        float d[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) d[u] = inner(B.b[2 * u], B.b[2 * u + 1]);
        // lanes 2, 3 of the four will own steps 2, 3: they keep d[2], d[3] and receive the partner's, and hand over d[0], d[1]
        const float keep_a = up ? d[2] : d[0], keep_b = up ? d[3] : d[1];
        const float send_a = up ? d[0] : d[2], send_b = up ? d[1] : d[3];
        const float a2 = keep_a + dpp_f32<0x4E>(send_a);   // from lane ^ 2
        const float b2 = keep_b + dpp_f32<0x4E>(send_b);
        const float keep = odd ? b2 : a2, send = odd ? a2 : b2;
        const float total = keep + dpp_f32<0xB1>(send);    // from lane ^ 1: the sum over the four lanes for step `sub`
        const int k_own = k0 + sub * 16 + g;
        if (k_own < hi) {
            const float v = B.v + total;
            acc[k_own] = v;
            own(k_own, v, B.aux);
        }
    };
    SliceBatch A, B;
    const int c0 = col_at(lo);
    int c1 = col_at(lo + 64);
    issue(A, c0, lo);
    for (int k0 = lo;; k0 += 128) {
        const int c2 = col_at(k0 + 128);
        const bool more_b = k0 + 64 < hi;
        if (more_b) issue(B, c1, k0 + 64);
        consume(A, k0);
        if (!more_b) break;
        c1 = col_at(k0 + 192);
        const bool more_a = k0 + 128 < hi;
        if (more_a) issue(A, c2, k0 + 128);
        consume(B, k0 + 64);
        if (!more_a) break;
    }
}

// Rows of one chunk for a walk that needs no row sums: piece(i, lo, hi) for every row piece.  The row pointers of
// the next 64 rows are fetched at once and handed out by lane reads, so a new row costs no memory round trip.
template <class Piece>
__device__ __forceinline__ void walk_row_pieces(const NnzArgs &a, int chunk, int lane, Piece piece) {
    const long long lo_ll = (long long)chunk * a.chunk_nnz;
    const int lo = (int)lo_ll;
    const int hi = (int)((lo_ll + a.chunk_nnz < (long long)a.nnz) ? lo_ll + a.chunk_nnz : (long long)a.nnz);
    if (lo >= hi) return;
    const int i0 = a.chunk_row[chunk];
    int i = __builtin_amdgcn_readfirstlane((a.row_ptr[i0] > lo) ? i0 - 1 : i0);
    int base = i;
    auto fetch_ends = [&]() {
        const int q = base + 1 + lane;
        return a.row_ptr[q < a.n_rows ? q : a.n_rows];
    };
    int ends = fetch_ends();
    int pos = lo;
    while (pos < hi) {
        if (i - base == 64) {
            base = i;
            ends = fetch_ends();
        }
        const int re = __builtin_amdgcn_readlane(ends, __builtin_amdgcn_readfirstlane(i - base));
        if (re > pos) {
            const int seg_hi = re < hi ? re : hi;
            piece(i, pos, seg_hi);
            pos = seg_hi;
        }
        i = __builtin_amdgcn_readfirstlane(i + 1);
    }
}

struct GatBwdArgs {
    NnzArgs n;
    const float *theta, *dP;  // slice-major (tiles of 32 columns): Theta over the source nodes, dP over the destinations
    const float *logits;      // e_ij per stored entry
    const float2 *mz;         // per row: (max logit, sum of exp(logit - max))
    float *dalpha;            // out, per stored entry: <dP_i, Theta_j>
    float *rowdot, *carry;    // out, per row: sum_j alpha_ij dalpha_ij (+ per-chunk carry slots)
    long long theta_tile, dp_tile;  // floats from one tile to the next
    int n_tiles;
    float scale;  // factor on every dot product (1 in the attention backward; the 1 / sqrt(d) of a key-query score)
};

// dalpha_ij = <dP[i,:], Theta[j,:]> for every stored entry (Eq. 2 with a dot product as the inner operator) together
// with the row sums sum_j alpha_ij dalpha_ij that the softmax backward needs.  One launch per 32-column slice: every
// wavefront of the GPU then gathers from the same contiguous slice of Theta (as the SpMM keeps one slice per L2), and
// the lane that owns an entry adds the slice's share to dalpha[k] - launches follow each other on the stream, so no
// atomics.  The last launch sees the complete dot products and forms the row sums.
template <bool LAST>
__global__ __launch_bounds__(kBlock) void k_gat_dalpha(GatBwdArgs a, int tile, int first) {
    const int chunk = wave_chunk();
    if (chunk >= a.n.n_chunks) return;
    const int lane = threadIdx.x & 63;
    const int sub = lane & 3;
    const float *theta = a.theta + (size_t)tile * a.theta_tile + sub * 4;
    const float *dP = a.dP + (size_t)tile * a.dp_tile + sub * 4;
    auto piece = [&](int i, int lo, int hi) {
        float4 p = *reinterpret_cast<const float4 *>(dP + (size_t)i * 32);
        float4 q = *reinterpret_cast<const float4 *>(dP + (size_t)i * 32 + 16);
        p.x *= a.scale; p.y *= a.scale; p.z *= a.scale; p.w *= a.scale;   // exact when the factor is 1
        q.x *= a.scale; q.y *= a.scale; q.z *= a.scale; q.w *= a.scale;
        float m = 0.f, iz = 0.f, s = 0.f;
        if (LAST) {
            const float2 st = a.mz[i];
            m = st.x;
            iz = inv_z(st.y);
        }
        slice_piece<LAST>(a.n.col_idx, theta, a.dalpha, a.logits, first != 0, lane, lo, hi,
                          [&](const float4 &b, const float4 &c) {
                              return fmaf(b.x, p.x, fmaf(b.y, p.y, fmaf(b.z, p.z, fmaf(b.w, p.w, fmaf(c.x, q.x, fmaf(c.y, q.y, fmaf(c.z, q.z, c.w * q.w)))))));
                          },
                          [&](int, float v, float e) { if (LAST) s = fmaf(expf(e - m) * iz, v, s); });
        return s;
    };
    if (LAST) reduce_rows(a.n, chunk, lane, a.rowdot, a.carry, piece);
    else walk_row_pieces(a.n, chunk, lane, [&](int i, int lo, int hi) { (void)piece(i, lo, hi); });
}

// dalpha of every stored entry from its two sources when the pattern carries a dense-tile split: where[k] >= 0 is the place of
// entry k in the remainder (dalpha_rem), a negative value -(cell + 1) the cell of the dense product Dt that holds it.  Writes
// dalpha in the order of the pattern and forms the row sums sum_j alpha_ij dalpha_ij.
__global__ __launch_bounds__(kBlock) void k_gat_dalpha_merge(NnzArgs a, const int32_t *__restrict__ where, const float *__restrict__ dalpha_rem,
                                                              const float *__restrict__ Dt, const float *__restrict__ logits,
                                                              const float2 *__restrict__ mz, float *__restrict__ dalpha,
                                                              float *__restrict__ rowdot, float *__restrict__ carry) {
    const int chunk = wave_chunk();
    if (chunk >= a.n_chunks) return;
    const int lane = threadIdx.x & 63;
    reduce_rows(a, chunk, lane, rowdot, carry, [&](int i, int lo, int hi) {
        const float2 st = mz[i];
        const float m = st.x, iz = inv_z(st.y);
        float s = 0.f;
        for (int k0 = lo + lane; k0 < hi; k0 += 64 * 4) {
            int w[4];
            float e[4], v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = k0 + 64 * u < hi ? k0 + 64 * u : lo;
                w[u] = where[k];
                e[u] = logits[k];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = w[u] >= 0 ? dalpha_rem[w[u]] : Dt[-(long long)w[u] - 1];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (k0 + 64 * u < hi) {
                    dalpha[k0 + 64 * u] = v[u];
                    s = fmaf(expf(e[u] - m) * iz, v[u], s);
                }
            }
        }
        return s;
    });
}

struct ScoreV2Args {
    NnzArgs n;
    const float *theta_l, *theta_r;  // slice-major: W_l x over the destinations, W_r x over the sources
    const float *att;                // attention vector padded with zeros to a multiple of 32
    float *logits;                   // out, per stored entry
    long long tl_tile, tr_tile;      // floats from one tile to the next
    float slope;
};

// Logits of the GATv2 score, e_ij = sum_m a[m] LeakyReLU(Theta_l[i, m] + Theta_r[j, m]): Eq. 2 with an inner operator
// that is neither a product nor a sum alone.  Same walk as k_gat_dalpha, one launch per 32-column slice.
__global__ __launch_bounds__(kBlock) void k_score_v2(ScoreV2Args a, int tile, int first) {
    const int chunk = wave_chunk();
    if (chunk >= a.n.n_chunks) return;
    const int lane = threadIdx.x & 63;
    const int sub = lane & 3;
    const float *theta_r = a.theta_r + (size_t)tile * a.tr_tile + sub * 4;
    const float *theta_l = a.theta_l + (size_t)tile * a.tl_tile + sub * 4;
    const float4 w = *reinterpret_cast<const float4 *>(a.att + tile * 32 + sub * 4);
    const float4 w2 = *reinterpret_cast<const float4 *>(a.att + tile * 32 + 16 + sub * 4);
    const float slope = a.slope;
    auto term = [&](float wt, float x, float y) {
        const float t = x + y;
        return wt * (t > 0.f ? t : slope * t);
    };
    walk_row_pieces(a.n, chunk, lane, [&](int i, int lo, int hi) {
        const float4 p = *reinterpret_cast<const float4 *>(theta_l + (size_t)i * 32);
        const float4 q = *reinterpret_cast<const float4 *>(theta_l + (size_t)i * 32 + 16);
        slice_piece<false>(a.n.col_idx, theta_r, a.logits, nullptr, first != 0, lane, lo, hi,
                           [&](const float4 &b, const float4 &c) {
                               return ((term(w.x, p.x, b.x) + term(w.y, p.y, b.y)) + (term(w.z, p.z, b.z) + term(w.w, p.w, b.w))) +
                                      ((term(w2.x, q.x, c.x) + term(w2.y, q.y, c.y)) + (term(w2.z, q.z, c.z) + term(w2.w, q.w, c.w)));
                           },
                           [](int, float, float) {});
    });
}

struct GatDtArgs {
    NnzArgs n;
    const float *logits, *dalpha, *rowdot;
    const float2 *mz;
    const int32_t *t_pos;   // place of entry k in the transposed pattern
    float *dt;
    float2 *adt_t;          // (alpha, dt) at the entry's place in the transposed pattern: one 8-byte scattered store
    float slope;
};

// Softmax and LeakyReLU backward per stored entry: alpha = exp(e - m_i) / z_i, de = alpha (dalpha - rowdot_i),
// dt = de * (e > 0 ? 1 : slope) (e > 0 exactly when the pre-activation is).  dt is kept in row order (for the row
// sums ds_l) and, together with alpha, written at its place in the transposed pattern (for ds_r and alpha^T dP).
__global__ __launch_bounds__(kBlock) void k_gat_dt(GatDtArgs a) {
    const int chunk = wave_chunk();
    if (chunk >= a.n.n_chunks) return;
    struct RowData { float m, iz, dot; };
    struct Got { float e, da; int p; };
    walk_chunk2(a.n, chunk, threadIdx.x & 63,
                [&](int i) { const float2 st = a.mz[i]; return RowData{st.x, inv_z(st.y), a.rowdot[i]}; },
                [&](int k, const RowData &) { return Got{a.logits[k], a.dalpha[k], a.t_pos[k]}; },
                [&](int k, const RowData &rd, const Got &g) {
                    const float al = expf(g.e - rd.m) * rd.iz;
                    const float dt = al * (g.da - rd.dot) * (g.e > 0.f ? 1.f : a.slope);
                    a.dt[k] = dt;
                    a.adt_t[g.p] = make_float2(al, dt);
                });
}

// dTheta[j, :] += ds_l[j] a_l + ds_r[j] a_r (ds_l counts only for j < n_l)
__global__ void k_rank1_add(float *__restrict__ D, long long ldd, long long n, int f, const float *__restrict__ ds_l, long long n_l,
                            const float *__restrict__ ds_r, const float *__restrict__ a_l, const float *__restrict__ a_r) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * f) return;
    const long long j = t / f;
    const int q = (int)(t % f);
    const float l = j < n_l ? ds_l[j] : 0.f;
    D[j * ldd + q] += l * a_l[q] + ds_r[j] * a_r[q];
}

// D[i, m] = (accumulate ? D[i, m] : 0) + v[m] G[i, m]: a column scaling, on its own or added to what D holds (G may be D itself)
__global__ void k_scale_cols(float *D, long long ldd, const float *G, long long ldg, const float *__restrict__ v, long long n, int f,
                             int accumulate) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * f) return;
    const long long i = t / f;
    const int m = (int)(t % f);
    const float g = v[m] * G[i * ldg + m];
    D[i * ldd + m] = accumulate ? D[i * ldd + m] + g : g;
}

__global__ void k_set_f32(float *p, long long n, float v) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) p[t] = v;
}

// part[slab][0][q] = sum_j Theta[j, q] v_l[j], part[slab][1][q] = sum_j Theta[j, q] v_r[j] over the rows of the slab,
// Theta slice-major, sums in fp64.  One workgroup per (tile, slab): 32 columns x 8 rows per pass.
__global__ __launch_bounds__(256) void k_theta_t_vec(const float *__restrict__ theta, long long n, int f_pad, const float *__restrict__ v_l,
                                                     long long n_l, const float *__restrict__ v_r, int rows_per_slab,
                                                     double *__restrict__ part) {
    __shared__ double red[2][8][32];
    const int tile = blockIdx.x, slab = blockIdx.y;
    const int c = threadIdx.x & 31, rr = threadIdx.x >> 5;
    const long long j_lo = (long long)slab * rows_per_slab;
    const long long j_hi = (j_lo + rows_per_slab < n) ? j_lo + rows_per_slab : n;
    const float *th = theta + (size_t)tile * (size_t)n * 32;
    double sl = 0.0, sr = 0.0;
    for (long long j = j_lo + rr; j < j_hi; j += 8) {
        const double x = (double)th[j * 32 + c];
        if (j < n_l) sl += x * (double)v_l[j];
        sr += x * (double)v_r[j];
    }
    red[0][rr][c] = sl;
    red[1][rr][c] = sr;
    __syncthreads();
    if (rr < 2) {
        double s = 0.0;
        for (int y = 0; y < 8; ++y) s += red[rr][y][c];
        part[((size_t)slab * 2 + rr) * f_pad + tile * 32 + c] = s;
    }
}

__global__ void k_sum_slabs(const double *__restrict__ part, int slabs, int f_pad, int f, float *__restrict__ out_l, float *__restrict__ out_r) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= f) return;
    double l = 0.0, r = 0.0;
    for (int s = 0; s < slabs; ++s) {
        l += part[((size_t)s * 2 + 0) * f_pad + q];
        r += part[((size_t)s * 2 + 1) * f_pad + q];
    }
    out_l[q] = (float)l;
    out_r[q] = (float)r;
}

// pos[k] = index in the transposed pattern of the entry (i, j) stored at k: the place of i among the ascending
// columns of row j of At.  miss counts entries that are not there (At is not the transpose of A).
__global__ __launch_bounds__(kBlock) void k_transpose_pos(NnzArgs a, const int32_t *__restrict__ t_row_ptr, const int32_t *__restrict__ t_col_idx,
                                                           int32_t *__restrict__ pos, int32_t *__restrict__ miss) {
    const int chunk = wave_chunk();
    if (chunk >= a.n_chunks) return;
    walk_chunk(a, chunk, threadIdx.x & 63, [&](int i) { return i; },
               [&](int k, int i) {
                   const int j = a.col_idx[k];
                   int lo = t_row_ptr[j], hi = t_row_ptr[j + 1];
                   const int end = hi;
                   while (lo < hi) {
                       const int mid = (int)(((long long)lo + hi) >> 1);
                       if (t_col_idx[mid] < i) lo = mid + 1; else hi = mid;
                   }
                   const bool found = lo < end && t_col_idx[lo] == i;
                   pos[k] = found ? lo : 0;
                   if (!found) atomicAdd(miss, 1);
               });
}

// graph feature extractor: out[0] = largest row length, out[1] = sum of squared row lengths (as two 32-bit halves are
// not needed: 64-bit integer atomics), both exact
__global__ void k_row_moments(const int32_t *__restrict__ row_ptr, int n_rows, unsigned long long *__restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long d = 0;
    if (i < n_rows) d = (unsigned long long)(row_ptr[i + 1] - row_ptr[i]);
    unsigned long long mx = d, sq = d * d;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long m2 = __shfl_xor(mx, off, 64), s2 = __shfl_xor(sq, off, 64);
        mx = mx > m2 ? mx : m2;
        sq += s2;
    }
    if ((threadIdx.x & 63) == 0) {
        atomicMax(&out[0], mx);
        atomicAdd(&out[1], sq);
    }
}

__global__ void k_fill_u64(unsigned long long *p, int n, unsigned long long v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

NnzArgs nnz_args(const sensei_csr &A, const ChunkPlan &p) {
    NnzArgs n;
    n.row_ptr = A.row_ptr; n.col_idx = A.col_idx; n.chunk_row = p.chunk_row;
    n.n_rows = A.n_rows; n.nnz = (int)A.nnz; n.chunk_nnz = p.chunk_nnz; n.n_chunks = p.n_chunks;
    return n;
}

}  // namespace

// ----------------------------------------------------------------- host side

// Non-zeros per chunk (= per wavefront).  Large graphs: 512 - with 2048 the same kernels left the GPU short of
// wavefronts: the attention statistics pass took 0.92 ms instead of 0.59 on 115 M non-zeros, an SpMM 64 columns wide
// 1.46 ms instead of 1.34, one 256 wide 4.70 against 4.72 (1024: 4.66; 256: 4.92), the whole three-layer step 13.9 ms
// instead of 13.3 (sweep of 128 .. 2048); only SpMMs 512 or more columns wide lose 1-2 %.
int choose_chunk_nnz(int64_t nnz) {
    if (nnz >= (1LL << 19)) return 512;
    if (nnz >= (1LL << 18)) return 256;
    if (nnz >= (1LL << 17)) return 128;
    return 64;  // small graphs are latency bound: more, shorter wavefronts
}

static int n_chunks_for(int64_t nnz, int t) { return nnz <= 0 ? 1 : (int)((nnz + t - 1) / t); }

size_t plan_bytes(int64_t nnz) {
    return align_up(((size_t)n_chunks_for(nnz, choose_chunk_nnz(nnz)) + 1) * sizeof(int32_t), 256);
}

hipError_t launch_chunk_rows(const sensei_csr &A, const ChunkPlan &p, hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_rows, dim3(blocks_for(p.n_chunks + 1, kBlock)), dim3(kBlock), 0, s, A.row_ptr, A.n_rows,
                       p.chunk_nnz, p.n_chunks, p.chunk_row);
    return hipGetLastError();
}

SpmmShape spmm_shape(const float *B, int64_t ldb, int f) {
    SpmmShape sh;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(B);
    if (f % 4 == 0 && ldb % 4 == 0 && addr % 16 == 0) sh.vec = 4;
    else if (f % 2 == 0 && ldb % 2 == 0 && addr % 8 == 0) sh.vec = 2;
    else sh.vec = 1;
    const int fv = (f + sh.vec - 1) / sh.vec;  // vector columns
    // A neighbour group reads one 128-byte line per neighbour (32 floats) and the feature tiles are spread
    // over the XCDs.  Rows that do not fill whole groups use one wider group instead when that covers the
    // row in a single tile (measured faster than leaving a nearly empty last tile); very wide rows use
    // wider groups so the number of tiles stays moderate.
    const int base = 32 / sh.vec;
    int lpg = base;
    while (lpg > 8 && lpg / 2 >= fv) lpg >>= 1;
    if (fv > lpg && fv <= 32 && fv % lpg != 0) while (lpg < fv) lpg <<= 1;
    while (lpg < 64 && (fv + lpg - 1) / lpg > 32) lpg <<= 1;
    sh.lpg = lpg;
    sh.n_tiles = (fv + lpg - 1) / lpg;
    sh.f_carry = sh.n_tiles * lpg * sh.vec;
    return sh;
}

size_t spmm_carry_bytes(int64_t nnz, int f) {
    const int t = choose_chunk_nnz(nnz);
    // tiles are at most 256 floats wide, so the padded width stays below f + 256
    const size_t f_carry = align_up((size_t)(f > 0 ? f : 1), 32) + 256;
    return align_up((size_t)n_chunks_for(nnz, t) * f_carry * sizeof(float), 256);
}

hipError_t launch_spmm(const sensei_csr &A, int mode, const float *r, const float *c, const float *B, int64_t ldb,
                       int f, float *C, int64_t ldc, int f_store, int act, const ChunkPlan &p, float *carry,
                       hipStream_t s, KernelTimer *timer, bool accumulate, bool finalize, const float2 *mz, bool b_sliced, int val_stride,
                       bool c_sliced, bool defer_fixup, const AttnFusedArgs *fused, const SelfSumArgs *self) {
    SpmmShape sh = spmm_shape(B, ldb, f);
    if (b_sliced) {  // slices of 32 floats per row: one 128-byte line per neighbour and tile
        sh.vec = 4; sh.lpg = 8; sh.n_tiles = (f + 31) / 32; sh.f_carry = sh.n_tiles * 32;
        ldb = 32;
    }
    SpmmArgs a;
    a.tile_stride_b = b_sliced ? (long long)(A.n_cols > 0 ? A.n_cols : 1) * 128 : (long long)sh.vec * sh.lpg * 4;
    a.mz = (mode == kSpmmSoftmax) ? mz : nullptr;
    a.val_stride = val_stride;
    if (c_sliced) ldc = 32;  // requires b_sliced (tiles of 32 columns) and f_store == pad32(f): checked by the callers
    a.c_tf = sh.vec * sh.lpg;
    a.c_tile = c_sliced ? (long long)(A.n_rows > 0 ? A.n_rows : 1) * 32 : (long long)a.c_tf;
    a.row_ptr = A.row_ptr; a.col_idx = A.col_idx; a.chunk_row = p.chunk_row;
    a.val = A.val; a.r = r; a.c = c; a.B = B; a.C = C; a.carry = carry;
    a.ldb = ldb; a.ldc = ldc;
    a.n_rows = A.n_rows; a.nnz = (int)A.nnz; a.chunk_nnz = p.chunk_nnz; a.n_chunks = p.n_chunks;
    a.f = f; a.f_store = f_store; a.f_carry = sh.f_carry; a.n_tiles = sh.n_tiles; a.act = act;
    a.store_vec_ok = (ldc % sh.vec == 0) && (reinterpret_cast<uintptr_t>(C) % (4 * sh.vec) == 0);
    a.accumulate = accumulate ? 1 : 0; a.finalize = finalize ? 1 : 0;
    a.s_l = nullptr; a.s_r = nullptr; a.slope = 0.f; a.mz_out = nullptr; a.carry_mz = nullptr;
    if (mode == kSpmmAttnFused) {
        if (!fused || accumulate || !finalize || defer_fixup) return hipErrorInvalidValue;
        a.s_l = fused->s_l; a.s_r = fused->s_r; a.slope = fused->slope; a.mz_out = fused->row_mz; a.carry_mz = fused->chunk_mz;
    }
    a.self = nullptr; a.self_tile = 0;
    if (mode == kSpmmSignSum || mode == kSpmmLreluSum) {
        if (!self || !self->self_sliced || !b_sliced || !A.val) return hipErrorInvalidValue;
        a.self = self->self_sliced; a.slope = self->slope;
        a.self_tile = (long long)(A.n_rows > 0 ? A.n_rows : 1) * 32;
    }
    const unsigned groups = blocks_for(p.n_chunks, kWavesPerBlock);
    // Feature tiles worked on at the same time (consecutive XCDs take consecutive tiles of the live set): all eight
    // while a 128-byte slice of the gathered matrix is small, four beyond that (measured on the 233 k-node R-MAT graph
    // at F = 256: 6.5 / 6.1 / 5.9 / 6.0 ms with 1 / 2 / 4 / 8 live tiles; 2.45 M nodes at F = 1024: 52.2 / 51.5 / 50.7 / 51.6).
    const double slice_bytes = (double)(A.n_cols > 0 ? A.n_cols : 1) * sh.lpg * sh.vec * 4.0;
    a.tiles_live = slice_bytes > 8e6 ? 4 : 8;
    if (a.tiles_live > sh.n_tiles) a.tiles_live = sh.n_tiles;
    a.n_groups = (int)groups;
    const unsigned n_sets = (unsigned)((sh.n_tiles + a.tiles_live - 1) / a.tiles_live);
    dim3 grid(groups * (unsigned)a.tiles_live * n_sets);
    // byte offsets of the gathered matrix fit 32 bits?
    const bool off32 = (unsigned long long)(A.n_cols > 0 ? A.n_cols : 1) * (unsigned long long)ldb * 4ull + 4ull * (unsigned long long)f <= 0xffffffffull &&
                       A.n_cols < (1 << 24) && ldb * 4 < (1 << 24);
    hipError_t err;
    hipEvent_t t0 = timer ? timer->next() : nullptr, t1 = t0 ? timer->next() : nullptr;
    if (t1 && hipEventRecord(t0, s) != hipSuccess) return hipErrorUnknown;
    switch (sh.vec) {
        case 4: err = spmm_dispatch_lpg<4>(a, mode, sh.lpg, off32, grid, s); break;
        case 2: err = spmm_dispatch_lpg<2>(a, mode, sh.lpg, off32, grid, s); break;
        default: err = spmm_dispatch_lpg<1>(a, mode, sh.lpg, off32, grid, s); break;
    }
    if (err != hipSuccess) return err;
    if (t1 && hipEventRecord(t1, s) != hipSuccess) return hipErrorUnknown;
    if (p.n_chunks > 1 && !(defer_fixup && b_sliced && !finalize)) {
        dim3 fg(blocks_for(p.n_chunks - 1, kWavesPerBlock));
        if (mode == kSpmmAttnFused) hipLaunchKernelGGL(k_spmm_fixup_attn, fg, dim3(kBlock), 0, s, a);
        else hipLaunchKernelGGL(k_spmm_fixup, fg, dim3(kBlock), 0, s, a);
        err = hipGetLastError();
    }
    return err;
}

hipError_t launch_degrees(const sensei_csr &A, int32_t *deg_row, int32_t *deg_col, hipStream_t s) {
    if (A.n_rows > 0) hipLaunchKernelGGL(k_deg_row, dim3(blocks_for(A.n_rows, kBlock)), dim3(kBlock), 0, s, A.row_ptr, A.n_rows, deg_row);
    if (A.n_cols > 0) hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(A.n_cols, kBlock)), dim3(kBlock), 0, s, deg_col, (long long)A.n_cols, 0);
    const int n_ranges = (int)((A.n_cols + kDegRange - 1) / kDegRange);
    if (A.nnz >= (1 << 18) && n_ranges <= kDegRangesMax) {
        int shares = 256 / n_ranges / 8 * 8;  // about one workgroup per compute unit, a multiple of eight shares
        if (shares < 8) shares = 8;
        const long long per_share = (A.nnz + shares - 1) / shares;
        hipLaunchKernelGGL(k_deg_col_ranges, dim3(shares * n_ranges), dim3(kDegThreads), 0, s, A.col_idx, (long long)A.nnz, (int)A.n_cols, n_ranges,
                           per_share, deg_col);
    } else if (A.nnz > 0) {
        hipLaunchKernelGGL(k_deg_col, dim3(blocks_for(A.nnz, kBlock)), dim3(kBlock), 0, s, A.col_idx, (long long)A.nnz, deg_col);
    }
    return hipGetLastError();
}

hipError_t launch_norm_vectors(const int32_t *deg, int64_t n, float *out, hipStream_t s) {
    if (n > 0) hipLaunchKernelGGL(k_norm_vec, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, s, deg, (long long)n, out);
    return hipGetLastError();
}

hipError_t launch_sddmm_norm(const sensei_csr &A, const float *r, const float *c, float *val, const ChunkPlan &p, hipStream_t s) {
    if (A.nnz > 0) hipLaunchKernelGGL(k_sddmm_norm, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, nnz_args(A, p), r, c, val);
    return hipGetLastError();
}

hipError_t launch_score(const sensei_csr &A, const float *s_l, const float *s_r, float slope, float *e, const ChunkPlan &p, hipStream_t s) {
    if (A.nnz > 0) hipLaunchKernelGGL(k_score, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, nnz_args(A, p), s_l, s_r, slope, e);
    return hipGetLastError();
}

hipError_t launch_row_broadcast(const float *s_vec, const float *X, int64_t ldx, int64_t n, int f, float *Y, int64_t ldy, int act, hipStream_t s,
                                const float *mask, int64_t ldm) {
    if (n <= 0 || f <= 0) return hipSuccess;
    const bool a16 = reinterpret_cast<uintptr_t>(X) % 16 == 0 && reinterpret_cast<uintptr_t>(Y) % 16 == 0;
    if (f % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && a16)
        hipLaunchKernelGGL((k_row_broadcast<4>), dim3(blocks_for(n * (f / 4), kBlock)), dim3(kBlock), 0, s, s_vec, X, (long long)ldx, (long long)n, f, Y, (long long)ldy, act, mask, (long long)ldm);
    else
        hipLaunchKernelGGL((k_row_broadcast<1>), dim3(blocks_for(n * f, kBlock)), dim3(kBlock), 0, s, s_vec, X, (long long)ldx, (long long)n, f, Y, (long long)ldy, act, mask, (long long)ldm);
    return hipGetLastError();
}

hipError_t launch_reciprocal(const float *v, int64_t n, float *out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_reciprocal, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, s, v, (long long)n, out);
    return hipGetLastError();
}

hipError_t launch_stack_weights(const float *W, int64_t ldw, int hops, int f_in, int f_out, float *out, int64_t ldo, hipStream_t s) {
    const long long total = (long long)hops * pad32(f_in) * f_out;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_stack_weights, dim3(blocks_for(total, kBlock)), dim3(kBlock), 0, s, W, (long long)ldw, hops, f_in, pad32(f_in), f_out, out, (long long)ldo);
    return hipGetLastError();
}

hipError_t launch_to_slices(const float *s_vec, const float *X, int64_t ldx, int64_t n, int f, float *Y, hipStream_t s, const float *mask,
                            int64_t ldm) {
    if (n <= 0 || f <= 0) return hipSuccess;
    const int x_vec_ok = (ldx % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0) ? 1 : 0;
    const long long threads = n * (long long)(pad32(f) / 4);
    hipLaunchKernelGGL(k_to_slices, dim3(blocks_for(threads, kBlock)), dim3(kBlock), 0, s, s_vec, X, (long long)ldx, (long long)n, f, Y, x_vec_ok, mask, (long long)ldm);
    return hipGetLastError();
}

size_t softmax_ws_bytes(const sensei_csr &A) {
    const int t = choose_chunk_nnz(A.nnz);
    return align_up((size_t)(A.n_rows + 1) * sizeof(float2), 256) + align_up((size_t)n_chunks_for(A.nnz, t) * sizeof(float2), 256);
}

hipError_t launch_softmax(const sensei_csr &A, const float *e, float *alpha, const ChunkPlan &p, float2 *stats, float2 *carry_stats,
                          hipStream_t s) {
    SoftmaxArgs a;
    a.n = nnz_args(A, p);
    a.e = e; a.s_l = nullptr; a.s_r = nullptr; a.slope = 0.f; a.stats = stats; a.carry = carry_stats; a.alpha = alpha;
    a.logits = nullptr; a.dst_index = nullptr;
    dim3 g1(blocks_for(p.n_chunks, kWavesPerBlock));
    hipLaunchKernelGGL((k_softmax_stats<true>), g1, dim3(kBlock), 0, s, a);
    if (p.n_chunks > 1) hipLaunchKernelGGL(k_softmax_fixup, dim3(blocks_for(p.n_chunks - 1, kBlock)), dim3(kBlock), 0, s, a);
    if (A.nnz > 0) hipLaunchKernelGGL(k_softmax_alpha, g1, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attention_stats(const sensei_csr &A, const float *s_l, const float *s_r, float slope, float *logits,
                                  const int32_t *dst_index, const ChunkPlan &p, float2 *stats, float2 *carry_stats, hipStream_t s) {
    SoftmaxArgs a;
    a.n = nnz_args(A, p);
    a.e = nullptr; a.s_l = s_l; a.s_r = s_r; a.slope = slope; a.stats = stats; a.carry = carry_stats; a.alpha = nullptr;
    a.logits = logits; a.dst_index = dst_index;
    hipLaunchKernelGGL((k_softmax_stats<false>), dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, a);
    if (p.n_chunks > 1) hipLaunchKernelGGL(k_softmax_fixup, dim3(blocks_for(p.n_chunks - 1, kBlock)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}


// ------------------------------------------------------------ backward of the attention layer (host side)

hipError_t launch_row_sum(const sensei_csr &A, const float *val, int stride, float *out, const ChunkPlan &p, float *carry, hipStream_t s) {
    const NnzArgs n = nnz_args(A, p);
    hipLaunchKernelGGL(k_row_sum, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, n, val, stride, out, carry);
    if (p.n_chunks > 1) hipLaunchKernelGGL(k_sum_fixup, dim3(blocks_for(p.n_chunks - 1, kBlock)), dim3(kBlock), 0, s, n, out, carry);
    return hipGetLastError();
}

hipError_t launch_gat_dalpha(const sensei_csr &A, const float *theta, const float *dP, int f, const float *logits, const float2 *mz,
                             float *dalpha, float *rowdot, const ChunkPlan &p, float *carry, hipStream_t s, float scale) {
    GatBwdArgs a;
    a.scale = scale;
    a.n = nnz_args(A, p);
    a.theta = theta; a.dP = dP; a.logits = logits; a.mz = mz; a.dalpha = dalpha; a.rowdot = rowdot; a.carry = carry;
    a.theta_tile = (long long)(A.n_cols > 0 ? A.n_cols : 1) * 32;
    a.dp_tile = (long long)(A.n_rows > 0 ? A.n_rows : 1) * 32;
    a.n_tiles = (f + 31) / 32;
    const dim3 grid(blocks_for(p.n_chunks, kWavesPerBlock));
    if (A.nnz <= 0 && !rowdot) return hipSuccess;
    for (int t = 0; t < a.n_tiles; ++t) {
        if (t == a.n_tiles - 1 && rowdot) hipLaunchKernelGGL(k_gat_dalpha<true>, grid, dim3(kBlock), 0, s, a, t, t == 0 ? 1 : 0);
        else hipLaunchKernelGGL(k_gat_dalpha<false>, grid, dim3(kBlock), 0, s, a, t, t == 0 ? 1 : 0);
    }
    if (rowdot && p.n_chunks > 1) hipLaunchKernelGGL(k_sum_fixup, dim3(blocks_for(p.n_chunks - 1, kBlock)), dim3(kBlock), 0, s, a.n, rowdot, carry);
    return hipGetLastError();
}

hipError_t launch_gat_dalpha_merge(const sensei_csr &A, const int32_t *where, const float *dalpha_rem, const float *Dt, const float *logits,
                                   const float2 *mz, float *dalpha, float *rowdot, const ChunkPlan &p, float *carry, hipStream_t s) {
    const NnzArgs n = nnz_args(A, p);
    hipLaunchKernelGGL(k_gat_dalpha_merge, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, n, where, dalpha_rem, Dt, logits, mz, dalpha,
                       rowdot, carry);
    if (p.n_chunks > 1) hipLaunchKernelGGL(k_sum_fixup, dim3(blocks_for(p.n_chunks - 1, kBlock)), dim3(kBlock), 0, s, n, rowdot, carry);
    return hipGetLastError();
}

hipError_t launch_score_v2(const sensei_csr &A, const float *theta_l, const float *theta_r, int f, const float *att_padded, float slope,
                           float *logits, const ChunkPlan &p, hipStream_t s) {
    if (A.nnz <= 0) return hipSuccess;
    ScoreV2Args a;
    a.n = nnz_args(A, p);
    a.theta_l = theta_l; a.theta_r = theta_r; a.att = att_padded; a.logits = logits; a.slope = slope;
    a.tl_tile = (long long)(A.n_rows > 0 ? A.n_rows : 1) * 32;
    a.tr_tile = (long long)(A.n_cols > 0 ? A.n_cols : 1) * 32;
    const dim3 grid(blocks_for(p.n_chunks, kWavesPerBlock));
    const int n_tiles = (f + 31) / 32;
    for (int t = 0; t < n_tiles; ++t) hipLaunchKernelGGL(k_score_v2, grid, dim3(kBlock), 0, s, a, t, t == 0 ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_gat_dt(const sensei_csr &A, const float *logits, const float *dalpha, const float *rowdot, const float2 *mz,
                         const int32_t *t_pos, float slope, float *dt, float2 *adt_t, const ChunkPlan &p, hipStream_t s) {
    if (A.nnz <= 0) return hipSuccess;
    GatDtArgs a;
    a.n = nnz_args(A, p);
    a.logits = logits; a.dalpha = dalpha; a.rowdot = rowdot; a.mz = mz; a.t_pos = t_pos; a.dt = dt; a.adt_t = adt_t;
    a.slope = slope;
    hipLaunchKernelGGL(k_gat_dt, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_rank1_add(float *D, int64_t ldd, int64_t n, int f, const float *ds_l, int64_t n_l, const float *ds_r, const float *a_l,
                            const float *a_r, hipStream_t s) {
    if (n <= 0 || f <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_rank1_add, dim3(blocks_for(n * f, kBlock)), dim3(kBlock), 0, s, D, (long long)ldd, (long long)n, f, ds_l, (long long)n_l,
                       ds_r, a_l, a_r);
    return hipGetLastError();
}

hipError_t launch_scale_cols(float *D, int64_t ldd, const float *G, int64_t ldg, const float *v, int64_t n, int f, bool accumulate, hipStream_t s) {
    if (n <= 0 || f <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_scale_cols, dim3(blocks_for(n * f, kBlock)), dim3(kBlock), 0, s, D, (long long)ldd, G, (long long)ldg, v, (long long)n, f,
                       accumulate ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float *p, int64_t n, float v, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_set_f32, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, s, p, (long long)n, v);
    return hipGetLastError();
}

static int theta_t_slabs(int64_t n) {
    const long long s = (n + 4095) / 4096;
    return (int)(s < 1 ? 1 : s > 256 ? 256 : s);
}

size_t theta_t_vec_bytes(int64_t n, int f) { return align_up((size_t)theta_t_slabs(n) * 2 * (size_t)pad32(f) * sizeof(double), 256); }

hipError_t launch_theta_t_vec(const float *theta_sliced, int64_t n, int f, const float *v_l, int64_t n_l, const float *v_r, float *out_l,
                              float *out_r, double *part, hipStream_t s) {
    if (f <= 0) return hipSuccess;
    const int slabs = theta_t_slabs(n), f_pad = pad32(f);
    const int rows_per_slab = (int)((((n > 0 ? n : 1) + slabs - 1) / slabs + 7) / 8 * 8);
    hipLaunchKernelGGL(k_theta_t_vec, dim3((unsigned)(f_pad / 32), (unsigned)slabs), dim3(256), 0, s, theta_sliced, (long long)n, f_pad, v_l,
                       (long long)n_l, v_r, rows_per_slab, part);
    hipLaunchKernelGGL(k_sum_slabs, dim3(blocks_for(f, 256)), dim3(256), 0, s, part, slabs, f_pad, f, out_l, out_r);
    return hipGetLastError();
}

hipError_t launch_transpose_pos(const sensei_csr &A, const sensei_csr &At, const ChunkPlan &p, int32_t *pos, int32_t *miss, hipStream_t s) {
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, s, miss, 1LL, 0);  // a fill kernel, not a memset: safe under stream capture too
    if (A.nnz <= 0) return hipGetLastError();
    hipLaunchKernelGGL(k_transpose_pos, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, nnz_args(A, p), At.row_ptr, At.col_idx,
                       pos, miss);
    return hipGetLastError();
}


hipError_t launch_row_moments(const sensei_csr &A, unsigned long long *out2, hipStream_t s) {
    hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(64), 0, s, out2, 2, 0ull);
    if (A.n_rows > 0) hipLaunchKernelGGL(k_row_moments, dim3(blocks_for(A.n_rows, kBlock)), dim3(kBlock), 0, s, A.row_ptr, A.n_rows, out2);
    return hipGetLastError();
}

// ------------------------------------------------------------ column panels (host side)

hipError_t launch_exclusive_scan(int32_t *data, int n, int32_t *block_sums, hipStream_t s) {
    const unsigned nb = blocks_for(n, kScanPerBlock);
    hipLaunchKernelGGL(k_scan_local, dim3(nb), dim3(256), 0, s, data, n, block_sums);
    hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(64), 0, s, block_sums, (int)nb);
    hipLaunchKernelGGL(k_scan_add, dim3(nb), dim3(256), 0, s, data, n, (const int32_t *)block_sums);
    return hipGetLastError();
}

size_t scan_temp_bytes(int n) { return align_up(((size_t)blocks_for(n, kScanPerBlock) + 1) * sizeof(int32_t), 256); }

hipError_t launch_panel_build(const sensei_csr &A, const ChunkPlan &plan, int n_panels, int width, int32_t *const *rp, int32_t *off,
                              int32_t *col_out, int32_t *perm_out, int32_t *scan_temp, hipStream_t s) {
    PanelPtrs pp;
    for (int q = 0; q < kMaxPanels; ++q) pp.rp[q] = q < n_panels ? rp[q] : nullptr;
    hipLaunchKernelGGL(k_panel_count, dim3(blocks_for((long long)A.n_rows + 1, kBlock)), dim3(kBlock), 0, s, A.row_ptr, A.col_idx, A.n_rows,
                       n_panels, width, pp);
    hipError_t err = hipGetLastError();
    for (int q = 0; q < n_panels && err == hipSuccess; ++q) err = launch_exclusive_scan(rp[q], A.n_rows + 1, scan_temp, s);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(k_panel_offsets, dim3(1), dim3(64), 0, s, pp, A.n_rows, n_panels, off);
    if (A.nnz > 0)
        hipLaunchKernelGGL(k_panel_scatter, dim3(blocks_for(plan.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s, nnz_args(A, plan), n_panels,
                           width, pp, (const int32_t *)off, col_out, perm_out);
    return hipGetLastError();
}

hipError_t launch_panel_segments(int32_t *const *rp, const int32_t *off, int n_rows, int n_panels, int32_t *seg_ptr, hipStream_t s) {
    PanelPtrs pp;
    for (int q = 0; q < kMaxPanels; ++q) pp.rp[q] = q < n_panels ? rp[q] : nullptr;
    hipLaunchKernelGGL(k_panel_segments, dim3(blocks_for((long long)n_panels * n_rows + 1, kBlock)), dim3(kBlock), 0, s, pp, off, n_rows, n_panels, seg_ptr);
    return hipGetLastError();
}

hipError_t launch_replicate_stats(const float2 *src, int64_t n, int copies, float2 *dst, hipStream_t s) {
    if (n <= 0 || copies <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_replicate_f2, dim3(blocks_for(n * copies, kBlock)), dim3(kBlock), 0, s, src, (long long)n, copies, dst);
    return hipGetLastError();
}

// ------------------------------------------------------------ dense tiles (host side)

// exclusive scan of up to 2^31 ints: the block totals are scanned by the same three kernels instead of one thread
size_t scan_large_temp_bytes(long long n) {
    const long long nb = (n + kScanPerBlock - 1) / kScanPerBlock;
    return align_up((size_t)(nb + 1) * sizeof(int32_t), 256) + scan_temp_bytes((int)(nb + 1));
}

hipError_t launch_exclusive_scan_large(int32_t *data, long long n, int32_t *temp, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned nb = blocks_for(n, kScanPerBlock);
    int32_t *sums = temp;
    int32_t *temp2 = temp + align_up((size_t)(nb + 1) * sizeof(int32_t), 256) / sizeof(int32_t);
    hipLaunchKernelGGL(k_scan_local, dim3(nb), dim3(256), 0, s, data, (int)n, sums);
    const hipError_t e = launch_exclusive_scan(sums, (int)nb, temp2, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_scan_add, dim3(nb), dim3(256), 0, s, data, (int)n, (const int32_t *)sums);
    return hipGetLastError();
}

static TileMapArgs tile_map_args(const sensei_csr &A, const ChunkPlan &p, const int32_t *rank_r, const int32_t *rank_c, int h_r, int h_c, int nt_c) {
    TileMapArgs a;
    a.n = nnz_args(A, p);
    a.rank_r = rank_r; a.rank_c = rank_c; a.h_r = h_r; a.h_c = h_c; a.nt_c = nt_c;
    return a;
}

hipError_t launch_tile_select(const sensei_csr &A, const ChunkPlan &p, const int32_t *rank_r, const int32_t *rank_c, int h_r, int h_c,
                              int nt_r, int nt_c, int min_count, int32_t *hist, int32_t *sel_scan, int32_t *slot_of, int32_t *slot_ct,
                              int32_t *slot_rt, int32_t *rt_ptr, int32_t *scan_temp, hipStream_t s) {
    const int n_tiles = nt_r * nt_c;
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n_tiles, kBlock)), dim3(kBlock), 0, s, hist, (long long)n_tiles, 0);
    if (A.nnz > 0)
        hipLaunchKernelGGL(k_tile_hist, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s,
                           tile_map_args(A, p, rank_r, rank_c, h_r, h_c, nt_c), hist);
    hipLaunchKernelGGL(k_tile_flags, dim3(blocks_for(n_tiles + 1, kBlock)), dim3(kBlock), 0, s, (const int32_t *)hist, n_tiles, min_count, sel_scan);
    const hipError_t e = launch_exclusive_scan(sel_scan, n_tiles + 1, scan_temp, s);
    if (e != hipSuccess) return e;
    const int span = n_tiles > nt_r + 1 ? n_tiles : nt_r + 1;
    hipLaunchKernelGGL(k_tile_slots, dim3(blocks_for(span, kBlock)), dim3(kBlock), 0, s, (const int32_t *)hist, (const int32_t *)sel_scan, n_tiles,
                       nt_r, nt_c, min_count, slot_of, slot_ct, slot_rt, rt_ptr);
    return hipGetLastError();
}

hipError_t launch_tile_split(const sensei_csr &A, const ChunkPlan &p, const int32_t *rank_r, const int32_t *rank_c, int h_r, int h_c, int nt_c,
                             const int32_t *slot_of, int n_slots, unsigned *bits, int32_t *pos, int32_t *scan_temp, int32_t *col_rem,
                             int32_t *dst_rem, int32_t *row_ptr_rem, hipStream_t s) {
    if (n_slots > 0) hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for((long long)n_slots * 512, kBlock)), dim3(kBlock), 0, s,
                                        reinterpret_cast<int32_t *>(bits), (long long)n_slots * 512, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, s, pos + A.nnz, 1LL, 0);
    if (A.nnz > 0)
        hipLaunchKernelGGL(k_tile_mark, dim3(blocks_for(p.n_chunks, kWavesPerBlock)), dim3(kBlock), 0, s,
                           tile_map_args(A, p, rank_r, rank_c, h_r, h_c, nt_c), slot_of, bits, pos, dst_rem);
    const hipError_t e = launch_exclusive_scan_large(pos, (long long)A.nnz + 1, scan_temp, s);
    if (e != hipSuccess) return e;
    if (A.nnz > 0) hipLaunchKernelGGL(k_rem_scatter, dim3(blocks_for(A.nnz, kBlock)), dim3(kBlock), 0, s, nnz_args(A, p), (const int32_t *)pos, col_rem, dst_rem);
    hipLaunchKernelGGL(k_rem_rowptr, dim3(blocks_for((long long)A.n_rows + 1, kBlock)), dim3(kBlock), 0, s, A.row_ptr, A.n_rows, (const int32_t *)pos,
                       row_ptr_rem);
    return hipGetLastError();
}

hipError_t launch_compact_values(int64_t nnz, const int32_t *dst_rem, const float *src, int stride, float *out, hipStream_t s, const int32_t *place) {
    if (nnz <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_compact_values, dim3(blocks_for(nnz, kBlock)), dim3(kBlock), 0, s, (long long)nnz, dst_rem, src, stride, out, place);
    return hipGetLastError();
}

// C (n x f, row-major with ldc, or slice-major when `sliced`) = 0
hipError_t launch_zero_matrix(float *C, int64_t n, int f, int64_t ldc, bool sliced, hipStream_t s) {
    if (n <= 0 || f <= 0) return hipSuccess;
    if (sliced || ldc == f) {
        const long long total = (long long)n * (sliced ? pad32(f) : f);
        if (total % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0) {
            hipLaunchKernelGGL(k_zero_f32, dim3(blocks_for(total / 4, kBlock)), dim3(kBlock), 0, s, C, total / 4);
            return hipGetLastError();
        }
        hipLaunchKernelGGL(k_zero_rows, dim3(blocks_for(total, kBlock)), dim3(kBlock), 0, s, C, total, 1, 1LL);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_zero_rows, dim3(blocks_for((long long)n * f, kBlock)), dim3(kBlock), 0, s, C, (long long)n, f, (long long)ldc);
    return hipGetLastError();
}

}  // namespace sensei
