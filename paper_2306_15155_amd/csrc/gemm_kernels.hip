// Dense kernels for gfx950: the fp32 update GEMM on the matrix cores with the activation fused into the
// epilogue (small products: v_mfma_f32_32x32x2_f32; large ones: v_mfma_f32_32x32x16_bf16 on three exact
// bf16 pieces per fp32 operand), the dense tiles of the hub region of a skewed graph (the same bf16
// instruction), the weight-gradient GEMM with fp64 slabs, and a two-vector GEMV for the attention projections.
#include "sensei_internal.h"

#include <type_traits>

namespace sensei {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int KT = 16;  // k extent of one LDS tile

struct GemmArgs {
    const float *A, *W, *row_scale;  // row_scale: optional per-row factor applied before the activation
    float *Y;
    long long lda, ldw, ldy, n;
    int k, m, m_store, act, n_bn;
    int y_sliced;  // Y stored slice-major in tiles of 32 columns: (row, col) at Y[(col / 32) * n * 32 + row * 32 + col % 32]
    long long a_slice;   // floats from columns 32 s .. 32 s + 31 of A to the next 32: 32 for a row-major A, n * 32 (with lda = 32) for a slice-major one
    const float *add;    // optional n x pad32(m) slice-major matrix added to the product before scaling and activation
};

// Block tile BM x BN, 4 wavefronts laid out WGM x WGN, each computing TM x TN tiles of 32 x 32
// with the 32x32x2 fp32 MFMA.  LDS holds A as [k][row] and W as [k][col] so that the MFMA operand
// reads (lane l takes k = l / 32, row or col = l % 32) are consecutive words.  The next k-tile is
// fetched from HBM into registers while the current one is multiplied.
template <int BM, int BN, int WGM, int WGN, int AVEC, int BVEC>
__global__ __launch_bounds__(kThreads) void k_gemm(GemmArgs g) {
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
    constexpr int APAD = 36, BPAD = 36;  // row stride = 36 mod 64 words: the two k-rows an MFMA operand read touches fall on (nearly) disjoint LDS banks, and the four k-rows a stash writes are 16 banks apart
    constexpr int A_TPR = KT / AVEC;             // threads per A row
    constexpr int A_RPP = kThreads / A_TPR;      // A rows per pass
    constexpr int A_PASSES = BM / A_RPP;
    constexpr int B_TPR = BN / BVEC;             // threads per W row
    constexpr int B_RPP = kThreads / B_TPR;      // W rows per pass
    constexpr int B_PASSES = (KT + B_RPP - 1) / B_RPP;
    __shared__ float As[KT][BM + APAD];
    __shared__ __attribute__((aligned(16))) float Bs[KT][BN + BPAD];

    const int t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const long long m0 = (long long)(blockIdx.x / g.n_bn) * BM;
    const int n0 = (int)(blockIdx.x % g.n_bn) * BN;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float ra[A_PASSES][AVEC];
    float rb[B_PASSES][BVEC];
    const int a_row = t / A_TPR, a_kk = (t % A_TPR) * AVEC;
    const int b_row = t / B_TPR, b_nn = (t % B_TPR) * BVEC;

    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const long long row = m0 + p * A_RPP + a_row;
            const int kk = k0 + a_kk;
            if (row < g.n && kk < g.k) {
                const float *src = g.A + row * g.lda + (long long)(kk >> 5) * g.a_slice + (kk & 31);
                if (AVEC == 4) { float4 v = *reinterpret_cast<const float4 *>(src); ra[p][0] = v.x; ra[p][1 % AVEC] = v.y; ra[p][2 % AVEC] = v.z; ra[p][3 % AVEC] = v.w; }
                else if (AVEC == 2) { float2 v = *reinterpret_cast<const float2 *>(src); ra[p][0] = v.x; ra[p][1 % AVEC] = v.y; }
                else ra[p][0] = *src;
            } else {
#pragma unroll
                for (int e = 0; e < AVEC; ++e) ra[p][e] = 0.f;
            }
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int kr = p * B_RPP + b_row;
            const int kk = k0 + kr;
            const int col = n0 + b_nn;
            if (kr < KT && kk < g.k && col < g.m) {
                const float *src = g.W + (long long)kk * g.ldw + col;
                if (BVEC == 4) { float4 v = *reinterpret_cast<const float4 *>(src); rb[p][0] = v.x; rb[p][1 % BVEC] = v.y; rb[p][2 % BVEC] = v.z; rb[p][3 % BVEC] = v.w; }
                else rb[p][0] = *src;
            } else {
#pragma unroll
                for (int e = 0; e < BVEC; ++e) rb[p][e] = 0.f;
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p)
#pragma unroll
            for (int e = 0; e < AVEC; ++e) As[a_kk + e][p * A_RPP + a_row] = ra[p][e];
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int kr = p * B_RPP + b_row;
            if (kr < KT) {
#pragma unroll
                for (int e = 0; e < BVEC; ++e) Bs[kr][b_nn + e] = rb[p][e];
            }
        }
    };

    const int n_kt = (g.k + KT - 1) / KT;
    fetch(0);
    for (int kt = 0; kt < n_kt; ++kt) {
        stash();
        __syncthreads();
        if (kt + 1 < n_kt) fetch((kt + 1) * KT);
        const int kh = lane >> 5, ll = lane & 31;
#pragma unroll
        for (int kk = 0; kk < KT; kk += 2) {
            float av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[kk + kh][(wm * TM + i) * 32 + ll];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[j] = Bs[kk + kh][(wn * TN + j) * 32 + ll];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator layout of the 32x32 tile: register r of lane l holds
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const int kh = lane >> 5, ll = lane & 31;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + ll;
            if (col >= g.m_store) continue;
            const long long y_col = g.y_sliced ? (long long)(col >> 5) * g.n * 32 + (col & 31) : (long long)col;
            const long long y_ld = g.y_sliced ? 32 : g.ldy;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long long row = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * kh + (r % 4);
                if (row < g.n) {
                    float y = acc[i][j][r];
                    if (g.add) y += g.add[(long long)(col >> 5) * g.n * 32 + row * 32 + (col & 31)];
                    if (g.row_scale) y *= g.row_scale[row];
                    if (g.act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
                    g.Y[row * y_ld + y_col] = y;
                }
            }
        }
}

template <int BM, int BN, int WGM, int WGN>
hipError_t gemm_launch_vec(const GemmArgs &g, int avec, int bvec, hipStream_t s) {
    const long long n_bm = (g.n + BM - 1) / BM;
    dim3 grid((unsigned)(n_bm * g.n_bn));
#define SENSEI_GEMM_CASE(AV, BV) \
    hipLaunchKernelGGL((k_gemm<BM, BN, WGM, WGN, AV, BV>), grid, dim3(kThreads), 0, s, g)
    if (bvec == 4) {
        if (avec == 4) SENSEI_GEMM_CASE(4, 4); else if (avec == 2) SENSEI_GEMM_CASE(2, 4); else SENSEI_GEMM_CASE(1, 4);
    } else {
        if (avec == 4) SENSEI_GEMM_CASE(4, 1); else if (avec == 2) SENSEI_GEMM_CASE(2, 1); else SENSEI_GEMM_CASE(1, 1);
    }
#undef SENSEI_GEMM_CASE
    return hipGetLastError();
}

// ---- the same GEMM on the bf16 matrix cores, which run 16 times the fp32 rate, at fp32 accuracy.  Every fp32 operand element
// is cut into three bf16 pieces of eight significand bits (truncate, subtract, truncate, subtract: the pieces add up to the
// element exactly); of the nine piece products of a term the six of weight 2^-16 and above are formed (a1 b1, a1 b2, a2 b1, a1 b3,
// a2 b2, a3 b1), each exact, and accumulated in fp32 by the matrix core: what is left out is below 2^-23 of the term, the
// rounding of the fp32 instruction.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void split_bf16x3(float v, unsigned &hi, unsigned &mid, unsigned &lo) {
    hi = __float_as_uint(v) & 0xFFFF0000u;
    const float r1 = v - __uint_as_float(hi);          // exact: at most 16 significant bits remain
    mid = __float_as_uint(r1) & 0xFFFF0000u;
    lo = __float_as_uint(r1 - __uint_as_float(mid));   // exact: at most 8 significant bits, so its low half is zero
}
// two fp32 bit patterns whose low halves do not matter -> their high halves as a pair of bf16 (first in the low half)
__device__ __forceinline__ unsigned pack_bf16(unsigned first, unsigned second) { return __builtin_amdgcn_perm(second, first, 0x07060302u); }

// Block tile 256 x 32 TN: four wavefronts stacked over the rows, each 64 rows x 32 TN columns (2 x TN accumulators).  The
// 256 x 16 block of A of a step goes through LDS as fp32 (fetched with neighbouring lanes on one row, so that a row's 64 bytes
// are one request); a lane of the 32 x 32 x 16 instruction holds eight consecutive k of one row, reads them back as two 16-byte
// words and cuts them into pieces in registers.  The 16 x 32 TN block of W of a step is cut once per workgroup (a thread:
// eight k of one column) and left in LDS in lane order.  Two buffers each, filled for step s + 1 while step s multiplies: one
// barrier per step.  Rows past the end are computed from the last row and dropped.
template <int TN, int AVEC>
__global__ __launch_bounds__(kThreads, 2) void k_gemm_bf(GemmArgs g) {
    constexpr int BM = 256, BN = 32 * TN;
    constexpr int A_TPR = 16 / AVEC, A_RPP = kThreads / A_TPR, A_PASSES = BM / A_RPP;   // threads per row, rows per pass
    constexpr int ALD = 20;   // floats per row of A in LDS: 16 k and 16 bytes of padding (conflict-free 16-byte reads of 16 rows)
    __shared__ __attribute__((aligned(16))) float As[2][BM][ALD];
    __shared__ __attribute__((aligned(16))) unsigned short Bs[2][3][TN][2][32][8];
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63, kh = lane >> 5, ll = lane & 31;
    const long long m0 = (long long)(blockIdx.x / g.n_bn) * BM;
    const int n0 = (int)(blockIdx.x % g.n_bn) * BN;

    floatx16 acc[2][TN];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int a_row = t / A_TPR, a_kk = (t % A_TPR) * AVEC;
    float ra[A_PASSES][AVEC];
    // Addresses: a uniform base that moves with k, plus a 32-bit byte offset per lane and pass that never changes (the row within
    // the block, clamped to the last row of A, and the lane's k): nothing per step is left for the vector ALU.
    const float *a_blk = g.A + m0 * g.lda;
    unsigned a_off[A_PASSES];
#pragma unroll
    for (int p = 0; p < A_PASSES; ++p) {
        long long row = m0 + p * A_RPP + a_row;
        if (row > g.n - 1) row = g.n - 1;
        a_off[p] = (unsigned)(((row - m0) * g.lda + a_kk) * 4);
    }
    // a step whose 16 k all exist: vector fetches; the last step of a k that is no multiple of 16 (and the idle fetch past the
    // last step): element by element from a clamped k, zeros past k
    auto fetch_a = [&](int k0, auto whole) {
        const char *src = reinterpret_cast<const char *>(a_blk + (long long)(k0 >> 5) * g.a_slice + (k0 & 31));
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            if constexpr (decltype(whole)::value) {
                if (AVEC == 4) { const float4 v = *reinterpret_cast<const float4 *>(src + a_off[p]); ra[p][0] = v.x; ra[p][1 % AVEC] = v.y; ra[p][2 % AVEC] = v.z; ra[p][3 % AVEC] = v.w; }
                else if (AVEC == 2) { const float2 v = *reinterpret_cast<const float2 *>(src + a_off[p]); ra[p][0] = v.x; ra[p][1 % AVEC] = v.y; }
                else ra[p][0] = *reinterpret_cast<const float *>(src + a_off[p]);
            } else {
                const float *base = reinterpret_cast<const float *>(reinterpret_cast<const char *>(a_blk) + a_off[p]) - a_kk;   // the row's first element
#pragma unroll
                for (int e = 0; e < AVEC; ++e) {
                    const int k = k0 + a_kk + e, kc = k < g.k ? k : g.k - 1;
                    const float v = base[(long long)(kc >> 5) * g.a_slice + (kc & 31)];
                    ra[p][e] = __uint_as_float(__float_as_uint(v) & (k < g.k ? ~0u : 0u));   // a mask, not a branch around the fetch
                }
            }
        }
    };
    auto stash_a = [&](int buf) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            float *dst = &As[buf][p * A_RPP + a_row][a_kk];
            if (AVEC == 4) *reinterpret_cast<float4 *>(dst) = make_float4(ra[p][0], ra[p][1 % AVEC], ra[p][2 % AVEC], ra[p][3 % AVEC]);
            else if (AVEC == 2) *reinterpret_cast<float2 *>(dst) = make_float2(ra[p][0], ra[p][1 % AVEC]);
            else *dst = ra[p][0];
        }
    };
    const bool w_on = t < 2 * BN;
    const int wcol = t % BN, wkh = (t / BN) & 1;
    const bool wcol_ok = n0 + wcol < g.m;
    const unsigned wmask = wcol_ok ? ~0u : 0u;   // columns past m read the last column and are cleared: a mask, not a branch around the fetch
    const unsigned w_off = (unsigned)(((long long)wkh * 8 * g.ldw + (wcol_ok ? n0 + wcol : g.m - 1)) * 4);
    float w_raw[8];
    auto fetch_w = [&](int k0, auto whole) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if constexpr (decltype(whole)::value) {
                const char *row = reinterpret_cast<const char *>(g.W + (long long)(k0 + e) * g.ldw);   // uniform
                w_raw[e] = __uint_as_float(__float_as_uint(*reinterpret_cast<const float *>(row + w_off)) & wmask);
            } else {   // rows past k read the last row: their factors in A are zero
                const int k = k0 + wkh * 8 + e;
                const char *row = reinterpret_cast<const char *>(g.W + (long long)(k < g.k ? k : g.k - 1) * g.ldw - (long long)wkh * 8 * g.ldw);
                w_raw[e] = __uint_as_float(__float_as_uint(*reinterpret_cast<const float *>(row + w_off)) & wmask);
            }
        }
    };
    auto stash_w = [&](int buf) {
        unsigned pc[8][3];
#pragma unroll
        for (int e = 0; e < 8; ++e) split_bf16x3(w_raw[e], pc[e][0], pc[e][1], pc[e][2]);
        if (w_on) {
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                uintx4 w;
#pragma unroll
                for (int d = 0; d < 4; ++d) w[d] = pack_bf16(pc[2 * d][p], pc[2 * d + 1][p]);
                *reinterpret_cast<uintx4 *>(&Bs[buf][p][wcol >> 5][wkh][wcol & 31][0]) = w;
            }
        }
    };

    // one step: fetch what step st + 1 needs, multiply step st out of the buffers st & 1, then fill the other buffers
    auto step = [&](int st, auto next_whole) {
        const int k1 = (st + 1) * 16;
        fetch_a(k1, next_whole);   // past the last step: zeros, not used
        fetch_w(k1, next_whole);
        __builtin_amdgcn_sched_barrier(0);   // the fetches stay here and their use stays below the multiply: the scheduler would join them
        __syncthreads();   // this step's blocks are in As[st & 1], Bs[st & 1]; nobody reads the other buffers any more
        uintx4 af[2][3];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float *src = &As[st & 1][wave * 64 + i * 32 + ll][kh * 8];
            const float4 lo4 = *reinterpret_cast<const float4 *>(src), hi4 = *reinterpret_cast<const float4 *>(src + 4);
            const float av[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
            unsigned pc[8][3];
#pragma unroll
            for (int e = 0; e < 8; ++e) split_bf16x3(av[e], pc[e][0], pc[e][1], pc[e][2]);
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int d = 0; d < 4; ++d) af[i][p][d] = pack_bf16(pc[2 * d][p], pc[2 * d + 1][p]);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            uintx4 bf[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) bf[p] = *reinterpret_cast<const uintx4 *>(&Bs[st & 1][p][j][kh][ll][0]);
#pragma unroll
            for (int pa = 2; pa >= 0; --pa)
#pragma unroll
                for (int pb = 2 - pa; pb >= 0; --pb)   // smallest products first
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[i][pa]), __builtin_bit_cast(bf16x8, bf[pb]),
                                                                             acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        stash_a((st + 1) & 1);
        stash_w((st + 1) & 1);
    };
    const int n_full = g.k / 16, n_steps = (g.k + 15) / 16;
    if (n_full > 0) { fetch_a(0, std::true_type()); fetch_w(0, std::true_type()); }
    else { fetch_a(0, std::false_type()); fetch_w(0, std::false_type()); }
    stash_a(0);
    stash_w(0);
    int st = 0;
    for (; st + 1 < n_full; ++st) step(st, std::true_type());
    for (; st < n_steps; ++st) step(st, std::false_type());

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + j * 32 + ll;
            if (col >= g.m_store) continue;
            const long long y_col = g.y_sliced ? (long long)(col >> 5) * g.n * 32 + (col & 31) : (long long)col;
            const long long y_ld = g.y_sliced ? 32 : g.ldy;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long long row = m0 + wave * 64 + i * 32 + 8 * (r / 4) + 4 * kh + (r % 4);
                if (row < g.n) {
                    float y = acc[i][j][r];
                    if (g.add) y += g.add[(long long)(col >> 5) * g.n * 32 + row * 32 + (col & 31)];
                    if (g.row_scale) y *= g.row_scale[row];
                    if (g.act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
                    g.Y[row * y_ld + y_col] = y;
                }
            }
        }
}

template <int TN>
hipError_t gemm_bf_launch(const GemmArgs &g, int avec, hipStream_t s) {
    const dim3 grid((unsigned)(((g.n + 255) / 256) * g.n_bn));
    if (avec == 4) hipLaunchKernelGGL((k_gemm_bf<TN, 4>), grid, dim3(kThreads), 0, s, g);
    else if (avec == 2) hipLaunchKernelGGL((k_gemm_bf<TN, 2>), grid, dim3(kThreads), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf<TN, 1>), grid, dim3(kThreads), 0, s, g);
    return hipGetLastError();
}

// ---- dense tiles of the hub region: C[order_r[rank], :] = sum over the kept 128 x 128 tiles of the rank's row of tiles of
// (tile bits) . B[tile columns, :], B in rank order.  The rows of tiles of the largest hubs keep hundreds of tiles, the others a
// few: the kept tiles of a row are therefore cut into segments of at most kTilesPerSegment, one workgroup per (segment, group
// of 32-column blocks); a segment leaves its 128 x f partial product in `part`, and k_tiles_reduce adds the segments of a row
// in order (no atomics).
// The value-less product on the bf16 matrix cores, which run 16 times the fp32 rate, without giving up fp32 accuracy: a
// tile entry is 0 or 1, exact in bf16, and every fp32 element of the right-hand operand is cut into three bf16 pieces of
// eight significand bits each (truncate, subtract, truncate, subtract: the pieces add up to the element exactly), so the three
// products per piece are exact and only the fp32 accumulation of the matrix core rounds, as it does in the fp32 instruction.
// Neither operand passes through LDS and the wavefronts never synchronise:
//   - a lane of the 32 x 32 x 16 instruction holds eight consecutive k of one tile row, i.e. one byte of that row's 128-bit
//     mask, which it expands in registers (to 2.0 = 0x4000, a single bit per entry; the stored result is halved);
//   - the right-hand operand is cut into its pieces once per call, by the kernel that gathers it into rank order, and stored
//     in the order the instruction's lanes read it: per (piece, column tile, 16 k, 32 columns) one contiguous kilobyte, lane
//     (k half, column) holding its eight k, so an operand fetch is one 16-byte load per lane straight from global memory.
// A wavefront owns 128 tile rows x 32 columns (four accumulators) and walks its segment's tiles with the fetches running three
// steps of 16 k ahead; the wavefronts of a workgroup only share the segment.
// eight mask bits -> eight bf16 of value 0 or 2.0: bit k is copied to k and k + 15, then each pair (2d, 2d + 1) is moved onto
// bits 14 and 30 of its word
__device__ __forceinline__ uintx4 expand_mask_byte(unsigned byte) {
    unsigned twice = byte | (byte << 15);
    asm volatile("" : "+v"(twice));   // keeps the shifts below shifts: folded with the line above they become 32-bit multiplies, four times as slow
    uintx4 a;
#pragma unroll
    for (int d = 0; d < 4; ++d) a[d] = (twice << (14 - 2 * d)) & 0x40004000u;
    return a;
}

// Bq: the gathered matrix in rank order, cut into bf16 pieces, in the lane order described above.  Element (rank q = 128 ct +
// 16 k16 + 8 kh + e, column n = 32 nb + nl) of piece p sits at p * n_ranks * f + ((((ct * 8 + k16) * (f / 32) + nb) * 2 + kh) * 32 + nl) * 8 + e.
// One thread: eight consecutive ranks of one column (one 16-byte store per piece).  Rows are those of the slice-major matrix B
// (zeros where the rank has no node), times 1 / mz[node].y if mz is given.
__global__ void k_gather_ranked_split(const float *__restrict__ B, long long n_cols, int f, const int32_t *__restrict__ order_c, long long n_ranks,
                                      unsigned short *__restrict__ Bq, const float2 *__restrict__ mz) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int nb_count = f / 32;
    if (t >= n_ranks / 8 * f) return;
    const int nl = (int)(t & 31);
    const int nb = (int)((t >> 5) % nb_count);
    const long long g8 = (t >> 5) / nb_count;
    const long long q0 = g8 * 8;
    unsigned pc[8][3];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int j = order_c[q0 + e];
        float v = j >= 0 ? B[(long long)nb * n_cols * 32 + (long long)j * 32 + nl] : 0.f;
        if (mz && j >= 0) { const float z = mz[j].y; v *= z > 0.f ? 1.f / z : 0.f; }
        split_bf16x3(v, pc[e][0], pc[e][1], pc[e][2]);
    }
    const long long at = ((g8 >> 1) * nb_count + nb) * 512 + (g8 & 1) * 256 + nl * 8;   // g8 = (ct * 8 + k16) * 2 + kh
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        uintx4 w;
#pragma unroll
        for (int d = 0; d < 4; ++d) w[d] = pack_bf16(pc[2 * d][p], pc[2 * d + 1][p]);
        *reinterpret_cast<uintx4 *>(Bq + (long long)p * n_ranks * f + at) = w;
    }
}

struct DenseTilesBfArgs {
    const unsigned *bits;                  // n_slots x 128 rows x 4 words
    const int32_t *seg_first, *slot_ct;    // first slot of each segment (n_seg + 1 entries); column tile of a slot
    const unsigned short *Bq;              // k_gather_ranked_split's output
    float *part;                           // n_seg x 128 x f
    long long plane;                       // elements per piece: ranks x f
    int f, n_bn;                           // f: multiple of 32; n_bn: workgroups (of up to four 32-column blocks) per segment
};

__global__ __launch_bounds__(kThreads) void k_dense_tiles_bf(DenseTilesBfArgs g) {
    constexpr int PF = 3, RING = PF + 1;   // fetch distance in steps of 16 k; 8 steps per tile, so ring positions are static
    const int seg = blockIdx.x / g.n_bn;
    const int lane = threadIdx.x & 63;
    const int nb = (blockIdx.x % g.n_bn) * 4 + (threadIdx.x >> 6);   // this wavefront's block of 32 columns
    const int nb_count = g.f / 32;
    if (nb >= nb_count) return;            // wavefronts do not synchronise: an idle one may leave
    const int s0 = __builtin_amdgcn_readfirstlane(g.seg_first[seg]), s1 = __builtin_amdgcn_readfirstlane(g.seg_first[seg + 1]);
    if (s0 >= s1) return;
    const int kh = lane >> 5, ll = lane & 31;

    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    uintx4 ring[RING][3];
    uintx4 ab[4], ab_n[4];
    const unsigned short *bq = g.Bq + (long long)nb * 512 + lane * 8;
    auto fetch = [&](int ct, int k16, int pos) {
        const unsigned short *at = bq + ((long long)ct * 8 + k16) * nb_count * 512;
#pragma unroll
        for (int p = 0; p < 3; ++p) ring[pos][p] = *reinterpret_cast<const uintx4 *>(at + p * g.plane);
    };
    auto fetch_bits = [&](int slot) {
#pragma unroll
        for (int i = 0; i < 4; ++i) ab_n[i] = *reinterpret_cast<const uintx4 *>(g.bits + ((size_t)slot * 128 + i * 32 + ll) * 4);
    };

    int ct = g.slot_ct[s0], ct_next = g.slot_ct[s0 + 1 < s1 ? s0 + 1 : s0];
    fetch_bits(s0);
    __builtin_amdgcn_sched_barrier(0);   // the fetches complete in issue order: the order here is the one the loop continues
#pragma unroll
    for (int k = 0; k < PF; ++k) {
        fetch(ct, k, k);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int slot = s0; slot < s1; ++slot) {
        // the loop body has no branches, so that the fetches stay in flight across iterations: past the last tile it fetches
        // that tile again and drops the result
        const int slot_next = slot + 1 < s1 ? slot + 1 : slot;
        const int ct_after = g.slot_ct[slot + 2 < s1 ? slot + 2 : s1 - 1];   // needed one tile from now: by then it has long arrived
#pragma unroll
        for (int i = 0; i < 4; ++i) ab[i] = ab_n[i];
#pragma unroll
        for (int k16 = 0; k16 < 8; ++k16) {
            if (k16 + PF < 8) fetch(ct, k16 + PF, (k16 + PF) % RING);
            else fetch(ct_next, k16 + PF - 8, (k16 + PF) % RING);
            if (k16 == 4) fetch_bits(slot_next);
            __builtin_amdgcn_sched_barrier(0);   // keeps the fetches PF steps ahead of their use: the scheduler would sink them to it
            uintx4 av[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = expand_mask_byte((ab[i][k16 >> 1] >> ((k16 & 1) * 16 + kh * 8)) & 0xFFu);
#pragma unroll
            for (int p = 2; p >= 0; --p)   // smallest pieces first
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[i]), __builtin_bit_cast(bf16x8, ring[k16 % RING][p]),
                                                                     acc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        ct = ct_next;
        ct_next = __builtin_amdgcn_readfirstlane(ct_after);   // placed after the last scheduling barrier: it does not wait on the fetches in flight
    }

    float *out = g.part + (size_t)seg * 128 * g.f + nb * 32 + ll;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[(size_t)(i * 32 + 8 * (r / 4) + 4 * kh + (r % 4)) * g.f] = 0.5f * acc[i][r];
}

// The attention modes on the bf16 matrix cores.  Entry (i, k) of a tile weighs w = exp(LeakyReLU(u[i] + v[k]) - shift), an fp32
// number, which is cut into three bf16 pieces like the right-hand operand; of the nine piece products the six of weight
// 2^-16 and above are formed (w1 b1, w1 b2, w2 b1, w1 b3, w2 b2, w3 b1: what is left out is below 2^-23 of a term, the rounding
// of the fp32 instruction).  kTilesAttn: u = s_l, v = s_r, shift = the maximum of row i (tiles of the pattern itself).
// kTilesAttnT: the tiles are those of the transposed pattern, so the softmax row is the tile's column: u = s_r, v = s_l,
// shift = the maximum of column k.
// The weights of one step (128 rows x 16 k) are computed once per workgroup, every thread a few of them, and shared through
// LDS (two buffers: the weights of step s + 1 are written while step s multiplies, one barrier per step); a wavefront owns 128
// rows x 32 columns as in the value-less kernel and fetches its right-hand pieces straight from global memory one step ahead.
// NW wavefronts per workgroup (as many 32-column blocks, up to eight); a workgroup whose last blocks do not exist lets those
// wavefronts repeat the last block and drop the result, so that every wavefront reaches every barrier.
struct DenseTilesAttnArgs {
    const unsigned *bits;
    const int32_t *seg_first, *slot_ct, *seg_rt;
    const unsigned short *Bq;
    float *part;
    long long plane;
    int f, n_bn;
    const float *u_rank, *m_rank;    // by row rank: u, and (kTilesAttn) the shift
    const float *v_rank, *mc_rank;   // by column rank: v, and (kTilesAttnT) the shift
    float slope;
};
constexpr int kTilesAttn = 1, kTilesAttnT = 2;

template <int MODE, int NW>
__global__ __launch_bounds__(64 * NW) void k_dense_tiles_attn_bf(DenseTilesAttnArgs g) {
    constexpr int THREADS = 64 * NW;
    constexpr int KP = NW >= 8 ? 4 : NW == 4 ? 8 : 16;   // consecutive k per thread and row when the weights are formed
    constexpr int TPR = 16 / KP;                          // threads per row
    constexpr int RPT = 128 * TPR / THREADS;              // rows per thread (2 for a single wavefront)
    constexpr int AROW = 24;                              // bf16 per row of a piece in LDS: 16 k and 16 bytes of padding (conflict-free 16-byte reads)
    __shared__ __attribute__((aligned(16))) unsigned short As[2][3][128][AROW];
    const int seg = blockIdx.x / g.n_bn;
    const int t = threadIdx.x, lane = t & 63;
    const int nb_count = g.f / 32;
    const int nb_want = (blockIdx.x % g.n_bn) * NW + (t >> 6);
    const bool stores = nb_want < nb_count;
    const int nb = stores ? nb_want : nb_count - 1;
    const int s0 = __builtin_amdgcn_readfirstlane(g.seg_first[seg]), s1 = __builtin_amdgcn_readfirstlane(g.seg_first[seg + 1]);
    if (s0 >= s1) return;
    const int rt = g.seg_rt[seg];
    const int kh = lane >> 5, ll = lane & 31;
    const int a_row = t / TPR, a_kq = t % TPR;

    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    float u_t[RPT], m_t[RPT];
    uintx4 ab[RPT], ab_n[RPT];
#pragma unroll
    for (int rr = 0; rr < RPT; ++rr) {
        const int row = a_row + rr * (THREADS / TPR);
        u_t[rr] = g.u_rank[rt * 128 + row];
        m_t[rr] = MODE == kTilesAttn ? g.m_rank[rt * 128 + row] : 0.f;
    }
    auto fetch_bits = [&](int slot) {
#pragma unroll
        for (int rr = 0; rr < RPT; ++rr)
            ab_n[rr] = *reinterpret_cast<const uintx4 *>(g.bits + ((size_t)slot * 128 + a_row + rr * (THREADS / TPR)) * 4);
    };
    uintx4 ring[2][3];
    const unsigned short *bq = g.Bq + (long long)nb * 512 + lane * 8;
    auto fetch = [&](int ct, int k16, int pos) {
        const unsigned short *at = bq + ((long long)ct * 8 + k16) * nb_count * 512;
#pragma unroll
        for (int p = 0; p < 3; ++p) ring[pos][p] = *reinterpret_cast<const uintx4 *>(at + p * g.plane);
    };
    float4 vv[KP / 4], mc[KP / 4];
    auto fetch_v = [&](int ct, int k16) {
#pragma unroll
        for (int q = 0; q < KP / 4; ++q) {
            vv[q] = *reinterpret_cast<const float4 *>(g.v_rank + (size_t)ct * 128 + k16 * 16 + a_kq * KP + q * 4);
            if (MODE == kTilesAttnT) mc[q] = *reinterpret_cast<const float4 *>(g.mc_rank + (size_t)ct * 128 + k16 * 16 + a_kq * KP + q * 4);
        }
    };
    // the weights of step k16 of the tile whose mask rows are `mask`, from the vectors fetch_v has brought, into buffer `buf`
    auto weights = [&](const uintx4 (&mask)[RPT], int k16, int buf) {
#pragma unroll
        for (int rr = 0; rr < RPT; ++rr) {
            const unsigned present = (mask[rr][k16 >> 1] >> ((k16 & 1) * 16 + a_kq * KP)) & ((1u << KP) - 1u);
            unsigned pc[KP][3];
#pragma unroll
            for (int e = 0; e < KP; ++e) {
                const float4 v4 = vv[e / 4];
                const float ve = (e & 3) == 0 ? v4.x : (e & 3) == 1 ? v4.y : (e & 3) == 2 ? v4.z : v4.w;
                float tt = u_t[rr] + ve;
                tt = tt > 0.f ? tt : g.slope * tt;
                float shift = m_t[rr];
                if (MODE == kTilesAttnT) { const float4 c4 = mc[e / 4]; shift = (e & 3) == 0 ? c4.x : (e & 3) == 1 ? c4.y : (e & 3) == 2 ? c4.z : c4.w; }
                const float w = ((present >> e) & 1u) ? __expf(tt - shift) : 0.f;
                split_bf16x3(w, pc[e][0], pc[e][1], pc[e][2]);
            }
            const int row = a_row + rr * (THREADS / TPR);
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                unsigned short *dst = &As[buf][p][row][a_kq * KP];
#pragma unroll
                for (int q = 0; q < KP / 4; ++q)
                    *reinterpret_cast<uint2 *>(dst + q * 4) = make_uint2(pack_bf16(pc[q * 4][p], pc[q * 4 + 1][p]), pack_bf16(pc[q * 4 + 2][p], pc[q * 4 + 3][p]));
            }
        }
    };

    int ct = g.slot_ct[s0], ct_next = g.slot_ct[s0 + 1 < s1 ? s0 + 1 : s0];
    fetch_bits(s0);
    fetch_v(ct, 0);
    fetch(ct, 0, 0);
#pragma unroll
    for (int rr = 0; rr < RPT; ++rr) ab[rr] = ab_n[rr];
    weights(ab, 0, 0);
    for (int slot = s0; slot < s1; ++slot) {
        // no branches in the body (the fetches stay in flight across iterations): past the last tile it works on that tile again
        // and drops the result
        const int slot_next = slot + 1 < s1 ? slot + 1 : slot;
        const int ct_after = g.slot_ct[slot + 2 < s1 ? slot + 2 : s1 - 1];
#pragma unroll
        for (int k16 = 0; k16 < 8; ++k16) {
            // what the next step needs: its right-hand pieces, and the column vectors its weights are formed from
            if (k16 < 7) { fetch(ct, k16 + 1, (k16 + 1) & 1); fetch_v(ct, k16 + 1); }
            else { fetch(ct_next, 0, 0); fetch_v(ct_next, 0); }
            if (k16 == 3) fetch_bits(slot_next);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();   // the weights of this step are in As[k16 & 1]; nobody reads the other buffer any more
#pragma unroll
            for (int pa = 2; pa >= 0; --pa) {
                uintx4 av[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) av[i] = *reinterpret_cast<const uintx4 *>(&As[k16 & 1][pa][i * 32 + ll][kh * 8]);
#pragma unroll
                for (int pb = 2 - pa; pb >= 0; --pb)   // smallest products first
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[i]), __builtin_bit_cast(bf16x8, ring[k16 & 1][pb]),
                                                                         acc[i], 0, 0, 0);
            }
            if (k16 < 7) weights(ab, k16 + 1, (k16 + 1) & 1);
            else weights(ab_n, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int rr = 0; rr < RPT; ++rr) ab[rr] = ab_n[rr];
        ct = ct_next;
        ct_next = __builtin_amdgcn_readfirstlane(ct_after);
    }

    if (!stores) return;
    float *out = g.part + (size_t)seg * 128 * g.f + nb * 32 + ll;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[(size_t)(i * 32 + 8 * (r / 4) + 4 * kh + (r % 4)) * g.f] = acc[i][r];
}

// Dh[rank, :] = sum of the partial products of the segments of the rank's row of tiles, in segment order (zeros for a row of
// tiles that kept none)
__global__ void k_tiles_reduce(const float *__restrict__ part, const int32_t *__restrict__ rt_seg, int nt_r, int f, float *__restrict__ Dh) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int f4 = f / 4;
    if (t >= (long long)nt_r * 128 * f4) return;
    const int col = (int)(t % f4) * 4;
    const int rank = (int)(t / f4);
    const int rt = rank >> 7, row = rank & 127;
    const int g0 = rt_seg[rt], g1 = rt_seg[rt + 1];
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int sg = g0; sg < g1; ++sg) {
        const float4 v = *reinterpret_cast<const float4 *>(part + ((size_t)sg * 128 + row) * f + col);
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    *reinterpret_cast<float4 *>(Dh + (size_t)rank * f + col) = sum;
}

// C[i, :] = act(scale_i * (C[i, :] + Dh[rank of i, :])): joins the raw sums of the sparse remainder with those of the tiles
// and applies what the SpMM epilogue would have applied (scale_i = r[i], or 1 / z_i in attention mode)
__global__ void k_tiles_combine(float *__restrict__ C, long long n_rows, int f_store, long long ldc, long long c_tile, const float *__restrict__ Dh,
                                int f, const int32_t *__restrict__ rank_r, int n_ranks, const float *__restrict__ r, const float2 *__restrict__ mz,
                                int act, int vec4, const int32_t *__restrict__ row_ptr, int chunk_nnz, const float *__restrict__ carry, int f_carry,
                                const float *__restrict__ tile_shift) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int f4 = (f_store + 3) / 4;
    if (t >= n_rows * f4) return;
    const long long i = t / f4;
    const int col = (int)(t % f4) * 4;
    const int rank = rank_r[i];
    float sc = 1.f;
    if (mz) { const float z = mz[i].y; sc = z > 0.f ? 1.f / z : 0.f; }
    else if (r) sc = r[i];
    float *dst = C + (long long)(col >> 5) * c_tile + i * ldc + (col & 31);
    const float *add = (rank < n_ranks) ? Dh + (size_t)rank * f + col : nullptr;
    // attention tiles that were multiplied before the row maxima were known used the maximum over the row's tile entries as the shift:
    // exp(that - the row maximum) brings their sum to the row's scale
    float tf = 1.f;
    if (tile_shift && add) { const float ts = tile_shift[rank]; tf = ts > -INFINITY ? __expf(ts - mz[i].x) : 0.f; }
    // the SpMM's own fix-up, when the caller left it to this pass: a row that spans chunk boundaries has its later pieces in the
    // carry slots of the chunks it continues into, c * chunk_nnz strictly inside the row; they are added in chunk order
    long long c_first = 1, c_last = 0;
    if (row_ptr) {
        const long long rs = row_ptr[i], re = row_ptr[i + 1];
        if (re > rs) {
            c_first = rs / chunk_nnz + 1;
            c_last = (re - 1) / chunk_nnz;
        }
    }
    if (vec4 && col + 3 < f_store) {  // 16-byte accesses when the caller found every row start aligned
        float4 y = *reinterpret_cast<const float4 *>(dst);
#pragma unroll 4
        for (long long c = c_first; c <= c_last; ++c) {
            const float4 p = *reinterpret_cast<const float4 *>(carry + (size_t)c * f_carry + col);
            y.x += p.x; y.y += p.y; y.z += p.z; y.w += p.w;
        }
        if (add) {
            const float4 a4 = *reinterpret_cast<const float4 *>(add);
            y.x += tf * a4.x; y.y += tf * a4.y; y.z += tf * a4.z; y.w += tf * a4.w;
        }
        y.x *= sc; y.y *= sc; y.z *= sc; y.w *= sc;
        if (act == SENSEI_ACT_RELU) {
            y.x = y.x > 0.f ? y.x : 0.f; y.y = y.y > 0.f ? y.y : 0.f; y.z = y.z > 0.f ? y.z : 0.f; y.w = y.w > 0.f ? y.w : 0.f;
        }
        *reinterpret_cast<float4 *>(dst) = y;
        return;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (col + e < f_store) {
            float y = dst[e];
            for (long long c = c_first; c <= c_last; ++c) y += carry[(size_t)c * f_carry + col + e];
            y = (y + (add ? tf * add[e] : 0.f)) * sc;
            if (act == SENSEI_ACT_RELU) y = y > 0.f ? y : 0.f;
            dst[e] = y;
        }
    }
}

// The join for a remainder that ran panel-major: the row's raw sum is spread over its n_panels segments (panel q, row i), each with
// the carry slots of the chunks the segment continues into; they are added panel by panel, chunk by chunk (a fixed order).
__global__ void k_tiles_combine_pm(float *__restrict__ C, long long n_rows, int f_store, long long ldc, long long c_tile, const float *__restrict__ Dh,
                                   int f, const int32_t *__restrict__ rank_r, int n_ranks, const float *__restrict__ r, const float2 *__restrict__ mz,
                                   int act, int vec4, const float *__restrict__ part, int n_panels, const int32_t *__restrict__ seg_ptr, int chunk_nnz,
                                   const float *__restrict__ carry, int f_carry, const float *__restrict__ tile_shift) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int f4 = (f_store + 3) / 4;
    if (t >= n_rows * f4) return;
    const long long i = t / f4;
    const int col = (int)(t % f4) * 4;
    const int rank = rank_r[i];
    float sc = 1.f;
    if (mz) { const float z = mz[i].y; sc = z > 0.f ? 1.f / z : 0.f; }
    else if (r) sc = r[i];
    const long long part_tile = (long long)n_panels * n_rows * 32;
    float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int q = 0; q < n_panels; ++q) {
        const long long seg = (long long)q * n_rows + i;
        const float4 p = *reinterpret_cast<const float4 *>(part + (long long)(col >> 5) * part_tile + seg * 32 + (col & 31));
        y.x += p.x; y.y += p.y; y.z += p.z; y.w += p.w;
        const long long rs = seg_ptr[seg], re = seg_ptr[seg + 1];
        if (re > rs) {
            for (long long c = rs / chunk_nnz + 1; c <= (re - 1) / chunk_nnz; ++c) {
                const float4 v = *reinterpret_cast<const float4 *>(carry + (size_t)c * f_carry + col);
                y.x += v.x; y.y += v.y; y.z += v.z; y.w += v.w;
            }
        }
    }
    if (rank < n_ranks) {
        float tf = 1.f;   // see k_tiles_combine
        if (tile_shift) { const float ts = tile_shift[rank]; tf = ts > -INFINITY ? __expf(ts - mz[i].x) : 0.f; }
        const float4 a4 = *reinterpret_cast<const float4 *>(Dh + (size_t)rank * f + col);
        y.x += tf * a4.x; y.y += tf * a4.y; y.z += tf * a4.z; y.w += tf * a4.w;
    }
    y.x *= sc; y.y *= sc; y.z *= sc; y.w *= sc;
    if (act == SENSEI_ACT_RELU) {
        y.x = y.x > 0.f ? y.x : 0.f; y.y = y.y > 0.f ? y.y : 0.f; y.z = y.z > 0.f ? y.z : 0.f; y.w = y.w > 0.f ? y.w : 0.f;
    }
    float *dst = C + (long long)(col >> 5) * c_tile + i * ldc + (col & 31);
    if (vec4 && col + 3 < f_store) {
        *reinterpret_cast<float4 *>(dst) = y;
    } else {
        if (col < f_store) dst[0] = y.x;
        if (col + 1 < f_store) dst[1] = y.y;
        if (col + 2 < f_store) dst[2] = y.z;
        if (col + 3 < f_store) dst[3] = y.w;
    }
}

// Dt[slot] = Lh[rows of the slot's row tile] . Rh[rows of its column tile]^T, 128 x 128 per kept tile: the per-entry dot product
// <dP_i, Theta_j> of the attention backward for all entries of a tile at once, on the matrix cores (the cells outside the tile's
// bit mask are computed too and never read).  Both operands are rows with k contiguous, so both go through the transposing
// stash the GEMM uses for its left operand.
__global__ __launch_bounds__(kThreads) void k_tiles_sddmm(const float *__restrict__ Lh, const float *__restrict__ Rh, int f,
                                                           const int32_t *__restrict__ slot_rt, const int32_t *__restrict__ slot_ct,
                                                           float *__restrict__ Dt) {
    constexpr int BM = 128, BN = 128, WGN = 2, TM = 2, TN = 2, PAD = 36;
    __shared__ float As[KT][BM + PAD];
    __shared__ float Bs[KT][BN + PAD];
    const int slot = blockIdx.x;
    const int t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const float *Lt = Lh + (size_t)slot_rt[slot] * 128 * f;
    const float *Rt = Rh + (size_t)slot_ct[slot] * 128 * f;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[2], rb[2];
    const int a_row = t >> 2, a_kk = (t & 3) * 4;  // 64 rows per pass, 4 threads (16 k) per row
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            ra[p] = *reinterpret_cast<const float4 *>(Lt + (size_t)(p * 64 + a_row) * f + k0 + a_kk);
            rb[p] = *reinterpret_cast<const float4 *>(Rt + (size_t)(p * 64 + a_row) * f + k0 + a_kk);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const float va[4] = {ra[p].x, ra[p].y, ra[p].z, ra[p].w}, vb[4] = {rb[p].x, rb[p].y, rb[p].z, rb[p].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                As[a_kk + e][p * 64 + a_row] = va[e];
                Bs[a_kk + e][p * 64 + a_row] = vb[e];
            }
        }
    };
    const int n_kt = f / KT;  // f is a multiple of 32
    fetch(0);
    for (int kt = 0; kt < n_kt; ++kt) {
        stash();
        __syncthreads();
        if (kt + 1 < n_kt) fetch((kt + 1) * KT);
        const int kh = lane >> 5, ll = lane & 31;
#pragma unroll
        for (int kk = 0; kk < KT; kk += 2) {
            float av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[kk + kh][(wm * TM + i) * 32 + ll];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[j] = Bs[kk + kh][(wn * TN + j) * 32 + ll];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }
    const int kh = lane >> 5, ll = lane & 31;
    float *out = Dt + (size_t)slot * 128 * 128;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = (wm * TM + i) * 32 + 8 * (r / 4) + 4 * kh + (r % 4);
#pragma unroll
            for (int j = 0; j < TN; ++j) out[(size_t)row * 128 + (wn * TN + j) * 32 + ll] = acc[i][j][r];
        }
}

// the attention vectors in rank order (zeros where a rank has no node)
__global__ void k_gather_ranked_vecs(const float *__restrict__ s_l, const float *__restrict__ s_r, const float2 *__restrict__ mz,
                                     const int32_t *__restrict__ order_r, int n_r, const int32_t *__restrict__ order_c, int n_c,
                                     float *__restrict__ sl_rank, float *__restrict__ m_rank, float *__restrict__ sr_rank) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < n_r) {
        const int i = order_r[q];
        sl_rank[q] = i >= 0 ? s_l[i] : 0.f;
        if (mz) m_rank[q] = i >= 0 ? mz[i].x : 0.f;
    }
    if (q < n_c) {
        const int j = order_c[q];
        sr_rank[q] = j >= 0 ? s_r[j] : 0.f;
    }
}

// (max, sum of exp) of the attention logits over the entries of one segment of tiles, per row of its row of tiles: two threads per
// row, each walks the set bits of its half of the row's mask in every tile of the segment; the column vector of the tile sits in LDS.
// A tile is first searched for its maximum, then summed against the running maximum, so a row costs one rescale per tile.
__global__ __launch_bounds__(256) void k_tile_stats(const unsigned *__restrict__ bits, const int32_t *__restrict__ seg_first,
                                                    const int32_t *__restrict__ slot_ct, const int32_t *__restrict__ seg_rt,
                                                    const float *__restrict__ sl_rank, const float *__restrict__ sr_rank, float slope,
                                                    float2 *__restrict__ seg_stats) {
    __shared__ float sr_s[128];
    const int seg = blockIdx.x;
    const int s0 = seg_first[seg], s1 = seg_first[seg + 1];
    const int t = threadIdx.x, row = t >> 1, half = t & 1;
    const float sl = sl_rank[(size_t)seg_rt[seg] * 128 + row];
    float m = -INFINITY, z = 0.f;
    for (int slot = s0; slot < s1; ++slot) {
        __syncthreads();  // the previous tile's column vector is no longer read
        if (t < 128) sr_s[t] = sr_rank[(size_t)slot_ct[slot] * 128 + t];
        __syncthreads();
        const uint2 w = *reinterpret_cast<const uint2 *>(bits + ((size_t)slot * 128 + row) * 4 + half * 2);
        const float *sr = sr_s + half * 64;
        float tm = -INFINITY;
        for (unsigned b = w.x; b; b &= b - 1) {
            float e = sl + sr[__ffs(b) - 1];
            e = e > 0.f ? e : slope * e;
            tm = e > tm ? e : tm;
        }
        for (unsigned b = w.y; b; b &= b - 1) {
            float e = sl + sr[32 + __ffs(b) - 1];
            e = e > 0.f ? e : slope * e;
            tm = e > tm ? e : tm;
        }
        if (tm == -INFINITY) continue;  // no entry of this row in this half of the tile
        const float mm = m > tm ? m : tm;
        z *= __expf(m - mm);            // m = -inf at the start: exp(-inf) = 0 and z = 0
        m = mm;
        for (unsigned b = w.x; b; b &= b - 1) {
            float e = sl + sr[__ffs(b) - 1];
            e = e > 0.f ? e : slope * e;
            z += __expf(e - m);
        }
        for (unsigned b = w.y; b; b &= b - 1) {
            float e = sl + sr[32 + __ffs(b) - 1];
            e = e > 0.f ? e : slope * e;
            z += __expf(e - m);
        }
    }
    // the two halves of the row sit in neighbouring lanes
    const float m2 = __shfl_xor(m, 1, 64), z2 = __shfl_xor(z, 1, 64);
    const float mm = m > m2 ? m : m2;
    if (half == 0) {
        float2 out = make_float2(-INFINITY, 0.f);
        if (mm != -INFINITY) out = make_float2(mm, z * __expf(m - mm) + z2 * __expf(m2 - mm));
        seg_stats[(size_t)seg * 128 + row] = out;
    }
}

// stats[i] (the pair over the remainder's entries of row i) merged with the pairs of the segments of the row's row of tiles, in
// segment order
__global__ void k_tile_stats_merge(float2 *__restrict__ stats, long long n_rows, const int32_t *__restrict__ rank_r, int n_ranks,
                                   const int32_t *__restrict__ rt_seg, const float2 *__restrict__ seg_stats) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int rank = rank_r[i];
    if (rank >= n_ranks) return;
    float2 a = stats[i];
    const int rt = rank >> 7, lr = rank & 127;
    for (int seg = rt_seg[rt]; seg < rt_seg[rt + 1]; ++seg) {
        const float2 b = seg_stats[(size_t)seg * 128 + lr];
        const float mm = a.x > b.x ? a.x : b.x;
        if (mm == -INFINITY) continue;
        a.y = a.y * expf(a.x - mm) + b.y * expf(b.x - mm);
        a.x = mm;
    }
    stats[i] = a;
}

// m_rank[q] = the largest logit among the tile entries of the row of rank q (-inf: none): the shift the attention tiles can use before
// the row maxima over all entries are known
__global__ void k_tile_row_max(const int32_t *__restrict__ rt_seg, const float2 *__restrict__ seg_stats, int n_ranks, float *__restrict__ m_rank) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_ranks) return;
    float m = -INFINITY;
    for (int seg = rt_seg[q >> 7]; seg < rt_seg[(q >> 7) + 1]; ++seg) { const float v = seg_stats[(size_t)seg * 128 + (q & 127)].x; m = v > m ? v : m; }
    m_rank[q] = m;
}

// the same for the tiles of the transposed pattern: its rows are the sources (s_r), its columns the destinations (s_l and their maxima)
__global__ void k_gather_ranked_vecs_t(const float *__restrict__ s_l, const float *__restrict__ s_r, const float2 *__restrict__ mz,
                                       const int32_t *__restrict__ order_r, int n_r, const int32_t *__restrict__ order_c, int n_c,
                                       float *__restrict__ sr_rank, float *__restrict__ sl_rank, float *__restrict__ m_rank) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < n_r) {
        const int j = order_r[q];
        sr_rank[q] = j >= 0 ? s_r[j] : 0.f;
    }
    if (q < n_c) {
        const int i = order_c[q];
        sl_rank[q] = i >= 0 ? s_l[i] : 0.f;
        m_rank[q] = i >= 0 ? mz[i].x : 0.f;
    }
}

// Bh[q, 0:f) = row order_c[q] of the slice-major matrix B (zeros where the rank has no node), times 1 / mz[node].y if mz is given
__global__ void k_gather_ranked_rows(const float *__restrict__ B, long long n_cols, int f, const int32_t *__restrict__ order_c, long long n_ranks,
                                     float *__restrict__ Bh, const float2 *__restrict__ mz) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int f4 = f / 4;
    if (t >= n_ranks * f4) return;
    const long long q = t / f4;
    const int col = (int)(t % f4) * 4;
    const int j = order_c[q];
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j >= 0) v = *reinterpret_cast<const float4 *>(B + (long long)(col >> 5) * n_cols * 32 + (long long)j * 32 + (col & 31));
    if (mz && j >= 0) {
        const float z = mz[j].y, iz = z > 0.f ? 1.f / z : 0.f;
        v.x *= iz; v.y *= iz; v.z *= iz; v.w *= iz;
    }
    *reinterpret_cast<float4 *>(Bh + q * f + col) = v;
}

// ---- C[M x N] = A^T . B with A stored [K x M] and B stored [K x N] (both row-major), K very long: the weight
// gradient dW = X^T . G of a layer, reduced over all nodes.  The K range is cut into `splits` slabs, one
// workgroup per (output tile, slab); slab s writes its partial tile to part[s] and k_sum_splits adds the slabs
// in order, so the result does not depend on scheduling.  Both operands arrive k-major, which is the layout the
// MFMA operand reads want, so both use the loader the forward kernel uses for W.  A sum over 10^5..10^7 nodes
// in one fp32 accumulator would lose the small entries of dW (rounding grows with the running sum, about
// 6e-4 of a term's spread at K = 233,000): the fp32 MFMA accumulators are therefore emptied into fp64 registers
// after every kFlushTiles k-tiles, the slabs are stored and added in fp64, and only the final sum is rounded to fp32.
struct GemmTnArgs {
    const float *A, *B;
    double *part;     // splits x M x N
    long long lda, ldb, k;
    int m, n, n_bn, n_tiles, k_per_split;
};

constexpr int kFlushTiles = 1;  // k-tiles (of KT = 16) summed in fp32 before the accumulators move to fp64

template <int VA, int VB>
__global__ __launch_bounds__(kThreads) void k_gemm_tn(GemmTnArgs g) {
    constexpr int BM = 128, BN = 128, TM = 2, TN = 2, PAD = 4;
    __shared__ __attribute__((aligned(16))) float As[KT][BM + PAD];
    __shared__ __attribute__((aligned(16))) float Bs[KT][BN + PAD];
    const int t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int tile = (int)(blockIdx.x % g.n_tiles), split = (int)(blockIdx.x / g.n_tiles);
    const int m0 = (tile / g.n_bn) * BM, n0 = (tile % g.n_bn) * BN;
    const long long k_lo = (long long)split * g.k_per_split;
    const long long k_hi = (k_lo + g.k_per_split < g.k) ? k_lo + g.k_per_split : g.k;

    floatx16 acc[TM][TN];
    double dacc[TM][TN][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; dacc[i][j][r] = 0.0; }
    auto flush = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) { dacc[i][j][r] += (double)acc[i][j][r]; acc[i][j][r] = 0.f; }
    };

    // loader: KT rows of 128 floats per operand; VEC floats per thread and pass
    constexpr int A_TPR = BM / VA, A_RPP = kThreads / A_TPR, A_PASSES = (KT + A_RPP - 1) / A_RPP;
    constexpr int B_TPR = BN / VB, B_RPP = kThreads / B_TPR, B_PASSES = (KT + B_RPP - 1) / B_RPP;
    float ra[A_PASSES][VA], rb[B_PASSES][VB];
    const int a_row = t / A_TPR, a_cc = (t % A_TPR) * VA;
    const int b_row = t / B_TPR, b_cc = (t % B_TPR) * VB;

    auto fetch = [&](long long k0) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int kr = p * A_RPP + a_row;
            const long long kk = k0 + kr;
            const int col = m0 + a_cc;
            if (kr < KT && kk < k_hi && col < g.m) {  // VA == 4 implies m % 4 == 0: a piece never straddles the edge
                const float *src = g.A + kk * g.lda + col;
                if (VA == 4) { float4 v = *reinterpret_cast<const float4 *>(src); ra[p][0] = v.x; ra[p][1 % VA] = v.y; ra[p][2 % VA] = v.z; ra[p][3 % VA] = v.w; }
                else ra[p][0] = *src;
            } else {
#pragma unroll
                for (int e = 0; e < VA; ++e) ra[p][e] = 0.f;
            }
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int kr = p * B_RPP + b_row;
            const long long kk = k0 + kr;
            const int col = n0 + b_cc;
            if (kr < KT && kk < k_hi && col < g.n) {
                const float *src = g.B + kk * g.ldb + col;
                if (VB == 4) { float4 v = *reinterpret_cast<const float4 *>(src); rb[p][0] = v.x; rb[p][1 % VB] = v.y; rb[p][2 % VB] = v.z; rb[p][3 % VB] = v.w; }
                else rb[p][0] = *src;
            } else {
#pragma unroll
                for (int e = 0; e < VB; ++e) rb[p][e] = 0.f;
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int kr = p * A_RPP + a_row;
            if (kr < KT) {
#pragma unroll
                for (int e = 0; e < VA; ++e) As[kr][a_cc + e] = ra[p][e];
            }
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int kr = p * B_RPP + b_row;
            if (kr < KT) {
#pragma unroll
                for (int e = 0; e < VB; ++e) Bs[kr][b_cc + e] = rb[p][e];
            }
        }
    };

    const int kh = lane >> 5, ll = lane & 31;
    if (k_lo < k_hi) fetch(k_lo);
    int since_flush = 0;
    for (long long k0 = k_lo; k0 < k_hi; k0 += KT) {
        stash();
        __syncthreads();
        if (k0 + KT < k_hi) fetch(k0 + KT);
#pragma unroll
        for (int kk = 0; kk < KT; kk += 2) {
            float av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[kk + kh][(wm * TM + i) * 32 + ll];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[j] = Bs[kk + kh][(wn * TN + j) * 32 + ll];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        if (++since_flush == kFlushTiles) { flush(); since_flush = 0; }
        __syncthreads();
    }
    flush();

    double *out = g.part + (size_t)split * (size_t)g.m * (size_t)g.n;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + ll;
            if (col >= g.n) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * kh + (r % 4);
                if (row < g.m) out[(size_t)row * g.n + col] = dacc[i][j][r];
            }
        }
}

// The same reduction on the bf16 matrix instruction at fp32 accuracy (three exact bf16 pieces per operand element, six piece
// products per term, as in k_gemm_bf).  Both operands arrive k-major, while a lane of the 32 x 32 x 16 instruction wants eight
// consecutive k of one column: a thread fetches exactly that (eight rows of its column, neighbouring lanes on neighbouring columns),
// cuts the eight values into pieces and leaves them in LDS in lane order, for both operands alike; two buffers, one barrier per step
// of 16 k, fetches one step ahead.  The fp32 accumulators are emptied into fp64 registers after every second step.
constexpr int kFlushStepsBf = 2;

__global__ __launch_bounds__(kThreads) void k_gemm_tn_bf(GemmTnArgs g) {
    constexpr int BM = 128, BN = 128, TM = 2, TN = 2;
    __shared__ __attribute__((aligned(16))) unsigned short Ps[2][2][3][4][2][32][8];   // [buffer][operand][piece][32-column block][k half][column][8 k]
    const int t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int kh = lane >> 5, ll = lane & 31;
    const int tile = (int)(blockIdx.x % g.n_tiles), split = (int)(blockIdx.x / g.n_tiles);
    const int m0 = (tile / g.n_bn) * BM, n0 = (tile % g.n_bn) * BN;
    const long long k_lo = (long long)split * g.k_per_split;
    const long long k_hi = (k_lo + g.k_per_split < g.k) ? k_lo + g.k_per_split : g.k;

    floatx16 acc[TM][TN];
    double dacc[TM][TN][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; dacc[i][j][r] = 0.0; }
    // Every other group of steps multiplies -A and is subtracted: the instruction's sum of 16 products and the accumulator loses
    // low bits of the smaller addends downwards whatever their sign (measured: about -2^-29 of the sum of the terms' magnitudes),
    // which over 10^5 rows would add up to several units of fp32 rounding of the root-sum-square; in alternating groups it cancels.
    int neg = split & 1;   // slabs with an odd number of groups leave one over: neighbouring slabs start with opposite signs
    auto flush = [&]() {
        const double sg = neg ? -1.0 : 1.0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) { dacc[i][j][r] = fma(sg, (double)acc[i][j][r], dacc[i][j][r]); acc[i][j][r] = 0.f; }
    };

    // staging: thread -> (column of the 128, k half); columns past the edge read the last column and are cleared, rows past the slab
    // read its last row and are cleared (masks, not branches around the fetches)
    const int col = t & 127, skh = t >> 7;
    const bool a_ok = m0 + col < g.m, b_ok = n0 + col < g.n;
    const unsigned a_mask = a_ok ? ~0u : 0u, b_mask = b_ok ? ~0u : 0u;
    // addresses: a uniform row pointer per k plus one 32-bit byte offset per lane (its k half and column), fixed before the loop
    const unsigned a_off = (unsigned)(((long long)skh * 8 * g.lda + (a_ok ? m0 + col : g.m - 1)) * 4);
    const unsigned b_off = (unsigned)(((long long)skh * 8 * g.ldb + (b_ok ? n0 + col : g.n - 1)) * 4);
    float ra[8], rb[8];
    auto fetch = [&](long long k0, auto whole) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if constexpr (decltype(whole)::value) {   // all 16 rows of the step lie inside the slab
                const char *ar = reinterpret_cast<const char *>(g.A + (k0 + e) * g.lda), *br = reinterpret_cast<const char *>(g.B + (k0 + e) * g.ldb);
                ra[e] = __uint_as_float(__float_as_uint(*reinterpret_cast<const float *>(ar + a_off)) & a_mask);
                rb[e] = __uint_as_float(__float_as_uint(*reinterpret_cast<const float *>(br + b_off)) & b_mask);
            } else {
                const long long k = k0 + skh * 8 + e;
                const long long kc = (k < k_hi ? k : k_hi - 1) - skh * 8;
                const unsigned live = k < k_hi ? ~0u : 0u;
                const char *ar = reinterpret_cast<const char *>(g.A + kc * g.lda), *br = reinterpret_cast<const char *>(g.B + kc * g.ldb);
                ra[e] = __uint_as_float(__float_as_uint(*reinterpret_cast<const float *>(ar + a_off)) & a_mask & live);
                rb[e] = __uint_as_float(__float_as_uint(*reinterpret_cast<const float *>(br + b_off)) & b_mask);
            }
        }
    };
    auto stash_one = [&](const float (&src)[8], int buf, int operand) {
        unsigned pc[8][3];
#pragma unroll
        for (int e = 0; e < 8; ++e) split_bf16x3(src[e], pc[e][0], pc[e][1], pc[e][2]);
        const unsigned flip = (operand == 0 && neg) ? 0x80008000u : 0u;   // the sign bits of a pair of bf16
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            uintx4 w;
#pragma unroll
            for (int d = 0; d < 4; ++d) w[d] = pack_bf16(pc[2 * d][p], pc[2 * d + 1][p]) ^ flip;
            *reinterpret_cast<uintx4 *>(&Ps[buf][operand][p][col >> 5][skh][col & 31][0]) = w;
        }
    };
    auto stash = [&](int buf) {
        stash_one(ra, buf, 0);
        __builtin_amdgcn_sched_barrier(0);   // one operand's pieces at a time in registers
        stash_one(rb, buf, 1);
    };

    if (k_lo < k_hi) {
        int buf = 0, since_flush = 0;
        auto step = [&](long long k0, auto next_whole) {
            fetch(k0 + 16 < k_hi ? k0 + 16 : k0, next_whole);   // past the last step: this step again, not used
            __builtin_amdgcn_sched_barrier(0);      // the fetches stay here and their use stays below the multiply
            __syncthreads();                        // this step's pieces are in Ps[buf]; nobody reads the other buffer any more
            // few fragments live at a time (the fp64 accumulators take half the registers): the pieces of B are read again for each
            // piece of A they meet
#pragma unroll
            for (int pa = 2; pa >= 0; --pa) {
                uintx4 af[TM];
#pragma unroll
                for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const uintx4 *>(&Ps[buf][0][pa][wm * TM + i][kh][ll][0]);
#pragma unroll
                for (int pb = 2 - pa; pb >= 0; --pb)   // smallest products first
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const uintx4 bf = *reinterpret_cast<const uintx4 *>(&Ps[buf][1][pb][wn * TN + j][kh][ll][0]);
#pragma unroll
                        for (int i = 0; i < TM; ++i)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf), acc[i][j], 0, 0, 0);
                    }
            }
            if (++since_flush == kFlushStepsBf) { flush(); since_flush = 0; neg ^= 1; }   // the pieces stashed below belong to the next group
            __builtin_amdgcn_sched_barrier(0);
            stash(buf ^ 1);
            buf ^= 1;
        };
        if (k_lo + 16 <= k_hi) fetch(k_lo, std::true_type()); else fetch(k_lo, std::false_type());
        stash(0);
        long long k0 = k_lo;
        for (; k0 + 32 <= k_hi; k0 += 16) step(k0, std::true_type());   // the next step is whole
        for (; k0 < k_hi; k0 += 16) step(k0, std::false_type());
    }
    flush();

    double *out = g.part + (size_t)split * (size_t)g.m * (size_t)g.n;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int c = n0 + (wn * TN + j) * 32 + ll;
            if (c >= g.n) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * kh + (r % 4);
                if (row < g.m) out[(size_t)row * g.n + c] = dacc[i][j][r];
            }
        }
}

// C[i] = sum over the slabs, in slab order
__global__ void k_sum_splits(const double *__restrict__ part, int splits, long long mn, int n, float *__restrict__ C, long long ldc) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= mn) return;
    double s = 0.0;
    for (int p = 0; p < splits; ++p) s += part[(size_t)p * (size_t)mn + e];
    C[(e / n) * ldc + (e % n)] = (float)s;
}

// Wt[c][r] = W[r][c] for a small matrix (the layer weights)
__global__ void k_transpose(const float *__restrict__ W, long long ldw, int rows, int cols, float *__restrict__ Wt, long long ldt) {
    __shared__ float tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int y = ty; y < 32; y += 8)
        if (r0 + y < rows && c0 + tx < cols) tile[y][tx] = W[(long long)(r0 + y) * ldw + c0 + tx];
    __syncthreads();
    for (int y = ty; y < 32; y += 8)
        if (c0 + y < cols && r0 + tx < rows) Wt[(long long)(c0 + y) * ldt + r0 + tx] = tile[tx][y];
}

// y1 = A.v1, y2 = A.v2; one wavefront per row, lanes stride over k.
template <int VEC>
__global__ __launch_bounds__(kThreads) void k_gemv2(const float *__restrict__ A, long long lda, long long n, int k,
                                                     const float *__restrict__ v1, const float *__restrict__ v2,
                                                     float *__restrict__ y1, float *__restrict__ y2, int a_sliced) {
    const long long row = (long long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (row >= n) return;
    const int lane = threadIdx.x & 63;
    const float *a0 = a_sliced ? A + row * 32 : A + row * lda;
    float d1 = 0.f, d2 = 0.f;
    for (int kk = lane * VEC; kk < k; kk += 64 * VEC) {
        // slice-major: columns kk.. of this row sit in tile kk / 32 (a 4-float piece never straddles tiles)
        const float *a = a_sliced ? a0 + (long long)(kk >> 5) * n * 32 + (kk & 31) - kk : a0;
        float x[VEC];
        if (VEC == 4) { float4 v = *reinterpret_cast<const float4 *>(a + kk); x[0] = v.x; x[1 % VEC] = v.y; x[2 % VEC] = v.z; x[3 % VEC] = v.w; }
        else if (VEC == 2) { float2 v = *reinterpret_cast<const float2 *>(a + kk); x[0] = v.x; x[1 % VEC] = v.y; }
        else x[0] = a[kk];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            d1 = fmaf(x[e], v1[kk + e], d1);
            d2 = fmaf(x[e], v2[kk + e], d2);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        d1 += __shfl_xor(d1, off, 64);
        d2 += __shfl_xor(d2, off, 64);
    }
    if (lane == 0) { y1[row] = d1; y2[row] = d2; }
}

}  // namespace

// from one 256-row block per compute unit on, and at least one whole step of 16 k
bool gemm_uses_pieces(int64_t n, int k, int m_store) {
    const int tn = m_store <= 32 ? 1 : m_store <= 64 ? 2 : 4;
    const int n_bn = (m_store + 32 * tn - 1) / (32 * tn);
    return k >= 16 && m_store > 0 && ((n + 255) / 256) * n_bn >= 256;
}

hipError_t launch_gemm(const float *A, int64_t lda, const float *W, int64_t ldw, float *Y, int64_t ldy, int64_t n,
                       int k, int m, int m_store, int act, hipStream_t s, const float *row_scale, KernelTimer *timer, bool y_sliced,
                       bool a_sliced, const float *add_sliced) {
    if (n <= 0 || m_store <= 0) return hipSuccess;
    if (a_sliced) lda = 32;
    hipEvent_t t0 = timer ? timer->next() : nullptr, t1 = t0 ? timer->next() : nullptr;
    if (t1 && hipEventRecord(t0, s) != hipSuccess) return hipErrorUnknown;
    auto done = [&](hipError_t e) {
        if (e == hipSuccess && t1 && hipEventRecord(t1, s) != hipSuccess) return hipErrorUnknown;
        return e;
    };
    GemmArgs g;
    g.row_scale = row_scale;
    g.A = A; g.W = W; g.Y = Y; g.lda = lda; g.ldw = ldw; g.ldy = ldy; g.n = n;
    g.k = k; g.m = m; g.m_store = m_store; g.act = act; g.y_sliced = y_sliced ? 1 : 0;
    g.a_slice = a_sliced ? n * 32 : 32; g.add = add_sliced;
    int avec = 1, bvec = 1;
    const uintptr_t aa = reinterpret_cast<uintptr_t>(A), wa = reinterpret_cast<uintptr_t>(W);
    if (k % 4 == 0 && lda % 4 == 0 && aa % 16 == 0) avec = 4;
    else if (k % 2 == 0 && lda % 2 == 0 && aa % 8 == 0) avec = 2;
    if (m % 4 == 0 && ldw % 4 == 0 && wa % 16 == 0) bvec = 4;
    // Large products go to the bf16-piece kernel (256-row blocks)
    {
        const int tn = m_store <= 32 ? 1 : m_store <= 64 ? 2 : 4;
        const int n_bn = (m_store + 32 * tn - 1) / (32 * tn);
        if (gemm_uses_pieces(n, k, m_store) && lda < (1 << 21) && ldw < (1 << 21)) {   // leading dimensions: 32-bit byte offsets within a block
            g.n_bn = n_bn;
            int av = 1;
            if (lda % 4 == 0 && aa % 16 == 0) av = 4;
            else if (lda % 2 == 0 && aa % 8 == 0) av = 2;
            if (tn == 1) return done(gemm_bf_launch<1>(g, av, s));
            if (tn == 2) return done(gemm_bf_launch<2>(g, av, s));
            return done(gemm_bf_launch<4>(g, av, s));
        }
    }
    // tile choice: widest column tile that the output needs; small tiles when the big ones
    // would leave most of the 256 compute units without a workgroup
    const long long big_blocks = ((n + 127) / 128) * ((m_store + 127) / 128);
    if (m_store <= 32) {
        g.n_bn = 1;
        if ((n + 255) / 256 >= 256) return done(gemm_launch_vec<256, 32, 4, 1>(g, avec, bvec, s));
        g.n_bn = (m_store + 63) / 64;
        return done(gemm_launch_vec<64, 64, 2, 2>(g, avec, bvec, s));
    }
    if (m_store <= 64) {
        g.n_bn = 1;
        if ((n + 255) / 256 >= 256) return done(gemm_launch_vec<256, 64, 4, 1>(g, avec, bvec, s));
        return done(gemm_launch_vec<64, 64, 2, 2>(g, avec, bvec, s));
    }
    if (big_blocks >= 256) {
        g.n_bn = (m_store + 127) / 128;
        return done(gemm_launch_vec<128, 128, 2, 2>(g, avec, bvec, s));
    }
    g.n_bn = (m_store + 63) / 64;
    return done(gemm_launch_vec<64, 64, 2, 2>(g, avec, bvec, s));
}

hipError_t launch_tiles_gather(const TileSplit &T, const float *B_sliced, int64_t n_cols, int f, float *Bh, hipStream_t s) {
    if (T.n_slots <= 0 || f <= 0) return hipSuccess;
    const long long n_ranks = (long long)T.nt_c * 128;
    hipLaunchKernelGGL(k_gather_ranked_split, dim3((unsigned)((n_ranks / 8 * f + 255) / 256)), dim3(256), 0, s, B_sliced, (long long)n_cols, f,
                       T.order_c, n_ranks, reinterpret_cast<unsigned short *>(Bh), (const float2 *)nullptr);
    return hipGetLastError();
}

template <int MODE>
static void launch_attn_tiles(const DenseTilesAttnArgs &a, int n_seg, int nb_count, hipStream_t s) {
    DenseTilesAttnArgs g = a;
    const int nw = nb_count >= 5 ? 8 : nb_count >= 3 ? 4 : nb_count;   // wavefronts (32-column blocks) per workgroup
    g.n_bn = (nb_count + nw - 1) / nw;
    const dim3 grid((unsigned)(n_seg * g.n_bn));
    if (nw == 8) hipLaunchKernelGGL((k_dense_tiles_attn_bf<MODE, 8>), grid, dim3(512), 0, s, g);
    else if (nw == 4) hipLaunchKernelGGL((k_dense_tiles_attn_bf<MODE, 4>), grid, dim3(256), 0, s, g);
    else if (nw == 2) hipLaunchKernelGGL((k_dense_tiles_attn_bf<MODE, 2>), grid, dim3(128), 0, s, g);
    else hipLaunchKernelGGL((k_dense_tiles_attn_bf<MODE, 1>), grid, dim3(64), 0, s, g);
}

// f: a multiple of 32.  Bh: room for 6 bytes per (rank, column).
// local_shift (attention on the pattern itself): launch_tile_stats has run on this stream - the vectors are in rank order and the shift of a
// row is the maximum over its tile entries, so the call needs no row statistics; the join rescales (tile_shift of the combine launchers)
hipError_t launch_dense_tiles(const TileSplit &T, const float *B_sliced, int64_t n_cols, int f, float *Bh, hipStream_t s, const float *s_l,
                              const float *s_r, const float2 *mz, float slope, bool transposed, bool gathered, bool local_shift) {
    if (T.n_slots <= 0 || f <= 0) return hipSuccess;
    const long long n_ranks = (long long)T.nt_c * 128;
    unsigned short *Bq = reinterpret_cast<unsigned short *>(Bh);
    const int nb_count = f / 32;
    if (!gathered)   // pieces of the operand in lane order (the transposed attention mode folds 1 / z of the softmax row into them)
        hipLaunchKernelGGL(k_gather_ranked_split, dim3((unsigned)((n_ranks / 8 * f + 255) / 256)), dim3(256), 0, s, B_sliced, (long long)n_cols, f,
                           T.order_c, n_ranks, Bq, (s_l && transposed) ? mz : (const float2 *)nullptr);
    if (!s_l) {
        DenseTilesBfArgs b;
        b.bits = T.bits; b.seg_first = T.seg_first; b.slot_ct = T.slot_ct; b.Bq = Bq; b.part = T.part;
        b.plane = n_ranks * f; b.f = f;
        const int waves = nb_count < 4 ? nb_count : 4;
        b.n_bn = (nb_count + 3) / 4;
        hipLaunchKernelGGL(k_dense_tiles_bf, dim3((unsigned)(T.n_seg * b.n_bn)), dim3(64 * waves), 0, s, b);
    } else {
        DenseTilesAttnArgs g;
        g.bits = T.bits; g.seg_first = T.seg_first; g.slot_ct = T.slot_ct; g.seg_rt = T.seg_rt; g.Bq = Bq; g.part = T.part;
        g.plane = n_ranks * f; g.f = f; g.n_bn = 1; g.slope = slope;
        const int n_r = T.nt_r * 128, n_c = T.nt_c * 128;
        const dim3 vgrid((unsigned)(((n_r > n_c ? n_r : n_c) + 255) / 256));
        if (transposed) {
            g.u_rank = T.rank_vec; g.m_rank = nullptr; g.v_rank = T.rank_vec + n_r; g.mc_rank = T.rank_vec + n_r + n_c;
            hipLaunchKernelGGL(k_gather_ranked_vecs_t, vgrid, dim3(256), 0, s, s_l, s_r, mz, T.order_r, n_r, T.order_c, n_c, T.rank_vec,
                               T.rank_vec + n_r, T.rank_vec + n_r + n_c);
            launch_attn_tiles<kTilesAttnT>(g, T.n_seg, nb_count, s);
        } else {
            g.u_rank = T.rank_vec; g.m_rank = T.rank_vec + n_r; g.v_rank = T.rank_vec + 2 * n_r; g.mc_rank = nullptr;
            if (!local_shift)
                hipLaunchKernelGGL(k_gather_ranked_vecs, vgrid, dim3(256), 0, s, s_l, s_r, mz, T.order_r, n_r, T.order_c, n_c, T.rank_vec,
                                   T.rank_vec + n_r, T.rank_vec + 2 * n_r);
            launch_attn_tiles<kTilesAttn>(g, T.n_seg, nb_count, s);
        }
    }
    const long long threads = (long long)T.nt_r * 128 * (f / 4);
    hipLaunchKernelGGL(k_tiles_reduce, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, (const float *)T.part, T.rt_seg, T.nt_r, f, T.dh);
    return hipGetLastError();
}

hipError_t launch_tile_stats(const TileSplit &T, const float *s_l, const float *s_r, float slope, hipStream_t s) {
    if (T.n_slots <= 0 || T.n_seg <= 0) return hipSuccess;
    const int n_r = T.nt_r * 128, n_c = T.nt_c * 128;
    hipLaunchKernelGGL(k_gather_ranked_vecs, dim3((unsigned)(((n_r > n_c ? n_r : n_c) + 255) / 256)), dim3(256), 0, s, s_l, s_r, (const float2 *)nullptr,
                       T.order_r, n_r, T.order_c, n_c, T.rank_vec, T.rank_vec + n_r, T.rank_vec + 2 * n_r);
    hipLaunchKernelGGL(k_tile_stats, dim3((unsigned)T.n_seg), dim3(256), 0, s, T.bits, T.seg_first, T.slot_ct, T.seg_rt, (const float *)T.rank_vec,
                       (const float *)(T.rank_vec + 2 * n_r), slope, T.seg_stats);
    hipLaunchKernelGGL(k_tile_row_max, dim3((unsigned)((n_r + 255) / 256)), dim3(256), 0, s, T.rt_seg, (const float2 *)T.seg_stats, n_r, T.rank_vec + n_r);
    return hipGetLastError();
}

hipError_t launch_tile_stats_merge(const TileSplit &T, float2 *stats, int64_t n_rows, hipStream_t s) {
    if (T.n_slots <= 0 || T.n_seg <= 0 || n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_tile_stats_merge, dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, s, stats, (long long)n_rows, T.rank_r, T.nt_r * 128,
                       T.rt_seg, (const float2 *)T.seg_stats);
    return hipGetLastError();
}

hipError_t launch_tiles_sddmm(const TileSplit &T, const float *L_sliced, int64_t n_rows, const float *R_sliced, int64_t n_cols, int f, float *Lh,
                              float *Rh, float *Dt, hipStream_t s) {
    if (T.n_slots <= 0 || f <= 0) return hipSuccess;
    const long long nr = (long long)T.nt_r * 128, nc = (long long)T.nt_c * 128;
    hipLaunchKernelGGL(k_gather_ranked_rows, dim3((unsigned)((nr * (f / 4) + 255) / 256)), dim3(256), 0, s, L_sliced, (long long)n_rows, f, T.order_r, nr, Lh, (const float2 *)nullptr);
    hipLaunchKernelGGL(k_gather_ranked_rows, dim3((unsigned)((nc * (f / 4) + 255) / 256)), dim3(256), 0, s, R_sliced, (long long)n_cols, f, T.order_c, nc, Rh, (const float2 *)nullptr);
    hipLaunchKernelGGL(k_tiles_sddmm, dim3((unsigned)T.n_slots), dim3(kThreads), 0, s, (const float *)Lh, (const float *)Rh, f, T.slot_rt, T.slot_ct, Dt);
    return hipGetLastError();
}

hipError_t launch_tiles_combine(const TileSplit &T, float *C, int64_t n_rows, int f_store, int64_t ldc, bool c_sliced, int f, const float *r,
                                const float2 *mz, int act, hipStream_t s, const int32_t *row_ptr_rem, int chunk_nnz, const float *carry, int f_carry,
                                const float *tile_shift) {
    if (n_rows <= 0 || f_store <= 0) return hipSuccess;
    const long long threads = (long long)n_rows * ((f_store + 3) / 4);
    // T.dh rows are f floats, f a multiple of 32; carry slots are f_carry floats apart
    const int vec4 = (reinterpret_cast<uintptr_t>(C) % 16 == 0 && (c_sliced || ldc % 4 == 0) &&
                      (!carry || (f_carry % 4 == 0 && reinterpret_cast<uintptr_t>(carry) % 16 == 0))) ? 1 : 0;
    if (!carry || chunk_nnz <= 0) row_ptr_rem = nullptr;
    hipLaunchKernelGGL(k_tiles_combine, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, C, (long long)n_rows, f_store,
                       c_sliced ? 32LL : (long long)ldc, c_sliced ? (long long)n_rows * 32 : 32LL, (const float *)T.dh, f, T.rank_r, T.nt_r * 128, r, mz,
                       act, vec4, row_ptr_rem, chunk_nnz, carry, f_carry, mz ? tile_shift : nullptr);
    return hipGetLastError();
}

hipError_t launch_tiles_combine_pm(const TileSplit &T, float *C, int64_t n_rows, int f_store, int64_t ldc, bool c_sliced, int f, const float *r,
                                   const float2 *mz, int act, hipStream_t s, const float *part, int n_panels, const int32_t *seg_ptr, int chunk_nnz,
                                   const float *carry, int f_carry, const float *tile_shift) {
    if (n_rows <= 0 || f_store <= 0) return hipSuccess;
    if (f % 32 != 0 || f_carry % 4 != 0 || reinterpret_cast<uintptr_t>(part) % 16 != 0 || reinterpret_cast<uintptr_t>(carry) % 16 != 0 || chunk_nnz <= 0)
        return hipErrorInvalidValue;
    const long long threads = (long long)n_rows * ((f_store + 3) / 4);
    const int vec4 = (reinterpret_cast<uintptr_t>(C) % 16 == 0 && (c_sliced || ldc % 4 == 0)) ? 1 : 0;
    hipLaunchKernelGGL(k_tiles_combine_pm, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, C, (long long)n_rows, f_store,
                       c_sliced ? 32LL : (long long)ldc, c_sliced ? (long long)n_rows * 32 : 32LL, (const float *)T.dh, f, T.rank_r, T.nt_r * 128, r, mz,
                       act, vec4, part, n_panels, seg_ptr, chunk_nnz, carry, f_carry, mz ? tile_shift : nullptr);
    return hipGetLastError();
}

hipError_t launch_gemv2(const float *A, int64_t lda, int64_t n, int k, const float *v1, const float *v2, float *y1,
                        float *y2, hipStream_t s, bool a_sliced) {
    if (n <= 0) return hipSuccess;
    dim3 grid((unsigned)((n + kThreads / 64 - 1) / (kThreads / 64)));
    const uintptr_t aa = reinterpret_cast<uintptr_t>(A);
    if (a_sliced) lda = 32;
    const int sl = a_sliced ? 1 : 0;
    if (k % 4 == 0 && lda % 4 == 0 && aa % 16 == 0)
        hipLaunchKernelGGL((k_gemv2<4>), grid, dim3(kThreads), 0, s, A, (long long)lda, (long long)n, k, v1, v2, y1, y2, sl);
    else if (k % 2 == 0 && lda % 2 == 0 && aa % 8 == 0)
        hipLaunchKernelGGL((k_gemv2<2>), grid, dim3(kThreads), 0, s, A, (long long)lda, (long long)n, k, v1, v2, y1, y2, sl);
    else
        hipLaunchKernelGGL((k_gemv2<1>), grid, dim3(kThreads), 0, s, A, (long long)lda, (long long)n, k, v1, v2, y1, y2, sl);
    return hipGetLastError();
}

int gemm_tn_splits(int64_t k, int m, int n) {
    const long long tiles = (long long)((m + 127) / 128) * ((n + 127) / 128);
    long long s = (768 + tiles - 1) / tiles;              // about three workgroups per compute unit
    const long long max_s = (k + 4 * KT - 1) / (4 * KT);  // at least four k-tiles per slab
    if (s > max_s) s = max_s;
    return (int)(s < 1 ? 1 : s);
}

size_t gemm_tn_bytes(int64_t k, int m, int n) { return align_up((size_t)gemm_tn_splits(k, m, n) * (size_t)m * (size_t)n * sizeof(double), 256); }

hipError_t launch_gemm_tn(const float *A, int64_t lda, const float *B, int64_t ldb, int64_t k, int m, int n, float *C, int64_t ldc,
                          double *part, hipStream_t s) {
    if (m <= 0 || n <= 0) return hipSuccess;
    GemmTnArgs g;
    g.A = A; g.B = B; g.part = part; g.lda = lda; g.ldb = ldb; g.k = k > 0 ? k : 0; g.m = m; g.n = n;
    g.n_bn = (n + 127) / 128;
    g.n_tiles = ((m + 127) / 128) * g.n_bn;
    const int splits = gemm_tn_splits(k, m, n);
    g.k_per_split = (int)(((g.k + splits - 1) / splits + KT - 1) / KT * KT);
    if (g.k_per_split < KT) g.k_per_split = KT;
    const bool va = (m % 4 == 0 && lda % 4 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0);
    const bool vb = (n % 4 == 0 && ldb % 4 == 0 && reinterpret_cast<uintptr_t>(B) % 16 == 0);
    dim3 grid((unsigned)(g.n_tiles * splits));
    // long reductions (the weight gradients of a layer) take the bf16-piece kernel
    if (g.k >= 4096 && g.k_per_split >= 64) hipLaunchKernelGGL(k_gemm_tn_bf, grid, dim3(kThreads), 0, s, g);
    else if (va && vb) hipLaunchKernelGGL((k_gemm_tn<4, 4>), grid, dim3(kThreads), 0, s, g);
    else if (va) hipLaunchKernelGGL((k_gemm_tn<4, 1>), grid, dim3(kThreads), 0, s, g);
    else if (vb) hipLaunchKernelGGL((k_gemm_tn<1, 4>), grid, dim3(kThreads), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_tn<1, 1>), grid, dim3(kThreads), 0, s, g);
    const long long mn = (long long)m * n;
    hipLaunchKernelGGL(k_sum_splits, dim3((unsigned)((mn + 255) / 256)), dim3(256), 0, s, part, splits, mn, n, C, (long long)ldc);
    return hipGetLastError();
}

hipError_t launch_transpose(const float *W, int64_t ldw, int rows, int cols, float *Wt, int64_t ldt, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_transpose, dim3((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32)), dim3(256), 0, s, W, (long long)ldw, rows, cols,
                       Wt, (long long)ldt);
    return hipGetLastError();
}

}  // namespace sensei
