// Dense kernels for gfx950: the fp32 update GEMM on the matrix cores
// (v_mfma_f32_32x32x2_f32) with the activation fused into the epilogue, and a
// two-vector GEMV for the attention projections.
#include "sensei_internal.h"

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
};

// Block tile BM x BN, 4 wavefronts laid out WGM x WGN, each computing TM x TN tiles of 32 x 32
// with the 32x32x2 fp32 MFMA.  LDS holds A as [k][row] and W as [k][col] so that the MFMA operand
// reads (lane l takes k = l / 32, row or col = l % 32) are consecutive words.  The next k-tile is
// fetched from HBM into registers while the current one is multiplied.
template <int BM, int BN, int WGM, int WGN, int AVEC, int BVEC>
__global__ __launch_bounds__(kThreads) void k_gemm(GemmArgs g) {
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
    constexpr int APAD = 2, BPAD = 4;
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
                const float *src = g.A + row * g.lda + kk;
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

hipError_t launch_gemm(const float *A, int64_t lda, const float *W, int64_t ldw, float *Y, int64_t ldy, int64_t n,
                       int k, int m, int m_store, int act, hipStream_t s, const float *row_scale, KernelTimer *timer, bool y_sliced) {
    if (n <= 0 || m_store <= 0) return hipSuccess;
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
    int avec = 1, bvec = 1;
    const uintptr_t aa = reinterpret_cast<uintptr_t>(A), wa = reinterpret_cast<uintptr_t>(W);
    if (k % 4 == 0 && lda % 4 == 0 && aa % 16 == 0) avec = 4;
    else if (k % 2 == 0 && lda % 2 == 0 && aa % 8 == 0) avec = 2;
    if (m % 4 == 0 && ldw % 4 == 0 && wa % 16 == 0) bvec = 4;
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

}  // namespace sensei
