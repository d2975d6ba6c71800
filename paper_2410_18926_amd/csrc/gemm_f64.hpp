// Dense contraction out[M][N] = epilogue( sum_k X[m][k] * W[n][k] ) with float inputs and float output,
// accumulated in double on the fp64 matrix cores (v_mfma_f64_16x16x4_f64).
//
// Used for the query projection q' = P^T q (Sec. 4.1) and for the centroid dissimilarities (Sec. 2.2 routing,
// Sec. 3.1 Euclidean reduction, evaluated in the d'-dimensional space per Sec. 4.1).  Products of two floats
// are exact in double, so the result is the correctly rounded value of the exact sum up to reordering noise of
// ~1e-16 relative: routing decisions and the 8-bit query codes derived from these numbers do not depend on the
// summation order in practice.
//
// Register layout of v_mfma_f64_16x16x4_f64 (measured on gfx950): A operand lane l holds A[l%16][l/16],
// B operand lane l holds B[l/16][l%16], result register v of lane l holds D[4v + l/16][l%16].
#pragma once
#include <cmath>

#include "common.hpp"

namespace lorann {

enum { EPI_PLAIN = 0, EPI_NEG = 1, EPI_L2 = 2 };

constexpr int GM_BN = 64, GM_KT = 32, GM_LD = GM_KT + 1;

// One operand tile (rows x 16 k) is fetched as one float4 per thread.
__device__ __forceinline__ float4 gemm_fetch(const float* __restrict__ base, int rows, int K, int row, int k, bool vec_ok) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < rows) {
        const float* p = base + (size_t)row * K + k;
        if (vec_ok && k + 4 <= K) {
            v = *reinterpret_cast<const float4*>(p);
        } else {
            if (k + 0 < K) v.x = p[0];
            if (k + 1 < K) v.y = p[1];
            if (k + 2 < K) v.z = p[2];
            if (k + 3 < K) v.w = p[3];
        }
    }
    return v;
}

// grid = (ceil(N/64), ceil(M/BM)), block = 256 (2 x 2 wavefronts, each BM/2 x 32 of the BM x 64 block tile).
// BM = 64 or 32: the smaller tile is used when it fills the machine more evenly (see gemm_pick_bm).
// X [M][K], W [N][K] row-major, out [M][N].  nrm [N] (double) is used by EPI_L2 only: out = nrm[n] - 2 * acc.
template <int EPI, int BM>
__global__ __launch_bounds__(256) void k_gemm_nt_f64(const float* __restrict__ X, const float* __restrict__ W,
                                                      float* __restrict__ out, const double* __restrict__ nrm,
                                                      int M, int N, int K) {
    constexpr int TI = BM / 32;          // 16-row MFMA tiles per wavefront along M
    __shared__ float Xs[BM * GM_LD];
    __shared__ float Ws[GM_BN * GM_LD];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * GM_BN;
    const int lrow = tid >> 2, lk = (tid & 3) * 4;
    const bool vec_ok = (K % 4) == 0;
    const bool x_loader = lrow < BM;

    f64x4 acc[TI][2];
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = (f64x4){0.0, 0.0, 0.0, 0.0};

    float4 rx = make_float4(0.f, 0.f, 0.f, 0.f), rx2 = rx;
    if (x_loader) { rx = gemm_fetch(X, M, K, m0 + lrow, lk, vec_ok); rx2 = gemm_fetch(X, M, K, m0 + lrow, lk + 16, vec_ok); }
    float4 rw = gemm_fetch(W, N, K, n0 + lrow, lk, vec_ok), rw2 = gemm_fetch(W, N, K, n0 + lrow, lk + 16, vec_ok);
    const int i = lane & 15, g = lane >> 4;

    for (int k0 = 0; k0 < K; k0 += GM_KT) {
        if (x_loader) {
            float* xs = Xs + lrow * GM_LD + lk;
            xs[0] = rx.x; xs[1] = rx.y; xs[2] = rx.z; xs[3] = rx.w;
            xs[16] = rx2.x; xs[17] = rx2.y; xs[18] = rx2.z; xs[19] = rx2.w;
        }
        float* ws = Ws + lrow * GM_LD + lk;
        ws[0] = rw.x; ws[1] = rw.y; ws[2] = rw.z; ws[3] = rw.w;
        ws[16] = rw2.x; ws[17] = rw2.y; ws[18] = rw2.z; ws[19] = rw2.w;
        __syncthreads();
        if (k0 + GM_KT < K) {
            if (x_loader) { rx = gemm_fetch(X, M, K, m0 + lrow, k0 + GM_KT + lk, vec_ok); rx2 = gemm_fetch(X, M, K, m0 + lrow, k0 + GM_KT + lk + 16, vec_ok); }
            rw = gemm_fetch(W, N, K, n0 + lrow, k0 + GM_KT + lk, vec_ok); rw2 = gemm_fetch(W, N, K, n0 + lrow, k0 + GM_KT + lk + 16, vec_ok);
        }
#pragma unroll
        for (int kk = 0; kk < GM_KT; kk += 4) {
            double a[TI];
#pragma unroll
            for (int ti = 0; ti < TI; ++ti) a[ti] = (double)Xs[(wm * (BM / 2) + ti * 16 + i) * GM_LD + kk + g];
            const double b0 = (double)Ws[(wn * 32 + i) * GM_LD + kk + g];
            const double b1 = (double)Ws[(wn * 32 + 16 + i) * GM_LD + kk + g];
#pragma unroll
            for (int ti = 0; ti < TI; ++ti) {
                acc[ti][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ti], b0, acc[ti][0], 0, 0, 0);
                acc[ti][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ti], b1, acc[ti][1], 0, 0, 0);
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int ti = 0; ti < TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj) {
            const int col = n0 + wn * 32 + tj * 16 + i;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + wm * (BM / 2) + ti * 16 + 4 * v + g;
                if (row < M && col < N) {
                    const double s = acc[ti][tj][v];
                    float o;
                    if (EPI == EPI_PLAIN) o = (float)s;
                    else if (EPI == EPI_NEG) o = (float)(-s);
                    else o = (float)(nrm[col] - 2.0 * s);
                    out[(size_t)row * N + col] = o;
                }
            }
        }
}

// Tile height that loads the 256 CUs more evenly: the workgroups of this kernel are bound by the matrix cores
// of their CU, so the time follows the largest number of workgroups any CU receives.
inline int gemm_pick_bm(long M, long N) {
    const double t64 = (double)((M + 63) / 64) * (double)((N + 63) / 64) / 256.0;
    const double t32 = (double)((M + 31) / 32) * (double)((N + 63) / 64) / 256.0;
    const double e64 = t64 / std::ceil(t64), e32 = t32 / std::ceil(t32);
    return e32 > e64 + 0.05 ? 32 : 64;
}

// out[row] = sum_i x[row][i]^2 accumulated in double; one wavefront per row.  OUT = float or double.
template <typename OUT>
__global__ __launch_bounds__(256) void k_row_sqnorm(const float* __restrict__ x, OUT* __restrict__ out, int64_t rows, int d) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* p = x + (size_t)row * d;
    double acc = 0.0;
    for (int i = lane; i < d; i += 64) { const double v = (double)p[i]; acc += v * v; }
    acc = wave_sum_f64(acc);
    if (lane == 0) out[row] = (OUT)acc;
}

// Pt[j][i] = P[i][j]  (P is [d][dp]).
__global__ void k_transpose(const float* __restrict__ P, float* __restrict__ Pt, int d, int dp) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)d * dp) return;
    const int i = (int)(t / dp), j = (int)(t % dp);
    Pt[(size_t)j * d + i] = P[t];
}

}  // namespace lorann
