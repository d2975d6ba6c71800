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
//
// No LDS staging: both operands are K-contiguous in memory, and the instruction does not care WHICH four k a
// step contracts as long as A and B agree.  So lane (i = l%16, g = l/16) fetches 16-byte pieces
// X[row i][k0 + 16h + 4g .. +3] straight into registers and step (h, j) of the chunk contracts the k's
// {k0 + 16h + 4g + j : g = 0..3}.  Every global load is a full float4, a row's 128 bytes of a 32-k chunk are
// consumed by one wavefront, and there are no barriers; the two wavefronts of a block that share rows (or
// columns) find them in the vector cache.
#pragma once
#include <cmath>

#include "common.hpp"

namespace lorann {

enum { EPI_PLAIN = 0, EPI_NEG = 1, EPI_L2 = 2 };

constexpr int GM_BN = 64, GM_KC = 32;

// Guarded fetch of four floats p[k .. k+3] of a row of length K (zero beyond the end); any alignment.
__device__ __forceinline__ float4 gemm_fetch_tail(const float* __restrict__ p, int k, int K) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k + 0 < K) v.x = p[k + 0];
    if (k + 1 < K) v.y = p[k + 1];
    if (k + 2 < K) v.z = p[k + 2];
    if (k + 3 < K) v.w = p[k + 3];
    return v;
}

// One wavefront's tile: rows [m0, m0 + 16 TI), columns [n0, n0 + 32).
// X [M][K], W [N][K] row-major, out [M][N].  nrm [N] (double) is used by EPI_L2 only: out = nrm[n] - 2 * acc.
// vec_ok: rows of X and W are 16-byte aligned (K % 4 == 0 and aligned bases); otherwise every chunk takes the
// guarded scalar path.
template <int EPI, int TI>
__device__ __forceinline__ void gemm_wave_tile(const float* __restrict__ X, const float* __restrict__ W,
                                               float* __restrict__ out, const double* __restrict__ nrm,
                                               int M, int N, int K, int vec_ok, __bf16* __restrict__ out_bf,
                                               const int m0, const int n0) {
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, g = lane >> 4;

    // rows / columns beyond the matrix are clamped (loaded, never stored)
    const float* xa[TI];
    const float* wb[2];
#pragma unroll
    for (int ti = 0; ti < TI; ++ti) xa[ti] = X + (size_t)min(m0 + ti * 16 + i, M - 1) * K;
#pragma unroll
    for (int tj = 0; tj < 2; ++tj) wb[tj] = W + (size_t)min(n0 + tj * 16 + i, N - 1) * K;

    f64x4 acc[TI][2];
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = (f64x4){0.0, 0.0, 0.0, 0.0};

    auto contract = [&](const float4 (&a)[TI][2], const float4 (&b)[2][2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                double av[TI], bv[2];
#pragma unroll
                for (int ti = 0; ti < TI; ++ti) av[ti] = (double)(j == 0 ? a[ti][h].x : j == 1 ? a[ti][h].y : j == 2 ? a[ti][h].z : a[ti][h].w);
#pragma unroll
                for (int tj = 0; tj < 2; ++tj) bv[tj] = (double)(j == 0 ? b[tj][h].x : j == 1 ? b[tj][h].y : j == 2 ? b[tj][h].z : b[tj][h].w);
#pragma unroll
                for (int ti = 0; ti < TI; ++ti)
#pragma unroll
                    for (int tj = 0; tj < 2; ++tj)
                        acc[ti][tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[ti], bv[tj], acc[ti][tj], 0, 0, 0);
            }
        }
    };

    const int k_full = vec_ok ? (K / GM_KC) * GM_KC : 0;     // chunks fetched with unconditional float4 loads
    if (k_full > 0) {
        // Three register stages: the chunk contracted now, and the next two already requested (one chunk of matrix-core
        // work is shorter than a trip to the L2 under load, so one chunk of lead leaves the matrix cores waiting).
        float4 a_st[3][TI][2], b_st[3][2][2];
        auto fetch = [&](int k0, float4 (&a)[TI][2], float4 (&b)[2][2]) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = k0 + 16 * h + 4 * g;
#pragma unroll
                for (int ti = 0; ti < TI; ++ti) a[ti][h] = *reinterpret_cast<const float4*>(xa[ti] + k);
#pragma unroll
                for (int tj = 0; tj < 2; ++tj) b[tj][h] = *reinterpret_cast<const float4*>(wb[tj] + k);
            }
        };
        const int k_last = k_full - GM_KC;
        fetch(0, a_st[0], b_st[0]);
        fetch(min(GM_KC, k_last), a_st[1], b_st[1]);
        for (int k0 = 0; k0 < k_full; k0 += 3 * GM_KC) {
#pragma unroll
            for (int st = 0; st < 3; ++st) {
                const int kc = k0 + st * GM_KC;
                if (kc < k_full) {                                   // uniform
                    // (clamped: the last requests are repeats that are never contracted)
                    fetch(min(kc + 2 * GM_KC, k_last), a_st[(st + 2) % 3], b_st[(st + 2) % 3]);
                    contract(a_st[st], b_st[st]);
                }
            }
        }
    }
    for (int k0 = k_full; k0 < K; k0 += GM_KC) {             // remainder (or everything when rows are unaligned)
        float4 a[TI][2], b[2][2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = k0 + 16 * h + 4 * g;
#pragma unroll
            for (int ti = 0; ti < TI; ++ti) a[ti][h] = gemm_fetch_tail(xa[ti], k, K);
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) b[tj][h] = gemm_fetch_tail(wb[tj], k, K);
        }
        contract(a, b);
    }

#pragma unroll
    for (int ti = 0; ti < TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj) {
            const int col = n0 + tj * 16 + i;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + ti * 16 + 4 * v + g;
                if (row < M && col < N) {
                    const double s = acc[ti][tj][v];
                    float o;
                    if (EPI == EPI_PLAIN) o = (float)s;
                    else if (EPI == EPI_NEG) o = (float)(-s);
                    else o = (float)(nrm[col] - 2.0 * s);
                    out[(size_t)row * N + col] = o;
                    if (EPI == EPI_PLAIN && out_bf) out_bf[(size_t)row * N + col] = (__bf16)o;     // bfloat16 copy of the same matrix
                }
            }
        }
}

// grid = (ceil(N/64), ceil(M/BM)), block = 256 (2 x 2 wavefronts, each (BM/2) x 32 of the BM x 64 block tile).
// BM = 64 or 32: the smaller tile is used when it fills the machine more evenly (see gemm_pick_bm).
template <int EPI, int BM>
__global__ __launch_bounds__(256) void k_gemm_nt_f64(const float* __restrict__ X, const float* __restrict__ W,
                                                      float* __restrict__ out, const double* __restrict__ nrm,
                                                      int M, int N, int K, int vec_ok, __bf16* __restrict__ out_bf = nullptr) {
    const int wv = threadIdx.x >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    gemm_wave_tile<EPI, BM / 32>(X, W, out, nrm, M, N, K, vec_ok, out_bf, blockIdx.y * BM + wm * (BM / 2), blockIdx.x * GM_BN + wn * 32);
}

// The same contraction with both tile heights in one launch: the first n64 blocks take 64-row tiles over rows
// [0, rows64), the others 32-row tiles over the rest.  rows64 is a whole number of rounds of the 256 CUs, so the
// efficient tall tiles load every CU equally and the remainder is spread thinly over the machine by the small ones
// (10 000 x 256: two tall blocks per CU and one small one on 228 CUs, instead of three tall ones on some CUs and two on
// the others).  grid = n64 + (blocks of the remainder), block = 256.
template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_nt_f64_two_heights(const float* __restrict__ X, const float* __restrict__ W,
                                                                  float* __restrict__ out, const double* __restrict__ nrm,
                                                                  int M, int N, int K, int vec_ok, __bf16* __restrict__ out_bf,
                                                                  int n64, int rows64) {
    const int wv = threadIdx.x >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int nbx = (N + GM_BN - 1) / GM_BN;
    const int b = (int)blockIdx.x;
    if (b < n64) {                                   // uniform over the block
        const int by = b / nbx, bx = b - by * nbx;
        gemm_wave_tile<EPI, 2>(X, W, out, nrm, M, N, K, vec_ok, out_bf, by * 64 + wm * 32, bx * GM_BN + wn * 32);
    } else {
        const int by = (b - n64) / nbx, bx = (b - n64) - by * nbx;
        gemm_wave_tile<EPI, 1>(X, W, out, nrm, M, N, K, vec_ok, out_bf, rows64 + by * 32 + wm * 16, bx * GM_BN + wn * 32);
    }
}

// Tile height: the workgroups of this kernel are bound by the matrix cores of their CU, so the time follows the
// largest number of workgroups any CU receives, times the work of one, over the rate the tile shape reaches (measured:
// the 64-row tile, with four accumulators per wavefront and half the operand traffic, keeps the fp64 matrix cores
// 72 % busy, the 32-row tile 50 %).  The smaller tile wins only where it fills the machine much more evenly.
inline int gemm_pick_bm(long M, long N) {
    const double t64 = (double)((M + 63) / 64) * (double)((N + 63) / 64) / 256.0;
    const double t32 = (double)((M + 31) / 32) * (double)((N + 63) / 64) / 256.0;
    const double time64 = std::ceil(t64) * 1.0 / 0.72, time32 = std::ceil(t32) * 0.5 / 0.50;
    return time32 < time64 ? 32 : 64;
}

// The projection of a small batch (M <= kSmallBatch): out[m][n] = sum_k X[m][k] * W[n][k], double accumulation, one
// rounding to float, optional bfloat16 copy.  A matrix-core tile is mostly padding at this size and its K loop a
// chain of dependent steps; here one wavefront owns one output column n for kSmallM queries, its lanes stride over k
// (W row and X rows are read coalesced) and the sums meet in a wavefront reduction.
// MT = queries per wavefront (1 or 16: a single query does not pay for sixteen).  Four k-steps are requested
// together, so that a wavefront waits for memory K / 256 times instead of K / 64 times; a lane still adds its
// products in ascending k.
// grid = (ceil(N / 4), ceil(M / MT)), block = 256.
constexpr int kSmallM = 16, kSmallBatch = 512;
template <int MT>
__global__ __launch_bounds__(256) void k_project_small(const float* __restrict__ X, const float* __restrict__ W, float* __restrict__ out,
                                                       int M, int N, int K, __bf16* __restrict__ out_bf) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;                              // wavefronts are independent
    const int m0 = blockIdx.y * MT;
    X += (size_t)m0 * K; out += (size_t)m0 * N; if (out_bf) out_bf += (size_t)m0 * N;
    M = min(M - m0, MT);
    double acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0.0;
    constexpr int KU = MT == 1 ? 4 : 1;      // sixteen queries already keep sixteen loads in flight per step
    for (int k0 = lane; k0 < K; k0 += 64 * KU) {
        float wv[KU], x[KU][MT];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const int k = k0 + 64 * u;
            const bool ok = k < K;
            wv[u] = ok ? W[(size_t)n * K + k] : 0.0f;      // beyond K: + 0 * 0, which leaves the sum as it is
#pragma unroll
            for (int m = 0; m < MT; ++m) x[u][m] = ok ? X[(size_t)min(m, M - 1) * K + k] : 0.0f;   // rows beyond M repeat the last one (never stored)
        }
#pragma unroll
        for (int u = 0; u < KU; ++u)
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m] += (double)x[u][m] * (double)wv[u];
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const double s = wave_sum_f64(acc[m]);
        if (lane == 0 && m < M) {
            const float o = (float)s;
            out[(size_t)m * N + n] = o;
            if (out_bf) out_bf[(size_t)m * N + n] = (__bf16)o;
        }
    }
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

// out[row] = sum_i (x[row][i] - xb[row][i])^2 in double: the squared norm of the error of a bfloat16 copy of x.
__global__ __launch_bounds__(256) void k_row_bf16_err(const float* __restrict__ x, const __bf16* __restrict__ xb, double* __restrict__ out,
                                                      int64_t rows, int d) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    double acc = 0.0;
    for (int i = lane; i < d; i += 64) {
        const double v = (double)x[(size_t)row * d + i] - (double)(float)xb[(size_t)row * d + i];
        acc += v * v;
    }
    acc = wave_sum_f64(acc);
    if (lane == 0) out[row] = acc;
}

// Pt[j][i] = P[i][j]  (P is [d][dp]).
__global__ void k_transpose(const float* __restrict__ P, float* __restrict__ Pt, int d, int dp) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)d * dp) return;
    const int i = (int)(t / dp), j = (int)(t % dp);
    Pt[(size_t)j * d + i] = P[t];
}

}  // namespace lorann
