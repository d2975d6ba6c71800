// Routing (Sec. 2.2; in the d'-dimensional space, Sec. 4.1) by screening: the w clusters of smallest
// dissimilarity are found WITHOUT evaluating all L dissimilarities in double.
//
//   1. k_centroid_bf16: all L dissimilarities approximately - operands rounded to bfloat16, products on the
//      bf16 matrix cores (v_mfma_f32_32x32x16_bf16), float accumulation.
//   2. k_select_clusters_screen: a rigorous bound eps on |approximate - exact| turns the approximate values into
//      a short list that provably contains the exact w best (everything not above the w-th smallest approximate
//      value + 2 eps); only the list is evaluated exactly - double accumulation, one rounding to float, as the
//      definition says - and ranked by (value, cluster id).
//
// The result is identical to ranking all L exact values; the double-precision work drops from L to about w
// dot products per query.  A list that does not fit (huge norms, long runs of near-equal values) makes the
// block evaluate every cluster exactly instead, so correctness never rests on the bound being tight.
//
// Error bound.  Write qb = q + dq and mub = mu + dmu for the operands rounded to bfloat16.  Then
//   <qb, mub> - <q, mu> = <dq, mu> + <qb, dmu>     (an identity),  so by Cauchy-Schwarz
//   |<qb, mub> - <q, mu>| <= |dq|_2 |mu|_2 + |qb|_2 |dmu|_2.
// |dq|_2 and |qb|_2 are computed from the query's ACTUAL rounding errors (the selection kernels redo the rounding
// of their query), |mu|_2 and |dmu|_2 enter through their maxima over the centroids, computed when the index is
// loaded.  For operands with no special structure this is about 0.003 |q||mu|; in the worst case of bfloat16 (8
// significant bits: 1 + 2^-8 becomes 1, a relative error of 2^-8 per operand) it grows to the 2^-7 |q||mu| it has
// to be.  The products of rounded operands are exact in float; the K float additions of the matrix core add at
// most K 2^-23 |qb|_2 |mub|_2 even if it truncates.  All norms are rounded up by a relative 1e-3, which covers
// their own float arithmetic; the final float operations of both sides are covered by a relative slack of 2^-20.
//
// Register layout of v_mfma_f32_32x32x16_bf16 (measured on gfx950): both operands give lane l eight consecutive
// k (k-half l/32) of row / column l%32; result register v of lane l holds D[8*(v/4) + 4*(l/32) + v%4][l%32].
#pragma once
#include "common.hpp"
#include "route.hpp"

namespace lorann {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float kScreenAcc = 1.1920929e-7f;      // 2^-23: float accumulation error per term of the matrix-core sum

// o[i] = bfloat16(x[i]), round to nearest even.
__global__ void k_to_bf16(const float* __restrict__ x, __bf16* __restrict__ o, int64_t n) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) o[t] = (__bf16)x[t];
}

// out[q][l] = - <Q[q], C[l]>  (L2 = false)   or   nrm[l] - 2 <Q[q], C[l]>  (L2 = true), approximately.
// Q [M][K], C [N][K] bfloat16 row-major (K % 16 == 0, 16-byte aligned rows), out [M][N] float, nrm [N] float.
// grid = (ceil(N/128), ceil(M/(64 TI))), block = 256: 2 x 2 wavefronts, each a (32 TI) x 64 tile as TI x 2 MFMA
// tiles (TI = 2 moves fewer operand bytes; TI = 1 gives twice the blocks when the problem is small).
// Operands go from memory straight into the registers of the lanes that feed them to the matrix core (rows
// beyond the matrices are clamped, never stored); the two wavefronts that share rows meet in the vector cache.
// NT: the matrix is far larger than the caches and read once by the selection: written with streaming stores.
template <bool L2, int TI, bool NT = false>
__global__ __launch_bounds__(256) void k_centroid_bf16(const __bf16* __restrict__ Q, const __bf16* __restrict__ C,
                                                        float* __restrict__ out, const float* __restrict__ nrm,
                                                        int M, int N, int K) {
    constexpr int SB = 1;                 // k-steps (of 16) requested ahead
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * (64 * TI) + (wv >> 1) * (32 * TI), n0 = blockIdx.x * 128 + (wv & 1) * 64;
    const __bf16* qa[TI];
    const __bf16* cb[2];
#pragma unroll
    for (int t = 0; t < TI; ++t) qa[t] = Q + (size_t)min(m0 + 32 * t + i, M - 1) * K + 8 * h;
#pragma unroll
    for (int t = 0; t < 2; ++t) cb[t] = C + (size_t)min(n0 + 32 * t + i, N - 1) * K + 8 * h;
    f32x16 acc[TI][2];
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int steps = K >> 4;
    auto fetch = [&](int s0, bf16x8 (&a)[SB][TI], bf16x8 (&b)[SB][2]) {
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const int k = 16 * min(s0 + u, steps - 1);        // clamped: a repeat beyond the end, not used
#pragma unroll
            for (int t = 0; t < TI; ++t) a[u][t] = *reinterpret_cast<const bf16x8*>(qa[t] + k);
#pragma unroll
            for (int t = 0; t < 2; ++t) b[u][t] = *reinterpret_cast<const bf16x8*>(cb[t] + k);
        }
    };
    bf16x8 a_cur[SB][TI], b_cur[SB][2], a_nxt[SB][TI], b_nxt[SB][2];
    fetch(0, a_cur, b_cur);
    for (int s0 = 0; s0 < steps; s0 += SB) {
        fetch(s0 + SB, a_nxt, b_nxt);
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (s0 + u < steps) {                             // uniform
#pragma unroll
                for (int ta = 0; ta < TI; ++ta)
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb)
                        acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur[u][ta], b_cur[u][tb], acc[ta][tb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < SB; ++u) {
#pragma unroll
            for (int t = 0; t < TI; ++t) a_cur[u][t] = a_nxt[u][t];
#pragma unroll
            for (int t = 0; t < 2; ++t) b_cur[u][t] = b_nxt[u][t];
        }
    }
#pragma unroll
    for (int ta = 0; ta < TI; ++ta)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int col = n0 + 32 * tb + i;
            const float nb = (L2 && col < N) ? nrm[col] : 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + 32 * ta + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < M && col < N) {
                    const float g = L2 ? nb - 2.0f * acc[ta][tb][v] : -acc[ta][tb][v];
                    if (NT) __builtin_nontemporal_store(g, &out[(size_t)row * N + col]);
                    else out[(size_t)row * N + col] = g;
                }
            }
        }
}

// Sum of a double over each row of 16 lanes (data-parallel-primitive shifts with zero fill); the total is valid
// in the LAST lane of the row only.
__device__ __forceinline__ double row16_sum_f64_last(double x) {
    auto shr = [](double v, auto ctrl) {
        const long long b = __double_as_longlong(v);
        const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), decltype(ctrl)::value, 0xf, 0xf, true);
        const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), decltype(ctrl)::value, 0xf, 0xf, true);
        return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
    };
    x += shr(x, std::integral_constant<int, 0x111>{});
    x += shr(x, std::integral_constant<int, 0x112>{});
    x += shr(x, std::integral_constant<int, 0x114>{});
    x += shr(x, std::integral_constant<int, 0x118>{});
    return x;
}

struct ScreenArgs {
    float* ghat;                 // [nq][L] approximate dissimilarities (a row is overwritten with exact values
                                 //         when its list does not fit)
    const float* qp;             // [nq][dp] projected queries (float)
    const float* centroids;      // [L][dp]
    const double* cent_sqnorm;   // [L] (Euclidean) or NULL
    int32_t* sel;                // out [nq][w], ordered (dissimilarity ascending, cluster id ascending)
    int L, dp, w;
    float mu_max;                // >= max_l |mu_l|_2
    float dmu_max;               // >= max_l |mu_l - bfloat16(mu_l)|_2
    // optional: the absmax quantization of the query (Sec. 3.3) done here as well,
    // and the batch's counters cleared, so that no separate pass over the queries is needed
    int8_t* q8;                  // out [nq][dp] or NULL
    float* dx;                   // out [nq]
    int32_t* zero;               // [nzero] cleared by this launch, or NULL
    int nzero;
    float nrm_max;               // >= max_l |mu_l|_2^2 (Euclidean; else 0)
    // LISTS instantiation of the block kernel (screen_fused.hpp): the approximate values at or below thr[q] arrive
    // as lists of 16-value groups instead of a row of ghat (ghat is then only written and read when everything has
    // to be evaluated exactly)
    const float* thr;            // [nq]
    const float* hit_val;        // [nq][nlist][cap][16]
    const int32_t* hit_grp;      // [nq][nlist][cap]  2 * (64-centroid tile) + row half; value v of a group written by
                                 //                   lane half h = list % 2 is centroid 64 tile + 32 half + 8 (v/4) + 4 h + v%4
    const int32_t* hit_cnt;      // [nq][nlist]       groups found; more than cap: the list overflowed
    int nlist, cap;
};

// Bound on |<qb, mub> - <q, mu>| for every centroid (see the header): qe >= |dq|_2, qb >= |qb|_2.
__device__ __forceinline__ float screen_eps_ip(float qe, float qb, float mu_max, float dmu_max, int dp) {
    const float e = qe * mu_max + qb * dmu_max + (float)dp * kScreenAcc * qb * (mu_max + dmu_max);
    return e * 1.001f;
}

// One block (256 threads) per query; KPT approximate values per thread in registers (256 * KPT >= L).
// dynamic LDS = dp * 4 bytes (the query).
template <int KPT, bool NT = false, bool LISTS = false>
__global__ __launch_bounds__(256) void k_select_clusters_screen(ScreenArgs a) {
    constexpr int CAP = LISTS ? 512 : 2048;     // (lists hold a few more than w entries; less LDS, more blocks per CU)
    extern __shared__ __align__(16) unsigned char scr_smem[];
    float* qs = reinterpret_cast<float*>(scr_smem);                  // [dp]
    __shared__ __align__(16) unsigned long long tmin[LISTS ? 2 : 256];
    __shared__ __align__(16) unsigned long long cand[CAP + 2];     // (key, cluster) of the first, then the final list
    __shared__ int clist[CAP];                                       // clusters evaluated exactly
    __shared__ float s_part[16];
    __shared__ int s_cnt, s_cnt2, s_over;
    __shared__ uint32_t s_bound, s_gw;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int L = a.L, dp = a.dp, w = a.w;
    const bool l2 = a.cent_sqnorm != nullptr;
    float* row = a.ghat + (size_t)blockIdx.x * L;
    const float* qrow = a.qp + (size_t)blockIdx.x * dp;
    int32_t* out = a.sel + (size_t)blockIdx.x * w;

    // the query, its norm (rounded up), the approximate values
    float v[KPT];
#pragma unroll
    for (int i = 0; i < KPT; ++i) v[i] = LISTS ? 0.0f : NT ? __builtin_nontemporal_load(&row[min(i * 256 + tid, L - 1)]) : row[min(i * 256 + tid, L - 1)];
    if (a.zero) for (int i = blockIdx.x * 256 + tid; i < a.nzero; i += gridDim.x * 256) a.zero[i] = 0;
    float nn = 0.0f, ne = 0.0f, nb = 0.0f;      // |q|^2, |dq|^2, |qb|^2
    float amax = 0.0f;
    for (int i = tid; i < dp; i += 256) {
        const float x = qrow[i];
        qs[i] = x;
        const float xb = (float)(__bf16)x, e = x - xb;            // the rounding the approximate scores used; e is exact
        nn = fmaf(x, x, nn); ne = fmaf(e, e, ne); nb = fmaf(xb, xb, nb);
        amax = fmaxf(amax, fabsf(x));
    }
    nn = wave_sum_f32(nn); ne = wave_sum_f32(ne); nb = wave_sum_f32(nb); amax = wave_max_f32(amax);
    if (lane == 0) { s_part[wv] = nn; s_part[4 + wv] = ne; s_part[8 + wv] = nb; s_part[12 + wv] = amax; }
    if (tid == 0) { s_cnt = 0; s_cnt2 = 0; s_over = 0; }
    uint32_t mn = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        if (i * 256 + tid < L) mn = min(mn, float_key_asc(v[i]));
    }
    const unsigned long long mine = ((unsigned long long)mn << 32) | (unsigned)tid;
    if (!LISTS) tmin[tid] = mine;
    __syncthreads();
    if (a.q8) {     // uniform: absmax codes of the query, exactly as k_quantize_rows computes them
        const float am = fmaxf(fmaxf(s_part[12], s_part[13]), fmaxf(s_part[14], s_part[15]));
        const bool any = am > 0.0f;
        const float cx = any ? (float)(127.0 / (double)am) : 0.0f;
        int8_t* o = a.q8 + (size_t)blockIdx.x * dp;
        for (int i = tid; i < dp; i += 256) {
            const int c8 = max(-127, min(127, (int)rintf(__fmul_rn(qs[i], cx))));
            o[i] = (int8_t)(any ? c8 : 0);
        }
        if (tid == 0) a.dx[blockIdx.x] = any ? (float)((double)am / 127.0) : 0.0f;
    }
    const float qn = sqrtf((s_part[0] + s_part[1]) + (s_part[2] + s_part[3])) * 1.001f;
    const float qe = sqrtf((s_part[4] + s_part[5]) + (s_part[6] + s_part[7])) * 1.001f;
    const float qb = sqrtf((s_part[8] + s_part[9]) + (s_part[10] + s_part[11])) * 1.001f;
    // |approximate - exact| <= eps for every cluster (see the header); Euclidean: g = nrm - 2 ip, nrm rounded to float
    float eps = screen_eps_ip(qe, qb, a.mu_max, a.dmu_max, dp);
    if (l2) eps = 2.0f * eps + 2.4e-7f * (a.nrm_max + 2.0f * qn * a.mu_max);
    eps += 1e-30f;
    // w-th smallest of the 256 per-thread minima: an upper bound of the w-th smallest approximate value
    int rank = 0;
    if (!LISTS) {
        const ulonglong2* t2 = reinterpret_cast<const ulonglong2*>(tmin);
#pragma unroll 16
        for (int u = 0; u < 128; ++u) {
            const ulonglong2 t = t2[u];
            rank += (t.x < mine ? 1 : 0) + (t.y < mine ? 1 : 0);
        }
    }
    if (!LISTS && rank == w - 1) s_bound = mn;
    __syncthreads();
    auto widen = [&](float t) {                           // t + 2 eps, rounded up generously
        const float s = t + 2.0f * eps;
        return s + 1e-6f * (fabsf(s) + eps);
    };
    // first list: everything that may lie below (w-th smallest approximate value) + 2 eps
    if (LISTS) {
        // 16 threads per list, a thread takes every 16th group; the threshold is the one the lists were made with
        const float tf1 = a.thr[blockIdx.x];
        for (int li = tid >> 4; li < a.nlist; li += 16) {
            const size_t lb = (size_t)blockIdx.x * a.nlist + li;
            const int n = a.hit_cnt[lb];
            if (n > a.cap && (tid & 15) == 0) s_over = 1;
            for (int sl = tid & 15; sl < min(n, a.cap); sl += 16) {
                const int grp = a.hit_grp[lb * a.cap + sl];
                const float4* val = reinterpret_cast<const float4*>(a.hit_val + (lb * a.cap + sl) * 16);
                float g[16];
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) { const float4 x = val[g4]; g[4 * g4] = x.x; g[4 * g4 + 1] = x.y; g[4 * g4 + 2] = x.z; g[4 * g4 + 3] = x.w; }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int l = (grp >> 1) * 64 + (grp & 1) * 32 + 8 * (e >> 2) + 4 * (li & 1) + (e & 3);
                    if (l < L && !(g[e] > tf1)) {
                        const int p = atomicAdd(&s_cnt, 1);
                        if (p < CAP) cand[p] = ((unsigned long long)float_key_asc(g[e]) << 32) | (unsigned)l;
                    }
                }
            }
        }
    } else {
        const float tf1 = widen(key_to_float(s_bound));
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const int l = i * 256 + tid;
            if (l < L && !(v[i] > tf1)) {
                const int p = atomicAdd(&s_cnt, 1);
                if (p < CAP) cand[p] = ((unsigned long long)float_key_asc(v[i]) << 32) | (unsigned)l;
            }
        }
    }
    __syncthreads();
    const int c1 = s_cnt;
    bool all_exact = c1 > CAP || (LISTS && (s_over != 0 || c1 < w));      // uniform
    int c2 = 0;
    if (!all_exact) {
        // the w-th smallest approximate value itself (it is in the list), then the final list
        if (tid < 2) cand[c1 + tid] = ~0ull;
        __syncthreads();
        const ulonglong2* cc = reinterpret_cast<const ulonglong2*>(cand);
        const int c_pairs = (c1 + 1) >> 1;
        for (int e = tid; e < c1; e += 256) {
            const unsigned long long me = cand[e];
            int r = 0;
#pragma unroll 8
            for (int u = 0; u < c_pairs; ++u) {
                const ulonglong2 t = cc[u];
                r += (t.x < me ? 1 : 0) + (t.y < me ? 1 : 0);
            }
            if (r == w - 1) s_gw = (uint32_t)(me >> 32);
        }
        __syncthreads();
        const float tf2 = widen(key_to_float(s_gw));
        for (int e = tid; e < c1; e += 256) {
            const unsigned long long me = cand[e];
            if (!(key_to_float((uint32_t)(me >> 32)) > tf2)) clist[atomicAdd(&s_cnt2, 1)] = (int)(unsigned)(me & 0xFFFFFFFFull);
        }
        __syncthreads();
        c2 = s_cnt2;
    }
    // exact values: 16 lanes per cluster, double accumulation, one rounding to float
    const int grp = tid >> 4, l16 = tid & 15;
    const int n_exact = all_exact ? L : c2;
    const int d4 = dp >> 2;                               // d' is a multiple of 16
    __syncthreads();
    const float4* q4 = reinterpret_cast<const float4*>(qs);
    if (d4 <= 64) {
        // d' <= 256: a lane holds its share of a centroid in 4 float4; two clusters per group are in flight
        for (int e0 = 0; e0 < n_exact; e0 += 32) {
            int le[2];
            float4 m[2][4];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int e = min(e0 + 16 * r + grp, n_exact - 1);
                le[r] = all_exact ? e : clist[e];
                const float4* mu = reinterpret_cast<const float4*>(a.centroids + (size_t)le[r] * dp);
#pragma unroll
                for (int u = 0; u < 4; ++u) m[r][u] = mu[min(l16 + 16 * u, d4 - 1)];
            }
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                double acc = 0.0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (l16 + 16 * u < d4) {
                        const float4 x = q4[l16 + 16 * u];
                        acc += (double)x.x * (double)m[r][u].x;
                        acc += (double)x.y * (double)m[r][u].y;
                        acc += (double)x.z * (double)m[r][u].z;
                        acc += (double)x.w * (double)m[r][u].w;
                    }
                }
                acc = row16_sum_f64_last(acc);
                const int e = e0 + 16 * r + grp;
                if (l16 == 15 && e < n_exact) {
                    const float g = l2 ? (float)(a.cent_sqnorm[le[r]] - 2.0 * acc) : (float)(-acc);
                    if (all_exact) row[le[r]] = g;
                    else cand[e] = ((unsigned long long)float_key_asc(g) << 32) | (unsigned)le[r];
                }
            }
        }
    } else {
        for (int e0 = 0; e0 < n_exact; e0 += 16) {
            const int e = min(e0 + grp, n_exact - 1);
            const int l = all_exact ? e : clist[e];
            const float4* mu = reinterpret_cast<const float4*>(a.centroids + (size_t)l * dp);
            double acc = 0.0;
            for (int i4 = l16; i4 < d4; i4 += 16) {
                const float4 m = mu[i4], x = q4[i4];
                acc += (double)x.x * (double)m.x;
                acc += (double)x.y * (double)m.y;
                acc += (double)x.z * (double)m.z;
                acc += (double)x.w * (double)m.w;
            }
            acc = row16_sum_f64_last(acc);
            if (l16 == 15 && e0 + grp < n_exact) {
                const float g = l2 ? (float)(a.cent_sqnorm[l] - 2.0 * acc) : (float)(-acc);
                if (all_exact) row[l] = g;
                else cand[e] = ((unsigned long long)float_key_asc(g) << 32) | (unsigned)l;
            }
        }
    }
    __syncthreads();
    if (all_exact) {                                      // uniform: rank the whole (now exact) row
        // the row was rewritten through global memory by other threads of this block: complete the writes, meet,
        // and drop what the vector cache still holds of the old row
        __threadfence();
        __syncthreads();
        __threadfence();
        select_clusters_radix(row, L, w, out);
    } else {
        if (tid < 2) cand[c2 + tid] = ~0ull;
        __syncthreads();
        const ulonglong2* cc = reinterpret_cast<const ulonglong2*>(cand);
        const int c_pairs = (c2 + 1) >> 1;
        for (int e = tid; e < c2; e += 256) {
            const unsigned long long me = cand[e];
            int r = 0;
#pragma unroll 8
            for (int u = 0; u < c_pairs; ++u) {
                const ulonglong2 t = cc[u];
                r += (t.x < me ? 1 : 0) + (t.y < me ? 1 : 0);
            }
            if (r < w) out[r] = (int)(unsigned)(me & 0xFFFFFFFFull);
        }
    }
}

// The same screening by ONE WAVEFRONT per query (row of approximate values in registers, KPL per lane,
// L <= 64 * KPL): no block barriers, four queries per block.  grid = ceil(nq / 4), block = 256,
// dynamic LDS = 4 * dp * 4 bytes (the four queries).
// Per wavefront: radix select of the w-th smallest approximate value; the values up to it + 2 eps form the list
// (at most kScreenWaveCap clusters; a longer list makes the wavefront evaluate all L clusters exactly); 16 lanes
// evaluate one listed cluster exactly, four clusters at a time and two rounds in flight; the list is ranked by
// (exact value, cluster id).
constexpr int kScreenWaveCap = 256;
template <int KPL>
__global__ __launch_bounds__(256) void k_select_clusters_screen_wave(ScreenArgs a, int nq) {
    extern __shared__ __align__(16) unsigned char scrw_smem[];
    __shared__ int hist[4][256];
    // per wavefront: [cand (kScreenWaveCap + 2) x 8 B | clist kScreenWaveCap x 4 B]; when everything is evaluated
    // exactly the same bytes hold the L exact values (L <= 64 * KPL floats) instead
    constexpr int kListBytes = (kScreenWaveCap + 2) * 8 + kScreenWaveCap * 4;
    constexpr int kRowBytes = 64 * KPL * 4;
    constexpr int kUnion = kListBytes > kRowBytes ? kListBytes : kRowBytes;
    __shared__ __align__(16) unsigned char wbuf[4][kUnion];
    __shared__ uint32_t selk[4][256];
    __shared__ int seli[4][256];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (a.zero) for (int i = blockIdx.x * 256 + threadIdx.x; i < a.nzero; i += gridDim.x * 256) a.zero[i] = 0;
    const int q = blockIdx.x * 4 + wv;
    if (q >= nq) return;                       // wavefronts are independent: no block barrier below
    const int L = a.L, dp = a.dp, w = a.w;
    const bool l2 = a.cent_sqnorm != nullptr;
    float* qs = reinterpret_cast<float*>(scrw_smem) + (size_t)wv * dp;
    unsigned long long* cand = reinterpret_cast<unsigned long long*>(wbuf[wv]);
    int* clist = reinterpret_cast<int*>(wbuf[wv] + (kScreenWaveCap + 2) * 8);
    float* gex = reinterpret_cast<float*>(wbuf[wv]);
    float* row = a.ghat + (size_t)q * L;
    const float* qrow = a.qp + (size_t)q * dp;
    int32_t* out = a.sel + (size_t)q * w;
    const int d4 = dp >> 2;                    // d' is a multiple of 16

    float v[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) v[i] = row[min(64 * i + lane, L - 1)];
    float nn = 0.0f, ne = 0.0f, nb = 0.0f;      // |q|^2, |dq|^2, |qb|^2
    float amax = 0.0f;
    for (int i4 = lane; i4 < d4; i4 += 64) {
        const float4 x = reinterpret_cast<const float4*>(qrow)[i4];
        reinterpret_cast<float4*>(qs)[i4] = x;
        const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float xb = (float)(__bf16)xs[t], e = xs[t] - xb;   // the rounding the approximate scores used; e is exact
            nn = fmaf(xs[t], xs[t], nn); ne = fmaf(e, e, ne); nb = fmaf(xb, xb, nb);
            amax = fmaxf(amax, fabsf(xs[t]));
        }
    }
    if (a.q8) {     // uniform: absmax codes of the query, exactly as k_quantize_rows computes them
        amax = wave_max_f32(amax);
        int8_t* o = a.q8 + (size_t)q * dp;
        const bool any = amax > 0.0f;
        const float cx = any ? (float)(127.0 / (double)amax) : 0.0f;
        for (int i4 = lane; i4 < d4; i4 += 64) {
            const float4 x = reinterpret_cast<const float4*>(qrow)[i4];      // this lane's own elements: still in its cache
            const float xs[4] = {x.x, x.y, x.z, x.w};
            char4 c;
            int v0 = max(-127, min(127, (int)rintf(__fmul_rn(xs[0], cx)))), v1 = max(-127, min(127, (int)rintf(__fmul_rn(xs[1], cx))));
            int v2 = max(-127, min(127, (int)rintf(__fmul_rn(xs[2], cx)))), v3 = max(-127, min(127, (int)rintf(__fmul_rn(xs[3], cx))));
            c.x = (signed char)(any ? v0 : 0); c.y = (signed char)(any ? v1 : 0); c.z = (signed char)(any ? v2 : 0); c.w = (signed char)(any ? v3 : 0);
            reinterpret_cast<char4*>(o)[i4] = c;
        }
        if (lane == 0) a.dx[q] = any ? (float)((double)amax / 127.0) : 0.0f;
    }
    nn = wave_sum_f32(nn); ne = wave_sum_f32(ne); nb = wave_sum_f32(nb);
    const float qn = sqrtf(nn) * 1.001f, qe = sqrtf(ne) * 1.001f, qb = sqrtf(nb) * 1.001f;
    float eps = screen_eps_ip(qe, qb, a.mu_max, a.dmu_max, dp);
    if (l2) eps = 2.0f * eps + 2.4e-7f * (a.nrm_max + 2.0f * qn * a.mu_max);
    eps += 1e-30f;
    uint32_t key[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) key[i] = 64 * i + lane < L ? float_key_asc(v[i]) : 0xFFFFFFFFu;
    auto widen = [&](float t) {                           // t + 2 eps, rounded up generously
        const float s = t + 2.0f * eps;
        return s + 1e-6f * (fabsf(s) + eps);
    };
    auto lds_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    const unsigned long long below = (1ull << lane) - 1ull;
    int c2 = 0;
    bool listed = false;
    if (w <= 64) {
        // The w-th smallest of the 64 per-lane minima bounds the w-th smallest value from above, so the values up
        // to that bound + 2 eps contain the w smallest AND the whole list; the w-th smallest itself is found by
        // counting inside this first list (a few more than w entries when the row is in no special order).
        uint32_t mn = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < KPL; ++i) mn = min(mn, key[i]);
        const unsigned long long mine = ((unsigned long long)mn << 32) | (unsigned)lane;
        cand[lane] = mine;
        lds_sync();
        int rank = 0;
        {
            const ulonglong2* t2 = reinterpret_cast<const ulonglong2*>(cand);
#pragma unroll 8
            for (int u = 0; u < 32; ++u) {
                const ulonglong2 t = t2[u];
                rank += (t.x < mine ? 1 : 0) + (t.y < mine ? 1 : 0);
            }
        }
        const int src = __ffsll((unsigned long long)__ballot(rank == w - 1)) - 1;     // exactly one lane
        const float tf1 = widen(key_to_float((uint32_t)__shfl((int)mn, src, 64)));
        lds_sync();
        int c1 = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            const int l = 64 * i + lane;
            const bool in = l < L && !(v[i] > tf1);
            const unsigned long long mk = __ballot(in);
            const int p = c1 + __popcll(mk & below);
            if (in && p < kScreenWaveCap) cand[p] = ((unsigned long long)key[i] << 32) | (unsigned)l;
            c1 += __popcll(mk);
        }
        if (c1 <= kScreenWaveCap) {                        // uniform
            if (lane < 2) cand[c1 + lane] = ~0ull;
            lds_sync();
            const ulonglong2* cc = reinterpret_cast<const ulonglong2*>(cand);
            const int c_pairs = (c1 + 1) >> 1;
            uint32_t gw_mine = 0u;
            bool found = false;
            unsigned long long mine_e[kScreenWaveCap / 64];
#pragma unroll
            for (int j = 0; j < kScreenWaveCap / 64; ++j) {
                const int e = lane + 64 * j;
                mine_e[j] = e < c1 ? cand[e] : ~0ull;
                int r = 0;
                if (e < c1) {
                    for (int u = 0; u < c_pairs; ++u) {
                        const ulonglong2 t = cc[u];
                        r += (t.x < mine_e[j] ? 1 : 0) + (t.y < mine_e[j] ? 1 : 0);
                    }
                    if (r == w - 1) { found = true; gw_mine = (uint32_t)(mine_e[j] >> 32); }
                }
            }
            const int src2 = __ffsll((unsigned long long)__ballot(found)) - 1;
            const float tf2 = widen(key_to_float((uint32_t)__shfl((int)gw_mine, src2, 64)));
#pragma unroll
            for (int j = 0; j < kScreenWaveCap / 64; ++j) {
                const int e = lane + 64 * j;
                const bool in = e < c1 && !(key_to_float((uint32_t)(mine_e[j] >> 32)) > tf2);
                const unsigned long long mk = __ballot(in);
                if (in) clist[c2 + __popcll(mk & below)] = (int)(unsigned)(mine_e[j] & 0xFFFFFFFFull);
                c2 += __popcll(mk);
            }
            listed = true;
        }
    }
    if (!listed) {
        // radix select of the w-th smallest approximate value, then the list
        int need_unused;
        lds_sync();
        const uint32_t gw = wave_wth_smallest_key<KPL>(key, L, w, hist[wv], need_unused);
        const float tf2 = widen(key_to_float(gw));
        c2 = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            const int l = 64 * i + lane;
            const bool in = l < L && !(v[i] > tf2);
            const unsigned long long mk = __ballot(in);
            const int p = c2 + __popcll(mk & below);
            if (in && p < kScreenWaveCap) clist[p] = l;
            c2 += __popcll(mk);
        }
    }
    const bool all_exact = c2 > kScreenWaveCap;            // uniform over the wavefront
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // exact values: 16 lanes per cluster, 4 clusters at a time, 2 rounds (8 clusters) requested together
    const int grp = lane >> 4, l16 = lane & 15;
    const int n_exact = all_exact ? L : c2;
    const float4* q4 = reinterpret_cast<const float4*>(qs);
    auto exact_of = [&](int l, const float4* mu) {       // full rows of 16 lanes execute this together
        double acc = 0.0;
        for (int i4 = l16; i4 < d4; i4 += 16) {
            const float4 m = mu[i4], x = q4[i4];
            acc += (double)x.x * (double)m.x;
            acc += (double)x.y * (double)m.y;
            acc += (double)x.z * (double)m.z;
            acc += (double)x.w * (double)m.w;
        }
        acc = row16_sum_f64_last(acc);
        return l2 ? (float)(a.cent_sqnorm[l] - 2.0 * acc) : (float)(-acc);
    };
    if (d4 <= 64) {
        // d' <= 256: a lane holds its share of a centroid in 4 float4; two rounds are in flight
        for (int e0 = 0; e0 < n_exact; e0 += 8) {
            int le[2];
            float4 m[2][4];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int e = min(e0 + 4 * r + grp, n_exact - 1);
                le[r] = all_exact ? e : clist[e];
                const float4* mu = reinterpret_cast<const float4*>(a.centroids + (size_t)le[r] * dp);
#pragma unroll
                for (int u = 0; u < 4; ++u) m[r][u] = mu[min(l16 + 16 * u, d4 - 1)];
            }
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                double acc = 0.0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (l16 + 16 * u < d4) {
                        const float4 x = q4[l16 + 16 * u];
                        acc += (double)x.x * (double)m[r][u].x;
                        acc += (double)x.y * (double)m[r][u].y;
                        acc += (double)x.z * (double)m[r][u].z;
                        acc += (double)x.w * (double)m[r][u].w;
                    }
                }
                acc = row16_sum_f64_last(acc);
                const int e = e0 + 4 * r + grp;
                if (l16 == 15 && e < n_exact) {
                    const float g = l2 ? (float)(a.cent_sqnorm[le[r]] - 2.0 * acc) : (float)(-acc);
                    if (all_exact) gex[le[r]] = g;
                    else cand[e] = ((unsigned long long)float_key_asc(g) << 32) | (unsigned)le[r];
                }
            }
        }
    } else {
        for (int e0 = 0; e0 < n_exact; e0 += 4) {
            const int e = min(e0 + grp, n_exact - 1);
            const int l = all_exact ? e : clist[e];
            const float g = exact_of(l, reinterpret_cast<const float4*>(a.centroids + (size_t)l * dp));
            if (l16 == 15 && e0 + grp < n_exact) {
                if (all_exact) gex[l] = g;
                else cand[e] = ((unsigned long long)float_key_asc(g) << 32) | (unsigned)l;
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (all_exact) {                                       // rank the whole exact row
#pragma unroll
        for (int i = 0; i < KPL; ++i) key[i] = 64 * i + lane < L ? float_key_asc(gex[64 * i + lane]) : 0xFFFFFFFFu;
        wave_select_from_keys<KPL>(key, L, w, out, hist[wv], selk[wv], seli[wv]);
        return;
    }
    if (lane < 2) cand[c2 + lane] = ~0ull;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const ulonglong2* cc = reinterpret_cast<const ulonglong2*>(cand);
    const int c_pairs = (c2 + 1) >> 1;
    for (int e = lane; e < c2; e += 64) {
        const unsigned long long me = cand[e];
        int r = 0;
#pragma unroll 8
        for (int u = 0; u < c_pairs; ++u) {
            const ulonglong2 t = cc[u];
            r += (t.x < me ? 1 : 0) + (t.y < me ? 1 : 0);
        }
        if (r < w) out[r] = (int)(unsigned)(me & 0xFFFFFFFFull);
    }
}

}  // namespace lorann
