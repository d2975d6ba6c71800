// Routing by screening (Sec. 2.2, 4.1) for many queries x many clusters WITHOUT writing the nq x L matrix of
// approximate dissimilarities: the bf16 matrix-core product is computed twice and only digests leave the chip.
//
//   pass A (k_screen_pass<.., false>)  every approximate value is folded into the minimum of one of S = 32 * nsplit
//                                      disjoint subsets of the clusters; out: smin [nq][S].
//   threshold (k_screen_threshold)     the w-th smallest of the S subset minima is an upper bound of the w-th smallest
//                                      approximate value (w distinct clusters do not exceed it); thr = that bound
//                                      + 2 eps, eps the rigorous bound of screen.hpp on |approximate - exact|.
//   pass B (k_screen_pass<.., true>)   the same product again; a lane that finds one of its 16 results of a tile at
//                                      or below its query's thr appends the 16 values to a list that only this lane
//                                      writes (no atomics, no round trips).
//   finish (k_select_clusters_screen<.., LISTS>)  per query: the listed values up to thr are the "first list" of the
//                                      block kernel of screen.hpp, which continues unchanged - w-th smallest
//                                      approximate value, final list, exact evaluation in double, ranking.
//
// Why the result is still exact: the w subsets behind the bound each hold a cluster whose pass-A value is <= bound,
// so its exact value is <= bound + eps and the exact w-th best is too; every cluster of the exact w best therefore
// has a pass-B value <= bound + 2 eps = thr and is listed (pass A and pass B may even round differently: eps covers
// any order of the float additions).  At least w listed values are <= thr, so the w-th smallest approximate value
// of ALL clusters is the w-th smallest listed one, and from there on the argument of screen.hpp applies.  A lane's
// list that overflows, or a first list beyond the block's capacity, makes the finish kernel evaluate every cluster
// exactly, as before.
//
// The product itself: a wavefront keeps the bf16 operands of 64 queries in registers for its whole life (queries are
// the COLUMNS of v_mfma_f32_32x32x16_bf16, so a lane holds results of one query per column tile and all of a lane's
// comparisons use one threshold); tiles of 64 centroids are staged through LDS (double buffered, one barrier per
// tile) and shared by the block's wavefronts.  grid = (ceil(nq / (64 * waves)), nsplit): block (x, y) serves its
// queries against the y-th run of centroid tiles.
#pragma once
#include "screen.hpp"

namespace lorann {

constexpr int kFusedSplits = 8;                // runs of centroid tiles = blocks along y (long runs: a block's set-up - its
                                               // queries into registers, the first tile - is paid once per run)
constexpr int kFusedSubsets = 32 * kFusedSplits;   // subset = (run, lane half, result register): 256
constexpr int kFusedLists = 2 * kFusedSplits;   // lists per query: (run, lane half)
constexpr int kFusedCap = 32;                  // 16-value groups a list can hold

struct ScreenPassArgs {
    const __bf16* Q;             // [nq][dp] queries rounded to bfloat16
    const __bf16* C;             // [L][dp] centroids rounded to bfloat16
    const float* nrm;            // [L] |mu_l|^2 in float (Euclidean) or NULL
    int nq, L;
    int tiles_per_split;         // 64-centroid tiles per run
    float* smin;                 // pass A out: [nq][kFusedSubsets]
    const float* thr;            // pass B in:  [nq]
    float* hit_val;              // pass B out: [nq][kFusedLists][kFusedCap][16] values of a group
    int32_t* hit_grp;            //             [nq][kFusedLists][kFusedCap]     2 * tile + (row half of the tile)
    int32_t* hit_cnt;            //             [nq][kFusedLists]                groups found (may exceed kFusedCap)
};

// Cluster of value v of a group: result register v of a lane of half h holds row 8 * (v / 4) + 4 h + v % 4.
__device__ __forceinline__ int fused_group_cluster(int grp, int h, int v) {
    return (grp >> 1) * 64 + (grp & 1) * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
}

template <int KS, bool L2, bool EMIT, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_screen_pass(ScreenPassArgs a) {
    constexpr int DP = 16 * KS;
    constexpr int NT = 64 * WAVES;
    // A staged centroid row is padded by 16 bytes so that the 16-byte reads of 8 consecutive rows fall into different
    // banks; at d' = 256 two padded tiles would exceed 64 KB of LDS, so there the 16-byte pieces of a row are permuted
    // instead (piece p of row i sits in slot p ^ (i % 8): same effect, no padding) and the norms come from memory.
    constexpr bool SWZ = KS == 16;
    constexpr int ROWB = DP * 2 + (SWZ ? 0 : 16);
    constexpr int TILEB = 64 * ROWB + (SWZ ? 0 : 256);        // + the tile's 64 norms
    constexpr int RP = DP / 8;                    // 16-byte pieces per row
    constexpr int PPT = 64 * RP / NT;             // pieces per thread
    static_assert(64 * RP % NT == 0, "tile pieces divide over the block");
    extern __shared__ __align__(16) unsigned char sf_smem[];       // 2 * TILEB
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int q0 = ((int)blockIdx.x * WAVES + wv) * 64;
    const int split = blockIdx.y;
    const int ntiles = (a.L + 63) >> 6;
    const int t_beg = min(ntiles, split * a.tiles_per_split), t_end = min(ntiles, t_beg + a.tiles_per_split);

    // the wavefront's 64 queries, resident: operand of column tile qt, k-step ks (inner product: negated, exact in bfloat16)
    bf16x8 qreg[2][KS];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const __bf16* qrow = a.Q + (size_t)min(q0 + 32 * qt + i, a.nq - 1) * DP + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 u = *reinterpret_cast<const uint4*>(qrow + 16 * ks);
            if (!L2) { u.x ^= 0x80008000u; u.y ^= 0x80008000u; u.z ^= 0x80008000u; u.w ^= 0x80008000u; }
            qreg[qt][ks] = __builtin_bit_cast(bf16x8, u);
        }
    }
    uint4 stage[PPT];
    float nstage = 0.0f;
    auto g_load = [&](int tile) {               // unconditional loads, rows clamped into the matrix
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            const int p = tid + NT * u, row = p / RP, pc = p - row * RP;
            stage[u] = *reinterpret_cast<const uint4*>(a.C + (size_t)min(tile * 64 + row, a.L - 1) * DP + 8 * pc);
        }
        if (L2 && !SWZ && tid < 64) nstage = a.nrm[min(tile * 64 + tid, a.L - 1)];
    };
    auto s_store = [&](int buf) {
        unsigned char* tb = sf_smem + buf * TILEB;
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            const int p = tid + NT * u, row = p / RP, pc = p - row * RP;
            *reinterpret_cast<uint4*>(tb + row * ROWB + (SWZ ? (pc ^ (row & 7)) : pc) * 16) = stage[u];
        }
        if (L2 && !SWZ && tid < 64) reinterpret_cast<float*>(tb + 64 * ROWB)[tid] = nstage;
    };

    float mn[2][16];
    int cnt[2] = {0, 0};
    float thr[2] = {0.0f, 0.0f};
    bool qok[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        qok[qt] = q0 + 32 * qt + i < a.nq;
#pragma unroll
        for (int j = 0; j < 16; ++j) mn[qt][j] = INFINITY;
        if (EMIT) thr[qt] = a.thr[min(q0 + 32 * qt + i, a.nq - 1)];
    }

    if (t_beg < t_end) {
        g_load(t_beg);
        s_store(0);
    }
    __syncthreads();
    for (int t = t_beg; t < t_end; ++t) {
        const int buf = (t - t_beg) & 1;
        g_load(min(t + 1, t_end - 1));                        // unconditional (a repeat of the last tile at the end, not stored)
        const unsigned char* tb = sf_smem + buf * TILEB;
        f32x16 acc[2][2];
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[ct][qt][v] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int piece = SWZ ? ((2 * ks + h) ^ (i & 7)) : 2 * ks + h;        // ((32 + i) % 8 == i % 8)
            const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(tb + i * ROWB + piece * 16);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(tb + (32 + i) * ROWB + piece * 16);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qreg[0][ks], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qreg[1][ks], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qreg[0][ks], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qreg[1][ks], acc[1][1], 0, 0, 0);
        }
        const bool ragged = t * 64 + 64 > a.L;       // uniform: the last tile may hold rows beyond the matrix
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
            float nv[16];
            if (L2 && SWZ) {
#pragma unroll
                for (int v = 0; v < 16; ++v) nv[v] = a.nrm[min(t * 64 + 32 * ct + 8 * (v >> 2) + 4 * h + (v & 3), a.L - 1)];
            } else if (L2) {
                const float4* n4 = reinterpret_cast<const float4*>(tb + 64 * ROWB) + (32 * ct + 4 * h) / 4;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const float4 x = n4[2 * g4];
                    nv[4 * g4] = x.x; nv[4 * g4 + 1] = x.y; nv[4 * g4 + 2] = x.z; nv[4 * g4 + 3] = x.w;
                }
            }
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                float g[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) g[v] = L2 ? fmaf(-2.0f, acc[ct][qt][v], nv[v]) : acc[ct][qt][v];
                if (ragged) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (t * 64 + 32 * ct + 8 * (v >> 2) + 4 * h + (v & 3) >= a.L) g[v] = INFINITY;
                }
                if (!EMIT) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) mn[qt][v] = __builtin_fminimum_numf(mn[qt][v], g[v]);     // (minimumnum: no quieting of each input)
                } else {
                    float gm = __builtin_fminimum_numf(g[0], g[1]);        // (three-operand minima, no quieting of each input)
#pragma unroll
                    for (int v = 2; v < 16; ++v) gm = __builtin_fminimum_numf(gm, g[v]);
                    if (qok[qt] && !(gm > thr[qt])) {
                        const int sl = cnt[qt]++;
                        if (sl < kFusedCap) {
                            const size_t li = ((size_t)(q0 + 32 * qt + i) * kFusedLists + 2 * split + h) * kFusedCap + sl;
                            float4* dst = reinterpret_cast<float4*>(a.hit_val + li * 16);
#pragma unroll
                            for (int g4 = 0; g4 < 4; ++g4) dst[g4] = make_float4(g[4 * g4], g[4 * g4 + 1], g[4 * g4 + 2], g[4 * g4 + 3]);
                            a.hit_grp[li] = 2 * t + ct;
                        }
                    }
                }
            }
        }
        if (t + 1 < t_end) s_store(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        if (!qok[qt]) continue;
        const int q = q0 + 32 * qt + i;
        if (!EMIT) {
            float4* dst = reinterpret_cast<float4*>(a.smin + (size_t)q * kFusedSubsets + (2 * split + h) * 16);
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) dst[g4] = make_float4(mn[qt][4 * g4], mn[qt][4 * g4 + 1], mn[qt][4 * g4 + 2], mn[qt][4 * g4 + 3]);
        } else {
            a.hit_cnt[(size_t)q * kFusedLists + 2 * split + h] = cnt[qt];
        }
    }
}

// One wavefront per query (four per block): thr[q] = (w-th smallest of the kFusedSubsets subset minima) + 2 eps, widened
// as the finish kernel widens its own thresholds.  w <= kFusedSubsets.
__global__ __launch_bounds__(256) void k_screen_threshold(const float* __restrict__ smin, const float* __restrict__ qp, int nq, int dp, int w, bool l2,
                                                          float mu_max, float dmu_max, float nrm_max, float* __restrict__ thr) {
    constexpr int KPL = kFusedSubsets / 64;
    __shared__ int hist[4][256];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int q = blockIdx.x * 4 + wv;
    if (q >= nq) return;                        // wavefronts are independent: no block barrier below
    uint32_t key[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) key[i] = float_key_asc(smin[(size_t)q * kFusedSubsets + 64 * i + lane]);
    float nn = 0.0f, ne = 0.0f, nb = 0.0f;      // |q|^2, |dq|^2, |qb|^2
    for (int e = lane; e < dp; e += 64) {
        const float x = qp[(size_t)q * dp + e];
        const float xb = (float)(__bf16)x, er = x - xb;
        nn = fmaf(x, x, nn); ne = fmaf(er, er, ne); nb = fmaf(xb, xb, nb);
    }
    nn = wave_sum_f32(nn); ne = wave_sum_f32(ne); nb = wave_sum_f32(nb);
    int need_unused;
    const uint32_t bound = wave_wth_smallest_key<KPL>(key, kFusedSubsets, w, hist[wv], need_unused);
    if (lane == 0) {
        const float qn = sqrtf(nn) * 1.001f, qe = sqrtf(ne) * 1.001f, qb = sqrtf(nb) * 1.001f;
        float eps = screen_eps_ip(qe, qb, mu_max, dmu_max, dp);
        if (l2) eps = 2.0f * eps + 2.4e-7f * (nrm_max + 2.0f * qn * mu_max);
        eps += 1e-30f;
        const float s = key_to_float(bound) + 2.0f * eps;
        thr[q] = s + 1e-6f * (fabsf(s) + eps);
    }
}

}  // namespace lorann
