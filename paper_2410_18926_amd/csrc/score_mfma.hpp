// Second 8-bit product on the int8 matrix cores, organised by CLUSTER (Sec. 3.2-3.3; batching per cluster
// replaces the per-(query, cluster) gathers of the paper's GPU design, Sec. 4.3): the (query, cluster) pairs
// were bucketed by cluster, so a wavefront takes one cluster and up to 32*NZ of its pairs, streams the
// cluster's codes B_c once, and contracts each 32-point tile against its pairs with
// v_mfma_i32_32x32x32_i8:   Y[point][pair] = sum_t code[point][t] * z[pair][t]   (int32, exact).
//
// Register layout of that instruction (measured on gfx950): both operands give lane l sixteen consecutive
// k-bytes (k-half l/32) of row / column l%32; result register v of lane l holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32].  With points as rows and pairs as columns every lane owns ONE pair and
// sees 16 of its scores per tile, so per-pair state (scale, threshold) lives in registers.
//
// Exact top-m without materialising the scores: a lower bound tau_q on each query's m-th best score is known
// before this kernel runs (the m-th best score inside the query's nearest cluster(s), k_seed_threshold), so
// only scores >= tau_q - typically little more than m per query - are appended to the query's survivor list.
// The exact top-m of the survivors is the exact top-m overall.  Queries whose survivor list overflows are
// finished by the exact per-query kernel.
#pragma once
#include "common.hpp"
#include "stage_a.hpp"

namespace lorann {

struct ScoreArgs {
    const int8_t* Bp;            // [n][r_pad]
    const int8_t* Z;             // [npairs][r_pad] bucket order
    const float* sigma;          // [npairs] bucket order
    const int64_t* off;          // [L+1] corpus rows of each cluster
    const int32_t* bucket_off;   // [L+1] pairs of each cluster
    const int32_t* unit_off;     // [L+1] 32*NZ-pair units of each cluster
    const int32_t* slot_of_pos;  // [npairs]
    const float* sqnorm;         // [n] (Euclidean) or NULL
    const float* tau;            // in:  [nq] lower bounds on the m-th best score
    int32_t* surv_cnt;           // out: [nq] survivors found (may exceed cap; only the first cap are stored)
    float* surv_score;           // out: [nq][cap]
    int32_t* surv_row;           // out: [nq][cap]
    int L, w, cap;
};

// Row (within the 32-point tile) of result register v for lane half h.
__device__ __forceinline__ int tile_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// grid = ceil(max_units / 4), block = 256 (one unit per wavefront).
// NZ pair tiles per unit, KS = r_pad / 32 k-steps, L2 = Euclidean score epilogue (per-point bias, float domain;
// inner product and cosine compare in the integer domain, where sigma > 0 is constant per pair).
template <int NZ, int KS, bool L2>
__global__ __launch_bounds__(256) void k_score_filter(ScoreArgs a) {
    const int lane = threadIdx.x & 63;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= a.unit_off[a.L]) return;
    const int c = find_bucket(a.unit_off, a.L, unit);
    const int pb = a.bucket_off[c] + (unit - a.unit_off[c]) * (32 * NZ);
    const int pend = a.bucket_off[c + 1];
    const int64_t row0 = a.off[c];
    const int m_c = (int)(a.off[c + 1] - row0);
    const int j = lane & 31, h = lane >> 5;
    constexpr int RP = KS * 32;

    i32x4 zreg[NZ][KS];
    float sg[NZ];
    bool pok[NZ];
    int thr[NZ];          // inner product / cosine: integer threshold (no false negatives)
    float tauf[NZ];       // Euclidean: float threshold
    int qn[NZ];
#pragma unroll
    for (int z = 0; z < NZ; ++z) {
        const int p = pb + 32 * z + j;
        pok[z] = p < pend;
        sg[z] = 0.0f; thr[z] = 0x7fffffff; tauf[z] = INFINITY; qn[z] = 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) zreg[z][ks] = (i32x4){0, 0, 0, 0};
        if (pok[z]) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) zreg[z][ks] = load16(a.Z + (size_t)p * RP + 32 * ks + 16 * h);
            const float s = a.sigma[p];
            sg[z] = L2 ? 2.0f * s : s;
            qn[z] = a.slot_of_pos[p] / a.w;
            const float t = a.tau[qn[z]];
            tauf[z] = t;
            if (!L2) {
                // smallest integer score that can reach t, minus a safety margin of 2 (the survivors are
                // re-selected exactly later, so passing a few extra scores is harmless)
                if (s > 0.0f) {
                    const float y = t / s;
                    thr[z] = !(y > -2.0e6f) ? (int)0x80000000 : (y > 2.0e6f ? 0x7fffffff : (int)floorf(y) - 2);
                } else {
                    thr[z] = (0.0f >= t) ? (int)0x80000000 : 0x7fffffff;   // every score of the pair is 0
                }
            }
        }
    }

    const int ntiles = (m_c + 31) >> 5;
    i32x4 bnext[KS];
    auto fetch = [&](int t, i32x4* dst) {
        const int pt = 32 * t + j;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            dst[ks] = (i32x4){0, 0, 0, 0};
            if (pt < m_c) dst[ks] = load16(a.Bp + (size_t)(row0 + pt) * RP + 32 * ks + 16 * h);
        }
    };
    if (ntiles > 0) fetch(0, bnext);

    for (int t = 0; t < ntiles; ++t) {
        i32x4 breg[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) breg[ks] = bnext[ks];
        if (t + 1 < ntiles) fetch(t + 1, bnext);
        const bool tail = 32 * t + 32 > m_c;         // only the last tile can hold rows beyond the cluster
        float bias[16];
        if (L2) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int pt = 32 * t + tile_row(v, h);
                bias[v] = pt < m_c ? a.sqnorm[row0 + pt] : 0.0f;
            }
        }
#pragma unroll
        for (int z = 0; z < NZ; ++z) {
            i32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(breg[ks], zreg[z][ks], acc, 0, 0, 0);
            if (tail) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (32 * t + tile_row(v, h) >= m_c) acc[v] = (int)0x80000000;   // marks "no point"
            }
            {
                // count this lane's survivors of the tile, reserve room with one atomic, write them
                unsigned mask = 0;
                float sc[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    bool keep;
                    if (!L2) {
                        keep = acc[v] >= thr[z] && acc[v] != (int)0x80000000;
                    } else {
                        sc[v] = acc[v] == (int)0x80000000 ? -INFINITY : __fmaf_rn((float)acc[v], sg[z], -bias[v]);
                        keep = sc[v] >= tauf[z] && acc[v] != (int)0x80000000;
                    }
                    mask |= keep ? (1u << v) : 0u;
                }
                if (!pok[z]) mask = 0;
                if (mask) {
                    const int cntl = __popc(mask);
                    int base = atomicAdd(&a.surv_cnt[qn[z]], cntl);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        if ((mask >> v) & 1u) {
                            if (base < a.cap) {
                                const float s = L2 ? sc[v] : __fmaf_rn((float)acc[v], sg[z], -0.0f);
                                a.surv_score[(size_t)qn[z] * a.cap + base] = s;
                                a.surv_row[(size_t)qn[z] * a.cap + base] = (int32_t)(row0 + 32 * t + tile_row(v, h));
                            }
                            ++base;
                        }
                    }
                }
            }
        }
    }
}

}  // namespace lorann
