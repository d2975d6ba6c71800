// Second 8-bit product on the int8 matrix cores, organised by CLUSTER (Sec. 3.2-3.3; batching per cluster
// replaces the per-(query, cluster) gathers of the paper's GPU design, Sec. 4.3): the (query, cluster) pairs
// were bucketed by cluster, so a wavefront takes one cluster and up to 32*NZ of its pairs, streams the
// cluster's codes B_c once, and contracts each 32-point tile against its pairs with
// v_mfma_i32_32x32x32_i8:   Y[pair][point] = sum_t z[pair][t] * code[point][t]   (int32, exact).
//
// Register layout of that instruction (measured on gfx950): both operands give lane l sixteen consecutive
// k-bytes (k-half l/32) of row / column l%32; result register v of lane l holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32].  With pairs as rows and points as columns, lane l owns ONE point of the
// tile and register v belongs to ONE pair (per lane half), so "does pair i have a survivor in this tile" is
// one compare per register, and the 64-bit lane mask it produces says which points survived.
//
// Exact top-m without materialising the scores: a lower bound tau_q on each query's m-th best score is known
// before this kernel runs (the m-th best score inside the query's nearest cluster(s), k_seed_threshold), so
// only scores >= tau_q - typically little more than m per query, concentrated in few pairs - survive.  They
// are compacted into a small per-wavefront LDS buffer (prefix count over the lane mask) and drained to the
// query's survivor list with one atomic slot reservation each.  The exact top-m of the survivors is the
// exact top-m overall; queries whose list overflows are finished by the exact per-query kernel.
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

// Orders this wavefront's LDS writes before its later LDS reads (the buffers are private to the wavefront).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Drain a wavefront's buffered survivors (query, score, row) to the per-query lists: one atomic slot
// reservation per entry; entries beyond the list capacity are dropped (the count still records them).
// Kept out of line: it is called from many places of an unrolled loop and runs rarely.
__device__ __attribute__((noinline)) void drain_survivors(const int* eq, const float* es, const int* er, int count,
                                                          int32_t* surv_cnt, float* surv_score, int32_t* surv_row, int cap) {
    const int lane = threadIdx.x & 63;
    wave_lds_sync();
    for (int e = lane; e < count; e += 64) {
        const int q = eq[e];
        const int idx = atomicAdd(&surv_cnt[q], 1);
        if (idx < cap) {
            surv_score[(size_t)q * cap + idx] = es[e];
            surv_row[(size_t)q * cap + idx] = er[e];
        }
    }
    wave_lds_sync();
}

// grid = ceil(max_units / 4), block = 256 (one unit per wavefront).
// NZ pair tiles per unit, KS = r_pad / 32 k-steps, L2 = Euclidean score epilogue (per-point bias, float domain;
// inner product and cosine compare in the integer domain, where sigma > 0 is constant per pair).
template <int NZ, int KS, bool L2>
__global__ __launch_bounds__(256) void k_score_filter(ScoreArgs a) {
    constexpr int NP = 32 * NZ;        // pairs per unit
    constexpr int CW = 256;            // survivor entries buffered per wavefront
    constexpr int RP = KS * 32;
    constexpr int TB = 4;              // point tiles fetched per chunk
    __shared__ int s_q[4][NP];
    __shared__ float s_sig[4][NP];
    __shared__ int s_thr[4][NP];
    __shared__ int s_eq[4][CW];
    __shared__ float s_es[4][CW];
    __shared__ int s_er[4][CW];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int unit = blockIdx.x * 4 + wv;
    if (unit >= a.unit_off[a.L]) return;          // no block-wide barrier below: wavefronts are independent
    const int c = find_bucket(a.unit_off, a.L, unit);
    const int pb = a.bucket_off[c] + (unit - a.unit_off[c]) * NP;
    const int pend = a.bucket_off[c + 1];
    const int64_t row0 = a.off[c];
    const int m_c = (int)(a.off[c + 1] - row0);
    const int j = lane & 31, h = lane >> 5;

    // per-pair tables: query number, score scale, threshold
    for (int p = lane; p < NP; p += 64) {
        const int gp = pb + p;
        int q = 0, thr = 0x7fffffff;
        float sgm = 0.0f;
        if (gp < pend) {
            const float s = a.sigma[gp];
            q = a.slot_of_pos[gp] / a.w;
            const float t = a.tau[q];
            sgm = L2 ? 2.0f * s : s;
            if (L2) {
                thr = __float_as_int(t);
            } else if (s > 0.0f) {
                // smallest integer score that can reach t, minus a safety margin of 2 (survivors are re-selected
                // exactly later, so passing a few extra scores is harmless; missing one would not be)
                const float y = t / s;
                thr = !(y > -2.0e6f) ? (int)0x80000000 : (y > 2.0e6f ? 0x7fffffff : (int)floorf(y) - 2);
            } else {
                thr = (0.0f >= t) ? (int)0x80000000 : 0x7fffffff;       // every score of the pair is 0
            }
        } else if (L2) {
            thr = __float_as_int(INFINITY);
        }
        s_q[wv][p] = q; s_sig[wv][p] = sgm; s_thr[wv][p] = thr;
    }
    wave_lds_sync();

    i32x4 zreg[NZ][KS];
    int thr[NZ][16];           // threshold of the pair that register v of this lane half belongs to
    float sgv[NZ][16];         // Euclidean only: its scale
#pragma unroll
    for (int z = 0; z < NZ; ++z) {
        const int gp = pb + 32 * z + j;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            zreg[z][ks] = (i32x4){0, 0, 0, 0};
            if (gp < pend) zreg[z][ks] = load16(a.Z + (size_t)gp * RP + 32 * ks + 16 * h);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            thr[z][v] = s_thr[wv][32 * z + tile_row(v, h)];
            if (L2) sgv[z][v] = s_sig[wv][32 * z + tile_row(v, h)];
        }
    }

    int wcount = 0;            // entries in this wavefront's buffer (uniform)
    auto flush = [&]() {
        drain_survivors(s_eq[wv], s_es[wv], s_er[wv], wcount, a.surv_cnt, a.surv_score, a.surv_row, a.cap);
        wcount = 0;
    };

    const int ntiles = (m_c + 31) >> 5;
    const int nchunks = (ntiles + TB - 1) / TB;
    auto fetch_chunk = [&](int t0, i32x4 (*dst)[KS]) {
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int pt = 32 * (t0 + u) + j;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                dst[u][ks] = (i32x4){0, 0, 0, 0};
                if (pt < m_c) dst[u][ks] = load16(a.Bp + (size_t)(row0 + pt) * RP + 32 * ks + 16 * h);
            }
        }
    };
    i32x4 bnext[TB][KS];
    if (nchunks > 0) fetch_chunk(0, bnext);
    for (int c0 = 0; c0 < nchunks; ++c0) {
        i32x4 breg[TB][KS];
#pragma unroll
        for (int u = 0; u < TB; ++u)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) breg[u][ks] = bnext[u][ks];
        if (c0 + 1 < nchunks) fetch_chunk((c0 + 1) * TB, bnext);
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int t = c0 * TB + u;
            if (t < ntiles) {                        // uniform
                const int pt = 32 * t + j;           // this lane's point of the tile
                const unsigned long long okmask = __ballot(pt < m_c);
                float bias = 0.0f;
                if (L2 && pt < m_c) bias = a.sqnorm[row0 + pt];
#pragma unroll
                for (int z = 0; z < NZ; ++z) {
                    i32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(zreg[z][ks], breg[u][ks], acc, 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float sc = 0.0f;
                        bool keep;
                        if (!L2) {
                            keep = acc[v] >= thr[z][v];
                        } else {
                            sc = __fmaf_rn((float)acc[v], sgv[z][v], -bias);
                            keep = sc >= __int_as_float(thr[z][v]);
                        }
                        const unsigned long long m64 = __ballot(keep) & okmask;
                        if (m64 != 0ull) {           // uniform: some point of this tile survives for this pair
                            if (wcount + 64 > CW) flush();
                            const bool mine = (m64 >> lane) & 1ull;
                            const int pos = wcount + __popcll(m64 & ((1ull << lane) - 1ull));
                            if (mine) {
                                const int pr = 32 * z + tile_row(v, h);
                                if (!L2) sc = __fmaf_rn((float)acc[v], s_sig[wv][pr], -0.0f);
                                s_eq[wv][pos] = s_q[wv][pr];
                                s_es[wv][pos] = sc;
                                s_er[wv][pos] = (int32_t)(row0 + pt);
                            }
                            wcount += __popcll(m64);
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);       // keep the tiles sequential: bounds live accumulators
        }
    }
    if (wcount > 0) flush();
}

}  // namespace lorann
