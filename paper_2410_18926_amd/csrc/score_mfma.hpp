// Second 8-bit product on the int8 matrix cores, organised by CLUSTER (Sec. 3.2-3.3; batching per cluster
// replaces the per-(query, cluster) gathers of the paper's GPU design, Sec. 4.3): the (query, cluster) pairs
// were bucketed by cluster, so a wavefront takes one cluster, up to 32*NZ of its pairs and a range of its
// codes B_c, and contracts each 32-point tile against the pairs with
// v_mfma_i32_32x32x32_i8:   Y[point][pair] = sum_t code[point][t] * z[pair][t]   (int32, exact).
//
// Register layout of that instruction (measured on gfx950): both operands give lane l sixteen consecutive
// k-bytes (k-half l/32) of row / column l%32; result register v of lane l holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32].  With points as rows and pairs as columns, lane l owns ONE pair and its
// sixteen result registers are sixteen points of the tile: everything that belongs to a pair (its scale, its
// running maxima) is one value per lane, and a maximum over points is a maximum over the lane's own registers -
// no cross-lane reduction except joining the two lane halves.
//
// Exact top-m without materialising the scores: this kernel only computes MAXIMA - for every pair the best score
// of each CHUNK of 64 consecutive points of the cluster (one three-operand maximum per two scores, no per-score
// branch) and from them the best score of the pair.  The per-query kernel (select_query.hpp) derives from the
// chunk maxima a lower bound of the query's m-th best score and then scores point by point only the chunks whose
// maximum reaches the running m-th best score; every other chunk and pair is dismissed by its maximum alone.
#pragma once
#include "common.hpp"
#include "stage_a.hpp"

namespace lorann {

constexpr int kScoreChunk = 64;      // points per chunk maximum (two 32-point tiles)

struct ScoreArgs {
    const int8_t* Bp;            // [n][r_pad]
    const int8_t* Z;             // [npairs][r_pad] bucket order
    const float* sigma;          // [npairs] bucket order
    const int64_t* off;          // [L+1] corpus rows of each cluster
    const int32_t* bucket_off;   // [L+1] pairs of each cluster
    const int32_t* unit_off;     // [L+1] work items (pair group x point range) of each cluster
    const float* sqnorm;         // [n] (Euclidean) or NULL
    const float* pt_scale;       // [n] step size of each point's code (column-wise quantization) or NULL
    const float* pt_first;       // [n] unquantized first row of B_c (mixed-precision decomposition) or NULL
    const float* rho0;           // [npairs] bucket order: unquantized first component of each pair's r, or NULL
    uint32_t* pmax;              // out: [npairs] order-preserving key of the pair's best score (0 on entry)
    uint32_t* cmax;              // out: best score of every 64-point chunk of every pair's cluster (float epilogue:
                                 //      order-preserving key; else the int32 accumulator), or NULL.  The row of pair p
                                 //      starts at entry cm_off[p] (a multiple of 8; ~0u: the pair has no row) and is
                                 //      written in groups of eight chunks (entries past the cluster's last chunk, up
                                 //      to the next multiple of four, receive unspecified values)
    const uint32_t* cm_off;      // [npairs] bucket order
    int L;
    int chunk_tiles;             // 32-point tiles per work item (even)
    // verification only (DUMP instantiations): every int32 accumulator of the matrix-core product is written to
    // y[y_off[slot_of_pos[pair]] + point]
    const int32_t* slot_of_pos;  // [npairs] bucket position -> slot (query * w + rank)
    const int64_t* y_off;        // [npairs + 1] offsets of the slots into y
    int32_t* y;
};

// Row (within the 32-row tile) of result register v for lane half h.
__device__ __forceinline__ int tile_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// Orders this wavefront's LDS writes before its later LDS reads (the buffers are private to the wavefront).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// grid = any (persistent: wavefronts stride over the work items), block = 64 * WPB (independent wavefronts).
// A work item = one cluster, up to 32*NZ of its pairs, up to chunk_tiles 32-point tiles of its codes; items of
// bounded size keep the load balanced when cluster sizes and pair counts are skewed.
// NZ pair tiles per item, KS = r_pad / 32 k-steps, L2 = Euclidean score epilogue (per-point bias, float domain;
// inner product and cosine compare integer accumulators, sigma >= 0 being constant per pair).  COLS = column-wise
// quantization: every point has its own step size, so the maxima are taken over float scores for every metric.
// MIX (with COLS; Sec. 4.2 mixed-precision decomposition): score = fma(rho0', pt_first[t], score of the quantized
// rest), rho0' = rho0 of the pair (twice that for Euclidean).
// TB = point tiles fetched ahead (double buffered in registers; even: tiles are taken in pairs = chunks).
// STREAM = false: items as above.  STREAM = true (few pairs per cluster: the kernel is a pure stream of the
// codes from HBM): one wavefront per cluster takes all of its points, no search for the item's cluster, deeper
// fetch-ahead; clusters without pairs cost nothing.
// DUMP = true (verification): additionally stores every accumulator, so that a test can compare the matrix-core
// product itself, element by element, with a reference.
template <int NZ, int KS, bool L2, int TB, bool STREAM, int WPB, bool COLS = false, bool MIX = false, bool DUMP = false>
__global__ __launch_bounds__(64 * WPB) void k_pair_max(ScoreArgs a) {
    static_assert(!MIX || COLS, "the mixed-precision decomposition builds on the column-wise step sizes");
    static_assert(TB % 2 == 0, "tiles are taken in pairs");
    constexpr bool FLT = L2 || COLS;   // float-domain epilogue
    constexpr int NP = 32 * NZ;        // pairs per item
    constexpr int RP = KS * 32;
    constexpr int IMIN = (int)0x80000000;
    constexpr int NPT = (L2 ? 1 : 0) + (COLS ? 1 : 0) + (MIX ? 1 : 0);   // per-point floats of the float epilogue
    constexpr int NPT1 = NPT > 0 ? NPT : 1;
    // per-point values of the current chunk (bias, step size, first-row value), two buffers by chunk parity
    __shared__ __align__(16) float s_pt[WPB][2][NPT1][kScoreChunk];
    // chunk maxima of the wavefront's pairs, eight chunks per pair and separately for the sixteen rows each lane
    // half holds; joined and written out as 32 contiguous bytes per pair when eight chunks are gathered
    __shared__ uint32_t s_ck[WPB][8][2][NP];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int j = lane & 31, h = lane >> 5;
    // no block-wide barrier below: the wavefronts of a block are independent

    // pairs [pb, min(pb + NP, pend)) against rows [row0, row0 + m_c); row0 is point pt0 of its cluster (a multiple of 64)
    auto process = [&](int pb, int pend, int64_t row0, int m_c, int pt0) {
        i32x4 zreg[NZ][KS];
        float sg[NZ], r0p[NZ];          // the lane's pair: sigma' (float epilogue) and rho0' (MIX)
        int64_t yo[NZ];                 // DUMP: where the lane's pair stores its accumulators
#pragma unroll
        for (int z = 0; z < NZ; ++z) {
            const int gp = pb + 32 * z + j;
            const int gpc = min(gp, pend - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                zreg[z][ks] = load16(a.Z + (size_t)gpc * RP + 32 * ks + 16 * h);
                if (gp >= pend) zreg[z][ks] = (i32x4){0, 0, 0, 0};
            }
            sg[z] = FLT ? (L2 ? 2.0f : 1.0f) * a.sigma[gpc] : 0.0f;
            r0p[z] = 0.0f;
            if (MIX) r0p[z] = (L2 ? 2.0f : 1.0f) * a.rho0[gpc];
            yo[z] = 0;
            if (DUMP) yo[z] = a.y_off[a.slot_of_pos[gpc]] + pt0;
        }
        int pmi[NZ];                    // running best of the pair over the item
        float pmf[NZ];
#pragma unroll
        for (int z = 0; z < NZ; ++z) { pmi[z] = IMIN; pmf[z] = -INFINITY; }

        const int ntiles = (m_c + 31) >> 5;
        const int nchunks = (ntiles + TB - 1) / TB;
        // Whole tiles are requested under a uniform guard with addresses that are affine in the tile number: the
        // lanes of the cluster's last tile that lie past its end read the rows that follow (the allocation is
        // padded by 32 rows) and their results are masked out of the maxima below.
        const int8_t* bbase = a.Bp + (size_t)(row0 + j) * RP + 16 * h;
        // per-point floats: lane l of a tile pair (u, u+1) holds those of point 32 u + l
        auto fetch_chunk = [&](int t0, i32x4 (*dst)[KS], float (*npt)[NPT1]) {
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                if (t0 + u < ntiles) {                   // uniform
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const int8_t* cp = bbase + (size_t)(t0 + u) * (32 * RP) + 32 * ks;
                        // STREAM: one wavefront reads the whole cluster exactly once - streaming (non-temporal) loads keep
                        // the codes out of the caches (measured 68 -> 56 us at 10M points, batch 1024)
                        dst[u][ks] = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(cp)) : load16(cp);
                    }
                } else {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) dst[u][ks] = (i32x4){0, 0, 0, 0};
                }
            }
            if (NPT > 0) {
#pragma unroll
                for (int u = 0; u < TB; u += 2) {
                    const int64_t prow = row0 + min(32 * (t0 + u) + lane, m_c - 1);
                    int f = 0;
                    if (L2) npt[u / 2][f++] = a.sqnorm[prow];
                    if (COLS) npt[u / 2][f++] = a.pt_scale[prow];
                    if (MIX) npt[u / 2][f++] = a.pt_first[prow];
                }
            }
        };
        auto score_chunk = [&](int c0, i32x4 (*breg)[KS], float (*npt)[NPT1]) {
            // Two tiles (one chunk of 64 points) at a time, so that ONE three-operand maximum takes in two scores
            // (the epilogue is bound by the vector ALU: a plain maximum costs one instruction per score).
#pragma unroll
            for (int u = 0; u < TB; u += 2) {
                const int t = c0 * TB + u;
                if (t < ntiles) {                        // uniform
                    const bool full = 32 * t + 64 <= m_c;                          // uniform: both tiles complete
                    const int buf = (t >> 1) & 1;
                    float bias_a[16], bias_b[16], ns_a[16], ns_b[16], nf_a[16], nf_b[16];
                    if (NPT > 0) {
                        // the chunk's per-point values go through LDS: register v needs those of rows tile_row(v, h)
#pragma unroll
                        for (int f = 0; f < NPT; ++f) s_pt[wv][buf][f][lane] = npt[u / 2][f];
                        wave_lds_sync();
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int ra = 8 * g + 4 * h;
                            auto rd = [&](int f, float* da, float* db) {
                                const float4 va = *reinterpret_cast<const float4*>(&s_pt[wv][buf][f][ra]);
                                const float4 vb = *reinterpret_cast<const float4*>(&s_pt[wv][buf][f][32 + ra]);
                                da[4 * g] = va.x; da[4 * g + 1] = va.y; da[4 * g + 2] = va.z; da[4 * g + 3] = va.w;
                                db[4 * g] = vb.x; db[4 * g + 1] = vb.y; db[4 * g + 2] = vb.z; db[4 * g + 3] = vb.w;
                            };
                            int f = 0;
                            if (L2) rd(f++, bias_a, bias_b);
                            if (COLS) rd(f++, ns_a, ns_b);
                            if (MIX) rd(f++, nf_a, nf_b);
                        }
                    }
#pragma unroll
                    for (int z = 0; z < NZ; ++z) {
                        i32x16 acc_a = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc_b = acc_a;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) {
                            acc_a = __builtin_amdgcn_mfma_i32_32x32x32_i8(breg[u][ks], zreg[z][ks], acc_a, 0, 0, 0);
                            acc_b = __builtin_amdgcn_mfma_i32_32x32x32_i8(breg[u + 1][ks], zreg[z][ks], acc_b, 0, 0, 0);
                        }
                        const bool pair_ok = pb + 32 * z + j < pend;
                        if (DUMP) {
                            if (pair_ok) {
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const int pa = 32 * t + tile_row(v, h);
                                    if (pa < m_c) a.y[yo[z] + pa] = acc_a[v];
                                    if (pa + 32 < m_c) a.y[yo[z] + pa + 32] = acc_b[v];
                                }
                            }
                        }
                        uint32_t ckey;          // what the chunk stores: float key, or the integer maximum (of this lane half's rows)
                        if (!FLT) {
                            int cm0 = IMIN, cm1 = IMIN;         // two chains: the maxima do not wait for each other
                            if (full) {
#pragma unroll
                                for (int v = 0; v < 16; v += 2) {
                                    cm0 = max(max(cm0, acc_a[v]), acc_b[v]);
                                    cm1 = max(max(cm1, acc_a[v + 1]), acc_b[v + 1]);
                                }
                            } else {
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const int pa = 32 * t + tile_row(v, h);
                                    cm0 = max(max(cm0, pa < m_c ? acc_a[v] : IMIN), pa + 32 < m_c ? acc_b[v] : IMIN);
                                }
                            }
                            const int cm = max(cm0, cm1);
                            pmi[z] = max(pmi[z], cm);
                            ckey = (uint32_t)cm;
                        } else {
                            float cm0 = -INFINITY, cm1 = -INFINITY;
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const float mult_a = COLS ? __fmul_rn(sg[z], ns_a[v]) : sg[z];
                                const float mult_b = COLS ? __fmul_rn(sg[z], ns_b[v]) : sg[z];
                                float sc_a = __fmaf_rn((float)acc_a[v], mult_a, L2 ? -bias_a[v] : -0.0f);
                                float sc_b = __fmaf_rn((float)acc_b[v], mult_b, L2 ? -bias_b[v] : -0.0f);
                                if (MIX) {
                                    sc_a = __fmaf_rn(r0p[z], nf_a[v], sc_a);
                                    sc_b = __fmaf_rn(r0p[z], nf_b[v], sc_b);
                                }
                                if (!full) {
                                    const int pa = 32 * t + tile_row(v, h);
                                    sc_a = pa < m_c ? sc_a : -INFINITY;
                                    sc_b = pa + 32 < m_c ? sc_b : -INFINITY;
                                }
                                if (v & 1) cm1 = fmaxf(fmaxf(cm1, sc_a), sc_b); else cm0 = fmaxf(fmaxf(cm0, sc_a), sc_b);
                            }
                            const float cm = fmaxf(cm0, cm1);
                            pmf[z] = fmaxf(pmf[z], cm);
                            ckey = float_key_asc(cm);
                        }
                        s_ck[wv][(t >> 1) & 7][h][32 * z + j] = ckey;
                    }
                    // eight chunks gathered (or the range ends): every pair's eight maxima leave as two 16-byte stores
                    if (a.cmax != nullptr && (((t >> 1) & 7) == 7 || t + 2 >= ntiles)) {          // uniform
                        wave_lds_sync();
                        const int p = lane & (NP - 1);                                   // NP = 32: the halves share a pair, one
                        const int half = NP == 32 ? h : 0;                               // store each; NP = 64: one pair per lane
                        const int ch0 = ((pt0 + 32 * t) >> 6) & ~7;
                        const int nvalid = ((pt0 + 32 * t) >> 6) - ch0 + 1;              // chunks of this group that exist
                        const uint32_t row = pb + p < pend ? a.cm_off[pb + p] : ~0u;
                        auto joined = [&](int cc) -> uint32_t {                           // both lane halves' rows of chunk cc
                            const uint32_t x = s_ck[wv][cc][0][p], y = s_ck[wv][cc][1][p];
                            return FLT ? max(x, y) : (uint32_t)max((int)x, (int)y);
                        };
                        if (row != ~0u) {
                            uint32_t* dst = a.cmax + (size_t)row + ch0;
                            if (NP == 32) {
                                if (4 * half < nvalid)
                                    *reinterpret_cast<uint4*>(dst + 4 * half) = make_uint4(joined(4 * half), joined(4 * half + 1), joined(4 * half + 2), joined(4 * half + 3));
                            } else {
                                *reinterpret_cast<uint4*>(dst) = make_uint4(joined(0), joined(1), joined(2), joined(3));
                                if (nvalid > 4) *reinterpret_cast<uint4*>(dst + 4) = make_uint4(joined(4), joined(5), joined(6), joined(7));
                            }
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);       // keep the tile pairs sequential: bounds live accumulators
            }
        };
        {
            i32x4 bnext[TB][KS];
            float nptnext[TB / 2][NPT1];
            if (nchunks > 0) fetch_chunk(0, bnext, nptnext);
            for (int c0 = 0; c0 < nchunks; ++c0) {
                i32x4 breg[TB][KS];
                float npt[TB / 2][NPT1];
#pragma unroll
                for (int u = 0; u < TB; ++u) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) breg[u][ks] = bnext[u][ks];
                }
#pragma unroll
                for (int u = 0; u < TB / 2; ++u)
#pragma unroll
                    for (int f = 0; f < NPT1; ++f) npt[u][f] = nptnext[u][f];
                if (c0 + 1 < nchunks) fetch_chunk((c0 + 1) * TB, bnext, nptnext);
                score_chunk(c0, breg, npt);
            }
        }

        // the pair's best score over this item (other point ranges of the cluster contribute through the atomic)
#pragma unroll
        for (int z = 0; z < NZ; ++z) {                     // the other half holds the other sixteen rows of every tile
            pmi[z] = max(pmi[z], __shfl_xor(pmi[z], 32, 64));
            pmf[z] = fmaxf(pmf[z], __shfl_xor(pmf[z], 32, 64));
        }
        if (h == 0) {
#pragma unroll
            for (int z = 0; z < NZ; ++z) {
                const int gp = pb + 32 * z + j;
                if (gp < pend) {
                    uint32_t key = 0u;       // 0 = no point seen (below the key of every float)
                    if (!FLT) {
                        // sigma >= 0: the best score of the pair is the score of its largest integer score
                        if (pmi[z] != IMIN) key = float_key_asc(__fmaf_rn((float)pmi[z], a.sigma[gp], -0.0f));
                    } else if (pmf[z] != -INFINITY) {
                        key = float_key_asc(pmf[z]);
                    }
                    if (key != 0u) atomicMax(&a.pmax[gp], key);
                }
            }
        }
    };

    if (STREAM) {
        // the cluster number is uniform over the wavefront: say so, and its offsets come through scalar loads
        for (int c = blockIdx.x * WPB + __builtin_amdgcn_readfirstlane(wv); c < a.L; c += gridDim.x * WPB) {
            const int pbeg = a.bucket_off[c], pend = a.bucket_off[c + 1];
            if (pbeg == pend) continue;
            const int64_t row_c = a.off[c];
            const int m_all = (int)(a.off[c + 1] - row_c);
            for (int pb = pbeg; pb < pend; pb += NP) process(pb, pend, row_c, m_all, 0);
        }
    } else {
        const int n_items = a.unit_off[a.L];
        for (int item = blockIdx.x * WPB + wv; item < n_items; item += gridDim.x * WPB) {
            const int c = __builtin_amdgcn_readfirstlane(find_bucket_wave(a.unit_off, a.L, item));   // uniform: scalar loads below
            const int64_t row_c = a.off[c];
            const int m_all = (int)(a.off[c + 1] - row_c);
            const int pbeg = a.bucket_off[c], pend = a.bucket_off[c + 1];
            const int n_groups = (pend - pbeg + NP - 1) / NP;
            const int local = item - a.unit_off[c];
            // consecutive items (the wavefronts of one block) share the point range and differ in the pair group,
            // so the range's codes are fetched from L2 once per block
            const int pk = local / n_groups, ug = local - pk * n_groups;
            process(pbeg + ug * NP, pend, row_c + (int64_t)pk * 32 * a.chunk_tiles,
                    min(32 * a.chunk_tiles, m_all - pk * 32 * a.chunk_tiles), pk * 32 * a.chunk_tiles);
        }
    }
}

}  // namespace lorann
