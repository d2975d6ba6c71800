// Second 8-bit product on the int8 matrix cores, organised by CLUSTER (Sec. 3.2-3.3; batching per cluster
// replaces the per-(query, cluster) gathers of the paper's GPU design, Sec. 4.3): the (query, cluster) pairs
// were bucketed by cluster, so a wavefront takes one cluster, up to 32*NZ of its pairs and a chunk of its
// codes B_c, and contracts each 32-point tile against the pairs with
// v_mfma_i32_32x32x32_i8:   Y[pair][point] = sum_t z[pair][t] * code[point][t]   (int32, exact).
//
// Register layout of that instruction (measured on gfx950): both operands give lane l sixteen consecutive
// k-bytes (k-half l/32) of row / column l%32; result register v of lane l holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32].  With pairs as rows and points as columns, lane l owns ONE point of the
// tile and register v belongs to ONE pair (per lane half).
//
// Exact top-m without materialising the scores: this kernel only computes, for every pair, the MAXIMUM score
// over the cluster's points - one integer max per MFMA result register, no per-score branch.  The per-query
// kernel (select_query.hpp) then needs to score point by point only the very few clusters of a query whose
// maximum reaches its running m-th best score; every other pair is dismissed by its maximum alone.
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
    const int32_t* unit_off;     // [L+1] work items (pair group x point chunk) of each cluster
    const float* sqnorm;         // [n] (Euclidean) or NULL
    const float* pt_scale;       // [n] step size of each point's code (column-wise quantization) or NULL
    const float* pt_first;       // [n] unquantized first row of B_c (mixed-precision decomposition) or NULL
    const float* rho0;           // [npairs] bucket order: unquantized first component of each pair's r, or NULL
    uint32_t* pmax;              // out: [npairs] order-preserving key of the pair's best score (0 on entry)
    const int64_t* voff;         // small batches (STREAM shape only): [L][2] first and end row of "cluster" c, which
                                 // is then simply pair c (bucket_off is not read: pairs [c, c + 1)); else NULL
    int L;
    int chunk_tiles;             // 32-point tiles per work item
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
// inner product and cosine compare the integer maximum, sigma >= 0 being constant per pair).  COLS = column-wise
// quantization: every point has its own step size, so the maximum is taken over float scores for every metric.
// MIX (with COLS; Sec. 4.2 mixed-precision decomposition): score = fma(rho0', pt_first[t], score of the quantized
// rest), rho0' = rho0 of the pair (twice that for Euclidean).
// TB = point tiles fetched ahead (double buffered in registers).
// STREAM = false: items as above.  STREAM = true (few pairs per cluster: the kernel is a pure stream of the
// codes from HBM): one wavefront per cluster takes all of its points, no search for the item's cluster, deeper
// fetch-ahead; clusters without pairs cost nothing.
// DUMP = true (verification): additionally stores every accumulator, so that a test can compare the matrix-core
// product itself, element by element, with a reference.
template <int NZ, int KS, bool L2, int TB, bool STREAM, int WPB, bool COLS = false, bool MIX = false, bool DUMP = false>
__global__ __launch_bounds__(64 * WPB) void k_pair_max(ScoreArgs a) {
    static_assert(!MIX || COLS, "the mixed-precision decomposition builds on the column-wise step sizes");
    constexpr bool FLT = L2 || COLS;   // float-domain epilogue
    constexpr int NP = 32 * NZ;        // pairs per item
    constexpr int RP = KS * 32;
    constexpr int IMIN = (int)0x80000000;
    constexpr int TRS = NZ * 16 + 1;   // padded row of the transpose buffer
    __shared__ int s_tr[WPB][64 * TRS];
    __shared__ int s_red[WPB][NP];       // per-pair maxima of the item (int, or order-preserving keys for Euclidean)
    __shared__ float s_sig[WPB][NP];     // Euclidean: 2 sigma of each pair
    __shared__ float s_r0[WPB][MIX ? NP : 1];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int j = lane & 31, h = lane >> 5;
    // no block-wide barrier below: the wavefronts of a block are independent

    // pairs [pb, min(pb + NP, pend)) against rows [row0, row0 + m_c); row0 is point pt0 of its cluster
    auto process = [&](int pb, int pend, int64_t row0, int m_c, int pt0) {
        i32x4 zreg[NZ][KS];
#pragma unroll
        for (int z = 0; z < NZ; ++z) {
            const int gp = pb + 32 * z + j;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                zreg[z][ks] = (i32x4){0, 0, 0, 0};
                if (gp < pend) zreg[z][ks] = load16(a.Z + (size_t)gp * RP + 32 * ks + 16 * h);
            }
        }
        float sgv[NZ][16];             // float epilogue only: scale of the pair that register v belongs to
        float r0v[MIX ? NZ : 1][16];   // MIX: (doubled) first component of that pair's r
        if (FLT) {
            wave_lds_sync();
            for (int p = lane; p < NP; p += 64) {
                s_sig[wv][p] = (pb + p < pend) ? (L2 ? 2.0f : 1.0f) * a.sigma[pb + p] : 0.0f;
                if (MIX) s_r0[wv][p] = (pb + p < pend) ? (L2 ? 2.0f : 1.0f) * a.rho0[pb + p] : 0.0f;
            }
            wave_lds_sync();
#pragma unroll
            for (int z = 0; z < NZ; ++z)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    sgv[z][v] = s_sig[wv][32 * z + tile_row(v, h)];
                    if (MIX) r0v[z][v] = s_r0[wv][32 * z + tile_row(v, h)];
                }
        }
        int mxi[NZ][16];
        float mxf[NZ][16];
#pragma unroll
        for (int z = 0; z < NZ; ++z)
#pragma unroll
            for (int v = 0; v < 16; ++v) { mxi[z][v] = IMIN; mxf[z][v] = -INFINITY; }

        const int ntiles = (m_c + 31) >> 5;
        const int nchunks = (ntiles + TB - 1) / TB;
        // Whole tiles are requested under a uniform guard with addresses that are affine in the tile number: the
        // lanes of the cluster's last tile that lie past its end read the rows that follow (the allocation is
        // padded by 32 rows) and are masked out of the maxima below.
        const int8_t* bbase = a.Bp + (size_t)(row0 + j) * RP + 16 * h;
        auto fetch_chunk = [&](int t0, i32x4 (*dst)[KS], float* nb, float* ns, float* nf) {
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
                    if (L2) nb[u] = a.sqnorm[row0 + min(32 * (t0 + u) + j, m_c - 1)];
                    if (COLS) ns[u] = a.pt_scale[row0 + min(32 * (t0 + u) + j, m_c - 1)];
                    if (MIX) nf[u] = a.pt_first[row0 + min(32 * (t0 + u) + j, m_c - 1)];
                } else {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) dst[u][ks] = (i32x4){0, 0, 0, 0};
                    if (L2) nb[u] = 0.0f;
                    if (COLS) ns[u] = 0.0f;
                    if (MIX) nf[u] = 0.0f;
                }
            }
        };
        auto score_chunk = [&](int c0, i32x4 (*breg)[KS], const float* nb, const float* ns, const float* nf) {
            // Two tiles at a time, so that ONE three-operand maximum per result register takes in both tiles (the
            // epilogue is bound by the vector ALU: integer maxima cost one instruction per score otherwise).
            static_assert(TB % 2 == 0, "tiles are taken in pairs");
#pragma unroll
            for (int u = 0; u < TB; u += 2) {
                const int t = c0 * TB + u;
                if (t < ntiles) {                        // uniform
                    const bool has2 = t + 1 < ntiles;                              // uniform
                    const bool full = has2 && 32 * t + 64 <= m_c;                  // uniform: both tiles complete
                    const bool ok_a = 32 * t + j < m_c, ok_b = has2 && 32 * (t + 1) + j < m_c;
                    const float bias_a = L2 ? nb[u] : 0.0f, bias_b = L2 ? nb[u + 1] : 0.0f;
#pragma unroll
                    for (int z = 0; z < NZ; ++z) {
                        i32x16 acc_a = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc_b = acc_a;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) {
                            acc_a = __builtin_amdgcn_mfma_i32_32x32x32_i8(zreg[z][ks], breg[u][ks], acc_a, 0, 0, 0);
                            acc_b = __builtin_amdgcn_mfma_i32_32x32x32_i8(zreg[z][ks], breg[u + 1][ks], acc_b, 0, 0, 0);
                        }
                        if (DUMP) {
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const int gp = pb + 32 * z + tile_row(v, h);
                                if (gp < pend) {
                                    const int64_t yo = a.y_off[a.slot_of_pos[gp]] + pt0;
                                    if (ok_a) a.y[yo + 32 * t + j] = acc_a[v];
                                    if (ok_b) a.y[yo + 32 * (t + 1) + j] = acc_b[v];
                                }
                            }
                        }
                        if (!FLT) {
                            if (full) {
#pragma unroll
                                for (int v = 0; v < 16; ++v) mxi[z][v] = max(max(mxi[z][v], acc_a[v]), acc_b[v]);
                            } else {
#pragma unroll
                                for (int v = 0; v < 16; ++v) mxi[z][v] = max(max(mxi[z][v], ok_a ? acc_a[v] : IMIN), ok_b ? acc_b[v] : IMIN);
                            }
                        } else {
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const float mult_a = COLS ? __fmul_rn(sgv[z][v], ns[u]) : sgv[z][v];
                                const float mult_b = COLS ? __fmul_rn(sgv[z][v], ns[u + 1]) : sgv[z][v];
                                float sc_a = __fmaf_rn((float)acc_a[v], mult_a, -bias_a);
                                float sc_b = __fmaf_rn((float)acc_b[v], mult_b, -bias_b);
                                if (MIX) {
                                    sc_a = __fmaf_rn(r0v[MIX ? z : 0][v], nf[u], sc_a);
                                    sc_b = __fmaf_rn(r0v[MIX ? z : 0][v], nf[u + 1], sc_b);
                                }
                                mxf[z][v] = fmaxf(fmaxf(mxf[z][v], ok_a ? sc_a : -INFINITY), ok_b ? sc_b : -INFINITY);
                            }
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);       // keep the tile pairs sequential: bounds live accumulators
            }
        };
        {
            i32x4 bnext[TB][KS];
            float nbnext[TB], nsnext[TB], nfnext[TB];
            if (nchunks > 0) fetch_chunk(0, bnext, nbnext, nsnext, nfnext);
            for (int c0 = 0; c0 < nchunks; ++c0) {
                i32x4 breg[TB][KS];
                float nb[TB], ns[TB], nf[TB];
#pragma unroll
                for (int u = 0; u < TB; ++u) {
                    nb[u] = nbnext[u]; ns[u] = nsnext[u]; nf[u] = nfnext[u];
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) breg[u][ks] = bnext[u][ks];
                }
                if (c0 + 1 < nchunks) fetch_chunk((c0 + 1) * TB, bnext, nbnext, nsnext, nfnext);
                score_chunk(c0, breg, nb, ns, nf);
            }
        }

        // reduce over the 32 points held by the lanes of each half through an LDS transpose: every lane stores its
        // NZ*16 running maxima as one padded row, then lane p gathers the column of pair p from the 32 lanes of
        // the half that holds it (independent reads, one wait) instead of 5 dependent shuffles per register
        wave_lds_sync();
#pragma unroll
        for (int z = 0; z < NZ; ++z)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                s_tr[wv][lane * TRS + z * 16 + v] = FLT ? (int)float_key_asc(mxf[z][v]) : mxi[z][v];
        wave_lds_sync();
        for (int p = lane; p < NP; p += 64) {
            const int z = p >> 5, i = p & 31;
            const int hh = (i >> 2) & 1, v = 4 * (i >> 3) + (i & 3);        // inverse of tile_row
            const int* col = &s_tr[wv][hh * 32 * TRS + z * 16 + v];
            if (!FLT) {
                int r = IMIN;
#pragma unroll
                for (int jj = 0; jj < 32; ++jj) r = max(r, col[jj * TRS]);
                s_red[wv][p] = r;
            } else {
                unsigned r = 0u;
#pragma unroll
                for (int jj = 0; jj < 32; ++jj) r = max(r, (unsigned)col[jj * TRS]);
                s_red[wv][p] = (int)r;
            }
        }
        wave_lds_sync();
        for (int p = lane; p < NP; p += 64) {
            const int gp = pb + p;
            if (gp < pend) {
                uint32_t key = 0u;       // 0 = no point seen (below the key of every float)
                if (!FLT) {
                    const int y = s_red[wv][p];
                    // sigma >= 0: the best score of the pair is the score of its largest integer score
                    if (y != IMIN) key = float_key_asc(__fmaf_rn((float)y, a.sigma[gp], -0.0f));
                } else {
                    key = (uint32_t)s_red[wv][p];
                    if (key == float_key_asc(-INFINITY)) key = 0u;      // no point of the chunk seen
                }
                if (key != 0u) atomicMax(&a.pmax[gp], key);      // the cluster's other point chunks contribute too
            }
        }
    };

    if (STREAM) {
        // the cluster number is uniform over the wavefront: say so, and its offsets come through scalar loads
        for (int c = blockIdx.x * WPB + __builtin_amdgcn_readfirstlane(wv); c < a.L; c += gridDim.x * WPB) {
            const int pbeg = a.voff ? c : a.bucket_off[c], pend = a.voff ? c + 1 : a.bucket_off[c + 1];
            if (pbeg == pend) continue;
            const int64_t row_c = a.voff ? a.voff[2 * c] : a.off[c];
            const int m_all = (int)((a.voff ? a.voff[2 * c + 1] : a.off[c + 1]) - row_c);
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
            // consecutive items (the wavefronts of one block) share the point chunk and differ in the pair group,
            // so the chunk's codes are fetched from L2 once per block
            const int pk = local / n_groups, ug = local - pk * n_groups;
            process(pbeg + ug * NP, pend, row_c + (int64_t)pk * 32 * a.chunk_tiles,
                    min(32 * a.chunk_tiles, m_all - pk * 32 * a.chunk_tiles), pk * 32 * a.chunk_tiles);
        }
    }
}

}  // namespace lorann
