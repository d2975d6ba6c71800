// Small batches (a few dozen queries, Sec. 4.3's latency-oriented use): the batched path - bucket the (query, cluster)
// pairs by cluster so that each cluster's factors are read once per batch - pays for three counting-sort launches
// and a cluster-major A stage that a handful of queries cannot fill.  With so few queries hardly any two pairs
// share a cluster, so the path stays QUERY-major instead: the block that has just selected a query's w clusters
// goes on to the first 8-bit product and the re-quantization of Sec. 3.3 for those w pairs; pairs keep their slot
// order (slot = query * w + rank) everywhere, and the scoring kernel takes every pair as a cluster of its own.
#pragma once
#include "common.hpp"
#include "select_exact.hpp"

namespace lorann {

struct SmallArgs {
    // inputs
    const int8_t* q8;            // [nq][dp] query codes (written earlier in the same block or by the kernel before)
    const float* dx;             // [nq]
    const int8_t* A;             // [L][r][dp]
    const float* sA;             // [L]
    const float* sB;             // [L]
    const int64_t* off;          // [L+1]
    int r, r_pad;
    // outputs, all in slot order
    int8_t* Z;                   // [nq*w][r_pad]   NULL: the small-batch tail is off
    float* sigma;                // [nq*w]
    uint32_t* pmax;              // [nq*w] cleared
    int32_t* pos_of_slot;        // [nq*w] identity
    int32_t* slot_of_pos;        // [nq*w] identity
    int64_t* voff;               // [nq*w][2] first row and end row of the pair's cluster
    int32_t* qorder;             // [nq] identity
};

// The whole block (256 threads) serves query q whose w selected clusters are sel[0..w): wavefront wv takes pairs wv,
// wv + 4, ...; lane j < r computes R_j = sum_i q8[i] A_c[j][i] (A_c[j] is d' contiguous bytes), then the pair is
// re-quantized exactly as the cluster-major kernel does: M = max_j |R_j|, z_j = sign(R_j) floor((254 |R_j| + M) / (2 M)),
// sigma = M / 127 * dx * DeltaA_c * DeltaB_c in double, left to right, one rounding to float.
// q8s: LDS, d' bytes (16-byte aligned).  Contains one block barrier.
__device__ __forceinline__ void small_stage_a_block(const SmallArgs& s, int q, const int32_t* __restrict__ sel, int w, int dp,
                                                    int8_t* q8s) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    for (int i = tid; i < dp / 4; i += 256) reinterpret_cast<int*>(q8s)[i] = reinterpret_cast<const int*>(s.q8 + (size_t)q * dp)[i];
    if (tid == 0) s.qorder[q] = q;
    __syncthreads();
    const float dxq = s.dx[q];
    const int r = s.r, r_pad = s.r_pad;
    const int jc = min(lane, r - 1);
    for (int j = wv; j < w; j += 4) {
        const int c = sel[j];
        const int8_t* arow = s.A + ((size_t)c * r + jc) * dp;
        int acc = 0;
        for (int i0 = 0; i0 < dp; i0 += 64) {                    // four 16-byte pieces at a time (d' is a multiple of 16)
            i32x4 av[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) av[u] = *reinterpret_cast<const i32x4*>(arow + min(i0 + 16 * u, dp - 16));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (i0 + 16 * u < dp) {                          // uniform
                    const i32x4 qv = *reinterpret_cast<const i32x4*>(q8s + i0 + 16 * u);
                    acc = dot4_i8(av[u][0], qv[0], acc); acc = dot4_i8(av[u][1], qv[1], acc);
                    acc = dot4_i8(av[u][2], qv[2], acc); acc = dot4_i8(av[u][3], qv[3], acc);
                }
            }
        }
        const int R = lane < r ? acc : 0;
        uint32_t mx = (uint32_t)abs(R);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
        const size_t slot = (size_t)q * w + j;
        int zc = 0;
        if (mx != 0u && lane < r) {
            const uint32_t a = (uint32_t)abs(R);
            const uint32_t qq = (254u * a + mx) / (2u * mx);     // < 2^32 because d' <= 1024
            zc = R < 0 ? -(int)qq : (int)qq;
        }
        if (lane < r_pad) s.Z[slot * r_pad + lane] = (int8_t)zc;
        if (lane == 0) {
            float sg = 0.0f;
            if (mx != 0u) sg = (float)((double)mx / 127.0 * (double)dxq * (double)s.sA[c] * (double)s.sB[c]);
            s.sigma[slot] = sg;
            s.pmax[slot] = 0u;
            s.pos_of_slot[slot] = (int32_t)slot;
            s.slot_of_pos[slot] = (int32_t)slot;
            s.voff[2 * slot] = s.off[c];
            s.voff[2 * slot + 1] = s.off[c + 1];
        }
    }
}

}  // namespace lorann
