// Small batches (a few dozen queries, Sec. 4.3's latency-oriented use): the batched path - bucket the (query, cluster)
// pairs by cluster so that each cluster's factors are read once per batch - pays for three counting-sort launches
// and a cluster-major A stage that a handful of queries cannot fill.  With so few queries hardly any two pairs
// share a cluster, so the path stays QUERY-major instead: one launch does the first 8-bit product and the
// re-quantization of Sec. 3.3 pair by pair (all rows of all A_c in flight at once - at this size the step is pure
// memory latency); pairs keep their slot order (slot = query * w + rank) everywhere, and the scoring kernel takes
// every pair as a cluster of its own.
#pragma once
#include "common.hpp"
#include "select_exact.hpp"

namespace lorann {

struct SmallArgs {
    // inputs
    const int8_t* q8;            // [nq][dp] query codes
    const float* dx;             // [nq]
    const int8_t* A;             // [L][r][dp]
    const float* sA;             // [L]
    const float* sB;             // [L]
    const int64_t* off;          // [L+1]
    int r, r_pad;
    // outputs, all in slot order
    int8_t* Z;                   // [nq*w][r_pad]
    float* sigma;                // [nq*w]
    uint32_t* pmax;              // [nq*w] cleared
    int32_t* pos_of_slot;        // [nq*w] identity
    int32_t* slot_of_pos;        // [nq*w] identity
    int64_t* voff;               // [nq*w][2] first row and end row of the pair's cluster
    int32_t* qorder;             // [nq] identity
    int32_t* done;               // [nq] cleared here: tickets of the query's re-rank blocks
};

// grid = ceil(npairs / (4 * ppw)), block = 256; ppw = pairs per wavefront: 2 when r_pad <= 32 (lanes 0..31 the columns
// of one pair, lanes 32..63 those of the other), else 1 (lane = column).  Pair p = slot = query * w + rank: lane j
// computes R_j = sum_i q8[i] A_c[j][i] (A_c[j] is d' contiguous bytes; all pieces of a row are requested at once), then
// the pair is re-quantized exactly as the cluster-major kernel does: M = max_j |R_j|,
// z_j = sign(R_j) floor((254 |R_j| + M) / (2 M)), sigma = M / 127 * dx * DeltaA_c * DeltaB_c in double, left to right,
// one rounding to float.
__global__ __launch_bounds__(256) void k_small_stage_a(SmallArgs s, const int32_t* __restrict__ sel, int nq, int w, int dp) {
    const int lane = threadIdx.x & 63;
    const int r = s.r, r_pad = s.r_pad;
    const int ppw = r_pad <= 32 ? 2 : 1;
    const int width = 64 / ppw;
    const int sub = lane / width, col = lane - sub * width;
    const int npairs = nq * w;
    const int p = ((int)blockIdx.x * 4 + (int)(threadIdx.x >> 6)) * ppw + sub;
    if ((p - sub) >= npairs) return;                             // whole wavefront beyond the end (no block barrier below)
    const bool pair_ok = p < npairs;
    const int pc = min(p, npairs - 1);
    const int q = pc / w;
    const int c = sel[pc];
    const int jc = min(col, r - 1);
    const int8_t* arow = s.A + ((size_t)c * r + jc) * dp;
    const int8_t* qrow = s.q8 + (size_t)q * dp;
    const int pieces = dp >> 4;                                  // 16-byte pieces of a row (d' is a multiple of 16)
    int acc = 0;
    for (int p0 = 0; p0 < pieces; p0 += 16) {                    // sixteen pieces in flight (all of d' <= 256 at once)
        i32x4 av[16], qv[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            av[u] = *reinterpret_cast<const i32x4*>(arow + 16 * min(p0 + u, pieces - 1));
            qv[u] = *reinterpret_cast<const i32x4*>(qrow + 16 * min(p0 + u, pieces - 1));
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (p0 + u < pieces) {                               // uniform
                acc = dot4_i8(av[u][0], qv[u][0], acc); acc = dot4_i8(av[u][1], qv[u][1], acc);
                acc = dot4_i8(av[u][2], qv[u][2], acc); acc = dot4_i8(av[u][3], qv[u][3], acc);
            }
        }
    }
    const int R = col < r ? acc : 0;
    uint32_t mx = (uint32_t)abs(R);
    for (int o = width >> 1; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));     // within the pair's lanes
    int zc = 0;
    if (mx != 0u && col < r) {
        const uint32_t a = (uint32_t)abs(R);
        const uint32_t qq = (254u * a + mx) / (2u * mx);         // < 2^32 because d' <= 1024
        zc = R < 0 ? -(int)qq : (int)qq;
    }
    if (pair_ok && col < r_pad) s.Z[(size_t)p * r_pad + col] = (int8_t)zc;
    if (pair_ok && col == 0) {
        float sg = 0.0f;
        if (mx != 0u) sg = (float)((double)mx / 127.0 * (double)s.dx[q] * (double)s.sA[c] * (double)s.sB[c]);
        s.sigma[p] = sg;
        s.pmax[p] = 0u;
        s.pos_of_slot[p] = p;
        s.slot_of_pos[p] = p;
        s.voff[2 * (size_t)p] = s.off[c];
        s.voff[2 * (size_t)p + 1] = s.off[c + 1];
        if (p % w == 0) { s.qorder[q] = q; s.done[q] = 0; }
    }
}

}  // namespace lorann
