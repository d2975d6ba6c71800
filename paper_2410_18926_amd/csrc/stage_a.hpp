// First 8-bit product and re-quantization (Sec. 3.3): for every (query, cluster) pair,
// R = q'_i8^T A_c in int32, z = round(127 R / max|R|) as int8, and the pair's combined scale
// sigma = max|R|/127 * Delta_x * DeltaA_c * DeltaB_c.  With one scalar DeltaA per cluster the
// de-quantize / re-quantize pair of Sec. 3.3 reduces to this integer expression.
//
// Pairs are grouped by cluster (counting sort), so one wavefront handles 16 pairs of the same cluster as an
// int8 matrix-core product  [16 pairs x d'] . [d' x r]  with v_mfma_i32_16x16x64_i8.
// Register layout of that instruction (measured on gfx950): both operands give lane l sixteen consecutive
// k-bytes of row/column l%16 (k-group l/16); result register v of lane l holds D[4*(l/16) + v][l%16].
#pragma once
#include "common.hpp"

namespace lorann {

__device__ __forceinline__ i32x4 load16(const int8_t* p) { return *reinterpret_cast<const i32x4*>(p); }

// Find c with off[c] <= t < off[c+1] (off non-decreasing, off[0] = 0, t < off[L]).
__device__ __forceinline__ int find_bucket(const int32_t* __restrict__ off, int L, int t) {
    int lo = 0, hi = L;   // invariant: off[lo] <= t < off[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// The same search done by a whole wavefront for one (uniform) t: every round the 64 lanes probe 64 evenly
// spaced entries of the current range, so the range shrinks 64-fold per dependent load instead of 2-fold.
__device__ __forceinline__ int find_bucket_wave(const int32_t* __restrict__ off, int L, int t) {
    const int lane = threadIdx.x & 63;
    int lo = 0, hi = L;   // invariant: off[lo] <= t < off[hi]
    while (hi - lo > 1) {
        const int span = hi - lo;
        const int step = (span + 63) >> 6;                 // >= 1
        const int probe = lo + (lane + 1) * step;          // lo < probe; lanes beyond hi do not count
        const bool le = probe < hi && off[probe] <= t;
        const int n = __popcll(__ballot(le));              // off is non-decreasing: the first n probes are <= t
        const int nlo = lo + n * step;
        const int nhi = min(hi, nlo + step);
        lo = nlo; hi = nhi;
    }
    return lo;
}

// grid = ceil(max_tiles / 4), block = 256 (one 16-pair tile per wavefront).
// RT = r_pad / 16 result tiles (2 or 4).  A is [L][r][dp]; Z is [npairs][r_pad] in bucket order.
template <int RT>
__global__ __launch_bounds__(256) void k_stage_a(const int8_t* __restrict__ q8, const float* __restrict__ dx,
                                                  const int8_t* __restrict__ A, const float* __restrict__ sA,
                                                  const float* __restrict__ sB, const int32_t* __restrict__ bucket_off,
                                                  const int32_t* __restrict__ tile_off, const int32_t* __restrict__ slot_of_pos,
                                                  int L, int dp, int r, int w, int8_t* __restrict__ Z, float* __restrict__ sigma) {
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= tile_off[L]) return;
    const int c = __builtin_amdgcn_readfirstlane(find_bucket_wave(tile_off, L, tile));   // uniform: scalar loads below
    const int base = bucket_off[c] + (tile - tile_off[c]) * 16;
    const int end = bucket_off[c + 1];
    const int i = lane & 15, g = lane >> 4;

    const bool row_ok = base + i < end;
    const int8_t* qrow = q8;
    if (row_ok) qrow = q8 + (size_t)(slot_of_pos[base + i] / w) * dp;
    const int8_t* Ac = A + (size_t)c * r * dp;

    i32x4 acc[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) acc[t] = (i32x4){0, 0, 0, 0};

    // The operands of SB k-steps are requested together, with clamped addresses instead of branches around the
    // loads (so that they overlap), and what lies outside the matrices is zeroed in registers afterwards.
    constexpr int SB = 4;
    const int steps = (dp + 63) >> 6;                    // uniform trip count: the MFMA runs with all lanes on
    for (int s0 = 0; s0 < steps; s0 += SB) {
        i32x4 av[SB], bv[SB][RT];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const int kc = min(64 * (s0 + u) + 16 * g, dp - 16);
            av[u] = load16(qrow + kc);
#pragma unroll
            for (int t = 0; t < RT; ++t) bv[u][t] = load16(Ac + (size_t)min(t * 16 + i, r - 1) * dp + kc);
        }
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (s0 + u < steps) {                        // uniform
                // d' is a multiple of 16: a 16-byte group is all in or all out
                const bool a_ok = row_ok && 64 * (s0 + u) + 16 * g < dp;
                const i32x4 a = a_ok ? av[u] : (i32x4){0, 0, 0, 0};
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    const i32x4 b = t * 16 + i < r ? bv[u][t] : (i32x4){0, 0, 0, 0};
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[t], 0, 0, 0);
                }
            }
        }
    }

    // acc[t][v] = R[pair 4g+v][column 16t+i].  Row maximum over the r columns: over t here, over i by shuffles.
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        uint32_t mx = 0;
#pragma unroll
        for (int t = 0; t < RT; ++t) mx = max(mx, (uint32_t)abs(acc[t][v]));
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
        const int pos = base + 4 * g + v;
        if (pos < end) {
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                int zc = 0;
                if (mx != 0u) {
                    const int R = acc[t][v];
                    const uint32_t a = (uint32_t)abs(R);
                    const uint32_t q = (254u * a + mx) / (2u * mx);   // < 2^32 because d' <= 1024
                    zc = R < 0 ? -(int)q : (int)q;
                }
                Z[(size_t)pos * (RT * 16) + t * 16 + i] = (int8_t)zc;
            }
            if (i == 0) {
                float s = 0.0f;
                if (mx != 0u) {
                    const int qi = slot_of_pos[pos] / w;
                    s = (float)((double)mx / 127.0 * (double)dx[qi] * (double)sA[c] * (double)sB[c]);
                }
                sigma[pos] = s;
            }
        }
    }
}

}  // namespace lorann
