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

// The same search started from a guess: if t lies within the 63 buckets from c_guess - 31 on, ONE round of probes
// finds it (buckets of similar size make an interpolated guess land that close); otherwise the full search runs.
__device__ __forceinline__ int find_bucket_near(const int32_t* __restrict__ off, int L, int t, int c_guess) {
    const int lane = threadIdx.x & 63;
    const int lo = max(0, min(c_guess - 31, L - 63));
    const int probe = min(lo + lane, L);
    const int n = __popcll(__ballot(off[probe] <= t));     // off is non-decreasing: the first n probes are <= t
    if (n >= 1 && n <= 63 && lo + n <= L) return lo + n - 1;     // off[lo + n - 1] <= t < off[lo + n]
    return find_bucket_wave(off, L, t);
}

// grid = ceil((npairs / 16 + L) / (4 * tpw)) blocks of 256: the 16-pair tiles of all clusters form one list
// (tile_off: tiles before each cluster) and every wavefront takes tpw consecutive tiles of it, so the work per
// wavefront is the same however unevenly the pairs are spread over the clusters; a wavefront whose tiles span
// several clusters serves them one after the other.  A_c stays in registers across the tiles of one cluster when
// d' <= 256.
// RT = r_pad / 16 result tiles (2 or 4); RES: d' <= 256, A_c resident.  A is [L][r][dp]; Z is [npairs][r_pad] in
// bucket order.
// COLS: column-wise quantization (Sec. 3.3 as printed) - sA is [L][r], one step size per column of A_c; the float
// approximation rho_j = R_j * (Delta_x * DeltaA_cj) is re-quantized like a query: z = rint(rho * 127 / |rho|_inf),
// sigma = |rho|_inf / 127 (every operation a single IEEE float operation); sB is not used.
// COLS with A_first != NULL (Sec. 4.2 mixed-precision decomposition; the queries' codes then have 0 in component
// 0): rho_j = fma(x_0, A_first[c][j], R_j * (Delta_x * DeltaA_cj)) with x_0 = qproj[query][0]; rho_0 goes to
// rho0[pair] as it is, z_0 = 0, and the maximum and the codes come from rho_1.. alone.
template <int RT, bool RES, bool COLS = false>
__global__ __launch_bounds__(256) void k_stage_a(const int8_t* __restrict__ q8, const float* __restrict__ dx,
                                                  const int8_t* __restrict__ A, const float* __restrict__ sA,
                                                  const float* __restrict__ sB, const int32_t* __restrict__ bucket_off,
                                                  const int32_t* __restrict__ tile_off, int tpw, int tiles_guess,
                                                  const int32_t* __restrict__ slot_of_pos,
                                                  int L, int dp, int r, int w, int8_t* __restrict__ Z, float* __restrict__ sigma,
                                                  const float* __restrict__ qproj = nullptr, const float* __restrict__ A_first = nullptr,
                                                  float* __restrict__ rho0 = nullptr) {
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, g = lane >> 4;
    // this wavefront's tiles [g0, g1) of the list of all tiles; wavefronts are independent: no block barrier below
    const int gw = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int g0 = gw * tpw;
    const int g1 = min(g0 + tpw, tile_off[L]);
    if (g0 >= g1) return;
    // (tiles_guess: about how many tiles there are, for the first guess of the cluster that holds tile g0)
    int c = __builtin_amdgcn_readfirstlane(find_bucket_near(tile_off, L, g0, (int)((long long)g0 * L / max(1, tiles_guess))));
    for (; g0 < g1; ++c) {                                // clusters this wavefront's tiles belong to
    const int t_beg = tile_off[c], t_end = c + 1 < L ? tile_off[c + 1] : tile_off[L];
    if (t_end <= g0) continue;                            // (a cluster without pairs)
    const int first = g0 - t_beg, last = min(g1, t_end) - t_beg;      // its tiles [first, last) are ours
    g0 = t_beg + last;
    const int pbeg = bucket_off[c], end = bucket_off[c + 1];
    const int8_t* Ac = A + (size_t)c * r * dp;
    constexpr int SB = 4;                                // k-steps whose operands are requested together
    const int steps = (dp + 63) >> 6;                    // uniform trip count: the MFMA runs with all lanes on
    constexpr bool a_resident = RES;                     // requires steps <= SB
    const i32x4 zero4 = (i32x4){0, 0, 0, 0};

    // Operands are requested with clamped addresses instead of branches around the loads (so that they overlap)
    // and what lies outside the matrices is zeroed in registers afterwards.
    auto fetch_a = [&](int s0, i32x4 (&bv)[SB][RT]) {
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const int kc = min(64 * (s0 + u) + 16 * g, dp - 16);
#pragma unroll
            for (int t = 0; t < RT; ++t) bv[u][t] = load16(Ac + (size_t)min(t * 16 + i, r - 1) * dp + kc);
        }
#pragma unroll
        for (int u = 0; u < SB; ++u)
#pragma unroll
            for (int t = 0; t < RT; ++t)
                if (!(t * 16 + i < r)) bv[u][t] = zero4;
    };
    i32x4 bres[RES ? SB : 1][RT];
    if constexpr (RES) fetch_a(0, bres);

    int slot_next = slot_of_pos[min(pbeg + first * 16 + i, end - 1)];
    for (int tile = first; tile < last; ++tile) {
    const int base = pbeg + tile * 16;
    const bool row_ok = base + i < end;
    const int8_t* qrow = q8 + (size_t)(slot_next / w) * dp;
    // the next tile's pair numbers are requested now, its query rows when this tile is done
    slot_next = slot_of_pos[min(base + 16 + i, end - 1)];

    i32x4 acc[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) acc[t] = zero4;

    for (int s0 = 0; s0 < steps; s0 += SB) {
        i32x4 av[SB], bload[RES ? 1 : SB][RT];
#pragma unroll
        for (int u = 0; u < SB; ++u) av[u] = load16(qrow + min(64 * (s0 + u) + 16 * g, dp - 16));
        if constexpr (!RES) fetch_a(s0, bload);
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (s0 + u < steps) {                        // uniform
                // d' is a multiple of 16: a 16-byte group is all in or all out
                const bool a_ok = row_ok && 64 * (s0 + u) + 16 * g < dp;
                const i32x4 a = a_ok ? av[u] : zero4;
#pragma unroll
                for (int t = 0; t < RT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, RES ? bres[RES ? u : 0][t] : bload[RES ? 0 : u][t], acc[t], 0, 0, 0);
            }
        }
    }

    // acc[t][v] = R[pair 4g+v][column 16t+i].  Row maximum over the r columns: over t here, over i by shuffles.
    if constexpr (COLS) {
        const bool mixed = A_first != nullptr;           // uniform
        float dA[RT], a0[RT];
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            dA[t] = sA[(size_t)c * r + min(t * 16 + i, r - 1)];
            a0[t] = mixed ? A_first[(size_t)c * r + min(t * 16 + i, r - 1)] : 0.0f;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int pos = base + 4 * g + v;
            const int qv = slot_of_pos[min(pos, end - 1)] / w;
            const float dxq = dx[qv];
            const float x0 = mixed ? qproj[(size_t)qv * dp] : 0.0f;
            float rho[RT], mx = 0.0f;
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                rho[t] = t * 16 + i < r ? __fmul_rn((float)acc[t][v], __fmul_rn(dxq, dA[t])) : 0.0f;
                if (mixed) {
                    if (t * 16 + i < r) rho[t] = __fmaf_rn(x0, a0[t], rho[t]);
                    if (t == 0 && i == 0) {                  // the unquantized first component of r
                        if (pos < end) rho0[pos] = rho[0];
                        rho[0] = 0.0f;                       // out of the maximum; its code is rint(0) = 0
                    }
                }
                mx = fmaxf(mx, fabsf(rho[t]));
            }
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
            if (pos < end) {
                const bool any = mx > 0.0f;
                const float cx = any ? (float)(127.0 / (double)mx) : 0.0f;
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    int zc = (int)rintf(__fmul_rn(rho[t], cx));
                    zc = max(-127, min(127, zc));
                    Z[(size_t)pos * (RT * 16) + t * 16 + i] = (int8_t)(any ? zc : 0);
                }
                if (i == 0) sigma[pos] = any ? (float)((double)mx / 127.0) : 0.0f;
            }
        }
        continue;
    }
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
    }   // tiles of this cluster
    }   // clusters of this wavefront
}

}  // namespace lorann
