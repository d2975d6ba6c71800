// Second 8-bit product, score epilogue and exact candidate selection, one query per block (Sec. 3.2, 3.3,
// 2.2): for each of the query's w pairs the integer scores Y = z^T B_c of all points of the cluster, the
// estimated score s = sigma' * Y - bias as ONE float fused multiply-add (sigma' = sigma for inner product and
// cosine, 2 sigma for Euclidean; bias = |c_j|^2 for Euclidean, Sec. 3.1), and the m points of highest score
// with ties resolved toward the lower corpus row.
//
// This kernel is the exact, order-independent definition of the candidate set: a 4-pass radix select over
// order-preserving keys of the scores, recomputing the cheap integer scores in every pass.  It reads each
// cluster once per QUERY (not once per batch), so it is the reference path and the path for the few queries a
// faster batch kernel cannot finish, not the one that carries the throughput.
#pragma once
#include "common.hpp"

namespace lorann {

__device__ __forceinline__ int dot4_i8(int a, int b, int c) {
    return __builtin_amdgcn_sdot4(a, b, c, false);
}

// Integer score of one point: Y = sum_t z[t] * code[t] over r_pad bytes (RB 16-byte blocks).
template <int RB>
__device__ __forceinline__ int point_score(const int8_t* __restrict__ code, const int* __restrict__ zw) {
    const i32x4* bp = reinterpret_cast<const i32x4*>(code);
    int y = 0;
#pragma unroll
    for (int u = 0; u < RB; ++u) {
        const i32x4 bv = bp[u];
        y = dot4_i8(bv[0], zw[4 * u + 0], y);
        y = dot4_i8(bv[1], zw[4 * u + 1], y);
        y = dot4_i8(bv[2], zw[4 * u + 2], y);
        y = dot4_i8(bv[3], zw[4 * u + 3], y);
    }
    return y;
}

struct SelectArgs {
    const int32_t* qlist;        // optional list of query numbers to process (NULL: queries 0..nq-1)
    const int32_t* qcount;       // device count of entries in qlist (used only with qlist)
    const int32_t* sel;          // [nq][w]
    const int32_t* pos_of_slot;  // [nq*w]
    const int8_t* Z;             // [npairs][r_pad], bucket order
    const float* sigma;          // [npairs], bucket order
    const int8_t* Bp;            // [n][r_pad]
    const int64_t* off;          // [L+1]
    const float* sqnorm;         // [n] (Euclidean) or NULL
    const float* pt_scale;       // [n] step size of each point's code (column-wise quantization) or NULL
    const float* pt_first;       // [n] unquantized first row of B_c (mixed-precision decomposition) or NULL
    const float* rho0;           // [npairs] bucket order: unquantized first component of each pair's r, or NULL
    int32_t* cand;               // [nq][m] out: candidate rows, -1 padded
    int32_t* fb_total;           // optional running total of the list lengths seen (profiling), or NULL
    int w, m;
};

// One query: the whole block works on query q.  RB = r_pad / 16.
template <int RB>
__device__ __forceinline__ void select_exact_query(const SelectArgs& a, const int q) {
    constexpr int ZW = RB * 4;                    // 32-bit words per z vector
    __shared__ int pc[256], ppos[256], pcnt[256], pstart[257];
    __shared__ int64_t prow0[256];
    __shared__ float psig[256], pr0[256];
    __shared__ int zs[256 * ZW];
    __shared__ int hist[256];
    __shared__ int wsum[4];
    __shared__ uint32_t s_prefix;
    __shared__ int s_need, s_above;

    const int tid = threadIdx.x;
    const int w = a.w, m = a.m;
    const bool l2 = a.sqnorm != nullptr;

    // pairs of this query, re-ordered by cluster id so that enumeration order == ascending corpus row
    if (tid < w) pc[tid] = a.sel[(size_t)q * w + tid];
    __syncthreads();
    int myc = 0, myrank = 0, mypos = 0;
    if (tid < w) {
        myc = pc[tid];
        for (int u = 0; u < w; ++u) myrank += (pc[u] < myc) ? 1 : 0;
        mypos = a.pos_of_slot[(size_t)q * w + tid];
    }
    __syncthreads();
    if (tid < w) {
        pc[myrank] = myc;
        ppos[myrank] = mypos;
        const int64_t r0 = a.off[myc];
        prow0[myrank] = r0;
        pcnt[myrank] = (int)(a.off[myc + 1] - r0);
        const float s = a.sigma[mypos];
        psig[myrank] = l2 ? 2.0f * s : s;
        const float r0f = a.rho0 ? a.rho0[mypos] : 0.0f;
        pr0[myrank] = l2 ? 2.0f * r0f : r0f;
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int j = 0; j < w; ++j) { pstart[j] = acc; acc += pcnt[j]; }
        pstart[w] = acc;
        s_prefix = 0u; s_need = m; s_above = 0;
    }
    for (int idx = tid; idx < w * ZW; idx += 256) {
        const int j = idx / ZW, k = idx - j * ZW;
        zs[idx] = reinterpret_cast<const int*>(a.Z)[(size_t)ppos[j] * ZW + k];
    }
    __syncthreads();
    const int N = pstart[w];
    int32_t* out = a.cand + (size_t)q * m;

    if (N <= m) {      // fewer scored points than m: all of them are candidates
        for (int j = 0; j < w; ++j)
            for (int t = tid; t < pcnt[j]; t += 256) out[pstart[j] + t] = (int32_t)(prow0[j] + t);
        for (int t = N + tid; t < m; t += 256) out[t] = -1;
        return;
    }

    auto key_of = [&](int j, int t) -> uint32_t {
        const int64_t row = prow0[j] + t;
        const int y = point_score<RB>(a.Bp + (size_t)row * (RB * 16), zs + j * ZW);
        const float bias = l2 ? a.sqnorm[row] : 0.0f;
        const float mult = a.pt_scale ? __fmul_rn(psig[j], a.pt_scale[row]) : psig[j];
        float sc = __fmaf_rn((float)y, mult, -bias);
        if (a.pt_first) sc = __fmaf_rn(pr0[j], a.pt_first[row], sc);
        return float_key_asc(sc);
    };

    uint32_t mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        for (int j = 0; j < w; ++j)
            for (int t = tid; t < pcnt[j]; t += 256) {
                const uint32_t key = key_of(j, t);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
        __syncthreads();
        if (tid < 64) {     // descending digit walk: the digit where the count from the top reaches need
            const int need = s_need;
            const int h0 = hist[255 - 4 * tid], h1 = hist[254 - 4 * tid], h2 = hist[253 - 4 * tid], h3 = hist[252 - 4 * tid];
            const int mine = h0 + h1 + h2 + h3;
            int incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (tid >= o) incl += t; }
            const int excl = incl - mine;
            if (excl < need && incl >= need) {
                int cum = excl, dgt = 255 - 4 * tid;
                if (cum + h0 >= need) { }
                else { cum += h0; if (cum + h1 >= need) { dgt -= 1; } else { cum += h1; if (cum + h2 >= need) { dgt -= 2; } else { cum += h2; dgt -= 3; } } }
                s_prefix = prefix | ((uint32_t)dgt << shift);
                s_need = need - cum;
            }
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    // T = key of the m-th best score; take every key above it and the first need_ties equal to it (row order).
    const uint32_t T = s_prefix;
    const int need_ties = s_need;
    const int n_above = m - need_ties;
    int tie_base = 0;
    for (int j = 0; j < w; ++j) {
        const int cnt = pcnt[j];
        for (int t0 = 0; t0 < cnt; t0 += 256) {
            const int t = t0 + tid;
            const bool in = t < cnt;
            uint32_t key = 0u;
            if (in) key = key_of(j, t);
            if (in && key > T) out[atomicAdd(&s_above, 1)] = (int32_t)(prow0[j] + t);
            if (tie_base < need_ties) {      // uniform across the block
                const bool tie = in && key == T;
                int tot;
                const int rank = block_flag_scan<4>(tie, wsum, tot);
                if (tie && tie_base + rank < need_ties) out[n_above + tie_base + rank] = (int32_t)(prow0[j] + t);
                tie_base += tot;
            }
        }
    }
}

// grid = any (blocks stride over the work), block = 256.  Work = queries 0..nq-1, or the entries of a.qlist
// (their number is read from a.qcount on the device).
template <int RB>
__global__ __launch_bounds__(256) void k_select_exact(SelectArgs a, int nq) {
    const int total = a.qlist ? *a.qcount : nq;
    if (a.fb_total && a.qlist && blockIdx.x == 0 && threadIdx.x == 0 && total > 0) atomicAdd(a.fb_total, total);
    for (int e = blockIdx.x; e < total; e += gridDim.x) {
        select_exact_query<RB>(a, a.qlist ? a.qlist[e] : e);
        __syncthreads();
    }
}

// Search without the final re-ranking step (Sec. 7.1 memory usage, App. D.3): the candidates ARE the answer and their
// estimated scores are what is reported.  For every candidate row of a.cand ([nq][m], valid entries first) this
// recomputes the score exactly as the selection did - same integer product, same single fused multiply-add - and
// writes dissimilarity = -score and the row's id into the arrays the top-k kernels order.
// grid = ceil(nq / 4), block = 256 (one wavefront per query).
template <int RB>
__global__ __launch_bounds__(256) void k_candidate_scores(SelectArgs a, int nq, const int64_t* __restrict__ ids,
                                                           float* __restrict__ dist, int64_t* __restrict__ cid,
                                                           int32_t* __restrict__ ccount) {
    constexpr int ZW = RB * 4;
    const int lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;
    const int w = a.w, m = a.m;
    const bool l2 = a.sqnorm != nullptr;
    int cnt = 0;
    for (int t0 = 0; t0 < m; t0 += 64) {
        const int t = t0 + lane;
        const int row = t < m ? a.cand[(size_t)q * m + t] : -1;
        if (row >= 0) {
            int j = 0;                                  // the selected cluster that owns the row
            for (int u = 0; u < w; ++u) {
                const int c = a.sel[(size_t)q * w + u];
                if (a.off[c] <= row && row < a.off[c + 1]) j = u;
            }
            const int pos = a.pos_of_slot[(size_t)q * w + j];
            int zw[ZW];
#pragma unroll
            for (int i = 0; i < ZW; ++i) zw[i] = reinterpret_cast<const int*>(a.Z)[(size_t)pos * ZW + i];
            const int y = point_score<RB>(a.Bp + (size_t)row * (RB * 16), zw);
            const float sg = a.sigma[pos];
            const float bias = l2 ? a.sqnorm[row] : 0.0f;
            const float sp = l2 ? 2.0f * sg : sg;
            float sc = __fmaf_rn((float)y, a.pt_scale ? __fmul_rn(sp, a.pt_scale[row]) : sp, -bias);
            if (a.pt_first) sc = __fmaf_rn(l2 ? 2.0f * a.rho0[pos] : a.rho0[pos], a.pt_first[row], sc);
            dist[(size_t)q * m + t] = -sc;
            cid[(size_t)q * m + t] = ids ? ids[row] : (int64_t)row;
        }
        cnt += __popcll(__ballot(row >= 0));
    }
    if (lane == 0) ccount[q] = cnt;
}

// Integer scores of every point of every pair, for verification: y[y_off[slot] + t] = z_slot^T code(row0 + t).
// grid = npairs (one block per slot), block = 256.
template <int RB>
__global__ __launch_bounds__(256) void k_dump_pair_scores(const int32_t* __restrict__ sel, const int32_t* __restrict__ pos_of_slot,
                                                           const int8_t* __restrict__ Z, const int8_t* __restrict__ Bp,
                                                           const int64_t* __restrict__ off, const int64_t* __restrict__ y_off,
                                                           int32_t* __restrict__ y) {
    constexpr int ZW = RB * 4;
    __shared__ int zw[ZW];
    const int slot = blockIdx.x;
    const int c = sel[slot];
    const int64_t r0 = off[c];
    const int cnt = (int)(off[c + 1] - r0);
    if (threadIdx.x < ZW) zw[threadIdx.x] = reinterpret_cast<const int*>(Z)[(size_t)pos_of_slot[slot] * ZW + threadIdx.x];
    __syncthreads();
    for (int t = threadIdx.x; t < cnt; t += 256)
        y[y_off[slot] + t] = point_score<RB>(Bp + (size_t)(r0 + t) * (RB * 16), zw);
}

}  // namespace lorann
