// Per-query selection kernels of the batched scoring path (Sec. 2.2: "the t highest scoring points are
// selected into the candidate set"; t is called m here):
//   k_seed_threshold: tau_q = the m-th best score within the query's nearest cluster(s), a valid lower bound on
//                     its m-th best score overall;
//   k_select_final  : exact top-m of the query's survivor list, order (score descending, row ascending);
//                     queries whose list overflowed are put on the list for the exact per-query kernel.
#pragma once
#include "common.hpp"
#include "select_exact.hpp"

namespace lorann {

// m-th largest key among keys[0..n) held in LDS (n >= m >= 1).  Returns the key; need_ties = how many of the
// keys equal to it belong to the top m.  hist: 256 ints of LDS; sh: 2 words of LDS.  Block = 256 threads;
// contains barriers, so every thread must call it with the same arguments.
__device__ __forceinline__ uint32_t block_mth_largest(const uint32_t* keys, int n, int m, int* hist, uint32_t* sh, int& need_ties) {
    const int tid = threadIdx.x;
    if (tid == 0) { sh[0] = 0u; sh[1] = (uint32_t)m; }
    uint32_t mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh[0];
        for (int i = tid; i < n; i += 256) {
            const uint32_t key = keys[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid < 64) {
            const int need = (int)sh[1];
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
                sh[0] = prefix | ((uint32_t)dgt << shift);
                sh[1] = (uint32_t)(need - cum);
            }
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    need_ties = (int)sh[1];
    const uint32_t T = sh[0];
    __syncthreads();
    return T;
}

constexpr int kSeedCap = 8192;    // scores of the seed clusters held in LDS (32 KiB)

struct SeedArgs {
    const int32_t* sel;          // [nq][w] clusters, nearest centroid first
    const int32_t* pos_of_slot;  // [nq*w]
    const int8_t* Z;             // [npairs][r_pad] bucket order
    const float* sigma;          // [npairs] bucket order
    const int8_t* Bp;            // [n][r_pad]
    const int64_t* off;          // [L+1]
    const float* sqnorm;         // [n] (Euclidean) or NULL
    float* tau;                  // out [nq]
    int32_t* surv_cnt;           // out [nq]: cleared
    int w, m;
};

// tau_q = the m-th best estimated score among the points of the query's nearest clusters ("seed": the shortest
// prefix of its ranked cluster list that holds at least m points, at most kSeedCap of them).  Every seed score is
// a real score of the query, so at least m scores are >= tau_q: it is a valid lower bound on the m-th best
// score overall, and a tight one whenever the nearest clusters hold most of the best candidates.  -inf when all
// w clusters together hold fewer than m points.     grid = nq, block = 256.  RB = r_pad / 16.
template <int RB>
__global__ __launch_bounds__(256) void k_seed_threshold(SeedArgs a) {
    constexpr int ZW = RB * 4;
    __shared__ uint32_t keys[kSeedCap];
    __shared__ int zw[ZW];
    __shared__ int hist[256];
    __shared__ uint32_t sh[2];
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    const bool l2 = a.sqnorm != nullptr;
    if (tid == 0) a.surv_cnt[q] = 0;
    int n = 0;
    for (int jp = 0; jp < a.w && n < a.m; ++jp) {        // uniform loop: n is the same in every thread
        const int c = a.sel[(size_t)q * a.w + jp];
        const int64_t r0 = a.off[c];
        const int cnt = min((int)(a.off[c + 1] - r0), kSeedCap - n);
        const int pos = a.pos_of_slot[(size_t)q * a.w + jp];
        __syncthreads();
        if (tid < ZW) zw[tid] = reinterpret_cast<const int*>(a.Z)[(size_t)pos * ZW + tid];
        __syncthreads();
        const float s = a.sigma[pos];
        const float sp = l2 ? 2.0f * s : s;
        for (int t = tid; t < cnt; t += 256) {
            const int y = point_score<RB>(a.Bp + (size_t)(r0 + t) * (RB * 16), zw);
            const float bias = l2 ? a.sqnorm[r0 + t] : 0.0f;
            keys[n + t] = float_key_asc(__fmaf_rn((float)y, sp, -bias));
        }
        n += cnt;
    }
    __syncthreads();
    if (n < a.m) {
        if (tid == 0) a.tau[q] = -INFINITY;
        return;
    }
    int need_ties;
    const uint32_t T = block_mth_largest(keys, n, a.m, hist, sh, need_ties);
    if (tid == 0) {
        const uint32_t u = (T & 0x80000000u) ? (T & 0x7fffffffu) : ~T;   // inverse of float_key_asc
        a.tau[q] = __uint_as_float(u);
    }
}

struct FinalArgs {
    const float* surv_score;     // [nq][cap]
    const int32_t* surv_row;     // [nq][cap]
    const int32_t* surv_cnt;     // [nq]
    int32_t* cand;               // [nq][m] out
    const int32_t* qlist;        // queries to process (NULL: 0..nq-1) and their number on the device
    const int32_t* qcount;
    int32_t* big_list;           // out: queries with lds_cap < survivors <= cap (NULL: none expected)
    int32_t* big_count;
    int32_t* fb_list;            // out: queries whose survivor list overflowed cap
    int32_t* fb_count;
    int nq, cap, lds_cap, m;
};

// Exact top-m of one query's survivors, order (score descending, row ascending).  Block = 256,
// dynamic LDS = lds_cap * 12 bytes (keys, rows, tie keys).  Blocks stride over the work list.
// Queries with more than lds_cap survivors go to big_list (a second launch with more LDS takes them); queries
// whose list overflowed cap go to fb_list (the exact per-query kernel takes them).
__global__ __launch_bounds__(256) void k_select_final(FinalArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t* keys = reinterpret_cast<uint32_t*>(smem);
    int32_t* rows = reinterpret_cast<int32_t*>(smem + (size_t)a.lds_cap * 4);
    uint32_t* tkeys = reinterpret_cast<uint32_t*>(smem + (size_t)a.lds_cap * 8);
    __shared__ int hist[256];
    __shared__ uint32_t sh[2];
    __shared__ int s_out, s_nt;
    const int tid = threadIdx.x;
    const int total = a.qlist ? *a.qcount : a.nq;
    const int m = a.m;
    for (int e = blockIdx.x; e < total; e += gridDim.x) {
        const int q = a.qlist ? a.qlist[e] : e;
        const int cnt = a.surv_cnt[q];
        int32_t* out = a.cand + (size_t)q * m;
        __syncthreads();                       // LDS of the previous query is no longer read
        if (cnt > a.cap) {
            if (tid == 0) a.fb_list[atomicAdd(a.fb_count, 1)] = q;
            continue;
        }
        if (cnt > a.lds_cap) {
            if (tid == 0) a.big_list[atomicAdd(a.big_count, 1)] = q;
            continue;
        }
        for (int i = tid; i < cnt; i += 256) {
            keys[i] = float_key_asc(a.surv_score[(size_t)q * a.cap + i]);
            rows[i] = a.surv_row[(size_t)q * a.cap + i];
        }
        if (tid == 0) { s_out = 0; s_nt = 0; }
        __syncthreads();
        if (cnt <= m) {     // every survivor is a candidate
            for (int i = tid; i < m; i += 256) out[i] = i < cnt ? rows[i] : -1;
            continue;
        }
        int need_ties;
        const uint32_t T = block_mth_largest(keys, cnt, m, hist, sh, need_ties);
        const int n_above = m - need_ties;
        // ties at the threshold: the need_ties lowest rows win.  Collect ~row of the tied entries and select again.
        for (int i = tid; i < cnt; i += 256)
            if (keys[i] == T) tkeys[atomicAdd(&s_nt, 1)] = ~(uint32_t)rows[i];
        __syncthreads();
        const int nt = s_nt;
        uint32_t RT = 0u;      // threshold on ~row: tied entries with ~row >= RT are taken
        if (nt > need_ties) {
            int dummy;
            RT = block_mth_largest(tkeys, nt, need_ties, hist, sh, dummy);
        }
        for (int i = tid; i < cnt; i += 256) {
            const uint32_t key = keys[i];
            if (key > T) out[atomicAdd(&s_out, 1)] = rows[i];
            else if (key == T && (~(uint32_t)rows[i]) >= RT) out[n_above + atomicAdd(&s_nt, 1) - nt] = rows[i];
        }
    }
}

}  // namespace lorann
