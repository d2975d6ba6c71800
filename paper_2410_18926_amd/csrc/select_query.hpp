// Per-query candidate selection of the batched scoring path (the candidate-selection step of Sec. 2.2; the
// paper's candidate count t is called m here).
//
// k_pair_max has already computed, for every (query, cluster) pair, the best score of the cluster.  One block
// per query now walks the query's pairs in descending order of that best score and keeps a running threshold T =
// the m-th best score seen so far: a cluster whose best score is below T cannot contribute a candidate, and
// because the pairs are sorted the walk stops at the first such cluster.  A query's best candidates sit in very
// few of its w clusters, so typically one or two clusters are scored here (point-parallel, 4-way int8 dot
// products); all the others were dismissed by their maxima alone.  The scores that reach T are held in LDS, the
// threshold is tightened by an exact radix select whenever new ones arrive, and the final exact top-m (score
// descending, row ascending) is written out.  Only if more scores tie with T than LDS can hold does the query go
// to the exact per-query kernel.
#pragma once
#include "common.hpp"
#include "select_exact.hpp"

namespace lorann {

// m-th largest among the keys f(i), i in [0, n), for which f returns true (at least m of them, m >= 1).
// f(i, key&) -> bool.  Returns the key; need_ties = how many of the keys equal to it belong to the top m.
// hist: 256 ints of LDS; sh: 2 words of LDS.  Block = 256 threads; contains barriers, so every thread must
// call it with the same arguments.
template <typename F>
__device__ __forceinline__ uint32_t block_mth_largest(int n, int m, int* hist, uint32_t* sh, int& need_ties, F f) {
    const int tid = threadIdx.x;
    if (tid == 0) { sh[0] = 0u; sh[1] = (uint32_t)m; }
    uint32_t mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh[0];
        for (int i = tid; i < n; i += 256) {
            uint32_t key;
            if (f(i, key) && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid < 64) {     // descending digit walk: the digit where the count from the top reaches need
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


// (score, row) entries a query holds in LDS: 2048 (16 KiB, more blocks per CU) or 6144 for m > 1024.  A quarter
// of the capacity is scored between capacity checks.
inline int select_query_cap(int m) { return m <= 1024 ? 2048 : 6144; }

// Block-wide minimum of `v` written to *dst (scratch: one int of LDS, clobbered).  Contains barriers.
__device__ __forceinline__ void block_min_to(int32_t* dst, int v, int* scratch) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
    if (threadIdx.x == 0) *scratch = 0x7fffffff;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) atomicMin(scratch, v);
    __syncthreads();
    if (threadIdx.x == 0) *dst = *scratch;
}

struct QuerySelectArgs {
    const int32_t* sel;          // [nq][w] clusters of each query
    const int32_t* pos_of_slot;  // [nq*w]
    const uint32_t* pmax;        // [npairs] key of each pair's best score (0: the cluster is empty), bucket order
    const int8_t* Z;             // [npairs][r_pad] bucket order
    const float* sigma;          // [npairs] bucket order
    const int8_t* Bp;            // [n][r_pad]
    const int64_t* off;          // [L+1]
    const float* sqnorm;         // [n] (Euclidean) or NULL
    const float* pt_scale;       // [n] step size of each point's code (column-wise quantization) or NULL
    const float* pt_first;       // [n] unquantized first row of B_c (mixed-precision decomposition) or NULL
    const float* rho0;           // [npairs] bucket order: unquantized first component of each pair's r, or NULL
    int32_t* cand;               // out [nq][m]: candidate rows, unordered, -1 padded
    float* tau;                  // out [nq]: score of the m-th candidate (-inf if fewer than m points were scored)
    int32_t* n_kept;             // out [nq]: scores held in LDS when the walk ended (-1: handed to the exact kernel)
    int32_t* qkey;               // out [nq]: smallest candidate row (locality hint for the order of the re-rank)
    int32_t* fb_list;            // out: queries that need the exact per-query kernel
    int32_t* fb_count;           //      and their number (0 on entry)
    const int32_t* qorder;       // [nq] queries grouped by nearest cluster (visiting order)
    int nq, w, m;
    int cap;                     // select_query_cap(m)
    int run_shift;               // log2 of the queries per run (see the kernel)
};

// grid = 512 * ceil(nq / 512), block = 256, dynamic LDS = 8 * cap bytes.  RB = r_pad / 16.
// Queries are visited grouped by nearest cluster (workgroups are dealt round-robin over the 8 XCDs): queries that
// score the same cluster run together and share its codes in L2.
// PT = points a thread scores between two capacity checks = cap / 1024.
// INLINE_FB (small batches): a query whose survivor list overflows is finished right here by the exact per-query
// routine instead of being handed to a later launch.
template <int RB, int PT, bool INLINE_FB = false>
__global__ __launch_bounds__(256) void k_select_query(QuerySelectArgs a) {
    constexpr int ZW = RB * 4;
    extern __shared__ __align__(16) unsigned char qs_smem[];
    uint32_t* keys = reinterpret_cast<uint32_t*>(qs_smem);
    int32_t* rows = reinterpret_cast<int32_t*>(qs_smem + (size_t)a.cap * 4);
    const int kQCap = a.cap, kQChunk = a.cap >> 2;
    __shared__ int zw[ZW];
    __shared__ int hist[256];
    __shared__ int wsum[4];
    __shared__ uint32_t sh[2];
    __shared__ uint32_t pk[256];      // best-score keys of the query's pairs
    __shared__ int ppos[256], order[256];
    __shared__ int s_count, s_out, s_ties;
    const int tid = threadIdx.x;
    // position in the visiting order: runs of 64 consecutive queries go to one XCD (they share clusters and hence
    // codes in that XCD's L2), successive runs to successive XCDs - a popular, large cluster (many queries, each
    // with much to score) is spread over all of them instead of making one XCD the last to finish
    const int slot = (int)(blockIdx.x >> 3);
    const int rs = a.run_shift;
    const int si = ((((slot >> rs) << 3) + (int)(blockIdx.x & 7)) << rs) + (slot & ((1 << rs) - 1));
    if (si >= a.nq) return;
    const int q = __builtin_amdgcn_readfirstlane(a.qorder[si]);     // uniform over the block: scalar loads below
    const int w = a.w, m = a.m;
    const bool l2 = a.sqnorm != nullptr, cols = a.pt_scale != nullptr, mixed = a.pt_first != nullptr;
    if (tid == 0) s_count = 0;
    if (tid < w) {
        const int pos = a.pos_of_slot[(size_t)q * w + tid];
        ppos[tid] = pos;
        pk[tid] = a.pmax[pos];
    }
    __syncthreads();
    if (tid < w) {      // order the pairs by best score, descending (ties: lower rank first)
        const uint32_t k = pk[tid];
        int rank = 0;
        for (int u = 0; u < w; ++u) rank += (pk[u] > k || (pk[u] == k && u < tid)) ? 1 : 0;
        order[rank] = tid;
    }
    __syncthreads();

    uint32_t T = 0u;          // running threshold key: the m-th best score seen so far (0: none yet)
    int count = 0;            // entries in keys/rows, all >= T (uniform)
    bool overflow = false;

    // Tighten T to the m-th largest stored key and drop the entries below it (stable, in place).
    auto compact = [&]() {
        if (count < m) return;
        int need_ties;
        const uint32_t Tn = block_mth_largest(count, m, hist, sh, need_ties, [&](int i, uint32_t& key) { key = keys[i]; return true; });
        int kept = 0;
        for (int base = 0; base < count; base += 256) {
            const int i = base + tid;
            uint32_t k = 0u;
            int32_t r = 0;
            if (i < count) { k = keys[i]; r = rows[i]; }
            const bool keep = i < count && k >= Tn;
            int tot;
            const int rank = block_flag_scan<4>(keep, wsum, tot);     // barriers: the chunk is in registers before any write
            if (keep) { keys[kept + rank] = k; rows[kept + rank] = r; }
            kept += tot;
        }
        __syncthreads();
        T = Tn;
        count = kept;
        if (tid == 0) s_count = kept;
        __syncthreads();
    };

    // The codes of the PT points a thread scores between two capacity checks are requested together, with
    // clamped addresses instead of branches, so that the loads overlap.
    for (int o = 0; o < w && !overflow; ++o) {
        const int jp = __builtin_amdgcn_readfirstlane(order[o]);
        if (pk[jp] == 0u || pk[jp] < T) break;           // sorted: no later cluster can reach T either
        const int c = a.sel[(size_t)q * w + jp];
        const int64_t r0 = a.off[c];
        const int m_c = (int)(a.off[c + 1] - r0);
        const int pos = __builtin_amdgcn_readfirstlane(ppos[jp]);
        // requests that do not depend on each other go out together: the pair's z and sigma, the first codes
        const int zv = reinterpret_cast<const int*>(a.Z)[(size_t)pos * ZW + (tid < ZW ? tid : 0)];
        const float s = a.sigma[pos];
        const float rfirst = mixed ? a.rho0[pos] : 0.0f;
        i32x4 code[PT][RB];
        float bias[PT], psc[PT], pf[PT];
        auto fetch_codes = [&](int p0) {
#pragma unroll
            for (int e = 0; e < PT; ++e) {
                {
                    const int64_t row = r0 + min(p0 + e * 256 + tid, m_c - 1);
                    const i32x4* bp = reinterpret_cast<const i32x4*>(a.Bp + (size_t)row * (RB * 16));
#pragma unroll
                    for (int u = 0; u < RB; ++u) code[e][u] = bp[u];
                    bias[e] = l2 ? a.sqnorm[row] : 0.0f;
                    psc[e] = cols ? a.pt_scale[row] : 1.0f;     // times 1 is exact: one code path for both schemes
                    pf[e] = mixed ? a.pt_first[row] : 0.0f;
                }
            }
        };
        if (m_c > 0) fetch_codes(0);
        __syncthreads();
        if (tid < ZW) zw[tid] = zv;
        __syncthreads();
        const float sp = l2 ? 2.0f * s : s;
        const float r0p = l2 ? 2.0f * rfirst : rfirst;
        for (int p0 = 0; p0 < m_c; p0 += kQChunk) {
            if (count > kQCap - kQChunk) {
                compact();
                if (count > kQCap - kQChunk) { overflow = true; break; }   // too many scores tie with the threshold
            }
            if (p0 > 0) fetch_codes(p0);
#pragma unroll
            for (int e = 0; e < PT; ++e) {
                {
                    const int t = p0 + e * 256 + tid;
                    int y = 0;
#pragma unroll
                    for (int u = 0; u < RB; ++u) {
                        y = dot4_i8(code[e][u][0], zw[4 * u + 0], y);
                        y = dot4_i8(code[e][u][1], zw[4 * u + 1], y);
                        y = dot4_i8(code[e][u][2], zw[4 * u + 2], y);
                        y = dot4_i8(code[e][u][3], zw[4 * u + 3], y);
                    }
                    float sc = __fmaf_rn((float)y, __fmul_rn(sp, psc[e]), -bias[e]);
                    if (mixed) sc = __fmaf_rn(r0p, pf[e], sc);      // uniform
                    const uint32_t key = float_key_asc(sc);
                    if (t < m_c && key >= T) {
                        const int at = atomicAdd(&s_count, 1);
                        keys[at] = key;
                        rows[at] = (int32_t)(r0 + t);
                    }
                }
            }
            __syncthreads();
            count = s_count;
        }
        if (!overflow) compact();     // new scores arrived: raise the threshold before looking at the next cluster
    }

    int32_t* out = a.cand + (size_t)q * m;
    if (overflow && INLINE_FB) {       // uniform
        if (tid == 0) { a.n_kept[q] = -1; a.tau[q] = key_to_float(T); a.qkey[q] = 0; }
        SelectArgs sa;
        sa.qlist = nullptr; sa.qcount = nullptr; sa.sel = a.sel; sa.pos_of_slot = a.pos_of_slot; sa.Z = a.Z; sa.sigma = a.sigma;
        sa.Bp = a.Bp; sa.off = a.off; sa.sqnorm = a.sqnorm; sa.pt_scale = a.pt_scale; sa.pt_first = a.pt_first; sa.rho0 = a.rho0;
        sa.cand = a.cand; sa.fb_total = nullptr; sa.w = w; sa.m = m;
        __syncthreads();
        select_exact_query<RB>(sa, q);
        return;
    }
    if (overflow) {
        if (tid == 0) {
            a.fb_list[atomicAdd(a.fb_count, 1)] = q; a.n_kept[q] = -1; a.tau[q] = key_to_float(T);
            a.qkey[q] = (int32_t)a.off[a.sel[(size_t)q * w + order[0]]];     // first row of its most promising cluster
        }
        return;
    }
    if (tid == 0) { a.n_kept[q] = count; a.tau[q] = count >= m ? key_to_float(T) : -INFINITY; s_out = 0; s_ties = 0; }
    if (count <= m) {       // every kept score is a candidate (count < m: all scored points)
        int mn = 0x7fffffff;
        for (int i = tid; i < m; i += 256) { const int r = i < count ? rows[i] : -1; out[i] = r; if (r >= 0) mn = min(mn, r); }
        block_min_to(a.qkey + q, mn, &s_ties);
        return;
    }
    // count > m: T is the m-th largest key (compact() ran after the last arrivals); ties at T go to the lower rows
    __syncthreads();
    int above = 0;
    for (int i = tid; i < count; i += 256) above += keys[i] > T ? 1 : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) above += __shfl_xor(above, o, 64);
    if ((tid & 63) == 0) atomicAdd(&s_out, above);
    __syncthreads();
    const int n_above = s_out;
    const int need_ties = m - n_above;
    __syncthreads();
    if (tid == 0) s_out = 0;
    int dummy;
    const uint32_t RT = block_mth_largest(count, need_ties, hist, sh, dummy,
                                          [&](int i, uint32_t& key) { key = ~(uint32_t)rows[i]; return keys[i] == T; });
    int mn = 0x7fffffff;
    for (int i = tid; i < count; i += 256) {
        const uint32_t key = keys[i];
        if (key > T) { out[atomicAdd(&s_out, 1)] = rows[i]; mn = min(mn, rows[i]); }
        else if ((~(uint32_t)rows[i]) >= RT) { out[n_above + atomicAdd(&s_ties, 1)] = rows[i]; mn = min(mn, rows[i]); }
    }
    __syncthreads();
    block_min_to(a.qkey + q, mn, &s_out);
}

}  // namespace lorann
