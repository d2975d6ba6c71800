// Per-query candidate selection of the batched scoring path (the candidate-selection step of Sec. 2.2; the
// paper's candidate count t is called m here).
//
// k_pair_max has already computed, for every (query, cluster) pair, the best score of the cluster and of each of
// its chunks of 64 consecutive points.  One block per query keeps a running threshold T, a lower bound of the
// query's m-th best score, and scores point by point (4-way int8 dot products) only chunks whose maximum reaches
// T; everything else is dismissed by its maximum alone.
//   - T starts from the chunk maxima themselves: every chunk maximum is the score of a distinct point, so the
//     m-th largest of them is a lower bound of the m-th best score.  Where a query's best points are spread over
//     most of its clusters this bound is close to the final threshold at once, and about m chunks are scored
//     whatever the cluster sizes.
//   - The pairs are visited in descending order of their best score, the best pair first and on its own: where a
//     query's best points sit in one or two clusters, scoring that cluster makes T tight and every other pair is
//     dismissed by its maximum.
// The scores that reach T are held in LDS, T is tightened by an exact radix select when enough new ones have
// arrived, and the final exact top-m (score descending, row ascending) is written out.  Only if more scores tie
// with T than LDS can hold does the query go to the exact per-query kernel.
#pragma once
#include "common.hpp"
#include "select_exact.hpp"

namespace lorann {

// m-th largest among the keys f(i), i in [0, n), for which f returns true (at least m of them, m >= 1).
// f(i, key&) -> bool.  Returns the key; need_ties = how many of the keys equal to it belong to the top m.
// hist: 256 ints of LDS; sh: 2 words of LDS.  Block = 256 threads; contains barriers, so every thread must
// call it with the same arguments.
// LOW_SHIFT > 0 stops after the bytes above it: the result is then the m-th largest key with its low LOW_SHIFT bits
// cleared - a lower bound of it that at least m keys reach (need_ties is meaningless then).
template <int LOW_SHIFT = 0, typename F>
__device__ __forceinline__ uint32_t block_mth_largest(int n, int m, int* hist, uint32_t* sh, int& need_ties, F f) {
    const int tid = threadIdx.x;
    if (tid == 0) { sh[0] = 0u; sh[1] = (uint32_t)m; }
    uint32_t mask = 0u;
    for (int shift = 24; shift >= LOW_SHIFT; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh[0];
#pragma unroll 4
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
    const uint32_t* cmax;        // best score of each 64-point chunk of each pair's cluster (float key, or the int32
                                 // accumulator when int_domain), or NULL: no chunk maxima
    const uint32_t* cm_off;      // [npairs] bucket order: first entry of the pair's row in cmax (~0u: it has none)
    int int_domain;              // chunk maxima are integer accumulators: score = fma(float(Y), sigma, -0)
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
    int wpad;                    // w rounded up to a multiple of 64 (sizes the per-pair tables in LDS)
    long long* dbg;              // TEMPORARY [nq][8]
};

constexpr int kTodoCap = 384;        // chunks waiting to be scored (LDS list)
inline size_t select_query_lds(int cap, int wpad) { return (size_t)cap * 8 + (size_t)(7 * wpad + 64) * 4; }
constexpr int kWindow = 2048;        // most chunk maxima examined per round

// grid = 512 * ceil(nq / 512), block = 256, dynamic LDS = select_query_lds(cap, wpad) bytes.  RB = r_pad / 16.
// Queries are visited grouped by nearest cluster (workgroups are dealt round-robin over the 8 XCDs): queries that
// score the same cluster run together and share its codes in L2.
// PT = points a thread scores between two capacity checks (4 * PT chunks per batch of the block).
template <int RB, int PT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PT == 2 && RB == 2 ? 7 : 1, 8))) void k_select_query(QuerySelectArgs a) {
    constexpr int ZW = RB * 4;
    extern __shared__ __align__(16) unsigned char qs_smem[];
    uint32_t* keys = reinterpret_cast<uint32_t*>(qs_smem);
    int32_t* rows = reinterpret_cast<int32_t*>(qs_smem + (size_t)a.cap * 4);
    const int kQCap = a.cap;
    constexpr int kBatch = 256 * PT;         // points scored between two capacity checks (4 * PT chunks)
    __shared__ int hist[256];
    __shared__ int wsum[4];
    __shared__ uint32_t sh[2];
    // the query's pairs in descending order of their best score (ties: lower rank first); wpad entries each
    int* const ptab = reinterpret_cast<int*>(qs_smem + (size_t)a.cap * 8);
    const int wp = a.wpad;
    uint32_t* const opk = reinterpret_cast<uint32_t*>(ptab);            // best-score key
    int* const opos = ptab + wp;                                         // position in bucket order
    int* const omc = ptab + 2 * wp;                                      // points of the cluster
    int* const orow0 = ptab + 3 * wp;                                    // its first corpus row
    float* const osig = reinterpret_cast<float*>(ptab + 4 * wp);         // its pair scale
    uint32_t* const ocm = reinterpret_cast<uint32_t*>(ptab + 5 * wp);    // first entry of its row of chunk maxima (~0u: none)
    int* const cstart = ptab + 6 * wp;                                   // chunks before the pair, in this order (wpad + 1 entries)
    __shared__ uint32_t todo[kTodoCap];
    __shared__ int s_count, s_out, s_ties;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // position in the visiting order: runs of 64 consecutive queries go to one XCD (they share clusters and hence
    // codes in that XCD's L2), successive runs to successive XCDs (a popular, large cluster - many queries, each
    // with much to score - is spread over all of them)
    const int slot = (int)(blockIdx.x >> 3);
    const int si = (((slot >> 6) << 3) + (int)(blockIdx.x & 7)) * 64 + (slot & 63);
    if (si >= a.nq) return;
    const int q = __builtin_amdgcn_readfirstlane(a.qorder[si]);     // uniform over the block: scalar loads below
    const int w = a.w, m = a.m;
    const bool l2 = a.sqnorm != nullptr, cols = a.pt_scale != nullptr, mixed = a.pt_first != nullptr;
    const bool have_cmax = a.cmax != nullptr;
    const long long t_0 = wall_clock64();
    if (tid == 0) s_count = 0;
    {
        uint32_t k = 0u, cmo = ~0u;
        int pos = 0, mc = 0, row0 = 0;
        float sgm = 0.0f;
        if (tid < w) {
            pos = a.pos_of_slot[(size_t)q * w + tid];
            if (have_cmax) cmo = a.cm_off[pos];
            const int c = a.sel[(size_t)q * w + tid];
            const int64_t r0 = a.off[c];
            mc = (int)(a.off[c + 1] - r0);
            row0 = (int)r0;
            k = a.pmax[pos];
            sgm = a.sigma[pos];
            hist[tid] = (int)k;
        }
        __syncthreads();
        int rank = 0;
        if (tid < w) {
            for (int u = 0; u < w; ++u) { const uint32_t ku = (uint32_t)hist[u]; rank += (ku > k || (ku == k && u < tid)) ? 1 : 0; }
            opk[rank] = k; opos[rank] = pos; ocm[rank] = cmo; omc[rank] = mc; orow0[rank] = row0; osig[rank] = sgm;
        }
        __syncthreads();
        // exclusive prefix of the chunk counts in this order (block scan over 256 threads)
        const int nch = tid < w ? (omc[tid] + 63) >> 6 : 0;
        int incl = nch;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (lane >= o) incl += t; }
        if (lane == 63) wsum[wv] = incl;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) before += i < wv ? wsum[i] : 0;
        if (tid < wp) cstart[tid + 1] = before + incl;
        if (tid == 0) cstart[0] = 0;
        __syncthreads();
    }
    const int NCH = cstart[w];
    long long t_a = wall_clock64(), t_b = 0, t_c = 0, t_score = 0, t_comp = 0; int n_win = 0, n_bat = 0, n_flagged = 0, n_cmp = 0;

    // the ordered pair that owns flat chunk number i (0 <= i < NCH)
    auto pair_of = [&](int i) {
        int lo = 0, hi = w;
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (cstart[mid] <= i) lo = mid; else hi = mid; }
        return lo;
    };
    // key of the best score of flat chunk i of pair o (an upper bound of every score in it)
    auto chunk_key = [&](int o, int i) -> uint32_t {
        const uint32_t row = ocm[o];
        if (row == ~0u) return opk[o];                  // no chunk maxima for this pair: the pair's best score bounds every chunk
        const uint32_t raw = a.cmax[(size_t)row + (i - cstart[o])];
        return a.int_domain ? float_key_asc(__fmaf_rn((float)(int)raw, osig[o], -0.0f)) : raw;
    };

    uint32_t T = 0u;          // running threshold key: a lower bound of the m-th best score (0: none yet)
    int count = 0;            // entries in keys/rows, all >= T (uniform)
    bool overflow = false;

    // The first 256 * KR chunk keys are requested here, all at once, and are on their way while the best pair is
    // being scored (thread tid keeps those of the flat chunks tid, tid + 256, ...); later ones are read when needed.
    constexpr int KR = 3;
    uint32_t kreg[KR];
#pragma unroll
    for (int u = 0; u < KR; ++u) {
        kreg[u] = 0u;
        if (256 * u < NCH) {                        // uniform
            const int ic = min(256 * u + tid, NCH - 1);
            kreg[u] = chunk_key(pair_of(ic), ic);
        }
    }
    auto key_at = [&](int i) -> uint32_t {          // i < NCH, i = tid mod 256
        if (i >= 256 * KR) return chunk_key(pair_of(i), i);
        uint32_t k = kreg[0];
#pragma unroll
        for (int u = 1; u < KR; ++u) k = i >= 256 * u ? kreg[u] : k;
        return k;
    };

    // Where the chunk maxima outnumber m several times, the m-th largest of them (every one the score of a distinct
    // point) is a useful first threshold.
    if (have_cmax && NCH >= 4 * m) {
        int dummy;
        T = block_mth_largest<8>(NCH, m, hist, sh, dummy, [&](int i, uint32_t& key) { key = key_at(i); return true; });
    }

    t_c = wall_clock64();
    int settled = 0;          // entries held after the latest compaction
    // Tighten T to the m-th largest stored key and drop the entries below it (stable, in place).
    auto compact = [&]() {
        if (count < m) return;
        ++n_cmp; const long long tc0 = wall_clock64();
        int need_ties;
        const uint32_t Tn = block_mth_largest(count, m, hist, sh, need_ties, [&](int i, uint32_t& key) { key = keys[i]; return true; });
        // every thread takes its entries into registers, then all of them write the kept ones behind a counter
        // (the list is unordered: ties are resolved by row number at the end)
        constexpr int EPT = 4 * PT;               // capacity / 256
        uint32_t kk[EPT];
        int32_t rr[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int i = 256 * e + tid;
            kk[e] = 0u; rr[e] = 0;
            if (i < count) { kk[e] = keys[i]; rr[e] = rows[i]; }
        }
        if (tid == 0) s_count = 0;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (256 * e + tid < count && kk[e] >= Tn) { const int at = atomicAdd(&s_count, 1); keys[at] = kk[e]; rows[at] = rr[e]; }
        __syncthreads();
        const int kept = s_count;
        T = Tn;
        count = kept;
        settled = kept;
        t_comp += wall_clock64() - tc0;
    };

    // Score the n_todo chunks of the list point by point: wavefront wv takes chunks wv, wv + 4, ... of every batch
    // of 4 * PT, lane = point of the chunk.  The codes of a batch are requested together, with clamped addresses
    // instead of branches, so that the loads overlap; z, sigma and rho0 of a chunk's pair are uniform over the
    // wavefront.
    auto score_todo = [&](int n_todo) {
        const long long ts0 = wall_clock64(); const long long tcb = t_comp;
        for (int i0 = 0; i0 < n_todo && !overflow; i0 += 4 * PT) {
            ++n_bat;
            if (count > kQCap - kBatch) {
                compact();
                if (count > kQCap - kBatch) { overflow = true; break; }   // too many scores tie with the threshold
            }
            i32x4 code[PT][RB];
            float bias[PT], psc[PT], pf[PT];
            int o_of[PT], row_of[PT];
            bool in_of[PT];
#pragma unroll
            for (int e = 0; e < PT; ++e) {
                const int ti = i0 + 4 * e + wv;
                const uint32_t ent = todo[min(ti, n_todo - 1)];
                const int o = (int)(ent >> 24), ch = (int)(ent & 0xffffffu);
                const int pt = 64 * ch + lane;
                const int64_t row = (int64_t)orow0[o] + min(pt, omc[o] - 1);
                o_of[e] = o; row_of[e] = (int)row; in_of[e] = ti < n_todo && pt < omc[o];
                const i32x4* bp = reinterpret_cast<const i32x4*>(a.Bp + (size_t)row * (RB * 16));
#pragma unroll
                for (int u = 0; u < RB; ++u) code[e][u] = bp[u];
                bias[e] = l2 ? a.sqnorm[row] : 0.0f;
                psc[e] = cols ? a.pt_scale[row] : 1.0f;     // times 1 is exact: one code path for both schemes
                pf[e] = mixed ? a.pt_first[row] : 0.0f;
            }
#pragma unroll
            for (int e = 0; e < PT; ++e) {
                const int o = __builtin_amdgcn_readfirstlane(o_of[e]);
                const int upos = __builtin_amdgcn_readfirstlane(opos[o]);
                const int* zp = reinterpret_cast<const int*>(a.Z) + (size_t)upos * ZW;
                int y = 0;
#pragma unroll
                for (int u = 0; u < RB; ++u) {
                    y = dot4_i8(code[e][u][0], zp[4 * u + 0], y);
                    y = dot4_i8(code[e][u][1], zp[4 * u + 1], y);
                    y = dot4_i8(code[e][u][2], zp[4 * u + 2], y);
                    y = dot4_i8(code[e][u][3], zp[4 * u + 3], y);
                }
                const float s = osig[o], rfirst = mixed ? a.rho0[upos] : 0.0f;
                const float sp = l2 ? 2.0f * s : s;
                float sc = __fmaf_rn((float)y, __fmul_rn(sp, psc[e]), -bias[e]);
                if (mixed) sc = __fmaf_rn(l2 ? 2.0f * rfirst : rfirst, pf[e], sc);      // uniform
                const uint32_t key = float_key_asc(sc);
                if (in_of[e] && key >= T) {
                    const int at = atomicAdd(&s_count, 1);
                    keys[at] = key;
                    rows[at] = row_of[e];
                }
            }
            __syncthreads();
            count = s_count;
        }
        t_score += (wall_clock64() - ts0) - (t_comp - tcb);
    };

    // Rounds over the flat list of chunk maxima, pairs in descending order of their best score.  A round covers
    // whole pairs (at most kWindow chunks; a larger cluster takes several rounds): the best pair alone first, and
    // from then on four times, twice or once as many pairs as the round before, depending on how few of the round's
    // chunks still reached T - while most do, T is still rising quickly and is raised again after every pair; once
    // few do, many pairs are dismissed per round.
    int e0 = 0, pw = 1;
    while (e0 < NCH && !overflow) {
        const int o0 = pair_of(e0);
        if (opk[o0] == 0u || opk[o0] < T) break;          // sorted: no later pair can reach T either
        const int e1 = min(cstart[min(w, o0 + pw)], e0 + kWindow);
        int n_todo = 0, n_flag = 0; ++n_win;
        if (T == 0u) {
            // no threshold yet: nothing can be dismissed, every chunk of the round is scored
            for (int base = e0; base < e1 && !overflow; base += kTodoCap) {
                const int nb = min(kTodoCap, e1 - base);
                for (int i = tid; i < nb; i += 256) { const int o = pair_of(base + i); todo[i] = ((uint32_t)o << 24) | (uint32_t)(base + i - cstart[o]); }
                __syncthreads();
                score_todo(nb);
            }
            n_flag = e1 - e0;
        } else
        for (int base = e0 & ~255; base < e1 && !overflow; base += 256) {
            const int i = base + tid;
            bool flag = false;
            if (i >= e0 && i < e1) flag = key_at(i) >= T;
            int tot;
            const int rank = block_flag_scan<4>(flag, wsum, tot);
            if (flag) { const int o = pair_of(i); todo[n_todo + rank] = ((uint32_t)o << 24) | (uint32_t)(i - cstart[o]); }
            n_todo += tot; n_flag += tot; n_flagged += tot;
            __syncthreads();
            if (n_todo > kTodoCap - 256) { score_todo(n_todo); n_todo = 0; }      // the next round may add 256
        }
        if (!overflow) score_todo(n_todo);
        pw = 4 * n_flag < e1 - e0 ? min(4 * pw, 256) : 2 * n_flag < e1 - e0 ? min(2 * pw, 256) : 1;
        e0 = e1;
        if (!overflow && count >= m && count > settled) compact();   // new scores arrived: raise the threshold
    }

    if (a.dbg && tid == 0) { long long t_d = wall_clock64(); long long* d = a.dbg + (size_t)q * 8; d[0] = t_a - t_0; d[1] = t_score; d[2] = t_comp; d[7] = t_d - t_0; d[3] = n_win; d[4] = n_bat; d[5] = n_flagged; d[6] = n_cmp; }
    int32_t* out = a.cand + (size_t)q * m;
    if (overflow) {
        if (tid == 0) {
            a.fb_list[atomicAdd(a.fb_count, 1)] = q; a.n_kept[q] = -1; a.tau[q] = key_to_float(T);
            a.qkey[q] = orow0[0];     // first row of its most promising cluster
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
