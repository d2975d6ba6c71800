// Routing-side kernels: absmax quantization of the projected queries (Sec. 3.3), selection of the w nearest
// centroids per query (Sec. 2.2), and the counting sort that groups (query, cluster) pairs by cluster so that
// each cluster's factors are read once per batch.
#pragma once
#include "common.hpp"

namespace lorann {

// ---- Sec. 3.3: x_i8 = round(c_x x), c_x = 127 / |x|_inf; step size Delta_x = |x|_inf / 127. ----
// One wavefront per query row; block = 256 (4 rows).  Round-half-to-even, codes clamped to [-127, 127];
// a zero row gives zero codes and step 0.  The quotients are formed in double and rounded once, which equals
// IEEE float division.  The first blocks also clear the `nzero` counters of the counting sorts that follow.
// qb (optional): the row rounded to bfloat16, for the approximate centroid scores.
// first = 1 (Sec. 4.2 mixed-precision decomposition): component 0 is not quantized - it takes no part in the
// maximum and its code is 0, so that the integer products that follow skip it; first = 0 otherwise.
__global__ __launch_bounds__(256) void k_quantize_rows(const float* __restrict__ qp, int8_t* __restrict__ q8,
                                                        float* __restrict__ dx, int nq, int dp,
                                                        int32_t* __restrict__ zero, int nzero, __bf16* __restrict__ qb,
                                                        int first) {
    for (int i = blockIdx.x * 256 + threadIdx.x; i < nzero; i += gridDim.x * 256) zero[i] = 0;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nq) return;
    const float* p = qp + (size_t)row * dp;
    float a = 0.0f;
    for (int i = lane; i < dp; i += 64) {
        const float x = p[i];
        if (i >= first) a = fmaxf(a, fabsf(x));
        if (qb) qb[(size_t)row * dp + i] = (__bf16)x;
    }
    a = wave_max_f32(a);
    int8_t* o = q8 + (size_t)row * dp;
    if (!(a > 0.0f)) {
        for (int i = lane; i < dp; i += 64) o[i] = 0;
        if (lane == 0) dx[row] = 0.0f;
        return;
    }
    const float cx = (float)(127.0 / (double)a);
    for (int i = lane; i < dp; i += 64) {
        int v = (int)rintf(__fmul_rn(p[i], cx));
        v = max(-127, min(127, v));
        o[i] = (int8_t)(i >= first ? v : 0);
    }
    if (lane == 0) dx[row] = (float)((double)a / 127.0);
}

// ---- Sec. 2.2: tau(x) = the w centroids of smallest dissimilarity. ----
// Block-wide exact selection over one row of dissimilarities (256 threads; every thread of the block calls it).
// 4-pass radix select on order-preserving keys, ties at the threshold resolved toward the lower cluster id;
// the result is written ordered (dissimilarity ascending, cluster id ascending).  Reads the row five times.
__device__ __forceinline__ void select_clusters_radix(const float* __restrict__ row, int L, int w, int32_t* __restrict__ out) {
    __shared__ int hist[256];
    __shared__ int wsum[4];
    __shared__ uint32_t s_prefix;
    __shared__ int s_need;
    __shared__ uint32_t selk[256];
    __shared__ int seli[256];
    __shared__ int s_nless;
    const int tid = threadIdx.x;

    __syncthreads();
    if (tid == 0) { s_prefix = 0u; s_need = w; s_nless = 0; }
    uint32_t mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        for (int l = tid; l < L; l += 256) {
            const uint32_t key = float_key_asc(row[l]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid < 64) {   // first wavefront: find the digit where the ascending cumulative count reaches need
            const int need = s_need;
            const int h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
            const int mine = h0 + h1 + h2 + h3;
            int incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (tid >= o) incl += t; }
            const int excl = incl - mine;
            if (excl < need && incl >= need) {
                int cum = excl, dgt = 4 * tid;
                if (cum + h0 >= need) { dgt += 0; }
                else { cum += h0; if (cum + h1 >= need) { dgt += 1; } else { cum += h1; if (cum + h2 >= need) { dgt += 2; } else { cum += h2; dgt += 3; } } }
                s_prefix = prefix | ((uint32_t)dgt << shift);
                s_need = need - cum;      // still to take among keys with this longer prefix
            }
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    // s_prefix = key of the w-th smallest; s_need of the keys equal to it are taken, lowest cluster id first.
    const uint32_t T = s_prefix;
    const int need_ties = s_need;
    const int n_less = w - need_ties;
    int tie_base = 0;
    for (int l0 = 0; l0 < L; l0 += 256) {
        const int l = l0 + tid;
        uint32_t key = 0xFFFFFFFFu;
        bool in = l < L;
        if (in) key = float_key_asc(row[l]);
        const bool less = in && key < T;
        const bool tie = in && key == T;
        if (less) { const int p = atomicAdd(&s_nless, 1); selk[p] = key; seli[p] = l; }
        int tot;
        const int rank = block_flag_scan<4>(tie, wsum, tot);
        if (tie && tie_base + rank < need_ties) { selk[n_less + tie_base + rank] = key; seli[n_less + tie_base + rank] = l; }
        tie_base += tot;
    }
    __syncthreads();
    if (tid < w) {   // order the w selected by (key, id): rank by counting
        const uint32_t k = selk[tid];
        const int id = seli[tid];
        int rank = 0;
        for (int u = 0; u < w; ++u) {
            const uint32_t ku = selk[u];
            const int iu = seli[u];
            rank += (ku < k || (ku == k && iu < id)) ? 1 : 0;
        }
        out[rank] = id;
    }
}

// One block (256 threads) per query, any L.  g [nq][L] holds the centroid dissimilarities.
__global__ __launch_bounds__(256) void k_select_clusters(const float* __restrict__ g, int L, int w,
                                                          int32_t* __restrict__ sel) {
    select_clusters_radix(g + (size_t)blockIdx.x * L, L, w, sel + (size_t)blockIdx.x * w);
}

// One block per query with the row read ONCE into registers (KPT keys per thread, 256 * KPT >= L, L >= 256, w <= 256).
// The w-th smallest of the 256 per-thread minima bounds the w-th smallest key from above (w distinct keys do
// not exceed it), so only the keys up to that bound - a few more than w when the row is in no special order -
// are collected into LDS and ranked exactly by (key, cluster id).  A row whose keys up to the bound do not fit
// (long runs of equal keys, adversarial order) is selected by the radix routine instead.
template <int KPT>
__global__ __launch_bounds__(256) void k_select_clusters_regs(const float* __restrict__ g, int L, int w,
                                                               int32_t* __restrict__ sel) {
    constexpr int CAP = 2048;
    // (key, position) packed into one 64-bit word: a single unsigned compare orders by key, then position
    __shared__ __align__(16) unsigned long long tmin[256];
    __shared__ __align__(16) unsigned long long cand[CAP + 2];
    __shared__ int s_cnt;
    __shared__ uint32_t s_bound;
    const int tid = threadIdx.x;
    const float* row = g + (size_t)blockIdx.x * L;
    int32_t* out = sel + (size_t)blockIdx.x * w;
    uint32_t key[KPT];
    uint32_t mn = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < KPT; ++i) key[i] = __float_as_uint(row[min(i * 256 + tid, L - 1)]);   // independent loads, all in flight
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        key[i] = i * 256 + tid < L ? float_key_asc(__uint_as_float(key[i])) : 0xFFFFFFFFu;
        mn = min(mn, key[i]);
    }
    const unsigned long long mine = ((unsigned long long)mn << 32) | (unsigned)tid;
    tmin[tid] = mine;
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    int rank = 0;
    {
        const ulonglong2* t2 = reinterpret_cast<const ulonglong2*>(tmin);
#pragma unroll 16
        for (int u = 0; u < 128; ++u) {
            const ulonglong2 t = t2[u];
            rank += (t.x < mine ? 1 : 0) + (t.y < mine ? 1 : 0);
        }
    }
    if (rank == w - 1) s_bound = mn;
    __syncthreads();
    const uint32_t bound = s_bound;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int l = i * 256 + tid;
        if (l < L && key[i] <= bound) {
            const int p = atomicAdd(&s_cnt, 1);
            if (p < CAP) cand[p] = ((unsigned long long)key[i] << 32) | (unsigned)l;
        }
    }
    __syncthreads();
    const int c = s_cnt;
    if (c > CAP) {          // uniform over the block
        select_clusters_radix(row, L, w, out);
        return;
    }
    if (tid < 2) cand[c + tid] = ~0ull;      // pad to a whole 16-byte read
    __syncthreads();
    const ulonglong2* c2 = reinterpret_cast<const ulonglong2*>(cand);
    const int c_pairs = (c + 1) >> 1;
    for (int e = tid; e < c; e += 256) {
        const unsigned long long me = cand[e];
        int r = 0;
#pragma unroll 8
        for (int u = 0; u < c_pairs; ++u) {
            const ulonglong2 t = c2[u];
            r += (t.x < me ? 1 : 0) + (t.y < me ? 1 : 0);
        }
        if (r < w) out[r] = (int)(unsigned)(me & 0xFFFFFFFFull);
    }
}

// The same selection done by ONE WAVEFRONT over keys it holds in registers (KPL keys per lane, element
// l = 64 * i + lane, L <= 64 * KPL, padding = 0xFFFFFFFF): 4-pass radix select with a wavefront-private LDS
// histogram (`hist`, 256 ints); ties at the threshold go to the lower cluster id; the w selected are written to
// `out` ordered by (key, cluster id).  `selk`, `seli`: 256 entries of wavefront-private LDS each.  No block
// barrier inside.
template <int KPL>
__device__ __forceinline__ uint32_t wave_wth_smallest_key(const uint32_t (&key)[KPL], int L, int w, int* hist, int& need_out) {
    const int lane = threadIdx.x & 63;
    uint32_t prefix = 0u, mask = 0u;
    int need = w;
    for (int shift = 24; shift >= 0; shift -= 8) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int b = 0; b < 4; ++b) hist[lane + 64 * b] = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < KPL; ++i)
            if (64 * i + lane < L && (key[i] & mask) == prefix) atomicAdd(&hist[(key[i] >> shift) & 255u], 1);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
        const int mine = h0 + h1 + h2 + h3;
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (lane >= o) incl += t; }
        const int excl = incl - mine;
        const bool owner = excl < need && incl >= need;
        int cum = excl, dgt = 4 * lane;
        if (owner) {
            if (cum + h0 >= need) { }
            else { cum += h0; if (cum + h1 >= need) { dgt += 1; } else { cum += h1; if (cum + h2 >= need) { dgt += 2; } else { cum += h2; dgt += 3; } } }
        }
        const int src = __ffsll((unsigned long long)__ballot(owner)) - 1;      // exactly one owner lane
        dgt = __shfl(dgt, src, 64);
        cum = __shfl(cum, src, 64);
        prefix |= (uint32_t)dgt << shift;
        need -= cum;
        mask |= 255u << shift;
    }
    need_out = need;       // how many of the keys equal to the result belong to the w smallest
    return prefix;
}

template <int KPL>
__device__ __forceinline__ void wave_select_from_keys(const uint32_t (&key)[KPL], int L, int w, int32_t* __restrict__ out,
                                                      int* hist, uint32_t* selk, int* seli) {
    const int lane = threadIdx.x & 63;
    int need;
    const uint32_t T = wave_wth_smallest_key<KPL>(key, L, w, hist, need);
    // `need` of the keys equal to T are taken, lowest cluster id first
    int n_out = 0, ties_left = need;
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const int l = 64 * i + lane;
        const bool in = l < L;
        const bool less = in && key[i] < T;
        const bool tie = in && key[i] == T;
        const unsigned long long ml = __ballot(less), mt = __ballot(tie);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (less) { const int p = n_out + __popcll(ml & below); selk[p] = key[i]; seli[p] = l; }
        n_out += __popcll(ml);
        const int trank = __popcll(mt & below);
        if (tie && trank < ties_left) { const int p = n_out + trank; selk[p] = key[i]; seli[p] = l; }
        const int took = min(ties_left, __popcll(mt));
        n_out += took;
        ties_left -= took;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int t = lane; t < w; t += 64) {       // order the w selected by (key, id): rank by counting
        const uint32_t k = selk[t];
        const int id = seli[t];
        int rank = 0;
        for (int u = 0; u < w; ++u) {
            const uint32_t ku = selk[u];
            const int iu = seli[u];
            rank += (ku < k || (ku == k && iu < id)) ? 1 : 0;
        }
        out[rank] = id;
    }
}

// One WAVEFRONT per query with the row of dissimilarities read once into registers: no re-reading of the scores
// and no block barriers.  grid = ceil(nq / 4), block = 256 (4 queries per block).
template <int KPL>
__global__ __launch_bounds__(256) void k_select_clusters_wave(const float* __restrict__ g, int nq, int L, int w,
                                                               int32_t* __restrict__ sel) {
    __shared__ int hist[4][256];
    __shared__ uint32_t selk[4][256];
    __shared__ int seli[4][256];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int q = blockIdx.x * 4 + wv;
    if (q >= nq) return;                       // wavefronts are independent: no block barrier below
    const float* row = g + (size_t)q * L;
    uint32_t key[KPL];                         // element l = 64 * i + lane
#pragma unroll
    for (int i = 0; i < KPL; ++i) key[i] = __float_as_uint(row[min(64 * i + lane, L - 1)]);   // independent loads, all in flight
#pragma unroll
    for (int i = 0; i < KPL; ++i)       // padding sorts last (and is never selected: w <= L)
        key[i] = 64 * i + lane < L ? float_key_asc(__uint_as_float(key[i])) : 0xFFFFFFFFu;
    wave_select_from_keys<KPL>(key, L, w, sel + (size_t)q * w, hist[wv], selk[wv], seli[wv]);
}

// ---- Counting sort, step 1: count the pairs of every cluster. ----
// Two sorts share the machinery: (query, cluster) pairs by cluster, and queries by their nearest cluster (the
// order in which the re-rank visits them).  Each block takes kBucketQueries queries, histograms their pairs in
// LDS (the old value of the LDS counter is the pair's rank among the block's pairs of that cluster), then adds
// each non-zero LDS count to the global counter once; the value that add returns is the block's offset inside
// the cluster's bucket.  Global atomics per cluster drop from one per pair to one per block.
// grid = ceil(nq / kBucketQueries), block = 1024, dynamic LDS = 8 * L bytes.
constexpr int kBucketQueries = 256;
__global__ __launch_bounds__(1024) void k_bucket_count(const int32_t* __restrict__ sel, int nq, int w, int L,
                                                        int32_t* __restrict__ count, int32_t* __restrict__ count0,
                                                        int32_t* __restrict__ rank_in_bucket, int32_t* __restrict__ qrank,
                                                        int32_t* __restrict__ base_tab, int32_t* __restrict__ base0_tab) {
    extern __shared__ int lh[];          // [L] pairs per cluster, [L] nearest-cluster queries per cluster
    int* lh0 = lh + L;
    const int tid = threadIdx.x;
    for (int c = tid; c < 2 * L; c += 1024) lh[c] = 0;
    __syncthreads();
    const int q0 = blockIdx.x * kBucketQueries;
    const int q1 = min(nq, q0 + kBucketQueries);
    const int64_t p0 = (int64_t)q0 * w, p1 = (int64_t)q1 * w;
    for (int64_t p = p0 + tid; p < p1; p += 1024) {
        const int c = sel[p];
        rank_in_bucket[p] = atomicAdd(&lh[c], 1);
        if (p % w == 0) qrank[p / w] = atomicAdd(&lh0[c], 1);
    }
    __syncthreads();
    for (int c = tid; c < L; c += 1024) {
        const int n = lh[c], n0 = lh0[c];
        base_tab[(size_t)blockIdx.x * L + c] = n ? atomicAdd(&count[c], n) : 0;
        base0_tab[(size_t)blockIdx.x * L + c] = n0 ? atomicAdd(&count0[c], n0) : 0;
    }
}

// The same without LDS histograms (cluster counts too large for LDS): one global atomic per pair.
// grid = ceil(npairs / 256), block = 256.  The block offsets are all zero.
__global__ __launch_bounds__(256) void k_bucket_count_global(const int32_t* __restrict__ sel, int64_t npairs, int w,
                                                              int32_t* __restrict__ count, int32_t* __restrict__ count0,
                                                              int32_t* __restrict__ rank_in_bucket, int32_t* __restrict__ qrank) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= npairs) return;
    const int c = sel[p];
    rank_in_bucket[p] = atomicAdd(&count[c], 1);
    if (p % w == 0) qrank[p / w] = atomicAdd(&count0[c], 1);
}

// ---- Counting sort, step 2: exclusive scans over the clusters. ----
// bucket_off[c]  = number of pairs routed to clusters < c                  (bucket_off[L] = number of pairs)
// tile_off[c]    = number of 16-pair tiles of clusters < c                 (tile_off[L]   = number of tiles)
// unit_off[c]    = number of scoring work items of clusters < c            (unit_off[L]   = number of items);
//                  a cluster with a pairs and m_c points has ceil(a / unit_pairs) * ceil(m_c / chunk_points) items
//                  (both powers of two, given as shifts: two integer divisions per cluster are most of this kernel otherwise)
// off0[c]        = number of queries whose nearest cluster is < c
// grid = ceil(L / 1024), block = 1024: block b scans clusters [1024 b, 1024 b + 1024) and first adds up, on its
// own, everything that precedes them (at most L - 1024 independent loads spread over its threads), so the blocks
// need no communication and none of them waits for another.
__global__ __launch_bounds__(1024) void k_scan_buckets(const int32_t* __restrict__ count, const int32_t* __restrict__ count0,
                                                        const int64_t* __restrict__ off, int L, int unit_shift, int chunk_shift,
                                                        int32_t* __restrict__ bucket_off, int32_t* __restrict__ tile_off,
                                                        int32_t* __restrict__ unit_off, int32_t* __restrict__ off0) {
    __shared__ int wtot[4][16], wpre[4][16];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int c0 = blockIdx.x * 1024;
    auto fields = [&](int c, int (&f)[4]) {         // c < L
        const int a = count[c];
        const int m_c = (int)(off[c + 1] - off[c]);
        f[0] = a; f[1] = (a + 15) >> 4;
        f[2] = ((a + (1 << unit_shift) - 1) >> unit_shift) * ((m_c + (1 << chunk_shift) - 1) >> chunk_shift);
        f[3] = count0[c];
    };
    int pre[4] = {0, 0, 0, 0};                      // this thread's share of the clusters before c0
#pragma unroll 8
    for (int c = tid; c < c0; c += 1024) {
        int f[4];
        fields(c, f);
#pragma unroll
        for (int k = 0; k < 4; ++k) pre[k] += f[k];
    }
    const int c = c0 + tid;
    int v[4] = {0, 0, 0, 0};
    if (c < L) fields(c, v);
    int incl[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int x = v[k], y = pre[k];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(x, o, 64);
            if (lane >= o) x += t;
            y += __shfl_xor(y, o, 64);
        }
        incl[k] = x;
        if (lane == 63) wtot[k][wv] = x;
        if (lane == 0) wpre[k][wv] = y;
    }
    __syncthreads();
    int total[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int before = 0, tot = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) { const int t = wtot[k][i]; if (i < wv) before += t; tot += t + wpre[k][i]; before += wpre[k][i]; }
        incl[k] += before - v[k];                   // exclusive, including everything before this block
        total[k] = tot;
    }
    if (c < L) { bucket_off[c] = incl[0]; tile_off[c] = incl[1]; unit_off[c] = incl[2]; off0[c] = incl[3]; }
    if (blockIdx.x == gridDim.x - 1 && tid == 0) { bucket_off[L] = total[0]; tile_off[L] = total[1]; unit_off[L] = total[2]; }
}

// ---- Counting sort, step 3: place every pair (slot = query * w + rank) into its cluster's bucket, at
// bucket start + offset of its block + its rank inside the block (the order inside a bucket is arbitrary; no
// result depends on it).  Also clears the pair's best-score key for the scoring kernels, and places every query
// into the list ordered by nearest cluster.  base_tab == NULL: ranks are already bucket-wide.
// SCAN (L <= 1024): step 2 is done here as well - every block scans the L counters on its own in LDS (16 KB of
// cached reads per block is cheaper than one more kernel in the chain of a batch) and block 0 writes the four
// offset arrays of k_scan_buckets for the kernels that follow; bucket_off / off0 are then outputs.
struct ScanArgs {
    const int32_t* count; const int32_t* count0; const int64_t* off;
    int unit_shift, chunk_shift;      // log2 of the pairs and of the points of a scoring work item
    int32_t* tile_off; int32_t* unit_off;
};
template <bool SCAN>
__global__ __launch_bounds__(256) void k_scatter_pairs(const int32_t* __restrict__ sel, int64_t npairs, int w, int L,
                                                        int32_t* __restrict__ bucket_off, const int32_t* __restrict__ rank_in_bucket,
                                                        int32_t* __restrict__ off0, const int32_t* __restrict__ qrank,
                                                        const int32_t* __restrict__ base_tab, const int32_t* __restrict__ base0_tab,
                                                        int32_t* __restrict__ slot_of_pos, int32_t* __restrict__ pos_of_slot,
                                                        uint32_t* __restrict__ pmax, int32_t* __restrict__ qorder, ScanArgs sc) {
    __shared__ int s_boff[SCAN ? 1024 : 1], s_off0[SCAN ? 1024 : 1];
    __shared__ int wtot[4][4];
    if (SCAN) {
        const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
        int f[4][4], tot[4] = {0, 0, 0, 0};                   // thread t owns clusters 4t .. 4t+3
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = min(4 * tid + j, L - 1);
            const bool in = 4 * tid + j < L;
            const int a = sc.count[c];
            const int m_c = (int)(sc.off[c + 1] - sc.off[c]);
            f[j][0] = in ? a : 0;
            f[j][1] = in ? (a + 15) >> 4 : 0;
            f[j][2] = in ? ((a + (1 << sc.unit_shift) - 1) >> sc.unit_shift) * ((m_c + (1 << sc.chunk_shift) - 1) >> sc.chunk_shift) : 0;
            f[j][3] = in ? sc.count0[c] : 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) tot[k] += f[j][k];
        }
        int incl[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int x = tot[k];
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(x, o, 64); if (lane >= o) x += t; }
            incl[k] = x;
            if (lane == 63) wtot[k][wv] = x;
        }
        __syncthreads();
        int run[4], total[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int before = 0, all = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { const int t = wtot[k][i]; if (i < wv) before += t; all += t; }
            run[k] = incl[k] - tot[k] + before;                 // exclusive prefix of this thread's first cluster
            total[k] = all;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = 4 * tid + j;
            if (c < L) {
                s_boff[c] = run[0]; s_off0[c] = run[3];
                if (blockIdx.x == 0) { bucket_off[c] = run[0]; sc.tile_off[c] = run[1]; sc.unit_off[c] = run[2]; off0[c] = run[3]; }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) run[k] += f[j][k];
        }
        if (blockIdx.x == 0 && tid == 0) { bucket_off[L] = total[0]; sc.tile_off[L] = total[1]; sc.unit_off[L] = total[2]; }
        __syncthreads();
    }
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= npairs) return;                                   // no barrier below
    const int c = sel[p];
    const int q = (int)(p / w);
    const size_t tb = (size_t)(q / kBucketQueries) * L + c;
    const int pos = (SCAN ? s_boff[c] : bucket_off[c]) + (base_tab ? base_tab[tb] : 0) + rank_in_bucket[p];
    slot_of_pos[pos] = (int32_t)p;
    pos_of_slot[p] = pos;
    pmax[p] = 0u;
    if (p % w == 0) qorder[(SCAN ? s_off0[c] : off0[c]) + (base0_tab ? base0_tab[tb] : 0) + qrank[q]] = q;
}

__global__ void k_zero_i32(int32_t* __restrict__ p, int64_t n) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) p[t] = 0;
}

}  // namespace lorann
