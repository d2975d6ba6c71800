// Exact re-rank with shared row gathers (Sec. 2.2 last step; Sec. 4.1: the original d-dimensional query).
//
// The re-rank is a row gather from HBM and dominates the bytes of the whole search.  Queries of one batch that
// fall into the same region of the corpus share many candidates, so
//   k_order_queries : puts the queries in an order in which such queries are neighbours (by nearest cluster,
//                     then by smallest candidate row);
//   k_group_union   : for every group of G consecutive queries forms the union of their candidate rows in an
//                     LDS hash table and writes it out as a list of (row, which queries want it, where each of
//                     them keeps the distance);
//   k_group_gather  : streams the distinct rows - every row is gathered ONCE per group (16-byte loads per lane,
//                     a row is contiguous, several rows in flight per wavefront) and scored against each query
//                     that asked for it; work is cut into many small blocks so the machine stays evenly loaded;
//   k_topk          : per query, the k smallest (distance, id), ties toward the lower id.
// Distances are accumulated exactly as in the one-query-per-block kernel (same per-lane order, same reduction
// across lanes), so both paths return identical bits.
#pragma once
#include <algorithm>

#include "common.hpp"
#include "rerank.hpp"
#include "select_exact.hpp"

namespace lorann {

constexpr int kGroupMax = 16;     // queries per group: 8 or 16 (one 16-bit mask per distinct row)

// Order the queries inside each nearest-cluster segment of `qorder` by `qkey` (their smallest candidate row), so
// that queries with overlapping candidate sets become neighbours.  grid = L, block = 64 (one wavefront per
// cluster).  Segments longer than 1024 queries are copied unchanged (the order is only a locality hint).
__device__ __forceinline__ void order_segment(int c, const int32_t* __restrict__ qorder, const int32_t* __restrict__ off0,
                                              int L, int nq, const int32_t* __restrict__ qkey, int32_t* __restrict__ qorder2) {
    __shared__ int skey[1024], sq[1024];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int beg = off0[c], end = c + 1 < L ? off0[c + 1] : nq;
    const int len = end - beg;
    if (len <= 0) return;                              // uniform over the block
    if (len > 1024) {
        for (int e = tid; e < len; e += nt) qorder2[beg + e] = qorder[beg + e];
        return;
    }
    for (int e = tid; e < len; e += nt) { const int q = qorder[beg + e]; sq[e] = q; skey[e] = qkey[q]; }
    __syncthreads();
    for (int e = tid; e < len; e += nt) {
        const int k = skey[e], q = sq[e];
        int rank = 0;
        for (int u = 0; u < len; ++u) rank += (skey[u] < k || (skey[u] == k && sq[u] < q)) ? 1 : 0;
        qorder2[beg + rank] = q;
    }
}

__global__ __launch_bounds__(64) void k_order_queries(const int32_t* __restrict__ qorder, const int32_t* __restrict__ off0,
                                                      int L, int nq, const int32_t* __restrict__ qkey,
                                                      int32_t* __restrict__ qorder2) {
    order_segment(blockIdx.x, qorder, off0, L, nq, qkey, qorder2);
}

// Two short, mutually independent steps of a batch in ONE launch (every launch is several microseconds of latency in
// the chain of a batch, more when other batches keep the machine busy): blocks [0, fb_blocks) finish, with the exact
// per-query kernel, the queries that the batched selection handed over (usually none); block fb_blocks + c orders the
// queries of nearest-cluster segment c.  grid = fb_blocks + L, block = 256.
template <int RB>
__global__ __launch_bounds__(256) void k_finish_and_order(SelectArgs a, int fb_blocks, const int32_t* __restrict__ qorder,
                                                          const int32_t* __restrict__ off0, int L, int nq,
                                                          const int32_t* __restrict__ qkey, int32_t* __restrict__ qorder2) {
    if ((int)blockIdx.x >= fb_blocks) {                // uniform over the block
        order_segment((int)blockIdx.x - fb_blocks, qorder, off0, L, nq, qkey, qorder2);
        return;
    }
    const int total = *a.qcount;
    if (a.fb_total && blockIdx.x == 0 && threadIdx.x == 0 && total > 0) atomicAdd(a.fb_total, total);
    for (int e = blockIdx.x; e < total; e += fb_blocks) {
        select_exact_query<RB>(a, a.qlist[e]);
        __syncthreads();
    }
}

struct GroupArgs {
    const float* Q;              // [nq][d]
    const void* corpus;          // [n][d] float, or its binary16 copy (the gather kernel's row type says which)
    const int64_t* ids;          // [n] or NULL
    const int32_t* cand;         // [nq][m]
    const int32_t* qorder;       // [nq] visiting order
    int32_t* u_row;              // [ngroups][G*m]    distinct candidate rows of each group
    uint16_t* u_mask;            // [ngroups][G*m]    bit g: query g of the group wants the row
    uint16_t* u_pos;             // [ngroups][G*m][G] where query g keeps the distance of that row
    int32_t* u_count;            // [ngroups]         number of distinct rows
    float* dist;                 // [nq][m]  exact dissimilarities, in the query's own slot order
    int64_t* cid;                // [nq][m]  id of the row in each slot
    int32_t* ccount;             // [nq]     slots in use
    int64_t* out_ids;            // [nq][k]
    float* out_dists;            // [nq][k]
    int nq, d, m, k;
    int ht;                      // hash table slots (rerank_group_ht)
    int slices;                  // gather blocks per group
    int gq;                      // queries per group in this launch, <= G (the buffers keep their G-wide strides)
};

inline int rerank_group_ht(int G, int m) {      // hash table slots: power of two, load factor <= 0.8
    int ht = 16;
    while (ht * 4 < G * m * 5) ht <<= 1;
    return ht;
}

// Queries per group for rows of d floats: 8 when their copies fit 48 KB of LDS (0: they do not).  Groups of 16
// (the kernels take either) move 15 % fewer bytes on the 768-d benchmark but were measured slower overall: the
// union costs twice as much and only three 512-thread gather blocks fit a CU.
inline int rerank_group_size(int d) {
    return (size_t)8 * d * 4 <= 48 * 1024 ? 8 : 0;
}

// grid = ngroups, block = kUnionThreads, dynamic LDS = ht * 6 bytes.  G = queries per group.  All groups are
// resident at once (blocks of 1024 threads were measured: not faster).
constexpr int kUnionThreads = 256;
template <int G>
__global__ __launch_bounds__(kUnionThreads) void k_group_union(GroupArgs a) {
    constexpr int kGroupQ = G;
    extern __shared__ __align__(16) unsigned char smem[];
    const int ht = a.ht, m = a.m;
    int32_t* tkey = reinterpret_cast<int32_t*>(smem);              // [ht]
    uint32_t* tmask = reinterpret_cast<uint32_t*>(tkey + ht);      // [ht/2], 16 bits per slot
    __shared__ int s_q[kGroupQ], s_rcount[kGroupQ], s_nuniq;
    const int tid = threadIdx.x;
    const int grp = blockIdx.x;
    const int g0 = grp * a.gq;
    const int ng = min(a.gq, a.nq - g0);
    if (tid < kGroupQ) { s_q[tid] = tid < ng ? a.qorder[g0 + tid] : -1; s_rcount[tid] = 0; }
    if (tid == 0) s_nuniq = 0;
    for (int s = tid; s < ht; s += kUnionThreads) tkey[s] = -1;
    for (int s = tid; s < ht / 2; s += kUnionThreads) tmask[s] = 0u;
    __syncthreads();
    // open addressing, key = row, one 16-bit mask per slot (bit g: query g wants the row)
    for (int t0 = 0; t0 < ng * m; t0 += kUnionThreads * 8) {
        int rows[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {            // eight candidates per thread requested together (clamped addresses)
            const int t = min(t0 + kUnionThreads * u + tid, ng * m - 1);
            const int g = t / m;
            rows[u] = a.cand[(size_t)s_q[g] * m + (t - g * m)];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int t = t0 + kUnionThreads * u + tid;
            const int row = rows[u];
            if (t >= ng * m || row < 0) continue;
            const int g = t / m;
            uint32_t h = ((uint32_t)row * 2654435761u) >> 7;
            for (;;) {
                h &= (uint32_t)(ht - 1);
                const int old = atomicCAS(&tkey[h], -1, row);
                if (old == -1 || old == row) { atomicOr(&tmask[h >> 1], (1u << g) << (16 * (h & 1))); break; }
                ++h;
            }
        }
    }
    __syncthreads();
    const size_t gbase = (size_t)grp * kGroupQ * m;
    for (int s0 = 0; s0 < ht; s0 += kUnionThreads * 8) {
        int rowv[8];
        int64_t idv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {            // the ids of eight table slots per thread requested together
            const int s = s0 + kUnionThreads * u + tid;
            rowv[u] = s < ht ? tkey[s] : -1;
            idv[u] = a.ids ? a.ids[max(rowv[u], 0)] : (int64_t)rowv[u];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int s = s0 + kUnionThreads * u + tid;
            const int row = rowv[u];
            if (row == -1) continue;
            const uint32_t mk = (tmask[s >> 1] >> (16 * (s & 1))) & 0xffffu;
            const int at = atomicAdd(&s_nuniq, 1);
            a.u_row[gbase + at] = row;
            a.u_mask[gbase + at] = (uint16_t)mk;
            for (int g = 0; g < ng; ++g) {
                if (!((mk >> g) & 1u)) continue;
                const int pos = atomicAdd(&s_rcount[g], 1);
                a.u_pos[(gbase + at) * kGroupQ + g] = (uint16_t)pos;
                a.cid[(size_t)s_q[g] * m + pos] = idv[u];
            }
        }
    }
    __syncthreads();
    if (tid == 0) a.u_count[grp] = s_nuniq;
    if (tid < ng) a.ccount[s_q[tid]] = s_rcount[tid];
}

constexpr int kGatherThreads = 512, kGatherWaves = kGatherThreads / 64;

// grid = ngroups * slices, block = kGatherThreads, dynamic LDS = G * d * 4 bytes (G = queries per group).
// METRIC: 0 inner product, 1 squared
// Euclidean, 2 cosine.
// NV = number of 64-lane slices of four elements of a row, ceil(d / 256), for rows that live in registers
// (d % 4 == 0, d <= 1024); NV = 0: any d, rows are streamed element by element.
// T = element type of the stored rows: float (16-byte loads per lane) or _Float16 (8-byte loads, twice the rows in
// flight); a lane owns the same four elements of a slice in both, so the arithmetic is the same.
template <int METRIC, int NV, int G, typename T>
__global__ __launch_bounds__(kGatherThreads) void k_group_gather(GroupArgs a) {
    constexpr int kGroupQ = G;
    constexpr int RB = sizeof(T) == 2 ? 4 : 2;                     // rows in flight per wavefront
    using V = typename Row4<T>::type;
    const T* const corpus = static_cast<const T*>(a.corpus);
    extern __shared__ __align__(16) unsigned char smem[];
    float* qs = reinterpret_cast<float*>(smem);                    // [G][d]
    __shared__ int s_q[kGroupQ];
    __shared__ float s_qnorm[kGroupQ];
    const int d = a.d, m = a.m;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int grp = blockIdx.x / a.slices, sl = blockIdx.x - grp * a.slices;
    const int g0 = grp * a.gq;
    const int ng = min(a.gq, a.nq - g0);
    const int nuniq = a.u_count[grp];
    const int per = (nuniq + a.slices - 1) / a.slices;
    const int ubeg = sl * per, uend = min(nuniq, ubeg + per);
    if (ubeg >= uend) return;
    if (tid < kGroupQ) s_q[tid] = tid < ng ? a.qorder[g0 + tid] : -1;
    __syncthreads();
    if (d % 4 == 0) {       // one flat loop over the float4 of all the group's queries: the loads are independent
        const int q4n = d / 4;
#pragma unroll 4
        for (int t = tid; t < ng * q4n; t += kGatherThreads) {
            const int g = t / q4n, i = t - g * q4n;
            reinterpret_cast<float4*>(qs)[t] = reinterpret_cast<const float4*>(a.Q + (size_t)s_q[g] * d)[i];
        }
    } else {
        for (int t = tid; t < ng * d; t += kGatherThreads) {
            const int g = t / d, i = t - g * d;
            qs[t] = a.Q[(size_t)s_q[g] * d + i];
        }
    }
    __syncthreads();
    if (METRIC == 2) {
        if (tid < 64) {
            for (int g = 0; g < ng; ++g) {
                float acc = 0.0f;
                for (int i = lane; i < d; i += 64) acc = fmaf(qs[(size_t)g * d + i], qs[(size_t)g * d + i], acc);
                acc = wave_sum_f32(acc);
                if (lane == 0) s_qnorm[g] = sqrtf(acc);
            }
        }
        __syncthreads();
    }
    const size_t gbase = (size_t)grp * kGroupQ * m;
    const int d4 = (d % 4 == 0) ? d / 4 : 0;      // vector path needs 16-byte aligned rows
    auto emit = [&](int g, int pos, float acc) {  // one lane of the wavefront records one (query, row) distance
        float dist;
        if (METRIC == 1) dist = acc;
        else if (METRIC == 0) dist = -acc;
        else dist = s_qnorm[g] > 0.0f ? 1.0f - acc / s_qnorm[g] : 1.0f;
        a.dist[(size_t)s_q[g] * m + pos] = dist;
    };
    if (NV > 0) {
        // RB rows are fetched before any is used.  Every load below is unconditional (indices clamped into the
        // row / the list instead of branching around the load), so the loads of all RB rows are in flight together.
        int nrow[RB], nps[RB];
        uint32_t nmk[RB];
        auto fetch_meta = [&](int u0) {           // (row, mask, slots) of the next RB rows, one iteration ahead
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int u = u0 + r;
                const size_t uc = gbase + min(u, uend - 1);
                const int rw = a.u_row[uc];
                const uint32_t mkk = a.u_mask[uc];
                nps[r] = a.u_pos[uc * kGroupQ + (lane & (kGroupQ - 1))];   // lane l keeps the slot of query l % G
                nrow[r] = u < uend ? rw : 0;
                nmk[r] = u < uend ? mkk : 0u;
            }
        };
        fetch_meta(ubeg + wv * RB);
        for (int u0 = ubeg + wv * RB; u0 < uend; u0 += kGatherWaves * RB) {
            V x[RB][NV > 0 ? NV : 1];
            int ps[RB];
            uint32_t mk[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                mk[r] = nmk[r]; ps[r] = nps[r];
                const V* p4 = reinterpret_cast<const V*>(corpus + (size_t)nrow[r] * d);
#pragma unroll
                for (int v = 0; v < NV; ++v) x[r][v] = row_load(p4 + min(lane + 64 * v, d4 - 1));
            }
            fetch_meta(u0 + kGatherWaves * RB);
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                uint32_t todo = __builtin_amdgcn_readfirstlane(mk[r]);     // uniform: the queries that want this row
                while (todo) {
                    const int g = __builtin_ctz(todo);
                    todo &= todo - 1u;
                    const float4* q4 = reinterpret_cast<const float4*>(qs + (size_t)g * d);
                    float acc = 0.0f;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        if (v + 1 < NV || lane + 64 * v < d4) {            // only the last slice can be partial
                            const float4 y = q4[lane + 64 * v], xv = widen4(x[r][v]);
                            if (METRIC == 1) {
                                const float a0 = y.x - xv.x, a1 = y.y - xv.y, a2 = y.z - xv.z, a3 = y.w - xv.w;
                                acc = fmaf(a0, a0, acc); acc = fmaf(a1, a1, acc); acc = fmaf(a2, a2, acc); acc = fmaf(a3, a3, acc);
                            } else {
                                acc = fmaf(xv.x, y.x, acc); acc = fmaf(xv.y, y.y, acc); acc = fmaf(xv.z, y.z, acc); acc = fmaf(xv.w, y.w, acc);
                            }
                        }
                    }
                    acc = wave_sum_f32_lane63(acc);
                    const int pos = __builtin_amdgcn_readlane(ps[r], g);
                    if (lane == 63) emit(g, pos, acc);
                }
            }
        }
    } else {
        for (int u = ubeg + wv; u < uend; u += kGatherWaves) {
            const int row = a.u_row[gbase + u];
            const uint32_t mk = a.u_mask[gbase + u];
            const T* p = corpus + (size_t)row * d;
            for (int g = 0; g < ng; ++g) {
                if (!((mk >> g) & 1u)) continue;
                const float* qg = qs + (size_t)g * d;
                float acc = 0.0f;
                if (d4) {
                    const V* p4 = reinterpret_cast<const V*>(p);
                    const float4* q4 = reinterpret_cast<const float4*>(qg);
                    for (int i = lane; i < d4; i += 64) {
                        const float4 x = widen4(row_load(p4 + i)), y = q4[i];
                        if (METRIC == 1) {
                            const float a0 = y.x - x.x, a1 = y.y - x.y, a2 = y.z - x.z, a3 = y.w - x.w;
                            acc = fmaf(a0, a0, acc); acc = fmaf(a1, a1, acc); acc = fmaf(a2, a2, acc); acc = fmaf(a3, a3, acc);
                        } else {
                            acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc); acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
                        }
                    }
                } else {
                    for (int i = lane; i < d; i += 64) {
                        const float x = widen1(p[i]);
                        if (METRIC == 1) { const float t = qg[i] - x; acc = fmaf(t, t, acc); }
                        else acc = fmaf(x, qg[i], acc);
                    }
                }
                acc = wave_sum_f32_lane63(acc);
                if (lane == 63) emit(g, a.u_pos[(gbase + u) * kGroupQ + g], acc);
            }
        }
    }
}

// The k smallest (distance, id) of each query, one WAVEFRONT per query, candidates in registers (EPL per lane,
// m <= 64 * EPL): k rounds of "take the wavefront-wide minimum and retire it".  For k much smaller than m this is
// far cheaper than sorting.  A round is one minimum over order-preserving distance keys (data-parallel moves, no
// LDS traffic) and a ballot; only when several lanes hold that distance are their ids compared.
// grid = ceil(nq / 4), block = 256.
template <int EPL>
__device__ __forceinline__ void topk_wave_query(const GroupArgs& a, int64_t q, int cnt) {
    const int lane = threadIdx.x & 63;
    uint32_t kv[EPL];                       // order-preserving key of the distance; 0xFFFFFFFF = retired / padding
    int64_t iv[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {         // clamped addresses: the loads go out together
        const int t = min(64 * e + lane, max(cnt - 1, 0));
        kv[e] = __float_as_uint(a.dist[(size_t)q * a.m + t]);
        iv[e] = a.cid[(size_t)q * a.m + t];
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const bool in = 64 * e + lane < cnt;
        // a NaN distance would map to a key above +inf's: clamp to +inf's key so that 0xFFFFFFFF stays reserved
        kv[e] = in ? min(float_key_asc(__uint_as_float(kv[e])), float_key_asc(INFINITY)) : 0xFFFFFFFFu;
        iv[e] = in ? iv[e] : kPadId;
    }
    for (int r = 0; r < a.k; ++r) {
        uint32_t bk = kv[0];
        int64_t bi = iv[0];
#pragma unroll
        for (int e = 1; e < EPL; ++e)
            if (kv[e] < bk || (kv[e] == bk && iv[e] < bi)) { bk = kv[e]; bi = iv[e]; }
        const uint32_t wk = wave_min_u32(bk);
        int64_t wi = kPadId;
        if (wk != 0xFFFFFFFFu) {                                           // uniform
            const unsigned long long holders = __ballot(bk == wk);
            int src = __ffsll((unsigned long long)holders) - 1;
            if (holders & (holders - 1ull)) {                              // several lanes tie on the distance: lowest id
                int64_t mi = bk == wk ? bi : kPadId;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) { const int64_t oi = __shfl_xor(mi, o, 64); mi = oi < mi ? oi : mi; }
                src = __ffsll((unsigned long long)__ballot(bk == wk && bi == mi)) - 1;
            }
            wi = __shfl(bi, src, 64);
            if (lane == src) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (iv[e] == wi && kv[e] == wk) { kv[e] = 0xFFFFFFFFu; iv[e] = kPadId; }
            }
        }
        if (lane == 0) {
            a.out_ids[(size_t)q * a.k + r] = wi == kPadId ? -1 : wi;
            a.out_dists[(size_t)q * a.k + r] = wi == kPadId ? INFINITY : key_to_float(wk);
        }
    }
}

template <int EPL>
__global__ __launch_bounds__(256) void k_topk_wave(GroupArgs a) {
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= a.nq) return;
    topk_wave_query<EPL>(a, q, a.ccount[q]);
}

// The k smallest (distance, id) of each query: bitonic sort in LDS.  grid = nq, block = 256,
// dynamic LDS = mp2 * 12 bytes (mp2 = power of two >= m, >= 256).
__global__ __launch_bounds__(256) void k_topk(GroupArgs a, int mp2) {
    extern __shared__ __align__(16) unsigned char smem[];
    int64_t* sid = reinterpret_cast<int64_t*>(smem);
    float* sdist = reinterpret_cast<float*>(sid + mp2);
    const int tid = threadIdx.x;
    const int64_t q = blockIdx.x;
    const int cnt = a.ccount[q];
    for (int t = tid; t < mp2; t += 256) {
        if (t < cnt) { sdist[t] = a.dist[(size_t)q * a.m + t]; sid[t] = a.cid[(size_t)q * a.m + t]; }
        else { sdist[t] = INFINITY; sid[t] = kPadId; }
    }
    __syncthreads();
    for (int size = 2; size <= mp2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < (mp2 >> 1); t += 256) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const float dl = sdist[lo], dh = sdist[hi];
                const int64_t il = sid[lo], ih = sid[hi];
                const bool swap = up ? rr_less(dh, ih, dl, il) : rr_less(dl, il, dh, ih);
                if (swap) { sdist[lo] = dh; sdist[hi] = dl; sid[lo] = ih; sid[hi] = il; }
            }
            __syncthreads();
        }
    }
    for (int t = tid; t < a.k; t += 256) {
        const int64_t id = sid[t];
        a.out_ids[(size_t)q * a.k + t] = id == kPadId ? -1 : id;
        a.out_dists[(size_t)q * a.k + t] = id == kPadId ? INFINITY : sdist[t];
    }
}

// Re-rank and top-k of a SMALL batch in one launch: a query's candidates are distinct rows, so no union is needed;
// `slices` blocks per query each take a run of its candidate list (one wavefront per row, two rows in flight, the
// query's elements in registers), write distances and ids at the candidates' own positions, and the block that
// finishes a query last - a ticket per query, device-scope fences around it: a handful of blocks, not the thousands for
// which such fences are ruinous - orders the query's results with the wavefront top-k.  The distance arithmetic is that
// of k_group_gather, lane for lane (same element ownership, same order, same reduction): bit-identical results.
// grid = nq * slices, block = 256.  done [nq]: zero on entry.  NV = ceil(d / 256) <= 4, d % 4 == 0; m <= 64 * EPL.
template <int METRIC, int NV, typename T, int EPL>
__global__ __launch_bounds__(256) void k_small_rerank(GroupArgs a, int slices, int32_t* __restrict__ done) {
    using V = typename Row4<T>::type;
    __shared__ int s_last;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int q = (int)blockIdx.x / slices, sl = (int)blockIdx.x - q * slices;
    const int d = a.d, d4 = d >> 2, m = a.m;
    const int per = (m + slices - 1) / slices;
    const int t_beg = sl * per, t_end = min(m, t_beg + per);
    const T* corpus = reinterpret_cast<const T*>(a.corpus);
    const float4* q4 = reinterpret_cast<const float4*>(a.Q + (size_t)q * d);
    float4 y[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) y[v] = q4[min(lane + 64 * v, d4 - 1)];
    float qn = 0.0f;
    if (METRIC == 2) {
        float acc = 0.0f;
        for (int i = lane; i < d; i += 64) acc = fmaf(a.Q[(size_t)q * d + i], a.Q[(size_t)q * d + i], acc);
        qn = sqrtf(wave_sum_f32(acc));
    }
    for (int t0 = t_beg + wv; t0 < t_end; t0 += 8) {
        int row[2];
        V x[2][NV];
#pragma unroll
        for (int u = 0; u < 2; ++u) {                       // clamped: a repeat of the run's last candidate, not stored
            row[u] = a.cand[(size_t)q * m + min(t0 + 4 * u, t_end - 1)];
            const V* p4 = reinterpret_cast<const V*>(corpus + (size_t)max(row[u], 0) * d);
#pragma unroll
            for (int v = 0; v < NV; ++v) x[u][v] = row_load(p4 + min(lane + 64 * v, d4 - 1));
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int t = t0 + 4 * u;
            if (t >= t_end || row[u] < 0) continue;         // uniform over the wavefront
            float acc = 0.0f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if (v + 1 < NV || lane + 64 * v < d4) {
                    const float4 yy = y[v], xv = widen4(x[u][v]);
                    if (METRIC == 1) {
                        const float a0 = yy.x - xv.x, a1 = yy.y - xv.y, a2 = yy.z - xv.z, a3 = yy.w - xv.w;
                        acc = fmaf(a0, a0, acc); acc = fmaf(a1, a1, acc); acc = fmaf(a2, a2, acc); acc = fmaf(a3, a3, acc);
                    } else {
                        acc = fmaf(xv.x, yy.x, acc); acc = fmaf(xv.y, yy.y, acc); acc = fmaf(xv.z, yy.z, acc); acc = fmaf(xv.w, yy.w, acc);
                    }
                }
            }
            acc = wave_sum_f32_lane63(acc);
            if (lane == 63) {
                float dist;
                if (METRIC == 1) dist = acc;
                else if (METRIC == 0) dist = -acc;
                else dist = qn > 0.0f ? 1.0f - acc / qn : 1.0f;
                a.dist[(size_t)q * m + t] = dist;
                a.cid[(size_t)q * m + t] = a.ids ? a.ids[row[u]] : (int64_t)row[u];
            }
        }
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = atomicAdd(&done[q], 1) == slices - 1 ? 1 : 0;
    __syncthreads();
    if (!s_last || wv != 0) return;
    __threadfence();
    int cnt = 0;                                             // valid candidates come first
    for (int t = lane; t < m; t += 64) cnt += a.cand[(size_t)q * m + t] >= 0 ? 1 : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    topk_wave_query<EPL>(a, q, cnt);
}

}  // namespace lorann
