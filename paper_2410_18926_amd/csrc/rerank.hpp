// Exact re-rank (Sec. 2.2 last step; Sec. 4.1: the ORIGINAL d-dimensional query is used): for each candidate
// row the true dissimilarity of Sec. 2.1 - squared Euclidean distance, negative inner product, or
// 1 - <q, c>/|q| - then the k smallest, ties toward the lower id.
//
// HBM-bound row gather: one block per query, each wavefront streams whole corpus rows with 16-byte loads per
// lane (a row of d floats is contiguous), reduces with shuffles, and the block sorts the m distances in LDS.
#pragma once
#include "common.hpp"

namespace lorann {

constexpr int64_t kPadId = 0x7fffffffffffffffLL;

__device__ __forceinline__ bool rr_less(float da, int64_t ia, float db, int64_t ib) {
    return da < db || (da == db && ia < ib);
}

// grid = 8 * ceil(nq / 8), block = 256, dynamic LDS = d*4 + mp2*(4 + 8) bytes (mp2 = power of two >= m, >= 256).
// METRIC: 0 inner product, 1 squared Euclidean, 2 cosine.
// Queries are taken in the order of `qorder` (grouped by nearest cluster: queries that share candidates run at
// the same time, so a corpus row gathered for one of them is still in cache for the others), and consecutive
// entries of that order go to the same XCD (workgroups are dealt round-robin over the 8 XCDs, each with its own L2).
template <int METRIC>
__global__ __launch_bounds__(256) void k_rerank(const float* __restrict__ Q, const float* __restrict__ corpus,
                                                 const int64_t* __restrict__ ids, const int32_t* __restrict__ cand,
                                                 const int32_t* __restrict__ qorder, int nq,
                                                 int d, int m, int mp2, int k, int64_t* __restrict__ out_ids,
                                                 float* __restrict__ out_dists) {
    extern __shared__ __align__(16) unsigned char smem[];
    int64_t* sid = reinterpret_cast<int64_t*>(smem);                 // [mp2]
    float* sdist = reinterpret_cast<float*>(smem + (size_t)mp2 * 8); // [mp2]
    float* qs = sdist + mp2;                                         // [d]
    __shared__ float s_qnorm;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int per_xcd = (nq + 7) >> 3;
    const int si = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (si >= nq) return;
    const int64_t q = qorder[si];
    const float* qrow = Q + (size_t)q * d;
    for (int i = tid; i < d; i += 256) qs[i] = qrow[i];
    for (int t = tid; t < mp2; t += 256) { sdist[t] = INFINITY; sid[t] = kPadId; }
    __syncthreads();
    if (METRIC == 2) {
        if (wv == 0) {
            float acc = 0.0f;
            for (int i = lane; i < d; i += 64) acc = fmaf(qs[i], qs[i], acc);
            acc = wave_sum_f32(acc);
            if (lane == 0) s_qnorm = sqrtf(acc);
        }
        __syncthreads();
    }
    const int32_t* crow = cand + (size_t)q * m;
    const int d4 = (d % 4 == 0) ? d / 4 : 0;      // vector path needs 16-byte aligned rows

    for (int c = wv; c < m; c += 4) {
        const int row = crow[c];
        if (row < 0) continue;                    // uniform per wavefront
        const float* p = corpus + (size_t)row * d;
        float acc = 0.0f;
        if (d4) {
            const float4* p4 = reinterpret_cast<const float4*>(p);
            const float4* q4 = reinterpret_cast<const float4*>(qs);
            for (int i = lane; i < d4; i += 64) {
                const float4 x = p4[i], y = q4[i];
                if (METRIC == 1) {
                    const float a0 = y.x - x.x, a1 = y.y - x.y, a2 = y.z - x.z, a3 = y.w - x.w;
                    acc = fmaf(a0, a0, acc); acc = fmaf(a1, a1, acc); acc = fmaf(a2, a2, acc); acc = fmaf(a3, a3, acc);
                } else {
                    acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc); acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
                }
            }
        } else {
            for (int i = lane; i < d; i += 64) {
                if (METRIC == 1) { const float t = qs[i] - p[i]; acc = fmaf(t, t, acc); }
                else acc = fmaf(p[i], qs[i], acc);
            }
        }
        acc = wave_sum_f32_lane63(acc);
        if (lane == 63) {
            float dist;
            if (METRIC == 1) dist = acc;
            else if (METRIC == 0) dist = -acc;
            else dist = s_qnorm > 0.0f ? 1.0f - acc / s_qnorm : 1.0f;
            sdist[c] = dist;
            sid[c] = ids ? ids[row] : (int64_t)row;
        }
    }
    __syncthreads();

    // bitonic sort of mp2 (distance, id) pairs, ascending
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
    for (int t = tid; t < k; t += 256) {
        const int64_t id = sid[t];
        out_ids[(size_t)q * k + t] = id == kPadId ? -1 : id;
        out_dists[(size_t)q * k + t] = id == kPadId ? INFINITY : sdist[t];
    }
}

}  // namespace lorann
