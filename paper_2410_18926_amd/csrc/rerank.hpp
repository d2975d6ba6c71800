// Exact re-rank (Sec. 2.2 last step; Sec. 4.1: the ORIGINAL d-dimensional query is used): for each candidate
// row the true dissimilarity of Sec. 2.1 - squared Euclidean distance, negative inner product, or
// 1 - <q, c>/|q| - then the k smallest, ties toward the lower id.
//
// HBM-bound row gather: one block per query, each wavefront streams whole corpus rows with 16-byte loads per
// lane (a row of d floats is contiguous), reduces with shuffles, and the block sorts the m distances in LDS.
//
// The rows are read either from the float corpus or from a half-precision (IEEE binary16) copy of it (Sec. 4.3:
// 16-bit floating point on the GPU); a half is widened exactly and all arithmetic stays in float, element for
// element in the same order, so the two modes differ only by the rounding of the stored rows.
#pragma once
#include "common.hpp"

namespace lorann {

constexpr int64_t kPadId = 0x7fffffffffffffffLL;

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
template <typename T> struct Row4 { using type = float4; };          // four consecutive row elements as stored
template <> struct Row4<_Float16> { using type = f16x4; };
__device__ __forceinline__ float4 widen4(const float4& v) { return v; }
__device__ __forceinline__ float4 widen4(const f16x4& v) { return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]); }
__device__ __forceinline__ float widen1(float v) { return v; }
__device__ __forceinline__ float widen1(_Float16 v) { return (float)v; }

// A corpus row is read once per group of queries (once per query in the one-query-per-block kernel): it is loaded
// as streaming data (non-temporal), so that the gather does not evict what it re-reads itself (queries, row lists)
// and what the other kernels - of this batch and of the batches on other lanes - keep in the caches.
// Measured on the 768-d benchmark: 563 -> 531 us per launch of the grouped gather.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 row_load(const float4* p) {
    const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
    return make_float4(t[0], t[1], t[2], t[3]);
}
__device__ __forceinline__ f16x4 row_load(const f16x4* p) {
    return __builtin_nontemporal_load(p);
}

// The half-precision copy of the corpus: round to nearest even.  *max_abs_bits receives the largest |x| seen (as
// float bits; a NaN compares above everything) so that the host can refuse rows binary16 cannot hold.
// grid-stride over count elements, block = 256.
__global__ __launch_bounds__(256) void k_corpus_to_half(const float* __restrict__ src, _Float16* __restrict__ dst, size_t count,
                                                         uint32_t* __restrict__ max_abs_bits) {
    uint32_t mx = 0u;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) {
        const float v = src[i];
        mx = max(mx, __float_as_uint(v) & 0x7fffffffu);
        dst[i] = (_Float16)v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(max_abs_bits, mx);
}

__device__ __forceinline__ bool rr_less(float da, int64_t ia, float db, int64_t ib) {
    return da < db || (da == db && ia < ib);
}

// grid = 8 * ceil(nq / 8), block = 256, dynamic LDS = d*4 + mp2*(4 + 8) bytes (mp2 = power of two >= m, >= 256).
// METRIC: 0 inner product, 1 squared Euclidean, 2 cosine.
// Queries are taken in the order of `qorder` (grouped by nearest cluster: queries that share candidates run at
// the same time, so a corpus row gathered for one of them is still in cache for the others), and consecutive
// entries of that order go to the same XCD (workgroups are dealt round-robin over the 8 XCDs, each with its own L2).
template <int METRIC, typename T>
__global__ __launch_bounds__(256) void k_rerank(const float* __restrict__ Q, const T* __restrict__ corpus,
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
    const int d4 = (d % 4 == 0) ? d / 4 : 0;      // vector path needs rows aligned to four elements
    using V = typename Row4<T>::type;

    for (int c = wv; c < m; c += 4) {
        const int row = crow[c];
        if (row < 0) continue;                    // uniform per wavefront
        const T* p = corpus + (size_t)row * d;
        float acc = 0.0f;
        if (d4) {
            const V* p4 = reinterpret_cast<const V*>(p);
            const float4* q4 = reinterpret_cast<const float4*>(qs);
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
                if (METRIC == 1) { const float t = qs[i] - x; acc = fmaf(t, t, acc); }
                else acc = fmaf(x, qs[i], acc);
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
