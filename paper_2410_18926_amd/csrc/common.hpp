// Shared device helpers for the LoRANN gfx950 kernels: vector types, order-preserving float keys,
// wavefront (64-lane) reductions and block-wide flag scans.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lorann {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// Monotone map float -> uint32: a < b  <=>  key(a) < key(b); -0 and +0 share one key.
__device__ __forceinline__ uint32_t float_key_asc(float f) {
    if (f == 0.0f) f = 0.0f;
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Exclusive prefix count of `flag` over a block of NW wavefronts (thread order), plus the block total.
// `wsum` is LDS scratch of NW ints.  Contains two barriers; every thread of the block must call it.
template <int NW>
__device__ __forceinline__ int block_flag_scan(bool flag, int* wsum, int& total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned long long b = __ballot(flag);
    const int before = __popcll(b & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wv] = __popcll(b);
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int c = wsum[i];
        if (i < wv) base += c;
        tot += c;
    }
    __syncthreads();
    total = tot;
    return base + before;
}

}  // namespace lorann
