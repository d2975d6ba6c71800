// Shared device helpers for the LoRANN gfx950 kernels: vector types, order-preserving float keys,
// wavefront (64-lane) reductions and block-wide flag scans.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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

__device__ __forceinline__ float key_to_float(uint32_t key) {   // inverse of float_key_asc
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
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
// Sum over the 64 lanes with data-parallel-primitive moves (no LDS traffic, unlike the shuffles above): prefix
// sums inside each row of 16 lanes (shifts by 1, 2, 4, 8 with zero fill), then lane 15 of a row is added to the
// next row, then lane 31 to the upper half.  The TOTAL IS VALID IN LANE 63 ONLY.
__device__ __forceinline__ float wave_sum_f32_lane63(float v) {
    auto shifted = [](float x, auto ctrl, auto row_mask, auto bound) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, decltype(row_mask)::value, 0xf,
                                                          decltype(bound)::value));
    };
    using std::integral_constant;
    v += shifted(v, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});   // row_shr:1
    v += shifted(v, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});   // row_shr:2
    v += shifted(v, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});   // row_shr:4
    v += shifted(v, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});   // row_shr:8
    v += shifted(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{}, integral_constant<bool, false>{});  // row_bcast:15 -> rows 1, 3
    v += shifted(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{}, integral_constant<bool, false>{});  // row_bcast:31 -> rows 2, 3
    return v;
}
// Minimum of an unsigned over the 64 lanes, same scheme (lanes without a source keep 0xFFFFFFFF, the identity);
// the result is returned to every lane through a scalar read of lane 63.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    auto shifted = [](uint32_t x, auto ctrl, auto row_mask) {
        return (uint32_t)__builtin_amdgcn_update_dpp((int)0xFFFFFFFFu, (int)x, decltype(ctrl)::value, decltype(row_mask)::value, 0xf, false);
    };
    using std::integral_constant;
    v = min(v, shifted(v, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{}));   // row_shr:1
    v = min(v, shifted(v, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{}));   // row_shr:2
    v = min(v, shifted(v, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{}));   // row_shr:4
    v = min(v, shifted(v, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{}));   // row_shr:8
    v = min(v, shifted(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{}));   // row_bcast:15 -> rows 1, 3
    v = min(v, shifted(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{}));   // row_bcast:31 -> rows 2, 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
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
