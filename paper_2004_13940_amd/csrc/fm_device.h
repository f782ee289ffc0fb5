// Device-side helpers shared by the row and column kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

template <int VEC>
__device__ __forceinline__ void fm_load_vec(const float* __restrict__ p, float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void fm_store_vec(float* __restrict__ p, const float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
    } else {
        *p = v[0];
    }
}

// Sum over the L lanes of a group (L a power of two, groups aligned to L lanes);
// every lane of the group receives the total.  Fixed butterfly order.
template <int L, typename T>
__device__ __forceinline__ T fm_group_sum(T v)
{
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, L);
    return v;
}

// Sum over all 64 lanes of the wave, fixed butterfly order.
template <typename T>
__device__ __forceinline__ T fm_wave_sum(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Value of `v` held by lane `t` of the caller's L-lane group.
template <int L, typename T>
__device__ __forceinline__ T fm_group_bcast(T v, int t)
{
    if constexpr (L == 1) {
        return v;
    } else {
        return __shfl(v, t, L);
    }
}

// Block b of the floor split of n items into P blocks that holds index i:
// b = floor(((i+1) P - 1) / n)   (inverse of the bound floor(b n / P)).
__device__ __forceinline__ int32_t fm_block_of(int64_t i, int64_t n, int32_t P)
{
    return (int32_t)(((i + 1) * (int64_t)P - 1) / n);
}
