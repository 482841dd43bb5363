// Device helpers: a lane group of G consecutive lanes (G = 16, 32 or 64, aligned inside the
// 64-wide wavefront) owns one matrix row; lane l keeps float4 number l, l+G, ... of it.
#pragma once
#include "common.h"

namespace w2v {

__device__ __forceinline__ float4 f4zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }

template <int G, int NV>
__device__ __forceinline__ void load_row(const float4* __restrict__ row, uint32_t d4, int l,
                                         float4 (&r)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        uint32_t i = (uint32_t)l + (uint32_t)(G * v);
        r[v] = (i < d4) ? row[i] : f4zero();
    }
}

template <int G, int NV>
__device__ __forceinline__ void load_row_if(bool on, const float4* __restrict__ row, uint32_t d4,
                                            int l, float4 (&r)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        uint32_t i = (uint32_t)l + (uint32_t)(G * v);
        r[v] = (on && i < d4) ? row[i] : f4zero();
    }
}

typedef float v4f __attribute__((ext_vector_type(4)));

// The same with the non-temporal hint: rows that are touched once per minibatch and should not
// push reusable rows out of the caches.
template <int G, int NV>
__device__ __forceinline__ void load_row_nt_if(bool on, const float4* __restrict__ row, uint32_t d4,
                                               int l, float4 (&r)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        uint32_t i = (uint32_t)l + (uint32_t)(G * v);
        if (on && i < d4) {
            const v4f x = __builtin_nontemporal_load((const v4f*)row + i);
            r[v] = make_float4(x.x, x.y, x.z, x.w);
        } else {
            r[v] = f4zero();
        }
    }
}

template <int G, int NV>
__device__ __forceinline__ void store_row_nt(float4* __restrict__ row, uint32_t d4, int l,
                                             const float4 (&r)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        uint32_t i = (uint32_t)l + (uint32_t)(G * v);
        if (i < d4) {
            v4f x = {r[v].x, r[v].y, r[v].z, r[v].w};
            __builtin_nontemporal_store(x, (v4f*)row + i);
        }
    }
}

template <int G, int NV>
__device__ __forceinline__ void store_row(float4* __restrict__ row, uint32_t d4, int l,
                                          const float4 (&r)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        uint32_t i = (uint32_t)l + (uint32_t)(G * v);
        if (i < d4) row[i] = r[v];
    }
}

template <int NV>
__device__ __forceinline__ float dot_part(const float4 (&a)[NV], const float4 (&b)[NV]) {
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        s = fmaf(a[v].x, b[v].x, s);
        s = fmaf(a[v].y, b[v].y, s);
        s = fmaf(a[v].z, b[v].z, s);
        s = fmaf(a[v].w, b[v].w, s);
    }
    return s;
}

template <int NV>
__device__ __forceinline__ void axpy(float c, const float4 (&x)[NV], float4 (&acc)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        acc[v].x = fmaf(c, x[v].x, acc[v].x);
        acc[v].y = fmaf(c, x[v].y, acc[v].y);
        acc[v].z = fmaf(c, x[v].z, acc[v].z);
        acc[v].w = fmaf(c, x[v].w, acc[v].w);
    }
}

template <int NV>
__device__ __forceinline__ void clear(float4 (&acc)[NV]) {
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = f4zero();
}

// Sum over the G lanes of a group; every lane of the group ends with the same bits.
// Inside a 16-lane row the butterfly runs on DPP lane permutations (xor 1, xor 2, then the two
// mirror patterns, in which both partners of a step still add the same two operands).  The four
// row sums of a wavefront are then fetched with v_readlane and added in a fixed order.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);   // row_half_mirror: lane i <-> 7-i within 8
    x += dpp_move<0x140>(x);   // row_mirror: lane i <-> 15-i within 16
    return x;
}

__device__ __forceinline__ float lane_value(float x, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}

template <int G>
__device__ __forceinline__ float group_sum(float x) {
    x = row16_sum(x);
    if (G == 16) return x;
    const float lo = lane_value(x, 0) + lane_value(x, 16);
    const float hi = lane_value(x, 32) + lane_value(x, 48);
    if (G == 32) return (threadIdx.x & 32) ? hi : lo;
    return lo + hi;
}

// Choice of group shape for a row of d4 float4.
#define W2V_DISPATCH_GEOM(d4, CALL)                   \
    do {                                              \
        if ((d4) <= 16)       { CALL(16, 1); }        \
        else if ((d4) <= 32)  { CALL(32, 1); }        \
        else if ((d4) <= 64)  { CALL(64, 1); }        \
        else if ((d4) <= 128) { CALL(64, 2); }        \
        else if ((d4) <= 192) { CALL(64, 3); }        \
        else                  { CALL(64, 4); }        \
    } while (0)

}  // namespace w2v
