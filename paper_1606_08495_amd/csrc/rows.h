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

// Sum over the G lanes of a group by a butterfly; every lane ends with the same bits because each
// step adds the same two operands in both partners.
template <int G>
__device__ __forceinline__ float group_sum(float x) {
#pragma unroll
    for (int m = G / 2; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
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
