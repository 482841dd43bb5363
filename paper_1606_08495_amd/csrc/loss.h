// Device parts of the minibatch loss, shared by the kernels that form it on their own and by the
// launch that runs them beside other work of the step.  Blocks of 256 threads.
#pragma once
#include "common.h"

namespace w2v {

// Sums of doubles go in slices of this many elements per block; up to this many fit one block.
constexpr uint32_t LOSS_SUM_SPAN = 4096;

// log(1 + e^x) without overflow or cancellation
__device__ __forceinline__ float softplus(float x) {
    return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
}

// fixed tree over the 256 values of a block; the sum arrives in thread 0
__device__ __forceinline__ double block_tree_sum_256(double v, double* red) {
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    return red[0];
}

// Block vb of the loss terms: slot 0 of a pair contributes softplus(-f), the others softplus(f);
// the block's sum goes to block_loss[vb].
__device__ __forceinline__ void loss_terms_block(const float* __restrict__ dots, uint32_t total,
                                                 uint32_t T, double* __restrict__ block_loss,
                                                 uint32_t vb, double* red) {
    const uint32_t i = vb * 256 + threadIdx.x;
    double term = 0.0;
    if (i < total) {
        const float f = dots[i];
        term = (double)((i % T) == 0 ? softplus(-f) : softplus(f));
    }
    const double s = block_tree_sum_256(term, red);
    if (threadIdx.x == 0) block_loss[vb] = s;
}

// Sum of the slice [vb*span, (vb+1)*span) of x[n] in a fixed order: thread t adds elements t,
// t+256, ... of the slice in order, then the block reduces by the fixed tree.
__device__ __forceinline__ void sum_doubles_block(const double* __restrict__ x, uint32_t n,
                                                  uint32_t span, double* __restrict__ out,
                                                  uint32_t vb, double* red) {
    const uint64_t lo = (uint64_t)vb * span;
    const uint64_t hi = lo + span < n ? lo + span : n;
    double s = 0.0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += 256) s += x[i];
    const double r = block_tree_sum_256(s, red);
    if (threadIdx.x == 0) out[vb] = r;
}

}  // namespace w2v
