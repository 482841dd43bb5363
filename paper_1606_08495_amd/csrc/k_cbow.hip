// Continuous-bag-of-words variant (Section 5.1, footnote): the kernels that are specific to it.
// Everything else of the step -- negatives, dots, coefficients, both segmented reductions -- runs in
// the skip-gram kernels, which take the matrix of hidden vectors in place of the input vectors.
#include "common.h"
#include "rows.h"

namespace w2v {

static inline unsigned blocks_for(uint64_t items, unsigned per_block) {
    return (unsigned)((items + per_block - 1) / per_block);
}

// ---------------------------------------------------------------------------------------------
// Per context entry e: the checked word, the example it belongs to and the weight 1/|C_p| with
// which the example's summed output rows enter the word's input vector.  The example is found by
// bisection of the offsets, so malformed offsets can at worst give wrong (never out-of-range)
// example numbers; they raise the error flag.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cbow_entries_kernel(const uint32_t* __restrict__ ctx_off,
                                                           const uint32_t* __restrict__ ctx_idx,
                                                           uint32_t n, uint32_t m, uint32_t V,
                                                           uint32_t* __restrict__ ctx_safe,
                                                           uint32_t* __restrict__ ex_of,
                                                           float* __restrict__ weight,
                                                           uint32_t* err) {
    uint32_t e = blockIdx.x * 256 + threadIdx.x;
    if (e >= m) return;
    uint32_t w = ctx_idx[e];
    if (w >= V) { atomicOr(err, 1u); w = 0; }
    ctx_safe[e] = w;
    uint32_t lo = 0, hi = n;                    // largest p in [0, n) with ctx_off[p] <= e
    while (hi - lo > 1) {
        uint32_t mid = lo + (hi - lo) / 2;
        if (ctx_off[mid] <= e) lo = mid; else hi = mid;
    }
    const uint32_t a = ctx_off[lo], b = ctx_off[lo + 1];
    const bool inside = a <= e && e < b && b <= m;
    if (!inside) atomicOr(err, 1u);
    ex_of[e] = lo;
    weight[e] = inside ? 1.0f / (float)(b - a) : 0.0f;
}

// Offsets must start at 0, never decrease and end at m.
__global__ __launch_bounds__(256) void cbow_check_offsets_kernel(const uint32_t* __restrict__ ctx_off,
                                                                 uint32_t n, uint32_t m,
                                                                 uint32_t* err) {
    uint32_t p = blockIdx.x * 256 + threadIdx.x;
    if (p > n) return;
    bool bad = ctx_off[p] > m;
    if (p == 0) bad = bad || ctx_off[0] != 0;
    if (p == n) bad = bad || ctx_off[n] != m;
    if (p < n) bad = bad || ctx_off[p + 1] < ctx_off[p];
    if (bad) atomicOr(err, 1u);
}

__global__ __launch_bounds__(256) void iota_kernel(uint32_t* __restrict__ x, uint32_t n) {
    uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) x[i] = i;
}

// ---------------------------------------------------------------------------------------------
// Hidden vectors: one lane group per example adds the input rows of its context words in list
// order (four loads in flight) and divides by their number.  An example without context gets zeros.
// ---------------------------------------------------------------------------------------------
template <int G, int NV>
__global__ __launch_bounds__(256) void cbow_hidden_kernel(const float4* __restrict__ U, RowGeom g,
                                                          const uint32_t* __restrict__ ctx_off,
                                                          const uint32_t* __restrict__ ctx_safe,
                                                          uint32_t n, uint32_t m,
                                                          float4* __restrict__ H) {
    constexpr int UB = 4;
    const int l = threadIdx.x % G;
    const uint32_t p = (blockIdx.x * 256u + threadIdx.x) / G;
    if (p >= n) return;                                   // whole groups leave together
    uint32_t lo = min(ctx_off[p], m);
    uint32_t hi = min(max(ctx_off[p + 1], lo), m);
    float4 acc[NV];
    clear<NV>(acc);
    for (uint32_t e = lo; e < hi; e += UB) {
        float4 r[UB][NV];
#pragma unroll
        for (int t = 0; t < UB; ++t) {
            const bool on = e + t < hi;
            const uint32_t w = on ? ctx_safe[e + t] : 0u;
            load_row_if<G, NV>(on, U + (uint64_t)w * g.stride4, g.d4, l, r[t]);
        }
#pragma unroll
        for (int t = 0; t < UB; ++t)
            if (e + t < hi) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    acc[v].x += r[t][v].x; acc[v].y += r[t][v].y;
                    acc[v].z += r[t][v].z; acc[v].w += r[t][v].w;
                }
            }
    }
    if (hi > lo) {
        const float cnt = (float)(hi - lo);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            acc[v].x /= cnt; acc[v].y /= cnt; acc[v].z /= cnt; acc[v].w /= cnt;
        }
    }
    store_row<G, NV>(H + (uint64_t)p * g.stride4, g.d4, l, acc);
}

void launch_cbow_entries(const uint32_t* ctx_off, const uint32_t* ctx_idx, uint32_t n, uint32_t m,
                         uint32_t V, uint32_t* ctx_safe, uint32_t* ex_of, float* weight,
                         uint32_t* err, hipStream_t st) {
    hipLaunchKernelGGL(cbow_check_offsets_kernel, dim3(blocks_for((uint64_t)n + 1, 256)), dim3(256),
                       0, st, ctx_off, n, m, err);
    if (m == 0 || n == 0) return;
    hipLaunchKernelGGL(cbow_entries_kernel, dim3(blocks_for(m, 256)), dim3(256), 0, st, ctx_off,
                       ctx_idx, n, m, V, ctx_safe, ex_of, weight, err);
}

void launch_iota(uint32_t* x, uint32_t n, hipStream_t st) {
    if (n == 0) return;
    hipLaunchKernelGGL(iota_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, x, n);
}

void launch_cbow_hidden(const float* U, RowGeom g, const uint32_t* ctx_off, const uint32_t* ctx_safe,
                        uint32_t n, uint32_t m, float* H, hipStream_t st) {
    if (n == 0) return;
#define CALL(G, NV)                                                                               \
    hipLaunchKernelGGL((cbow_hidden_kernel<G, NV>), dim3(blocks_for((uint64_t)n * G, 256)),       \
                       dim3(256), 0, st, (const float4*)U, g, ctx_off, ctx_safe, n, m, (float4*)H)
    W2V_DISPATCH_GEOM(g.d4, CALL);
#undef CALL
}

// ---------------------------------------------------------------------------------------------
// Examples from text, on top of the pair formation's per-survivor results: survivor q with
// kcnt[q] > 0 context words becomes example number ex[q] (exclusive count of such survivors); its
// context words are the pair stream's output words poff[q] .. poff[q] + kcnt[q].
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cbow_example_flags_kernel(const uint32_t* __restrict__ kcnt,
                                                                 const uint32_t* __restrict__ n_kept,
                                                                 uint32_t n,
                                                                 uint32_t* __restrict__ flag) {
    uint32_t q = blockIdx.x * 256 + threadIdx.x;
    if (q >= n) return;
    flag[q] = (q < *n_kept && kcnt[q] > 0) ? 1u : 0u;
}

__global__ __launch_bounds__(256) void cbow_example_write_kernel(
    const uint32_t* __restrict__ kcnt, const uint32_t* __restrict__ kword,
    const uint32_t* __restrict__ poff, const uint32_t* __restrict__ ex,
    const uint32_t* __restrict__ n_kept, uint32_t n, uint32_t* __restrict__ ctx_off,
    uint32_t* __restrict__ out_idx, uint64_t cap_examples) {
    uint32_t q = blockIdx.x * 256 + threadIdx.x;
    if (q == 0) ctx_off[0] = 0;
    if (q >= n || q >= *n_kept || kcnt[q] == 0) return;
    const uint64_t x = ex[q];
    if (x >= cap_examples) return;
    out_idx[x] = kword[q];
    ctx_off[x + 1] = poff[q] + kcnt[q];
}

void launch_cbow_examples(const uint32_t* kcnt, const uint32_t* kword, const uint32_t* poff,
                          const uint32_t* n_kept, uint32_t n, uint32_t* flag, uint32_t* ex,
                          uint32_t* scan_tmp, uint32_t* ctx_off, uint32_t* out_idx,
                          uint64_t cap_examples, uint32_t* total_examples, hipStream_t st) {
    const dim3 grid(blocks_for(n ? n : 1, 256)), block(256);
    if (n > 0)
        hipLaunchKernelGGL(cbow_example_flags_kernel, grid, block, 0, st, kcnt, n_kept, n, flag);
    launch_exclusive_scan(flag, ex, n, scan_tmp, total_examples, st);
    hipLaunchKernelGGL(cbow_example_write_kernel, grid, block, 0, st, kcnt, kword, poff, ex, n_kept, n,
                       ctx_off, out_idx, cap_examples);
}

}  // namespace w2v
