// Initial values, row get/set, negative sampling (destination keys), gather dot products and the
// client's coefficient step.  gfx950, wave64.
#include <algorithm>

#include "rows.h"
#include "loss.h"

namespace w2v {

static inline unsigned blocks_for(uint64_t items, unsigned per_block) {
    return (unsigned)((items + per_block - 1) / per_block);
}

// ---------------------------------------------------------------------------------------------
// Initial vectors: component (word w, global column c) of matrix m is
//   ((R >> 8) * 2^-24 - 0.5) / d_total,  R = word (c mod 4) of Philox(counter = (w, c/4, m, INIT)).
// One thread per float4 of a row; columns past d_slice inside the stride stay zero.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void init_kernel(float4* __restrict__ M, uint32_t V, RowGeom g,
                                                   uint32_t d_slice, float d_total,
                                                   uint32_t col_begin, uint32_t k0, uint32_t k1,
                                                   uint32_t matrix, int zero) {
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    uint64_t total = (uint64_t)V * g.stride4;
    if (i >= total) return;
    uint32_t w = (uint32_t)(i / g.stride4);
    uint32_t q = (uint32_t)(i % g.stride4);
    float vals[4] = {0.f, 0.f, 0.f, 0.f};
    if (!zero) {
        uint32_t have_block = 0xFFFFFFFFu;
        U4 r{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t local = q * 4 + e;
            if (local < d_slice) {
                uint32_t c = col_begin + local;
                if ((c >> 2) != have_block) {
                    have_block = c >> 2;
                    r = philox4x32_10(w, have_block, matrix, DOM_INIT, k0, k1);
                }
                uint32_t lane = c & 3u;
                uint32_t bits = lane == 0 ? r.x : lane == 1 ? r.y : lane == 2 ? r.z : r.w;
                float x = (float)(bits >> 8) * (1.0f / 16777216.0f) - 0.5f;
                vals[e] = x / d_total;
            }
        }
    }
    M[i] = make_float4(vals[0], vals[1], vals[2], vals[3]);
}

void launch_init(float* M, uint32_t V, RowGeom g, uint32_t d_slice, uint32_t d_total,
                 uint32_t col_begin, uint64_t seed, uint32_t matrix, bool zero, hipStream_t st) {
    uint64_t total = (uint64_t)V * g.stride4;
    hipLaunchKernelGGL(init_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, st, (float4*)M, V,
                       g, d_slice, (float)d_total, col_begin, (uint32_t)seed,
                       (uint32_t)(seed >> 32), matrix, zero ? 1 : 0);
}

// ---------------------------------------------------------------------------------------------
// get / set of listed rows, dense [m][d_slice] on the caller's side.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ M,
                                                          uint32_t stride, uint32_t d_slice,
                                                          const uint32_t* __restrict__ rows,
                                                          uint32_t m, uint32_t V,
                                                          float* __restrict__ dst,
                                                          uint32_t* err) {
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (uint64_t)m * d_slice) return;
    uint32_t r = (uint32_t)(i / d_slice), c = (uint32_t)(i % d_slice);
    uint32_t w = rows[r];
    if (w >= V) { if (c == 0) atomicOr(err, 1u); w = 0; }
    dst[i] = M[(uint64_t)w * stride + c];
}

__global__ __launch_bounds__(256) void scatter_rows_kernel(float* __restrict__ M, uint32_t stride,
                                                           uint32_t d_slice,
                                                           const uint32_t* __restrict__ rows,
                                                           uint32_t m, uint32_t V,
                                                           const float* __restrict__ src,
                                                           uint32_t* err) {
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (uint64_t)m * d_slice) return;
    uint32_t r = (uint32_t)(i / d_slice), c = (uint32_t)(i % d_slice);
    uint32_t w = rows[r];
    if (w >= V) { if (c == 0) atomicOr(err, 1u); return; }
    M[(uint64_t)w * stride + c] = src[i];
}

void launch_gather_rows(const float* M, RowGeom g, uint32_t d_slice, const uint32_t* rows,
                        uint32_t m, uint32_t V, float* dst, uint32_t* err, hipStream_t st) {
    if (m == 0) return;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks_for((uint64_t)m * d_slice, 256)), dim3(256),
                       0, st, M, g.stride4 * 4, d_slice, rows, m, V, dst, err);
}

void launch_scatter_rows(float* M, RowGeom g, uint32_t d_slice, const uint32_t* rows, uint32_t m,
                         uint32_t V, const float* src, uint32_t* err, hipStream_t st) {
    if (m == 0) return;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks_for((uint64_t)m * d_slice, 256)), dim3(256),
                       0, st, M, g.stride4 * 4, d_slice, rows, m, V, src, err);
}

// ---------------------------------------------------------------------------------------------
// Destination keys: slot 0 of pair p is its positive output word, slot j >= 1 its j-th negative.
// A negative is the first alias-table candidate (attempt t = 0..15, Philox counter (p, j, t, NEG))
// that differs from the positive word; after 16 rejections it is the next word index, cyclically.
// One thread per slot, so the generator runs with all 64 lanes busy.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void dest_key_item(const uint2* __restrict__ bins, uint32_t V,
                                              const uint32_t* __restrict__ out_idx, uint32_t n,
                                              uint32_t T, uint32_t k0, uint32_t k1,
                                              uint32_t* __restrict__ keys, uint32_t* err, uint32_t i) {
    if (i >= n * T) return;
    uint32_t p = i / T, j = i - p * T;
    uint32_t wo = out_idx[p];
    if (wo >= V) { wo = 0; if (j == 0) atomicOr(err, 1u); }
    uint32_t key;
    if (j == 0) {
        key = wo;
    } else {
        key = wo + 1 == V ? 0u : wo + 1;           // the fallback
        for (uint32_t t = 0; t < 16; ++t) {
            U4 r = philox4x32_10(p, j, t, DOM_NEG, k0, k1);
            uint64_t r64 = ((uint64_t)r.y << 32) | (uint64_t)r.x;
            uint32_t bin = (uint32_t)__umul64hi(r64, (uint64_t)V);
            uint2 b = bins[bin];
            uint32_t cand = (r.z < b.x) ? bin : b.y;
            if (cand != wo) { key = cand; break; }
        }
    }
    keys[i] = key;
}

__global__ __launch_bounds__(256) void dest_keys_kernel(const uint2* __restrict__ bins, uint32_t V,
                                                        const uint32_t* __restrict__ out_idx,
                                                        uint32_t n, uint32_t T, uint32_t k0_arg,
                                                        uint32_t k1_arg, uint32_t* __restrict__ keys,
                                                        uint32_t* err, const CallScalars* dev) {
    const uint32_t k0 = dev ? dev->seed_lo : k0_arg, k1 = dev ? dev->seed_hi : k1_arg;
    dest_key_item(bins, V, out_idx, n, T, k0, k1, keys, err, blockIdx.x * 256 + threadIdx.x);
}

// After the sort of the destination keys: an entry whose two neighbours carry other keys is the
// only slot of the minibatch that names its row.  Such slots get KEY_ALONE set in the slot-ordered
// key array (each slot is written by at most one thread), so that the input-side kernel, which
// holds everything the row's update needs, can write it, and the output side can leave it out.
__global__ __launch_bounds__(256) void mark_alone_kernel(const uint32_t* __restrict__ skey,
                                                         const uint32_t* __restrict__ sidx,
                                                         uint32_t M, uint32_t* __restrict__ keys) {
    uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= M) return;
    const uint32_t k = skey[i];
    const bool left = i > 0 && skey[i - 1] == k;
    const bool right = i + 1 < M && skey[i + 1] == k;
    if (!left && !right) keys[sidx[i]] = k | KEY_ALONE;
}

void launch_dest_keys(NoiseTable nt, const uint32_t* out_idx, uint32_t n, uint32_t k, uint64_t seed,
                      uint32_t* keys, uint32_t* err, hipStream_t st, const CallScalars* dev) {
    if (n == 0) return;
    uint32_t T = k + 1;
    hipLaunchKernelGGL(dest_keys_kernel, dim3(blocks_for((uint64_t)n * T, 256)), dim3(256), 0, st,
                       nt.bins, nt.V, out_idx, n, T, (uint32_t)seed, (uint32_t)(seed >> 32), keys,
                       err, dev);
}

void launch_mark_alone(const uint32_t* skey, const uint32_t* sidx, uint32_t M, uint32_t* keys,
                       hipStream_t st) {
    if (M == 0) return;
    hipLaunchKernelGGL(mark_alone_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, st, skey, sidx, M,
                       keys);
}

// Range-checked copy of the input words: an index >= V raises *err and is replaced by word 0, so no
// later kernel can be sent outside the matrices.
__device__ __forceinline__ void check_input_item(const uint32_t* __restrict__ in_idx, uint32_t n,
                                                 uint32_t V, uint32_t* __restrict__ in_safe,
                                                 uint32_t* err, uint32_t p) {
    if (p >= n) return;
    uint32_t wi = in_idx[p];
    if (wi >= V) { atomicOr(err, 1u); wi = 0; }
    in_safe[p] = wi;
}

__global__ __launch_bounds__(256) void check_inputs_kernel(const uint32_t* __restrict__ in_idx,
                                                           uint32_t n, uint32_t V,
                                                           uint32_t* __restrict__ in_safe,
                                                           uint32_t* err) {
    check_input_item(in_idx, n, V, in_safe, err, blockIdx.x * 256 + threadIdx.x);
}

void launch_check_inputs(const uint32_t* in_idx, uint32_t n, uint32_t V, uint32_t* in_safe,
                         uint32_t* err, hipStream_t st) {
    if (n == 0) return;
    hipLaunchKernelGGL(check_inputs_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, in_idx, n, V,
                       in_safe, err);
}

// The index work that depends on nothing but the call's arguments, in ONE launch: destination
// keys, checked input words and up to two plain fills (the sort's counters, the output side's
// border slots).  Each block does one part, told by its number.  A step of a few thousand pairs is
// a chain of dependent launches of a few microseconds each, and these were four of them.
__global__ __launch_bounds__(256) void index_prologue_kernel(IndexPrologue a) {
    const uint32_t b = blockIdx.x;
    if (b < a.b_check) {
        const uint32_t k0 = a.dev ? a.dev->seed_lo : a.seed_lo, k1 = a.dev ? a.dev->seed_hi : a.seed_hi;
        dest_key_item(a.nt.bins, a.nt.V, a.out_idx, a.n, a.T, k0, k1, a.keys, a.err,
                      b * 256 + threadIdx.x);
        if (a.scalars_out && b == 0 && threadIdx.x == 0) {
            a.scalars_out->seed_lo = a.seed_lo; a.scalars_out->seed_hi = a.seed_hi;
            a.scalars_out->alpha = a.alpha;
        }
    } else if (b < a.b_fill[0]) {
        check_input_item(a.in_idx, a.n, a.nt.V, a.in_safe, a.err, (b - a.b_check) * 256 + threadIdx.x);
    } else {
        const int f = b < a.b_fill[1] ? 0 : 1;
        const uint32_t i = (b - a.b_fill[f]) * 256 + threadIdx.x;
        if (i < a.fill[f].count) a.fill[f].p[i] = a.fill[f].value;
    }
}

void launch_index_prologue(IndexPrologue a, hipStream_t st) {
    if (a.n == 0) { a.fill[0].count = 0; a.fill[1].count = 0; }   // (no pairs: nothing follows)
    a.b_check = blocks_for((uint64_t)a.n * a.T, 256);
    a.b_fill[0] = a.b_check + blocks_for(a.n, 256);
    a.b_fill[1] = a.b_fill[0] + blocks_for(a.fill[0].count, 256);
    const uint32_t blocks = a.b_fill[1] + blocks_for(a.fill[1].count, 256);
    if (blocks == 0) return;
    hipLaunchKernelGGL(index_prologue_kernel, dim3(blocks), dim3(256), 0, st, a);
}

__global__ __launch_bounds__(256) void copy_negatives_kernel(const uint32_t* __restrict__ keys,
                                                             uint32_t n, uint32_t k,
                                                             uint32_t* __restrict__ neg) {
    uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n * k) return;
    uint32_t p = i / k, j = i - p * k;
    neg[i] = keys[p * (k + 1) + 1 + j];
}

void launch_copy_negatives(const uint32_t* keys, uint32_t n, uint32_t k, uint32_t* neg,
                           hipStream_t st) {
    if (n == 0 || k == 0) return;
    hipLaunchKernelGGL(copy_negatives_kernel, dim3(blocks_for((uint64_t)n * k, 256)), dim3(256), 0,
                       st, keys, n, k, neg);
}

// ---------------------------------------------------------------------------------------------
// Gather dot products: one lane group per pair.  The group loads u once, then the T output rows in
// batches of TB with every load of a batch issued before the first multiply.
// ---------------------------------------------------------------------------------------------
constexpr int DOT_THREADS = 128;     // (256: the kernel 40 % slower beside other work, 64: the same)
template <int G, int NV, int TB>
__global__ __launch_bounds__(DOT_THREADS) void dots_kernel(const float4* __restrict__ U,
                                                   const float4* __restrict__ W, RowGeom g,
                                                   const uint32_t* __restrict__ in_idx,
                                                   const uint32_t* __restrict__ keys, uint32_t n,
                                                   uint32_t T, float* __restrict__ dots) {
    const int l = threadIdx.x % G;
    uint32_t grp = (blockIdx.x * (uint32_t)DOT_THREADS + threadIdx.x) / G;
    const bool live = grp < n;
    const uint32_t p = live ? grp : n - 1;
    const uint32_t wi = in_idx[p];          // already range-checked (launch_check_inputs)
    float4 u[NV];
    load_row<G, NV>(U + (uint64_t)wi * g.stride4, g.d4, l, u);
    for (uint32_t jb = 0; jb < T; jb += TB) {
        float4 w[TB][NV];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            uint32_t j = jb + t;
            bool on = j < T;
            uint32_t r = on ? (keys[p * T + j] & ~KEY_ALONE) : 0u;   // (a prepared set may carry the mark)
            load_row_if<G, NV>(on, W + (uint64_t)r * g.stride4, g.d4, l, w[t]);
        }
        float s[TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) s[t] = dot_part<NV>(u, w[t]);
#pragma unroll
        for (int t = 0; t < TB; ++t) s[t] = group_sum<G>(s[t]);
#pragma unroll
        for (int t = 0; t < TB; ++t)
            if (l == t && live && jb + t < T) dots[p * T + jb + t] = s[t];
    }
}

void launch_dots(const float* U, const float* W, RowGeom g, const uint32_t* in_idx,
                 const uint32_t* keys, uint32_t n, uint32_t T, float* dots, hipStream_t st) {
    if (n == 0) return;
#define CALL(G, NV)                                                                               \
    hipLaunchKernelGGL((dots_kernel<G, NV, (NV <= 2 ? 6 : 4)>),                                   \
                       dim3(blocks_for((uint64_t)n * G, DOT_THREADS)), dim3(DOT_THREADS), 0, st, (const float4*)U, \
                       (const float4*)W, g, in_idx, keys, n, T, dots)
    W2V_DISPATCH_GEOM(g.d4, CALL);
#undef CALL
}

// ---------------------------------------------------------------------------------------------
// Client step between the two calls: f = sum over shards of the partial dots (shard order), then
// the coefficient label - sigma(f), written as sigma(-f) for the positive slot so that it keeps
// its relative accuracy when f is large.  Loss terms are softplus(-f) / softplus(f), summed per
// block in double by a fixed tree, then over blocks in index order by one thread.
// ---------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void coeffs_kernel(PartialPtrs parts, uint32_t S, uint32_t total,
                                                     uint32_t T, float* __restrict__ coeffs,
                                                     double* __restrict__ block_loss) {
    __shared__ double red[256];
    uint32_t i = blockIdx.x * 256 + threadIdx.x;
    double term = 0.0;
    if (i < total) {
        float f = 0.f;
        for (uint32_t s = 0; s < S; ++s) f += parts.p[s][i];
        uint32_t j = i % T;
        float gcoef;
        if (j == 0) { gcoef = 1.0f / (1.0f + expf(f)); term = (double)softplus(-f); }
        else        { gcoef = -1.0f / (1.0f + expf(-f)); term = (double)softplus(f); }
        coeffs[i] = gcoef;
    }
    if (block_loss) {
        red[threadIdx.x] = term;
        __syncthreads();
        for (int s = 128; s >= 1; s >>= 1) {
            if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
            __syncthreads();
        }
        if (threadIdx.x == 0) block_loss[blockIdx.x] = red[0];
    }
}

// Sum of n doubles in a fixed order: block b of a grid takes the slice [b*span, (b+1)*span), its
// thread t adds elements t, t+256, ... of the slice in order, then the block reduces by a fixed
// tree.  Called once over the data (-> one partial per block) and once, with a single block, over
// the partials.
__global__ __launch_bounds__(256) void sum_doubles_kernel(const double* __restrict__ x, uint32_t n,
                                                          uint32_t span,
                                                          double* __restrict__ out) {
    __shared__ double red[256];
    sum_doubles_block(x, n, span, out, blockIdx.x, red);
}


// x[n] -> *out, using tmp[ceil(n / LOSS_SUM_SPAN)] doubles.
static void launch_sum_doubles(const double* x, uint32_t n, double* tmp, double* out,
                               hipStream_t st) {
    uint32_t nb = (n + LOSS_SUM_SPAN - 1) / LOSS_SUM_SPAN;
    if (nb <= 1) {
        hipLaunchKernelGGL(sum_doubles_kernel, dim3(1), dim3(256), 0, st, x, n, n ? n : 1u, out);
        return;
    }
    hipLaunchKernelGGL(sum_doubles_kernel, dim3(nb), dim3(256), 0, st, x, n, LOSS_SUM_SPAN, tmp);
    hipLaunchKernelGGL(sum_doubles_kernel, dim3(1), dim3(256), 0, st, (const double*)tmp, nb, nb,
                       out);
}

// doubles of scratch for the loss: the per-block (or per-pair) terms plus the second-stage partials
size_t coeffs_loss_scratch_doubles(uint32_t n, uint32_t T) {
    size_t terms = std::max<size_t>(blocks_for((uint64_t)n * T, 256), n);
    return terms + (terms + LOSS_SUM_SPAN - 1) / LOSS_SUM_SPAN + 8;
}

void launch_coeffs(PartialPtrs parts, uint32_t S, uint32_t n, uint32_t T, float* coeffs,
                   double* block_loss, double* loss_out, hipStream_t st) {
    uint32_t total = n * T;
    if (total == 0) {
        if (loss_out) launch_sum_doubles(nullptr, 0, nullptr, loss_out, st);
        return;
    }
    unsigned nb = blocks_for(total, 256);
    hipLaunchKernelGGL(coeffs_kernel, dim3(nb), dim3(256), 0, st, parts, S, total, T, coeffs,
                       loss_out ? block_loss : (double*)nullptr);
    if (loss_out) launch_sum_doubles(block_loss, nb, block_loss + nb, loss_out, st);
}

// Minibatch loss of the fused step, from the dots the input-side kernel leaves behind: the same
// softplus terms as coeffs_kernel, so that the fused and the unfused form of a step report the
// same loss, finite however far sigma saturates.
__global__ __launch_bounds__(256) void loss_from_dots_kernel(const float* __restrict__ dots,
                                                             uint32_t total, uint32_t T,
                                                             double* __restrict__ block_loss) {
    __shared__ double red[256];
    loss_terms_block(dots, total, T, block_loss, blockIdx.x, red);
}

void launch_loss_from_dots(const float* dots, uint32_t n, uint32_t T, double* tmp, double* loss_out,
                           hipStream_t st) {
    uint32_t total = n * T;
    if (total == 0) { launch_sum_doubles(nullptr, 0, nullptr, loss_out, st); return; }
    unsigned nb = blocks_for(total, 256);
    hipLaunchKernelGGL(loss_from_dots_kernel, dim3(nb), dim3(256), 0, st, dots, total, T, tmp);
    launch_sum_doubles(tmp, nb, tmp + nb, loss_out, st);
}

}  // namespace w2v
