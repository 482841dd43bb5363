// Client-side pair formation on the device (Eq.1's index sets): subsample each token, then pair
// every surviving center with the surviving tokens at most b positions away inside its sentence,
// b uniform on 1..B per center.  Three passes joined by two prefix sums:
//   draws   : per token, keep flag and b from Philox(counter = (position lo, position hi, epoch,
//             TOKEN)): word 0 < keep threshold keeps the token; b = 1 + ((word 1 * B) >> 32)
//   compact : surviving tokens get consecutive numbers (scan of the flags); each learns the range
//             of surviving neighbours it pairs with and how many pairs that is
//   emit    : scan of the pair counts gives each center its place in the output
#include "common.h"

namespace w2v {

static inline unsigned blocks_for(uint64_t items, unsigned per_block) {
    return (unsigned)((items + per_block - 1) / per_block);
}

__global__ __launch_bounds__(256) void token_draws_kernel(const uint32_t* __restrict__ tokens,
                                                          uint32_t n_tokens, uint64_t token_base,
                                                          uint32_t epoch, uint32_t k0, uint32_t k1,
                                                          uint32_t B,
                                                          const uint64_t* __restrict__ keep,
                                                          uint32_t V, uint32_t* __restrict__ flag,
                                                          uint32_t* __restrict__ width,
                                                          uint32_t* err) {
    uint32_t t = blockIdx.x * 256 + threadIdx.x;
    if (t > n_tokens) return;
    if (t == n_tokens) { flag[t] = 0; return; }       // sentinel so the scan has n_tokens+1 entries
    uint64_t gpos = token_base + t;
    U4 r = philox4x32_10((uint32_t)gpos, (uint32_t)(gpos >> 32), epoch, DOM_TOKEN, k0, k1);
    uint32_t w = tokens[t];
    if (w >= V) { atomicOr(err, 1u); w = 0; }
    bool kept = keep ? ((uint64_t)r.x < keep[w]) : true;
    flag[t] = kept ? 1u : 0u;
    width[t] = 1u + (uint32_t)(((uint64_t)r.y * (uint64_t)B) >> 32);
}

// kpos[t] = number of surviving tokens before t (exclusive scan of flag, n_tokens+1 entries).
__global__ __launch_bounds__(256) void compact_kernel(const uint32_t* __restrict__ tokens,
                                                      uint32_t n_tokens,
                                                      const uint64_t* __restrict__ sent_off,
                                                      uint32_t n_sent,
                                                      const uint32_t* __restrict__ flag,
                                                      const uint32_t* __restrict__ kpos,
                                                      const uint32_t* __restrict__ width,
                                                      uint32_t V, uint32_t* __restrict__ kword,
                                                      uint32_t* __restrict__ klo,
                                                      uint32_t* __restrict__ khi,
                                                      uint32_t* __restrict__ kcnt,
                                                      uint32_t* __restrict__ kj) {
    uint32_t t = blockIdx.x * 256 + threadIdx.x;
    if (t >= n_tokens || !flag[t]) return;
    // sentence of t: the last s with sent_off[s] <= t
    uint32_t lo = 0, hi = n_sent;            // invariant: sent_off[lo] <= t < sent_off[hi]
    while (hi - lo > 1) {
        uint32_t mid = lo + (hi - lo) / 2;
        if (sent_off[mid] <= (uint64_t)t) lo = mid; else hi = mid;
    }
    uint64_t ob = sent_off[lo], oe = sent_off[lo + 1];        // clamped: never index past kpos
    uint32_t s_begin = kpos[ob < n_tokens ? (uint32_t)ob : n_tokens];
    uint32_t s_end = kpos[oe < n_tokens ? (uint32_t)oe : n_tokens];
    uint32_t q = kpos[t];
    uint32_t j = q - s_begin, m = s_end - s_begin, b = width[t];
    uint32_t left = j < b ? j : b;
    uint32_t right = (m - 1 - j) < b ? (m - 1 - j) : b;
    uint32_t w = tokens[t];
    kword[q] = w < V ? w : 0u;
    klo[q] = q - left;
    khi[q] = q + right;
    kcnt[q] = left + right;
    if (kj) kj[q] = j;                        // position among the sentence's survivors
}

__global__ __launch_bounds__(256) void set_u32_kernel(uint32_t* __restrict__ x, uint32_t n,
                                                      uint32_t value) {
    uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) x[i] = value;
}

// Interleaved order: pair counts of the survivors taken in the order perm[0], perm[1], ...
__global__ __launch_bounds__(256) void permuted_counts_kernel(const uint32_t* __restrict__ kcnt,
                                                              const uint32_t* __restrict__ perm,
                                                              const uint32_t* __restrict__ n_kept,
                                                              uint32_t n,
                                                              uint32_t* __restrict__ out) {
    uint32_t r = blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    out[r] = r < *n_kept ? kcnt[perm[r]] : 0u;
}

__global__ __launch_bounds__(256) void emit_pairs_kernel(const uint32_t* __restrict__ kword,
                                                         const uint32_t* __restrict__ klo,
                                                         const uint32_t* __restrict__ khi,
                                                         const uint32_t* __restrict__ poff,
                                                         const uint32_t* __restrict__ n_kept,
                                                         const uint32_t* __restrict__ perm,
                                                         uint32_t* __restrict__ in_idx,
                                                         uint32_t* __restrict__ out_idx,
                                                         uint64_t capacity) {
    uint32_t r = blockIdx.x * 256 + threadIdx.x;        // place in the order of emission
    if (r >= *n_kept) return;
    uint32_t q = perm ? perm[r] : r;                      // which survivor is the center
    uint32_t w = kword[q];
    uint64_t o = poff[r];
    uint32_t last = khi[q] < *n_kept ? khi[q] : *n_kept - 1;   // holds for well-formed sentences
    for (uint32_t c = klo[q]; c <= last; ++c) {
        if (c == q) continue;
        if (o < capacity) {
            if (in_idx) in_idx[o] = w;
            out_idx[o] = kword[c];
        }
        ++o;
    }
}

// scratch layout (uint32): flag[n+1] kpos[n+1] width[n] kword[n] klo[n] khi[n] kcnt[n] poff[n]
// n_kept[8] scan_tmp[...]; interleaved order adds kj[n] cs[n] b0[2n] b1[2n] sort_tmp[...]
size_t pairs_scratch_u32(uint32_t n_tokens, bool interleave) {
    size_t n = n_tokens;
    size_t base = 2 * (n + 1) + 6 * n + 8 + scan_scratch_u32(n_tokens + 1);
    if (interleave) base += 6 * n + 4 + sort_scratch_u32(n_tokens);
    return base;
}

void launch_make_pairs(const PairArgs& a, hipStream_t st) {
    const uint32_t n = a.n_tokens;
    uint32_t* flag = a.scratch;
    uint32_t* kpos = flag + (n + 1);
    uint32_t* width = kpos + (n + 1);
    uint32_t* kword = width + n;
    uint32_t* klo = kword + n;
    uint32_t* khi = klo + n;
    uint32_t* kcnt = khi + n;
    uint32_t* poff = kcnt + n;
    uint32_t* n_kept = poff + n;
    uint32_t* scan_tmp = n_kept + 8;
    uint32_t* extra = scan_tmp + scan_scratch_u32(n + 1);
    uint32_t* kj = a.interleave ? extra : nullptr;
    uint32_t* cs = extra + n;
    // sort buffers (8-byte words) and sort scratch start on 8-byte boundaries
    uint32_t* after_cs = cs + n;
    after_cs += ((uintptr_t)after_cs & 4) ? 1 : 0;
    uint2 *b0 = (uint2*)after_cs, *b1 = b0 + n;
    uint32_t* sort_tmp = (uint32_t*)(b1 + n);
    hipLaunchKernelGGL(token_draws_kernel, dim3(blocks_for((uint64_t)n + 1, 256)), dim3(256), 0, st,
                       a.tokens, n, a.token_base, a.epoch, (uint32_t)a.seed,
                       (uint32_t)(a.seed >> 32), a.B, a.keep, a.V, flag, width, a.err);
    launch_exclusive_scan(flag, kpos, n + 1, scan_tmp, n_kept, st);
    // pair counts of the survivors; entries of kcnt beyond n_kept must read as zero for the scan
    if (n == 0) {
        launch_exclusive_scan(kcnt, poff, 0, scan_tmp, a.total_pairs, st);
        if (a.ctx_off)
            launch_cbow_examples(kcnt, kword, poff, n_kept, 0, flag, kpos, scan_tmp, a.ctx_off,
                                 a.centers, a.cap_examples, a.total_examples, st);
        return;
    }
    const dim3 grid(blocks_for(n, 256)), block(256);
    hipLaunchKernelGGL(set_u32_kernel, grid, block, 0, st, kcnt, n, 0u);
    if (a.interleave) hipLaunchKernelGGL(set_u32_kernel, grid, block, 0, st, kj, n, n);   // sorts last
    hipLaunchKernelGGL(compact_kernel, grid, block, 0, st, a.tokens, n, a.sent_off, a.n_sent, flag,
                       kpos, width, a.V, kword, klo, khi, kcnt, kj);
    if (!a.interleave) {
        launch_exclusive_scan(kcnt, poff, n, scan_tmp, a.total_pairs, st);
        hipLaunchKernelGGL(emit_pairs_kernel, grid, block, 0, st, kword, klo, khi, poff, n_kept,
                           (const uint32_t*)nullptr, a.in_idx, a.out_idx, a.capacity);
        // bag-of-words examples: flag and kpos are free again after the compaction
        if (a.ctx_off)
            launch_cbow_examples(kcnt, kword, poff, n_kept, n, flag, kpos, scan_tmp, a.ctx_off,
                                 a.centers, a.cap_examples, a.total_examples, st);
        return;
    }
    // Round-robin over the sentences: a stable sort of the survivors by their position within the
    // sentence keeps the sentences in order among equal positions.
    uint32_t bits = 1;
    while (bits < 32 && (1ull << bits) <= (uint64_t)n) ++bits;
    uint32_t *sk = nullptr, *perm = nullptr;
    launch_sort_pairs(kj, b0, b1, n, bits, sort_tmp, &sk, &perm, a.err, st);
    hipLaunchKernelGGL(permuted_counts_kernel, grid, block, 0, st, kcnt, perm, n_kept, n, cs);
    launch_exclusive_scan(cs, poff, n, scan_tmp, a.total_pairs, st);
    hipLaunchKernelGGL(emit_pairs_kernel, grid, block, 0, st, kword, klo, khi, poff, n_kept,
                       (const uint32_t*)perm, a.in_idx, a.out_idx, a.capacity);
}

}  // namespace w2v
