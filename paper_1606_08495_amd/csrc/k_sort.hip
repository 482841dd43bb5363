// Device-wide exclusive scan and a stable least-significant-digit radix sort of (key, value)
// pairs, 8 bits per pass.  Used to group the contributions of adjust by destination row: equal
// keys end up adjacent and, the sort being stable, in increasing order of their original slot, so
// the order in which a row's contributions are summed is fixed by the input alone.
#include "common.h"

namespace w2v {

static inline unsigned blocks_for(uint64_t items, unsigned per_block) {
    return (unsigned)((items + per_block - 1) / per_block);
}

// ---------------------------------------------------------------------------------------------
// Scan.  Blocks of 256 threads x 8 items: (1) per-block sums, (2) one block scans the sums with a
// running carry, (3) per-block local scan plus the block's offset.
// ---------------------------------------------------------------------------------------------
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

// Exclusive scan of one value per thread across a 256-thread block; returns the exclusive prefix
// and leaves the block total in *total_out (shared).
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* wave_sums,
                                                         uint32_t* total_out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = x;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < SCAN_THREADS / 64; ++w) {
        uint32_t s = wave_sums[w];
        if (w < wave) base += s;
    }
    if (threadIdx.x == SCAN_THREADS - 1) *total_out = base + incl;
    __syncthreads();
    return base + incl - x;
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_block_sums_kernel(
    const uint32_t* __restrict__ in, uint32_t n, uint32_t* __restrict__ sums) {
    __shared__ uint32_t wave_sums[4];
    __shared__ uint32_t total;
    uint64_t base = (uint64_t)blockIdx.x * SCAN_TILE + (uint64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t s = 0;
#pragma unroll
    for (int e = 0; e < SCAN_ITEMS; ++e)
        if (base + e < n) s += in[base + e];
    block_exclusive_scan(s, wave_sums, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_sums_kernel(uint32_t* __restrict__ sums,
                                                                 uint32_t nb,
                                                                 uint32_t* __restrict__ total_out) {
    __shared__ uint32_t wave_sums[4];
    __shared__ uint32_t total;
    uint32_t carry = 0;
    for (uint32_t start = 0; start < nb; start += SCAN_THREADS) {
        uint32_t i = start + threadIdx.x;
        uint32_t x = i < nb ? sums[i] : 0u;
        uint32_t ex = block_exclusive_scan(x, wave_sums, &total);
        if (i < nb) sums[i] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0 && total_out) *total_out = carry;
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_apply_kernel(const uint32_t* __restrict__ in,
                                                                  uint32_t* __restrict__ out,
                                                                  uint32_t n,
                                                                  const uint32_t* __restrict__ sums) {
    __shared__ uint32_t wave_sums[4];
    __shared__ uint32_t total;
    uint64_t base = (uint64_t)blockIdx.x * SCAN_TILE + (uint64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS];
    uint32_t s = 0;
#pragma unroll
    for (int e = 0; e < SCAN_ITEMS; ++e) {
        v[e] = (base + e < n) ? in[base + e] : 0u;
        s += v[e];
    }
    uint32_t run = block_exclusive_scan(s, wave_sums, &total) + sums[blockIdx.x];
#pragma unroll
    for (int e = 0; e < SCAN_ITEMS; ++e) {
        if (base + e < n) out[base + e] = run;
        run += v[e];
    }
}

size_t scan_scratch_u32(uint32_t n) { return blocks_for(n, SCAN_TILE) + 1; }

void launch_exclusive_scan(const uint32_t* in, uint32_t* out, uint32_t n, uint32_t* tmp,
                           uint32_t* total, hipStream_t st) {
    unsigned nb = blocks_for(n, SCAN_TILE);
    if (n == 0) {
        hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(SCAN_THREADS), 0, st, tmp, 0u, total);
        return;
    }
    hipLaunchKernelGGL(scan_block_sums_kernel, dim3(nb), dim3(SCAN_THREADS), 0, st, in, n, tmp);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(SCAN_THREADS), 0, st, tmp, nb, total);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(nb), dim3(SCAN_THREADS), 0, st, in, out, n, tmp);
}

// ---------------------------------------------------------------------------------------------
// Radix sort pass.  A block owns a tile of 256 x ITEMS consecutive elements; wave w of the block owns
// the w-th quarter of the tile and walks it in order, 64 elements at a time.
//   histogram : per-block digit counts, stored digit-major [256][blocks]
//   digit scan: per digit, exclusive prefix of its counts over the blocks, and the digit's total
//   (prefix of the totals + that prefix = where a block's elements of a digit start in the output)
//   scatter   : each element's position = that start + its rank among the block's elements with
//               the same digit, counted in tile order -> stable.  The tile is first put in that
//               order in LDS and then written out position by position, so that the stores of
//               neighbouring threads fall into the same digit run (coalesced pieces of about
//               tile/256 elements) instead of single 4-byte stores all over the output.
// ---------------------------------------------------------------------------------------------
constexpr int SORT_THREADS = 256;
constexpr int SORT_WAVES = SORT_THREADS / 64;
// Elements per thread (ITEMS): 16 for large inputs (long coalesced pieces, few blocks to scan over),
// 4 below SORT_SMALL_N elements, where 16 would leave most of the chip without a block.
constexpr int SORT_ITEMS_LARGE = 16;
constexpr int SORT_ITEMS_SMALL = 4;
constexpr uint32_t SORT_SMALL_N = 1u << 22;
static inline int sort_items_for(uint32_t n) { return n < SORT_SMALL_N ? SORT_ITEMS_SMALL : SORT_ITEMS_LARGE; }

template <int SORT_ITEMS>
__global__ __launch_bounds__(SORT_THREADS) void sort_hist_kernel(const uint32_t* __restrict__ keys,
                                                                 uint32_t n, uint32_t shift,
                                                                 uint32_t nblocks,
                                                                 uint32_t* __restrict__ hist) {
    constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS;
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    uint64_t base = (uint64_t)blockIdx.x * SORT_TILE;
#pragma unroll
    for (int e = 0; e < SORT_ITEMS; ++e) {
        uint64_t i = base + (uint64_t)e * SORT_THREADS + threadIdx.x;
        const bool valid = i < n;
        const uint32_t d = valid ? (keys[i] >> shift) & 255u : 0u;
        // long stretches of one key (a very frequent word, or the sentinel of slots that are left
        // out) would serialise 64 atomics on one counter: one lane adds for the whole wavefront
        const uint64_t live = __ballot(valid);
        const uint32_t d0 = __shfl(d, live ? __ffsll((long long)live) - 1 : 0, 64);
        if (live && __ballot(valid && d == d0) == live) {
            if ((threadIdx.x & 63) == __ffsll((long long)live) - 1) atomicAdd(&h[d0], (uint32_t)__popcll(live));
        } else if (valid) {
            atomicAdd(&h[d], 1u);
        }
    }
    __syncthreads();
    hist[(uint64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

template <int SORT_ITEMS>
__global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(
    const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in,
    uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out, uint32_t n, uint32_t shift,
    uint32_t nblocks, const uint32_t* __restrict__ offsets, const uint32_t* __restrict__ digit_total) {
    constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS;
    constexpr int SORT_WAVE_SPAN = 64 * SORT_ITEMS;
    __shared__ uint32_t cnt[SORT_WAVES][256];
    __shared__ uint32_t to_global[256];
    __shared__ uint32_t s_key[SORT_TILE];
    __shared__ uint32_t s_val[SORT_TILE];
    __shared__ uint32_t wave_sums[4];
    __shared__ uint32_t total_all;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // where each digit's elements start in the output: exclusive scan of the 256 digit totals
    const uint32_t digit_base = block_exclusive_scan(digit_total[threadIdx.x], wave_sums, &total_all);
#pragma unroll
    for (int w = 0; w < SORT_WAVES; ++w) cnt[w][threadIdx.x] = 0;
    __syncthreads();

    uint64_t base = (uint64_t)blockIdx.x * SORT_TILE + (uint64_t)wave * SORT_WAVE_SPAN;
    uint32_t key[SORT_ITEMS], val[SORT_ITEMS], rank[SORT_ITEMS];
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int e = 0; e < SORT_ITEMS; ++e) {
        uint64_t i = base + (uint64_t)e * 64 + lane;
        bool valid = i < n;
        key[e] = valid ? keys_in[i] : 0u;
        val[e] = valid ? (vals_in ? vals_in[i] : (uint32_t)i) : 0u;
        uint32_t d = (key[e] >> shift) & 255u;
        // lanes of this wave holding the same digit
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            uint64_t bal = __ballot((d >> b) & 1u);
            same &= ((d >> b) & 1u) ? bal : ~bal;
        }
        uint32_t before = 0;
        if (valid) {
            before = cnt[wave][d];
            rank[e] = before + (uint32_t)__popcll(same & below);
        } else {
            rank[e] = 0;
        }
        // The reads above are issued before the write below by every lane of the wave (one
        // instruction stream), so the leader's update cannot be seen by this step's readers.
        if (valid && (same & below) == 0) cnt[wave][d] = before + (uint32_t)__popcll(same);
    }
    __syncthreads();
    // Thread t owns digit t.  The tile is first put in sorted order in LDS (digit by digit, within
    // a digit wave by wave), then copied out position by position: neighbouring threads then write
    // neighbouring addresses inside each digit's run instead of 4-byte pieces all over the output.
    {
        const uint32_t d = threadIdx.x;
        uint32_t c[SORT_WAVES], tile_count = 0;
#pragma unroll
        for (int w = 0; w < SORT_WAVES; ++w) { c[w] = cnt[w][d]; tile_count += c[w]; }
        const uint32_t local_start = block_exclusive_scan(tile_count, wave_sums, &total_all);
        uint32_t run = local_start;
#pragma unroll
        for (int w = 0; w < SORT_WAVES; ++w) { cnt[w][d] = run; run += c[w]; }
        // output position = to_global[digit] + position in the sorted tile (mod 2^32 arithmetic)
        to_global[d] = digit_base + offsets[(uint64_t)d * nblocks + blockIdx.x] - local_start;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < SORT_ITEMS; ++e) {
        uint64_t i = base + (uint64_t)e * 64 + lane;
        if (i < n) {
            const uint32_t d = (key[e] >> shift) & 255u;
            const uint32_t lp = cnt[wave][d] + rank[e];
            s_key[lp] = key[e];
            s_val[lp] = val[e];
        }
    }
    __syncthreads();
    const uint64_t tile_base = (uint64_t)blockIdx.x * SORT_TILE;
    const uint32_t in_tile = (uint32_t)min((uint64_t)SORT_TILE, (uint64_t)n - tile_base);
#pragma unroll
    for (int e = 0; e < SORT_ITEMS; ++e) {
        const uint32_t lp = (uint32_t)e * SORT_THREADS + threadIdx.x;
        if (lp < in_tile) {
            const uint32_t k = s_key[lp];
            const uint32_t pos = to_global[(k >> shift) & 255u] + lp;
            keys_out[pos] = k;
            vals_out[pos] = s_val[lp];
        }
    }
}

// Block d turns the per-block counts of digit d into exclusive prefixes over the blocks (in place)
// and writes the digit's total.
__global__ __launch_bounds__(SCAN_THREADS) void sort_digit_scan_kernel(uint32_t* __restrict__ hist,
                                                                       uint32_t nblocks,
                                                                       uint32_t* __restrict__ digit_total) {
    __shared__ uint32_t wave_sums[4];
    __shared__ uint32_t total;
    uint32_t* row = hist + (uint64_t)blockIdx.x * nblocks;
    uint32_t carry = 0;
    for (uint32_t start = 0; start < nblocks; start += SCAN_THREADS) {
        uint32_t i = start + threadIdx.x;
        uint32_t x = i < nblocks ? row[i] : 0u;
        uint32_t ex = block_exclusive_scan(x, wave_sums, &total);
        if (i < nblocks) row[i] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) digit_total[blockIdx.x] = carry;
}

size_t sort_scratch_u32(uint32_t n) {
    uint32_t nblocks = blocks_for(n, SORT_THREADS * sort_items_for(n));
    uint32_t hist = 256u * (nblocks ? nblocks : 1u);
    return (size_t)hist + 256 + 8;
}

void launch_sort_pairs(const uint32_t* keys_in, uint32_t* k0, uint32_t* v0, uint32_t* k1, uint32_t* v1,
                       uint32_t n, uint32_t bits, uint32_t* tmp, uint32_t** out_keys,
                       uint32_t** out_vals, hipStream_t st) {
    if (bits == 0) bits = 1;
    uint32_t passes = (bits + 7) / 8;
    const bool small = sort_items_for(n) == SORT_ITEMS_SMALL;
    uint32_t nblocks = blocks_for(n, SORT_THREADS * sort_items_for(n));
    uint32_t hist_len = 256u * nblocks;
    uint32_t* hist = tmp;
    uint32_t* digit_total = tmp + hist_len;
    *out_keys = k0;
    *out_vals = v0;
    if (n == 0) return;
    const uint32_t* kin = keys_in;
    const uint32_t* vin = nullptr;           // first pass: value i = i
    uint32_t *kout = k0, *vout = v0;
    for (uint32_t ps = 0; ps < passes; ++ps) {
        uint32_t shift = ps * 8;
        if (small)
            hipLaunchKernelGGL(sort_hist_kernel<SORT_ITEMS_SMALL>, dim3(nblocks), dim3(SORT_THREADS), 0,
                               st, kin, n, shift, nblocks, hist);
        else
            hipLaunchKernelGGL(sort_hist_kernel<SORT_ITEMS_LARGE>, dim3(nblocks), dim3(SORT_THREADS), 0,
                               st, kin, n, shift, nblocks, hist);
        hipLaunchKernelGGL(sort_digit_scan_kernel, dim3(256), dim3(SCAN_THREADS), 0, st, hist,
                           nblocks, digit_total);
        if (small)
            hipLaunchKernelGGL(sort_scatter_kernel<SORT_ITEMS_SMALL>, dim3(nblocks), dim3(SORT_THREADS),
                               0, st, kin, vin, kout, vout, n, shift, nblocks, hist, digit_total);
        else
            hipLaunchKernelGGL(sort_scatter_kernel<SORT_ITEMS_LARGE>, dim3(nblocks), dim3(SORT_THREADS),
                               0, st, kin, vin, kout, vout, n, shift, nblocks, hist, digit_total);
        *out_keys = kout;
        *out_vals = vout;
        kin = kout; vin = vout;
        if (kout == k0) { kout = k1; vout = v1; } else { kout = k0; vout = v0; }
    }
}

}  // namespace w2v
