// Device-wide exclusive scan and a stable least-significant-digit radix sort of (key, index)
// pairs, up to 8 bits per pass.  Used to group the contributions of adjust by destination row:
// equal keys end up adjacent and, the sort being stable, in increasing order of their original
// slot, so the order in which a row's contributions are summed is fixed by the input alone.
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

// Exclusive scan of one value per thread across the first 256 threads of a block (larger blocks
// pass through with the rest of their threads, for the barriers); returns the exclusive prefix
// and leaves the total in *total_out (shared).
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* wave_sums,
                                                         uint32_t* total_out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = x;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63 && wave < SCAN_THREADS / 64) wave_sums[wave] = incl;
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
// Radix sort.  One or two independent arrays ("jobs") are sorted by the same launches:
//   fill      : clears the digit totals, the tile tickets and the first tile-state array
//   totals    : one read of the keys gives, for every pass at once, how many keys carry each digit
//               (the totals do not depend on the order the earlier passes leave behind)
//   pass x P  : ONE launch per pass.  A block takes the next tile of 256 x ITEMS consecutive elements
//               (ticket counter), ranks its elements among the tile's elements of the same digit in
//               tile order (-> stable), and learns how many elements of each digit the tiles before
//               it hold by looking back over the tile states: a tile first publishes its own digit
//               counts ("partial"), then walks back over its predecessors, adding partial counts
//               until it meets a tile that has already published its prefix ("inclusive"), and
//               publishes its own prefix.  A tile only ever waits for tiles with smaller tickets,
//               which are running or done; the wait is bounded all the same: past the limit the
//               block raises the error flag and goes on with what it has, so every wave ends.
//               The tile is then put in sorted order in LDS and written out position by position,
//               so that neighbouring threads write neighbouring addresses inside a digit's run.
// Between passes an element travels as one 8-byte word (key, index): one coalesced load and one
// store per element and pass, runs of 16 elements filling whole 128-byte lines.  The first pass
// reads the keys alone (the index is the position), the last one writes keys and indices to
// separate arrays, which is what the kernels of adjust read.
// Two tile-state arrays alternate between passes; each block clears its own row of the array the
// next pass will use, so no pass starts on stale states and nothing is cleared between passes.
// ---------------------------------------------------------------------------------------------
constexpr int SORT_THREADS = 256;                    // of the totals kernel
constexpr uint32_t SORT_SMALL_N = 1u << 19;
constexpr int SORT_MAX_PASSES = 4;
constexpr uint32_t SORT_SPIN_LIMIT = 1u << 22;       // fruitless look-back polls before giving up (~ a second)
constexpr int LB_WINDOW = 8;                         // tiles examined per look-back round
constexpr uint64_t ST_PARTIAL = 1ull << 62, ST_INCLUSIVE = 2ull << 62, ST_VALUE = (1ull << 62) - 1;
// Tile shapes.  Large inputs: 512 threads x 16 elements = 8192 per tile -- with 256 digits a digit's
// run in a tile is 32 elements, 256 bytes, on average (tiles of 4096 measured 15 % slower, and
// 1024 threads x 8 or 512 x 8 slower still).  Below SORT_SMALL_N elements: 256 x 4, so that small
// sorts still spread over the chip (2^18 keys: 51 us against 60; from 2^20 keys on the large shape
// wins, 77 us against 123: fewer tiles, shorter look-back).
static inline int sort_shape_for(uint64_t n) { return n < SORT_SMALL_N ? 0 : 1; }
static inline uint32_t sort_tile_of(int shape) { return shape == 0 ? 1024u : 8192u; }

struct SortJobDev {
    const uint32_t* keys_in;     // the caller's keys (pass 0 reads them; never written)
    uint2* buf[2];               // ping-pong buffers of (key, index) words, n each
    uint32_t* out_keys;          // last pass: separate arrays (inside the buffer it does not read)
    uint32_t* out_vals;
    uint32_t n, tiles;
};
struct SortArgs {
    SortJobDev job[2];
    uint32_t njobs, tiles0;      // tiles of job 0 come first in ticket order
    uint32_t passes, shift[SORT_MAX_PASSES], width[SORT_MAX_PASSES];
    uint32_t* totals;            // [2][SORT_MAX_PASSES][256] digit totals
    uint32_t* tickets;           // [SORT_MAX_PASSES]
    uint64_t* state[2];          // [tiles0 + tiles1][256] each
    uint32_t* err;               // sticky error flag of the shard (may be null)
};

__global__ __launch_bounds__(256) void sort_fill_kernel(uint64_t* __restrict__ p, uint64_t count) {
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0ull;
}

// Digit totals of every pass in one read of the keys.  A block covers 256 x 16 keys of one job and
// counts in LDS, one atomic per key and pass.  Word frequencies are skewed, so many lanes of a
// wavefront hold the same digit (in the top pass, most of them): each counter is kept in
// TOT_COPIES copies, chosen by lane number, which divides the number of lanes that queue up on
// one address by that many (integer sums: the order does not matter).
constexpr int TOT_ITEMS = 16;
constexpr int TOT_COPIES = 8;
__global__ __launch_bounds__(SORT_THREADS) void sort_totals_kernel(SortArgs a, uint32_t blocks0) {
    __shared__ uint32_t h[SORT_MAX_PASSES][256 * TOT_COPIES];
    for (int i = threadIdx.x; i < SORT_MAX_PASSES * 256 * TOT_COPIES; i += SORT_THREADS) (&h[0][0])[i] = 0;
    __syncthreads();
    const uint32_t j = blockIdx.x >= blocks0 ? 1u : 0u;
    const uint32_t b = blockIdx.x - (j ? blocks0 : 0u);
    const uint32_t* __restrict__ keys = a.job[j].keys_in;
    const uint32_t n = a.job[j].n;
    const uint32_t base = b * (uint32_t)(SORT_THREADS * TOT_ITEMS) + threadIdx.x;
    const uint32_t copy = threadIdx.x & (TOT_COPIES - 1);
    uint32_t k[TOT_ITEMS];
#pragma unroll
    for (int e = 0; e < TOT_ITEMS; ++e) {
        const uint32_t i = base + (uint32_t)e * SORT_THREADS;
        k[e] = i < n ? keys[i] : 0u;
    }
    for (uint32_t p = 0; p < a.passes; ++p) {
        const uint32_t shift = a.shift[p], mask = (1u << a.width[p]) - 1u;
#pragma unroll
        for (int e = 0; e < TOT_ITEMS; ++e) {
            const uint32_t d = (k[e] >> shift) & mask;
            if (base + (uint32_t)e * SORT_THREADS < n) atomicAdd(&h[p][d * TOT_COPIES + copy], 1u);
        }
    }
    __syncthreads();
    for (uint32_t p = 0; p < a.passes; ++p) {
        uint32_t c = 0;
#pragma unroll
        for (int q = 0; q < TOT_COPIES; ++q) c += h[p][threadIdx.x * TOT_COPIES + q];
        if (c) atomicAdd(&a.totals[(j * SORT_MAX_PASSES + p) * 256 + threadIdx.x], c);
    }
}

template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void sort_pass_kernel(SortArgs a, uint32_t pass) {
    constexpr int TILE = THREADS * ITEMS;
    constexpr int WAVE_SPAN = 64 * ITEMS;
    constexpr int WAVES = THREADS / 64;
    static_assert(THREADS >= 256 && THREADS % 256 == 0, "one thread per digit for the tile's bookkeeping");
    __shared__ uint32_t cnt[WAVES][256];
    __shared__ uint32_t to_global[256];
    __shared__ uint2 s_item[TILE];
    __shared__ uint32_t wave_sums[4];
    __shared__ uint32_t total_all;
    __shared__ uint32_t s_ticket;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool owner = threadIdx.x < 256;                 // thread d < 256 keeps the books of digit d
    if (threadIdx.x == 0) s_ticket = atomicAdd(&a.tickets[pass], 1u);
    for (int i = threadIdx.x; i < WAVES * 256; i += THREADS) (&cnt[0][0])[i] = 0;
    __syncthreads();
    // (< tiles0 + tiles1: one block per tile; the same in every lane, hence a scalar)
    const uint32_t ticket = __builtin_amdgcn_readfirstlane(s_ticket);
    const uint32_t j = (a.njobs > 1 && ticket >= a.tiles0) ? 1u : 0u;
    const uint32_t first_tile = j ? a.tiles0 : 0u;       // ticket of this job's first tile
    const uint32_t tile = ticket - first_tile;
    const SortJobDev& jb = a.job[j];
    const uint32_t n = jb.n;
    const uint32_t shift = a.shift[pass], width = a.width[pass], mask = (1u << width) - 1u;
    const bool first_pass = pass == 0, last_pass = pass + 1 == a.passes;
    const uint2* __restrict__ in = jb.buf[(pass + 1) & 1];       // written by the pass before
    uint64_t* __restrict__ state = a.state[pass & 1];
    // the row of this tile in the array the next pass will use must be clear by then
    if (owner) a.state[(pass + 1) & 1][(uint64_t)ticket * 256 + threadIdx.x] = 0ull;
    // where each digit's elements start in the output: exclusive scan of the job's digit totals
    const uint32_t digit_base = block_exclusive_scan(
        owner ? a.totals[(j * SORT_MAX_PASSES + pass) * 256 + threadIdx.x] : 0u, wave_sums, &total_all);

    // element e of lane l of wave w is number w * WAVE_SPAN + e * 64 + l of the tile (n < 2^31)
    const uint32_t base = tile * (uint32_t)TILE + (uint32_t)wave * WAVE_SPAN + (uint32_t)lane;
    uint32_t key[ITEMS], val[ITEMS], rank[ITEMS];
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
        const uint32_t i = base + (uint32_t)e * 64;
        if (i < n) {
            if (first_pass) { key[e] = jb.keys_in[i]; val[e] = i; }
            else { const uint2 x = in[i]; key[e] = x.x; val[e] = x.y; }
        } else {
            key[e] = 0u; val[e] = 0u;
        }
    }
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
        const bool valid = base + (uint32_t)e * 64 < n;
        const uint32_t d = (key[e] >> shift) & mask;
        // lanes of this wave holding the same digit
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            if (b < (int)width) {                        // (same in every lane)
                const uint64_t bal = __ballot((d >> b) & 1u);
                same &= ((d >> b) & 1u) ? bal : ~bal;
            }
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
    // Thread d owns digit d: the tile's count of the digit, its place in the sorted tile, and the
    // look-back over the tiles before this one.
    uint32_t c[WAVES], tile_count = 0;
    if (owner) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) { c[w] = cnt[w][threadIdx.x]; tile_count += c[w]; }
    }
    uint64_t* mine = state + (uint64_t)ticket * 256 + (threadIdx.x & 255);
    if (owner)
        __hip_atomic_store(mine, (tile == 0 ? ST_INCLUSIVE : ST_PARTIAL) | (uint64_t)tile_count,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t local_start = block_exclusive_scan(tile_count, wave_sums, &total_all);
    if (owner) {
        const uint32_t d = threadIdx.x;
        uint32_t run = local_start;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) { cnt[w][d] = run; run += c[w]; }
        // Look-back, a window of LB_WINDOW tiles at a time: their states are requested together
        // (one memory round trip for the window) and taken in order from the nearest tile back,
        // up to the first that has not published yet (asked for again in the next round) or that
        // carries its prefix (done).
        uint64_t before_tiles = 0;
        if (tile > 0) {
            uint32_t cur = ticket;                       // the next tile to take is cur - 1
            uint32_t polls = 0;
            bool done = false, gave_up = false;
            while (!done) {                              // (the job's first tile is always "inclusive")
                uint64_t s[LB_WINDOW];
#pragma unroll
                for (int w = 0; w < LB_WINDOW; ++w) {
                    const bool inside = cur - first_tile > (uint32_t)w;      // tile cur-1-w is of this job
                    const uint32_t t = inside ? cur - 1u - (uint32_t)w : first_tile;
                    s[w] = __hip_atomic_load(state + (uint64_t)t * 256 + d, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
                }
                uint32_t taken = 0;
#pragma unroll
                for (int w = 0; w < LB_WINDOW; ++w) {
                    const bool inside = cur - first_tile > (uint32_t)w;
                    if (!done && taken == (uint32_t)w && inside && (s[w] >> 62) != 0) {
                        before_tiles += s[w] & ST_VALUE;
                        ++taken;
                        if ((s[w] >> 62) == 2) done = true;
                    }
                }
                cur -= taken;
                if (!done && taken == 0) {               // the nearest tile has not published yet
                    if (++polls >= SORT_SPIN_LIMIT) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
            if (gave_up && a.err) atomicOr(a.err, 2u);
            __hip_atomic_store(mine, ST_INCLUSIVE | ((before_tiles + tile_count) & ST_VALUE),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // output position = to_global[digit] + position in the sorted tile (mod 2^32 arithmetic)
        to_global[d] = digit_base + (uint32_t)before_tiles - local_start;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
        if (base + (uint32_t)e * 64 < n) {
            const uint32_t d = (key[e] >> shift) & mask;
            s_item[cnt[wave][d] + rank[e]] = make_uint2(key[e], val[e]);
        }
    }
    __syncthreads();
    const uint32_t tile_base = tile * (uint32_t)TILE;
    const uint32_t in_tile = min((uint32_t)TILE, n - tile_base);
    uint2* __restrict__ out = jb.buf[pass & 1];
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
        const uint32_t lp = (uint32_t)e * THREADS + threadIdx.x;
        if (lp < in_tile) {
            const uint2 x = s_item[lp];
            const uint32_t pos = to_global[(x.x >> shift) & mask] + lp;   // < n: ranks are a permutation
            if (pos < n) {                               // (only a timed-out look-back can fail this)
                if (last_pass) { jb.out_keys[pos] = x.x; jb.out_vals[pos] = x.y; }
                else out[pos] = x;
            }
        }
    }
}

static inline uint32_t sort_tiles(uint32_t n, int shape) { return blocks_for(n, sort_tile_of(shape)); }

// Scratch of one call over arrays of n0 and n1 elements (n1 = 0: one array), in uint32 (the
// region must be 8-byte aligned).
size_t sort_scratch_u32(uint32_t n0, uint32_t n1) {
    const int shape = sort_shape_for((uint64_t)n0 + n1);
    const uint64_t tiles = (uint64_t)sort_tiles(n0, shape) + sort_tiles(n1, shape);
    return 2 * SORT_MAX_PASSES * 256 + 8 + 2 * (size_t)(2 * tiles * 256) + 16;
}

// totals, tickets and the first state array: one stretch of 8-byte words at the start of tmp
static uint64_t sort_clear_words64(uint32_t tiles) {
    return (2 * SORT_MAX_PASSES * 256 + 8) / 2 + (uint64_t)tiles * 256;
}

FillJob sort_clear_job(const SortJob* jobs, int njobs, uint32_t* tmp) {
    uint64_t n_all = 0;
    for (int i = 0; i < njobs && i < 2; ++i) n_all += jobs[i].n;
    if (n_all == 0) return FillJob{tmp, 0u, 0u};
    const int shape = sort_shape_for(n_all);
    uint32_t tiles = 0;
    for (int i = 0; i < njobs && i < 2; ++i)
        if (jobs[i].n) tiles += sort_tiles(jobs[i].n, shape);
    return FillJob{tmp, (uint32_t)(2 * sort_clear_words64(tiles)), 0u};
}

void launch_sort_jobs(const SortJob* jobs, int njobs, uint32_t bits, uint32_t* tmp, uint32_t* err,
                      hipStream_t st, bool cleared) {
    if (bits == 0) bits = 1;
    if (bits > 32) bits = 32;
    SortArgs a{};
    // empty arrays need nothing; results of an empty job are its first buffer
    int live = 0;
    uint64_t n_all = 0;
    for (int i = 0; i < njobs && i < 2; ++i) {
        *jobs[i].out_keys = (uint32_t*)jobs[i].buf0;
        *jobs[i].out_vals = (uint32_t*)jobs[i].buf0;
        if (jobs[i].n) n_all += jobs[i].n;
    }
    if (n_all == 0) return;
    const int shape = sort_shape_for(n_all);
    a.passes = (bits + 7) / 8;
    for (uint32_t p = 0, lo = 0; p < a.passes; ++p) {      // digits of nearly equal width
        const uint32_t w = (bits - lo + (a.passes - p) - 1) / (a.passes - p);
        a.shift[p] = lo; a.width[p] = w; lo += w;
    }
    for (int i = 0; i < njobs && i < 2; ++i) {
        if (jobs[i].n == 0) continue;
        SortJobDev& d = a.job[live];
        d.keys_in = jobs[i].keys_in; d.n = jobs[i].n; d.tiles = sort_tiles(jobs[i].n, shape);
        d.buf[0] = jobs[i].buf0; d.buf[1] = jobs[i].buf1;
        // the last pass reads buf[passes & 1] (or the caller's keys) and writes the other buffer
        uint2* dst = d.buf[(a.passes - 1) & 1];
        d.out_keys = (uint32_t*)dst;
        d.out_vals = (uint32_t*)dst + d.n;
        *jobs[i].out_keys = d.out_keys;
        *jobs[i].out_vals = d.out_vals;
        ++live;
    }
    a.njobs = live;
    a.tiles0 = a.job[0].tiles;
    const uint32_t tiles = a.job[0].tiles + (live > 1 ? a.job[1].tiles : 0u);
    a.totals = tmp;
    a.tickets = tmp + 2 * SORT_MAX_PASSES * 256;
    a.state[0] = (uint64_t*)(tmp + 2 * SORT_MAX_PASSES * 256 + 8);
    a.state[1] = a.state[0] + (uint64_t)tiles * 256;
    a.err = err;
    if (!cleared) {
        const uint64_t clear64 = sort_clear_words64(tiles);
        hipLaunchKernelGGL(sort_fill_kernel, dim3(blocks_for(clear64, 256)), dim3(256), 0, st,
                           (uint64_t*)tmp, clear64);
    }
    const uint32_t blocks0 = blocks_for(a.job[0].n, SORT_THREADS * TOT_ITEMS);
    const uint32_t blocks1 = live > 1 ? blocks_for(a.job[1].n, SORT_THREADS * TOT_ITEMS) : 0u;
    hipLaunchKernelGGL(sort_totals_kernel, dim3(blocks0 + blocks1), dim3(SORT_THREADS), 0, st, a, blocks0);
    for (uint32_t p = 0; p < a.passes; ++p) {
        if (shape == 0)
            hipLaunchKernelGGL((sort_pass_kernel<256, 4>), dim3(tiles), dim3(256), 0, st, a, p);
        else
            hipLaunchKernelGGL((sort_pass_kernel<512, 16>), dim3(tiles), dim3(512), 0, st, a, p);
    }
}

void launch_sort_pairs(const uint32_t* keys_in, uint2* buf0, uint2* buf1, uint32_t n, uint32_t bits,
                       uint32_t* tmp, uint32_t** out_keys, uint32_t** out_vals, uint32_t* err,
                       hipStream_t st) {
    SortJob job{keys_in, n, buf0, buf1, out_keys, out_vals};
    launch_sort_jobs(&job, 1, bits, tmp, err, st);
}

}  // namespace w2v
