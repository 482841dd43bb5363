// adjust: segmented, fixed-order reduction of row contributions and the single write-back.
//
// After the destination keys are sorted, the contributions to one row are a run of adjacent
// entries.  The entry list is cut into chunks of a fixed number of entries; one lane group walks one
// chunk in order with the running sum in registers.  A run that lies inside a chunk is finished by
// that group (one read-modify-write of the destination row).  A run cut by a chunk border leaves
// one partial row on each side of the border ("slots" 2b and 2b+1 of border b, tagged with the
// row); the list of slots is then reduced by the same scheme, level after level, until a level
// fits one chunk.  Which entries meet in which partial sum depends only on the entry positions, so
// the result is bitwise reproducible, and a row that collects millions of contributions is spread
// over as many groups as it has chunks.
#include "rows.h"
#include "loss.h"

namespace w2v {

static inline unsigned blocks_for(uint64_t items, unsigned per_block) {
    return (unsigned)((items + per_block - 1) / per_block);
}

// Block sizes, measured per kernel family: the input-side kernels run 6 % faster in blocks of 128
// than of 256 (and no faster in 64); the output-side kernel is 7 % slower in 128 at one wavefront
// per row and 8 % faster at sixteen lanes per row.
constexpr int ADJ_THREADS = 256;                   // higher levels, write-back
constexpr int USEG_THREADS = 128;                  // input-side kernels
constexpr int wown_threads(int G) { return G == 16 ? 128 : 256; }     // output-side kernel
constexpr int TAIL_C = 16;     // entries per chunk, higher levels (even, so a border's two slots
                               // fall into one chunk)
constexpr uint32_t NOKEY = 0xFFFFFFFFu;   // compares unequal to every masked key
constexpr uint32_t ALONE = KEY_ALONE;

uint32_t tail_entries_per_chunk() { return TAIL_C; }
// Pairs per chunk of the input-side kernel: about useg_e(G) entries (pairs x slots), 2..useg_maxp(G)
// pairs.  Longer chunks cut fewer runs (fewer partial rows for the higher levels: -2.7 % on the
// benchmark step, -6 % with k = 25, against chunks of 48 entries); with sixteen groups to a block
// (rows of up to 64 floats) the short chunks stay: there the longer ones measured 1 % slower.
constexpr int useg_e(int G) { return G == 16 ? 48 : 192; }
constexpr int useg_maxp(int G) { return G == 16 ? 16 : 32; }            // pairs per chunk, at most
constexpr int useg_maxe(int G) {                 // entries, at most: c T < E + T, and 2 T, T <= 65
    return useg_e(G) + 66 < 136 ? 136 : useg_e(G) + 66;
}
// A lane group walks its chunk pair by pair, one memory round trip each, so a small minibatch cut
// into long chunks leaves the chip to a handful of groups (4096 pairs in chunks of 32: 128 groups,
// 109 us of row latency in a row): below USEG_MIN_CHUNKS chunks the chunks shrink, down to two pairs.
// (32768: from 2^20 pairs on the long chunks stay; 2^18 pairs run 5 % faster per step than with
// 4096, the 2^17 examples of a bag-of-words minibatch 4 %; 4096 pairs the same.)
constexpr uint32_t USEG_MIN_CHUNKS = 32768;
uint32_t useg_pairs_per_chunk(uint32_t T, uint32_t d4, uint32_t n) {
    const int G = d4 <= 16 ? 16 : (d4 <= 32 ? 32 : 64);                 // as W2V_DISPATCH_GEOM
    uint32_t c = ((uint32_t)useg_e(G) + T - 1) / T;
    if (c < 2) c = 2;
    if (c > (uint32_t)useg_maxp(G)) c = useg_maxp(G);
    const uint32_t fill = n / USEG_MIN_CHUNKS;                          // pairs per chunk that still give that many
    if (c > fill) c = fill < 2 ? 2 : fill;
    return c;
}

// ---------------------------------------------------------------------------------------------
// Generic chunk walker for entries that each name ONE source row.
//   SRC = 0: output-vector side, level 1: source U[in_idx[sidx / T]], weight coeffs[sidx]
//   SRC = 1: higher level: source src_rows[entry], weight 1 (or none when flagged empty)
// C entries per group (C <= G), loads issued D entries at a time (source rows and, for runs that
// finish inside the chunk, the destination rows as well).
// ---------------------------------------------------------------------------------------------
struct SegArgs {
    const float4* src;          // SRC 0: U; SRC 1: partial rows of the previous level
    float4* dst;                // matrix updated in place
    RowGeom g;
    const uint32_t* skey;       // destination key per entry
    const uint32_t* sidx;       // SRC 0 only
    const uint32_t* in_idx;     // SRC 0 only
    const float* coeffs;        // SRC 0 only
    uint32_t entries, T;
    float alpha;
    float4* prows; uint32_t* pkeys;    // this level's partial slots
    bool skip_alone;                   // wown_kernel: runs of length one are handled elsewhere
    // DEFER: finished sums are not added to dst but parked in the input side's delta buffer
    float4* defer_rows; uint32_t* defer_keys;
    uint32_t level, cp;                // level of this pass (1 = first), pairs per input-side chunk
    const CallScalars* dev;            // optional: the learning rate is read from here
};

// DEFER (higher levels of the input side): a run finished here must not touch the input matrix
// yet -- the output side may still be reading it -- so its sum goes to the delta buffer, from
// where apply_delta_kernel adds it with the same fma.  Its place there: every entry of a higher
// level stands at a chunk border of the level below, and so, level by level, at a border of the
// input-side kernel's chunk grid; the pair position right after that border lies inside the run,
// is not the run's first pair (the run was cut there), and so holds no sum of its own.  Runs are
// disjoint ranges of pair positions, hence no two finished runs share a place.
// (vb: the block's number among the blocks of this walk -- the kernel below passes blockIdx.x, a
// launch that carries several walks the block's offset within its own)
template <int G, int NV, int C, int D, int SRC, bool DEFER = false>
__device__ __forceinline__ void seg_body(const SegArgs& a, uint32_t vb) {
    static_assert(C <= G && C % D == 0, "chunk must fit a lane group");
    const float alpha = a.dev ? a.dev->alpha : a.alpha;
    const int l = threadIdx.x % G;
    const uint32_t c = (vb * (uint32_t)ADJ_THREADS + threadIdx.x) / G;
    const uint32_t nchunks = (a.entries + C - 1) / C;
    if (c >= nchunks) return;
    const uint32_t e0 = c * C;
    const uint32_t cnt = min((uint32_t)C, a.entries - e0);
    const uint32_t d4 = a.g.d4;
    const uint64_t s4 = a.g.stride4;

    // ---- per-entry facts, entry e0+l in lane l ----
    const bool valid = (uint32_t)l < cnt;
    uint32_t key = NOKEY, srow = 0;
    float coef = 1.0f;
    int has = 0;
    if (valid) {
        uint32_t raw = a.skey[e0 + l];
        if (SRC == 0) {
            key = raw;
            uint32_t q = a.sidx[e0 + l];
            srow = a.in_idx[q / a.T];          // range-checked copy
            coef = a.coeffs[q];
            has = 1;
        } else {
            key = raw & KEY_MASK;
            srow = e0 + l;
            has = (raw != KEY_NONE) && !(raw & KEY_ZERO);
        }
    }
    const uint32_t real_limit = (SRC == 0) ? NOKEY : KEY_MASK;   // keys >= this name no row
    if (SRC == 1) {
        // Most slots of a level are unused.  No run passes through a chunk of unused slots only:
        // its own two slots are unused as well, and that is all there is to do.
        const uint64_t any = __ballot(valid && key < real_limit);
        const int first_lane = (int)(threadIdx.x % 64) / G * G;
        const uint64_t group_bits = G >= 64 ? ~0ull : ((1ull << (G & 63)) - 1ull);
        if (((any >> first_lane) & group_bits) == 0) {
            if (l == 0) {
                if (c > 0) a.pkeys[2 * c - 1] = KEY_NONE;
                if (c + 1 < nchunks) a.pkeys[2 * c] = KEY_NONE;
            }
            return;
        }
    }
    uint32_t key_prev = NOKEY, key_after = NOKEY;
    if (e0 > 0) { uint32_t r = a.skey[e0 - 1]; key_prev = (SRC == 0) ? r : (r & KEY_MASK); }
    if (e0 + cnt < a.entries) { uint32_t r = a.skey[e0 + cnt]; key_after = (SRC == 0) ? r : (r & KEY_MASK); }
    uint32_t next = __shfl(key, l + 1, G);
    if ((uint32_t)l + 1 >= cnt) next = key_after;
    const uint32_t key0 = __shfl(key, 0, G);
    const bool open_head = (key_prev == key0);
    const int ends = valid && (next != key);
    const int in_head = open_head && (key == key0);
    const int real = key < real_limit;
    const int complete = ends && !in_head && real;

    float4 acc[NV];
    clear<NV>(acc);
    uint32_t head_key = KEY_NONE, tail_key = KEY_NONE;
    const uint32_t head_slot = 2 * c - 1, tail_slot = 2 * c;   // used only when they exist

    // Register sets srcv[t] / dstv[t] hold the source row of an entry and, when its run finishes
    // inside the chunk, the destination row.  Entry e uses set e % D; as soon as an entry has been
    // consumed its set is refilled with entry e + D, so D entries' rows stay in flight.
    float4 srcv[D][NV], dstv[D][NV];
    auto fetch = [&](int e, float4 (&sv)[NV], float4 (&dv)[NV]) {
        uint32_t sr = __shfl(srow, e, G);
        int h = __shfl(has, e, G);
        int cm = __shfl(complete, e, G);
        uint32_t dk = __shfl(key, e, G);
        load_row_if<G, NV>(h != 0, a.src + (uint64_t)sr * s4, d4, l, sv);
        load_row_if<G, NV>(cm != 0 && !DEFER, a.dst + (uint64_t)(cm ? dk : 0u) * s4, d4, l, dv);
    };
#pragma unroll
    for (int t = 0; t < D; ++t) fetch(t, srcv[t], dstv[t]);
#pragma unroll
    for (int b = 0; b < C; b += D) {
#pragma unroll
        for (int t = 0; t < D; ++t) {
            const int e = b + t;
            float cf = __shfl(coef, e, G);
            int h = __shfl(has, e, G);
            int en = __shfl(ends, e, G);
            int cm = __shfl(complete, e, G);
            int ih = __shfl(in_head, e, G);
            int rl = __shfl(real, e, G);
            uint32_t dk = __shfl(key, e, G);
            if (h) axpy<NV>(cf, srcv[t], acc);
            if (en) {
                if (cm && DEFER) {
                    uint32_t pos = e0 + (uint32_t)e;
                    for (uint32_t lv = a.level; lv > 1; --lv) pos = ((pos + 2) >> 1) * (uint32_t)C;
                    pos = ((pos + 2) >> 1) * a.cp;
                    store_row<G, NV>(a.defer_rows + (uint64_t)pos * s4, d4, l, acc);
                    if (l == 0) a.defer_keys[pos] = dk;
                } else if (cm) {
                    float4 out[NV];
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        out[v].x = fmaf(alpha, acc[v].x, dstv[t][v].x);
                        out[v].y = fmaf(alpha, acc[v].y, dstv[t][v].y);
                        out[v].z = fmaf(alpha, acc[v].z, dstv[t][v].z);
                        out[v].w = fmaf(alpha, acc[v].w, dstv[t][v].w);
                    }
                    store_row<G, NV>(a.dst + (uint64_t)dk * s4, (uint32_t)s4, l, out);
                } else if (ih && rl) {      // the run came in from the previous chunk and ends here
                    store_row<G, NV>(a.prows + (uint64_t)head_slot * s4, d4, l, acc);
                    head_key = dk;
                }
                clear<NV>(acc);
            }
            if (b + D < C) fetch(e + D, srcv[t], dstv[t]);
        }
    }
    // ---- the last run may go on into the next chunk ----
    {
        const int last = (int)cnt - 1;
        int en = __shfl(ends, last, G);
        int ih = __shfl(in_head, last, G);
        int rl = __shfl(real, last, G);
        uint32_t dk = __shfl(key, last, G);
        if (!en && rl) {
            if (ih) {               // one run covers the whole chunk: one partial, in the head slot
                store_row<G, NV>(a.prows + (uint64_t)head_slot * s4, d4, l, acc);
                head_key = dk;
                tail_key = dk | KEY_ZERO;
            } else {
                store_row<G, NV>(a.prows + (uint64_t)tail_slot * s4, d4, l, acc);
                tail_key = dk;
            }
        }
    }
    if (l == 0) {
        if (c > 0) a.pkeys[head_slot] = head_key;
        if (c + 1 < nchunks) a.pkeys[tail_slot] = tail_key;
    }
}

template <int G, int NV, int C, int D, int SRC, bool DEFER = false>
__global__ __launch_bounds__(ADJ_THREADS) void seg_kernel(SegArgs a) {
    seg_body<G, NV, C, D, SRC, DEFER>(a, blockIdx.x);
}

// ---------------------------------------------------------------------------------------------
// Output-vector side, level 1, with run ownership.  A grid of chunks of C entries only decides WHO
// sums a run, not where it is cut:
//  * a run that starts in chunk c and ends before the end of chunk c+1 ("short", at most 2C entries)
//    is summed entirely by group c, which reads on past its chunk's end and finishes the row with
//    one read-modify-write; the group of chunk c+1 skips those entries;
//  * a run that reaches chunk c+2 ("long": a frequent word) is cut only at multiples of L entries
//    (cells).  Each piece is summed by one group -- the group of the chunk in which the run starts,
//    or of the chunk at the cell's start -- which streams on through the cell.  A piece that is the
//    whole run is finished at once; otherwise it is left in the cell's border slots (two per cell
//    border, as in seg_kernel) for the higher levels.
// Short or long follows from the run's own extent on the chunk grid, so every group that meets a
// run decides alike, from the keys at six fixed positions around its chunk.  No partial row is
// written unless a word collects more than L contributions or so.
// ---------------------------------------------------------------------------------------------
constexpr int WOWN_C = 16;
constexpr int WOWN_L = 64;                   // cell size for long runs, a multiple of C (128: the
                                             // output-side kernel 9 % slower, 32: more levels above)
constexpr int WOWN_WIN = 3 * WOWN_C + 2;     // keys staged: positions base-C-1 .. base+2C
constexpr int WOWN_E = 2 * WOWN_C;           // positions summed from LDS facts: base .. base+2C-1
enum : uint32_t { ACT_SKIP = 0, ACT_ADD = 1, ACT_COMPLETE = 2, ACT_HEAD = 3 };

uint32_t wseg_entries_per_chunk() { return WOWN_L; }

template <int G, int NV, int D>
__device__ __forceinline__ void wown_body(const SegArgs& a, uint32_t vb) {
    constexpr int WOWN_THREADS = wown_threads(G);
    constexpr int GROUPS = WOWN_THREADS / G;
    constexpr int C = WOWN_C, L = WOWN_L;
    static_assert(L % C == 0 && C == 16 && G >= 16, "grid shapes");
    const float alpha = a.dev ? a.dev->alpha : a.alpha;
    __shared__ uint32_t s_key[GROUPS][WOWN_WIN];
    __shared__ uint32_t s_srow[GROUPS][WOWN_E];
    __shared__ float s_coef[GROUPS][WOWN_E];
    __shared__ uint32_t s_act[GROUPS][WOWN_E];
    __shared__ uint32_t s_list[GROUPS][WOWN_E];
    const int l = threadIdx.x % G, grp = threadIdx.x / G;
    const uint32_t c = vb * (uint32_t)GROUPS + grp;
    const uint32_t nchunks = (a.entries + C - 1) / C;
    const bool active = c < nchunks;
    const int64_t base = (int64_t)c * C;
    for (int i = l; i < WOWN_WIN; i += G) {
        int64_t pos = base - C - 1 + i;
        s_key[grp][i] = (active && pos >= 0 && pos < (int64_t)a.entries) ? a.skey[pos] : NOKEY;
    }
    __syncthreads();
    auto K = [&](int rel) -> uint32_t { return s_key[grp][rel + C + 1]; };   // rel = position - base
    const uint32_t kbm = K(-C - 1), kb = K(-1), k0 = K(0), kC = K(C), k2C = K(2 * C), klast = K(C - 1);
    const bool head_exists = active && kb == k0;
    const bool head_long = head_exists && !(kbm != k0 && kC != k0);
    const bool own_head = head_long && (base % L) == 0;          // a cell begins here: the piece is ours
    const bool last_in_head = head_exists && klast == k0;
    const bool ext_ok = klast != NOKEY && !last_in_head && k2C != klast;
    // does the run through the chunk's last entry go on, as a long piece that this group owns?
    const bool cont = active && klast != NOKEY && kC == klast && (last_in_head ? own_head : k2C == klast);
    // The positions this group sums are listed densely in s_list (positions that are skipped --
    // another group's, or rows handled elsewhere -- take no place in the load pipeline below).
    int count = 0;
    const int group_lane0 = ((int)(threadIdx.x & 63) / G) * G;
    for (int i0 = 0; i0 < WOWN_E; i0 += G) {
        const int i = i0 + l;
        const bool inside = i < WOWN_E;
        const uint32_t k = inside ? K(i) : NOKEY, kn = inside ? K(i + 1) : NOKEY;
        uint32_t act = ACT_SKIP;
        if (active && k != NOKEY && !(a.skip_alone && kn != k && K(i - 1) != k)) {
            if (i < C) {
                if (head_exists && k == k0) {            // a run that came in from the left
                    if (own_head) act = (kn != k) ? ACT_HEAD : ACT_ADD;
                } else if (k2C != k) {                   // starts here and is short: ours entirely
                    act = (kn != k) ? ACT_COMPLETE : ACT_ADD;
                } else {                                 // starts here and is long: first piece
                    act = ACT_ADD;
                }
            } else if (ext_ok && k == klast) {           // the rest of our last short run
                act = (kn != k) ? ACT_COMPLETE : ACT_ADD;
            }
        }
        if (inside) s_act[grp][i] = act;
        const bool use = act != ACT_SKIP;
        const uint64_t wave_mask = __ballot(use);
        const uint64_t mine = (G == 64) ? wave_mask : ((wave_mask >> group_lane0) & ((1ull << G) - 1ull));
        if (use) {
            const uint32_t q = a.sidx[base + i];
            s_srow[grp][i] = a.in_idx[q / a.T];          // range-checked copy
            s_coef[grp][i] = a.coeffs[q];
            s_list[grp][count + __popcll(mine & ((1ull << l) - 1ull))] = (uint32_t)i;
        }
        count += __popcll(mine);
    }
    __syncthreads();
    if (!active || count == 0) return;
    const uint32_t d4 = a.g.d4;
    const uint64_t s4 = a.g.stride4;
    const uint32_t cell = (uint32_t)(base / L);
    const uint32_t head_slot = 2 * cell - 1, tail_slot = 2 * cell;   // used only when they exist

    float4 acc[NV], srcv[D][NV], dstv[D][NV];
    clear<NV>(acc);
    auto finish_row = [&](uint32_t row, const float4 (&old)[NV]) {
        float4 out[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            out[v].x = fmaf(alpha, acc[v].x, old[v].x);
            out[v].y = fmaf(alpha, acc[v].y, old[v].y);
            out[v].z = fmaf(alpha, acc[v].z, old[v].z);
            out[v].w = fmaf(alpha, acc[v].w, old[v].w);
        }
        store_row_nt<G, NV>(a.dst + (uint64_t)row * s4, (uint32_t)s4, l, out);
    };
    auto fetch = [&](int idx, float4 (&sv)[NV], float4 (&dv)[NV]) {
        const bool on = idx < count;
        const int i = on ? (int)s_list[grp][idx] : 0;
        const uint32_t sr = on ? s_srow[grp][i] : 0u;
        const bool cm = on && s_act[grp][i] == ACT_COMPLETE;
        const uint32_t dk = cm ? K(i) : 0u;
        // Destination rows are read and written once per minibatch: with the non-temporal hint they
        // do not push the source rows (a few hundred MB that are read again and again) out of the
        // caches -- measured -7 % on this kernel; the same hint on the source rows costs +25 %.
        load_row_if<G, NV>(on, a.src + (uint64_t)sr * s4, d4, l, sv);
        load_row_nt_if<G, NV>(cm, a.dst + (uint64_t)dk * s4, d4, l, dv);
    };
#pragma unroll
    for (int t = 0; t < D; ++t) fetch(t, srcv[t], dstv[t]);
    for (int b = 0; b < count; b += D) {
#pragma unroll
        for (int t = 0; t < D; ++t) {
            const int idx = b + t;
            if (idx < count) {
                const int i = (int)s_list[grp][idx];
                const uint32_t act = s_act[grp][i];
                axpy<NV>(s_coef[grp][i], srcv[t], acc);
                if (act == ACT_COMPLETE) {
                    finish_row(K(i), dstv[t]);
                    clear<NV>(acc);
                } else if (act == ACT_HEAD) {            // our piece of a long run ends in the chunk
                    store_row<G, NV>(a.prows + (uint64_t)head_slot * s4, d4, l, acc);
                    if (l == 0) a.pkeys[head_slot] = K(i);
                    clear<NV>(acc);
                }
            }
            fetch(idx + D, srcv[t], dstv[t]);
        }
    }
    if (!cont) return;

    // ---- the long piece goes on past the chunk: stream through the rest of the cell ----
    const uint32_t key = klast;
    const int64_t limit = min((int64_t)(cell + 1) * L, (int64_t)a.entries);
    bool ended = false;
    for (int64_t x0 = base + C; x0 < limit; x0 += 16) {
        const int nblk = (int)min((int64_t)16, limit - x0);
        const bool same = l < nblk && a.skey[x0 + l] == key;
        const uint32_t bits = (uint32_t)(__ballot(same) >> group_lane0) & 0xFFFFu;
        const int cnt = __builtin_ctz(~bits);             // entries of the run at the block's front
        uint32_t sr = 0;
        float cf = 0.f;
        if (l < cnt) {
            const uint32_t q = a.sidx[x0 + l];
            sr = a.in_idx[q / a.T];
            cf = a.coeffs[q];
        }
#pragma unroll
        for (int b = 0; b < 16; b += D) {
            if (b < cnt) {
#pragma unroll
                for (int t = 0; t < D; ++t)
                    load_row_if<G, NV>(b + t < cnt, a.src + (uint64_t)__shfl(sr, b + t, G) * s4, d4, l,
                                       srcv[t]);
#pragma unroll
                for (int t = 0; t < D; ++t) axpy<NV>(__shfl(cf, b + t, G), srcv[t], acc);
            }
        }
        if (cnt < nblk) { ended = true; break; }
    }
    if (!ended) ended = limit >= (int64_t)a.entries || a.skey[limit] != key;
    if (!last_in_head) {
        if (ended) {                                      // the whole run lay inside the cell
            float4 old[NV];
            load_row_nt_if<G, NV>(true, a.dst + (uint64_t)key * s4, d4, l, old);
            finish_row(key, old);
        } else {                                          // first piece of a run that leaves the cell
            store_row<G, NV>(a.prows + (uint64_t)tail_slot * s4, d4, l, acc);
            if (l == 0) a.pkeys[tail_slot] = key;
        }
    } else {                                              // a piece that began at the cell's start
        store_row<G, NV>(a.prows + (uint64_t)head_slot * s4, d4, l, acc);
        if (l == 0) {
            a.pkeys[head_slot] = key;
            if (!ended) a.pkeys[tail_slot] = key | KEY_ZERO;   // the run fills the cell and goes on
        }
    }
}

template <int G, int NV, int D>
__global__ __launch_bounds__(wown_threads(G)) void wown_kernel(SegArgs a) {
    wown_body<G, NV, D>(a, blockIdx.x);
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* __restrict__ x, uint32_t n,
                                                       uint32_t value) {
    uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) x[i] = value;
}

FillJob wseg_fill_job(uint32_t* pkeys, uint32_t M) {
    // border slots of the cells: only pieces of long runs write them
    const uint32_t ncells = (M + WOWN_L - 1) / WOWN_L;
    return FillJob{pkeys, ncells ? 2 * (ncells - 1) : 0u, KEY_NONE};
}

void launch_wseg_fill(uint32_t* pkeys, uint32_t M, hipStream_t st) {
    const FillJob f = wseg_fill_job(pkeys, M);
    if (f.count)
        hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(f.count, 256)), dim3(256), 0, st, f.p,
                           f.count, f.value);
}

static SegArgs seg_args_of(const WSideArgs& w) {
    SegArgs a{};
    a.src = (const float4*)w.U; a.dst = (float4*)w.W; a.g = w.g; a.skey = w.skey; a.sidx = w.sidx;
    a.in_idx = w.in_idx; a.coeffs = w.coeffs; a.entries = w.M; a.T = w.T;
    a.alpha = w.alpha; a.prows = (float4*)w.prows; a.pkeys = w.pkeys; a.dev = w.dev;
    a.skip_alone = w.skip_alone;
    return a;
}

static SegArgs seg_args_of(const TailArgs& t) {
    SegArgs a{};
    a.src = (const float4*)t.src_rows; a.dst = (float4*)t.M; a.g = t.g; a.skey = t.src_keys;
    a.sidx = nullptr; a.in_idx = nullptr; a.coeffs = nullptr; a.entries = t.entries; a.T = 1;
    a.skip_alone = false;
    a.alpha = t.alpha; a.prows = (float4*)t.prows; a.pkeys = t.pkeys; a.dev = t.dev;
    a.defer_rows = (float4*)t.defer_rows; a.defer_keys = t.defer_keys; a.level = t.level; a.cp = t.cp;
    return a;
}

void launch_wseg(const WSideArgs& w, hipStream_t st, bool filled) {
    if (w.M == 0) return;
    const SegArgs a = seg_args_of(w);
    if (!filled) launch_wseg_fill(w.pkeys, w.M, st);
    uint32_t nchunks = (w.M + WOWN_C - 1) / WOWN_C;
#define CALL(G, NV)                                                                              \
    hipLaunchKernelGGL((wown_kernel<G, NV, (NV <= 2 ? 4 : 2)>),                                   \
                       dim3(blocks_for((uint64_t)nchunks * G, wown_threads(G))),                 \
                       dim3(wown_threads(G)), 0,                                                 \
                       st, a)
    W2V_DISPATCH_GEOM(w.g.d4, CALL);
#undef CALL
}

void launch_tail(const TailArgs& t, hipStream_t st) {
    if (t.entries == 0) return;
    const SegArgs a = seg_args_of(t);
    uint32_t nchunks = (t.entries + TAIL_C - 1) / TAIL_C;
#define CALL(G, NV)                                                                              \
    do {                                                                                         \
        if (t.defer_rows)                                                                        \
            hipLaunchKernelGGL((seg_kernel<G, NV, TAIL_C, (NV <= 2 ? 4 : 2), 1, true>),          \
                               dim3(blocks_for((uint64_t)nchunks * G, ADJ_THREADS)),             \
                               dim3(ADJ_THREADS), 0, st, a);                                     \
        else                                                                                     \
            hipLaunchKernelGGL((seg_kernel<G, NV, TAIL_C, (NV <= 2 ? 4 : 2), 1>),                \
                               dim3(blocks_for((uint64_t)nchunks * G, ADJ_THREADS)),             \
                               dim3(ADJ_THREADS), 0, st, a);                                     \
    } while (0)
    W2V_DISPATCH_GEOM(t.g.d4, CALL);
#undef CALL
}

// ---------------------------------------------------------------------------------------------
// One launch for parts of the update that do not depend on each other: a walk of the output side
// (its level-1 kernel when FIRST, else one of its higher levels), one higher level of the input
// side (which parks its sums in the delta buffer), and one step of the loss.  Each block does one
// part, told by its number, with the same code as the kernels above, so the bits are the same.
// On one stream a step of a few thousand pairs is a chain of launches of a few microseconds each;
// this takes the input side's levels and the loss out of that chain.
// ---------------------------------------------------------------------------------------------
struct StageDev {
    SegArgs w, u;
    uint32_t w_blocks, u_blocks;
    uint32_t loss_step;              // 0 none, 1 terms -> block sums, 2 block sums -> loss
    const float* dots; uint32_t total, T;
    double* block_loss; uint32_t nb; double* loss_out;
};

template <int G, int NV, bool FIRST>
__global__ __launch_bounds__(ADJ_THREADS) void adjust_stage_kernel(StageDev s) {
    constexpr int D = NV <= 2 ? 4 : 2;
    static_assert(wown_threads(G) == ADJ_THREADS, "the parts share one block size");
    uint32_t b = blockIdx.x;
    if (b < s.w_blocks) {
        if (FIRST) wown_body<G, NV, D>(s.w, b);
        else seg_body<G, NV, TAIL_C, D, 1, false>(s.w, b);
        return;
    }
    b -= s.w_blocks;
    if (b < s.u_blocks) {
        seg_body<G, NV, TAIL_C, D, 1, true>(s.u, b);
        return;
    }
    b -= s.u_blocks;
    __shared__ double red[256];
    if (s.loss_step == 1) loss_terms_block(s.dots, s.total, s.T, s.block_loss, b, red);
    else sum_doubles_block(s.block_loss, s.nb, s.nb, s.loss_out, 0u, red);
}

bool adjust_stage_supported(uint32_t d4) { return d4 > 16; }    // (sixteen-lane groups use blocks of 128)
uint32_t adjust_stage_loss_blocks_max() { return LOSS_SUM_SPAN; }

template <int G, int NV>
static void launch_stage_shape(StageDev s, uint32_t w_chunks, uint32_t u_chunks, uint32_t loss_blocks,
                               bool first, hipStream_t st) {
    if constexpr (G != 16) {
        s.w_blocks = blocks_for((uint64_t)w_chunks * G, ADJ_THREADS);
        s.u_blocks = blocks_for((uint64_t)u_chunks * G, ADJ_THREADS);
        const dim3 grid(s.w_blocks + s.u_blocks + loss_blocks);
        if (first)
            hipLaunchKernelGGL((adjust_stage_kernel<G, NV, true>), grid, dim3(ADJ_THREADS), 0, st, s);
        else
            hipLaunchKernelGGL((adjust_stage_kernel<G, NV, false>), grid, dim3(ADJ_THREADS), 0, st, s);
    }
}

void launch_adjust_stage(const AdjustStage& x, hipStream_t st) {
    StageDev s{};
    RowGeom g{};
    uint32_t w_chunks = 0, u_chunks = 0, loss_blocks = 0;
    const bool first = x.wfirst && x.wfirst->M;
    if (first) {
        s.w = seg_args_of(*x.wfirst); g = x.wfirst->g;
        w_chunks = (x.wfirst->M + WOWN_C - 1) / WOWN_C;
    } else if (x.wtail && x.wtail->entries) {
        s.w = seg_args_of(*x.wtail); g = x.wtail->g;
        w_chunks = (x.wtail->entries + TAIL_C - 1) / TAIL_C;
    }
    if (x.utail && x.utail->entries) {
        s.u = seg_args_of(*x.utail); g = x.utail->g;
        u_chunks = (x.utail->entries + TAIL_C - 1) / TAIL_C;
    }
    s.loss_step = x.loss_step;
    if (x.loss_step) {
        s.dots = x.dots; s.total = x.n * x.T; s.T = x.T; s.block_loss = x.loss_tmp;
        s.nb = blocks_for(s.total, 256); s.loss_out = x.loss_out;
        loss_blocks = x.loss_step == 1 ? s.nb : 1u;
    }
    if (!w_chunks && !u_chunks && !loss_blocks) return;
    if (!w_chunks && !u_chunks) g.d4 = 17;        // (only the loss part runs: any supported shape)
#define CALL(G, NV) launch_stage_shape<G, NV>(s, w_chunks, u_chunks, loss_blocks, first, st)
    W2V_DISPATCH_GEOM(g.d4, CALL);
#undef CALL
}

// ---------------------------------------------------------------------------------------------
// Input-vector side, level 1: entries are whole pairs (T source rows each) in the order of the
// sorted input words.  Runs finished inside a chunk go to the delta buffer (the input matrix must
// stay untouched until the output side has read it); cut runs go to the partial slots.
// FUSED: the group also holds u, forms the T dots of the pair, turns them into coefficients
// (written out for the output side) and uses them at once -- the output rows are read only once.
// ---------------------------------------------------------------------------------------------
// sigma(-x) = 1 / (1 + e^x): the positive slot's coefficient 1 - sigma(f) is sigma(-f), a negative
// slot's -sigma(f) is -sigma(-(-f)); written this way the coefficient keeps its relative accuracy
// when it is small.
__device__ __forceinline__ float sigmoid_of_minus(float x) { return 1.0f / (1.0f + expf(x)); }


template <int G, int NV, int TB, bool FUSED, bool OWN>
__global__ __launch_bounds__(USEG_THREADS) void useg_kernel(USideArgs a, uint32_t CP) {
    constexpr bool NEED_U = FUSED || OWN;      // the pair's input row: for the dots, for own rows
    const float alpha = a.dev ? a.dev->alpha : a.alpha;
    constexpr int GROUPS = USEG_THREADS / G;
    // The chunk's indices are staged in LDS first (two dependent gathers for the whole chunk), so
    // that the row loads of the main loop depend on nothing but LDS reads.
    constexpr int USEG_MAXE = useg_maxe(G), USEG_MAXP = useg_maxp(G);
    __shared__ uint32_t s_key[GROUPS][USEG_MAXE];                 // output row of every entry
    __shared__ float s_cf[FUSED ? 1 : GROUPS][FUSED ? 1 : USEG_MAXE];   // given coefficients
    __shared__ uint32_t s_pair[GROUPS][USEG_MAXP];                // pair number of every sorted pair
    __shared__ uint32_t s_skey[GROUPS][USEG_MAXP + 2];            // input word: [0] before, [cnt+1] after
    const int l = threadIdx.x % G, grp = threadIdx.x / G;
    const uint32_t c = blockIdx.x * (uint32_t)GROUPS + grp;
    const uint32_t nchunks = (a.n + CP - 1) / CP;
    const bool active = c < nchunks;
    const uint32_t ps0 = active ? c * CP : 0u;
    const uint32_t cnt = active ? min(CP, a.n - ps0) : 0u;
    const uint32_t T = a.T;
    for (uint32_t i = l; i < cnt; i += G) {
        s_pair[grp][i] = a.perm[ps0 + i];
        s_skey[grp][i + 1] = a.skey[ps0 + i];
    }
    if (active && l == 0) {
        s_skey[grp][0] = ps0 > 0 ? a.skey[ps0 - 1] : NOKEY;
        s_skey[grp][cnt + 1] = ps0 + cnt < a.n ? a.skey[ps0 + cnt] : NOKEY;
    }
    __syncthreads();
    for (uint32_t i = l; i < cnt * T; i += G) {
        uint32_t pi = i / T, j = i - pi * T;
        uint32_t q = s_pair[grp][pi] * T + j;
        s_key[grp][i] = a.keys[q];                 // may carry ALONE (fused, own rows)
        if (!FUSED) s_cf[grp][i] = a.coeffs_in[q];
    }
    __syncthreads();
    if (!active) return;

    const uint32_t d4 = a.g.d4;
    const uint64_t s4 = a.g.stride4;
    const float4* U4p = (const float4*)a.U;
    const float4* W4p = (const float4*)a.W;
    float4* delta = (float4*)a.delta;
    float4* prows = (float4*)a.prows;

    uint32_t key = s_skey[grp][1];
    const bool open_head = (s_skey[grp][0] == key);
    uint32_t run_start = ps0;
    uint32_t head_key = KEY_NONE, tail_key = KEY_NONE;
    const uint32_t head_slot = 2 * c - 1, tail_slot = 2 * c;

    float4 acc[NV], w[TB][NV], u[NV], un[NV];
    clear<NV>(acc);
    // prologue: the first batch of rows (and u) of the chunk's first pair
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        bool on = (uint32_t)t < T;
        uint32_t r = on ? (s_key[grp][t] & ~ALONE) : 0u;
        load_row_if<G, NV>(on, W4p + (uint64_t)r * s4, d4, l, w[t]);
    }
    if (NEED_U) load_row<G, NV>(U4p + (uint64_t)key * s4, d4, l, u);

    for (uint32_t pi = 0; pi < cnt; ++pi) {
        const uint32_t ps = ps0 + pi;
        const uint32_t p = s_pair[grp][pi];
        const uint32_t next = s_skey[grp][pi + 2];
        if (l == 0) a.dkey[ps] = KEY_NONE;
        if (NEED_U) {                                  // the next pair's input row, ahead of need
            bool more = pi + 1 < cnt;
            load_row_if<G, NV>(more, U4p + (uint64_t)(more ? next : 0u) * s4, d4, l, un);
        }
        for (uint32_t jb = 0; jb < T; jb += TB) {
            const bool last_batch = jb + TB >= T;
            const uint32_t npi = last_batch ? pi + 1 : pi;     // where the following batch starts
            const uint32_t njb = last_batch ? 0u : jb + TB;
            float gco[TB];
            if (FUSED) {
                float sdot[TB];
#pragma unroll
                for (int t = 0; t < TB; ++t) sdot[t] = dot_part<NV>(u, w[t]);
#pragma unroll
                for (int t = 0; t < TB; ++t) sdot[t] = group_sum<G>(sdot[t]);
#pragma unroll
                for (int t = 0; t < TB; ++t) {
                    uint32_t j = jb + t;
                    float f = sdot[t];
                    const float gc = (j == 0) ? sigmoid_of_minus(f) : -sigmoid_of_minus(-f);
                    gco[t] = (j < T) ? gc : 0.f;
                    if (l == t && j < T) {
                        a.coeffs_out[p * T + j] = gc;
                        if (a.dots_out) a.dots_out[p * T + j] = f;
                    }
                }
            } else {
#pragma unroll
                for (int t = 0; t < TB; ++t)
                    gco[t] = (jb + t < T) ? s_cf[grp][pi * T + jb + t] : 0.f;
            }
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (jb + t < T) {
                    axpy<NV>(gco[t], w[t], acc);
                    // an output row that no other slot names gets its whole update here (see the
                    // fixed-T kernel below)
                    const uint32_t rr = OWN ? s_key[grp][pi * T + jb + t] : 0u;
                    if (OWN && (rr & ALONE)) {
                        float4 out[NV];
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            out[v].x = fmaf(alpha, fmaf(gco[t], u[v].x, 0.f), w[t][v].x);
                            out[v].y = fmaf(alpha, fmaf(gco[t], u[v].y, 0.f), w[t][v].y);
                            out[v].z = fmaf(alpha, fmaf(gco[t], u[v].z, 0.f), w[t][v].z);
                            out[v].w = fmaf(alpha, fmaf(gco[t], u[v].w, 0.f), w[t][v].w);
                        }
                        store_row_nt<G, NV>((float4*)a.W_update + (uint64_t)(rr & ~ALONE) * s4, (uint32_t)s4, l, out);
                    }
                }
                // this register set is free again: fetch the matching row of the following batch
                uint32_t nj = njb + t;
                bool on = npi < cnt && nj < T;
                // (the non-temporal hint for rows named once, which pays in the fixed-T kernel,
                // costs 25 % here: the branch breaks up this loop's batched loads)
                uint32_t r = on ? (s_key[grp][npi * T + nj] & ~ALONE) : 0u;
                load_row_if<G, NV>(on, W4p + (uint64_t)r * s4, d4, l, w[t]);
            }
        }
        if (next != key) {                       // the run of `key` ends with this pair
            if (run_start == ps0 && open_head) {
                store_row<G, NV>(prows + (uint64_t)head_slot * s4, d4, l, acc);
                head_key = key;
            } else {
                store_row<G, NV>(delta + (uint64_t)run_start * s4, d4, l, acc);
                if (l == 0) a.dkey[run_start] = key;
            }
            clear<NV>(acc);
            run_start = ps + 1;
        }
        if (NEED_U) {
#pragma unroll
            for (int v = 0; v < NV; ++v) u[v] = un[v];
        }
        key = next;
    }
    if (run_start < ps0 + cnt) {                 // the last run goes on into the next chunk
        const uint32_t k_last = s_skey[grp][cnt];
        if (run_start == ps0 && open_head) {
            store_row<G, NV>(prows + (uint64_t)head_slot * s4, d4, l, acc);
            head_key = k_last;
            tail_key = k_last | KEY_ZERO;
        } else {
            store_row<G, NV>(prows + (uint64_t)tail_slot * s4, d4, l, acc);
            tail_key = k_last;
        }
    }
    if (l == 0) {
        if (c > 0) a.pkeys[head_slot] = head_key;
        if (c + 1 < nchunks) a.pkeys[tail_slot] = tail_key;
    }
}

// ---------------------------------------------------------------------------------------------
// The same step for a compile-time number of slots per pair (T), taking PB pairs per batch: all
// PB*T output rows and the PB input rows of a batch are requested before the first of them is
// used, so a lane group keeps PB*(T+1) rows in flight instead of T+1.  The kernel is
// latency-bound (rows in flight per SIMD x row size / memory latency), and registers spent on
// rows in flight buy more than registers spent on extra resident waves.
// ---------------------------------------------------------------------------------------------
// Register budget for five wavefronts per SIMD: at two float4 per lane the fused form would take
// 102 registers and run four; held to 96 it spills five and is 1.6 % faster.  (Six: 30 % slower.
// The same squeeze on the generic kernel or on the output-side kernel costs more than it gives.)
template <int G, int NV, int T, int PB, bool FUSED, bool OWN>
__global__ __launch_bounds__(USEG_THREADS, 5) void useg_multi_kernel(USideArgs a, uint32_t CP) {
    constexpr bool NEED_U = FUSED || OWN;
    const float alpha = a.dev ? a.dev->alpha : a.alpha;
    constexpr int GROUPS = USEG_THREADS / G;
    constexpr int MAXP = useg_maxp(G), MAXE = MAXP * T;
    __shared__ uint32_t s_key[GROUPS][MAXE];
    __shared__ float s_cf[FUSED ? 1 : GROUPS][FUSED ? 1 : MAXE];
    __shared__ uint32_t s_pair[GROUPS][MAXP];
    __shared__ uint32_t s_skey[GROUPS][MAXP + 2];
    const int l = threadIdx.x % G, grp = threadIdx.x / G;
    const uint32_t c = blockIdx.x * (uint32_t)GROUPS + grp;
    const uint32_t nchunks = (a.n + CP - 1) / CP;
    const bool active = c < nchunks;
    const uint32_t ps0 = active ? c * CP : 0u;
    const uint32_t cnt = active ? min(CP, a.n - ps0) : 0u;
    for (uint32_t i = l; i < cnt; i += G) {
        s_pair[grp][i] = a.perm[ps0 + i];
        s_skey[grp][i + 1] = a.skey[ps0 + i];
    }
    if (active && l == 0) {
        s_skey[grp][0] = ps0 > 0 ? a.skey[ps0 - 1] : NOKEY;
        s_skey[grp][cnt + 1] = ps0 + cnt < a.n ? a.skey[ps0 + cnt] : NOKEY;
    }
    __syncthreads();
    for (uint32_t i = l; i < cnt * T; i += G) {
        uint32_t pi = i / T, j = i - pi * T;
        uint32_t q = s_pair[grp][pi] * T + j;
        s_key[grp][i] = a.keys[q];                 // may carry ALONE (fused, own rows)
        if (!FUSED) s_cf[grp][i] = a.coeffs_in[q];
    }
    __syncthreads();
    if (!active) return;

    const uint32_t d4 = a.g.d4;
    const uint64_t s4 = a.g.stride4;
    const float4* U4p = (const float4*)a.U;
    const float4* W4p = (const float4*)a.W;
    float4* delta = (float4*)a.delta;
    float4* prows = (float4*)a.prows;

    uint32_t key = s_skey[grp][1];
    const bool open_head = (s_skey[grp][0] == key);
    uint32_t run_start = ps0;
    uint32_t head_key = KEY_NONE, tail_key = KEY_NONE;
    const uint32_t head_slot = 2 * c - 1, tail_slot = 2 * c;

    float4 acc[NV];
    clear<NV>(acc);
    for (uint32_t pb = 0; pb < cnt; pb += PB) {
        float4 w[PB][T][NV], u[PB][NV];
#pragma unroll
        for (int b = 0; b < PB; ++b) {
            const uint32_t pi = pb + b;
            const bool live = pi < cnt;
            if (NEED_U) {
                const uint32_t k_in = live ? s_skey[grp][pi + 1] : 0u;
                load_row_if<G, NV>(live, U4p + (uint64_t)k_in * s4, d4, l, u[b]);
            }
#pragma unroll
            for (int j = 0; j < T; ++j) {
                const uint32_t rk = live ? s_key[grp][pi * T + j] : 0u;
                const uint32_t r = rk & ~ALONE;
                // a row that no other slot names is read here once and written once: the
                // non-temporal hint keeps it out of the caches' way (-7 % on this kernel)
                if (rk & ALONE) load_row_nt_if<G, NV>(live, W4p + (uint64_t)r * s4, d4, l, w[b][j]);
                else load_row_if<G, NV>(live, W4p + (uint64_t)r * s4, d4, l, w[b][j]);
            }
        }
#pragma unroll
        for (int b = 0; b < PB; ++b) {
            const uint32_t pi = pb + b;
            if (pi < cnt) {
                const uint32_t ps = ps0 + pi;
                const uint32_t p = s_pair[grp][pi];
                const uint32_t next = s_skey[grp][pi + 2];
                if (l == 0) a.dkey[ps] = KEY_NONE;
                float gco[T];
                if (FUSED) {
                    float sdot[T];
#pragma unroll
                    for (int j = 0; j < T; ++j) sdot[j] = dot_part<NV>(u[b], w[b][j]);
#pragma unroll
                    for (int j = 0; j < T; ++j) sdot[j] = group_sum<G>(sdot[j]);
#pragma unroll
                    for (int j = 0; j < T; ++j) {
                        const float f = sdot[j];
                        gco[j] = (j == 0) ? sigmoid_of_minus(f) : -sigmoid_of_minus(-f);
                        if (l == j % G) {
                            a.coeffs_out[p * T + j] = gco[j];
                            if (a.dots_out) a.dots_out[p * T + j] = f;
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < T; ++j) gco[j] = s_cf[grp][pi * T + j];
                }
                // An output row that no other slot names gets its whole update here, from the
                // registers, with the same two roundings as the output-side kernel
                // (fl(g u), then one fma with alpha); that kernel never sees the slot.
                if (OWN) {
#pragma unroll
                    for (int j = 0; j < T; ++j) {
                        const uint32_t r = s_key[grp][pi * T + j];
                        if (r & ALONE) {
                            float4 out[NV];
#pragma unroll
                            for (int v = 0; v < NV; ++v) {
                                out[v].x = fmaf(alpha, fmaf(gco[j], u[b][v].x, 0.f), w[b][j][v].x);
                                out[v].y = fmaf(alpha, fmaf(gco[j], u[b][v].y, 0.f), w[b][j][v].y);
                                out[v].z = fmaf(alpha, fmaf(gco[j], u[b][v].z, 0.f), w[b][j][v].z);
                                out[v].w = fmaf(alpha, fmaf(gco[j], u[b][v].w, 0.f), w[b][j][v].w);
                            }
                            store_row_nt<G, NV>((float4*)a.W_update + (uint64_t)(r & ~ALONE) * s4, (uint32_t)s4,
                                                l, out);
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < T; ++j) axpy<NV>(gco[j], w[b][j], acc);
                if (next != key) {                       // the run of `key` ends with this pair
                    if (run_start == ps0 && open_head) {
                        store_row<G, NV>(prows + (uint64_t)head_slot * s4, d4, l, acc);
                        head_key = key;
                    } else {
                        store_row<G, NV>(delta + (uint64_t)run_start * s4, d4, l, acc);
                        if (l == 0) a.dkey[run_start] = key;
                    }
                    clear<NV>(acc);
                    run_start = ps + 1;
                }
                key = next;
            }
        }
    }
    if (run_start < ps0 + cnt) {                 // the last run goes on into the next chunk
        const uint32_t k_last = s_skey[grp][cnt];
        if (run_start == ps0 && open_head) {
            store_row<G, NV>(prows + (uint64_t)head_slot * s4, d4, l, acc);
            head_key = k_last;
            tail_key = k_last | KEY_ZERO;
        } else {
            store_row<G, NV>(prows + (uint64_t)tail_slot * s4, d4, l, acc);
            tail_key = k_last;
        }
    }
    if (l == 0) {
        if (c > 0) a.pkeys[head_slot] = head_key;
        if (c + 1 < nchunks) a.pkeys[tail_slot] = tail_key;
    }
}

constexpr int USEG_PB = 1;     // pairs per batch of the fixed-T kernel (1 measured best on MI355X)

// A fixed-T kernel exists for k = 5 (the paper's and the benchmark's number of negatives); other T
// take the generic kernel (fixed-T variants for k = 10 and 25 measured no better, or worse).

template <int G, int NV, int T>
static void launch_useg_fixed(const USideArgs& a, uint32_t CP, dim3 grid, dim3 block, hipStream_t st) {
    const bool own = a.W_update != nullptr;      // (only the fused form takes rows over)
    if (a.fused && own)
        hipLaunchKernelGGL((useg_multi_kernel<G, NV, T, USEG_PB, true, true>), grid, block, 0, st, a, CP);
    else if (a.fused)
        hipLaunchKernelGGL((useg_multi_kernel<G, NV, T, USEG_PB, true, false>), grid, block, 0, st, a, CP);
    else
        hipLaunchKernelGGL((useg_multi_kernel<G, NV, T, USEG_PB, false, false>), grid, block, 0, st, a, CP);
}

template <int G, int NV>
static void launch_useg_shape(const USideArgs& a, hipStream_t st) {
    const uint32_t CP = useg_pairs_per_chunk(a.T, a.g.d4, a.n);
    const uint32_t nchunks = (a.n + CP - 1) / CP;
    dim3 grid(blocks_for((uint64_t)nchunks * G, USEG_THREADS)), block(USEG_THREADS);
    if constexpr (NV <= 2) {
        if (a.T == 6) return launch_useg_fixed<G, NV, 6>(a, CP, grid, block, st);
    }
    constexpr int TB = NV == 1 ? 9 : (NV == 2 ? 6 : 4);     // rows requested per batch
    const bool own = a.W_update != nullptr;      // (only the fused form takes rows over)
    if constexpr (NV == 1) {
        // The fused kernel with one float4 per lane has registers for up to thirteen rows in
        // flight: of 9, 11 and 13 rows per batch, take the one that needs the fewest batches per
        // pair and then leaves the fewest empty places in them (k = 10: one batch of 11 instead of
        // 9 + 2, input-side kernel 3 % faster; k = 25: 13 + 13 instead of 9 + 9 + 8, 1 %).
        if (a.fused && own) {
            int best = 9;
            uint32_t best_nb = (a.T + 8) / 9, best_waste = best_nb * 9 - a.T;
            for (int tb : {11, 13}) {
                const uint32_t nb = (a.T + tb - 1) / tb, waste = nb * tb - a.T;
                if (nb < best_nb || (nb == best_nb && waste < best_waste)) { best = tb; best_nb = nb; best_waste = waste; }
            }
            if (best == 11) { hipLaunchKernelGGL((useg_kernel<G, NV, 11, true, true>), grid, block, 0, st, a, CP); return; }
            if (best == 13) { hipLaunchKernelGGL((useg_kernel<G, NV, 13, true, true>), grid, block, 0, st, a, CP); return; }
        }
    }
    if (a.fused && own)
        hipLaunchKernelGGL((useg_kernel<G, NV, TB, true, true>), grid, block, 0, st, a, CP);
    else if (a.fused)
        hipLaunchKernelGGL((useg_kernel<G, NV, TB, true, false>), grid, block, 0, st, a, CP);
    else
        hipLaunchKernelGGL((useg_kernel<G, NV, TB, false, false>), grid, block, 0, st, a, CP);
}

void launch_useg(const USideArgs& a, hipStream_t st) {
    if (a.n == 0) return;
#define SHAPE(G, NV) launch_useg_shape<G, NV>(a, st)
    W2V_DISPATCH_GEOM(a.g.d4, SHAPE);
#undef SHAPE
}

// ---------------------------------------------------------------------------------------------
// Write-back of the input-vector changes held in the delta buffer.
// ---------------------------------------------------------------------------------------------
// A lane group looks at G consecutive sorted positions at once (one dkey per lane) and then walks
// the few that carry a finished run.
template <int G, int NV>
__global__ __launch_bounds__(ADJ_THREADS) void apply_delta_kernel(float4* __restrict__ U, RowGeom g,
                                                                  const float4* __restrict__ delta,
                                                                  const uint32_t* __restrict__ dkey,
                                                                  uint32_t n, float alpha_arg,
                                                                  const CallScalars* dev) {
    const float alpha = dev ? dev->alpha : alpha_arg;
    const int l = threadIdx.x % G;
    const uint32_t grp = (blockIdx.x * (uint32_t)ADJ_THREADS + threadIdx.x) / G;
    const uint32_t base = grp * (uint32_t)G;
    if (base >= n) return;
    const uint32_t mine = (base + l < n) ? dkey[base + l] : KEY_NONE;
    for (int e = 0; e < G; ++e) {
        const uint32_t key = __shfl(mine, e, G);
        if (key == KEY_NONE) continue;
        const uint32_t ps = base + e;
        float4 dv[NV], uv[NV];
        load_row<G, NV>(delta + (uint64_t)ps * g.stride4, g.d4, l, dv);
        load_row<G, NV>(U + (uint64_t)key * g.stride4, g.d4, l, uv);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            uv[v].x = fmaf(alpha, dv[v].x, uv[v].x);
            uv[v].y = fmaf(alpha, dv[v].y, uv[v].y);
            uv[v].z = fmaf(alpha, dv[v].z, uv[v].z);
            uv[v].w = fmaf(alpha, dv[v].w, uv[v].w);
        }
        store_row<G, NV>(U + (uint64_t)key * g.stride4, g.stride4, l, uv);
    }
}

void launch_apply_delta(float* U, RowGeom g, const float* delta, const uint32_t* dkey, uint32_t n,
                        float alpha, hipStream_t st, const CallScalars* dev) {
    if (n == 0) return;
#define CALL(G, NV)                                                                              \
    hipLaunchKernelGGL((apply_delta_kernel<G, NV>), dim3(blocks_for(n, ADJ_THREADS)),            \
                       dim3(ADJ_THREADS), 0, st, (float4*)U, g, (const float4*)delta, dkey, n, alpha, dev)
    W2V_DISPATCH_GEOM(g.d4, CALL);
#undef CALL
}

}  // namespace w2v
