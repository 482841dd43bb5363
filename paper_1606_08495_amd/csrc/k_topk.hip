// Retrieval by cosine similarity (Section 2; Section 7.3: K = 30, threshold tau): for every query
// vector the K most similar candidate vectors.  The similarities are a dense contraction
// (Q x d) . (d x N) and run on the fp32 matrix cores; they are never written out -- a tile's scores
// are compared with the query's current K-th best right in the accumulators, and only the few that
// pass are appended to the query's pending list, which a small selection kernel folds into the
// sorted best list after every round of candidates.
#include "common.h"

#include <math.h>

namespace w2v {

static inline unsigned blocks_for(uint64_t items, unsigned per_block) {
    return (unsigned)((items + per_block - 1) / per_block);
}

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int TK_BQ = 128;          // queries per block tile (2 x 2 wavefronts x 2 x 2 tiles of 32)
constexpr int TK_BC = 128;          // candidates per block tile; granularity of a round
constexpr int TK_BK = 16;           // columns per panel; two panels are held in LDS
constexpr int TK_LD = TK_BK + 1;    // LDS row pitch (odd: conflict-free column reads)
constexpr int TK_THREADS = 256;     // four wavefronts
constexpr int TK_RPM = TK_THREADS / (TK_BK / 4);            // rows covered by one move of the block
constexpr int TK_LIST = 64;         // slots of a query's best list (K <= 64)
constexpr uint32_t TK_NONE = 0xFFFFFFFFu;

// ---------------------------------------------------------------------------------------------
// 1 / |row| (0 for an all-zero row): one wavefront per row.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void inv_norm_kernel(const float* __restrict__ M, uint32_t rows,
                                                       uint32_t d, float* __restrict__ inv) {
    const uint32_t r = (blockIdx.x * 256u + threadIdx.x) / 64u;
    const int lane = threadIdx.x % 64;
    if (r >= rows) return;                                  // whole wavefronts leave together
    const float* row = M + (uint64_t)r * d;
    float s = 0.f;
    for (uint32_t i = lane; i < d; i += 64) s = fmaf(row[i], row[i], s);
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) inv[r] = s > 0.f ? 1.0f / sqrtf(s) : 0.f;
}

__global__ __launch_bounds__(256) void topk_init_kernel(uint32_t Q, float theta0,
                                                        float* __restrict__ theta,
                                                        uint32_t* __restrict__ cnt,
                                                        uint32_t* __restrict__ best_cnt,
                                                        uint32_t* __restrict__ err) {
    uint32_t q = blockIdx.x * 256 + threadIdx.x;
    if (q == 0) *err = 0u;
    if (q >= Q) return;
    theta[q] = theta0;
    cnt[q] = 0u;
    best_cnt[q] = 0u;
}

// ---------------------------------------------------------------------------------------------
// Scores of 128 queries x 128 candidates over all d columns, then the filter.
// Block b of the grid is mapped so that the blocks an XCD receives (b mod 8) walk through the
// query tiles of one candidate tile after the other: the candidate tile stays in that XCD's L2.
// v_mfma_f32_32x32x2_f32: lane l feeds A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32];
// accumulator register v of lane l is D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32].
// ---------------------------------------------------------------------------------------------
struct TopkArgs {
    const float* Qm; const float* Cm; uint32_t Q, N, d;
    uint32_t c_begin, c_end;            // candidates of this round
    uint32_t nq_tiles, nc_tiles;
    const float* invq; const float* invc; const float* theta;
    uint32_t* cnt; uint2* pend; uint32_t cap;
    uint32_t* err;
};

template <bool VEC4>
__device__ __forceinline__ float4 load_cols(const float* __restrict__ row, bool row_ok, uint32_t k,
                                            uint32_t d) {
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!row_ok) return r;
    if (VEC4) {
        if (k < d) r = *(const float4*)(row + k);            // d % 4 == 0: all four inside
    } else {
        if (k + 0 < d) r.x = row[k + 0];
        if (k + 1 < d) r.y = row[k + 1];
        if (k + 2 < d) r.z = row[k + 2];
        if (k + 3 < d) r.w = row[k + 3];
    }
    return r;
}

// The block is 2 x 2 wavefronts; a wavefront owns TM x TN matrix-core tiles of 32 x 32, so the
// block tile is (64 TM) queries x (64 TN) candidates.  WPE = wavefronts per SIMD the register
// budget is set for.
template <int TM, int TN, int WPE, bool VEC4>
__global__ __launch_bounds__(TK_THREADS, WPE) void topk_scores_kernel(TopkArgs a) {
    constexpr int BQ = 64 * TM, BC = 64 * TN;
    constexpr int MOVES_A = BQ * TK_BK / 4 / TK_THREADS, MOVES_B = BC * TK_BK / 4 / TK_THREADS;
    __shared__ float As[2][BQ][TK_LD];
    __shared__ float Bs[2][BC][TK_LD];
    __shared__ float s_invq[BQ];
    __shared__ float s_theta[BQ];
    __shared__ __align__(16) float s_tq[BQ];

    const uint32_t total = a.nq_tiles * a.nc_tiles;
    const uint32_t per_xcd = (total + 7u) / 8u;
    const uint32_t logical = (blockIdx.x % 8u) * per_xcd + blockIdx.x / 8u;
    if (logical >= total) return;                            // uniform per block, before any barrier
    const uint32_t q0 = (logical % a.nq_tiles) * BQ;
    const uint32_t c0 = a.c_begin + (logical / a.nq_tiles) * BC;

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / 2, wn = wave % 2;
    for (int i = tid; i < BQ; i += TK_THREADS) {
        const uint32_t q = q0 + i;
        const float iq = q < a.Q ? a.invq[q] : 0.f;
        const float th = q < a.Q ? a.theta[q] : INFINITY;
        s_invq[i] = iq;
        s_theta[i] = th;
        // The same threshold for the raw product dot x (1/|c|), lowered by 2^-20 of itself so that
        // no score the exact test below accepts is missed (the two roundings of the score and the
        // ones made here stay under 2^-22 relative); -inf sends every element to the exact test.
        float t;
        if (iq == 0.f) {
            t = th <= 0.f ? -INFINITY : INFINITY;         // every score of a zero query is 0
        } else {
            const float r = th / iq;
            t = fabsf(r) < INFINITY ? r - fabsf(r) * 0x1p-20f : (r > 0.f && th == INFINITY ? INFINITY : -INFINITY);
        }
        s_tq[i] = t;
    }

    // Staging through two LDS buffers of TK_BK columns: while a panel is multiplied, the next one
    // is written to the other buffer (from registers loaded during the panel before) and the one
    // after is requested from memory; one barrier per panel.  Thread t moves float4 number t,
    // t + 256, ... of a panel, i.e. the same four columns of rows srow0, srow0 + TK_RPM, ...
    // (One buffer of 32 columns with a barrier on either side of its refill measured 1 % slower.)
    const int srow0 = tid / (TK_BK / 4), scol = (tid % (TK_BK / 4)) * 4;
    const float* arow0 = a.Qm + (uint64_t)(q0 + srow0) * a.d;      // not dereferenced past Q / c_end
    const float* brow0 = a.Cm + (uint64_t)(c0 + srow0) * a.d;
    const uint64_t row_step = (uint64_t)TK_RPM * a.d;
    float4 ra[MOVES_A], rb[MOVES_B];
    auto fetch = [&](uint32_t col0) {
#pragma unroll
        for (int i = 0; i < MOVES_A; ++i)
            ra[i] = load_cols<VEC4>(arow0 + i * row_step, q0 + srow0 + i * TK_RPM < a.Q, col0 + scol, a.d);
#pragma unroll
        for (int i = 0; i < MOVES_B; ++i)
            rb[i] = load_cols<VEC4>(brow0 + i * row_step, c0 + srow0 + i * TK_RPM < a.c_end, col0 + scol, a.d);
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MOVES_A; ++i) {
            float* pa = &As[buf][srow0 + i * TK_RPM][scol];
            pa[0] = ra[i].x; pa[1] = ra[i].y; pa[2] = ra[i].z; pa[3] = ra[i].w;
        }
#pragma unroll
        for (int i = 0; i < MOVES_B; ++i) {
            float* pb = &Bs[buf][srow0 + i * TK_RPM][scol];
            pb[0] = rb[i].x; pb[1] = rb[i].y; pb[2] = rb[i].z; pb[3] = rb[i].w;
        }
    };
    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int fr = lane & 31, fk = lane >> 5;
    fetch(0);
    stash(0);
    if (TK_BK < a.d) fetch(TK_BK);
    __syncthreads();
    int cur = 0;
    for (uint32_t kb = 0; kb < a.d; kb += TK_BK, cur ^= 1) {
        if (kb + TK_BK < a.d) {
            stash(cur ^ 1);
            if (kb + 2 * TK_BK < a.d) fetch(kb + 2 * TK_BK);
        }
        const int kmax = (int)min((uint32_t)TK_BK, a.d - kb);     // columns beyond d hold zeros: skipped
        // one step of two columns per trip (longer straight runs, which would let the compiler
        // issue LDS reads under earlier products, measured the same; 16-byte LDS accesses on a
        // column order that gives each lane four adjacent floats per four steps measured slower)
#pragma unroll 1
        for (int kk = 0; kk < kmax; kk += 2) {
            float av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[cur][wm * 32 * TM + i * 32 + fr][kk + fk];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[j] = Bs[cur][wn * 32 * TN + j * 32 + fr][kk + fk];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // filter: a score at or above the query's threshold joins the query's pending list.  For a
    // given accumulator register the 32 lanes of a half-wavefront hold 32 candidates of one query,
    // so each half reserves its slots with a single atomic.
    // Most tiles hold no such score once the thresholds have risen, so each 32 x 32 tile is first
    // screened with two instructions per element (raw product against the lowered threshold);
    // only a tile with a hit goes through the exact test.
#pragma unroll
    for (int ti = 0; ti < TM; ++ti) {
        const int qbase = wm * 32 * TM + ti * 32 + 4 * fk;   // this lane's queries: qbase + 8 (v/4) + v%4
        float tq[16];
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const float4 t4 = *reinterpret_cast<const float4*>(&s_tq[qbase + 8 * v4]);
            tq[4 * v4 + 0] = t4.x; tq[4 * v4 + 1] = t4.y; tq[4 * v4 + 2] = t4.z; tq[4 * v4 + 3] = t4.w;
        }
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const uint32_t c = c0 + wn * 32 * TN + tj * 32 + fr;
            const bool c_ok = c < a.c_end;
            const float ic = c_ok ? a.invc[c] : 0.f;
            float over = -INFINITY;
#pragma unroll
            for (int v = 0; v < 16; ++v) over = fmaxf(over, fmaf(acc[ti][tj][v], ic, -tq[v]));
            if (__ballot(over >= 0.f) == 0) continue;        // uniform per wavefront
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int ql = qbase + 8 * (v / 4) + (v % 4);
                const float s = acc[ti][tj][v] * s_invq[ql] * ic;
                const bool pass = c_ok && s >= s_theta[ql];  // padded queries carry +inf: never
                const uint64_t both = __ballot(pass);
                const uint32_t half = fk ? (uint32_t)(both >> 32) : (uint32_t)both;
                if (half) {
                    const uint32_t q = q0 + ql;
                    const int leader = __ffs(half) - 1 + 32 * fk;
                    uint32_t base = 0;
                    if (lane == leader) base = atomicAdd(&a.cnt[q], (uint32_t)__popc(half));
                    base = __shfl(base, leader, 64);
                    if (pass) {
                        const uint32_t slot = base + (uint32_t)__popc(half & ((1u << fr) - 1u));
                        if (slot < a.cap)
                            a.pend[(uint64_t)q * a.cap + slot] = make_uint2(__float_as_uint(s), c);
                        else
                            atomicOr(a.err, 1u);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Selection: one wavefront per query folds the pending entries, 64 at a time, into the sorted best
// list (bitonic sort of 128 in LDS; order: higher score first, equal scores by lower index), then
// raises the query's threshold to its K-th best and empties the pending list.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ bool ranks_before(float sa, uint32_t ia, float sb, uint32_t ib) {
    return sa > sb || (sa == sb && ia < ib);
}

__global__ __launch_bounds__(64) void topk_select_kernel(uint32_t Q, uint32_t K, uint32_t cap,
                                                         uint32_t* __restrict__ cnt,
                                                         const uint2* __restrict__ pend,
                                                         uint2* __restrict__ best,
                                                         uint32_t* __restrict__ best_cnt,
                                                         float* __restrict__ theta) {
    __shared__ float s_sc[2 * TK_LIST];
    __shared__ uint32_t s_ix[2 * TK_LIST];
    const uint32_t q = blockIdx.x;
    const int t = threadIdx.x;
    if (q >= Q) return;
    const uint32_t n_new = min(cnt[q], cap);
    if (n_new == 0) return;
    const uint32_t bc = best_cnt[q];
    {
        const uint2 e = (uint32_t)t < bc ? best[(uint64_t)q * TK_LIST + t] : make_uint2(0u, TK_NONE);
        s_sc[t] = (uint32_t)t < bc ? __uint_as_float(e.x) : -INFINITY;
        s_ix[t] = e.y;
    }
    for (uint32_t base = 0; base < n_new; base += TK_LIST) {
        const uint32_t e = base + t;
        const uint2 p = e < n_new ? pend[(uint64_t)q * cap + e] : make_uint2(0u, TK_NONE);
        s_sc[TK_LIST + t] = e < n_new ? __uint_as_float(p.x) : -INFINITY;
        s_ix[TK_LIST + t] = p.y;
        __syncthreads();
        for (int k = 2; k <= 2 * TK_LIST; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int i = 2 * t - (t & (j - 1)), l = i + j;
                const bool up = (i & k) == 0;
                const float si = s_sc[i], sl = s_sc[l];
                const uint32_t ii = s_ix[i], il = s_ix[l];
                const bool swap = up ? ranks_before(sl, il, si, ii) : ranks_before(si, ii, sl, il);
                if (swap) { s_sc[i] = sl; s_ix[i] = il; s_sc[l] = si; s_ix[l] = ii; }
                __syncthreads();
            }
        }
    }
    const uint32_t have = min((uint64_t)K, (uint64_t)bc + n_new);
    best[(uint64_t)q * TK_LIST + t] = make_uint2(__float_as_uint(s_sc[t]), s_ix[t]);
    if (t == 0) {
        best_cnt[q] = have;
        if (have == K) theta[q] = s_sc[K - 1];
        cnt[q] = 0u;
    }
}

// Result: the first K of the best list with similarity > tau; unused slots get TK_NONE and 0.
__global__ __launch_bounds__(64) void topk_finish_kernel(uint32_t Q, uint32_t K, float tau,
                                                         const uint2* __restrict__ best,
                                                         const uint32_t* __restrict__ best_cnt,
                                                         uint32_t* __restrict__ out_idx,
                                                         float* __restrict__ out_score,
                                                         uint32_t* __restrict__ out_count) {
    const uint32_t q = blockIdx.x;
    const uint32_t t = threadIdx.x;
    if (q >= Q) return;
    const uint32_t bc = best_cnt[q];
    const uint2 e = t < bc ? best[(uint64_t)q * TK_LIST + t] : make_uint2(0u, TK_NONE);
    const float s = __uint_as_float(e.x);
    const bool ok = t < bc && t < K && s > tau;
    if (t < K) {
        out_idx[(uint64_t)q * K + t] = ok ? e.y : TK_NONE;
        out_score[(uint64_t)q * K + t] = ok ? s : 0.f;
    }
    const uint64_t mask = __ballot(ok);
    if (t == 0 && out_count) out_count[q] = (uint32_t)__popcll(mask);
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct TopkLayout {
    size_t invq, invc, theta, cnt, best_cnt, err, best, pend, fixed_bytes;
};

static TopkLayout topk_layout(uint32_t Q, uint32_t N) {
    TopkLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
    L.invq = take(sizeof(float) * Q);
    L.invc = take(sizeof(float) * N);
    L.theta = take(sizeof(float) * Q);
    L.cnt = take(sizeof(uint32_t) * Q);
    L.best_cnt = take(sizeof(uint32_t) * Q);
    L.err = take(256);
    L.best = take(sizeof(uint2) * (size_t)Q * TK_LIST);
    L.pend = off;
    L.fixed_bytes = off;
    return L;
}

size_t topk_workspace_bytes(uint32_t Q, uint32_t N, uint32_t round_candidates) {
    uint32_t cap = ((round_candidates + TK_BC - 1) / TK_BC) * TK_BC;
    return topk_layout(Q, N).fixed_bytes + sizeof(uint2) * (size_t)Q * cap;
}

uint32_t topk_round_capacity(uint32_t Q, uint32_t N, size_t workspace_bytes) {
    const size_t fixed = topk_layout(Q, N).fixed_bytes;
    if (workspace_bytes <= fixed) return 0;
    size_t cap = (workspace_bytes - fixed) / (sizeof(uint2) * (size_t)Q);
    cap = (cap / TK_BC) * TK_BC;
    const size_t all = ((size_t)N + TK_BC - 1) / TK_BC * TK_BC;
    return (uint32_t)(cap < all ? cap : all);
}

uint32_t* launch_topk_cosine(const float* Qm, uint32_t Q, const float* Cm, uint32_t N, uint32_t d,
                             uint32_t K, float tau, uint32_t* out_idx, float* out_score,
                             uint32_t* out_count, void* workspace, uint32_t cap, hipStream_t st) {
    const TopkLayout L = topk_layout(Q, N);
    char* ws = (char*)workspace;
    float* invq = (float*)(ws + L.invq);
    float* invc = (float*)(ws + L.invc);
    float* theta = (float*)(ws + L.theta);
    uint32_t* cnt = (uint32_t*)(ws + L.cnt);
    uint32_t* best_cnt = (uint32_t*)(ws + L.best_cnt);
    uint32_t* err = (uint32_t*)(ws + L.err);
    uint2* best = (uint2*)(ws + L.best);
    uint2* pend = (uint2*)(ws + L.pend);

    hipLaunchKernelGGL(inv_norm_kernel, dim3(blocks_for((uint64_t)Q * 64, 256)), dim3(256), 0, st, Qm,
                       Q, d, invq);
    hipLaunchKernelGGL(inv_norm_kernel, dim3(blocks_for((uint64_t)N * 64, 256)), dim3(256), 0, st, Cm,
                       N, d, invc);
    // nothing below the threshold is ever wanted; without one, every cosine passes (-2 < -1)
    const float theta0 = tau > -2.0f ? tau : -2.0f;
    hipLaunchKernelGGL(topk_init_kernel, dim3(blocks_for(Q, 256)), dim3(256), 0, st, Q, theta0, theta,
                       cnt, best_cnt, err);
    TopkArgs a{};
    a.Qm = Qm; a.Cm = Cm; a.Q = Q; a.N = N; a.d = d;
    a.invq = invq; a.invc = invc; a.theta = theta; a.cnt = cnt; a.pend = pend; a.cap = cap;
    a.err = err;
    // 2 x 2 tiles per wavefront at four wavefronts per SIMD (128 registers, accumulators included)
    // measured best: 2 x 4 and 4 x 2 tiles (two wavefronts per SIMD) ran 9 % slower, 4 x 4 (one) 2.3
    // times slower -- this kernel lives on having other wavefronts to switch to at its barriers.
    constexpr int TK_TM = 2, TK_TN = 2, TK_WPE = 4;
    constexpr int BQ = 64 * TK_TM, BC = 64 * TK_TN;
    a.nq_tiles = (Q + BQ - 1) / BQ;
    // The first rounds are short and grow fourfold: with a threshold from the first few hundred
    // candidates only a small share of a full round's scores reaches the pending lists.
    uint64_t len = TK_BC;
    for (uint64_t begin = 0; begin < N; begin += len, len = (len * 4 < cap ? len * 4 : cap)) {
        if (len > cap) len = cap;
        a.c_begin = (uint32_t)begin;
        a.c_end = (uint32_t)(begin + len < N ? begin + len : N);
        a.nc_tiles = (a.c_end - a.c_begin + BC - 1) / BC;
        const uint32_t total = a.nq_tiles * a.nc_tiles;
        const dim3 grid(((total + 7u) / 8u) * 8u), block(TK_THREADS);
        if (d % 4 == 0 && ((uintptr_t)Qm % 16 == 0) && ((uintptr_t)Cm % 16 == 0))
            hipLaunchKernelGGL((topk_scores_kernel<TK_TM, TK_TN, TK_WPE, true>), grid, block, 0, st, a);
        else
            hipLaunchKernelGGL((topk_scores_kernel<TK_TM, TK_TN, TK_WPE, false>), grid, block, 0, st, a);
        hipLaunchKernelGGL(topk_select_kernel, dim3(Q), dim3(64), 0, st, Q, K, cap, cnt, pend, best,
                           best_cnt, theta);
    }
    hipLaunchKernelGGL(topk_finish_kernel, dim3(Q), dim3(64), 0, st, Q, K, tau, best, best_cnt,
                       out_idx, out_score, out_count);
    return err;
}

// Column slice of the listed rows written into full-width vectors: dst[i][col_begin + c] =
// M[rows[i]][c] (Section 6.1.4: partial vectors of the shards joined into whole vectors).
__global__ __launch_bounds__(256) void export_rows_kernel(const float* __restrict__ M,
                                                          uint32_t stride, uint32_t d_slice,
                                                          const uint32_t* __restrict__ rows,
                                                          uint32_t m, uint32_t V,
                                                          float* __restrict__ dst, uint32_t d_total,
                                                          uint32_t col_begin, uint32_t* err) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (uint64_t)m * d_slice) return;
    const uint32_t r = (uint32_t)(i / d_slice), c = (uint32_t)(i % d_slice);
    uint32_t w = rows[r];
    if (w >= V) { if (c == 0) atomicOr(err, 1u); w = 0; }
    dst[(uint64_t)r * d_total + col_begin + c] = M[(uint64_t)w * stride + c];
}

void launch_export_rows(const float* M, RowGeom g, uint32_t d_slice, const uint32_t* rows, uint32_t m,
                        uint32_t V, float* dst, uint32_t d_total, uint32_t col_begin, uint32_t* err,
                        hipStream_t st) {
    if (m == 0) return;
    hipLaunchKernelGGL(export_rows_kernel, dim3(blocks_for((uint64_t)m * d_slice, 256)), dim3(256), 0,
                       st, M, g.stride4 * 4, d_slice, rows, m, V, dst, d_total, col_begin, err);
}

}  // namespace w2v
