// Shared declarations of the shard library's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace w2v {

// ---- counter-based generator (Philox4x32, 10 rounds; Salmon et al., SC'11) -----------------------
// The fourth counter word separates the uses of the generator.
enum : uint32_t { DOM_INIT = 1, DOM_TOKEN = 2, DOM_NEG = 4, DOM_MBSEED = 5 };

struct U4 { uint32_t x, y, z, w; };

__host__ __device__ inline uint32_t mulhi32(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);
#endif
}

__host__ __device__ inline U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1) {
    const uint32_t MA = 0xD2511F53u, MB = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t hiA = mulhi32(MA, c0), loA = MA * c0;
        uint32_t hiB = mulhi32(MB, c2), loB = MB * c2;
        uint32_t t0 = hiB ^ c1 ^ k0;
        uint32_t t2 = hiA ^ c3 ^ k1;
        c0 = t0; c1 = loB; c2 = t2; c3 = loA;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

// ---- row geometry ------------------------------------------------------------------------------
// A row of either matrix is `stride4` float4 in memory, of which the first d4 = ceil(d_slice/4)
// carry data (columns >= d_slice inside the last float4 are kept at zero).  A group of G lanes owns
// one row at a time; lane l holds float4 number l, l+G, ..., l+(NV-1)G.
struct RowGeom {
    uint32_t d4;        // float4 per row that carry data
    uint32_t stride4;   // float4 between consecutive rows
};

constexpr uint32_t KEY_NONE = 0xFFFFFFFFu;   // "no destination" in partial-sum key arrays
constexpr uint32_t KEY_ZERO = 0x80000000u;   // flag: slot belongs to the row but holds no data
constexpr uint32_t KEY_MASK = 0x7FFFFFFFu;
constexpr uint32_t KEY_ALONE = 0x80000000u;  // slot-ordered keys: no other slot names this row

// The per-call scalars a captured graph cannot take as kernel arguments (those are fixed when the
// graph is captured): where a `dev` pointer is given, the kernels read the minibatch seed and the
// learning rate from this block in device memory instead of from their arguments.
struct CallScalars { uint32_t seed_lo, seed_hi; float alpha; uint32_t reserved; };

// ---- launch wrappers (defined in the .hip files) -------------------------------------------------
struct NoiseTable { const uint2* bins; uint32_t V; };   // {keep threshold, alias} per word

void launch_init(float* M, uint32_t V, RowGeom g, uint32_t d_slice, uint32_t d_total,
                 uint32_t col_begin, uint64_t seed, uint32_t matrix, bool zero, hipStream_t st);
void launch_gather_rows(const float* M, RowGeom g, uint32_t d_slice, const uint32_t* rows,
                        uint32_t m, uint32_t V, float* dst, uint32_t* err, hipStream_t st);
void launch_scatter_rows(float* M, RowGeom g, uint32_t d_slice, const uint32_t* rows, uint32_t m,
                         uint32_t V, const float* src, uint32_t* err, hipStream_t st);

// keys[p*T + 0] = out_idx[p], keys[p*T + j] = negative j.  An output word >= V raises *err and is
// replaced by 0.  in_safe[p] (launch_check_inputs) is the checked copy of in_idx[p] that every
// later kernel uses.
void launch_dest_keys(NoiseTable nt, const uint32_t* out_idx, uint32_t n, uint32_t k, uint64_t seed,
                      uint32_t* keys, uint32_t* err, hipStream_t st,
                      const CallScalars* dev = nullptr);
// keys[sidx[i]] |= KEY_ALONE for every sorted entry i whose neighbours carry other keys.
void launch_mark_alone(const uint32_t* skey, const uint32_t* sidx, uint32_t M, uint32_t* keys,
                       hipStream_t st);
void launch_check_inputs(const uint32_t* in_idx, uint32_t n, uint32_t V, uint32_t* in_safe,
                         uint32_t* err, hipStream_t st);
// launch_dest_keys + launch_check_inputs + two fills of 32-bit words in one launch (n pairs, T = k+1
// slots each).  With `dev` the seed is read from device memory; with `scalars_out` the seed and the
// learning rate given here are also written there, for the kernels that follow.
struct FillJob { uint32_t* p; uint32_t count; uint32_t value; };
struct IndexPrologue {
    NoiseTable nt; const uint32_t* out_idx; uint32_t n, T; uint32_t seed_lo, seed_hi; uint32_t* keys;
    const CallScalars* dev;
    const uint32_t* in_idx; uint32_t* in_safe;
    uint32_t* err;
    FillJob fill[2];
    CallScalars* scalars_out; float alpha;
    uint32_t b_check, b_fill[2];        // first block of each part (set by the launcher)
};
void launch_index_prologue(IndexPrologue a, hipStream_t st);
void launch_copy_negatives(const uint32_t* keys, uint32_t n, uint32_t k, uint32_t* neg,
                           hipStream_t st);

void launch_dots(const float* U, const float* W, RowGeom g, const uint32_t* in_safe,
                 const uint32_t* keys, uint32_t n, uint32_t T, float* dots, hipStream_t st);

struct PartialPtrs { const float* p[32]; };
void launch_coeffs(PartialPtrs parts, uint32_t S, uint32_t n, uint32_t T, float* coeffs,
                   double* block_loss, double* loss_out, hipStream_t st);
size_t coeffs_loss_scratch_doubles(uint32_t n, uint32_t T);

// Stable least-significant-digit radix sort of (keys_in[i], i) on `bits` key bits.  keys_in is
// only read; the passes ping-pong between buf0 and buf1 (n 8-byte words each, 8-byte aligned), and
// the sorted keys and indices end up as two arrays of n uint32 inside one of the two buffers,
// returned through out_keys/out_vals.  tmp holds sort_scratch_u32(n0, n1) uint32 (8-byte aligned).
// launch_sort_jobs sorts one or two independent arrays with the same launches (the second rides
// along with the first: no launches of its own).  err: sticky flag, bit 1 is raised if a bounded
// wait inside the sort runs out (cannot happen unless the device stalls a running block for about
// a second); may be null.
struct SortJob {
    const uint32_t* keys_in; uint32_t n; uint2* buf0; uint2* buf1;
    uint32_t** out_keys; uint32_t** out_vals;
};
size_t sort_scratch_u32(uint32_t n0, uint32_t n1 = 0);
void launch_sort_jobs(const SortJob* jobs, int njobs, uint32_t bits, uint32_t* tmp, uint32_t* err,
                      hipStream_t st, bool cleared = false);
// The part of tmp that must read zero when the sort starts (launch_sort_jobs clears it itself unless
// told that the caller has).
FillJob sort_clear_job(const SortJob* jobs, int njobs, uint32_t* tmp);
void launch_sort_pairs(const uint32_t* keys_in, uint2* buf0, uint2* buf1, uint32_t n, uint32_t bits,
                       uint32_t* tmp, uint32_t** out_keys, uint32_t** out_vals, uint32_t* err,
                       hipStream_t st);

// Exclusive prefix sum of n uint32 (in place allowed); total (may be null) gets the sum.
size_t scan_scratch_u32(uint32_t n);
void launch_exclusive_scan(const uint32_t* in, uint32_t* out, uint32_t n, uint32_t* tmp,
                           uint32_t* total, hipStream_t st);

// ---- adjust ------------------------------------------------------------------------------------
// Chunk sizes of the segmented reductions (entries per lane group).
uint32_t useg_pairs_per_chunk(uint32_t T, uint32_t d4, uint32_t n);   // by slots per pair, row geometry and minibatch size;
                                                          // smallest for the narrowest rows (d4 = 1)
uint32_t wseg_entries_per_chunk();
uint32_t tail_entries_per_chunk();

// Input-vector side, level 1.  Sorted pairs ps = 0..n-1 (key skey[ps] = in_idx of pair perm[ps]).
// A lane group sums coeffs[p][j] * W[keys[p][j]] over the pairs of its chunk; a run of equal keys
// that lies inside the chunk is written to delta[first ps of run] with dkey[ps] = key (KEY_NONE
// elsewhere); runs cut by a chunk border go to the partial slots (pkeys/prows), two per border.
// With `fused` the group also loads u = U[key], forms the dots, writes coefficients
// and uses those coefficients.
struct USideArgs {
    const float* U; const float* W; RowGeom g;
    const uint32_t* skey; const uint32_t* perm; const uint32_t* keys; uint32_t n; uint32_t T;
    const float* coeffs_in;      // unfused: coefficients to use
    float* coeffs_out;           // fused: coefficients written here [n][T]
    float* dots_out;             // fused, optional: the dots themselves
    float* delta; uint32_t* dkey;
    float* prows; uint32_t* pkeys;
    bool fused;
    // fused only, optional (W_update != null): keys carrying KEY_ALONE name rows that no other slot
    // of the minibatch names; the kernel then writes W[row] += alpha * g * u itself (nobody else
    // reads or writes that row in this minibatch) and the output side must leave those slots out.
    float* W_update; float alpha;
    const CallScalars* dev;      // optional: the learning rate is read from here
};
void launch_useg(const USideArgs& a, hipStream_t st);
// Minibatch loss from the dots of the fused step: slot 0 of a pair contributes softplus(-f), the
// others softplus(f).  tmp holds coeffs_loss_scratch_doubles(n, T) doubles.
void launch_loss_from_dots(const float* dots, uint32_t n, uint32_t T, double* tmp, double* loss_out,
                           hipStream_t st);

// Output-vector side, level 1.  Sorted contributions i = 0..M-1 with destination skey[i] and
// original slot sidx[i] = p*T + j: adds alpha * sum coeffs[sidx] * U[in_idx[p]] to W[skey] for runs
// inside a chunk; cut runs go to the partial slots.
struct WSideArgs {
    const float* U; float* W; RowGeom g;
    const uint32_t* skey; const uint32_t* sidx; uint32_t M; uint32_t T;
    bool skip_alone;             // entries whose neighbours carry other keys are handled elsewhere
    const uint32_t* in_idx; const float* coeffs; float alpha;
    float* prows; uint32_t* pkeys;
    const CallScalars* dev;      // optional: the learning rate is read from here
};
// (the cells' border slots must read KEY_NONE when the kernel starts: launch_wseg_fill writes that;
// launch_wseg does it itself unless told that the caller already has)
FillJob wseg_fill_job(uint32_t* pkeys, uint32_t M);
void launch_wseg_fill(uint32_t* pkeys, uint32_t M, hipStream_t st);
void launch_wseg(const WSideArgs& a, hipStream_t st, bool filled = false);

// Higher levels (both sides): entries are partial rows src_rows[i] with destination src_keys[i]
// (KEY_NONE = nothing, KEY_ZERO flag = belongs to the run but empty).
struct TailArgs {
    float* M; RowGeom g; float alpha;
    const float* src_rows; const uint32_t* src_keys; uint32_t entries;
    float* prows; uint32_t* pkeys;
    // input side only: finished sums go to the delta buffer (rows, keys) instead of into M;
    // level = 1 for the first pass over the input-side kernel's slots, cp = its pairs per chunk
    float* defer_rows = nullptr; uint32_t* defer_keys = nullptr; uint32_t level = 0, cp = 0;
    const CallScalars* dev = nullptr;      // optional: the learning rate is read from here
};
void launch_tail(const TailArgs& a, hipStream_t st);

// Parts of one update that do not depend on each other, in ONE launch (each may be absent): the
// output side's level-1 kernel (wfirst; its border slots already cleared) or one of its higher
// levels (wtail), one higher level of the input side (utail, with defer_rows), and one step of the
// loss of the fused form (loss_step 1: dots -> block sums in loss_tmp, needs at most
// adjust_stage_loss_blocks_max() blocks of 256 terms; 2: block sums -> *loss_out).  Same code and
// same bits as the separate launches.  Only for the row geometries adjust_stage_supported names.
struct AdjustStage {
    const WSideArgs* wfirst = nullptr; const TailArgs* wtail = nullptr; const TailArgs* utail = nullptr;
    uint32_t loss_step = 0; const float* dots = nullptr; uint32_t n = 0, T = 0;
    double* loss_tmp = nullptr; double* loss_out = nullptr;
};
bool adjust_stage_supported(uint32_t d4);
uint32_t adjust_stage_loss_blocks_max();
void launch_adjust_stage(const AdjustStage& x, hipStream_t st);

// U[dkey[ps]] += alpha * delta[ps] wherever dkey[ps] != KEY_NONE.
void launch_apply_delta(float* U, RowGeom g, const float* delta, const uint32_t* dkey, uint32_t n,
                        float alpha, hipStream_t st, const CallScalars* dev = nullptr);

// ---- pair formation ------------------------------------------------------------------------------
struct PairArgs {
    const uint32_t* tokens; const uint64_t* sent_off; uint32_t n_sent; uint32_t n_tokens;
    uint64_t token_base; uint32_t epoch; uint64_t seed; uint32_t B; const uint64_t* keep; uint32_t V;
    uint32_t* in_idx; uint32_t* out_idx; uint64_t capacity;
    bool interleave;        // centers round-robin over the sentences instead of corpus order
    // bag-of-words examples (plain order only; in_idx may then be null): ctx_off[cap_examples+1],
    // centers[cap_examples], *total_examples; out_idx holds the context words
    uint32_t* ctx_off; uint32_t* centers; uint64_t cap_examples; uint32_t* total_examples;
    uint32_t* scratch;      // pairs_scratch_u32(n_tokens, interleave) uint32
    uint32_t* total_pairs;  // device, one uint32
    uint32_t* err;
};
size_t pairs_scratch_u32(uint32_t n_tokens, bool interleave);
void launch_make_pairs(const PairArgs& a, hipStream_t st);

// ---- export and retrieval ----------------------------------------------------------------------------
void launch_export_rows(const float* M, RowGeom g, uint32_t d_slice, const uint32_t* rows, uint32_t m,
                        uint32_t V, float* dst, uint32_t d_total, uint32_t col_begin, uint32_t* err,
                        hipStream_t st);
// Workspace of the top-K search for rounds of `round_candidates` candidates, and the largest round a
// given workspace allows (multiple of 128; 0: too small).
size_t topk_workspace_bytes(uint32_t Q, uint32_t N, uint32_t round_candidates);
uint32_t topk_round_capacity(uint32_t Q, uint32_t N, size_t workspace_bytes);
uint32_t* launch_topk_cosine(const float* Qm, uint32_t Q, const float* Cm, uint32_t N, uint32_t d,
                             uint32_t K, float tau, uint32_t* out_idx, float* out_score,
                             uint32_t* out_count, void* workspace, uint32_t cap, hipStream_t st);

// ---- continuous bag of words ----------------------------------------------------------------------
// Per context entry: checked word, example number, weight 1/|C|; offsets are validated (error flag).
void launch_cbow_entries(const uint32_t* ctx_off, const uint32_t* ctx_idx, uint32_t n, uint32_t m,
                         uint32_t V, uint32_t* ctx_safe, uint32_t* ex_of, float* weight,
                         uint32_t* err, hipStream_t st);
void launch_iota(uint32_t* x, uint32_t n, hipStream_t st);
// H[p] = mean of U[ctx_safe[e]] over the entries of example p (row geometry g).
void launch_cbow_hidden(const float* U, RowGeom g, const uint32_t* ctx_off, const uint32_t* ctx_safe,
                        uint32_t n, uint32_t m, float* H, hipStream_t st);
void launch_cbow_examples(const uint32_t* kcnt, const uint32_t* kword, const uint32_t* poff,
                          const uint32_t* n_kept, uint32_t n, uint32_t* flag, uint32_t* ex,
                          uint32_t* scan_tmp, uint32_t* ctx_off, uint32_t* out_idx,
                          uint64_t cap_examples, uint32_t* total_examples, hipStream_t st);

}  // namespace w2v
