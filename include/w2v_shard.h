/*
 * w2v_shard.h -- C ABI of the MI355X shard library (libw2v_shard.so).
 *
 * One `w2v_shard` is one parameter-server shard of the column-partitioned word2vec system of
 * Ordentlich et al., arXiv 1606.08495 (Section 5.1): it holds d_slice consecutive columns of EVERY
 * input vector u(w) and output vector v(w), w = 0..V-1 (word index = rank in the vocabulary
 * ordering), as two fp32 matrices U and W in the HBM of the current HIP device, plus the noise
 * table the negatives are drawn from.  The calls below are the paper's remote procedure calls
 * (dotprod, adjust, get), the client's aggregation between them, and the client's pair formation.
 *
 * Conventions for every call
 *   - returns 0 on success and a negative W2V_ERR_* code otherwise; w2v_last_error() gives the text
 *     of the calling thread's last failure.  Nothing throws across this boundary.
 *   - "dev" pointers are device memory of the shard's GPU, owned by the caller, read or written only
 *     by work queued on `stream` (a hipStream_t passed as void*, NULL = the default stream).  The
 *     library keeps none of them after the call.  "host" pointers are ordinary host memory, used
 *     before the call returns.
 *   - calls that take a stream only queue work on it; they return before the work has run.  Calls on
 *     one shard share that shard's scratch memory and must be stream-ordered with one another (same
 *     stream, or the caller orders them).  Scratch grows to the largest request seen and is then
 *     reused, so a steady-state training loop allocates nothing (cf. Section 6.1.3: the paper's
 *     shards also create no objects in steady state).  Part of a call's work may run on streams
 *     the shard owns (one for work beside the call's main kernels, one for announced minibatches),
 *     forked from `stream` and joined back into it by events before the call returns: for the
 *     caller everything is ordered on `stream`.
 *   - index arrays are uint32 word indices < V.  An index >= V never causes an out-of-range access:
 *     the kernel substitutes word 0 and raises a sticky flag that w2v_shard_status() reports.
 *   - layouts are row-major and dense: partial_dots / coeffs are [n][k+1] with the positive output
 *     word in column 0 and the k negatives in columns 1..k (the paper's F+ / F- and G+ / G-
 *     arrays, interleaved per pair).
 *
 * Limits: 2 <= V <= 2^31-1 (V = 1 is accepted when k = 0), 1 <= d_slice <= W2V_D_MAX,
 * 0 <= k <= W2V_K_MAX, n*(k+1) < 2^31, S <= W2V_S_MAX.
 */
#ifndef W2V_SHARD_H
#define W2V_SHARD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define W2V_K_MAX 64
#define W2V_D_MAX 1024
#define W2V_S_MAX 32

#define W2V_OK             0
#define W2V_ERR_NULL      -1   /* a required pointer is NULL */
#define W2V_ERR_ARG       -2   /* a size or mode outside the limits above */
#define W2V_ERR_ALLOC     -3   /* device or host allocation failed */
#define W2V_ERR_HIP       -4   /* a HIP runtime call failed (text in w2v_last_error) */
#define W2V_ERR_STATE     -5   /* the noise table has not been set (w2v_shard_set_counts) */
#define W2V_ERR_INDEX     -6   /* some earlier call saw a word index >= V */
#define W2V_ERR_MISMATCH  -7   /* shards passed together differ in V, device or noise table */

typedef struct w2v_shard w2v_shard;

const char* w2v_last_error(void);

/* ---- shard life cycle (Section 5.1: column-wise partition; word2vec-style initial values) ------
 * Allocates U and W ([V][d_slice] fp32 each, kept with an internal row stride) on the current HIP
 * device and fills them on the device: every component is a pure function of (seed, word, GLOBAL
 * column, matrix), uniform on [-0.5/d_total, 0.5/d_total), so the S slices of one vector agree with
 * the unsliced vector.  init_mode 0: U uniform, W zero (the word2vec default).  init_mode 1: both
 * uniform.  w2v_shard_create(V, d, seed) is create_ex(V, d, 0, d, seed, 0).
 * The shard is bound to the device that was current at creation.  *out is owned by the caller until
 * w2v_shard_destroy, which synchronises the device and frees everything the shard holds. */
int w2v_shard_create(uint32_t V, uint32_t d_slice, uint64_t seed, w2v_shard** out);
int w2v_shard_create_ex(uint32_t V, uint32_t d_total, uint32_t col_begin, uint32_t d_slice,
                        uint64_t seed, int init_mode, w2v_shard** out);
int w2v_shard_destroy(w2v_shard* shard);

/* ---- vocabulary histogram -> noise table and subsample thresholds ---------------------------------
 * Section 3 defers to the word2vec paper for the noise distribution of the negatives (count^0.75)
 * and for the subsampling of frequent words.  counts_host[V] are occurrence counts.
 * Builds, on the host, a Vose alias table {keep threshold, alias}[V] for the count^0.75 law and the
 * per-word keep thresholds floor(min(1, sqrt(t/f)+t/f) * 2^32) (f = count share; subsample_t <= 0
 * disables subsampling), and uploads them.  Synchronous.  Must be called before any call that draws
 * negatives or forms pairs.  w2v_shard_get_tables copies the tables back (any pointer may be NULL). */
int w2v_shard_set_counts(w2v_shard* shard, const uint64_t* counts_host, double subsample_t);
int w2v_shard_get_tables(w2v_shard* shard, uint32_t* thresh_host, uint32_t* alias_host,
                         uint64_t* keep_host);

/* ---- get (Section 6.1.4, vector export) and its inverse ------------------------------------------
 * which: 0 = input vectors U, 1 = output vectors W.  rows_dev[m] word indices; dst_dev/src_dev is
 * [m][d_slice] dense.  set_rows with a word listed twice leaves one of the two values. */
int w2v_shard_get_rows(w2v_shard* shard, int which, const uint32_t* rows_dev, uint32_t m,
                       float* dst_dev, void* stream);
int w2v_shard_set_rows(w2v_shard* shard, int which, const uint32_t* rows_dev, uint32_t m,
                       const float* src_dev, void* stream);

/* Waits for `stream` and for the shard's own streams (announced minibatches are checked there), then
 * reports and clears the sticky bad-index flag (W2V_ERR_INDEX) or a pending HIP error. */
int w2v_shard_status(w2v_shard* shard, void* stream);

/* ---- negatives (Appendix, dotprod / adjust: N word indices other than the positive output word) -
 * neg_dev[n][k]: the negatives of pair p, slot j = 1..k, a pure function of (seed, p, j, out_idx[p])
 * and the noise table; exactly the ones w2v_dotprod and w2v_adjust use for the same arguments. */
int w2v_negatives(w2v_shard* shard, const uint32_t* out_idx_dev, uint32_t n, uint32_t k,
                  uint64_t seed, uint32_t* neg_dev, void* stream);

/* ---- dotprod (Appendix, "Server side computation - dotprod"; Section 5.1) ------------------------
 * For every pair p: partial_dots[p][0] = u_s(in_idx[p]) . v_s(out_idx[p]) and, for the k negatives
 * regenerated from `seed`, partial_dots[p][j] = u_s(in_idx[p]) . v_s(neg[p][j]), over this shard's
 * columns.  Does not modify the shard. */
int w2v_dotprod(w2v_shard* shard, const uint32_t* in_idx_dev, const uint32_t* out_idx_dev,
                uint32_t n, uint32_t k, uint64_t seed, float* partial_dots_dev, void* stream);

/* ---- w2v_dotprod for callers that cannot allocate ------------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid allocation: the
 * same operation, arguments, results (bit for bit) and errors as w2v_dotprod, but the call never
 * allocates or frees memory -- its scratch (the checked input words and the regenerated negatives)
 * lives in a fixed array of W2V_NOALLOC_SCRATCH_U32 uint32 (8 MiB) that is part of the library's
 * device code, one copy per GPU, held until the process ends.  A minibatch needs
 * roundup64(n*(k+1)) + n entries; larger ones are refused with W2V_ERR_ARG (use w2v_dotprod).
 * Every call on a GPU, from any shard, uses that GPU's one array: calls that may overlap on one
 * GPU (different streams, different threads) race and must be ordered by the caller.  Nothing in
 * the array needs to start at zero; it keeps the last call's contents.  Announced minibatches
 * (w2v_prefetch_minibatch) are not consulted, and no timing spans are recorded. */
#define W2V_NOALLOC_SCRATCH_U32 (1u << 21)
int w2v_dotprod_noalloc(w2v_shard* shard, const uint32_t* in_idx_dev, const uint32_t* out_idx_dev,
                        uint32_t n, uint32_t k, uint64_t seed, float* partial_dots_dev, void* stream);

/* ---- client aggregation (Appendix, "Grid based word2vec": F = sum_s F_s, then G+ and G-) ----------
 * partials_host[S] are S device arrays [n][k+1].  coeffs[p][0] = 1 - sigma(f), coeffs[p][j>0] =
 * -sigma(f), f the sum over shards in shard order.  The learning rate is NOT folded in; adjust takes
 * it separately and the product is the paper's G.  loss_dev (device double, may be NULL) receives
 * -sum[log sigma(f+) + sum log(1 - sigma(f-))], reduced in a fixed order.  Uses shard's scratch. */
int w2v_coeffs(w2v_shard* shard, const float* const* partials_host, uint32_t S, uint32_t n,
               uint32_t k, float* coeffs_dev, double* loss_dev, void* stream);

/* ---- adjust (Appendix, "Server side computation - adjust"; Section 5.1 last paragraph) -----------
 * Regenerates the negatives from `seed`, then for every pair p and slot j
 *     du(in_idx[p]) += coeffs[p][j] * v_s(row[p][j]),   dv(row[p][j]) += coeffs[p][j] * u_s(in_idx[p])
 * with every v_s, u_s read as it was when the call began, and finally adds alpha*du, alpha*dv to the
 * stored vectors, each touched row written once.  Contributions to one row are summed in an order
 * fixed by (n, k) alone, so results are bitwise reproducible. */
int w2v_adjust(w2v_shard* shard, const uint32_t* in_idx_dev, const uint32_t* out_idx_dev,
               uint32_t n, uint32_t k, uint64_t seed, const float* coeffs_dev, float alpha,
               void* stream);

/* ---- one client step in this process (Appendix, "Grid based word2vec", body of the minibatch loop)
 * dotprod on each of the S shards (shards_host[S], all on one device, same V and noise table),
 * aggregation, adjust on each shard.  With S = 1 the three phases are fused where that changes no
 * result beyond fp32 rounding.  loss_dev as in w2v_coeffs. */
int w2v_train_minibatch(w2v_shard* const* shards_host, uint32_t S, const uint32_t* in_idx_dev,
                        const uint32_t* out_idx_dev, uint32_t n, uint32_t k, uint64_t seed,
                        float alpha, double* loss_dev, void* stream);

/* ---- client-side pair formation (Eq.1 index sets; Section 3 footnote on "dirty" contexts) --------
 * tokens_dev[n_tokens] word indices; sent_off_dev[n_sent+1] token offsets of the sentences
 * (sent_off[0] = 0, sent_off[n_sent] = n_tokens); token_base = corpus position of tokens_dev[0].
 * Each token is kept or dropped by the subsample rule; on the surviving tokens of each sentence every
 * center draws a half-width b uniform on 1..B and pairs (center, context) are emitted for the
 * survivors within b positions, centers in corpus order, contexts by increasing position.  All draws
 * are functions of (corpus_seed, token position, epoch).  Writes at most `capacity` pairs to
 * in_idx_dev/out_idx_dev and the full count to *n_pairs_host.  Synchronises `stream`.
 * The formation calls keep scratch of their own in the shard and read only its subsample table:
 * on a stream of their own they may run beside a training call on the same shard (one formation
 * call at a time per shard).
 * Requires n_tokens * 2B < 2^32. */
int w2v_make_pairs(w2v_shard* shard, const uint32_t* tokens_dev, const uint64_t* sent_off_dev,
                   uint32_t n_sent, uint32_t n_tokens, uint64_t token_base, uint32_t epoch,
                   uint64_t corpus_seed, uint32_t B, uint32_t* in_idx_dev, uint32_t* out_idx_dev,
                   uint64_t capacity, uint64_t* n_pairs_host, void* stream);

/* ---- a training step captured once and replayed (the paper's minibatch sizes) ----------------------
 * Section 6.2 and Section 7.1 train with minibatches of 200, 50 or a single input word -- a few
 * thousand pairs at most.  At that size a step is a chain of some twenty small kernels and its time
 * is their launches.  w2v_step_graph_create captures w2v_train_minibatch(S = 1) for a fixed (n, k)
 * on this shard into a HIP graph, all but the step's first kernel, the only one that reads the
 * caller's arrays (it forms the destination keys and the checked input words); w2v_step_graph_run
 * queues that kernel on `stream` with this run's arrays, seed and learning rate (the last two it
 * also leaves in device memory, where the captured kernels read them) and replays the graph behind
 * it: the same kernels on the same data, hence the same bits as w2v_train_minibatch(in_idx, out_idx,
 * n, k, seed, alpha, loss).  The two arrays are read only by work queued on `stream` during the
 * call.  loss_dev (may be NULL) is fixed at creation and written by every run.
 * The captured step runs on one stream and uses the shard's scratch like any other call: order it
 * with other calls on the shard through `stream`.  Creating the graph allocates and synchronises;
 * running it does neither.  A call between creation and a run that needs a larger scratch region
 * (a larger n or k on the same shard) invalidates the graph: w2v_step_graph_run then returns
 * W2V_ERR_STATE and the graph has to be created again. */
typedef struct w2v_step_graph w2v_step_graph;
int w2v_step_graph_create(w2v_shard* shard, uint32_t n, uint32_t k, double* loss_dev,
                          w2v_step_graph** out);
int w2v_step_graph_run(w2v_step_graph* graph, const uint32_t* in_idx_dev, const uint32_t* out_idx_dev,
                       uint64_t seed, float alpha, void* stream);
int w2v_step_graph_destroy(w2v_step_graph* graph);

/* Optional look-ahead for a training loop on one shard.  Everything w2v_train_minibatch derives from
 * the indices alone -- the negatives, and the grouping of the minibatch's input and output rows that
 * makes the update deterministic -- depends on neither the vectors nor earlier minibatches.  This call
 * queues that work for a LATER minibatch on a stream the shard owns, ordered after the work queued
 * on `stream` so far, so that it runs beside the training call that is queued next:
 *     prefetch(h+1); train(h); prefetch(h+2); train(h+1); ...
 * or, on a column shard that serves the two calls of Section 5.1,
 *     prefetch(h+1); dotprod(h); adjust(h); prefetch(h+2); dotprod(h+1); adjust(h+1); ...
 * A w2v_train_minibatch whose first shard is this one, a w2v_dotprod or a w2v_adjust on this shard
 * with the same in_idx_dev, out_idx_dev (same pointers, contents unchanged in between), n, k and
 * seed uses the prepared work (w2v_dotprod leaves it in place for the w2v_adjust of the same
 * minibatch; an update consumes it); otherwise the call computes everything itself as if this call
 * had not been made.  Results are identical either way.  w2v_shard_set_counts voids what was
 * announced before it (the negatives came from the old table).
 * The two index arrays are read on the shard's own stream, possibly after this call has returned
 * (the one exception to the rule above that only work queued on `stream` touches the caller's
 * arrays): keep them allocated and unchanged until the call that uses the prepared work has been
 * queued on `stream`, or, if no such call follows, until the device has been synchronised.
 * Three announcements can be held at a time (a fourth replaces the oldest), so that a loop may run
 * two minibatches ahead -- prefetch(h+2); train(h); prefetch(h+3); train(h+1); ... -- which gives the
 * index work two steps to finish in where it does not fit beside one; each keeps its own device
 * buffers (about 20 (k+2) n bytes, allocated on first use and reused).  An announcement serves one of
 * the next three update calls on the shard; after that it is void (w2v_prefetch_cancel). */
int w2v_prefetch_minibatch(w2v_shard* shard, const uint32_t* in_idx_dev, const uint32_t* out_idx_dev,
                           uint32_t n, uint32_t k, uint64_t seed, void* stream);

/* Drops every announcement of either kind (w2v_prefetch_minibatch, w2v_cbow_prefetch_minibatch) that
 * has not been used, after waiting for the shard's look-ahead stream: on return the announced index
 * arrays are no longer read and may be changed or freed.  An announcement is matched by the
 * addresses of its arrays, so call this (or synchronise and never pass those addresses again)
 * before reusing an announced array's memory for other indices under the same n, k and seed.
 * Independently of this call, an announcement that the next three update calls on the shard
 * (w2v_adjust, w2v_train_minibatch and their bag-of-words forms) do not use is void. */
int w2v_prefetch_cancel(w2v_shard* shard);

/* ---- interleaved minibatch formation (Section 5.1, last paragraph) -------------------------------
 * Same arguments and the same set of pairs as w2v_make_pairs, in another order: the centers are
 * visited round-robin over the sentences of the block -- every sentence's first surviving token (in
 * sentence order), then every sentence's second, ... -- so that a minibatch cut from the pair stream
 * takes its input words from many different sentences, and the input words of one sentence fall
 * into successive minibatches.  Contexts of a center keep their order. */
int w2v_make_pairs_interleaved(w2v_shard* shard, const uint32_t* tokens_dev,
                               const uint64_t* sent_off_dev, uint32_t n_sent, uint32_t n_tokens,
                               uint64_t token_base, uint32_t epoch, uint64_t corpus_seed,
                               uint32_t B, uint32_t* in_idx_dev, uint32_t* out_idx_dev,
                               uint64_t capacity, uint64_t* n_pairs_host, void* stream);

/* ---- continuous-bag-of-words variant (Section 5.1, footnote: the architecture carries over) ----------
 * Example p (p = 0..n-1) has a center word out_idx[p], which plays the output role, and the context
 * words ctx_idx[ctx_off[p] .. ctx_off[p+1]), which play the input role.  Its hidden vector is the
 * mean of the context words' input vectors, h_p = (1/|C_p|) sum u_c, and it takes the place of the
 * input vector in Eq.1: the dots are h_p . v_row for row = center word and the k negatives (drawn as
 * for w2v_dotprod: functions of seed, p and the slot, different from the center word).  A column
 * slice of h_p is the mean of the slices, so partial dots of the shards add up as in Eq.3.  The update
 * is gradient ascent on that objective (Eq.4 / Eq.5 with h in place of u), from start-of-call
 * vectors:  v_row += alpha * g_pj * h_p  and, for every entry c of C_p,
 * u_c += alpha * (1/|C_p|) * sum_j g_pj * v_row_pj  (a word listed twice receives it twice).
 * An example with an empty context list has h = 0: zero dots, no change.
 *
 * ctx_off_dev[n+1] (first 0, non-decreasing, last m), ctx_idx_dev[m], out_idx_dev[n] are device
 * arrays owned by the caller; m < 2^31.  Offsets that break these rules, and words >= V, raise the
 * sticky index flag (w2v_shard_status) and are made harmless; they never fault.  Other arguments,
 * layouts of partial_dots / coeffs, errors and stream behaviour are those of w2v_dotprod,
 * w2v_adjust and w2v_train_minibatch. */
int w2v_cbow_dotprod(w2v_shard* shard, const uint32_t* ctx_off_dev, const uint32_t* ctx_idx_dev,
                     uint32_t m, const uint32_t* out_idx_dev, uint32_t n, uint32_t k, uint64_t seed,
                     float* partial_dots_dev, void* stream);
int w2v_cbow_adjust(w2v_shard* shard, const uint32_t* ctx_off_dev, const uint32_t* ctx_idx_dev,
                    uint32_t m, const uint32_t* out_idx_dev, uint32_t n, uint32_t k, uint64_t seed,
                    const float* coeffs_dev, float alpha, void* stream);
int w2v_cbow_train_minibatch(w2v_shard* const* shards, uint32_t S, const uint32_t* ctx_off_dev,
                             const uint32_t* ctx_idx_dev, uint32_t m, const uint32_t* out_idx_dev,
                             uint32_t n, uint32_t k, uint64_t seed, float alpha, double* loss_dev,
                             void* stream);

/* Look-ahead for the bag-of-words calls, as w2v_prefetch_minibatch is for the skip-gram ones: the
 * checked context entries, the negatives and both groupings of a LATER minibatch are computed on a
 * stream the shard owns, beside the calls queued next.  A w2v_cbow_train_minibatch whose first
 * shard is this one, a w2v_cbow_dotprod or a w2v_cbow_adjust on this shard with the same three
 * index arrays (same pointers, contents unchanged in between), m, n, k and seed uses the prepared
 * work (the dotprod leaves it in place, an update consumes it); results are identical either way.
 * Two announcements can be held at a time (each serves one of the next three update calls on the
 * shard); w2v_shard_set_counts voids what was announced before it.
 * As there, the three index arrays are read on the shard's own stream: keep them allocated and
 * unchanged until the call that uses the prepared work has been queued (or the device synchronised). */
int w2v_cbow_prefetch_minibatch(w2v_shard* shard, const uint32_t* ctx_off_dev,
                                const uint32_t* ctx_idx_dev, uint32_t m, const uint32_t* out_idx_dev,
                                uint32_t n, uint32_t k, uint64_t seed, void* stream);

/* Examples from text: the same subsampling and window draws as w2v_make_pairs.  Every surviving
 * center with at least one surviving neighbour inside its window gives one example; its contexts are
 * those neighbours by increasing position (the pair stream's output words, grouped by center).
 * Writes at most cap_examples centers (out_idx_dev) with their offsets (ctx_off_dev, cap_examples+1
 * entries, always starting with 0) and at most cap_ctx context words; *n_examples_host and
 * *n_ctx_host receive the full counts.  Synchronises the stream, like w2v_make_pairs. */
int w2v_make_cbow_examples(w2v_shard* shard, const uint32_t* tokens_dev, const uint64_t* sent_off_dev,
                           uint32_t n_sent, uint32_t n_tokens, uint64_t token_base, uint32_t epoch,
                           uint64_t corpus_seed, uint32_t B, uint32_t* ctx_off_dev,
                           uint32_t* ctx_idx_dev, uint32_t* out_idx_dev, uint64_t cap_examples,
                           uint64_t cap_ctx, uint64_t* n_examples_host, uint64_t* n_ctx_host,
                           void* stream);

/* ---- vector export (Section 6.1.4) ------------------------------------------------------------------
 * Joins the partial vectors of the column shards into whole vectors: dst_dev[i][0..d_total) is row
 * rows_dev[i] of matrix `which` (0 = input vectors, 1 = output vectors), shard s contributing columns
 * [col_begin_s, col_begin_s + d_slice_s).  The shards must agree in V and d_total and their column
 * ranges must tile [0, d_total) exactly (W2V_ERR_MISMATCH otherwise); any order.  dst_dev is a dense
 * [m][d_total] device array owned by the caller.  A row >= V raises the sticky index flag of the shard
 * and yields row 0. */
int w2v_export_rows(w2v_shard* const* shards, uint32_t S, int which, const uint32_t* rows_dev,
                    uint32_t m, float* dst_dev, void* stream);

/* ---- retrieval by cosine similarity (Section 2; Section 7.3: K = 30, threshold 0.65) ----------------
 * For each of the Q query vectors (queries_dev, dense [Q][d]) the K candidates (cands_dev, dense
 * [N][d]) with the highest cosine similarity (q.c)/(|q||c|), ranked by decreasing similarity, equal
 * similarities by increasing index; an all-zero vector has similarity 0 with everything.  Only
 * similarities strictly above tau are returned (pass tau <= -2 for no threshold):
 * out_idx_dev[q][0..count) / out_score_dev[q][0..count) hold them, the remaining slots of the K hold
 * 0xFFFFFFFF / 0, and out_count_dev[q] (may be NULL) the count.  fp32 throughout; 1 <= K <=
 * W2V_TOPK_MAX.
 *
 * The call allocates nothing: workspace_dev (256-byte aligned device memory, contents irrelevant
 * before and after) holds the norms, the running best lists and, per query, room for one round of
 * candidates.  w2v_topk_cosine_workspace(Q, N, r) is the size for rounds of r candidates (r = 0 or
 * r >= N: a single round); a smaller workspace means more, shorter rounds (the minimum is r = 128),
 * never a different result.  All work is queued on the stream; nothing is synchronised. */
#define W2V_TOPK_MAX 64
size_t w2v_topk_cosine_workspace(uint32_t Q, uint32_t N, uint32_t round_candidates);
int w2v_topk_cosine(const float* queries_dev, uint32_t Q, const float* cands_dev, uint32_t N,
                    uint32_t d, uint32_t K, float tau, uint32_t* out_idx_dev, float* out_score_dev,
                    uint32_t* out_count_dev, void* workspace_dev, size_t workspace_bytes,
                    void* stream);

/* Seed of minibatch number h (the client picks a fresh seed per minibatch), a function of a master seed. */
uint64_t w2v_minibatch_seed(uint64_t master_seed, uint64_t h);

/* ---- per-phase GPU timing ------------------------------------------------------------------------
 * When enabled, the library brackets each phase it queues with HIP events on the caller's stream.
 * w2v_shard_timing_read synchronises, adds the elapsed times into ms_host[W2V_PHASES] and the launch
 * counts into launches_host[W2V_PHASES], and resets the accumulators.  Phase order: */
#define W2V_PH_NEG     0   /* negatives + destination keys */
#define W2V_PH_DOT     1   /* gather dot products */
#define W2V_PH_COEFF   2   /* aggregation + coefficients */
#define W2V_PH_SORT    3   /* radix sorts of destination keys */
#define W2V_PH_USIDE   4   /* input-vector changes (and, fused, dots + coefficients) */
#define W2V_PH_WSIDE   5   /* output-vector changes, applied in place */
#define W2V_PH_APPLY   6   /* write-back of the input-vector changes and multi-level tails */
#define W2V_PH_PAIRS   7   /* pair formation */
#define W2V_PHASES     8
int w2v_shard_timing_enable(w2v_shard* shard, int on);
int w2v_shard_timing_read(w2v_shard* shard, double* ms_host, uint64_t* launches_host);

#ifdef __cplusplus
}
#endif
#endif
