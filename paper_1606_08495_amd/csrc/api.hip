// C ABI of the shard library: argument checks, scratch planning and the order in which the
// kernels of dotprod / adjust / train_minibatch are queued.  See include/w2v_shard.h for the
// contract of every entry point.
#include "../../include/w2v_shard.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "common.h"

namespace w2v {
bool build_noise_table_host(const uint64_t* counts, uint32_t V, uint32_t* thresh, uint32_t* alias);
void build_keep_thresholds_host(const uint64_t* counts, uint32_t V, double t, uint64_t* keep);
}  // namespace w2v

using namespace w2v;

// ---------------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------------
static thread_local std::string g_last_error;

static int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

#define HIP_TRY(expr)                                                                   \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess)                                                           \
            return fail(e_ == hipErrorOutOfMemory ? W2V_ERR_ALLOC : W2V_ERR_HIP,        \
                        "%s failed: %s", #expr, hipGetErrorString(e_));                 \
    } while (0)

extern "C" const char* w2v_last_error(void) { return g_last_error.c_str(); }

// ---------------------------------------------------------------------------------------------
// Scratch of w2v_dotprod_noalloc: one array per GPU, part of the loaded code object, so the entry
// point never allocates.  In host code the array's name is only a handle for hipGetSymbolAddress;
// the device address it yields (one per device) is what kernels and copies are given.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) uint32_t scratch[W2V_NOALLOC_SCRATCH_U32];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
uint32_t* g_scratch_ptr[MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the CURRENT device (which must be `device`), resolved once.
int static_scratch(int device, uint32_t** out) {
    if (device < 0 || device >= MAX_DEVICES)
        return -1;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) { (void)hipGetLastError(); return -1; }
        g_scratch_ptr[device] = (uint32_t*)ptr;
    }
    *out = g_scratch_ptr[device];
    return 0;
}
}  // namespace

// ---------------------------------------------------------------------------------------------
// shard object
// ---------------------------------------------------------------------------------------------
struct TimedSpan { int phase; hipEvent_t a, b; };

// Index work of one minibatch computed ahead of its training call (w2v_prefetch_minibatch): the
// checked input words and their sort, the destination keys and their sort.  Two sets alternate, so
// that the one a running step reads is never the one being filled.
struct IndexSet {
    char* base = nullptr; size_t cap = 0;
    uint32_t *keys = nullptr, *in_safe = nullptr;
    uint2 *ub0 = nullptr, *ub1 = nullptr;       // sort buffers, input side (n)
    uint2 *wb0 = nullptr, *wb1 = nullptr;       // sort buffers, output side (M)
    uint32_t *sort_tmp = nullptr;               // of the joint sort of both sides
    uint32_t *sku = nullptr, *perm = nullptr, *skw = nullptr, *sidx = nullptr;   // sorted results
    hipEvent_t ready = nullptr;
};

struct Prepared {
    bool valid = false; int set = 0; bool own_rows = false;
    uint64_t born = 0;              // value of the shard's update counter at the announcement
    const uint32_t* in_idx = nullptr; const uint32_t* out_idx = nullptr;
    uint32_t n = 0, k = 0; uint64_t seed = 0;
};

// The same for a bag-of-words minibatch (w2v_cbow_prefetch_minibatch): the checked context entries
// with their example numbers and weights, the destination keys, and both sorts.
struct CbowSet {
    char* base = nullptr; size_t cap = 0;
    uint32_t *keys = nullptr, *ctx_safe = nullptr, *ex_of = nullptr, *iota = nullptr;
    float* weight = nullptr;
    uint2 *wb0 = nullptr, *wb1 = nullptr;       // sort buffers of the M destinations
    uint2 *cb0 = nullptr, *cb1 = nullptr;       // sort buffers of the m context entries
    uint32_t *sort_tmp = nullptr;               // of the joint sort of both
    uint32_t *skw = nullptr, *sidx = nullptr, *skc = nullptr, *cidx = nullptr;   // sorted results
    hipEvent_t ready = nullptr;
};

struct CbowPrepared {
    bool valid = false; bool own_rows = false;
    uint64_t born = 0;
    const uint32_t* ctx_off = nullptr; const uint32_t* ctx_idx = nullptr; const uint32_t* out_idx = nullptr;
    uint32_t n = 0, k = 0, m = 0; uint64_t seed = 0;
};

struct w2v_shard {
    int device = 0;
    uint32_t V = 0, d_total = 0, col_begin = 0, d_slice = 0;
    uint64_t seed = 0;
    int init_mode = 0;
    RowGeom g{0, 0};
    float* U = nullptr;
    float* W = nullptr;
    uint2* bins = nullptr;          // noise table
    uint64_t* keep = nullptr;       // subsample thresholds (nullptr: keep everything)
    bool has_tables = false;
    uint64_t table_tag = 0;         // checksum of the noise table, to compare shards
    uint32_t* err = nullptr;        // sticky device flag
    uint32_t* static_ws = nullptr;  // this device's copy of the no-allocation scratch array
    uint64_t updates = 0;           // update calls seen (adjust / train_minibatch, either variant)
    IndexPrologue* prologue_sink = nullptr;  // set while a step is captured: the first launch of the
                                             // step is not queued but handed back (it takes the
                                             // caller's arrays, which change from call to call)
    const CallScalars* call_dev = nullptr;   // set while a step is captured into a graph: the
                                    // kernels then read seed and learning rate from device memory
    // scratch: one region, carved per call
    char* ws = nullptr;
    size_t ws_cap = 0;
    // scratch of the pair formation, apart from the training calls' so that the two may overlap
    char* pairs_ws = nullptr;
    size_t pairs_ws_cap = 0;
    // second stream: the part of a call that can run beside its main kernels (key generation and
    // output-side sort; loss, the input side's higher levels, the write-back of the delta buffer),
    // forked from the caller's stream and joined back into it by events
    hipStream_t side = nullptr;
    // third stream: the index work of announced minibatches (w2v_prefetch_minibatch), apart from
    // `side` so that the current step's own second-stream work does not queue up behind it
    hipStream_t ahead = nullptr;
    hipEvent_t ev_fork = nullptr, ev_keys = nullptr, ev_join = nullptr;
    hipEvent_t ev_coeffs = nullptr, ev_wdone = nullptr, ev_tails = nullptr;
    bool overlap = true;
    bool own_rows = true;           // fused step: singly named output rows updated by the input side
    bool last_update_fused = true;  // what the last update on this shard was: an announced minibatch
                                    // gets its rows-named-once marks only if the fused step is likely
    static constexpr int N_SETS = 3;   // two announced minibatches besides the one in use
    IndexSet sets[N_SETS];
    Prepared prep[N_SETS];          // what sets[i] holds
    CbowSet csets[2];
    CbowPrepared cprep[2];
    int next_cset = 0;
    hipEvent_t ev_pfork = nullptr;
    // timing
    bool timing = false;
    std::vector<TimedSpan> spans;
    std::vector<hipEvent_t> pool;
    double ms[W2V_PHASES] = {0};
    uint64_t launches[W2V_PHASES] = {0};
};

namespace {

struct Carver {
    char* base; size_t off = 0;
    explicit Carver(char* b) : base(b) {}
    template <typename T> T* take(size_t count) {
        off = (off + 255) & ~(size_t)255;
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

// Grow a scratch region to at least `bytes` (it is never shrunk; growing waits for the device).
int ensure_region(char*& region, size_t& cap, size_t bytes) {
    if (bytes <= cap) return W2V_OK;
    if (region) { HIP_TRY(hipDeviceSynchronize()); HIP_TRY(hipFree(region)); region = nullptr; cap = 0; }
    size_t want = bytes + bytes / 8 + 4096;
    hipError_t e = hipMalloc((void**)&region, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        want = bytes;
        e = hipMalloc((void**)&region, want);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(W2V_ERR_ALLOC, "scratch allocation of %zu bytes failed: %s", want,
                    hipGetErrorString(e));
    }
    cap = want;
    return W2V_OK;
}

int ensure_ws(w2v_shard* sh, size_t bytes) { return ensure_region(sh->ws, sh->ws_cap, bytes); }

struct Phase {
    w2v_shard* sh; int phase; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
    Phase(w2v_shard* s, int ph, hipStream_t stream) : sh(s), phase(ph), st(stream) {
        if (!sh->timing) return;
        a = grab(); b = grab();
        if (a && b) (void)hipEventRecord(a, st);
    }
    ~Phase() {
        if (!sh->timing || !a || !b) return;
        (void)hipEventRecord(b, st);
        sh->spans.push_back(TimedSpan{phase, a, b});
    }
    hipEvent_t grab() {
        if (!sh->pool.empty()) { hipEvent_t e = sh->pool.back(); sh->pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

int check_device(const w2v_shard* sh) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != sh->device)
        return fail(W2V_ERR_MISMATCH, "shard lives on device %d but device %d is current",
                    sh->device, dev);
    return W2V_OK;
}

int check_batch(const w2v_shard* sh, uint32_t n, uint32_t k, bool needs_tables) {
    if (k > W2V_K_MAX) return fail(W2V_ERR_ARG, "k = %u exceeds W2V_K_MAX = %d", k, W2V_K_MAX);
    if ((uint64_t)n * (k + 1) >= (1ull << 31))
        return fail(W2V_ERR_ARG, "n*(k+1) = %llu must stay below 2^31",
                    (unsigned long long)((uint64_t)n * (k + 1)));
    if (k > 0 && sh->V < 2) return fail(W2V_ERR_ARG, "negatives need a vocabulary of at least 2 words");
    if (needs_tables && k > 0 && !sh->has_tables)
        return fail(W2V_ERR_STATE, "w2v_shard_set_counts has not been called on this shard");
    return W2V_OK;
}

uint32_t key_bits(uint32_t V) {
    uint32_t bits = 1;
    while (bits < 32 && (1ull << bits) < (uint64_t)V) ++bits;
    return bits;
}

uint32_t slots_after(uint32_t entries, uint32_t per_chunk) {
    if (entries == 0) return 0;
    uint32_t chunks = (entries + per_chunk - 1) / per_chunk;
    return 2 * (chunks - 1);
}

// Everything one minibatch needs in scratch, carved in a fixed order.
struct Plan {
    uint32_t n, T, M;
    uint32_t* keys; uint32_t* in_safe;
    bool own_rows;                         // fused step: singly named output rows go to the input side
    uint2 *ub0, *ub1;                      // sort buffers, input side (n)
    uint2 *wb0, *wb1;                      // sort buffers, output side (M)
    uint32_t* sort_tmp; uint32_t* sort_tmp_u;
    float* coeffs; float* dots; double* loss_tmp;
    float* delta; uint32_t* dkey;
    float* pa_rows; uint32_t* pa_keys;     // input side, level 1 slots
    float* pb_rows; uint32_t* pb_keys;     // output side, level 1 slots
    float* pc_rows; uint32_t* pc_keys;     // level 2 slots, output side
    float* pe_rows; uint32_t* pe_keys;     // level 2 slots, input side (the two sides' tails may overlap)
    uint32_t slots_u1, slots_w1, slots_2;
    bool wfill_done;                       // the output side's border slots are cleared already
    size_t bytes;
};

Plan make_plan(char* base, uint32_t n, uint32_t k, uint32_t stride4_max, uint32_t S_dots,
               bool want_adjust, bool want_coeffs, uint32_t V_own_rows = 0) {
    Plan p{};
    p.n = n; p.T = k + 1; p.M = n * p.T;
    Carver c(base);
    p.keys = c.take<uint32_t>(p.M);
    p.in_safe = c.take<uint32_t>(n);
    p.own_rows = V_own_rows != 0;
    if (want_coeffs) p.coeffs = c.take<float>(p.M);
    if (S_dots) p.dots = c.take<float>((size_t)S_dots * p.M);
    p.loss_tmp = c.take<double>(coeffs_loss_scratch_doubles(n, p.T));
    if (want_adjust) {
        p.ub0 = c.take<uint2>(n); p.ub1 = c.take<uint2>(n);
        p.wb0 = c.take<uint2>(p.M); p.wb1 = c.take<uint2>(p.M);
        p.sort_tmp = c.take<uint32_t>(sort_scratch_u32(p.M, n));     // (room for the joint sort)
        p.sort_tmp_u = c.take<uint32_t>(sort_scratch_u32(n));
        const size_t row = (size_t)stride4_max * 4;
        p.delta = c.take<float>((size_t)n * row);
        p.dkey = c.take<uint32_t>(n);
        p.slots_u1 = slots_after(n, useg_pairs_per_chunk(p.T, 1, n));    // the most any shard needs
        p.slots_w1 = slots_after(p.M, wseg_entries_per_chunk());
        uint32_t s2u = slots_after(p.slots_u1, tail_entries_per_chunk());
        uint32_t s2w = slots_after(p.slots_w1, tail_entries_per_chunk());
        p.slots_2 = std::max(s2u, s2w);
        p.pa_rows = c.take<float>((size_t)p.slots_u1 * row); p.pa_keys = c.take<uint32_t>(p.slots_u1 + 1);
        p.pb_rows = c.take<float>((size_t)p.slots_w1 * row); p.pb_keys = c.take<uint32_t>(p.slots_w1 + 1);
        p.pc_rows = c.take<float>((size_t)p.slots_2 * row);  p.pc_keys = c.take<uint32_t>(p.slots_2 + 1);
        p.pe_rows = c.take<float>((size_t)p.slots_2 * row);  p.pe_keys = c.take<uint32_t>(p.slots_2 + 1);
    }
    p.bytes = c.off + 256;
    return p;
}

// Reduce the partial slots of one side level by level into matrix M (in place) -- or, for the
// input side of the skip-gram step (defer_rows given), into the delta buffer, so that these passes
// need not wait for the output side to finish reading M.
void run_tails(w2v_shard* sh, float* M, float alpha, float* rows_a, uint32_t* keys_a, uint32_t slots,
               float* rows_b, uint32_t* keys_b, hipStream_t st, float* defer_rows = nullptr,
               uint32_t* defer_keys = nullptr, uint32_t cp = 0, const CallScalars* dev = nullptr) {
    float* src_rows = rows_a; uint32_t* src_keys = keys_a;
    float* dst_rows = rows_b; uint32_t* dst_keys = keys_b;
    uint32_t level = 0;
    while (slots > 0) {
        TailArgs t{M, sh->g, alpha, src_rows, src_keys, slots, dst_rows, dst_keys};
        t.defer_rows = defer_rows; t.defer_keys = defer_keys; t.level = ++level; t.cp = cp; t.dev = dev;
        launch_tail(t, st);
        slots = slots_after(slots, tail_entries_per_chunk());
        std::swap(src_rows, dst_rows);
        std::swap(src_keys, dst_keys);
    }
}

int ensure_side_stream(w2v_shard* sh) {
    if (sh->side) return W2V_OK;
    HIP_TRY(hipStreamCreateWithFlags(&sh->side, hipStreamNonBlocking));
    HIP_TRY(hipStreamCreateWithFlags(&sh->ahead, hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&sh->ev_fork, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&sh->ev_keys, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&sh->ev_join, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&sh->ev_coeffs, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&sh->ev_wdone, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&sh->ev_tails, hipEventDisableTiming));
    return W2V_OK;
}

// Buffers of one prefetched minibatch, carved from the set's own allocation (grown on demand).
int ensure_set(w2v_shard* sh, IndexSet& x, uint32_t n, uint32_t M) {
    for (int pass = 0; pass < 2; ++pass) {
        Carver c(pass ? x.base : nullptr);
        uint32_t* keys = c.take<uint32_t>(M);
        uint32_t* in_safe = c.take<uint32_t>(n);
        uint2* ub0 = c.take<uint2>(n); uint2* ub1 = c.take<uint2>(n);
        uint2* wb0 = c.take<uint2>(M); uint2* wb1 = c.take<uint2>(M);
        uint32_t* tw = c.take<uint32_t>(sort_scratch_u32(M, n));
        const size_t need = c.off + 256;
        if (pass == 0) {
            if (need > x.cap) {
                if (x.base) { HIP_TRY(hipDeviceSynchronize()); HIP_TRY(hipFree(x.base)); x.base = nullptr; x.cap = 0; }
                hipError_t e = hipMalloc((void**)&x.base, need);
                if (e != hipSuccess) {
                    (void)hipGetLastError();
                    return fail(W2V_ERR_ALLOC, "allocation of %zu bytes for a prefetched minibatch failed: %s",
                                need, hipGetErrorString(e));
                }
                x.cap = need;
            }
        } else {
            x.keys = keys; x.in_safe = in_safe; x.ub0 = ub0; x.ub1 = ub1;
            x.wb0 = wb0; x.wb1 = wb1; x.sort_tmp = tw;
        }
    }
    if (!x.ready) HIP_TRY(hipEventCreateWithFlags(&x.ready, hipEventDisableTiming));
    if (!sh->ev_pfork) HIP_TRY(hipEventCreateWithFlags(&sh->ev_pfork, hipEventDisableTiming));
    return W2V_OK;
}

// Everything adjust needs before its first row kernel: the checked input words, the destination
// keys (positive word + regenerated negatives) and both sorts.
// The input-side kernel needs the keys and the (small) input-side sort; the output-side sort is only
// needed later.  So the key generation and the output-side sort are queued on the shard's second
// stream, forked from the caller's stream by an event, while the caller's stream checks the inputs
// and sorts the input side; the caller's stream then waits for the keys (ev_keys) and, just before
// the first kernel that reads the output-side order, for that sort (join_output_sort).
int queue_keys_and_sorts(w2v_shard* sh, Plan& p, const uint32_t* in_idx, const uint32_t* out_idx,
                         uint32_t k, uint64_t seed, uint32_t** sku, uint32_t** perm, uint32_t** skw,
                         uint32_t** sidx, hipStream_t st) {
    const uint32_t bits = key_bits(sh->V);

    const NoiseTable nt{sh->bins, sh->V};
    if (!sh->overlap) {
        // one stream: keys, checked inputs and both fills in one launch, then the two sides' keys
        // through the same sort launches
        const SortJob jobs[2] = {{p.keys, p.M, p.wb0, p.wb1, skw, sidx},
                                 {p.in_safe, p.n, p.ub0, p.ub1, sku, perm}};
        {
            Phase ph(sh, W2V_PH_NEG, st);
            IndexPrologue pro{};
            pro.nt = nt; pro.out_idx = out_idx; pro.n = p.n; pro.T = p.T;
            pro.seed_lo = (uint32_t)seed; pro.seed_hi = (uint32_t)(seed >> 32);
            pro.keys = p.keys; pro.dev = sh->call_dev; pro.in_idx = in_idx; pro.in_safe = p.in_safe;
            pro.err = sh->err;
            pro.fill[0] = sort_clear_job(jobs, 2, p.sort_tmp);
            pro.fill[1] = wseg_fill_job(p.pb_keys, p.M);
            p.wfill_done = true;
            if (sh->prologue_sink) *sh->prologue_sink = pro;
            else launch_index_prologue(pro, st);
        }
        Phase ph(sh, W2V_PH_SORT, st);
        launch_sort_jobs(jobs, 2, bits, p.sort_tmp, sh->err, st, true);
        if (p.own_rows) launch_mark_alone(*skw, *sidx, p.M, p.keys, st);
        return W2V_OK;
    }
    hipStream_t wst = st;
    if (sh->overlap) {
        int rc = ensure_side_stream(sh);
        if (rc) return rc;
        HIP_TRY(hipEventRecord(sh->ev_fork, st));
        HIP_TRY(hipStreamWaitEvent(sh->side, sh->ev_fork, 0));
        wst = sh->side;
    }
    {
        Phase ph(sh, W2V_PH_NEG, wst);
        launch_dest_keys(nt, out_idx, p.n, k, seed, p.keys, sh->err, wst, sh->call_dev);
    }
    if (sh->overlap) HIP_TRY(hipEventRecord(sh->ev_keys, sh->side));
    {
        Phase ph(sh, W2V_PH_SORT, wst);
        launch_sort_pairs(p.keys, p.wb0, p.wb1, p.M, bits, p.sort_tmp, skw, sidx, sh->err, wst);
        // fused single-shard step: output rows named by one slot only are updated by the
        // input-side kernel (which then has to wait for this sort) and skipped by the output side
        if (p.own_rows) launch_mark_alone(*skw, *sidx, p.M, p.keys, wst);
    }
    if (sh->overlap) HIP_TRY(hipEventRecord(sh->ev_join, sh->side));
    {
        Phase ph(sh, W2V_PH_SORT, st);
        launch_check_inputs(in_idx, p.n, sh->V, p.in_safe, sh->err, st);
        launch_sort_pairs(p.in_safe, p.ub0, p.ub1, p.n, bits, p.sort_tmp_u, sku, perm, sh->err, st);
    }
    if (sh->overlap) HIP_TRY(hipStreamWaitEvent(st, p.own_rows ? sh->ev_join : sh->ev_keys, 0));
    return W2V_OK;
}

// The index work of a minibatch announced by w2v_prefetch_minibatch, queued on the second stream
// behind everything queued on `st` so far.
int run_prefetch_chain(w2v_shard* sh, const Prepared& want, hipStream_t st) {
    // a set that holds no live announcement (its last user was queued on `st` before this call, and
    // the chain waits for `st`), else the one announced longest ago
    int which = 0;
    for (int i = 0; i < w2v_shard::N_SETS; ++i) {
        if (!sh->prep[i].valid) { which = i; break; }
        if (sh->prep[i].born < sh->prep[which].born) which = i;
    }
    IndexSet& x = sh->sets[which];
    sh->prep[which].valid = false;
    const uint32_t n = want.n, k = want.k, M = n * (k + 1);
    int rc = ensure_set(sh, x, n, M);
    if (rc) return rc;
    HIP_TRY(hipEventRecord(sh->ev_pfork, st));
    HIP_TRY(hipStreamWaitEvent(sh->ahead, sh->ev_pfork, 0));
    hipStream_t side = sh->ahead;
    const uint32_t bits = key_bits(sh->V);
    const bool marks = sh->own_rows && sh->last_update_fused;
    // both sides' keys in the same launches: the small input-side sort rides along
    const SortJob jobs[2] = {{x.keys, M, x.wb0, x.wb1, &x.skw, &x.sidx},
                             {x.in_safe, n, x.ub0, x.ub1, &x.sku, &x.perm}};
    {
        Phase ph(sh, W2V_PH_NEG, side);
        IndexPrologue pro{};
        pro.nt = NoiseTable{sh->bins, sh->V}; pro.out_idx = want.out_idx; pro.n = n; pro.T = k + 1;
        pro.seed_lo = (uint32_t)want.seed; pro.seed_hi = (uint32_t)(want.seed >> 32);
        pro.keys = x.keys; pro.in_idx = want.in_idx; pro.in_safe = x.in_safe; pro.err = sh->err;
        pro.fill[0] = sort_clear_job(jobs, 2, x.sort_tmp);
        launch_index_prologue(pro, side);
    }
    {
        Phase ph(sh, W2V_PH_SORT, side);
        launch_sort_jobs(jobs, 2, bits, x.sort_tmp, sh->err, side, true);
        if (marks) launch_mark_alone(x.skw, x.sidx, M, x.keys, side);
    }
    HIP_TRY(hipEventRecord(x.ready, side));
    HIP_TRY(hipGetLastError());
    Prepared& pr = sh->prep[which];
    pr = want;
    pr.valid = true; pr.set = which; pr.own_rows = marks; pr.born = sh->updates;
    return W2V_OK;
}

// The set that w2v_prefetch_minibatch filled for exactly this minibatch, or -1.
// An announcement is good for the next PREP_MAX_AGE update calls on the shard (a loop may announce
// two minibatches ahead of the one it trains); an older one is void, so that a forgotten set cannot be matched much later by
// arrays that happen to live at the same addresses.
constexpr uint64_t PREP_MAX_AGE = 3;

int find_prepared(w2v_shard* sh, const uint32_t* in_idx, const uint32_t* out_idx, uint32_t n,
                  uint32_t k, uint64_t seed) {
    for (int i = 0; i < w2v_shard::N_SETS; ++i) {
        Prepared& pr = sh->prep[i];
        if (pr.valid && sh->updates - pr.born >= PREP_MAX_AGE) pr.valid = false;
        if (pr.valid && pr.in_idx == in_idx && pr.out_idx == out_idx && pr.n == n && pr.k == k &&
            pr.seed == seed)
            return i;
    }
    return -1;
}

void join_output_sort(w2v_shard* sh, hipStream_t st) {
    if (sh->overlap && sh->side) (void)hipStreamWaitEvent(st, sh->ev_join, 0);
}

// First part of a shard's update, the same on one stream or several: the output-side kernel's border
// slots are cleared here, ahead of the input-side kernel, so that the two row kernels follow each
// other with nothing in between (unless the call's first launch has cleared them already: good for
// one shard's update); then the input-side kernel.
void queue_input_side(w2v_shard* ws_owner, w2v_shard* sh, Plan& p, const uint32_t* sku,
                      const uint32_t* perm, const float* coeffs_in, float* coeffs_out, bool fused,
                      float alpha, bool keep_dots, hipStream_t st) {
    if (p.wfill_done) p.wfill_done = false;
    else launch_wseg_fill(p.pb_keys, p.M, st);
    Phase ph(ws_owner, W2V_PH_USIDE, st);
    USideArgs a{};
    a.U = sh->U; a.W = sh->W; a.g = sh->g; a.skey = sku; a.perm = perm; a.keys = p.keys;
    a.n = p.n; a.T = p.T; a.coeffs_in = coeffs_in; a.coeffs_out = coeffs_out;
    a.dots_out = (fused && keep_dots) ? p.dots : nullptr; a.delta = p.delta; a.dkey = p.dkey;
    a.prows = p.pa_rows; a.pkeys = p.pa_keys; a.fused = fused;
    if (p.own_rows) { a.W_update = sh->W; a.alpha = alpha; }
    a.dev = ws_owner->call_dev;
    launch_useg(a, st);
}

// The same update on ONE stream (a captured step, or a shard told not to use its second stream),
// for the row geometries that have the joint launch: after the input-side kernel, each launch
// carries one walk of the output side together with one higher level of the input side and one
// step of the loss, which depend on different things; the delta buffer is written back last.
// Same kernels' code on the same data as queue_adjust below: the same bits.
void queue_adjust_one_stream(w2v_shard* ws_owner, w2v_shard* sh, Plan& p, const uint32_t* sku,
                             const uint32_t* perm, const uint32_t* skw, const uint32_t* sidx,
                             const float* coeffs_in, float* coeffs_out, bool fused, float alpha,
                             double* loss_out, hipStream_t st) {
    queue_input_side(ws_owner, sh, p, sku, perm, coeffs_in, coeffs_out, fused, alpha, loss_out != nullptr, st);
    const uint32_t cp = useg_pairs_per_chunk(p.T, sh->g.d4, p.n);
    struct Side { float* src_rows; uint32_t* src_keys; float* dst_rows; uint32_t* dst_keys; uint32_t slots, level; };
    Side us{p.pa_rows, p.pa_keys, p.pe_rows, p.pe_keys, slots_after(p.n, cp), 0u};
    Side ws{p.pb_rows, p.pb_keys, p.pc_rows, p.pc_keys, p.slots_w1, 0u};
    uint32_t loss_step = (loss_out && fused) ? 1u : 0u;
    if (loss_step && (uint64_t)p.n * p.T > 256ull * adjust_stage_loss_blocks_max()) {
        Phase ph(ws_owner, W2V_PH_COEFF, st);                 // too many terms for one final block
        launch_loss_from_dots(p.dots, p.n, p.T, p.loss_tmp, loss_out, st);
        loss_step = 0;
    }
    auto advance = [](Side& x) {
        x.slots = slots_after(x.slots, tail_entries_per_chunk());
        std::swap(x.src_rows, x.dst_rows);
        std::swap(x.src_keys, x.dst_keys);
    };
    for (bool first = true; first || us.slots || ws.slots || loss_step; first = false) {
        Phase ph(ws_owner, first ? W2V_PH_WSIDE : W2V_PH_APPLY, st);
        AdjustStage x;
        WSideArgs w{};
        TailArgs wt{}, ut{};
        const bool w_level = !first && ws.slots > 0, u_level = us.slots > 0;
        if (first) {
            w.U = sh->U; w.W = sh->W; w.g = sh->g; w.skey = skw; w.sidx = sidx; w.M = p.M; w.T = p.T;
            w.in_idx = p.in_safe; w.coeffs = fused ? coeffs_out : coeffs_in; w.alpha = alpha;
            w.prows = p.pb_rows; w.pkeys = p.pb_keys; w.skip_alone = p.own_rows;
            w.dev = ws_owner->call_dev;
            x.wfirst = &w;
        } else if (w_level) {
            wt = TailArgs{sh->W, sh->g, alpha, ws.src_rows, ws.src_keys, ws.slots, ws.dst_rows, ws.dst_keys};
            wt.level = ++ws.level; wt.dev = ws_owner->call_dev;
            x.wtail = &wt;
        }
        if (u_level) {
            ut = TailArgs{sh->U, sh->g, alpha, us.src_rows, us.src_keys, us.slots, us.dst_rows, us.dst_keys};
            ut.defer_rows = p.delta; ut.defer_keys = p.dkey; ut.level = ++us.level; ut.cp = cp;
            ut.dev = ws_owner->call_dev;
            x.utail = &ut;
        }
        if (loss_step) {
            x.loss_step = loss_step; x.dots = p.dots; x.n = p.n; x.T = p.T;
            x.loss_tmp = p.loss_tmp; x.loss_out = loss_out;
            loss_step = loss_step == 1 ? 2u : 0u;
        }
        launch_adjust_stage(x, st);
        if (w_level) advance(ws);
        if (u_level) advance(us);
    }
    {
        Phase ph(ws_owner, W2V_PH_APPLY, st);
        launch_apply_delta(sh->U, sh->g, p.delta, p.dkey, p.n, alpha, st, ws_owner->call_dev);
    }
}

// The update of one shard from given coefficients (or, fused, from its own dots).
// After the input-side kernel the coefficients and the input side's partial sums exist, so the
// minibatch loss (if asked for, fused form only) and the input side's higher reduction levels --
// which park their results in the delta buffer and leave the input matrix alone -- run on the
// second stream beside the output-side kernel.  After that kernel the output side's higher levels
// follow on the caller's stream while the second stream writes the delta buffer back; the
// caller's stream finally waits for the second one.
void queue_adjust(w2v_shard* ws_owner, w2v_shard* sh, Plan& p, const uint32_t* sku,
                  const uint32_t* perm, const uint32_t* skw, const uint32_t* sidx,
                  const float* coeffs_in, float* coeffs_out, bool fused, float alpha,
                  double* loss_out, hipStream_t st) {
    // (loss_out: fused form only; the dots it is formed from go to p.dots)
    const bool two = ws_owner->overlap && ws_owner->side;
    if (!two && adjust_stage_supported(sh->g.d4))
        return queue_adjust_one_stream(ws_owner, sh, p, sku, perm, skw, sidx, coeffs_in, coeffs_out, fused,
                                       alpha, loss_out, st);
    hipStream_t side = two ? ws_owner->side : st;
    queue_input_side(ws_owner, sh, p, sku, perm, coeffs_in, coeffs_out, fused, alpha, loss_out != nullptr, st);
    // The input side's higher levels only touch its slots and the delta buffer, and the loss only
    // reads the coefficients: both go to the second stream and run beside the output-side kernel.
    if (two) {
        (void)hipEventRecord(ws_owner->ev_coeffs, st);
        (void)hipStreamWaitEvent(side, ws_owner->ev_coeffs, 0);
    }
    if (loss_out && fused) {
        Phase ph(ws_owner, W2V_PH_COEFF, side);
        launch_loss_from_dots(p.dots, p.n, p.T, p.loss_tmp, loss_out, side);
    }
    {
        Phase ph(ws_owner, W2V_PH_APPLY, side);
        const uint32_t cp = useg_pairs_per_chunk(p.T, sh->g.d4, p.n);      // this shard's chunk size
        run_tails(sh, sh->U, alpha, p.pa_rows, p.pa_keys, slots_after(p.n, cp), p.pe_rows, p.pe_keys,
                  side, p.delta, p.dkey, cp, ws_owner->call_dev);
    }
    join_output_sort(ws_owner, st);
    {
        Phase ph(ws_owner, W2V_PH_WSIDE, st);
        WSideArgs w{};
        w.U = sh->U; w.W = sh->W; w.g = sh->g; w.skey = skw; w.sidx = sidx; w.M = p.M; w.T = p.T;
        w.in_idx = p.in_safe; w.coeffs = fused ? coeffs_out : coeffs_in; w.alpha = alpha;
        w.prows = p.pb_rows; w.pkeys = p.pb_keys;
        w.skip_alone = p.own_rows;
        w.dev = ws_owner->call_dev;
        launch_wseg(w, st, true);
    }
    // After the output-side kernel: its higher levels stay on the caller's stream (no wait in
    // between), the write-back of the delta buffer goes to the second stream, behind the input
    // side's levels there.
    if (two) {
        (void)hipEventRecord(ws_owner->ev_wdone, st);
        (void)hipStreamWaitEvent(side, ws_owner->ev_wdone, 0);
    }
    {
        Phase ph(ws_owner, W2V_PH_APPLY, side);
        launch_apply_delta(sh->U, sh->g, p.delta, p.dkey, p.n, alpha, side, ws_owner->call_dev);
    }
    if (two) (void)hipEventRecord(ws_owner->ev_tails, side);
    {
        Phase ph(ws_owner, W2V_PH_APPLY, st);
        run_tails(sh, sh->W, alpha, p.pb_rows, p.pb_keys, p.slots_w1, p.pc_rows, p.pc_keys, st, nullptr,
                  nullptr, 0, ws_owner->call_dev);
    }
    if (two) (void)hipStreamWaitEvent(st, ws_owner->ev_tails, 0);
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// life cycle
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_shard_create_ex(uint32_t V, uint32_t d_total, uint32_t col_begin,
                                   uint32_t d_slice, uint64_t seed, int init_mode,
                                   w2v_shard** out) {
    if (!out) return fail(W2V_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (V == 0 || V > 0x7FFFFFFFu) return fail(W2V_ERR_ARG, "V = %u outside 1..2^31-1", V);
    if (d_slice == 0 || d_slice > W2V_D_MAX)
        return fail(W2V_ERR_ARG, "d_slice = %u outside 1..%d", d_slice, W2V_D_MAX);
    if (d_total == 0 || (uint64_t)col_begin + d_slice > d_total)
        return fail(W2V_ERR_ARG, "columns [%u, %u) do not fit d_total = %u", col_begin,
                    col_begin + d_slice, d_total);
    if (init_mode != 0 && init_mode != 1) return fail(W2V_ERR_ARG, "init_mode must be 0 or 1");

    w2v_shard* sh = new (std::nothrow) w2v_shard();
    if (!sh) return fail(W2V_ERR_ALLOC, "host allocation failed");
    HIP_TRY(hipGetDevice(&sh->device));
    sh->V = V; sh->d_total = d_total; sh->col_begin = col_begin; sh->d_slice = d_slice;
    sh->seed = seed; sh->init_mode = init_mode;
    sh->g.d4 = (d_slice + 3) / 4;
    // Row stride.  A row that straddles 128-byte lines costs an extra line per gather (a 240-byte
    // row touches 2.75 lines on average, 2 when aligned; a 1200-byte row 10.25 against 10) and
    // its write-back leaves two lines partly written instead of one, so rows are padded to a
    // multiple of 128 bytes when that adds at most an eighth (d = 60: +20 % gather rate; d = 300:
    // the benchmark step 2.8 % shorter for 6.7 % more memory; d = 200: 2 % for 12 %).
    // W2V_ROW_ALIGN_FLOATS overrides the granularity (for experiments).
    uint32_t align4 = 1;                     // row stride granularity in float4
    {
        uint32_t padded = ((sh->g.d4 + 7) / 8) * 8;
        if ((padded - sh->g.d4) * 8 <= sh->g.d4) align4 = 8;
    }
    if (const char* env = getenv("W2V_ROW_ALIGN_FLOATS")) {
        long v = atol(env);
        if (v >= 4 && v <= 256 && (v % 4) == 0) align4 = (uint32_t)v / 4;
    }
    sh->g.stride4 = ((sh->g.d4 + align4 - 1) / align4) * align4;
    if (const char* env = getenv("W2V_NO_OVERLAP")) sh->overlap = (atoi(env) == 0);
    if (const char* env = getenv("W2V_NO_OWN_ROWS")) sh->own_rows = (atoi(env) == 0);

    size_t bytes = (size_t)V * sh->g.stride4 * 16;
    hipError_t e = hipMalloc((void**)&sh->U, bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&sh->W, bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&sh->err, 256);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        int rc = fail(W2V_ERR_ALLOC, "allocating 2 x %zu bytes of vectors failed: %s", bytes,
                      hipGetErrorString(e));
        if (sh->U) (void)hipFree(sh->U);
        if (sh->W) (void)hipFree(sh->W);
        if (sh->err) (void)hipFree(sh->err);
        delete sh;
        return rc;
    }
    if (static_scratch(sh->device, &sh->static_ws) != 0) {
        int rc = fail(W2V_ERR_HIP, "hipGetSymbolAddress of the static scratch array failed on device %d",
                      sh->device);
        (void)hipFree(sh->U); (void)hipFree(sh->W); (void)hipFree(sh->err);
        delete sh;
        return rc;
    }
    launch_init(sh->U, V, sh->g, d_slice, d_total, col_begin, seed, 0, false, nullptr);
    launch_init(sh->W, V, sh->g, d_slice, d_total, col_begin, seed, 1, init_mode == 0, nullptr);
    hipError_t le = hipGetLastError();
    if (le == hipSuccess) le = hipMemset(sh->err, 0, 256);
    hipError_t se = hipDeviceSynchronize();
    if (le != hipSuccess || se != hipSuccess) {
        int rc = fail(W2V_ERR_HIP, "initialisation kernels failed: %s",
                      hipGetErrorString(le != hipSuccess ? le : se));
        (void)hipFree(sh->U); (void)hipFree(sh->W); (void)hipFree(sh->err);
        delete sh;
        return rc;
    }
    *out = sh;
    return W2V_OK;
}

extern "C" int w2v_shard_create(uint32_t V, uint32_t d_slice, uint64_t seed, w2v_shard** out) {
    return w2v_shard_create_ex(V, d_slice, 0, d_slice, seed, 0, out);
}

extern "C" int w2v_shard_destroy(w2v_shard* sh) {
    if (!sh) return W2V_OK;
    (void)hipDeviceSynchronize();
    for (auto& s : sh->spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
    for (auto e : sh->pool) (void)hipEventDestroy(e);
    if (sh->U) (void)hipFree(sh->U);
    if (sh->W) (void)hipFree(sh->W);
    if (sh->bins) (void)hipFree(sh->bins);
    if (sh->keep) (void)hipFree(sh->keep);
    if (sh->err) (void)hipFree(sh->err);
    if (sh->ws) (void)hipFree(sh->ws);
    if (sh->pairs_ws) (void)hipFree(sh->pairs_ws);
    if (sh->ev_fork) (void)hipEventDestroy(sh->ev_fork);
    if (sh->ev_keys) (void)hipEventDestroy(sh->ev_keys);
    if (sh->ev_join) (void)hipEventDestroy(sh->ev_join);
    if (sh->ev_coeffs) (void)hipEventDestroy(sh->ev_coeffs);
    if (sh->ev_wdone) (void)hipEventDestroy(sh->ev_wdone);
    if (sh->ev_tails) (void)hipEventDestroy(sh->ev_tails);
    if (sh->ev_pfork) (void)hipEventDestroy(sh->ev_pfork);
    for (auto& x : sh->sets) {
        if (x.ready) (void)hipEventDestroy(x.ready);
        if (x.base) (void)hipFree(x.base);
    }
    for (auto& x : sh->csets) {
        if (x.ready) (void)hipEventDestroy(x.ready);
        if (x.base) (void)hipFree(x.base);
    }
    if (sh->side) (void)hipStreamDestroy(sh->side);
    if (sh->ahead) (void)hipStreamDestroy(sh->ahead);
    delete sh;
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// tables
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_shard_set_counts(w2v_shard* sh, const uint64_t* counts, double subsample_t) {
    if (!sh || !counts) return fail(W2V_ERR_NULL, "shard or counts is NULL");
    int rc = check_device(sh);
    if (rc) return rc;
    const uint32_t V = sh->V;
    std::vector<uint32_t> thresh, alias;
    std::vector<uint64_t> keep;
    std::vector<uint2> packed;
    try {
        thresh.resize(V); alias.resize(V); keep.resize(V); packed.resize(V);
    } catch (const std::bad_alloc&) {
        return fail(W2V_ERR_ALLOC, "host allocation for the tables failed");
    }
    if (!build_noise_table_host(counts, V, thresh.data(), alias.data()))
        return fail(W2V_ERR_ALLOC, "host allocation for the alias construction failed");
    build_keep_thresholds_host(counts, V, subsample_t, keep.data());
    uint64_t tag = 1469598103934665603ull;
    for (uint32_t w = 0; w < V; ++w) {
        packed[w] = make_uint2(thresh[w], alias[w]);
        tag = (tag ^ thresh[w]) * 1099511628211ull;
        tag = (tag ^ alias[w]) * 1099511628211ull;
    }
    HIP_TRY(hipDeviceSynchronize());
    if (!sh->bins) HIP_TRY(hipMalloc((void**)&sh->bins, sizeof(uint2) * (size_t)V));
    if (!sh->keep) HIP_TRY(hipMalloc((void**)&sh->keep, sizeof(uint64_t) * (size_t)V));
    HIP_TRY(hipMemcpy(sh->bins, packed.data(), sizeof(uint2) * (size_t)V, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(sh->keep, keep.data(), sizeof(uint64_t) * (size_t)V, hipMemcpyHostToDevice));
    sh->has_tables = true;
    sh->table_tag = tag;
    for (Prepared& pr : sh->prep) pr.valid = false;   // negatives drawn from the old table are void
    sh->cprep[0].valid = sh->cprep[1].valid = false;
    return W2V_OK;
}

extern "C" int w2v_shard_get_tables(w2v_shard* sh, uint32_t* thresh, uint32_t* alias,
                                    uint64_t* keep) {
    if (!sh) return fail(W2V_ERR_NULL, "shard is NULL");
    if (!sh->has_tables) return fail(W2V_ERR_STATE, "no tables set");
    int rc = check_device(sh);
    if (rc) return rc;
    const uint32_t V = sh->V;
    if (thresh || alias) {
        std::vector<uint2> packed(V);
        HIP_TRY(hipMemcpy(packed.data(), sh->bins, sizeof(uint2) * (size_t)V, hipMemcpyDeviceToHost));
        for (uint32_t w = 0; w < V; ++w) {
            if (thresh) thresh[w] = packed[w].x;
            if (alias) alias[w] = packed[w].y;
        }
    }
    if (keep) HIP_TRY(hipMemcpy(keep, sh->keep, sizeof(uint64_t) * (size_t)V, hipMemcpyDeviceToHost));
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// rows, status
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_shard_get_rows(w2v_shard* sh, int which, const uint32_t* rows, uint32_t m,
                                  float* dst, void* stream) {
    if (!sh || (m && (!rows || !dst))) return fail(W2V_ERR_NULL, "NULL argument");
    if (which != 0 && which != 1) return fail(W2V_ERR_ARG, "which must be 0 (U) or 1 (W)");
    int rc = check_device(sh);
    if (rc) return rc;
    launch_gather_rows(which ? sh->W : sh->U, sh->g, sh->d_slice, rows, m, sh->V, dst, sh->err,
                       (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_shard_set_rows(w2v_shard* sh, int which, const uint32_t* rows, uint32_t m,
                                  const float* src, void* stream) {
    if (!sh || (m && (!rows || !src))) return fail(W2V_ERR_NULL, "NULL argument");
    if (which != 0 && which != 1) return fail(W2V_ERR_ARG, "which must be 0 (U) or 1 (W)");
    int rc = check_device(sh);
    if (rc) return rc;
    launch_scatter_rows(which ? sh->W : sh->U, sh->g, sh->d_slice, rows, m, sh->V, src, sh->err,
                        (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_shard_status(w2v_shard* sh, void* stream) {
    if (!sh) return fail(W2V_ERR_NULL, "shard is NULL");
    int rc = check_device(sh);
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    // announced minibatches are checked on the shard's own streams, which join the caller's stream
    // only when the set is used: wait for them too, so that a bad index announced just now is seen
    if (sh->ahead) HIP_TRY(hipStreamSynchronize(sh->ahead));
    if (sh->side) HIP_TRY(hipStreamSynchronize(sh->side));
    uint32_t flag = 0;
    HIP_TRY(hipMemcpy(&flag, sh->err, sizeof(flag), hipMemcpyDeviceToHost));
    if (flag) {
        uint32_t zero = 0;
        HIP_TRY(hipMemcpy(sh->err, &zero, sizeof(zero), hipMemcpyHostToDevice));
        if (flag & 2u)
            return fail(W2V_ERR_HIP, "a bounded wait inside the key sort ran out (device stalled?): "
                        "the vectors of that minibatch are not to be trusted");
        return fail(W2V_ERR_INDEX, "a word index >= V = %u was passed to an earlier call", sh->V);
    }
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// negatives, dotprod, coeffs
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_negatives(w2v_shard* sh, const uint32_t* out_idx, uint32_t n, uint32_t k,
                             uint64_t seed, uint32_t* neg, void* stream) {
    if (!sh || (n && (!out_idx || (k && !neg)))) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (n == 0 || k == 0) return W2V_OK;
    hipStream_t st = (hipStream_t)stream;
    Plan sz = make_plan(nullptr, n, k, sh->g.stride4, 0, false, false);
    rc = ensure_ws(sh, sz.bytes);
    if (rc) return rc;
    Plan p = make_plan(sh->ws, n, k, sh->g.stride4, 0, false, false);
    {
        Phase ph(sh, W2V_PH_NEG, st);
        launch_dest_keys(NoiseTable{sh->bins, sh->V}, out_idx, n, k, seed, p.keys, sh->err, st);
        launch_copy_negatives(p.keys, n, k, neg, st);
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_dotprod(w2v_shard* sh, const uint32_t* in_idx, const uint32_t* out_idx,
                           uint32_t n, uint32_t k, uint64_t seed, float* partial_dots,
                           void* stream) {
    if (!sh || (n && (!in_idx || !out_idx || !partial_dots)))
        return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (n == 0) return W2V_OK;
    hipStream_t st = (hipStream_t)stream;
    Plan sz = make_plan(nullptr, n, k, sh->g.stride4, 0, false, false);
    rc = ensure_ws(sh, sz.bytes);
    if (rc) return rc;
    Plan p = make_plan(sh->ws, n, k, sh->g.stride4, 0, false, false);
    const int ahead = find_prepared(sh, in_idx, out_idx, n, k, seed);
    if (ahead >= 0) {                 // announced: the checked words and the keys exist already; the
        IndexSet& x = sh->sets[ahead];                   // set stays valid for the adjust call
        HIP_TRY(hipStreamWaitEvent(st, x.ready, 0));
        p.keys = x.keys; p.in_safe = x.in_safe;
    } else {
        Phase ph(sh, W2V_PH_NEG, st);
        launch_check_inputs(in_idx, n, sh->V, p.in_safe, sh->err, st);
        launch_dest_keys(NoiseTable{sh->bins, sh->V}, out_idx, n, k, seed, p.keys, sh->err, st);
    }
    {
        Phase ph(sh, W2V_PH_DOT, st);
        launch_dots(sh->U, sh->W, sh->g, p.in_safe, p.keys, n, p.T, partial_dots, st);
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

// w2v_dotprod without any allocation: the checked input words and the destination keys go to this
// device's static scratch array instead of the shard's growable region; same kernels.  No timing
// spans either (they take events from a pool that may have to grow).
extern "C" int w2v_dotprod_noalloc(w2v_shard* sh, const uint32_t* in_idx, const uint32_t* out_idx,
                                   uint32_t n, uint32_t k, uint64_t seed, float* partial_dots,
                                   void* stream) {
    if (!sh || (n && (!in_idx || !out_idx || !partial_dots)))
        return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (n == 0) return W2V_OK;
    const uint64_t M = (uint64_t)n * (k + 1);
    const uint64_t keys_u32 = (M + 63) & ~(uint64_t)63;           // keeps the second array 256-byte aligned
    if (keys_u32 + n > (uint64_t)W2V_NOALLOC_SCRATCH_U32)
        return fail(W2V_ERR_ARG, "n*(k+2) = %llu exceeds the %u entries of the static scratch array "
                    "(W2V_NOALLOC_SCRATCH_U32); use w2v_dotprod for larger minibatches",
                    (unsigned long long)(M + n), (unsigned)W2V_NOALLOC_SCRATCH_U32);
    if (!sh->static_ws) return fail(W2V_ERR_STATE, "the static scratch array was not resolved");
    hipStream_t st = (hipStream_t)stream;
    uint32_t* keys = sh->static_ws;
    uint32_t* in_safe = sh->static_ws + keys_u32;
    launch_check_inputs(in_idx, n, sh->V, in_safe, sh->err, st);
    launch_dest_keys(NoiseTable{sh->bins, sh->V}, out_idx, n, k, seed, keys, sh->err, st);
    launch_dots(sh->U, sh->W, sh->g, in_safe, keys, n, k + 1, partial_dots, st);
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_coeffs(w2v_shard* sh, const float* const* partials, uint32_t S, uint32_t n,
                          uint32_t k, float* coeffs, double* loss, void* stream) {
    if (!sh || !partials || (n && !coeffs)) return fail(W2V_ERR_NULL, "NULL argument");
    if (S == 0 || S > W2V_S_MAX) return fail(W2V_ERR_ARG, "S = %u outside 1..%d", S, W2V_S_MAX);
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, false);
    if (rc) return rc;
    PartialPtrs pp{};
    for (uint32_t s = 0; s < S; ++s) {
        if (n && !partials[s]) return fail(W2V_ERR_NULL, "partials[%u] is NULL", s);
        pp.p[s] = partials[s];
    }
    hipStream_t st = (hipStream_t)stream;
    size_t need = sizeof(double) * coeffs_loss_scratch_doubles(n, k + 1) + 512;
    rc = ensure_ws(sh, need);
    if (rc) return rc;
    {
        Phase ph(sh, W2V_PH_COEFF, st);
        launch_coeffs(pp, S, n, k + 1, coeffs, (double*)sh->ws, loss, st);
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// adjust
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_adjust(w2v_shard* sh, const uint32_t* in_idx, const uint32_t* out_idx,
                          uint32_t n, uint32_t k, uint64_t seed, const float* coeffs, float alpha,
                          void* stream) {
    if (!sh || (n && (!in_idx || !out_idx || !coeffs))) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (n == 0) return W2V_OK;
    hipStream_t st = (hipStream_t)stream;
    Plan sz = make_plan(nullptr, n, k, sh->g.stride4, 0, true, false);
    rc = ensure_ws(sh, sz.bytes);
    if (rc) return rc;
    Plan p = make_plan(sh->ws, n, k, sh->g.stride4, 0, true, false);
    uint32_t *sku, *perm, *skw, *sidx;
    sh->last_update_fused = false;
    const int ahead = find_prepared(sh, in_idx, out_idx, n, k, seed);
    sh->updates++;
    if (ahead >= 0) {
        IndexSet& x = sh->sets[ahead];
        sh->prep[ahead].valid = false;                   // a set serves one update
        HIP_TRY(hipStreamWaitEvent(st, x.ready, 0));
        // (the keys may carry the marks of rows named once; the two-call form does not use them:
        // its input-side kernel would have to read the input rows for that, which costs more)
        p.keys = x.keys; p.in_safe = x.in_safe;
        sku = x.sku; perm = x.perm; skw = x.skw; sidx = x.sidx;
    } else {
        rc = queue_keys_and_sorts(sh, p, in_idx, out_idx, k, seed, &sku, &perm, &skw, &sidx, st);
        if (rc) return rc;
    }
    queue_adjust(sh, sh, p, sku, perm, skw, sidx, coeffs, nullptr, false, alpha, nullptr, st);
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// one client step
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_train_minibatch(w2v_shard* const* shards, uint32_t S, const uint32_t* in_idx,
                                   const uint32_t* out_idx, uint32_t n, uint32_t k, uint64_t seed,
                                   float alpha, double* loss, void* stream) {
    if (!shards || (n && (!in_idx || !out_idx))) return fail(W2V_ERR_NULL, "NULL argument");
    if (S == 0 || S > W2V_S_MAX) return fail(W2V_ERR_ARG, "S = %u outside 1..%d", S, W2V_S_MAX);
    uint32_t stride_max = 0;
    for (uint32_t s = 0; s < S; ++s) {
        if (!shards[s]) return fail(W2V_ERR_NULL, "shards[%u] is NULL", s);
        if (shards[s]->V != shards[0]->V || shards[s]->device != shards[0]->device)
            return fail(W2V_ERR_MISMATCH, "shard %u differs from shard 0 in V or device", s);
        if (k > 0 && shards[s]->has_tables && shards[0]->has_tables &&
            shards[s]->table_tag != shards[0]->table_tag)
            return fail(W2V_ERR_MISMATCH, "shard %u holds a different noise table", s);
        stride_max = std::max(stride_max, shards[s]->g.stride4);
    }
    w2v_shard* s0 = shards[0];
    int rc = check_device(s0);
    if (!rc) rc = check_batch(s0, n, k, true);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) {
        if (loss) launch_loss_from_dots(nullptr, 0, k + 1, nullptr, loss, st);
        return W2V_OK;
    }
    const bool fused = (S == 1);
    const uint32_t own = (fused && s0->own_rows) ? s0->V : 0u;
    const uint32_t S_dots = fused ? (loss ? 1u : 0u) : S;    // fused: the dots are kept for the loss only
    Plan sz = make_plan(nullptr, n, k, stride_max, S_dots, true, true, own);
    rc = ensure_ws(s0, sz.bytes);
    if (rc) return rc;
    Plan p = make_plan(s0->ws, n, k, stride_max, S_dots, true, true, own);
    uint32_t *sku, *perm, *skw, *sidx;
    // a set computed by w2v_prefetch_minibatch on shard 0 (every shard holds the same noise table)
    s0->last_update_fused = fused;
    const int ahead = find_prepared(s0, in_idx, out_idx, n, k, seed);
    s0->updates++;
    if (ahead >= 0) {
        IndexSet& x = s0->sets[ahead];
        s0->prep[ahead].valid = false;                   // a set serves one update
        HIP_TRY(hipStreamWaitEvent(st, x.ready, 0));
        p.keys = x.keys; p.in_safe = x.in_safe; p.own_rows = fused && s0->prep[ahead].own_rows;
        sku = x.sku; perm = x.perm; skw = x.skw; sidx = x.sidx;
    } else {
        rc = queue_keys_and_sorts(s0, p, in_idx, out_idx, k, seed, &sku, &perm, &skw, &sidx, st);
        if (rc) return rc;
    }
    if (fused) {
        queue_adjust(s0, s0, p, sku, perm, skw, sidx, nullptr, p.coeffs, true, alpha, loss, st);
    } else {
        PartialPtrs pp{};
        {
            Phase ph(s0, W2V_PH_DOT, st);
            for (uint32_t s = 0; s < S; ++s) {
                float* d = p.dots + (size_t)s * p.M;
                launch_dots(shards[s]->U, shards[s]->W, shards[s]->g, p.in_safe, p.keys, n, p.T, d, st);
                pp.p[s] = d;
            }
        }
        {
            Phase ph(s0, W2V_PH_COEFF, st);
            launch_coeffs(pp, S, n, p.T, p.coeffs, p.loss_tmp, loss, st);
        }
        for (uint32_t s = 0; s < S; ++s)
            queue_adjust(s0, shards[s], p, sku, perm, skw, sidx, p.coeffs, nullptr, false, alpha, nullptr, st);
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_prefetch_minibatch(w2v_shard* sh, const uint32_t* in_idx, const uint32_t* out_idx,
                                      uint32_t n, uint32_t k, uint64_t seed, void* stream) {
    if (!sh || (n && (!in_idx || !out_idx))) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (n == 0 || !sh->overlap) return W2V_OK;            // nothing to gain without the second stream
    hipStream_t st = (hipStream_t)stream;
    rc = ensure_side_stream(sh);
    if (rc) return rc;
    Prepared want;
    want.in_idx = in_idx; want.out_idx = out_idx; want.n = n; want.k = k; want.seed = seed;
    // Queued at once, so that it runs beside the whole of the training call that is queued next.
    // (Queued behind that call's input-side kernel instead, it left the benchmark step unchanged but
    // did not fit beside the output-side kernel alone when k is large: the next step then waited.)
    return run_prefetch_chain(sh, want, st);
}

extern "C" int w2v_prefetch_cancel(w2v_shard* sh) {
    if (!sh) return fail(W2V_ERR_NULL, "shard is NULL");
    int rc = check_device(sh);
    if (rc) return rc;
    // the chains may still be reading the caller's arrays: wait for them before the caller is told
    // that the arrays are its own again
    if (sh->ahead) HIP_TRY(hipStreamSynchronize(sh->ahead));
    for (Prepared& pr : sh->prep) pr.valid = false;
    sh->cprep[0].valid = sh->cprep[1].valid = false;
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// a training step captured once and replayed (small minibatches are bound by launches, not bytes)
// ---------------------------------------------------------------------------------------------
struct w2v_step_graph {
    w2v_shard* sh = nullptr;
    uint32_t n = 0, k = 0;
    IndexPrologue first{};              // the step's first launch: queued by every run, with that
                                        // run's arrays and seed (not part of the graph)
    CallScalars* scalars = nullptr;     // the captured kernels read seed and learning rate from here
    const char* ws_at_capture = nullptr; // the shard's scratch region the captured kernels point into
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

static void free_step_graph(w2v_step_graph* g) {
    if (!g) return;
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    if (g->scalars) (void)hipFree(g->scalars);
    delete g;
}

extern "C" int w2v_step_graph_create(w2v_shard* sh, uint32_t n, uint32_t k, double* loss,
                                     w2v_step_graph** out) {
    if (!sh || !out) return fail(W2V_ERR_NULL, "NULL argument");
    *out = nullptr;
    int rc = check_device(sh);
    if (!rc) rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (n == 0) return fail(W2V_ERR_ARG, "a captured step needs at least one pair");
    w2v_step_graph* g = new (std::nothrow) w2v_step_graph();
    if (!g) return fail(W2V_ERR_ALLOC, "host allocation failed");
    g->sh = sh; g->n = n; g->k = k;
    hipStream_t cap = nullptr;
    auto bail = [&](int code) { if (cap) (void)hipStreamDestroy(cap); free_step_graph(g); return code; };
    hipError_t e = hipMalloc((void**)&g->scalars, 256);
    if (e == hipSuccess) e = hipMemset(g->scalars, 0, 256);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return bail(fail(W2V_ERR_ALLOC, "allocating the scalar block of a captured step failed: %s",
                         hipGetErrorString(e)));
    }
    // everything the step allocates must exist before the capture begins: its scratch ...
    const uint32_t own = sh->own_rows ? sh->V : 0u;
    Plan sz = make_plan(nullptr, n, k, sh->g.stride4, loss ? 1u : 0u, true, true, own);
    rc = ensure_ws(sh, sz.bytes);
    if (rc) return bail(rc);
    e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&cap, hipStreamNonBlocking);
    if (e != hipSuccess) return bail(fail(W2V_ERR_HIP, "set-up of the capture failed: %s", hipGetErrorString(e)));
    // ... and the capture runs the step on ONE stream, without timing spans and without looking at
    // announced minibatches (none can match the stand-in arrays).  The step's first launch -- keys,
    // checked inputs, fills -- is the only one that reads the caller's arrays: it is handed back
    // instead of captured, and every run queues it itself in front of the graph.  (Captured with its side stream,
    // as parallel branches of the graph, a 4096-pair step replays in 0.176 ms instead of 0.115 ms:
    // the two sorts are then separate chains of launches, and branches cost more than they hide.)
    const bool overlap = sh->overlap, timing = sh->timing;
    sh->overlap = false; sh->timing = false; sh->call_dev = g->scalars; sh->prologue_sink = &g->first;
    e = hipStreamBeginCapture(cap, hipStreamCaptureModeThreadLocal);
    if (e == hipSuccess) {
        w2v_shard* one[1] = {sh};
        const uint32_t* stand_in = (const uint32_t*)g->scalars;      // recorded, never read
        rc = w2v_train_minibatch(one, 1, stand_in, stand_in, n, k, 0, 0.f, loss, cap);
        hipError_t e2 = hipStreamEndCapture(cap, &g->graph);
        if (rc == W2V_OK && e2 != hipSuccess) e = e2;
    }
    sh->overlap = overlap; sh->timing = timing; sh->call_dev = nullptr; sh->prologue_sink = nullptr;
    if (rc == W2V_OK && e == hipSuccess && g->first.keys == nullptr)
        rc = fail(W2V_ERR_STATE, "the captured step did not hand back its first launch");
    if (rc) return bail(rc);
    if (e == hipSuccess) e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return bail(fail(W2V_ERR_HIP, "capturing the step failed: %s", hipGetErrorString(e)));
    }
    (void)hipStreamDestroy(cap);
    g->ws_at_capture = sh->ws;
    *out = g;
    return W2V_OK;
}

extern "C" int w2v_step_graph_run(w2v_step_graph* g, const uint32_t* in_idx, const uint32_t* out_idx,
                                  uint64_t seed, float alpha, void* stream) {
    if (!g || !in_idx || !out_idx) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(g->sh);
    if (rc) return rc;
    if (g->sh->ws != g->ws_at_capture)
        return fail(W2V_ERR_STATE, "the shard's scratch region was reallocated by a larger call after this "
                    "step was captured: create the graph again");
    hipStream_t st = (hipStream_t)stream;
    IndexPrologue first = g->first;
    first.in_idx = in_idx; first.out_idx = out_idx;
    first.seed_lo = (uint32_t)seed; first.seed_hi = (uint32_t)(seed >> 32);
    first.dev = nullptr; first.scalars_out = g->scalars; first.alpha = alpha;
    launch_index_prologue(first, st);
    HIP_TRY(hipGraphLaunch(g->exec, st));
    g->sh->updates++;
    g->sh->last_update_fused = true;
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_step_graph_destroy(w2v_step_graph* g) {
    if (!g) return W2V_OK;
    (void)hipDeviceSynchronize();
    free_step_graph(g);
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// continuous bag of words (Section 5.1, footnote)
// ---------------------------------------------------------------------------------------------
namespace {

// Scratch of one bag-of-words minibatch: n examples, M = n(k+1) dot slots, m context entries.
struct CbowPlan {
    uint32_t n, T, M, m;
    bool own_rows;                                   // fused step: rows named once go to the per-example pass
    uint32_t* keys;                                  // [M] center word + negatives per example
    uint32_t* ctx_safe; uint32_t* ex_of; float* weight;   // [m]
    uint32_t* iota;                                  // [n] 0, 1, 2, ...
    float* H; float* E; uint32_t* dkey;              // [n] rows: hidden vectors, summed output rows
    float* coeffs; float* dots; double* loss_tmp;
    uint2 *wb0, *wb1; uint32_t* sort_tmp_w;          // sort of the M destinations
    uint2 *cb0, *cb1; uint32_t* sort_tmp_c;          // sort of the m context entries
    float* pa_rows; uint32_t* pa_keys;               // unused slots of the per-example pass
    float* pb_rows; uint32_t* pb_keys;               // output side, level 1
    float* pd_rows; uint32_t* pd_keys;               // input side, level 1
    float* pc_rows; uint32_t* pc_keys;               // level 2, output side
    float* pe_rows; uint32_t* pe_keys;               // level 2, input side (the two sides overlap)
    uint32_t slots_a, slots_w1, slots_c1, slots_2;
    size_t bytes;
};

CbowPlan make_cbow_plan(char* base, uint32_t n, uint32_t k, uint32_t m, uint32_t stride4_max,
                        uint32_t S_dots, bool want_adjust, bool want_coeffs) {
    CbowPlan p{};
    p.n = n; p.T = k + 1; p.M = n * p.T; p.m = m;
    Carver c(base);
    const size_t row = (size_t)stride4_max * 4;
    p.keys = c.take<uint32_t>(p.M);
    p.ctx_safe = c.take<uint32_t>(m); p.ex_of = c.take<uint32_t>(m); p.weight = c.take<float>(m);
    p.iota = c.take<uint32_t>(n);
    p.H = c.take<float>((size_t)n * row);
    if (want_coeffs) p.coeffs = c.take<float>(p.M);
    if (S_dots) p.dots = c.take<float>((size_t)S_dots * p.M);
    p.loss_tmp = c.take<double>(coeffs_loss_scratch_doubles(n, p.T));
    if (want_adjust) {
        p.E = c.take<float>((size_t)n * row);
        p.dkey = c.take<uint32_t>(n);
        p.wb0 = c.take<uint2>(p.M); p.wb1 = c.take<uint2>(p.M);
        p.sort_tmp_w = c.take<uint32_t>(sort_scratch_u32(p.M));
        p.cb0 = c.take<uint2>(m); p.cb1 = c.take<uint2>(m);
        p.sort_tmp_c = c.take<uint32_t>(sort_scratch_u32(m));
        p.slots_a = slots_after(n, useg_pairs_per_chunk(p.T, 1, n));
        p.slots_w1 = slots_after(p.M, wseg_entries_per_chunk());
        p.slots_c1 = slots_after(m, wseg_entries_per_chunk());
        p.slots_2 = std::max(slots_after(p.slots_w1, tail_entries_per_chunk()),
                             slots_after(p.slots_c1, tail_entries_per_chunk()));
        p.pa_rows = c.take<float>((size_t)p.slots_a * row);  p.pa_keys = c.take<uint32_t>(p.slots_a + 1);
        p.pb_rows = c.take<float>((size_t)p.slots_w1 * row); p.pb_keys = c.take<uint32_t>(p.slots_w1 + 1);
        p.pd_rows = c.take<float>((size_t)p.slots_c1 * row); p.pd_keys = c.take<uint32_t>(p.slots_c1 + 1);
        p.pc_rows = c.take<float>((size_t)p.slots_2 * row);  p.pc_keys = c.take<uint32_t>(p.slots_2 + 1);
        p.pe_rows = c.take<float>((size_t)p.slots_2 * row);  p.pe_keys = c.take<uint32_t>(p.slots_2 + 1);
    }
    p.bytes = c.off + 256;
    return p;
}

int check_cbow_batch(const w2v_shard* sh, uint32_t n, uint32_t k, uint32_t m) {
    int rc = check_batch(sh, n, k, true);
    if (rc) return rc;
    if (m >= (1u << 31)) return fail(W2V_ERR_ARG, "m = %u context entries must stay below 2^31", m);
    return W2V_OK;
}

// Checked context entries, example numbers and weights, the destination keys, and (for adjust)
// both sorts: destinations of the M output-side contributions, words of the m context entries.
// With the second stream, the keys and the sorts are queued there (they depend on the indices
// only) while the caller's stream forms the hidden vectors; cbow_wait_keys / join_output_sort make
// the caller's stream wait for them where they are first needed.
int queue_cbow_indices(w2v_shard* sh, CbowPlan& p, const uint32_t* ctx_off, const uint32_t* ctx_idx,
                       const uint32_t* out_idx, uint32_t k, uint64_t seed, bool sorts,
                       uint32_t** skw, uint32_t** sidx, uint32_t** skc, uint32_t** cidx,
                       hipStream_t st) {
    {
        Phase ph(sh, W2V_PH_NEG, st);
        launch_cbow_entries(ctx_off, ctx_idx, p.n, p.m, sh->V, p.ctx_safe, p.ex_of, p.weight,
                            sh->err, st);
        launch_iota(p.iota, p.n, st);
    }
    hipStream_t wst = st;
    const bool two = sorts && sh->overlap;
    if (two) {
        int rc = ensure_side_stream(sh);
        if (rc) return rc;
        HIP_TRY(hipEventRecord(sh->ev_fork, st));
        HIP_TRY(hipStreamWaitEvent(sh->side, sh->ev_fork, 0));
        wst = sh->side;
    }
    {
        Phase ph(sh, W2V_PH_NEG, wst);
        launch_dest_keys(NoiseTable{sh->bins, sh->V}, out_idx, p.n, k, seed, p.keys, sh->err, wst);
    }
    if (two && !p.own_rows) HIP_TRY(hipEventRecord(sh->ev_keys, wst));
    if (!sorts) return W2V_OK;
    {
        Phase ph(sh, W2V_PH_SORT, wst);
        const uint32_t bits = key_bits(sh->V);
        launch_sort_pairs(p.keys, p.wb0, p.wb1, p.M, bits, p.sort_tmp_w, skw, sidx, sh->err, wst);
        if (p.own_rows) {           // the per-example pass needs the marks: "keys ready" moves here
            launch_mark_alone(*skw, *sidx, p.M, p.keys, wst);
            if (two) HIP_TRY(hipEventRecord(sh->ev_keys, wst));
        }
        launch_sort_pairs(p.ctx_safe, p.cb0, p.cb1, p.m, bits, p.sort_tmp_c, skc, cidx, sh->err, wst);
    }
    if (two) HIP_TRY(hipEventRecord(sh->ev_join, wst));
    return W2V_OK;
}

// The caller's stream needs the keys from here on (only after a queue_cbow_indices with sorts).
void cbow_wait_keys(w2v_shard* sh, hipStream_t st) {
    if (sh->overlap && sh->side) (void)hipStreamWaitEvent(st, sh->ev_keys, 0);
}

void queue_cbow_hidden(w2v_shard* owner, w2v_shard* sh, CbowPlan& p, const uint32_t* ctx_off,
                       hipStream_t st) {
    Phase ph(owner, W2V_PH_DOT, st);
    launch_cbow_hidden(sh->U, sh->g, ctx_off, p.ctx_safe, p.n, p.m, p.H, st);
}

// The update of one shard.  The hidden vectors stand in for the input vectors in the skip-gram
// kernels: the per-example pass (every example is its own run) leaves e_p = sum_j g_pj v_row_pj in
// E, forming dots and coefficients on the way when fused; the output side adds g_pj h_p to its
// rows; the input side adds e_p / |C_p| to the input vector of every context entry.  H holds the
// start-of-call input vectors and E the start-of-call output vectors, so the order of the two
// write-backs does not matter -- with the second stream they run beside each other: the input side
// there, behind its sort, the output side on the caller's stream.
void queue_cbow_adjust(w2v_shard* owner, w2v_shard* sh, CbowPlan& p, const uint32_t* skw,
                       const uint32_t* sidx, const uint32_t* skc, const uint32_t* cidx,
                       const float* coeffs_in, float* coeffs_out, float* dots_out, bool fused,
                       float alpha, bool join_sorts, hipStream_t st) {
    // border slots of both write-back kernels, cleared ahead of the per-example pass (the second
    // stream's kernel starts behind an event recorded after that pass)
    launch_wseg_fill(p.pd_keys, p.m, st);
    launch_wseg_fill(p.pb_keys, p.M, st);
    {
        Phase ph(owner, W2V_PH_USIDE, st);
        USideArgs a{};
        a.U = p.H; a.W = sh->W; a.g = sh->g; a.skey = p.iota; a.perm = p.iota; a.keys = p.keys;
        a.n = p.n; a.T = p.T; a.coeffs_in = coeffs_in; a.coeffs_out = coeffs_out;
        a.dots_out = fused ? dots_out : nullptr; a.delta = p.E; a.dkey = p.dkey;
        a.prows = p.pa_rows; a.pkeys = p.pa_keys; a.fused = fused;
        if (fused && p.own_rows) { a.W_update = sh->W; a.alpha = alpha; }   // source: the hidden vector
        launch_useg(a, st);
    }
    const bool two = owner->overlap && owner->side;
    hipStream_t side = two ? owner->side : st;
    if (two) {
        (void)hipEventRecord(owner->ev_coeffs, st);
        (void)hipStreamWaitEvent(side, owner->ev_coeffs, 0);
    }
    {
        Phase ph(owner, W2V_PH_APPLY, side);
        WSideArgs u{};
        u.U = p.E; u.W = sh->U; u.g = sh->g; u.skey = skc; u.sidx = cidx; u.M = p.m; u.T = 1;
        u.in_idx = p.ex_of; u.coeffs = p.weight; u.alpha = alpha;
        u.prows = p.pd_rows; u.pkeys = p.pd_keys;
        launch_wseg(u, side, true);
        run_tails(sh, sh->U, alpha, p.pd_rows, p.pd_keys, p.slots_c1, p.pe_rows, p.pe_keys, side);
    }
    if (two) (void)hipEventRecord(owner->ev_tails, side);
    if (join_sorts) join_output_sort(owner, st);
    {
        Phase ph(owner, W2V_PH_WSIDE, st);
        WSideArgs w{};
        w.U = p.H; w.W = sh->W; w.g = sh->g; w.skey = skw; w.sidx = sidx; w.M = p.M; w.T = p.T;
        w.in_idx = p.iota; w.coeffs = fused ? coeffs_out : coeffs_in; w.alpha = alpha;
        w.prows = p.pb_rows; w.pkeys = p.pb_keys;
        w.skip_alone = fused && p.own_rows;
        launch_wseg(w, st, true);
        run_tails(sh, sh->W, alpha, p.pb_rows, p.pb_keys, p.slots_w1, p.pc_rows, p.pc_keys, st);
    }
    if (two) (void)hipStreamWaitEvent(st, owner->ev_tails, 0);
}

// Buffers of one announced bag-of-words minibatch, carved from the set's own allocation.
int ensure_cset(w2v_shard* sh, CbowSet& x, uint32_t n, uint32_t M, uint32_t m) {
    for (int pass = 0; pass < 2; ++pass) {
        Carver c(pass ? x.base : nullptr);
        uint32_t* keys = c.take<uint32_t>(M);
        uint32_t* ctx_safe = c.take<uint32_t>(m); uint32_t* ex_of = c.take<uint32_t>(m);
        float* weight = c.take<float>(m);
        uint32_t* iota = c.take<uint32_t>(n);
        uint2* wb0 = c.take<uint2>(M); uint2* wb1 = c.take<uint2>(M);
        uint2* cb0 = c.take<uint2>(m); uint2* cb1 = c.take<uint2>(m);
        uint32_t* tw = c.take<uint32_t>(sort_scratch_u32(M, m));
        const size_t need = c.off + 256;
        if (pass == 0) {
            int rc = ensure_region(x.base, x.cap, need);
            if (rc) return rc;
        } else {
            x.keys = keys; x.ctx_safe = ctx_safe; x.ex_of = ex_of; x.weight = weight; x.iota = iota;
            x.wb0 = wb0; x.wb1 = wb1; x.cb0 = cb0; x.cb1 = cb1; x.sort_tmp = tw;
        }
    }
    if (!x.ready) HIP_TRY(hipEventCreateWithFlags(&x.ready, hipEventDisableTiming));
    if (!sh->ev_pfork) HIP_TRY(hipEventCreateWithFlags(&sh->ev_pfork, hipEventDisableTiming));
    return W2V_OK;
}

// The index work of an announced bag-of-words minibatch, queued on the third stream behind
// everything queued on `st` so far.
int run_cbow_prefetch_chain(w2v_shard* sh, const CbowPrepared& want, hipStream_t st) {
    const int which = sh->next_cset;
    CbowSet& x = sh->csets[which];
    sh->cprep[which].valid = false;
    const uint32_t n = want.n, k = want.k, m = want.m, M = n * (k + 1);
    int rc = ensure_cset(sh, x, n, M, m);
    if (rc) return rc;
    HIP_TRY(hipEventRecord(sh->ev_pfork, st));
    HIP_TRY(hipStreamWaitEvent(sh->ahead, sh->ev_pfork, 0));
    hipStream_t ah = sh->ahead;
    const uint32_t bits = key_bits(sh->V);
    {
        Phase ph(sh, W2V_PH_NEG, ah);
        launch_cbow_entries(want.ctx_off, want.ctx_idx, n, m, sh->V, x.ctx_safe, x.ex_of, x.weight,
                            sh->err, ah);
        launch_iota(x.iota, n, ah);
        launch_dest_keys(NoiseTable{sh->bins, sh->V}, want.out_idx, n, k, want.seed, x.keys, sh->err, ah);
    }
    {
        Phase ph(sh, W2V_PH_SORT, ah);
        const SortJob jobs[2] = {{x.keys, M, x.wb0, x.wb1, &x.skw, &x.sidx},
                                 {x.ctx_safe, m, x.cb0, x.cb1, &x.skc, &x.cidx}};
        launch_sort_jobs(jobs, 2, bits, x.sort_tmp, sh->err, ah);
        if (sh->own_rows) launch_mark_alone(x.skw, x.sidx, M, x.keys, ah);
    }
    HIP_TRY(hipEventRecord(x.ready, ah));
    HIP_TRY(hipGetLastError());
    CbowPrepared& pr = sh->cprep[which];
    pr = want;
    pr.valid = true; pr.own_rows = sh->own_rows; pr.born = sh->updates;
    sh->next_cset = which ^ 1;
    return W2V_OK;
}

// The set that w2v_cbow_prefetch_minibatch filled for exactly this minibatch, or -1.
int find_cbow_prepared(w2v_shard* sh, const uint32_t* ctx_off, const uint32_t* ctx_idx,
                       uint32_t m, const uint32_t* out_idx, uint32_t n, uint32_t k, uint64_t seed) {
    for (int i = 0; i < 2; ++i) {
        CbowPrepared& pr = sh->cprep[i];
        if (pr.valid && sh->updates - pr.born >= PREP_MAX_AGE) pr.valid = false;
        if (pr.valid && pr.ctx_off == ctx_off && pr.ctx_idx == ctx_idx && pr.out_idx == out_idx &&
            pr.n == n && pr.k == k && pr.m == m && pr.seed == seed)
            return i;
    }
    return -1;
}

// Point the plan at a prepared set (the caller's stream waits for it) ...
int use_cbow_prepared(w2v_shard* sh, int which, CbowPlan& p, bool spend, bool fused, uint32_t** skw,
                      uint32_t** sidx, uint32_t** skc, uint32_t** cidx, hipStream_t st) {
    CbowSet& x = sh->csets[which];
    if (spend) sh->cprep[which].valid = false;            // a set serves one update
    HIP_TRY(hipStreamWaitEvent(st, x.ready, 0));
    p.keys = x.keys; p.ctx_safe = x.ctx_safe; p.ex_of = x.ex_of; p.weight = x.weight; p.iota = x.iota;
    p.own_rows = fused && sh->cprep[which].own_rows;
    if (skw) { *skw = x.skw; *sidx = x.sidx; *skc = x.skc; *cidx = x.cidx; }
    return W2V_OK;
}

// ... or compute the index work within the call.
int cbow_indices(w2v_shard* sh, CbowPlan& p, const uint32_t* ctx_off, const uint32_t* ctx_idx,
                 uint32_t m, const uint32_t* out_idx, uint32_t n, uint32_t k, uint64_t seed,
                 bool sorts, bool spend, bool fused, uint32_t** skw, uint32_t** sidx, uint32_t** skc,
                 uint32_t** cidx, bool* prepared, hipStream_t st) {
    const int ahead = find_cbow_prepared(sh, ctx_off, ctx_idx, m, out_idx, n, k, seed);
    if (spend) sh->updates++;                             // an update call
    *prepared = ahead >= 0;
    if (ahead >= 0) return use_cbow_prepared(sh, ahead, p, spend, fused, skw, sidx, skc, cidx, st);
    return queue_cbow_indices(sh, p, ctx_off, ctx_idx, out_idx, k, seed, sorts, skw, sidx, skc, cidx, st);
}

int check_cbow_pointers(const uint32_t* ctx_off, const uint32_t* ctx_idx, uint32_t m,
                        const uint32_t* out_idx, uint32_t n) {
    if (n && (!ctx_off || !out_idx)) return fail(W2V_ERR_NULL, "NULL argument");
    if (m && !ctx_idx) return fail(W2V_ERR_NULL, "ctx_idx is NULL");
    if (n == 0 && m != 0) return fail(W2V_ERR_ARG, "context entries without examples");
    return W2V_OK;
}

}  // namespace

extern "C" int w2v_cbow_dotprod(w2v_shard* sh, const uint32_t* ctx_off, const uint32_t* ctx_idx,
                                uint32_t m, const uint32_t* out_idx, uint32_t n, uint32_t k,
                                uint64_t seed, float* partial_dots, void* stream) {
    if (!sh || (n && !partial_dots)) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_cbow_pointers(ctx_off, ctx_idx, m, out_idx, n);
    if (!rc) rc = check_device(sh);
    if (!rc) rc = check_cbow_batch(sh, n, k, m);
    if (rc) return rc;
    if (n == 0) return W2V_OK;
    hipStream_t st = (hipStream_t)stream;
    CbowPlan sz = make_cbow_plan(nullptr, n, k, m, sh->g.stride4, 0, false, false);
    rc = ensure_ws(sh, sz.bytes);
    if (rc) return rc;
    CbowPlan p = make_cbow_plan(sh->ws, n, k, m, sh->g.stride4, 0, false, false);
    bool prepared = false;              // an announced set is used and left for the update
    rc = cbow_indices(sh, p, ctx_off, ctx_idx, m, out_idx, n, k, seed, false, false, false, nullptr,
                      nullptr, nullptr, nullptr, &prepared, st);
    if (rc) return rc;
    queue_cbow_hidden(sh, sh, p, ctx_off, st);
    {
        Phase ph(sh, W2V_PH_DOT, st);
        launch_dots(p.H, sh->W, sh->g, p.iota, p.keys, n, p.T, partial_dots, st);
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_cbow_adjust(w2v_shard* sh, const uint32_t* ctx_off, const uint32_t* ctx_idx,
                               uint32_t m, const uint32_t* out_idx, uint32_t n, uint32_t k,
                               uint64_t seed, const float* coeffs, float alpha, void* stream) {
    if (!sh || (n && !coeffs)) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_cbow_pointers(ctx_off, ctx_idx, m, out_idx, n);
    if (!rc) rc = check_device(sh);
    if (!rc) rc = check_cbow_batch(sh, n, k, m);
    if (rc) return rc;
    if (n == 0) return W2V_OK;
    hipStream_t st = (hipStream_t)stream;
    CbowPlan sz = make_cbow_plan(nullptr, n, k, m, sh->g.stride4, 0, true, false);
    rc = ensure_ws(sh, sz.bytes);
    if (rc) return rc;
    CbowPlan p = make_cbow_plan(sh->ws, n, k, m, sh->g.stride4, 0, true, false);
    uint32_t *skw, *sidx, *skc, *cidx;
    bool prepared = false;
    rc = cbow_indices(sh, p, ctx_off, ctx_idx, m, out_idx, n, k, seed, true, true, false, &skw, &sidx,
                      &skc, &cidx, &prepared, st);
    if (rc) return rc;
    queue_cbow_hidden(sh, sh, p, ctx_off, st);
    if (!prepared) cbow_wait_keys(sh, st);
    queue_cbow_adjust(sh, sh, p, skw, sidx, skc, cidx, coeffs, nullptr, nullptr, false, alpha, !prepared, st);
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_cbow_train_minibatch(w2v_shard* const* shards, uint32_t S,
                                        const uint32_t* ctx_off, const uint32_t* ctx_idx,
                                        uint32_t m, const uint32_t* out_idx, uint32_t n, uint32_t k,
                                        uint64_t seed, float alpha, double* loss, void* stream) {
    if (!shards) return fail(W2V_ERR_NULL, "NULL argument");
    if (S == 0 || S > W2V_S_MAX) return fail(W2V_ERR_ARG, "S = %u outside 1..%d", S, W2V_S_MAX);
    uint32_t stride_max = 0;
    for (uint32_t s = 0; s < S; ++s) {
        if (!shards[s]) return fail(W2V_ERR_NULL, "shards[%u] is NULL", s);
        if (shards[s]->V != shards[0]->V || shards[s]->device != shards[0]->device)
            return fail(W2V_ERR_MISMATCH, "shard %u differs from shard 0 in V or device", s);
        if (k > 0 && shards[s]->has_tables && shards[0]->has_tables &&
            shards[s]->table_tag != shards[0]->table_tag)
            return fail(W2V_ERR_MISMATCH, "shard %u holds a different noise table", s);
        stride_max = std::max(stride_max, shards[s]->g.stride4);
    }
    w2v_shard* s0 = shards[0];
    int rc = check_cbow_pointers(ctx_off, ctx_idx, m, out_idx, n);
    if (!rc) rc = check_device(s0);
    if (!rc) rc = check_cbow_batch(s0, n, k, m);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) {
        if (loss) launch_loss_from_dots(nullptr, 0, k + 1, nullptr, loss, st);
        return W2V_OK;
    }
    const bool fused = (S == 1);
    const uint32_t S_dots = fused ? (loss ? 1u : 0u) : S;    // fused: the dots are kept for the loss only
    CbowPlan sz = make_cbow_plan(nullptr, n, k, m, stride_max, S_dots, true, true);
    rc = ensure_ws(s0, sz.bytes);
    if (rc) return rc;
    CbowPlan p = make_cbow_plan(s0->ws, n, k, m, stride_max, S_dots, true, true);
    p.own_rows = fused && s0->own_rows;
    uint32_t *skw, *sidx, *skc, *cidx;
    bool prepared = false;
    rc = cbow_indices(s0, p, ctx_off, ctx_idx, m, out_idx, n, k, seed, true, true, fused, &skw, &sidx,
                      &skc, &cidx, &prepared, st);
    if (rc) return rc;
    if (fused) {
        queue_cbow_hidden(s0, s0, p, ctx_off, st);
        if (!prepared) cbow_wait_keys(s0, st);
        queue_cbow_adjust(s0, s0, p, skw, sidx, skc, cidx, nullptr, p.coeffs, loss ? p.dots : nullptr, true,
                          alpha, !prepared, st);
        if (loss) {
            Phase ph(s0, W2V_PH_COEFF, st);
            launch_loss_from_dots(p.dots, n, p.T, p.loss_tmp, loss, st);
        }
    } else {
        // As in the two-call protocol, every shard forms its hidden vectors once for the dots and
        // once more for the update (its input vectors do not change in between).
        PartialPtrs pp{};
        for (uint32_t s = 0; s < S; ++s) {
            float* d = p.dots + (size_t)s * p.M;
            queue_cbow_hidden(s0, shards[s], p, ctx_off, st);
            if (!prepared) cbow_wait_keys(s0, st);
            Phase ph(s0, W2V_PH_DOT, st);
            launch_dots(p.H, shards[s]->W, shards[s]->g, p.iota, p.keys, n, p.T, d, st);
            pp.p[s] = d;
        }
        {
            Phase ph(s0, W2V_PH_COEFF, st);
            launch_coeffs(pp, S, n, p.T, p.coeffs, p.loss_tmp, loss, st);
        }
        for (uint32_t s = 0; s < S; ++s) {
            queue_cbow_hidden(s0, shards[s], p, ctx_off, st);
            queue_cbow_adjust(s0, shards[s], p, skw, sidx, skc, cidx, p.coeffs, nullptr, nullptr, false,
                              alpha, !prepared, st);
        }
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" int w2v_cbow_prefetch_minibatch(w2v_shard* sh, const uint32_t* ctx_off,
                                           const uint32_t* ctx_idx, uint32_t m,
                                           const uint32_t* out_idx, uint32_t n, uint32_t k,
                                           uint64_t seed, void* stream) {
    if (!sh) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_cbow_pointers(ctx_off, ctx_idx, m, out_idx, n);
    if (!rc) rc = check_device(sh);
    if (!rc) rc = check_cbow_batch(sh, n, k, m);
    if (rc) return rc;
    if (n == 0 || !sh->overlap) return W2V_OK;            // nothing to gain without the other streams
    rc = ensure_side_stream(sh);
    if (rc) return rc;
    CbowPrepared want;
    want.ctx_off = ctx_off; want.ctx_idx = ctx_idx; want.out_idx = out_idx;
    want.n = n; want.k = k; want.m = m; want.seed = seed;
    return run_cbow_prefetch_chain(sh, want, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// export and retrieval
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_export_rows(w2v_shard* const* shards, uint32_t S, int which,
                               const uint32_t* rows, uint32_t m, float* dst, void* stream) {
    if (!shards || (m && (!rows || !dst))) return fail(W2V_ERR_NULL, "NULL argument");
    if (S == 0 || S > W2V_S_MAX) return fail(W2V_ERR_ARG, "S = %u outside 1..%d", S, W2V_S_MAX);
    if (which != 0 && which != 1) return fail(W2V_ERR_ARG, "which must be 0 (input) or 1 (output)");
    for (uint32_t s = 0; s < S; ++s) {
        if (!shards[s]) return fail(W2V_ERR_NULL, "shards[%u] is NULL", s);
        if (shards[s]->V != shards[0]->V || shards[s]->device != shards[0]->device ||
            shards[s]->d_total != shards[0]->d_total)
            return fail(W2V_ERR_MISMATCH, "shard %u differs from shard 0 in V, d_total or device", s);
    }
    // the column ranges must tile [0, d_total) exactly
    std::vector<uint32_t> order(S);
    for (uint32_t s = 0; s < S; ++s) order[s] = s;
    std::sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
        return shards[x]->col_begin < shards[y]->col_begin;
    });
    uint32_t next = 0;
    for (uint32_t s = 0; s < S; ++s) {
        if (shards[order[s]]->col_begin != next)
            return fail(W2V_ERR_MISMATCH, "the shards' columns do not tile [0, d_total): gap or "
                        "overlap at column %u", next);
        next += shards[order[s]]->d_slice;
    }
    if (next != shards[0]->d_total)
        return fail(W2V_ERR_MISMATCH, "the shards cover %u of %u columns", next, shards[0]->d_total);
    int rc = check_device(shards[0]);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    for (uint32_t s = 0; s < S; ++s) {
        w2v_shard* sh = shards[s];
        launch_export_rows(which ? sh->W : sh->U, sh->g, sh->d_slice, rows, m, sh->V, dst,
                           sh->d_total, sh->col_begin, sh->err, st);
    }
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

extern "C" size_t w2v_topk_cosine_workspace(uint32_t Q, uint32_t N, uint32_t round_candidates) {
    if (Q == 0 || N == 0) return 0;
    if (round_candidates == 0 || round_candidates > N) round_candidates = N;
    return topk_workspace_bytes(Q, N, round_candidates);
}

extern "C" int w2v_topk_cosine(const float* queries, uint32_t Q, const float* cands, uint32_t N,
                               uint32_t d, uint32_t K, float tau, uint32_t* out_idx,
                               float* out_score, uint32_t* out_count, void* workspace,
                               size_t workspace_bytes, void* stream) {
    if (Q == 0) return W2V_OK;
    if (K == 0 || K > W2V_TOPK_MAX) return fail(W2V_ERR_ARG, "K = %u outside 1..%d", K, W2V_TOPK_MAX);
    if (N == 0 || d == 0) return fail(W2V_ERR_ARG, "N and d must be at least 1");
    if (!queries || !cands || !out_idx || !out_score || !workspace)
        return fail(W2V_ERR_NULL, "NULL argument");
    if (N >= 0xFFFFFF00u || Q >= 0xFFFFFF00u) return fail(W2V_ERR_ARG, "Q and N must stay below 2^32 - 256");
    if (!(tau == tau)) return fail(W2V_ERR_ARG, "tau is not a number");
    if ((uintptr_t)workspace % 256) return fail(W2V_ERR_ARG, "workspace must be 256-byte aligned");
    const uint32_t cap = topk_round_capacity(Q, N, workspace_bytes);
    if (cap == 0)
        return fail(W2V_ERR_ARG, "workspace of %zu bytes is too small: %zu are needed for rounds of "
                    "128 candidates", workspace_bytes, topk_workspace_bytes(Q, N, 128));
    launch_topk_cosine(queries, Q, cands, N, d, K, tau, out_idx, out_score, out_count, workspace, cap,
                       (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return W2V_OK;
}

// ---------------------------------------------------------------------------------------------
// pair formation
// ---------------------------------------------------------------------------------------------
// Outputs of the bag-of-words example formation on top of the pair stream.
struct CbowOut { uint32_t* ctx_off; uint32_t* centers; uint64_t cap_examples; uint64_t* n_examples; };

static int make_pairs_impl(w2v_shard* sh, const uint32_t* tokens, const uint64_t* sent_off,
                           uint32_t n_sent, uint32_t n_tokens, uint64_t token_base, uint32_t epoch,
                           uint64_t corpus_seed, uint32_t B, uint32_t* in_idx, uint32_t* out_idx,
                           uint64_t capacity, uint64_t* n_pairs, bool interleave,
                           const CbowOut* cbow, void* stream) {
    if (!sh || !n_pairs) return fail(W2V_ERR_NULL, "NULL argument");
    *n_pairs = 0;
    if (n_tokens && (!tokens || !sent_off)) return fail(W2V_ERR_NULL, "NULL argument");
    if (capacity && ((!in_idx && !cbow) || !out_idx)) return fail(W2V_ERR_NULL, "NULL output");
    if (B == 0) return fail(W2V_ERR_ARG, "window B must be at least 1");
    if (n_tokens && n_sent == 0) return fail(W2V_ERR_ARG, "tokens without sentences");
    if ((uint64_t)n_tokens * 2 * B >= (1ull << 32))
        return fail(W2V_ERR_ARG, "n_tokens * 2B must stay below 2^32; pass the corpus in blocks");
    int rc = check_device(sh);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (n_tokens == 0) {
        if (cbow) {                          // the closing offset of an empty example list
            launch_iota(cbow->ctx_off, 1, st);
            HIP_TRY(hipStreamSynchronize(st));
        }
        return W2V_OK;
    }
    size_t need = sizeof(uint32_t) * (pairs_scratch_u32(n_tokens, interleave) + 64) + 512;
    rc = ensure_region(sh->pairs_ws, sh->pairs_ws_cap, need);
    if (rc) return rc;
    PairArgs a{};
    a.tokens = tokens; a.sent_off = sent_off; a.n_sent = n_sent; a.n_tokens = n_tokens;
    a.token_base = token_base; a.epoch = epoch; a.seed = corpus_seed; a.B = B;
    a.keep = sh->has_tables ? sh->keep : nullptr; a.V = sh->V;
    a.in_idx = in_idx; a.out_idx = out_idx; a.capacity = capacity; a.interleave = interleave;
    a.total_pairs = (uint32_t*)sh->pairs_ws;
    if (cbow) {
        a.ctx_off = cbow->ctx_off; a.centers = cbow->centers; a.cap_examples = cbow->cap_examples;
        a.total_examples = (uint32_t*)sh->pairs_ws + 1;
    }
    a.scratch = (uint32_t*)sh->pairs_ws + 64;
    a.err = sh->err;
    {
        Phase ph(sh, W2V_PH_PAIRS, st);
        launch_make_pairs(a, st);
    }
    HIP_TRY(hipGetLastError());
    uint32_t total[2] = {0, 0};
    HIP_TRY(hipMemcpyAsync(total, a.total_pairs, sizeof(uint32_t) * (cbow ? 2 : 1),
                           hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    *n_pairs = total[0];
    if (cbow) *cbow->n_examples = total[1];
    return W2V_OK;
}

extern "C" int w2v_make_cbow_examples(w2v_shard* sh, const uint32_t* tokens,
                                      const uint64_t* sent_off, uint32_t n_sent, uint32_t n_tokens,
                                      uint64_t token_base, uint32_t epoch, uint64_t corpus_seed,
                                      uint32_t B, uint32_t* ctx_off, uint32_t* ctx_idx,
                                      uint32_t* out_idx, uint64_t cap_examples, uint64_t cap_ctx,
                                      uint64_t* n_examples, uint64_t* n_ctx, void* stream) {
    if (!n_examples || !ctx_off) return fail(W2V_ERR_NULL, "NULL argument");
    *n_examples = 0;
    if (cap_examples && !out_idx) return fail(W2V_ERR_NULL, "NULL output");
    CbowOut co{ctx_off, out_idx, cap_examples, n_examples};
    return make_pairs_impl(sh, tokens, sent_off, n_sent, n_tokens, token_base, epoch, corpus_seed,
                           B, nullptr, ctx_idx, cap_ctx, n_ctx, false, &co, stream);
}

extern "C" int w2v_make_pairs(w2v_shard* sh, const uint32_t* tokens, const uint64_t* sent_off,
                              uint32_t n_sent, uint32_t n_tokens, uint64_t token_base,
                              uint32_t epoch, uint64_t corpus_seed, uint32_t B, uint32_t* in_idx,
                              uint32_t* out_idx, uint64_t capacity, uint64_t* n_pairs,
                              void* stream) {
    return make_pairs_impl(sh, tokens, sent_off, n_sent, n_tokens, token_base, epoch, corpus_seed,
                           B, in_idx, out_idx, capacity, n_pairs, false, nullptr, stream);
}

extern "C" int w2v_make_pairs_interleaved(w2v_shard* sh, const uint32_t* tokens,
                                          const uint64_t* sent_off, uint32_t n_sent,
                                          uint32_t n_tokens, uint64_t token_base, uint32_t epoch,
                                          uint64_t corpus_seed, uint32_t B, uint32_t* in_idx,
                                          uint32_t* out_idx, uint64_t capacity, uint64_t* n_pairs,
                                          void* stream) {
    return make_pairs_impl(sh, tokens, sent_off, n_sent, n_tokens, token_base, epoch, corpus_seed,
                           B, in_idx, out_idx, capacity, n_pairs, true, nullptr, stream);
}

extern "C" uint64_t w2v_minibatch_seed(uint64_t master_seed, uint64_t h) {
    U4 r = philox4x32_10((uint32_t)h, (uint32_t)(h >> 32), 0, DOM_MBSEED, (uint32_t)master_seed,
                         (uint32_t)(master_seed >> 32));
    return ((uint64_t)r.y << 32) | (uint64_t)r.x;
}

// ---------------------------------------------------------------------------------------------
// timing
// ---------------------------------------------------------------------------------------------
extern "C" int w2v_shard_timing_enable(w2v_shard* sh, int on) {
    if (!sh) return fail(W2V_ERR_NULL, "shard is NULL");
    sh->timing = on != 0;
    return W2V_OK;
}

extern "C" int w2v_shard_timing_read(w2v_shard* sh, double* ms, uint64_t* launches) {
    if (!sh || !ms || !launches) return fail(W2V_ERR_NULL, "NULL argument");
    int rc = check_device(sh);
    if (rc) return rc;
    HIP_TRY(hipDeviceSynchronize());
    for (auto& s : sh->spans) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, s.a, s.b) == hipSuccess) {
            sh->ms[s.phase] += (double)t;
            sh->launches[s.phase] += 1;
        } else {
            (void)hipGetLastError();
        }
        sh->pool.push_back(s.a);
        sh->pool.push_back(s.b);
    }
    sh->spans.clear();
    for (int i = 0; i < W2V_PHASES; ++i) {
        ms[i] = sh->ms[i]; launches[i] = sh->launches[i];
        sh->ms[i] = 0; sh->launches[i] = 0;
    }
    return W2V_OK;
}
