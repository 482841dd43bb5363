// Reference ("oracle") implementation of the per-shard skip-gram negative-sampling step of the
// column-partitioned word2vec parameter server (Ordentlich et al., arXiv 1606.08495).
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, single-threaded CPU program that
// the GPU library is checked against.  It shares no code with the GPU library, is never tuned, and
// may only be used by the tests, by the smoke check and by the benchmark's "cpu_baseline" leg.
//
// What it follows in the paper:
//   * the dotprod server routine  (Appendix, algorithm "Server side computation - dotprod")
//   * the adjust server routine   (Appendix, algorithm "Server side computation - adjust")
//   * the client's aggregation    (Appendix, algorithm "Grid based word2vec", the two lines that
//                                  sum the partial dots and form G+ / G-)
//   * Eq.1 / Eq.3 (objective), Eq.4 (gradient), Eq.5 (update), Section 5.1 (column slices, and
//     the rule that adjust reads the vectors as they stood when the call began).
//   * Section 6.1.4 (vector export: the shards' partial vectors joined column-wise) and the
//     retrieval the vectors are trained for (Section 2, Section 7.3: top-K by cosine similarity).
//   * Section 5.1's two extensions: interleaved minibatch formation (last paragraph) and the
//     continuous-bag-of-words variant (footnote), the latter with the word2vec paper's model.
// Where the paper only names a seeded random number generator, or defers to the word2vec paper
// for the noise distribution and the subsampling rule, the readings taken are:
// Philox4x32-10 (Salmon et al., SC'11) as a counter-based generator, the unigram^0.75 noise
// distribution held in a Vose alias table, and the keep probability sqrt(t/f)+t/f.
//
// Floating point: every sum is accumulated in double, left to right, in the order the paper's
// loops visit the terms, and rounded to float once.  Build with -ffp-contract=off.
//
// Parity pins (tests/test_oracle_*.py): Philox known-answer vectors; brute-force tiny cases;
// closed forms for zero output vectors; finite differences of the objective; the column-slice
// invariant; chi-square of the sampler; alias-table reconstruction; window / subsample laws;
// for the bag-of-words variant a matrix formulation, finite differences, and its reduction to
// skip-gram when every example has one context word; for the retrieval, planar vectors with
// known angles, scaled basis vectors, and an independent library's cosine matrix.
// Nothing in this file is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

typedef unsigned __int128 u128;

// ---------------------------------------------------------------------------------------------
// Philox4x32-10.  One call maps a 128-bit counter and a 64-bit key to four 32-bit words.
// ---------------------------------------------------------------------------------------------
namespace {

struct Quad { uint32_t r[4]; };

Quad philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t seed) {
    uint32_t k0 = (uint32_t)(seed & 0xffffffffu);
    uint32_t k1 = (uint32_t)(seed >> 32);
    for (int round = 0; round < 10; ++round) {
        uint64_t prodA = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prodB = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prodB >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prodB;
        uint32_t n2 = (uint32_t)(prodA >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prodA;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Quad q; q.r[0] = c0; q.r[1] = c1; q.r[2] = c2; q.r[3] = c3;
    return q;
}

// The fourth counter word says what a draw is for, so that streams never collide.
const uint32_t DOMAIN_INIT   = 1;   // initial vector components
const uint32_t DOMAIN_TOKEN  = 2;   // per-token subsample decision and window width
const uint32_t DOMAIN_NEG    = 4;   // negative examples
const uint32_t DOMAIN_MBSEED = 5;   // the per-minibatch seed chosen by the client

// One initial component: word w, global column c of the full d_total-wide vector, matrix 0=U, 1=W.
// The draw depends on the global column so that column slices of a vector agree with the unsliced one.
float init_component(uint64_t seed, uint32_t w, uint32_t c, uint32_t matrix, uint32_t d_total) {
    Quad q = philox(w, c / 4, matrix, DOMAIN_INIT, seed);
    uint32_t bits = q.r[c % 4];
    float x = (float)(bits >> 8) * (1.0f / 16777216.0f) - 0.5f;   // exact: 24-bit fraction
    return x / (float)d_total;
}

// One candidate from the alias table.
uint32_t alias_candidate(uint64_t seed, uint32_t p, uint32_t slot, uint32_t attempt, uint32_t V,
                         const uint32_t* thresh, const uint32_t* alias) {
    Quad q = philox(p, slot, attempt, DOMAIN_NEG, seed);
    uint64_t r64 = ((uint64_t)q.r[1] << 32) | (uint64_t)q.r[0];
    uint32_t bin = (uint32_t)(((u128)r64 * (u128)V) >> 64);
    return (q.r[2] < thresh[bin]) ? bin : alias[bin];
}

// The negative for pair p, slot j in 1..k: first candidate that differs from the positive output
// word; after 16 rejected candidates, the next word index (cyclically).
uint32_t negative(uint64_t seed, uint32_t p, uint32_t j, uint32_t w_out, uint32_t V,
                  const uint32_t* thresh, const uint32_t* alias) {
    for (uint32_t attempt = 0; attempt < 16; ++attempt) {
        uint32_t cand = alias_candidate(seed, p, j, attempt, V, thresh, alias);
        if (cand != w_out) return cand;
    }
    return (uint32_t)(((uint64_t)w_out + 1) % V);
}

double sigmoid(double x) { return 1.0 / (1.0 + std::exp(-x)); }

// log sigma(x), the term of the objective (Eq.1; log(1 - sigma(x)) is log sigma(-x)).  Written as
// -log(1 + e^-x) on the side where e^-x is small and as x - log(1 + e^x) on the other, it is the
// same function as log(sigmoid(x)) but stays finite and accurate when sigma saturates.
double log_sigmoid(double x) {
    return x >= 0.0 ? -std::log1p(std::exp(-x)) : x - std::log1p(std::exp(x));
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------------------------
// Randomness
// ---------------------------------------------------------------------------------------------
void orc_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    Quad q = philox(ctr[0], ctr[1], ctr[2], ctr[3], ((uint64_t)key[1] << 32) | key[0]);
    for (int i = 0; i < 4; ++i) out[i] = q.r[i];
}

// Seed of minibatch number h (the client algorithm picks a fresh random seed per minibatch).
uint64_t orc_minibatch_seed(uint64_t master_seed, uint64_t h) {
    Quad q = philox((uint32_t)h, (uint32_t)(h >> 32), 0, DOMAIN_MBSEED, master_seed);
    return ((uint64_t)q.r[1] << 32) | (uint64_t)q.r[0];
}

// ---------------------------------------------------------------------------------------------
// Initial vectors (Section 5.1 defers to word2vec for the initial values): input vectors uniform in
// (-0.5/d, 0.5/d); the caller zeroes the output vectors when it wants the word2vec default.
// rows[m] lists the words wanted; out is [m][d_slice].
// ---------------------------------------------------------------------------------------------
void orc_init_rows(uint64_t seed, uint32_t d_total, uint32_t col_begin, uint32_t d_slice,
                   uint32_t matrix, const uint32_t* rows, uint64_t m, float* out) {
    for (uint64_t i = 0; i < m; ++i)
        for (uint32_t c = 0; c < d_slice; ++c)
            out[i * d_slice + c] = init_component(seed, rows[i], col_begin + c, matrix, d_total);
}

// ---------------------------------------------------------------------------------------------
// Noise distribution: weight of word w is count^0.75, written sqrt(sqrt(c*c*c)) so that only
// correctly rounded IEEE operations are involved.  probs[w] = weight / total.
// ---------------------------------------------------------------------------------------------
void orc_noise_probs(const uint64_t* counts, uint32_t V, double* probs) {
    double total = 0.0;
    for (uint32_t w = 0; w < V; ++w) {
        double c = (double)counts[w];
        probs[w] = std::sqrt(std::sqrt(c * c * c));
        total += probs[w];
    }
    for (uint32_t w = 0; w < V; ++w) probs[w] = probs[w] / total;
}

// Vose's alias method.  Bin w keeps itself with probability thresh[w]/2^32 and otherwise yields
// alias[w].  Work lists are filled in increasing word order and used last-in first-out.
void orc_build_alias(const uint64_t* counts, uint32_t V, uint32_t* thresh, uint32_t* alias) {
    std::vector<double> scaled(V);
    double total = 0.0;
    for (uint32_t w = 0; w < V; ++w) {
        double c = (double)counts[w];
        scaled[w] = std::sqrt(std::sqrt(c * c * c));
        total += scaled[w];
    }
    for (uint32_t w = 0; w < V; ++w) scaled[w] = (scaled[w] * (double)V) / total;

    std::vector<uint32_t> small, large;
    for (uint32_t w = 0; w < V; ++w) (scaled[w] < 1.0 ? small : large).push_back(w);

    const double two32 = 4294967296.0;
    for (uint32_t w = 0; w < V; ++w) { thresh[w] = 0xffffffffu; alias[w] = w; }
    while (!small.empty() && !large.empty()) {
        uint32_t s = small.back(); small.pop_back();
        uint32_t l = large.back(); large.pop_back();
        double t = std::floor(scaled[s] * two32);
        thresh[s] = (t >= two32 - 1.0) ? 0xffffffffu : (uint32_t)t;
        alias[s] = l;
        scaled[l] = (scaled[l] + scaled[s]) - 1.0;
        (scaled[l] < 1.0 ? small : large).push_back(l);
    }
    // Whatever is left keeps itself with certainty (already set above).
}

// Keep thresholds for subsampling: a token of word w survives when a uniform 32-bit draw is
// below keep_thresh[w]; 2^32 means "always".  keep = sqrt(t/f) + t/f with f the word's share.
void orc_build_keep(const uint64_t* counts, uint32_t V, double t, uint64_t* keep_thresh) {
    uint64_t total = 0;
    for (uint32_t w = 0; w < V; ++w) total += counts[w];
    for (uint32_t w = 0; w < V; ++w) {
        double f = (double)counts[w] / (double)total;
        double ratio = t / f;
        double keep = std::sqrt(ratio) + ratio;
        if (!(keep < 1.0)) keep_thresh[w] = (uint64_t)1 << 32;
        else keep_thresh[w] = (uint64_t)std::floor(keep * 4294967296.0);
    }
}

// ---------------------------------------------------------------------------------------------
// Negative examples (dotprod / adjust: N word indices different from the positive output word,
// drawn from the seeded generator).
// pair_ids == NULL means pairs 0..n-1; otherwise the negatives of the listed pair numbers
// (out_idx is then indexed by position in the list, not by pair number).
// neg is [n][k].
// ---------------------------------------------------------------------------------------------
void orc_negatives(const uint32_t* out_idx, const uint32_t* pair_ids, uint64_t n, uint32_t k,
                   uint64_t seed, uint32_t V, const uint32_t* thresh, const uint32_t* alias,
                   uint32_t* neg) {
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t p = pair_ids ? pair_ids[i] : (uint32_t)i;
        for (uint32_t j = 1; j <= k; ++j)
            neg[i * k + (j - 1)] = negative(seed, p, j, out_idx[i], V, thresh, alias);
    }
}

// ---------------------------------------------------------------------------------------------
// Partial dot products over a column slice.  rows is [n][T] (T = k+1): column 0 is the positive
// output word, columns 1..k the negatives.  U and W are dense [V][d] row-major.
// ---------------------------------------------------------------------------------------------
void orc_dots(const float* U, const float* W, uint32_t d, const uint32_t* in_idx,
              const uint32_t* rows, uint64_t n, uint32_t T, float* dots) {
    for (uint64_t p = 0; p < n; ++p) {
        const float* u = U + (uint64_t)in_idx[p] * d;
        for (uint32_t j = 0; j < T; ++j) {
            const float* v = W + (uint64_t)rows[p * T + j] * d;
            double acc = 0.0;
            for (uint32_t c = 0; c < d; ++c) acc += (double)u[c] * (double)v[c];
            dots[p * T + j] = (float)acc;
        }
    }
}

// The dotprod routine as the paper states it: seed the generator, draw the negatives, return the
// partial dots (F+ is column 0 of each row of `dots`, F- the other columns).
void orc_dotprod(const float* U, const float* W, uint32_t V, uint32_t d, const uint32_t* in_idx,
                 const uint32_t* out_idx, uint64_t n, uint32_t k, uint64_t seed,
                 const uint32_t* thresh, const uint32_t* alias, float* dots) {
    uint32_t T = k + 1;
    std::vector<uint32_t> rows(n * T);
    for (uint64_t p = 0; p < n; ++p) {
        rows[p * T] = out_idx[p];
        for (uint32_t j = 1; j <= k; ++j)
            rows[p * T + j] = negative(seed, (uint32_t)p, j, out_idx[p], V, thresh, alias);
    }
    orc_dots(U, W, d, in_idx, rows.data(), n, T, dots);
}

// ---------------------------------------------------------------------------------------------
// Client aggregation: sum the S partial-dot arrays, then the gradient coefficients
// (1 - sigma) for the positive slot and (-sigma) for a negative slot.  The learning rate is kept
// out of the coefficients here and applied by adjust; the product is the paper's G.
// loss (may be NULL) receives  - sum [ log sigma(f+) + sum log(1 - sigma(f-)) ].
// ---------------------------------------------------------------------------------------------
void orc_coeffs(const float* const* partial, uint32_t S, uint64_t n, uint32_t T, float* coeffs,
                double* loss) {
    double total_loss = 0.0;
    for (uint64_t p = 0; p < n; ++p) {
        for (uint32_t j = 0; j < T; ++j) {
            double f = 0.0;
            for (uint32_t s = 0; s < S; ++s) f += (double)partial[s][p * T + j];
            double sg = sigmoid(f);
            if (j == 0) { coeffs[p * T + j] = (float)(1.0 - sg); total_loss -= log_sigmoid(f); }
            else        { coeffs[p * T + j] = (float)(-sg);      total_loss -= log_sigmoid(-f); }
        }
    }
    if (loss) *loss = total_loss;
}

// ---------------------------------------------------------------------------------------------
// adjust, given the row lists.  All reads are of the vectors as they were when the call began;
// the summed changes are added at the end.  sequential_fp32 != 0 keeps the scratch sums in float
// (for information; the default double sum is the reference).
// ---------------------------------------------------------------------------------------------
typedef std::unordered_map<uint32_t, std::vector<double>> ScratchArea;   // word -> summed change

// The loop of the adjust routine: fills the scratch area (du per input word, dv per output word)
// from the start-of-call vectors, touching neither matrix.
static void adjust_accumulate(const float* U, const float* W, uint32_t d, const uint32_t* in_idx,
                              const uint32_t* rows, uint64_t n, uint32_t T, const float* coeffs,
                              int sequential_fp32, ScratchArea& dU, ScratchArea& dW) {
    for (uint64_t p = 0; p < n; ++p) {
        uint32_t wi = in_idx[p];
        const float* u = U + (uint64_t)wi * d;
        std::vector<double>& du = dU[wi];
        if (du.empty()) du.assign(d, 0.0);
        for (uint32_t j = 0; j < T; ++j) {
            uint32_t wo = rows[p * T + j];
            const float* v = W + (uint64_t)wo * d;
            std::vector<double>& dv = dW[wo];
            if (dv.empty()) dv.assign(d, 0.0);
            double g = (double)coeffs[p * T + j];
            for (uint32_t c = 0; c < d; ++c) {
                if (sequential_fp32) {
                    du[c] = (double)((float)du[c] + (float)g * v[c]);
                    dv[c] = (double)((float)dv[c] + (float)g * u[c]);
                } else {
                    du[c] += g * (double)v[c];
                    dv[c] += g * (double)u[c];
                }
            }
        }
    }
}

void orc_adjust_rows(float* U, float* W, uint32_t d, const uint32_t* in_idx, const uint32_t* rows,
                     uint64_t n, uint32_t T, const float* coeffs, float alpha,
                     int sequential_fp32) {
    ScratchArea dU, dW;
    adjust_accumulate(U, W, d, in_idx, rows, n, T, coeffs, sequential_fp32, dU, dW);
    for (auto& kv : dU) {
        float* u = U + (uint64_t)kv.first * d;
        for (uint32_t c = 0; c < d; ++c) u[c] = (float)((double)u[c] + (double)alpha * kv.second[c]);
    }
    for (auto& kv : dW) {
        float* v = W + (uint64_t)kv.first * d;
        for (uint32_t c = 0; c < d; ++c) v[c] = (float)((double)v[c] + (double)alpha * kv.second[c]);
    }
}

// Read-only view of the adjust routine's scratch area: the summed changes du, dv (double, before the
// learning rate is applied) of the listed words, zero for a word the minibatch does not touch.
// want_u[mu], want_w[mw] are word indices; dU_out is [mu][d], dW_out is [mw][d].  Changes nothing.
void orc_adjust_deltas(const float* U, const float* W, uint32_t d, const uint32_t* in_idx,
                       const uint32_t* rows, uint64_t n, uint32_t T, const float* coeffs,
                       const uint32_t* want_u, uint64_t mu, const uint32_t* want_w, uint64_t mw,
                       double* dU_out, double* dW_out) {
    ScratchArea dU, dW;
    adjust_accumulate(U, W, d, in_idx, rows, n, T, coeffs, 0, dU, dW);
    for (uint64_t i = 0; i < mu; ++i) {
        auto it = dU.find(want_u[i]);
        for (uint32_t c = 0; c < d; ++c) dU_out[i * d + c] = it == dU.end() ? 0.0 : it->second[c];
    }
    for (uint64_t i = 0; i < mw; ++i) {
        auto it = dW.find(want_w[i]);
        for (uint32_t c = 0; c < d; ++c) dW_out[i * d + c] = it == dW.end() ? 0.0 : it->second[c];
    }
}

// The adjust routine as the paper states it: re-seed, regenerate the same negatives, accumulate
// the changes from the start-of-call vectors, add them at the end.
void orc_adjust(float* U, float* W, uint32_t V, uint32_t d, const uint32_t* in_idx,
                const uint32_t* out_idx, uint64_t n, uint32_t k, uint64_t seed,
                const uint32_t* thresh, const uint32_t* alias, const float* coeffs, float alpha) {
    uint32_t T = k + 1;
    std::vector<uint32_t> rows(n * T);
    for (uint64_t p = 0; p < n; ++p) {
        rows[p * T] = out_idx[p];
        for (uint32_t j = 1; j <= k; ++j)
            rows[p * T + j] = negative(seed, (uint32_t)p, j, out_idx[p], V, thresh, alias);
    }
    orc_adjust_rows(U, W, d, in_idx, rows.data(), n, T, coeffs, alpha, 0);
}

// One client step over S column shards held in this process: dotprod on every shard, aggregate,
// adjust on every shard.  Us[s], Ws[s] are dense [V][ds[s]].
void orc_train_minibatch(float* const* Us, float* const* Ws, const uint32_t* ds, uint32_t S,
                         uint32_t V, const uint32_t* in_idx, const uint32_t* out_idx, uint64_t n,
                         uint32_t k, uint64_t seed, const uint32_t* thresh, const uint32_t* alias,
                         float alpha, double* loss) {
    uint32_t T = k + 1;
    std::vector<std::vector<float>> partial(S, std::vector<float>(n * T));
    std::vector<const float*> ptrs(S);
    for (uint32_t s = 0; s < S; ++s) {
        orc_dotprod(Us[s], Ws[s], V, ds[s], in_idx, out_idx, n, k, seed, thresh, alias,
                    partial[s].data());
        ptrs[s] = partial[s].data();
    }
    std::vector<float> coeffs(n * T);
    orc_coeffs(ptrs.data(), S, n, T, coeffs.data(), loss);
    for (uint32_t s = 0; s < S; ++s)
        orc_adjust(Us[s], Ws[s], V, ds[s], in_idx, out_idx, n, k, seed, thresh, alias,
                   coeffs.data(), alpha);
}

// ---------------------------------------------------------------------------------------------
// The same step on a vocabulary too large to hold densely on the host: rows are created on first
// touch from the initialisation function (which is a pure function of word and column), and kept
// in a map.  Used only to time the oracle on large-vocabulary workloads and to check sampled
// outputs; the arithmetic is the dense routines above applied to a compacted copy.
// ---------------------------------------------------------------------------------------------
struct LazyShard {
    uint64_t seed; uint32_t V, d_total, col_begin, d; int w_uniform;
    std::unordered_map<uint32_t, std::vector<float>> U, W;
};

void* orc_lazy_create(uint32_t V, uint32_t d_total, uint32_t col_begin, uint32_t d_slice,
                      uint64_t seed, int w_uniform) {
    LazyShard* sh = new LazyShard();
    sh->seed = seed; sh->V = V; sh->d_total = d_total; sh->col_begin = col_begin;
    sh->d = d_slice; sh->w_uniform = w_uniform;
    return sh;
}
void orc_lazy_destroy(void* h) { delete (LazyShard*)h; }

static std::vector<float>& lazy_row(LazyShard* sh, int which, uint32_t w) {
    auto& table = which ? sh->W : sh->U;
    auto it = table.find(w);
    if (it != table.end()) return it->second;
    std::vector<float> row(sh->d, 0.0f);
    if (which == 0 || sh->w_uniform)
        orc_init_rows(sh->seed, sh->d_total, sh->col_begin, sh->d, (uint32_t)which, &w, 1, row.data());
    return table.emplace(w, std::move(row)).first->second;
}

void orc_lazy_get_row(void* h, int which, uint32_t w, float* out) {
    LazyShard* sh = (LazyShard*)h;
    std::vector<float>& r = lazy_row(sh, which, w);
    std::memcpy(out, r.data(), sizeof(float) * sh->d);
}

uint64_t orc_lazy_rows_held(void* h) {
    LazyShard* sh = (LazyShard*)h;
    return sh->U.size() + sh->W.size();
}

// train_minibatch on one lazy shard: compact the touched rows, run the dense routines, copy back.
void orc_lazy_train_minibatch(void* h, const uint32_t* in_idx, const uint32_t* out_idx, uint64_t n,
                              uint32_t k, uint64_t seed, const uint32_t* thresh,
                              const uint32_t* alias, float alpha, double* loss) {
    LazyShard* sh = (LazyShard*)h;
    uint32_t T = k + 1, d = sh->d;
    std::vector<uint32_t> rows(n * T), cin(n), crows(n * T);
    std::unordered_map<uint32_t, uint32_t> idU, idW;
    std::vector<uint32_t> wordsU, wordsW;
    for (uint64_t p = 0; p < n; ++p) {
        rows[p * T] = out_idx[p];
        for (uint32_t j = 1; j <= k; ++j)
            rows[p * T + j] = negative(seed, (uint32_t)p, j, out_idx[p], sh->V, thresh, alias);
        auto r = idU.emplace(in_idx[p], (uint32_t)wordsU.size());
        if (r.second) wordsU.push_back(in_idx[p]);
        cin[p] = r.first->second;
        for (uint32_t j = 0; j < T; ++j) {
            auto q = idW.emplace(rows[p * T + j], (uint32_t)wordsW.size());
            if (q.second) wordsW.push_back(rows[p * T + j]);
            crows[p * T + j] = q.first->second;
        }
    }
    std::vector<float> Uc(wordsU.size() * (size_t)d), Wc(wordsW.size() * (size_t)d);
    for (size_t i = 0; i < wordsU.size(); ++i)
        std::memcpy(&Uc[i * d], lazy_row(sh, 0, wordsU[i]).data(), sizeof(float) * d);
    for (size_t i = 0; i < wordsW.size(); ++i)
        std::memcpy(&Wc[i * d], lazy_row(sh, 1, wordsW[i]).data(), sizeof(float) * d);

    std::vector<float> dots(n * T), coeffs(n * T);
    orc_dots(Uc.data(), Wc.data(), d, cin.data(), crows.data(), n, T, dots.data());
    const float* one[1] = { dots.data() };
    orc_coeffs(one, 1, n, T, coeffs.data(), loss);
    orc_adjust_rows(Uc.data(), Wc.data(), d, cin.data(), crows.data(), n, T, coeffs.data(), alpha, 0);

    for (size_t i = 0; i < wordsU.size(); ++i)
        std::memcpy(lazy_row(sh, 0, wordsU[i]).data(), &Uc[i * d], sizeof(float) * d);
    for (size_t i = 0; i < wordsW.size(); ++i)
        std::memcpy(lazy_row(sh, 1, wordsW[i]).data(), &Wc[i * d], sizeof(float) * d);
}

// ---------------------------------------------------------------------------------------------
// Pair generation (Eq.1's index sets; footnote on "dirty" contexts).  For every sentence: drop
// tokens by the subsample rule, then for each surviving center draw a half-width b in 1..B and
// emit (center, context) for the surviving neighbours within b positions, contexts in increasing
// position.  The draws of a token depend only on its global position in the corpus and the epoch.
// sent_off[n_sent+1] are token offsets relative to tokens[0]; token_base is the global position
// of tokens[0].  keep_thresh == NULL disables subsampling.  Returns the number of pairs; writes at
// most `capacity` of them.
// ---------------------------------------------------------------------------------------------
uint64_t orc_make_pairs(const uint32_t* tokens, const uint64_t* sent_off, uint64_t n_sent,
                        uint64_t token_base, uint32_t epoch, uint64_t corpus_seed, uint32_t B,
                        const uint64_t* keep_thresh, uint32_t* in_idx, uint32_t* out_idx,
                        uint64_t capacity) {
    uint64_t count = 0;
    std::vector<uint32_t> kept_word;
    std::vector<uint32_t> kept_b;
    for (uint64_t s = 0; s < n_sent; ++s) {
        kept_word.clear(); kept_b.clear();
        for (uint64_t t = sent_off[s]; t < sent_off[s + 1]; ++t) {
            uint64_t g = token_base + t;
            Quad q = philox((uint32_t)g, (uint32_t)(g >> 32), epoch, DOMAIN_TOKEN, corpus_seed);
            uint32_t w = tokens[t];
            bool keep = keep_thresh ? ((uint64_t)q.r[0] < keep_thresh[w]) : true;
            if (!keep) continue;
            kept_word.push_back(w);
            kept_b.push_back(1 + (uint32_t)(((uint64_t)q.r[1] * (uint64_t)B) >> 32));
        }
        int64_t m = (int64_t)kept_word.size();
        for (int64_t j = 0; j < m; ++j) {
            int64_t b = (int64_t)kept_b[j];
            for (int64_t c = j - b; c <= j + b; ++c) {
                if (c == j || c < 0 || c >= m) continue;
                if (count < capacity) { in_idx[count] = kept_word[j]; out_idx[count] = kept_word[c]; }
                ++count;
            }
        }
    }
    return count;
}

// Interleaved minibatch formation (Section 5.1, last paragraph: an option that keeps the input words
// of one minibatch far apart in the corpus, ideally in different sentences).  Reading taken here:
// the same pairs as orc_make_pairs, but the centers are visited round-robin over the sentences of
// the token block -- first every sentence's first surviving token (in sentence order), then every
// sentence's second, and so on -- so that a minibatch cut from the pair stream takes at most a few
// centers from any one sentence.  The contexts of a center keep their order.
uint64_t orc_make_pairs_interleaved(const uint32_t* tokens, const uint64_t* sent_off,
                                    uint64_t n_sent, uint64_t token_base, uint32_t epoch,
                                    uint64_t corpus_seed, uint32_t B, const uint64_t* keep_thresh,
                                    uint32_t* in_idx, uint32_t* out_idx, uint64_t capacity) {
    struct Center { uint64_t sentence; int64_t j; };
    std::vector<std::vector<uint32_t>> words(n_sent), widths(n_sent);
    std::vector<Center> centers;
    for (uint64_t s = 0; s < n_sent; ++s) {
        for (uint64_t t = sent_off[s]; t < sent_off[s + 1]; ++t) {
            uint64_t g = token_base + t;
            Quad q = philox((uint32_t)g, (uint32_t)(g >> 32), epoch, DOMAIN_TOKEN, corpus_seed);
            uint32_t w = tokens[t];
            bool keep = keep_thresh ? ((uint64_t)q.r[0] < keep_thresh[w]) : true;
            if (!keep) continue;
            centers.push_back(Center{s, (int64_t)words[s].size()});
            words[s].push_back(w);
            widths[s].push_back(1 + (uint32_t)(((uint64_t)q.r[1] * (uint64_t)B) >> 32));
        }
    }
    // by position within the sentence; sentences stay in order among equal positions
    std::stable_sort(centers.begin(), centers.end(),
                     [](const Center& a, const Center& b) { return a.j < b.j; });
    uint64_t count = 0;
    for (const Center& ce : centers) {
        const std::vector<uint32_t>& sw = words[ce.sentence];
        int64_t m = (int64_t)sw.size(), j = ce.j, b = (int64_t)widths[ce.sentence][j];
        for (int64_t c = j - b; c <= j + b; ++c) {
            if (c == j || c < 0 || c >= m) continue;
            if (count < capacity) { in_idx[count] = sw[j]; out_idx[count] = sw[c]; }
            ++count;
        }
    }
    return count;
}

// ---------------------------------------------------------------------------------------------
// Continuous-bag-of-words variant (Section 5.1, footnote: the same architecture carries over to
// it; the model itself is the word2vec paper's).  An example p has a center word out_idx[p], which
// plays the output role, and the list of its context words ctx_idx[ctx_off[p] .. ctx_off[p+1]),
// which play the input role.  The hidden vector is the mean of the context words' input vectors,
//     h_p = (1/|C_p|) sum_{c in C_p} u_c ,
// and the objective is Eq.1's with u replaced by h:  log sigma(h.v_center) + sum log sigma(-h.v_neg).
// A column slice of h is the mean of the column slices, so the partial dots of the shards still
// add up (Eq.3's decomposition), and the update is gradient ascent as in Eq.4 / Eq.5:
//     v_row += alpha * g * h              (row = center or negative, g its coefficient)
//     u_c   += alpha * (1/|C_p|) * sum_j g_j v_row_j     for every occurrence c in C_p
// (the exact derivative of the mean; a word that occurs twice in C_p receives it twice).
// An example with no context has h = 0: zero dots, no change.
// ---------------------------------------------------------------------------------------------
void orc_cbow_dots(const float* U, const float* W, uint32_t d, const uint32_t* ctx_off,
                   const uint32_t* ctx_idx, const uint32_t* rows, uint64_t n, uint32_t T,
                   float* dots) {
    std::vector<double> h(d);
    for (uint64_t p = 0; p < n; ++p) {
        uint32_t lo = ctx_off[p], hi = ctx_off[p + 1];
        std::fill(h.begin(), h.end(), 0.0);
        for (uint32_t e = lo; e < hi; ++e) {
            const float* u = U + (uint64_t)ctx_idx[e] * d;
            for (uint32_t c = 0; c < d; ++c) h[c] += (double)u[c];
        }
        if (hi > lo) for (uint32_t c = 0; c < d; ++c) h[c] /= (double)(hi - lo);
        for (uint32_t j = 0; j < T; ++j) {
            const float* v = W + (uint64_t)rows[p * T + j] * d;
            double acc = 0.0;
            for (uint32_t c = 0; c < d; ++c) acc += h[c] * (double)v[c];
            dots[p * T + j] = (float)acc;
        }
    }
}

void orc_cbow_adjust_rows(float* U, float* W, uint32_t d, const uint32_t* ctx_off,
                          const uint32_t* ctx_idx, const uint32_t* rows, uint64_t n, uint32_t T,
                          const float* coeffs, float alpha) {
    std::unordered_map<uint32_t, std::vector<double>> dU, dW;   // the scratch area
    std::vector<double> h(d), e(d);
    for (uint64_t p = 0; p < n; ++p) {
        uint32_t lo = ctx_off[p], hi = ctx_off[p + 1];
        std::fill(h.begin(), h.end(), 0.0);
        std::fill(e.begin(), e.end(), 0.0);
        for (uint32_t x = lo; x < hi; ++x) {
            const float* u = U + (uint64_t)ctx_idx[x] * d;
            for (uint32_t c = 0; c < d; ++c) h[c] += (double)u[c];
        }
        if (hi > lo) for (uint32_t c = 0; c < d; ++c) h[c] /= (double)(hi - lo);
        for (uint32_t j = 0; j < T; ++j) {
            uint32_t wo = rows[p * T + j];
            const float* v = W + (uint64_t)wo * d;
            std::vector<double>& dv = dW[wo];
            if (dv.empty()) dv.assign(d, 0.0);
            double g = (double)coeffs[p * T + j];
            for (uint32_t c = 0; c < d; ++c) {
                e[c] += g * (double)v[c];
                dv[c] += g * h[c];
            }
        }
        for (uint32_t x = lo; x < hi; ++x) {
            std::vector<double>& du = dU[ctx_idx[x]];
            if (du.empty()) du.assign(d, 0.0);
            for (uint32_t c = 0; c < d; ++c) du[c] += e[c] / (double)(hi - lo);
        }
    }
    for (auto& kv : dU) {
        float* u = U + (uint64_t)kv.first * d;
        for (uint32_t c = 0; c < d; ++c) u[c] = (float)((double)u[c] + (double)alpha * kv.second[c]);
    }
    for (auto& kv : dW) {
        float* v = W + (uint64_t)kv.first * d;
        for (uint32_t c = 0; c < d; ++c) v[c] = (float)((double)v[c] + (double)alpha * kv.second[c]);
    }
}

static void cbow_rows(const uint32_t* out_idx, uint64_t n, uint32_t k, uint64_t seed, uint32_t V,
                      const uint32_t* thresh, const uint32_t* alias, std::vector<uint32_t>& rows) {
    uint32_t T = k + 1;
    rows.resize(n * T);
    for (uint64_t p = 0; p < n; ++p) {
        rows[p * T] = out_idx[p];
        for (uint32_t j = 1; j <= k; ++j)
            rows[p * T + j] = negative(seed, (uint32_t)p, j, out_idx[p], V, thresh, alias);
    }
}

// The two server calls and the client step, with the negatives drawn exactly as for skip-gram
// (k words different from the example's center word, from the seed).
void orc_cbow_dotprod(const float* U, const float* W, uint32_t V, uint32_t d,
                      const uint32_t* ctx_off, const uint32_t* ctx_idx, const uint32_t* out_idx,
                      uint64_t n, uint32_t k, uint64_t seed, const uint32_t* thresh,
                      const uint32_t* alias, float* dots) {
    std::vector<uint32_t> rows;
    cbow_rows(out_idx, n, k, seed, V, thresh, alias, rows);
    orc_cbow_dots(U, W, d, ctx_off, ctx_idx, rows.data(), n, k + 1, dots);
}

void orc_cbow_adjust(float* U, float* W, uint32_t V, uint32_t d, const uint32_t* ctx_off,
                     const uint32_t* ctx_idx, const uint32_t* out_idx, uint64_t n, uint32_t k,
                     uint64_t seed, const uint32_t* thresh, const uint32_t* alias,
                     const float* coeffs, float alpha) {
    std::vector<uint32_t> rows;
    cbow_rows(out_idx, n, k, seed, V, thresh, alias, rows);
    orc_cbow_adjust_rows(U, W, d, ctx_off, ctx_idx, rows.data(), n, k + 1, coeffs, alpha);
}

void orc_cbow_train_minibatch(float* const* Us, float* const* Ws, const uint32_t* ds, uint32_t S,
                              uint32_t V, const uint32_t* ctx_off, const uint32_t* ctx_idx,
                              const uint32_t* out_idx, uint64_t n, uint32_t k, uint64_t seed,
                              const uint32_t* thresh, const uint32_t* alias, float alpha,
                              double* loss) {
    uint32_t T = k + 1;
    std::vector<std::vector<float>> partial(S, std::vector<float>(n * T));
    std::vector<const float*> ptrs(S);
    for (uint32_t s = 0; s < S; ++s) {
        orc_cbow_dotprod(Us[s], Ws[s], V, ds[s], ctx_off, ctx_idx, out_idx, n, k, seed, thresh,
                         alias, partial[s].data());
        ptrs[s] = partial[s].data();
    }
    std::vector<float> coeffs(n * T);
    orc_coeffs(ptrs.data(), S, n, T, coeffs.data(), loss);
    for (uint32_t s = 0; s < S; ++s)
        orc_cbow_adjust(Us[s], Ws[s], V, ds[s], ctx_off, ctx_idx, out_idx, n, k, seed, thresh,
                        alias, coeffs.data(), alpha);
}

// Examples from text: the same subsampling and window draws as orc_make_pairs; every surviving
// center with at least one surviving neighbour in its window gives one example whose contexts are
// those neighbours in increasing position.  Returns the number of examples, *n_ctx the number of
// context entries; writes at most cap_examples / cap_ctx of them (ctx_off is filled for the examples
// written, plus the closing offset).
uint64_t orc_make_cbow_examples(const uint32_t* tokens, const uint64_t* sent_off, uint64_t n_sent,
                                uint64_t token_base, uint32_t epoch, uint64_t corpus_seed,
                                uint32_t B, const uint64_t* keep_thresh, uint32_t* ctx_off,
                                uint32_t* ctx_idx, uint32_t* out_idx, uint64_t cap_examples,
                                uint64_t cap_ctx, uint64_t* n_ctx) {
    uint64_t examples = 0, entries = 0;
    ctx_off[0] = 0;
    std::vector<uint32_t> kept_word, kept_b;
    for (uint64_t s = 0; s < n_sent; ++s) {
        kept_word.clear(); kept_b.clear();
        for (uint64_t t = sent_off[s]; t < sent_off[s + 1]; ++t) {
            uint64_t g = token_base + t;
            Quad q = philox((uint32_t)g, (uint32_t)(g >> 32), epoch, DOMAIN_TOKEN, corpus_seed);
            uint32_t w = tokens[t];
            bool keep = keep_thresh ? ((uint64_t)q.r[0] < keep_thresh[w]) : true;
            if (!keep) continue;
            kept_word.push_back(w);
            kept_b.push_back(1 + (uint32_t)(((uint64_t)q.r[1] * (uint64_t)B) >> 32));
        }
        int64_t m = (int64_t)kept_word.size();
        for (int64_t j = 0; j < m; ++j) {
            int64_t b = (int64_t)kept_b[j];
            int64_t lo = std::max<int64_t>(0, j - b), hi = std::min<int64_t>(m - 1, j + b);
            if (hi - lo == 0) continue;                   // no neighbour survives
            for (int64_t c = lo; c <= hi; ++c) {
                if (c == j) continue;
                if (entries < cap_ctx) ctx_idx[entries] = kept_word[c];
                ++entries;
            }
            if (examples < cap_examples) {
                out_idx[examples] = kept_word[j];
                ctx_off[examples + 1] = (uint32_t)entries;
            }
            ++examples;
        }
    }
    *n_ctx = entries;
    return examples;
}

// Per-token view of the same decisions, for the statistical pins: keep[t] in {0,1}, b[t].
void orc_token_draws(const uint32_t* tokens, uint64_t n_tokens, uint64_t token_base, uint32_t epoch,
                     uint64_t corpus_seed, uint32_t B, const uint64_t* keep_thresh, uint8_t* keep,
                     uint32_t* b) {
    for (uint64_t t = 0; t < n_tokens; ++t) {
        uint64_t g = token_base + t;
        Quad q = philox((uint32_t)g, (uint32_t)(g >> 32), epoch, DOMAIN_TOKEN, corpus_seed);
        keep[t] = keep_thresh ? (uint8_t)((uint64_t)q.r[0] < keep_thresh[tokens[t]]) : (uint8_t)1;
        b[t] = 1 + (uint32_t)(((uint64_t)q.r[1] * (uint64_t)B) >> 32);
    }
}

// ---------------------------------------------------------------------------------------------
// Retrieval by cosine similarity (Section 2: the K candidates most similar to a query vector are
// retrieved; Section 7.3: K = 30, and only similarities above a threshold tau are kept).
// Qm is [Q][d], Cm is [N][d], both dense row-major.  For query q the similarity with candidate c is
//     (q . c) / (|q| |c|)          (0 when either vector is all zeros),
// everything in double.  The candidates are ranked by decreasing similarity, equal similarities by
// increasing index; the first K with similarity > tau are returned: idx[q][0..count[q]) and
// score[q][0..count[q]), the rest of the K slots filled with 0xFFFFFFFF and 0.
// ---------------------------------------------------------------------------------------------
void orc_topk_cosine(const float* Qm, uint32_t Q, const float* Cm, uint32_t N, uint32_t d,
                     uint32_t K, double tau, uint32_t* idx, double* score, uint32_t* count) {
    std::vector<double> cnorm(N);
    for (uint32_t c = 0; c < N; ++c) {
        double s = 0.0;
        for (uint32_t i = 0; i < d; ++i) s += (double)Cm[(uint64_t)c * d + i] * (double)Cm[(uint64_t)c * d + i];
        cnorm[c] = std::sqrt(s);
    }
    std::vector<double> sim(N);
    std::vector<uint32_t> order(N);
    for (uint32_t q = 0; q < Q; ++q) {
        const float* qv = Qm + (uint64_t)q * d;
        double qs = 0.0;
        for (uint32_t i = 0; i < d; ++i) qs += (double)qv[i] * (double)qv[i];
        double qnorm = std::sqrt(qs);
        for (uint32_t c = 0; c < N; ++c) {
            const float* cv = Cm + (uint64_t)c * d;
            double dot = 0.0;
            for (uint32_t i = 0; i < d; ++i) dot += (double)qv[i] * (double)cv[i];
            sim[c] = (qnorm > 0.0 && cnorm[c] > 0.0) ? dot / (qnorm * cnorm[c]) : 0.0;
            order[c] = c;
        }
        std::stable_sort(order.begin(), order.end(),
                         [&](uint32_t a, uint32_t b) { return sim[a] > sim[b]; });
        uint32_t kept = 0;
        for (uint32_t r = 0; r < K; ++r) {
            bool ok = r < N && sim[order[r]] > tau;
            idx[(uint64_t)q * K + r] = ok ? order[r] : 0xFFFFFFFFu;
            score[(uint64_t)q * K + r] = ok ? sim[order[r]] : 0.0;
            if (ok) ++kept;
        }
        count[q] = kept;
    }
}

}  // extern "C"
