// Host-side construction of the noise (alias) table and the subsample keep thresholds from a
// vocabulary histogram.  Compiled without floating-point contraction: every value below comes from
// correctly rounded IEEE double operations (*, /, +, -, sqrt, floor), so any conforming
// implementation of the same recipe produces the same integers.
//
// Recipe (Section 3 of arXiv 1606.08495 defers to word2vec for both laws):
//   noise weight of word w     q_w = sqrt(sqrt(c_w^3))            (c_w^0.75)
//   scaled probability         s_w = q_w * V / sum(q), the sum taken in word order
//   Vose's alias method with two stacks, filled in word order and popped from the top:
//       words with s_w < 1 go to `small`, the others to `large`;
//       pop s, pop l: bin s keeps itself with probability s_s and otherwise yields l;
//       s_l <- (s_l + s_s) - 1 and l is pushed again on the stack its new value selects
//   keep threshold of a bin = min(2^32 - 1, floor(s * 2^32)); bins left on either stack keep
//   themselves always (threshold 2^32 - 1, alias = self)
//   subsample keep probability min(1, sqrt(t/f) + t/f), f = c_w / sum(c); threshold
//   floor(keep * 2^32) as 64-bit, 2^32 meaning "always keep"
#include <cmath>
#include <cstdint>
#include <memory>
#include <new>

namespace w2v {

bool build_noise_table_host(const uint64_t* counts, uint32_t V, uint32_t* thresh, uint32_t* alias) {
    std::unique_ptr<double[]> s(new (std::nothrow) double[V]);
    std::unique_ptr<uint32_t[]> stack_small(new (std::nothrow) uint32_t[V]);
    std::unique_ptr<uint32_t[]> stack_large(new (std::nothrow) uint32_t[V]);
    if (!s || !stack_small || !stack_large) return false;

    double sum = 0.0;
    for (uint32_t w = 0; w < V; ++w) {
        const double c = (double)counts[w];
        const double cube = c * c * c;
        s[w] = std::sqrt(std::sqrt(cube));
        sum += s[w];
    }
    const double Vd = (double)V;
    size_t ns = 0, nl = 0;
    for (uint32_t w = 0; w < V; ++w) {
        const double scaled = (s[w] * Vd) / sum;
        s[w] = scaled;
        thresh[w] = 0xFFFFFFFFu;
        alias[w] = w;
        if (scaled < 1.0) stack_small[ns++] = w; else stack_large[nl++] = w;
    }
    const double two32 = 4294967296.0;
    while (ns > 0 && nl > 0) {
        const uint32_t a = stack_small[--ns];
        const uint32_t b = stack_large[--nl];
        const double fl = std::floor(s[a] * two32);
        thresh[a] = fl >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)fl;
        alias[a] = b;
        const double rest = (s[b] + s[a]) - 1.0;
        s[b] = rest;
        if (rest < 1.0) stack_small[ns++] = b; else stack_large[nl++] = b;
    }
    return true;
}

void build_keep_thresholds_host(const uint64_t* counts, uint32_t V, double t, uint64_t* keep) {
    const uint64_t always = (uint64_t)1 << 32;
    if (!(t > 0.0)) {
        for (uint32_t w = 0; w < V; ++w) keep[w] = always;
        return;
    }
    uint64_t total = 0;
    for (uint32_t w = 0; w < V; ++w) total += counts[w];
    const double totald = (double)total;
    for (uint32_t w = 0; w < V; ++w) {
        const double f = (double)counts[w] / totald;
        const double r = t / f;
        const double p = std::sqrt(r) + r;
        keep[w] = (p < 1.0) ? (uint64_t)std::floor(p * 4294967296.0) : always;
    }
}

}  // namespace w2v
