"""Seeded synthetic inputs for the word2vec shard path (numpy only).

This module produces *inputs* -- token streams, sentence boundaries, vocabulary counts, (input,
output) index pairs, coefficient arrays -- with the shapes and distributions of the paper's
workloads (Section 6.2: very large vocabularies of generalized words, Zipf-like frequencies,
sessions of a few tens of tokens).  It holds none of the method's arithmetic: no negative
sampling, no subsampling, no windows, no dot products.  The GPU library and the CPU oracle are
both driven from the arrays made here.

Word id == frequency rank (Section 5.1: the vocabulary is ordered by decreasing frequency).
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One of the benchmark shapes.  ``d_slice`` columns [col_begin, col_begin+d_slice) of d_total."""
    name: str
    V: int
    d_total: int
    col_begin: int
    d_slice: int
    zipf_s: float
    n_pairs: int          # pairs per minibatch
    k: int                # negatives per pair
    window: int           # per-side maximum B
    sent_min: int
    sent_max: int
    corpus_tokens: int
    subsample_t: float    # 0 disables subsampling
    alpha: float
    alpha_min: float
    w_uniform: bool       # False: output vectors start at zero (word2vec default)
    seed: int
    pairs_from_corpus: bool   # False: (in,out) drawn iid from the Zipf law


WORKLOADS = {
    "tiny": Workload("tiny", 10_000, 100, 0, 100, 1.0, 4096, 5, 5, 20, 20, 200_000, 1e-4,
                     0.025, 0.025, False, 1, True),
    "slice60": Workload("slice60", 1_000_000, 300, 0, 60, 1.0, 1 << 20, 5, 5, 20, 20,
                        1_000_000_000, 0.0, 0.025, 0.025, True, 2, False),
    "full300": Workload("full300", 10_000_000, 300, 0, 300, 1.05, 1 << 20, 5, 10, 30, 30,
                        500_000_000, 1e-5, 0.025, 1e-4, False, 3, True),
    "search200m": Workload("search200m", 200_000_000, 300, 0, 60, 0.9, 1 << 21, 10, 5, 10, 40,
                           2_000_000_000, 0.0, 0.025, 0.025, False, 4, True),
    "stress25": Workload("stress25", 50_000_000, 200, 0, 200, 1.2, 1 << 22, 25, 8, 30, 30,
                         1_000_000_000, 0.0, 0.025, 0.025, False, 5, True),
}


def zipf_cdf(V, s):
    """Cumulative distribution of p_r ~ r^-s over ranks 1..V (float64, last entry exactly 1)."""
    r = np.arange(1, V + 1, dtype=np.float64)
    w = r ** (-float(s))
    c = np.cumsum(w)
    c /= c[-1]
    c[-1] = 1.0
    return c


def zipf_probs(V, s):
    r = np.arange(1, V + 1, dtype=np.float64)
    w = r ** (-float(s))
    return w / w.sum()


def zipf_draw(cdf, n, rng):
    """n word ids (uint32) from the law whose cumulative table is ``cdf``."""
    out = np.empty(n, np.uint32)
    step = 1 << 22
    for a in range(0, n, step):
        b = min(n, a + step)
        u = rng.random(b - a)
        out[a:b] = np.minimum(np.searchsorted(cdf, u, side="right"), cdf.size - 1)
    return out


def analytic_counts(V, s, corpus_tokens):
    """Expected occurrence counts max(1, round(N p_r)) -- stands in for a counted histogram."""
    p = zipf_probs(V, s)
    return np.maximum(1, np.rint(p * float(corpus_tokens))).astype(np.uint64)


def counted(tokens, V):
    return np.bincount(tokens, minlength=V).astype(np.uint64)


def sentence_offsets(n_tokens, lo, hi, rng):
    """Token offsets of consecutive sentences with lengths uniform on lo..hi (last one clipped)."""
    if lo == hi:
        off = np.arange(0, n_tokens + lo, lo, dtype=np.uint64)
        off = off[off <= n_tokens]
        if off[-1] != n_tokens:
            off = np.append(off, np.uint64(n_tokens))
        return off
    est = int(n_tokens / ((lo + hi) / 2.0) * 1.2) + 16
    lens = rng.integers(lo, hi + 1, size=est)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = off[off < n_tokens]
    off = np.append(off, n_tokens)
    return off.astype(np.uint64)


def corpus(wl, n_tokens=None, seed=None, cdf=None):
    """(tokens uint32[n], sentence offsets uint64[m+1]) shaped like ``wl``; n_tokens may be a slice
    of the nominal corpus size."""
    n = int(wl.corpus_tokens if n_tokens is None else n_tokens)
    rng = np.random.Generator(np.random.PCG64(wl.seed if seed is None else seed))
    if cdf is None:
        cdf = zipf_cdf(wl.V, wl.zipf_s)
    tokens = zipf_draw(cdf, n, rng)
    off = sentence_offsets(n, wl.sent_min, wl.sent_max, rng)
    return tokens, off


def iid_pairs(wl, n=None, seed=None, cdf=None):
    """(in_idx, out_idx), each iid from the workload's Zipf law (the single-slice shard shape)."""
    n = int(wl.n_pairs if n is None else n)
    rng = np.random.Generator(np.random.PCG64((wl.seed if seed is None else seed) + 1000))
    if cdf is None:
        cdf = zipf_cdf(wl.V, wl.zipf_s)
    return zipf_draw(cdf, n, rng), zipf_draw(cdf, n, rng)


def embedding_like(n, d, seed, n_clusters=1000, spread=0.6, cluster_seed=0):
    """n vectors of width d shaped like trained embeddings: a cluster direction (one of n_clusters
    drawn from ``cluster_seed``, Zipf-popular) plus isotropic unit-variance noise times ``spread``,
    with log-normal lengths.  Calls with the same cluster_seed share the directions, so queries
    generated by one call have close neighbours among candidates generated by another.
    float32 [n, d]."""
    crng = np.random.Generator(np.random.PCG64(cluster_seed + 5000))
    centers = crng.standard_normal((n_clusters, d)).astype(np.float32)
    rng = np.random.Generator(np.random.PCG64(seed + 4000))
    which = zipf_draw(zipf_cdf(n_clusters, 1.0), n, rng)
    length = (np.exp(0.3 * rng.standard_normal(n)) / np.sqrt(d)).astype(np.float32)
    x = np.empty((n, d), np.float32)
    step = 1 << 16                                   # in slices: no second array of the full size
    for a in range(0, n, step):
        b = min(n, a + step)
        part = rng.random((b - a, d), dtype=np.float32)
        part -= np.float32(0.5)
        part *= np.float32(spread * np.sqrt(12.0))
        part += centers[which[a:b]]
        part *= length[a:b, None]
        x[a:b] = part
    return x


def uniform_coeffs(n, T, seed):
    """Harness-supplied coefficients uniform(-1, 1), float32 [n, T]."""
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    return (rng.random((n, T), dtype=np.float32) * 2.0 - 1.0).astype(np.float32)


def alpha_schedule(wl, h, H):
    """Learning rate of minibatch h of H: linear from alpha to alpha_min (constant when equal)."""
    a = wl.alpha - (wl.alpha - wl.alpha_min) * (float(h) / float(max(H, 1)))
    return float(np.float32(a))
