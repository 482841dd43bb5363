"""Pins of the oracle's integer side: the noise table, the negative sampler, the subsample rule and
the window law -- against exact bounds, brute force, and the distributions they must follow.
"""
import math

import numpy as np
import pytest
from scipy import stats

import oracle


# --- alias table (T7) -------------------------------------------------------------------------

def reconstruct(thresh, alias):
    V = thresh.size
    keep = thresh.astype(np.float64) / 2.0 ** 32
    # a draw below thresh keeps the bin; thresh == 2^32-1 with alias == self keeps it always
    p = np.zeros(V)
    np.add.at(p, np.arange(V), keep)
    np.add.at(p, alias, 1.0 - keep)
    return p / V


@pytest.mark.parametrize("V,seed", [(1, 0), (2, 1), (7, 2), (1000, 3), (50_000, 4)])
def test_T7_alias_table_reconstructs_the_noise_distribution(V, seed):
    rng = np.random.default_rng(seed)
    counts = np.maximum(1, (1e6 / np.arange(1, V + 1) ** 1.1)).astype(np.uint64)
    rng.shuffle(counts)
    th, al = oracle.build_alias(counts)
    want = counts.astype(np.float64) ** 0.75
    want /= want.sum()
    np.testing.assert_allclose(oracle.noise_probs(counts), want, rtol=1e-12)
    got = reconstruct(th, al)
    # each bin's keep probability is floored to a multiple of 2^-32
    assert np.max(np.abs(got - want)) <= 2.0 ** -32 + 1e-15 * V
    assert abs(got.sum() - 1.0) < 1e-12
    assert np.all(al < V)


def test_alias_table_with_zero_counts_never_yields_those_words():
    counts = np.array([5, 0, 0, 9, 1, 0, 3], np.uint64)
    th, al = oracle.build_alias(counts)
    got = reconstruct(th, al)
    assert np.all(got[counts == 0] == 0.0)
    out = np.zeros(20000, np.uint32)       # positive word 0; negatives must avoid 0 and zero-count words
    neg = oracle.negatives(out, 3, 123, th, al)
    assert set(np.unique(neg).tolist()) <= {3, 4, 6}


def test_T7_negatives_follow_unigram_to_the_three_quarters():
    V, n, k = 1000, 400_000, 5
    counts = np.maximum(1, (1e7 / np.arange(1, V + 1))).astype(np.uint64)
    th, al = oracle.build_alias(counts)
    out = np.full(n, V - 1, np.uint32)        # exclude one rare word, renormalise the rest
    neg = oracle.negatives(out, k, 2024, th, al)
    assert not np.any(neg == V - 1)
    p = oracle.noise_probs(counts)[: V - 1]
    p = p / p.sum()
    obs = np.bincount(neg.ravel(), minlength=V)[: V - 1]
    chi2 = ((obs - p * obs.sum()) ** 2 / (p * obs.sum())).sum()
    assert stats.chi2.sf(chi2, V - 2) > 1e-4
    # slots and pairs are separate streams: slot 1 and slot 2 are uncorrelated
    r = np.corrcoef(neg[:, 0].astype(float), neg[:, 1].astype(float))[0, 1]
    assert abs(r) < 0.01


def test_bin_choice_is_the_high_word_of_a_64_bit_product():
    # with every bin keeping itself, a negative is floor(r64 * V / 2^64) of the generator's
    # first two words (low word first) at counter (pair, slot, attempt, 4)
    V = 1000
    th, al = oracle.build_alias(np.ones(V, np.uint64))
    assert np.all(al == np.arange(V))
    out = np.full(50, V + 5, np.uint32) % V
    seed = (0xABCDEF01 << 32) | 0x12345678
    neg = oracle.negatives(out, 2, seed, th, al)
    for p in range(50):
        for j in (1, 2):
            t = 0
            while True:
                q = oracle.philox([p, j, t, 4], [seed & 0xffffffff, seed >> 32])
                cand = (((int(q[1]) << 32) | int(q[0])) * V) >> 64
                if cand != out[p]:
                    break
                t += 1
            assert neg[p, j - 1] == cand


# --- negatives: exclusion, fallback, regeneration (T5, T6) ---------------------------------------

def test_T6_negatives_never_equal_the_positive_word():
    rng = np.random.default_rng(6)
    V = 5
    counts = np.array([1000, 1, 1, 1, 1], np.uint64)     # word 0 dominates the noise distribution
    th, al = oracle.build_alias(counts)
    out = np.zeros(5000, np.uint32)                     # ... and is the positive word everywhere
    neg = oracle.negatives(out, 4, 77, th, al)
    assert not np.any(neg == 0)
    assert neg.max() < V
    out = rng.integers(0, V, 5000).astype(np.uint32)
    neg = oracle.negatives(out, 4, 78, th, al)
    assert not np.any(neg == out[:, None])


def test_T6_sixteen_rejections_fall_back_to_the_next_word():
    # two words, the noise distribution puts (almost) all mass on word 0: with out=0 nearly every
    # slot exhausts its 16 candidates and must return (0+1) mod 2 = 1; with out=1 every slot is 0.
    counts = np.array([10 ** 12, 1], np.uint64)
    th, al = oracle.build_alias(counts)
    neg0 = oracle.negatives(np.zeros(1000, np.uint32), 3, 5, th, al)
    assert np.all(neg0 == 1)
    neg1 = oracle.negatives(np.ones(1000, np.uint32), 3, 5, th, al)
    assert np.all(neg1 == 0)
    # wrap-around of the fallback: V=3, out = 2, all mass on word 2 -> 0
    th, al = oracle.build_alias(np.array([1, 1, 10 ** 15], np.uint64))
    neg = oracle.negatives(np.full(200, 2, np.uint32), 2, 9, th, al)
    assert np.mean(neg == 0) > 0.9 and not np.any(neg == 2)


def test_T5_dotprod_and_adjust_regenerate_the_same_negatives():
    rng = np.random.default_rng(5)
    V, d, n, k, seed = 40, 6, 60, 4, 31337
    U = (rng.random((V, d)).astype(np.float32) - 0.5)
    W = (rng.random((V, d)).astype(np.float32) - 0.5)
    th, al = oracle.build_alias(rng.integers(1, 30, V).astype(np.uint64))
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    neg = oracle.negatives(out_idx, k, seed, th, al)
    rows = np.concatenate([out_idx[:, None], neg], axis=1)
    assert np.array_equal(oracle.dotprod(U, W, in_idx, out_idx, k, seed, th, al),
                          oracle.dots(U, W, in_idx, rows))
    g = (rng.random((n, k + 1)).astype(np.float32) - 0.5)
    Ua, Wa, Ub, Wb = U.copy(), W.copy(), U.copy(), W.copy()
    oracle.adjust(Ua, Wa, in_idx, out_idx, k, seed, th, al, g, 0.1)
    oracle.adjust_rows(Ub, Wb, in_idx, rows, g, 0.1)
    assert np.array_equal(Ua, Ub) and np.array_equal(Wa, Wb)
    # another seed gives other negatives; a subset of pair numbers gives the same rows
    assert not np.array_equal(neg, oracle.negatives(out_idx, k, seed + 1, th, al))
    ids = np.array([3, 17, 59], np.uint32)
    assert np.array_equal(oracle.negatives(out_idx[ids], k, seed, th, al, pair_ids=ids), neg[ids])


# --- subsampling (T10) ---------------------------------------------------------------------------

def test_T10_keep_thresholds_and_rates():
    counts = np.array([500_000, 100_000, 10_000, 1000, 100, 10, 0], np.uint64)
    t = 1e-3
    kt = oracle.build_keep(counts, t)
    f = counts.astype(np.float64) / counts.sum()
    with np.errstate(divide="ignore"):
        keep = np.minimum(1.0, np.sqrt(t / f) + t / f)
    for w in range(counts.size):
        if keep[w] >= 1.0:
            assert kt[w] == 2 ** 32
        else:
            assert abs(int(kt[w]) - keep[w] * 2 ** 32) <= 1.0
    assert kt[0] < kt[1] < kt[2] <= 2 ** 32
    # empirical keep fraction per word inside a binomial interval
    n = 200_000
    for w in (0, 1, 2):
        tokens = np.full(n, w, np.uint32)
        kept, _ = oracle.token_draws(tokens, 10 ** 10, 0, 42, 5, kt)
        p = keep[w]
        assert abs(kept.mean() - p) < 5 * math.sqrt(p * (1 - p) / n)
    # a huge threshold keeps everything; no table keeps everything
    kept, _ = oracle.token_draws(np.zeros(1000, np.uint32), 0, 0, 1, 5, oracle.build_keep(counts, 1e9))
    assert kept.all()
    kept, _ = oracle.token_draws(np.zeros(1000, np.uint32), 0, 0, 1, 5, None)
    assert kept.all()


def test_token_draws_depend_on_global_position_epoch_and_seed_only():
    tokens = np.zeros(64, np.uint32)
    kt = oracle.build_keep(np.array([9, 1], np.uint64), 0.05)
    k0, b0 = oracle.token_draws(tokens, 1000, 0, 7, 6, kt)
    k1, b1 = oracle.token_draws(tokens[:32], 1032, 0, 7, 6, kt)
    assert np.array_equal(k0[32:], k1) and np.array_equal(b0[32:], b1)
    assert not np.array_equal(b0, oracle.token_draws(tokens, 1000, 1, 7, 6, kt)[1])
    assert not np.array_equal(b0, oracle.token_draws(tokens, 1000, 0, 8, 6, kt)[1])
    # positions beyond 2^32 use the high counter word
    _, bh = oracle.token_draws(tokens, (1 << 32) + 1000, 0, 7, 6, kt)
    assert not np.array_equal(b0, bh)


# --- windows (T11) -------------------------------------------------------------------------------

def test_T11_window_width_is_uniform_on_1_to_B():
    B = 7
    _, b = oracle.token_draws(np.zeros(350_000, np.uint32), 0, 0, 3, B, None)
    assert b.min() == 1 and b.max() == B
    obs = np.bincount(b, minlength=B + 1)[1:]
    assert stats.chisquare(obs).pvalue > 1e-4


def pairs_by_hand(tokens, off, base, epoch, seed, B, kt):
    keep, b = oracle.token_draws(tokens, base, epoch, seed, B, kt)
    a_out, b_out = [], []
    for s in range(off.size - 1):
        pos = [t for t in range(int(off[s]), int(off[s + 1])) if keep[t]]
        for j, t in enumerate(pos):
            lo, hi = max(0, j - int(b[t])), min(len(pos) - 1, j + int(b[t]))
            for c in range(lo, hi + 1):
                if c != j:
                    a_out.append(tokens[t])
                    b_out.append(tokens[pos[c]])
    return np.array(a_out, np.uint32), np.array(b_out, np.uint32)


def test_T11_pairs_against_a_hand_written_walk():
    rng = np.random.default_rng(111)
    V = 30
    counts = rng.integers(1, 2000, V).astype(np.uint64)
    kt = oracle.build_keep(counts, 0.01)
    tokens = rng.integers(0, V, 600).astype(np.uint32)
    lens = rng.integers(1, 25, 60)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = off[off < 600]
    off = np.append(off, 600).astype(np.uint64)
    for B in (1, 3, 8):
        a, b, cnt = oracle.make_pairs(tokens, off, 12345, 2, 99, B, kt)
        ha, hb = pairs_by_hand(tokens, off, 12345, 2, 99, B, kt)
        assert cnt == ha.size and np.array_equal(a, ha) and np.array_equal(b, hb)


def test_T11_window_one_without_subsampling_gives_adjacent_tokens():
    tokens = np.arange(10, dtype=np.uint32)
    off = np.array([0, 4, 5, 10], np.uint64)           # sentences of 4, 1 and 5 tokens
    a, b, cnt = oracle.make_pairs(tokens, off, 0, 0, 1, 1, None)
    want = [(0, 1), (1, 0), (1, 2), (2, 1), (2, 3), (3, 2),
            (5, 6), (6, 5), (6, 7), (7, 6), (7, 8), (8, 7), (8, 9), (9, 8)]
    assert cnt == len(want) and list(zip(a.tolist(), b.tolist())) == want


def test_T11_interleaved_order_on_a_hand_case():
    # Section 5.1, last paragraph: centers are taken round-robin over the sentences.  Sentences of
    # 4, 1 and 5 tokens, window 1, no subsampling: first tokens 0 and 5 (the one-word sentence has
    # no pair), second tokens 1 and 6, third 2 and 7, fourth 3 and 8, and 9 alone at the end.
    tokens = np.arange(10, dtype=np.uint32)
    off = np.array([0, 4, 5, 10], np.uint64)
    a, b, cnt = oracle.make_pairs(tokens, off, 0, 0, 1, 1, None, interleaved=True)
    want = [(0, 1), (5, 6), (1, 0), (1, 2), (6, 5), (6, 7), (2, 1), (2, 3), (7, 6), (7, 8),
            (3, 2), (8, 7), (8, 9), (9, 8)]
    assert cnt == len(want) and list(zip(a.tolist(), b.tolist())) == want


def test_T11_interleaved_is_a_reordering_with_centers_round_robin():
    rng = np.random.default_rng(113)
    V, n = 5000, 4000
    tokens = rng.permutation(V)[:n].astype(np.uint32)     # distinct words: a pair names its positions
    lens = rng.integers(0, 30, 400)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.append(off[off < n], n).astype(np.uint64)
    kt = np.full(V, int(0.7 * 2 ** 32), np.uint64)
    for B in (1, 4):
        a0, b0, c0 = oracle.make_pairs(tokens, off, 77, 1, 9, B, kt)
        a1, b1, c1 = oracle.make_pairs(tokens, off, 77, 1, 9, B, kt, interleaved=True)
        assert c0 == c1
        key0 = a0.astype(np.uint64) << 32 | b0
        key1 = a1.astype(np.uint64) << 32 | b1
        assert np.array_equal(np.sort(key0), np.sort(key1)) and not np.array_equal(key0, key1)
        # rank of every word among its sentence's survivors, and its sentence, from the draws
        keep, _ = oracle.token_draws(tokens, 77, 1, 9, B, kt)
        sent = np.searchsorted(off, np.arange(n), side="right") - 1
        rank = np.zeros(V, np.int64)
        sent_of = np.zeros(V, np.int64)
        for s in range(off.size - 1):
            pos = [t for t in range(int(off[s]), int(off[s + 1])) if keep[t]]
            for j, t in enumerate(pos):
                rank[tokens[t]], sent_of[tokens[t]] = j, s
        order = rank[a1] * (off.size + 1) + sent_of[a1]
        assert np.all(np.diff(order) >= 0)                # by rank, then by sentence
        # contexts of one center stay in corpus order, as in the plain walk
        for w in rng.choice(np.unique(a1), 50, replace=False):
            assert np.array_equal(b1[a1 == w], b0[a0 == w])
        # the truncated call returns a prefix of the full one
        a2, _, c2 = oracle.make_pairs(tokens, off, 77, 1, 9, B, kt, capacity=37, interleaved=True)
        assert c2 == c1 and np.array_equal(a2, a1[:37])
        assert sent.max() == off.size - 2


def test_T11_interleaved_minibatches_take_every_center_from_a_different_sentence():
    # The purpose of the option (Section 5.1, last paragraph): with more sentences in the block than
    # centers in a minibatch, the input words of a minibatch come from (nearly) as many sentences --
    # a sentence gives a second one only where the minibatch runs over the end of a round -- while
    # the corpus-order walk takes them from a handful of sentences.
    n_sent, L, B, n = 3000, 20, 5, 4096
    tokens = np.arange(n_sent * L, dtype=np.uint32)       # word id == position
    off = np.arange(0, n_sent * L + 1, L).astype(np.uint64)
    kt = np.full(tokens.size, int(0.4 * 2 ** 32), np.uint64)
    per_batch = {}
    for inter in (False, True):
        a, _, cnt = oracle.make_pairs(tokens, off, 0, 0, 3, B, kt, interleaved=inter)
        got = []
        for h in range(cnt // n):
            centers = np.unique(a[h * n:(h + 1) * n])
            got.append((centers.size, np.unique(centers // L).size))
        per_batch[inter] = np.array(got)
    plain, inter = per_batch[False], per_batch[True]
    assert inter[0, 0] == inter[0, 1]                     # first round: one center per sentence
    assert np.all(inter[:, 1] * 2 >= inter[:, 0])         # a minibatch spans at most two rounds ...
    assert inter[:, 1].sum() > 0.85 * inter[:, 0].sum()   # ... and mostly one
    assert np.all(plain[:, 1] * 4 < plain[:, 0])          # corpus order: several centers per sentence
    assert abs(plain[:, 0].mean() - inter[:, 0].mean()) < 0.1 * plain[:, 0].mean()


def test_T11_pair_count_is_the_sum_of_clipped_windows_and_no_pair_crosses_a_sentence():
    rng = np.random.default_rng(112)
    n, L, B = 3000, 15, 4
    tokens = np.arange(n, dtype=np.uint32)              # word id == position, so pairs reveal positions
    off = np.arange(0, n + 1, L).astype(np.uint64)
    a, b, cnt = oracle.make_pairs(tokens, off, 0, 0, 5, B, None)
    _, bw = oracle.token_draws(tokens, 0, 0, 5, B, None)
    j = np.arange(n) % L
    assert cnt == int((np.minimum(j, bw) + np.minimum(L - 1 - j, bw)).sum())
    assert np.all(a // L == b // L)
    assert np.all(np.abs(a.astype(np.int64) - b) <= bw[a]) and np.all(a != b)
    assert np.all(np.diff(a.astype(np.int64)) >= 0)     # centers in corpus order
    # capacity is respected and the full count still reported
    a2, b2, cnt2 = oracle.make_pairs(tokens, off, 0, 0, 5, B, None, capacity=100)
    assert cnt2 == cnt and a2.size == 100 and np.array_equal(a2, a[:100])
    # removed tokens do not count toward the window: with subsampling, neighbours can be far apart
    kt = np.full(n, int(0.3 * 2 ** 32), np.uint64)
    a3, b3, _ = oracle.make_pairs(tokens, off, 0, 0, 5, 1, kt)
    assert np.max(np.abs(a3.astype(np.int64) - b3)) > 1 and np.all(a3 // L == b3 // L)
