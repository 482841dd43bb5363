"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot hold a 10M x 300 model densely in a test, so it is asked for exactly the outputs
sampled here: integer results (pairs, negatives) are compared in full, bit for bit; dots and updated
rows are compared on samples chosen to include the hottest rows (long runs that go through several
reduction levels) and random cold ones.  For a sampled row, every pair that contributes to it is
handed to the oracle as one sub-minibatch over a compacted copy of the touched rows, so the
oracle's result for that row is complete.  Initial values on both sides come from the same
counter-based recipe, never from the GPU.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_08495_amd import w2v, workloads
from util import delta_error, dev, dot_error, vec_error, vec_error_elem

pytestmark = pytest.mark.gpu
TOL1 = 1e-5


def say(*a):
    print(*a, flush=True)


def compact_problem(wl, in_idx, rows, init_w):
    """Oracle-side dense copy of just the touched rows; returns (U, W, cin, crows, words_u, words_w)."""
    words_u, cin = np.unique(in_idx, return_inverse=True)
    words_w, cr = np.unique(rows.ravel(), return_inverse=True)
    U = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 0, words_u.astype(np.uint32))
    if init_w:
        W = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 1, words_w.astype(np.uint32))
    else:
        W = np.zeros((words_w.size, wl.d_slice), np.float32)
    return U, W, cin.astype(np.uint32), cr.reshape(rows.shape).astype(np.uint32), words_u, words_w


def sample_rows(ids, n_hot, n_cold, rng):
    """The n_hot most frequent values of ids plus n_cold random other ones."""
    vals, cnt = np.unique(ids, return_counts=True)
    order = np.argsort(-cnt, kind="stable")
    hot = vals[order[:n_hot]]
    rest = vals[order[n_hot:]]
    cold = rng.choice(rest, size=min(n_cold, rest.size), replace=False) if rest.size else rest
    return np.concatenate([hot, cold]).astype(np.uint32)


def check_sampled_update(sh, wl, in_idx, rows, coeffs, alpha, init_w, samp_u, samp_w):
    """Oracle adjust on every pair touching a sampled row; compares those rows with the shard's:
    the updated rows, and the change itself ((after - before) / alpha against the oracle's summed
    change; the shard started from the initial values, which the oracle reproduces bit for bit)."""
    sel = np.isin(in_idx, samp_u) | np.isin(rows, samp_w).any(axis=1)
    ii, rr = in_idx[sel], rows[sel]
    say("   sub-minibatch of", int(sel.sum()), "pairs for", samp_u.size, "+", samp_w.size, "rows")
    U, W, cin, cr, words_u, words_w = compact_problem(wl, ii, rr, init_w)
    if coeffs is None:
        g = oracle.coeffs([oracle.dots(U, W, cin, cr)])
    else:
        g = coeffs[sel]
    at_u, at_w = np.searchsorted(words_u, samp_u), np.searchsorted(words_w, samp_w)
    dU, dW = oracle.adjust_deltas(U, W, cin, cr, g, want_u=at_u, want_w=at_w)
    U0, W0 = U[at_u].copy(), W[at_w].copy()
    oracle.adjust_rows(U, W, cin, cr, g, alpha)
    gu = sh.get_rows(0, dev(samp_u)).cpu().numpy()
    gw = sh.get_rows(1, dev(samp_w)).cpu().numpy()
    ru, rw = U[at_u], W[at_w]
    du, dw = delta_error(gu, U0, alpha, dU), delta_error(gw, W0, alpha, dW)
    say("   change of U", du, "of W", dw, "| element-relative", vec_error_elem(gu, ru), vec_error_elem(gw, rw))
    assert du <= TOL1 and dw <= TOL1, (du, dw)
    return vec_error(gu, ru), vec_error(gw, rw)


@pytest.mark.parametrize("init_w", [True, False])
def test_full300_step_sampled(init_w):
    """V = 10M, d = 300, 2^20 pairs from the corpus, k = 5: make_pairs + train_minibatch."""
    wl = workloads.WORKLOADS["full300"]
    rng = np.random.default_rng(7)
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    tokens, off = workloads.corpus(wl, 400_000, cdf=cdf)
    del cdf
    say("full300: building shard", "W uniform" if init_w else "W zero")
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, init_mode=1 if init_w else 0)
    sh.set_counts(counts, wl.subsample_t)
    th, al = oracle.build_alias(counts)
    kt = oracle.build_keep(counts, wl.subsample_t)

    # pairs: full comparison
    cap = wl.n_pairs * 2
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    # (init_w: as bench.py runs it -- pairs formed on a stream of their own, the minibatch announced
    # to the shard before the step; otherwise everything on one stream, nothing announced)
    tok_dev, off_dev = dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda()
    with torch.cuda.stream(torch.cuda.Stream() if init_w else torch.cuda.current_stream()):
        cnt = sh.make_pairs(tok_dev, off_dev, 0, 0, wl.seed, wl.window, gi, go)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, 0, 0, wl.seed, wl.window, kt)
    assert cnt == ocnt and cnt >= wl.n_pairs
    assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi) and np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    n = wl.n_pairs
    in_idx, out_idx = oi[:n], oo[:n]
    a, b = gi[:n], go[:n]
    seed = w2v.minibatch_seed(wl.seed, 0)

    # negatives: full comparison
    say("   negatives")
    neg = oracle.negatives(out_idx, wl.k, seed, th, al)
    assert np.array_equal(w2v.index_to_numpy(sh.negatives(b, wl.k, seed)), neg)
    rows = np.concatenate([out_idx[:, None], neg], axis=1)

    # dots: 4096 sampled pairs
    say("   dots")
    dots = sh.dotprod(a, b, wl.k, seed).cpu().numpy()
    pick = rng.choice(n, 4096, replace=False)
    U, W, cin, cr, _, _ = compact_problem(wl, in_idx[pick], rows[pick], init_w)
    ref = oracle.dots(U, W, cin, cr)
    err = dot_error(dots[pick], ref, U, W, cin, cr)
    say("   dot error", err)
    assert err <= TOL1
    if not init_w:
        assert not dots.any()

    # the fused step, then sampled rows
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    alpha = workloads.alpha_schedule(wl, 0, 1000)
    if init_w:
        sh.prefetch_minibatch(a, b, wl.k, seed)
    w2v.train_minibatch([sh], a, b, wl.k, seed, alpha, loss=loss)
    sh.status()
    samp_u = sample_rows(in_idx, 24, 200, rng)
    samp_w = sample_rows(rows.ravel(), 24, 1500, rng)
    eu, ew = check_sampled_update(sh, wl, in_idx, rows, None, alpha, init_w, samp_u, samp_w)
    say("   U error", eu, "W error", ew)
    assert eu <= TOL1 and ew <= TOL1
    if not init_w:
        # closed form: every dot is zero, so the loss is n (k+1) ln 2 and the input vectors stay put
        assert abs(loss.item() - n * (wl.k + 1) * np.log(2.0)) <= 1e-6 * loss.item()
        untouched = sh.get_rows(0, dev(samp_u)).cpu().numpy()
        assert np.array_equal(untouched, oracle.init_rows(wl.seed, wl.d_total, 0, wl.d_slice, 0, samp_u))
    # rows no pair touches are bitwise unchanged
    never = np.setdiff1d(rng.integers(0, wl.V, 4000).astype(np.uint32), rows.ravel())[:1000]
    w_init = oracle.init_rows(wl.seed, wl.d_total, 0, wl.d_slice, 1, never) if init_w else 0.0
    assert np.array_equal(sh.get_rows(1, dev(never)).cpu().numpy(), w_init + np.zeros((never.size, wl.d_slice), np.float32))
    sh.destroy()


def test_slice60_dotprod_adjust_sampled():
    """V = 1M, d_slice = 60 of 300, 2^20 iid Zipf pairs, k = 5, harness coefficients."""
    wl = workloads.WORKLOADS["slice60"]
    rng = np.random.default_rng(8)
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    in_idx, out_idx = workloads.iid_pairs(wl, cdf=cdf)
    n, T = wl.n_pairs, wl.k + 1
    g = workloads.uniform_coeffs(n, T, wl.seed)
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin, init_mode=1)
    sh.set_counts(counts, 0.0)
    th, al = oracle.build_alias(counts)
    seed = w2v.minibatch_seed(wl.seed, 0)
    a, b = dev(in_idx), dev(out_idx)
    neg = oracle.negatives(out_idx, wl.k, seed, th, al)
    assert np.array_equal(w2v.index_to_numpy(sh.negatives(b, wl.k, seed)), neg)
    rows = np.concatenate([out_idx[:, None], neg], axis=1)

    sh.prefetch_minibatch(a, b, wl.k, seed)          # as bench.py runs it: the minibatch announced
    dots = sh.dotprod(a, b, wl.k, seed).cpu().numpy()
    pick = rng.choice(n, 8192, replace=False)
    U, W, cin, cr, _, _ = compact_problem(wl, in_idx[pick], rows[pick], True)
    err = dot_error(dots[pick], oracle.dots(U, W, cin, cr), U, W, cin, cr)
    say("slice60 dot error", err)
    assert err <= TOL1

    sh.adjust(a, b, wl.k, seed, torch.from_numpy(g).cuda(), wl.alpha)
    sh.status()
    samp_u = sample_rows(in_idx, 8, 600, rng)      # word 0 is the input of ~7% of the pairs
    samp_w = sample_rows(rows.ravel(), 8, 1500, rng)
    eu, ew = check_sampled_update(sh, wl, in_idx, rows, g, wl.alpha, True, samp_u, samp_w)
    say("slice60 U error", eu, "W error", ew)
    assert eu <= TOL1 and ew <= TOL1
    sh.destroy()


def reduced_n_step(name, n, n_tokens):
    """Full vocabulary, dimension, k and token law of a large workload; one minibatch of n pairs."""
    wl = workloads.WORKLOADS[name]
    rng = np.random.default_rng(11)
    say(name, ": tables for V =", wl.V)
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    tokens, off = workloads.corpus(wl, n_tokens, cdf=cdf)
    del cdf
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin, init_mode=1)
    sh.set_counts(counts, wl.subsample_t)
    th, al = oracle.build_alias(counts)
    gth, gal, _ = sh.get_tables()
    assert np.array_equal(gth, th) and np.array_equal(gal, al)
    del gth, gal, counts
    say("   pairs")
    cap = n_tokens * 2 * wl.window
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    cnt = sh.make_pairs(dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda(), 0, 0, wl.seed,
                        wl.window, gi, go)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, 0, 0, wl.seed, wl.window, None)
    assert cnt == ocnt and cnt >= n
    assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi) and np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    in_idx, out_idx = oi[:n], oo[:n]
    a, b = gi[:n].contiguous(), go[:n].contiguous()
    seed = w2v.minibatch_seed(wl.seed, 0)
    say("   negatives")
    neg = oracle.negatives(out_idx, wl.k, seed, th, al)
    assert np.array_equal(w2v.index_to_numpy(sh.negatives(b, wl.k, seed)), neg)
    rows = np.concatenate([out_idx[:, None], neg], axis=1)
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    w2v.train_minibatch([sh], a, b, wl.k, seed, wl.alpha, loss=loss)
    sh.status()
    samp_u = sample_rows(in_idx, 8, 100, rng)
    samp_w = sample_rows(rows.ravel(), 8, 600, rng)
    eu, ew = check_sampled_update(sh, wl, in_idx, rows, None, wl.alpha, True, samp_u, samp_w)
    say("   U error", eu, "W error", ew)
    assert eu <= TOL1 and ew <= TOL1
    first = (sh.get_rows(0, dev(samp_u)).cpu().numpy(), sh.get_rows(1, dev(samp_w)).cpu().numpy(), loss.item())
    sh.destroy()
    # the same step on a fresh shard gives the same bits (fixed-order reduction, no float atomics)
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin, init_mode=1)
    sh.set_counts(workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens), wl.subsample_t)
    w2v.train_minibatch([sh], a, b, wl.k, seed, wl.alpha, loss=loss)
    assert np.array_equal(sh.get_rows(0, dev(samp_u)).cpu().numpy(), first[0])
    assert np.array_equal(sh.get_rows(1, dev(samp_w)).cpu().numpy(), first[1])
    assert loss.item() == first[2]
    sh.destroy()


def streamed_input_row_change(wl, in_idx, rows, word, chunk=1 << 15):
    """The oracle's summed change (double) of input row `word`: every pair that names it as its input
    word, handed to the oracle in chunks over a compacted copy of the output rows those pairs touch
    (initial values from the counter-based recipe); the chunks' sums are added in double."""
    sel = np.flatnonzero(in_idx == word)
    U = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 0, np.array([word], np.uint32))
    total = np.zeros(wl.d_slice)
    none = np.zeros(0, np.uint32)
    for lo in range(0, sel.size, chunk):
        rr = rows[sel[lo:lo + chunk]]
        words_w, cr = np.unique(rr.ravel(), return_inverse=True)
        W = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 1, words_w.astype(np.uint32))
        cr = cr.reshape(rr.shape).astype(np.uint32)
        cin = np.zeros(rr.shape[0], np.uint32)
        g = oracle.coeffs([oracle.dots(U, W, cin, cr)])
        dU, _ = oracle.adjust_deltas(U, W, cin, cr, g, want_u=[0], want_w=none)
        total += dU[0]
    return total, sel.size


def streamed_output_row_change(wl, in_idx, rows, word, chunk=1 << 17):
    """The same for output row `word`: every SLOT that names it.  A slot in column 0 (the word as the
    positive output word) goes to the oracle as a pair without negatives; a slot in a column j > 0
    (the word as a negative) as a pair [its own positive word, `word`] with one negative, whose
    second column carries the slot's coefficient -sigma and its change -- the positive word of such
    a pair is never `word` itself (negatives differ from it), so nothing else lands in the row."""
    total = np.zeros(wl.d_slice)
    slots = 0
    none = np.zeros(0, np.uint32)
    for col0 in (True, False):
        if col0:
            pp = np.flatnonzero(rows[:, 0] == word)
            sub_rows = np.full((pp.size, 1), word, np.uint32)
        else:
            pp, jj = np.nonzero(rows[:, 1:] == word)
            assert not np.any(rows[pp, 0] == word)
            sub_rows = np.stack([rows[pp, 0], np.full(pp.size, word, np.uint32)], axis=1)
        slots += pp.size
        for lo in range(0, pp.size, chunk):
            ii, rr = in_idx[pp[lo:lo + chunk]], sub_rows[lo:lo + chunk]
            words_u, cin = np.unique(ii, return_inverse=True)
            words_w, cr = np.unique(rr.ravel(), return_inverse=True)
            U = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 0, words_u.astype(np.uint32))
            W = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 1, words_w.astype(np.uint32))
            cr = cr.reshape(rr.shape).astype(np.uint32)
            g = oracle.coeffs([oracle.dots(U, W, cin.astype(np.uint32), cr)])
            at = np.searchsorted(words_w, [word])
            _, dW = oracle.adjust_deltas(U, W, cin.astype(np.uint32), cr, g, want_u=none, want_w=at)
            total += dW[0]
    return total, slots


def check_hottest_rows(sh, wl, in_idx, rows, alpha):
    """The most frequent input word and the most frequently named output row of the minibatch --
    the rows whose contributions pass through every level of the reduction -- against the oracle."""
    for which, ids, fn in ((0, in_idx, streamed_input_row_change), (1, rows.ravel(), streamed_output_row_change)):
        vals, cnt = np.unique(ids, return_counts=True)
        word = int(vals[np.argmax(cnt)])
        change, m = fn(wl, in_idx, rows, word)
        before = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, which, np.array([word], np.uint32))
        ref = (before.astype(np.float64) + float(np.float32(alpha)) * change[None]).astype(np.float32)
        got = sh.get_rows(which, dev(np.array([word], np.uint32))).cpu().numpy()
        e, de = vec_error(got, ref), delta_error(got, before, alpha, change[None])
        say("   hottest", "input" if which == 0 else "output", "row: word", word, "with", m,
            "contributions" if which else "pairs", "| row error", e, "| change", de)
        assert e <= TOL1 and de <= TOL1, (which, word, e, de)


def full_n_step(name, n_tokens):
    """The benchmark's own launch configuration (full vocabulary, dimension, k and n): pairs and
    negatives compared in full; updated rows compared on sampled rows that collect few
    contributions (for those the oracle can be given every pair that touches them) and on the
    hottest input row and the hottest output row (the oracle streams through every pair / slot that
    names them); the whole step repeated on a fresh shard must give the same bits."""
    wl = workloads.WORKLOADS[name]
    n = wl.n_pairs
    rng = np.random.default_rng(23)
    say(name, "full n =", n, ": tables")
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    tokens, off = workloads.corpus(wl, n_tokens, cdf=cdf)
    del cdf
    th, al = oracle.build_alias(counts)

    def fresh():
        sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin, init_mode=1)
        sh.set_counts(counts, wl.subsample_t)
        return sh
    sh = fresh()
    cap = n_tokens * 2 * wl.window
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    cnt = sh.make_pairs(dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda(), 0, 0, wl.seed,
                        wl.window, gi, go)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, 0, 0, wl.seed, wl.window, None)
    assert cnt == ocnt and cnt >= n
    assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi) and np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    in_idx, out_idx = oi[:n], oo[:n]
    a, b = gi[:n].contiguous(), go[:n].contiguous()
    del gi, go
    seed = w2v.minibatch_seed(wl.seed, 0)
    say("   negatives, all", n * wl.k)
    neg = oracle.negatives(out_idx, wl.k, seed, th, al)
    assert np.array_equal(w2v.index_to_numpy(sh.negatives(b, wl.k, seed)), neg)
    rows = np.concatenate([out_idx[:, None], neg], axis=1)
    del neg
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    w2v.train_minibatch([sh], a, b, wl.k, seed, wl.alpha, loss=loss)
    sh.status()
    # rows with at most four contributions, found from a random sample of slots
    cand_w = np.unique(rows.ravel()[rng.integers(0, rows.size, 3000)])
    hits = rows.ravel()[np.isin(rows.ravel(), cand_w)]
    vals, c = np.unique(hits, return_counts=True)
    samp_w = vals[c <= 4][:600].astype(np.uint32)
    vals, c = np.unique(in_idx, return_counts=True)
    few = vals[c <= 4]
    samp_u = rng.choice(few, size=min(150, few.size), replace=False).astype(np.uint32)
    assert samp_w.size >= 100 and samp_u.size >= 50
    eu, ew = check_sampled_update(sh, wl, in_idx, rows, None, wl.alpha, True, samp_u, samp_w)
    say("   U error", eu, "W error", ew)
    assert eu <= TOL1 and ew <= TOL1
    check_hottest_rows(sh, wl, in_idx, rows, wl.alpha)
    hot_u = sample_rows(in_idx, 8, 100, rng)
    hot_w = sample_rows(out_idx, 8, 300, rng)
    keep = [sh.get_rows(0, dev(x)).cpu().numpy() for x in (samp_u, hot_u)] + \
           [sh.get_rows(1, dev(x)).cpu().numpy() for x in (samp_w, hot_w)] + [loss.item()]
    sh.destroy()
    del sh
    say("   the same step on a fresh shard, announced ahead as bench.py does")
    sh = fresh()
    sh.prefetch_minibatch(a, b, wl.k, seed)
    w2v.train_minibatch([sh], a, b, wl.k, seed, wl.alpha, loss=loss)
    again = [sh.get_rows(0, dev(x)).cpu().numpy() for x in (samp_u, hot_u)] + \
            [sh.get_rows(1, dev(x)).cpu().numpy() for x in (samp_w, hot_w)] + [loss.item()]
    for x, y in zip(keep[:4], again[:4]):
        assert np.array_equal(x, y)
    assert keep[4] == again[4]
    sh.status()
    sh.destroy()


def test_stress25_full_n_properties():
    full_n_step("stress25", 700_000)


def test_search200m_full_n_properties():
    full_n_step("search200m", 520_000)


def test_stress25_reduced_n_sampled():
    """V = 50M, d = 200, k = 25, Zipf(1.2): the most frequent word is the input of ~18% of the pairs,
    so its row collects hundreds of thousands of contributions through several reduction levels."""
    reduced_n_step("stress25", 1 << 18, 40_000)


def test_search200m_reduced_n_sampled():
    """V = 200M, d_slice = 60 of 300, k = 10, Zipf(0.9): heavy tail, rows rarely reused."""
    reduced_n_step("search200m", 1 << 18, 64_000)


@pytest.mark.parametrize("init_w", [True, False])
def test_full300_cbow_step_sampled(init_w):
    """The bag-of-words benchmark configuration: V = 10M, d = 300, 2^17 examples from the corpus,
    k = 5: make_cbow_examples + cbow_train_minibatch; examples in full, updated rows on samples."""
    wl = workloads.WORKLOADS["full300"]
    rng = np.random.default_rng(17)
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    tokens, off = workloads.corpus(wl, 400_000, cdf=cdf)
    del cdf
    say("full300 cbow: building shard", "W uniform" if init_w else "W zero")
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, init_mode=1 if init_w else 0)
    sh.set_counts(counts, wl.subsample_t)
    th, al = oracle.build_alias(counts)
    kt = oracle.build_keep(counts, wl.subsample_t)
    n_tok = tokens.size
    co = torch.empty(n_tok + 1, dtype=torch.int32, device="cuda")
    cx = torch.empty(n_tok * 2 * wl.window, dtype=torch.int32, device="cuda")
    ce = torch.empty(n_tok, dtype=torch.int32, device="cuda")
    n_ex, n_ctx = sh.make_cbow_examples(dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda(), 0, 0,
                                        wl.seed, wl.window, co, cx, ce)
    ooff, octx, oout, ocnt, onctx = oracle.make_cbow_examples(tokens, off, 0, 0, wl.seed, wl.window, kt)
    assert (n_ex, n_ctx) == (ocnt, onctx)
    assert np.array_equal(w2v.index_to_numpy(co[:n_ex + 1]), ooff)
    assert np.array_equal(w2v.index_to_numpy(cx[:n_ctx]), octx)
    assert np.array_equal(w2v.index_to_numpy(ce[:n_ex]), oout)
    n = 1 << 17
    assert n_ex >= n
    m = int(ooff[n])
    off_n, ctx_n, out_n = ooff[:n + 1], octx[:m], oout[:n]
    seed = w2v.minibatch_seed(wl.seed, 0)
    alpha = workloads.alpha_schedule(wl, 0, 1000)
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    w2v.cbow_train_minibatch([sh], co[:n + 1].contiguous(), cx[:m].contiguous(), ce[:n].contiguous(),
                             wl.k, seed, alpha, loss=loss)
    sh.status()
    neg = oracle.negatives(out_n, wl.k, seed, th, al)
    rows = np.concatenate([out_n[:, None], neg], axis=1)
    samp_u = sample_rows(ctx_n, 16, 200, rng)
    samp_w = sample_rows(rows.ravel(), 16, 800, rng)
    # every example that touches a sampled row, whole
    ex_of = np.repeat(np.arange(n), np.diff(off_n.astype(np.int64)))
    hit = np.zeros(n, bool)
    hit[ex_of[np.isin(ctx_n, samp_u)]] = True
    hit |= np.isin(rows, samp_w).any(axis=1)
    sel = np.flatnonzero(hit)
    say("   sub-minibatch of", sel.size, "examples for", samp_u.size, "+", samp_w.size, "rows")
    lens = np.diff(off_n.astype(np.int64))[sel]
    sub_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    sub_ctx = np.concatenate([ctx_n[off_n[p]:off_n[p + 1]] for p in sel])
    sub_rows = rows[sel]
    words_u, cctx = np.unique(sub_ctx, return_inverse=True)
    words_w, cr = np.unique(sub_rows.ravel(), return_inverse=True)
    U = oracle.init_rows(wl.seed, wl.d_total, 0, wl.d_slice, 0, words_u.astype(np.uint32))
    W = (oracle.init_rows(wl.seed, wl.d_total, 0, wl.d_slice, 1, words_w.astype(np.uint32)) if init_w
         else np.zeros((words_w.size, wl.d_slice), np.float32))
    cr = cr.reshape(sub_rows.shape).astype(np.uint32)
    g = oracle.coeffs([oracle.cbow_dots(U, W, sub_off, cctx.astype(np.uint32), cr)])
    oracle.cbow_adjust_rows(U, W, sub_off, cctx.astype(np.uint32), cr, g, alpha)
    gu = sh.get_rows(0, dev(samp_u)).cpu().numpy()
    gw = sh.get_rows(1, dev(samp_w)).cpu().numpy()
    eu = vec_error(gu, U[np.searchsorted(words_u, samp_u)])
    ew = vec_error(gw, W[np.searchsorted(words_w, samp_w)])
    say("   U error", eu, "W error", ew)
    assert eu <= TOL1 and ew <= TOL1
    if not init_w:
        assert abs(loss.item() - n * (wl.k + 1) * np.log(2.0)) <= 1e-6 * loss.item()
        assert np.array_equal(gu, oracle.init_rows(wl.seed, wl.d_total, 0, wl.d_slice, 0, samp_u))
    sh.destroy()
