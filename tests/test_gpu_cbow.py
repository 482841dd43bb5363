"""GPU parity of the continuous-bag-of-words entry points (Section 5.1, footnote) against the CPU
oracle, through the C ABI: examples from text bit for bit; dots, coefficients and updated vectors
within 1e-5 after one minibatch and 1e-3 after a hundred.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_08495_amd import w2v, workloads
from util import all_rows, dev, dot_error, vec_error, zipf_counts

pytestmark = pytest.mark.gpu

TOL1 = 1e-5
TOL100 = 1e-3


def say(*a):
    print(*a, flush=True)


def make_shard(V, d, seed, counts, d_total=None, col_begin=0, init_mode=1, t=0.0):
    sh = w2v.Shard(V, d, seed, d_total=d_total, col_begin=col_begin, init_mode=init_mode)
    sh.set_counts(counts, t)
    return sh


def oracle_state(V, d, seed, d_total=None, col_begin=0, init_mode=1):
    rows = np.arange(V, dtype=np.uint32)
    dt = d if d_total is None else d_total
    U = oracle.init_rows(seed, dt, col_begin, d, 0, rows)
    W = oracle.init_rows(seed, dt, col_begin, d, 1, rows) if init_mode else np.zeros((V, d), np.float32)
    return U, W


def examples(V, n, max_ctx, rng, skew=1.0, empty=False):
    cdf = workloads.zipf_cdf(V, skew)
    lens = rng.integers(0 if empty else 1, max_ctx + 1, n)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    return off, workloads.zipf_draw(cdf, int(off[-1]), rng), workloads.zipf_draw(cdf, n, rng)


def mean_abs_rows(U, off, ctx):
    """Row p: mean over the contexts of p of |u_c| (the scale of the hidden vector's rounding)."""
    n = off.size - 1
    H = np.zeros((n, U.shape[1]))
    for p in range(n):
        if off[p + 1] > off[p]:
            H[p] = np.abs(U[ctx[off[p]:off[p + 1]]].astype(np.float64)).mean(axis=0)
    return H


SHAPES = [(5000, 60, 300, 4099, 5, 12), (3000, 300, 300, 2500, 5, 20), (2000, 100, 100, 1000, 10, 7),
          (500, 7, 7, 777, 3, 40), (64, 1000, 1000, 130, 2, 5), (40, 200, 200, 1, 25, 3)]


@pytest.mark.parametrize("V,d,d_total,n,k,max_ctx", SHAPES)
def test_cbow_dotprod_parity(V, d, d_total, n, k, max_ctx):
    say("cbow dotprod", V, d, n, k, max_ctx)
    rng = np.random.default_rng(V + d + n)
    counts = zipf_counts(V)
    sh = make_shard(V, d, 3, counts, d_total=d_total)
    U, W = oracle_state(V, d, 3, d_total)
    th, al = oracle.build_alias(counts)
    off, ctx, out = examples(V, n, max_ctx, rng, empty=True)
    got = sh.cbow_dotprod(dev(off), dev(ctx), dev(out), k, 99).cpu().numpy()
    ref = oracle.cbow_dotprod(U, W, off, ctx, out, k, 99, th, al)
    rows = np.concatenate([out[:, None], oracle.negatives(out, k, 99, th, al)], axis=1)
    err = dot_error(got, ref, mean_abs_rows(U, off, ctx), W, np.arange(n), rows)
    say("  dot error", err)
    assert err <= TOL1
    empty = np.diff(off.astype(np.int64)) == 0
    assert np.all(got[empty] == 0)
    sh.status()
    sh.destroy()


@pytest.mark.parametrize("V,d,d_total,n,k,max_ctx", SHAPES)
def test_cbow_adjust_parity(V, d, d_total, n, k, max_ctx):
    say("cbow adjust", V, d, n, k, max_ctx)
    rng = np.random.default_rng(V + d + n + 1)
    counts = zipf_counts(V)
    sh = make_shard(V, d, 4, counts, d_total=d_total)
    U, W = oracle_state(V, d, 4, d_total)
    th, al = oracle.build_alias(counts)
    off, ctx, out = examples(V, n, max_ctx, rng, empty=True)
    g = workloads.uniform_coeffs(n, k + 1, 5)
    sh.cbow_adjust(dev(off), dev(ctx), dev(out), k, 1234, torch.from_numpy(g).cuda(), 0.025)
    oracle.cbow_adjust(U, W, off, ctx, out, k, 1234, th, al, g, 0.025)
    eu, ew = vec_error(all_rows(sh, 0), U), vec_error(all_rows(sh, 1), W)
    say("  errors", eu, ew)
    assert eu <= TOL1 and ew <= TOL1
    sh.status()
    sh.destroy()


@pytest.mark.parametrize("S,d,V,n,k", [(1, 300, 4000, 3000, 5), (1, 60, 3000, 5000, 5), (5, 60, 2000, 2049, 5),
                                       (3, 20, 500, 300, 10), (1, 128, 1000, 2000, 0)])
def test_cbow_train_minibatch_parity(S, d, V, n, k):
    say("cbow train", S, d, V, n, k)
    rng = np.random.default_rng(S * 1000 + d)
    counts = zipf_counts(V)
    th, al = oracle.build_alias(counts)
    dt = S * d
    shards = [make_shard(V, d, 8, counts, d_total=dt, col_begin=s * d) for s in range(S)]
    st = [oracle_state(V, d, 8, dt, s * d) for s in range(S)]
    Us, Ws = [a for a, _ in st], [b for _, b in st]
    off, ctx, out = examples(V, n, 16, rng)
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    goff, gctx, gout = dev(off), dev(ctx), dev(out)
    for step in range(2):
        seed = w2v.minibatch_seed(11, step)
        w2v.cbow_train_minibatch(shards, goff, gctx, gout, k, seed, 0.025, loss=loss)
        ref_loss = oracle.cbow_train_minibatch(Us, Ws, off, ctx, out, k, seed, th, al, 0.025)
        assert abs(loss.item() - ref_loss) <= 1e-5 * abs(ref_loss)
    for s in range(S):
        eu, ew = vec_error(all_rows(shards[s], 0), Us[s]), vec_error(all_rows(shards[s], 1), Ws[s])
        say("  shard", s, eu, ew)
        assert eu <= 2 * TOL1 and ew <= 2 * TOL1
        shards[s].status()
        shards[s].destroy()


def test_cbow_heavy_rows_and_reproducibility():
    # every example has the same center and draws its contexts from three words: the longest
    # possible runs on both sides (many levels of partial sums), checked against the closed form
    # the oracle gives, and run twice for bitwise equality.
    V, d, n, k = 50, 60, 40_000, 2
    counts = np.ones(V, np.uint64)
    th, al = oracle.build_alias(counts)
    rng = np.random.default_rng(9)
    lens = rng.integers(1, 9, n)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    ctx = rng.integers(0, 3, int(off[-1])).astype(np.uint32)
    out = np.full(n, 7, np.uint32)
    g = workloads.uniform_coeffs(n, k + 1, 6) * np.float32(1e-2)
    results = []
    for rep in range(2):
        sh = make_shard(V, d, 2, counts)
        sh.cbow_adjust(dev(off), dev(ctx), dev(out), k, 55, torch.from_numpy(g).cuda(), 0.05)
        results.append((all_rows(sh, 0), all_rows(sh, 1)))
        sh.status()
        sh.destroy()
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    U, W = oracle_state(V, d, 2)
    oracle.cbow_adjust(U, W, off, ctx, out, k, 55, th, al, g, 0.05)
    eu, ew = vec_error(results[0][0], U), vec_error(results[0][1], W)
    say("  heavy rows", eu, ew)
    assert eu <= TOL1 and ew <= TOL1


@pytest.mark.parametrize("B,t", [(1, 0.0), (5, 1e-3), (8, 1e-2)])
def test_make_cbow_examples_bit_exact(B, t):
    rng = np.random.default_rng(20 + B)
    V, n_tok = 300, 30_011
    tokens = workloads.zipf_draw(workloads.zipf_cdf(V, 1.0), n_tok, rng)
    counts = workloads.counted(tokens, V)
    lens = rng.integers(0, 45, 3000)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.append(off[off < n_tok], n_tok).astype(np.uint64)
    sh = make_shard(V, 4, 1, counts, t=t)
    kt = oracle.build_keep(counts, t) if t > 0 else None
    base = (1 << 35) + 5
    doff = torch.from_numpy(off.astype(np.int64)).cuda()
    co = torch.empty(n_tok + 1, dtype=torch.int32, device="cuda")
    cx = torch.empty(n_tok * 2 * B, dtype=torch.int32, device="cuda")
    ce = torch.empty(n_tok, dtype=torch.int32, device="cuda")
    n_ex, n_ctx = sh.make_cbow_examples(dev(tokens), doff, base, 1, 77, B, co, cx, ce)
    ooff, octx, oout, ocnt, onctx = oracle.make_cbow_examples(tokens, off, base, 1, 77, B, kt)
    assert (n_ex, n_ctx) == (ocnt, onctx) and n_ex > 0
    assert np.array_equal(w2v.index_to_numpy(co[:n_ex + 1]), ooff)
    assert np.array_equal(w2v.index_to_numpy(cx[:n_ctx]), octx)
    assert np.array_equal(w2v.index_to_numpy(ce[:n_ex]), oout)
    # short outputs: prefixes, full counts
    co2 = torch.empty(101, dtype=torch.int32, device="cuda")
    cx2 = torch.empty(150, dtype=torch.int32, device="cuda")
    ce2 = torch.empty(100, dtype=torch.int32, device="cuda")
    n2, m2 = sh.make_cbow_examples(dev(tokens), doff, base, 1, 77, B, co2, cx2, ce2)
    assert (n2, m2) == (n_ex, n_ctx)
    assert np.array_equal(w2v.index_to_numpy(co2), ooff[:101])
    assert np.array_equal(w2v.index_to_numpy(ce2), oout[:100])
    assert np.array_equal(w2v.index_to_numpy(cx2), octx[:150])
    sh.status()
    sh.destroy()


def test_cbow_hundred_minibatches_from_text():
    wl = workloads.WORKLOADS["tiny"]
    tokens, soff = workloads.corpus(wl)
    counts = workloads.counted(tokens, wl.V)
    th, al = oracle.build_alias(counts)
    kt = oracle.build_keep(counts, wl.subsample_t)
    sh = make_shard(wl.V, wl.d_slice, wl.seed, counts, init_mode=0, t=wl.subsample_t)
    U, W = oracle_state(wl.V, wl.d_slice, wl.seed, init_mode=0)
    n_tok = tokens.size
    co = torch.empty(n_tok + 1, dtype=torch.int32, device="cuda")
    cx = torch.empty(n_tok * 2 * wl.window, dtype=torch.int32, device="cuda")
    ce = torch.empty(n_tok, dtype=torch.int32, device="cuda")
    n_ex, n_ctx = sh.make_cbow_examples(dev(tokens), torch.from_numpy(soff.astype(np.int64)).cuda(), 0, 0,
                                        wl.seed, wl.window, co, cx, ce)
    ooff, octx, oout, ocnt, onctx = oracle.make_cbow_examples(tokens, soff, 0, 0, wl.seed, wl.window, kt)
    assert (n_ex, n_ctx) == (ocnt, onctx)
    nb, n = 100, 512
    assert n_ex >= nb * n
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    losses, ref_losses = [], []
    for h in range(nb):
        a, b = h * n, (h + 1) * n
        lo, hi = int(ooff[a]), int(ooff[b])
        seed = w2v.minibatch_seed(wl.seed, h)
        goff = (co[a:b + 1] - co[a]).contiguous()
        w2v.cbow_train_minibatch([sh], goff, cx[lo:hi].contiguous(), ce[a:b].contiguous(), wl.k, seed,
                                 wl.alpha, loss=loss)
        losses.append(loss.item())
        ref_losses.append(oracle.cbow_train_minibatch([U], [W], ooff[a:b + 1] - ooff[a], octx[lo:hi],
                                                      oout[a:b], wl.k, seed, th, al, wl.alpha))
        if h == 0:
            e1 = max(vec_error(all_rows(sh, 0), U), vec_error(all_rows(sh, 1), W))
            say("  after 1 minibatch:", e1)
            assert e1 <= TOL1
    eu, ew = vec_error(all_rows(sh, 0), U), vec_error(all_rows(sh, 1), W)
    say("  after", nb, "minibatches:", eu, ew, "loss", losses[0], "->", losses[-1])
    assert eu <= TOL100 and ew <= TOL100
    assert np.allclose(losses, ref_losses, rtol=1e-4)
    assert np.mean(losses[-10:]) < np.mean(losses[:10])
    sh.status()
    sh.destroy()


def test_cbow_bad_offsets_and_words_raise_the_flag_without_a_fault():
    V = 100
    sh = make_shard(V, 60, 1, np.ones(V, np.uint64))
    out = dev(np.array([1, 2, 3], np.uint32))
    ctx = dev(np.array([4, 5, 6, 7, 8], np.uint32))
    good = dev(np.array([0, 2, 3, 5], np.uint32))
    sh.cbow_dotprod(good, ctx, out, 3, 1)
    sh.status()
    for bad in ([0, 4, 3, 5], [1, 2, 3, 5], [0, 2, 3, 4], [0, 2, 3, 4_000_000_000]):
        sh.cbow_dotprod(dev(np.array(bad, np.uint32)), ctx, out, 3, 1)
        with pytest.raises(w2v.W2VError) as e:
            sh.status()
        assert e.value.code == -6
        sh.cbow_adjust(dev(np.array(bad, np.uint32)), ctx, out, 3, 1,
                       torch.zeros((3, 4), dtype=torch.float32, device="cuda"), 0.1)
        with pytest.raises(w2v.W2VError):
            sh.status()
    sh.cbow_dotprod(good, dev(np.array([4, 5, 100, 7, 8], np.uint32)), out, 3, 1)
    with pytest.raises(w2v.W2VError) as e:
        sh.status()
    assert e.value.code == -6
    with pytest.raises(w2v.W2VError) as e:
        sh.cbow_dotprod(good, ctx, out, 65, 1)
    assert e.value.code == -2
    sh.status()
    sh.destroy()


@pytest.mark.parametrize("V,d,n,k,ctx_len", [(2, 60, 50, 3, 5), (1000, 60, 3, 64, 2000), (300, 300, 1, 5, 1),
                                             (5000, 8, 9000, 1, 3)])
def test_cbow_edge_shapes(V, d, n, k, ctx_len):
    say("cbow edge", V, d, n, k, ctx_len)
    rng = np.random.default_rng(V + n)
    counts = zipf_counts(V)
    th, al = oracle.build_alias(counts)
    sh = make_shard(V, d, 6, counts)
    U, W = oracle_state(V, d, 6)
    lens = np.full(n, ctx_len)
    lens[0] = 0 if n > 1 else ctx_len            # an empty context in front
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    ctx = rng.integers(0, V, int(off[-1])).astype(np.uint32)
    out = rng.integers(0, V, n).astype(np.uint32)
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    alpha = 0.025 if V > 2 else 1e-4
    w2v.cbow_train_minibatch([sh], dev(off), dev(ctx), dev(out), k, 31, alpha, loss=loss)
    ref = oracle.cbow_train_minibatch([U], [W], off, ctx, out, k, 31, th, al, alpha)
    eu, ew = vec_error(all_rows(sh, 0), U), vec_error(all_rows(sh, 1), W)
    say("  errors", eu, ew)
    assert eu <= TOL1 and ew <= TOL1 and abs(loss.item() - ref) <= 1e-5 * abs(ref)
    sh.status()
    sh.destroy()


def test_cbow_no_examples_and_no_text():
    V = 50
    sh = make_shard(V, 12, 1, np.ones(V, np.uint64))
    before = (all_rows(sh, 0), all_rows(sh, 1))
    empty = torch.empty(0, dtype=torch.int32, device="cuda")
    loss = torch.ones(1, dtype=torch.float64, device="cuda")
    w2v.cbow_train_minibatch([sh], dev(np.zeros(1, np.uint32)), empty, empty, 5, 1, 0.1, loss=loss)
    assert loss.item() == 0.0
    # examples whose contexts are all empty: nothing moves
    off = dev(np.zeros(4, np.uint32))
    w2v.cbow_train_minibatch([sh], off, empty, dev(np.array([1, 2, 3], np.uint32)), 5, 1, 0.1)
    assert np.array_equal(all_rows(sh, 0), before[0]) and np.array_equal(all_rows(sh, 1), before[1])
    # text of one-word sentences gives no example; so does no text at all
    co = torch.full((11,), 7, dtype=torch.int32, device="cuda")
    cx = torch.empty(40, dtype=torch.int32, device="cuda")
    ce = torch.empty(10, dtype=torch.int32, device="cuda")
    toks = dev(np.arange(10, dtype=np.uint32))
    n_ex, n_ctx = sh.make_cbow_examples(toks, torch.arange(11, dtype=torch.int64, device="cuda"), 0, 0, 1, 3,
                                        co, cx, ce)
    assert (n_ex, n_ctx) == (0, 0) and co[0].item() == 0
    co.fill_(7)
    n_ex, n_ctx = sh.make_cbow_examples(empty, torch.zeros(1, dtype=torch.int64, device="cuda"), 0, 0, 1, 3,
                                        co, cx, ce)
    assert (n_ex, n_ctx) == (0, 0) and co[0].item() == 0
    sh.status()
    sh.destroy()


@pytest.mark.parametrize("S,V,d,k,max_ctx,empty", [(1, 3000, 300, 5, 12, False), (1, 2000, 60, 10, 20, True),
                                                   (3, 1500, 100, 5, 8, False), (1, 30, 64, 2, 40, True)])
def test_announced_cbow_minibatches_give_the_same_bits(S, V, d, k, max_ctx, empty):
    # each minibatch announced one step ahead (w2v_cbow_prefetch_minibatch): the fused step, the
    # step over several shards and the two calls must give the bits of shards that were told nothing
    say("announced cbow", S, V, d, k)
    n, steps = 2049, 4
    rng = np.random.default_rng(V + S)
    counts = zipf_counts(V)
    data = []
    for _ in range(steps + 1):
        off, ctx, ctr = examples(V, n, max_ctx, rng, empty=empty)
        data.append((dev(off), dev(ctx), dev(ctr)))
    seeds = [w2v.minibatch_seed(4, h) for h in range(steps + 1)]
    cuts = [(0, d)] if S == 1 else [(0, 20), (20, 50), (70, d - 70)]
    told = [make_shard(V, w, 5, counts, d_total=d, col_begin=b) for b, w in cuts]
    plain = [make_shard(V, w, 5, counts, d_total=d, col_begin=b) for b, w in cuts]
    la, lb = (torch.zeros(1, dtype=torch.float64, device="cuda") for _ in range(2))
    told[0].cbow_prefetch_minibatch(*data[0], k, seeds[0])
    for h in range(steps):
        told[0].cbow_prefetch_minibatch(*data[h + 1], k, seeds[h + 1])
        w2v.cbow_train_minibatch(told, *data[h], k, seeds[h], 0.02, loss=la)
        w2v.cbow_train_minibatch(plain, *data[h], k, seeds[h], 0.02, loss=lb)
        assert la.item() == lb.item()
    for a, b in zip(told, plain):
        for which in (0, 1):
            assert np.array_equal(all_rows(a, which), all_rows(b, which))
    # the two calls on the first shard: dots from the announced set, then the update spends it;
    # a mismatching announcement (other seed) is ignored
    g = torch.from_numpy(workloads.uniform_coeffs(n, k + 1, 9)).cuda()
    told[0].cbow_prefetch_minibatch(*data[steps], k, seeds[steps] + 1)
    da = told[0].cbow_dotprod(*data[steps], k, seeds[steps]).cpu().numpy()
    dp = plain[0].cbow_dotprod(*data[steps], k, seeds[steps]).cpu().numpy()
    assert np.array_equal(da, dp)
    told[0].cbow_adjust(*data[steps], k, seeds[steps], g, 0.02)
    plain[0].cbow_adjust(*data[steps], k, seeds[steps], g, 0.02)
    for which in (0, 1):
        assert np.array_equal(all_rows(told[0], which), all_rows(plain[0], which))
    for s in told + plain:
        s.status()
        s.destroy()
    # and the oracle agrees with the announced fused step
    if S == 1:
        sh = make_shard(V, d, 5, counts)
        U, W = oracle_state(V, d, 5)
        th, al = oracle.build_alias(counts)
        for h in range(2):
            sh.cbow_prefetch_minibatch(*data[h], k, seeds[h])
            w2v.cbow_train_minibatch([sh], *data[h], k, seeds[h], 0.02)
            oracle.cbow_train_minibatch([U], [W], *(w2v.index_to_numpy(x) for x in data[h]), k, seeds[h],
                                        th, al, 0.02)
        assert vec_error(all_rows(sh, 0), U) <= 2 * TOL1 and vec_error(all_rows(sh, 1), W) <= 2 * TOL1
        sh.status()
        sh.destroy()
