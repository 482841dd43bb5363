"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
inputs.  Integer results (tables, negatives, pairs) must match bit for bit; fp32 results within
1e-5 after one minibatch and 1e-3 after a hundred (error measures in tests/util.py).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_08495_amd import w2v, workloads
from util import all_rows, delta_error, dev, dot_error, set_all_rows, vec_error, vec_error_elem, zipf_counts

pytestmark = pytest.mark.gpu

TOL1 = 1e-5
TOL100 = 1e-3
TOL_ELEM = 1e-4     # element-relative measure (floor 1e-2 of the row's largest): reported, loosely bounded


def step_rows(out_idx, k, seed, th, al):
    """[n][k+1] output rows of a minibatch: the positive word, then the oracle's negatives."""
    return np.concatenate([out_idx[:, None], oracle.negatives(out_idx, k, seed, th, al)], axis=1)


def oracle_step_deltas(U, W, in_idx, out_idx, k, seed, th, al):
    """The summed changes (double) that one oracle training step would add, times 1/alpha."""
    rows = step_rows(out_idx, k, seed, th, al)
    g = oracle.coeffs([oracle.dots(U, W, in_idx, rows)])
    return oracle.adjust_deltas(U, W, in_idx, rows, g)


def safe_alpha(n, k, p_top, alpha_max=0.05):
    """A learning rate under which one minibatch moves the most frequently named row by about a
    tenth of itself at most (coefficients are about a half, vectors of about equal length), so that
    small vocabularies do not diverge, and no smaller than that, so that updates stay far above the
    tolerance."""
    m_top = max(1.0, n * (k + 1) * p_top)
    return float(min(alpha_max, 0.2 / m_top))


def say(*a):
    print(*a, flush=True)


def make_shard(V, d, seed, counts=None, t=0.0, d_total=None, col_begin=0, init_mode=1):
    sh = w2v.Shard(V, d, seed, d_total=d_total, col_begin=col_begin, init_mode=init_mode)
    if counts is not None:
        sh.set_counts(counts, t)
    return sh


def oracle_state(V, d, seed, d_total=None, col_begin=0, init_mode=1):
    rows = np.arange(V, dtype=np.uint32)
    dt = d if d_total is None else d_total
    U = oracle.init_rows(seed, dt, col_begin, d, 0, rows)
    W = oracle.init_rows(seed, dt, col_begin, d, 1, rows) if init_mode else np.zeros((V, d), np.float32)
    return U, W


# --- initial vectors and tables: bit exact ---------------------------------------------------

@pytest.mark.parametrize("V,d,d_total,col_begin,mode", [
    (1000, 60, 300, 60, 1), (300, 300, 300, 0, 0), (257, 7, 23, 5, 1), (64, 100, 100, 0, 1),
    (50, 1000, 1000, 0, 1), (33, 1, 1, 0, 1)])
def test_initial_vectors_bit_exact(V, d, d_total, col_begin, mode):
    say("init", V, d, d_total, col_begin, mode)
    sh = make_shard(V, d, 12345, d_total=d_total, col_begin=col_begin, init_mode=mode)
    U, W = oracle_state(V, d, 12345, d_total, col_begin, mode)
    assert np.array_equal(all_rows(sh, 0), U)
    assert np.array_equal(all_rows(sh, 1), W)
    sh.destroy()


def test_tables_bit_exact():
    V = 50_000
    counts = zipf_counts(V, 1.07, 3e8)
    counts[100:120] = 0
    sh = make_shard(V, 8, 1, counts, 1e-4)
    th, al, kp = sh.get_tables()
    oth, oal = oracle.build_alias(counts)
    assert np.array_equal(th, oth) and np.array_equal(al, oal)
    assert np.array_equal(kp, oracle.build_keep(counts, 1e-4))
    sh.set_counts(counts, 0.0)
    assert np.all(sh.get_tables()[2] == 2 ** 32)
    sh.destroy()


# --- negatives: bit exact ------------------------------------------------------------------------

@pytest.mark.parametrize("V,n,k,skew", [(2, 3000, 3, 12.0), (5, 5000, 4, 3.0), (1000, 4099, 5, 1.0),
                                        (100_000, 70_001, 25, 1.05), (3, 257, 64, 6.0)])
def test_negatives_bit_exact(V, n, k, skew):
    say("negatives", V, n, k, skew)
    rng = np.random.default_rng(V + k)
    counts = np.maximum(1, 1e12 / np.arange(1, V + 1) ** skew).astype(np.uint64)
    sh = make_shard(V, 4, 7, counts)
    th, al = oracle.build_alias(counts)
    out = (rng.random(n) ** 3 * V).astype(np.uint32)        # mostly the frequent words
    seed = 0x9E3779B97F4A7C15
    neg = w2v.index_to_numpy(sh.negatives(dev(out), k, seed))
    ref = oracle.negatives(out, k, seed, th, al)
    assert np.array_equal(neg, ref)
    assert not np.any(neg == out[:, None])
    sh.status()
    sh.destroy()


# --- dotprod ----------------------------------------------------------------------------------------

@pytest.mark.parametrize("V,d,n,k", [(5000, 60, 4099, 5), (3000, 300, 2050, 5), (2000, 100, 1000, 10),
                                     (1500, 200, 777, 25), (400, 7, 513, 0), (300, 1000, 300, 3),
                                     (900, 129, 1, 6), (64, 256, 65, 64)])
def test_dotprod_parity(V, d, n, k):
    say("dotprod", V, d, n, k)
    rng = np.random.default_rng(d + n)
    counts = zipf_counts(V)
    sh = make_shard(V, d, 99, counts)
    U, W = oracle_state(V, d, 99)
    th, al = oracle.build_alias(counts)
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    seed = 4242
    got = sh.dotprod(dev(in_idx), dev(out_idx), k, seed).cpu().numpy()
    ref = oracle.dotprod(U, W, in_idx, out_idx, k, seed, th, al)
    rows = np.concatenate([out_idx[:, None], oracle.negatives(out_idx, k, seed, th, al)], axis=1)
    err = dot_error(got, ref, U, W, in_idx, rows)
    say("  dot error", err)
    assert err <= TOL1
    # dotprod does not modify the shard
    assert np.array_equal(all_rows(sh, 0), U) and np.array_equal(all_rows(sh, 1), W)
    sh.status()
    sh.destroy()


def test_dotprod_empty_batch_and_zero_output_vectors():
    V, d = 100, 60
    counts = zipf_counts(V)
    sh = make_shard(V, d, 5, counts, init_mode=0)
    e = torch.empty(0, dtype=torch.int32, device="cuda")
    assert sh.dotprod(e, e, 5, 1).shape == (0, 6)
    idx = dev(np.arange(50, dtype=np.uint32))
    assert torch.all(sh.dotprod(idx, idx, 5, 1) == 0)
    sh.destroy()


# --- coefficients ------------------------------------------------------------------------------------

def test_coeffs_parity():
    rng = np.random.default_rng(3)
    n, k, S = 3001, 5, 3
    sh = make_shard(10, 4, 1)
    parts = [(rng.standard_normal((n, k + 1)) * 4).astype(np.float32) for _ in range(S)]
    parts[0][0, :] = 60.0
    parts[0][1, :] = -60.0
    got, loss = sh.coeffs([torch.from_numpy(p).cuda() for p in parts], k, want_loss=True)
    ref, ref_loss = oracle.coeffs(parts, want_loss=True)
    got = got.cpu().numpy()
    # the three float partials are added in float on the GPU and in double by the oracle: the sum
    # differs by a few ulp of its magnitude, and d(coefficient)/df <= 1/4
    ftot = np.sum([np.abs(p.astype(np.float64)) for p in parts], axis=0)
    assert np.all(np.abs(got - ref) <= 1e-6 * np.maximum(np.abs(ref), 1e-30) + 0.25 * 3e-7 * ftot)
    assert abs(float(loss.item()) - ref_loss) <= 1e-5 * abs(ref_loss)
    sh.destroy()


def test_loss_with_saturated_sigmoids_is_finite_and_the_same_in_both_forms():
    """Dots far out on either side (rows set by hand): the minibatch loss of the fused single-shard
    step, of the step over two column shards and of the client call must all be finite and agree
    with the oracle, whose loss term is log(1 + e^-x) evaluated without cancellation."""
    V, d, k = 64, 64, 3
    rng = np.random.default_rng(21)
    counts = np.ones(V, np.uint64)
    th, al = oracle.build_alias(counts)
    U = np.zeros((V, d), np.float32)
    W = np.zeros((V, d), np.float32)
    scale = np.linspace(-9.0, 9.0, V).astype(np.float32)       # dots u_a . v_b = scale_a * scale_b
    U[:, 0] = scale
    W[:, 0] = scale
    U[:, 1:] = (rng.random((V, d - 1), dtype=np.float32) - 0.5) * 1e-3
    W[:, 1:] = (rng.random((V, d - 1), dtype=np.float32) - 0.5) * 1e-3
    n = 3000
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    seed = 5
    one = make_shard(V, d, 1, counts)
    halves = [make_shard(V, 32, 1, counts, d_total=d, col_begin=0),
              make_shard(V, 32, 1, counts, d_total=d, col_begin=32)]
    set_all_rows(one, 0, U); set_all_rows(one, 1, W)
    for s, sh in enumerate(halves):
        set_all_rows(sh, 0, U[:, 32 * s:32 * s + 32]); set_all_rows(sh, 1, W[:, 32 * s:32 * s + 32])
    ref_dots = oracle.dotprod(U, W, in_idx, out_idx, k, seed, th, al)
    assert np.abs(ref_dots).max() > 70 and np.abs(ref_dots).min() < 1     # both regimes present
    _, ref_loss = oracle.coeffs([ref_dots], want_loss=True)
    assert np.isfinite(ref_loss)
    a, b = dev(in_idx), dev(out_idx)
    dots = one.dotprod(a, b, k, seed)
    _, client_loss = one.coeffs([dots], k, want_loss=True)
    l1 = torch.zeros(1, dtype=torch.float64, device="cuda")
    l2 = torch.zeros(1, dtype=torch.float64, device="cuda")
    w2v.train_minibatch([one], a, b, k, seed, 0.0, loss=l1)
    w2v.train_minibatch(halves, a, b, k, seed, 0.0, loss=l2)
    say("  saturated loss: oracle", ref_loss, "client", client_loss.item(), "fused", l1.item(), "two shards", l2.item())
    for got in (client_loss.item(), l1.item(), l2.item()):
        assert np.isfinite(got) and abs(got - ref_loss) <= 1e-5 * ref_loss
    for sh in [one] + halves:
        sh.status()
        sh.destroy()


# --- adjust ------------------------------------------------------------------------------------------

def run_adjust_case(V, d, n, k, in_idx, out_idx, seed=77, alpha=0.025, label=""):
    counts = zipf_counts(V)
    sh = make_shard(V, d, 31, counts)
    U, W = oracle_state(V, d, 31)
    th, al = oracle.build_alias(counts)
    g = workloads.uniform_coeffs(n, k + 1, seed)
    dU, dW = oracle.adjust_deltas(U, W, in_idx, step_rows(out_idx, k, seed, th, al), g)
    U0, W0 = U.copy(), W.copy()
    sh.adjust(dev(in_idx), dev(out_idx), k, seed, torch.from_numpy(g).cuda(), alpha)
    oracle.adjust(U, W, in_idx, out_idx, k, seed, th, al, g, alpha)
    gU, gW = all_rows(sh, 0), all_rows(sh, 1)
    eu, ew = vec_error(gU, U), vec_error(gW, W)
    du, dw = delta_error(gU, U0, alpha, dU), delta_error(gW, W0, alpha, dW)
    say("  adjust", label, "U error", eu, "W error", ew, "| change of U", du, "of W", dw,
        "| element-relative", vec_error_elem(gU, U), vec_error_elem(gW, W))
    assert du <= TOL1 and dw <= TOL1, (du, dw)
    assert vec_error_elem(gU, U) <= TOL_ELEM and vec_error_elem(gW, W) <= TOL_ELEM
    sh.status()
    sh.destroy()
    return eu, ew


@pytest.mark.parametrize("V,d,n,k", [(3000, 60, 4099, 5), (2000, 300, 2050, 5), (50, 100, 3000, 5),
                                     (4000, 200, 999, 25), (30, 7, 1025, 2), (500, 1000, 200, 3),
                                     (7, 16, 1, 0), (100, 128, 257, 10), (300, 60, 130, 64),
                                     (2, 300, 700, 1), (20_000, 60, 127, 10), (9, 300, 4096, 5)])
def test_adjust_parity(V, d, n, k):
    say("adjust", V, d, n, k)
    rng = np.random.default_rng(V + d)
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    eu, ew = run_adjust_case(V, d, n, k, in_idx, out_idx)
    assert eu <= TOL1 and ew <= TOL1


def test_adjust_heavy_rows_many_levels():
    # every pair shares one input word and one output word: both runs span every chunk, so the
    # partial sums go through several levels of the reduction (T13)
    V, d, n, k = 10, 60, 20_000, 1
    in_idx = np.full(n, 3, np.uint32)
    out_idx = np.full(n, 7, np.uint32)
    eu, ew = run_adjust_case(V, d, n, k, in_idx, out_idx, label="heavy")
    assert eu <= TOL1 and ew <= TOL1
    # a Zipf(1.2)-like head: word 0 takes a fifth of the pairs
    rng = np.random.default_rng(8)
    V, d, n, k = 2000, 200, 30_000, 5
    cdf = workloads.zipf_cdf(V, 1.2)
    in_idx = workloads.zipf_draw(cdf, n, rng)
    out_idx = workloads.zipf_draw(cdf, n, rng)
    eu, ew = run_adjust_case(V, d, n, k, in_idx, out_idx, label="zipf1.2")
    assert eu <= TOL1 and ew <= TOL1


def test_adjust_reads_start_of_call_vectors():
    # the same pair twice in one call gives exactly twice the change of one call (T8)
    V, d = 6, 60
    sh = make_shard(V, d, 3, np.ones(V, np.uint64))
    U0, W0 = all_rows(sh, 0), all_rows(sh, 1)
    a, b = np.array([2, 2], np.uint32), np.array([4, 4], np.uint32)
    g = torch.tensor([[0.3], [0.3]], dtype=torch.float32, device="cuda")
    sh.adjust(dev(a), dev(b), 0, 1, g, 1.0)
    U1, W1 = all_rows(sh, 0), all_rows(sh, 1)
    np.testing.assert_allclose(U1[2] - U0[2], 2 * np.float32(0.3) * W0[4], rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(W1[4] - W0[4], 2 * np.float32(0.3) * U0[2], rtol=1e-6, atol=1e-9)
    untouched = [r for r in range(V) if r != 2]
    assert np.array_equal(U1[untouched], U0[untouched])
    sh.destroy()


def test_adjust_null_updates_are_bitwise_noops():
    rng = np.random.default_rng(9)
    V, d, n, k = 200, 100, 1500, 5
    counts = zipf_counts(V)
    sh = make_shard(V, d, 4, counts)
    U0, W0 = all_rows(sh, 0), all_rows(sh, 1)
    in_idx, out_idx = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    g = torch.from_numpy(workloads.uniform_coeffs(n, k + 1, 1)).cuda()
    sh.adjust(in_idx, out_idx, k, 5, g, 0.0)
    assert np.array_equal(all_rows(sh, 0), U0) and np.array_equal(all_rows(sh, 1), W0)
    sh.adjust(in_idx, out_idx, k, 5, torch.zeros_like(g), 0.5)
    assert np.array_equal(all_rows(sh, 0), U0) and np.array_equal(all_rows(sh, 1), W0)
    sh.adjust(in_idx[:0], out_idx[:0], k, 5, g[:0], 0.5)
    assert np.array_equal(all_rows(sh, 0), U0)
    sh.destroy()


def test_runs_are_bitwise_reproducible():
    rng = np.random.default_rng(10)
    V, d, n, k = 500, 300, 6000, 5
    counts = zipf_counts(V)
    in_idx, out_idx = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    results = []
    for rep in range(2):
        sh = make_shard(V, d, 8, counts)
        dots = sh.dotprod(in_idx, out_idx, k, 123).cpu().numpy()
        loss = torch.zeros(1, dtype=torch.float64, device="cuda")
        for h in range(3):
            w2v.train_minibatch([sh], in_idx, out_idx, k, 1000 + h, 0.025, loss=loss)
        results.append((dots, all_rows(sh, 0), all_rows(sh, 1), loss.item()))
        sh.destroy()
    for a, b in zip(results[0], results[1]):
        assert np.array_equal(a, b)


# --- the whole step --------------------------------------------------------------------------------

@pytest.mark.parametrize("V,d,n,k,mode", [(3000, 300, 4099, 5, 1), (2000, 60, 2500, 5, 1),
                                          (800, 100, 4096, 5, 0), (500, 200, 1111, 25, 1),
                                          (40, 300, 1, 5, 1), (5, 60, 3000, 64, 1), (600, 320, 515, 10, 1)])
def test_train_minibatch_parity_one_shard(V, d, n, k, mode):
    say("train S=1", V, d, n, k, mode)
    rng = np.random.default_rng(n)
    counts = zipf_counts(V)
    sh = make_shard(V, d, 21, counts, init_mode=mode)
    U, W = oracle_state(V, d, 21, init_mode=mode)
    th, al = oracle.build_alias(counts)
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    # (a handful of words named 10^5 times each would diverge under the usual learning rate; a
    # single pair must still move its rows by far more than the tolerance)
    alpha = safe_alpha(n, k, 1.0 / V)
    for h in range(2):
        in_idx = rng.integers(0, V, n).astype(np.uint32)
        out_idx = rng.integers(0, V, n).astype(np.uint32)
        seed = w2v.minibatch_seed(5, h)
        assert seed == oracle.minibatch_seed(5, h)
        gU0, gW0 = all_rows(sh, 0), all_rows(sh, 1)
        dU, dW = oracle_step_deltas(U, W, in_idx, out_idx, k, seed, th, al)
        w2v.train_minibatch([sh], dev(in_idx), dev(out_idx), k, seed, alpha, loss=loss)
        ref_loss = oracle.train_minibatch([U], [W], in_idx, out_idx, k, seed, th, al, alpha)
        assert abs(loss.item() - ref_loss) <= 1e-5 * abs(ref_loss)
        # the change of this minibatch alone, from the shard's own rows before it
        gU, gW = all_rows(sh, 0), all_rows(sh, 1)
        du, dw = delta_error(gU, gU0, alpha, dU), delta_error(gW, gW0, alpha, dW)
        say("  minibatch", h, "alpha", alpha, "change of U", du, "of W", dw)
        assert du <= (h + 1) * TOL1 and dw <= (h + 1) * TOL1
    eu, ew = vec_error(gU, U), vec_error(gW, W)
    say("  errors", eu, ew, "element-relative", vec_error_elem(gU, U), vec_error_elem(gW, W))
    assert eu <= 2 * TOL1 and ew <= 2 * TOL1      # two minibatches
    assert vec_error_elem(gU, U) <= TOL_ELEM and vec_error_elem(gW, W) <= TOL_ELEM
    sh.status()
    sh.destroy()


def test_train_minibatch_five_column_shards_match_one_wide_shard():
    # T4: S = 5 slices of 60 columns against the oracle's single 300-wide vectors
    rng = np.random.default_rng(55)
    V, n, k = 1500, 3000, 5
    counts = zipf_counts(V)
    shards = [make_shard(V, 60, 77, counts, d_total=300, col_begin=60 * s) for s in range(5)]
    U, W = oracle_state(V, 300, 77)
    assert np.array_equal(np.concatenate([all_rows(s, 0) for s in shards], axis=1), U)
    th, al = oracle.build_alias(counts)
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    # partial dots sum to the full dot
    parts = [s.dotprod(dev(in_idx), dev(out_idx), k, 9).cpu().numpy().astype(np.float64) for s in shards]
    full = oracle.dotprod(U, W, in_idx, out_idx, k, 9, th, al)
    rows = np.concatenate([out_idx[:, None], oracle.negatives(out_idx, k, 9, th, al)], axis=1)
    assert dot_error(np.sum(parts, axis=0), full, U, W, in_idx, rows) <= TOL1
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    w2v.train_minibatch(shards, dev(in_idx), dev(out_idx), k, 9, 0.05, loss=loss)
    ref_loss = oracle.train_minibatch([U], [W], in_idx, out_idx, k, 9, th, al, 0.05)
    assert abs(loss.item() - ref_loss) <= 1e-5 * abs(ref_loss)
    Ug = np.concatenate([all_rows(s, 0) for s in shards], axis=1)
    Wg = np.concatenate([all_rows(s, 1) for s in shards], axis=1)
    assert vec_error(Ug, U) <= TOL1 and vec_error(Wg, W) <= TOL1
    for s in shards:
        s.destroy()


def test_unequal_slices_and_two_call_form_match_the_fused_step():
    rng = np.random.default_rng(56)
    V, n, k = 400, 1200, 5
    counts = zipf_counts(V)
    cuts = [(0, 7), (7, 143), (150, 150)]
    shards = [make_shard(V, w, 3, counts, d_total=300, col_begin=b) for b, w in cuts]
    one = make_shard(V, 300, 3, counts)
    in_idx, out_idx = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    w2v.train_minibatch(shards, in_idx, out_idx, k, 1, 0.05)
    w2v.train_minibatch([one], in_idx, out_idx, k, 1, 0.05)
    Ug = np.concatenate([all_rows(s, 0) for s in shards], axis=1)
    Wg = np.concatenate([all_rows(s, 1) for s in shards], axis=1)
    assert vec_error(Ug, all_rows(one, 0)) <= TOL1 and vec_error(Wg, all_rows(one, 1)) <= TOL1
    for s in shards + [one]:
        s.destroy()


def test_tiny_config_hundred_minibatches():
    # BASELINE config 1: V = 10,000, d = 100, window 5, k = 5, t = 1e-4, minibatches of 4096 pairs
    wl = workloads.WORKLOADS["tiny"]
    tokens, off = workloads.corpus(wl)
    counts = workloads.counted(tokens, wl.V)
    sh = make_shard(wl.V, wl.d_slice, wl.seed, counts, wl.subsample_t, init_mode=0)
    U, W = oracle_state(wl.V, wl.d_slice, wl.seed, init_mode=0)
    th, al = oracle.build_alias(counts)
    kt = oracle.build_keep(counts, wl.subsample_t)
    cap = tokens.size * 2 * wl.window
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    off_dev = torch.from_numpy(off.astype(np.int64)).cuda()
    cnt = sh.make_pairs(dev(tokens), off_dev, 0, 0, wl.seed, wl.window, gi, go)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, 0, 0, wl.seed, wl.window, kt)
    assert cnt == ocnt
    assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi) and np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    nb = min(100, cnt // wl.n_pairs)
    say("  tiny config:", cnt, "pairs,", nb, "minibatches")
    assert nb >= 100
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    losses, ref_losses = [], []
    for h in range(nb):
        a, b = h * wl.n_pairs, (h + 1) * wl.n_pairs
        seed = w2v.minibatch_seed(wl.seed, h)
        if h + 1 < nb and h % 3 != 2:      # as the benchmark loop does: the next minibatch announced
            sh.prefetch_minibatch(gi[b:b + wl.n_pairs], go[b:b + wl.n_pairs], wl.k,
                                  w2v.minibatch_seed(wl.seed, h + 1))   # (every third one is not)
        w2v.train_minibatch([sh], gi[a:b], go[a:b], wl.k, seed, wl.alpha, loss=loss)
        losses.append(loss.item())
        ref_losses.append(oracle.train_minibatch([U], [W], oi[a:b], oo[a:b], wl.k, seed, th, al, wl.alpha))
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


@pytest.mark.parametrize("V,d,n,k,mode", [(10_000, 100, 4096, 5, 0), (3000, 300, 1000, 5, 1),
                                          (500, 60, 257, 10, 1), (40, 64, 1, 0, 1)])
def test_captured_step_replays_give_the_same_bits_as_the_plain_call(V, d, n, k, mode):
    """w2v_step_graph: every replay (different indices, seed and learning rate each time, eager
    work and synchronisations in between) must leave the same bits as w2v_train_minibatch on a
    shard that was never captured, the loss included -- and both agree with the oracle."""
    say("captured step", V, d, n, k, mode)
    rng = np.random.default_rng(V + n)
    counts = zipf_counts(V)
    cdf = workloads.zipf_cdf(V, 1.0)
    plain = make_shard(V, d, 9, counts, init_mode=mode)
    graphed = make_shard(V, d, 9, counts, init_mode=mode)
    U, W = oracle_state(V, d, 9, init_mode=mode)
    th, al = oracle.build_alias(counts)
    la = torch.zeros(1, dtype=torch.float64, device="cuda")
    lb = torch.zeros(1, dtype=torch.float64, device="cuda")
    graph = w2v.StepGraph(graphed, n, k, loss=lb)
    steps = 7
    for h in range(steps):
        in_idx, out_idx = workloads.zipf_draw(cdf, n, rng), workloads.zipf_draw(cdf, n, rng)
        a, b = dev(in_idx), dev(out_idx)
        seed, alpha = w2v.minibatch_seed(77, h), 0.05 / (1 + h)
        w2v.train_minibatch([plain], a, b, k, seed, alpha, loss=la)
        graph.run(a, b, seed, alpha)
        if h % 2:                                # eager work on the captured shard between replays
            assert np.array_equal(graphed.dotprod(a, b, k, seed).cpu().numpy(),
                                  plain.dotprod(a, b, k, seed).cpu().numpy())
        torch.cuda.synchronize()
        assert la.item() == lb.item(), h
        for which in (0, 1):
            assert np.array_equal(all_rows(graphed, which), all_rows(plain, which)), (h, which)
        ref_loss = oracle.train_minibatch([U], [W], in_idx, out_idx, k, seed, th, al, alpha)
        assert abs(lb.item() - ref_loss) <= 1e-5 * abs(ref_loss) + 1e-12
    assert vec_error(all_rows(graphed, 0), U) <= steps * TOL1
    assert vec_error(all_rows(graphed, 1), W) <= steps * TOL1
    # a plain call on the captured shard in between leaves the graph usable
    a, b = dev(workloads.zipf_draw(cdf, n, rng)), dev(workloads.zipf_draw(cdf, n, rng))
    w2v.train_minibatch([graphed], a, b, k, 5, 0.01)
    w2v.train_minibatch([plain], a, b, k, 5, 0.01)
    graph.run(b, a, 6, 0.02)
    w2v.train_minibatch([plain], b, a, k, 6, 0.02, loss=la)
    torch.cuda.synchronize()
    assert la.item() == lb.item()
    for which in (0, 1):
        assert np.array_equal(all_rows(graphed, which), all_rows(plain, which))
    with pytest.raises(ValueError):
        graph.run(a[:-1], b[:-1], 1, 0.1) if n > 1 else graph.run(torch.cat([a, a]), torch.cat([b, b]), 1, 0.1)
    # a larger call moves the shard's scratch region: the captured step must refuse to run
    big = dev(rng.integers(0, V, 8 * n + 4096))
    w2v.train_minibatch([graphed], big, big, k, 9, 0.0)
    with pytest.raises(w2v.W2VError) as e:
        graph.run(a, b, 7, 0.01)
    assert e.value.code == -5
    graph.destroy()
    for sh in (plain, graphed):
        sh.status()
        sh.destroy()


@pytest.mark.parametrize("V,d,n,k", [(3000, 100, 5000, 5), (40, 300, 20_000, 3), (5000, 72, 180_000, 5),
                                     (300, 60, 3000, 5), (7, 520, 900, 2)])
def test_a_shard_kept_on_one_stream_gives_the_same_bits(V, d, n, k, monkeypatch):
    """A shard created with W2V_NO_OVERLAP=1 queues everything on the caller's stream; where the row
    geometry allows it carries the output side's walks, the input side's higher levels and the loss
    in joint launches.  Two-call form, fused step with loss, and a step over two column halves:
    the same bits as a shard that spreads the work over its own streams (few words: rows that
    collect thousands of contributions, several levels on both sides; 180 000 pairs: more loss terms
    than the joint launch takes)."""
    say("one stream", V, d, n, k)
    rng = np.random.default_rng(V * 31 + n)
    counts = zipf_counts(V)
    cdf = workloads.zipf_cdf(V, 1.0)
    half = (d // 2 + 3) // 4 * 4

    def shards():
        return (make_shard(V, d, 4, counts), make_shard(V, half, 4, counts, d_total=d),
                make_shard(V, d - half, 4, counts, d_total=d, col_begin=half))

    spread = shards()
    monkeypatch.setenv("W2V_NO_OVERLAP", "1")
    single = shards()
    monkeypatch.delenv("W2V_NO_OVERLAP")
    la = torch.zeros(1, dtype=torch.float64, device="cuda")
    lb = torch.zeros(1, dtype=torch.float64, device="cuda")
    for h in range(3):
        a, b = dev(workloads.zipf_draw(cdf, n, rng)), dev(workloads.zipf_draw(cdf, n, rng))
        coeffs_ = torch.tensor(rng.uniform(-1, 1, n * (k + 1)).astype(np.float32), device="cuda")
        seed, alpha = w2v.minibatch_seed(5, h), 0.03 / (1 + h)
        for group, loss in ((spread, la), (single, lb)):
            assert group[0].dotprod(a, b, k, seed).numel() == n * (k + 1)
            group[0].adjust(a, b, k, seed, coeffs_, alpha)                       # two-call form
            w2v.train_minibatch([group[0]], a, b, k, seed + 1, alpha, loss=loss)  # fused
        torch.cuda.synchronize()
        assert la.item() == lb.item(), h
        for group, loss in ((spread, la), (single, lb)):
            w2v.train_minibatch(list(group[1:]), a, b, k, seed + 2, alpha, loss=loss)   # S = 2
        torch.cuda.synchronize()
        assert la.item() == lb.item(), h
        for x, y in zip(spread, single):
            for which in (0, 1):
                assert np.array_equal(all_rows(x, which), all_rows(y, which)), (h, which)
    for sh in spread + single:
        sh.status()
        sh.destroy()


def test_tiny_config_hundred_minibatches_through_the_captured_step():
    # BASELINE config 1 again, every minibatch a replay of one captured step
    wl = workloads.WORKLOADS["tiny"]
    tokens, off = workloads.corpus(wl)
    counts = workloads.counted(tokens, wl.V)
    sh = make_shard(wl.V, wl.d_slice, wl.seed, counts, wl.subsample_t, init_mode=0)
    U, W = oracle_state(wl.V, wl.d_slice, wl.seed, init_mode=0)
    th, al = oracle.build_alias(counts)
    kt = oracle.build_keep(counts, wl.subsample_t)
    cap = tokens.size * 2 * wl.window
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    cnt = sh.make_pairs(dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda(), 0, 0, wl.seed,
                        wl.window, gi, go)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, 0, 0, wl.seed, wl.window, kt)
    assert cnt == ocnt and cnt // wl.n_pairs >= 100
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    graph = w2v.StepGraph(sh, wl.n_pairs, wl.k, loss=loss)
    losses, ref_losses = [], []
    for h in range(100):
        a, b = h * wl.n_pairs, (h + 1) * wl.n_pairs
        seed = w2v.minibatch_seed(wl.seed, h)
        graph.run(gi[a:b], go[a:b], seed, wl.alpha)
        losses.append(loss.item())
        ref_losses.append(oracle.train_minibatch([U], [W], oi[a:b], oo[a:b], wl.k, seed, th, al, wl.alpha))
        if h == 0:
            e1 = max(vec_error(all_rows(sh, 0), U), vec_error(all_rows(sh, 1), W))
            assert e1 <= TOL1
    eu, ew = vec_error(all_rows(sh, 0), U), vec_error(all_rows(sh, 1), W)
    say("  captured step, after 100 minibatches:", eu, ew, "loss", losses[0], "->", losses[-1])
    assert eu <= TOL100 and ew <= TOL100
    assert np.allclose(losses, ref_losses, rtol=1e-4)
    graph.destroy()
    sh.status()
    sh.destroy()


# --- pair formation: bit exact -------------------------------------------------------------------------

@pytest.mark.parametrize("B,t", [(1, 0.0), (5, 1e-3), (10, 1e-2), (3, 1e9)])
def test_make_pairs_bit_exact(B, t):
    rng = np.random.default_rng(B)
    V, n_tok = 300, 20_011
    tokens = workloads.zipf_draw(workloads.zipf_cdf(V, 1.0), n_tok, rng)
    counts = workloads.counted(tokens, V)
    lens = rng.integers(0, 45, 2000)                 # includes empty and one-word sentences
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.append(off[off < n_tok], n_tok).astype(np.uint64)
    sh = make_shard(V, 4, 1, counts, t)
    kt = oracle.build_keep(counts, t) if t > 0 else None
    base = (1 << 33) + 12345
    cap = n_tok * 2 * B
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    cnt = sh.make_pairs(dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda(), base, 3, 99, B, gi, go)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, base, 3, 99, B, kt)
    assert cnt == ocnt
    assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi)
    assert np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    # a too-small output still reports the full count and fills what fits
    gi2 = torch.empty(1000, dtype=torch.int32, device="cuda")
    go2 = torch.empty(1000, dtype=torch.int32, device="cuda")
    cnt2 = sh.make_pairs(dev(tokens), torch.from_numpy(off.astype(np.int64)).cuda(), base, 3, 99, B, gi2, go2)
    assert cnt2 == cnt and np.array_equal(w2v.index_to_numpy(gi2), oi[:1000])
    sh.status()
    sh.destroy()


@pytest.mark.parametrize("B,t,n_tok,n_sent", [(1, 0.0, 5_000, 600), (5, 1e-3, 20_011, 2000),
                                              (4, 1e-2, 70_001, 90), (3, 1e9, 3, 1)])
def test_make_pairs_interleaved_bit_exact(B, t, n_tok, n_sent):
    rng = np.random.default_rng(100 + B)
    V = 300
    tokens = workloads.zipf_draw(workloads.zipf_cdf(V, 1.0), n_tok, rng)
    counts = workloads.counted(tokens, V)
    lens = rng.integers(0, 2 * max(1, n_tok // n_sent) + 2, n_sent)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.append(off[off < n_tok], n_tok).astype(np.uint64)
    sh = make_shard(V, 4, 1, counts, t)
    kt = oracle.build_keep(counts, t) if t > 0 else None
    base = (1 << 34) + 777
    cap = n_tok * 2 * B
    doff = torch.from_numpy(off.astype(np.int64)).cuda()
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    cnt = sh.make_pairs(dev(tokens), doff, base, 2, 5, B, gi, go, interleaved=True)
    oi, oo, ocnt = oracle.make_pairs(tokens, off, base, 2, 5, B, kt, interleaved=True)
    assert cnt == ocnt
    assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi)
    assert np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    # the plain order is unchanged by a call of the other entry point on the same shard
    cnt0 = sh.make_pairs(dev(tokens), doff, base, 2, 5, B, gi, go)
    pi, po, pcnt = oracle.make_pairs(tokens, off, base, 2, 5, B, kt)
    assert cnt0 == pcnt and np.array_equal(w2v.index_to_numpy(gi[:cnt0]), pi)
    assert np.array_equal(w2v.index_to_numpy(go[:cnt0]), po)
    # a short output holds the first pairs of the interleaved order
    m = min(500, max(1, cnt // 2))
    gi2 = torch.empty(m, dtype=torch.int32, device="cuda")
    go2 = torch.empty(m, dtype=torch.int32, device="cuda")
    cnt2 = sh.make_pairs(dev(tokens), doff, base, 2, 5, B, gi2, go2, interleaved=True)
    k = min(m, cnt)
    assert cnt2 == cnt and np.array_equal(w2v.index_to_numpy(gi2)[:k], oi[:k])
    assert np.array_equal(w2v.index_to_numpy(go2)[:k], oo[:k])
    sh.status()
    sh.destroy()


# --- errors are reported, never faults -------------------------------------------------------------------

def test_argument_errors():
    sh = make_shard(100, 60, 1)
    idx = dev(np.arange(10, dtype=np.uint32))
    with pytest.raises(w2v.W2VError) as e:
        sh.dotprod(idx, idx, 5, 1)                        # no noise table yet
    assert e.value.code == -5
    sh.set_counts(np.ones(100, np.uint64))
    with pytest.raises(w2v.W2VError) as e:
        sh.dotprod(idx, idx, 65, 1)
    assert e.value.code == -2
    with pytest.raises(w2v.W2VError):
        w2v.Shard(0, 60, 1)
    with pytest.raises(w2v.W2VError):
        w2v.Shard(10, 2000, 1)
    other = make_shard(101, 60, 1, np.ones(101, np.uint64))
    with pytest.raises(w2v.W2VError) as e:
        w2v.train_minibatch([sh, other], idx, idx, 5, 1, 0.1)
    assert e.value.code == -7
    other.destroy()
    sh.destroy()


def test_out_of_range_index_raises_the_sticky_flag_without_a_fault():
    sh = make_shard(100, 60, 1, np.ones(100, np.uint64))
    bad = dev(np.array([1, 2, 100, 4_000_000_000], np.uint32))
    good = dev(np.array([1, 2, 3, 4], np.uint32))
    sh.dotprod(bad, good, 5, 1)
    with pytest.raises(w2v.W2VError) as e:
        sh.status()
    assert e.value.code == -6
    sh.status()                                           # cleared
    g = torch.zeros((4, 6), dtype=torch.float32, device="cuda")
    sh.adjust(good, bad, 5, 1, g, 0.1)
    with pytest.raises(w2v.W2VError):
        sh.status()
    w2v.train_minibatch([sh], bad, bad, 5, 1, 0.1)
    with pytest.raises(w2v.W2VError):
        sh.status()
    sh.get_rows(0, bad)
    with pytest.raises(w2v.W2VError):
        sh.status()
    sh.destroy()


# --- the C ABI from plain C ----------------------------------------------------------------------------

def test_plain_c_client_gets_the_same_bits_as_the_binding(tmp_path):
    """tests/c_client/abi_client.c (C99, gcc, no Python or torch) runs dotprod / coeffs / adjust /
    train_minibatch through the header; the binding must return the same bits for the same inputs."""
    import os
    import subprocess
    from paper_1606_08495_amd import build as hip_build
    if not os.path.exists(hip_build.C_CLIENT):
        hip_build.build_c_client()                       # a sub-second gcc compile
    out = tmp_path / "client.bin"
    r = subprocess.run([hip_build.C_CLIENT, str(out)], capture_output=True, text=True, timeout=300)
    say(r.stdout.strip(), r.stderr.strip())
    assert r.returncode == 0
    V, D, N, K = 1000, 64, 3000, 5
    T = K + 1
    raw = np.fromfile(out, dtype=np.uint8)
    pos = 0

    def take(dtype, count):
        nonlocal pos
        a = raw[pos:pos + np.dtype(dtype).itemsize * count].view(dtype)
        pos += a.nbytes
        return a
    in_idx, out_idx = take(np.uint32, N), take(np.uint32, N)
    c_dots, c_coeffs = take(np.float32, N * T).reshape(N, T), take(np.float32, N * T).reshape(N, T)
    c_loss = take(np.float64, 2)
    c_U, c_W = take(np.float32, V * D).reshape(V, D), take(np.float32, V * D).reshape(V, D)
    assert pos == raw.size
    counts = (1000000 // (np.arange(V, dtype=np.uint64) + 1) + 1).astype(np.uint64)
    sh = make_shard(V, D, 77, counts, 0.0, init_mode=1)
    a, b = dev(in_idx), dev(out_idx)
    seed = w2v.minibatch_seed(99, 0)
    dots = sh.dotprod(a, b, K, seed)
    g, loss0 = sh.coeffs([dots], K, want_loss=True)
    sh.adjust(a, b, K, seed, g, 0.05)
    loss1 = torch.zeros(1, dtype=torch.float64, device="cuda")
    w2v.train_minibatch([sh], a, b, K, w2v.minibatch_seed(99, 1), 0.05, loss=loss1)
    assert np.array_equal(dots.cpu().numpy(), c_dots) and np.array_equal(g.cpu().numpy(), c_coeffs)
    assert loss0.item() == c_loss[0] and loss1.item() == c_loss[1]
    assert np.array_equal(all_rows(sh, 0), c_U) and np.array_equal(all_rows(sh, 1), c_W)
    # and both agree with the oracle
    U, W = oracle_state(V, D, 77)
    th, al = oracle.build_alias(counts)
    oracle.train_minibatch([U], [W], in_idx, out_idx, K, seed, th, al, 0.05)
    oracle.train_minibatch([U], [W], in_idx, out_idx, K, w2v.minibatch_seed(99, 1), th, al, 0.05)
    assert vec_error(c_U, U) <= 2 * TOL1 and vec_error(c_W, W) <= 2 * TOL1
    sh.destroy()


# --- random shapes ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("case", range(24))
def test_random_shapes_skipgram_and_bag_of_words(case):
    """Shapes, skews and shard splits drawn at random inside the documented limits: one skip-gram
    step and one bag-of-words step per case against the oracle."""
    rng = np.random.default_rng(9000 + case)
    V = int(rng.choice([2, 3, 17, 100, 1000, 3000]))
    S = int(rng.choice([1, 1, 2, 3]))
    widths = [int(rng.integers(1, 120)) if S > 1 else int(rng.choice([1, 7, 60, 64, 65, 100, 128, 200, 257, 330]))
              for _ in range(S)]
    n = int(rng.choice([1, 2, 15, 16, 17, 300, 2047, 4097, 9000]))
    k = int(rng.choice([0, 1, 5, 5, 12, 31]))
    skew = float(rng.choice([0.0, 1.0, 2.5]))
    say("random case", case, "V", V, "widths", widths, "n", n, "k", k, "skew", skew)
    counts = np.maximum(1, 1e9 / np.arange(1, V + 1) ** skew).astype(np.uint64)
    th, al = oracle.build_alias(counts)
    dt = sum(widths)
    begins = np.concatenate([[0], np.cumsum(widths)[:-1]])
    cdf = workloads.zipf_cdf(V, skew)
    alpha = safe_alpha(n, k, float(cdf[0]), 0.02)
    for variant in ("sgns", "cbow"):
        shards = [make_shard(V, w, 31, counts, d_total=dt, col_begin=int(b)) for w, b in zip(widths, begins)]
        st = [oracle_state(V, w, 31, dt, int(b)) for w, b in zip(widths, begins)]
        Us, Ws = [a for a, _ in st], [b for _, b in st]
        out = workloads.zipf_draw(cdf, n, rng)
        loss = torch.zeros(1, dtype=torch.float64, device="cuda")
        deltas = None
        if variant == "sgns":
            inn = workloads.zipf_draw(cdf, n, rng)
            rows = step_rows(out, k, 4242, th, al)
            g = oracle.coeffs([oracle.dots(Us[s], Ws[s], inn, rows) for s in range(S)])
            deltas = [oracle.adjust_deltas(Us[s], Ws[s], inn, rows, g) for s in range(S)]
            before = [(Us[s].copy(), Ws[s].copy()) for s in range(S)]     # = the shards' initial rows
            w2v.train_minibatch(shards, dev(inn), dev(out), k, 4242, alpha, loss=loss)
            ref = oracle.train_minibatch(Us, Ws, inn, out, k, 4242, th, al, alpha)
        else:
            lens = rng.integers(0, 9, n)
            off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
            ctx = workloads.zipf_draw(cdf, int(off[-1]), rng)
            w2v.cbow_train_minibatch(shards, dev(off), dev(ctx), dev(out), k, 4242, alpha, loss=loss)
            ref = oracle.cbow_train_minibatch(Us, Ws, off, ctx, out, k, 4242, th, al, alpha)
        assert abs(loss.item() - ref) <= 1e-5 * abs(ref) + 1e-12
        for s in range(S):
            gU, gW = all_rows(shards[s], 0), all_rows(shards[s], 1)
            eu, ew = vec_error(gU, Us[s]), vec_error(gW, Ws[s])
            assert eu <= TOL1 and ew <= TOL1, (variant, s, eu, ew)
            if deltas is not None:
                du = delta_error(gU, before[s][0], alpha, deltas[s][0])
                dw = delta_error(gW, before[s][1], alpha, deltas[s][1])
                assert du <= TOL1 and dw <= TOL1, (variant, s, du, dw)
            shards[s].status()
            shards[s].destroy()


@pytest.mark.parametrize("case", range(12))
def test_random_text_blocks_pairs_interleaved_pairs_and_examples(case):
    rng = np.random.default_rng(7000 + case)
    V = int(rng.choice([2, 50, 5000]))
    n_tok = int(rng.choice([1, 2, 63, 4096, 4097, 30_000]))
    B = int(rng.choice([1, 2, 5, 10, 15]))
    t = float(rng.choice([0.0, 1e-4, 1e-2, 1e6]))
    max_len = int(rng.choice([1, 2, 8, 60, 1000]))
    say("text case", case, "V", V, "tokens", n_tok, "B", B, "t", t, "max sentence", max_len)
    tokens = workloads.zipf_draw(workloads.zipf_cdf(V, 1.0), n_tok, rng)
    counts = np.maximum(1, workloads.counted(tokens, V))
    lens = rng.integers(0, max_len + 1, n_tok + 1)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.append(off[off < n_tok], n_tok).astype(np.uint64)
    sh = make_shard(V, 4, 1, counts, t)
    kt = oracle.build_keep(counts, t) if t > 0 else None
    base, epoch, seed = int(rng.integers(0, 1 << 40)), int(rng.integers(0, 5)), int(rng.integers(0, 1 << 62))
    doff = torch.from_numpy(off.astype(np.int64)).cuda()
    cap = max(1, n_tok * 2 * B)
    gi = torch.empty(cap, dtype=torch.int32, device="cuda")
    go = torch.empty(cap, dtype=torch.int32, device="cuda")
    for inter in (False, True):
        cnt = sh.make_pairs(dev(tokens), doff, base, epoch, seed, B, gi, go, interleaved=inter)
        oi, oo, ocnt = oracle.make_pairs(tokens, off, base, epoch, seed, B, kt, interleaved=inter)
        assert cnt == ocnt
        assert np.array_equal(w2v.index_to_numpy(gi[:cnt]), oi) and np.array_equal(w2v.index_to_numpy(go[:cnt]), oo)
    co = torch.empty(n_tok + 1, dtype=torch.int32, device="cuda")
    ce = torch.empty(n_tok, dtype=torch.int32, device="cuda")
    n_ex, n_ctx = sh.make_cbow_examples(dev(tokens), doff, base, epoch, seed, B, co, go, ce)
    ooff, octx, oout, ocnt, onctx = oracle.make_cbow_examples(tokens, off, base, epoch, seed, B, kt)
    assert (n_ex, n_ctx) == (ocnt, onctx)
    assert np.array_equal(w2v.index_to_numpy(co[:n_ex + 1]), ooff)
    assert np.array_equal(w2v.index_to_numpy(go[:n_ctx]), octx)
    assert np.array_equal(w2v.index_to_numpy(ce[:n_ex]), oout)
    sh.status()
    sh.destroy()


# --- look-ahead ------------------------------------------------------------------------------------------

def test_prefetch_gives_the_same_bits_and_a_mismatch_is_harmless():
    V, d, n, k, steps = 3000, 300, 4099, 5, 6
    rng = np.random.default_rng(77)
    counts = zipf_counts(V)
    cdf = workloads.zipf_cdf(V, 1.0)
    ins = [dev(workloads.zipf_draw(cdf, n, rng)) for _ in range(steps + 1)]
    outs = [dev(workloads.zipf_draw(cdf, n, rng)) for _ in range(steps + 1)]
    seeds = [w2v.minibatch_seed(3, h) for h in range(steps + 1)]
    plain, ahead, mixed = (make_shard(V, d, 5, counts) for _ in range(3))
    la, lb = (torch.zeros(1, dtype=torch.float64, device="cuda") for _ in range(2))
    for h in range(steps):
        w2v.train_minibatch([plain], ins[h], outs[h], k, seeds[h], 0.05, loss=la)
        ahead.prefetch_minibatch(ins[h + 1], outs[h + 1], k, seeds[h + 1])      # next one, before this one
        w2v.train_minibatch([ahead], ins[h], outs[h], k, seeds[h], 0.05, loss=lb)
        assert la.item() == lb.item()
        # announcements that do not match what is trained next: other seed, other arrays, other k
        mixed.prefetch_minibatch(ins[h], outs[h], k, seeds[h] + 1)
        mixed.prefetch_minibatch(outs[h], ins[h], k, seeds[h])
        w2v.train_minibatch([mixed], ins[h], outs[h], k, seeds[h], 0.05)
        mixed.prefetch_minibatch(ins[h], outs[h], k + 1, seeds[h])
    for which in (0, 1):
        ref = all_rows(plain, which)
        assert np.array_equal(all_rows(ahead, which), ref)
        assert np.array_equal(all_rows(mixed, which), ref)
    # and the oracle agrees
    U, W = oracle_state(V, d, 5)
    th, al = oracle.build_alias(counts)
    for h in range(steps):
        oracle.train_minibatch([U], [W], w2v.index_to_numpy(ins[h]), w2v.index_to_numpy(outs[h]), k,
                               seeds[h], th, al, 0.05)
    assert vec_error(all_rows(ahead, 0), U) <= 6 * TOL1 and vec_error(all_rows(ahead, 1), W) <= 6 * TOL1
    for sh in (plain, ahead, mixed):
        sh.status()
        sh.destroy()


@pytest.mark.parametrize("V,d,k,d_total,col", [(3000, 60, 5, 300, 120), (2500, 300, 5, 300, 0),
                                               (1500, 100, 10, 100, 0), (40, 64, 5, 64, 0),
                                               (5000, 1000, 2, 1000, 0)])
def test_announced_dotprod_and_adjust_give_the_same_bits(V, d, k, d_total, col):
    # a column shard serving the two calls, with each minibatch announced one step ahead: dots and
    # vectors must equal, bit for bit, those of a shard that was told nothing -- and match the oracle
    say("announced two-call form", V, d, k)
    n, steps = 4099, 4
    rng = np.random.default_rng(V + k)
    counts = zipf_counts(V)
    cdf = workloads.zipf_cdf(V, 1.0)
    ins = [dev(workloads.zipf_draw(cdf, n, rng)) for _ in range(steps + 1)]
    outs = [dev(workloads.zipf_draw(cdf, n, rng)) for _ in range(steps + 1)]
    seeds = [w2v.minibatch_seed(9, h) for h in range(steps + 1)]
    gs = [torch.from_numpy(workloads.uniform_coeffs(n, k + 1, 100 + h)).cuda() for h in range(steps)]
    plain = make_shard(V, d, 5, counts, d_total=d_total, col_begin=col)
    ahead = make_shard(V, d, 5, counts, d_total=d_total, col_begin=col)
    U, W = oracle_state(V, d, 5, d_total=d_total, col_begin=col)
    th, al = oracle.build_alias(counts)
    ahead.prefetch_minibatch(ins[0], outs[0], k, seeds[0])
    for h in range(steps):
        ahead.prefetch_minibatch(ins[h + 1], outs[h + 1], k, seeds[h + 1])
        da = ahead.dotprod(ins[h], outs[h], k, seeds[h]).cpu().numpy()
        dp = plain.dotprod(ins[h], outs[h], k, seeds[h]).cpu().numpy()
        assert np.array_equal(da, dp)
        ahead.adjust(ins[h], outs[h], k, seeds[h], gs[h], 0.05)
        plain.adjust(ins[h], outs[h], k, seeds[h], gs[h], 0.05)
        oracle.adjust(U, W, w2v.index_to_numpy(ins[h]), w2v.index_to_numpy(outs[h]), k, seeds[h], th,
                      al, gs[h].cpu().numpy(), 0.05)
    for which, ref in ((0, U), (1, W)):
        assert np.array_equal(all_rows(ahead, which), all_rows(plain, which))
        assert vec_error(all_rows(ahead, which), ref) <= steps * TOL1
    # an adjust without the dotprod before it, and a second adjust of the same minibatch (the set
    # is spent: it recomputes), are the same updates as on the shard that was told nothing
    ahead.adjust(ins[steps], outs[steps], k, seeds[steps], gs[0], 0.05)
    ahead.adjust(ins[steps], outs[steps], k, seeds[steps], gs[0], 0.05)
    plain.adjust(ins[steps], outs[steps], k, seeds[steps], gs[0], 0.05)
    plain.adjust(ins[steps], outs[steps], k, seeds[steps], gs[0], 0.05)
    for which in (0, 1):
        assert np.array_equal(all_rows(ahead, which), all_rows(plain, which))
    for sh in (plain, ahead):
        sh.status()
        sh.destroy()


def test_announced_step_over_column_shards_gives_the_same_bits():
    rng = np.random.default_rng(58)
    V, n, k, steps = 1200, 3000, 5, 3
    counts = zipf_counts(V)
    cuts = [(0, 60), (60, 100), (160, 140)]
    told = [make_shard(V, w, 3, counts, d_total=300, col_begin=b) for b, w in cuts]
    plain = [make_shard(V, w, 3, counts, d_total=300, col_begin=b) for b, w in cuts]
    ins = [dev(rng.integers(0, V, n)) for _ in range(steps + 1)]
    outs = [dev(rng.integers(0, V, n)) for _ in range(steps + 1)]
    la, lb = (torch.zeros(1, dtype=torch.float64, device="cuda") for _ in range(2))
    for h in range(steps):
        told[0].prefetch_minibatch(ins[h + 1], outs[h + 1], k, 40 + h + 1)
        if h == 0:
            told[0].prefetch_minibatch(ins[0], outs[0], k, 40)
        w2v.train_minibatch(told, ins[h], outs[h], k, 40 + h, 0.05, loss=la)
        w2v.train_minibatch(plain, ins[h], outs[h], k, 40 + h, 0.05, loss=lb)
        assert la.item() == lb.item()
    for a, b in zip(told, plain):
        for which in (0, 1):
            assert np.array_equal(all_rows(a, which), all_rows(b, which))
    for s in told + plain:
        s.status()
        s.destroy()


def test_cancelled_and_stale_announcements_are_not_used():
    """An announcement is matched by the addresses of its arrays.  After w2v_prefetch_cancel, or
    once three update calls have gone by without using it, new contents at the same addresses must be
    trained as what they are."""
    V, d, n, k = 900, 60, 2000, 5
    rng = np.random.default_rng(41)
    counts = zipf_counts(V)
    a, b = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    a2, b2 = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    x, y = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    for mode in ("cancel", "stale"):
        told, plain = make_shard(V, d, 2, counts), make_shard(V, d, 2, counts)
        buf_in, buf_out = a.clone(), b.clone()
        told.prefetch_minibatch(buf_in, buf_out, k, 11)
        if mode == "cancel":
            told.prefetch_cancel()
        else:                                   # three other updates go by: the announcement is void
            torch.cuda.synchronize()
            for sh in (told, plain):
                w2v.train_minibatch([sh], x, y, k, 7, 0.05)
                w2v.train_minibatch([sh], y, x, k, 8, 0.05)
                w2v.train_minibatch([sh], x, x, k, 9, 0.05)
        torch.cuda.synchronize()
        buf_in.copy_(a2); buf_out.copy_(b2)     # same addresses, same n, k, seed -- other words
        w2v.train_minibatch([told], buf_in, buf_out, k, 11, 0.05)
        w2v.train_minibatch([plain], a2, b2, k, 11, 0.05)
        for which in (0, 1):
            assert np.array_equal(all_rows(told, which), all_rows(plain, which)), mode
        for sh in (told, plain):
            sh.status()
            sh.destroy()


def test_status_sees_a_bad_index_in_an_announcement_at_once():
    sh = make_shard(100, 60, 1, np.ones(100, np.uint64))
    good = dev(np.arange(50, dtype=np.uint32))
    bad = dev(np.full(50, 100, np.uint32))
    sh.prefetch_minibatch(bad, good, 5, 1)
    with pytest.raises(w2v.W2VError) as e:
        sh.status()                             # no training call in between
    assert e.value.code == -6
    sh.prefetch_cancel()
    sh.status()
    sh.destroy()


def test_new_counts_void_an_announced_minibatch():
    # the announced negatives came from the old noise table: after w2v_shard_set_counts the step
    # must draw them again
    V, d, n, k = 900, 60, 2000, 5
    rng = np.random.default_rng(4)
    a, b = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    old, new = zipf_counts(V), zipf_counts(V)[::-1].copy()
    told = make_shard(V, d, 2, old)
    plain = make_shard(V, d, 2, new)
    told.prefetch_minibatch(a, b, k, 11)
    told.set_counts(new)
    w2v.train_minibatch([told], a, b, k, 11, 0.05)
    w2v.train_minibatch([plain], a, b, k, 11, 0.05)
    for which in (0, 1):
        assert np.array_equal(all_rows(told, which), all_rows(plain, which))
    for sh in (told, plain):
        sh.status()
        sh.destroy()


def test_pair_formation_on_its_own_stream_beside_training():
    # blocks of text are turned into pairs on a second stream while the training calls on the
    # pairs of the block before are still queued on the first: same pairs, same vectors as one
    # stream doing one thing after the other
    V, d, k, B, blocks, n_tok = 2000, 300, 5, 5, 4, 60_000
    rng = np.random.default_rng(12)
    cdf = workloads.zipf_cdf(V, 1.0)
    counts = zipf_counts(V)
    texts = [workloads.zipf_draw(cdf, n_tok, rng) for _ in range(blocks)]
    off = torch.from_numpy(np.arange(0, n_tok + 1, 20, dtype=np.int64)).cuda()
    side = torch.cuda.Stream()
    results = []
    for overlapped in (False, True):
        sh = make_shard(V, d, 6, counts, t=1e-3)
        bufs = [(torch.empty(n_tok * 2 * B, dtype=torch.int32, device="cuda"),
                 torch.empty(n_tok * 2 * B, dtype=torch.int32, device="cuda")) for _ in range(blocks)]
        formed = []
        for j in range(blocks):
            gi, go = bufs[j]
            if overlapped:
                with torch.cuda.stream(side):
                    cnt = sh.make_pairs(dev(texts[j]), off, j * n_tok, 0, 77, B, gi, go)
            else:
                cnt = sh.make_pairs(dev(texts[j]), off, j * n_tok, 0, 77, B, gi, go)
            formed.append(cnt)
            for h, lo in enumerate(range(0, cnt - 4095, 4096)):          # whole minibatches
                w2v.train_minibatch([sh], gi[lo:lo + 4096], go[lo:lo + 4096], k,
                                    w2v.minibatch_seed(j, h), 0.002)
        torch.cuda.synchronize()
        results.append((formed, [w2v.index_to_numpy(a[:c]).copy() for (a, _), c in zip(bufs, formed)],
                        all_rows(sh, 0), all_rows(sh, 1)))
        sh.status()
        sh.destroy()
    assert results[0][0] == results[1][0] and min(results[0][0]) > 4096
    for a, b in zip(results[0][1], results[1][1]):
        assert np.array_equal(a, b)
    assert np.isfinite(results[0][2]).all() and np.isfinite(results[0][3]).all()
    assert np.array_equal(results[0][2], results[1][2]) and np.array_equal(results[0][3], results[1][3])


@pytest.mark.parametrize("V,d,n,k", [(50, 60, 1, 0), (50, 60, 700, 0), (3, 300, 1, 5), (2000, 100, 4097, 64)])
def test_announced_edge_shapes_give_the_same_bits(V, d, n, k):
    rng = np.random.default_rng(n + k)
    counts = zipf_counts(V)
    a, b = dev(rng.integers(0, V, n)), dev(rng.integers(0, V, n))
    told, plain = make_shard(V, d, 2, counts), make_shard(V, d, 2, counts)
    la, lb = (torch.zeros(1, dtype=torch.float64, device="cuda") for _ in range(2))
    told.prefetch_minibatch(a[:0], b[:0], k, 1)                # an empty announcement is a no-op
    for h in range(3):
        told.prefetch_minibatch(a, b, k, 10 + h)
        w2v.train_minibatch([told], a, b, k, 10 + h, 0.01, loss=la)
        w2v.train_minibatch([plain], a, b, k, 10 + h, 0.01, loss=lb)
        assert la.item() == lb.item()
    for which in (0, 1):
        assert np.array_equal(all_rows(told, which), all_rows(plain, which))
    for sh in (told, plain):
        sh.status()
        sh.destroy()


@pytest.mark.parametrize("form", ["fused", "two calls"])
def test_announcing_two_minibatches_ahead_gives_the_same_bits(form):
    """prefetch(h+2); train(h); prefetch(h+3); train(h+1); ...: three announcements are alive at a
    time, each in buffers of its own, and each serves the step it was made for.  A fourth
    announcement in a row replaces the oldest, whose step then does its index work itself."""
    V, d, n, k, steps = 3000, 100, 6000, 5, 7
    rng = np.random.default_rng(17)
    counts = zipf_counts(V)
    cdf = workloads.zipf_cdf(V, 1.0)
    told, plain = make_shard(V, d, 3, counts), make_shard(V, d, 3, counts)
    batches = [(dev(workloads.zipf_draw(cdf, n, rng)), dev(workloads.zipf_draw(cdf, n, rng)))
               for _ in range(steps + 3)]
    coeffs_ = torch.tensor(rng.uniform(-1, 1, n * (k + 1)).astype(np.float32), device="cuda")
    la, lb = (torch.zeros(1, dtype=torch.float64, device="cuda") for _ in range(2))

    def step(sh, h, loss):
        a, b = batches[h]
        if form == "fused":
            w2v.train_minibatch([sh], a, b, k, 100 + h, 0.02, loss=loss)
        else:
            sh.dotprod(a, b, k, 100 + h)
            sh.adjust(a, b, k, 100 + h, coeffs_, 0.02)

    told.prefetch_minibatch(*batches[0], k, 100)
    told.prefetch_minibatch(*batches[1], k, 101)
    for h in range(steps):
        told.prefetch_minibatch(*batches[h + 2], k, 100 + h + 2)
        if h == 3:                    # one announcement too many: the oldest (this step's) is dropped
            told.prefetch_minibatch(*batches[h + 3], k, 100 + h + 3)
        step(told, h, la)
        step(plain, h, lb)
        torch.cuda.synchronize()
        if form == "fused":
            assert la.item() == lb.item(), h
        for which in (0, 1):
            assert np.array_equal(all_rows(told, which), all_rows(plain, which)), (h, which)
    for sh in (told, plain):
        sh.prefetch_cancel()
        sh.status()
        sh.destroy()
