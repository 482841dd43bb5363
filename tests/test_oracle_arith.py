"""Pins of the oracle's arithmetic (dots, coefficients, adjust) against things the oracle does not
compute itself: brute-force loops written here, closed forms, finite differences of the objective
(Eq.1/Eq.3), the column-slice invariant (Section 5.1) and the start-of-call rule of adjust.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def sigma(x):
    return 1.0 / (1.0 + math.exp(-x))


def rand_model(rng, V, d, scale=0.5):
    U = (rng.random((V, d)) * 2 - 1).astype(np.float32) * np.float32(scale)
    W = (rng.random((V, d)) * 2 - 1).astype(np.float32) * np.float32(scale)
    return U, W


def flat_table(V):
    """Alias table of a uniform noise distribution (every bin keeps itself)."""
    return oracle.build_alias(np.ones(V, np.uint64))


# --- Philox ---------------------------------------------------------------------------------

def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = oracle.philox(v[0:4], v[4:6])
        assert [int(x) for x in got] == v[6:10]


def test_minibatch_seed_is_a_function_of_master_and_index():
    a = [oracle.minibatch_seed(7, h) for h in range(200)]
    assert len(set(a)) == 200
    assert a == [oracle.minibatch_seed(7, h) for h in range(200)]
    assert oracle.minibatch_seed(8, 0) != a[0]
    # it is the first two output words of the generator at counter (h, 0, 0, 5)
    q = oracle.philox([3, 0, 0, 5], [7, 0])
    assert a[3] == (int(q[1]) << 32) | int(q[0])


# --- T1 brute force ----------------------------------------------------------------------------

def brute_force_step(U, W, in_idx, rows, alpha):
    """Independent double-precision loops: dots, coefficients, start-of-call update."""
    U0 = U.astype(np.float64)
    W0 = W.astype(np.float64)
    n, T = rows.shape
    d = U.shape[1]
    f = np.zeros((n, T))
    for p in range(n):
        for j in range(T):
            s = 0.0
            for c in range(d):
                s += U0[in_idx[p], c] * W0[rows[p, j], c]
            f[p, j] = s
    f32 = f.astype(np.float32).astype(np.float64)     # the client sees float32 partial dots
    g = np.zeros((n, T))
    for p in range(n):
        for j in range(T):
            label = 1.0 if j == 0 else 0.0
            g[p, j] = label - sigma(f32[p, j])
    g32 = g.astype(np.float32).astype(np.float64)
    dU = np.zeros_like(U0)
    dW = np.zeros_like(W0)
    for p in range(n):
        for j in range(T):
            for c in range(d):
                dU[in_idx[p], c] += g32[p, j] * W0[rows[p, j], c]
                dW[rows[p, j], c] += g32[p, j] * U0[in_idx[p], c]
    a = float(np.float32(alpha))
    return f, g, (U0 + a * dU), (W0 + a * dW)


def test_T1_brute_force_tiny():
    rng = np.random.default_rng(11)
    V, d, n, k = 8, 4, 3, 2
    U, W = rand_model(rng, V, d)
    in_idx = np.array([1, 5, 1], np.uint32)                      # a repeated input row
    rows = np.array([[2, 3, 7], [2, 6, 6], [4, 2, 0]], np.uint32)  # repeated output rows too
    f, g, U1, W1 = brute_force_step(U, W, in_idx, rows, 0.25)

    dots = oracle.dots(U, W, in_idx, rows)
    np.testing.assert_allclose(dots, f, rtol=0, atol=1e-7)
    co = oracle.coeffs([dots])
    np.testing.assert_allclose(co, g, rtol=0, atol=1e-7)
    Uo, Wo = U.copy(), W.copy()
    oracle.adjust_rows(Uo, Wo, in_idx, rows, co, 0.25)
    np.testing.assert_allclose(Uo, U1, rtol=0, atol=1e-7)
    np.testing.assert_allclose(Wo, W1, rtol=0, atol=1e-7)
    # untouched rows are bitwise unchanged
    touched_u = set(in_idx.tolist())
    touched_w = set(rows.ravel().tolist())
    for r in range(V):
        if r not in touched_u:
            assert np.array_equal(Uo[r], U[r])
        if r not in touched_w:
            assert np.array_equal(Wo[r], W[r])


def test_T1b_brute_force_random_shapes():
    rng = np.random.default_rng(12)
    for V, d, n, k in [(5, 3, 7, 1), (9, 5, 6, 3), (4, 1, 9, 0)]:
        U, W = rand_model(rng, V, d)
        in_idx = rng.integers(0, V, n).astype(np.uint32)
        rows = rng.integers(0, V, (n, k + 1)).astype(np.uint32)
        f, g, U1, W1 = brute_force_step(U, W, in_idx, rows, 0.1)
        dots = oracle.dots(U, W, in_idx, rows)
        co = oracle.coeffs([dots])
        Uo, Wo = U.copy(), W.copy()
        oracle.adjust_rows(Uo, Wo, in_idx, rows, co, 0.1)
        np.testing.assert_allclose(dots, f, atol=1e-7, rtol=0)
        np.testing.assert_allclose(co, g, atol=1e-7, rtol=0)
        np.testing.assert_allclose(Uo, U1, atol=1e-7, rtol=0)
        np.testing.assert_allclose(Wo, W1, atol=1e-7, rtol=0)


# --- T2 closed form for zero output vectors ------------------------------------------------------

def test_T2_zero_output_vectors():
    rng = np.random.default_rng(2)
    V, d, n, k = 50, 8, 40, 3
    U = ((rng.random((V, d)) - 0.5) / d).astype(np.float32)
    W = np.zeros((V, d), np.float32)
    th, al = oracle.build_alias(rng.integers(1, 100, V).astype(np.uint64))
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    seed = 99
    dots = oracle.dotprod(U, W, in_idx, out_idx, k, seed, th, al)
    assert np.all(dots == 0.0)
    co, loss = oracle.coeffs([dots], want_loss=True)
    assert np.all(co[:, 0] == np.float32(0.5)) and np.all(co[:, 1:] == np.float32(-0.5))
    assert abs(loss - n * (k + 1) * math.log(2.0)) < 1e-9
    U1, W1 = U.copy(), W.copy()
    alpha = 0.025
    oracle.adjust(U1, W1, in_idx, out_idx, k, seed, th, al, co, alpha)
    assert np.array_equal(U1, U)                      # every source row is zero
    neg = oracle.negatives(out_idx, k, seed, th, al)
    expect = np.zeros((V, d))
    for p in range(n):
        expect[out_idx[p]] += 0.5 * U[in_idx[p]].astype(np.float64)
        for j in range(k):
            expect[neg[p, j]] -= 0.5 * U[in_idx[p]].astype(np.float64)
    expect *= float(np.float32(alpha))
    np.testing.assert_allclose(W1, expect, rtol=0, atol=1e-9)


# --- T3 finite differences of the minibatch objective -------------------------------------------

def objective(U, W, in_idx, rows):
    """Lambda of Eq.3 for explicit negatives, in double."""
    total = 0.0
    for p in range(rows.shape[0]):
        u = U[in_idx[p]]
        total += math.log(sigma(float(u @ W[rows[p, 0]])))
        for j in range(1, rows.shape[1]):
            total += math.log(1.0 - sigma(float(u @ W[rows[p, j]])))
    return total


def test_T3_update_is_alpha_times_gradient_of_objective():
    rng = np.random.default_rng(3)
    V, d, n, k = 20, 6, 30, 3
    U, W = rand_model(rng, V, d, scale=0.8)
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    in_idx[5] = in_idx[4]                     # repeated rows on both sides
    rows = rng.integers(0, V, (n, k + 1)).astype(np.uint32)
    rows[7, 2] = rows[7, 1]
    alpha = 0.5
    co = oracle.coeffs([oracle.dots(U, W, in_idx, rows)])
    U1, W1 = U.copy(), W.copy()
    oracle.adjust_rows(U1, W1, in_idx, rows, co, alpha)
    gU = (U1.astype(np.float64) - U) / alpha
    gW = (W1.astype(np.float64) - W) / alpha

    Ud, Wd = U.astype(np.float64), W.astype(np.float64)
    h = 1e-4
    for M, G, which in ((Ud, gU, "U"), (Wd, gW, "W")):
        for r in range(V):
            for c in range(d):
                old = M[r, c]
                M[r, c] = old + h
                up = objective(Ud, Wd, in_idx, rows)
                M[r, c] = old - h
                dn = objective(Ud, Wd, in_idx, rows)
                M[r, c] = old
                fd = (up - dn) / (2 * h)
                assert abs(fd - G[r, c]) < 2e-6, (which, r, c, fd, G[r, c])


# --- T4 column slices ----------------------------------------------------------------------------

def test_T4_slices_of_the_initial_vectors_concatenate():
    rows = np.array([0, 1, 17, 123456, 9_999_999], np.uint32)
    for matrix in (0, 1):
        full = oracle.init_rows(42, 300, 0, 300, matrix, rows)
        parts = [oracle.init_rows(42, 300, 60 * s, 60, matrix, rows) for s in range(5)]
        assert np.array_equal(np.concatenate(parts, axis=1), full)
        odd = [oracle.init_rows(42, 300, b, e - b, matrix, rows) for b, e in ((0, 7), (7, 150), (150, 300))]
        assert np.array_equal(np.concatenate(odd, axis=1), full)
    assert np.all(np.abs(full) <= 0.5 / 300)
    a = oracle.init_rows(42, 300, 0, 300, 0, rows)
    b = oracle.init_rows(42, 300, 0, 300, 1, rows)
    assert not np.array_equal(a, b)


def test_T4_initial_vectors_look_uniform():
    rows = np.arange(4000, dtype=np.uint32)
    x = oracle.init_rows(5, 100, 0, 100, 0, rows).astype(np.float64) * 100   # -> uniform(-0.5,0.5)
    assert abs(x.mean()) < 3 * (1 / math.sqrt(12)) / math.sqrt(x.size)
    assert abs(x.var() - 1 / 12) < 1e-3
    assert x.min() >= -0.5 and x.max() < 0.5
    # columns and rows are not correlated copies of each other
    assert abs(np.corrcoef(x[:, 0], x[:, 1])[0, 1]) < 0.06
    assert abs(np.corrcoef(x[0], x[1])[0, 1]) < 0.35


def test_T4_partial_dots_sum_to_the_full_dot_and_updates_concatenate():
    rng = np.random.default_rng(4)
    V, d, S, n, k = 64, 20, 5, 50, 4
    U, W = rand_model(rng, V, d)
    th, al = oracle.build_alias(rng.integers(1, 50, V).astype(np.uint64))
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    ds = d // S
    Us = [np.ascontiguousarray(U[:, s * ds:(s + 1) * ds]) for s in range(S)]
    Ws = [np.ascontiguousarray(W[:, s * ds:(s + 1) * ds]) for s in range(S)]
    full = oracle.dotprod(U, W, in_idx, out_idx, k, 5, th, al)
    parts = [oracle.dotprod(Us[s], Ws[s], in_idx, out_idx, k, 5, th, al) for s in range(S)]
    np.testing.assert_allclose(np.sum([p.astype(np.float64) for p in parts], axis=0), full,
                               rtol=0, atol=2e-7)
    U1, W1 = U.copy(), W.copy()
    l1 = oracle.train_minibatch([U1], [W1], in_idx, out_idx, k, 5, th, al, 0.05)
    l5 = oracle.train_minibatch(Us, Ws, in_idx, out_idx, k, 5, th, al, 0.05)
    assert abs(l1 - l5) < 1e-5
    np.testing.assert_allclose(np.concatenate(Us, axis=1), U1, rtol=0, atol=1e-7)
    np.testing.assert_allclose(np.concatenate(Ws, axis=1), W1, rtol=0, atol=1e-7)


# --- T8 / T9 / T13 special cases of adjust --------------------------------------------------------

def test_T8_reads_are_of_the_start_of_call_vectors():
    rng = np.random.default_rng(8)
    V, d = 6, 5
    U, W = rand_model(rng, V, d)
    a, b = 2, 4
    g = np.array([[0.3]], np.float32)
    alpha = 1.0
    # one pair
    U1, W1 = U.copy(), W.copy()
    oracle.adjust_rows(U1, W1, np.array([a], np.uint32), np.array([[b]], np.uint32), g, alpha)
    du = U1[a].astype(np.float64) - U[a]
    dw = W1[b].astype(np.float64) - W[b]
    np.testing.assert_allclose(du, 0.3 * W[b].astype(np.float64) * (np.float32(0.3) / 0.3), atol=1e-7)
    # the same pair twice in one call: exactly twice the change, both from the old vectors
    U2, W2 = U.copy(), W.copy()
    oracle.adjust_rows(U2, W2, np.array([a, a], np.uint32), np.array([[b], [b]], np.uint32),
                       np.array([[0.3], [0.3]], np.float32), alpha)
    np.testing.assert_allclose(U2[a].astype(np.float64) - U[a], 2 * du, atol=2e-7)
    np.testing.assert_allclose(W2[b].astype(np.float64) - W[b], 2 * dw, atol=2e-7)
    # applying the pair in two successive calls is different (the second call sees moved vectors)
    U3, W3 = U1.copy(), W1.copy()
    oracle.adjust_rows(U3, W3, np.array([a], np.uint32), np.array([[b]], np.uint32), g, alpha)
    assert np.max(np.abs(U3[a] - U2[a])) > 1e-3
    # and within one pair the input row's change uses the OLD output row and vice versa
    np.testing.assert_allclose(dw, float(np.float32(0.3)) * U[a].astype(np.float64), atol=1e-7)


def test_T9_null_updates_leave_the_store_bitwise_unchanged():
    rng = np.random.default_rng(9)
    V, d, n, k = 30, 7, 25, 2
    U, W = rand_model(rng, V, d)
    th, al = flat_table(V)
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    out_idx = rng.integers(0, V, n).astype(np.uint32)
    co = oracle.coeffs([oracle.dotprod(U, W, in_idx, out_idx, k, 1, th, al)])
    U1, W1 = U.copy(), W.copy()
    oracle.adjust(U1, W1, in_idx, out_idx, k, 1, th, al, co, 0.0)
    assert np.array_equal(U1, U) and np.array_equal(W1, W)
    oracle.adjust(U1, W1, in_idx, out_idx, k, 1, th, al, np.zeros_like(co), 0.3)
    assert np.array_equal(U1, U) and np.array_equal(W1, W)
    # k = 0: positive pairs only
    d0 = oracle.dotprod(U, W, in_idx, out_idx, 0, 1, th, al)
    assert d0.shape == (n, 1)
    np.testing.assert_allclose(
        d0[:, 0], np.einsum("ij,ij->i", U[in_idx].astype(np.float64), W[out_idx].astype(np.float64)),
        atol=1e-7)


def test_T13_heavy_row_closed_form():
    rng = np.random.default_rng(13)
    V, d, n = 10, 9, 5000
    U, W = rand_model(rng, V, d)
    a, b = 3, 7
    g = (rng.random((n, 1)) * 2 - 1).astype(np.float32)
    alpha = 0.01
    U1, W1 = U.copy(), W.copy()
    oracle.adjust_rows(U1, W1, np.full(n, a, np.uint32), np.full((n, 1), b, np.uint32), g, alpha)
    G = g.astype(np.float64).sum()
    a32 = float(np.float32(alpha))
    np.testing.assert_allclose(U1[a], U[a].astype(np.float64) + a32 * G * W[b], rtol=0, atol=1e-7)
    np.testing.assert_allclose(W1[b], W[b].astype(np.float64) + a32 * G * U[a], rtol=0, atol=1e-7)
    rest = [r for r in range(V) if r != a]
    assert np.array_equal(U1[rest], U[rest])


def test_coefficients_are_label_minus_sigmoid_of_the_summed_partials():
    rng = np.random.default_rng(14)
    n, T, S = 40, 4, 3
    parts = [(rng.standard_normal((n, T)) * 3).astype(np.float32) for _ in range(S)]
    co, loss = oracle.coeffs(parts, want_loss=True)
    tot = np.sum([p.astype(np.float64) for p in parts], axis=0)
    exp_loss = 0.0
    for p in range(n):
        for j in range(T):
            s = sigma(tot[p, j])
            want = (1.0 - s) if j == 0 else -s
            assert abs(float(co[p, j]) - want) <= 1e-7
            exp_loss -= math.log(s) if j == 0 else math.log(1.0 - s)
    assert abs(loss - exp_loss) < 1e-9 * max(1.0, abs(exp_loss))
    # extreme dots saturate but stay finite and keep their sign
    big = np.array([[40.0, 40.0], [-40.0, -40.0]], np.float32)
    c = oracle.coeffs([big])
    assert np.all(np.isfinite(c)) and c[0, 0] >= 0 and c[0, 1] == -1.0 and c[1, 0] == 1.0


def test_loss_stays_finite_and_exact_when_sigma_saturates():
    """-log sigma(x) = log(1 + e^-x): for x = -60 that is 60 + e^-60, for x = +60 it is
    log1p(e^-60) = e^-60 to first order (e^-60 = 8.7565107626965203e-27); a negative slot's term
    -log(1 - sigma(x)) is the same function of -x."""
    tiny = 8.7565107626965203e-27
    for x, slot, want in ((-60.0, 0, 60.0), (60.0, 0, tiny), (60.0, 1, 60.0), (-60.0, 1, tiny),
                          (-700.0, 0, 700.0), (800.0, 1, 800.0), (0.0, 0, math.log(2.0))):
        if slot == 0:                               # a pair without negatives: the loss is the term
            _, loss = oracle.coeffs([np.full((1, 1), x, np.float32)], want_loss=True)
            assert abs(loss - want) <= 1e-12 * want, (x, loss)
        else:                                       # the positive slot's zero dot adds log 2
            f = np.zeros((1, 2), np.float32)
            f[0, 1] = x
            _, loss = oracle.coeffs([f], want_loss=True)
            assert math.isfinite(loss) and abs((loss - math.log(2.0)) - want) <= 1e-12 * max(want, 1.0), (x, loss)


def test_sequential_float_mode_differs_only_by_rounding():
    rng = np.random.default_rng(15)
    V, d, n, k = 12, 6, 400, 2
    U, W = rand_model(rng, V, d)
    in_idx = rng.integers(0, V, n).astype(np.uint32)
    rows = rng.integers(0, V, (n, k + 1)).astype(np.uint32)
    g = (rng.random((n, k + 1)) * 2 - 1).astype(np.float32)
    Ua, Wa, Ub, Wb = U.copy(), W.copy(), U.copy(), W.copy()
    oracle.adjust_rows(Ua, Wa, in_idx, rows, g, 0.025)
    oracle.adjust_rows(Ub, Wb, in_idx, rows, g, 0.025, sequential_fp32=True)
    assert np.max(np.abs(Ua - Ub)) < 1e-5 and np.max(np.abs(Wa - Wb)) < 1e-5


def test_lazy_store_matches_dense_store():
    rng = np.random.default_rng(16)
    V, d, n, k = 300, 12, 200, 3
    counts = rng.integers(1, 1000, V).astype(np.uint64)
    th, al = oracle.build_alias(counts)
    allrows = np.arange(V, dtype=np.uint32)
    U = oracle.init_rows(77, 24, 12, d, 0, allrows)
    W = oracle.init_rows(77, 24, 12, d, 1, allrows)
    lazy = oracle.LazyShard(V, 24, 12, d, 77, True)
    for h in range(3):
        in_idx = rng.integers(0, V, n).astype(np.uint32)
        out_idx = rng.integers(0, V, n).astype(np.uint32)
        l1 = oracle.train_minibatch([U], [W], in_idx, out_idx, k, 1000 + h, th, al, 0.05)
        l2 = lazy.train_minibatch(in_idx, out_idx, k, 1000 + h, th, al, 0.05)
        assert abs(l1 - l2) < 1e-9
    for r in range(0, V, 7):
        assert np.array_equal(lazy.row(0, r), U[r]) and np.array_equal(lazy.row(1, r), W[r])
    lazy.close()


def test_scratch_sums_match_a_brute_force_loop_and_the_applied_update():
    """oracle.adjust_deltas hands out the adjust routine's scratch area (Appendix, adjust: the summed
    changes before they are added to the store).  Pin: an independent loop written here, and the
    update that adjust_rows applies from the same sums."""
    rng = np.random.default_rng(17)
    V, d, n, T = 23, 7, 160, 4
    U, W = rand_model(rng, V, d)
    in_idx = rng.integers(0, V - 2, n).astype(np.uint32)        # words V-2, V-1 are never inputs
    rows = rng.integers(0, V, (n, T)).astype(np.uint32)
    g = (rng.random((n, T)) * 2 - 1).astype(np.float32)
    U_before, W_before = U.copy(), W.copy()
    dU, dW = oracle.adjust_deltas(U, W, in_idx, rows, g)
    assert np.array_equal(U, U_before) and np.array_equal(W, W_before)      # read-only
    bU, bW = np.zeros((V, d)), np.zeros((V, d))
    for p in range(n):
        for j in range(T):
            bU[in_idx[p]] += float(g[p, j]) * W[rows[p, j]].astype(np.float64)
            bW[rows[p, j]] += float(g[p, j]) * U[in_idx[p]].astype(np.float64)
    np.testing.assert_allclose(dU, bU, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dW, bW, rtol=0, atol=1e-12)
    # a word the minibatch never names has a zero sum; a subset is the matching rows of the whole
    unused = np.setdiff1d(np.arange(V), in_idx)
    assert unused.size > 0 and not dU[unused].any()
    sU, sW = oracle.adjust_deltas(U, W, in_idx, rows, g, want_u=[5, 0, 5], want_w=[22])
    assert np.array_equal(sU, dU[[5, 0, 5]]) and np.array_equal(sW, dW[[22]])
    # and these are the sums that adjust_rows adds: new = fl(old + alpha * sum)
    alpha = np.float32(0.05)
    U1, W1 = U.copy(), W.copy()
    oracle.adjust_rows(U1, W1, in_idx, rows, g, alpha)
    assert np.array_equal(U1, (U.astype(np.float64) + float(alpha) * dU).astype(np.float32))
    assert np.array_equal(W1, (W.astype(np.float64) + float(alpha) * dW).astype(np.float32))
