"""Pins of the oracle's continuous-bag-of-words functions (Section 5.1, footnote) against things
they do not compute themselves: a dense-matrix formulation written here, finite differences of the
objective, the reduction to the (separately pinned) skip-gram functions when every example has one
context word, the column-slice invariant, the start-of-call rule, and a hand-written walk for the
example generator.
"""
import math

import numpy as np

import oracle


def rand_model(rng, V, d, scale=0.5):
    U = (rng.random((V, d)) * 2 - 1).astype(np.float32) * np.float32(scale)
    W = (rng.random((V, d)) * 2 - 1).astype(np.float32) * np.float32(scale)
    return U, W


def rand_examples(rng, V, n, max_ctx, allow_empty=False):
    lens = rng.integers(0 if allow_empty else 1, max_ctx + 1, n)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    ctx = rng.integers(0, V, int(off[-1])).astype(np.uint32)
    return off, ctx


def averaging_matrix(off, ctx, V):
    """A[p][w] = (occurrences of w among the contexts of p) / |C_p|."""
    n = off.size - 1
    A = np.zeros((n, V))
    for p in range(n):
        for w in ctx[off[p]:off[p + 1]]:
            A[p, w] += 1.0 / (off[p + 1] - off[p])
    return A


def objective(U, W, A, rows):
    """Eq.1 with the hidden vector in place of the input vector, in double."""
    H = A @ U
    total = 0.0
    for p in range(rows.shape[0]):
        for j in range(rows.shape[1]):
            f = float(H[p] @ W[rows[p, j]])
            total += math.log(1.0 / (1.0 + math.exp(-f if j == 0 else f)))
    return total


def test_cbow_dots_and_adjust_against_a_dense_matrix_formulation():
    rng = np.random.default_rng(401)
    V, d, n, T = 23, 7, 40, 4
    U, W = rand_model(rng, V, d)
    off, ctx = rand_examples(rng, V, n, 6, allow_empty=True)
    assert np.any(np.diff(off.astype(np.int64)) == 0)            # the empty-context case is in
    rows = rng.integers(0, V, (n, T)).astype(np.uint32)
    A = averaging_matrix(off, ctx, V)
    H = A @ U.astype(np.float64)
    want = np.einsum("pc,pjc->pj", H, W.astype(np.float64)[rows])
    got = oracle.cbow_dots(U, W, off, ctx, rows)
    assert np.allclose(got, want, rtol=0, atol=1e-7)
    g = (rng.random((n, T)) * 2 - 1).astype(np.float32)
    alpha = np.float32(0.05)
    E = np.einsum("pj,pjc->pc", g.astype(np.float64), W.astype(np.float64)[rows])
    dU = A.T @ E
    dW = np.zeros((V, d))
    np.add.at(dW, rows.reshape(-1), (g.astype(np.float64)[:, :, None] * H[:, None, :]).reshape(-1, d))
    U1, W1 = U.copy(), W.copy()
    oracle.cbow_adjust_rows(U1, W1, off, ctx, rows, g, alpha)
    assert np.allclose(U1, U + float(alpha) * dU, rtol=0, atol=2e-7)
    assert np.allclose(W1, W + float(alpha) * dW, rtol=0, atol=2e-7)
    assert not np.allclose(U1, U) and not np.allclose(W1, W)
    # the word with no occurrence as a context keeps its input vector bit for bit
    untouched = np.setdiff1d(np.arange(V), ctx)
    assert np.array_equal(U1[untouched], U[untouched])


def test_cbow_update_is_the_gradient_of_the_objective():
    rng = np.random.default_rng(402)
    V, d, n, k = 12, 5, 9, 3
    U, W = rand_model(rng, V, d, 0.8)
    lens = rng.integers(1, 6, n)
    lens[2] = 3
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    ctx = rng.integers(0, V, int(off[-1])).astype(np.uint32)
    ctx[off[2]:off[2] + 2] = 4                                  # a word twice in one context list
    rows = rng.integers(0, V, (n, k + 1)).astype(np.uint32)
    A = averaging_matrix(off, ctx, V)
    dots = oracle.cbow_dots(U, W, off, ctx, rows)
    g = oracle.coeffs([dots])
    alpha = 1.0
    U1, W1 = U.copy(), W.copy()
    oracle.cbow_adjust_rows(U1, W1, off, ctx, rows, g, alpha)
    Ud, Wd = U.astype(np.float64), W.astype(np.float64)
    h = 1e-5
    for M, M1, name in ((Ud, U1, "U"), (Wd, W1, "W")):
        grad = np.zeros_like(M)
        for w in range(V):
            for c in range(d):
                old = M[w, c]
                M[w, c] = old + h
                up = objective(Ud, Wd, A, rows)
                M[w, c] = old - h
                dn = objective(Ud, Wd, A, rows)
                M[w, c] = old
                grad[w, c] = (up - dn) / (2 * h)
        step = M1.astype(np.float64) - M
        assert np.abs(step - grad).max() <= 5e-6, name
        assert np.abs(grad).max() > 1e-2


def test_cbow_with_one_context_word_per_example_is_skip_gram():
    # h = u_c, so dots, coefficients and both updates are those of the pair (in = c, out = center).
    rng = np.random.default_rng(403)
    V, d, n, k = 50, 12, 300, 4
    U, W = rand_model(rng, V, d)
    th, al = oracle.build_alias(rng.integers(1, 100, V).astype(np.uint64))
    ctx = rng.integers(0, V, n).astype(np.uint32)
    off = np.arange(n + 1, dtype=np.uint32)
    out = rng.integers(0, V, n).astype(np.uint32)
    a = oracle.cbow_dotprod(U, W, off, ctx, out, k, 77, th, al)
    b = oracle.dotprod(U, W, ctx, out, k, 77, th, al)
    assert np.array_equal(a, b)
    Ua, Wa, Ub, Wb = U.copy(), W.copy(), U.copy(), W.copy()
    la = oracle.cbow_train_minibatch([Ua], [Wa], off, ctx, out, k, 77, th, al, 0.05)
    lb = oracle.train_minibatch([Ub], [Wb], ctx, out, k, 77, th, al, 0.05)
    assert la == lb
    assert np.allclose(Ua, Ub, rtol=0, atol=1e-7) and np.allclose(Wa, Wb, rtol=0, atol=1e-7)
    assert not np.array_equal(Ua, U)


def test_cbow_column_slices_add_up_and_concatenate():
    rng = np.random.default_rng(404)
    V, d, n, k, S = 40, 30, 120, 5, 5
    U, W = rand_model(rng, V, d)
    th, al = oracle.build_alias(rng.integers(1, 100, V).astype(np.uint64))
    off, ctx = rand_examples(rng, V, n, 8)
    out = rng.integers(0, V, n).astype(np.uint32)
    ds = d // S
    Us = [np.ascontiguousarray(U[:, s * ds:(s + 1) * ds]) for s in range(S)]
    Ws = [np.ascontiguousarray(W[:, s * ds:(s + 1) * ds]) for s in range(S)]
    full = oracle.cbow_dotprod(U, W, off, ctx, out, k, 5, th, al)
    parts = [oracle.cbow_dotprod(Us[s], Ws[s], off, ctx, out, k, 5, th, al) for s in range(S)]
    assert np.allclose(np.sum(np.array(parts, np.float64), axis=0), full, rtol=0, atol=2e-7)
    U1, W1 = U.copy(), W.copy()
    l1 = oracle.cbow_train_minibatch([U1], [W1], off, ctx, out, k, 5, th, al, 0.05)
    lS = oracle.cbow_train_minibatch(Us, Ws, off, ctx, out, k, 5, th, al, 0.05)
    assert abs(l1 - lS) <= 1e-5 * abs(l1)
    assert np.allclose(np.concatenate(Us, axis=1), U1, rtol=0, atol=2e-7)
    assert np.allclose(np.concatenate(Ws, axis=1), W1, rtol=0, atol=2e-7)


def test_cbow_adjust_reads_start_of_call_vectors():
    # The same example twice changes every row by exactly twice the single-example change; two
    # calls in a row (which see the first call's result) do not.
    rng = np.random.default_rng(405)
    V, d = 10, 6
    U, W = rand_model(rng, V, d)
    off1, ctx1 = np.array([0, 3], np.uint32), np.array([1, 2, 1], np.uint32)
    rows1 = np.array([[5, 6, 2]], np.uint32)
    g1 = np.array([[0.4, -0.3, -0.2]], np.float32)
    Ua, Wa = U.copy(), W.copy()
    oracle.cbow_adjust_rows(Ua, Wa, off1, ctx1, rows1, g1, 0.5)
    off2, ctx2 = np.array([0, 3, 6], np.uint32), np.tile(ctx1, 2)
    Ub, Wb = U.copy(), W.copy()
    oracle.cbow_adjust_rows(Ub, Wb, off2, ctx2, np.tile(rows1, (2, 1)), np.tile(g1, (2, 1)), 0.5)
    assert np.allclose(Ub - U, 2 * (Ua - U), rtol=0, atol=1e-7)
    assert np.allclose(Wb - W, 2 * (Wa - W), rtol=0, atol=1e-7)
    Uc, Wc = Ua.copy(), Wa.copy()
    oracle.cbow_adjust_rows(Uc, Wc, off1, ctx1, rows1, g1, 0.5)
    assert np.abs((Uc - U) - 2 * (Ua - U)).max() > 1e-4
    # row 2 is both a context word and a negative: its input and output vectors both move, each
    # from the other matrix's start-of-call values
    assert not np.array_equal(Ua[2], U[2]) and not np.array_equal(Wa[2], W[2])
    h = (2 * U[1].astype(np.float64) + U[2]) / 3
    assert np.allclose(Wa[2], W[2] + 0.5 * np.float64(g1[0, 2]) * h, rtol=0, atol=1e-7)
    e = (g1[0].astype(np.float64)[:, None] * W[rows1[0]].astype(np.float64)).sum(axis=0)
    assert np.allclose(Ua[1], U[1] + 0.5 * 2 * e / 3, rtol=0, atol=1e-7)
    assert np.allclose(Ua[2], U[2] + 0.5 * e / 3, rtol=0, atol=1e-7)


def test_cbow_null_updates():
    rng = np.random.default_rng(406)
    V, d, n, T = 15, 4, 20, 3
    U, W = rand_model(rng, V, d)
    off, ctx = rand_examples(rng, V, n, 4)
    rows = rng.integers(0, V, (n, T)).astype(np.uint32)
    g = (rng.random((n, T)) - 0.5).astype(np.float32)
    U1, W1 = U.copy(), W.copy()
    oracle.cbow_adjust_rows(U1, W1, off, ctx, rows, g, 0.0)
    assert np.array_equal(U1, U) and np.array_equal(W1, W)
    oracle.cbow_adjust_rows(U1, W1, off, ctx, rows, np.zeros_like(g), 0.3)
    assert np.array_equal(U1, U) and np.array_equal(W1, W)


# --- examples from text ----------------------------------------------------------------------------

def examples_by_hand(tokens, off, base, epoch, seed, B, kt):
    keep, b = oracle.token_draws(tokens, base, epoch, seed, B, kt)
    centers, lists = [], []
    for s in range(off.size - 1):
        pos = [t for t in range(int(off[s]), int(off[s + 1])) if keep[t]]
        for j, t in enumerate(pos):
            near = [tokens[pos[c]] for c in range(max(0, j - int(b[t])), min(len(pos) - 1, j + int(b[t])) + 1)
                    if c != j]
            if near:
                centers.append(tokens[t])
                lists.append(near)
    return centers, lists


def test_cbow_examples_hand_case_and_walk():
    tokens = np.arange(10, dtype=np.uint32)
    off = np.array([0, 4, 5, 10], np.uint64)               # sentences of 4, 1 and 5 tokens
    co, cx, out, cnt, nctx = oracle.make_cbow_examples(tokens, off, 0, 0, 1, 1, None)
    assert out.tolist() == [0, 1, 2, 3, 5, 6, 7, 8, 9] and cnt == 9 and nctx == 14
    assert [cx[co[p]:co[p + 1]].tolist() for p in range(9)] == \
        [[1], [0, 2], [1, 3], [2], [6], [5, 7], [6, 8], [7, 9], [8]]
    rng = np.random.default_rng(407)
    V = 30
    counts = rng.integers(1, 2000, V).astype(np.uint64)
    kt = oracle.build_keep(counts, 0.01)
    tokens = rng.integers(0, V, 700).astype(np.uint32)
    lens = rng.integers(1, 25, 70)
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.append(off[off < 700], 700).astype(np.uint64)
    for B in (1, 3, 8):
        co, cx, out, cnt, nctx = oracle.make_cbow_examples(tokens, off, 999, 1, 42, B, kt)
        centers, lists = examples_by_hand(tokens, off, 999, 1, 42, B, kt)
        assert cnt == len(centers) and out.tolist() == [int(c) for c in centers]
        assert [cx[co[p]:co[p + 1]].tolist() for p in range(cnt)] == [[int(x) for x in l] for l in lists]
        # the same (center, context) pairs as the skip-gram walk, grouped by center
        a, b, pc = oracle.make_pairs(tokens, off, 999, 1, 42, B, kt)
        assert pc == nctx and np.array_equal(b, cx)
        assert np.array_equal(a, np.repeat(out, np.diff(co.astype(np.int64))))
        # truncated outputs are prefixes, full counts still reported
        co2, cx2, out2, cnt2, nctx2 = oracle.make_cbow_examples(tokens, off, 999, 1, 42, B, kt,
                                                                 cap_examples=11, cap_ctx=17)
        assert (cnt2, nctx2) == (cnt, nctx) and np.array_equal(out2, out[:11])
        assert np.array_equal(co2, co[:12]) and np.array_equal(cx2, cx[:17])
