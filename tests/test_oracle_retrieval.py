"""Pins of the oracle's export and top-K cosine retrieval (Section 6.1.4, Section 2, Section 7.3)
against things it does not compute itself: planar vectors whose angles are known, scaled basis
vectors, an independent library's cosine matrix, and invariances of the cosine.
"""
import numpy as np
from sklearn.metrics.pairwise import cosine_similarity

import oracle


def test_topk_planar_vectors_rank_by_angle():
    # candidate i sits at angle a_i with radius r_i; the query at angle phi: cosine = cos(a_i - phi)
    rng = np.random.default_rng(501)
    N, K = 200, 17
    ang = rng.random(N) * 2 * np.pi
    rad = rng.random(N) * 5 + 0.1
    C = np.stack([rad * np.cos(ang), rad * np.sin(ang)], axis=1).astype(np.float32)
    phis = np.array([0.3, 2.0, 4.4, 6.0])
    Qm = np.stack([3 * np.cos(phis), 3 * np.sin(phis)], axis=1).astype(np.float32)
    idx, score, count = oracle.topk_cosine(Qm, C, K)
    for q, phi in enumerate(phis):
        want = np.cos(ang - phi)
        order = np.argsort(-want, kind="stable")[:K]
        assert np.array_equal(idx[q], order)
        assert np.allclose(score[q], want[order], rtol=0, atol=1e-6)   # float32 coordinates
        assert count[q] == K
    # threshold: only the candidates within the cone cos > 0.65 survive
    idx, score, count = oracle.topk_cosine(Qm, C, 150, tau=0.65)
    for q, phi in enumerate(phis):
        inside = np.sum(np.cos(ang - phi) > 0.65 + 1e-6)
        assert abs(int(count[q]) - int(inside)) <= 1
        assert np.all(score[q, :count[q]] > 0.65) and np.all(idx[q, count[q]:] == 0xFFFFFFFF)
        assert np.all(score[q, count[q]:] == 0)


def test_topk_scaled_basis_vectors_and_ties_by_index():
    d = 6
    rows, axis, sign = [], [], []
    for i, (a, s) in enumerate([(0, 2.0), (1, 1.0), (0, 0.5), (2, -3.0), (0, -1.0), (1, 7.0), (3, 0.0)]):
        v = np.zeros(d, np.float32)
        v[a] = s
        rows.append(v); axis.append(a); sign.append(np.sign(s))
    C = np.array(rows)
    Qm = np.zeros((2, d), np.float32)
    Qm[0, 0] = 4.0          # along axis 0
    Qm[1, 1] = -1.0         # against axis 1
    idx, score, count = oracle.topk_cosine(Qm, C, 7)
    # query 0: +1 for candidates 0 and 2 (index order), 0 for 1, 3, 5, 6 (6 is the zero vector), -1 for 4
    assert idx[0].tolist() == [0, 2, 1, 3, 5, 6, 4]
    assert score[0].tolist() == [1, 1, 0, 0, 0, 0, -1]
    assert idx[1].tolist() == [0, 2, 3, 4, 6, 1, 5]
    assert score[1].tolist() == [0, 0, 0, 0, 0, -1, -1]
    # K larger than N: everything, then padding
    idx, score, count = oracle.topk_cosine(Qm, C, 10)
    assert count.tolist() == [7, 7] and np.all(idx[:, 7:] == 0xFFFFFFFF)
    # strict threshold: similarities equal to tau are dropped
    idx, score, count = oracle.topk_cosine(Qm, C, 7, tau=0.0)
    assert count.tolist() == [2, 0] and idx[0, :2].tolist() == [0, 2]


def test_topk_against_an_independent_cosine_matrix_and_invariances():
    rng = np.random.default_rng(502)
    Q, N, d, K = 9, 500, 37, 30
    Qm = (rng.random((Q, d)) - 0.5).astype(np.float32)
    C = (rng.random((N, d)) - 0.3).astype(np.float32)
    idx, score, count = oracle.topk_cosine(Qm, C, K)
    S = cosine_similarity(Qm.astype(np.float64), C.astype(np.float64))
    for q in range(Q):
        order = np.argsort(-S[q], kind="stable")[:K]
        assert np.array_equal(idx[q], order)
        assert np.allclose(score[q], S[q, order], rtol=0, atol=1e-12)
    # positive rescaling of any vector changes nothing (power-of-two factors: exact in float32)
    fc = (2.0 ** rng.integers(-3, 4, N)).astype(np.float32)
    fq = (2.0 ** rng.integers(-3, 4, Q)).astype(np.float32)
    idx2, score2, _ = oracle.topk_cosine(Qm * fq[:, None], C * fc[:, None], K)
    assert np.array_equal(idx2, idx) and np.allclose(score2, score, rtol=0, atol=1e-12)
    # a permutation of the candidates permutes the answer
    perm = rng.permutation(N)
    idx3, score3, _ = oracle.topk_cosine(Qm, C[perm], K)
    assert np.array_equal(perm[idx3], idx) and np.allclose(score3, score, rtol=0, atol=1e-12)
    # a vector is its own nearest neighbour with similarity one
    idx4, score4, _ = oracle.topk_cosine(C[:20], C, 1)
    assert np.array_equal(idx4[:, 0], np.arange(20)) and np.allclose(score4, 1.0, rtol=0, atol=1e-12)


def test_export_joins_the_column_slices():
    rng = np.random.default_rng(503)
    V, widths = 50, [7, 1, 12, 4]
    full = rng.random((V, sum(widths))).astype(np.float32)
    begins = np.concatenate([[0], np.cumsum(widths)[:-1]])
    Ms = [np.ascontiguousarray(full[:, b:b + w]) for b, w in zip(begins, widths)]
    rows = rng.integers(0, V, 23)
    got = oracle.export_rows(Ms, begins, sum(widths), rows)
    assert np.array_equal(got, full[rows])
    # the initial vectors of column shards join into the unsliced initial vectors
    whole = oracle.init_rows(5, 24, 0, 24, 0, np.arange(V, dtype=np.uint32))
    parts = [oracle.init_rows(5, 24, b, w, 0, np.arange(V, dtype=np.uint32)) for b, w in zip(begins, widths)]
    assert np.array_equal(oracle.export_rows(parts, begins, 24, np.arange(V)), whole)
