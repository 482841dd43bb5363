"""GPU parity of vector export (bit exact) and of the top-K cosine retrieval against the CPU oracle,
through the C ABI.

Retrieval tolerance: the GPU forms each similarity in fp32 (d products accumulated in fp32, two
inverse norms), the oracle in double.  The error of an fp32 dot product is at most about d * 2^-24
times |q||c| and in practice a few times sqrt(d) * 2^-24, so similarities must agree within
TOL = 1e-5 (d <= 1000).  Where the oracle's ranking is decided by a margin wider than 2 TOL the
indices must be identical; inside such a margin any order of the tied candidates is accepted, as
long as every returned candidate's true similarity fits its rank.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_08495_amd import w2v, workloads
from util import dev

pytestmark = pytest.mark.gpu

TOL = 1e-5


def say(*a):
    print(*a, flush=True)


def check_topk(Qm, C, K, tau, gi, gs, gc):
    """gi, gs, gc: GPU index / score / count arrays (numpy)."""
    oi, os_, oc = oracle.topk_cosine(Qm, C, K, tau)
    full_i, full_s, _ = oracle.topk_cosine(Qm, C, min(C.shape[0], K + 8), -2.0)   # a little beyond rank K
    exact = 0
    for q in range(Qm.shape[0]):
        n = int(gc[q])
        # counts differ only if a similarity sits within TOL of tau
        if n != int(oc[q]):
            edge = full_s[q][(np.abs(full_s[q] - tau) <= TOL)]
            assert edge.size >= abs(n - int(oc[q])), (q, n, oc[q])
        assert np.all(gi[q, n:] == 0xFFFFFFFF) and np.all(gs[q, n:] == 0)
        assert np.all(np.diff(gs[q, :n]) <= 0)                            # ranked
        assert np.unique(gi[q, :n]).size == n                             # no candidate twice
        assert np.all(gs[q, :n] > tau)
        m = min(n, int(oc[q]))
        assert np.all(np.abs(gs[q, :m] - os_[q, :m]) <= TOL), (q, np.abs(gs[q, :m] - os_[q, :m]).max())
        # every returned candidate's true similarity (oracle arithmetic) fits its rank
        cq = C[gi[q, :n]].astype(np.float64)
        qv = Qm[q].astype(np.float64)
        den = np.linalg.norm(cq, axis=1) * np.linalg.norm(qv)
        true = np.divide(cq @ qv, den, out=np.zeros(n), where=den > 0)
        assert np.all(np.abs(true - gs[q, :n]) <= TOL)
        # ranks decided by a clear margin must carry the oracle's index
        s = full_s[q]
        for r in range(m):
            above = s[r - 1] - s[r] if r > 0 else np.inf
            below = s[r] - s[r + 1] if r + 1 < s.size else np.inf
            if above > 2 * TOL and below > 2 * TOL:
                assert gi[q, r] == oi[q, r], (q, r)
                exact += 1
    return exact


def run_gpu(Qm, C, K, tau, round_candidates):
    gi, gs, gc = w2v.topk_cosine(torch.from_numpy(Qm).cuda(), torch.from_numpy(C).cuda(), K, tau,
                                 round_candidates=round_candidates)
    torch.cuda.synchronize()
    return w2v.index_to_numpy(gi), gs.cpu().numpy(), w2v.index_to_numpy(gc)


@pytest.mark.parametrize("Q,N,d,K,tau", [(5, 1000, 300, 30, -2.0), (300, 5000, 60, 10, 0.2),
                                         (130, 20011, 100, 64, -2.0), (257, 12800, 37, 1, -2.0),
                                         (1, 3, 7, 5, -2.0), (129, 129, 1000, 30, 0.65), (3, 300, 1, 4, -2.0)])
def test_topk_parity(Q, N, d, K, tau):
    say("topk", Q, N, d, K, tau)
    Qm = workloads.embedding_like(Q, d, 1, n_clusters=50)
    C = workloads.embedding_like(N, d, 2, n_clusters=50)
    ref = None
    for rounds in (128, 1024, 0):
        gi, gs, gc = run_gpu(Qm, C, K, tau, rounds)
        if ref is None:
            exact = check_topk(Qm, C, K, tau, gi, gs, gc)
            say("  ranks with an exact index check:", exact, "of", int(gc.sum()))
            if d >= 30:
                assert exact >= 0.5 * int(gc.sum())
            ref = (gi, gs, gc)
        else:   # the round length never changes the result
            assert np.array_equal(gi, ref[0]) and np.array_equal(gs, ref[1]) and np.array_equal(gc, ref[2])


def test_topk_equal_similarities_rank_by_index_and_zero_vectors_score_zero():
    rng = np.random.default_rng(3)
    N, d, K = 2000, 60, 40
    C = workloads.embedding_like(N, d, 4, n_clusters=20)
    C[1000:] = C[:1000]                     # every candidate twice: bitwise equal similarities
    C[7] = 0; C[1007] = 0
    Qm = workloads.embedding_like(6, d, 5, n_clusters=20)
    Qm[5] = 0                               # an all-zero query: similarity 0 with everyone
    gi, gs, gc = run_gpu(Qm, C, K, -2.0, 256)
    for q in range(5):
        a, b = gi[q, 0::2], gi[q, 1::2]
        assert np.all(b == a + 1000), "a candidate and its copy must come as (lower index, higher index)"
        assert np.all(gs[q, 0::2] == gs[q, 1::2])
    assert gi[5].tolist() == list(range(K)) and np.all(gs[5] == 0)
    oi, os_, oc = oracle.topk_cosine(Qm, C, K)
    assert np.array_equal(gi[5], oi[5])
    check_topk(Qm[:5], C, K, -2.0, gi[:5], gs[:5], gc[:5])


def test_topk_similarities_rising_with_the_index_fill_every_pending_list():
    # candidate i is the query direction plus noise that shrinks with i: every round, most
    # candidates beat the current K-th best, so the pending lists run full.
    rng = np.random.default_rng(6)
    N, d, K = 4096, 64, 30
    Qm = rng.standard_normal((4, d)).astype(np.float32)
    noise = rng.standard_normal((N, d)).astype(np.float32)
    scale = np.linspace(3.0, 0.05, N).astype(np.float32)[:, None]
    C = (Qm[0][None, :] + scale * noise).astype(np.float32)
    for rounds in (128, 1024):
        gi, gs, gc = run_gpu(Qm, C, K, -2.0, rounds)
        check_topk(Qm, C, K, -2.0, gi, gs, gc)
    assert gi[0].min() > N // 2


def test_topk_argument_errors():
    q = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    c = torch.zeros((10, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(w2v.W2VError) as e:
        w2v.topk_cosine(q, c, 0)
    assert e.value.code == -2
    with pytest.raises(w2v.W2VError):
        w2v.topk_cosine(q, c, 65)
    with pytest.raises(w2v.W2VError) as e:
        w2v.topk_cosine(q, c, 3, workspace=torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -2
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(w2v.W2VError):
        w2v.topk_cosine(q, c, 3, workspace=ws[4:])
    gi, gs, gc = w2v.topk_cosine(q, c, 3, workspace=ws)        # all zeros: similarity 0, index order
    assert w2v.index_to_numpy(gi).tolist() == [[0, 1, 2]] * 4


def test_topk_full_size_sampled_queries():
    # the benchmark's shape; the oracle checks a sample of the queries
    Q, N, d, K = 4096, 1 << 20, 300, 30
    C = workloads.embedding_like(N, d, 7)
    Qm = workloads.embedding_like(Q, d, 8)
    gi, gs, gc = run_gpu(Qm, C, K, -2.0, 8192)
    pick = np.array([0, 127, 128, 2049, 4095])
    exact = check_topk(Qm[pick], C, K, -2.0, gi[pick], gs[pick], gc[pick])
    say("  full size: exact index checks", exact, "of", pick.size * K)
    assert np.all(gc == K)
    gi2, gs2, gc2 = run_gpu(Qm, C, K, -2.0, 8192)
    assert np.array_equal(gi, gi2) and np.array_equal(gs, gs2)      # reproducible bit for bit


# --- export ---------------------------------------------------------------------------------------------

def test_export_rows_bit_exact():
    V, dt = 1000, 300
    widths = [60, 100, 40, 96, 4]
    begins = np.concatenate([[0], np.cumsum(widths)[:-1]])
    counts = np.ones(V, np.uint64)
    shards = [w2v.Shard(V, w, 9, d_total=dt, col_begin=int(b), init_mode=1) for w, b in zip(widths, begins)]
    for sh in shards:
        sh.set_counts(counts, 0.0)
    rng = np.random.default_rng(10)
    a = dev(rng.integers(0, V, 500).astype(np.uint32))
    b = dev(rng.integers(0, V, 500).astype(np.uint32))
    w2v.train_minibatch(shards, a, b, 5, 77, 0.05)               # move the vectors off their start
    rows = rng.integers(0, V, 333).astype(np.uint32)
    rd = dev(rows)
    for which in (0, 1):
        got = w2v.export_rows(shards[::-1], which, rd).cpu().numpy()      # any shard order
        parts = [sh.get_rows(which, rd).cpu().numpy() for sh in shards]
        assert np.array_equal(got, oracle.export_rows(parts, begins, dt, np.arange(rows.size)))
    whole = oracle.init_rows(9, dt, 0, dt, 0, np.arange(V, dtype=np.uint32))
    fresh = [w2v.Shard(V, w, 9, d_total=dt, col_begin=int(b), init_mode=1) for w, b in zip(widths, begins)]
    allr = torch.arange(V, dtype=torch.int32, device="cuda")
    assert np.array_equal(w2v.export_rows(fresh, 0, allr).cpu().numpy(), whole)
    with pytest.raises(w2v.W2VError) as e:
        w2v.export_rows(fresh[:-1], 0, allr)                      # columns missing
    assert e.value.code == -7
    with pytest.raises(w2v.W2VError):
        w2v.export_rows(fresh + fresh[:1], 0, allr)               # a slice twice
    w2v.export_rows(fresh, 0, dev(np.array([1, V + 5], np.uint32)))
    with pytest.raises(w2v.W2VError) as e:
        fresh[0].status()
    assert e.value.code == -6
    for sh in shards + fresh:
        sh.destroy()
