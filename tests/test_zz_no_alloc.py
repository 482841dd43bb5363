"""The entry point that allocates nothing (w2v_dotprod_noalloc), through the C ABI, against
w2v_dotprod: the same bits, on two calls in a row of which the second is smaller (the static
scratch array keeps the first call's contents), and against the oracle; sizes beyond the static
array are refused."""
import numpy as np
import pytest
import torch

import oracle
from paper_1606_08495_amd import w2v
from util import dev, dot_error, zipf_counts

pytestmark = pytest.mark.gpu


def test_no_alloc_dotprod_matches_dotprod_on_two_calls_in_a_row():
    V, d, k = 5000, 300, 5
    rng = np.random.default_rng(321)
    counts = zipf_counts(V)
    sh = w2v.Shard(V, d, 17, init_mode=1)
    sh.set_counts(counts)
    rows_all = np.arange(V, dtype=np.uint32)
    U = oracle.init_rows(17, d, 0, d, 0, rows_all)
    W = oracle.init_rows(17, d, 0, d, 1, rows_all)
    th, al = oracle.build_alias(counts)
    for n, seed in ((70_001, 11), (4_099, 12)):          # the second call is smaller
        print("no-alloc dotprod: n", n, "k", k, "seed", seed, flush=True)
        in_idx = rng.integers(0, V, n).astype(np.uint32)
        out_idx = rng.integers(0, V, n).astype(np.uint32)
        a, b = dev(in_idx), dev(out_idx)
        out = torch.full((n, k + 1), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        sh.dotprod_noalloc(a, b, k, seed, out)
        assert torch.cuda.memory_allocated() == before
        got = out.cpu().numpy()
        want = sh.dotprod(a, b, k, seed).cpu().numpy()
        assert np.array_equal(got, want)
        ref = oracle.dotprod(U, W, in_idx, out_idx, k, seed, th, al)
        rows = np.concatenate([out_idx[:, None], oracle.negatives(out_idx, k, seed, th, al)], axis=1)
        assert dot_error(got, ref, U, W, in_idx, rows) <= 1e-5
    sh.status()
    # a second shard on the same GPU shares the array; narrow rows, other k
    sh2 = w2v.Shard(300, 60, 3, d_total=300, col_begin=60, init_mode=1)
    sh2.set_counts(zipf_counts(300))
    a, b = dev(rng.integers(0, 300, 1000)), dev(rng.integers(0, 300, 1000))
    out = torch.empty((1000, 11), dtype=torch.float32, device="cuda")
    sh2.dotprod_noalloc(a, b, 10, 5, out)
    assert np.array_equal(out.cpu().numpy(), sh2.dotprod(a, b, 10, 5).cpu().numpy())
    # beyond the static array: refused with a clear error, nothing launched
    n_big = w2v.NOALLOC_SCRATCH_U32 // (k + 2) + 1
    big = torch.zeros(n_big, dtype=torch.int32, device="cuda")
    out = torch.empty((n_big, k + 1), dtype=torch.float32, device="cuda")
    with pytest.raises(w2v.W2VError) as e:
        sh.dotprod_noalloc(big, big, k, 1, out)
    assert e.value.code == -2 and "static scratch" in str(e.value)
    # the largest size that fits still works
    n_fit = (w2v.NOALLOC_SCRATCH_U32 - 64) // (k + 2)
    fit = dev(rng.integers(0, V, n_fit))
    out = torch.empty((n_fit, k + 1), dtype=torch.float32, device="cuda")
    sh.dotprod_noalloc(fit, fit, k, 2, out)
    assert np.array_equal(out.cpu().numpy(), sh.dotprod(fit, fit, k, 2).cpu().numpy())
    e0 = torch.empty(0, dtype=torch.int32, device="cuda")
    sh.dotprod_noalloc(e0, e0, k, 1, torch.empty((0, k + 1), dtype=torch.float32, device="cuda"))
    sh.status()
    sh2.status()
    sh.destroy()
    sh2.destroy()
