"""Helpers shared by the GPU parity tests: error measures and small conveniences.

Error measures (the tolerances are the ones the task fixes: 1e-5 after one minibatch, 1e-3 after a
hundred):
  * dots: |gpu - ref| / sum_c |u_c v_c|.  The forward error of an fp32 dot product is bounded by a
    small multiple of eps * sum|u_c v_c|, whatever the cancellation in the sum, so this is the
    quantity that 1e-5 can meaningfully bound; a dropped or misplaced term shows up at about
    1/d >> 1e-5.
  * vectors: |gpu - ref| / max(|ref|, max_c |ref_row,c|), i.e. relative to the element, but
    elements that happen to be tiny are measured against their row's scale.
"""
import numpy as np
import torch

from paper_1606_08495_amd import w2v


def dot_error(gpu, ref, U, W, in_idx, rows):
    """max over slots of |gpu-ref| / sum_c|u_c v_c| (slots with a zero denominator must match exactly)."""
    au = np.abs(U[in_idx].astype(np.float64))                     # [n, d]
    worst = 0.0
    for j in range(rows.shape[1]):
        den = np.einsum("ij,ij->i", au, np.abs(W[rows[:, j]].astype(np.float64)))
        diff = np.abs(gpu[:, j].astype(np.float64) - ref[:, j].astype(np.float64))
        zero = den == 0
        assert np.all(diff[zero] == 0), "non-zero dot where every product is zero"
        if np.any(~zero):
            worst = max(worst, float(np.max(diff[~zero] / den[~zero])))
    return worst


def vec_error(gpu, ref):
    """max over elements of |gpu-ref| / max(|ref|, row max |ref|); all-zero rows must match exactly."""
    gpu = gpu.astype(np.float64)
    ref = ref.astype(np.float64)
    scale = np.max(np.abs(ref), axis=1, keepdims=True)
    diff = np.abs(gpu - ref)
    zero = scale[:, 0] == 0
    assert np.all(diff[zero] == 0), "a row that must stay zero changed"
    if np.all(zero):
        return 0.0
    den = np.maximum(np.abs(ref[~zero]), scale[~zero])
    return float(np.max(diff[~zero] / den))


def dev(a):
    return w2v.as_index_tensor(a)


def all_rows(shard, which):
    rows = torch.arange(shard.V, dtype=torch.int32, device="cuda")
    return shard.get_rows(which, rows).cpu().numpy()


def set_all_rows(shard, which, M):
    rows = torch.arange(shard.V, dtype=torch.int32, device="cuda")
    shard.set_rows(which, rows, torch.from_numpy(np.ascontiguousarray(M, np.float32)).cuda())


def zipf_counts(V, s=1.0, total=1e7):
    return np.maximum(1, total / np.arange(1, V + 1) ** s).astype(np.uint64)
