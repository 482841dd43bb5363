"""Helpers shared by the GPU parity tests: error measures and small conveniences.

Error measures (the tolerances are the ones the task fixes: 1e-5 after one minibatch, 1e-3 after a
hundred):
  * dots: |gpu - ref| / sum_c |u_c v_c|.  The forward error of an fp32 dot product is bounded by a
    small multiple of eps * sum|u_c v_c|, whatever the cancellation in the sum, so this is the
    quantity that 1e-5 can meaningfully bound; a dropped or misplaced term shows up at about
    1/d >> 1e-5.
  * vectors, three measures:
      vec_error       |gpu - ref| / max_c |ref_row,c|: relative to the row's largest component
                      (row-normwise).  This is what a fixed bound can hold against: a component that
                      nearly cancels has an error set by the terms that went into it, not by what is
                      left of them.
      vec_error_elem  |gpu - ref| / max(|ref|, floor * max_c |ref_row,c|): relative to the element
                      itself, down to components `floor` times smaller than the row's largest.
                      Reported beside the first one (floor 1e-2).
      delta_error     the CHANGE of a row, (after - before) / alpha, against the oracle's summed
                      change, relative to that sum's largest component.  With both matrices
                      initialised one update moves a row by about a per cent, so a row-level bound
                      of 1e-5 resolves the change only to 1e-3; this measure looks at the change
                      itself.  The stored row is fl(before + alpha * sum), so what can be recovered
                      from it is the sum plus up to half an ulp of the stored value divided by
                      alpha; that slack is subtracted element by element before the comparison.
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
    """max over elements of |gpu-ref| / (largest |component| of the element's ref row);
    all-zero rows must match exactly."""
    return vec_error_elem(gpu, ref, floor=1.0)


def vec_error_elem(gpu, ref, floor=1e-2):
    """max over elements of |gpu-ref| / max(|ref|, floor * row max |ref|); all-zero rows must match
    exactly.  floor = 1 is the row-normwise measure."""
    gpu = gpu.astype(np.float64)
    ref = ref.astype(np.float64)
    scale = np.max(np.abs(ref), axis=1, keepdims=True)
    diff = np.abs(gpu - ref)
    zero = scale[:, 0] == 0
    assert np.all(diff[zero] == 0), "a row that must stay zero changed"
    if np.all(zero):
        return 0.0
    den = np.maximum(np.abs(ref[~zero]), floor * scale[~zero])
    return float(np.max(diff[~zero] / den))


def delta_error(after, before, alpha, delta_ref):
    """The update itself: (after - before) / alpha against the oracle's summed change delta_ref
    (double), as max over elements of max(0, |difference| - store slack) / (largest |component| of the
    element's delta_ref row), the store slack being half an ulp of the stored fp32 value over alpha.
    Rows whose summed change is all zero must be bitwise unchanged."""
    alpha = float(np.float32(alpha))
    after32 = np.ascontiguousarray(after, np.float32)
    got = (after32.astype(np.float64) - np.asarray(before, np.float64)) / alpha
    ref = np.asarray(delta_ref, np.float64)
    scale = np.max(np.abs(ref), axis=1, keepdims=True)
    zero = scale[:, 0] == 0
    assert np.array_equal(after32[zero], np.asarray(before, np.float32)[zero]), \
        "a row without contributions changed"
    if np.all(zero):
        return 0.0
    slack = 0.5 * np.spacing(np.abs(after32)).astype(np.float64) / alpha
    excess = np.maximum(0.0, np.abs(got - ref) - slack)
    return float(np.max(excess[~zero] / scale[~zero]))


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
