"""ctypes front end of the CPU oracle (w2v_oracle.cpp).

Test infrastructure only: importable from tests/, from the smoke check and from the benchmark's
cpu_baseline leg.  Nothing here touches the GPU library, and the GPU library never imports this.

Every function takes and returns numpy arrays; shapes follow the paper's routines:
``rows`` is [n, k+1] with the positive output word in column 0 and the negatives after it.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w2v_oracle.cpp")
_SO = os.path.join(_HERE, "libw2v_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with g++ (no GPU toolchain involved)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
               "-o", _SO, _SRC]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        L.orc_minibatch_seed.restype = ctypes.c_uint64
        L.orc_minibatch_seed.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        L.orc_make_pairs.restype = ctypes.c_uint64
        L.orc_make_pairs_interleaved.restype = ctypes.c_uint64
        L.orc_make_cbow_examples.restype = ctypes.c_uint64
        L.orc_lazy_create.restype = ctypes.c_void_p
        L.orc_lazy_rows_held.restype = ctypes.c_uint64
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


U64 = ctypes.c_uint64
U32 = ctypes.c_uint32


def philox(ctr, key):
    c = _u32(ctr)
    k = _u32(key)
    out = np.zeros(4, np.uint32)
    lib().orc_philox(_p(c), _p(k), _p(out))
    return out


def minibatch_seed(master_seed, h):
    return int(lib().orc_minibatch_seed(U64(master_seed), U64(h)))


def init_rows(seed, d_total, col_begin, d_slice, matrix, rows):
    rows = _u32(rows)
    out = np.empty((rows.size, d_slice), np.float32)
    lib().orc_init_rows(U64(seed), U32(d_total), U32(col_begin), U32(d_slice), U32(matrix),
                        _p(rows), U64(rows.size), _p(out))
    return out


def noise_probs(counts):
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    out = np.empty(counts.size, np.float64)
    lib().orc_noise_probs(_p(counts), U32(counts.size), _p(out))
    return out


def build_alias(counts):
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    thresh = np.empty(counts.size, np.uint32)
    alias = np.empty(counts.size, np.uint32)
    lib().orc_build_alias(_p(counts), U32(counts.size), _p(thresh), _p(alias))
    return thresh, alias


def build_keep(counts, t):
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    out = np.empty(counts.size, np.uint64)
    lib().orc_build_keep(_p(counts), U32(counts.size), ctypes.c_double(t), _p(out))
    return out


def negatives(out_idx, k, seed, thresh, alias, pair_ids=None):
    out_idx = _u32(out_idx)
    n = out_idx.size
    pid = None if pair_ids is None else _u32(pair_ids)
    neg = np.empty((n, k), np.uint32)
    lib().orc_negatives(_p(out_idx), _p(pid), U64(n), U32(k), U64(seed), U32(thresh.size),
                        _p(thresh), _p(alias), _p(neg))
    return neg


def dots(U, W, in_idx, rows):
    U = _f32(U)
    W = _f32(W)
    in_idx = _u32(in_idx)
    rows = _u32(rows)
    n, T = rows.shape
    out = np.empty((n, T), np.float32)
    lib().orc_dots(_p(U), _p(W), U32(U.shape[1]), _p(in_idx), _p(rows), U64(n), U32(T), _p(out))
    return out


def dotprod(U, W, in_idx, out_idx, k, seed, thresh, alias):
    U = _f32(U)
    W = _f32(W)
    in_idx = _u32(in_idx)
    out_idx = _u32(out_idx)
    n = in_idx.size
    out = np.empty((n, k + 1), np.float32)
    lib().orc_dotprod(_p(U), _p(W), U32(U.shape[0]), U32(U.shape[1]), _p(in_idx), _p(out_idx),
                      U64(n), U32(k), U64(seed), _p(thresh), _p(alias), _p(out))
    return out


def coeffs(partials, want_loss=False):
    """partials: list of S arrays [n, T] -> coefficient array [n, T] (and the minibatch loss)."""
    parts = [_f32(a) for a in partials]
    n, T = parts[0].shape
    arr = (ctypes.c_void_p * len(parts))(*[a.ctypes.data for a in parts])
    out = np.empty((n, T), np.float32)
    loss = ctypes.c_double(0.0)
    lib().orc_coeffs(arr, U32(len(parts)), U64(n), U32(T), _p(out), ctypes.byref(loss))
    return (out, loss.value) if want_loss else out


def adjust_rows(U, W, in_idx, rows, coeffs_, alpha, sequential_fp32=False):
    """In place on U and W (float32, C-contiguous)."""
    assert U.dtype == np.float32 and W.dtype == np.float32
    assert U.flags.c_contiguous and W.flags.c_contiguous
    in_idx = _u32(in_idx)
    rows = _u32(rows)
    g = _f32(coeffs_)
    n, T = rows.shape
    lib().orc_adjust_rows(_p(U), _p(W), U32(U.shape[1]), _p(in_idx), _p(rows), U64(n), U32(T),
                          _p(g), ctypes.c_float(alpha), ctypes.c_int(int(sequential_fp32)))


def adjust_deltas(U, W, in_idx, rows, coeffs_, want_u=None, want_w=None):
    """The adjust routine's scratch sums (double, learning rate not applied) for the listed words
    (default: every row of U / W); U and W are left as they are.  Returns (dU, dW)."""
    U, W = _f32(U), _f32(W)
    in_idx = _u32(in_idx)
    rows = _u32(rows)
    g = _f32(coeffs_)
    n, T = rows.shape
    want_u = _u32(np.arange(U.shape[0]) if want_u is None else want_u)
    want_w = _u32(np.arange(W.shape[0]) if want_w is None else want_w)
    d = U.shape[1]
    dU = np.empty((want_u.size, d), np.float64)
    dW = np.empty((want_w.size, d), np.float64)
    lib().orc_adjust_deltas(_p(U), _p(W), U32(d), _p(in_idx), _p(rows), U64(n), U32(T), _p(g),
                            _p(want_u), U64(want_u.size), _p(want_w), U64(want_w.size), _p(dU), _p(dW))
    return dU, dW


def adjust(U, W, in_idx, out_idx, k, seed, thresh, alias, coeffs_, alpha):
    assert U.dtype == np.float32 and W.dtype == np.float32
    assert U.flags.c_contiguous and W.flags.c_contiguous
    in_idx = _u32(in_idx)
    out_idx = _u32(out_idx)
    g = _f32(coeffs_)
    lib().orc_adjust(_p(U), _p(W), U32(U.shape[0]), U32(U.shape[1]), _p(in_idx), _p(out_idx),
                     U64(in_idx.size), U32(k), U64(seed), _p(thresh), _p(alias), _p(g),
                     ctypes.c_float(alpha))


def train_minibatch(Us, Ws, in_idx, out_idx, k, seed, thresh, alias, alpha):
    """One client step over S in-process column shards (lists of float32 arrays); returns loss."""
    S = len(Us)
    for a in list(Us) + list(Ws):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    in_idx = _u32(in_idx)
    out_idx = _u32(out_idx)
    up = (ctypes.c_void_p * S)(*[a.ctypes.data for a in Us])
    wp = (ctypes.c_void_p * S)(*[a.ctypes.data for a in Ws])
    ds = np.array([a.shape[1] for a in Us], np.uint32)
    loss = ctypes.c_double(0.0)
    lib().orc_train_minibatch(up, wp, _p(ds), U32(S), U32(Us[0].shape[0]), _p(in_idx), _p(out_idx),
                              U64(in_idx.size), U32(k), U64(seed), _p(thresh), _p(alias),
                              ctypes.c_float(alpha), ctypes.byref(loss))
    return loss.value


class LazyShard:
    """Rows created on first touch from the initialisation function; for large vocabularies."""

    def __init__(self, V, d_total, col_begin, d_slice, seed, w_uniform):
        self.d = d_slice
        self.h = ctypes.c_void_p(lib().orc_lazy_create(U32(V), U32(d_total), U32(col_begin),
                                                       U32(d_slice), U64(seed),
                                                       ctypes.c_int(int(w_uniform))))

    def close(self):
        if self.h:
            lib().orc_lazy_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def row(self, which, w):
        out = np.empty(self.d, np.float32)
        lib().orc_lazy_get_row(self.h, ctypes.c_int(which), U32(w), _p(out))
        return out

    def rows_held(self):
        return int(lib().orc_lazy_rows_held(self.h))

    def train_minibatch(self, in_idx, out_idx, k, seed, thresh, alias, alpha):
        in_idx = _u32(in_idx)
        out_idx = _u32(out_idx)
        loss = ctypes.c_double(0.0)
        lib().orc_lazy_train_minibatch(self.h, _p(in_idx), _p(out_idx), U64(in_idx.size), U32(k),
                                       U64(seed), _p(thresh), _p(alias), ctypes.c_float(alpha),
                                       ctypes.byref(loss))
        return loss.value


def make_pairs(tokens, sent_off, token_base, epoch, corpus_seed, B, keep_thresh, capacity=None,
               interleaved=False):
    tokens = _u32(tokens)
    sent_off = np.ascontiguousarray(sent_off, dtype=np.uint64)
    kt = None if keep_thresh is None else np.ascontiguousarray(keep_thresh, dtype=np.uint64)
    if capacity is None:
        capacity = int(tokens.size) * 2 * B
    a = np.empty(capacity, np.uint32)
    b = np.empty(capacity, np.uint32)
    fn = lib().orc_make_pairs_interleaved if interleaved else lib().orc_make_pairs
    cnt = fn(_p(tokens), _p(sent_off), U64(sent_off.size - 1), U64(token_base), U32(epoch),
             U64(corpus_seed), U32(B), _p(kt), _p(a), _p(b), U64(capacity))
    cnt = int(cnt)
    m = min(cnt, capacity)
    return a[:m].copy(), b[:m].copy(), cnt


def token_draws(tokens, token_base, epoch, corpus_seed, B, keep_thresh):
    tokens = _u32(tokens)
    kt = None if keep_thresh is None else np.ascontiguousarray(keep_thresh, dtype=np.uint64)
    keep = np.empty(tokens.size, np.uint8)
    b = np.empty(tokens.size, np.uint32)
    lib().orc_token_draws(_p(tokens), U64(tokens.size), U64(token_base), U32(epoch),
                          U64(corpus_seed), U32(B), _p(kt), _p(keep), _p(b))
    return keep, b


# --- continuous bag of words ------------------------------------------------------------------------

def cbow_dots(U, W, ctx_off, ctx_idx, rows):
    U, W, ctx_off, ctx_idx, rows = _f32(U), _f32(W), _u32(ctx_off), _u32(ctx_idx), _u32(rows)
    n, T = rows.shape
    out = np.empty((n, T), np.float32)
    lib().orc_cbow_dots(_p(U), _p(W), U32(U.shape[1]), _p(ctx_off), _p(ctx_idx), _p(rows), U64(n),
                        U32(T), _p(out))
    return out


def cbow_adjust_rows(U, W, ctx_off, ctx_idx, rows, coeffs_, alpha):
    """In place on U and W (float32, C-contiguous)."""
    assert U.dtype == np.float32 and W.dtype == np.float32
    assert U.flags.c_contiguous and W.flags.c_contiguous
    ctx_off, ctx_idx, rows, g = _u32(ctx_off), _u32(ctx_idx), _u32(rows), _f32(coeffs_)
    n, T = rows.shape
    lib().orc_cbow_adjust_rows(_p(U), _p(W), U32(U.shape[1]), _p(ctx_off), _p(ctx_idx), _p(rows),
                               U64(n), U32(T), _p(g), ctypes.c_float(alpha))


def cbow_dotprod(U, W, ctx_off, ctx_idx, out_idx, k, seed, thresh, alias):
    U, W, ctx_off, ctx_idx, out_idx = _f32(U), _f32(W), _u32(ctx_off), _u32(ctx_idx), _u32(out_idx)
    n = out_idx.size
    out = np.empty((n, k + 1), np.float32)
    lib().orc_cbow_dotprod(_p(U), _p(W), U32(U.shape[0]), U32(U.shape[1]), _p(ctx_off), _p(ctx_idx),
                           _p(out_idx), U64(n), U32(k), U64(seed), _p(thresh), _p(alias), _p(out))
    return out


def cbow_adjust(U, W, ctx_off, ctx_idx, out_idx, k, seed, thresh, alias, coeffs_, alpha):
    assert U.dtype == np.float32 and W.dtype == np.float32
    assert U.flags.c_contiguous and W.flags.c_contiguous
    ctx_off, ctx_idx, out_idx, g = _u32(ctx_off), _u32(ctx_idx), _u32(out_idx), _f32(coeffs_)
    lib().orc_cbow_adjust(_p(U), _p(W), U32(U.shape[0]), U32(U.shape[1]), _p(ctx_off), _p(ctx_idx),
                          _p(out_idx), U64(out_idx.size), U32(k), U64(seed), _p(thresh), _p(alias),
                          _p(g), ctypes.c_float(alpha))


def cbow_train_minibatch(Us, Ws, ctx_off, ctx_idx, out_idx, k, seed, thresh, alias, alpha):
    S = len(Us)
    for a in list(Us) + list(Ws):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    ctx_off, ctx_idx, out_idx = _u32(ctx_off), _u32(ctx_idx), _u32(out_idx)
    up = (ctypes.c_void_p * S)(*[a.ctypes.data for a in Us])
    wp = (ctypes.c_void_p * S)(*[a.ctypes.data for a in Ws])
    ds = np.array([a.shape[1] for a in Us], np.uint32)
    loss = ctypes.c_double(0.0)
    lib().orc_cbow_train_minibatch(up, wp, _p(ds), U32(S), U32(Us[0].shape[0]), _p(ctx_off),
                                   _p(ctx_idx), _p(out_idx), U64(out_idx.size), U32(k), U64(seed),
                                   _p(thresh), _p(alias), ctypes.c_float(alpha), ctypes.byref(loss))
    return loss.value


def make_cbow_examples(tokens, sent_off, token_base, epoch, corpus_seed, B, keep_thresh,
                       cap_examples=None, cap_ctx=None):
    """Returns (ctx_off[m+1], ctx_idx, out_idx[m], n_examples, n_ctx) with m = min(n_examples, cap)."""
    tokens = _u32(tokens)
    sent_off = np.ascontiguousarray(sent_off, dtype=np.uint64)
    kt = None if keep_thresh is None else np.ascontiguousarray(keep_thresh, dtype=np.uint64)
    if cap_examples is None:
        cap_examples = int(tokens.size)
    if cap_ctx is None:
        cap_ctx = int(tokens.size) * 2 * B
    off = np.zeros(cap_examples + 1, np.uint32)
    ctx = np.empty(cap_ctx, np.uint32)
    out = np.empty(cap_examples, np.uint32)
    nctx = ctypes.c_uint64(0)
    cnt = int(lib().orc_make_cbow_examples(_p(tokens), _p(sent_off), U64(sent_off.size - 1),
                                           U64(token_base), U32(epoch), U64(corpus_seed), U32(B),
                                           _p(kt), _p(off), _p(ctx), _p(out), U64(cap_examples),
                                           U64(cap_ctx), ctypes.byref(nctx)))
    m = min(cnt, cap_examples)
    return off[:m + 1].copy(), ctx[:min(int(nctx.value), cap_ctx)].copy(), out[:m].copy(), cnt, int(nctx.value)


# --- export and retrieval ----------------------------------------------------------------------------

def export_rows(Ms, col_begins, d_total, rows):
    """Vector export (Section 6.1.4): the shards' column slices of the listed rows, joined into
    full vectors [m, d_total].  Ms[s] is the dense [V, d_s] matrix of shard s."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, d_total), np.float32)
    for M, c0 in zip(Ms, col_begins):
        out[:, c0:c0 + M.shape[1]] = M[rows]
    return out


def topk_cosine(Qm, Cm, K, tau=-2.0):
    """(idx uint32[Q,K], score float64[Q,K], count uint32[Q]) of orc_topk_cosine."""
    Qm, Cm = _f32(Qm), _f32(Cm)
    Q, d = Qm.shape
    N = Cm.shape[0]
    assert Cm.shape[1] == d
    idx = np.empty((Q, K), np.uint32)
    score = np.empty((Q, K), np.float64)
    count = np.empty(Q, np.uint32)
    lib().orc_topk_cosine(_p(Qm), U32(Q), _p(Cm), U32(N), U32(d), U32(K), ctypes.c_double(tau),
                          _p(idx), _p(score), _p(count))
    return idx, score, count
