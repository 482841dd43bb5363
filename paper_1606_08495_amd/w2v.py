"""Thin ctypes binding over libw2v_shard.so -- same names as include/w2v_shard.h.

Argument marshalling only: every step of the shard path runs in the library's HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the stream.  There is no fallback: if
the library has not been built, or a call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("W2V_LIB", os.path.join(_HERE, "libw2v_shard.so"))
_lib = None

PHASES = ["neg", "dot", "coeff", "sort", "uside", "wside", "apply", "pairs"]
K_MAX, D_MAX, S_MAX = 64, 1024, 32
NOALLOC_SCRATCH_U32 = 1 << 21

c_u32, c_u64, c_vp = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p

_SIGNATURES = {
    "w2v_last_error": (ctypes.c_char_p, []),
    "w2v_shard_create": (ctypes.c_int, [c_u32, c_u32, c_u64, ctypes.POINTER(c_vp)]),
    "w2v_shard_create_ex": (ctypes.c_int, [c_u32, c_u32, c_u32, c_u32, c_u64, ctypes.c_int,
                                           ctypes.POINTER(c_vp)]),
    "w2v_shard_destroy": (ctypes.c_int, [c_vp]),
    "w2v_shard_set_counts": (ctypes.c_int, [c_vp, c_vp, ctypes.c_double]),
    "w2v_shard_get_tables": (ctypes.c_int, [c_vp, c_vp, c_vp, c_vp]),
    "w2v_shard_get_rows": (ctypes.c_int, [c_vp, ctypes.c_int, c_vp, c_u32, c_vp, c_vp]),
    "w2v_shard_set_rows": (ctypes.c_int, [c_vp, ctypes.c_int, c_vp, c_u32, c_vp, c_vp]),
    "w2v_shard_status": (ctypes.c_int, [c_vp, c_vp]),
    "w2v_negatives": (ctypes.c_int, [c_vp, c_vp, c_u32, c_u32, c_u64, c_vp, c_vp]),
    "w2v_dotprod": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_vp, c_vp]),
    "w2v_dotprod_noalloc": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_vp, c_vp]),
    "w2v_prefetch_cancel": (ctypes.c_int, [c_vp]),
    "w2v_coeffs": (ctypes.c_int, [c_vp, ctypes.POINTER(c_vp), c_u32, c_u32, c_u32, c_vp, c_vp, c_vp]),
    "w2v_adjust": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_vp, ctypes.c_float, c_vp]),
    "w2v_train_minibatch": (ctypes.c_int, [ctypes.POINTER(c_vp), c_u32, c_vp, c_vp, c_u32, c_u32,
                                           c_u64, ctypes.c_float, c_vp, c_vp]),
    "w2v_step_graph_create": (ctypes.c_int, [c_vp, c_u32, c_u32, c_vp, ctypes.POINTER(c_vp)]),
    "w2v_step_graph_run": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u64, ctypes.c_float, c_vp]),
    "w2v_step_graph_destroy": (ctypes.c_int, [c_vp]),
    "w2v_prefetch_minibatch": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_vp]),
    "w2v_cbow_prefetch_minibatch": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_vp, c_u32, c_u32, c_u64,
                                                   c_vp]),
    "w2v_make_pairs": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_u32, c_u64, c_u32,
                                      c_vp, c_vp, c_u64, ctypes.POINTER(c_u64), c_vp]),
    "w2v_make_pairs_interleaved": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_u32, c_u64,
                                                  c_u32, c_vp, c_vp, c_u64, ctypes.POINTER(c_u64),
                                                  c_vp]),
    "w2v_cbow_dotprod": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_vp, c_u32, c_u32, c_u64, c_vp, c_vp]),
    "w2v_cbow_adjust": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_vp, c_u32, c_u32, c_u64, c_vp,
                                       ctypes.c_float, c_vp]),
    "w2v_cbow_train_minibatch": (ctypes.c_int, [ctypes.POINTER(c_vp), c_u32, c_vp, c_vp, c_u32, c_vp,
                                                c_u32, c_u32, c_u64, ctypes.c_float, c_vp, c_vp]),
    "w2v_make_cbow_examples": (ctypes.c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u64, c_u32, c_u64,
                                              c_u32, c_vp, c_vp, c_vp, c_u64, c_u64,
                                              ctypes.POINTER(c_u64), ctypes.POINTER(c_u64), c_vp]),
    "w2v_export_rows": (ctypes.c_int, [ctypes.POINTER(c_vp), c_u32, ctypes.c_int, c_vp, c_u32, c_vp, c_vp]),
    "w2v_topk_cosine_workspace": (ctypes.c_size_t, [c_u32, c_u32, c_u32]),
    "w2v_topk_cosine": (ctypes.c_int, [c_vp, c_u32, c_vp, c_u32, c_u32, c_u32, ctypes.c_float, c_vp,
                                       c_vp, c_vp, c_vp, ctypes.c_size_t, c_vp]),
    "w2v_minibatch_seed": (c_u64, [c_u64, c_u64]),
    "w2v_shard_timing_enable": (ctypes.c_int, [c_vp, ctypes.c_int]),
    "w2v_shard_timing_read": (ctypes.c_int, [c_vp, c_vp, c_vp]),
}
EXPORTS = sorted(_SIGNATURES)


class W2VError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("w2v error %d: %s" % (code, text))
        self.code = code


def lib():
    """Opens the built library; a missing library is an error (run paper_1606_08495_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_1606_08495_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise W2VError(rc, lib().w2v_last_error().decode("utf-8", "replace"))


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_vp(stream.cuda_stream)


def _dev(t, dtype, name):
    if t is None:
        return c_vp(0)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))
    return c_vp(t.data_ptr())


# uint32 index arrays are carried in int32 tensors (torch has no arithmetic on uint32; the bit
# patterns are what the library reads).
IDX = torch.int32


def as_index_tensor(a, device="cuda"):
    """numpy uint32/int array -> int32 device tensor with the same bit pattern."""
    a = np.ascontiguousarray(a, dtype=np.uint32)
    return torch.from_numpy(a.view(np.int32)).to(device)


def index_to_numpy(t):
    return t.detach().cpu().numpy().view(np.uint32)


def minibatch_seed(master_seed, h):
    return int(lib().w2v_minibatch_seed(c_u64(master_seed), c_u64(h)))


class Shard:
    """One column shard (w2v_shard).  Methods mirror the C entry points one to one."""

    def __init__(self, V, d_slice, seed, d_total=None, col_begin=0, init_mode=0):
        self.V, self.d_slice = int(V), int(d_slice)
        self.d_total = int(d_slice if d_total is None else d_total)
        self.col_begin = int(col_begin)
        h = c_vp(0)
        _check(lib().w2v_shard_create_ex(self.V, self.d_total, self.col_begin, self.d_slice,
                                         int(seed), int(init_mode), ctypes.byref(h)))
        self.h = h

    def destroy(self):
        if getattr(self, "h", None):
            lib().w2v_shard_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- tables ------------------------------------------------------------------------------
    def set_counts(self, counts, subsample_t=0.0):
        counts = np.ascontiguousarray(counts, dtype=np.uint64)
        if counts.size != self.V:
            raise ValueError("counts must have V entries")
        _check(lib().w2v_shard_set_counts(self.h, c_vp(counts.ctypes.data), float(subsample_t)))

    def get_tables(self):
        th = np.empty(self.V, np.uint32)
        al = np.empty(self.V, np.uint32)
        kp = np.empty(self.V, np.uint64)
        _check(lib().w2v_shard_get_tables(self.h, c_vp(th.ctypes.data), c_vp(al.ctypes.data),
                                          c_vp(kp.ctypes.data)))
        return th, al, kp

    # -- rows ----------------------------------------------------------------------------------
    def get_rows(self, which, rows, stream=None):
        out = torch.empty((rows.numel(), self.d_slice), dtype=torch.float32, device=rows.device)
        _check(lib().w2v_shard_get_rows(self.h, int(which), _dev(rows, IDX, "rows"), rows.numel(),
                                        _dev(out, torch.float32, "dst"), _stream(stream)))
        return out

    def set_rows(self, which, rows, src, stream=None):
        if src.shape != (rows.numel(), self.d_slice):
            raise ValueError("src must be [m, d_slice]")
        _check(lib().w2v_shard_set_rows(self.h, int(which), _dev(rows, IDX, "rows"), rows.numel(),
                                        _dev(src, torch.float32, "src"), _stream(stream)))

    def status(self, stream=None):
        _check(lib().w2v_shard_status(self.h, _stream(stream)))

    # -- the calls of the paper ------------------------------------------------------------------
    def negatives(self, out_idx, k, seed, stream=None):
        n = out_idx.numel()
        neg = torch.empty((n, k), dtype=IDX, device=out_idx.device)
        _check(lib().w2v_negatives(self.h, _dev(out_idx, IDX, "out_idx"), n, int(k), int(seed),
                                   _dev(neg, IDX, "neg"), _stream(stream)))
        return neg

    def dotprod(self, in_idx, out_idx, k, seed, out=None, stream=None):
        n = in_idx.numel()
        if out is None:
            out = torch.empty((n, k + 1), dtype=torch.float32, device=in_idx.device)
        _check(lib().w2v_dotprod(self.h, _dev(in_idx, IDX, "in_idx"), _dev(out_idx, IDX, "out_idx"),
                                 n, int(k), int(seed), _dev(out, torch.float32, "partial_dots"),
                                 _stream(stream)))
        return out

    def dotprod_noalloc(self, in_idx, out_idx, k, seed, out, stream=None):
        """w2v_dotprod_noalloc: `out` ([n, k+1] float32) must be given; the library allocates nothing."""
        _check(lib().w2v_dotprod_noalloc(self.h, _dev(in_idx, IDX, "in_idx"),
                                         _dev(out_idx, IDX, "out_idx"), in_idx.numel(), int(k),
                                         int(seed), _dev(out, torch.float32, "partial_dots"),
                                         _stream(stream)))
        return out

    def prefetch_cancel(self):
        _check(lib().w2v_prefetch_cancel(self.h))

    def coeffs(self, partials, k, want_loss=False, out=None, stream=None):
        S = len(partials)
        n = partials[0].shape[0]
        arr = (c_vp * S)(*[p.data_ptr() for p in partials])
        for p in partials:
            _dev(p, torch.float32, "partials")
        if out is None:
            out = torch.empty((n, k + 1), dtype=torch.float32, device=partials[0].device)
        loss = torch.zeros(1, dtype=torch.float64, device=out.device) if want_loss else None
        _check(lib().w2v_coeffs(self.h, arr, S, n, int(k), _dev(out, torch.float32, "coeffs"),
                                _dev(loss, torch.float64, "loss"), _stream(stream)))
        return (out, loss) if want_loss else out

    def adjust(self, in_idx, out_idx, k, seed, coeffs, alpha, stream=None):
        n = in_idx.numel()
        _check(lib().w2v_adjust(self.h, _dev(in_idx, IDX, "in_idx"), _dev(out_idx, IDX, "out_idx"),
                                n, int(k), int(seed), _dev(coeffs, torch.float32, "coeffs"),
                                float(alpha), _stream(stream)))

    def prefetch_minibatch(self, in_idx, out_idx, k, seed, stream=None):
        """Index work of the next minibatch, queued beside the current one (w2v_prefetch_minibatch)."""
        _check(lib().w2v_prefetch_minibatch(self.h, _dev(in_idx, IDX, "in_idx"),
                                            _dev(out_idx, IDX, "out_idx"), in_idx.numel(), int(k),
                                            int(seed), _stream(stream)))

    def make_pairs(self, tokens, sent_off, token_base, epoch, corpus_seed, B, in_idx, out_idx,
                   stream=None, interleaved=False):
        """tokens int32[n] (uint32 bits), sent_off int64[m+1] on the device; fills in_idx/out_idx
        (capacity = their length) and returns the full pair count.  ``interleaved`` calls
        w2v_make_pairs_interleaved instead of w2v_make_pairs."""
        cnt = c_u64(0)
        fn = lib().w2v_make_pairs_interleaved if interleaved else lib().w2v_make_pairs
        _check(fn(self.h, _dev(tokens, IDX, "tokens"),
                                    _dev(sent_off, torch.int64, "sent_off"), sent_off.numel() - 1,
                                    tokens.numel(), int(token_base), int(epoch), int(corpus_seed),
                                    int(B), _dev(in_idx, IDX, "in_idx"), _dev(out_idx, IDX, "out_idx"),
                                    min(in_idx.numel(), out_idx.numel()), ctypes.byref(cnt),
                                    _stream(stream)))
        return int(cnt.value)

    # -- continuous bag of words -----------------------------------------------------------------
    def cbow_dotprod(self, ctx_off, ctx_idx, out_idx, k, seed, out=None, stream=None):
        """ctx_off int32[n+1], ctx_idx int32[m], out_idx int32[n] (uint32 bits) on the device."""
        n = out_idx.numel()
        if out is None:
            out = torch.empty((n, k + 1), dtype=torch.float32, device=out_idx.device)
        _check(lib().w2v_cbow_dotprod(self.h, _dev(ctx_off, IDX, "ctx_off"),
                                      _dev(ctx_idx, IDX, "ctx_idx"), ctx_idx.numel(),
                                      _dev(out_idx, IDX, "out_idx"), n, int(k), int(seed),
                                      _dev(out, torch.float32, "partial_dots"), _stream(stream)))
        return out

    def cbow_adjust(self, ctx_off, ctx_idx, out_idx, k, seed, coeffs, alpha, stream=None):
        _check(lib().w2v_cbow_adjust(self.h, _dev(ctx_off, IDX, "ctx_off"),
                                     _dev(ctx_idx, IDX, "ctx_idx"), ctx_idx.numel(),
                                     _dev(out_idx, IDX, "out_idx"), out_idx.numel(), int(k), int(seed),
                                     _dev(coeffs, torch.float32, "coeffs"), float(alpha),
                                     _stream(stream)))

    def cbow_prefetch_minibatch(self, ctx_off, ctx_idx, out_idx, k, seed, stream=None):
        """Index work of a later bag-of-words minibatch, queued beside the calls that follow."""
        _check(lib().w2v_cbow_prefetch_minibatch(self.h, _dev(ctx_off, IDX, "ctx_off"),
                                                 _dev(ctx_idx, IDX, "ctx_idx"), ctx_idx.numel(),
                                                 _dev(out_idx, IDX, "out_idx"), out_idx.numel(),
                                                 int(k), int(seed), _stream(stream)))

    def make_cbow_examples(self, tokens, sent_off, token_base, epoch, corpus_seed, B, ctx_off, ctx_idx,
                           out_idx, stream=None):
        """Fills ctx_off (length cap+1), ctx_idx and out_idx (length cap) on the device; returns
        the full (number of examples, number of context entries)."""
        n_ex, n_ctx = c_u64(0), c_u64(0)
        cap = min(out_idx.numel(), ctx_off.numel() - 1)
        _check(lib().w2v_make_cbow_examples(
            self.h, _dev(tokens, IDX, "tokens"), _dev(sent_off, torch.int64, "sent_off"),
            sent_off.numel() - 1, tokens.numel(), int(token_base), int(epoch), int(corpus_seed), int(B),
            _dev(ctx_off, IDX, "ctx_off"), _dev(ctx_idx, IDX, "ctx_idx"), _dev(out_idx, IDX, "out_idx"),
            cap, ctx_idx.numel(), ctypes.byref(n_ex), ctypes.byref(n_ctx), _stream(stream)))
        return int(n_ex.value), int(n_ctx.value)

    # -- timing ----------------------------------------------------------------------------------
    def timing_enable(self, on=True):
        _check(lib().w2v_shard_timing_enable(self.h, int(bool(on))))

    def timing_read(self):
        ms = np.zeros(len(PHASES), np.float64)
        cnt = np.zeros(len(PHASES), np.uint64)
        _check(lib().w2v_shard_timing_read(self.h, c_vp(ms.ctypes.data), c_vp(cnt.ctypes.data)))
        return {PHASES[i]: (float(ms[i]), int(cnt[i])) for i in range(len(PHASES))}


class StepGraph:
    """w2v_step_graph: w2v_train_minibatch on one shard for a fixed (n, k), captured once and replayed."""

    def __init__(self, shard, n, k, loss=None):
        self.n, self.k, self.shard, self.loss = int(n), int(k), shard, loss
        h = c_vp(0)
        _check(lib().w2v_step_graph_create(shard.h, self.n, self.k, _dev(loss, torch.float64, "loss"),
                                           ctypes.byref(h)))
        self.h = h

    def run(self, in_idx, out_idx, seed, alpha, stream=None):
        if in_idx.numel() != self.n or out_idx.numel() != self.n:
            raise ValueError("the graph was captured for %d pairs" % self.n)
        _check(lib().w2v_step_graph_run(self.h, _dev(in_idx, IDX, "in_idx"), _dev(out_idx, IDX, "out_idx"),
                                        int(seed), float(alpha), _stream(stream)))

    def destroy(self):
        if getattr(self, "h", None):
            lib().w2v_step_graph_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def train_minibatch(shards, in_idx, out_idx, k, seed, alpha, loss=None, stream=None):
    """One client step over the given shards (w2v_train_minibatch).  ``loss``: optional float64
    device tensor of one element that receives the minibatch loss."""
    S = len(shards)
    arr = (c_vp * S)(*[s.h.value for s in shards])
    n = in_idx.numel()
    _check(lib().w2v_train_minibatch(arr, S, _dev(in_idx, IDX, "in_idx"),
                                     _dev(out_idx, IDX, "out_idx"), n, int(k), int(seed),
                                     float(alpha), _dev(loss, torch.float64, "loss"),
                                     _stream(stream)))


def cbow_train_minibatch(shards, ctx_off, ctx_idx, out_idx, k, seed, alpha, loss=None, stream=None):
    """One client step of the bag-of-words variant over the given shards
    (w2v_cbow_train_minibatch)."""
    S = len(shards)
    arr = (c_vp * S)(*[s.h.value for s in shards])
    _check(lib().w2v_cbow_train_minibatch(arr, S, _dev(ctx_off, IDX, "ctx_off"),
                                          _dev(ctx_idx, IDX, "ctx_idx"), ctx_idx.numel(),
                                          _dev(out_idx, IDX, "out_idx"), out_idx.numel(), int(k),
                                          int(seed), float(alpha), _dev(loss, torch.float64, "loss"),
                                          _stream(stream)))


def export_rows(shards, which, rows, out=None, stream=None):
    """Whole vectors [m, d_total] of the listed rows, joined from the column shards
    (w2v_export_rows)."""
    S = len(shards)
    arr = (c_vp * S)(*[s.h.value for s in shards])
    m = rows.numel()
    if out is None:
        out = torch.empty((m, shards[0].d_total), dtype=torch.float32, device=rows.device)
    _check(lib().w2v_export_rows(arr, S, int(which), _dev(rows, IDX, "rows"), m,
                                 _dev(out, torch.float32, "dst"), _stream(stream)))
    return out


def topk_cosine(queries, cands, K, tau=-2.0, round_candidates=32768, workspace=None, stream=None):
    """(idx int32[Q, K] (uint32 bits), score float32[Q, K], count int32[Q]) of w2v_topk_cosine.
    ``workspace``: optional uint8 device tensor to reuse; otherwise one for rounds of
    ``round_candidates`` candidates is allocated here."""
    Q, d = queries.shape
    N = cands.shape[0]
    if cands.shape[1] != d:
        raise ValueError("queries and candidates differ in width")
    if workspace is None:
        need = int(lib().w2v_topk_cosine_workspace(Q, N, int(round_candidates)))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=queries.device)
    idx = torch.empty((Q, K), dtype=IDX, device=queries.device)
    score = torch.empty((Q, K), dtype=torch.float32, device=queries.device)
    count = torch.empty(Q, dtype=IDX, device=queries.device)
    _check(lib().w2v_topk_cosine(_dev(queries, torch.float32, "queries"), Q,
                                 _dev(cands, torch.float32, "cands"), N, d, int(K), float(tau),
                                 _dev(idx, IDX, "out_idx"), _dev(score, torch.float32, "out_score"),
                                 _dev(count, IDX, "out_count"), c_vp(workspace.data_ptr()),
                                 workspace.numel(), _stream(stream)))
    return idx, score, count
