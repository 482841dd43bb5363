#!/usr/bin/env python3
"""Benchmark of the word2vec shard path on one MI355X.

One step = one pass of the whole hot path over one minibatch: pair formation from the token stream
(amortised over the minibatches a token block yields), negatives, dot products, coefficients and
the deterministic adjust -- i.e. w2v_make_pairs + w2v_train_minibatch (workload "full300", the
10M-word d=300 configuration the bandwidth target is stated on), or w2v_dotprod + w2v_adjust with
harness coefficients (workload "slice60", one of five column shards).  In the text workloads the
next minibatch is announced to the shard (w2v_prefetch_minibatch) before the current one is
trained, so its index work runs beside the current step; every minibatch's index work is still done
exactly once inside the timed region (--no-prefetch turns the announcement off).

Prints one JSON line: pairs/s (k negatives included), ms per step, the roofline entry of the
dominant kernel (algorithmic bytes / its measured HIP-event time, against 8 TB/s) and the CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# the row kernel that makes up a timed phase (names as rocprofv3 lists them)
KERNEL_OF_PHASE = {"wside": "wown_kernel", "uside": "useg_multi_kernel / useg_kernel", "dot": "dots_kernel",
                   "apply": "wown_kernel (input side)"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class PairStream:
    """Feeds minibatches of n pairs cut from the pair stream of a token corpus (device side).  Pairs
    are formed block by block into one pair of buffers sized for the whole run and never moved, so
    that the minibatch after the current one can be announced to the shard ahead of time.  Pair
    formation runs on a stream of its own (it keeps its own scratch in the shard), so a block is
    formed while the training calls queued before it are still running; the call returns the pair
    count, i.e. waits for that stream only."""

    def __init__(self, shard, wl, tokens, sent_off, block_tokens, torch, minibatches, own_stream=True):
        self.torch = torch
        self.sh, self.wl = shard, wl
        self.tok = torch.from_numpy(tokens.view(np.int32)).cuda()
        self.off_host = sent_off.astype(np.int64)
        self.off_dev = torch.from_numpy(self.off_host).cuda()
        self.side = torch.cuda.Stream() if own_stream else torch.cuda.current_stream()
        self.block_tokens = block_tokens
        cap = (minibatches + 2) * wl.n_pairs + block_tokens * 2 * wl.window
        self.a = torch.empty(cap, dtype=torch.int32, device="cuda")
        self.b = torch.empty(cap, dtype=torch.int32, device="cuda")
        self.have = 0           # pairs formed so far
        self.pos = 0            # pairs handed out
        self.sent = 0           # next sentence
        self.epoch = 0
        self.tokens_used = 0

    def _more(self):
        torch = self.torch
        off = self.off_host
        if self.sent >= off.size - 1:
            self.sent, self.epoch = 0, self.epoch + 1
        s0 = self.sent
        t0 = int(off[s0])
        s1 = int(np.searchsorted(off, t0 + self.block_tokens, side="right")) - 1
        s1 = max(s1, s0 + 1)
        s1 = min(s1, off.size - 1)
        t1 = int(off[s1])
        with torch.cuda.stream(self.side):
            rel = self.off_dev[s0:s1 + 1] - t0
            cnt = self.sh.make_pairs(self.tok[t0:t1], rel, t0, self.epoch, self.wl.seed,
                                     self.wl.window, self.a[self.have:], self.b[self.have:])
        assert cnt <= self.a.numel() - self.have, "pair buffers too small for this run"
        self.have += cnt
        self.sent = s1
        self.tokens_used += t1 - t0

    def next(self):
        """The current minibatch; the one after it is formed as well (see peek)."""
        n = self.wl.n_pairs
        while self.have - self.pos < 3 * n:
            self._more()
        a = self.a[self.pos:self.pos + n]
        b = self.b[self.pos:self.pos + n]
        self.pos += n
        return a, b

    def peek(self, ahead=0):
        """The minibatch the following next() will return (same device addresses); ahead = 1: the
        one after that."""
        n = self.wl.n_pairs
        lo = self.pos + ahead * n
        return self.a[lo:lo + n], self.b[lo:lo + n]


def host_cpu():
    """CPU model, sockets and cores of the box the oracle is timed on (from /proc/cpuinfo)."""
    model, phys, cores_per, logical = "unknown", set(), {}, 0
    try:
        cur = None
        for line in open("/proc/cpuinfo"):
            key, _, val = line.partition(":")
            key, val = key.strip(), val.strip()
            if key == "processor":
                logical += 1
            elif key == "model name":
                model = val
            elif key == "physical id":
                cur = val
                phys.add(val)
            elif key == "cpu cores" and cur is not None:
                cores_per[cur] = int(val)
    except OSError:
        pass
    sockets = max(1, len(phys))
    cores = sum(cores_per.values()) if cores_per else logical
    return {"model": model, "sockets": sockets, "cores_total": cores, "logical_cpus": logical,
            "visible_to_process": len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else logical}


def step_time_stats(torch, events):
    """Median, minimum and mean of the per-step times between consecutive events (ms)."""
    ms = [events[i].elapsed_time(events[i + 1]) for i in range(len(events) - 1)]
    return {"ms_per_step_median": float(np.median(ms)), "ms_per_step_min": float(np.min(ms)),
            "ms_per_step_mean_events": float(np.mean(ms))}


def cpu_baseline_full(wl, counts, in_idx, out_idx, seed, sample_pairs):
    import oracle
    th, al = oracle.build_alias(counts)
    lazy = oracle.LazyShard(wl.V, wl.d_total, wl.col_begin, wl.d_slice, wl.seed, wl.w_uniform)
    m = min(sample_pairs, in_idx.size)
    t0 = time.perf_counter()
    lazy.train_minibatch(in_idx[:m], out_idx[:m], wl.k, seed, th, al, wl.alpha)
    dt = time.perf_counter() - t0
    lazy.close()
    return {"value": m / dt, "unit": "pairs/s", "cores": 1, "kind": "oracle", "host": host_cpu(),
            "sample": "first %d pairs of minibatch 0 of workload %s, oracle train_minibatch on "
                      "lazily initialised rows, %.1f s" % (m, wl.name, dt)}


def cpu_baseline_slice(wl, counts, in_idx, out_idx, coeffs, seed, sample_pairs):
    import oracle
    th, al = oracle.build_alias(counts)
    m = min(sample_pairs, in_idx.size)
    ii, oo = in_idx[:m], out_idx[:m]
    neg = oracle.negatives(oo, wl.k, seed, th, al)
    rows = np.concatenate([oo[:, None], neg], axis=1)
    words, inv = np.unique(np.concatenate([ii, rows.ravel()]), return_inverse=True)
    U = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 0, words.astype(np.uint32))
    W = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 1, words.astype(np.uint32))
    ci = inv[:m].astype(np.uint32)
    cr = inv[m:].reshape(rows.shape).astype(np.uint32)
    t0 = time.perf_counter()
    oracle.negatives(oo, wl.k, seed, th, al)
    oracle.dots(U, W, ci, cr)
    oracle.negatives(oo, wl.k, seed, th, al)
    oracle.adjust_rows(U, W, ci, cr, coeffs[:m], wl.alpha)
    dt = time.perf_counter() - t0
    return {"value": m / dt, "unit": "pairs/s", "cores": 1, "kind": "oracle", "host": host_cpu(),
            "sample": "first %d pairs of the minibatch of workload %s, oracle dotprod + adjust on "
                      "the touched rows, %.1f s" % (m, wl.name, dt)}


def copy_probe(torch, mb):
    """One plain device copy of mb MiB (calibrates the HBM traffic counters of a profiler run)."""
    if not mb:
        return
    src = torch.ones(mb << 18, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)              # one copy kernel: reads and writes mb MiB
    torch.cuda.synchronize()
    del src, dst


class ExampleStream:
    """Feeds minibatches of n bag-of-words examples formed from a token corpus (device side).  A
    token block gives a run of examples; whole minibatches are cut from it and the block's last,
    incomplete minibatch is dropped (its formation cost still counts).  Blocks alternate between
    two sets of buffers and are formed on a stream of their own, beside the training calls queued
    before; a set is refilled only after the training calls that read it have finished (event).
    Minibatches are cut ahead of their use (cut_ahead, after a training call has been queued): the
    next one can then be announced to the shard, and a block is formed -- a call that waits for the
    example count -- while the device still has that training call to run."""

    def __init__(self, shard, wl, tokens, sent_off, block_tokens, n, torch):
        self.torch, self.sh, self.wl, self.n = torch, shard, wl, n
        self.tok = torch.from_numpy(tokens.view(np.int32)).cuda()
        self.off_host = sent_off.astype(np.int64)
        self.off_dev = torch.from_numpy(self.off_host).cuda()
        self.block_tokens = block_tokens
        self.sets = [(torch.empty(block_tokens + 64, dtype=torch.int32, device="cuda"),
                      torch.empty((block_tokens + 63) * 2 * wl.window, dtype=torch.int32, device="cuda"),
                      torch.empty(block_tokens + 63, dtype=torch.int32, device="cuda")) for _ in range(2)]
        self.done = [None, None]        # event after the last training call queued on set i
        self.which = 1
        self.queue = []                 # minibatches cut ahead: (set, arrays), oldest first
        self.current_set = None
        self.side = torch.cuda.Stream()
        self.have = self.pos = self.sent = self.epoch = 0
        self.tokens_used = 0

    def _refill(self):
        torch, off = self.torch, self.off_host
        if self.sent >= off.size - 1:
            self.sent, self.epoch = 0, self.epoch + 1
        s0 = self.sent
        t0 = int(off[s0])
        s1 = int(np.searchsorted(off, t0 + self.block_tokens, side="right")) - 1
        s1 = min(max(s1, s0 + 1), off.size - 1)
        t1 = int(off[s1])
        self.which ^= 1
        self.co, self.cx, self.ce = self.sets[self.which]
        with torch.cuda.stream(self.side):
            if self.done[self.which] is not None:
                self.side.wait_event(self.done[self.which])
            rel = self.off_dev[s0:s1 + 1] - t0
            n_ex, n_ctx = self.sh.make_cbow_examples(self.tok[t0:t1], rel, t0, self.epoch, self.wl.seed,
                                                     self.wl.window, self.co, self.cx, self.ce)
            assert n_ex <= self.ce.numel() and n_ctx <= self.cx.numel()
            self.co_host = self.co[:n_ex + 1].cpu().numpy()  # offsets, to slice the context words
        self.have, self.pos, self.sent = n_ex, 0, s1
        self.tokens_used += t1 - t0

    def _cut(self):
        while self.have - self.pos < self.n:
            self._refill()
        a, b = self.pos, self.pos + self.n
        self.pos = b
        lo, hi = int(self.co_host[a]), int(self.co_host[b])
        return self.which, ((self.co[a:b + 1] - lo), self.cx[lo:hi], self.ce[a:b])

    def next(self):
        """The current minibatch (the arrays peek() returned before, if it was called)."""
        if not self.queue:
            self.queue.append(self._cut())
        self.current_set, arrays = self.queue.pop(0)
        return arrays

    def peek(self):
        """The minibatch the following next() will return (same device arrays)."""
        if not self.queue:
            self.queue.append(self._cut())
        return self.queue[0][1]

    def cut_ahead(self):
        """Call after consumed(): cuts the minibatches of the next two steps, forming a block if
        they need one (the set it goes to was last read by training calls queued before)."""
        while len(self.queue) < 2:
            self.queue.append(self._cut())

    def consumed(self):
        """Call after the training call on the current minibatch has been queued."""
        ev = self.torch.cuda.Event()
        ev.record(self.torch.cuda.current_stream())
        self.done[self.current_set] = ev


def run_cbow(args, torch, w2v, workloads):
    """Bag-of-words variant on the full300 shape: make_cbow_examples + cbow_train_minibatch."""
    wl = workloads.WORKLOADS[args.workload]
    if not wl.pairs_from_corpus or wl.name == "tiny":
        print("bench.py: --variant cbow runs on a text workload (full300, search200m, stress25)",
              file=sys.stderr)
        sys.exit(2)
    K, Wm = args.steps, args.warmup
    n = args.cbow_examples
    R, T = 4 * wl.d_slice, wl.k + 1
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin,
                   init_mode=1 if wl.w_uniform else 0)
    sh.set_counts(counts, wl.subsample_t)
    copy_probe(torch, args.copy_probe_mb)
    tokens, off = workloads.corpus(wl, args.corpus_tokens or 12_000_000, cdf=cdf)
    del cdf
    stream = ExampleStream(sh, wl, tokens, off, min(tokens.size, 1 << 21), n, torch)
    loss = None if args.no_loss else torch.zeros(1, dtype=torch.float64, device="cuda")
    H = max(1, wl.corpus_tokens // (2 * n))

    def step(h):
        co, cx, ce = stream.next()
        if not args.no_prefetch:                           # the next minibatch's index work, ahead
            sh.cbow_prefetch_minibatch(*stream.peek(), wl.k, w2v.minibatch_seed(wl.seed, h + 1))
        w2v.cbow_train_minibatch([sh], co, cx, ce, wl.k, w2v.minibatch_seed(wl.seed, h),
                                 workloads.alpha_schedule(wl, h, H), loss=loss)
        stream.consumed()
        stream.cut_ahead()
        return co, cx, ce

    first = None
    for h in range(max(Wm, 1)):
        e = step(h)
        if first is None:
            first = tuple(w2v.index_to_numpy(x).copy() for x in e)
    Wm = max(Wm, 1)
    sh.status()
    # A bag-of-words step is about a millisecond and the host needs nearly as long to queue it, so
    # the two event records per phase of the library's timing spans would cost the step 5 %: the K
    # timed steps run without them, and the phase times come from a second run of up to 20 steps
    # right after, with the spans on.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx_total = 0
    for h in range(Wm, Wm + K):
        last = step(h)
        ctx_total += last[1].numel()
    t_queued = time.perf_counter() - t0          # the host's share: all K steps are queued by now
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    K2 = min(K, 20)
    sh.timing_enable(True)
    sh.timing_read()
    t2 = time.perf_counter()
    for h in range(Wm + K, Wm + K + K2):
        last = step(h)
    torch.cuda.synchronize()
    dt_spans = time.perf_counter() - t2
    phases = sh.timing_read()
    sh.timing_enable(False)
    sh.status()
    m = ctx_total / K
    neg = sh.negatives(last[2], wl.k, w2v.minibatch_seed(wl.seed, Wm + K - 1))
    du = int(torch.unique(last[1]).numel())
    _, c = torch.unique(torch.cat([last[2], neg.reshape(-1)]), return_counts=True)
    dw, single = int(c.numel()), int((c == 1).sum().item())    # single: output rows named by one slot
    if os.environ.get("W2V_NO_OWN_ROWS", "0") not in ("", "0"):
        single = 0
    M = n * T
    # algorithmic bytes per launch (= per minibatch):
    #   dot   (hidden vectors)      : m input rows read + n rows written + 4 B per entry
    #   uside (per-example pass)    : T output rows + the hidden row per example, one row written,
    #                                 + one row written per output row that a single slot names
    #   wside (output-side update)  : one hidden row per contribution + 12 B + RMW of distinct rows
    #                                 (without the slots and rows the per-example pass has taken over)
    #   apply (input-side update)   : one summed row per context entry + 12 B + RMW of distinct rows
    algo = {
        "dot": (m + n) * R + 4 * m,
        "uside": n * (T + 2) * R + 8 * M + single * R,
        "wside": (M - single) * R + 12 * M + 2 * (dw - single) * R,
        "apply": m * R + 12 * m + 2 * du * R,
    }
    per_phase = {name: {"ms_per_launch": ms / cnt, "launches": cnt}
                 for name, (ms, cnt) in phases.items() if cnt}
    dom = max((p for p in per_phase if p in algo),
              key=lambda p: per_phase[p]["ms_per_launch"] * per_phase[p]["launches"])
    launches_per_step = per_phase[dom]["launches"] / K2
    dom_ms = per_phase[dom]["ms_per_launch"] * launches_per_step      # per minibatch
    achieved = algo[dom] / (dom_ms * 1e-3) / 1e9
    traffic = None          # L2<->fabric bytes per launch, from the committed rocprofv3 counter summary
    tfile = os.path.join(ROOT, "profiles", "%s_cbow_hbm_traffic.txt" % wl.name)
    if os.path.exists(tfile):
        for line in open(tfile):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic" and parts[1] == dom:
                traffic = float(parts[2])
    out = {
        "metric": "CBOW training examples/s (k negatives incl.) on 1 MI355X",
        "value": n * K / dt, "unit": "examples/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": dt * 1e3 / K, "host_queue_ms_per_step": t_queued * 1e3 / K,
        "ms_per_step_with_phase_spans": dt_spans * 1e3 / K2, "steps_with_phase_spans": K2,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name + "/cbow", "V": wl.V, "d_slice": wl.d_slice,
                   "examples_per_minibatch": n, "context_words_per_minibatch": m, "k": wl.k,
                   "zipf_s": wl.zipf_s, "window": wl.window, "subsample_t": wl.subsample_t,
                   "path": "make_cbow_examples+cbow_train_minibatch",
                   "distinct_input_rows": du, "distinct_output_rows": dw,
                   "output_rows_named_once": single, "prefetch": not args.no_prefetch},
        "context_words_per_s": ctx_total / dt,
        "roofline": {"bound": "hbm", "kernel": "cbow_hidden_kernel" if dom == "dot" else
                     KERNEL_OF_PHASE.get(dom, dom), "phase": dom, "achieved": achieved,
                     "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": algo[dom], "ms_per_launch": dom_ms},
        "phases": per_phase,
        "tokens_per_minibatch": stream.tokens_used / (K + Wm),
    }
    if not args.no_cpu_baseline:
        import oracle
        th, al = oracle.build_alias(counts)
        co, cx, ce = first
        e = min(args.cpu_sample_pairs or (1 << 17), ce.size)
        co, cx, ce = co[:e + 1], cx[:int(co[e])], ce[:e]
        seed0 = w2v.minibatch_seed(wl.seed, 0)
        rows = np.concatenate([ce[:, None], oracle.negatives(ce, wl.k, seed0, th, al)], axis=1)
        words, inv = np.unique(np.concatenate([cx, rows.ravel()]), return_inverse=True)
        U = oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 0, words.astype(np.uint32))
        W = (oracle.init_rows(wl.seed, wl.d_total, wl.col_begin, wl.d_slice, 1, words.astype(np.uint32))
             if wl.w_uniform else np.zeros_like(U))
        cc = inv[:cx.size].astype(np.uint32)
        cr = inv[cx.size:].reshape(rows.shape).astype(np.uint32)
        t0 = time.perf_counter()
        oracle.negatives(ce, wl.k, seed0, th, al)
        g = oracle.coeffs([oracle.cbow_dots(U, W, co, cc, cr)])
        oracle.negatives(ce, wl.k, seed0, th, al)
        oracle.cbow_adjust_rows(U, W, co, cc, cr, g, wl.alpha)
        dtc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": e / dtc, "unit": "examples/s", "cores": 1, "kind": "oracle",
                               "host": host_cpu(),
                               "sample": "first %d examples of minibatch 0, oracle cbow dots + "
                                         "coefficients + adjust on the touched rows, %.1f s" % (e, dtc)}
    sh.destroy()
    print(json.dumps(out), flush=True)


def run_topk(args, torch, w2v, workloads):
    """Retrieval: the K most similar of N candidate vectors for each of Q queries (w2v_topk_cosine).
    One step = one whole search.  The contraction runs on the fp32 matrix cores, so the roofline is
    the dense fp32 MFMA peak; flops counted: 2 Q N d."""
    Q, N, d, K = args.topk_queries, args.topk_candidates, 300, args.topk_k
    steps, Wm = args.steps, max(args.warmup, 1)
    t0 = time.perf_counter()
    C = workloads.embedding_like(N, d, 7)
    Qm = workloads.embedding_like(Q, d, 8)
    log("setup: %d x %d candidates, %d queries generated in %.1f s" % (N, d, Q, time.perf_counter() - t0))
    cd, qd = torch.from_numpy(C).cuda(), torch.from_numpy(Qm).cuda()
    need = int(w2v.lib().w2v_topk_cosine_workspace(Q, N, args.topk_round))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    copy_probe(torch, args.copy_probe_mb)
    for _ in range(Wm):
        out = w2v.topk_cosine(qd, cd, K, -2.0, workspace=ws)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        out = w2v.topk_cosine(qd, cd, K, -2.0, workspace=ws)
        ev[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    flops = 2.0 * Q * N * d
    achieved = flops / (np.mean(ms) * 1e-3) / 1e12
    res = {
        "metric": "top-K cosine retrieval, queries/s on 1 MI355X", "value": Q * steps / dt,
        "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": Wm, "ms_per_step": dt * 1e3 / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "topk_cosine", "Q": Q, "N": N, "d": d, "K": K, "tau": None,
                   "round_candidates": args.topk_round, "workspace_bytes": need},
        "roofline": {"bound": "mfma", "kernel": "topk_scores_kernel (+ selection, whole call)",
                     "achieved": achieved, "peak": 157.3, "unit": "TFLOP/s", "frac": achieved / 157.3,
                     "traffic": None, "algorithmic_flops_per_launch": flops,
                     "ms_per_launch": float(np.mean(ms))},
    }
    if not args.no_cpu_baseline:
        import oracle
        m = min(Q, args.cpu_sample_pairs or 48)
        t0 = time.perf_counter()
        oi, osc, oc = oracle.topk_cosine(Qm[:m], C, K)
        dtc = time.perf_counter() - t0
        gi = w2v.index_to_numpy(out[0][:m])
        res["cpu_baseline"] = {"value": m / dtc, "unit": "queries/s", "cores": 1, "kind": "oracle",
                               "host": host_cpu(),
                               "sample": "first %d queries against all %d candidates, %.1f s; %d of %d "
                                         "indices equal the GPU's" % (m, N, dtc, int((gi == oi).sum()), m * K)}
    print(json.dumps(res), flush=True)


def run_gather_probe(args, torch, w2v, workloads):
    """What random row gathers reach on this part: w2v_dotprod alone on the chosen workload's shard
    with uniformly random input and output words (no frequent words, so no cache help beyond what
    the row size gives): (k+2) row reads per pair and 4(k+1) bytes written.  A measured ceiling for
    the access pattern of the training kernels, next to the 8 TB/s data-sheet figure."""
    wl = workloads.WORKLOADS[args.workload]
    n, k, R = wl.n_pairs, wl.k, 4 * wl.d_slice
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin, init_mode=1)
    sh.set_counts(np.ones(wl.V, np.uint64), 0.0)          # uniform noise distribution
    g = torch.Generator(device="cuda").manual_seed(5)
    a = torch.randint(0, wl.V, (n,), generator=g, device="cuda", dtype=torch.int32)
    b = torch.randint(0, wl.V, (n,), generator=g, device="cuda", dtype=torch.int32)
    dots = torch.empty((n, k + 1), dtype=torch.float32, device="cuda")
    for h in range(max(args.warmup, 1)):
        sh.dotprod(a, b, k, h, out=dots)
    sh.timing_enable(True)
    sh.timing_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for h in range(args.steps):
        sh.dotprod(a, b, k, 100 + h, out=dots)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms, cnt = sh.timing_read()["dot"]
    sh.status()
    sh.destroy()
    algo = n * (k + 2) * R + 8 * n * (k + 1)
    achieved = algo / (ms / cnt * 1e-3) / 1e9
    print(json.dumps({
        "metric": "random row gather (dots_kernel alone, uniform words) on 1 MI355X",
        "value": achieved, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 1),
        "ms_per_step": dt * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name + "/gather-probe", "V": wl.V, "d_slice": wl.d_slice,
                   "row_bytes": R, "pairs": n, "k": k},
        "roofline": {"bound": "hbm", "kernel": "dots_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": algo, "ms_per_launch": ms / cnt}}), flush=True)


def distinct_rows(torch, shard, in_idx, out_idx, k, seed):
    """Distinct input rows, distinct output/negative rows, and output rows named by one slot only,
    of one minibatch (for byte counts)."""
    neg = shard.negatives(out_idx, k, seed)
    du = int(torch.unique(in_idx).numel())
    _, c = torch.unique(torch.cat([out_idx, neg.reshape(-1)]), return_counts=True)
    return du, int(c.numel()), int((c == 1).sum().item())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 1500 for the skip-gram run on full300 or slice60, a few "
                         "seconds of device time; 20 otherwise)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before (default 20 / 5)")
    ap.add_argument("--workload", default="full300",
                    choices=["full300", "slice60", "tiny", "search200m", "stress25"])
    ap.add_argument("--variant", default="sgns", choices=["sgns", "cbow", "topk", "gather"],
                    help="cbow: the bag-of-words variant on the same text workload; "
                         "topk: cosine retrieval over exported vectors; gather: the rate plain "
                         "random row gathers reach (dotprod alone, uniform words)")
    ap.add_argument("--topk-queries", type=int, default=4096)
    ap.add_argument("--topk-candidates", type=int, default=1 << 20)
    ap.add_argument("--topk-k", type=int, default=30)
    ap.add_argument("--topk-round", type=int, default=32768, help="candidates per round")
    ap.add_argument("--cbow-examples", type=int, default=1 << 17, help="examples per cbow minibatch")
    ap.add_argument("--corpus-tokens", type=int, default=0, help="tokens of the corpus slice to generate")
    ap.add_argument("--cpu-sample-pairs", type=int, default=0,
                    help="pairs the CPU oracle is timed on (default: about 10-30 s of one core)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-loss", action="store_true", help="do not request the minibatch loss")
    ap.add_argument("--pairs-on-main-stream", action="store_true",
                    help="form the pairs on the training stream instead of a stream of their own")
    ap.add_argument("--no-prefetch", action="store_true",
                    help="do not announce the next minibatch to the shard (w2v_prefetch_minibatch)")
    ap.add_argument("--graph", action="store_true",
                    help="text workloads: run every step as a replay of one captured step "
                         "(w2v_step_graph), the form meant for small minibatches")
    ap.add_argument("--pairs-per-minibatch", type=int, default=0,
                    help="override the workload's minibatch size (pairs)")
    ap.add_argument("--prefetch-depth", type=int, default=1, choices=[1, 2],
                    help="text workloads: announce minibatch h+1 before step h (1) or minibatch h+2 "
                         "after step h (2)")
    ap.add_argument("--copy-probe-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibrates HBM counters)")
    args = ap.parse_args()
    # The default run lasts a few seconds on the device (long enough for an outside observer's
    # utilisation sampler to see it); step time is the same over 20, 300 or 1500 steps.
    long_run = args.variant == "sgns" and args.workload in ("full300", "slice60") and not args.graph
    if args.steps is None:
        args.steps = 1500 if long_run else 20
    if args.warmup is None:
        args.warmup = 20 if long_run else 5
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (a shard is one GPU's column slice); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1606_08495_amd import w2v, workloads

    if not os.path.exists(w2v.LIB_PATH):
        from paper_1606_08495_amd import build as hip_build
        hip_build.build()
    torch.cuda.set_device(0)
    if args.variant == "cbow":
        return run_cbow(args, torch, w2v, workloads)
    if args.variant == "topk":
        return run_topk(args, torch, w2v, workloads)
    if args.variant == "gather":
        return run_gather_probe(args, torch, w2v, workloads)
    wl = workloads.WORKLOADS[args.workload]
    if args.pairs_per_minibatch:
        import dataclasses
        wl = dataclasses.replace(wl, n_pairs=args.pairs_per_minibatch)
    K, Wm = args.steps, args.warmup
    if not args.cpu_sample_pairs:
        args.cpu_sample_pairs = {"full300": 1 << 20, "slice60": 1 << 20, "tiny": 1 << 16,
                                 "search200m": 1 << 19, "stress25": 1 << 17}[wl.name]
    R = 4 * wl.d_slice
    T = wl.k + 1

    t_setup = time.perf_counter()
    cdf = workloads.zipf_cdf(wl.V, wl.zipf_s)
    if wl.name == "tiny":
        tokens, off = workloads.corpus(wl, cdf=cdf)
        counts = workloads.counted(tokens, wl.V)
    else:
        counts = workloads.analytic_counts(wl.V, wl.zipf_s, wl.corpus_tokens)
    sh = w2v.Shard(wl.V, wl.d_slice, wl.seed, d_total=wl.d_total, col_begin=wl.col_begin,
                   init_mode=1 if wl.w_uniform else 0)
    sh.set_counts(counts, wl.subsample_t)
    log("setup: shard V=%d d_slice=%d (%.1f GB of vectors) ready in %.1f s"
        % (wl.V, wl.d_slice, 2.0 * wl.V * R / 1e9, time.perf_counter() - t_setup))

    copy_probe(torch, args.copy_probe_mb)

    loss = None if args.no_loss else torch.zeros(1, dtype=torch.float64, device="cuda")
    total_steps = K + Wm
    result_extra = {}

    if wl.pairs_from_corpus:
        # ---- end-to-end: make_pairs + train_minibatch ------------------------------------------
        if wl.name != "tiny":
            # tokens the timed run will consume, with a margin (pairs per token differ by workload)
            n_tok = args.corpus_tokens or {"full300": 12_000_000, "search200m": 700_000 * (K + Wm + 2),
                                           "stress25": 700_000 * (K + Wm + 2)}[wl.name]
            tokens, off = workloads.corpus(wl, n_tok, cdf=cdf)
        del cdf
        stream = PairStream(sh, wl, tokens, off, block_tokens=min(tokens.size, 1 << 21), torch=torch,
                            minibatches=total_steps + 2, own_stream=not args.pairs_on_main_stream)
        H = max(1, wl.corpus_tokens * 4 // wl.n_pairs)     # minibatches in the nominal corpus

        step_graph = w2v.StepGraph(sh, wl.n_pairs, wl.k, loss=loss) if args.graph else None

        def step(h):
            a, b = stream.next()
            if step_graph is not None:          # one captured step, replayed (small minibatches)
                step_graph.run(a, b, w2v.minibatch_seed(wl.seed, h), workloads.alpha_schedule(wl, h, H))
                return a, b
            if args.prefetch_depth == 2:
                # two ahead: minibatch h+2 is announced before step h is queued, so its index work
                # starts beside step h and has until step h+2 to finish
                if h == 0:
                    sh.prefetch_minibatch(*stream.peek(), wl.k, w2v.minibatch_seed(wl.seed, 1))
                sh.prefetch_minibatch(*stream.peek(1), wl.k, w2v.minibatch_seed(wl.seed, h + 2))
                w2v.train_minibatch([sh], a, b, wl.k, w2v.minibatch_seed(wl.seed, h),
                                    workloads.alpha_schedule(wl, h, H), loss=loss)
                return a, b
            if not args.no_prefetch:                       # the next minibatch's index work, ahead
                na, nb = stream.peek()
                sh.prefetch_minibatch(na, nb, wl.k, w2v.minibatch_seed(wl.seed, h + 1))
            w2v.train_minibatch([sh], a, b, wl.k, w2v.minibatch_seed(wl.seed, h),
                                workloads.alpha_schedule(wl, h, H), loss=loss)
            return a, b

        first = None
        for h in range(Wm):
            ab = step(h)
            if first is None:
                first = (w2v.index_to_numpy(ab[0]).copy(), w2v.index_to_numpy(ab[1]).copy())
        if first is None:
            a0, b0 = stream.next()
            first = (w2v.index_to_numpy(a0).copy(), w2v.index_to_numpy(b0).copy())
            stream.pos -= wl.n_pairs
        sh.status()
        sh.timing_enable(True)
        sh.timing_read()
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        t0 = time.perf_counter()
        marks[0].record()
        last = None
        for h in range(Wm, total_steps):
            last = step(h)
            marks[h - Wm + 1].record()      # every stream of the step has joined the caller's by now
        result_extra["host_queue_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / K
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        result_extra.update(step_time_stats(torch, marks))
        phases = sh.timing_read()
        sh.timing_enable(False)
        sh.status()
        du, dw, single = distinct_rows(torch, sh, last[0], last[1], wl.k,
                                       w2v.minibatch_seed(wl.seed, total_steps - 1))
        if os.environ.get("W2V_NO_OWN_ROWS", "0") not in ("", "0"):
            single = 0
        result_extra["tokens_per_minibatch"] = stream.tokens_used / max(1, total_steps)
        if not args.no_cpu_baseline:
            cpu = cpu_baseline_full(wl, counts, first[0], first[1], w2v.minibatch_seed(wl.seed, 0),
                                    args.cpu_sample_pairs)
    else:
        # ---- two-call form on one column slice: dotprod + adjust with harness coefficients --------
        ii, oo = workloads.iid_pairs(wl, cdf=cdf)
        del cdf
        g = workloads.uniform_coeffs(wl.n_pairs, T, wl.seed)
        a, b = w2v.as_index_tensor(ii), w2v.as_index_tensor(oo)
        gd = torch.from_numpy(g).cuda()
        dots = torch.empty((wl.n_pairs, T), dtype=torch.float32, device="cuda")

        def step(h):
            seed = w2v.minibatch_seed(wl.seed, h)
            if not args.no_prefetch:          # the next minibatch's index work, beside this one's rows
                if args.prefetch_depth == 2:  # ... or that of the one after it as well
                    if h == 0:
                        sh.prefetch_minibatch(a, b, wl.k, w2v.minibatch_seed(wl.seed, 1))
                    sh.prefetch_minibatch(a, b, wl.k, w2v.minibatch_seed(wl.seed, h + 2))
                else:
                    sh.prefetch_minibatch(a, b, wl.k, w2v.minibatch_seed(wl.seed, h + 1))
            sh.dotprod(a, b, wl.k, seed, out=dots)
            sh.adjust(a, b, wl.k, seed, gd, wl.alpha)

        if not args.no_prefetch:
            sh.prefetch_minibatch(a, b, wl.k, w2v.minibatch_seed(wl.seed, 0))

        for h in range(Wm):
            step(h)
        sh.status()
        sh.timing_enable(True)
        sh.timing_read()
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        t0 = time.perf_counter()
        marks[0].record()
        for h in range(Wm, total_steps):
            step(h)
            marks[h - Wm + 1].record()
        result_extra["host_queue_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / K
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        result_extra.update(step_time_stats(torch, marks))
        phases = sh.timing_read()
        sh.timing_enable(False)
        sh.status()
        du, dw, _ = distinct_rows(torch, sh, a, b, wl.k, w2v.minibatch_seed(wl.seed, total_steps - 1))
        single = 0                      # the two-call form sums every output row on the output side
        if not args.no_cpu_baseline:
            cpu = cpu_baseline_slice(wl, counts, ii, oo, g, w2v.minibatch_seed(wl.seed, 0),
                                     args.cpu_sample_pairs)

    n = wl.n_pairs
    M = n * T
    ms_per_step = dt * 1e3 / K
    pairs_per_s = n * K / dt

    # ---- algorithmic bytes of each gather/scatter phase, per launch (= per minibatch) -------------
    #   dot      : (k+2) rows per pair + keys + dots written
    #   uside    : T output rows per pair (+ the input row when fused) + keys/coefficients/sort data
    #              + one delta row written per distinct input row
    #              + (fused) one row written per output row that a single slot names
    #   wside    : one input row per contribution + 12 B of key/slot/coefficient
    #              + one read and one write of every distinct destination row
    #              (fused: without the slots and rows that the input side has taken over)
    fused = wl.pairs_from_corpus
    algo = {
        "dot": n * (wl.k + 2) * R + 8 * M,
        "uside": n * (T + (1 if fused else 0)) * R + 8 * M + 8 * n + du * R + single * R,
        "wside": (M - single) * R + 12 * M + 2 * (dw - single) * R,
    }
    # ---- compulsory bytes: what a launch would move if every DISTINCT row crossed the memory
    # interface once per direction (no re-read of a row named several times is counted; index and
    # coefficient arrays are streamed once either way).  A lower bound on the HBM traffic of the
    # launch; the logical figure above is what the kernel asks of the memory system, caches included.
    #   dot   : the distinct input and output rows, read
    #   uside : the distinct output rows (+ the distinct input rows when fused), read; one delta row
    #           per distinct input row and the rows named once, written
    #   wside : the distinct input rows, read; every other distinct output row read and written
    compulsory = {
        "dot": (du + dw) * R + 8 * M,
        "uside": (dw + (du if fused else 0)) * R + (du + single) * R + 8 * M + 8 * n,
        "wside": du * R + 2 * (dw - single) * R + 12 * M,
    }
    per_phase = {}
    for name, (ms, cnt) in phases.items():
        if cnt:
            per_phase[name] = {"ms_per_launch": ms / cnt, "launches": cnt}
    timed = [p for p in per_phase if p in algo]
    if timed:
        dom = max(timed, key=lambda p: per_phase[p]["ms_per_launch"] * per_phase[p]["launches"])
        dom_ms = per_phase[dom]["ms_per_launch"]
    else:
        # a captured step records no per-phase events: the roofline entry is the whole step's, its
        # bytes the sum over the row kernels
        dom, dom_ms = "step", ms_per_step
        algo["step"] = algo["uside"] + algo["wside"] + (0 if fused else algo["dot"])
        compulsory["step"] = 2 * (du + dw) * R + 8 * n
    achieved = algo[dom] / (dom_ms * 1e-3) / 1e9
    compulsory_gbs = compulsory[dom] / (dom_ms * 1e-3) / 1e9
    # L2<->fabric bytes per launch: NOT measured in this run -- read from the committed rocprofv3
    # counter summary of the same command (counters and timing cannot share a run)
    traffic, traffic_source = None, None
    tfile = os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % wl.name)
    if os.path.exists(tfile):
        for line in open(tfile):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic" and parts[1] == dom:
                traffic = float(parts[2])
                traffic_source = "profiles/%s_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE " \
                                 "of this command in a run of its own; L2<->fabric, an upper bound on " \
                                 "HBM bytes)" % wl.name
    step_algo = 3 * (wl.k + 2) * R * n      # the paper-style logical figure: 3 (k+2) rows per pair
    # the whole step at its least: every distinct row of either matrix read once and written once
    step_compulsory = 2 * (du + dw) * R + 8 * n + (4 * M if not fused else 0)
    out = {
        "metric": "SGNS training pairs/s (k negatives incl.) on 1 MI355X",
        "value": pairs_per_s,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "V": wl.V, "d_slice": wl.d_slice, "d_total": wl.d_total,
                   "pairs_per_minibatch": n, "k": wl.k, "zipf_s": wl.zipf_s, "window": wl.window,
                   "subsample_t": wl.subsample_t,
                   "path": "make_pairs+train_minibatch" if fused else "dotprod+adjust",
                   "distinct_input_rows": du, "distinct_output_rows": dw,
                   "output_rows_named_once": single,
                   "prefetch": not args.no_prefetch and not args.graph, "captured_step": bool(args.graph)},
        "roofline": {"bound": "hbm", "kernel": KERNEL_OF_PHASE.get(dom, dom), "phase": dom,
                     "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": algo[dom], "ms_per_launch": dom_ms,
                     "compulsory_bytes_per_launch": compulsory[dom],
                     "compulsory_GBps": compulsory_gbs,
                     "compulsory_frac": compulsory_gbs / HBM_PEAK_GBS,
                     "hbm_frac_bracket": [compulsory_gbs / HBM_PEAK_GBS,
                                          (traffic / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS) if traffic
                                          else achieved / HBM_PEAK_GBS]},
        "step_logical_GBps": step_algo / (ms_per_step * 1e-3) / 1e9,
        "step_compulsory_GBps": step_compulsory / (ms_per_step * 1e-3) / 1e9,
        "step_compulsory_frac": step_compulsory / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "phases": per_phase,
    }
    out.update(result_extra)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu
    sh.destroy()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
