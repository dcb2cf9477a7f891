#!/usr/bin/env python3
"""Benchmark of the AASD hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input of the chosen
workload, with all inputs resident in HBM before the timed region starts:
    aasd_align_sample   over all prefill rows,
    aasd_retrieve_drafts over the token buffers of every decode step,
    aasd_verify         over the verify logits of every decode step
(for the single-stream workloads the decode steps are processed as one batch, which is the
throughput form; the sequential per-step latency is reported beside it).
The metric is logit rows per second (prefill rows sampled + verify rows verified); the roofline
block gives the achieved HBM bandwidth of the dominant kernel, the fused row sweep.

The workloads tree_single and tree_batch run the draft-tree form of the same path instead (alignment
sampling, retrieval with the extras, tree build, tree verification over one row per tree node).

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# the oracle leg repeats its sample until it has run this long (a short workload alone gives too short a timing)
CPU_BASELINE_MIN_S = 10.0
CPU_BASELINE_MAX_PASSES = 8


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_single",
                    choices=["tiny", "llama3_single", "long_context", "batched_serving", "stress_tree",
                             "tree_single", "tree_batch"])
    ap.add_argument("--decode-steps", type=int, default=None, help="override the workload's number of decode steps")
    ap.add_argument("--prefill-rows", type=int, default=None, help="cap on prefill rows held in HBM")
    ap.add_argument("--max-nodes", type=int, default=None, help="tree_* workloads: node budget per sequence (default min(256, 1 + C*k*(1+m)))")
    ap.add_argument("--extras-mode", default="top", choices=["top", "sample", "gumbel"],
                    help="how alignment sampling chooses the extras: best-ranked (Fig. 2), seeded draws among the top-c, "
                         "or seeded draws from the whole row (a second, ALU-bound kernel over the misaligned rows)")
    ap.add_argument("--streams", type=int, default=2, choices=[1, 2],
                    help="2 (default): alignment sampling (the prefill rows of new requests) is enqueued on a second HIP stream of the "
                         "same priority and overlaps with retrieval and verification of the running batch, which do not depend on it; "
                         "1: every call on one stream.  Kernel times for the roofline block are always taken on one stream")
    ap.add_argument("--retrieval", default="scan", choices=["scan", "pool"],
                    help="n-gram retrieval by the stateless scan of the token buffer, or through the persistent draft pool "
                         "(built in set-up; the latency loop then does an incremental update and a lookup per step)")
    ap.add_argument("--verifier", default="adaptive", choices=["adaptive", "topk"],
                    help="conditional verification with the entropy-adaptive threshold (Eq. 4-6), or the top-k ablation (Sec. 4.4)")
    ap.add_argument("--topk", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="skip the per_step block (the decode step at its real shape)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "row_sweep_traffic.txt"),
                    help="text file with HBM bytes per launch measured by rocprofv3 --pmc (key = value lines)")
    return ap.parse_args()


_hip = None


def hip_event():
    """A raw hipEvent_t: the library's measurement hook records these around the sweep kernel alone."""
    global _hip
    import ctypes
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
    e = ctypes.c_void_p()
    assert _hip.hipEventCreate(ctypes.byref(e)) == 0
    return e


def hip_elapsed(a, b):
    import ctypes
    ms = ctypes.c_float()
    assert _hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
    return ms.value


def read_traffic(path):
    measured = {}
    if path and os.path.exists(path):
        for line in open(path):
            if "=" in line and not line.lstrip().startswith("#"):
                k_, v_ = line.split("=", 1)
                measured[k_.strip()] = v_.strip()
    return measured


def kernel_source_sha():
    """Hash of the kernel sources: figures copied from a rocprofv3 run under profiles/ carry the hash of the sources
    they were measured on, and are only quoted while it still matches."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_13204_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def check_batch_against_loop(np, name, batch, loop_accept, loop_best, alpha, beta, C, k):
    """The batched pass must reproduce the sequential loop it stands for.  The two run in different launch shapes, so
    their sums are formed in different orders: a decision may differ only where the token that decides it lies within
    1e-6 of its threshold, and not at all where the threshold is the row's maximum probability itself (then passing
    means "the logit equals the row's largest", which no rounding touches).  Returns the report for the JSON line."""
    acc = batch["accept_len"].cpu().numpy()
    best = batch["best_cand"].cpu().numpy()
    tok_p = batch["tok_p"].cpu().numpy().astype(np.float64)
    tok_d = batch["tok_delta"].cpu().numpy().astype(np.float64)
    H = batch["row_entropy"].cpu().numpy().astype(np.float64)
    pmax = batch["row_pmax"].cpu().numpy().astype(np.float64)
    clamp_everywhere = bool((alpha * H + beta > pmax * (1 + 1e-5)).all())
    differ = np.nonzero(acc != loop_accept)[0]
    outside = 0
    for b in differ:
        j = int(min(acc[b], loop_accept[b]))            # the first token on which the two disagree
        close = False
        for c in {int(best[b]), int(loop_best[b])}:
            if j < k and abs(tok_p[b, c, j] - tok_d[b, c, j]) < 1e-6:
                close = True
        outside += 0 if close else 1
    assert outside == 0, f"{name}: {outside} sequences decide differently in the batch and in the loop away from any threshold"
    if clamp_everywhere:
        assert len(differ) == 0, f"{name}: {len(differ)} decisions differ although every threshold is the row maximum"
    near = int(batch["near_count"].cpu().numpy().astype(np.int64).sum())
    return {"sequences": int(len(acc)), "batch_vs_loop_differences": int(len(differ)),
            "differences_outside_1e-6_of_threshold": int(outside), "every_threshold_is_row_max": clamp_everywhere,
            "near_threshold_decisions": near}


def time_steps(torch, fn, n, reps=3):
    """Microseconds per call of fn(i), i = 0..n-1: launched back to back (no host synchronisation inside), and
    replayed from a HIP graph captured once (None if the capture fails)."""
    fn_all = lambda: [fn(i) for i in range(n)]
    fn_all()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn_all()
    e1.record()
    torch.cuda.synchronize()
    eager = e0.elapsed_time(e1) * 1e3 / (reps * n)
    graph_us = None
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn_all()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        graph_us = e0.elapsed_time(e1) * 1e3 / (reps * n)
    except Exception as exc:  # context only: a failed capture must not cost the benchmark line
        print(f"bench.py: HIP graph capture failed ({exc}); not reported", file=sys.stderr)
    return eager, graph_us


def per_step_block(torch, np, aasd, label, logits_steps, tokens, lens, plens, w, note="", use_pool=False):
    """One decode step at its real shape: aasd_retrieve_drafts (or aasd_pool_step) + aasd_verify for the B sequences of a
    step, over per-step logits that rotate through more than the 256 MB Infinity Cache, so every step reads cold HBM.
    logits_steps: list of [B, R, V] tensors; tokens/lens/plens: per step [B, cap], [B], [B]."""
    dev = logits_steps[0].device
    n = len(logits_steps)
    B, R, V = logits_steps[0].shape
    elt = logits_steps[0].element_size()
    dt_code = aasd.BF16 if elt == 2 else aasd.F32
    step_bytes = B * R * V * elt
    ws_bytes = max(128, aasd.verify_workspace_bytes(B, w.C, w.k, V, dt_code))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    ws_zeroed = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)   # only ever passed with AASD_VERIFY_ZEROED_WORKSPACE
    r = aasd.retrieve_drafts(tokens[0], lens[0], plens, w.n_min, w.n_max, w.k, w.C)
    kw = dict(alpha=w.alpha, beta=w.beta, want_rows=False, want_tokens=False, want_near=True)
    v = aasd.verify(logits_steps[0], r["drafts"], r["draft_len"], r["strict"], zeroed_workspace=True, workspace=ws_zeroed, **kw)
    v2 = aasd.verify(logits_steps[0], r["drafts"], r["draft_len"], r["strict"], workspace=ws, **kw)
    # Retrieval both ways: the stateless scan, and the persistent pool: built once over the longest context (timed:
    # the cost at the end of prefill), then rebuilt at the first step's length; aasd_pool_step indexes what a step
    # added and looks up.  The step lengths ascend through the first pass over the buffers (real incremental updates);
    # later passes look up at lengths that are indexed already.
    pool = aasd.DraftPool(B, tokens[0].shape[1], w.n_min, w.n_max, dev)
    pool.update(tokens[n - 1], lens[n - 1], reset=True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        pool.update(tokens[n - 1], lens[n - 1], reset=True)
    e1.record()
    torch.cuda.synchronize()
    pool_build_us = e0.elapsed_time(e1) * 1e3 / 10
    pool.update(tokens[0], lens[0], reset=True)

    def step(i, one_launch=False, with_retrieve=True, through_pool=use_pool):
        if with_retrieve and through_pool:
            pool.step(tokens[i % n], lens[i % n], plens, w.k, w.C, out=r)
        elif with_retrieve:
            aasd.retrieve_drafts(tokens[i % n], lens[i % n], plens, w.n_min, w.n_max, w.k, w.C, out=r)
        aasd.verify(logits_steps[i % n], r["drafts"], r["draft_len"], r["strict"], zeroed_workspace=one_launch,
                    workspace=ws_zeroed if one_launch else ws, out=v if one_launch else v2, **kw)

    m = max(n, 64)
    scan_eager, scan_graph = time_steps(torch, lambda i: step(i, through_pool=False), m)
    pool_eager, pool_graph = time_steps(torch, lambda i: step(i, through_pool=True), m)
    eager, graph_us = (pool_eager, pool_graph) if use_pool else (scan_eager, scan_graph)
    t_eager, t_graph = time_steps(torch, lambda i: step(i, False, False), m)      # aasd_verify alone, as it is called by default
    v_eager, v_graph = time_steps(torch, lambda i: step(i, True, False), m)       # and with AASD_VERIFY_ZEROED_WORKSPACE
    # the sweep kernel alone (the default form), from the library's hook: the kernel's own begin and end
    evs = [(hip_event(), hip_event()) for _ in range(m)]
    for i in range(m):
        aasd.set_sweep_events(evs[i][0], evs[i][1])
        step(i, False, False)
    aasd.set_sweep_events(None, None)
    torch.cuda.synchronize()
    kern = sorted(hip_elapsed(a, b) * 1e3 for a, b in evs)[m // 2]
    best = min(x for x in (v_eager, v_graph, t_eager, t_graph) if x is not None)
    rnd = lambda x: None if x is None else round(x, 2)
    return {"shape": label, "sequences": B, "rows_per_step": B * R, "bytes_per_step": step_bytes,
            "rotating_step_buffers": n, "resident_MB": round(n * step_bytes / 1e6, 1),
            "retrieval": "pool" if use_pool else "scan",
            "pool_build_us": round(pool_build_us, 1), "pool_build_tokens": int(lens[n - 1].sum().item()),
            "retrieve_plus_verify_us": {"eager": rnd(eager), "hip_graph": rnd(graph_us)},
            "scan_plus_verify_us": {"eager": rnd(scan_eager), "hip_graph": rnd(scan_graph)},
            "pool_step_plus_verify_us": {"eager": rnd(pool_eager), "hip_graph": rnd(pool_graph)},
            "verify_us": {"eager": rnd(t_eager), "hip_graph": rnd(t_graph), "sweep_kernel_event_median": rnd(kern), "launches": 2},
            "verify_zeroed_workspace_us": {"eager": rnd(v_eager), "hip_graph": rnd(v_graph),
                                           "launches": aasd.verify_launches(B, w.C, w.k, V, dt_code, True),
                                           "note": "with AASD_VERIFY_ZEROED_WORKSPACE a small call goes out as one launch: fewer launches "
                                                   "for the host (the eager figure), no faster on the GPU (the graph figure)"},
            "verify_GB/s": round(step_bytes / best / 1e3, 1), "verify_frac_of_hbm_peak": round(step_bytes / best / 1e3 / HBM_PEAK_GBS, 4),
            "note": ("logit bytes of one step / time of the aasd_verify call alone (its faster launch mode); the time includes "
                     "launch and ramp of a launch this short" + (": " + note if note else ""))}


def prewarm(torch, step_fn, seconds=0.25):
    """Part of set-up: run the step for a quarter of a second so that clocks and caches of a fresh process are
    in their steady state before the W warm-up steps and the K timed ones (the first ~50 ms of work after start-up
    run 5-8 % slower on this GPU, which a handful of sub-millisecond warm-up steps does not cover)."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(5):
            step_fn()
        torch.cuda.synchronize()


def graph_latency_us(torch, steps_fn, check, n_steps):
    """Capture the launches of steps_fn() in one HIP graph, check that a replay reproduces `check` (the eager
    loop's last result: same launches, bit-identical), and time replays.  Context only: None if capture fails."""
    try:
        eager_last = check.clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            steps_fn()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        if not bool((check == eager_last).all()):
            print("bench.py: HIP graph replay differs from the eager loop; not reported", file=sys.stderr)
            return None
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(3):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        return round(g0.elapsed_time(g1) * 1e3 / (3 * n_steps), 2)
    except Exception as exc:  # the figure is context: a failed capture must not cost the benchmark line
        print(f"bench.py: HIP graph capture failed ({exc}); not reported", file=sys.stderr)
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {args.gpus} is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2505_13204_amd as aasd
    from paper_2505_13204_amd import _lib
    from tests import harness, synth

    _lib.load()  # no CPU fallback: fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.WORKLOADS[args.workload]
    if args.decode_steps:
        w = synth.scaled(w, steps=args.decode_steps)
    elt = 2 if w.dtype == "bf16" else 4
    if w.name.startswith("tree_"):
        return bench_tree(args, w, dev)
    mode = {"top": aasd.EXTRAS_TOP, "sample": aasd.EXTRAS_SAMPLE, "gumbel": aasd.EXTRAS_GUMBEL}[args.extras_mode]
    dt_code = aasd.BF16 if w.dtype == "bf16" else aasd.F32
    topk = args.verifier == "topk"

    def verify_ws(nseq):
        nbytes = (aasd.verify_topk_workspace_bytes if topk else aasd.verify_workspace_bytes)(nseq, w.C, w.k, w.V, dt_code)
        # zeroed once: aasd_verify may then take its one-launch form where all workgroups of the call fit the GPU at
        # once (the `tiny` workload; the larger batches take the two launches), and leaves the counters zero
        return torch.zeros(max(128, nbytes), dtype=torch.uint8, device=dev)

    def do_verify(logits, drafts, draft_len, strict, workspace=None, out=None):
        if topk:
            return aasd.verify_topk(logits, drafts, draft_len, topk=args.topk, want_rows=False, want_tokens=False,
                                    workspace=workspace, out=out)
        return aasd.verify(logits, drafts, draft_len, strict, alpha=w.alpha, beta=w.beta, want_rows=False,
                           want_tokens=False, want_near=True, workspace=workspace, out=out,
                           zeroed_workspace=workspace is not None)

    # ---------------------------------------------------------------- setup (untimed)
    t_setup = time.time()
    n_prefill_seq = w.B
    prefill_rows = w.B * w.L
    if args.prefill_rows and prefill_rows > args.prefill_rows:
        n_prefill_seq = max(1, args.prefill_rows // w.L)
        prefill_rows = n_prefill_seq * w.L
    prefill = torch.empty((prefill_rows, w.V), dtype=w.torch_dtype, device=dev)
    next_tok = np.empty(prefill_rows, dtype=np.int32)
    for b in range(n_prefill_seq):
        g, copied = synth.token_stream(w, b)
        synth.prefill_logits(w, b, g, copied, dev, out=prefill[b * w.L:(b + 1) * w.L])
        next_tok[b * w.L:(b + 1) * w.L] = synth.next_tokens(w, g)
    next_tok_d = torch.from_numpy(next_tok).to(dev)
    align_out = aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=mode, seed=w.seed)

    # run the synthetic decode loop once on the HIP path to obtain every step's inputs
    class Recorder(harness.Backend):
        def __init__(self):
            self.logits = []

        def _d(self, a, dt):
            return torch.as_tensor(np.ascontiguousarray(a), device=dev).to(dt)

        def retrieve(self, tokens, length, prompt_len, w_, extras, n_extras):
            out = aasd.retrieve_drafts(self._d(tokens, torch.int32), self._d(length, torch.int32),
                                       self._d(prompt_len, torch.int32), w_.n_min, w_.n_max, w_.k, w_.C)
            return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}

        def make_logits(self, w_, step, gs, copieds, length, drafts, draft_len, peaked):
            z = synth.verify_logits(w_, step, gs, copieds, length, drafts, draft_len, dev)
            self.logits.append(z)
            return z

        def verify(self, logits, drafts, draft_len, strict, w_):
            out = do_verify(logits, self._d(drafts, torch.int32), self._d(draft_len, torch.int32),
                            self._d(strict, torch.uint8))
            return {k: v.cpu().numpy() for k, v in out.items() if v is not None and k != "workspace"}

    # hold at most ~24 GiB of verify logits: later steps reuse the buffers of earlier ones in rotation
    step_bytes = w.B * w.R * w.V * elt
    max_steps_resident = max(1, min(w.steps, int(24 * 2 ** 30 // step_bytes)))
    rec = Recorder()
    trace = harness.decode(synth.scaled(w, steps=max_steps_resident), rec)
    S = len(trace.steps)
    BB = S * w.B  # decode steps x sequences, processed as one batch
    verify_logits = torch.stack(rec.logits).view(BB, w.R, w.V)
    rec.logits = None
    tok_cap = trace.tokens.shape[1]
    tokens_b = torch.from_numpy(np.tile(trace.tokens, (S, 1))).to(dev).contiguous()          # [S*B, cap]
    len_b = torch.from_numpy(np.concatenate([s.length for s in trace.steps]).astype(np.int32)).to(dev)
    plen_b = torch.full((BB,), w.L, dtype=torch.int32, device=dev)
    use_pool = args.retrieval == "pool"
    pool = None
    if use_pool:   # one pool per sequence of the batch, indexed up to the final length of the token buffers
        pool = aasd.DraftPool(BB, tok_cap, w.n_min, w.n_max, dev)
        full_len = torch.from_numpy(np.tile(trace.length, S).astype(np.int32)).to(dev)
        t_build = time.perf_counter()
        pool.update(tokens_b, full_len, reset=True)
        torch.cuda.synchronize()
        pool_build_ms = (time.perf_counter() - t_build) * 1e3

    def do_retrieve(out=None):
        if use_pool:
            return pool.retrieve(tokens_b, len_b, plen_b, w.k, w.C, out=out)
        return aasd.retrieve_drafts(tokens_b, len_b, plen_b, w.n_min, w.n_max, w.k, w.C, out=out)

    r_out = do_retrieve()
    ws = verify_ws(BB)
    v_out = do_verify(verify_logits, r_out["drafts"], r_out["draft_len"], r_out["strict"], workspace=ws)
    torch.cuda.synchronize()
    seq_accept = np.concatenate([s.verified["accept_len"] for s in trace.steps])
    seq_best = np.concatenate([s.verified["best_cand"] for s in trace.steps])
    if topk:   # logit comparisons only: the batch must equal the loop exactly
        self_check = {"sequences": BB, "batch_vs_loop_differences": int((v_out["accept_len"].cpu().numpy() != seq_accept).sum())}
        assert self_check["batch_vs_loop_differences"] == 0, "batched top-k verification differs from the decode loop"
    else:
        full = aasd.verify(verify_logits, r_out["drafts"], r_out["draft_len"], r_out["strict"], alpha=w.alpha, beta=w.beta)
        torch.cuda.synchronize()
        assert bool((full["accept_len"] == v_out["accept_len"]).all())
        self_check = check_batch_against_loop(np, w.name, full, seq_accept, seq_best, float(np.float32(w.alpha)),
                                              float(np.float32(w.beta)), w.C, w.k)
        del full
    setup_s = time.time() - t_setup

    verify_rows = BB * w.R
    rows_per_step = prefill_rows + verify_rows

    side = torch.cuda.Stream(device=dev)   # default priority, like the main stream

    def one_pass(two_streams=False):
        if two_streams:     # prefill alignment and decode verification are independent pieces of work
            with torch.cuda.stream(side):
                aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=mode, seed=w.seed, out=align_out)
        else:
            aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=mode, seed=w.seed, out=align_out)
        do_retrieve(out=r_out)
        do_verify(verify_logits, r_out["drafts"], r_out["draft_len"], r_out["strict"], workspace=ws, out=v_out)

    prewarm(torch, lambda: one_pass(args.streams == 2))
    for _ in range(args.warmup):
        one_pass(args.streams == 2)
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- timed region: exactly K steps
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        one_pass(args.streams == 2)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    value = rows_per_step / (ms_per_step * 1e-3)
    ms_per_step_one_stream = ms_per_step
    if args.streams == 2:   # for comparison: the same K steps on one stream
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        for i in range(K):
            one_pass(False)
        torch.cuda.synchronize()
        ms_per_step_one_stream = (time.perf_counter() - ts0) * 1e3 / K

    # ---------------------------------------------------------------- the same K steps again, instrumented (one stream)
    # (a) With the library's measurement hook only: the sweep (and draw) kernels are launched with start and stop
    # events that take the kernel's own begin and end; no packet is added to the stream, the kernels follow one another
    # as in the timed region.  (b) With one pair of events around each API call, for the call times: every event record
    # is a packet of its own between two kernels and costs a few microseconds of idle GPU.
    kev = [[hip_event() for _ in range(6)] for _ in range(K)]
    torch.cuda.synchronize()
    for i in range(K):
        aasd.set_sweep_events(kev[i][0], kev[i][1])
        if mode == aasd.EXTRAS_GUMBEL:
            aasd.set_draw_events(kev[i][4], kev[i][5])
        aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=mode, seed=w.seed, out=align_out)
        aasd.set_draw_events(None, None)
        do_retrieve(out=r_out)
        aasd.set_sweep_events(kev[i][2], kev[i][3])
        do_verify(verify_logits, r_out["drafts"], r_out["draft_len"], r_out["strict"], workspace=ws, out=v_out)
    aasd.set_sweep_events(None, None)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
    ti0 = time.perf_counter()
    for i in range(K):
        ev[i][0].record()
        aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=mode, seed=w.seed, out=align_out)
        ev[i][1].record()
        do_retrieve(out=r_out)
        ev[i][2].record()
        do_verify(verify_logits, r_out["drafts"], r_out["draft_len"], r_out["strict"], workspace=ws, out=v_out)
        ev[i][3].record()
    torch.cuda.synchronize()
    ms_per_step_instrumented = (time.perf_counter() - ti0) * 1e3 / K
    draws = None
    if mode == aasd.EXTRAS_GUMBEL:
        # The draw kernel is bound by the vector ALUs.  A rocprofv3 --pmc run of this command (profiles/
        # gumbel_extras_counters.txt) gives, per launch: SQ_ACTIVE_INST_VALU (time the vector ALUs spend on instructions, in
        # units of 4 cycles, summed over the SIMDs), SQ_INSTS_VALU (wave instructions) and GRBM_GUI_ACTIVE (cycles, summed
        # over the 8 dies: the shader clock of that run).  Busy cycles scale with the tokens drawn; the cycles available are
        # 256 CUs x 4 SIMDs x clock x this run's kernel time.  Waves of one SIMD overlap the end of one instruction with
        # the start of the next, so the counter can exceed the cycles by a few percent: frac is capped at 1, frac_raw is not.
        draw_ms = float(np.mean([hip_elapsed(kev[i][4], kev[i][5]) for i in range(K)]))
        n_mis = int(align_out["misaligned"].sum().item())
        tokens = n_mis * w.V
        draws = {"kernel": "aasd::gumbel_extras_kernel", "rows_drawn": n_mis, "tokens": tokens, "kernel_ms": round(draw_ms, 4),
                 "Gtokens/s": round(tokens / (draw_ms * 1e-3) / 1e9, 1), "roofline": None}
        cnt = read_traffic(os.path.join(ROOT, "profiles", "gumbel_extras_counters.txt"))
        if cnt.get("kernel_source_sha") == kernel_source_sha() and f"{w.name}.gumbel.valu_active_quadcycles" in cnt:
            g = lambda k: float(cnt[f"{w.name}.gumbel.{k}"])
            scale = tokens / g("tokens")
            clock_ghz = g("shader_clock_ghz")
            busy = g("valu_active_quadcycles") * 4 * scale              # SIMD-cycles of vector-ALU work per launch
            ach = busy / (draw_ms * 1e-3) / 1e9
            peak = 256 * 4 * clock_ghz                                  # G SIMD-cycles per second
            draws["roofline"] = {"bound": "alu", "achieved": round(ach, 1), "peak": round(peak, 1),
                                 "unit": "G SIMD-cycles/s of vector-ALU work", "frac": round(min(1.0, ach / peak), 4),
                                 "frac_raw": round(ach / peak, 4), "shader_clock_ghz": clock_ghz,
                                 "wave_insts_per_token": round(g("valu_wave_insts") / g("tokens"), 4),
                                 "G_wave_insts/s": round(g("valu_wave_insts") * scale / (draw_ms * 1e-3) / 1e9, 1),
                                 "source": "profiles/gumbel_extras_counters.txt"}
        else:
            draws["roofline_note"] = "no instruction counters under profiles/ for the kernel sources built now"
    align_ms = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(K)]))
    retr_ms = float(np.mean([ev[i][1].elapsed_time(ev[i][2]) for i in range(K)]))
    verify_ms = float(np.mean([ev[i][2].elapsed_time(ev[i][3]) for i in range(K)]))
    align_sweep_ms = float(np.mean([hip_elapsed(kev[i][0], kev[i][1]) for i in range(K)]))
    verify_sweep_ms = float(np.mean([hip_elapsed(kev[i][2], kev[i][3]) for i in range(K)]))

    row_bytes = w.V * elt
    align_gbs = prefill_rows * row_bytes / (align_sweep_ms * 1e-3) / 1e9
    verify_gbs = verify_rows * row_bytes / (verify_sweep_ms * 1e-3) / 1e9
    # HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), if this workload was profiled
    traffic, traffic_note = None, None
    measured = read_traffic(args.traffic_file)
    # the dominant kernel is the row sweep; of its two launches per step the one that runs longer is reported
    dom = "verify" if verify_sweep_ms >= align_sweep_ms else "align"
    key = f"{w.name}.{dom}_sweep.hbm_bytes_per_launch"
    if key in measured and measured.get(f"{w.name}.{dom}_sweep.rows") == str(verify_rows if dom == "verify" else prefill_rows):
        if measured.get("kernel_source_sha") == kernel_source_sha():
            traffic = int(float(measured[key]))
            traffic_note = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command on these kernel sources, copied from " + \
                           os.path.relpath(args.traffic_file, ROOT)
        else:
            traffic_note = "not quoted: the counters under profiles/ were taken on other kernel sources than the ones built now"
    dom_rows, dom_ms, dom_gbs = ((verify_rows, verify_sweep_ms, verify_gbs) if dom == "verify"
                                 else (prefill_rows, align_sweep_ms, align_gbs))
    roofline = {
        "bound": "hbm", "kernel": f"aasd::row_sweep_kernel ({dom} launch, {dom_rows} rows)",
        "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
        "traffic": traffic, "traffic_source": traffic_note, "bytes_per_launch": dom_rows * row_bytes, "avg_launch_ms": round(dom_ms, 4),
        "align_sample": {"rows": prefill_rows, "sweep_kernel_ms": round(align_sweep_ms, 4), "GB/s": round(align_gbs, 1),
                         "frac": round(align_gbs / HBM_PEAK_GBS, 4), "call_ms": round(align_ms, 4)},
        "verify": {"rows": verify_rows, "sweep_kernel_ms": round(verify_sweep_ms, 4), "GB/s": round(verify_gbs, 1),
                   "frac": round(verify_gbs / HBM_PEAK_GBS, 4), "call_ms": round(verify_ms, 4)},
        "retrieve_drafts": {"sequences": BB, "call_ms": round(retr_ms, 4), "through": args.retrieval,
                            **({"pool_build_ms": round(pool_build_ms, 3), "pool_MB": round(pool.nbytes / 1e6, 1)} if use_pool else {})},
        "ms_per_step_one_stream": round(ms_per_step_one_stream, 4),
        "ms_per_step_instrumented": round(ms_per_step_instrumented, 4),
        "note": "kernel times: the sweep kernels' own begin and end (start and stop events of their launches, set through the "
                "library's measurement hook) over a one-stream repeat of the K timed steps; call times: events around every "
                "call in a second repeat (ms_per_step_instrumented; the events cost idle time between kernels, so the timed "
                "region runs without them) and include the finish kernels",
    }

    # ---------------------------------------------------------------- the decode step at its real shape
    # Steps of one sequence are sequential (Algorithm 1): what a decode loop launches per step is one retrieval and one
    # verification over B x R rows.  Timed here over the resident per-step logits in rotation (cold HBM), for this
    # workload's shape and, always, for the 288-row step of batched_serving.
    per_step = None
    if not args.no_latency:
        per_step = []
        n_own = max(1, min(S, 256, int(4e9 // step_bytes)))
        own = per_step_block(
            torch, np, aasd, f"{w.name}: B={w.B}, R={w.R}, V={w.V}",
            [verify_logits[s * w.B:(s + 1) * w.B] for s in range(n_own)],
            [tokens_b[s * w.B:(s + 1) * w.B] for s in range(n_own)], [len_b[s * w.B:(s + 1) * w.B] for s in range(n_own)],
            plen_b[:w.B], w, use_pool=use_pool)
        if n_own * step_bytes < 300e6:
            own["note"] += "; CAUTION: fewer step buffers resident than the 256 MB Infinity Cache holds"
        per_step.append(own)
        if w.name != "batched_serving" and w.dtype == "bf16":
            w4 = synth.scaled(synth.WORKLOADS["batched_serving"], steps=8)     # 8 x 73.9 MB = 591 MB in rotation

            class Recorder4(Recorder):
                def verify(self, logits, drafts, draft_len, strict, w_):
                    out = aasd.verify(logits, self._d(drafts, torch.int32), self._d(draft_len, torch.int32),
                                      self._d(strict, torch.uint8), alpha=w_.alpha, beta=w_.beta)
                    return {k: v.cpu().numpy() for k, v in out.items() if v is not None and k != "workspace"}

            rec4 = Recorder4()
            tr4 = harness.decode(w4, rec4)
            S4 = len(tr4.steps)
            toks4 = torch.from_numpy(tr4.tokens).to(dev).contiguous()
            per_step.append(per_step_block(
                torch, np, aasd, f"batched_serving: B={w4.B}, R={w4.R}, V={w4.V}", rec4.logits, [toks4] * S4,
                [torch.from_numpy(st.length.astype(np.int32)).to(dev) for st in tr4.steps],
                torch.full((w4.B,), w4.L, dtype=torch.int32, device=dev), w4, use_pool=use_pool))
            rec4.logits = None

    # ---------------------------------------------------------------- CPU oracle on a bounded sample (context)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_a = min(prefill_rows, 8192)
        n_s = max(1, min(S, 9216 // (w.B * w.R)))
        nb = n_s * w.B
        bits_a = synth.to_host_bits(prefill[:n_a])
        bits_v = synth.to_host_bits(verify_logits[:nb])
        tok_h = tokens_b[:nb].cpu().numpy()
        len_h = len_b[:nb].cpu().numpy()
        plen_h = plen_b[:nb].cpu().numpy()
        tc = time.perf_counter()
        passes = 0
        while passes < CPU_BASELINE_MAX_PASSES and (passes == 0 or time.perf_counter() - tc < CPU_BASELINE_MIN_S):
            oracle.align_sample(bits_a, next_tok[:n_a], m_x=w.m, c=w.c, mode=mode)
            r = oracle.retrieve_drafts(tok_h, len_h, plen_h, w.n_min, w.n_max, w.k, w.C)
            if topk:
                oracle.verify_topk(bits_v, r["drafts"], r["draft_len"], topk=args.topk)
            else:
                oracle.verify(bits_v, r["drafts"], r["draft_len"], r["strict"], alpha=float(np.float32(w.alpha)),
                              beta=float(np.float32(w.beta)))
            passes += 1
        dt = time.perf_counter() - tc
        cpu = {"value": round(passes * (n_a + nb * w.R) / dt, 1), "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n_a} prefill rows + first {n_s} decode steps ({nb * w.R} verify rows) of the same "
                         f"workload, {passes} pass{'es' if passes > 1 else ''}, {dt:.1f} s", "host_cores_present": os.cpu_count()}

    out = {
        "metric": "logit rows/sec verified+sampled at V=%d %s" % (w.V, w.dtype),
        "value": round(value, 1), "unit": "rows/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "prompt_len": w.L, "V": w.V, "logits_dtype": w.dtype, "k": w.k, "C": w.C,
                   "n_gram": [w.n_min, w.n_max], "decode_steps": S, "prefill_rows": prefill_rows,
                   "verify_rows": verify_rows, "rows_per_step": rows_per_step,
                   "form": "all resident decode steps verified as one batch: the throughput form, an upper bound for a decode loop "
                           "whose steps are sequential (see per_step for the step at its real shape)",
                   "extras_mode": args.extras_mode,
                   "verifier": "top-%d" % args.topk if topk else "adaptive threshold", "retrieval": args.retrieval,
                   "streams": args.streams},
        "roofline": roofline, "cpu_baseline": cpu, "per_step": per_step, "self_check": self_check,
        "near_threshold_decisions": {"verify": None if topk else int(v_out["near_count"].sum().item()),
                                     "note": "evaluated draft tokens with |p - delta| < 1e-6 in the timed batch, counted by the kernel "
                                             "(a draft token that IS the row's most likely token has p = delta when the threshold is clamped)"},
        "tokens_per_decode_step": round(trace.mean_accept_len, 3), "setup_s": round(setup_s, 1),
    }
    if draws is not None:
        out["draws"] = draws
    print(json.dumps(out))


def bench_tree(args, w, dev):
    """The draft-tree form of the path (Sec. 3.2, Eq. 2): per step align_sample over the resident prefill
    rows, then for every recorded decode step retrieval with the alignment extras, tree build and tree
    verification (one logits row per tree node; rows beyond a sequence's node count are not read)."""
    import numpy as np
    import torch

    import paper_2505_13204_amd as aasd
    from tests import harness, synth

    elt = 2 if w.dtype == "bf16" else 4
    dt_code = aasd.BF16 if w.dtype == "bf16" else aasd.F32
    N = args.max_nodes or min(aasd.MAX_TREE_NODES, 1 + w.C * w.k * (1 + w.m))
    t_setup = time.time()
    streams = [synth.tree_stream(w, b) for b in range(w.B)]
    cap_rows = args.prefill_rows or 16384
    n_prefill_seq = max(1, min(w.B, cap_rows // w.L))
    prefill_rows = n_prefill_seq * w.L
    prefill = torch.empty((prefill_rows, w.V), dtype=w.torch_dtype, device=dev)
    scratch = torch.empty((w.L, w.V), dtype=w.torch_dtype, device=dev)
    next_tok = np.empty(w.B * w.L, dtype=np.int32)
    extras = torch.empty((w.B * w.L, w.m), dtype=torch.int32, device=dev)
    n_extras = torch.empty((w.B * w.L,), dtype=torch.uint8, device=dev)
    for b in range(w.B):   # alignment sampling of every prompt (setup); the first sequences stay resident for the timed pass
        g, alt, slot = streams[b]
        buf = prefill[b * w.L:(b + 1) * w.L] if b < n_prefill_seq else scratch
        synth.tree_prefill_logits(w, b, g, alt, slot, dev, out=buf)
        next_tok[b * w.L:(b + 1) * w.L] = synth.next_tokens(w, g)
        o = aasd.align_sample(buf, torch.from_numpy(next_tok[b * w.L:(b + 1) * w.L]).to(dev), m=w.m, c=w.c,
                              mode=aasd.EXTRAS_TOP, seed=w.seed, row_id_base=b * w.L)
        extras[b * w.L:(b + 1) * w.L] = o["extras"]
        n_extras[b * w.L:(b + 1) * w.L] = o["n_extras"]
    del scratch
    next_tok_d = torch.from_numpy(next_tok[:prefill_rows]).to(dev)
    align_out = aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=aasd.EXTRAS_TOP, seed=w.seed)
    extras_h, n_extras_h = extras.cpu().numpy(), n_extras.cpu().numpy()

    class Recorder(harness.Backend):
        def __init__(self):
            self.logits = []

        def _d(self, a, dt):
            return torch.as_tensor(np.ascontiguousarray(a), device=dev).to(dt)

        def retrieve(self, tokens, length, prompt_len, w_, ex, nx):
            out = aasd.retrieve_drafts(self._d(tokens, torch.int32), self._d(length, torch.int32),
                                       self._d(prompt_len, torch.int32), w_.n_min, w_.n_max, w_.k, w_.C,
                                       extras=extras, n_extras=n_extras, m=w_.m, extras_stride=w_.L)
            return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}

        def build_tree(self, r, root_tok, max_nodes):
            out = aasd.build_tree(self._d(r["drafts"], torch.int32), self._d(r["draft_len"], torch.int32),
                                  self._d(r["strict"], torch.uint8), self._d(r["draft_extras"], torch.int32),
                                  self._d(root_tok, torch.int32), max_nodes=max_nodes)
            return {k: v.cpu().numpy() for k, v in out.items() if v is not None}

        def make_tree_logits(self, w_, step, gs, length, tree):
            z = synth.tree_verify_logits(w_, step, gs, length, tree, dev)
            self.logits.append(z)
            return z

        def verify_tree(self, logits, tree, w_):
            out = aasd.verify_tree(logits, self._d(tree["node_token"], torch.int32), self._d(tree["node_parent"], torch.int32),
                                   self._d(tree["n_nodes"], torch.int32), self._d(tree["node_strict"], torch.uint8),
                                   alpha=w_.alpha, beta=w_.beta, want_rows=False, want_nodes=False, want_near=False)
            return {k: v.cpu().numpy() for k, v in out.items() if v is not None and k != "workspace"}

    step_bytes = w.B * N * w.V * elt
    max_steps_resident = max(1, min(w.steps, int(96 * 2 ** 30 // step_bytes)))   # room for max_nodes rows per tree is held, a tree uses a few of them
    rec = Recorder()
    trace = harness.decode_tree(synth.scaled(w, steps=max_steps_resident), rec, streams, extras_h, n_extras_h,
                                max_nodes=N)
    S = len(trace.steps)
    BB = S * w.B
    tree_logits = torch.stack(rec.logits).view(BB, N, w.V)
    rec.logits = None
    tokens_b = torch.from_numpy(np.tile(trace.tokens, (S, 1))).to(dev).contiguous()
    len_h = np.concatenate([s.length for s in trace.steps]).astype(np.int32)
    len_b = torch.from_numpy(len_h).to(dev)
    plen_b = torch.full((BB,), w.L, dtype=torch.int32, device=dev)
    root_b = torch.from_numpy(np.tile(trace.tokens, (S, 1))[np.arange(BB), len_h - 1].astype(np.int32)).to(dev)
    # sequence s*B + b of the batch reads the extras of prompt b: tile them like the token buffers
    extras_b = extras.view(w.B, w.L, w.m).repeat(S, 1, 1).view(BB * w.L, w.m).contiguous()
    n_extras_b = n_extras.view(w.B, w.L).repeat(S, 1).view(BB * w.L).contiguous()
    ws = torch.empty(max(16, aasd.verify_tree_workspace_bytes(BB, N, w.V, dt_code)), dtype=torch.uint8, device=dev)
    r_out = aasd.retrieve_drafts(tokens_b, len_b, plen_b, w.n_min, w.n_max, w.k, w.C, extras=extras_b,
                                 n_extras=n_extras_b, m=w.m, extras_stride=w.L)
    t_out = aasd.build_tree(r_out["drafts"], r_out["draft_len"], r_out["strict"], r_out["draft_extras"], root_b, max_nodes=N)
    v_out = aasd.verify_tree(tree_logits, t_out["node_token"], t_out["node_parent"], t_out["n_nodes"], t_out["node_strict"],
                             alpha=w.alpha, beta=w.beta, workspace=ws, want_rows=False, want_nodes=False)
    torch.cuda.synchronize()
    # the batched pass must reproduce the sequential loop it stands for: a decision may differ only where some
    # evaluated node lies within 1e-6 of its threshold (the two launch shapes sum in different orders)
    seq_accept = np.concatenate([s.verified["accept_len"] for s in trace.steps])
    full = aasd.verify_tree(tree_logits, t_out["node_token"], t_out["node_parent"], t_out["n_nodes"], t_out["node_strict"],
                            alpha=w.alpha, beta=w.beta, want_rows=False)
    torch.cuda.synchronize()
    differ = np.nonzero(v_out["accept_len"].cpu().numpy() != seq_accept)[0]
    node_gap = (full["node_p"].double() - full["node_delta"].double()).abs().cpu().numpy()
    used = np.arange(N)[None, :] < t_out["n_nodes"].cpu().numpy()[:, None]
    used[:, 0] = False
    outside = sum(0 if (node_gap[b][used[b]] < 1e-6).any() else 1 for b in differ)
    assert outside == 0, f"{outside} trees decide differently in the batch and in the loop away from any threshold"
    self_check = {"sequences": BB, "batch_vs_loop_differences": int(len(differ)), "differences_outside_1e-6_of_threshold": int(outside),
                  "near_threshold_decisions": int(full["near_count"].cpu().numpy().astype(np.int64).sum())}
    del full, node_gap
    n_nodes_h = t_out["n_nodes"].cpu().numpy()
    tree_rows = int(n_nodes_h.sum())
    setup_s = time.time() - t_setup
    rows_per_step = prefill_rows + tree_rows

    side = torch.cuda.Stream(device=dev)   # default priority, like the main stream

    def one_pass(i=None, ev=None, kev=None, two_streams=False):
        if ev: ev[0].record()
        if kev: aasd.set_sweep_events(kev[0], kev[1])
        if two_streams:     # prefill alignment does not feed the decode steps of this batch: it may overlap with them
            with torch.cuda.stream(side):
                aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=aasd.EXTRAS_TOP, seed=w.seed, out=align_out)
        else:
            aasd.align_sample(prefill, next_tok_d, m=w.m, c=w.c, mode=aasd.EXTRAS_TOP, seed=w.seed, out=align_out)
        if ev: ev[1].record()
        aasd.retrieve_drafts(tokens_b, len_b, plen_b, w.n_min, w.n_max, w.k, w.C, extras=extras_b, n_extras=n_extras_b,
                             m=w.m, extras_stride=w.L, out=r_out)
        if ev: ev[2].record()
        aasd.build_tree(r_out["drafts"], r_out["draft_len"], r_out["strict"], r_out["draft_extras"], root_b, max_nodes=N,
                        out=t_out)
        if ev: ev[3].record()
        if kev: aasd.set_sweep_events(kev[2], kev[3])
        aasd.verify_tree(tree_logits, t_out["node_token"], t_out["node_parent"], t_out["n_nodes"], t_out["node_strict"],
                         alpha=w.alpha, beta=w.beta, workspace=ws, want_rows=False, want_nodes=False, out=v_out)
        if ev: ev[4].record()

    prewarm(torch, lambda: one_pass(two_streams=args.streams == 2))
    for _ in range(args.warmup):
        one_pass(two_streams=args.streams == 2)
    torch.cuda.synchronize()
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        one_pass(two_streams=args.streams == 2)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    ms_per_step_one_stream = ms_per_step
    if args.streams == 2:
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        for i in range(K):
            one_pass()
        torch.cuda.synchronize()
        ms_per_step_one_stream = (time.perf_counter() - ts0) * 1e3 / K
    # the same K steps again: with the hook's events that take the sweep kernels' own begin and end, then with events
    # around every call (see main())
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
    kev = [[hip_event() for _ in range(4)] for _ in range(K)]
    torch.cuda.synchronize()
    for i in range(K):
        one_pass(i, None, kev[i])
    aasd.set_sweep_events(None, None)
    torch.cuda.synchronize()
    ti0 = time.perf_counter()
    for i in range(K):
        one_pass(i, ev[i], None)
    torch.cuda.synchronize()
    ms_per_step_instrumented = (time.perf_counter() - ti0) * 1e3 / K
    mean = lambda a, b: float(np.mean([ev[i][a].elapsed_time(ev[i][b]) for i in range(K)]))
    align_ms, retr_ms, build_ms, verify_ms = mean(0, 1), mean(1, 2), mean(2, 3), mean(3, 4)
    align_sweep_ms = float(np.mean([hip_elapsed(kev[i][0], kev[i][1]) for i in range(K)]))
    tree_sweep_ms = float(np.mean([hip_elapsed(kev[i][2], kev[i][3]) for i in range(K)]))
    row_bytes = w.V * elt
    align_gbs = prefill_rows * row_bytes / (align_sweep_ms * 1e-3) / 1e9
    tree_gbs = tree_rows * row_bytes / (tree_sweep_ms * 1e-3) / 1e9
    measured = read_traffic(args.traffic_file)
    traffic, traffic_note = None, None
    if measured.get(f"{w.name}.tree_sweep.rows") == str(tree_rows):
        if measured.get("kernel_source_sha") == kernel_source_sha():
            traffic = int(float(measured[f"{w.name}.tree_sweep.hbm_bytes_per_launch"]))
            traffic_note = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command on these kernel sources, copied from " + \
                           os.path.relpath(args.traffic_file, ROOT)
        else:
            traffic_note = "not quoted: the counters under profiles/ were taken on other kernel sources than the ones built now"
    roofline = {
        "bound": "hbm", "kernel": f"aasd::row_sweep_used_kernel (tree verification launch, {tree_rows} used rows of {BB * N})",
        "achieved": round(tree_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(tree_gbs / HBM_PEAK_GBS, 4),
        "traffic": traffic, "traffic_source": traffic_note, "bytes_per_launch": tree_rows * row_bytes, "avg_launch_ms": round(tree_sweep_ms, 4),
        "align_sample": {"rows": prefill_rows, "sweep_kernel_ms": round(align_sweep_ms, 4), "GB/s": round(align_gbs, 1),
                         "frac": round(align_gbs / HBM_PEAK_GBS, 4), "call_ms": round(align_ms, 4)},
        "verify_tree": {"rows_used": tree_rows, "rows_launched": BB * N, "sweep_kernel_ms": round(tree_sweep_ms, 4),
                        "GB/s": round(tree_gbs, 1), "frac": round(tree_gbs / HBM_PEAK_GBS, 4), "call_ms": round(verify_ms, 4)},
        "retrieve_drafts": {"sequences": BB, "call_ms": round(retr_ms, 4)},
        "build_tree": {"sequences": BB, "call_ms": round(build_ms, 4), "mean_nodes": round(float(n_nodes_h.mean()), 2),
                       "max_nodes": int(n_nodes_h.max())},
        "ms_per_step_one_stream": round(ms_per_step_one_stream, 4),
        "ms_per_step_instrumented": round(ms_per_step_instrumented, 4),
        "note": "only the rows of existing tree nodes are read and counted; kernel times: the sweep kernels' own begin and end "
                "(start and stop events of their launches) over a one-stream repeat of the K timed steps; call times from a "
                "second repeat with events around every call",
    }

    # ---------------------------------------------------------------- sequential per-step latency (context)
    latency = None
    if not args.no_latency and w.B * N <= 512:
        n_lat = min(S, 256)
        sl0 = slice(0, w.B)
        ws1 = torch.empty(max(16, aasd.verify_tree_workspace_bytes(w.B, N, w.V, dt_code)), dtype=torch.uint8, device=dev)
        r1 = aasd.retrieve_drafts(tokens_b[sl0], len_b[sl0], plen_b[sl0], w.n_min, w.n_max, w.k, w.C, extras=extras,
                                  n_extras=n_extras, m=w.m, extras_stride=w.L)
        t1_ = aasd.build_tree(r1["drafts"], r1["draft_len"], r1["strict"], r1["draft_extras"], root_b[sl0], max_nodes=N)
        v1 = aasd.verify_tree(tree_logits[sl0], t1_["node_token"], t1_["node_parent"], t1_["n_nodes"], t1_["node_strict"],
                              alpha=w.alpha, beta=w.beta, workspace=ws1, want_rows=False, want_nodes=False, want_near=False)

        def lat_steps():
            for s_ in range(n_lat):
                sl = slice(s_ * w.B, (s_ + 1) * w.B)
                aasd.retrieve_drafts(tokens_b[sl], len_b[sl], plen_b[sl], w.n_min, w.n_max, w.k, w.C, extras=extras,
                                     n_extras=n_extras, m=w.m, extras_stride=w.L, out=r1)
                aasd.build_tree(r1["drafts"], r1["draft_len"], r1["strict"], r1["draft_extras"], root_b[sl], max_nodes=N, out=t1_)
                aasd.verify_tree(tree_logits[sl], t1_["node_token"], t1_["node_parent"], t1_["n_nodes"], t1_["node_strict"],
                                 alpha=w.alpha, beta=w.beta, workspace=ws1, want_rows=False, want_nodes=False,
                                 want_near=False, out=v1)

        lat_steps()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        lat_steps()
        e1.record()
        torch.cuda.synchronize()
        graph_us = graph_latency_us(torch, lat_steps, v1["accept_len"], n_lat)
        latency = {"decode_steps": n_lat, "rows_per_step": "%d of %d" % (int(n_nodes_h[:n_lat * w.B].sum()) // n_lat, w.B * N),
                   "us_per_decode_step": round(e0.elapsed_time(e1) * 1e3 / n_lat, 2),
                   "hip_graph_us_per_decode_step": graph_us,
                   "note": "retrieve + build_tree + verify_tree launched back to back per decode step, no host sync"}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_a = min(prefill_rows, 4096)
        nb = max(1, min(BB, 4096 // max(1, int(n_nodes_h.mean()))))
        bits_a = synth.to_host_bits(prefill[:n_a])
        bits_v = synth.to_host_bits(tree_logits[:nb])
        tok_h = tokens_b[:nb].cpu().numpy()
        ex_h, nx_h = extras_b[:nb * w.L].cpu().numpy(), n_extras_b[:nb * w.L].cpu().numpy()
        root_h = root_b[:nb].cpu().numpy()
        tc = time.perf_counter()
        passes = 0
        while passes < CPU_BASELINE_MAX_PASSES and (passes == 0 or time.perf_counter() - tc < CPU_BASELINE_MIN_S):
            oracle.align_sample(bits_a, next_tok[:n_a], m_x=w.m, c=w.c)
            r = oracle.retrieve_drafts(tok_h, len_h[:nb], np.full(nb, w.L, np.int32), w.n_min, w.n_max, w.k, w.C,
                                       extras=ex_h, n_extras=nx_h, m_x=w.m, extras_stride=w.L)
            t = oracle.build_tree(r["drafts"], r["draft_len"], r["strict"], r["draft_extras"], root_tok=root_h, max_nodes=N)
            oracle.verify_tree(bits_v, t["node_token"], t["node_parent"], t["node_strict"], t["n_nodes"],
                               alpha=float(np.float32(w.alpha)), beta=float(np.float32(w.beta)))
            passes += 1
        dtc = time.perf_counter() - tc
        used = int(t["n_nodes"].sum())
        cpu = {"value": round(passes * (n_a + used) / dtc, 1), "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n_a} prefill rows + first {nb} trees ({used} tree rows) of the same workload, "
                         f"{passes} pass{'es' if passes > 1 else ''}, {dtc:.1f} s",
               "host_cores_present": os.cpu_count()}

    out = {
        "metric": "logit rows/sec verified+sampled at V=%d %s" % (w.V, w.dtype),
        "value": round(rows_per_step / (ms_per_step * 1e-3), 1), "unit": "rows/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "prompt_len": w.L, "V": w.V, "logits_dtype": w.dtype,
                   "k": w.k, "C": w.C, "m": w.m, "n_gram": [w.n_min, w.n_max], "max_nodes": N, "decode_steps": S,
                   "prefill_rows": prefill_rows, "tree_rows": tree_rows, "rows_per_step": rows_per_step,
                   "form": "all decode steps built and verified as one batch of trees", "streams": args.streams},
        "roofline": roofline, "cpu_baseline": cpu, "latency": latency, "self_check": self_check,
        "tokens_per_decode_step": round(trace.mean_accept_len, 3), "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
