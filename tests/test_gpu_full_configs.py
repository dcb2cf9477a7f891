"""Configurations 3, 4 and 5 against the oracle at their full sizes, in the launch shapes bench.py times.

long_context (config 3) and batched_serving (config 4) are checked in full: every prefill row in both extras
modes, every retrieval, every verify row of every decode step.  stress_tree (config 5; 80 GB of prefill logits and
321 GB of verify logits in total) is checked on every row of its first and last decode step, every prefill row
of its first and last sequence, and every retrieval of all 64 x 128 lookups.  The oracle is the single-threaded
C code, run over disjoint row ranges on the host's threads (tests/backends.py).  Each test prints what it covered.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_13204_amd as aasd
from tests import harness, synth
from tests import backends as bk

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _t(a, dt):
    return torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)


def _prefill(w, seqs):
    """Prefill logits and next tokens of the given sequences, stacked: [len(seqs) * L, V] on the device."""
    z = torch.empty((len(seqs) * w.L, w.V), dtype=w.torch_dtype, device=DEV)
    nt = np.empty(len(seqs) * w.L, np.int32)
    for i, b in enumerate(seqs):
        g, copied = synth.token_stream(w, b)
        synth.prefill_logits(w, b, g, copied, DEV, out=z[i * w.L:(i + 1) * w.L])
        nt[i * w.L:(i + 1) * w.L] = synth.next_tokens(w, g)
    return z, nt


def _check_align(w, z, nt, mode, tally, row_id_base=0, chunk=8192):
    """One launch over all rows of z (the shape bench.py times), the oracle over every row, chunk by chunk."""
    got = bk.hip_align(z, nt, w.m, w.c, mode, seed=w.seed, row_id_base=row_id_base)
    for lo in range(0, z.shape[0], chunk):
        hi = min(lo + chunk, z.shape[0])
        ref = bk.oracle_align_rows(synth.to_host_bits(z[lo:hi]), nt[lo:hi], w.m, w.c, mode, seed=w.seed,
                                   row_id_base=row_id_base + lo)
        bk.compare_align({k: (v[lo:hi] if v is not None else None) for k, v in got.items()}, ref, tally, mode)
    return got


def _decode_and_check(w, tally, keep_steps=None, one_launch=False):
    """The decode loop on the HIP path (one aasd_retrieve_drafts and one aasd_verify per step, the per-step shape),
    then the oracle: every retrieval of every step, and the verify rows of the kept steps (all steps if
    keep_steps is None).  one_launch: the steps pass a zeroed workspace with AASD_VERIFY_ZEROED_WORKSPACE, and the
    library takes the one-launch form up to 32 MiB of logits (9-row steps; the 288-row steps of batched_serving go out
    as two kernels, the sweep writing one partial per workgroup).  As every checked step's outputs equal the oracle's on the same inputs, the loop has
    followed the oracle's trajectory up to that step.  Returns the trace and the number of verify rows checked."""
    hip = bk.HipBackend(DEV, one_launch=one_launch)
    kept = {}

    def on_step(step, rec):
        if keep_steps is None or step in keep_steps:
            kept[step] = rec.logits
        rec.logits = None

    trace = harness.decode(w, hip, keep_logits=True, on_step=on_step)
    S = len(trace.steps)
    # every retrieval: the final token buffer holds every step's context as a prefix
    lens = np.concatenate([s.length for s in trace.steps]).astype(np.int32)
    toks = np.tile(trace.tokens, (S, 1))
    ref_r = oracle.retrieve_drafts(toks, lens, np.full(S * w.B, w.L, np.int32), w.n_min, w.n_max, w.k, w.C)
    got_r = {k: np.concatenate([s.retrieved[k] for s in trace.steps]) for k in
             ("n_cand", "key_len", "src_pos", "draft_len", "drafts", "strict")}
    bk.compare_retrieve(got_r, ref_r)
    rows = 0
    for step in sorted(kept):
        st = trace.steps[step]
        ref = bk.oracle_verify_seqs(synth.to_host_bits(kept[step]), st.retrieved["drafts"], st.retrieved["draft_len"],
                                    st.retrieved["strict"], bk.f32(w.alpha), bk.f32(w.beta))
        bk.compare_verify(st.verified, ref, tally)
        rows += w.B * w.R
    return trace, kept, rows


def _check_batched_verify(w, trace, kept, tally):
    """All kept steps verified as ONE batch (bench.py's throughput form): must reproduce the per-step results."""
    steps = sorted(kept)
    logits = torch.cat([kept[s] for s in steps]).view(len(steps) * w.B, w.R, w.V)
    cat = lambda name: np.concatenate([trace.steps[s].retrieved[name] for s in steps])
    v = bk.to_np(aasd.verify(logits, _t(cat("drafts"), torch.int32), _t(cat("draft_len"), torch.int32),
                             _t(cat("strict"), torch.uint8), alpha=w.alpha, beta=w.beta))
    torch.cuda.synchronize()
    ref = {k: np.concatenate([trace.steps[s].verified[k] for s in steps]) for k in ("accept_len", "best_cand", "next_token")}
    near = np.concatenate([trace.steps[s].verified["near_count"] for s in steps]) > 0
    for name in ref:   # the two launch shapes sum in different orders: only a decision within rounding of its threshold may differ
        assert (v[name] == ref[name])[~near].all(), name
    np.testing.assert_array_equal(v["row_argmax"], np.concatenate([trace.steps[s].verified["row_argmax"] for s in steps]))
    return int(near.sum())


def test_long_context_in_full():
    """Config 3: 8192 prefill rows (TOP and SAMPLE), 1024 decode steps of 9 rows, every row against the oracle."""
    w = synth.WORKLOADS["long_context"]
    tally = bk.Tally()
    z, nt = _prefill(w, [0])
    _check_align(w, z, nt, oracle.EXTRAS_TOP, tally)
    _check_align(w, z, nt, oracle.EXTRAS_SAMPLE, tally)
    del z
    trace, kept, rows = _decode_and_check(w, tally, one_launch=True)
    assert len(trace.steps) == w.steps == 1024 and rows == 1024 * 9
    near = _check_batched_verify(w, trace, kept, tally)
    print(f"long_context covered: prefill rows {w.L} of {w.L} x 2 modes, retrievals {w.steps} of {w.steps}, "
          f"verify rows {rows} of {w.steps * w.R} (per step, in the one-launch form) and again as one batch; near {near}; {tally}")


def test_batched_serving_in_full():
    """Config 4: 65,536 prefill rows in one launch (TOP and SAMPLE), 256 decode steps of 32 x 9 rows."""
    w = synth.WORKLOADS["batched_serving"]
    tally = bk.Tally()
    z, nt = _prefill(w, list(range(w.B)))
    assert z.shape[0] == 65536
    _check_align(w, z, nt, oracle.EXTRAS_TOP, tally)
    _check_align(w, z, nt, oracle.EXTRAS_SAMPLE, tally)
    del z
    torch.cuda.empty_cache()
    trace, kept, rows = _decode_and_check(w, tally, one_launch=True)
    assert len(trace.steps) == w.steps == 256 and rows == 256 * 288
    near = _check_batched_verify(w, trace, kept, tally)
    print(f"batched_serving covered: prefill rows 65536 of 65536 x 2 modes, retrievals {w.steps * w.B} of {w.steps * w.B}, "
          f"verify rows {rows} of {w.steps * w.B * w.R} (per step) and again as one batch of 8192 sequences; near {near}; {tally}")


def test_stress_tree_first_and_last_step_and_sequence():
    """Config 5: every row of the first and the last of the 128 decode steps (64 x 129 rows of V = 152064 each),
    every prefill row of sequences 0 and 63, every one of the 64 x 128 retrievals."""
    w = synth.WORKLOADS["stress_tree"]
    tally = bk.Tally()
    # prefill: sequences 0 and 63 stacked into one 8192-row launch (the many-rows launch shape of the full set)
    z, nt = _prefill(w, [0, w.B - 1])
    _check_align(w, z, nt, oracle.EXTRAS_TOP, tally)
    for i, b in enumerate((0, w.B - 1)):   # seeded draws are keyed by the global row id: one launch per sequence
        _check_align(w, z[i * w.L:(i + 1) * w.L], nt[i * w.L:(i + 1) * w.L], oracle.EXTRAS_SAMPLE, tally, row_id_base=b * w.L)
    del z
    torch.cuda.empty_cache()
    trace, kept, rows = _decode_and_check(w, tally, keep_steps={0, w.steps - 1})
    assert len(trace.steps) == w.steps == 128 and rows == 2 * 64 * 129
    print(f"stress_tree covered: prefill rows {2 * w.L} of {w.B * w.L} (sequences 0 and 63; TOP in one 8192-row launch, SAMPLE "
          f"per sequence), retrievals {w.steps * w.B} of {w.steps * w.B}, verify rows {rows} of {w.steps * w.B * w.R} "
          f"(steps 0 and 127 in full); {tally}")
