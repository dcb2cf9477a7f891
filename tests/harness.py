"""Synthetic decode driver: the loop of Algorithm 1 with the model forward replaced by seeded
logits.  It only orchestrates - retrieve drafts, obtain verify logits, verify, append - through a
backend object, so the same driver runs the HIP library and (in tests) the CPU oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional

import numpy as np

from . import synth


@dataclass
class StepRecord:
    length: np.ndarray        # [B] context length before the step
    retrieved: dict           # host copies of the retrieval outputs
    verified: dict            # host copies of the verification outputs
    logits: object = None     # the step's verify logits (backend-native), kept only on request


@dataclass
class DecodeTrace:
    tokens: np.ndarray        # [B, tok_cap] final token buffers
    length: np.ndarray        # [B]
    steps: List[StepRecord] = field(default_factory=list)

    @property
    def mean_accept_len(self) -> float:
        """Tokens committed per step (accepted draft tokens + the one token of the target model)."""
        a = np.concatenate([s.verified["accept_len"] for s in self.steps])
        return float(a.mean() + 1.0)


class Backend:
    """What the driver needs from an implementation; all arrays cross this interface as numpy."""

    def retrieve(self, tokens: np.ndarray, length: np.ndarray, prompt_len: np.ndarray, w: synth.Workload,
                 extras, n_extras) -> dict:
        raise NotImplementedError

    def make_logits(self, w: synth.Workload, step: int, gs, copieds, length, drafts, draft_len, peaked: bool):
        raise NotImplementedError

    def verify(self, logits, drafts: np.ndarray, draft_len: np.ndarray, strict: np.ndarray, w: synth.Workload) -> dict:
        raise NotImplementedError

    # ---- draft-tree path (Sec. 3.2): only needed by decode_tree
    def build_tree(self, retrieved: dict, root_tok: np.ndarray, max_nodes: int) -> dict:
        raise NotImplementedError

    def make_tree_logits(self, w: synth.Workload, step: int, gs, length, tree: dict):
        raise NotImplementedError

    def verify_tree(self, logits, tree: dict, w: synth.Workload) -> dict:
        raise NotImplementedError


def decode(w: synth.Workload, backend: Backend, steps: Optional[int] = None, peaked: bool = False,
           extras=None, n_extras=None, keep_logits: bool = False,
           on_step: Optional[Callable[[int, StepRecord], None]] = None) -> DecodeTrace:
    """Run `steps` decode steps of workload `w` for all B sequences in lock step."""
    steps = w.steps if steps is None else steps
    streams = [synth.token_stream(w, b) for b in range(w.B)]
    gs = [s[0] for s in streams]
    copieds = [s[1] for s in streams]
    tokens = np.zeros((w.B, w.tok_cap), dtype=np.int32)
    for b in range(w.B):
        tokens[b, :w.L] = gs[b][:w.L]
    length = np.full(w.B, w.L, dtype=np.int32)
    prompt_len = np.full(w.B, w.L, dtype=np.int32)
    trace = DecodeTrace(tokens=tokens, length=length)
    for step in range(steps):
        r = backend.retrieve(tokens, length, prompt_len, w, extras, n_extras)
        logits = backend.make_logits(w, step, gs, copieds, length, r["drafts"], r["draft_len"], peaked)
        v = backend.verify(logits, r["drafts"], r["draft_len"], r["strict"], w)
        rec = StepRecord(length=length.copy(), retrieved=r, verified=v, logits=logits if keep_logits else None)
        trace.steps.append(rec)
        if on_step is not None:
            on_step(step, rec)
        for b in range(w.B):
            a, c = int(v["accept_len"][b]), int(v["best_cand"][b])
            n = int(length[b])
            tokens[b, n:n + a] = r["drafts"][b, c, :a]
            tokens[b, n + a] = v["next_token"][b]
            length[b] = n + a + 1
    trace.length = length
    return trace


def decode_tree(w: synth.Workload, backend: Backend, streams, extras, n_extras, steps: Optional[int] = None,
                max_nodes: int = 64, keep_logits: bool = False,
                on_step: Optional[Callable[[int, StepRecord], None]] = None) -> DecodeTrace:
    """The same loop with the candidates and their alignment extras merged into a draft tree
    (Sec. 3.2, Eq. 2): retrieve, build the tree, obtain one row per node, verify the tree, append
    the accepted path and the next token.  `streams` = [synth.tree_stream(w, b) for b]; extras and
    n_extras are the alignment-sampling outputs of the prefill rows ([B*L, m], [B*L])."""
    steps = w.steps if steps is None else steps
    gs = [s[0] for s in streams]
    tokens = np.zeros((w.B, w.tok_cap), dtype=np.int32)
    for b in range(w.B):
        tokens[b, :w.L] = gs[b][:w.L]
    length = np.full(w.B, w.L, dtype=np.int32)
    prompt_len = np.full(w.B, w.L, dtype=np.int32)
    trace = DecodeTrace(tokens=tokens, length=length)
    for step in range(steps):
        r = backend.retrieve(tokens, length, prompt_len, w, extras, n_extras)
        root = tokens[np.arange(w.B), length - 1].copy()
        t = backend.build_tree(r, root, max_nodes)
        logits = backend.make_tree_logits(w, step, gs, length, t)
        v = backend.verify_tree(logits, t, w)
        rec = StepRecord(length=length.copy(), retrieved={**r, "tree": t}, verified=v,
                         logits=logits if keep_logits else None)
        trace.steps.append(rec)
        if on_step is not None:
            on_step(step, rec)
        for b in range(w.B):
            a, n = int(v["accept_len"][b]), int(length[b])
            path = v["accept_path"][b, :a]
            tokens[b, n:n + a] = t["node_token"][b, path]
            tokens[b, n + a] = v["next_token"][b]
            length[b] = n + a + 1
    trace.length = length
    return trace
