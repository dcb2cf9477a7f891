"""Seeded synthetic workloads shaped like the paper's (Sec. 4.1, Appendix B): token streams with
planted repeats and logits with a peak on the continuation token.

This module only GENERATES inputs (random tokens, Gaussian logits, which row gets a peak).  It
holds none of the method's arithmetic - no softmax, no threshold, no matching - and is the one
module that both the HIP tests/benchmark and the CPU-oracle tests may use.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int                 # sequences
    L: int                 # prompt length
    V: int                 # vocabulary
    dtype: str             # "f32" | "bf16"
    sigma2: float          # variance of the Gaussian logits
    bump: float            # added to the continuation token's logit ...
    q: float               # ... with this probability
    q_copy: float          # ... or this one when the position lies in a planted copy
    n_min: int
    n_max: int
    k: int                 # draft length
    C: int                 # candidates per step
    steps: int             # decode steps
    coverage: float        # fraction of the stream covered by planted copies (0 = use `spans`)
    spans: int = 0         # exact number of planted 8-token spans (config "tiny")
    motifs: int = 0        # > 0: copies are drawn from a pool of this many 12-token motifs
    m: int = 2             # extras per misaligned position (Sec. 4.1: at most two)
    c: int = 4             # candidate-set size
    alpha: float = 0.1     # Sec. 4.1: 0.1 (LLaMA-3.1), 0.2 (Qwen-2.5)
    beta: float = 0.1
    seed: int = 0
    mis_rate: float = 0.3  # draft-tree workloads: fraction of misaligned prompt positions (Sec. 2.3 reports about 45 %
                           # of the retrieved tokens; 0.3 of all positions gives a comparable share of the drafts)

    @property
    def R(self) -> int:
        return 1 + self.C * self.k

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def stream_len(self) -> int:
        return self.L + self.steps * (self.k + 1) + self.k + 1

    @property
    def tok_cap(self) -> int:
        return self.L + self.steps * (self.k + 1)


# The five configurations the build is measured on; sizes follow the paper's models
# (V = 128256 LLaMA-3.1, 152064 Qwen-2.5) and context lengths (Appendix B: 3.6k-15.3k tokens).
WORKLOADS = {
    "tiny": Workload("tiny", B=1, L=256, V=32000, dtype="f32", sigma2=2.0, bump=6.0, q=0.7, q_copy=0.7,
                     n_min=3, n_max=3, k=4, C=1, steps=64, coverage=0.0, spans=3, seed=0),
    "llama3_single": Workload("llama3_single", B=1, L=2048, V=128256, dtype="bf16", sigma2=3.0, bump=8.0, q=0.6,
                              q_copy=0.8, n_min=3, n_max=3, k=8, C=1, steps=512, coverage=0.30),
    "long_context": Workload("long_context", B=1, L=8192, V=128256, dtype="bf16", sigma2=3.0, bump=8.0, q=0.65,
                             q_copy=0.65, n_min=4, n_max=4, k=8, C=1, steps=1024, coverage=0.50),
    "batched_serving": Workload("batched_serving", B=32, L=2048, V=128256, dtype="bf16", sigma2=3.0, bump=8.0,
                                q=0.6, q_copy=0.8, n_min=3, n_max=3, k=8, C=1, steps=256, coverage=0.30),
    "stress_tree": Workload("stress_tree", B=64, L=4096, V=152064, dtype="bf16", sigma2=1.0, bump=0.0, q=0.0,
                            q_copy=0.0, n_min=2, n_max=4, k=8, C=16, steps=128, coverage=0.50, motifs=8, alpha=0.2),
    # Draft-tree form of the path (Sec. 3.2): the same model shapes, prompts made by tree_stream.
    "tree_single": Workload("tree_single", B=1, L=2048, V=128256, dtype="bf16", sigma2=3.0, bump=0.0, q=0.0, q_copy=0.0,
                            n_min=1, n_max=3, k=8, C=4, steps=256, coverage=0.80),
    "tree_batch": Workload("tree_batch", B=64, L=4096, V=152064, dtype="bf16", sigma2=1.0, bump=0.0, q=0.0, q_copy=0.0,
                           n_min=1, n_max=4, k=8, C=16, steps=64, coverage=0.80, motifs=8, alpha=0.2),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller copy of a workload (same recipe, fewer rows/steps) for quick parity cases."""
    return replace(w, **kw)


# --------------------------------------------------------------------------- token streams
def token_stream(w: Workload, b: int):
    """Stream G_b of w.stream_len token ids and a mask of the positions that lie in a planted copy.
    The prompt is G[:L]; the rest is the text the synthetic model prefers to continue with."""
    rng = np.random.default_rng([w.seed, b, 0x70C])
    n = w.stream_len
    g = rng.integers(0, w.V, size=n, dtype=np.int64).astype(np.int32)
    copied = np.zeros(n, dtype=bool)
    if w.spans > 0:
        # exactly `spans` 8-token spans of the first half of the prompt, each copied once later in the
        # prompt and once into the continuation
        src = np.sort(rng.choice(np.arange(8, w.L // 2 - 8, 16), size=w.spans, replace=False))
        dst_p = np.sort(rng.choice(np.arange(w.L // 2 + 8, w.L - 16, 16), size=w.spans, replace=False))
        dst_c = np.sort(rng.choice(np.arange(w.L + 8, n - 16, 16), size=w.spans, replace=False))
        for s, d1, d2 in zip(src, dst_p, dst_c):
            g[d1:d1 + 8] = g[s:s + 8]; copied[d1:d1 + 8] = True
            g[d2:d2 + 8] = g[s:s + 8]; copied[d2:d2 + 8] = True
        return g, copied
    if w.motifs > 0:
        pool = rng.integers(0, w.V, size=(w.motifs, 12), dtype=np.int64).astype(np.int32)
        pos = 16
        while pos + 12 < n:
            if rng.random() < w.coverage:
                g[pos:pos + 12] = pool[rng.integers(0, w.motifs)]
                copied[pos:pos + 12] = True
            pos += 12
        return g, copied
    # copies of earlier segments (length uniform in [16, 64]) until `coverage` of the stream is covered
    pos = 96
    while pos < n:
        ln = int(rng.integers(16, 65))
        ln = min(ln, n - pos)
        if rng.random() < w.coverage and pos > ln:
            s = int(rng.integers(0, pos - ln))
            g[pos:pos + ln] = g[s:s + ln]
            copied[pos:pos + ln] = True
        pos += ln
    return g, copied


def next_tokens(w: Workload, g: np.ndarray) -> np.ndarray:
    """Row i of the prefill logits predicts prompt token i+1; the last row has no next prompt token."""
    nt = np.empty(w.L, dtype=np.int32)
    nt[:-1] = g[1:w.L]
    nt[-1] = -1
    return nt


# --------------------------------------------------------------------------- logits
def _generator(device, *key) -> torch.Generator:
    gen = torch.Generator(device=device)
    seed = 0
    for x in key:
        seed = (seed * 1000003 + int(x) + 0x9E37) % (2 ** 62)
    gen.manual_seed(seed)
    return gen


def logits_rows(w: Workload, targets: torch.Tensor, q: torch.Tensor, gen: torch.Generator, device,
                peaked: bool = False, out: Optional[torch.Tensor] = None, chunk: int = 512,
                slot: Optional[torch.Tensor] = None, lead: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[n, V] logits: i.i.d. N(0, sigma2) noise, plus `bump` on targets[i] with probability q[i]
    (targets[i] < 0: no peak).  peaked=True instead plants LLM-like rows: four tokens at logits 24, 23,
    22, 21 (probabilities about 0.64, 0.24, 0.09, 0.03), the target being the first, second or third
    of them with probability 0.80 / 0.14 / 0.06.  slot[i] in {0, 1, 2} fixes the target's rank instead of
    drawing it, and lead[i] >= 0 names the best of the other three tokens (the row's top token when slot > 0)."""
    n = targets.numel()
    targets = targets.to(device=device, dtype=torch.long)
    q = q.to(device=device, dtype=torch.float32)
    if out is None:
        out = torch.empty((n, w.V), dtype=w.torch_dtype, device=device)
    sigma = math.sqrt(w.sigma2)
    for lo in range(0, n, chunk):
        hi = min(lo + chunk, n)
        z = torch.randn((hi - lo, w.V), generator=gen, device=device, dtype=torch.float32) * sigma
        t = targets[lo:hi]
        rows = torch.arange(hi - lo, device=device)
        has = t >= 0
        if peaked:
            # four distinct-valued top tokens at 24, 23, 22, 21; the target is the top one with
            # probability 0.80, the runner-up with 0.14, the third with 0.06
            others = torch.randint(0, w.V, (hi - lo, 3), generator=gen, device=device)
            place = torch.rand(hi - lo, generator=gen, device=device)
            slot_c = (place >= 0.80).long() + (place >= 0.94).long()  # 0, 1 or 2: rank of the target
            if slot is not None:
                slot_c = slot[lo:hi].to(device=device, dtype=torch.long)
            if lead is not None:
                ld = lead[lo:hi].to(device=device, dtype=torch.long)
                others[:, 0] = torch.where(ld >= 0, ld, others[:, 0])
            levels = torch.tensor([24.0, 23.0, 22.0, 21.0], device=device)
            r = rows[has]
            for i in range(3):
                # the i-th other token takes the i-th level that the target does not occupy
                lvl = levels[(i + (i >= slot_c[has]).long())]
                z[r, others[has, i]] = lvl
            z[r, t[has]] = levels[slot_c[has]]
        else:
            hit = has & (torch.rand(hi - lo, generator=gen, device=device) < q[lo:hi])
            z[rows[hit], t[hit]] += w.bump
        out[lo:hi] = z.to(w.torch_dtype)
    return out


def prefill_logits(w: Workload, b: int, g: np.ndarray, copied: np.ndarray, device, rows: Optional[slice] = None,
                   peaked: bool = False, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Prefill logits of sequence b: row i predicts absolute position i+1."""
    rows = rows or slice(0, w.L)
    idx = np.arange(w.L)[rows]
    targets = torch.from_numpy(g[idx + 1].astype(np.int64))
    q = torch.from_numpy(np.where(copied[idx + 1], w.q_copy, w.q).astype(np.float32))
    gen = _generator(device, w.seed, b, 1, idx[0] if len(idx) else 0)
    return logits_rows(w, targets, q, gen, device, peaked=peaked, out=out)


def verify_targets(w: Workload, g: np.ndarray, copied: np.ndarray, length: int, drafts: np.ndarray,
                   draft_len: np.ndarray):
    """Targets and peak probabilities of the R verify rows of one sequence at context length `length`.
    Row 0 predicts position `length`; the row after the j-th draft token of candidate c predicts
    position length+j, and gets a peak only while the candidate has followed the stream."""
    R = w.R
    tg = np.full(R, -1, dtype=np.int64)
    qq = np.zeros(R, dtype=np.float32)
    tg[0] = g[length]
    qq[0] = w.q_copy if copied[length] else w.q
    for c in range(w.C):
        on = True
        for j in range(1, w.k + 1):
            if j > draft_len[c]:
                break
            on = on and drafts[c, j - 1] == g[length + j - 1]
            if on:
                P = length + j
                r = 1 + c * w.k + (j - 1)
                tg[r] = g[P]
                qq[r] = w.q_copy if copied[P] else w.q
    return tg, qq


def verify_logits(w: Workload, step: int, gs, copieds, lengths, drafts, draft_len, device, peaked: bool = False,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[B, R, V] verify logits of one decode step ("drawn the same way" as the prefill rows)."""
    tg, qq = [], []
    for b in range(w.B):
        t, q = verify_targets(w, gs[b], copieds[b], int(lengths[b]), drafts[b], draft_len[b])
        tg.append(t); qq.append(q)
    targets = torch.from_numpy(np.concatenate(tg))
    q = torch.from_numpy(np.concatenate(qq))
    gen = _generator(device, w.seed, step, 2)
    flat = None if out is None else out.view(w.B * w.R, w.V)
    z = logits_rows(w, targets, q, gen, device, peaked=peaked, out=flat)
    return z.view(w.B, w.R, w.V)


# --------------------------------------------------------------------------- draft-tree workloads
def tree_stream(w: Workload, b: int):
    """Token stream for the draft-tree path (Sec. 3.2): returns (g, alt, slot).
    g[:L] is the prompt and alt[i] the token the synthetic model prefers at prompt position i: g[i] itself
    (aligned, slot[i] = 0) or another token, the prompt token being the model's second or third choice
    (misaligned, slot[i] = 1 or 2; Sec. 2.3).  The continuation g[L:] repeats prompt material in the
    model's wording (alt), covering w.coverage of it, with novel tokens in between.
    w.motifs = 0: random prompt, a fraction w.mis_rate of its positions misaligned; the continuation copies
    prompt segments of 8..24 tokens.
    w.motifs > 0: the prompt holds instances of w.motifs 12-token motifs, each token of an instance
    replaced with probability 0.1, so that one key has many occurrences whose continuations share prefixes
    and then part; the model's wording of a motif differs from it at a fraction w.mis_rate of its offsets,
    the same ones in every instance; the continuation strings motifs in the model's wording together."""
    rng = np.random.default_rng([w.seed, b, 0x7EE])
    n = w.stream_len
    g = rng.integers(0, w.V, size=n, dtype=np.int64).astype(np.int32)
    alt = g.copy()
    rand_tokens = lambda k: rng.integers(0, w.V, size=k, dtype=np.int64).astype(np.int32)
    if w.motifs > 0:
        pool = rand_tokens(w.motifs * 12).reshape(w.motifs, 12)
        wording = pool.copy()
        differs = rng.random((w.motifs, 12)) < w.mis_rate
        wording[differs] = rand_tokens(int(differs.sum()))
        for pos in range(1, w.L - 12, 12):
            if rng.random() < w.coverage:
                mid = int(rng.integers(0, w.motifs))
                inst = pool[mid].copy()
                change = rng.random(12) < 0.1
                inst[change] = rand_tokens(int(change.sum()))
                g[pos:pos + 12] = inst
                alt[pos:pos + 12] = wording[mid]
        pos = w.L + 2
        while pos + 12 <= n:
            if rng.random() < w.coverage:
                g[pos:pos + 12] = wording[int(rng.integers(0, w.motifs))]
            pos += 12
    else:
        mis = rng.random(w.L) < w.mis_rate
        mis[0] = False
        alt[:w.L][mis] = rand_tokens(int(mis.sum()))
        pos = w.L + 2
        while pos < n:
            ln = min(int(rng.integers(8, 25)), n - pos)
            if rng.random() < w.coverage and w.L > ln + 2:
                s0 = int(rng.integers(1, w.L - ln))
                g[pos:pos + ln] = alt[s0:s0 + ln]
            pos += ln
    alt[0] = g[0]
    alt[w.L:] = g[w.L:]
    slot = np.where(alt != g, 1 + (rng.random(n) < 0.5), 0).astype(np.int64)
    return g, alt, slot


def tree_prefill_logits(w: Workload, b: int, g: np.ndarray, alt: np.ndarray, slot: np.ndarray, device,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Prefill logits for tree_stream: row i predicts position i+1; the prompt token g[i+1] sits at rank
    slot[i+1] and, where it is not the top one, the row's top token is alt[i+1]."""
    idx = np.arange(w.L)
    nxt = np.minimum(idx + 1, w.L - 1)
    targets = torch.from_numpy(g[nxt].astype(np.int64))
    sl = torch.from_numpy(slot[nxt])
    lead = torch.from_numpy(np.where(slot[nxt] > 0, alt[nxt], -1).astype(np.int64))
    gen = _generator(device, w.seed, b, 5)
    return logits_rows(w, targets, torch.zeros(w.L), gen, device, peaked=True, out=out, slot=sl, lead=lead)


def tree_verify_targets(g: np.ndarray, length: int, node_token: np.ndarray, node_parent: np.ndarray,
                        node_depth: np.ndarray, n_nodes: int) -> np.ndarray:
    """Target token of every tree row of one sequence: the row of a node whose path from the root has
    followed the stream g predicts the stream's next token; any other row gets no peak (-1)."""
    N = node_token.shape[0]
    tg = np.full(N, -1, dtype=np.int64)
    on = np.zeros(N, dtype=bool)
    on[0] = True
    tg[0] = g[length]
    for i in range(1, n_nodes):
        pa, d = int(node_parent[i]), int(node_depth[i])
        on[i] = 0 <= pa < i and on[pa] and node_token[i] == g[length + d - 1]
        if on[i]:
            tg[i] = g[length + d]
    return tg


def tree_verify_logits(w: Workload, step: int, gs, lengths, tree: dict, device,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[B, N, V] logits of one tree-verification step; rows at or beyond n_nodes hold noise."""
    B, N = tree["node_token"].shape
    tg = [tree_verify_targets(gs[b], int(lengths[b]), tree["node_token"][b], tree["node_parent"][b],
                              tree["node_depth"][b], int(tree["n_nodes"][b])) for b in range(B)]
    targets = torch.from_numpy(np.concatenate(tg))
    gen = _generator(device, w.seed, step, 6)
    place = torch.rand(B * N, generator=gen, device=device)
    slot = (place >= 0.90).long() + (place >= 0.97).long()   # the stream's token leads the row 9 times in 10
    flat = None if out is None else out.view(B * N, w.V)
    z = logits_rows(w, targets, torch.zeros(B * N), gen, device, peaked=True, out=flat, slot=slot)
    return z.view(B, N, w.V)


# --------------------------------------------------------------------------- host copies for the oracle
def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Device logits -> the same bit patterns on the host (float32, or uint16 for bf16)."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
