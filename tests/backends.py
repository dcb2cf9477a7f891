"""Backends of the synthetic decode driver used by the tests, and the parity comparators.

OracleBackend runs the CPU oracle; HipBackend runs the HIP library through the Python binding;
ParityBackend runs both on the same bits, asserts parity at every call and returns the oracle's
results, so that a decode loop stays on the oracle's trajectory.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2505_13204_amd as aasd
from tests import harness, synth

NEAR = 1e-6        # decisions whose oracle margin is below this are counted, not compared
NEAR_GUMBEL = 5e-5 # the same for Gumbel-top-k draws: gap between neighbouring keys z + G (fp32 keys err by < 1e-5)
REL_TOL = 1e-5     # probabilities and entropies
P_FLOOR = 1e-30
H_FLOOR = 0.05     # nats: below this the entropy is compared absolutely (5e-7); fp32 S resolves ln S to ~1e-7


def f32(x) -> float:
    return float(np.float32(x))


def rel_err(got, ref, floor):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.abs(got - ref) / np.maximum(np.abs(ref), floor)


class Tally:
    """Accumulates what the parity report needs: worst errors and near-threshold counts."""

    def __init__(self):
        self.max_rel_p = 0.0
        self.max_rel_h = 0.0
        self.near_decisions = 0
        self.near_disagreements = 0
        self.rows = 0
        self.tokens = 0

    def __repr__(self):
        return (f"rows={self.rows} tokens={self.tokens} max_rel_p={self.max_rel_p:.2e} max_rel_H={self.max_rel_h:.2e} "
                f"near={self.near_decisions} near_disagree={self.near_disagreements}")


# --------------------------------------------------------------------------- comparators
def compare_align(got: dict, ref: dict, tally: Tally, mode: int):
    """got: numpy copies of the HIP outputs; ref: oracle outputs."""
    np.testing.assert_array_equal(got["argmax"], ref["argmax"])
    np.testing.assert_array_equal(got["misaligned"], ref["misaligned"])
    if got.get("rank") is not None:
        np.testing.assert_array_equal(got["rank"], ref["rank"])
    e_h = rel_err(got["entropy"], ref["entropy"], H_FLOOR)
    e_p = np.maximum(rel_err(got["p_max"], ref["p_max"], P_FLOOR), rel_err(got["p_next"], ref["p_next"], P_FLOOR))
    tally.max_rel_h = max(tally.max_rel_h, float(e_h.max(initial=0.0)))
    tally.max_rel_p = max(tally.max_rel_p, float(e_p.max(initial=0.0)))
    assert e_h.max(initial=0.0) <= REL_TOL, f"entropy rel err {e_h.max():.3e} at row {int(e_h.argmax())}"
    assert e_p.max(initial=0.0) <= REL_TOL, f"probability rel err {e_p.max():.3e} at row {int(e_p.argmax())}"
    tally.rows += len(ref["argmax"])
    np.testing.assert_array_equal(got["n_extras"], ref["n_extras"])
    if ref["extras"].shape[1] == 0:
        return
    if mode == oracle.EXTRAS_TOP:
        np.testing.assert_array_equal(got["extras"], ref["extras"])
        return
    # SAMPLE / GUMBEL: rows whose draws all stay clear of a CDF edge / of the next key must agree exactly
    margin = np.where(ref["draw_margin"] < 0, np.inf, ref["draw_margin"]).min(axis=1)
    near = margin < (NEAR_GUMBEL if mode == oracle.EXTRAS_GUMBEL else NEAR)
    tally.near_decisions += int(near.sum())
    same = (got["extras"] == ref["extras"]).all(axis=1)
    assert same[~near].all(), f"sampled extras differ at rows {np.nonzero(~same & ~near)[0][:8]}"
    tally.near_disagreements += int((~same & near).sum())


def compare_retrieve(got: dict, ref: dict):
    for name in ("n_cand", "key_len", "src_pos", "draft_len", "drafts", "strict"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    if ref.get("draft_extras") is not None:
        np.testing.assert_array_equal(got["draft_extras"], ref["draft_extras"], err_msg="draft_extras")


def compare_verify(got: dict, ref: dict, tally: Tally):
    np.testing.assert_array_equal(got["row_argmax"], ref["row_argmax"])
    e_h = rel_err(got["row_entropy"], ref["row_entropy"], H_FLOOR)
    e_p = rel_err(got["row_pmax"], ref["row_pmax"], P_FLOOR)
    assert e_h.max(initial=0.0) <= REL_TOL, f"row entropy rel err {e_h.max():.3e}"
    assert e_p.max(initial=0.0) <= REL_TOL, f"row p_max rel err {e_p.max():.3e}"
    e_tp = rel_err(got["tok_p"], ref["tok_p"], P_FLOOR)
    e_td = rel_err(got["tok_delta"], ref["tok_delta"], P_FLOOR)
    assert e_tp.max(initial=0.0) <= REL_TOL, f"token p rel err {e_tp.max():.3e}"
    assert e_td.max(initial=0.0) <= REL_TOL, f"token delta rel err {e_td.max():.3e}"
    tally.max_rel_h = max(tally.max_rel_h, float(e_h.max(initial=0.0)))
    tally.max_rel_p = max(tally.max_rel_p, float(max(e_p.max(initial=0.0), e_tp.max(initial=0.0), e_td.max(initial=0.0))))
    tally.rows += ref["row_argmax"].size
    tally.tokens += int((ref["tok_margin"] >= 0).sum())
    # decisions: exact unless the oracle's margin of some evaluated token of the sequence is below NEAR
    B = len(ref["accept_len"])
    margin = np.where(ref["tok_margin"] < 0, np.inf, ref["tok_margin"]).reshape(B, -1).min(axis=1)
    near = margin < NEAR
    tally.near_decisions += int((ref["tok_margin"] >= 0).__and__(ref["tok_margin"] < NEAR).sum())
    same = ((got["accept_len"] == ref["accept_len"]) & (got["best_cand"] == ref["best_cand"])
            & (got["next_token"] == ref["next_token"]))
    assert same[~near].all(), f"decisions differ at sequences {np.nonzero(~same & ~near)[0][:8]}"
    tally.near_disagreements += int((~same & near).sum())
    # the kernel's own near counter brackets the oracle's (its margins differ from the oracle's by rounding)
    if got.get("near_count") is not None:
        lo = ((ref["tok_margin"] >= 0) & (ref["tok_margin"] < 0.5 * NEAR)).reshape(B, -1).sum(axis=1)
        hi = ((ref["tok_margin"] >= 0) & (ref["tok_margin"] < 2.0 * NEAR)).reshape(B, -1).sum(axis=1)
        ok = (got["near_count"] >= lo) & (got["near_count"] <= hi)
        assert ok[same].all()


def compare_tree(got: dict, ref: dict):
    for name in ("n_nodes", "node_token", "node_parent", "node_depth", "node_strict", "cand_node", "mask"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)


def compare_verify_tree(got: dict, ref: dict, tally: Tally):
    np.testing.assert_array_equal(got["row_argmax"], ref["row_argmax"])
    e_h = rel_err(got["row_entropy"], ref["row_entropy"], H_FLOOR)
    e_p = rel_err(got["row_pmax"], ref["row_pmax"], P_FLOOR)
    e_np = rel_err(got["node_p"], ref["node_p"], P_FLOOR)
    e_nd = rel_err(got["node_delta"], ref["node_delta"], P_FLOOR)
    for name, e in (("row entropy", e_h), ("row p_max", e_p), ("node p", e_np), ("node delta", e_nd)):
        assert e.max(initial=0.0) <= REL_TOL, f"{name} rel err {e.max():.3e}"
    tally.max_rel_h = max(tally.max_rel_h, float(e_h.max(initial=0.0)))
    tally.max_rel_p = max(tally.max_rel_p, float(max(e_p.max(initial=0.0), e_np.max(initial=0.0), e_nd.max(initial=0.0))))
    tally.rows += int((ref["row_argmax"] >= 0).sum())
    ev = ref["node_margin"] >= 0                     # nodes that were evaluated: all ancestors accepted
    tally.tokens += int(ev.sum())
    B = len(ref["accept_len"])
    near = (np.where(ev, ref["node_margin"], np.inf).reshape(B, -1).min(axis=1)) < NEAR
    tally.near_decisions += int((ev & (ref["node_margin"] < NEAR)).sum())
    same = ((got["accept_len"] == ref["accept_len"]) & (got["best_node"] == ref["best_node"])
            & (got["next_token"] == ref["next_token"]) & (got["accept_path"] == ref["accept_path"]).all(axis=1))
    assert same[~near].all(), f"tree decisions differ at sequences {np.nonzero(~same & ~near)[0][:8]}"
    tally.near_disagreements += int((~same & near).sum())
    if got.get("near_count") is not None:
        lo = (ev & (ref["node_margin"] < 0.5 * NEAR)).reshape(B, -1).sum(axis=1)
        hi = (ev & (ref["node_margin"] < 2.0 * NEAR)).reshape(B, -1).sum(axis=1)
        ok = (got["near_count"] >= lo) & (got["near_count"] <= hi)
        assert ok[same].all()


# --------------------------------------------------------------------------- host/device helpers
def to_np(d: dict) -> dict:
    return {k: (v.cpu().numpy() if isinstance(v, torch.Tensor) else v) for k, v in d.items() if k != "workspace"}


def hip_align(logits_dev, next_tok, m, c, mode, seed=0, row_id_base=0, V=None, want_rank=True):
    nt = None if next_tok is None else torch.as_tensor(np.asarray(next_tok, dtype=np.int32), device=logits_dev.device)
    out = aasd.align_sample(logits_dev, nt, m=m, c=c, mode=mode, seed=seed, row_id_base=row_id_base, V=V,
                            want_rank=want_rank)
    torch.cuda.synchronize()
    return to_np(out)


def oracle_align(logits_dev, next_tok, m, c, mode, seed=0, row_id_base=0, V=None):
    bits = synth.to_host_bits(logits_dev)
    return oracle.align_sample(bits, next_tok, m_x=m, c=c, mode=mode, seed=seed, row_id_base=row_id_base, V=V)


# --------------------------------------------------------------------------- driver backends
class OracleBackend(harness.Backend):
    def __init__(self, device="cpu"):
        self.device = device

    def retrieve(self, tokens, length, prompt_len, w, extras, n_extras):
        return oracle.retrieve_drafts(tokens, length, prompt_len, w.n_min, w.n_max, w.k, w.C, extras=extras,
                                      n_extras=n_extras, m_x=w.m if extras is not None else 0, extras_stride=w.L)

    def make_logits(self, w, step, gs, copieds, length, drafts, draft_len, peaked):
        return synth.to_host_bits(synth.verify_logits(w, step, gs, copieds, length, drafts, draft_len, self.device,
                                                      peaked=peaked))

    def verify(self, logits, drafts, draft_len, strict, w):
        return oracle.verify(logits, drafts, draft_len, strict, alpha=f32(w.alpha), beta=f32(w.beta))


    def build_tree(self, r, root_tok, max_nodes):
        return oracle.build_tree(r["drafts"], r["draft_len"], r["strict"], r.get("draft_extras"), root_tok=root_tok,
                                 max_nodes=max_nodes)

    def make_tree_logits(self, w, step, gs, length, tree):
        return synth.to_host_bits(synth.tree_verify_logits(w, step, gs, length, tree, self.device))

    def verify_tree(self, logits, tree, w):
        return oracle.verify_tree(logits, tree["node_token"], tree["node_parent"], tree["node_strict"], tree["n_nodes"],
                                  alpha=f32(w.alpha), beta=f32(w.beta))


class HipBackend(harness.Backend):
    def __init__(self, device="cuda:0", one_launch=False):
        self.device = torch.device(device)
        self.one_launch = one_launch      # aasd_verify in its one-launch form, over a zero-filled workspace kept per shape
        self._ws = {}

    def _dev(self, a, dtype):
        return torch.as_tensor(np.ascontiguousarray(a), device=self.device).to(dtype)

    def retrieve(self, tokens, length, prompt_len, w, extras, n_extras):
        have = extras is not None
        out = aasd.retrieve_drafts(
            self._dev(tokens, torch.int32), self._dev(length, torch.int32), self._dev(prompt_len, torch.int32),
            w.n_min, w.n_max, w.k, w.C,
            extras=self._dev(extras, torch.int32) if have else None,
            n_extras=self._dev(n_extras, torch.uint8) if have else None,
            m=w.m if have else 0, extras_stride=w.L)
        torch.cuda.synchronize()
        return to_np(out)

    def make_logits(self, w, step, gs, copieds, length, drafts, draft_len, peaked):
        return synth.verify_logits(w, step, gs, copieds, length, drafts, draft_len, self.device, peaked=peaked)

    def verify(self, logits, drafts, draft_len, strict, w):
        kw = {}
        if self.one_launch:
            B, C, k = drafts.shape
            key = (B, C, k, logits.shape[2], logits.dtype)
            if key not in self._ws:
                nbytes = aasd.verify_workspace_bytes(B, C, k, logits.shape[2], aasd.BF16 if logits.dtype == torch.bfloat16 else aasd.F32)
                self._ws[key] = torch.zeros(nbytes, dtype=torch.uint8, device=self.device)
            kw = dict(workspace=self._ws[key], zeroed_workspace=True)
        out = aasd.verify(logits, self._dev(drafts, torch.int32), self._dev(draft_len, torch.int32),
                          self._dev(strict, torch.uint8), alpha=w.alpha, beta=w.beta, **kw)
        torch.cuda.synchronize()
        return to_np(out)


    def build_tree(self, r, root_tok, max_nodes):
        dx = r.get("draft_extras")
        out = aasd.build_tree(self._dev(r["drafts"], torch.int32), self._dev(r["draft_len"], torch.int32),
                              self._dev(r["strict"], torch.uint8), None if dx is None else self._dev(dx, torch.int32),
                              self._dev(root_tok, torch.int32), max_nodes=max_nodes)
        torch.cuda.synchronize()
        t = to_np(out)
        t["mask"] = t["mask"].view(np.uint32)
        return t

    def make_tree_logits(self, w, step, gs, length, tree):
        return synth.tree_verify_logits(w, step, gs, length, tree, self.device)

    def verify_tree(self, logits, tree, w):
        out = aasd.verify_tree(logits, self._dev(tree["node_token"], torch.int32), self._dev(tree["node_parent"], torch.int32),
                               self._dev(tree["n_nodes"], torch.int32), self._dev(tree["node_strict"], torch.uint8),
                               alpha=w.alpha, beta=w.beta)
        torch.cuda.synchronize()
        return to_np(out)


class ParityBackend(harness.Backend):
    """Runs both, asserts parity on every call, returns the oracle's results."""

    def __init__(self, device="cuda:0", one_launch=False):
        self.hip = HipBackend(device, one_launch=one_launch)
        self.orc = OracleBackend()
        self.tally = Tally()

    def retrieve(self, tokens, length, prompt_len, w, extras, n_extras):
        ref = self.orc.retrieve(tokens, length, prompt_len, w, extras, n_extras)
        got = self.hip.retrieve(tokens, length, prompt_len, w, extras, n_extras)
        compare_retrieve(got, ref)
        return ref

    def make_logits(self, w, step, gs, copieds, length, drafts, draft_len, peaked):
        dev = self.hip.make_logits(w, step, gs, copieds, length, drafts, draft_len, peaked)
        return dev, synth.to_host_bits(dev)

    def verify(self, logits, drafts, draft_len, strict, w):
        dev, bits = logits
        ref = self.orc.verify(bits, drafts, draft_len, strict, w)
        got = self.hip.verify(dev, drafts, draft_len, strict, w)
        compare_verify(got, ref, self.tally)
        return ref

    def build_tree(self, r, root_tok, max_nodes):
        ref = self.orc.build_tree(r, root_tok, max_nodes)
        got = self.hip.build_tree(r, root_tok, max_nodes)
        compare_tree(got, ref)
        return ref

    def make_tree_logits(self, w, step, gs, length, tree):
        dev = self.hip.make_tree_logits(w, step, gs, length, tree)
        return dev, synth.to_host_bits(dev)

    def verify_tree(self, logits, tree, w):
        dev, bits = logits
        ref = self.orc.verify_tree(bits, tree, w)
        got = self.hip.verify_tree(dev, tree, w)
        compare_verify_tree(got, ref, self.tally)
        return ref


# --------------------------------------------------------------------------- the oracle over many rows
# The oracle is single-threaded C without global state, and ctypes releases the interpreter lock during a
# call: disjoint ranges of rows (or of sequences) can be handed to a few host threads.  Every range is still
# computed by the same plain code; the threads share nothing but read-only inputs.
def host_threads() -> int:
    import os
    return max(1, min(16, os.cpu_count() or 1))


def _ranges(n, parts):
    parts = max(1, min(parts, n))
    edges = np.linspace(0, n, parts + 1).astype(np.int64)
    return [(int(a), int(b)) for a, b in zip(edges[:-1], edges[1:]) if b > a]


def oracle_align_rows(bits, next_tok, m, c, mode, seed=0, row_id_base=0, V=None):
    """oracle.align_sample over all rows of `bits`, row ranges spread over the host's threads."""
    from concurrent.futures import ThreadPoolExecutor
    rows = bits.shape[0]
    nt = None if next_tok is None else np.asarray(next_tok, dtype=np.int32)
    rs = _ranges(rows, host_threads() * 4)
    def run(ab):
        a, b = ab
        return oracle.align_sample(bits[a:b], None if nt is None else nt[a:b], m_x=m, c=c, mode=mode, seed=seed,
                                   row_id_base=row_id_base + a, V=V)
    with ThreadPoolExecutor(host_threads()) as ex:
        parts = list(ex.map(run, rs))
    return {k: np.concatenate([p[k] for p in parts]) for k in parts[0]}


def oracle_verify_seqs(bits, drafts, draft_len, strict, alpha, beta, flags=0):
    """oracle.verify over all sequences of `bits` [B, R, V], sequence ranges spread over the host's threads."""
    from concurrent.futures import ThreadPoolExecutor
    B = bits.shape[0]
    rs = _ranges(B, host_threads() * 2)
    def run(ab):
        a, b = ab
        return oracle.verify(bits[a:b], drafts[a:b], draft_len[a:b], None if strict is None else strict[a:b],
                             alpha=alpha, beta=beta, flags=flags)
    with ThreadPoolExecutor(host_threads()) as ex:
        parts = list(ex.map(run, rs))
    return {k: np.concatenate([p[k] for p in parts]) for k in parts[0]}
