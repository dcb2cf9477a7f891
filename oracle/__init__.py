"""ctypes wrapper around the CPU oracle (``aasd_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module: only ``tests/``, the smoke check and the benchmark's ``cpu_baseline``
leg use it.  The oracle shares no code with the HIP library.

All arrays are numpy arrays on the host.  Logits are passed as their raw bit
patterns: ``float32`` arrays for fp32, ``uint16`` arrays for bf16.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_int, c_int32, c_int64, c_uint8, c_uint32, c_uint64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aasd_oracle.c")
_LIB = os.path.join(_HERE, "libaasd_oracle.so")

F32, BF16 = 0, 1
EXTRAS_TOP, EXTRAS_SAMPLE, EXTRAS_GUMBEL = 0, 1, 2
VERIFY_NO_CLAMP = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no intrinsics, single-threaded)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "aasd_oracle.h")))
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_philox4x32_10.restype = None
        for name in ("orc_widen_row", "orc_row_softmax", "orc_row_stats", "orc_align_sample",
                     "orc_retrieve_drafts", "orc_verify", "orc_build_tree", "orc_verify_tree"):
            getattr(_lib, name).restype = c_int
    return _lib


def _ptr(a, ctype):
    if a is None:
        return ctypes.cast(None, POINTER(ctype))
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(POINTER(ctype))


def _dtype_of(logits: np.ndarray) -> int:
    if logits.dtype == np.float32:
        return F32
    if logits.dtype == np.uint16:
        return BF16
    raise TypeError("logits must be float32 (fp32) or uint16 (bf16 bit patterns)")


def philox4x32_10(ctr, key):
    c = (c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = (c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def row_softmax(row: np.ndarray) -> np.ndarray:
    row = np.ascontiguousarray(row)
    p = np.empty(row.shape[0], dtype=np.float64)
    rc = lib().orc_row_softmax(c_void_p(row.ctypes.data), _dtype_of(row), c_int32(row.shape[0]),
                               _ptr(p, c_double))
    assert rc == 0, rc
    return p


def row_stats(row: np.ndarray):
    """-> (m, S, H, argmax) of one row."""
    row = np.ascontiguousarray(row)
    m, S, H, am = c_double(), c_double(), c_double(), c_int32()
    rc = lib().orc_row_stats(c_void_p(row.ctypes.data), _dtype_of(row), c_int32(row.shape[0]),
                             ctypes.byref(m), ctypes.byref(S), ctypes.byref(H), ctypes.byref(am))
    assert rc == 0, rc
    return m.value, S.value, H.value, am.value


def align_sample(logits: np.ndarray, next_tok, m_x: int = 2, c: int = 4, mode: int = EXTRAS_TOP,
                 seed: int = 0, row_id_base: int = 0, V: int | None = None):
    """logits: [rows, row_stride] (float32 or uint16).  Returns a dict of numpy arrays."""
    assert logits.ndim == 2 and logits.flags["C_CONTIGUOUS"]
    rows, row_stride = logits.shape
    V = row_stride if V is None else V
    nt = None if next_tok is None else np.ascontiguousarray(next_tok, dtype=np.int32)
    out = dict(
        argmax=np.empty(rows, np.int32), misaligned=np.empty(rows, np.uint8),
        entropy=np.empty(rows, np.float64), p_next=np.empty(rows, np.float64),
        p_max=np.empty(rows, np.float64), rank=np.empty(rows, np.int32),
        extras=np.empty((rows, m_x), np.int32), n_extras=np.empty(rows, np.uint8),
        draw_margin=np.empty((rows, m_x), np.float64))
    rc = lib().orc_align_sample(
        c_void_p(logits.ctypes.data), _dtype_of(logits), c_int64(rows), c_int32(V), c_int64(row_stride),
        _ptr(nt, c_int32), c_int32(m_x), c_int32(c), c_int(mode), c_uint64(seed), c_uint64(row_id_base),
        _ptr(out["argmax"], c_int32), _ptr(out["misaligned"], c_uint8), _ptr(out["entropy"], c_double),
        _ptr(out["p_next"], c_double), _ptr(out["p_max"], c_double), _ptr(out["rank"], c_int32),
        _ptr(out["extras"], c_int32), _ptr(out["n_extras"], c_uint8), _ptr(out["draw_margin"], c_double))
    if rc != 0:
        raise ValueError(f"orc_align_sample rc={rc}")
    return out


def retrieve_drafts(tokens: np.ndarray, length, prompt_len, n_min: int, n_max: int, k: int, C: int,
                    extras=None, n_extras=None, m_x: int = 0, extras_stride: int = 0):
    """tokens: [B, tok_stride] int32.  Returns a dict of numpy arrays."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    assert tokens.ndim == 2
    B, tok_stride = tokens.shape
    length = np.ascontiguousarray(length, dtype=np.int32)
    prompt_len = np.ascontiguousarray(prompt_len, dtype=np.int32)
    have_x = extras is not None and m_x > 0
    if have_x:
        extras = np.ascontiguousarray(extras, dtype=np.int32)
        n_extras = np.ascontiguousarray(n_extras, dtype=np.uint8)
    out = dict(
        drafts=np.empty((B, C, k), np.int32), draft_len=np.empty((B, C), np.int32),
        src_pos=np.empty((B, C), np.int32), n_cand=np.empty(B, np.int32), key_len=np.empty(B, np.int32),
        strict=np.empty((B, C, k), np.uint8),
        draft_extras=np.empty((B, C, k, m_x), np.int32) if have_x else None)
    rc = lib().orc_retrieve_drafts(
        _ptr(tokens, c_int32), c_int64(tok_stride), _ptr(length, c_int32), _ptr(prompt_len, c_int32),
        c_int32(B), c_int32(n_min), c_int32(n_max), c_int32(k), c_int32(C),
        _ptr(extras if have_x else None, c_int32), _ptr(n_extras if have_x else None, c_uint8),
        c_int32(m_x), c_int64(extras_stride),
        _ptr(out["drafts"], c_int32), _ptr(out["draft_len"], c_int32), _ptr(out["src_pos"], c_int32),
        _ptr(out["n_cand"], c_int32), _ptr(out["key_len"], c_int32),
        _ptr(out["draft_extras"], c_int32), _ptr(out["strict"], c_uint8))
    if rc != 0:
        raise ValueError(f"orc_retrieve_drafts rc={rc}")
    return out


def verify(logits: np.ndarray, drafts, draft_len, strict=None, alpha: float = 0.1, beta: float = 0.1,
           flags: int = 0, V: int | None = None):
    """logits: [B, R, row_stride] with R = 1 + C*k; drafts [B, C, k]; draft_len [B, C].

    alpha/beta are used exactly as given (pass float32-rounded values to mirror
    an fp32 caller)."""
    assert logits.ndim == 3 and logits.flags["C_CONTIGUOUS"]
    B, R, row_stride = logits.shape
    V = row_stride if V is None else V
    drafts = np.ascontiguousarray(drafts, dtype=np.int32)
    draft_len = np.ascontiguousarray(draft_len, dtype=np.int32)
    _, C, k = drafts.shape
    assert R == 1 + C * k, (R, C, k)
    st = None if strict is None else np.ascontiguousarray(strict, dtype=np.uint8)
    out = dict(
        accept_len=np.empty(B, np.int32), best_cand=np.empty(B, np.int32), next_token=np.empty(B, np.int32),
        row_entropy=np.empty((B, R), np.float64), row_pmax=np.empty((B, R), np.float64),
        row_argmax=np.empty((B, R), np.int32), tok_p=np.empty((B, C, k), np.float64),
        tok_delta=np.empty((B, C, k), np.float64), tok_margin=np.empty((B, C, k), np.float64),
        near_count=np.empty(B, np.uint32))
    rc = lib().orc_verify(
        c_void_p(logits.ctypes.data), _dtype_of(logits), c_int32(B), c_int32(C), c_int32(k), c_int32(V),
        c_int64(row_stride), c_int64(R * row_stride), _ptr(drafts, c_int32), _ptr(draft_len, c_int32),
        _ptr(st, c_uint8), c_double(alpha), c_double(beta), c_uint32(flags),
        _ptr(out["accept_len"], c_int32), _ptr(out["best_cand"], c_int32), _ptr(out["next_token"], c_int32),
        _ptr(out["row_entropy"], c_double), _ptr(out["row_pmax"], c_double), _ptr(out["row_argmax"], c_int32),
        _ptr(out["tok_p"], c_double), _ptr(out["tok_delta"], c_double), _ptr(out["tok_margin"], c_double),
        _ptr(out["near_count"], c_uint32))
    if rc != 0:
        raise ValueError(f"orc_verify rc={rc}")
    return out


def verify_topk(logits: np.ndarray, drafts, draft_len, topk: int = 5, V: int | None = None):
    """Top-k verification (Sec. 4.4): logits [B, R, row_stride], R = 1 + C*k; drafts [B,C,k]; draft_len [B,C]."""
    assert logits.ndim == 3 and logits.flags["C_CONTIGUOUS"]
    B, R, row_stride = logits.shape
    V = row_stride if V is None else V
    drafts = np.ascontiguousarray(drafts, dtype=np.int32)
    draft_len = np.ascontiguousarray(draft_len, dtype=np.int32)
    _, C, k = drafts.shape
    assert R == 1 + C * k, (R, C, k)
    out = dict(accept_len=np.empty(B, np.int32), best_cand=np.empty(B, np.int32), next_token=np.empty(B, np.int32),
               row_argmax=np.empty((B, R), np.int32), tok_rank=np.empty((B, C, k), np.int32))
    rc = lib().orc_verify_topk(
        c_void_p(logits.ctypes.data), _dtype_of(logits), c_int32(B), c_int32(C), c_int32(k), c_int32(V),
        c_int64(row_stride), c_int64(R * row_stride), _ptr(drafts, c_int32), _ptr(draft_len, c_int32), c_int32(topk),
        _ptr(out["accept_len"], c_int32), _ptr(out["best_cand"], c_int32), _ptr(out["next_token"], c_int32),
        _ptr(out["row_argmax"], c_int32), _ptr(out["tok_rank"], c_int32))
    if rc != 0:
        raise ValueError(f"orc_verify_topk rc={rc}")
    return out


def build_tree(drafts, draft_len, strict=None, draft_extras=None, root_tok=None, max_nodes: int = 64):
    """drafts [B,C,k], draft_len [B,C], strict [B,C,k] or None, draft_extras [B,C,k,m] or None."""
    drafts = np.ascontiguousarray(drafts, dtype=np.int32)
    draft_len = np.ascontiguousarray(draft_len, dtype=np.int32)
    B, C, k = drafts.shape
    st = None if strict is None else np.ascontiguousarray(strict, dtype=np.uint8)
    dx = None if draft_extras is None else np.ascontiguousarray(draft_extras, dtype=np.int32)
    m_x = 0 if dx is None else dx.shape[3]
    rt = None if root_tok is None else np.ascontiguousarray(root_tok, dtype=np.int32)
    N, W = max_nodes, (max_nodes + 31) // 32
    out = dict(
        node_token=np.empty((B, N), np.int32), node_parent=np.empty((B, N), np.int32),
        node_depth=np.empty((B, N), np.int32), node_strict=np.empty((B, N), np.uint8),
        n_nodes=np.empty(B, np.int32), mask=np.empty((B, N, W), np.uint32), cand_node=np.empty((B, C, k), np.int32))
    rc = lib().orc_build_tree(
        _ptr(drafts, c_int32), _ptr(draft_len, c_int32), _ptr(st, c_uint8), _ptr(dx, c_int32), c_int32(m_x),
        _ptr(rt, c_int32), c_int32(B), c_int32(C), c_int32(k), c_int32(N),
        _ptr(out["node_token"], c_int32), _ptr(out["node_parent"], c_int32), _ptr(out["node_depth"], c_int32),
        _ptr(out["node_strict"], c_uint8), _ptr(out["n_nodes"], c_int32), _ptr(out["mask"], c_uint32),
        _ptr(out["cand_node"], c_int32))
    if rc != 0:
        raise ValueError(f"orc_build_tree rc={rc}")
    return out


def verify_tree(logits: np.ndarray, node_token, node_parent, node_strict, n_nodes, alpha: float = 0.1,
                beta: float = 0.1, flags: int = 0, V: int | None = None):
    """logits [B, N, row_stride]; node arrays [B, N]."""
    assert logits.ndim == 3 and logits.flags["C_CONTIGUOUS"]
    B, N, row_stride = logits.shape
    V = row_stride if V is None else V
    nt = np.ascontiguousarray(node_token, dtype=np.int32)
    npar = np.ascontiguousarray(node_parent, dtype=np.int32)
    ns = None if node_strict is None else np.ascontiguousarray(node_strict, dtype=np.uint8)
    nn = np.ascontiguousarray(n_nodes, dtype=np.int32)
    out = dict(
        accept_len=np.empty(B, np.int32), best_node=np.empty(B, np.int32), accept_path=np.empty((B, 16), np.int32),
        next_token=np.empty(B, np.int32), row_entropy=np.empty((B, N), np.float64), row_pmax=np.empty((B, N), np.float64),
        row_argmax=np.empty((B, N), np.int32), node_p=np.empty((B, N), np.float64), node_delta=np.empty((B, N), np.float64),
        node_margin=np.empty((B, N), np.float64), near_count=np.empty(B, np.uint32))
    rc = lib().orc_verify_tree(
        c_void_p(logits.ctypes.data), _dtype_of(logits), c_int32(B), c_int32(N), c_int32(V), c_int64(row_stride),
        c_int64(N * row_stride), _ptr(nt, c_int32), _ptr(npar, c_int32), _ptr(ns, c_uint8), _ptr(nn, c_int32),
        c_double(alpha), c_double(beta), c_uint32(flags),
        _ptr(out["accept_len"], c_int32), _ptr(out["best_node"], c_int32), _ptr(out["accept_path"], c_int32),
        _ptr(out["next_token"], c_int32), _ptr(out["row_entropy"], c_double), _ptr(out["row_pmax"], c_double),
        _ptr(out["row_argmax"], c_int32), _ptr(out["node_p"], c_double), _ptr(out["node_delta"], c_double),
        _ptr(out["node_margin"], c_double), _ptr(out["near_count"], c_uint32))
    if rc != 0:
        raise ValueError(f"orc_verify_tree rc={rc}")
    return out
