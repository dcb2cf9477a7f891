"""Randomized parity: for every seed a random mix of shapes, element types, value distributions and parameters
goes through every entry point and is compared with the oracle.  The fixed cases elsewhere pin the known edge
cases; this one guards against the combinations nobody thought of (a longer run of the same generator, over
several hundred seeds, found that align_sample left n_extras undefined for m = 0)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_13204_amd as aasd
from tests import synth
from tests import backends as bk
from tests import test_gpu_parity as P
from tests import test_gpu_tree as T

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _t(a, dt):
    return None if a is None else torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)


@pytest.mark.parametrize("seed", range(24))
def test_random_rows_candidates_and_trees(seed):
    rng = np.random.default_rng(1000 + seed)
    tally = bk.Tally()
    V = int(rng.choice([37, 1000, 4099, 32000, 50257, 128256]))
    rows = int(rng.integers(1, 300 if V < 60000 else 60))
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    z = P._random_rows(rng, rows, V, dtype, sigma=float(rng.uniform(0.5, 4.0)), coarse=bool(rng.random() < 0.3))
    if rng.random() < 0.5:      # LLM-like peaks
        for r in range(rows):
            idx = rng.choice(V, min(4, V), replace=False)
            z[r, idx] = torch.tensor([24.0, 23.0, 22.0, 21.0][:len(idx)], device=DEV, dtype=z.dtype)
    nt = rng.integers(-1, V, size=rows).astype(np.int32)
    m = int(rng.integers(0, 5))
    c = int(rng.integers(max(m, 1), 9))
    for mode in (oracle.EXTRAS_TOP, oracle.EXTRAS_SAMPLE, oracle.EXTRAS_GUMBEL):
        got = bk.hip_align(z, nt, m, c, mode, seed=seed, row_id_base=seed * 1000)
        ref = bk.oracle_align(z, nt, m, c, mode, seed=seed, row_id_base=seed * 1000)
        bk.compare_align(got, ref, tally, mode)
    B, C, k = int(rng.integers(1, 6)), int(rng.integers(1, 9)), int(rng.integers(1, 9))
    Vv = int(rng.choice([50, 2000, 32000]))
    zd, drafts, dl, strict = P._verify_case(rng, B, C, k, Vv, dtype, peaked=bool(rng.random() < 0.7))
    P._verify_both(zd, drafts, dl, strict if rng.random() < 0.5 else None, float(rng.uniform(0, 0.3)),
                   float(rng.uniform(0, 0.3)), int(rng.random() < 0.2), tally)
    topk = int(rng.integers(1, 9))
    ref = oracle.verify_topk(synth.to_host_bits(zd), drafts, dl, topk=topk)
    got = bk.to_np(aasd.verify_topk(zd, _t(drafts, torch.int32), _t(dl, torch.int32), topk=topk))
    for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    mm, N = int(rng.integers(0, 4)), int(rng.integers(2, 80))
    d2, dl2, st2, dx2 = T._random_candidates(rng, B, C, k, mm, alphabet=int(rng.integers(2, 30)))
    tree = T._build_both(d2, dl2, st2, dx2, np.zeros(B, np.int32), N)
    zt = T._tree_logits(rng, tree, Vv, dtype, peaked=bool(rng.random() < 0.7), p_lead=float(rng.random()))
    T._verify_tree_both(zt, tree, tree["node_strict"], float(rng.uniform(0, 0.3)), float(rng.uniform(0, 0.3)), 0, tally)


@pytest.mark.parametrize("seed", range(24))
def test_random_contexts_scan_and_pool(seed):
    rng = np.random.default_rng(2000 + seed)
    B = int(rng.integers(1, 9))
    cap = int(rng.choice([5, 64, 700, 3000, 12000, 25000]))
    toks = rng.integers(0, int(rng.choice([2, 3, 8, 100, 50000])), size=(B, cap)).astype(np.int32)
    for b in range(B):          # planted repeats
        for _ in range(int(rng.integers(0, 6))):
            ln = int(rng.integers(1, max(2, min(60, cap // 3))))
            if cap > 2 * ln + 2:
                s = int(rng.integers(0, cap - 2 * ln))
                d = int(rng.integers(s + ln, cap - ln + 1))
                toks[b, d:d + ln] = toks[b, s:s + ln]
    n_min = int(rng.integers(1, 5))
    n_max = int(rng.integers(n_min, 9))
    k, C, m = int(rng.integers(1, 17)), int(rng.integers(1, 33)), int(rng.integers(0, 4))
    L0 = int(rng.integers(1, cap + 1))
    extras = n_extras = None
    if m:
        extras = rng.integers(0, 99, size=(B * L0, m)).astype(np.int32)
        n_extras = rng.integers(0, m + 1, size=B * L0).astype(np.uint8)
        extras[np.arange(m)[None, :] >= n_extras[:, None]] = -1
    td = _t(toks, torch.int32)
    pool = aasd.DraftPool(B, cap, n_min, n_max, DEV)
    lens = np.minimum(rng.integers(0, L0 + 1, size=B), cap).astype(np.int32)
    plens = np.minimum(lens, rng.integers(0, cap + 1, size=B)).astype(np.int32)
    first = True
    for step in range(int(rng.integers(1, 8))):
        ref = oracle.retrieve_drafts(toks, lens, plens, n_min, n_max, k, C, extras=extras, n_extras=n_extras, m_x=m,
                                     extras_stride=L0)
        kw = dict(extras=_t(extras, torch.int32), n_extras=_t(n_extras, torch.uint8), m=m, extras_stride=L0)
        got = aasd.retrieve_drafts(td, _t(lens, torch.int32), _t(plens, torch.int32), n_min, n_max, k, C, **kw)
        bk.compare_retrieve(bk.to_np(got), ref)
        if first or rng.random() < 0.3:
            pool.update(td, _t(lens, torch.int32), reset=first or rng.random() < 0.2)
            gotp = pool.retrieve(td, _t(lens, torch.int32), _t(plens, torch.int32), k, C, **kw)
        else:
            gotp = pool.step(td, _t(lens, torch.int32), _t(plens, torch.int32), k, C, **kw)
        first = False
        torch.cuda.synchronize()
        bk.compare_retrieve(bk.to_np(gotp), ref)
        lens = np.minimum(lens + rng.integers(0, 20, size=B), cap).astype(np.int32)
