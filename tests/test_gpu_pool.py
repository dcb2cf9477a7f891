"""The persistent draft pool (Algorithm 1's dictionary with incremental update) on the GPU returns exactly
what the stateless oracle retrieval returns, after a full build and after every incremental update."""
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
    return None if a is None else torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)


def _check(pool, toks_d, toks, lens, plens, n_min, n_max, k, C, extras=None, n_extras=None, m=0, xs=0):
    ref = oracle.retrieve_drafts(toks, lens, plens, n_min, n_max, k, C, extras=extras, n_extras=n_extras, m_x=m,
                                 extras_stride=xs)
    out = pool.retrieve(toks_d, _t(lens, torch.int32), _t(plens, torch.int32), k, C, extras=_t(extras, torch.int32),
                        n_extras=_t(n_extras, torch.uint8), m=m, extras_stride=xs)
    torch.cuda.synchronize()
    bk.compare_retrieve(bk.to_np(out), ref)
    return ref


@pytest.mark.parametrize("n_min,n_max,k,C", [(1, 1, 1, 1), (1, 6, 6, 4), (3, 3, 4, 2), (2, 4, 8, 16), (1, 8, 16, 32)])
@pytest.mark.parametrize("cap", [1, 90, 1500, 30011])
def test_pool_full_build_random_small_alphabet(n_min, n_max, k, C, cap):
    rng = np.random.default_rng(cap + n_max)
    B = 12
    alphabet = 3 if cap < 2000 else 40
    toks = rng.integers(0, alphabet, size=(B, cap)).astype(np.int32)
    lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
    lens[0], lens[1] = cap, 0
    plens = np.minimum(lens, rng.integers(0, cap + 1, size=B)).astype(np.int32)
    pool = aasd.DraftPool(B, cap, n_min, n_max, DEV)
    toks_d = _t(toks, torch.int32)
    pool.update(toks_d, _t(lens, torch.int32), reset=True)
    ref = _check(pool, toks_d, toks, lens, plens, n_min, n_max, k, C)
    if cap >= 1500:
        assert (ref["n_cand"] > 0).any()
    # a lookup at a shorter context than was indexed ignores the later positions
    shorter = (lens * 0.7).astype(np.int32)
    _check(pool, toks_d, toks, shorter, np.minimum(plens, shorter), n_min, n_max, k, C)
    # a second full build over the same memory starts from nothing
    toks2 = rng.integers(0, alphabet, size=(B, cap)).astype(np.int32)
    toks2_d = _t(toks2, torch.int32)
    pool.update(toks2_d, _t(lens, torch.int32), reset=True)
    _check(pool, toks2_d, toks2, lens, plens, n_min, n_max, k, C)


@pytest.mark.parametrize("alphabet", [2, 6, 5000])
def test_pool_build_in_pieces_and_many_keys(alphabet):
    """The build path taken for many positions at once (tiles of 8192, batches of 64): from empty tables, continued
    without a reset across a tile boundary, then by a decode step's few tokens.  After each, lookups at 24 different
    context lengths (so 24 different keys per sequence and key length) with C = 32 walk many chains to depth 32."""
    rng = np.random.default_rng(alphabet)
    B, cap, n_min, n_max, k, C = 5, 20000, 1, 5, 4, 32
    toks = rng.integers(0, alphabet, size=(B, cap)).astype(np.int32)
    for b in range(B):    # long repeats, so that the longest keys have several occurrences
        for _ in range(30):
            ln = int(rng.integers(5, 200))
            s = int(rng.integers(0, cap - 2 * ln))
            d = int(rng.integers(s + ln, cap - ln + 1))
            toks[b, d:d + ln] = toks[b, s:s + ln]
    toks_d = _t(toks, torch.int32)
    pool = aasd.DraftPool(B, cap, n_min, n_max, DEV)
    stages = [np.array([3000, 64, 8191, 9000, 70], np.int32), np.array([12000, 8300, 8192, 19999, 71], np.int32),
              np.array([12040, 8364, 8200, 20000, 20000], np.int32)]
    for si, lens in enumerate(stages):
        pool.update(toks_d, _t(lens, torch.int32), reset=(si == 0))
        for _ in range(24):
            at = np.maximum(1, (lens * rng.uniform(0.05, 1.0, size=B)).astype(np.int32))
            at = np.minimum(at, lens)
            _check(pool, toks_d, toks, at, np.minimum(at, 2500), n_min, n_max, k, C)
        _check(pool, toks_d, toks, lens, np.minimum(lens, 2500), n_min, n_max, k, C)


def test_pool_at_the_largest_capacity():
    """2^24 tokens, the most a pool takes: buckets use all 25 bits that the build kernel's notes leave them, the build
    runs over 2048 tiles, and the lookup still returns what the scan of the whole context returns."""
    cap = 1 << 24
    rng = np.random.default_rng(24)
    toks = rng.integers(0, 3000, size=(1, cap)).astype(np.int32)
    toks[0, cap - 40:cap] = toks[0, 1000:1040]                       # the context ends in a copy of an early span
    toks[0, 9_000_000:9_000_040] = toks[0, 1000:1040]                # which also occurs in the middle
    lens = np.array([cap], np.int32)
    toks_d = _t(toks, torch.int32)
    pool = aasd.DraftPool(1, cap, 2, 6, DEV)
    pool.update(toks_d, _t(lens, torch.int32), reset=True)
    ref = _check(pool, toks_d, toks, lens, np.array([cap // 2], np.int32), 2, 6, 8, 8)
    assert ref["n_cand"][0] >= 2 and ref["key_len"][0] == 6
    shorter = np.array([9_000_030], np.int32)                         # a key that ends inside the middle copy
    ref = _check(pool, toks_d, toks, shorter, shorter, 2, 6, 8, 8)
    assert ref["n_cand"][0] >= 1


def test_pool_incremental_updates_with_extras():
    """Prompt indexed once, then 60 steps that append 1..9 tokens each; after every update the pool answers
    like the oracle on the context of that step.  Updates cross the 64-position batches of the insert kernel."""
    rng = np.random.default_rng(21)
    B, L0, cap, m = 5, 700, 1400, 2
    n_min, n_max, k, C = 2, 5, 8, 8
    stream = rng.integers(0, 6, size=(B, cap)).astype(np.int32)
    for b in range(B):          # planted repeats so that long keys occur
        for dst in range(100, cap - 40, 97):
            src = int(rng.integers(0, dst - 30))
            stream[b, dst:dst + 30] = stream[b, src:src + 30]
    extras = rng.integers(0, 50, size=(B * L0, m)).astype(np.int32)
    n_extras = rng.integers(0, m + 1, size=B * L0).astype(np.uint8)
    extras[np.arange(m)[None, :] >= n_extras[:, None]] = -1
    toks_d = _t(stream, torch.int32)
    pool = aasd.DraftPool(B, cap, n_min, n_max, DEV)
    lens = np.full(B, L0, np.int32)
    plens = np.full(B, L0, np.int32)
    pool.update(toks_d, _t(lens, torch.int32), reset=True)
    hits = 0
    for step in range(60):
        ref = _check(pool, toks_d, stream, lens, plens, n_min, n_max, k, C, extras, n_extras, m, L0)
        hits += int((ref["n_cand"] > 0).sum())
        lens = np.minimum(lens + rng.integers(1, 10, size=B), cap).astype(np.int32)
        if step % 2:
            pool.update(toks_d, _t(lens, torch.int32))
        else:      # the fused form: update and lookup in one launch
            got = pool.step(toks_d, _t(lens, torch.int32), _t(plens, torch.int32), k, C, extras=_t(extras, torch.int32),
                            n_extras=_t(n_extras, torch.uint8), m=m, extras_stride=L0)
            torch.cuda.synchronize()
            bk.compare_retrieve(bk.to_np(got), oracle.retrieve_drafts(stream, lens, plens, n_min, n_max, k, C, extras=extras,
                                                                      n_extras=n_extras, m_x=m, extras_stride=L0))
    assert hits > 100


def test_pool_colliding_ngrams_are_told_apart_and_capacity_cuts():
    step = (1 << 32) - aasd.HASH_BASE   # (a+1)*B + (b+step) == a*B + b (mod 2^32): same window hash, same bucket
    a, b = 1000, 2000
    toks = np.array([[5, a + 1, b + step, 77, 6, a, b, 88, 9, a, b]], np.int32)
    pool = aasd.DraftPool(1, 16, 2, 2, DEV)
    td = _t(toks, torch.int32)
    pool.update(td, _t([11], torch.int32), reset=True)
    ref = _check(pool, td, toks, np.array([11], np.int32), np.array([11], np.int32), 2, 2, 3, 4)
    assert ref["src_pos"][0].tolist() == [7, -1, -1, -1]
    # a context longer than the pool's capacity is indexed up to the capacity only
    rng = np.random.default_rng(2)
    long = rng.integers(0, 3, size=(1, 300)).astype(np.int32)
    small = aasd.DraftPool(1, 200, 1, 3, DEV)
    ld = _t(long, torch.int32)
    small.update(ld, _t([300], torch.int32), reset=True)
    _check(small, ld, long, np.array([200], np.int32), np.array([200], np.int32), 1, 3, 4, 6)


def test_decode_loop_with_the_pool_matches_the_oracle():
    """The synthetic decode loop with retrieval served by the pool (one full build, then an update per step)."""
    w = synth.scaled(synth.WORKLOADS["llama3_single"], B=3, L=300, V=3000, steps=30, n_min=2, n_max=4, C=4, coverage=0.9)

    class PoolParity(bk.ParityBackend):
        def __init__(self, dev):
            super().__init__(dev)
            self.pool = aasd.DraftPool(w.B, w.tok_cap, w.n_min, w.n_max, dev)
            self.first = True

        def retrieve(self, tokens, length, prompt_len, w_, extras, n_extras):
            ref = self.orc.retrieve(tokens, length, prompt_len, w_, extras, n_extras)
            td = _t(tokens, torch.int32)
            if self.first:
                self.pool.update(td, _t(length, torch.int32), reset=True)
            self.first = False
            got = self.pool.step(td, _t(length, torch.int32), _t(prompt_len, torch.int32), w_.k, w_.C)   # update + lookup
            torch.cuda.synchronize()
            bk.compare_retrieve(bk.to_np(got), ref)
            return ref

    pb = PoolParity(DEV)
    trace = harness.decode(w, pb, peaked=True)
    assert trace.mean_accept_len > 1.5
