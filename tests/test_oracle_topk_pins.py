"""Pins of the oracle's top-k verifier (the ablation of Sec. 4.4) against numpy ranking, the already
pinned strict verifier (k = 1), brute force on the cascade, and monotonicity in k.  No GPU."""
import itertools

import numpy as np
import pytest

import oracle
from tests.util import to_bf16_bits, bf16_bits_to_f32


def _case(rng, B, C, k, V, ties=False):
    R = 1 + C * k
    z = rng.standard_normal((B, R, V)).astype(np.float32)
    if ties:
        z = np.round(z * 2) / 2
    order = np.argsort(-z, axis=2, kind="stable")
    drafts = np.empty((B, C, k), np.int32)
    for b in range(B):
        for c in range(C):
            for j in range(k):
                rho = 0 if j == 0 else 1 + c * k + (j - 1)
                drafts[b, c, j] = order[b, rho, min(V - 1, int(rng.geometric(0.3)) - 1)]
    drafts[rng.random((B, C, k)) < 0.03] = V + 2
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    return z, drafts, dl


@pytest.mark.parametrize("topk", [1, 2, 5, 8])
def test_ranks_and_decisions_against_numpy(topk):
    rng = np.random.default_rng(topk)
    B, C, k, V = 6, 3, 5, 40
    for ties in (False, True):
        z, drafts, dl = _case(rng, B, C, k, V, ties)
        out = oracle.verify_topk(z, drafts, dl, topk=topk)
        for b in range(B):
            best = (0, 0)
            for c in range(C):
                a, alive = 0, True
                for j in range(k):
                    rho = 0 if j == 0 else 1 + c * k + (j - 1)
                    t = drafts[b, c, j]
                    if j >= dl[b, c]:
                        assert out["tok_rank"][b, c, j] == -1
                        continue
                    rk = int((z[b, rho] > z[b, rho, t]).sum()) if t < V else -1
                    assert out["tok_rank"][b, c, j] == rk
                    ok = 0 <= rk < topk
                    if alive and ok:
                        a += 1
                    else:
                        alive = False
                if a > best[0]:
                    best = (a, c)
            assert (out["accept_len"][b], out["best_cand"][b]) == best
            rho = 0 if best[0] == 0 else 1 + best[1] * k + best[0] - 1
            assert out["next_token"][b] == int(np.argmax(z[b, rho]))
        assert (out["row_argmax"] == z.argmax(axis=2)).all()


def test_top1_is_strict_verification():
    """k = 1 accepts exactly the tokens that attain the row maximum: the strict limit of Sec. 3.3, which the
    conditional verifier (pinned elsewhere) reaches when every token is flagged strict."""
    rng = np.random.default_rng(3)
    for ties in (False, True):
        z, drafts, dl = _case(rng, 8, 4, 6, 30, ties)
        bits = to_bf16_bits(z)
        a = oracle.verify_topk(bits, drafts, dl, topk=1)
        s = oracle.verify(bits, drafts, dl, np.ones_like(drafts, dtype=np.uint8), alpha=0.1, beta=0.1)
        for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
            assert (a[name] == s[name]).all(), name


def test_monotone_in_k_and_limits():
    rng = np.random.default_rng(5)
    z, drafts, dl = _case(rng, 10, 4, 6, 25)
    drafts = np.minimum(drafts, 24)            # all ids valid
    prev = None
    for topk in range(1, 26):
        a = oracle.verify_topk(z, drafts, dl, topk=topk)["accept_len"]
        if prev is not None:
            assert (a >= prev).all()
        prev = a
    assert (prev == dl.max(axis=1)).all()       # k = V accepts everything: the longest candidate wins
    with pytest.raises(ValueError):
        oracle.verify_topk(z, drafts, dl, topk=0)


def test_cascade_brute_force():
    """Every pass/fail pattern of one candidate of 4 tokens: the accepted length is the number of leading passes."""
    V, k = 12, 4
    for pattern in itertools.product([0, 1], repeat=k):
        z = np.zeros((1, 1 + k, V), np.float32)
        z[0, :, :6] = np.arange(6, 0, -1)        # tokens 0..5 ranked 0..5 in every row
        drafts = np.array([[[2 if ok else 5 for ok in pattern]]], np.int32)   # rank 2 passes at k = 3, rank 5 fails
        out = oracle.verify_topk(z, drafts, [[k]], topk=3)
        lead = next((i for i, ok in enumerate(pattern) if not ok), k)
        assert out["accept_len"][0] == lead
        assert out["tok_rank"][0, 0].tolist() == [2 if ok else 5 for ok in pattern]
