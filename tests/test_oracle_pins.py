"""Pins of the CPU oracle against things other than itself.

Each test fixes the oracle to a value the paper prints, a closed form, an
independent library routine (scipy / numpy), an invariant, or brute force on
tiny inputs, so that a dropped term, a wrong sign or index, or a transposed
operand in the oracle fails at least one of them.  None of these tests needs a GPU.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

import oracle
from tests.util import bf16_bits_to_f32, logits_from_probs, read_golden, to_bf16_bits

F32A = float(np.float32(0.1))  # alpha/beta as an fp32 caller passes them
F32B = float(np.float32(0.1))


# --------------------------------------------------------------------------- Philox
def test_philox_known_answers(golden_dir):
    rows = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            assert oracle.philox4x32_10(w[0:4], w[4:6]) == w[6:10]
            rows += 1
    assert rows == 3


def test_philox_counter_and_key_sensitivity():
    # a counter-based generator: every counter word and key word changes the block
    base = oracle.philox4x32_10([1, 2, 3, 4], [5, 6])
    for i in range(4):
        c = [1, 2, 3, 4]
        c[i] ^= 1
        assert oracle.philox4x32_10(c, [5, 6]) != base
    assert oracle.philox4x32_10([1, 2, 3, 4], [5, 7]) != base
    assert oracle.philox4x32_10([1, 2, 3, 4], [4, 6]) != base


# --------------------------------------------------------------------------- softmax / entropy
@pytest.mark.parametrize("V", [1, 2, 7, 1000])
def test_softmax_matches_scipy_and_sums_to_one(V):
    rng = np.random.default_rng(V)
    z = (rng.standard_normal(V) * 3).astype(np.float32)
    p = oracle.row_softmax(z)
    assert abs(p.sum() - 1.0) < 1e-12
    np.testing.assert_allclose(p, scipy.special.softmax(z.astype(np.float64)), rtol=1e-12, atol=0)
    # shift invariance (exactly representable shift)
    p2 = oracle.row_softmax((z.astype(np.float64) + 4.0).astype(np.float32))
    np.testing.assert_allclose(p2, p, rtol=1e-5)


def test_softmax_bf16_widening_is_exact():
    z = np.array([1.0, -2.5, 3.140625, 0.0, -0.0, 100.0], dtype=np.float32)
    bits = to_bf16_bits(z)
    np.testing.assert_array_equal(bf16_bits_to_f32(bits), z)  # all exactly representable in bf16
    np.testing.assert_allclose(oracle.row_softmax(bits), scipy.special.softmax(z.astype(np.float64)), rtol=1e-12)


@pytest.mark.parametrize("V", [32000, 128256, 152064])
def test_entropy_uniform_row_is_ln_V(V):
    z = np.full(V, 1.25, dtype=np.float32)
    m, S, H, am = oracle.row_stats(z)
    assert m == 1.25 and am == 0
    assert abs(S - V) < 1e-6
    assert abs(H - math.log(V)) < 1e-9
    # printed to six decimals in closed form: ln 32000 = 10.373491, ln 128256 = 11.761784, ln 152064 = 11.932057
    assert round(H, 6) == {32000: 10.373491, 128256: 11.761784, 152064: 11.932057}[V]


def test_entropy_special_rows():
    # one-hot limit
    z = np.full(100, -1.0e4, dtype=np.float32)
    z[17] = 0.0
    m, S, H, am = oracle.row_stats(z)
    assert (m, S, H, am) == (0.0, 1.0, 0.0, 17)
    # two equal tokens, everything else negligible
    z[40] = 0.0
    m, S, H, am = oracle.row_stats(z)
    assert am == 17 and abs(S - 2.0) < 1e-12 and abs(H - math.log(2)) < 1e-12
    # single-token vocabulary
    assert oracle.row_stats(np.array([3.0], np.float32)) == (3.0, 1.0, 0.0, 0)
    # -inf logits carry zero probability and do not poison the entropy
    z = np.array([0.0, -np.inf, 0.0, -np.inf], np.float32)
    m, S, H, am = oracle.row_stats(z)
    assert am == 0 and S == 2.0 and abs(H - math.log(2)) < 1e-15


def test_entropy_geometric_closed_form():
    # logits z_v = -a v  =>  p_v = r^v (1-r)/(1-r^V), r = e^-a; closed-form entropy of a truncated geometric law
    a, V = 0.25, 64
    z = (-a * np.arange(V)).astype(np.float32)  # exactly representable
    r = math.exp(-a)
    norm = (1 - r) / (1 - r ** V)
    mean_v = r / (1 - r) - V * r ** V / (1 - r ** V)
    H_closed = -math.log(norm) + a * mean_v
    m, S, H, am = oracle.row_stats(z)
    assert am == 0 and m == 0.0
    assert abs(S - 1.0 / norm) < 1e-12
    assert abs(H - H_closed) < 1e-12


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_stats_match_scipy(dtype):
    rng = np.random.default_rng(7)
    z = (rng.standard_normal(5000) * math.sqrt(3.0)).astype(np.float32)
    z[1234] += 8.0
    if dtype == "bf16":
        bits = to_bf16_bits(z)
        zz, arg = bf16_bits_to_f32(bits).astype(np.float64), bits
    else:
        zz, arg = z.astype(np.float64), z
    m, S, H, am = oracle.row_stats(arg)
    p = scipy.special.softmax(zz)
    assert m == zz.max() and am == int(np.argmax(zz))
    assert abs(1.0 / S - p.max()) < 1e-14
    assert abs(H - scipy.stats.entropy(p)) < 1e-11


def test_argmax_tie_takes_lowest_index():
    bits = to_bf16_bits(np.array([0.5, 2.0, -1.0, 2.0, 2.0], np.float32))
    assert oracle.row_stats(bits)[3] == 1


# --------------------------------------------------------------------------- alignment mask / extras
LETTERS = 6  # A..F


def _rows_with_ranking(rankings, V, gap=1.0):
    """fp32 logits [len(rankings), V]: row r ranks the tokens in rankings[r] first (descending)."""
    z = np.full((len(rankings), V), -5.0, dtype=np.float32)
    for r, order in enumerate(rankings):
        for i, tok in enumerate(order):
            z[r, tok] = 10.0 - gap * i
    return z


def test_alignment_example_sec_2_3(golden_dir):
    row = [r for r in read_golden(os.path.join(golden_dir, "alignment_examples.txt")) if r[0] == "sec2.3"][0]
    prompt = [int(x) for x in row[1].split()]
    picks = [int(x) for x in row[2].split()]
    expect = [int(x) for x in row[3].split()]
    z = _rows_with_ranking([[p] for p in picks], LETTERS)
    next_tok = prompt[1:] + [-1]
    out = oracle.align_sample(z, next_tok, m_x=2, c=4)
    assert out["argmax"].tolist() == picks
    assert out["misaligned"].tolist() == expect
    assert out["rank"].tolist()[3] == -1 and out["n_extras"].tolist()[3] == 0
    # the aligned rows get no extras, the misaligned one gets the greedy pick F
    assert out["n_extras"].tolist()[:3] == [0, 0, 1]
    assert out["extras"][2].tolist() == [5, -1]


def test_alignment_sampling_fig2(golden_dir):
    V = 50
    order = [11, 22, 33, 44, 5, 6]  # ranking of one prefill row, best first
    for name, rk, n_exp, ranks in [r for r in read_golden(os.path.join(golden_dir, "alignment_examples.txt"))
                                   if r[0].startswith("fig2") and r[0] != "fig2.tree"]:
        rk, n_exp = int(rk), int(n_exp)
        ranks = [int(x) for x in ranks.split()]
        z = _rows_with_ranking([order], V)
        out = oracle.align_sample(z, [order[rk]], m_x=2, c=4, mode=oracle.EXTRAS_TOP)
        assert out["rank"][0] == rk, name
        assert out["misaligned"][0] == (1 if rk > 0 else 0), name
        assert out["n_extras"][0] == n_exp, name
        assert out["extras"][0].tolist()[:n_exp] == [order[i] for i in ranks], name
        assert all(x == -1 for x in out["extras"][0].tolist()[n_exp:]), name


def test_rank_and_topc_against_numpy_sort_with_ties():
    rng = np.random.default_rng(3)
    V, rows = 97, 200
    # coarse values -> many exact ties, also at the top
    zf = np.round(rng.standard_normal((rows, V)) * 2.0) / 2.0
    bits = to_bf16_bits(zf.astype(np.float32))
    z = bf16_bits_to_f32(bits).astype(np.float64)
    next_tok = rng.integers(0, V, size=rows)
    out = oracle.align_sample(bits, next_tok, m_x=4, c=8, mode=oracle.EXTRAS_TOP)
    for r in range(rows):
        order = np.lexsort((np.arange(V), -z[r]))  # logit descending, id ascending
        zs = z[r, next_tok[r]]
        rank = int((z[r] > zs).sum())
        assert out["rank"][r] == rank
        assert out["argmax"][r] == order[0]
        assert out["misaligned"][r] == (rank > 0)
        K = [int(v) for v in order[:8] if z[r, v] > zs]
        want = K[:4]
        assert out["n_extras"][r] == len(want)
        assert out["extras"][r].tolist()[:len(want)] == want
        assert abs(out["p_next"][r] - scipy.special.softmax(z[r])[next_tok[r]]) < 1e-14


def test_tied_with_max_counts_as_aligned():
    # reading: aligned iff no token is STRICTLY more likely than the prompt token
    bits = to_bf16_bits(np.array([[1.0, 3.0, 3.0, 0.0]], np.float32))
    out = oracle.align_sample(bits, [2], m_x=2, c=4)
    assert out["argmax"][0] == 1 and out["misaligned"][0] == 0 and out["rank"][0] == 0 and out["n_extras"][0] == 0


def test_extras_parameters_m0_and_invalid():
    z = _rows_with_ranking([[3, 2, 1]], 8)
    out = oracle.align_sample(z, [1], m_x=0, c=4)
    assert out["misaligned"][0] == 1 and out["n_extras"][0] == 0 and out["extras"].shape == (1, 0)
    with pytest.raises(ValueError):
        oracle.align_sample(z, [1], m_x=3, c=2)  # c < m


# --------------------------------------------------------------------------- seeded draws
def _uniform_of(seed, row_id, j):
    x = oracle.philox4x32_10([row_id & 0xFFFFFFFF, row_id >> 32, j, 0x41415344], [seed & 0xFFFFFFFF, seed >> 32])[0]
    return (x >> 8) / 2.0 ** 24


def test_sample_mode_pick_is_inverse_cdf_of_the_documented_uniform():
    """Brute force: recompute every draw with numpy's cumsum/searchsorted from the uniform
    that the (pinned) Philox block yields for (seed, row id, draw index)."""
    rng = np.random.default_rng(11)
    V, rows, seed, base = 12, 3000, 0x1234567800000042, (1 << 33) + 5
    z = rng.standard_normal((rows, V)).astype(np.float32) * 1.5
    next_tok = np.argsort(z, axis=1)[:, 2]  # a low-ranked token: many candidates above it
    out = oracle.align_sample(z, next_tok, m_x=2, c=4, mode=oracle.EXTRAS_SAMPLE, seed=seed, row_id_base=base)
    zd = z.astype(np.float64)
    for r in range(rows):
        order = np.lexsort((np.arange(V), -zd[r]))
        K = [int(v) for v in order[:4] if zd[r, v] > zd[r, next_tok[r]]]
        assert len(K) == 4
        remaining, want = list(K), []
        for j in range(2):
            w = np.exp(zd[r, remaining] - zd[r].max())
            cum = np.cumsum(w)
            u = _uniform_of(seed, base + r, j)
            i = min(int(np.searchsorted(cum, u * cum[-1], side="right")), len(remaining) - 1)
            want.append(remaining.pop(i))
        if out["draw_margin"][r].min() > 1e-9:  # away from a CDF edge the pick is unambiguous
            assert out["extras"][r].tolist() == want
        assert len(set(out["extras"][r].tolist())) == 2  # without replacement


def test_sample_mode_frequencies_follow_softmax():
    rows, V = 100000, 6
    z = np.tile(np.array([2.0, 1.0, 0.5, 0.0, -3.0, -9.0], np.float32), (rows, 1))
    next_tok = np.full(rows, 4)  # tokens 0..3 are the candidates
    out = oracle.align_sample(z, next_tok, m_x=1, c=4, mode=oracle.EXTRAS_SAMPLE, seed=99)
    w = np.exp(np.array([2.0, 1.0, 0.5, 0.0]))
    p = w / w.sum()
    counts = np.bincount(out["extras"][:, 0], minlength=4)[:4]
    sigma = np.sqrt(rows * p * (1 - p))
    assert np.all(np.abs(counts - rows * p) < 4 * sigma)
    # a different seed gives a different stream, the same seed the same stream
    out2 = oracle.align_sample(z, next_tok, m_x=1, c=4, mode=oracle.EXTRAS_SAMPLE, seed=100)
    out3 = oracle.align_sample(z, next_tok, m_x=1, c=4, mode=oracle.EXTRAS_SAMPLE, seed=99)
    assert (out2["extras"] != out["extras"]).any() and (out3["extras"] == out["extras"]).all()


def test_sample_mode_consumes_no_randomness_when_candidates_fit():
    z = _rows_with_ranking([[7, 3, 5, 1]], 10)
    a = oracle.align_sample(z, [5], m_x=2, c=4, mode=oracle.EXTRAS_SAMPLE, seed=1)
    b = oracle.align_sample(z, [5], m_x=2, c=4, mode=oracle.EXTRAS_TOP)
    assert a["extras"].tolist() == b["extras"].tolist() == [[7, 3]]
    assert (a["draw_margin"] == -1).all()


def test_row_id_base_partitioning():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((64, 20)).astype(np.float32)
    nt = rng.integers(0, 20, 64)
    full = oracle.align_sample(z, nt, 2, 4, oracle.EXTRAS_SAMPLE, seed=3, row_id_base=1000)
    lo = oracle.align_sample(z[:32].copy(), nt[:32], 2, 4, oracle.EXTRAS_SAMPLE, seed=3, row_id_base=1000)
    hi = oracle.align_sample(z[32:].copy(), nt[32:], 2, 4, oracle.EXTRAS_SAMPLE, seed=3, row_id_base=1032)
    np.testing.assert_array_equal(full["extras"], np.concatenate([lo["extras"], hi["extras"]]))


# --------------------------------------------------------------------------- retrieval
def _suffix_match_lookup(tok, n_min, n_max, C):
    """What the draft pool of Sec. 3.1 must answer, stated without a pool: for every position p that still has a
    token after it, how many tokens before p agree with the end of the context (the length of the common
    suffix of tok[:p] and tok, counted backwards one token at a time)?  The key that the lookup settles on is the
    longest such agreement, capped at n_max and of at least n_min tokens; the hits are the positions that reach it,
    latest first."""
    L = len(tok)
    agree = {}
    for p in range(1, L):                      # p <= L - 1: one continuation token at least
        n = 0
        while n < min(p, n_max, L - 1) and tok[p - 1 - n] == tok[L - 1 - n]:
            n += 1
        agree[p] = n
    best = max(agree.values(), default=0)
    if best < n_min:
        return 0, []
    return best, sorted((p for p, n in agree.items() if n >= best), reverse=True)[:C]


def test_retrieval_equals_direct_suffix_matching():
    rng = np.random.default_rng(0)
    B, cap = 60, 90
    toks = rng.integers(0, 4, size=(B, cap)).astype(np.int32)  # tiny alphabet: many repeats
    lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
    plens = np.minimum(lens, rng.integers(0, cap, size=B)).astype(np.int32)
    for (n_min, n_max, k, C) in [(1, 6, 6, 4), (3, 3, 4, 2), (2, 4, 8, 16), (1, 8, 16, 32)]:
        out = oracle.retrieve_drafts(toks, lens, plens, n_min, n_max, k, C)
        for b in range(B):
            L = int(lens[b])
            t = toks[b, :L].tolist()
            klen, hits = _suffix_match_lookup(t, n_min, n_max, C)
            assert out["key_len"][b] == klen
            assert out["n_cand"][b] == len(hits)
            assert out["src_pos"][b].tolist() == hits + [-1] * (C - len(hits))
            for c in range(C):
                if c < len(hits):
                    p = hits[c]
                    cont = t[p:p + k]
                    assert out["draft_len"][b, c] == len(cont) >= 1
                    assert out["drafts"][b, c].tolist() == cont + [-1] * (k - len(cont))
                    assert out["strict"][b, c].tolist() == [int(p + j >= plens[b]) for j in range(len(cont))] + [0] * (k - len(cont))
                else:
                    assert out["draft_len"][b, c] == 0
                    assert (out["drafts"][b, c] == -1).all() and (out["strict"][b, c] == 0).all()


def test_incrementally_updated_pool_returns_what_a_rebuilt_pool_returns():
    """Algorithm 1 keeps one dictionary and adds, after every step, the windows that end in the new tokens.
    A dictionary grown that way, looked up at every step, gives what the oracle's stateless retrieval gives
    for the context of that step (so a persistent index may be checked against the stateless oracle)."""
    rng = np.random.default_rng(11)
    n_min, n_max, k, C = 1, 4, 5, 6
    stream = rng.integers(0, 3, size=140).astype(np.int32)
    pool, indexed = {}, 0
    L = 40
    while L <= len(stream):
        tok = stream[:L].tolist()
        for end in range(indexed + 1, L + 1):            # windows that end in a new token: tok[end-klen:end]
            for klen in range(1, min(n_max, end) + 1):
                pool.setdefault(tuple(tok[end - klen:end]), []).append(end)
        indexed = L
        ref = oracle.retrieve_drafts(stream[None, :], [L], [40], n_min, n_max, k, C)
        klen_found, hits = 0, []
        for klen in range(n_max, n_min - 1, -1):
            if klen >= L:
                continue
            hits = sorted((p for p in pool.get(tuple(tok[L - klen:]), []) if p <= L - 1), reverse=True)[:C]
            if hits:
                klen_found = klen
                break
        assert ref["key_len"][0] == klen_found and ref["src_pos"][0].tolist() == hits + [-1] * (C - len(hits))
        L += int(rng.integers(1, 7))


def test_retrieval_planted_span_and_fallback():
    # context: noise, SPAN, noise, SPAN[:5] -> the suffix SPAN[2:5] occurs once before, continuation SPAN[5:]
    span = [101, 102, 103, 104, 105, 106, 107, 108]
    noise1, noise2 = list(range(1, 21)), list(range(30, 45))
    t = noise1 + span + noise2 + span[:5]
    L = len(t)
    toks = np.array([t + [0] * 7], np.int32)
    out = oracle.retrieve_drafts(toks, [L], [L], 3, 3, 4, 2)
    assert out["key_len"][0] == 3 and out["n_cand"][0] == 1
    assert out["src_pos"][0, 0] == len(noise1) + 5
    assert out["drafts"][0, 0].tolist() == [106, 107, 108, 30]
    # a longer key than the repeated part falls back to the longest length that occurs
    out = oracle.retrieve_drafts(toks, [L], [L], 2, 8, 4, 2)
    assert out["key_len"][0] == 5
    # no repeat at all
    out = oracle.retrieve_drafts(np.arange(50, dtype=np.int32)[None], [50], [50], 1, 6, 4, 2)
    assert out["n_cand"][0] == 0 and out["key_len"][0] == 0 and (out["src_pos"] == -1).all()
    # context not longer than the key: no hit
    out = oracle.retrieve_drafts(np.array([[5, 5, 5]], np.int32), [3], [3], 3, 3, 4, 2)
    assert out["n_cand"][0] == 0
    # hit whose only continuation is the last token
    out = oracle.retrieve_drafts(np.array([[9, 8, 7, 1, 9, 8, 9, 8]], np.int32), [8], [8], 2, 2, 4, 4)
    assert out["src_pos"][0].tolist()[:2] == [6, 2] and out["draft_len"][0].tolist()[:2] == [2, 4]
    out = oracle.retrieve_drafts(np.array([[4, 4, 4]], np.int32), [3], [3], 1, 1, 4, 4)
    assert out["src_pos"][0].tolist() == [2, 1, -1, -1] and out["draft_len"][0].tolist() == [1, 2, 0, 0]


def test_retrieval_extras_gather_and_strict_split():
    # prompt of 10 tokens, then generated tokens; key (1,2) occurs in the prompt at 1..2 and in generated text
    t = [7, 1, 2, 3, 4, 5, 6, 8, 9, 10, 1, 2, 3, 1, 2]
    toks = np.array([t], np.int32)
    PL, L = 10, len(t)
    m_x = 2
    extras = -np.ones((PL, m_x), np.int32)
    n_extras = np.zeros(PL, np.uint8)
    extras[2] = [50, 51]; n_extras[2] = 2      # row 2 predicted the token at position 3: misaligned, two extras
    extras[4] = [60, -1]; n_extras[4] = 1      # row 4 predicted the token at position 5
    extras[9] = [70, 71]; n_extras[9] = 2      # the last prompt row predicts generated text: never gathered
    out = oracle.retrieve_drafts(toks, [L], [PL], 2, 2, 8, 2, extras=extras, n_extras=n_extras, m_x=m_x, extras_stride=PL)
    assert out["src_pos"][0].tolist() == [12, 3]
    assert out["draft_len"][0].tolist() == [3, 8]
    assert out["drafts"][0].tolist() == [[3, 1, 2, -1, -1, -1, -1, -1], [3, 4, 5, 6, 8, 9, 10, 1]]
    assert out["strict"][0].tolist() == [[1, 1, 1, 0, 0, 0, 0, 0], [0, 0, 0, 0, 0, 0, 0, 1]]
    assert out["draft_extras"][0, 0].tolist() == [[-1, -1]] * 8          # generated context has no prefill rows
    assert out["draft_extras"][0, 1].tolist() == [[50, 51], [-1, -1], [60, -1]] + [[-1, -1]] * 5


# --------------------------------------------------------------------------- verification
def _verify_rows(B, C, k, V, fill=-30.0):
    return np.full((B, 1 + C * k, V), fill, dtype=np.float32)


def test_threshold_worked_values(golden_dir):
    for alpha, beta, probs, H, delta, flags in read_golden(os.path.join(golden_dir, "threshold_examples.txt")):
        alpha, beta = float(np.float32(float(alpha))), float(np.float32(float(beta)))
        probs = [float(x) for x in probs.split()]
        flags = [int(x) for x in flags.split()]
        n = len(probs)
        # one candidate per token, each of length 1: all are verified by row 0
        C, k = n, 1
        z = _verify_rows(1, C, k, n)
        z[0, :, :] = logits_from_probs(probs)
        drafts = np.arange(n, dtype=np.int32).reshape(1, C, k)
        out = oracle.verify(z, drafts, np.ones((1, C), np.int32), alpha=alpha, beta=beta)
        assert abs(out["row_entropy"][0, 0] - float(H)) < 2e-6
        np.testing.assert_allclose(out["tok_delta"][0, :, 0], float(delta), atol=2e-6)
        np.testing.assert_allclose(out["tok_p"][0, :, 0], probs, rtol=1e-6)
        passed = (out["tok_p"][0, :, 0] >= out["tok_delta"][0, :, 0]).astype(int).tolist()
        assert passed == flags
        # accepted length 1 iff some candidate passes; the first passing candidate is reported
        assert out["accept_len"][0] == (1 if any(flags) else 0)
        assert out["best_cand"][0] == (flags.index(1) if any(flags) else 0)


def test_extreme_cases_of_sec_3_3():
    V = 1000
    # all tokens equally likely: they are accepted together (p = Delta >= delta)
    z = np.zeros((1, 1 + 3, V), np.float32)
    out = oracle.verify(z, np.array([[[5], [700], [999]]], np.int32), np.ones((1, 3), np.int32), alpha=F32A, beta=F32B)
    assert (out["tok_p"] >= out["tok_delta"]).all() and out["accept_len"][0] == 1
    # one token close to 1: nothing else is accepted
    z[:] = -20.0
    z[0, 0, 123] = 5.0
    out = oracle.verify(z, np.array([[[122], [123], [124]]], np.int32), np.ones((1, 3), np.int32), alpha=F32A, beta=F32B)
    assert out["best_cand"][0] == 1 and out["accept_len"][0] == 1
    assert out["tok_margin"][0, 0, 0] > 0.09 and out["tok_margin"][0, 2, 0] > 0.09


@pytest.mark.parametrize("k,C", [(1, 1), (3, 2), (4, 3)])
def test_accept_prefix_brute_force(k, C):
    """Every pass/fail pattern: tokens GOOD (p ~ 0.9) pass, tokens BAD (p ~ 1e-7) fail."""
    V, GOOD, BAD = 16, 3, 9
    for pattern in itertools.product([0, 1], repeat=C * k):
        pat = np.array(pattern).reshape(C, k)
        z = _verify_rows(1, C, k, V, fill=-16.0)
        for r in range(1 + C * k):
            z[0, r, GOOD] = 0.0
            z[0, r, (r * 5 + 1) % V if (r * 5 + 1) % V not in (GOOD, BAD) else 0] = -2.0  # a distinct runner-up per row
        drafts = np.where(pat == 1, GOOD, BAD).astype(np.int32)[None]
        out = oracle.verify(z, drafts, np.full((1, C), k, np.int32), alpha=F32A, beta=F32B)
        lead = [int(np.argmin(np.append(pat[c], 0))) for c in range(C)]  # index of the first 0
        a = max(lead)
        assert out["accept_len"][0] == a
        assert out["best_cand"][0] == lead.index(a)
        assert out["next_token"][0] == GOOD
        # tokens after the first failure are not evaluated
        for c in range(C):
            ev = (out["tok_margin"][0, c] >= 0).astype(int).tolist()
            assert ev == [1] * min(lead[c] + 1, k) + [0] * (k - min(lead[c] + 1, k))


def test_next_token_comes_from_the_row_after_the_last_accepted_token():
    V, C, k = 32, 2, 3
    z = _verify_rows(1, C, k, V)
    R = 1 + C * k
    for r in range(R):
        z[0, r, r + 10] = 4.0  # greedy pick of row r is token r+10
    # candidate 1 follows the greedy picks of its own rows for two tokens, then deviates
    drafts = np.array([[[10, 0, 0], [10, 1 + 1 * k + 0 + 10, 7]]], np.int32)
    out = oracle.verify(z, drafts, np.array([[3, 3]], np.int32), alpha=F32A, beta=F32B)
    assert out["accept_len"][0] == 2 and out["best_cand"][0] == 1
    assert out["next_token"][0] == (1 + 1 * k + 1) + 10  # row after candidate 1's second token
    # nothing accepted: the bonus token is the greedy pick of row 0 (one token per step, as in autoregressive decoding)
    drafts = np.array([[[0, 0, 0], [1, 1, 1]]], np.int32)
    out = oracle.verify(z, drafts, np.array([[3, 3]], np.int32), alpha=F32A, beta=F32B)
    assert out["accept_len"][0] == 0 and out["best_cand"][0] == 0 and out["next_token"][0] == 10
    # draft_len limits what can be accepted
    drafts = np.array([[[10, 11, 12], [10, 14, 15]]], np.int32)
    out = oracle.verify(z, drafts, np.array([[0, 1]], np.int32), alpha=F32A, beta=F32B)
    assert out["accept_len"][0] == 1 and out["best_cand"][0] == 1 and out["next_token"][0] == 14


def _random_verify_case(seed, B=3, C=3, k=4, V=200, peaked=True):
    rng = np.random.default_rng(seed)
    R = 1 + C * k
    z = rng.standard_normal((B, R, V)).astype(np.float32)
    if peaked:
        for b in range(B):
            for r in range(R):
                top = rng.choice(V, 4, replace=False)
                z[b, r, top] = [9.0, 8.0, 7.0, 6.0]
    drafts = np.empty((B, C, k), np.int32)
    for b in range(B):
        for c in range(C):
            for j in range(k):
                rho = 0 if j == 0 else 1 + c * k + (j - 1)
                order = np.argsort(-z[b, rho])
                drafts[b, c, j] = order[rng.choice(4, p=[0.55, 0.25, 0.1, 0.1])]
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    return z, drafts, dl


def test_verify_invariants():
    for seed in range(20):
        z, drafts, dl = _random_verify_case(seed)
        B, C, k = drafts.shape
        base = oracle.verify(z, drafts, dl, alpha=F32A, beta=F32B)
        assert ((0 <= base["accept_len"]) & (base["accept_len"] <= dl.max(axis=1))).all()
        assert (base["tok_delta"] <= np.repeat(base["row_pmax"][:, :1], C * k, 1).reshape(B, C, k) + 1).all()
        # delta never exceeds Delta of the verifying row
        for b in range(B):
            for c in range(C):
                for j in range(dl[b, c]):
                    rho = 0 if j == 0 else 1 + c * k + (j - 1)
                    assert base["tok_delta"][b, c, j] <= base["row_pmax"][b, rho]
        # the greedy token of every row passes: drafting the greedy chain accepts everything
        greedy = np.empty_like(drafts)
        for b in range(B):
            for c in range(C):
                for j in range(k):
                    rho = 0 if j == 0 else 1 + c * k + (j - 1)
                    greedy[b, c, j] = base["row_argmax"][b, rho]
        g = oracle.verify(z, greedy, dl, alpha=F32A, beta=F32B, strict=np.ones_like(greedy, dtype=np.uint8))
        assert (g["accept_len"] == dl.max(axis=1)).all()
        # raising alpha or beta never lengthens the accepted prefix
        prev = None
        for a_, b_ in [(0.0, 0.0), (0.05, 0.05), (F32A, F32B), (0.2, 0.1), (0.5, 0.3), (0.0, 1.0)]:
            cur = oracle.verify(z, drafts, dl, alpha=a_, beta=b_)["accept_len"]
            if prev is not None:
                assert (cur <= prev).all()
            prev = cur
        # alpha = beta = 0 accepts every drafted token
        assert (oracle.verify(z, drafts, dl, alpha=0.0, beta=0.0)["accept_len"] == dl.max(axis=1)).all()


def test_strict_limit_is_exact_match_greedy_verification():
    for seed in range(20):
        z, drafts, dl = _random_verify_case(100 + seed)
        B, C, k = drafts.shape
        strict = oracle.verify(z, drafts, dl, alpha=F32A, beta=F32B, strict=np.ones_like(drafts, dtype=np.uint8))
        beta1 = oracle.verify(z, drafts, dl, alpha=0.0, beta=1.0)
        for b in range(B):
            lead = []
            for c in range(C):
                a = 0
                for j in range(dl[b, c]):
                    rho = 0 if j == 0 else 1 + c * k + (j - 1)
                    if drafts[b, c, j] != int(np.argmax(z[b, rho])):  # rows here have a unique maximum
                        break
                    a += 1
                lead.append(a)
            assert strict["accept_len"][b] == beta1["accept_len"][b] == max(lead)
            assert strict["best_cand"][b] == beta1["best_cand"][b] == lead.index(max(lead))


def test_strict_flag_is_per_token_and_ties_with_the_maximum_pass():
    V = 10
    z = _verify_rows(1, 1, 2, V)
    z[0, 0, [1, 2]] = [3.0, 2.0]      # p ~ 0.73, 0.27
    z[0, 1, [4, 5]] = [1.0, 1.0]      # exact tie at the maximum
    drafts = np.array([[[2, 5]]], np.int32)
    dl = np.array([[2]], np.int32)
    loose = oracle.verify(z, drafts, dl, alpha=F32A, beta=F32B)
    assert loose["accept_len"][0] == 2      # 0.27 >= 0.1*H+0.1, and the tied token passes
    tight = oracle.verify(z, drafts, dl, alpha=F32A, beta=F32B, strict=np.array([[[1, 0]]], np.uint8))
    assert tight["accept_len"][0] == 0      # strict on the first token: 2 is not a greedy token
    tie = oracle.verify(z, np.array([[[1, 5]]], np.int32), dl, alpha=F32A, beta=F32B, strict=np.ones((1, 1, 2), np.uint8))
    assert tie["accept_len"][0] == 2        # token 5 ties with token 4 at the row maximum


def test_fixed_threshold_flag_is_eq_3():
    # Eq. 3 with delta = 0.1 (the ablation's value): no Delta clamp, so even the top token can fail
    V = 100
    z = np.zeros((1, 2, V), np.float32)  # uniform: every p = 0.01 < 0.1
    out = oracle.verify(z, np.array([[[0]]], np.int32), np.array([[1]], np.int32), alpha=0.0, beta=F32B,
                        flags=oracle.VERIFY_NO_CLAMP)
    assert out["accept_len"][0] == 0 and abs(out["tok_delta"][0, 0, 0] - F32B) < 1e-15
    out = oracle.verify(z, np.array([[[0]]], np.int32), np.array([[1]], np.int32), alpha=0.0, beta=F32B)
    assert out["accept_len"][0] == 1


def test_near_threshold_counter():
    # p = (0.6, 0.3, 0.1): with alpha = 0, beta = 0.3 (in double) the second token sits on the threshold
    z = np.empty((1, 2, 3), np.float32)
    z[0, :, :] = logits_from_probs([0.6, 0.3, 0.1])
    out = oracle.verify(z, np.array([[[1]]], np.int32), np.array([[1]], np.int32), alpha=0.0, beta=0.3)
    assert out["near_count"][0] == 1 and out["tok_margin"][0, 0, 0] < 1e-6
    out = oracle.verify(z, np.array([[[1]]], np.int32), np.array([[1]], np.int32), alpha=0.0, beta=0.2)
    assert out["near_count"][0] == 0


def test_out_of_vocabulary_draft_token_is_rejected():
    z = np.zeros((1, 3, 8), np.float32)
    out = oracle.verify(z, np.array([[[8, 0]]], np.int32), np.array([[2]], np.int32), alpha=0.0, beta=0.0)
    assert out["accept_len"][0] == 0
    out = oracle.verify(z, np.array([[[-1, 0]]], np.int32), np.array([[2]], np.int32), alpha=0.0, beta=0.0)
    assert out["accept_len"][0] == 0
