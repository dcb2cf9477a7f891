"""Pins of the oracle's full-vocabulary seeded sampling (alignment sampling read literally, Sec. 3.2:
extras drawn from the whole output distribution of the prefill row; Gumbel-top-k).  The picks must
follow the softmax law without replacement (Plackett-Luce), which is checked statistically against
closed forms; the counter layout that the GPU has to share is checked against the pinned Philox.  No GPU."""
import itertools

import numpy as np
import pytest
from scipy import stats

import oracle

G = oracle.EXTRAS_GUMBEL


def _rows(p, n):
    return np.tile(np.log(np.asarray(p, dtype=np.float64)).astype(np.float32), (n, 1))


def test_first_draw_follows_the_softmax_law_without_the_prompt_token():
    p = np.array([0.05, 0.40, 0.25, 0.02, 0.18, 0.10])
    n, nt = 60000, 0                     # the prompt token is the fifth most likely: every row is misaligned
    out = oracle.align_sample(_rows(p, n), np.full(n, nt), m_x=1, c=1, mode=G, seed=11)
    assert out["misaligned"].all() and (out["n_extras"] == 1).all()
    first = out["extras"][:, 0]
    assert (first != nt).all()
    q = p.copy(); q[nt] = 0; q /= q.sum()
    obs = np.bincount(first, minlength=6)[1:]
    assert stats.chisquare(obs, q[1:] * n).pvalue > 1e-3
    # a different seed gives different draws, the same seed the same ones
    again = oracle.align_sample(_rows(p, n), np.full(n, nt), m_x=1, c=1, mode=G, seed=11)
    other = oracle.align_sample(_rows(p, n), np.full(n, nt), m_x=1, c=1, mode=G, seed=12)
    assert (again["extras"] == out["extras"]).all() and (other["extras"] != out["extras"]).mean() > 0.5


def test_ordered_pairs_follow_plackett_luce():
    p = np.array([0.10, 0.35, 0.30, 0.15, 0.10])
    n, nt = 80000, 4
    out = oracle.align_sample(_rows(p, n), np.full(n, nt), m_x=2, c=2, mode=G, seed=5)
    ex = out["extras"]
    assert (ex[:, 0] != ex[:, 1]).all() and (ex != nt).all() and (out["n_extras"] == 2).all()
    q = p[:4] / p[:4].sum()
    pairs = [(a, b) for a, b in itertools.permutations(range(4), 2)]
    expect = np.array([q[a] * q[b] / (1 - q[a]) for a, b in pairs]) * n
    obs = np.array([((ex[:, 0] == a) & (ex[:, 1] == b)).sum() for a, b in pairs])
    assert stats.chisquare(obs, expect).pvalue > 1e-3
    # margins: gap of each pick's key to the next one, always positive here
    assert (out["draw_margin"] > 0).all()


def test_draws_use_one_philox_word_per_token_keyed_by_row_and_seed():
    """Token v of row id r uses word v mod 4 of Philox4x32-10(counter = (lo32 r, hi32 r, v div 4,
    0x47554D42), key = seed): x = ((word >> 9) + 0.5) / 2^23, E = -ln(1 - x), key = z - ln E."""
    rng = np.random.default_rng(2)
    V, rows, base, seed = 37, 5, (1 << 33) + 7, (9 << 32) | 1234
    z = rng.standard_normal((rows, V)).astype(np.float32)
    nt = z.argmin(axis=1)
    out = oracle.align_sample(z, nt, m_x=3, c=3, mode=G, seed=seed, row_id_base=base)
    for r in range(rows):
        rid = base + r
        kap = np.empty(V)
        for v in range(V):
            w = oracle.philox4x32_10([rid & 0xffffffff, rid >> 32, v >> 2, 0x47554D42], [seed & 0xffffffff, seed >> 32])[v & 3]
            x = ((int(w) >> 9) + 0.5) / 2 ** 23
            kap[v] = float(z[r, v]) - np.log(-np.log1p(-x))
        kap[nt[r]] = -np.inf
        order = np.lexsort((np.arange(V), -kap))
        assert out["extras"][r].tolist() == order[:3].tolist()
        np.testing.assert_allclose(out["draw_margin"][r], kap[order[:3]] - kap[order[1:4]], rtol=1e-12)


def test_partition_shift_invariance_and_degenerate_rows():
    rng = np.random.default_rng(4)
    V, rows = 50, 40
    z = (np.round(rng.standard_normal((rows, V)) * 1024) / 1024).astype(np.float32)   # few bits: z + 8 is exact
    nt = rng.integers(0, V, size=rows)
    full = oracle.align_sample(z, nt, m_x=2, c=4, mode=G, seed=3, row_id_base=100)
    # rows keep their draws when the batch is split (the counter is the global row id)
    lo = oracle.align_sample(z[:17], nt[:17], m_x=2, c=4, mode=G, seed=3, row_id_base=100)
    hi = oracle.align_sample(z[17:], nt[17:], m_x=2, c=4, mode=G, seed=3, row_id_base=117)
    assert (np.concatenate([lo["extras"], hi["extras"]]) == full["extras"]).all()
    # softmax is shift invariant, so are the draws (the shift is exact in fp32 for these values)
    zs = (z.astype(np.float64) + 8.0).astype(np.float32)
    assert ((zs.astype(np.float64) - 8.0) == z).all()
    assert (oracle.align_sample(zs, nt, m_x=2, c=4, mode=G, seed=3, row_id_base=100)["extras"] == full["extras"]).all()
    # aligned rows get nothing, and consume nothing
    am = z.argmax(axis=1)
    al = oracle.align_sample(z, am, m_x=2, c=4, mode=G, seed=3)
    assert (al["n_extras"] == 0).all() and (al["extras"] == -1).all() and (al["draw_margin"] == -1).all()
    # V = 2: the only other token; V = 1: nothing to draw (and the row is aligned anyway)
    two = oracle.align_sample(np.array([[0.0, 1.0]], np.float32), [0], m_x=2, c=2, mode=G, seed=1)
    assert two["extras"].tolist() == [[1, -1]] and two["n_extras"].tolist() == [1]
    assert np.isinf(two["draw_margin"][0, 0]) and two["draw_margin"][0, 1] == -1
    one = oracle.align_sample(np.array([[0.3]], np.float32), [0], m_x=1, c=1, mode=G, seed=1)
    assert one["n_extras"].tolist() == [0]
    # tokens of probability zero (-inf logits) are never drawn
    zi = np.full((50, 8), -np.inf, np.float32)
    zi[:, 2], zi[:, 5], zi[:, 6] = 0.0, 1.0, -1.0
    out = oracle.align_sample(zi, np.full(50, 6), m_x=4, c=4, mode=G, seed=2)
    assert (out["n_extras"] == 2).all() and (np.sort(out["extras"][:, :2], axis=1) == [2, 5]).all()
    assert (out["extras"][:, 2:] == -1).all()


def test_a_dominant_token_is_drawn_first_almost_surely():
    V, n = 200, 3000
    z = np.zeros((n, V), np.float32)
    z[:, 7] = 25.0                       # p(7) = 1 - 199 e^-25
    out = oracle.align_sample(z, np.full(n, 3), m_x=2, c=2, mode=G, seed=8)
    assert (out["extras"][:, 0] == 7).all()
    second = out["extras"][:, 1]
    assert ((second != 7) & (second != 3)).all()
    assert stats.chisquare(np.bincount(second, minlength=V)[np.r_[0:3, 4:7, 8:V]]).pvalue > 1e-3   # uniform over the rest
