"""Parity of the HIP path with the CPU oracle, element by element, on the same seeded inputs.

Bar: integers, bytes and indices bit-exact (decisions whose oracle margin is below 1e-6 are
counted instead); probabilities and entropies within 1e-5 relative (fp32 accumulation).
All calls go through the Python binding, i.e. through the C ABI of libaasd.so.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2505_13204_amd as aasd
from tests import harness, synth
from tests import backends as bk
from tests.util import to_bf16_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"



def _dev_logits(z: np.ndarray, dtype: str):
    t = torch.from_numpy(np.ascontiguousarray(z, dtype=np.float32)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def _random_rows(rng, rows, V, dtype, sigma=1.7, coarse=False):
    z = rng.standard_normal((rows, V)).astype(np.float32) * sigma
    if coarse:
        z = np.round(z * 2) / 2  # many exact ties
    return _dev_logits(z, dtype)


# --------------------------------------------------------------------------- alignment sampling
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V", [1, 5, 8, 9, 63, 1000, 4099, 32000])
def test_align_shapes_and_tails(dtype, V):
    rng = np.random.default_rng(V)
    rows = 37
    z = _random_rows(rng, rows, V, dtype)
    nt = rng.integers(-1, V, size=rows).astype(np.int32)
    tally = bk.Tally()
    for mode in (oracle.EXTRAS_TOP, oracle.EXTRAS_SAMPLE):
        got = bk.hip_align(z, nt, 2, 4, mode, seed=5, row_id_base=77)
        ref = bk.oracle_align(z, nt, 2, 4, mode, seed=5, row_id_base=77)
        bk.compare_align(got, ref, tally, mode)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("pad", [1, 3, 8, 13])
def test_align_unaligned_row_stride(dtype, pad):
    """row_stride != V: rows start at every 16-byte phase, so head and tail scalars are exercised."""
    rng = np.random.default_rng(pad)
    rows, V = 41, 5003
    full = _random_rows(rng, rows, V + pad, dtype)
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    got = bk.hip_align(full, nt, 2, 4, oracle.EXTRAS_TOP, V=V)
    ref = oracle.align_sample(synth.to_host_bits(full), nt, m_x=2, c=4, V=V)
    bk.compare_align(got, ref, bk.Tally(), oracle.EXTRAS_TOP)


@pytest.mark.parametrize("m,c", [(0, 1), (1, 1), (1, 2), (2, 2), (2, 4), (3, 5), (4, 4), (4, 8)])
def test_align_extras_parameters_with_ties(m, c):
    rng = np.random.default_rng(100 * m + c)
    rows, V = 300, 777
    z = _random_rows(rng, rows, V, "bf16", coarse=True)
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    for mode in (oracle.EXTRAS_TOP, oracle.EXTRAS_SAMPLE):
        got = bk.hip_align(z, nt, m, c, mode, seed=9)
        ref = bk.oracle_align(z, nt, m, c, mode, seed=9)
        bk.compare_align(got, ref, bk.Tally(), mode)


def test_align_no_next_tokens_and_no_rank():
    rng = np.random.default_rng(1)
    z = _random_rows(rng, 20, 3000, "bf16")
    got = bk.hip_align(z, None, 2, 4, oracle.EXTRAS_TOP, want_rank=False)
    ref = bk.oracle_align(z, None, 2, 4, oracle.EXTRAS_TOP)
    assert got["rank"] is None
    bk.compare_align(got, ref, bk.Tally(), oracle.EXTRAS_TOP)
    assert (got["n_extras"] == 0).all() and (got["extras"] == -1).all()


def test_align_without_extras_defines_the_count_array():
    """m = 0: no extras are chosen; an n_extras array that the caller passes anyway comes back as zeros."""
    rng = np.random.default_rng(44)
    z = _random_rows(rng, 70, 3000, "bf16")
    nt = torch.from_numpy(rng.integers(0, 3000, size=70).astype(np.int32)).to(DEV)
    for mode in (aasd.EXTRAS_TOP, aasd.EXTRAS_SAMPLE, aasd.EXTRAS_GUMBEL):
        out = {"n_extras": torch.full((70,), 0xAB, dtype=torch.uint8, device=DEV)}
        got = aasd.align_sample(z, nt, m=0, c=1, mode=mode, out=out)
        torch.cuda.synchronize()
        assert (got["n_extras"] == 0).all()


def test_align_degenerate_rows():
    V = 4096
    z = np.zeros((6, V), np.float32)
    z[1, :] = -3.0                      # uniform
    z[2, :] = -1.0e4; z[2, 1234] = 0.0  # one-hot limit
    z[3, :] = -np.inf; z[3, [5, 4000]] = [1.0, 1.0]   # -inf logits (masked vocabulary)
    z[4, :] = np.linspace(-40, 40, V)   # wide dynamic range, maximum at the end
    z[5, :] = np.linspace(60, -60, V)   # maximum at the start
    nt = np.array([7, 9, 1234, 4000, 0, 0], np.int32)
    for dtype in ("f32", "bf16"):
        zd = _dev_logits(z, dtype)
        got = bk.hip_align(zd, nt, 2, 4, oracle.EXTRAS_TOP)
        ref = bk.oracle_align(zd, nt, 2, 4, oracle.EXTRAS_TOP)
        bk.compare_align(got, ref, bk.Tally(), oracle.EXTRAS_TOP)
        assert abs(got["entropy"][0] - math.log(V)) < 1e-4 and got["misaligned"][0] == 0
        assert got["entropy"][2] == 0.0 and abs(got["p_max"][2] - 1.0) < 1e-6
        assert abs(got["entropy"][3] - math.log(2)) < 1e-5


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_low_entropy_rows_with_a_dominant_logit(dtype):
    """One logit far above the rest, met late in the sweep: the entropy is small and its error must not
    grow with the height of the peak above what the lane had seen before."""
    rng = np.random.default_rng(77)
    rows, V = 96, 40000
    z = rng.standard_normal((rows, V)).astype(np.float32) * 1.7
    for r in range(rows):
        pos = rng.choice(np.arange(V // 2, V), 3, replace=False)
        h = 8.0 + 0.5 * r      # 8 .. 55 nats above the bulk
        z[r, pos] = [h, h - 5.0, h - 6.0]
    zd = _dev_logits(z, dtype)
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    tally = bk.Tally()
    ref = bk.oracle_align(zd, nt, 2, 4, oracle.EXTRAS_TOP)
    assert 0.03 < ref["entropy"].min() < 0.06
    bk.compare_align(bk.hip_align(zd, nt, 2, 4, oracle.EXTRAS_TOP), ref, tally, oracle.EXTRAS_TOP)
    B = rows // 3
    drafts = rng.integers(0, V, size=(B, 1, 2)).astype(np.int32)
    _verify_both(zd.view(B, 3, V), drafts, np.full((B, 1), 2, np.int32), None, 0.1, 0.1, 0, tally)
    print("low entropy", dtype, tally)


def test_align_many_ties_above_next_token_overflows_candidate_buffer():
    """More than 256 tokens tied above the prompt token: the exact fallback selection runs."""
    V = 6000
    z = np.full((3, V), -2.0, np.float32)
    z[0, 100:700] = 3.0                 # 600-way tie at the top
    z[1, 100:700] = 3.0; z[1, 5555] = 4.0; z[1, 17] = 3.5
    z[2, ::2] = 1.0                     # 3000-way tie
    nt = np.array([0, 1, 1], np.int32)
    for dtype in ("f32", "bf16"):
        zd = _dev_logits(z, dtype)
        for (m, c) in [(2, 4), (4, 8)]:
            for mode in (oracle.EXTRAS_TOP, oracle.EXTRAS_SAMPLE):
                got = bk.hip_align(zd, nt, m, c, mode, seed=3)
                ref = bk.oracle_align(zd, nt, m, c, mode, seed=3)
                bk.compare_align(got, ref, bk.Tally(), mode)
    assert got["extras"][1].tolist()[:2] == ref["extras"][1].tolist()[:2]


def test_align_row_id_base_partition_and_determinism():
    rng = np.random.default_rng(8)
    z = _random_rows(rng, 64, 2048, "bf16")
    nt = rng.integers(0, 2048, size=64).astype(np.int32)
    full = bk.hip_align(z, nt, 2, 4, oracle.EXTRAS_SAMPLE, seed=11, row_id_base=500)
    again = bk.hip_align(z, nt, 2, 4, oracle.EXTRAS_SAMPLE, seed=11, row_id_base=500)
    for name in full:
        if full[name] is not None:
            assert full[name].tobytes() == again[name].tobytes(), name  # byte-identical reruns
    lo = bk.hip_align(z[:32], nt[:32], 2, 4, oracle.EXTRAS_SAMPLE, seed=11, row_id_base=500)
    hi = bk.hip_align(z[32:], nt[32:], 2, 4, oracle.EXTRAS_SAMPLE, seed=11, row_id_base=532)
    np.testing.assert_array_equal(full["extras"], np.concatenate([lo["extras"], hi["extras"]]))


def test_align_sample_frequencies_on_device():
    rows = 20000
    z = torch.tensor([2.0, 1.0, 0.5, 0.0, -3.0, -9.0], device=DEV).repeat(rows, 1).contiguous()
    nt = np.full(rows, 4, np.int32)
    got = bk.hip_align(z, nt, 1, 4, oracle.EXTRAS_SAMPLE, seed=99)
    ref = bk.oracle_align(z, nt, 1, 4, oracle.EXTRAS_SAMPLE, seed=99)
    bk.compare_align(got, ref, bk.Tally(), oracle.EXTRAS_SAMPLE)
    w = np.exp(np.array([2.0, 1.0, 0.5, 0.0])); p = w / w.sum()
    counts = np.bincount(got["extras"][:, 0], minlength=4)[:4]
    assert np.all(np.abs(counts - rows * p) < 4 * np.sqrt(rows * p * (1 - p)))


@pytest.mark.parametrize("shape", ["256,1", "256,2", "256,4", "512,2", "512,4", "1024,1", "1024,2",
                                   "256,4,1", "256,4,2", "256,2,5", "256,1,16", "512,2,8", "1024,1,4"])
def test_every_compiled_launch_shape(shape, forced_plan):
    """The sweep is compiled for several (threads per workgroup, loads in flight) shapes and cuts rows into
    segments when there are few of them; the library picks by row count.  Every plan must give the same
    answers: force them one by one ("block,unroll[,segments]")."""
    forced_plan(shape)
    rng = np.random.default_rng(17)
    rows, V = 24, 128256 // 4 + 5   # several full batches for the widest shape, plus a ragged tail
    for dtype in ("bf16", "f32"):
        z = _random_rows(rng, rows, V, dtype, coarse=(dtype == "bf16"))
        nt = rng.integers(-1, V, size=rows).astype(np.int32)
        got = bk.hip_align(z, nt, 2, 4, oracle.EXTRAS_SAMPLE, seed=2)
        ref = bk.oracle_align(z, nt, 2, 4, oracle.EXTRAS_SAMPLE, seed=2)
        bk.compare_align(got, ref, bk.Tally(), oracle.EXTRAS_SAMPLE)
    zd, drafts, dl, strict = _verify_case(rng, 2, 2, 3, 40000, "bf16")
    _verify_both(zd, drafts, dl, strict, 0.1, 0.1, 0, bk.Tally())
    # top-k verification runs the alignment form of the sweep over verify rows
    ref = oracle.verify_topk(synth.to_host_bits(zd), drafts, dl, topk=3)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    got = bk.to_np(aasd.verify_topk(zd, t(drafts, torch.int32), t(dl, torch.int32), topk=3))
    for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)


@pytest.mark.parametrize("dtype,V", [("f32", 1_000_003), ("bf16", 4_000_037)])
def test_vocabularies_too_large_for_the_chunk_maxima_in_lds(dtype, V):
    """A row so long that a segment's chunk maxima do not fit LDS even in 16 segments: the alignment sweep then finds
    a lane's candidate chunks by a second look at its share.  Odd V, so rows start at every alignment; all three
    extras modes, and verification in both launch forms over rows of the same length."""
    rng = np.random.default_rng(31)
    rows = 5
    z = _random_rows(rng, rows, V, dtype, coarse=(dtype == "bf16"))
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    nt[0] = -1
    tally = bk.Tally()
    for mode in (oracle.EXTRAS_TOP, oracle.EXTRAS_SAMPLE, oracle.EXTRAS_GUMBEL):
        got = bk.hip_align(z, nt, 2, 4, mode, seed=9)
        ref = bk.oracle_align(z, nt, 2, 4, mode, seed=9)
        bk.compare_align(got, ref, tally, mode)
    assert ref["misaligned"].sum() >= 2
    zd, drafts, dl, strict = _verify_case(rng, 1, 2, 2, V, dtype, peaked=True)
    _verify_both(zd, drafts, dl, strict, 0.1, 0.1, 0, tally)
    # top-k verification runs the alignment form of the sweep (every row lists its best tokens) over the same rows
    ref = oracle.verify_topk(synth.to_host_bits(zd), drafts, dl, topk=5)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    got = bk.to_np(aasd.verify_topk(zd, t(drafts, torch.int32), t(dl, torch.int32), topk=5))
    for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    print("large vocabulary", dtype, V, tally)


# --------------------------------------------------------------------------- retrieval
def _retrieve_both(tokens, lens, plens, n_min, n_max, k, C, extras=None, n_extras=None, m=0, xs=0):
    ref = oracle.retrieve_drafts(tokens, lens, plens, n_min, n_max, k, C, extras=extras, n_extras=n_extras, m_x=m,
                                 extras_stride=xs)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    out = aasd.retrieve_drafts(t(tokens, torch.int32), t(lens, torch.int32), t(plens, torch.int32), n_min, n_max, k, C,
                               extras=None if extras is None else t(extras, torch.int32),
                               n_extras=None if extras is None else t(n_extras, torch.uint8), m=m, extras_stride=xs)
    torch.cuda.synchronize()
    bk.compare_retrieve(bk.to_np(out), ref)
    return ref


@pytest.mark.parametrize("n_min,n_max,k,C", [(1, 1, 1, 1), (1, 6, 6, 4), (3, 3, 4, 2), (2, 4, 8, 16), (1, 8, 16, 32)])
@pytest.mark.parametrize("cap", [1, 90, 1500, 12000, 30011])
@pytest.mark.parametrize("B", [24, 520])    # up to 512 sequences: 1024 threads each; more: 256 threads each, smaller tiles
def test_retrieve_random_small_alphabet(n_min, n_max, k, C, cap, B):
    rng = np.random.default_rng(cap + n_max + B)
    alphabet = 3 if cap < 2000 else 40
    toks = rng.integers(0, alphabet, size=(B, cap)).astype(np.int32)
    lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
    lens[0], lens[1] = cap, 0
    plens = np.minimum(lens, rng.integers(0, cap + 1, size=B)).astype(np.int32)
    ref = _retrieve_both(toks, lens, plens, n_min, n_max, k, C)
    if cap >= 1500:
        assert (ref["n_cand"] > 0).any()


@pytest.mark.parametrize("B", [3, 513])
def test_retrieve_planted_spans_multi_tile_and_extras(B):
    """A 20000-token context (two LDS tiles) with spans repeated across the tile boundary, plus
    gathering of the alignment extras."""
    rng = np.random.default_rng(4)
    L, V, m = 20000, 50000, 2
    toks = rng.integers(0, V, size=(B, L + 64)).astype(np.int32)
    for b in range(B):
        span = toks[b, 100:140].copy()
        for dst in (5000, 2 * 4352 - 5, 11200, 11264 - 5, 19000):  # tiles: 11264 positions with few sequences, 4352 with many
            toks[b, dst:dst + 40] = span
        toks[b, L - 6:L] = span[10:16]  # the context ends inside the span
    lens = np.full(B, L, np.int32)
    plens = np.resize(np.array([L, 12000, 0], np.int32), B)
    extras = rng.integers(0, V, size=(B * L, m)).astype(np.int32)
    n_extras = rng.integers(0, m + 1, size=B * L).astype(np.uint8)
    extras[np.arange(m)[None, :] >= n_extras[:, None]] = -1
    ref = _retrieve_both(toks, lens, plens, 2, 6, 8, 8, extras=extras, n_extras=n_extras, m=m, xs=L)
    assert (ref["key_len"] == 6).all() and (ref["n_cand"] == 6).all()
    assert ref["src_pos"][0].tolist()[:6] == [19016, 11264 - 5 + 16, 11200 + 16, 2 * 4352 - 5 + 16, 5016, 116]


def test_retrieve_hash_collision_is_not_a_hit():
    """Two different bigrams with the same polynomial window hash: only the exact one is returned."""
    step = (1 << 32) - aasd.HASH_BASE  # (a+1)*B + (b+step) == a*B + b  (mod 2^32)
    a, b = 1000, 2000
    toks = np.array([[5, a + 1, b + step, 77, 6, a, b, 88, 9, a, b]], np.int32)
    assert ((a + 1) * aasd.HASH_BASE + (b + step)) % (1 << 32) == (a * aasd.HASH_BASE + b) % (1 << 32)
    ref = _retrieve_both(toks, [11], [11], 2, 2, 3, 4)
    assert ref["src_pos"][0].tolist() == [7, -1, -1, -1]


# --------------------------------------------------------------------------- verification
def _verify_case(rng, B, C, k, V, dtype, peaked=True):
    R = 1 + C * k
    z = rng.standard_normal((B, R, V)).astype(np.float32) * 1.5
    drafts = np.empty((B, C, k), np.int32)
    for b in range(B):
        for r in range(R):
            if peaked:
                top = rng.choice(V, 4, replace=False)
                z[b, r, top] = [24.0, 23.0, 22.0, 21.0]
    order = np.argsort(-z, axis=2)[:, :, :6]
    for b in range(B):
        for c in range(C):
            for j in range(k):
                rho = 0 if j == 0 else 1 + c * k + (j - 1)
                pick = rng.choice(6, p=[0.55, 0.25, 0.08, 0.06, 0.03, 0.03])
                drafts[b, c, j] = order[b, rho, pick]
    drafts[rng.random((B, C, k)) < 0.02] = V + 5       # out-of-vocabulary ids fail
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    strict = (rng.random((B, C, k)) < 0.3).astype(np.uint8)
    return _dev_logits(z.reshape(B * R, V), dtype).view(B, R, V), drafts, dl, strict


def _verify_both(zd, drafts, dl, strict, alpha, beta, flags, tally):
    """Oracle against both launch forms of aasd_verify: sweep + tail, and the one-launch form over a workspace
    whose counters are zero (twice in a row on the same workspace: the kernel leaves them at zero)."""
    ref = oracle.verify(synth.to_host_bits(zd), drafts, dl, strict, alpha=bk.f32(alpha), beta=bk.f32(beta), flags=flags)
    t = lambda a, dt: None if a is None else torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    args = (zd, t(drafts, torch.int32), t(dl, torch.int32), t(strict, torch.uint8))
    out = bk.to_np(aasd.verify(*args, alpha=alpha, beta=beta, flags=flags))
    torch.cuda.synchronize()
    bk.compare_verify(out, ref, tally)
    B, C, k = drafts.shape
    ws = torch.zeros(aasd.verify_workspace_bytes(B, C, k, zd.shape[2], aasd.BF16 if zd.dtype == torch.bfloat16 else aasd.F32),
                     dtype=torch.uint8, device=DEV)
    first = None
    for rep in range(2):
        one = bk.to_np(aasd.verify(*args, alpha=alpha, beta=beta, flags=flags, workspace=ws, zeroed_workspace=True))
        torch.cuda.synchronize()
        if first is None:
            first = one
            bk.compare_verify(one, ref, bk.Tally())      # its sums are formed in another order: to the oracle's bar on its own
            np.testing.assert_array_equal(one["row_argmax"], out["row_argmax"])
        for name, a in first.items():
            if a is not None:
                assert a.tobytes() == one[name].tobytes(), (name, rep)     # byte-identical reruns
    assert int(ws[:128].view(torch.int32).abs().sum().item()) == 0          # the first sequence's counter is back at zero
    return ref


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,C,k,V", [(1, 1, 1, 50), (3, 1, 4, 32000), (2, 3, 5, 4099), (5, 16, 8, 1000), (2, 32, 16, 300)])
def test_verify_random_cases(dtype, B, C, k, V):
    rng = np.random.default_rng(B * 1000 + C * 10 + k)
    tally = bk.Tally()
    for peaked in (True, False):
        zd, drafts, dl, strict = _verify_case(rng, B, C, k, V, dtype, peaked)
        for alpha, beta, flags, st in [(0.1, 0.1, 0, strict), (0.2, 0.1, 0, None), (0.0, 0.1, aasd.VERIFY_NO_CLAMP, None),
                                       (0.0, 0.0, 0, None), (0.0, 1.0, 0, strict)]:
            _verify_both(zd, drafts, dl, st, alpha, beta, flags, tally)
    print("verify", dtype, B, C, k, V, tally)


def test_verify_strided_sequences_and_determinism():
    rng = np.random.default_rng(12)
    B, C, k, V = 3, 2, 4, 2000
    R = 1 + C * k
    zd, drafts, dl, strict = _verify_case(rng, B, C, k, V, "bf16")
    big = torch.zeros((B, R + 2, V + 24), dtype=torch.bfloat16, device=DEV)
    big[:, :R, :V] = zd
    view = big[:, :R, :V]
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    a = bk.to_np(aasd.verify(zd, t(drafts, torch.int32), t(dl, torch.int32), t(strict, torch.uint8)))
    b = bk.to_np(aasd.verify(view, t(drafts, torch.int32), t(dl, torch.int32), t(strict, torch.uint8)))
    torch.cuda.synchronize()
    for name in a:
        if a[name] is not None:
            assert a[name].tobytes() == b[name].tobytes(), name


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_verify_short_launch_of_many_segments_with_masked_logits_and_unaligned_rows(dtype):
    """Few rows of a large vocabulary: the sweep cuts every row into many segments and its workgroups merge their
    waves' partials.  Rows start at any element offset (odd row stride inside a larger buffer), a third of the
    logits are -inf, one row has a single finite logit and one segment of one row is -inf throughout."""
    rng = np.random.default_rng(77)
    B, C, k, V = 2, 2, 3, 40003
    R = 1 + C * k
    zd, drafts, dl, strict = _verify_case(rng, B, C, k, V, dtype, peaked=True)
    z = zd.float().cpu().numpy()
    z[rng.random(z.shape) < 0.33] = -np.inf
    z[0, 1, :] = -np.inf; z[0, 1, 31111] = 0.5
    z[1, 2, 10000:13000] = -np.inf
    for b in range(B):      # the first draft of every candidate is the bonus row's best finite token: something is accepted
        drafts[b, :, 0] = int(np.argmax(z[b, 0]))
    big = torch.full((B, R + 1, V + 7), 77.0, dtype=zd.dtype, device=DEV)     # the padding would win every row if it were read
    big[:, :R, :V] = torch.from_numpy(z).to(DEV).to(zd.dtype)
    tally = bk.Tally()
    for alpha, beta, flags, st in [(0.1, 0.1, 0, strict), (0.3, 0.05, 0, None), (0.0, 0.2, aasd.VERIFY_NO_CLAMP, None)]:
        ref = _verify_both(big[:, :R, :V], drafts, dl, st, alpha, beta, flags, tally)
    assert aasd.verify_launches(B, C, k, V, aasd.BF16 if dtype == "bf16" else aasd.F32) == 2
    assert ref["accept_len"].max() >= 1
    print("masked short launch", dtype, tally)


# --------------------------------------------------------------------------- the five workloads
def _align_workload(w, b, rows, tally, peaked=False, mode=oracle.EXTRAS_TOP):
    g, copied = synth.token_stream(w, b)
    z = synth.prefill_logits(w, b, g, copied, DEV, rows=rows, peaked=peaked)
    nt = synth.next_tokens(w, g)[rows]
    base = b * w.L + (rows.start or 0)
    got = bk.hip_align(z, nt, w.m, w.c, mode, seed=w.seed, row_id_base=base)
    ref = bk.oracle_align(z, nt, w.m, w.c, mode, seed=w.seed, row_id_base=base)
    bk.compare_align(got, ref, tally, mode)
    return got


def test_workload_tiny_full():
    """Config 1 in full: all 256 prefill rows (both modes) and the 64-step decode loop."""
    w = synth.WORKLOADS["tiny"]
    tally = bk.Tally()
    got = _align_workload(w, 0, slice(0, w.L), tally, mode=oracle.EXTRAS_TOP)
    _align_workload(w, 0, slice(0, w.L), tally, mode=oracle.EXTRAS_SAMPLE)
    assert 0.2 < got["misaligned"].mean() < 0.8
    pb = bk.ParityBackend(DEV)
    trace = harness.decode(w, pb)
    assert len(trace.steps) == w.steps
    print("tiny", tally, pb.tally, "tokens/step", trace.mean_accept_len)
    # LLM-like rows (exercise the unclamped alpha*H + beta branch) over a context dense in repeats, with
    # the alignment extras gathered along the drafts: drafts are found and accepted
    wd = synth.scaled(w, coverage=0.9, spans=0)
    g, copied = synth.token_stream(wd, 0)
    z = synth.prefill_logits(wd, 0, g, copied, DEV, peaked=True)
    al = bk.hip_align(z, synth.next_tokens(wd, g), wd.m, wd.c, oracle.EXTRAS_TOP)
    pb2 = bk.ParityBackend(DEV, one_launch=True)
    tr2 = harness.decode(wd, pb2, peaked=True, extras=al["extras"], n_extras=al["n_extras"])
    hits = sum(int(s.retrieved["n_cand"][0] > 0) for s in tr2.steps)
    print("tiny dense/peaked", pb2.tally, "tokens/step", tr2.mean_accept_len, "steps with drafts", hits)
    assert hits > 5 and tr2.mean_accept_len > 1.2


@pytest.mark.parametrize("name,rows_n,steps", [("llama3_single", 192, 24), ("long_context", 128, 12),
                                               ("batched_serving", 64, 6), ("stress_tree", 64, 3)])
def test_workloads_scaled(name, rows_n, steps):
    """Configs 2-5 at full vocabulary and full per-step shape, with fewer rows and steps."""
    w0 = synth.WORKLOADS[name]
    tally = bk.Tally()
    _align_workload(w0, 0, slice(0, rows_n), tally, mode=oracle.EXTRAS_TOP)
    _align_workload(w0, w0.B - 1, slice(w0.L - rows_n, w0.L), tally, mode=oracle.EXTRAS_SAMPLE)
    _align_workload(w0, 0, slice(0, 32), tally, peaked=True)
    w = synth.scaled(w0, B=min(w0.B, 4), steps=steps)
    pb = bk.ParityBackend(DEV)
    trace = harness.decode(w, pb)
    pb2 = bk.ParityBackend(DEV, one_launch=True)
    harness.decode(synth.scaled(w, steps=4), pb2, peaked=True)
    print(name, tally, pb.tally, pb2.tally, "MAL", trace.mean_accept_len)


# --------------------------------------------------------------------------- full sizes, in the launch plans bench.py times
# (configs 3-5: tests/test_gpu_full_configs.py)
def test_full_size_llama3_single_as_benched():
    """Config 2 at full size in bench.py's launch configuration: alignment sampling over all 2048 prefill
    rows in one call, verification of all 512 decode steps as one batch of 512 x 9 rows.  The oracle checks
    every prefill row and every decode step."""
    w = synth.WORKLOADS["llama3_single"]
    tally = bk.Tally()
    _align_workload(w, 0, slice(0, w.L), tally, mode=oracle.EXTRAS_TOP)
    # decode loop on the HIP path (sequential 9-row steps), then the batched pass over the same inputs
    hip = bk.HipBackend(DEV)
    trace = harness.decode(w, hip, keep_logits=True)
    S = len(trace.steps)
    logits = torch.stack([s.logits for s in trace.steps]).view(S, w.R, w.V)
    tokens = torch.from_numpy(np.tile(trace.tokens, (S, 1))).to(DEV)
    lens = torch.from_numpy(np.concatenate([s.length for s in trace.steps]).astype(np.int32)).to(DEV)
    plens = torch.full((S,), w.L, dtype=torch.int32, device=DEV)
    r = aasd.retrieve_drafts(tokens, lens, plens, w.n_min, w.n_max, w.k, w.C)
    v = aasd.verify(logits, r["drafts"], r["draft_len"], r["strict"], alpha=w.alpha, beta=w.beta)
    torch.cuda.synchronize()
    r_np, v_np = bk.to_np(r), bk.to_np(v)
    # batched == sequential, bit for bit
    for name in ("drafts", "draft_len", "src_pos", "n_cand", "key_len", "strict"):
        np.testing.assert_array_equal(r_np[name], np.concatenate([s.retrieved[name] for s in trace.steps]), err_msg=name)
    for name in ("accept_len", "best_cand", "next_token"):
        np.testing.assert_array_equal(v_np[name], np.concatenate([s.verified[name] for s in trace.steps]), err_msg=name)
    # oracle on every decode step
    ref_r = oracle.retrieve_drafts(np.tile(trace.tokens, (S, 1)), lens.cpu().numpy(), plens.cpu().numpy(),
                                   w.n_min, w.n_max, w.k, w.C)
    bk.compare_retrieve(r_np, ref_r)
    ref_v = oracle.verify(synth.to_host_bits(logits), ref_r["drafts"], ref_r["draft_len"], ref_r["strict"],
                          alpha=bk.f32(w.alpha), beta=bk.f32(w.beta))
    bk.compare_verify(v_np, ref_v, tally)
    print("llama3_single full", tally)


# --------------------------------------------------------------------------- full-vocabulary draws
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V,m", [(2, 1), (5, 2), (9, 4), (1000, 2), (4099, 3), (32000, 2), (128256, 2)])
def test_gumbel_extras_parity(dtype, V, m):
    """EXTRAS_GUMBEL: the draws are the m largest keys z + G over the whole row; same picks as the oracle
    unless two neighbouring keys are closer than the fp32 keys can tell apart (counted)."""
    rng = np.random.default_rng(V * 7 + m)
    rows = 48 if V > 20000 else 200
    zd = _random_rows(rng, rows, V, dtype)
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    nt[::7] = -1
    tally = bk.Tally()
    for seed, base in [(1, 0), ((5 << 32) | 9, (1 << 32) + 3)]:
        ref = bk.oracle_align(zd, nt, m, max(m, 1), oracle.EXTRAS_GUMBEL, seed=seed, row_id_base=base)
        got = bk.hip_align(zd, nt, m, max(m, 1), oracle.EXTRAS_GUMBEL, seed=seed, row_id_base=base)
        bk.compare_align(got, ref, tally, oracle.EXTRAS_GUMBEL)
        mis = ref["misaligned"] == 1
        assert (ref["n_extras"][mis] == min(m, V - 1)).all() and (ref["n_extras"][~mis] == 0).all()
    assert tally.near_disagreements <= tally.near_decisions
    print("gumbel", dtype, V, m, tally)


@pytest.mark.parametrize("segments", [1, 2, 5, 16])
def test_gumbel_extras_with_few_and_many_shares_per_row(segments, forced_plan):
    """The draw kernel skips tokens below the wave's running bound; how soon the bound bites depends on how many
    tokens a lane sees, i.e. on the workgroups per row: 1 (500 tokens per lane at this V), 2, 5 and 16 (31 per lane).
    Rows with a dominant token, with equal logits everywhere (every key then hangs on the random word alone) and with
    most tokens at probability zero are in."""
    forced_plan(f"0,0,{segments}")
    rng = np.random.default_rng(segments)
    rows, V, m = 24, 128256, 2
    z = rng.standard_normal((rows, V)).astype(np.float32) * 2
    z[0:4, 77] = 30.0                      # dominant
    z[4:8, :] = 0.0                        # all equal
    z[8:12, :] = -np.inf                   # nearly everything impossible
    z[8:12, 1000:1010] = 1.0
    zd = _dev_logits(z, "bf16")
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    nt[8:12] = 5                           # a token of probability zero as the prompt's: the row is misaligned
    tally = bk.Tally()
    for seed in (3, 11):
        ref = bk.oracle_align(zd, nt, m, m, oracle.EXTRAS_GUMBEL, seed=seed, row_id_base=1 << 33)
        got = bk.hip_align(zd, nt, m, m, oracle.EXTRAS_GUMBEL, seed=seed, row_id_base=1 << 33)
        bk.compare_align(got, ref, tally, oracle.EXTRAS_GUMBEL)
    assert tally.near_disagreements <= tally.near_decisions
    print("gumbel shares", segments, tally)


def test_gumbel_extras_unaligned_rows_peaked_rows_and_near_counter():
    rng = np.random.default_rng(31)
    rows, V = 300, 5003
    big = torch.zeros((rows, V + 5), dtype=torch.bfloat16, device=DEV)   # odd stride: rows start at any 2-byte offset
    z = rng.standard_normal((rows, V)).astype(np.float32) * 2
    z[:, 17] = 16.0                                                      # one dominant token: it is (nearly) always drawn first
    big[:, :V] = torch.from_numpy(z).to(DEV).to(torch.bfloat16)
    view = big[:, :V]
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    tally = bk.Tally()
    ref = bk.oracle_align(view, nt, 3, 3, oracle.EXTRAS_GUMBEL, seed=4)
    near = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = aasd.align_sample(view, torch.from_numpy(nt).to(DEV), m=3, c=3, mode=aasd.EXTRAS_GUMBEL, seed=4, near_count=near)
    torch.cuda.synchronize()
    bk.compare_align(bk.to_np(out), ref, tally, oracle.EXTRAS_GUMBEL)
    assert (ref["extras"][nt != 17, 0] == 17).mean() > 0.97
    margin = np.where(ref["draw_margin"] < 0, np.inf, ref["draw_margin"]).min(axis=1)
    lo, hi = int((margin < 0.5 * bk.NEAR_GUMBEL).sum()), int((margin < 2 * bk.NEAR_GUMBEL).sum())
    assert lo <= int(near.item()) <= hi


def test_gumbel_extras_many_rows_hit_near_decisions_and_zero_probability_tokens():
    """Enough draws that some neighbouring keys fall within the fp32 resolution: those rows are counted, all
    others must agree exactly, and the kernel's own counter brackets the oracle's.  Some tokens have p = 0."""
    rng = np.random.default_rng(9)
    rows, V, m = 40000, 24, 4
    z = (rng.standard_normal((rows, V)) * 1.5).astype(np.float32)
    z[rng.random((rows, V)) < 0.1] = -np.inf
    zd = _dev_logits(z, "f32")
    nt = rng.integers(0, V, size=rows).astype(np.int32)
    tally = bk.Tally()
    ref = bk.oracle_align(zd, nt, m, m, oracle.EXTRAS_GUMBEL, seed=77)
    near = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = aasd.align_sample(zd, torch.from_numpy(nt).to(DEV), m=m, c=m, mode=aasd.EXTRAS_GUMBEL, seed=77, near_count=near)
    torch.cuda.synchronize()
    bk.compare_align(bk.to_np(out), ref, tally, oracle.EXTRAS_GUMBEL)
    assert tally.near_decisions >= 2, tally
    margin = np.where(ref["draw_margin"] < 0, np.inf, ref["draw_margin"]).min(axis=1)
    lo, hi = int((margin < 0.5 * bk.NEAR_GUMBEL).sum()), int((margin < 2 * bk.NEAR_GUMBEL).sum())
    assert lo <= int(near.item()) <= hi, (lo, int(near.item()), hi)
    print("gumbel many rows", tally, "kernel near", int(near.item()), "oracle bracket", lo, hi)


# --------------------------------------------------------------------------- top-k verification (Sec. 4.4 ablation)
def _topk_case(rng, B, C, k, V, dtype, ties):
    R = 1 + C * k
    z = rng.standard_normal((B, R, V)).astype(np.float32) * 1.5
    if ties:
        z = np.round(z * 2) / 2
    zd = _dev_logits(z.reshape(B * R, V), dtype).view(B, R, V)
    zf = zd.float().cpu().numpy()
    order = np.argsort(-zf, axis=2, kind="stable")
    drafts = np.empty((B, C, k), np.int32)
    for b in range(B):
        for c in range(C):
            for j in range(k):
                rho = 0 if j == 0 else 1 + c * k + (j - 1)
                drafts[b, c, j] = order[b, rho, min(V - 1, int(rng.geometric(0.25)) - 1)]
    drafts[rng.random((B, C, k)) < 0.02] = V + 3
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    return zd, drafts, dl


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,C,k,V", [(1, 1, 1, 3), (3, 1, 4, 32000), (2, 3, 5, 4099), (5, 16, 8, 1000), (2, 32, 16, 300),
                                     (600, 1, 8, 2000)])
def test_verify_topk_parity(dtype, B, C, k, V):
    rng = np.random.default_rng(B * 100 + C + k)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    for ties in (False, True):
        zd, drafts, dl = _topk_case(rng, B, C, k, V, dtype, ties)
        bits = synth.to_host_bits(zd)
        for topk in (1, 2, 5, 8):
            ref = oracle.verify_topk(bits, drafts, dl, topk=topk)
            got = bk.to_np(aasd.verify_topk(zd, t(drafts, torch.int32), t(dl, torch.int32), topk=topk))
            torch.cuda.synchronize()
            for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
                np.testing.assert_array_equal(got[name], ref[name], err_msg=f"{name} topk={topk} ties={ties}")
            want = ((ref["tok_rank"] >= 0) & (ref["tok_rank"] < topk)).astype(np.uint8)
            np.testing.assert_array_equal(got["tok_pass"], want, err_msg=f"tok_pass topk={topk} ties={ties}")
        assert ref["accept_len"].max() >= min(1, dl.max())


def test_verify_topk_top1_equals_strict_verification_and_full_shape():
    """k = 1 is strict verification (same decisions as aasd_verify with every token strict); also the benched
    shape of config 2 (512 x 9 rows of V = 128256 bf16) against the oracle on sampled sequences."""
    w = synth.WORKLOADS["llama3_single"]
    rng = np.random.default_rng(6)
    B = 512
    g = torch.Generator(device=DEV).manual_seed(2)
    zd = (torch.randn((B, w.R, w.V), generator=g, device=DEV) * 1.7).to(torch.bfloat16)
    top = torch.topk(zd.float(), 6, dim=2).indices.cpu().numpy()
    drafts = np.empty((B, 1, w.k), np.int32)
    for j in range(w.k):
        drafts[:, 0, j] = top[np.arange(B), j, rng.geometric(0.5, size=B).clip(1, 6) - 1]
    dl = np.full((B, 1), w.k, np.int32)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    one = bk.to_np(aasd.verify_topk(zd, t(drafts, torch.int32), t(dl, torch.int32), topk=1))
    strict = bk.to_np(aasd.verify(zd, t(drafts, torch.int32), t(dl, torch.int32), t(np.ones_like(drafts), torch.uint8)))
    five = bk.to_np(aasd.verify_topk(zd, t(drafts, torch.int32), t(dl, torch.int32), topk=5))
    torch.cuda.synchronize()
    for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
        np.testing.assert_array_equal(one[name], strict[name], err_msg=name)
    assert (five["accept_len"] >= one["accept_len"]).all() and five["accept_len"].mean() > one["accept_len"].mean() + 1
    for b in rng.choice(B, 4, replace=False):
        ref = oracle.verify_topk(synth.to_host_bits(zd[b:b + 1]), drafts[b:b + 1], dl[b:b + 1], topk=5)
        assert ref["accept_len"][0] == five["accept_len"][b] and ref["next_token"][0] == five["next_token"][b]
        assert (((ref["tok_rank"] >= 0) & (ref["tok_rank"] < 5)) == five["tok_pass"][b:b + 1].astype(bool)).all()


@pytest.mark.parametrize("one_launch", [False, True])
def test_decode_steps_captured_in_a_hip_graph_match_the_eager_launches(one_launch):
    """Retrieval and verification of several decode steps captured once and replayed: every replay, with eager
    work and synchronisations in between, gives the eager results (the library launches kernels only: no
    allocation, no memset, no host synchronisation inside its calls).  In the one-launch form the kernel itself
    puts its arrival counters back to zero, so a replay finds them as the capture did."""
    rng = np.random.default_rng(41)
    w = synth.scaled(synth.WORKLOADS["llama3_single"], V=6000, L=300, steps=12, coverage=0.9)
    g, cp = synth.token_stream(w, 0)
    S = 8
    toks = torch.from_numpy(g[:w.tok_cap].astype(np.int32)[None]).to(DEV)
    z = [_verify_case(rng, 1, w.C, w.k, w.V, "bf16")[0] for _ in range(S)]
    lens = [torch.tensor([w.L + 5 * s], dtype=torch.int32, device=DEV) for s in range(S)]
    plen = torch.tensor([w.L], dtype=torch.int32, device=DEV)
    r = aasd.retrieve_drafts(toks, lens[0], plen, w.n_min, w.n_max, w.k, w.C)
    ws = torch.zeros(aasd.verify_workspace_bytes(1, w.C, w.k, w.V, aasd.BF16), dtype=torch.uint8, device=DEV)
    v = aasd.verify(z[0], r["drafts"], r["draft_len"], r["strict"], workspace=ws, zeroed_workspace=one_launch)
    rec = [torch.zeros(4, dtype=torch.int32, device=DEV) for _ in range(S)]

    def steps():
        for s in range(S):
            aasd.retrieve_drafts(toks, lens[s], plen, w.n_min, w.n_max, w.k, w.C, out=r)
            aasd.verify(z[s], r["drafts"], r["draft_len"], r["strict"], workspace=ws, out=v, zeroed_workspace=one_launch)
            rec[s][0:1].copy_(v["accept_len"]); rec[s][1:2].copy_(v["next_token"]); rec[s][2:3].copy_(r["n_cand"])
            rec[s][3:4].copy_(r["src_pos"][0, :1])

    steps()
    torch.cuda.synchronize()
    eager = [x.clone() for x in rec]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        steps()
    torch.cuda.synchronize()
    for i in range(4):
        for x in rec:
            x.fill_(-9)
        other = aasd.verify(z[(i + 1) % S], r["drafts"], r["draft_len"], r["strict"])   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for s in range(S):
            assert (rec[s] == eager[s]).all(), (i, s, rec[s].tolist(), eager[s].tolist())
    assert any(int(e[2]) > 0 for e in eager)


def test_verify_topk_strided_rows_zero_probability_tokens_and_tiny_vocabularies():
    rng = np.random.default_rng(52)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    # rows embedded in a larger buffer: odd row stride (rows start at any 2-byte offset), gap between sequences
    B, C, k, V = 4, 3, 4, 1501
    R = 1 + C * k
    zd, drafts, dl = _topk_case(rng, B, C, k, V, "bf16", ties=True)
    big = torch.full((B, R + 2, V + 7), 99.0, dtype=torch.bfloat16, device=DEV)   # the padding would win every row if it were read
    big[:, :R, :V] = zd
    ref = oracle.verify_topk(synth.to_host_bits(zd), drafts, dl, topk=4)
    got = bk.to_np(aasd.verify_topk(big[:, :R, :V], t(drafts, torch.int32), t(dl, torch.int32), topk=4))
    for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    # tokens of probability zero, and vocabularies smaller than k
    for V in (1, 3, 7, 40):
        B, C, k = 6, 2, 3
        R = 1 + C * k
        z = rng.standard_normal((B, R, V)).astype(np.float32)
        z[rng.random((B, R, V)) < 0.4] = -np.inf
        z[:, :, 0] = np.where(np.isinf(z).all(axis=2), 0.0, z[:, :, 0])      # at least one finite logit per row
        zd = torch.from_numpy(z).to(DEV)
        drafts = rng.integers(0, V, size=(B, C, k)).astype(np.int32)
        dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
        for topk in (1, 2, 8):
            ref = oracle.verify_topk(z, drafts, dl, topk=topk)
            got = bk.to_np(aasd.verify_topk(zd, t(drafts, torch.int32), t(dl, torch.int32), topk=topk))
            for name in ("accept_len", "best_cand", "next_token", "row_argmax"):
                np.testing.assert_array_equal(got[name], ref[name], err_msg=f"{name} V={V} topk={topk}")
            want = ((ref["tok_rank"] >= 0) & (ref["tok_rank"] < topk)).astype(np.uint8)
            np.testing.assert_array_equal(got["tok_pass"], want, err_msg=f"tok_pass V={V} topk={topk}")


def test_more_work_than_one_launch_covers():
    """A launch covers at most 2^22 workgroups: 5,000,000 prefill rows and 500,000 sequences of 9 verify rows go
    out as two launches each (tiny vocabulary, so that the oracle can follow)."""
    rng = np.random.default_rng(71)
    rows, V = 5_000_000, 8
    z = (rng.standard_normal((rows, V)) * 2).astype(np.float32)
    zd = torch.from_numpy(z).to(DEV).to(torch.bfloat16)
    nt = rng.integers(-1, V, size=rows).astype(np.int32)
    tally = bk.Tally()
    got = bk.hip_align(zd, nt, 1, 2, oracle.EXTRAS_TOP)
    ref = bk.oracle_align(zd, nt, 1, 2, oracle.EXTRAS_TOP)
    bk.compare_align(got, ref, tally, oracle.EXTRAS_TOP)
    got = bk.hip_align(zd, nt, 1, 1, oracle.EXTRAS_GUMBEL, seed=5, want_rank=False)     # the draw kernel is chunked too
    ref = bk.oracle_align(zd, nt, 1, 1, oracle.EXTRAS_GUMBEL, seed=5)
    bk.compare_align(got, ref, tally, oracle.EXTRAS_GUMBEL)
    B, C, k = 500_000, 1, 8
    R = 1 + C * k
    zv = zd[:B * R].view(B, R, V)
    drafts = rng.integers(0, V, size=(B, C, k)).astype(np.int32)
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    _verify_both(zv, drafts, dl, None, 0.1, 0.1, 0, tally)
    print("large counts", tally)


# --------------------------------------------------------------------------- measurement hooks
def test_event_hooks_time_the_kernel_and_change_nothing():
    """With the hooks set, the sweep (and draw) kernels are launched with start and stop events: the results are
    byte for byte those of a call without hooks, and the events hold a duration that is positive and no longer than
    the whole call as the stream sees it."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")

    def event():
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def elapsed_ms(a, b):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value

    rng = np.random.default_rng(5)
    z = _random_rows(rng, 600, 32000, "bf16")
    nt = torch.from_numpy(rng.integers(0, 32000, size=600).astype(np.int32)).to(DEV)
    zd, drafts, dl, strict = _verify_case(rng, 4, 2, 4, 32000, "bf16")
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    vargs = (zd, t(drafts, torch.int32), t(dl, torch.int32), t(strict, torch.uint8))
    ws = torch.zeros(aasd.verify_workspace_bytes(4, 2, 4, 32000, aasd.BF16), dtype=torch.uint8, device=DEV)
    calls = {
        "align top": (aasd.set_sweep_events, lambda: aasd.align_sample(z, nt, m=2, c=4)),
        "align gumbel, sweep": (aasd.set_sweep_events, lambda: aasd.align_sample(z, nt, m=2, c=2, mode=aasd.EXTRAS_GUMBEL, seed=3)),
        "align gumbel, draws": (aasd.set_draw_events, lambda: aasd.align_sample(z, nt, m=2, c=2, mode=aasd.EXTRAS_GUMBEL, seed=3)),
        "verify, two launches": (aasd.set_sweep_events, lambda: aasd.verify(*vargs)),
        "verify, one launch": (aasd.set_sweep_events, lambda: aasd.verify(*vargs, workspace=ws, zeroed_workspace=True)),
        "verify top-k": (aasd.set_sweep_events, lambda: aasd.verify_topk(*vargs[:3], topk=3)),
    }
    for name, (hook, call) in calls.items():
        plain = bk.to_np(call())
        torch.cuda.synchronize()
        a, b = event(), event()
        o0, o1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        hook(a, b)
        try:
            o0.record()
            timed = bk.to_np(call())
            o1.record()
        finally:
            hook(None, None)
        torch.cuda.synchronize()
        for key, v in plain.items():
            if v is not None:
                assert v.tobytes() == timed[key].tobytes(), (name, key)
        inner, outer = elapsed_ms(a, b), o0.elapsed_time(o1)
        assert 0.0 < inner <= outer, (name, inner, outer)
        assert hip.hipEventDestroy(a) == 0 and hip.hipEventDestroy(b) == 0


def test_more_workgroups_than_one_launch_takes(forced_plan):
    """1.5 million verify rows cut into 3 segments each are 4.5 million workgroups: more than one launch takes
    (2^22), so the sweep is launched twice, the second time starting at a row far from zero.  Every sequence is checked."""
    forced_plan("0,0,3")
    rng = np.random.default_rng(4500000)
    B, C, k, V = 500_000, 1, 2, 64
    R = 1 + C * k
    z = (rng.standard_normal((B, R, V)) * 2).astype(np.float32)
    z[:, :, 7] += 9.0
    drafts = rng.integers(0, V, size=(B, C, k)).astype(np.int32)
    drafts[rng.random((B, C, k)) < 0.5] = 7
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    zd = _dev_logits(z.reshape(B * R, V), "bf16").view(B, R, V)
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    out = bk.to_np(aasd.verify(zd, t(drafts, torch.int32), t(dl, torch.int32), None, alpha=0.1, beta=0.1))
    torch.cuda.synchronize()
    ref = bk.oracle_verify_seqs(synth.to_host_bits(zd), drafts, dl, None, bk.f32(0.1), bk.f32(0.1))
    tally = bk.Tally()
    bk.compare_verify(out, ref, tally)
    assert ref["accept_len"].max() == 2 and 0.2 < (ref["accept_len"] > 0).mean() < 0.9
    print("4.5 million workgroups", tally)
