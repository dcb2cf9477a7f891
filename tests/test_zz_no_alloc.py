"""aasd_verify_static (verification on the library's built-in scratch memory, for callers that cannot
allocate) against aasd_verify, through the C ABI: same kernels, so the same bits as the form of aasd_verify
that runs the same launches; two calls in a row on the shared scratch, the second on a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_13204_amd as aasd
from tests import synth
from tests import backends as bk

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(rng, B, C, k, V, dtype):
    R = 1 + C * k
    z = rng.standard_normal((B, R, V)).astype(np.float32) * 1.5
    for b in range(B):
        for r in range(R):
            z[b, r, rng.choice(V, 4, replace=False)] = [24.0, 23.0, 22.0, 21.0]
    order = np.argsort(-z, axis=2)[:, :, :4]
    drafts = np.empty((B, C, k), np.int32)
    for b in range(B):
        for c in range(C):
            for j in range(k):
                rho = 0 if j == 0 else 1 + c * k + (j - 1)
                drafts[b, c, j] = order[b, rho, rng.choice(4, p=[0.6, 0.25, 0.1, 0.05])]
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    strict = (rng.random((B, C, k)) < 0.3).astype(np.uint8)
    zd = torch.from_numpy(z).to(DEV)
    zd = zd.to(torch.bfloat16) if dtype == "bf16" else zd
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dt)
    return zd, t(drafts, torch.int32), t(dl, torch.int32), t(strict, torch.uint8), (drafts, dl, strict)


def _outputs(B, C, k):
    R = 1 + C * k
    e = lambda shape, dt: torch.full(shape, -7, dtype=dt, device=DEV)
    return dict(accept_len=e((B,), torch.int32), best_cand=e((B,), torch.int32), next_token=e((B,), torch.int32),
                row_entropy=e((B, R), torch.float32), row_pmax=e((B, R), torch.float32), row_argmax=e((B, R), torch.int32),
                tok_p=e((B, C, k), torch.float32), tok_delta=e((B, C, k), torch.float32), near_count=e((B,), torch.int32))


def _check(rng, B, C, k, V, dtype, alpha=0.1, beta=0.1, flags=0):
    zd, drafts, dl, strict, host = _case(rng, B, C, k, V, dtype)
    got = bk.to_np(aasd.verify_static(zd, drafts, dl, strict, _outputs(B, C, k), alpha=alpha, beta=beta, flags=flags))
    torch.cuda.synchronize()
    # the existing entry point, in the form that runs the same launches
    dt = aasd.BF16 if dtype == "bf16" else aasd.F32
    ws = torch.zeros(aasd.verify_workspace_bytes(B, C, k, V, dt), dtype=torch.uint8, device=DEV)
    same = bk.to_np(aasd.verify(zd, drafts, dl, strict, alpha=alpha, beta=beta, flags=flags, workspace=ws, zeroed_workspace=True))
    torch.cuda.synchronize()
    for name, a in same.items():
        assert a.tobytes() == got[name].tobytes(), name
    # and its default form (two launches; sums in another order), to the bar of the oracle tests
    two = bk.to_np(aasd.verify(zd, drafts, dl, strict, alpha=alpha, beta=beta, flags=flags))
    np.testing.assert_array_equal(got["row_argmax"], two["row_argmax"])
    for name in ("row_entropy", "row_pmax", "tok_p", "tok_delta"):
        floor = bk.H_FLOOR if name == "row_entropy" else bk.P_FLOOR
        assert bk.rel_err(got[name], two[name], floor).max(initial=0.0) <= bk.REL_TOL, name
    clear = two["near_count"] == 0
    for name in ("accept_len", "best_cand", "next_token"):
        assert (got[name] == two[name])[clear].all(), name
    # and the oracle
    ref = oracle.verify(synth.to_host_bits(zd), *host, alpha=bk.f32(alpha), beta=bk.f32(beta), flags=flags)
    bk.compare_verify(got, ref, bk.Tally())
    return got


def test_verify_static_matches_verify_on_two_calls_in_a_row():
    rng = np.random.default_rng(7)
    assert aasd.verify_static_max_bytes() == 4 << 20
    a = _check(rng, 32, 1, 8, 128256, "bf16")       # a decode step of config 4: one launch, counters in groups
    b = _check(rng, 3, 2, 4, 5003, "bf16")          # right after it, smaller: same scratch, counters were left at zero
    assert a["accept_len"].max() >= 1 and b["accept_len"].max() >= 1
    _check(rng, 1, 1, 8, 128256, "bf16")            # a decode step of config 2
    _check(rng, 5, 4, 3, 777, "f32", alpha=0.0, beta=0.1, flags=aasd.VERIFY_NO_CLAMP)
    _check(rng, 64, 16, 8, 4099, "bf16")            # 8256 rows: served in two launches from the same scratch
    _check(rng, 2, 1, 2, 300, "f32")


def test_verify_static_rejects_what_its_scratch_cannot_hold():
    B, C, k, V = 300, 16, 8, 64                      # 38700 rows of 4 partials: more than 4 MiB
    z = torch.zeros((B, 1 + C * k, V), dtype=torch.bfloat16, device=DEV)
    drafts = torch.zeros((B, C, k), dtype=torch.int32, device=DEV)
    dl = torch.zeros((B, C), dtype=torch.int32, device=DEV)
    out = _outputs(B, C, k)
    with pytest.raises(aasd.AasdError) as e:
        aasd.verify_static(z, drafts, dl, None, out)
    assert e.value.code == -2 and "built-in scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (out["accept_len"] == -7).all()           # nothing was enqueued
    with pytest.raises(aasd.AasdError):
        aasd.verify_static(z[:2], drafts[:2], dl[:2], None, out, flags=aasd.VERIFY_ZEROED_WORKSPACE)


def test_verify_static_in_a_captured_graph():
    """The callers it is for: capture once, replay with eager work in between; every replay gives the eager result."""
    rng = np.random.default_rng(9)
    B, C, k, V = 4, 2, 4, 6000
    cases = [_case(rng, B, C, k, V, "bf16") for _ in range(3)]
    outs = [_outputs(B, C, k) for _ in cases]
    eager = []
    for (zd, d, dl, st, _), o in zip(cases, outs):
        eager.append({n: v.clone() for n, v in aasd.verify_static(zd, d, dl, st, o).items()})
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for (zd, d, dl, st, _), o in zip(cases, outs):
            aasd.verify_static(zd, d, dl, st, o)
    torch.cuda.synchronize()
    for i in range(3):
        for o in outs:
            for v in o.values():
                v.fill_(-9)
        aasd.verify_static(*cases[i][:4], _outputs(B, C, k))      # eager work on the same scratch between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            for n in o:
                assert (o[n] == e[n]).all(), (i, n)
