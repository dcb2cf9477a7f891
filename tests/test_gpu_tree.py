"""Parity of the HIP draft-tree path (tree build, tree attention mask, tree verification; Sec. 3.2
Eq. 2 and Sec. 3.3) with the CPU oracle, through the C ABI.  Integers bit-exact; decisions whose
oracle margin is below 1e-6 are counted instead; probabilities and entropies within 1e-5."""
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


def _random_candidates(rng, B, C, k, m, alphabet=3):
    drafts = rng.integers(0, alphabet, size=(B, C, k)).astype(np.int32)   # tiny alphabet: many shared prefixes
    drafts[rng.random((B, C, k)) < 0.05] = -1                             # a missing token ends the path
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    strict = (rng.random((B, C, k)) < 0.4).astype(np.uint8)
    dx = None
    if m:
        dx = rng.integers(0, alphabet + 1, size=(B, C, k, m)).astype(np.int32)
        dx[rng.random((B, C, k, m)) < 0.5] = -1
    return drafts, dl, strict, dx


def _build_both(drafts, dl, strict, dx, root, N):
    ref = oracle.build_tree(drafts, dl, strict, dx, root_tok=root, max_nodes=N)
    got = bk.to_np(aasd.build_tree(_t(drafts, torch.int32), _t(dl, torch.int32), _t(strict, torch.uint8),
                                   _t(dx, torch.int32), _t(root, torch.int32), max_nodes=N))
    torch.cuda.synchronize()
    for name in ("n_nodes", "node_token", "node_parent", "node_depth", "node_strict", "cand_node"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    np.testing.assert_array_equal(got["mask"].view(np.uint32), ref["mask"], err_msg="mask")
    return ref


@pytest.mark.parametrize("C,k,m,N", [(1, 1, 0, 1), (1, 4, 0, 8), (3, 4, 2, 64), (8, 8, 2, 40), (16, 8, 2, 256),
                                     (32, 16, 4, 256), (4, 6, 3, 5), (32, 16, 4, 33), (16, 8, 0, 129),
                                     (16, 8, 2, 385), (16, 8, 2, 512), (32, 16, 4, 512), (16, 8, 2, 300),
                                     (16, 5, 3, 200), (13, 5, 4, 200), (8, 16, 2, 300), (32, 3, 1, 97), (21, 4, 2, 33)])   # 64 and 65 events per layer: the last shape one wave builds, the first it does not
def test_build_tree_random_small_alphabet(C, k, m, N):
    rng = np.random.default_rng(C * 100 + k)
    for B, alphabet in [(12, 3), (5, 50), (1, 2)]:
        drafts, dl, strict, dx = _random_candidates(rng, B, C, k, m, alphabet)
        ref = _build_both(drafts, dl, strict, dx, np.arange(B, dtype=np.int32) + 7, N)
        assert ref["n_nodes"].max() <= N
    # optional inputs absent: no strict flags, no extras, no root token
    drafts, dl, _, _ = _random_candidates(rng, 4, C, k, 0)
    _build_both(drafts, dl, None, None, None, N)


@pytest.mark.parametrize("block", range(4))
def test_build_tree_random_shapes(block):
    """Random candidate counts, draft lengths, extras, node budgets and alphabets: layers of up to 64 events are
    built by one wave, larger ones by the whole workgroup; both against the oracle."""
    shapes = {True: 0, False: 0}
    for seed in range(block * 30, block * 30 + 30):
        rng = np.random.default_rng(50000 + seed)
        C, k, m = int(rng.integers(1, 33)), int(rng.integers(1, 17)), int(rng.integers(0, 5))
        N = int(rng.choice([1, 2, 5, 31, 32, 33, 64, 97, 129, 256, 385, 512, int(rng.integers(1, 513))]))
        B = int(rng.integers(1, 7))
        drafts, dl, strict, dx = _random_candidates(rng, B, C, k, m, int(rng.choice([1, 2, 3, 6, 50, 5000])))
        _build_both(drafts, dl, strict if rng.random() < 0.7 else None, dx,
                    np.arange(B, dtype=np.int32) if rng.random() < 0.5 else None, N)
        shapes[C * (1 + m) <= 64] += 1
    assert shapes[True] > 0 and shapes[False] > 0


def test_build_tree_full_and_empty():
    # all candidates identical -> one chain; all different -> C*k nodes; no candidate -> the root alone
    C, k = 16, 8
    same = np.tile(np.arange(k, dtype=np.int32), (1, C, 1))
    ref = _build_both(same, np.full((1, C), k, np.int32), None, None, np.array([3], np.int32), 256)
    assert ref["n_nodes"][0] == 1 + k
    diff = (np.arange(C * k, dtype=np.int32).reshape(1, C, k) * 7 + 11)
    ref = _build_both(diff, np.full((1, C), k, np.int32), None, None, np.array([3], np.int32), 256)
    assert ref["n_nodes"][0] == 1 + C * k
    ref = _build_both(diff, np.zeros((1, C), np.int32), None, None, np.array([3], np.int32), 64)
    assert ref["n_nodes"][0] == 1
    out = aasd.build_tree(torch.empty((0, C, k), dtype=torch.int32, device=DEV),
                          torch.empty((0, C), dtype=torch.int32, device=DEV), max_nodes=64)
    assert out["n_nodes"].numel() == 0


def test_tree_at_the_papers_largest_parameters():
    """16 candidates of 8 tokens with two extras at every position and nothing shared: 385 nodes (Sec. 3.2 Eq. 2
    with Sec. 4.1's cap of two extras).  Built and verified on the GPU against the oracle, also under a budget
    (256) that cuts the tree, and with prefixes shared between candidates so that the count varies."""
    rng = np.random.default_rng(385)
    B, C, k, m, V = 3, 16, 8, 2, 9000
    perm = np.stack([rng.permutation(V) for _ in range(B)]).astype(np.int32)           # all tokens of a sequence distinct
    drafts = perm[:, :C * k].reshape(B, C, k).copy()
    dx = perm[:, C * k:C * k * (1 + m)].reshape(B, C, k, m).copy()
    drafts[1, 8:, :3] = drafts[1, :8, :3]               # sequence 1: candidates share three-token prefixes in pairs
    drafts[2, 1:] = drafts[2, 0]                        # sequence 2: all candidates identical, one chain with extras
    dx[2, 1:] = dx[2, 0]
    dl = np.full((B, C), k, np.int32)
    strict = (rng.random((B, C, k)) < 0.3).astype(np.uint8)
    root = np.array([1, 2, 3], np.int32)
    dx_in_vocab = dx
    for N in (512, 385, 256):
        ref = _build_both(drafts, dl, strict, dx_in_vocab, root, N)
        if N >= 385:
            assert ref["n_nodes"][0] == 385 and 256 < ref["n_nodes"][1] < 385 and ref["n_nodes"][2] == 1 + k * 3
        else:
            assert ref["n_nodes"][0] == 256
    tree = oracle.build_tree(drafts, dl, strict, dx_in_vocab, root_tok=root, max_nodes=512)
    tally = bk.Tally()
    for dtype in ("bf16", "f32"):
        zd = _tree_logits(rng, tree, V, dtype, p_lead=0.8)
        ref, _ = _verify_tree_both(zd, tree, tree["node_strict"], 0.1, 0.1, 0, tally)
    assert ref["accept_len"].max() >= 3 and tally.tokens > 100
    print("385-node trees", tally)


def test_build_tree_from_retrieval_outputs():
    """Retrieval -> tree on the device, on a stream with planted copies and prefill extras."""
    w = synth.scaled(synth.WORKLOADS["stress_tree"], B=6, L=1500, steps=8)
    rng = np.random.default_rng(3)
    toks = np.stack([synth.token_stream(w, b)[0][:w.L] for b in range(w.B)]).astype(np.int32)
    lens = np.full(w.B, w.L, np.int32)
    m = 2
    extras = rng.integers(0, w.V, size=(w.B * w.L, m)).astype(np.int32)
    nx = rng.integers(0, m + 1, size=w.B * w.L).astype(np.uint8)
    extras[np.arange(m)[None, :] >= nx[:, None]] = -1
    r = aasd.retrieve_drafts(_t(toks, torch.int32), _t(lens, torch.int32), _t(lens, torch.int32), w.n_min, w.n_max, w.k,
                             w.C, extras=_t(extras, torch.int32), n_extras=_t(nx, torch.uint8), m=m, extras_stride=w.L)
    ref_r = oracle.retrieve_drafts(toks, lens, lens, w.n_min, w.n_max, w.k, w.C, extras=extras, n_extras=nx, m_x=m,
                                   extras_stride=w.L)
    root = toks[:, -1].copy()
    got = bk.to_np(aasd.build_tree(r["drafts"], r["draft_len"], r["strict"], r["draft_extras"], _t(root, torch.int32),
                                   max_nodes=160))
    ref = oracle.build_tree(ref_r["drafts"], ref_r["draft_len"], ref_r["strict"], ref_r["draft_extras"], root_tok=root,
                            max_nodes=160)
    torch.cuda.synchronize()
    assert ref["n_nodes"].max() > 8     # the planted copies give candidates
    for name in ("n_nodes", "node_token", "node_parent", "node_depth", "node_strict", "cand_node"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    np.testing.assert_array_equal(got["mask"].view(np.uint32), ref["mask"])


# --------------------------------------------------------------------------- tree verification
compare_verify_tree = bk.compare_verify_tree


def _tree_logits(rng, tree, V, dtype, peaked=True, poison=True, p_lead=0.0):
    """Rows for every node; the token of node i is put among the leaders of its parent's row."""
    B, N = tree["node_token"].shape
    z = rng.standard_normal((B, N, V)).astype(np.float32) * 1.5
    levels = [24.0, 23.0, 22.0, 21.0, 19.0, 12.0]
    for b in range(B):
        n = int(tree["n_nodes"][b])
        kids = {}
        for i in range(1, n):
            kids.setdefault(int(tree["node_parent"][b, i]), []).append(int(tree["node_token"][b, i]))
        for r in range(n):
            if not peaked:
                continue
            want = [t for t in dict.fromkeys(kids.get(r, [])) if 0 <= t < V][:6]
            fill = [int(x) for x in rng.permutation(V)[:6 + len(want)] if int(x) not in want]
            ids = (want + fill)[:min(6, V)]
            if rng.random() >= p_lead:      # else the first child keeps the top level
                rng.shuffle(ids)
            z[b, r, ids] = levels[:len(ids)]
    zd = torch.from_numpy(z).to(DEV)
    zd = zd.to(torch.bfloat16) if dtype == "bf16" else zd
    if poison:   # rows beyond n_nodes are never read: fill them with NaN
        for b in range(B):
            zd[b, int(tree["n_nodes"][b]):] = float("nan")
    return zd


def _verify_tree_both(zd, tree, strict, alpha, beta, flags, tally):
    ref = oracle.verify_tree(synth.to_host_bits(zd), tree["node_token"], tree["node_parent"], strict, tree["n_nodes"],
                             alpha=bk.f32(alpha), beta=bk.f32(beta), flags=flags)
    out = aasd.verify_tree(zd, _t(tree["node_token"], torch.int32), _t(tree["node_parent"], torch.int32),
                           _t(tree["n_nodes"], torch.int32), _t(strict, torch.uint8), alpha=alpha, beta=beta, flags=flags)
    torch.cuda.synchronize()
    compare_verify_tree(bk.to_np(out), ref, tally)
    return ref, out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,C,k,m,N,V", [(1, 1, 1, 0, 2, 50), (3, 2, 4, 2, 32, 32000), (2, 4, 5, 2, 64, 4099),
                                         (5, 16, 8, 2, 160, 1000), (2, 32, 16, 4, 256, 300), (9, 8, 8, 2, 40, 2000)])
def test_verify_tree_random_cases(dtype, B, C, k, m, N, V):
    rng = np.random.default_rng(B * 1000 + C * 10 + k)
    tally = bk.Tally()
    depth_seen = 0
    for peaked in (True, False):
        drafts, dl, strict, dx = _random_candidates(rng, B, C, k, m, alphabet=min(V, 40))
        drafts[rng.random(drafts.shape) < 0.03] = V + 5        # out-of-vocabulary ids fail
        tree = oracle.build_tree(drafts, dl, strict, dx, root_tok=np.zeros(B, np.int32), max_nodes=N)
        zd = _tree_logits(rng, tree, V, dtype, peaked)
        for alpha, beta, flags, st in [(0.1, 0.1, 0, tree["node_strict"]), (0.2, 0.1, 0, None),
                                       (0.0, 0.1, aasd.VERIFY_NO_CLAMP, None), (0.0, 0.0, 0, None),
                                       (0.0, 1.0, 0, tree["node_strict"])]:
            ref, _ = _verify_tree_both(zd, tree, st, alpha, beta, flags, tally)
            depth_seen = max(depth_seen, int(ref["accept_len"].max()))
    if k >= 4:
        assert depth_seen >= 2      # the cases do accept paths, not only roots
    print("verify_tree", dtype, B, C, k, V, tally)


def test_verify_tree_chain_equals_candidate_verification():
    """A tree that is one chain is the C = 1 case of aasd_verify: same rows, same decisions, same bits."""
    rng = np.random.default_rng(5)
    B, k, V = 6, 8, 5000
    drafts = rng.integers(0, V, size=(B, 1, k)).astype(np.int32)
    dl = rng.integers(0, k + 1, size=(B, 1)).astype(np.int32)
    strict = (rng.random((B, 1, k)) < 0.3).astype(np.uint8)
    tree = oracle.build_tree(drafts, dl, strict, None, root_tok=np.zeros(B, np.int32), max_nodes=1 + k)
    zd = _tree_logits(rng, tree, V, "bf16", poison=False, p_lead=0.8)
    a = bk.to_np(aasd.verify(zd, _t(drafts, torch.int32), _t(dl, torch.int32), _t(strict, torch.uint8)))
    t = bk.to_np(aasd.verify_tree(zd, _t(tree["node_token"], torch.int32), _t(tree["node_parent"], torch.int32),
                                  _t(tree["n_nodes"], torch.int32), _t(tree["node_strict"], torch.uint8)))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a["accept_len"], t["accept_len"])
    np.testing.assert_array_equal(a["next_token"], t["next_token"])
    assert a["accept_len"].max() >= 2
    for b in range(B):
        n = int(tree["n_nodes"][b])
        assert a["row_entropy"][b, :n].tobytes() == t["row_entropy"][b, :n].tobytes()
        assert a["tok_p"][b, 0, :n - 1].tobytes() == t["node_p"][b, 1:n].tobytes()
        assert a["tok_delta"][b, 0, :n - 1].tobytes() == t["node_delta"][b, 1:n].tobytes()


def test_verify_tree_hand_made_trees_and_bad_parents():
    """Trees not made by the builder: deep chains, stars, parents that do not precede their children,
    node counts outside [1, N]."""
    rng = np.random.default_rng(8)
    B, N, V = 6, 48, 3000
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    par = np.full((B, N), -1, np.int32)
    par[0, 1:] = np.arange(N - 1)                    # one chain of depth 47 (longer than the 16 path slots)
    par[1, 1:] = 0                                   # a star
    par[2, 1:] = (np.arange(1, N) - 1) // 2          # a binary heap
    par[3, 1:] = rng.integers(0, np.arange(1, N))    # random recursive tree
    par[4, 1:] = par[3, 1:]
    par[4, 5] = 5; par[4, 9] = 20; par[4, 12] = -3   # self, forward and negative parents: rejected
    par[5, 1:] = par[3, 1:]
    n_nodes = np.array([N, N, N, N, N, N], np.int32)
    tree = dict(node_token=tok, node_parent=par, n_nodes=n_nodes)
    zd = _tree_logits(rng, tree, V, "bf16", poison=False, p_lead=0.5)
    zd[0, torch.arange(0, 40, device=DEV), torch.as_tensor(tok[0, 1:41].astype(np.int64), device=DEV)] = 30.0
    tally = bk.Tally()
    ref, _ = _verify_tree_both(zd, tree, None, 0.1, 0.1, 0, tally)
    assert ref["accept_len"][0] >= 40 and (ref["accept_path"][0] == np.arange(1, 17)).all()
    for nn in ([0, 1, 7, N + 5, -4, 2],):
        tree2 = dict(node_token=tok, node_parent=par, n_nodes=np.array(nn, np.int32))
        _verify_tree_both(zd, tree2, None, 0.3, 0.05, 0, tally)
    print(tally)


def test_verify_tree_strided_rows_and_determinism():
    rng = np.random.default_rng(13)
    B, C, k, N, V = 3, 4, 6, 40, 2000
    drafts, dl, strict, dx = _random_candidates(rng, B, C, k, 2, alphabet=30)
    tree = oracle.build_tree(drafts, dl, strict, dx, root_tok=np.zeros(B, np.int32), max_nodes=N)
    zd = _tree_logits(rng, tree, V, "bf16", poison=False)
    big = torch.zeros((B, N + 3, V + 24), dtype=torch.bfloat16, device=DEV)
    big[:, :N, :V] = zd
    args = (_t(tree["node_token"], torch.int32), _t(tree["node_parent"], torch.int32), _t(tree["n_nodes"], torch.int32),
            _t(tree["node_strict"], torch.uint8))
    a = bk.to_np(aasd.verify_tree(zd, *args))
    b = bk.to_np(aasd.verify_tree(big[:, :N, :V], *args))
    c = bk.to_np(aasd.verify_tree(zd, *args))
    torch.cuda.synchronize()
    for name in a:
        if a[name] is not None:
            assert a[name].tobytes() == b[name].tobytes() == c[name].tobytes(), name


@pytest.mark.parametrize("N", [129, 256])
def test_verify_tree_full_size_stress_shape_sampled(N):
    """The batch shapes as benched: B = 64 sequences, V = 152064 bf16, trees of up to 129 nodes (1 + C*k) or with
    the node budget of 256 that the tree workloads use.  Decisions and statistics are checked on sampled
    sequences whose rows the oracle recomputes, structural properties on all."""
    w = synth.WORKLOADS["stress_tree"]
    rng = np.random.default_rng(21 + N)
    B, V = w.B, w.V
    drafts, dl, strict, dx = _random_candidates(rng, B, w.C, w.k, 2, alphabet=6 if N == 129 else 12)
    tree = oracle.build_tree(drafts, dl, strict, dx, root_tok=np.zeros(B, np.int32), max_nodes=N)
    g = torch.Generator(device=DEV).manual_seed(4)
    zd = torch.randn((B, N, V), generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    nt, npar = tree["node_token"], tree["node_parent"]
    for b in range(B):      # the tokens of the nodes lead their parents' rows, with decreasing weight
        for i in range(1, int(tree["n_nodes"][b])):
            zd[b, npar[b, i], nt[b, i]] = 9.0 - 0.5 * (i % 4)
    out = aasd.verify_tree(zd, _t(nt, torch.int32), _t(npar, torch.int32), _t(tree["n_nodes"], torch.int32),
                           _t(tree["node_strict"], torch.uint8), alpha=w.alpha, beta=0.1)
    torch.cuda.synchronize()
    got = bk.to_np(out)
    tally = bk.Tally()
    for b in rng.choice(B, 3, replace=False):
        sub = {kk: v[b:b + 1] for kk, v in tree.items() if kk in ("node_token", "node_parent", "n_nodes", "node_strict")}
        ref = oracle.verify_tree(synth.to_host_bits(zd[b:b + 1]), sub["node_token"], sub["node_parent"], sub["node_strict"],
                                 sub["n_nodes"], alpha=bk.f32(w.alpha), beta=bk.f32(0.1))
        compare_verify_tree({kk: (v[b:b + 1] if v is not None else None) for kk, v in got.items()}, ref, tally)
    # properties that hold for every sequence
    for b in range(B):
        a, best = int(got["accept_len"][b]), int(got["best_node"][b])
        assert 0 <= a <= w.k and tree["node_depth"][b, best] == a
        path = got["accept_path"][b]
        assert (path[a:] == -1).all() and (a == 0 or path[a - 1] == best)
        for d in range(a - 1, 0, -1):
            assert npar[b, path[d]] == path[d - 1]
        assert got["next_token"][b] == got["row_argmax"][b, best]
    assert got["accept_len"].max() >= 2
    print("stress tree", tally, "mean accept", float(got["accept_len"].mean()))


def test_tree_decode_parity_and_gain_over_chain():
    """Alignment sampling -> retrieval with extras -> tree -> tree verification, step by step in parity
    with the oracle, on a stream whose continuation follows the model's wording of the prompt: the tree
    with the extras commits more tokens per step than the same tree without them."""
    w = synth.scaled(synth.WORKLOADS["llama3_single"], B=3, L=640, V=6000, steps=40, n_min=1, n_max=3, C=4, k=6,
                     coverage=0.9)
    streams = [synth.tree_stream(w, b) for b in range(w.B)]
    tally = bk.Tally()
    ex, nx = [], []
    for b in range(w.B):
        g, alt, slot = streams[b]
        zd = synth.tree_prefill_logits(w, b, g, alt, slot, DEV)
        nt = synth.next_tokens(w, g)
        ref = bk.oracle_align(zd, nt, w.m, w.c, oracle.EXTRAS_TOP)
        bk.compare_align(bk.hip_align(zd, nt, w.m, w.c, oracle.EXTRAS_TOP), ref, tally, oracle.EXTRAS_TOP)
        mis = slot[1:w.L] > 0
        assert (ref["misaligned"][:w.L - 1] == mis).all()
        assert (ref["extras"][:w.L - 1, 0][mis] == alt[1:w.L][mis]).all()   # the model's own pick is the first extra
        ex.append(ref["extras"]); nx.append(ref["n_extras"])
    extras, n_extras = np.concatenate(ex), np.concatenate(nx)
    pb = bk.ParityBackend(DEV)
    with_x = harness.decode_tree(w, pb, streams, extras, n_extras, max_nodes=1 + w.C * w.k * (1 + w.m))
    without = harness.decode_tree(w, pb, streams, None, None, max_nodes=1 + w.C * w.k)
    print("tree decode", pb.tally, "tokens/step with extras", with_x.mean_accept_len, "without", without.mean_accept_len)
    assert pb.tally.tokens > 100
    assert with_x.mean_accept_len > without.mean_accept_len + 0.1
    assert with_x.mean_accept_len > 1.5


@pytest.mark.parametrize("B,N,V", [(1100, 4, 300), (300, 8, 700), (2100, 2, 64)])
def test_verify_tree_more_sequences_than_one_launch_covers(B, N, V):
    """The used-rows sweep numbers the rows of at most one workgroup-size of sequences per launch."""
    rng = np.random.default_rng(B)
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    par = np.full((B, N), -1, np.int32)
    for i in range(1, N):
        par[:, i] = rng.integers(0, i, size=B)
    tree = dict(node_token=tok, node_parent=par, n_nodes=rng.integers(1, N + 1, size=B).astype(np.int32))
    zd = _tree_logits(rng, tree, V, "bf16", p_lead=0.6)
    tally = bk.Tally()
    ref, _ = _verify_tree_both(zd, tree, None, 0.1, 0.1, 0, tally)
    assert ref["accept_len"].max() >= 1


@pytest.mark.parametrize("shape", ["256,1", "256,2", "256,4", "512,2", "512,4", "1024,1", "1024,2", "256,2,5", "512,2,8", "1024,1,4"])
def test_verify_tree_under_every_compiled_launch_shape(shape, forced_plan):
    """The used-rows sweep is compiled for the same (threads, loads in flight[, segments]) shapes as the plain
    sweep; every one of them must give the oracle's answers, for both element types."""
    forced_plan(shape)
    rng = np.random.default_rng(19)
    B, C, k, N, V = 7, 4, 5, 24, 128256 // 4 + 5
    drafts, dl, strict, dx = _random_candidates(rng, B, C, k, 2, alphabet=30)
    tree = oracle.build_tree(drafts, dl, strict, dx, root_tok=np.zeros(B, np.int32), max_nodes=N)
    tally = bk.Tally()
    for dtype in ("bf16", "f32"):
        zd = _tree_logits(rng, tree, V, dtype, p_lead=0.5)
        _verify_tree_both(zd, tree, tree["node_strict"], 0.1, 0.1, 0, tally)
    assert tally.tokens > 20


@pytest.mark.parametrize("V", [1, 3, 9, 70])
def test_verify_tree_tiny_vocabularies_and_zero_probability_tokens(V):
    rng = np.random.default_rng(60 + V)
    B, N = 8, 12
    tok = rng.integers(-1, V + 2, size=(B, N)).astype(np.int32)      # some ids outside the vocabulary: they fail
    par = np.full((B, N), -1, np.int32)
    for i in range(1, N):
        par[:, i] = rng.integers(0, i, size=B)
    tree = dict(node_token=tok, node_parent=par, n_nodes=rng.integers(1, N + 1, size=B).astype(np.int32))
    z = rng.standard_normal((B, N, V)).astype(np.float32) * 2
    z[rng.random((B, N, V)) < 0.35] = -np.inf
    z[:, :, 0] = np.where(np.isinf(z).all(axis=2), 0.5, z[:, :, 0])   # at least one finite logit per row
    tally = bk.Tally()
    for dtype in ("f32", "bf16"):
        zd = torch.from_numpy(z).to(DEV)
        zd = zd.to(torch.bfloat16) if dtype == "bf16" else zd
        for alpha, beta, flags in [(0.1, 0.1, 0), (0.0, 0.0, 0), (0.0, 0.3, aasd.VERIFY_NO_CLAMP)]:
            _verify_tree_both(zd, tree, None, alpha, beta, flags, tally)
