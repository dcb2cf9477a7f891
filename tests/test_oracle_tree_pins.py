"""Pins of the oracle's draft-tree functions (Sec. 3.2, Eq. 2; verification as in Sec. 3.3) against
the paper's worked example, an independent dictionary trie, the already pinned chain verifier and
brute force on small trees.  No GPU."""
import itertools
import os

import numpy as np
import pytest

import oracle
from tests.util import read_golden

F32A = float(np.float32(0.1))


def test_tree_of_fig2(golden_dir):
    row = [r for r in read_golden(os.path.join(golden_dir, "alignment_examples.txt")) if r[0] == "fig2.tree"][0]
    root, draft = int(row[1]), [int(x) for x in row[2].split()]
    extras = [[] if e == "-" else [int(x) for x in e.split(",")] for e in row[3].split()]
    expect = [tuple(int(x) for x in e.split(":")) for e in row[4].split()]
    k, m = len(draft), 2
    dx = -np.ones((1, 1, k, m), np.int32)
    for j, e in enumerate(extras):
        dx[0, 0, j, :len(e)] = e
    t = oracle.build_tree(np.array([[draft]], np.int32), [[k]], None, dx, root_tok=[root], max_nodes=16)
    n = int(t["n_nodes"][0])
    assert n == len(expect) == 6
    assert list(zip(t["node_token"][0, :n].tolist(), t["node_parent"][0, :n].tolist())) == expect
    assert t["node_depth"][0, :n].tolist() == [0, 1, 1, 1, 2, 3]
    # tree attention mask: "great" sees Jackson, is, a, great; the extras see only the root and themselves
    assert t["mask"][0, 5, 0] == 0b110011 and t["mask"][0, 2, 0] == 0b000101 and t["mask"][0, 3, 0] == 0b001001
    assert t["cand_node"][0, 0].tolist() == [1, 4, 5]


def _trie_reference(drafts, draft_len, strict, dx, max_nodes):
    """Independent construction: a dictionary keyed by (parent, token), filled layer by layer."""
    C, k = drafts.shape
    m = 0 if dx is None else dx.shape[2]
    nodes = [(-1, -1, 0)]  # (token, parent, depth); root token filled by the caller
    is_strict = [0]
    index = {}
    cur = [0] * C
    cand_node = -np.ones((C, k), np.int64)
    for j in range(1, k + 1):
        nxt = [-1] * C
        for c in range(C):
            if cur[c] < 0 or j > draft_len[c]:
                continue
            toks = [(int(drafts[c, j - 1]), int(strict[c, j - 1]) if strict is not None else 0, True)]
            if toks[0][0] < 0:
                continue
            toks += [(int(x), 0, False) for x in (dx[c, j - 1] if dx is not None else []) if x >= 0]
            for tok, st, main in toks:
                key = (cur[c], tok)
                if key not in index and len(nodes) < max_nodes:
                    index[key] = len(nodes)
                    nodes.append((tok, cur[c], j))
                    is_strict.append(st)
                elif key in index and not st:
                    is_strict[index[key]] = 0
                if main:
                    nxt[c] = index.get(key, -1)
                    cand_node[c, j - 1] = nxt[c]
        cur = nxt
    return nodes, is_strict, cand_node


@pytest.mark.parametrize("C,k,m,N,alphabet", [(1, 4, 0, 8, 3), (3, 4, 2, 64, 3), (8, 8, 2, 40, 3), (16, 8, 2, 256, 3),
                                              (32, 16, 4, 256, 3), (4, 6, 3, 5, 3),
                                              # the paper's parameters (Sec. 4.1: up to two extras per position) need up to
                                              # 1 + 16*8*3 = 385 nodes; a wider alphabet shares fewer prefixes and fills them
                                              (16, 8, 2, 385, 12), (16, 8, 2, 512, 40), (32, 16, 4, 512, 6), (16, 8, 2, 300, 40)])
def test_tree_build_against_dictionary_trie(C, k, m, N, alphabet):
    rng = np.random.default_rng(C * 100 + k + alphabet)
    B = 12
    drafts = rng.integers(0, alphabet, size=(B, C, k)).astype(np.int32)   # small alphabet: shared prefixes
    drafts[rng.random((B, C, k)) < 0.05] = -1                      # a missing token ends the candidate's path
    dl = rng.integers(0, k + 1, size=(B, C)).astype(np.int32)
    strict = (rng.random((B, C, k)) < 0.4).astype(np.uint8)
    dx = None
    if m:
        dx = rng.integers(0, alphabet + 1, size=(B, C, k, m)).astype(np.int32)
        dx[rng.random((B, C, k, m)) < (0.5 if alphabet == 3 else 0.1)] = -1
    if alphabet > 3:
        dl[:] = np.maximum(dl, k - 1)                                     # long candidates: large trees
    t = oracle.build_tree(drafts, dl, strict, dx, root_tok=np.arange(B), max_nodes=N)
    if N >= 385:
        assert t["n_nodes"].max() > 256                                   # the case needs the larger budget
    W = (N + 31) // 32
    for b in range(B):
        nodes, st, cand_node = _trie_reference(drafts[b], dl[b], strict[b], None if dx is None else dx[b], N)
        n = len(nodes)
        assert t["n_nodes"][b] == n <= N
        assert t["node_token"][b, 0] == b and t["node_parent"][b, 0] == -1
        assert t["node_token"][b, 1:n].tolist() == [x[0] for x in nodes[1:]]
        assert t["node_parent"][b, 1:n].tolist() == [x[1] for x in nodes[1:]]
        assert t["node_depth"][b, :n].tolist() == [x[2] for x in nodes]
        assert t["node_strict"][b, :n].tolist() == st
        assert (t["node_token"][b, n:] == -1).all() and (t["node_parent"][b, n:] == -1).all()
        np.testing.assert_array_equal(t["cand_node"][b], cand_node)
        for i in range(N):
            want = np.zeros(W, np.uint32)
            a = i if i < n else -1
            while a >= 0:
                want[a // 32] |= np.uint32(1 << (a % 32))
                a = nodes[a][1]
            np.testing.assert_array_equal(t["mask"][b, i], want)
        # parents precede children; depth = parent's depth + 1; a candidate's nodes chain up to the root
        for i in range(1, n):
            p = nodes[i][1]
            assert 0 <= p < i and nodes[i][2] == nodes[p][2] + 1


def test_tree_at_the_papers_largest_parameters_has_385_nodes():
    """16 candidates of 8 tokens, every position misaligned with two extras (the shape of Fig. 2's caption at every
    position; Sec. 4.1 allows at most two), all tokens distinct: nothing merges, so the tree is known in closed form.
    Layer j holds 48 nodes in (candidate, slot) order; the retrieved token of (j, c) is the parent of layer j+1's
    three nodes of candidate c; every extra is a leaf."""
    C, k, m = 16, 8, 2
    per = 1 + m
    drafts = (1000 + np.arange(C * k)).reshape(1, C, k).astype(np.int32)
    dx = (5000 + np.arange(C * k * m)).reshape(1, C, k, m).astype(np.int32)
    dl = np.full((1, C), k, np.int32)
    strict = np.zeros((1, C, k), np.uint8)
    strict[0, :, 4:] = 1
    node = lambda j, c, s: 1 + (j - 1) * C * per + c * per + s      # j = 1..k
    t = oracle.build_tree(drafts, dl, strict, dx, root_tok=[7], max_nodes=512)
    assert t["n_nodes"][0] == 1 + C * k * per == 385
    for j in range(1, k + 1):
        for c in range(C):
            for s in range(per):
                i = node(j, c, s)
                want_tok = drafts[0, c, j - 1] if s == 0 else dx[0, c, j - 1, s - 1]
                want_par = 0 if j == 1 else node(j - 1, c, 0)
                assert (t["node_token"][0, i], t["node_parent"][0, i], t["node_depth"][0, i]) == (want_tok, want_par, j)
                assert t["node_strict"][0, i] == (1 if s == 0 and j > 4 else 0)
                row = t["mask"][0, i]
                bits = {a for a in range(512) if (row[a // 32] >> (a % 32)) & 1}
                assert bits == {0, i} | {node(jj, c, 0) for jj in range(1, j)}
            assert t["cand_node"][0, c, j - 1] == node(j, c, 0)
    assert (t["node_token"][0, 385:] == -1).all() and (t["mask"][0, 385:] == 0).all()
    # the same input under a budget of 256: creation order is kept, the rest is dropped with what hangs below it
    t2 = oracle.build_tree(drafts, dl, strict, dx, root_tok=[7], max_nodes=256)
    assert t2["n_nodes"][0] == 256
    np.testing.assert_array_equal(t2["node_token"][0], t["node_token"][0, :256])
    np.testing.assert_array_equal(t2["node_parent"][0], t["node_parent"][0, :256])
    dropped = t["cand_node"][0] >= 256
    assert (t2["cand_node"][0][dropped] == -1).all() and (t2["cand_node"][0][~dropped] == t["cand_node"][0][~dropped]).all()
    # verification over all 385 rows: the stream follows candidate 9 to its end
    V = 7000
    z = np.full((1, 512, V), -20.0, np.float32)
    for i in range(385):
        z[0, i, 3] = 0.0                                             # a token no node carries wins every row ...
    path = [0] + [node(j, 9, 0) for j in range(1, k + 1)]
    for a, nxt in zip(path[:-1], path[1:]):
        z[0, a, t["node_token"][0, nxt]] = 5.0                       # ... except along the path of candidate 9
    out = oracle.verify_tree(z, t["node_token"], t["node_parent"], t["node_strict"], t["n_nodes"], alpha=F32A, beta=F32A)
    assert out["accept_len"][0] == k and out["best_node"][0] == node(k, 9, 0) and out["next_token"][0] == 3
    assert out["accept_path"][0, :k].tolist() == path[1:]


def _random_rows(rng, B, R, V):
    z = rng.standard_normal((B, R, V)).astype(np.float32)
    for b in range(B):
        for r in range(R):
            top = rng.choice(V, 4, replace=False)
            z[b, r, top] = [9.0, 8.0, 7.0, 6.0]
    return z


def test_tree_of_disjoint_chains_equals_chain_verification():
    """A tree whose candidates share no prefix is the chain layout re-indexed: both verifiers must agree."""
    rng = np.random.default_rng(2)
    B, C, k, V = 6, 3, 4, 120
    R = 1 + C * k
    for trial in range(10):
        z = _random_rows(rng, B, R, V)
        order = np.argsort(-z, axis=2)
        drafts = np.empty((B, C, k), np.int32)
        for b in range(B):
            for c in range(C):
                for j in range(k):
                    rho = 0 if j == 0 else 1 + c * k + (j - 1)
                    drafts[b, c, j] = order[b, rho, rng.choice(4, p=[0.6, 0.25, 0.1, 0.05])]
                drafts[b, c, 0] = order[b, 0, c]      # distinct first tokens: no shared prefixes
        dl = rng.integers(1, k + 1, size=(B, C)).astype(np.int32)
        strict = (rng.random((B, C, k)) < 0.3).astype(np.uint8)
        chain = oracle.verify(z, drafts, dl, strict, alpha=F32A, beta=F32A)
        t = oracle.build_tree(drafts, dl, strict, None, max_nodes=R)
        # tree logits: the row of node (c, j) is the chain row after candidate c's j-th token
        zt = np.zeros((B, R, V), np.float32)
        zt[:, 0] = z[:, 0]
        for b in range(B):
            for c in range(C):
                for j in range(dl[b, c]):
                    zt[b, t["cand_node"][b, c, j]] = z[b, 1 + c * k + j]
        tree = oracle.verify_tree(zt, t["node_token"], t["node_parent"], t["node_strict"], t["n_nodes"],
                                  alpha=F32A, beta=F32A)
        np.testing.assert_array_equal(tree["accept_len"], chain["accept_len"])
        np.testing.assert_array_equal(tree["next_token"], chain["next_token"])
        for b in range(B):
            a, c = chain["accept_len"][b], chain["best_cand"][b]
            assert tree["accept_path"][b, :a].tolist() == t["cand_node"][b, c, :a].tolist()
            assert (tree["accept_path"][b, a:] == -1).all()
            assert tree["near_count"][b] == chain["near_count"][b]


def test_tree_verify_brute_force_over_pass_patterns():
    """Every pass/fail assignment on a fixed 7-node tree: the deepest all-pass path wins, lowest index on ties."""
    V, GOOD, BAD = 12, 3, 9
    parent = [-1, 0, 0, 1, 1, 2, 5]
    depth = [0, 1, 1, 2, 2, 2, 3]
    N = len(parent)
    z = np.full((1, N, V), -16.0, np.float32)
    z[0, :, GOOD] = 0.0
    for r in range(N):
        z[0, r, (r + 4) % V if (r + 4) % V not in (GOOD, BAD) else 0] = -2.0
    for pattern in itertools.product([0, 1], repeat=N - 1):
        ok = [1] + list(pattern)
        tok = np.array([[-1] + [GOOD if p else BAD for p in pattern]], np.int32)
        out = oracle.verify_tree(z, tok, np.array([parent], np.int32), None, [N], alpha=F32A, beta=F32A)
        acc = [1] * N
        for i in range(1, N):
            acc[i] = ok[i] and acc[parent[i]]
        best = max(range(N), key=lambda i: (depth[i] if acc[i] else -1, -i))
        assert out["best_node"][0] == best and out["accept_len"][0] == depth[best]
        path = []
        a = best
        while a > 0:
            path.append(a); a = parent[a]
        assert out["accept_path"][0, :len(path)].tolist() == path[::-1]
        assert out["next_token"][0] == GOOD
        evaluated = [int(acc[parent[i]]) for i in range(1, N)]
        assert (out["node_margin"][0, 1:] >= 0).astype(int).tolist() == evaluated


def test_tree_verify_uses_the_parent_row_and_per_node_strictness():
    V = 10
    z = np.full((1, 4, V), -30.0, np.float32)
    z[0, 0, [1, 2]] = [3.0, 2.0]     # root row: p ~ 0.73, 0.27
    z[0, 1, [4, 5]] = [1.0, 1.0]     # row of node 1: a tie at the maximum
    z[0, 2, 7] = 0.0
    tok = np.array([[-1, 2, 5, 7]], np.int32)           # node 1 = runner-up, node 2 child of 1, node 3 child of 0
    par = np.array([[-1, 0, 1, 0]], np.int32)
    out = oracle.verify_tree(z, tok, par, None, [4], alpha=F32A, beta=F32A)
    assert out["accept_len"][0] == 2 and out["best_node"][0] == 2          # 0.27 passes, the tied token passes
    assert out["next_token"][0] == 7                                        # greedy pick of node 2's row
    out = oracle.verify_tree(z, tok, par, np.array([[0, 1, 0, 0]], np.uint8), [4], alpha=F32A, beta=F32A)
    assert out["accept_len"][0] == 0 and out["next_token"][0] == 1          # strict node 1 fails; node 3 (p=0) fails
    out = oracle.verify_tree(z, tok, par, None, [2], alpha=F32A, beta=F32A)  # only two nodes in the tree
    assert out["accept_len"][0] == 1 and out["best_node"][0] == 1 and out["row_argmax"][0, 2] == -1
