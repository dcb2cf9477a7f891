"""Host-side checks of the synthetic workloads and of the decode driver (oracle backend, no GPU)."""
import numpy as np
import torch

import oracle

from tests import harness, synth
from tests import backends as bk


def test_token_streams_are_seeded_and_have_planted_repeats():
    for name, w in synth.WORKLOADS.items():
        g, copied = synth.token_stream(w, 0)
        g2, _ = synth.token_stream(w, 0)
        assert (g == g2).all() and len(g) == w.stream_len
        assert g.min() >= 0 and g.max() < w.V
        other, _ = synth.token_stream(w, 1)
        assert (other != g).any()
        if w.spans:
            assert copied.sum() == 2 * 8 * w.spans
        else:
            assert abs(copied.mean() - w.coverage) < 0.1, (name, copied.mean())
    nt = synth.next_tokens(synth.WORKLOADS["tiny"], synth.token_stream(synth.WORKLOADS["tiny"], 0)[0])
    assert nt[-1] == -1 and len(nt) == 256


def test_logits_recipe():
    w = synth.scaled(synth.WORKLOADS["llama3_single"], V=4000, L=512)
    g, copied = synth.token_stream(w, 0)
    z = synth.prefill_logits(w, 0, g, copied, "cpu")
    assert z.shape == (512, 4000) and z.dtype == torch.bfloat16
    zf = z.float()
    assert abs(zf.var().item() - w.sigma2) < 0.1
    top_is_next = (zf.argmax(1)[:-1].numpy() == g[1:512]).mean()
    assert 0.4 < top_is_next < 0.95  # the peak wins most, not all, rows
    z2 = synth.prefill_logits(w, 0, g, copied, "cpu")
    assert torch.equal(z.view(torch.int16), z2.view(torch.int16))
    zp = synth.prefill_logits(w, 0, g, copied, "cpu", rows=slice(0, 8), peaked=True).float()
    assert (zp.max(1).values == 24.0).all()


def test_decode_driver_with_oracle_backend():
    w = synth.scaled(synth.WORKLOADS["llama3_single"], V=3000, L=400, steps=48)
    trace = harness.decode(w, bk.OracleBackend())
    assert len(trace.steps) == 48
    assert (trace.length >= w.L + 48).all() and (trace.length <= w.tok_cap).all()
    # planted spans are found and followed: more than one token per step on average
    assert trace.mean_accept_len > 1.0
    for s in trace.steps:
        assert 0 <= s.verified["accept_len"][0] <= w.k
    again = harness.decode(w, bk.OracleBackend())
    assert (again.tokens == trace.tokens).all()
    batched = synth.scaled(synth.WORKLOADS["stress_tree"], V=2000, L=600, B=3, steps=5)
    tr = harness.decode(batched, bk.OracleBackend(), peaked=True)
    assert tr.steps[0].retrieved["drafts"].shape == (3, 16, 8)
    assert any((s.retrieved["n_cand"] > 1).any() for s in tr.steps)


def test_tree_decode_on_the_oracle_gains_from_alignment_extras():
    """The draft-tree loop end to end on the CPU oracle: prefill alignment sampling finds the model's own
    wording at the misaligned prompt positions, and the tree that carries those extras commits more tokens
    per step than the tree without them (the effect Sec. 3.2 is after)."""
    w = synth.scaled(synth.WORKLOADS["llama3_single"], B=2, L=400, V=3000, steps=30, n_min=1, n_max=3, C=4, k=6,
                     coverage=0.9)
    streams = [synth.tree_stream(w, b) for b in range(w.B)]
    ex, nx = [], []
    for b in range(w.B):
        g, alt, slot = streams[b]
        z = synth.tree_prefill_logits(w, b, g, alt, slot, "cpu")
        out = oracle.align_sample(synth.to_host_bits(z), synth.next_tokens(w, g), m_x=w.m, c=w.c, mode=oracle.EXTRAS_TOP)
        mis = slot[1:w.L] > 0
        assert 0.2 < mis.mean() < 0.4
        assert (out["misaligned"][:w.L - 1] == mis).all()
        assert (out["extras"][:w.L - 1, 0][mis] == alt[1:w.L][mis]).all()
        ex.append(out["extras"]); nx.append(out["n_extras"])
    ob = bk.OracleBackend()
    with_x = harness.decode_tree(w, ob, streams, np.concatenate(ex), np.concatenate(nx), max_nodes=1 + w.C * w.k * 3)
    without = harness.decode_tree(w, ob, streams, None, None, max_nodes=1 + w.C * w.k)
    assert with_x.mean_accept_len > without.mean_accept_len + 0.1
    # every committed token came from the accepted path of that step's tree, then the model's next token
    for s in with_x.steps:
        t, v = s.retrieved["tree"], s.verified
        for b in range(w.B):
            a = int(v["accept_len"][b])
            assert 0 <= a <= w.k and (v["accept_path"][b, a:] == -1).all()
            assert a == 0 or t["node_depth"][b, v["best_node"][b]] == a
