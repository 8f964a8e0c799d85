"""Invariants the verification operator must satisfy, checked on the oracle.

The central one is the lossless property the method rests on (Section 3.2: verification preserves
autoregressive conditioning; related work: the verifier accepts the longest matching prefix): running
verification rounds over ANY draft yields exactly the tokens plain token-by-token greedy decoding yields.
"""
import itertools

import numpy as np
import pytest

import oracle as O
import workloads as W

SHAPES = list(itertools.product([1, 2], [32, 64], [(1, 1), (2, 1), (4, 1), (4, 2), (4, 4)], [64, 257]))


def _setup(desc, seed, n_vis=5, n_prompt=3):
    w = W.make_weights(desc, seed)
    vis, prompt = W.make_prefix(desc, seed, 0, n_vis, n_prompt)
    return w, vis, prompt


@pytest.mark.parametrize("L,d,heads,V", SHAPES)
def test_lossless_invariant_random_models(L, d, heads, V):
    Hq, Hkv = heads
    desc = W.tiny_model(n_layers=L, d_model=d, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d // Hq, d_ffn=2 * d, vocab=V)
    n = 14
    for trial, p in enumerate([0.0, 0.1, 0.5, 1.0]):
        seed = 1000 * L + d + 7 * Hq + Hkv + V + trial
        w, vis, prompt = _setup(desc, seed)
        cache, pending = O.prefill(desc, w, vis, prompt)
        g = O.greedy_decode(desc, w, cache, pending, n)
        draft, mask = W.corrupt_draft(g, p, V, seed, "d")
        cache, pending = O.prefill(desc, w, vis, prompt)
        out, rounds = O.spec_decode(desc, w, cache, pending, draft, n)
        np.testing.assert_array_equal(out, g)
        assert len(cache) == len(vis) + len(prompt) - 1 + sum(r.alpha + 1 for r in rounds)
        # a completely random draft (not derived from the target) changes nothing either
        rnd = np.random.default_rng(seed).integers(0, V, size=n)
        cache, pending = O.prefill(desc, w, vis, prompt)
        out2, _ = O.spec_decode(desc, w, cache, pending, rnd, n)
        np.testing.assert_array_equal(out2, g)


def test_alpha_closed_form_from_corruption_positions():
    """With draft = greedy output corrupted at positions B by different tokens, a round starting at
    draft offset o accepts alpha = (first b in B with b >= o) - o tokens (all remaining if none), and
    the number of rounds is |B| + 1, minus one if the last draft token is corrupted... computed by replay."""
    desc = W.tiny_model(n_layers=1, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ffn=64, vocab=97)
    w, vis, prompt = _setup(desc, 77)
    n = 40
    cache, pending = O.prefill(desc, w, vis, prompt)
    g = O.greedy_decode(desc, w, cache, pending, n)
    for p in (0.05, 0.2, 0.6):
        draft, mask = W.corrupt_draft_forced(g, p, desc.vocab, 77, f"p{p}")
        B = np.nonzero(mask)[0]
        cache, pending = O.prefill(desc, w, vis, prompt)
        out, rounds = O.spec_decode(desc, w, cache, pending, draft, n)
        np.testing.assert_array_equal(out, g)
        o = 0
        for r in rounds:
            assert r.offset == o and r.k == n - o
            later = B[B >= o]
            expect = int(later[0] - o) if len(later) else n - o
            assert r.alpha == expect
            assert r.bonus == (g[o + r.alpha] if o + r.alpha < n else r.bonus)
            o += r.alpha + 1
        assert o >= n


def test_verify_rollback_reverify_is_idempotent():
    desc = W.tiny_model(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=64, vocab=50)
    w, vis, prompt = _setup(desc, 5)
    cache, pending = O.prefill(desc, w, vis, prompt)
    draft = np.random.default_rng(0).integers(0, 50, size=10)
    base = len(cache)
    a1 = O.verify_block(desc, w, cache, pending, draft)
    cache.truncate(base)
    a2 = O.verify_block(desc, w, cache, pending, draft)
    assert a1[0] == a2[0] and a1[1] == a2[1]
    np.testing.assert_array_equal(a1[3], a2[3])


def test_block_length_one_is_a_decode_step_and_max_block_cap():
    desc = W.tiny_model(n_layers=1, d_model=32, n_q_heads=2, n_kv_heads=2, head_dim=16, d_ffn=64, vocab=60)
    w, vis, prompt = _setup(desc, 9)
    cache, pending = O.prefill(desc, w, vis, prompt)
    g = O.greedy_decode(desc, w, cache, pending, 25)
    cache, pending = O.prefill(desc, w, vis, prompt)
    alpha, bonus, u_hat, _ = O.verify_block(desc, w, cache, pending, np.array([], dtype=np.int32))
    assert (alpha, bonus) == (0, g[0])
    # capping the packed block (the paper caps it at 128 tokens, Section 4.3) changes rounds, not output
    draft, _ = W.corrupt_draft_forced(g, 0.1, desc.vocab, 9, "c")
    for cap in (1, 4, 128):
        cache, pending = O.prefill(desc, w, vis, prompt)
        out, rounds = O.spec_decode(desc, w, cache, pending, draft, 25, max_block=cap)
        np.testing.assert_array_equal(out, g)
        assert all(r.k <= cap for r in rounds)


def test_aal_expectation_iid_corruption():
    """AAL (Eq. 15) of the first round over many i.i.d.-corrupted drafts is sum_{j=1..k} (1-p)^j.
    Acceptance here is replayed from the mask alone (closed form pinned above), so this checks the
    corruption generator's statistics that the workloads rely on."""
    k, p, n = 64, 0.05, 4000
    target = np.zeros(k, dtype=np.int32)
    alphas = []
    for i in range(n):
        _, mask = W.corrupt_draft_forced(target, p, 1000, 123, f"s{i}")
        nz = np.nonzero(mask)[0]
        alphas.append(int(nz[0]) if len(nz) else k)
    expect = sum((1 - p) ** j for j in range(1, k + 1))
    assert abs(np.mean(alphas) - expect) < 4 * np.std(alphas) / np.sqrt(n)


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_lossless_invariant_with_bf16_storage(seed):
    """The invariant is a property of the operator, not of the precision: it also holds when the decoder
    stores its activations in bf16."""
    desc = W.tiny_model(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=128, vocab=257, dtype="bf16")
    w, vis, prompt = _setup(desc, seed)
    cache, pending = O.prefill(desc, w, vis, prompt, act_dtype="bf16")
    g = O.greedy_decode(desc, w, cache, pending, 16, act_dtype="bf16")
    draft, _ = W.corrupt_draft(g, 0.3, desc.vocab, seed, "b")
    cache, pending = O.prefill(desc, w, vis, prompt, act_dtype="bf16")
    out, rounds = O.spec_decode(desc, w, cache, pending, draft, 16, act_dtype="bf16")
    np.testing.assert_array_equal(out, g)
