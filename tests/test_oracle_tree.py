"""Pins of the oracle's prefix-tree verification (paper Section 3.2: prefix-tree batching, tree-ancestry attention
mask, greedy traversal Eq. 9-12): structure of the worked example, node logits against independent chain
evaluations, reduction to the chain case, and the lossless property with KV compaction."""
import math

import numpy as np
import pytest

import oracle as O
import workloads as W


def test_tree_of_the_worked_example():
    """The worked example of the method's figure: three candidates that share the first word and then continue
    with `in parallel`, `simultaneously`, `together`.  Next(`tokens`) has three members; `parallel` sits under
    `in`.  (Words are mapped to arbitrary ids.)"""
    TOK, IN, PAR, SIM, TOG, PEND = 11, 12, 13, 14, 15, 99
    tokens, parent, depth, end = O.build_prefix_tree(PEND, [[TOK, IN, PAR], [TOK, SIM], [TOK, TOG]])
    assert tokens.tolist() == [PEND, TOK, IN, PAR, SIM, TOG]          # pre-order, children in order of appearance
    assert parent.tolist() == [-1, 0, 1, 2, 1, 1]
    assert depth.tolist() == [0, 1, 2, 3, 2, 2]
    assert end.tolist() == [6, 6, 4, 4, 5, 6]
    next_of_tokens = {int(tokens[i]) for i in range(len(tokens)) if parent[i] == 1}
    assert next_of_tokens == {IN, SIM, TOG}
    m = O.ancestry_mask(parent)
    assert m[3].tolist() == [True, True, True, True, False, False]   # `parallel` sees root, tokens, in, itself
    assert m[4].tolist() == [True, True, False, False, True, False]  # `simultaneously` does not see `in parallel`


def test_subtree_intervals_are_the_ancestry_relation():
    rng = np.random.default_rng(3)
    for _ in range(50):
        cands = [rng.integers(0, 4, size=int(rng.integers(1, 7))).tolist() for _ in range(int(rng.integers(1, 8)))]
        tokens, parent, depth, end = O.build_prefix_tree(0, cands)
        n = len(tokens)
        m = O.ancestry_mask(parent)
        for i in range(n):
            for j in range(n):
                assert m[i, j] == (j <= i < end[j])
            assert depth[i] == m[i].sum() - 1
        # every candidate is a root-to-node path, and the tree has no other leaves than candidate ends
        paths = set()
        for i in range(n):
            p, v = [], i
            while v > 0:
                p.append(int(tokens[v]))
                v = int(parent[v])
            paths.add(tuple(reversed(p)))
        for c in cands:
            assert tuple(c) in paths
        assert n - 1 == len({tuple(c[:k]) for c in cands for k in range(1, len(c) + 1)})


def _setup(seed=41, dtype="fp32"):
    desc = W.tiny_model(2, 64, 2, 1, 32, 128, 60, dtype)
    weights = W.make_weights(desc, seed)
    vis, prompt = W.make_prefix(desc, seed, 0, 10, 3)
    cache, pending = O.prefill(desc, weights, vis, prompt)
    return desc, weights, cache, pending


def test_node_logits_equal_independent_chain_evaluations():
    """Each node's row must be what a plain causal pass over context + pending + path(node) gives at its last row:
    pins the mask, the per-node positions and the slot/position split in one go."""
    desc, weights, cache, pending = _setup()
    base = len(cache)
    rng = np.random.default_rng(8)
    cands = [rng.integers(0, desc.vocab, size=5).tolist(), rng.integers(0, desc.vocab, size=3).tolist()]
    cands.append(cands[0][:2] + [7, 8, 9])
    cands.append(cands[0][:4] + [5])
    tokens, parent, depth, end = O.build_prefix_tree(pending, cands)
    logits = O.decoder_forward(desc, weights, O.embed_tokens(weights, tokens), cache, depth=depth,
                               block_mask=O.ancestry_mask(parent))
    cache.truncate(base)
    for i in range(len(tokens)):
        path, v = [], i
        while v >= 0:
            path.append(int(tokens[v]))
            v = int(parent[v])
        chain = O.decoder_forward(desc, weights, O.embed_tokens(weights, list(reversed(path))), cache)
        cache.truncate(base)
        np.testing.assert_allclose(logits[i], chain[-1], rtol=0, atol=1e-9)


@pytest.mark.parametrize("log_tau", [0.0, math.log(0.75)])
def test_single_candidate_tree_is_the_chain(log_tau):
    desc, weights, cache, pending = _setup(seed=42)
    base = len(cache)
    target = O.greedy_decode(desc, weights, cache, pending, 12)
    cache.truncate(base)
    draft, _ = W.corrupt_draft_forced(target, 0.2, desc.vocab, 42, "tree1")
    alpha, bonus, _, logits = O.verify_block(desc, weights, cache, pending, draft, log_tau=log_tau)
    cache.truncate(base)
    acc, bonus_t, logits_t, _ = O.verify_tree(desc, weights, cache, pending, [draft], log_tau=log_tau)
    assert (len(acc), bonus_t) == (alpha, bonus) and acc == draft[:alpha].tolist()
    np.testing.assert_allclose(logits_t, logits, rtol=0, atol=1e-9)
    assert len(cache) == base + 1 + alpha


def test_tree_rounds_are_lossless_and_leave_an_ordinary_cache():
    """Rounds of tree verification over several imperfect candidates reproduce token-by-token greedy decoding;
    each round accepts the longest prefix of the greedy continuation present in the tree, and the compacted
    cache continues exactly like one built token by token."""
    desc, weights, cache, pending = _setup(seed=43)
    base = len(cache)
    n = 40
    target = O.greedy_decode(desc, weights, cache, pending, n)
    cache.truncate(base)
    rng = np.random.default_rng(17)
    committed, pend, rounds = [], pending, 0
    while len(committed) < n:
        o = len(committed)
        rest = target[o:o + 10]
        cands = []
        for c in range(3):                      # three drafts, each wrong from a different point on
            d = rest.copy()
            cut = int(rng.integers(0, len(d) + 1))
            d[cut:] = rng.integers(0, desc.vocab, size=len(d) - cut)
            cands.append(d.tolist())
        acc, bonus, _, (tokens, parent, depth, end) = O.verify_tree(desc, weights, cache, pend, cands)
        in_tree = {tuple(c[:k]) for c in cands for k in range(len(c) + 1)}
        expect = max(k for k in range(len(rest) + 1) if tuple(rest[:k].tolist()) in in_tree)
        assert len(acc) == expect and acc == rest[:expect].tolist()
        committed.extend(acc)
        committed.append(bonus)
        pend = bonus
        rounds += 1
        assert len(cache) == base + len(committed)
    np.testing.assert_array_equal(np.asarray(committed[:n]), target)
    assert rounds >= 3
    # the cache after compaction equals the cache of plain decoding over the same tokens
    ref = O.KVCache(desc.n_layers, desc.n_kv_heads, desc.head_dim)
    vis, prompt = W.make_prefix(desc, 43, 0, 10, 3)
    ref, p0 = O.prefill(desc, weights, vis, prompt)
    O.decoder_forward(desc, weights, O.embed_tokens(weights, [p0] + committed[:-1]), ref)
    for l in range(desc.n_layers):
        np.testing.assert_allclose(cache.keys(l, len(cache)), ref.keys(l, len(cache)), rtol=0, atol=1e-9)
        np.testing.assert_allclose(cache.values(l, len(cache)), ref.values(l, len(cache)), rtol=0, atol=1e-9)


def test_relaxed_walk_equals_probability_form():
    rng = np.random.default_rng(23)
    for _ in range(100):
        cands = [rng.integers(0, 6, size=int(rng.integers(1, 6))).tolist() for _ in range(int(rng.integers(1, 6)))]
        tokens, parent, depth, end = O.build_prefix_tree(0, cands)
        V = 8
        logits = rng.normal(0, 1.2, size=(len(tokens), V))
        tau = float(rng.choice([0.9, 0.6, 0.2]))
        path, bonus = O.walk_prefix_tree(logits, tokens, parent, math.log(tau))
        # brute force with probabilities (Eq. 9-11)
        e = np.exp(logits - logits.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        s, ref = 0, []
        while True:
            kids = [i for i in range(len(tokens)) if parent[i] == s]
            if not kids:
                break
            best = max(kids, key=lambda c: p[s, tokens[c]])
            if p[s, tokens[best]] / p[s].max() >= tau:
                ref.append(best)
                s = best
            else:
                break
        assert path == ref and bonus == int(np.argmax(p[s]))
