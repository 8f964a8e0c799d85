"""Pins of the oracle's decoupled-verification driver (paper Section 3.2: draft-target matching Eq. 5-6, the
cap on the packed sequence, rounds over a FIXED draft set): the set definitions by brute force, and the lossless
property under insert / delete / reorder corruption of the drafts."""
import numpy as np

import oracle as O
import workloads as W


def test_match_candidates_is_the_set_definition():
    rng = np.random.default_rng(2)
    for _ in range(300):
        n = int(rng.integers(1, 4))
        acc = rng.integers(0, 3, size=int(rng.integers(0, 8))).tolist()
        drafts = [rng.integers(0, 3, size=int(rng.integers(0, 10))).tolist() for _ in range(int(rng.integers(0, 4)))]
        got = O.match_candidates(acc, drafts, n)
        if len(acc) >= n:
            w = acc[-n:]
            # Eq. 5: 1-based j with draft[j..j+n-1] = w and j <= |draft|-n+1; Eq. 6: suffix from j+n, non-empty
            ref = {tuple(d[j + n:]) for d in drafts for j in range(len(d) - n + 1) if d[j:j + n] == w and j + n < len(d)}
            assert {tuple(c) for c in got} == ref
        assert len({tuple(c) for c in got}) == len(got) and all(len(c) for c in got)
    assert O.match_candidates([], [[4, 5], [6]], 3) == [[4, 5], [6]]          # nothing accepted yet
    assert O.match_candidates([9, 1, 2, 3], [[7, 1, 2, 3, 8, 1, 2, 3, 5]], 3) == [[8, 1, 2, 3, 5], [5]]


def test_cap_candidates_bounds_the_packed_tree():
    rng = np.random.default_rng(4)
    for _ in range(200):
        cands = [rng.integers(0, 3, size=int(rng.integers(1, 30))).tolist() for _ in range(int(rng.integers(1, 6)))]
        cap = int(rng.integers(8, 64))
        capped = O.cap_candidates(cands, cap)
        tokens, _, depth, _ = O.build_prefix_tree(0, capped)
        L = max(len(c) for c in capped)
        assert len(tokens) <= cap or L == 1
        assert all(tuple(c) in {tuple(x[:len(c)]) for x in cands} for c in capped)          # prefixes of the inputs
        longer = [c[:L + 1] for c in cands]
        if L < max(len(c) for c in cands):                                                  # L is maximal
            assert len(O.build_prefix_tree(0, longer)[0]) > cap
    assert O.cap_candidates([], 128) == []


def _corrupt_set(rng, target, vocab):
    """Draft set with the defects the decoupled setting has to survive: the target cut into segments that come in
    another order, with tokens deleted, inserted and substituted."""
    cuts = sorted(rng.choice(np.arange(5, len(target) - 5), size=3, replace=False).tolist())
    segs = [target[a:b].tolist() for a, b in zip([0] + cuts, cuts + [len(target)])]
    rng.shuffle(segs)
    out = []
    for sgm in segs:
        d = []
        for t in sgm:
            r = rng.random()
            if r < 0.04:
                continue                                  # deletion
            if r < 0.08:
                d.append(int(rng.integers(0, vocab)))     # insertion
            d.append(int(rng.integers(0, vocab)) if r > 0.95 else int(t))
        out.append(d)
    return out


def test_decoupled_rounds_are_lossless_under_insert_delete_reorder():
    desc = W.tiny_model(2, 64, 2, 1, 32, 128, 72, "fp32")
    seed = 51
    weights = W.make_weights(desc, seed)
    vis, prompt = W.make_prefix(desc, seed, 0, 9, 3)
    cache, pending = O.prefill(desc, weights, vis, prompt)
    base = len(cache)
    n = 90
    target = O.greedy_decode(desc, weights, cache, pending, n)
    cache.truncate(base)
    rng = np.random.default_rng(9)
    drafts = _corrupt_set(rng, target, desc.vocab)
    out, rounds = O.spec_decode_matching(desc, weights, cache, pending, drafts, n, n_window=3, max_packed=32)
    np.testing.assert_array_equal(out, target)            # whatever the drafts are, the output is the greedy one
    assert len(rounds) < 0.7 * n                          # and it took far fewer passes than tokens
    assert max(r[0] for r in rounds) <= 32
    assert any(r[0] == 1 for r in rounds)                 # some rounds had no candidate: plain decoding steps
    cache.truncate(base)
    # a perfect single draft is consumed several tokens per pass (repeated windows may split the cap among
    # several candidates, so not always at the cap's pace)
    out, rounds = O.spec_decode_matching(desc, weights, cache, pending, [target.tolist()], n, max_packed=32)
    np.testing.assert_array_equal(out, target)
    assert len(rounds) <= n // 8 and all(a == r - 1 for r, a in rounds[:1])
