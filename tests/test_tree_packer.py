"""The host-side tree packer and window matching of the product against the oracle's independently written
versions (CPU only)."""
import numpy as np

import oracle as O


def test_runtime_packer_matches_oracle_tree():
    from paper_2602_12957_amd.runtime import pack_prefix_tree
    rng = np.random.default_rng(0)
    for _ in range(300):
        cands = [rng.integers(0, 4, size=int(rng.integers(0, 7))).tolist() for _ in range(int(rng.integers(0, 8)))]
        tokens, parent, depth, end = O.build_prefix_tree(5, cands)
        t2, e2, d2 = pack_prefix_tree(5, cands)
        assert t2.dtype == np.int32 and e2.dtype == np.int32 and d2.dtype == np.int32
        np.testing.assert_array_equal(tokens, t2)
        np.testing.assert_array_equal(end, e2)
        np.testing.assert_array_equal(depth, d2)
    t, e, d = pack_prefix_tree(9, [])
    assert t.tolist() == [9] and e.tolist() == [1] and d.tolist() == [0]
    long = list(range(5000))                       # a chain far deeper than Python's default recursion limit
    t, e, d = pack_prefix_tree(1, [long])
    assert d.tolist() == list(range(5001)) and (e == 5001).all()


def test_host_matching_equals_oracle_matching():
    from paper_2602_12957_amd.specdecode import cap_candidates, match_candidates
    rng = np.random.default_rng(3)
    for _ in range(300):
        n = int(rng.integers(1, 4))
        acc = rng.integers(0, 3, size=int(rng.integers(0, 9))).tolist()
        drafts = [rng.integers(0, 3, size=int(rng.integers(0, 12))).tolist() for _ in range(int(rng.integers(0, 4)))]
        c1, c2 = match_candidates(acc, drafts, n), O.match_candidates(acc, drafts, n)
        assert c1 == c2
        cap = int(rng.integers(4, 40))
        assert cap_candidates(c1, cap) == O.cap_candidates(c2, cap)
