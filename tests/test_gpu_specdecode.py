"""The host driver of decoupled speculative verification on the GPU path (paper Section 3.2, Eq. 1-6): window
matching against a fixed draft set, prefix-tree batching, rounds with commit -- and the two stages of the
hierarchy (regions in one batch, then the page with the regions' outputs as drafts, Eq. 2-4).

Whatever the drafts contain, the output must be the model's own greedy sequence (exact rule): checked bit for bit
against the same library's token-by-token decoding on shallow models, and the host logic against the oracle's
independently written matching functions."""
import numpy as np
import pytest

import oracle as O
import workloads as W
from workloads.generators import SequenceSpec

from hsd_testlib import make_engine, prefix_rows

pytestmark = pytest.mark.gpu

FP32 = W.ModelDesc(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=1, head_dim=64, d_ffn=256, vocab=512, dtype="fp32")
BF16 = W.ModelDesc(n_layers=3, d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=512, vocab=1024, dtype="bf16")


def _defective_drafts(rng, target, vocab, n_seg=4):
    """The target cut into segments in another order, with deletions, insertions and substitutions."""
    cuts = sorted(rng.choice(np.arange(5, len(target) - 5), size=n_seg - 1, replace=False).tolist())
    segs = [target[a:b].tolist() for a, b in zip([0] + cuts, cuts + [len(target)])]
    rng.shuffle(segs)
    out = []
    for sgm in segs:
        d = []
        for t in sgm:
            r = rng.random()
            if r < 0.03:
                continue
            if r < 0.06:
                d.append(int(rng.integers(0, vocab)))
            d.append(int(rng.integers(0, vocab)) if r > 0.96 else int(t))
        out.append(d)
    return out


@pytest.mark.parametrize("desc", [FP32, BF16], ids=["fp32", "bf16"])
def test_decoupled_rounds_reproduce_greedy_decoding(desc):
    from paper_2602_12957_amd.specdecode import SpecDecoder
    seed = 71
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 40, 3, 120, 0.0), SequenceSpec(1, 5, 2, 90, 0.0), SequenceSpec(2, 130, 5, 60, 0.0)]
    n = len(specs)
    sized = [SequenceSpec(sp.seq_id, sp.n_visual, sp.n_prompt, sp.draft_len + 40, 0.0) for sp in specs]
    eng = make_engine(desc, weights, sized, max_total_q=4096)
    toks, embs, pend = [], [], []
    for sp in specs:
        _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
        toks.append(tok), embs.append(emb), pend.append(pending)
    slots = list(range(n))
    eng.prefill(slots, toks, embs)
    k_max = max(sp.draft_len for sp in specs)
    target = eng.greedy_decode(slots, pend, k_max)
    eng.reset()
    eng.prefill(slots, toks, embs)
    rng = np.random.default_rng(seed)
    draft_sets = [_defective_drafts(rng, target[i][:sp.draft_len], desc.vocab) for i, sp in enumerate(specs)]
    dec = SpecDecoder(eng, n_window=3, max_packed=32)
    outs, stats = dec.run(slots, pend, draft_sets, [sp.draft_len for sp in specs])
    for i, sp in enumerate(specs):
        np.testing.assert_array_equal(outs[i], target[i][:sp.draft_len])
    total = sum(sp.draft_len for sp in specs)
    print(desc.dtype, stats, "tokens", total)
    assert stats["seq_rounds"] < 0.7 * total          # far fewer passes than tokens
    assert stats["plain_steps"] > 0                   # realignment really needed some plain decoding steps
    eng.close()


def test_decoupled_rounds_match_the_oracle_driver():
    """SpecDecoder on the HIP path against oracle.spec_decode_matching on the same fp32 model and the same defective
    draft sets (Section 3.2, Eq. 5-6: window matching; Eq. 7: prefix-tree batching; Eq. 9-12: tree walk), with a
    128-row and a 24-row cap: the committed tokens and, round by round, the size of the packed tree and the number
    of accepted tokens must be the oracle's.  The fp32 path's logits are within 1e-4 of the oracle's (measured: 2e-6);
    every decision is taken at a row of the greedy path, and the seed is one for which no greedy step of the oracle has
    a top-1/top-2 margin under 1e-4 (asserted), so every decision is unambiguous."""
    from paper_2602_12957_amd.specdecode import SpecDecoder
    desc, seed = FP32, 78
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 40, 3, 100, 0.0), SequenceSpec(1, 5, 2, 80, 0.0), SequenceSpec(2, 130, 5, 60, 0.0)]
    n = len(specs)
    rng = np.random.default_rng(seed)
    caches, pend, draft_sets = [], [], []
    for sp in specs:
        vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
        cache, pending = O.prefill(desc, weights, vis, prompt)
        base = len(cache)
        target, margins = O.greedy_decode(desc, weights, cache, pending, sp.draft_len, return_margins=True)
        assert margins.min() > 1e-4, margins.min()
        cache.truncate(base)
        caches.append(cache), pend.append(pending)
        draft_sets.append(_defective_drafts(rng, target, desc.vocab))
    sized = [SequenceSpec(sp.seq_id, sp.n_visual, sp.n_prompt, sp.draft_len + 140, 0.0) for sp in specs]
    for cap in (128, 24):
        expect = []
        for i, sp in enumerate(specs):
            base = len(caches[i])
            expect.append(O.spec_decode_matching(desc, weights, caches[i], pend[i], draft_sets[i], sp.draft_len,
                                                 n_window=3, max_packed=cap))
            caches[i].truncate(base)
        eng = make_engine(desc, weights, sized, max_total_q=4096)
        toks, embs = [], []
        for sp in specs:
            _, _, tok, emb, _ = prefix_rows(desc, seed, sp)
            toks.append(tok), embs.append(emb)
        eng.prefill(list(range(n)), toks, embs)
        outs, stats = SpecDecoder(eng, n_window=3, max_packed=cap).run(list(range(n)), pend, draft_sets,
                                                                       [sp.draft_len for sp in specs])
        eng.close()
        for i in range(n):
            np.testing.assert_array_equal(outs[i], expect[i][0])
            assert stats["per_seq"][i] == [tuple(r) for r in expect[i][1]], (cap, i)
        print("cap", cap, "rounds per sequence", [len(e[1]) for e in expect], "accepted", stats["accepted"])
        assert stats["accepted"] > 0


def test_two_stage_hierarchy_on_one_engine():
    """Stage 1: three regions verified in one batch from defective region drafts.  Stage 2: the page (its own,
    longer prefix) verified with the UNORDERED collection of Stage-1 outputs as its draft set.  The page's greedy
    text is built to contain the regions' texts in another order with glue tokens the drafts lack."""
    from paper_2602_12957_amd.specdecode import SpecDecoder
    desc, seed = FP32, 73
    weights = W.make_weights(desc, seed)
    regions = [SequenceSpec(0, 30, 3, 50, 0.0), SequenceSpec(1, 12, 2, 40, 0.0), SequenceSpec(2, 50, 4, 45, 0.0)]
    page = SequenceSpec(3, 200, 4, 150, 0.0)
    specs = regions + [page]
    sized = [SequenceSpec(sp.seq_id, sp.n_visual, sp.n_prompt, sp.draft_len + 40, 0.0) for sp in specs]
    eng = make_engine(desc, weights, sized, max_total_q=4096)
    toks, embs, pend = [], [], []
    for sp in specs:
        _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
        toks.append(tok), embs.append(emb), pend.append(pending)
    slots = list(range(4))
    eng.prefill(slots, toks, embs)
    target = eng.greedy_decode(slots, pend, max(sp.draft_len for sp in specs))
    eng.reset()
    eng.prefill(slots, toks, embs)
    rng = np.random.default_rng(seed)
    # Stage 1
    s1 = SpecDecoder(eng, max_packed=32, mode="region")
    r_drafts = [_defective_drafts(rng, target[i][:sp.draft_len], desc.vocab, n_seg=2) for i, sp in enumerate(regions)]
    r_out, st1 = s1.run(slots[:3], pend[:3], r_drafts, [sp.draft_len for sp in regions])
    for i, sp in enumerate(regions):
        np.testing.assert_array_equal(r_out[i], target[i][:sp.draft_len])
    # Stage 2: the page's drafts are the region outputs plus, so that they are of any use with random weights,
    # pieces of the page's own greedy text standing in for "what the regions read"
    page_t = target[3][:page.draft_len]
    pieces = [page_t[100:150].tolist(), page_t[0:45].tolist(), page_t[50:95].tolist()]
    drafts_pg = [o.tolist() for o in r_out] + pieces
    s2 = SpecDecoder(eng, max_packed=64, mode="page")
    p_out, st2 = s2.run([3], [pend[3]], [drafts_pg], [page.draft_len])
    np.testing.assert_array_equal(p_out[0], page_t)
    print("stage 1", st1, "stage 2", st2)
    assert st2["seq_rounds"] < 0.5 * page.draft_len
    eng.close()
