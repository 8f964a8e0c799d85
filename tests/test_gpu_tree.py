"""GPU parity of prefix-tree batching (paper Section 3.2: prefix tree, tree-ancestry attention mask, greedy
traversal Eq. 9-12, commit of the accepted path) through the C ABI.

(1) One pass over a ragged batch of packed trees against the oracle: every row's logits element-wise, the per-row
    candidate gaps, and (alpha, bonus, stop node) exactly where the oracle's margins clear the gate.
(2) Rounds of tree verification WITH commit (KV compaction of the accepted path) against the same library's
    token-by-token greedy decoding: bit-exact, no oracle involved -- any error in the mask, the node positions, the
    slot/position split or the compaction breaks it."""
import math

import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from workloads.generators import SequenceSpec

from hsd_testlib import make_engine, prefix_rows

pytestmark = pytest.mark.gpu

FP32 = W.ModelDesc(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=1, head_dim=64, d_ffn=256, vocab=512, dtype="fp32")
BF16 = W.ModelDesc(n_layers=3, d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=512, vocab=1024, dtype="bf16")
TOL = {"fp32": 1e-4, "bf16": 2e-2}


def _candidates(rng, target, vocab, n_cand, length):
    """Drafts of the next `length` target tokens, each wrong from a random point on; some share long prefixes."""
    rest = np.asarray(target[:length])
    out = []
    for _ in range(n_cand):
        d = rest.copy()
        cut = int(rng.integers(0, len(d) + 1))
        d[cut:] = rng.integers(0, vocab, size=len(d) - cut)
        out.append(d.tolist())
    return out


def _walk(argmax, tokens, end, gap, want, log_tau):
    """The traversal rule applied to the GPU's own per-row outputs (numpy re-statement for the closed-form check)."""
    s, alpha = 0, 0
    while True:
        kids, c = [], s + 1
        while c < end[s]:
            kids.append(c)
            c = end[c]
        if not kids:
            break
        if log_tau < 0:
            best = max(kids, key=lambda k: (want[k], -k))
            if not gap[best] >= np.float32(log_tau):
                break
        else:
            hit = [k for k in kids if tokens[k] == argmax[s]]
            if not hit:
                break
            best = hit[0]
        s, alpha = best, alpha + 1
    return alpha, int(argmax[s]), s


@pytest.mark.parametrize("desc,chunk", [(FP32, None), (BF16, None), (BF16, 128)], ids=["fp32", "bf16", "bf16-keysplit128"])
@pytest.mark.parametrize("log_tau", [0.0, math.log(0.75)], ids=["exact", "tau0.75"])
@pytest.mark.parametrize("mode", ["region", "page"])
def test_one_pass_over_packed_trees(desc, chunk, log_tau, mode):
    shapes = [(40, 3, 30), (5, 2, 70), (17, 1, 12), (64, 8, 45), (0, 4, 20)]
    specs = [SequenceSpec(i, nv, npr, k, 0.0) for i, (nv, npr, k) in enumerate(shapes)]
    decided = _one_pass_trees(desc, chunk, log_tau, mode, 61, specs, [1, 4, 0, 6, 3], np.random.default_rng(7), 3)
    assert decided >= 1


def test_random_packed_trees_against_oracle():
    """Thirty seeded random combinations of model shape, GQA grouping, storage type, entry point, acceptance rule,
    attention key split and per-sequence candidate sets (0 to 6 drafts of up to 60 tokens that share prefixes of
    random length with the greedy continuation and with each other)."""
    rng = np.random.default_rng(20260213)
    decided = 0
    for it in range(30):
        heads = [(4, 1), (4, 2), (8, 2), (4, 4), (16, 4)][rng.integers(0, 5)]
        dt = "bf16" if rng.random() < 0.7 else "fp32"
        desc = W.ModelDesc(n_layers=int(rng.integers(1, 4)), d_model=int(rng.choice([128, 256])), n_q_heads=heads[0],
                           n_kv_heads=heads[1], head_dim=64, d_ffn=256, vocab=int(rng.choice([512, 1024])), dtype=dt)
        specs, n_cands = [], []
        for i in range(int(rng.integers(1, 5))):
            nv = int(rng.choice([0, 1, 16, 47, 64, 130]))
            specs.append(SequenceSpec(i, nv, int(rng.integers(1 if nv == 0 else 0, 5)), int(rng.choice([1, 7, 31, 60])), 0.0))
            n_cands.append(int(rng.integers(0, 7)))
        log_tau = 0.0 if rng.random() < 0.5 else math.log(0.75)
        mode = "page" if rng.random() < 0.4 else "region"
        chunk = int(rng.choice([0, 128])) if dt == "bf16" else 0
        seed = int(rng.integers(1, 10000))
        print(it, desc, [(s.n_visual, s.n_prompt, s.draft_len) for s in specs], n_cands, mode, log_tau, chunk, seed, flush=True)
        decided += _one_pass_trees(desc, chunk or None, log_tau, mode, seed, specs, n_cands, rng, -1)
    assert decided >= 30


def _one_pass_trees(desc, chunk, log_tau, mode, seed, specs, n_cands, rng, with_target):
    """One verification pass over packed prefix trees against the oracle; returns the number of sequences whose
    acceptance could be compared exactly (every deciding row clear of the tie gate).  `with_target`: index of the
    sequence whose candidate set also holds the greedy continuation itself (-1: none)."""
    from paper_2602_12957_amd.runtime import pack_prefix_tree
    weights = W.make_weights(desc, seed)
    n = len(specs)
    ora, blocks, trees = [], [], []
    for sp in specs:
        vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
        cache, pending = O.prefill(desc, weights, vis, prompt)
        base = len(cache)
        target = O.greedy_decode(desc, weights, cache, pending, sp.draft_len)
        cache.truncate(base)
        cands = _candidates(rng, target, desc.vocab, n_cands[sp.seq_id], sp.draft_len)
        if sp.seq_id == with_target:
            cands.append(target.tolist())           # the greedy continuation itself is among the drafts
        acc, bonus, logits, (tokens, parent, depth, end) = O.verify_tree(desc, weights, cache, pending, cands,
                                                                         log_tau=log_tau)
        ora.append((acc, bonus, logits, tokens, parent, end))
        t, e, d = pack_prefix_tree(pending, cands)
        np.testing.assert_array_equal(t, tokens)
        blocks.append(t)
        trees.append((e, d))
    total = sum(len(b) for b in blocks)
    sized = [SequenceSpec(sp.seq_id, sp.n_visual, sp.n_prompt, len(b), 0.0) for sp, b in zip(specs, blocks)]
    eng = make_engine(desc, weights, sized, max_dump=total, attn_key_chunk=chunk)
    toks, embs = [], []
    for sp in specs:
        _, _, tok, emb, _ = prefix_rows(desc, seed, sp)
        toks.append(tok), embs.append(emb)
    eng.prefill(list(range(n)), toks, embs)
    out = eng.verify(list(range(n)), blocks, mode, dump_rows=np.arange(total), log_tau=log_tau, trees=trees)
    g_alpha, g_bonus, status = eng.read_acceptance(n)
    assert status == 0
    g_logits = out.logits.cpu().numpy()
    g_arg = out.argmax.cpu().numpy()
    g_stop = out.stop_row.cpu().numpy()
    g_gap = out.gap.cpu().numpy() if log_tau < 0 else None
    gate = 2 * TOL[desc.dtype]
    decided = 0
    for i, (acc, bonus, logits, tokens, parent, end) in enumerate(ora):
        lo, hi = out.cu_q[i], out.cu_q[i + 1]
        assert hi - lo == len(tokens)
        err = float(np.abs(g_logits[lo:hi] - logits).max())
        assert err <= TOL[desc.dtype], (i, err)
        want = None
        if log_tau < 0:
            ref_gap = np.full(len(tokens), -np.inf)
            for c in range(1, len(tokens)):
                ref_gap[c] = logits[parent[c], tokens[c]] - logits[parent[c]].max()
            assert g_gap[lo] == -np.inf
            assert np.abs(g_gap[lo + 1:hi] - ref_gap[1:]).max(initial=0.0) <= gate
            want = np.array([g_logits[lo + parent[c], tokens[c]] if c else -np.inf for c in range(len(tokens))])
        a_closed, b_closed, s_closed = _walk(g_arg[lo:hi], tokens, end, None if g_gap is None else g_gap[lo:hi], want, log_tau)
        assert (g_alpha[i], g_bonus[i], g_stop[i]) == (a_closed, b_closed, s_closed), i
        # against the oracle where every deciding row clears the gate
        path_rows = [0]
        for t in acc:
            path_rows.append(next(c for c in range(len(tokens)) if parent[c] == path_rows[-1] and tokens[c] == t))
        margin = O.top2_margin(logits)
        clear = all(margin[r] > gate for r in path_rows)
        if log_tau < 0:
            kids_gap = [ref_gap[c] for r in path_rows for c in range(len(tokens)) if parent[c] == r]
            clear = clear and all(abs(g - log_tau) > gate for g in kids_gap)
        if clear:
            assert (g_alpha[i], g_bonus[i], g_stop[i]) == (len(acc), bonus, path_rows[-1]), i
            decided += 1
    eng.close()
    print(desc.dtype, mode, log_tau, "decided", decided, "of", n)
    return decided


def _row_of_path(tokens, end, path):
    """Packed row of the node reached from the root along `path` (it exists by construction)."""
    s = 0
    for t in path:
        c = s + 1
        while tokens[c] != t:
            c = end[c]
        s = c
    return s


def _tree_rounds_lossless(desc, specs, seed, mode, n_cand, window, tie_gate=0.0):
    """tie_gate = 0: bit-exact agreement with greedy decoding is required.  tie_gate > 0 (deep models): a tree row
    keeps its K/V in another cache slot than the one it would have in a chain, so the attention sums group the
    keys differently and results agree only to rounding; a round may then stop early at a row whose own
    top-1/top-2 margin is below tie_gate, is counted, and is re-synchronised to the greedy sequence."""
    from paper_2602_12957_amd.runtime import pack_prefix_tree
    weights = W.make_weights(desc, seed)
    n = len(specs)
    worst = SequenceSpec(0, 0, 0, n_cand * window + 1, 0.0)
    sized = [SequenceSpec(sp.seq_id, sp.n_visual, sp.n_prompt, sp.draft_len + worst.draft_len, 0.0) for sp in specs]
    eng = make_engine(desc, weights, sized, max_total_q=max(4096, n * (worst.draft_len + 1)))
    toks, embs, pend = [], [], []
    for sp in specs:
        _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
        toks.append(tok), embs.append(emb), pend.append(pending)
    slots = list(range(n))
    eng.prefill(slots, toks, embs)
    k_max = max(sp.draft_len for sp in specs)
    target = eng.greedy_decode(slots, pend, k_max, mode)
    eng.reset()
    eng.prefill(slots, toks, embs)
    rng = np.random.default_rng(seed)
    committed = [[] for _ in range(n)]
    pending = list(pend)
    active, rounds, moved, ties = slots, 0, 0, []
    while active:
        blocks, trees, expect = [], [], []
        for i in active:
            o = len(committed[i])
            rest = target[i][o:specs[i].draft_len]
            cands = _candidates(rng, rest, desc.vocab, n_cand, min(window, len(rest)))
            t, e, d = pack_prefix_tree(pending[i], cands)
            blocks.append(t), trees.append((e, d))
            in_tree = {tuple(c[:k]) for c in cands for k in range(len(c) + 1)}
            expect.append(max(k for k in range(min(window, len(rest)) + 1) if tuple(rest[:k].tolist()) in in_tree))
        out = eng.verify(active, blocks, mode, trees=trees)
        alpha, bonus, status = eng.read_acceptance(len(active))
        stop = out.stop_row.cpu().numpy()
        margin = out.margin.cpu().numpy()
        assert status == 0
        fix_a, fix_b, fix_s, nxt = [], [], [], []
        for j, i in enumerate(active):
            o = len(committed[i])
            known = o + expect[j] < target.shape[1]        # the greedy token after the accepted path, if generated
            want_b = int(target[i][o + expect[j]]) if known else int(bonus[j])
            if (alpha[j], bonus[j]) != (expect[j], want_b):
                # only a near-tie at the GPU's stop row may explain an early stop or another bonus token
                assert tie_gate > 0 and alpha[j] <= expect[j], f"seq {i} round {rounds}: alpha {alpha[j]} != {expect[j]}"
                assert margin[out.cu_q[j] + stop[j]] < tie_gate, (i, rounds, float(margin[out.cu_q[j] + stop[j]]))
                ties.append((i, rounds))
            path = target[i][o:o + expect[j]].tolist()
            fix_a.append(expect[j]), fix_b.append(want_b), fix_s.append(_row_of_path(blocks[j], trees[j][0], path))
            moved += int(fix_s[-1] != expect[j])
            committed[i].extend(path)
            committed[i].append(want_b)
            pending[i] = want_b
            if len(committed[i]) < specs[i].draft_len:
                nxt.append(i)
        if tie_gate > 0:
            eng.override_acceptance(np.asarray(fix_a), np.asarray(fix_b), np.asarray(fix_s))
        eng.commit()
        active = nxt
        rounds += 1
    for i, sp in enumerate(specs):
        np.testing.assert_array_equal(np.asarray(committed[i][:sp.draft_len]), target[i][:sp.draft_len])
    torch.cuda.synchronize()
    seq_len = eng.seq_len.cpu().numpy()
    for i, sp in enumerate(specs):
        assert seq_len[i] == sp.n_visual + max(sp.n_prompt - 1, 0) + len(committed[i])
    owned = int((eng.block_table.cpu().numpy() >= 0).sum())
    assert owned == sum((int(x) + 15) // 16 for x in seq_len[:n])
    assert owned + int(eng.free_count.item()) == eng.n_blocks
    eng.close()
    return rounds, moved, ties


@pytest.mark.parametrize("mode", ["region", "page"])
def test_tree_rounds_with_commit_are_lossless_small_models(mode):
    for desc in (FP32, BF16):
        specs = [SequenceSpec(0, 40, 3, 90, 0.0), SequenceSpec(1, 5, 2, 70, 0.0), SequenceSpec(2, 130, 5, 33, 0.0),
                 SequenceSpec(3, 0, 4, 150, 0.0)]
        rounds, moved, _ = _tree_rounds_lossless(desc, specs, 13, mode, n_cand=4, window=24)
        assert rounds >= 3 and moved > 0        # some accepted paths really had to be moved


def test_tree_rows_equal_chain_rows_to_rounding_model_m():
    """24-layer bf16 model: the logits of the nodes on one root-to-leaf path of a packed tree against the logits of
    the same tokens verified as a chain, both on the GPU.  The two differ only in the cache slots the path's K/V
    occupy during the pass (hence in how the attention sums group the keys): agreement to the model's rounding
    noise floor (sigma ~ 1e-2 for this model, see tests/test_oracle_noise_floor.py), nowhere near a masking or
    position error (which changes logits by O(1))."""
    from paper_2602_12957_amd.runtime import pack_prefix_tree
    desc, seed = W.MODEL_M, W.SEED_BASE
    weights = W.make_weights(desc, seed)
    sp = SequenceSpec(0, 300, 8, 40, 0.0)
    rng = np.random.default_rng(5)
    path = rng.integers(0, desc.vocab, size=24).tolist()
    cands = [path[:6] + rng.integers(0, desc.vocab, size=10).tolist(), path, path[:15] + [3, 4, 5],
             rng.integers(0, desc.vocab, size=12).tolist()]
    sized = [SequenceSpec(0, sp.n_visual, sp.n_prompt, 80, 0.0)]
    eng = make_engine(desc, weights, sized, max_total_q=4096, max_dump=32)
    _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
    eng.prefill([0], [tok], [emb])
    chain = np.concatenate([[pending], path]).astype(np.int32)
    out = eng.verify([0], [chain], "region", dump_rows=np.arange(len(chain)))
    ref = out.logits.cpu().numpy().copy()
    eng.override_acceptance(np.array([-1]), np.array([0]))
    eng.commit()                                           # roll the chain pass back
    t, e, d = pack_prefix_tree(pending, cands)
    rows = [0]
    for tk in path:
        rows.append(_row_of_path(t, e, path[:len(rows)]))
    assert rows != list(range(len(rows)))                  # the path is not stored contiguously in the tree
    out = eng.verify([0], [t], "region", dump_rows=np.asarray(rows), trees=[(e, d)])
    got = out.logits.cpu().numpy()
    diff = got - ref
    rms, worst = float(np.sqrt((diff ** 2).mean())), float(np.abs(diff).max())
    print("tree vs chain rows: rms", rms, "max", worst)
    eng.close()
    assert rms <= 2e-2 and worst <= 1e-1


def test_tree_rounds_with_commit_are_lossless_model_m():
    """24-layer bf16 model, 8 regions with 1055 cached tokens, 5 candidates of up to 48 tokens per round."""
    specs = [SequenceSpec(i, 1024, 32, 120, 0.0) for i in range(8)]
    rounds, moved, ties = _tree_rounds_lossless(W.MODEL_M, specs, W.SEED_BASE, "region", n_cand=5, window=48,
                                                tie_gate=0.07)
    print("model M tree rounds", rounds, "moved paths", moved, "near-tie stops", ties)
    assert moved > 0 and len(ties) <= rounds * len(specs) // 4


def test_malformed_tree_is_clamped_and_flagged():
    """tree_end / tree_depth entries that do not describe a packed pre-order tree are clamped on the device to a
    valid one (so nothing can index outside its block) and reported in the status word; a well-formed call on the
    same engine afterwards is unaffected."""
    import paper_2602_12957_amd.binding as B
    from paper_2602_12957_amd.runtime import pack_prefix_tree
    desc, seed = BF16, 5
    weights = W.make_weights(desc, seed)
    sp = SequenceSpec(0, 20, 3, 40, 0.0)
    eng = make_engine(desc, weights, [sp], max_dump=0)
    _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
    eng.prefill([0], [tok], [emb])
    cands = [[1, 2, 3, 4], [1, 2, 9], [7, 8]]
    t, e, d = pack_prefix_tree(pending, cands)
    for bad_e, bad_d in ((np.zeros_like(e), d), (np.full_like(e, 10 ** 6), d), (e, np.full_like(d, -3)),
                         (e[::-1].copy(), d[::-1].copy())):
        eng.status.zero_()
        for lt in (0.0, math.log(0.5)):
            eng.verify([0], [t], "region", log_tau=lt, trees=[(bad_e, bad_d)])
            alpha, bonus, status = eng.read_acceptance(1)
            assert status & B.HSD_STATUS_BAD_TREE
            assert 0 <= alpha[0] < len(t)
            eng.commit()                                   # compaction walks the same (clamped) structure
            torch.cuda.synchronize()
            # roll the sequence back to its prefix for the next case
            eng.reset()
            eng.prefill([0], [tok], [emb])
    eng.status.zero_()
    out = eng.verify([0], [t], "region", trees=[(e, d)])
    alpha, bonus, status = eng.read_acceptance(1)
    assert status == 0 and 0 <= out.stop_row.cpu().numpy()[0] < len(t)
    eng.close()
