"""GPU parity: the HIP verification path against the CPU oracle, element by element, through the C ABI.

Bars: fp32 path logits max-abs <= 1e-4; bf16 path logits max-abs <= 2e-2; arg-max, alpha and bonus
bit-exact wherever the oracle's top-1/top-2 margin of every deciding row exceeds 1e-2.
"""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from workloads.generators import SequenceSpec

from hsd_testlib import MARGIN_GATE, make_engine, prefix_rows, oracle_targets, gated_compare_argmax

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def _oracle_state(desc, weights, seed, specs):
    st = []
    for sp in specs:
        vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
        cache, pending = O.prefill(desc, weights, vis, prompt)
        st.append([cache, pending])
    return st


def _gpu_prefill(eng, desc, seed, specs):
    toks, embs, pend = [], [], []
    for sp in specs:
        _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
        toks.append(tok)
        embs.append(emb)
        pend.append(pending)
    eng.prefill(list(range(len(specs))), toks, embs)
    return pend


def run_rounds_parity(desc, weights, seed, specs, drafts, mode="region", check_logits=True, attn_key_chunk=None):
    """Runs verification rounds to completion on both sides, teacher-forcing the GPU to the oracle's state
    after each round, and compares every output of every round."""
    n = len(specs)
    total_q = sum(len(d) + 1 for d in drafts)
    eng = make_engine(desc, weights, specs, max_total_q=max(total_q, max(s.n_visual + s.n_prompt for s in specs)),
                      max_dump=total_q if check_logits else 0, attn_key_chunk=attn_key_chunk)
    ora = _oracle_state(desc, weights, seed, specs)
    pend = _gpu_prefill(eng, desc, seed, specs)
    assert pend == [o[1] for o in ora]
    committed = [0] * n
    active = list(range(n))
    stats = dict(rounds=0, rows=0, gated_rows=0, gated_rounds=0, max_logit_err=0.0)
    tol = TOL[desc.dtype]
    while active:
        blocks, recs = [], []
        for s in active:
            rest = drafts[s][committed[s]:]
            blocks.append(np.concatenate([[ora[s][1]], rest]).astype(np.int32))
            base = len(ora[s][0])
            alpha, bonus, u_hat, logits = O.verify_block(desc, weights, ora[s][0], ora[s][1], rest)
            ora[s][0].truncate(base + 1 + alpha)
            recs.append((alpha, bonus, u_hat, logits, O.top2_margin(logits)))
        T = sum(len(b) for b in blocks)
        out = eng.verify(active, blocks, mode, dump_rows=np.arange(T) if check_logits else None)
        g_alpha, g_bonus, status = eng.read_acceptance(len(active))
        assert status == 0
        g_argmax = out.argmax.cpu().numpy()
        g_margin = out.margin.cpu().numpy()
        g_logits = out.logits.cpu().numpy() if check_logits else None
        for i, s in enumerate(active):
            alpha, bonus, u_hat, logits, margin = recs[i]
            lo, hi = out.cu_q[i], out.cu_q[i + 1]
            if check_logits:
                err = float(np.abs(g_logits[lo:hi] - logits).max())
                stats["max_logit_err"] = max(stats["max_logit_err"], err)
                assert err <= tol, f"seq {s}: logits differ by {err}"
                assert np.abs(g_margin[lo:hi] - margin).max() <= 2 * tol
            bad, n_ok = gated_compare_argmax(g_argmax[lo:hi], u_hat, margin)
            assert len(bad) == 0, f"seq {s}: arg-max differs at rows {bad} with margins {margin[bad]}"
            stats["rows"] += hi - lo
            stats["gated_rows"] += (hi - lo) - n_ok
            if np.all(margin[:alpha + 1] > MARGIN_GATE):
                assert (g_alpha[i], g_bonus[i]) == (alpha, bonus), f"seq {s} round {stats['rounds']}"
            else:
                stats["gated_rounds"] += 1
        # re-synchronise the GPU to the oracle's decisions, then commit
        eng.override_acceptance(np.array([r[0] for r in recs]), np.array([r[1] for r in recs]))
        eng.commit()
        nxt = []
        for i, s in enumerate(active):
            committed[s] += recs[i][0] + 1
            ora[s][1] = recs[i][1]
            if committed[s] < len(drafts[s]):
                nxt.append(s)
        active = nxt
        stats["rounds"] += 1
    # KV accounting after the last commit: every block is either free or owned by a committed position
    torch.cuda.synchronize()
    seq_len = eng.seq_len.cpu().numpy()
    for s in range(n):
        assert seq_len[s] == len(ora[s][0])
    owned = int((eng.block_table.cpu().numpy() >= 0).sum())
    assert owned == sum((int(x) + 15) // 16 for x in seq_len)
    assert owned + int(eng.free_count.item()) == eng.n_blocks
    eng.close()
    return stats


def test_config0_tiny_fp32_full_rounds():
    """BASELINE config 0: 2 layers, d 256, 4x64 heads, FFN 1024, vocab 4096, fp32; 4 regions of 256 visual
    + 16 prompt tokens; draft 32 = oracle greedy output corrupted at p = 0.1."""
    desc, seed = W.MODEL_T, W.SEED_BASE
    weights = W.make_weights(desc, seed)
    specs = W.draw_sequences(0, seed)
    targets = oracle_targets(desc, weights, seed, specs)
    drafts = [W.corrupt_draft(g, sp.corrupt_p, desc.vocab, seed, f"cfg0.{sp.seq_id}")[0] for (g, _), sp in zip(targets, specs)]
    stats = run_rounds_parity(desc, weights, seed, specs, drafts)
    print("cfg0", stats)
    assert stats["rounds"] >= 2 and stats["max_logit_err"] <= 1e-4


SMALL_BF16 = W.ModelDesc(n_layers=3, d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=512, vocab=1024, dtype="bf16")
SMALL_FP32 = W.ModelDesc(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=1, head_dim=64, d_ffn=256, vocab=512, dtype="fp32")
# two 64-wide K slices per projection: the shortest GEMM pipeline, and every large-tile configuration falls back
NARROW_BF16 = W.ModelDesc(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=256, vocab=640, dtype="bf16")


@pytest.mark.parametrize("desc", [SMALL_FP32, SMALL_BF16, NARROW_BF16], ids=["fp32", "bf16", "bf16-narrow"])
@pytest.mark.parametrize("mode", ["region", "page"])
def test_ragged_batch_rounds(desc, mode):
    """Ragged prefixes and drafts spanning several tiles with ragged tails, GQA, both entry points.
    Draft lengths hit alpha = 0, 63, 64, 65 and full acceptance to cross wave boundaries of the scan."""
    seed = 77
    weights = W.make_weights(desc, seed)
    shapes = [(40, 3, 1), (5, 2, 70), (130, 5, 131), (17, 1, 64), (64, 8, 200), (0, 4, 66), (33, 0, 90)]
    specs = [SequenceSpec(i, nv, npr, k, 0.0) for i, (nv, npr, k) in enumerate(shapes)]
    targets = oracle_targets(desc, weights, seed, specs)
    drafts = []
    first_bad = {1: 0, 2: 63, 3: None, 4: 65, 5: None, 6: 64}     # position of the first forced mismatch
    for (g, _), sp in zip(targets, specs):
        d = g.copy()
        fb = first_bad.get(sp.seq_id, None)
        if fb is not None and fb < len(d):
            d[fb] = (d[fb] + 1) % desc.vocab
            if fb + 7 < len(d):
                d[fb + 7] = (d[fb + 7] + 3) % desc.vocab
        drafts.append(d)
    stats = run_rounds_parity(desc, weights, seed, specs, drafts, mode=mode)
    print(desc.dtype, mode, stats)
    assert stats["gated_rows"] < 0.5 * stats["rows"]


@pytest.mark.parametrize("chunk", [128, 256])
def test_key_split_attention_rounds(chunk):
    """The same rounds against the oracle with the attention keys cut into chunks (hsd_model_desc.attn_key_chunk):
    contexts of 4 to 539 tokens give rows with one to five chunks, query tiles whose rows see different numbers of
    chunks, and chunks that hold no visible key for some rows of a tile."""
    desc, seed = SMALL_BF16, 78
    weights = W.make_weights(desc, seed)
    shapes = [(40, 3, 1), (5, 2, 70), (130, 5, 131), (125, 3, 64), (320, 8, 210), (0, 4, 130), (33, 0, 90)]
    specs = [SequenceSpec(i, nv, npr, k, 0.0) for i, (nv, npr, k) in enumerate(shapes)]
    targets = oracle_targets(desc, weights, seed, specs)
    drafts = []
    for (g, _), sp in zip(targets, specs):
        d = g.copy()
        if sp.seq_id % 2 and len(d) > 40:
            d[37] = (d[37] + 1) % desc.vocab
        drafts.append(d)
    stats = run_rounds_parity(desc, weights, seed, specs, drafts, mode="region", attn_key_chunk=chunk)
    print("key split", chunk, stats)
    assert stats["gated_rows"] < 0.5 * stats["rows"]


def test_key_split_last_chunk_is_open_ended():
    """More keys than 8 chunks hold: the last chunk takes the rest (one pass against the oracle, 128-key chunks,
    contexts up to 1300 tokens), and the result agrees with the unsplit kernel to rounding."""
    desc, seed = SMALL_BF16, 79
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 1200, 4, 96, 0.0), SequenceSpec(1, 1010, 2, 40, 0.0)]
    rng = np.random.default_rng(5)
    drafts = [rng.integers(0, desc.vocab, size=sp.draft_len).astype(np.int32) for sp in specs]
    stats = run_rounds_parity(desc, weights, seed, specs, drafts, mode="page", attn_key_chunk=128)
    print("key split open-ended", stats)
    logits = []
    for chunk in (0, 128):
        eng = make_engine(desc, weights, specs, max_total_q=2048, max_dump=256, attn_key_chunk=chunk)
        pend = _gpu_prefill(eng, desc, seed, specs)
        blocks = [np.concatenate([[p], d]).astype(np.int32) for p, d in zip(pend, drafts)]
        logits.append(_one_round(eng, [0, 1], blocks)[1])
        eng.close()
    diff = np.abs(logits[0].astype(np.float64) - logits[1])
    assert diff.max() > 0 and np.sqrt((diff ** 2).mean()) < 2e-2, (diff.max(), np.sqrt((diff ** 2).mean()))


def test_random_shapes_against_oracle():
    """Forty seeded random combinations of depth, width, GQA grouping (1, 2, 4 query heads per kv head and
    kv-head counts of 1 to 8), storage type, vocabulary, entry point, attention key split and ragged sequences whose
    prefix and draft lengths sit on and around the tile and page boundaries (0, 1, 15-17, 63-65, ...), drafts
    corrupted at 4 % of the positions: every round of every case against the oracle."""
    rng = np.random.default_rng(20260212)
    for it in range(40):
        heads = [(4, 1), (4, 2), (8, 2), (4, 4), (8, 8), (16, 4)][rng.integers(0, 6)]
        dt = "bf16" if rng.random() < 0.7 else "fp32"
        desc = W.ModelDesc(n_layers=int(rng.integers(1, 4)), d_model=int(rng.choice([128, 256])), n_q_heads=heads[0],
                           n_kv_heads=heads[1], head_dim=64, d_ffn=int(rng.choice([256, 512])),
                           vocab=int(rng.choice([512, 640, 1024])), dtype=dt)
        seed = int(rng.integers(1, 10000))
        specs = []
        for i in range(int(rng.integers(1, 6))):
            nv = int(rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 130, 300]))
            npr = int(rng.integers(1 if nv == 0 else 0, 6))
            specs.append(SequenceSpec(i, nv, npr, int(rng.choice([1, 2, 31, 32, 33, 64, 65, 100, 190])), 0.0))
        mode = "page" if rng.random() < 0.4 else "region"
        chunk = int(rng.choice([0, 0, 128, 256])) if dt == "bf16" else 0
        weights = W.make_weights(desc, seed)
        drafts = []
        for (g, _) in oracle_targets(desc, weights, seed, specs):
            d = g.copy()
            for pos in np.nonzero(rng.random(len(d)) < 0.04)[0]:
                d[pos] = (d[pos] + 1 + rng.integers(0, desc.vocab - 1)) % desc.vocab
            drafts.append(d)
        print(it, desc, [(s.n_visual, s.n_prompt, s.draft_len) for s in specs], mode, chunk, seed, flush=True)
        run_rounds_parity(desc, weights, seed, specs, drafts, mode=mode, attn_key_chunk=chunk or None)


def test_large_pass_dispatch_agrees_bitwise_with_plain_tiles():
    """A pass of 16,880 rows (the shape of the prefix prefill) takes the dispatch paths that small batches never reach:
    the persistent form of the 256x256 GEMM (gate/up: 528 tiles for 256 compute units) and the rounds-aware row split
    (O and down: 66 x 4 tiles would be 1.03 rounds; 64 rows of tiles go to the large kernel, 496 rows to the small
    one).  None of it may change a bit: arg-max rows and sampled logit rows equal those of the same pass forced onto
    128x128 tiles everywhere."""
    desc = W.ModelDesc(n_layers=2, d_model=1024, n_q_heads=16, n_kv_heads=4, head_dim=64, d_ffn=1024, vocab=1024, dtype="bf16")
    seed = 21
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(i, 3, 2, 4219, 0.0) for i in range(4)]
    rng = np.random.default_rng(8)
    drafts = [rng.integers(0, desc.vocab, size=sp.draft_len).astype(np.int32) for sp in specs]
    total_q = sum(len(d) + 1 for d in drafts)
    assert total_q == 16880
    rows = np.unique(np.concatenate([np.arange(0, total_q, 97), np.arange(total_q - 600, total_q)])).astype(np.int32)
    results = []
    for debug in (None, {"gemm_cfg": (0, 0, 0, 0, 0)}):
        eng = make_engine(desc, weights, specs, max_total_q=total_q, max_dump=len(rows), debug=debug)
        pend = _gpu_prefill(eng, desc, seed, specs)
        blocks = [np.concatenate([[p], d]).astype(np.int32) for p, d in zip(pend, drafts)]
        out = eng.verify([0, 1, 2, 3], blocks, "page", dump_rows=rows)
        results.append((out.argmax.cpu().numpy().copy(), out.logits.cpu().numpy().copy()))
        eng.close()
    np.testing.assert_array_equal(results[0][0], results[1][0])
    np.testing.assert_array_equal(results[0][1], results[1][1])
    assert np.isfinite(results[0][1]).all()


def test_many_sequences_take_the_plain_task_order():
    """More sequences than the attention task table places group by group (over 1024 task groups: here 300 sequences
    x 4 kv heads) fall back to the plain task order; one pass of such a batch, ragged, against the oracle."""
    desc = W.ModelDesc(n_layers=2, d_model=256, n_q_heads=8, n_kv_heads=4, head_dim=64, d_ffn=256, vocab=512, dtype="bf16")
    seed = 90
    weights = W.make_weights(desc, seed)
    rng = np.random.default_rng(90)
    specs = [SequenceSpec(i, int(rng.integers(0, 40)), int(rng.integers(1, 4)), int(rng.integers(1, 70)), 0.0)
             for i in range(300)]
    drafts = [rng.integers(0, desc.vocab, size=sp.draft_len).astype(np.int32) for sp in specs]
    total_q = sum(len(d) + 1 for d in drafts)
    eng = make_engine(desc, weights, specs, max_total_q=total_q, max_dump=total_q)
    ora = _oracle_state(desc, weights, seed, specs)
    pend = _gpu_prefill(eng, desc, seed, specs)
    blocks = [np.concatenate([[p], d]).astype(np.int32) for p, d in zip(pend, drafts)]
    out = eng.verify(list(range(300)), blocks, "region", dump_rows=np.arange(total_q))
    g_alpha, g_bonus, status = eng.read_acceptance(300)
    assert status == 0
    g_logits = out.logits.cpu().numpy()
    worst = 0.0
    for i, sp in enumerate(specs):
        alpha, bonus, u_hat, logits = O.verify_block(desc, weights, ora[i][0], ora[i][1], drafts[i])
        lo, hi = out.cu_q[i], out.cu_q[i + 1]
        worst = max(worst, float(np.abs(g_logits[lo:hi] - logits).max()))
        if np.all(O.top2_margin(logits)[:alpha + 1] > MARGIN_GATE):
            assert (g_alpha[i], g_bonus[i]) == (alpha, bonus), i
    assert worst <= TOL["bf16"], worst
    eng.close()


def test_prefill_takes_device_resident_embeddings():
    """Visual embedding rows handed over as device tensors (what a vision encoder leaves behind) give the same cache
    as host arrays uploaded chunk by chunk, also when the prefill runs in several passes."""
    import torch
    desc, seed = SMALL_BF16, 31
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 150, 3, 40, 0.0), SequenceSpec(1, 33, 2, 25, 0.0)]
    rng = np.random.default_rng(6)
    drafts = [rng.integers(0, desc.vocab, size=sp.draft_len).astype(np.int32) for sp in specs]
    outs = []
    for on_device, chunk in ((False, None), (True, None), (True, 64)):
        eng = make_engine(desc, weights, specs, max_total_q=256, max_dump=128)
        toks, embs, pend = [], [], []
        for sp in specs:
            _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
            toks.append(tok), pend.append(pending)
            embs.append(torch.from_numpy(emb).to("cuda:0") if on_device else emb)
        eng.prefill([0, 1], toks, embs, chunk=chunk)
        blocks = [np.concatenate([[p], d]).astype(np.int32) for p, d in zip(pend, drafts)]
        outs.append(_one_round(eng, [0, 1], blocks))
        eng.close()
    for other in outs[1:]:
        np.testing.assert_array_equal(outs[0][0], other[0])
        np.testing.assert_array_equal(outs[0][1], other[1])


def test_greedy_decode_matches_oracle_fp32():
    """Blocks of length 1 (k = 0) are plain decode steps; the GPU greedy loop reproduces the oracle's
    token-by-token output.  The fp32 path's logits are within 1e-4 of the oracle's, so the comparison runs
    over all steps whose oracle margin exceeds 1e-3 (seed 9: every step, smallest margin 1.5e-3)."""
    desc, seed = SMALL_FP32, 9
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 20, 4, 40, 0.0), SequenceSpec(1, 3, 9, 40, 0.0)]
    targets = oracle_targets(desc, weights, seed, specs)
    eng = make_engine(desc, weights, specs)
    pend = _gpu_prefill(eng, desc, seed, specs)
    got = eng.greedy_decode([0, 1], pend, 40)
    for s, (g, margins) in enumerate(targets):
        ok = margins > 1e-3
        upto = int(np.argmin(ok)) if not ok.all() else len(g)
        np.testing.assert_array_equal(got[s][:upto], g[:upto])
        assert upto == 40
    eng.close()


def _one_round(eng, slots, blocks, mode="region", dump=True):
    T = sum(len(b) for b in blocks)
    out = eng.verify(slots, blocks, mode, dump_rows=np.arange(T) if dump else None)
    a, b, st = eng.read_acceptance(len(slots))
    return out.argmax.cpu().numpy().copy(), out.logits.cpu().numpy().copy() if dump else None, a, b, st


@pytest.mark.parametrize("desc", [SMALL_FP32, SMALL_BF16], ids=["fp32", "bf16"])
def test_metamorphic_paging_batching_rollback(desc):
    """Properties that hold at any size: results do not depend on which physical blocks hold the cache, on
    the batch a sequence is verified in, or on garbage in freed/rejected slots; verify -> rollback -> verify
    is idempotent; a pure rollback returns every speculative block."""
    seed = 31
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 37, 3, 50, 0.0), SequenceSpec(1, 16, 1, 81, 0.0), SequenceSpec(2, 70, 2, 20, 0.0)]
    rng = np.random.default_rng(3)
    drafts = [rng.integers(0, desc.vocab, size=sp.draft_len).astype(np.int32) for sp in specs]
    total_q = sum(len(d) + 1 for d in drafts)

    def fresh(perm_seed=None):
        eng = make_engine(desc, weights, specs, max_total_q=max(total_q, 80), max_dump=total_q, n_blocks=64)
        if perm_seed is not None:
            perm = np.random.default_rng(perm_seed).permutation(eng.n_blocks).astype(np.int32)
            eng.free_list.copy_(torch.from_numpy(perm))
        pend = _gpu_prefill(eng, desc, seed, specs)
        return eng, [np.concatenate([[p], d]).astype(np.int32) for p, d in zip(pend, drafts)]

    eng, blocks = fresh()
    free0 = int(eng.free_count.item())
    ref = _one_round(eng, [0, 1, 2], blocks)
    assert ref[4] == 0
    # (1) rollback returns all speculative blocks, and re-verification is bitwise identical
    eng.override_acceptance(np.array([-1, -1, -1]), np.array([0, 0, 0]))
    eng.commit()
    torch.cuda.synchronize()
    assert int(eng.free_count.item()) == free0
    # (2) poison everything that is not committed context: free blocks and the tail of each last block
    bt = eng.block_table.cpu().numpy()
    sl = eng.seq_len.cpu().numpy()
    owned = set(int(b) for b in bt.ravel() if b >= 0)
    poison = float("nan") if desc.dtype == "fp32" else 0x7FC0     # bf16 NaN bit pattern held in the int16 view
    v_slot = lambda t: ((t >> 2) & 1) * 8 + (t >> 3) * 4 + (t & 3)      # token order inside a transposed V page
    for pool, is_v in ((eng.k_pool, False), (eng.v_pool, True)):
        p = pool.view(desc.n_layers, eng.n_blocks, desc.n_kv_heads, 64, 16) if is_v else \
            pool.view(desc.n_layers, eng.n_blocks, desc.n_kv_heads, 16, 64)
        for b in range(eng.n_blocks):
            if b not in owned:
                p[:, b] = poison
        for s in range(3):
            for tok in range(sl[s] % 16, 16 if sl[s] % 16 else 0):
                if is_v:
                    p[:, int(bt[s, sl[s] // 16]), :, :, v_slot(tok)] = poison
                else:
                    p[:, int(bt[s, sl[s] // 16]), :, tok, :] = poison
    again = _one_round(eng, [0, 1, 2], blocks)
    np.testing.assert_array_equal(again[0], ref[0])
    np.testing.assert_array_equal(again[1], ref[1])
    assert not np.isnan(again[1]).any()
    eng.close()
    # (3) another physical block assignment gives bitwise identical results
    eng2, blocks2 = fresh(perm_seed=9)
    other = _one_round(eng2, [0, 1, 2], blocks2)
    np.testing.assert_array_equal(other[0], ref[0])
    np.testing.assert_array_equal(other[1], ref[1])
    eng2.override_acceptance(np.array([-1, -1, -1]), np.array([0, 0, 0]))
    eng2.commit()
    # (4) a sequence verified alone, or in another batch order, gives the same rows
    cu = np.concatenate([[0], np.cumsum([len(b) for b in blocks])])
    alone = _one_round(eng2, [1], [blocks2[1]])
    np.testing.assert_array_equal(alone[0], ref[0][cu[1]:cu[2]])
    np.testing.assert_allclose(alone[1], ref[1][cu[1]:cu[2]], rtol=0, atol=0)
    eng2.override_acceptance(np.array([-1]), np.array([0]))
    eng2.commit()
    swapped = _one_round(eng2, [2, 0], [blocks2[2], blocks2[0]])
    np.testing.assert_array_equal(swapped[0], np.concatenate([ref[0][cu[2]:cu[3]], ref[0][cu[0]:cu[1]]]))
    np.testing.assert_array_equal(swapped[2], [ref[2][2], ref[2][0]])
    eng2.close()


def test_device_side_error_flags():
    """Pool exhaustion and block-table overflow are reported in the status word and never fault."""
    desc, seed = SMALL_FP32, 2
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 30, 2, 40, 0.0)]
    from paper_2602_12957_amd.runtime import Engine
    import paper_2602_12957_amd.binding as B
    eng = Engine(desc, weights, n_blocks=3, n_slots=1, max_blocks_per_seq=8, max_total_q=64)
    _, _, tok, emb, pending = prefix_rows(desc, seed, specs[0])
    eng.prefill([0], [tok], [emb])                      # 31 rows -> 2 blocks, 1 left
    blk = np.concatenate([[pending], np.zeros(40, np.int32)]).astype(np.int32)   # needs 3 more blocks
    eng.verify([0], [blk])
    _, _, status = eng.read_acceptance(1)
    assert status & B.HSD_STATUS_POOL_EXHAUSTED
    eng.close()
    eng = Engine(desc, weights, n_blocks=32, n_slots=1, max_blocks_per_seq=3, max_total_q=64)
    eng.prefill([0], [tok], [emb])
    eng.verify([0], [blk])                              # 31 + 41 rows need 5 table entries, only 3 exist
    _, _, status = eng.read_acceptance(1)
    assert status & B.HSD_STATUS_TABLE_OVERFLOW
    eng.close()


def test_tile_configurations_agree_bitwise():
    """Every GEMM call site picks its tile shape from the row count.  The choice must never change a result bit
    (each output element sums its K slices in one fixed order, and the folded RMSNorm adds a row's 64-column pieces
    in one fixed order), or a row's result would depend on the batch it was computed in."""
    desc, seed = SMALL_BF16, 13
    weights = W.make_weights(desc, seed)
    specs = [SequenceSpec(0, 37, 3, 150, 0.0), SequenceSpec(1, 16, 1, 81, 0.0)]
    rng = np.random.default_rng(4)
    drafts = [rng.integers(0, desc.vocab, size=sp.draft_len).astype(np.int32) for sp in specs]
    results = []
    for debug in (None, {"gemm_cfg": (5, 2, 8, 8, 8)}, {"gemm_cfg": (7, 9, 7, 9, 0)}, {"gemm_cfg": (0, 0, 0, 6, 1)},
                  {"gemm_cfg": (10, 10, 10, 10, 0)}, {"gemm_cfg": (11, 11, 11, 11, 0)},
                  {"gemm_cfg": (12, 12, 12, 12, 0)}, {"gemm_cfg": (13, 13, 13, 13, 0)}):
        eng = make_engine(desc, weights, specs, max_total_q=256, max_dump=256, debug=debug)
        pend = _gpu_prefill(eng, desc, seed, specs)
        blocks = [np.concatenate([[p], d]).astype(np.int32) for p, d in zip(pend, drafts)]
        results.append(_one_round(eng, [0, 1], blocks))
        eng.close()
    for other in results[1:]:
        np.testing.assert_array_equal(results[0][0], other[0])
        np.testing.assert_array_equal(results[0][1], other[1])
