"""The lossless property on the GPU path itself, at full model size and exactly.

Speculative verification must reproduce plain token-by-token greedy decoding of the same model (the premise
of the method, Section 3.2: verification preserves autoregressive conditioning; the verifier accepts the longest
matching prefix).  Here BOTH sides are the HIP path: greedy decoding with blocks of length 1, and verification
rounds over corrupted drafts run freely (no teacher forcing).  Because every kernel computes a row's result
independently of which other rows share the launch, the two agree bit for bit, for any model depth -- a property
that holds at any size and does not involve the oracle (whose parity is tested separately).  Acceptance lengths
are also checked against the closed form given by the corruption positions.
"""
import numpy as np
import pytest
import torch

import workloads as W
from workloads.generators import SequenceSpec

from hsd_testlib import make_engine, prefix_rows

pytestmark = pytest.mark.gpu


def _lossless(desc, specs, seed, mode, attn_key_chunk=None):
    weights = W.make_weights(desc, seed)
    n = len(specs)
    eng = make_engine(desc, weights, specs, max_total_q=max(sum(s.draft_len + 1 for s in specs), 4096),
                      attn_key_chunk=attn_key_chunk)
    toks, embs, pend = [], [], []
    for sp in specs:
        _, _, tok, emb, pending = prefix_rows(desc, seed, sp)
        toks.append(tok), embs.append(emb), pend.append(pending)
    slots = list(range(n))
    eng.prefill(slots, toks, embs)
    k_max = max(sp.draft_len for sp in specs)
    target = eng.greedy_decode(slots, pend, k_max, mode)   # same entry point: the two are tiled differently
    eng.reset()
    eng.prefill(slots, toks, embs)
    drafts, masks = [], []
    for i, sp in enumerate(specs):
        d, m = W.corrupt_draft_forced(target[i][:sp.draft_len], sp.corrupt_p, desc.vocab, seed, f"ll.{sp.seq_id}")
        drafts.append(d), masks.append(np.nonzero(m)[0])
    committed = [[] for _ in range(n)]
    pending = list(pend)
    rounds = 0
    active = slots
    while active:
        blocks = [np.concatenate([[pending[i]], drafts[i][len(committed[i]):]]).astype(np.int32) for i in active]
        eng.verify(active, blocks, mode)
        eng.commit()
        alpha, bonus, status = eng.read_acceptance(len(active))
        assert status == 0
        nxt = []
        for j, i in enumerate(active):
            o = len(committed[i])
            later = masks[i][masks[i] >= o]
            expect = int(later[0] - o) if len(later) else specs[i].draft_len - o
            assert alpha[j] == expect, f"seq {i} round {rounds}: alpha {alpha[j]} != {expect}"
            committed[i].extend(drafts[i][o:o + alpha[j]].tolist())
            committed[i].append(int(bonus[j]))
            pending[i] = int(bonus[j])
            if len(committed[i]) < specs[i].draft_len:
                nxt.append(i)
        active = nxt
        rounds += 1
    for i, sp in enumerate(specs):
        np.testing.assert_array_equal(np.asarray(committed[i][:sp.draft_len]), target[i][:sp.draft_len])
    torch.cuda.synchronize()
    owned = int((eng.block_table.cpu().numpy() >= 0).sum())
    assert owned + int(eng.free_count.item()) == eng.n_blocks
    eng.close()
    return rounds


@pytest.mark.parametrize("mode", ["region", "page"])
def test_lossless_small_models(mode):
    for desc in (W.ModelDesc(2, 128, 4, 1, 64, 256, 512, "fp32"), W.ModelDesc(3, 256, 8, 2, 64, 512, 1024, "bf16")):
        specs = [SequenceSpec(0, 40, 3, 90, 0.1), SequenceSpec(1, 5, 2, 70, 0.3), SequenceSpec(2, 130, 5, 33, 0.0),
                 SequenceSpec(3, 0, 4, 150, 0.05)]
        assert _lossless(desc, specs, 11, mode) >= 2


def test_lossless_with_attention_key_split():
    """The key split cuts at absolute positions, so a row's bits still do not depend on the block it is scored in:
    verification and token-by-token decoding agree exactly with the split on (128-key chunks on a small model; the
    page-level configuration with the 1024-key chunks that suit it)."""
    specs = [SequenceSpec(0, 40, 3, 90, 0.1), SequenceSpec(1, 5, 2, 70, 0.3), SequenceSpec(2, 330, 5, 33, 0.0),
             SequenceSpec(3, 0, 4, 290, 0.05)]
    assert _lossless(W.ModelDesc(3, 256, 8, 2, 64, 512, 1024, "bf16"), specs, 12, "region", attn_key_chunk=128) >= 2
    rounds = _lossless(W.MODEL_M, W.draw_sequences(2, W.SEED_BASE), W.SEED_BASE, "page", attn_key_chunk=1024)
    print("cfg2 lossless rounds with 1024-key chunks", rounds)


def test_lossless_random_shapes():
    """Twenty-five seeded random combinations of depth, width, GQA grouping, storage type, entry point, key split and
    ragged sequences (prefixes of 0 to 700 tokens, drafts of 1 to 260, corruption 0 / 5 / 30 %): verification rounds
    reproduce token-by-token decoding exactly in every one."""
    rng = np.random.default_rng(20260214)
    for it in range(25):
        heads = [(4, 1), (4, 2), (8, 2), (4, 4), (16, 4), (8, 8)][rng.integers(0, 6)]
        dt = "bf16" if rng.random() < 0.8 else "fp32"
        desc = W.ModelDesc(int(rng.integers(1, 5)), int(rng.choice([128, 256, 512])), heads[0], heads[1], 64,
                           int(rng.choice([256, 512, 1024])), int(rng.choice([512, 1024, 2048])), dt)
        specs = []
        for i in range(int(rng.integers(1, 7))):
            nv = int(rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 130, 300, 700]))
            specs.append(SequenceSpec(i, nv, int(rng.integers(1 if nv == 0 else 0, 6)),
                                      int(rng.choice([1, 2, 31, 33, 64, 65, 150, 260])), float(rng.choice([0.0, 0.05, 0.3]))))
        mode = "page" if rng.random() < 0.4 else "region"
        chunk = int(rng.choice([0, 128, 256, 384])) if dt == "bf16" else 0
        seed = int(rng.integers(1, 10000))
        print(it, desc, [(s.n_visual, s.n_prompt, s.draft_len, s.corrupt_p) for s in specs], mode, chunk, seed, flush=True)
        _lossless(desc, specs, seed, mode, attn_key_chunk=chunk or None)


def test_lossless_through_every_row_count_regime():
    """Drafts long enough that round 1 scores more than 6 k rows (256x256 tiles on QKV and O, the down projection's K
    chunks walked inside one workgroup, row-band tile order) and the following rounds shrink through every tile
    choice down to a few rows: all of them must reproduce token-by-token decoding bit for bit, on small models with
    ragged tile tails."""
    for desc, lens in ((W.ModelDesc(3, 256, 8, 2, 64, 512, 1024, "bf16"), [1500, 1300, 1700, 999, 801]),
                       (W.ModelDesc(2, 256, 16, 4, 64, 1536, 2048, "bf16"), [3000, 3200, 67, 1])):
        specs = [SequenceSpec(i, 40 + 13 * i, 3, k, 0.02) for i, k in enumerate(lens)]
        assert _lossless(desc, specs, 17, "region") >= 20


def test_lossless_config1_model_m():
    """configs[1] shapes (16 regions, 1055 cached tokens, drafts U[16,256], 5 % corruption), 24-layer bf16 model."""
    specs = W.draw_sequences(1, W.SEED_BASE)
    rounds = _lossless(W.MODEL_M, specs, W.SEED_BASE, "region")
    print("cfg1 lossless rounds", rounds)


def test_lossless_config2_page_level():
    """configs[2] shape: one page, 4127 cached tokens, a 2048-token draft, first mismatch Geometric(0.002)."""
    specs = W.draw_sequences(2, W.SEED_BASE)
    rounds = _lossless(W.MODEL_M, specs, W.SEED_BASE, "page")
    print("cfg2 lossless rounds", rounds)


def test_lossless_config3_long_documents():
    """configs[3] shape at full size: 4 pages of 8192 cached tokens with 8192-token drafts at 1 % corruption
    (about 80 rounds, 32,772 rows in the first).  The CPU oracle needs hours per page here; this property needs
    no oracle and is exact."""
    specs = W.draw_sequences(3, W.SEED_BASE)
    rounds = _lossless(W.MODEL_M, specs, W.SEED_BASE, "page")
    print("cfg3 lossless rounds", rounds)
    assert rounds >= 40
