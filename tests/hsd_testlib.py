"""Shared helpers of the GPU parity tests: build the same seeded workload for the oracle and the HIP path.
The oracle is always taken in its plain form (fp64, nothing rounded), whatever the storage type of the model."""
from __future__ import annotations

import numpy as np

import oracle as O
import workloads as W

MARGIN_GATE = 1e-2   # acceptance decisions are compared only where the oracle's top-1/top-2 margin exceeds this


def blocks_needed(specs, extra=4, uniform_len=False):
    k_max = max(s.draft_len for s in specs)
    return sum((s.n_visual + s.n_prompt + (k_max if uniform_len else s.draft_len) + 1 + 15) // 16 + 1 for s in specs) + extra


def make_engine(desc, weights, specs, max_total_q=None, max_dump=0, n_blocks=None, attn_key_chunk=None, debug=None):
    """Engine sized for the given sequences.  The pool and block tables leave room for every sequence to grow by
    the LONGEST draft length (Engine.greedy_decode advances all sequences in lock step)."""
    from paper_2602_12957_amd.runtime import Engine
    n = len(specs)
    k_max = max(s.draft_len for s in specs)
    maxb = max((s.n_visual + s.n_prompt + k_max + 1 + 15) // 16 + 1 for s in specs)
    n_blocks = n_blocks or blocks_needed(specs, uniform_len=True)
    if max_total_q is None:
        max_total_q = max(sum(s.draft_len + 1 for s in specs), max(s.n_visual + s.n_prompt for s in specs))
    return Engine(desc, weights, n_blocks or blocks_needed(specs), n, maxb, max_total_q, max_dump,
                  attn_key_chunk=attn_key_chunk or 0, debug=debug)


def prefix_rows(desc, seed, spec):
    """(tokens with -1 for visual rows, embeds, pending token) of a sequence's prefix, pending excluded."""
    vis, prompt = W.make_prefix(desc, seed, spec.seq_id, spec.n_visual, spec.n_prompt)
    if spec.n_prompt == 0:
        tok = np.full(spec.n_visual, -1, dtype=np.int32)
        emb = vis
        pending = 0
    else:
        tok = np.concatenate([np.full(spec.n_visual, -1, dtype=np.int32), prompt[:-1]]).astype(np.int32)
        emb = np.concatenate([vis, np.zeros((spec.n_prompt - 1, desc.d_model), np.float32)], axis=0)
        pending = int(prompt[-1])
    return vis, prompt, tok, emb, pending


def oracle_targets(desc, weights, seed, specs, dtype=np.float64):
    """Oracle prefill + greedy decode of every sequence: the 'target greedy output' drafts are derived from."""
    out = []
    for sp in specs:
        vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
        cache, pending = O.prefill(desc, weights, vis, prompt, dtype)
        g, margins = O.greedy_decode(desc, weights, cache, pending, sp.draft_len, dtype, return_margins=True)
        out.append((g, margins))
    return out


def gated_compare_argmax(gpu_argmax, ora_argmax, ora_margin):
    ok = ora_margin > MARGIN_GATE
    bad = np.nonzero(ok & (gpu_argmax != ora_argmax))[0]
    return bad, int(ok.sum())
