"""Host orchestration of decoupled speculative verification on top of the HIP verification library
(paper Section 3.2; host logic only: everything numeric runs in the library's kernels).

Per round and sequence: match the reference window (the last n accepted tokens) against the fixed draft set
(Eq. 5-6), cap and pack the candidate continuations into one prefix tree, verify all sequences' trees in one
batched pass, commit, and continue from the bonus token.  A sequence without candidates takes a plain decoding
step in the same pass (its tree is the root alone).  Stage 1 / Stage 2 of the hierarchy (Eq. 2-4) are two calls
of the same driver: regions in one batch, then the page with the regions' outputs as its draft set.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .runtime import Engine, pack_prefix_tree


def match_candidates(accepted: Sequence[int], drafts: Sequence[Sequence[int]], n: int) -> List[List[int]]:
    """Suffixes that follow an occurrence of the window (last n accepted tokens) in any draft (Eq. 5-6); while fewer
    than n tokens are accepted the window is everything accepted so far, and with nothing accepted every draft is
    a candidate from its start.  Duplicates removed; order: by draft, then by position."""
    w = [int(t) for t in accepted[-n:]] if n > 0 and len(accepted) else []
    out, seen = [], set()
    for d in drafts:
        d = [int(t) for t in d]
        if not w:
            starts = [0]
        else:
            arr = np.asarray(d, dtype=np.int64)
            hit = np.ones(max(len(d) - len(w) + 1, 0), dtype=bool)
            for k, t in enumerate(w):
                hit &= arr[k:k + len(hit)] == t
            starts = np.nonzero(hit)[0].tolist()
        for j in starts:
            suf = tuple(d[j + len(w):])
            if suf and suf not in seen:
                seen.add(suf)
                out.append(list(suf))
    return out


def cap_candidates(candidates: Sequence[Sequence[int]], max_packed: int) -> List[List[int]]:
    """Cuts every candidate at one common depth, the largest whose packed tree (root included) has at most
    max_packed rows.  The tree has one row per distinct candidate prefix, so its size at cut depth L is
    1 + sum over depths k <= L of the number of distinct length-k prefixes: one pass over the depths."""
    cands = [tuple(int(t) for t in c) for c in candidates if len(c)]
    if not cands:
        return []
    rows, depth = 1, 0
    for k in range(1, max(len(c) for c in cands) + 1):
        level = len({c[:k] for c in cands if len(c) >= k})
        if rows + level > max_packed and k > 1:
            break
        rows, depth = rows + level, k
    out, seen = [], set()
    for c in cands:
        head = c[:depth]
        if head not in seen:
            seen.add(head)
            out.append(list(head))
    return out


class SpecDecoder:
    """SpecDecode(p_theta, z, Y~) (Eq. 1) for a batch of sequences whose prefixes are already in the engine's cache."""

    def __init__(self, engine: Engine, n_window: int = 3, max_packed: int = 128, log_tau: float = 0.0,
                 mode: str = "region"):
        self.eng, self.n_window, self.max_packed, self.log_tau, self.mode = engine, n_window, max_packed, log_tau, mode

    def run(self, slots: Sequence[int], pending: Sequence[int], draft_sets: Sequence[Sequence[Sequence[int]]],
            n_tokens: Sequence[int], eos: Optional[int] = None):
        """Generates n_tokens[i] tokens (or up to `eos`) for sequence slots[i] from its draft set.
        Returns (outputs: list of int arrays, stats: dict with rounds, verified rows, accepted tokens, plain steps)."""
        n = len(slots)
        out: List[List[int]] = [[] for _ in range(n)]
        pend = [int(p) for p in pending]
        done = [False] * n
        stats = dict(rounds=0, rows=0, accepted=0, plain_steps=0, seq_rounds=0,
                     per_seq=[[] for _ in range(n)])      # per sequence: (tree rows, accepted) of each of its rounds
        while not all(done):
            active = [i for i in range(n) if not done[i]]
            blocks, trees = [], []
            for i in active:
                cands = cap_candidates(match_candidates(out[i], draft_sets[i], self.n_window), self.max_packed)
                t, e, d = pack_prefix_tree(pend[i], cands)
                blocks.append(t), trees.append((e, d))
                stats["plain_steps"] += int(len(t) == 1)
                stats["rows"] += len(t)
            o = self.eng.verify([slots[i] for i in active], blocks, self.mode, log_tau=self.log_tau, trees=trees)
            self.eng.commit()
            alpha, bonus, status = self.eng.read_acceptance(len(active))
            if status:
                raise RuntimeError(f"SpecDecoder: device status {status}")
            stop = o.stop_row.cpu().numpy()
            for j, i in enumerate(active):
                # the accepted path: walk from the stop node up through the packed tree
                e, d = trees[j]
                path, s = [], int(stop[j])
                row = 0
                for depth in range(1, int(alpha[j]) + 1):
                    c = row + 1
                    while not (c <= s < e[c]):
                        c = int(e[c])
                    path.append(int(blocks[j][c]))
                    row = c
                out[i].extend(path)
                out[i].append(int(bonus[j]))
                pend[i] = int(bonus[j])
                stats["accepted"] += int(alpha[j])
                stats["seq_rounds"] += 1
                stats["per_seq"][i].append((len(blocks[j]), int(alpha[j])))
                if len(out[i]) >= n_tokens[i] or (eos is not None and eos in path + [int(bonus[j])]):
                    done[i] = True
            stats["rounds"] += 1
        res = []
        for i in range(n):
            seq = out[i][: n_tokens[i]]
            if eos is not None and eos in seq:
                seq = seq[: seq.index(eos) + 1]
            res.append(np.asarray(seq, dtype=np.int32))
        return res, stats
