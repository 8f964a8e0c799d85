"""Plain CPU oracle of HSD's verification pass.  TEST INFRASTRUCTURE ONLY.

This file is the slow, obviously-correct definition that the HIP kernels are compared with.  It
shares no code with them and is never used by the product path.

What it computes (paper, Section 3.2 "Verification and acceptance", Eq. 8-12, in the linear-draft
case the related-work section describes: one candidate continuation per sequence, so the prefix
tree is a chain and the tree-ancestry mask is the causal mask):

  * the target decoder's next-token distribution at every draft position in one causal forward
    pass over [pending token, d_1 .. d_k] on top of the already accepted context (Eq. 8);
  * the model's own top-1 token u_hat at every position (Eq. 10);
  * exact greedy acceptance: descend while the draft token equals u_hat (Eq. 9 and Eq. 11 in the
    limit tau -> 1, where log p(u*) - log p(u_hat) >= 0 holds only for u* = u_hat); with log_tau < 0 the
    relaxed rule of Eq. 11 itself (accept while log p(u*) - log p(u_hat) >= log tau);
  * the accepted-sequence update  y <- y + accepted path + u_hat at the stop node (Eq. 12);
  * alpha = number of consecutive draft tokens accepted before the first mismatch, the quantity
    averaged by the AAL metric (Eq. 15, Section 4.2).

The decoder architecture is not fixed by the paper (it runs off-the-shelf checkpoints on the
Hugging Face Transformers stack, Section 4.3), so the oracle implements the Llama family that
stack defines: pre-norm RMSNorm, rotary embedding with rotate-half pairing, grouped-query causal
attention, SwiGLU feed-forward, untied LM head, no biases.  tests/test_oracle_pins.py pins this
forward against the Transformers implementation itself.

Precision: every function takes `dtype` (default float64).  The paper states no precision.  A decoder whose
configuration says "bf16" stores its activations in bf16 between operators; `act_dtype="bf16"` makes the
oracle round to the nearest bf16 value (ties to even) at exactly those storage points -- the normalised
hidden state fed to each projection, q/k after the rotary embedding, v, the un-normalised attention
probabilities entering the weighted sum of values, the attention output, the SwiGLU output -- while every
sum is still formed in `dtype`.  With act_dtype=None nothing is rounded.  Decisions that floating point
feeds (arg-max, acceptance) are compared with the HIP path at the HIP path's storage precision.

Pins (tests/test_oracle_pins.py, tests/test_oracle_invariants.py): Transformers' LlamaForCausalLM
logits and greedy generation; torch's scaled_dot_product_attention, rms_norm and silu; complex-number
form of the rotary embedding; pure-Python brute-force attention; the lossless invariant (verification
rounds reproduce token-by-token greedy decoding exactly); closed-form alpha from the corruption
positions; for the relaxed rule (tests/test_oracle_relaxed.py) the probability-ratio form of Eq. 11, the
tau -> 1 and tau -> 0 limits, monotonicity in tau, a closed form on near-miss drafts and the replay invariant
(every committed token passes the rule in its own context); for prefix-tree batching (tests/test_oracle_tree.py)
the worked example's tree, subtree intervals = ancestry, every node's logits against an independent chain
evaluation of its root-to-node path, reduction to the chain for one candidate, lossless tree rounds whose
compacted cache equals a token-by-token one.  No function here is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "round_bf16", "rmsnorm", "rope_rotate_half", "causal_gqa_attention", "swiglu", "KVCache", "decoder_forward",
    "argmax_lowest_index", "top2_margin", "accept_longest_prefix", "draft_gap", "accept_relaxed", "verify_block",
    "greedy_decode", "prefill", "spec_decode", "RoundRecord", "embed_tokens",
    "build_prefix_tree", "ancestry_mask", "walk_prefix_tree", "verify_tree",
    "match_candidates", "cap_candidates", "spec_decode_matching",
]


# ----------------------------------------------------------------------------------------------
# Decoder building blocks (Llama family as defined by the Transformers stack, paper Section 4.3)
# ----------------------------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bf16-representable value, ties to even (via the fp32 bit pattern); dtype of x is kept."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)).view(np.float32)
    return r.astype(np.asarray(x).dtype)


def _act_round(act_dtype):
    if act_dtype is None:
        return lambda a: a
    if act_dtype == "bf16":
        return round_bf16
    raise ValueError(f"unknown act_dtype {act_dtype!r}")


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope_rotate_half(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding with rotate-half pairing.

    x: [n, heads, hd]; positions: [n] absolute token positions.  Dimension i (< hd/2) is paired
    with dimension i + hd/2; the pair is rotated by angle pos * theta^(-2i/hd)."""
    n, _, hd = x.shape
    half = hd // 2
    inv_freq = theta ** (-np.arange(half, dtype=x.dtype) * 2.0 / hd)
    ang = positions.astype(x.dtype)[:, None] * inv_freq[None, :]          # [n, half]
    cos = np.cos(ang)[:, None, :]
    sin = np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos0: int, act_dtype=None,
                         block_mask: Optional[np.ndarray] = None) -> np.ndarray:
    """Softmax attention of a block of queries over a key/value history.

    q: [Lq, Hq, hd] queries at absolute positions q_pos0 .. q_pos0+Lq-1.
    k, v: [n_keys, Hkv, hd] keys/values at absolute positions 0 .. n_keys-1 (n_keys >= q_pos0+Lq).
    Query at position p attends to keys at positions <= p.  Query head h uses kv head
    h // (Hq // Hkv).  Scores are scaled by 1/sqrt(hd).  Returns [Lq, Hq, hd].
    With act_dtype set, the un-normalised probabilities are rounded before they weight the values and the
    normaliser is the sum of the unrounded ones.  Softmax is invariant to the reference point c in
    2^(t - c) / sum 2^(t - c)  (t = score * log2 e); for the rounded form c is the smallest integer >= max t, so
    that the stored value is the probability's own floating-point rounding whatever order the keys are visited in
    (rounding commutes with powers of two)."""
    rnd = _act_round(act_dtype)
    Lq, Hq, hd = q.shape
    n_keys, Hkv, _ = k.shape
    group = Hq // Hkv
    out = np.empty_like(q)
    key_pos = np.arange(n_keys)[None, :]
    qry_pos = (q_pos0 + np.arange(Lq))[:, None]
    allowed = key_pos <= qry_pos                                           # [Lq, n_keys]
    if block_mask is not None:
        # tree-ancestry mask (Section 3.2): every key before the block is visible, key q_pos0 + j of the block is
        # visible to query row i iff block_mask[i, j]
        allowed = np.concatenate([np.ones((Lq, q_pos0), dtype=bool), np.asarray(block_mask, dtype=bool)], axis=1)
    for h in range(Hq):
        kh = k[:, h // group, :]
        vh = v[:, h // group, :]
        s = (q[:, h, :] @ kh.T) / np.sqrt(np.asarray(hd, dtype=q.dtype))
        s = np.where(allowed, s, -np.inf)
        if act_dtype is None:
            p = np.exp(s - np.max(s, axis=-1, keepdims=True))
        else:
            t = s * np.log2(np.e)
            p = np.exp2(t - np.ceil(np.max(t, axis=-1, keepdims=True)))
        out[:, h, :] = (rnd(p) @ vh) / np.sum(p, axis=-1, keepdims=True)
    return out


def swiglu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """silu(gate) * up with silu(x) = x / (1 + exp(-x))."""
    return gate / (1.0 + np.exp(-gate)) * up


class KVCache:
    """Contiguous per-layer key/value history of ONE sequence (the oracle has no paging).

    Storage grows geometrically so that token-by-token decoding does not copy the history every step;
    `k[l]` / `v[l]` are views of the first len(self) positions."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int, dtype=np.float64):
        self._n = 0
        self._shape = (n_kv_heads, head_dim)
        self._dtype = dtype
        self._kbuf = [np.zeros((0,) + self._shape, dtype=dtype) for _ in range(n_layers)]
        self._vbuf = [np.zeros((0,) + self._shape, dtype=dtype) for _ in range(n_layers)]

    def __len__(self) -> int:
        return self._n

    def keys(self, layer: int, n: int) -> np.ndarray:
        return self._kbuf[layer][:n]

    def values(self, layer: int, n: int) -> np.ndarray:
        return self._vbuf[layer][:n]

    def write(self, layer: int, pos0: int, k: np.ndarray, v: np.ndarray) -> None:
        """Stores keys/values of positions pos0 .. pos0+len(k)-1 of one layer."""
        need = pos0 + k.shape[0]
        if need > self._kbuf[layer].shape[0]:
            cap = max(need, 2 * self._kbuf[layer].shape[0], 64)
            for buf in (self._kbuf, self._vbuf):
                grown = np.zeros((cap,) + self._shape, dtype=self._dtype)
                grown[: self._n] = buf[layer][: self._n]
                buf[layer] = grown
        self._kbuf[layer][pos0:need] = k
        self._vbuf[layer][pos0:need] = v

    def advance(self, n_new: int) -> None:
        self._n += n_new

    def compact(self, base: int, slots: Sequence[int]) -> None:
        """Moves the keys/values stored at positions `slots` (increasing, each >= its target) to the contiguous
        positions base, base+1, ...: the accepted root-to-node path of a packed tree becomes ordinary context."""
        for layer in range(len(self._kbuf)):
            for d, src in enumerate(slots):
                self._kbuf[layer][base + d] = self._kbuf[layer][src]
                self._vbuf[layer][base + d] = self._vbuf[layer][src]

    def truncate(self, n: int) -> None:
        """Rollback: forget every position >= n."""
        assert n <= self._n
        self._n = n


def _cast_weights(weights: Dict, dtype) -> Dict:
    cache = weights.setdefault("_cast", {})
    key = np.dtype(dtype).name
    if key not in cache:
        cw = {n: np.asarray(weights[n], dtype=dtype) for n in ("tok_embed", "lm_head", "final_norm")}
        cw["layers"] = [{n: np.asarray(a, dtype=dtype) for n, a in lay.items()} for lay in weights["layers"]]
        cache[key] = cw
    return cache[key]


def decoder_forward(desc, weights: Dict, x_rows: np.ndarray, cache: KVCache, dtype=np.float64,
                    want_logits: bool = True, act_dtype=None, depth: Optional[np.ndarray] = None,
                    block_mask: Optional[np.ndarray] = None) -> Optional[np.ndarray]:
    """Causal forward of the decoder over a block of new rows of one sequence.

    x_rows: [n, d_model] input embeddings of the new rows (token rows already looked up).  The rows
    sit at absolute positions len(cache) .. len(cache)+n-1.  Their keys/values are appended to
    `cache`.  Returns logits [n, vocab] (or None when want_logits is False).

    Packed prefix tree (Section 3.2): with `depth` [n] and `block_mask` [n, n] given, row i sits at position
    len(cache) + depth[i] (its position on its own root-to-node path) and sees, inside the block, exactly the rows
    j with block_mask[i, j]; its keys/values are still stored at cache slot len(cache) + i."""
    w = _cast_weights(weights, dtype)
    rnd = _act_round(act_dtype)
    x = np.asarray(x_rows, dtype=dtype).copy()
    n = x.shape[0]
    pos0 = len(cache)
    positions = pos0 + (np.arange(n) if depth is None else np.asarray(depth, dtype=np.int64))
    Hq, Hkv, hd = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    for l, lay in enumerate(w["layers"]):
        h = rnd(rmsnorm(x, lay["attn_norm"], desc.rms_eps))
        qkv = h @ lay["wqkv"].T
        q = qkv[:, : Hq * hd].reshape(n, Hq, hd)
        k = qkv[:, Hq * hd: (Hq + Hkv) * hd].reshape(n, Hkv, hd)
        v = qkv[:, (Hq + Hkv) * hd:].reshape(n, Hkv, hd)
        q = rnd(rope_rotate_half(q, positions, desc.rope_theta))
        k = rnd(rope_rotate_half(k, positions, desc.rope_theta))
        cache.write(l, pos0, k, rnd(v))
        a = rnd(causal_gqa_attention(q, cache.keys(l, pos0 + n), cache.values(l, pos0 + n), pos0, act_dtype,
                                     block_mask))
        x = x + a.reshape(n, Hq * hd) @ lay["wo"].T
        h = rnd(rmsnorm(x, lay["ffn_norm"], desc.rms_eps))
        gu = h @ lay["w_gate_up"].T
        x = x + rnd(swiglu(gu[:, : desc.d_ffn], gu[:, desc.d_ffn:])) @ lay["w_down"].T
    cache.advance(n)
    if not want_logits:
        return None
    return rnd(rmsnorm(x, w["final_norm"], desc.rms_eps)) @ w["lm_head"].T


def embed_tokens(weights: Dict, tokens: Sequence[int], dtype=np.float64) -> np.ndarray:
    return _cast_weights(weights, dtype)["tok_embed"][np.asarray(tokens, dtype=np.int64)]


# ----------------------------------------------------------------------------------------------
# Acceptance (Eq. 9-12 with one candidate per node and exact match) and AAL's alpha (Eq. 15)
# ----------------------------------------------------------------------------------------------

def argmax_lowest_index(logits: np.ndarray) -> np.ndarray:
    """u_hat per row (Eq. 10); among equal maxima the lowest token id wins."""
    return np.argmax(logits, axis=-1).astype(np.int32)


def top2_margin(logits: np.ndarray) -> np.ndarray:
    """Largest minus second-largest logit per row (used only to gate parity comparisons)."""
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def accept_longest_prefix(u_hat: np.ndarray, draft: np.ndarray) -> Tuple[int, int]:
    """Greedy walk down the chain.

    u_hat[i] is the model's top-1 after context + d_1..d_i (row 0 = after the pending token alone),
    i = 0..k.  draft = (d_1..d_k).  Node i+1 is entered iff d_{i+1} == u_hat[i].  Returns
    (alpha, bonus): alpha = number of draft tokens accepted, bonus = u_hat at the stop node."""
    k = len(draft)
    alpha = 0
    while alpha < k and int(draft[alpha]) == int(u_hat[alpha]):
        alpha += 1
    return alpha, int(u_hat[alpha])


def draft_gap(logits: np.ndarray, draft: np.ndarray) -> np.ndarray:
    """gap[i] = logit of the draft token d_{i+1} at row i minus the row's largest logit (<= 0), i = 0..k-1.

    The two log-probabilities of the relaxed acceptance test (Eq. 11) share their normaliser, so their
    difference is this difference of logits."""
    k = len(draft)
    rows = np.arange(k)
    return logits[rows, np.asarray(draft, dtype=np.int64)] - logits[:k].max(axis=1)


def accept_relaxed(logits: np.ndarray, draft: np.ndarray, log_tau: float) -> Tuple[int, int]:
    """Relaxed walk down the chain (Eq. 9-12 with a single candidate per node): the draft token d_{i+1} is the
    only candidate u* at node i; it is accepted iff log p(u*) - log p(u_hat) >= log tau.  Returns (alpha, bonus):
    the number of accepted draft tokens and the model's own top-1 token at the stop node (Eq. 12)."""
    gap = draft_gap(logits, draft)
    k = len(draft)
    alpha = 0
    while alpha < k and gap[alpha] >= log_tau:
        alpha += 1
    return alpha, int(argmax_lowest_index(logits[alpha:alpha + 1])[0])


def verify_block(desc, weights, cache: KVCache, pending: int, draft: np.ndarray, dtype=np.float64, act_dtype=None,
                 log_tau: float = 0.0):
    """One verification pass for one sequence.

    cache holds the accepted context except its last token `pending` (whose keys/values are not
    cached yet).  Feeds [pending, d_1..d_k] in one causal pass (Eq. 8), takes u_hat at every row
    (Eq. 10), walks the chain (Eq. 9, 11; log_tau = 0 is the exact-match rule, log_tau < 0 the relaxed one) and
    returns (alpha, bonus, u_hat[k+1], logits[k+1,V]).
    All k+1 rows are appended to the cache; the caller commits by truncating to
    len_before + 1 + alpha."""
    block = np.concatenate([[pending], np.asarray(draft, dtype=np.int64)]).astype(np.int64)
    logits = decoder_forward(desc, weights, embed_tokens(weights, block, dtype), cache, dtype, act_dtype=act_dtype)
    u_hat = argmax_lowest_index(logits)
    if log_tau < 0.0:    # relaxed acceptance (the paper's operating point is tau = 0.75)
        alpha, bonus = accept_relaxed(logits, draft, log_tau)
    else:                # tau -> 1: exact greedy match, ties resolved to the lowest token id
        alpha, bonus = accept_longest_prefix(u_hat, draft)
    return alpha, bonus, u_hat, logits


# ----------------------------------------------------------------------------------------------
# Prefix-tree batching (Section 3.2, Eq. 7 and the tree-ancestry mask; acceptance Eq. 9-12 over Next(s))
# ----------------------------------------------------------------------------------------------

def build_prefix_tree(pending: int, candidates: Sequence[Sequence[int]]):
    """Merges the candidate continuations into a prefix tree and linearises it in depth-first pre-order.

    Row 0 is the root (empty prefix): it carries the pending token, whose row produces the distribution the
    root's children are tested against.  Children of a node keep the order in which their tokens first appear
    in `candidates`.  Returns int arrays over the packed rows: tokens, parent (-1 for the root), depth (0 for the
    root) and end (row index one past the node's subtree, so j is an ancestor-or-self of i iff j <= i < end[j])."""
    children: List[Dict[int, int]] = [{}]          # per node: token -> node id (creation order)
    tok, par = [int(pending)], [-1]
    for c in candidates:
        v = 0
        for t in c:
            t = int(t)
            if t not in children[v]:
                children[v][t] = len(tok)
                tok.append(t)
                par.append(v)
                children.append({})
            v = children[v][t]
    order, new_id = [], {}
    stack = [0]
    while stack:                                   # pre-order, children in creation order
        v = stack.pop()
        new_id[v] = len(order)
        order.append(v)
        stack.extend(reversed(list(children[v].values())))
    n = len(order)
    tokens = np.array([tok[v] for v in order], dtype=np.int64)
    parent = np.array([-1 if par[v] < 0 else new_id[par[v]] for v in order], dtype=np.int64)
    depth = np.zeros(n, dtype=np.int64)
    end = np.arange(1, n + 1, dtype=np.int64)
    for i in range(1, n):
        depth[i] = depth[parent[i]] + 1
    for i in range(n - 1, 0, -1):                  # a node's subtree ends where its last descendant's does
        end[parent[i]] = max(end[parent[i]], end[i])
    return tokens, parent, depth, end


def ancestry_mask(parent: np.ndarray) -> np.ndarray:
    """mask[i, j] = row j is row i itself or one of its ancestors (the tree-ancestry attention mask)."""
    n = len(parent)
    mask = np.zeros((n, n), dtype=bool)
    for i in range(n):
        v = i
        while v >= 0:
            mask[i, v] = True
            v = int(parent[v])
    return mask


def walk_prefix_tree(logits: np.ndarray, tokens: np.ndarray, parent: np.ndarray, log_tau: float = 0.0):
    """Greedy traversal (Eq. 9-12).  At node s the candidate u* is the child whose token has the highest logit at
    row s (lowest row index among equals); it is entered iff logit(u*) - max logit >= log_tau (log_tau = 0: iff u*
    is the arg-max token itself, lowest id among equal maxima).  Returns (path rows excluding the root, bonus =
    arg-max token at the stop node)."""
    n = len(tokens)
    kids: List[List[int]] = [[] for _ in range(n)]
    for i in range(1, n):
        kids[int(parent[i])].append(i)
    s, path = 0, []
    while kids[s]:
        row = logits[s]
        best = max(kids[s], key=lambda c: (row[tokens[c]], -c))
        u_hat = int(argmax_lowest_index(row[None, :])[0])
        ok = (row[tokens[best]] - row.max() >= log_tau) if log_tau < 0.0 else (int(tokens[best]) == u_hat)
        if not ok:
            break
        path.append(best)
        s = best
    return path, int(argmax_lowest_index(logits[s:s + 1])[0])


def verify_tree(desc, weights, cache: KVCache, pending: int, candidates: Sequence[Sequence[int]], dtype=np.float64,
                act_dtype=None, log_tau: float = 0.0):
    """One verification pass over the prefix tree of `candidates` (all of them continuations of the accepted
    context + pending token).  Returns (accepted tokens, bonus, logits [n, V], (tokens, parent, depth, end)).
    On return the cache holds the accepted context extended by the pending token and the accepted path
    (the path's keys/values are moved to contiguous positions, everything else of the block is rolled back)."""
    tokens, parent, depth, end = build_prefix_tree(pending, candidates)
    base = len(cache)
    logits = decoder_forward(desc, weights, embed_tokens(weights, tokens, dtype), cache, dtype, act_dtype=act_dtype,
                             depth=depth, block_mask=ancestry_mask(parent))
    path, bonus = walk_prefix_tree(logits, tokens, parent, log_tau)
    cache.compact(base + 1, [base + r for r in path])
    cache.truncate(base + 1 + len(path))
    return [int(tokens[r]) for r in path], bonus, logits, (tokens, parent, depth, end)


# ----------------------------------------------------------------------------------------------
# Decoupled speculative verification driver: draft-target matching (Eq. 5-6), candidate cap, rounds
# ----------------------------------------------------------------------------------------------

def match_candidates(accepted: Sequence[int], drafts: Sequence[Sequence[int]], n: int) -> List[List[int]]:
    """Candidate continuations C (Eq. 5-6): slide the reference window w = the last n accepted tokens over every
    draft; each occurrence that is followed by at least one token contributes the suffix after it.
    While fewer than n tokens are accepted the window is the whole accepted sequence; with nothing accepted yet
    every draft is a candidate from its first token (the paper leaves the start-up unspecified).
    Duplicates are kept out (C is a set); order: by draft, then by match position."""
    accepted = [int(t) for t in accepted]
    w = accepted[-n:] if n > 0 else []
    out: List[List[int]] = []
    seen = set()
    for d in drafts:
        d = [int(t) for t in d]
        starts = [0] if not w else [j for j in range(len(d) - len(w) + 1) if d[j:j + len(w)] == w]
        for j in starts:
            suf = d[j + len(w):]
            if suf and tuple(suf) not in seen:
                seen.add(tuple(suf))
                out.append(suf)
    return out


def cap_candidates(candidates: Sequence[Sequence[int]], max_packed: int) -> List[List[int]]:
    """Cuts all candidates to one common length L, the largest for which the packed prefix tree (root included)
    has at most max_packed rows (the paper caps the packed sequence at 128 tokens but not how; cutting every
    candidate at the same depth keeps all alternatives alive).  At least one token per candidate is kept if
    max_packed allows a root and one child per distinct first token."""
    cands = [list(c) for c in candidates if len(c)]
    if not cands:
        return []

    def size(L):
        return 1 + len({tuple(c[:k]) for c in cands for k in range(1, min(L, len(c)) + 1)})

    lo, hi = 1, max(len(c) for c in cands)
    if size(hi) <= max_packed:
        lo = hi
    else:
        while lo < hi:                       # size is non-decreasing in L
            mid = (lo + hi + 1) // 2
            if size(mid) <= max_packed:
                lo = mid
            else:
                hi = mid - 1
    out, seen = [], set()
    for c in cands:
        t = tuple(c[:lo])
        if t not in seen:
            seen.add(t)
            out.append(list(t))
    return out


def spec_decode_matching(desc, weights, cache: KVCache, pending: int, drafts: Sequence[Sequence[int]],
                         n_commit: int, n_window: int = 3, max_packed: int = 128, dtype=np.float64,
                         act_dtype=None, log_tau: float = 0.0):
    """SpecDecode (Eq. 1) with a fixed draft SET and decoupled verification: every round matches the reference
    window against all drafts, packs the candidate continuations into one prefix tree and verifies it in one
    pass; a round without candidates is a plain decoding step (the tree is its root alone).
    Returns (committed tokens [n_commit], list of (tree rows, accepted) per round)."""
    committed: List[int] = []
    rounds = []
    while len(committed) < n_commit:
        cands = cap_candidates(match_candidates(committed, drafts, n_window), max_packed)
        acc, bonus, _, (tokens, _, _, _) = verify_tree(desc, weights, cache, pending, cands, dtype, act_dtype, log_tau)
        committed.extend(acc)
        committed.append(bonus)
        rounds.append((len(tokens), len(acc)))
        pending = bonus
    return np.asarray(committed[:n_commit], dtype=np.int32), rounds


def prefill(desc, weights, visual: np.ndarray, prompt: Sequence[int], dtype=np.float64, act_dtype=None):
    """Build the cache for [visual rows, prompt tokens except the last]; the last prompt token is
    returned as the pending token.  With an empty prompt the pending token is id 0 and all visual
    rows are cached."""
    cache = KVCache(desc.n_layers, desc.n_kv_heads, desc.head_dim, dtype)
    prompt = np.asarray(prompt, dtype=np.int64)
    if len(prompt) == 0:
        rows, pending = np.asarray(visual, dtype=dtype), 0
    else:
        rows = np.concatenate([np.asarray(visual, dtype=dtype), embed_tokens(weights, prompt[:-1], dtype)], axis=0)
        pending = int(prompt[-1])
    if rows.shape[0]:
        decoder_forward(desc, weights, rows, cache, dtype, want_logits=False, act_dtype=act_dtype)
    return cache, pending


def greedy_decode(desc, weights, cache: KVCache, pending: int, n_tokens: int, dtype=np.float64,
                  return_margins: bool = False, act_dtype=None):
    """Plain autoregressive decoding, one token per forward pass: the definition that verification
    must reproduce.  Returns the n_tokens generated tokens (and each step's top-1/top-2 margin)."""
    out, margins = [], []
    tok = pending
    for _ in range(n_tokens):
        logits = decoder_forward(desc, weights, embed_tokens(weights, [tok], dtype), cache, dtype, act_dtype=act_dtype)
        tok = int(argmax_lowest_index(logits)[0])
        out.append(tok)
        if return_margins:
            margins.append(float(top2_margin(logits)[0]))
    res = np.asarray(out, dtype=np.int32)
    return (res, np.asarray(margins)) if return_margins else res


@dataclass
class RoundRecord:
    offset: int            # index into the full draft of d_1 of this round
    k: int                 # draft tokens scored this round
    alpha: int
    bonus: int
    u_hat: np.ndarray      # [k+1]
    margins: np.ndarray    # [k+1] top-1/top-2 margins of the rows


def spec_decode(desc, weights, cache: KVCache, pending: int, draft: np.ndarray, n_commit: int,
                dtype=np.float64, max_block: Optional[int] = None, act_dtype=None, log_tau: float = 0.0):
    """SpecDecode (Eq. 1) for one sequence with a single fixed, index-aligned draft.

    Repeats verification passes until n_commit tokens are committed.  The draft stays fixed (it
    is produced once, Section 3.2); because the synthetic corruption only substitutes tokens, the
    draft stays aligned by index: after a round that started at draft offset o and accepted alpha
    tokens, alpha+1 tokens are committed (Eq. 12) and the next round's draft starts at
    o + alpha + 1.  Returns (committed tokens [n_commit], list of RoundRecord)."""
    draft = np.asarray(draft, dtype=np.int32)
    committed: List[int] = []
    rounds: List[RoundRecord] = []
    while len(committed) < n_commit:
        o = len(committed)
        rest = draft[o:]
        if max_block is not None:
            rest = rest[: max_block]
        base = len(cache)
        alpha, bonus, u_hat, logits = verify_block(desc, weights, cache, pending, rest, dtype, act_dtype, log_tau)
        cache.truncate(base + 1 + alpha)                      # commit accepted rows, roll back the rest
        committed.extend(int(t) for t in rest[:alpha])
        committed.append(bonus)
        rounds.append(RoundRecord(o, len(rest), alpha, bonus, u_hat, top2_margin(logits)))
        pending = bonus
    return np.asarray(committed[:n_commit], dtype=np.int32), rounds
