"""Device-memory plumbing around the C-ABI library.

`Engine` allocates every device buffer through torch (weights, paged KV pools, per-sequence state,
workspace, batch staging), marshals arguments into the structs of include/hsd.h and calls the
library on torch's current stream.  It performs no arithmetic of the method itself: the decoder
forward, arg-max, acceptance and KV maintenance all run inside libhsd.so.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _pack_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (round to nearest even), as int16 for transport."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16).view(np.int16)


def _ptr(t: Optional[torch.Tensor]):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def pack_prefix_tree(pending: int, candidates: Sequence[Sequence[int]]):
    """Host-side batching of candidate continuations into one packed prefix tree (depth-first pre-order; row 0 is
    the root and carries the pending token; children keep the order in which their tokens first appear).
    Returns (tokens, tree_end, tree_depth) int32 arrays as the C ABI expects them."""
    nodes = [{}]                   # per trie node: token -> child node
    toks, depth_of = [int(pending)], [0]
    for cand in candidates:
        v = 0
        for t in cand:
            t = int(t)
            nxt = nodes[v].get(t)
            if nxt is None:
                nxt = len(nodes)
                nodes[v][t] = nxt
                nodes.append({})
                toks.append(t)
                depth_of.append(depth_of[v] + 1)
            v = nxt
    tokens, end, depth = [], [], []

    def emit(v):                   # pre-order; recursion depth = longest candidate
        i = len(tokens)
        tokens.append(toks[v]), depth.append(depth_of[v]), end.append(0)
        for c in nodes[v].values():
            emit(c)
        end[i] = len(tokens)

    import sys
    limit = sys.getrecursionlimit()
    need = max((len(c) for c in candidates), default=0) + 50
    if need > limit:
        sys.setrecursionlimit(need)
    try:
        emit(0)
    finally:
        sys.setrecursionlimit(limit)
    return (np.asarray(tokens, dtype=np.int32), np.asarray(end, dtype=np.int32), np.asarray(depth, dtype=np.int32))


@dataclass
class VerifyOutput:
    n_seq: int
    total_q: int
    cu_q: np.ndarray          # host copy [n_seq+1]
    argmax: torch.Tensor      # device int32 [total_q]
    margin: torch.Tensor      # device fp32 [total_q]
    accept_len: torch.Tensor  # device int32 [n_seq]
    bonus: torch.Tensor       # device int32 [n_seq]
    logits: Optional[torch.Tensor] = None  # device fp32 [n_dump, vocab]
    gap: Optional[torch.Tensor] = None     # device fp32 [total_q]: row's own token under its parent row, minus that
                                           #   row's maximum logit (relaxed acceptance only)
    stop_row: Optional[torch.Tensor] = None  # device int32 [n_seq]: local row of the stop node (tree blocks only)


class Engine:
    def __init__(self, desc, weights: dict, n_blocks: int, n_slots: int, max_blocks_per_seq: int,
                 max_total_q: int, max_dump: int = 0, device: str = "cuda:0", attn_key_chunk: int = 0,
                 debug: Optional[dict] = None):
        """debug: {"sync_layers" | "force_simple": int, "gemm_cfg": (qkv, o, gate_up, down, lm_head)} ->
        hsd_debug_set (experiments and cross-checks only)."""
        if not torch.cuda.is_available():
            raise RuntimeError("the HSD verification path needs a GPU (MI355X); there is no CPU fallback")
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.bf16 = desc.dtype == "bf16"
        self.cdesc = B.hsd_model_desc(desc.n_layers, desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim,
                                      desc.d_ffn, desc.vocab, B.HSD_BF16 if self.bf16 else B.HSD_FP32,
                                      desc.kv_block_tokens, desc.rms_eps, desc.rope_theta, 0)
        self.cdesc.attn_key_chunk = int(attn_key_chunk or 0)    # attention key split (hsd_model_desc.attn_key_chunk)
        code = B.hsd_validate_model(self.cdesc)
        B.check("hsd_validate_model", code)
        self.desc = desc
        self.n_blocks, self.n_slots, self.maxb = n_blocks, n_slots, max_blocks_per_seq
        self.max_total_q, self.max_dump = max_total_q, max_dump

        # ---- weights
        self._keep: List[torch.Tensor] = []
        L = desc.n_layers
        cw = B.hsd_weights()
        cw.tok_embed = self._up_mat(weights["tok_embed"])
        cw.lm_head = self._up_mat(weights["lm_head"])
        cw.final_norm = self._up_f32(weights["final_norm"])
        arrays = {}
        for name, is_mat in (("attn_norm", False), ("wqkv", True), ("wo", True), ("ffn_norm", False),
                             ("w_gate_up", True), ("w_down", True)):
            arr = (C.c_void_p * L)()
            for l in range(L):
                a = weights["layers"][l][name]
                arr[l] = self._up_mat(a) if is_mat else self._up_f32(a)
            arrays[name] = arr
            setattr(cw, name, C.cast(arr, C.POINTER(C.c_void_p)))
        self._cw, self._arrays = cw, arrays
        self.ctx = B.hsd_create(self.cdesc, cw)
        for name, val in (debug or {}).items():
            if name == "gemm_cfg":
                for site, v in enumerate(val):
                    B.hsd_debug_set(self.ctx, B.HSD_DEBUG_GEMM_CFG_QKV + site, int(v))
            else:
                B.hsd_debug_set(self.ctx, getattr(B, "HSD_DEBUG_" + name.upper()), int(val))

        # ---- paged KV pools + per-sequence state
        es = torch.int16 if self.bf16 else torch.float32
        pool_elems = L * n_blocks * desc.n_kv_heads * B.HSD_KV_BLOCK_TOKENS * B.HSD_HEAD_DIM
        self.k_pool = torch.zeros(pool_elems, dtype=es, device=self.dev)
        self.v_pool = torch.zeros(pool_elems, dtype=es, device=self.dev)
        # all KV bookkeeping lives in one int32 buffer so that a snapshot/restore is a single device copy
        # (the outputs the host reads back every round -- status, alpha, bonus -- sit together at its end: one copy)
        n_state = n_blocks + 1 + n_slots + n_slots * max_blocks_per_seq + 1 + 2 * n_slots
        self._state = torch.zeros(n_state, dtype=torch.int32, device=self.dev)
        o = 0
        self.free_list = self._state[o:o + n_blocks]; o += n_blocks
        self.free_count = self._state[o:o + 1]; o += 1
        self.seq_len = self._state[o:o + n_slots]; o += n_slots
        self.block_table = self._state[o:o + n_slots * max_blocks_per_seq].view(n_slots, max_blocks_per_seq)
        o += n_slots * max_blocks_per_seq
        self.status = self._state[o:o + 1]
        self.accept_len = self._state[o + 1:o + 1 + n_slots]
        self.bonus = self._state[o + 1 + n_slots:o + 1 + 2 * n_slots]
        self._readback = self._state[o:o + 1 + 2 * n_slots]
        self._snapshot = torch.zeros_like(self._state)
        self.cpool = B.hsd_kv_pool(_ptr(self.k_pool), _ptr(self.v_pool), n_blocks, _ptr(self.free_list),
                                   _ptr(self.free_count))

        # ---- workspace and batch staging
        self.ws_bytes = B.hsd_workspace_bytes(self.cdesc, max_total_q, n_slots)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        n_meta = (n_slots + 1) + n_slots + 3 * max_total_q + max(max_dump, 1)
        self._h_meta = torch.empty(n_meta, dtype=torch.int32).pin_memory()
        self._d_meta = torch.empty(n_meta, dtype=torch.int32, device=self.dev)
        self.argmax = torch.zeros(max_total_q, dtype=torch.int32, device=self.dev)
        self.margin = torch.zeros(max_total_q, dtype=torch.float32, device=self.dev)
        self.gap = torch.zeros(max_total_q, dtype=torch.float32, device=self.dev)
        self.stop_row = torch.zeros(n_slots, dtype=torch.int32, device=self.dev)
        self.pending = torch.zeros(n_slots, dtype=torch.int32, device=self.dev)
        self._h_out = torch.empty(2 * n_slots + 1, dtype=torch.int32).pin_memory()
        self.embeds = None
        self.logits_dump = (torch.zeros((max_dump, desc.vocab), dtype=torch.float32, device=self.dev)
                            if max_dump > 0 else None)
        self._batch: Optional[B.hsd_batch] = None
        self._meta_event = None
        self.reset()

    # ------------------------------------------------------------------ uploads
    def _up_mat(self, a: np.ndarray):
        t = torch.from_numpy(_pack_bf16(a) if self.bf16 else np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)
        self._keep.append(t)
        return t.data_ptr()

    def _up_f32(self, a: np.ndarray):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)
        self._keep.append(t)
        return t.data_ptr()

    @property
    def stream(self):
        return C.c_void_p(torch.cuda.current_stream(self.dev).cuda_stream)

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize(self.dev)
            B.hsd_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ state
    def reset(self):
        self.seq_len.zero_()
        self.block_table.fill_(-1)
        self.status.zero_()
        B.hsd_kv_pool_init(self.stream, self.cpool)

    def snapshot(self):
        """Remembers the KV bookkeeping (free stack, lengths, block tables); cached K/V data is not copied."""
        self._snapshot.copy_(self._state)

    def restore(self):
        """Returns the bookkeeping to the last snapshot (one small device copy on the current stream)."""
        self._state.copy_(self._snapshot)

    def profile(self, which: int, max_launches: int):
        B.hsd_profile_enable(self.ctx, which, max_launches)

    def profile_read(self):
        return B.hsd_profile_read(self.ctx)

    def _make_batch(self, slots: Sequence[int], blocks: Sequence[np.ndarray], dump_rows=None,
                    with_outputs: bool = True, embeds: Optional[torch.Tensor] = None,
                    log_tau: float = 0.0, trees=None) -> B.hsd_batch:
        n = len(slots)
        lens = [len(b) for b in blocks]
        total = int(sum(lens))
        if n < 1 or n > self.n_slots or total > self.max_total_q or min(lens) < 1:
            raise ValueError(f"bad batch: n_seq={n}, total_q={total}, min q_len={min(lens) if lens else 0}")
        nd = 0 if dump_rows is None else len(dump_rows)
        if nd > self.max_dump:
            raise ValueError("too many dump rows")
        if self._meta_event is not None:
            self._meta_event.synchronize()       # the previous upload has left the pinned staging buffer
        h = self._h_meta.numpy()
        o_cu, o_slot, o_tok, o_dump = 0, n + 1, 2 * n + 1, 2 * n + 1 + total
        cu = np.zeros(n + 1, dtype=np.int32)
        np.cumsum(lens, out=cu[1:])
        h[o_cu:o_cu + n + 1] = cu
        h[o_slot:o_slot + n] = np.asarray(slots, dtype=np.int32)
        h[o_tok:o_tok + total] = np.concatenate([np.asarray(b, dtype=np.int32) for b in blocks])
        if nd:
            h[o_dump:o_dump + nd] = np.asarray(dump_rows, dtype=np.int32)
        used = o_dump + nd
        o_end = o_dep = None
        if trees is not None:      # per sequence (tree_end, tree_depth) of its packed prefix tree
            o_end, o_dep = used, used + total
            h[o_end:o_end + total] = np.concatenate([np.asarray(t[0], dtype=np.int32) for t in trees])
            h[o_dep:o_dep + total] = np.concatenate([np.asarray(t[1], dtype=np.int32) for t in trees])
            used = o_dep + total
        self._d_meta[:used].copy_(self._h_meta[:used], non_blocking=True)
        self._meta_event = torch.cuda.Event()
        self._meta_event.record(torch.cuda.current_stream(self.dev))
        base = self._d_meta.data_ptr()
        b = B.hsd_batch()
        b.n_seq, b.total_q, b.max_blocks_per_seq, b.n_slots = n, total, self.maxb, self.n_slots
        b.cu_q = base + 4 * o_cu
        b.seq_slot = base + 4 * o_slot
        b.tokens = base + 4 * o_tok
        b.embeds = _ptr(embeds)
        b.seq_len, b.block_table = _ptr(self.seq_len), _ptr(self.block_table)
        b.status = _ptr(self.status)
        if with_outputs:
            b.argmax, b.top2_margin = _ptr(self.argmax), _ptr(self.margin)
            b.accept_len, b.bonus = _ptr(self.accept_len), _ptr(self.bonus)
            b.log_tau = float(log_tau)
            if log_tau < 0:
                b.draft_gap = _ptr(self.gap)
            if trees is not None:
                b.tree_end, b.tree_depth = base + 4 * o_end, base + 4 * o_dep
                b.stop_row = _ptr(self.stop_row)
        if nd:
            b.logits_dump, b.dump_rows, b.n_dump = _ptr(self.logits_dump), base + 4 * o_dump, nd
        self._cu = cu
        return b

    # ------------------------------------------------------------------ library calls
    def prefill(self, slots: Sequence[int], tokens: Sequence[np.ndarray], embeds: Optional[Sequence] = None,
                chunk: Optional[int] = None):
        """Appends rows to the sequences' caches.  tokens[i][r] < 0 takes row r of embeds[i] (fp32 [n, d]): a numpy
        array (uploaded chunk by chunk) or a tensor already on the device (the output of a vision encoder)."""
        chunk = chunk or self.max_total_q
        n_max = max(len(t) for t in tokens)
        per = max(1, chunk // len(slots))
        for c0 in range(0, n_max, per):
            sl, tk, src = [], [], []
            for i, s in enumerate(slots):
                t = np.asarray(tokens[i][c0:c0 + per], dtype=np.int32)
                if len(t) == 0:
                    continue
                sl.append(s)
                tk.append(t)
                src.append(embeds[i] if embeds is not None else None)
            dev_emb = None
            if any((t < 0).any() for t in tk):
                em = []
                for t, e in zip(tk, src):
                    if e is None:
                        em.append(torch.zeros((len(t), self.desc.d_model), dtype=torch.float32, device=self.dev))
                    elif isinstance(e, torch.Tensor):
                        em.append(e[c0:c0 + per].to(device=self.dev, dtype=torch.float32))
                    else:
                        em.append(torch.from_numpy(np.ascontiguousarray(e[c0:c0 + per], dtype=np.float32)).to(self.dev))
                dev_emb = torch.cat(em, dim=0).contiguous()
            b = self._make_batch(sl, tk, with_outputs=False, embeds=dev_emb)
            B.hsd_prefill(self.ctx, self.stream, self.cpool, b, _ptr(self.ws), self.ws_bytes)
            if dev_emb is not None:
                torch.cuda.current_stream(self.dev).synchronize()   # dev_emb must outlive the pass

    def verify(self, slots: Sequence[int], blocks: Sequence[np.ndarray], mode: str = "region",
               dump_rows=None, log_tau: float = 0.0, trees=None, noalloc: bool = False) -> VerifyOutput:
        """One verification pass; blocks[i] = [pending token, d_1..d_k] of sequence slots[i].  Asynchronous.
        log_tau = 0 is the exact-match rule; log_tau < 0 the relaxed acceptance test with threshold tau.
        With trees[i] = (tree_end, tree_depth), blocks[i] holds the tokens of a packed prefix tree
        (see pack_prefix_tree) instead of a chain."""
        b = self._make_batch(slots, blocks, dump_rows, log_tau=log_tau, trees=trees)
        if noalloc:       # the library's own fixed scratch array instead of this engine's workspace
            B.hsd_verify_region_batch_noalloc(self.ctx, self.stream, self.cpool, b)
        else:
            fn = B.hsd_verify_region_batch if mode == "region" else B.hsd_verify_page
            fn(self.ctx, self.stream, self.cpool, b, _ptr(self.ws), self.ws_bytes)
        self._batch = b
        n, T = b.n_seq, b.total_q
        return VerifyOutput(n, T, self._cu.copy(), self.argmax[:T], self.margin[:T], self.accept_len[:n],
                            self.bonus[:n], self.logits_dump[:b.n_dump] if b.n_dump else None,
                            self.gap[:T] if log_tau < 0 else None, self.stop_row[:n] if trees is not None else None)

    def prepare(self, slots: Sequence[int], blocks: Sequence[np.ndarray], log_tau: float = 0.0) -> B.hsd_batch:
        """Uploads a batch description once; verify_prepared/commit can then be replayed on it."""
        b = self._make_batch(slots, blocks, log_tau=log_tau)
        self._batch = b
        return b

    def verify_prepared(self, b: B.hsd_batch, mode: str = "region"):
        fn = B.hsd_verify_region_batch if mode == "region" else B.hsd_verify_page
        fn(self.ctx, self.stream, self.cpool, b, _ptr(self.ws), self.ws_bytes)
        self._batch = b

    def override_acceptance(self, accept_len: np.ndarray, bonus: np.ndarray, stop_row: Optional[np.ndarray] = None):
        """Test hook: replaces the device-side alpha/bonus (and, for tree blocks, the stop node) of the last verify
        before commit."""
        n = len(accept_len)
        self.accept_len[:n].copy_(torch.from_numpy(np.asarray(accept_len, dtype=np.int32)))
        self.bonus[:n].copy_(torch.from_numpy(np.asarray(bonus, dtype=np.int32)))
        if stop_row is not None:
            self.stop_row[:n].copy_(torch.from_numpy(np.asarray(stop_row, dtype=np.int32)))

    def commit(self, pending_out: Optional[torch.Tensor] = None):
        """Commit/rollback for the batch of the last verify (alpha < 0 entries roll back)."""
        B.hsd_kv_commit_rollback(self.ctx, self.stream, self.cpool, self._batch,
                                 _ptr(pending_out if pending_out is not None else self.pending))

    def read_acceptance(self, n: int):
        """Small device-to-host readback of (alpha, bonus, status); synchronises the stream."""
        self._h_out.copy_(self._readback, non_blocking=True)
        torch.cuda.current_stream(self.dev).synchronize()
        h = self._h_out.numpy()
        return h[1:1 + n].copy(), h[1 + self.n_slots:1 + self.n_slots + n].copy(), int(h[0])

    def greedy_decode(self, slots: Sequence[int], pending: Sequence[int], n_tokens: int,
                      mode: str = "region") -> np.ndarray:
        """Plain autoregressive decoding with blocks of length 1 (no draft): each step's bonus token is
        written by the commit kernel straight into the next step's token buffer.  Returns [n_seq, n_tokens]."""
        n = len(slots)
        hist = torch.zeros((n_tokens, n), dtype=torch.int32, device=self.dev)
        b = self._make_batch(slots, [np.asarray([p], dtype=np.int32) for p in pending])
        tok_view = self._d_meta[2 * n + 1: 3 * n + 1]
        fn = B.hsd_verify_region_batch if mode == "region" else B.hsd_verify_page
        for step in range(n_tokens):
            fn(self.ctx, self.stream, self.cpool, b, _ptr(self.ws), self.ws_bytes)
            B.hsd_kv_commit_rollback(self.ctx, self.stream, self.cpool, b, _ptr(tok_view))
            hist[step].copy_(self.bonus[:n])
        torch.cuda.current_stream(self.dev).synchronize()
        status = int(self.status.item())
        if status:
            raise RuntimeError(f"greedy_decode: device status {status} (KV pool exhausted or block table too short)")
        return hist.cpu().numpy().T.copy()
