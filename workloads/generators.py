"""Seeded generators for model weights and verification workloads.

Every tensor is drawn from its own Philox stream keyed by (seed, tag), so any
tensor can be regenerated independently of the others.  Shapes, sizes and
distributions follow the five workload configurations this repository is
measured on (region-level, page-level, long-document and ragged verification;
Section 3.1 of the paper describes the two stages whose shapes they mimic).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

SEED_BASE = 20260212


@dataclass(frozen=True)
class ModelDesc:
    """Llama-style decoder dimensions (pre-norm, RMSNorm, RoPE, SwiGLU, GQA)."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"            # "bf16" or "fp32": storage type of weights / KV on the device
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0
    kv_block_tokens: int = 16

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def gemm_params(self) -> int:
        per_layer = (self.d_model * (self.q_dim + 2 * self.kv_dim) + self.q_dim * self.d_model
                     + self.d_model * 2 * self.d_ffn + self.d_ffn * self.d_model)
        return per_layer * self.n_layers + self.d_model * self.vocab


# config 0 model ("T") and configs 1-4 model ("M")
MODEL_T = ModelDesc(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                    d_ffn=1024, vocab=4096, dtype="fp32")
MODEL_M = ModelDesc(n_layers=24, d_model=1024, n_q_heads=16, n_kv_heads=4, head_dim=64,
                    d_ffn=4096, vocab=32768, dtype="bf16")


def tiny_model(n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=64, d_ffn=128,
               vocab=256, dtype="fp32") -> ModelDesc:
    return ModelDesc(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype)


def _rng(seed: int, tag: str) -> np.random.Generator:
    h = hashlib.blake2b(f"{seed}:{tag}".encode(), digest_size=16).digest()
    key = np.frombuffer(h, dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of bf16-representable fp32 values, as uint16 (for upload to the device)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _normal(seed, tag, shape, std, bf16):
    w = _rng(seed, tag).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return round_to_bf16(w) if bf16 else w


def make_weights(desc: ModelDesc, seed: int = SEED_BASE) -> Dict[str, object]:
    """All decoder weights as fp32 numpy arrays (bf16-representable when desc.dtype == 'bf16').

    Linear weights are stored [out_features, in_features] (row-major), i.e. y = x @ W.T.
    wqkv rows are [all q heads | all k heads | all v heads]; w_gate_up rows are [gate | up].
    Matrices ~ N(0, 0.02).  RMSNorm gains ~ 1 + 0.1 N(0,1), always plain fp32 (kept away from
    exactly 1 so that a forgotten gain shows up in parity tests).
    """
    bf = desc.dtype == "bf16"
    d, F, V = desc.d_model, desc.d_ffn, desc.vocab
    w: Dict[str, object] = {
        "tok_embed": _normal(seed, "tok_embed", (V, d), 0.02, bf),
        "lm_head": _normal(seed, "lm_head", (V, d), 0.02, bf),
        "final_norm": 1.0 + _normal(seed, "final_norm", (d,), 0.1, False),
        "layers": [],
    }
    for l in range(desc.n_layers):
        lay = {
            "attn_norm": 1.0 + _normal(seed, f"L{l}.attn_norm", (d,), 0.1, False),
            "wqkv": _normal(seed, f"L{l}.wqkv", (desc.q_dim + 2 * desc.kv_dim, d), 0.02, bf),
            "wo": _normal(seed, f"L{l}.wo", (d, desc.q_dim), 0.02, bf),
            "ffn_norm": 1.0 + _normal(seed, f"L{l}.ffn_norm", (d,), 0.1, False),
            "w_gate_up": _normal(seed, f"L{l}.w_gate_up", (2 * F, d), 0.02, bf),
            "w_down": _normal(seed, f"L{l}.w_down", (d, F), 0.02, bf),
        }
        w["layers"].append(lay)
    return w


def make_prefix(desc: ModelDesc, seed: int, seq_id: int, n_visual: int, n_prompt: int):
    """Visual-prefix embeddings N(0,1) [n_visual, d] and prompt tokens U[0,V) [n_prompt]."""
    emb = _normal(seed, f"seq{seq_id}.visual", (n_visual, desc.d_model), 1.0, desc.dtype == "bf16")
    prompt = _rng(seed, f"seq{seq_id}.prompt").integers(0, desc.vocab, size=n_prompt, dtype=np.int64)
    return emb, prompt.astype(np.int32)


def corrupt_draft(target: np.ndarray, p: float, vocab: int, seed: int, tag: str):
    """Replace each token, independently with probability p, by a uniform draw from [0, vocab).

    The redraw may reproduce the original token.  Returns (draft, replaced_mask)."""
    g = _rng(seed, f"corrupt.{tag}")
    target = np.asarray(target, dtype=np.int32)
    mask = g.random(target.shape[0]) < p
    repl = g.integers(0, vocab, size=target.shape[0], dtype=np.int64).astype(np.int32)
    return np.where(mask, repl, target).astype(np.int32), mask


def corrupt_draft_forced(target: np.ndarray, p: float, vocab: int, seed: int, tag: str):
    """As corrupt_draft, but a replaced token always differs from the original, so the first
    replaced position is exactly Geometric(p)."""
    g = _rng(seed, f"corruptf.{tag}")
    target = np.asarray(target, dtype=np.int32)
    mask = g.random(target.shape[0]) < p
    shift = g.integers(1, vocab, size=target.shape[0], dtype=np.int64)
    repl = ((target.astype(np.int64) + shift) % vocab).astype(np.int32)
    return np.where(mask, repl, target).astype(np.int32), mask


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    model: ModelDesc
    n_seq: int
    kind: str                 # "region" or "page"
    description: str = ""


@dataclass
class SequenceSpec:
    seq_id: int
    n_visual: int
    n_prompt: int             # prompt tokens after the visual prefix (0 => pending token id 0)
    draft_len: int
    corrupt_p: float
    forced_different: bool = False


CONFIGS: List[WorkloadConfig] = [
    WorkloadConfig("cfg0_tiny", MODEL_T, 4, "region",
                   "4 regions, 256 visual + 16 prompt, draft 32, p=0.1, fp32"),
    WorkloadConfig("cfg1_region", MODEL_M, 16, "region",
                   "16 regions, 1024 visual + 32 prompt, draft U[16,256], p=0.05"),
    WorkloadConfig("cfg2_page", MODEL_M, 1, "page",
                   "1 page, 4096 visual + 32 prompt, draft 2048, first mismatch Geometric(0.002)"),
    WorkloadConfig("cfg3_longdoc", MODEL_M, 4, "page",
                   "4 pages, 8192 visual, draft 8192, p=0.01"),
    WorkloadConfig("cfg4_ragged", MODEL_M, 64, "region",
                   "64 regions, prefix U[512,2048], draft lognormal(4.5,0.8) in [8,1024], p~U[0,0.2]"),
]


def draw_sequences(cfg_index: int, seed: int = SEED_BASE) -> List[SequenceSpec]:
    """Per-sequence shape parameters (prefix length, draft length, corruption rate) of a config."""
    g = _rng(seed, f"cfg{cfg_index}.shapes")
    if cfg_index == 0:
        return [SequenceSpec(i, 256, 16, 32, 0.1) for i in range(4)]
    if cfg_index == 1:
        ks = g.integers(16, 257, size=16)
        return [SequenceSpec(i, 1024, 32, int(ks[i]), 0.05) for i in range(16)]
    if cfg_index == 2:
        return [SequenceSpec(0, 4096, 32, 2048, 0.002, True)]
    if cfg_index == 3:
        return [SequenceSpec(i, 8192, 0, 8192, 0.01) for i in range(4)]
    if cfg_index == 4:
        S = g.integers(512, 2049, size=64)
        k = np.clip(np.rint(g.lognormal(4.5, 0.8, size=64)), 8, 1024).astype(int)
        p = g.random(64) * 0.2
        return [SequenceSpec(i, int(S[i]), 0, int(k[i]), float(p[i])) for i in range(64)]
    raise ValueError(f"unknown config {cfg_index}")
