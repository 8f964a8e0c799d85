"""Pins of the CPU oracle against things other than itself.

Each oracle function is checked against a library routine, a different mathematical formulation,
or a brute-force definition, so that a dropped term, a wrong sign or index, or a transposed operand
in the oracle fails here.  The decoder family (Llama: pre-norm RMSNorm, rotate-half RoPE, GQA,
SwiGLU, untied head) is the one defined by the Hugging Face Transformers stack the paper runs on
(Section 4.3), so the whole forward is pinned to that stack's own implementation.
"""
import math

import numpy as np
import pytest
import torch

import oracle as O
import workloads as W


# ---------------------------------------------------------------- building blocks

def test_rmsnorm_matches_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 48))
    g = 1 + 0.3 * rng.standard_normal(48)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-6), ref, rtol=1e-13, atol=1e-13)


def test_swiglu_matches_torch_silu():
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal((5, 33)) * 3, rng.standard_normal((5, 33))
    ref = (torch.nn.functional.silu(torch.from_numpy(a)) * torch.from_numpy(b)).numpy()
    np.testing.assert_allclose(O.swiglu(a, b), ref, rtol=1e-13, atol=1e-14)


def test_rope_equals_complex_rotation():
    """Rotate-half pairing (i, i+hd/2) is multiplication of z_i = x_i + j*x_{i+hd/2} by exp(j*pos*theta^(-2i/hd))."""
    rng = np.random.default_rng(2)
    n, H, hd, theta = 9, 3, 16, 10000.0
    x = rng.standard_normal((n, H, hd))
    pos = rng.integers(0, 5000, size=n)
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    freq = np.array([theta ** (-2.0 * i / hd) for i in range(hd // 2)])
    zr = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    ref = np.concatenate([zr.real, zr.imag], axis=-1)
    np.testing.assert_allclose(O.rope_rotate_half(x, pos, theta), ref, rtol=1e-12, atol=1e-12)


def test_rope_invariants():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 1, 64))
    k = rng.standard_normal((1, 1, 64))
    # position 0 is the identity; rotation preserves norms
    np.testing.assert_allclose(O.rope_rotate_half(q, np.array([0]), 1e4), q, atol=0)
    assert abs(np.linalg.norm(O.rope_rotate_half(q, np.array([123]), 1e4)) - np.linalg.norm(q)) < 1e-12
    # the score depends only on the relative position
    def score(m, n):
        return float(np.sum(O.rope_rotate_half(q, np.array([m]), 1e4) * O.rope_rotate_half(k, np.array([n]), 1e4)))
    assert abs(score(17, 5) - score(1012, 1000)) < 1e-10
    assert abs(score(17, 5) - score(5, 17)) > 1e-6       # and it is not symmetric in (m, n)


def _brute_force_attention(q, k, v, pos0):
    """Scalar loops straight from the definition of causal softmax attention with grouped heads."""
    Lq, Hq, hd = q.shape
    Hkv = k.shape[1]
    out = np.zeros_like(q)
    for i in range(Lq):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            scores = []
            for j in range(pos0 + i + 1):
                scores.append(sum(q[i, h, t] * k[j, g, t] for t in range(hd)) / math.sqrt(hd))
            m = max(scores)
            e = [math.exp(s - m) for s in scores]
            Z = sum(e)
            for t in range(hd):
                out[i, h, t] = sum(e[j] / Z * v[j, g, t] for j in range(len(e)))
    return out


@pytest.mark.parametrize("Lq,S,Hq,Hkv", [(1, 7, 2, 2), (5, 0, 4, 2), (4, 6, 4, 1), (3, 3, 3, 3)])
def test_attention_brute_force(Lq, S, Hq, Hkv):
    rng = np.random.default_rng(Lq * 100 + S)
    hd = 8
    q = rng.standard_normal((Lq, Hq, hd))
    k = rng.standard_normal((S + Lq, Hkv, hd))
    v = rng.standard_normal((S + Lq, Hkv, hd))
    np.testing.assert_allclose(O.causal_gqa_attention(q, k, v, S), _brute_force_attention(q, k, v, S),
                               rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("Lq,S,Hq,Hkv", [(33, 70, 8, 2), (1, 50, 4, 4), (40, 0, 4, 1)])
def test_attention_matches_torch_sdpa(Lq, S, Hq, Hkv):
    rng = np.random.default_rng(7)
    hd = 64
    q = rng.standard_normal((Lq, Hq, hd))
    k = rng.standard_normal((S + Lq, Hkv, hd))
    v = rng.standard_normal((S + Lq, Hkv, hd))
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    mask = torch.arange(S + Lq)[None, :] <= (S + torch.arange(Lq))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(O.causal_gqa_attention(q, k, v, S), ref, rtol=1e-11, atol=1e-12)


def test_attention_properties():
    rng = np.random.default_rng(8)
    q = rng.standard_normal((6, 2, 8))
    k = rng.standard_normal((10, 1, 8))
    v = np.broadcast_to(rng.standard_normal((1, 1, 8)), (10, 1, 8)).copy()
    # all values equal -> every output row equals that value (softmax weights sum to one)
    out = O.causal_gqa_attention(q, k, v, 4)
    np.testing.assert_allclose(out, np.broadcast_to(v[0], out.shape), atol=1e-13)
    # future keys do not matter: changing keys after the query position leaves the row unchanged
    v2 = rng.standard_normal((10, 1, 8))
    base = O.causal_gqa_attention(q, k, v2, 4)
    k3, v3 = k.copy(), v2.copy()
    k3[7:] += 5.0
    v3[7:] -= 3.0
    pert = O.causal_gqa_attention(q, k3, v3, 4)
    np.testing.assert_allclose(pert[:3], base[:3], atol=1e-13)      # rows at positions 4,5,6 see keys <= 6
    assert np.abs(pert[3:] - base[3:]).max() > 1e-3


# ---------------------------------------------------------------- whole forward vs Transformers

def _hf_model(desc, weights):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=desc.vocab, hidden_size=desc.d_model, intermediate_size=desc.d_ffn,
                      num_hidden_layers=desc.n_layers, num_attention_heads=desc.n_q_heads,
                      num_key_value_heads=desc.n_kv_heads, head_dim=desc.head_dim, rms_norm_eps=desc.rms_eps,
                      rope_theta=desc.rope_theta, attention_bias=False, mlp_bias=False,
                      tie_word_embeddings=False, max_position_embeddings=4096)
    cfg._attn_implementation = "eager"
    m = LlamaForCausalLM(cfg).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    Hq, Hkv, hd, F = desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.d_ffn
    sd = {"model.embed_tokens.weight": t(weights["tok_embed"]), "model.norm.weight": t(weights["final_norm"]),
          "lm_head.weight": t(weights["lm_head"])}
    for l, lay in enumerate(weights["layers"]):
        p = f"model.layers.{l}."
        sd[p + "self_attn.q_proj.weight"] = t(lay["wqkv"][: Hq * hd])
        sd[p + "self_attn.k_proj.weight"] = t(lay["wqkv"][Hq * hd: (Hq + Hkv) * hd])
        sd[p + "self_attn.v_proj.weight"] = t(lay["wqkv"][(Hq + Hkv) * hd:])
        sd[p + "self_attn.o_proj.weight"] = t(lay["wo"])
        sd[p + "mlp.gate_proj.weight"] = t(lay["w_gate_up"][:F])
        sd[p + "mlp.up_proj.weight"] = t(lay["w_gate_up"][F:])
        sd[p + "mlp.down_proj.weight"] = t(lay["w_down"])
        sd[p + "input_layernorm.weight"] = t(lay["attn_norm"])
        sd[p + "post_attention_layernorm.weight"] = t(lay["ffn_norm"])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return m


def _hf_logits(m, rows):
    with torch.no_grad():
        return m(inputs_embeds=torch.from_numpy(rows)[None]).logits[0].numpy()


@pytest.mark.parametrize("Hq,Hkv,hd,L", [(4, 2, 16, 2), (4, 4, 64, 1), (8, 2, 32, 3)])
def test_forward_matches_transformers_llama(Hq, Hkv, hd, L):
    desc = W.tiny_model(n_layers=L, d_model=64, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=hd, d_ffn=96, vocab=200)
    w = W.make_weights(desc, seed=11)
    vis, prompt = W.make_prefix(desc, 11, 0, 10, 6)
    draft = np.random.default_rng(5).integers(0, desc.vocab, size=9)
    rows = np.concatenate([vis.astype(np.float64), np.asarray(w["tok_embed"], np.float64)[np.concatenate([prompt, draft])]])
    ref = _hf_logits(_hf_model(desc, w), rows)
    # (a) one shot
    full = O.decoder_forward(desc, w, rows, O.KVCache(L, Hkv, hd))
    np.testing.assert_allclose(full, ref, rtol=0, atol=1e-6)   # Transformers keeps its rotary tables in fp32
    # (b) prefix cached first, then the verification block [pending, draft] on top of it:
    #     pins the cache, the absolute positions and the prefix+causal mask of the block
    cache, pending = O.prefill(desc, w, vis, prompt)
    assert len(cache) == 10 + 6 - 1 and pending == prompt[-1]
    alpha, bonus, u_hat, logits = O.verify_block(desc, w, cache, pending, draft)
    np.testing.assert_allclose(logits, ref[15:], rtol=0, atol=1e-6)
    np.testing.assert_array_equal(u_hat, ref[15:].argmax(-1))


def test_greedy_and_spec_decode_match_transformers_greedy():
    """Token-by-token greedy with Transformers as the next-token function (full recompute each step)
    equals the oracle's cached greedy decode, and equals the oracle's verification rounds."""
    desc = W.tiny_model(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=150)
    w = W.make_weights(desc, seed=21)
    vis, prompt = W.make_prefix(desc, 21, 0, 6, 5)
    m = _hf_model(desc, w)
    E = np.asarray(w["tok_embed"], np.float64)
    rows = np.concatenate([vis.astype(np.float64), E[prompt]])
    hf_tokens = []
    for _ in range(12):
        nxt = int(_hf_logits(m, rows)[-1].argmax())
        hf_tokens.append(nxt)
        rows = np.concatenate([rows, E[[nxt]]])
    cache, pending = O.prefill(desc, w, vis, prompt)
    g = O.greedy_decode(desc, w, cache, pending, 12)
    np.testing.assert_array_equal(g, hf_tokens)
    draft, _ = W.corrupt_draft_forced(g, 0.3, desc.vocab, 21, "x")
    cache, pending = O.prefill(desc, w, vis, prompt)
    out, _ = O.spec_decode(desc, w, cache, pending, draft, 12)
    np.testing.assert_array_equal(out, hf_tokens)


def test_fp32_oracle_close_to_fp64():
    desc = W.tiny_model(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=150)
    w = W.make_weights(desc, seed=3)
    vis, prompt = W.make_prefix(desc, 3, 0, 12, 4)
    rows = np.concatenate([vis, np.asarray(w["tok_embed"])[prompt]])
    a = O.decoder_forward(desc, w, rows, O.KVCache(2, 2, 16, np.float64), np.float64)
    b = O.decoder_forward(desc, w, rows, O.KVCache(2, 2, 16, np.float32), np.float32)
    assert b.dtype == np.float32
    assert np.abs(a - b).max() < 1e-5


# ---------------------------------------------------------------- acceptance (Eq. 9-12) and helpers

def test_accept_longest_prefix_brute_force():
    rng = np.random.default_rng(4)
    for _ in range(300):
        k = int(rng.integers(0, 12))
        u = rng.integers(0, 3, size=k + 1)
        d = rng.integers(0, 3, size=k)
        # definition: the largest j such that every one of the first j draft tokens equals the model's top-1
        best = max(j for j in range(k + 1) if all(d[i] == u[i] for i in range(j)))
        alpha, bonus = O.accept_longest_prefix(u, d)
        assert alpha == best and bonus == u[best]
    assert O.accept_longest_prefix(np.array([5]), np.array([], dtype=int)) == (0, 5)       # k = 0: plain decode step
    assert O.accept_longest_prefix(np.array([1, 2, 3]), np.array([1, 2])) == (2, 3)        # full acceptance: bonus from last row
    assert O.accept_longest_prefix(np.array([9, 2, 3]), np.array([1, 2])) == (0, 9)        # later matches do not count


def test_argmax_ties_and_margin():
    x = np.array([[0.0, 2.0, 2.0, 1.0], [3.0, 1.0, 2.5, -1.0]])
    np.testing.assert_array_equal(O.argmax_lowest_index(x), [1, 0])
    np.testing.assert_allclose(O.top2_margin(x), [0.0, 0.5])
    rng = np.random.default_rng(0)
    y = rng.standard_normal((20, 50))
    s = np.sort(y, axis=-1)
    np.testing.assert_allclose(O.top2_margin(y), s[:, -1] - s[:, -2])


# ---------------------------------------------------------------- bf16 storage-precision mode

def test_round_bf16_matches_torch_conversion():
    rng = np.random.default_rng(12)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, size=5000),
                        # exact ties between two bf16 neighbours (must go to the even one) and exact bf16 values
                        np.array([1.00390625, 1.01171875, -1.00390625, 3.0, 0.0, 65280.0 + 128.0, 2.0 ** -120])])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_bf16(x), ref)
    assert O.round_bf16(x).dtype == x.dtype
    assert O.round_bf16(np.array([1.00390625]))[0] == 1.0 and O.round_bf16(np.array([1.01171875]))[0] == 1.015625


def test_bf16_mode_is_the_same_forward_with_rounded_storage():
    """act_dtype=None leaves the pinned fp64 forward untouched; act_dtype='bf16' perturbs it by rounding noise only;
    attention with rounded probabilities keeps the unrounded normaliser."""
    desc = W.tiny_model(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=150, dtype="bf16")
    w = W.make_weights(desc, seed=8)
    vis, prompt = W.make_prefix(desc, 8, 0, 10, 5)
    rows = np.concatenate([vis, np.asarray(w["tok_embed"])[prompt]]).astype(np.float64)
    a = O.decoder_forward(desc, w, rows, O.KVCache(2, 2, 16))
    b = O.decoder_forward(desc, w, rows, O.KVCache(2, 2, 16), act_dtype="bf16")
    rel = np.abs(a - b).max() / np.abs(a).max()
    assert 1e-5 < rel < 5e-2
    rng = np.random.default_rng(0)
    q, k, v = rng.standard_normal((3, 2, 8)), rng.standard_normal((7, 2, 8)), rng.standard_normal((7, 2, 8))
    out = O.causal_gqa_attention(q, k, v, 4, act_dtype="bf16")
    for i in range(3):
        for h in range(2):
            t = (k[: 5 + i, h] @ q[i, h]) / np.sqrt(8) * np.log2(np.e)
            e = 2.0 ** (t - np.ceil(t.max()))
            np.testing.assert_allclose(out[i, h], (O.round_bf16(e) @ v[: 5 + i, h]) / e.sum(), rtol=1e-12)
            # the rounded probabilities do not depend on the order/grouping in which keys are visited:
            # any other integer reference point only moves the exponent
            e2 = 2.0 ** (t - np.ceil(t.max()) - 3)
            np.testing.assert_array_equal(O.round_bf16(e2) * 8, O.round_bf16(e))
