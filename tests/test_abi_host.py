"""Host-side tests of the C-ABI library that need no GPU: it loads, exports every declared symbol, and
rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

import paper_2602_12957_amd.binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _desc(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024, vocab=4096,
                dtype=B.HSD_FP32, kv_block_tokens=16, rms_eps=1e-6, rope_theta=10000.0, attn_key_chunk=0)
    base.update(kw)
    return B.hsd_model_desc(*[base[n] for n, _ in B.hsd_model_desc._fields_])


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "hsd.h")).read()
    declared = set(re.findall(r"\b(hsd_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_status_strings():
    assert B.hsd_status_string(0) == "ok"
    for code in range(-6, 0):
        assert B.hsd_status_string(code) not in ("ok", "unknown status")
    assert B.hsd_status_string(-99) == "unknown status"


@pytest.mark.parametrize("kw,code", [
    ({}, B.HSD_OK), ({"dtype": B.HSD_BF16}, B.HSD_OK),
    ({"head_dim": 128}, B.HSD_EINVAL), ({"kv_block_tokens": 32}, B.HSD_EINVAL), ({"dtype": 7}, B.HSD_EINVAL),
    ({"n_q_heads": 6, "n_kv_heads": 4}, B.HSD_EINVAL), ({"d_model": 200}, B.HSD_EINVAL),
    ({"vocab": 1000}, B.HSD_EINVAL), ({"n_layers": 0}, B.HSD_EINVAL), ({"rms_eps": 0.0}, B.HSD_EINVAL),
    ({"n_layers": 5000}, B.HSD_ERANGE),
    ({"attn_key_chunk": 512}, B.HSD_OK), ({"attn_key_chunk": 100}, B.HSD_EINVAL), ({"attn_key_chunk": -128}, B.HSD_EINVAL), ({"attn_key_chunk": 64}, B.HSD_EINVAL),
])
def test_validate_model(kw, code):
    assert B.hsd_validate_model(_desc(**kw)) == code


def _batch(**kw):
    fake = 0x1000  # never dereferenced by the host-side checks
    b = B.hsd_batch()
    b.n_seq, b.total_q, b.max_blocks_per_seq, b.n_slots = 4, 132, 32, 4
    for name in ("cu_q", "tokens", "seq_len", "block_table", "argmax", "accept_len", "bonus", "status"):
        setattr(b, name, fake)
    for k, v in kw.items():
        setattr(b, k, v)
    return b


def _pool(**kw):
    p = B.hsd_kv_pool(0x1000, 0x1000, 64, 0x1000, 0x1000)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_workspace_grows_with_key_split():
    """The key-split attention keeps 8 partial records of 264 bytes per (row, head); bf16 models only."""
    plain = B.hsd_workspace_bytes(_desc(dtype=B.HSD_BF16), 1000, 4)
    split = B.hsd_workspace_bytes(_desc(dtype=B.HSD_BF16, attn_key_chunk=512), 1000, 4)
    assert 8 * 1000 * 4 * 264 <= split - plain <= 8 * 1000 * 4 * 264 + 1024
    assert B.hsd_workspace_bytes(_desc(attn_key_chunk=512), 1000, 4) == B.hsd_workspace_bytes(_desc(), 1000, 4)


def test_validate_batch():
    d = _desc()
    need = B.hsd_workspace_bytes(d, 132, 4)
    assert need > 132 * 256 * 4
    assert B.hsd_validate_batch(d, _pool(), _batch(), need) == B.HSD_OK
    assert B.hsd_validate_batch(d, _pool(), _batch(), need - 1) == B.HSD_ENOSPC
    assert B.hsd_validate_batch(d, _pool(), _batch(n_seq=0), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(total_q=3), need) == B.HSD_EINVAL          # q_len >= 1 each
    assert B.hsd_validate_batch(d, _pool(), _batch(n_seq=5000, total_q=5000, n_slots=5000), 1 << 40) == B.HSD_ERANGE
    assert B.hsd_validate_batch(d, _pool(), _batch(cu_q=None), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(status=None), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(n_slots=2), need) == B.HSD_EINVAL          # identity slots need n_slots >= n_seq
    assert B.hsd_validate_batch(d, _pool(), _batch(n_slots=2, seq_slot=0x1000), need) == B.HSD_OK
    assert B.hsd_validate_batch(d, _pool(), _batch(n_dump=2), need) == B.HSD_EINVAL           # dump without buffers
    # acceptance threshold: log(tau) of a tau in (0, 1]; the relaxed rule needs its output buffer
    assert B.hsd_validate_batch(d, _pool(), _batch(log_tau=0.1), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(log_tau=float("nan")), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(log_tau=float("-inf"), draft_gap=0x1000), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(log_tau=-0.3), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(log_tau=-0.3, draft_gap=0x1000), need) == B.HSD_OK
    # packed prefix trees: the depths and the stop-node output come with tree_end
    assert B.hsd_validate_batch(d, _pool(), _batch(tree_end=0x1000), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(tree_end=0x1000, tree_depth=0x1000), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(), _batch(tree_end=0x1000, tree_depth=0x1000, stop_row=0x1000), need) == B.HSD_OK
    assert B.hsd_validate_batch(d, _pool(n_blocks=0), _batch(), need) == B.HSD_EINVAL
    assert B.hsd_validate_batch(d, _pool(k_pool=None), _batch(), need) == B.HSD_EINVAL
    assert B.hsd_workspace_bytes(_desc(head_dim=32), 10, 1) == 0


def test_entry_points_reject_null_context_without_a_device():
    d, b, p = _desc(), _batch(), _pool()
    for fn in (B.lib.hsd_verify_region_batch, B.lib.hsd_verify_page, B.lib.hsd_prefill):
        assert fn(None, None, C.byref(p), C.byref(b), 0x1000, 1 << 30) == B.HSD_EINVAL
    assert B.lib.hsd_kv_commit_rollback(None, None, C.byref(p), C.byref(b), None) == B.HSD_EINVAL
    assert B.lib.hsd_kv_pool_init(None, None) == B.HSD_EINVAL
    out = C.c_void_p()
    assert B.lib.hsd_create(C.byref(d), None, C.byref(out)) == B.HSD_EINVAL
    assert B.lib.hsd_create(C.byref(_desc(head_dim=8)), None, C.byref(out)) == B.HSD_EINVAL


def test_create_without_gpu_reports_no_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    d = _desc(n_layers=1)
    w = B.hsd_weights()
    arr = (C.c_void_p * 1)(0x1000)
    w.tok_embed = w.final_norm = w.lm_head = 0x1000
    for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down"):
        setattr(w, n, C.cast(arr, C.POINTER(C.c_void_p)))
    out = C.c_void_p()
    assert B.lib.hsd_create(C.byref(d), C.byref(w), C.byref(out)) == B.HSD_ENODEV
    assert not out.value


def test_probe_launch_rejects_bad_arguments_before_touching_a_device():
    """hsd_probe_launch validates its arguments on the host: nothing is launched for any of these."""
    fake = C.c_void_p(0x1000)   # never dereferenced: every call below fails validation first
    for kind, n_wg, iters, arg, scratch, nbytes in (
            (B.HSD_PROBE_MFMA, 0, 10, 0, fake, 64), (B.HSD_PROBE_MFMA, 8, 0, 0, fake, 64),
            (B.HSD_PROBE_MFMA, 8, 10, 0, None, 64), (B.HSD_PROBE_MFMA, 8, 10, 0, fake, 0),
            (7, 8, 10, 0, fake, 64), (B.HSD_PROBE_LOAD_REG, 8, 10, 0, fake, 8 * 32768 - 8),
            (B.HSD_PROBE_LOAD_LDS, 8, 10, 0, fake, 8 * 40000), (B.HSD_PROBE_LDS_READ, 8, 10, 0, fake, 64),
            (B.HSD_PROBE_LDS_READ, 8, 10, 17, fake, 64)):
        assert B.lib.hsd_probe_launch(None, kind, n_wg, iters, arg, scratch, nbytes) == B.HSD_EINVAL
