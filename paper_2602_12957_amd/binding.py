"""ctypes mirror of include/hsd.h: same names, argument marshalling only."""
import ctypes as C
import os

# torch is the device-memory provider and ships its own HIP runtime (libamdhip64.so.7).  Import it first so
# that libhsd.so binds to that same runtime instance: pointers and streams are only meaningful within one.
import torch  # noqa: F401

from .build import LIB_PATH

LIB_PATH = os.environ.get("HSD_LIB_PATH", LIB_PATH)   # experiments: load an alternative build of the library

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2602_12957_amd.build, or "
        "__graft_entry__.build()).  There is no fallback path.")

lib = C.CDLL(LIB_PATH)

HSD_OK, HSD_EINVAL, HSD_ENOSPC, HSD_ERANGE, HSD_EARCH, HSD_ENODEV, HSD_EHIP = 0, -1, -2, -3, -4, -5, -6
HSD_FP32, HSD_BF16 = 0, 1
HSD_STATUS_POOL_EXHAUSTED, HSD_STATUS_TABLE_OVERFLOW, HSD_STATUS_BAD_SLOT, HSD_STATUS_BAD_TREE = 1, 2, 4, 8
HSD_KV_BLOCK_TOKENS, HSD_HEAD_DIM, HSD_MAX_SEQ = 16, 64, 4096

i32, f32, vp = C.c_int32, C.c_float, C.c_void_p


class hsd_model_desc(C.Structure):
    _fields_ = [(n, i32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                                   "dtype", "kv_block_tokens")] + [("rms_eps", f32), ("rope_theta", f32),
                                                                       ("attn_key_chunk", i32)]


class hsd_weights(C.Structure):
    _fields_ = [("tok_embed", vp), ("final_norm", vp), ("lm_head", vp),
                ("attn_norm", C.POINTER(vp)), ("wqkv", C.POINTER(vp)), ("wo", C.POINTER(vp)),
                ("ffn_norm", C.POINTER(vp)), ("w_gate_up", C.POINTER(vp)), ("w_down", C.POINTER(vp))]


class hsd_kv_pool(C.Structure):
    _fields_ = [("k_pool", vp), ("v_pool", vp), ("n_blocks", i32), ("free_list", vp), ("free_count", vp)]


class hsd_batch(C.Structure):
    _fields_ = [("n_seq", i32), ("total_q", i32), ("max_blocks_per_seq", i32), ("n_slots", i32),
                ("cu_q", vp), ("seq_slot", vp), ("tokens", vp), ("embeds", vp), ("seq_len", vp),
                ("block_table", vp), ("argmax", vp), ("top2_margin", vp), ("accept_len", vp), ("bonus", vp),
                ("status", vp), ("logits_dump", vp), ("dump_rows", vp), ("n_dump", i32),
                ("log_tau", f32), ("draft_gap", vp), ("tree_end", vp), ("tree_depth", vp), ("stop_row", vp)]


_P = C.POINTER
lib.hsd_status_string.restype = C.c_char_p
lib.hsd_status_string.argtypes = [C.c_int]
lib.hsd_validate_model.argtypes = [_P(hsd_model_desc)]
lib.hsd_validate_batch.argtypes = [_P(hsd_model_desc), _P(hsd_kv_pool), _P(hsd_batch), C.c_size_t]
lib.hsd_create.argtypes = [_P(hsd_model_desc), _P(hsd_weights), _P(vp)]
lib.hsd_destroy.argtypes = [vp]
lib.hsd_destroy.restype = None
lib.hsd_workspace_bytes.argtypes = [_P(hsd_model_desc), i32, i32]
lib.hsd_workspace_bytes.restype = C.c_size_t
lib.hsd_kv_pool_init.argtypes = [vp, _P(hsd_kv_pool)]
for _n in ("hsd_verify_region_batch", "hsd_verify_page", "hsd_prefill"):
    getattr(lib, _n).argtypes = [vp, vp, _P(hsd_kv_pool), _P(hsd_batch), vp, C.c_size_t]
lib.hsd_verify_region_batch_noalloc.argtypes = [vp, vp, _P(hsd_kv_pool), _P(hsd_batch)]
lib.hsd_noalloc_scratch_bytes.argtypes = []
lib.hsd_noalloc_scratch_bytes.restype = C.c_size_t
lib.hsd_kv_commit_rollback.argtypes = [vp, vp, _P(hsd_kv_pool), _P(hsd_batch), vp]

lib.hsd_profile_enable.argtypes = [vp, C.c_int, i32]
lib.hsd_profile_read.argtypes = [vp, _P(i32), _P(f32)]
(HSD_PROF_NONE, HSD_PROF_GEMM_QKV, HSD_PROF_ATTENTION, HSD_PROF_GEMM_O, HSD_PROF_GEMM_GATE_UP, HSD_PROF_GEMM_DOWN,
 HSD_PROF_GEMM_LM_HEAD, HSD_PROF_RMSNORM) = range(8)

lib.hsd_debug_set.argtypes = [vp, C.c_int, C.c_int64]
HSD_DEBUG_SYNC_LAYERS, HSD_DEBUG_FORCE_SIMPLE = 1, 2
(HSD_DEBUG_GEMM_CFG_QKV, HSD_DEBUG_GEMM_CFG_O, HSD_DEBUG_GEMM_CFG_GATE_UP, HSD_DEBUG_GEMM_CFG_DOWN,
 HSD_DEBUG_GEMM_CFG_LM_HEAD) = range(6, 11)

lib.hsd_probe_launch.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_size_t]
HSD_PROBE_MFMA, HSD_PROBE_LOAD_REG, HSD_PROBE_LOAD_LDS, HSD_PROBE_LDS_READ = range(4)

EXPORTS = ["hsd_probe_launch", "hsd_verify_region_batch_noalloc", "hsd_noalloc_scratch_bytes", "hsd_debug_set", "hsd_profile_enable", "hsd_profile_read", "hsd_status_string", "hsd_validate_model", "hsd_validate_batch", "hsd_create", "hsd_destroy",
           "hsd_workspace_bytes", "hsd_kv_pool_init", "hsd_verify_region_batch", "hsd_verify_page",
           "hsd_kv_commit_rollback", "hsd_prefill"]


class HsdError(RuntimeError):
    def __init__(self, where, code):
        super().__init__(f"{where}: {lib.hsd_status_string(code).decode()} ({code})")
        self.code = code


def check(where, code):
    if code != HSD_OK:
        raise HsdError(where, code)


def hsd_status_string(code): return lib.hsd_status_string(code).decode()
def hsd_validate_model(desc): return lib.hsd_validate_model(C.byref(desc))
def hsd_validate_batch(desc, pool, batch, ws_bytes):
    return lib.hsd_validate_batch(C.byref(desc), C.byref(pool) if pool is not None else None, C.byref(batch), ws_bytes)
def hsd_workspace_bytes(desc, max_total_q, max_n_seq): return lib.hsd_workspace_bytes(C.byref(desc), max_total_q, max_n_seq)
def hsd_create(desc, weights):
    out = vp()
    check("hsd_create", lib.hsd_create(C.byref(desc), C.byref(weights), C.byref(out)))
    return out
def hsd_destroy(ctx): lib.hsd_destroy(ctx)
def hsd_kv_pool_init(stream, pool): check("hsd_kv_pool_init", lib.hsd_kv_pool_init(stream, C.byref(pool)))
def hsd_verify_region_batch(ctx, stream, pool, batch, ws, ws_bytes):
    check("hsd_verify_region_batch", lib.hsd_verify_region_batch(ctx, stream, C.byref(pool), C.byref(batch), ws, ws_bytes))
def hsd_verify_region_batch_noalloc(ctx, stream, pool, batch):
    check("hsd_verify_region_batch_noalloc", lib.hsd_verify_region_batch_noalloc(ctx, stream, C.byref(pool), C.byref(batch)))
def hsd_noalloc_scratch_bytes(): return lib.hsd_noalloc_scratch_bytes()
def hsd_verify_page(ctx, stream, pool, batch, ws, ws_bytes):
    check("hsd_verify_page", lib.hsd_verify_page(ctx, stream, C.byref(pool), C.byref(batch), ws, ws_bytes))
def hsd_prefill(ctx, stream, pool, batch, ws, ws_bytes):
    check("hsd_prefill", lib.hsd_prefill(ctx, stream, C.byref(pool), C.byref(batch), ws, ws_bytes))
def hsd_kv_commit_rollback(ctx, stream, pool, batch, pending_out):
    check("hsd_kv_commit_rollback", lib.hsd_kv_commit_rollback(ctx, stream, C.byref(pool), C.byref(batch), pending_out))

def hsd_profile_enable(ctx, which, max_launches):
    check("hsd_profile_enable", lib.hsd_profile_enable(ctx, which, max_launches))
def hsd_profile_read(ctx):
    n, ms = i32(), f32()
    check("hsd_profile_read", lib.hsd_profile_read(ctx, C.byref(n), C.byref(ms)))
    return n.value, ms.value

def hsd_debug_set(ctx, knob, value):
    check("hsd_debug_set", lib.hsd_debug_set(ctx, knob, value))
def hsd_probe_launch(stream, kind, n_workgroups, iters, arg, scratch, scratch_bytes):
    check("hsd_probe_launch", lib.hsd_probe_launch(stream, kind, n_workgroups, iters, arg, scratch, scratch_bytes))
