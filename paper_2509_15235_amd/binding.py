"""ctypes binding: same names and argument order as include/vispec_verify.h."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# VISPEC_VERIFY_LIB names another build of the same library (e.g. the one whose host code is
# compiled with sanitizers, see build.py)
_LIB_PATH = os.environ.get("VISPEC_VERIFY_LIB") or os.path.join(_HERE, "libvispec_verify.so")

VS_BF16, VS_F32 = 0, 1
VS_IMPL_AUTO, VS_IMPL_GENERIC, VS_IMPL_MFMA = 0, 1, 2
VS_SCHED_AUTO, VS_SCHED_LOOP, VS_SCHED_PIPELINED, VS_SCHED_RESIDENT, VS_SCHED_BALANCED = 0, 1, 2, 3, 4

EXPORTED_SYMBOLS = [
    "vs_version", "vs_strerror", "vs_status_string", "vs_tree_validate_host", "vs_tree_mask_build",
    "vs_attention_plan", "vs_attention_workspace_bytes", "vs_tree_verify_attention",
    "vs_accept_workspace_bytes", "vs_tree_accept", "vs_tree_accept_noalloc", "vs_accept_sample_workspace_bytes", "vs_tree_accept_sample",
    "vs_draft_expand_workspace_bytes", "vs_draft_expand", "vs_draft_tree_build", "vs_tree_kv_commit",
    "vs_compress_attention_workspace_bytes", "vs_compress_attention",
]
# measurement helpers declared in include/vispec_peaks.h
PEAK_SYMBOLS = ["vs_peak_hbm_read", "vs_peak_hbm_copy", "vs_peak_mfma_bf16", "vs_peak_mfma_flops"]


class VSError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: vs_error {code} ({vs_strerror(code)})")
        self.code = code


class AttnDesc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("d", ctypes.c_int32), ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("max_prefix_len", ctypes.c_int32), ("paged", ctypes.c_int32), ("block_size", ctypes.c_int32),
        ("max_blocks", ctypes.c_int32), ("num_blocks", ctypes.c_int32), ("capacity", ctypes.c_int64),
        ("stride_seq", ctypes.c_int64), ("stride_block", ctypes.c_int64), ("stride_head", ctypes.c_int64),
        ("stride_tok", ctypes.c_int64), ("block_table", ctypes.c_void_p), ("impl", ctypes.c_int32),
        ("num_splits", ctypes.c_int32), ("rows_per_wave", ctypes.c_int32), ("waves_per_group", ctypes.c_int32),
        ("schedule", ctypes.c_int32),
    ]


class KVDesc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("num_layers", ctypes.c_int32), ("stride_layer", ctypes.c_int64),
        ("paged", ctypes.c_int32), ("block_size", ctypes.c_int32), ("max_blocks", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32), ("capacity", ctypes.c_int64), ("stride_seq", ctypes.c_int64),
        ("stride_block", ctypes.c_int64), ("stride_head", ctypes.c_int64), ("stride_tok", ctypes.c_int64),
        ("block_table", ctypes.c_void_p),
    ]


class AttnPlan(ctypes.Structure):
    _fields_ = [
        ("impl", ctypes.c_int32), ("num_splits", ctypes.c_int32), ("keys_per_split", ctypes.c_int32),
        ("row_groups", ctypes.c_int32), ("waves_per_group", ctypes.c_int32), ("rows_per_wave", ctypes.c_int32),
        ("workgroups", ctypes.c_int32),
        ("combine", ctypes.c_int32), ("schedule", ctypes.c_int32),
    ]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2509_15235_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.vs_version.restype = i32
        L.vs_strerror.argtypes = [i32]
        L.vs_strerror.restype = ctypes.c_char_p
        L.vs_status_string.argtypes = [i32]
        L.vs_status_string.restype = ctypes.c_char_p
        L.vs_tree_validate_host.argtypes = [vp, i32]
        L.vs_tree_validate_host.restype = i32
        L.vs_tree_mask_build.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.vs_tree_mask_build.restype = i32
        L.vs_attention_plan.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(AttnPlan)]
        L.vs_attention_plan.restype = i32
        L.vs_attention_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
        L.vs_attention_workspace_bytes.restype = sz
        L.vs_tree_verify_attention.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_tree_verify_attention.restype = i32
        L.vs_compress_attention_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
        L.vs_compress_attention_workspace_bytes.restype = sz
        L.vs_compress_attention.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_compress_attention.restype = i32
        L.vs_accept_workspace_bytes.argtypes = [i32, i32, i32]
        L.vs_accept_workspace_bytes.restype = sz
        L.vs_tree_accept.argtypes = [vp, i64, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_tree_accept.restype = i32
        L.vs_tree_accept_noalloc.argtypes = [vp, i64, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        L.vs_tree_accept_noalloc.restype = i32
        L.vs_accept_sample_workspace_bytes.argtypes = [i32, i32, i32]
        L.vs_accept_sample_workspace_bytes.restype = sz
        L.vs_tree_accept_sample.argtypes = [vp, i64, i32, ctypes.c_float, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp,
                                            sz, vp]
        L.vs_tree_accept_sample.restype = i32
        L.vs_draft_expand_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.vs_draft_expand_workspace_bytes.restype = sz
        L.vs_draft_expand.argtypes = [vp, i64, i32, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_draft_expand.restype = i32
        L.vs_draft_tree_build.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.vs_draft_tree_build.restype = i32
        L.vs_tree_kv_commit.argtypes = [ctypes.POINTER(KVDesc), vp, vp, vp, vp, vp, vp, vp, vp]
        L.vs_tree_kv_commit.restype = i32
        L.vs_peak_hbm_read.argtypes = [vp, sz, vp, i32, vp]
        L.vs_peak_hbm_read.restype = i32
        L.vs_peak_hbm_copy.argtypes = [vp, vp, sz, i32, vp]
        L.vs_peak_hbm_copy.restype = i32
        L.vs_peak_mfma_bf16.argtypes = [vp, i32, vp, i32, vp]
        L.vs_peak_mfma_bf16.restype = i32
        L.vs_peak_mfma_flops.argtypes = [i32, i32]
        L.vs_peak_mfma_flops.restype = ctypes.c_double
        _lib = L
    return _lib


def _ptr(x):
    """Device (or host) address of x: None, an int, a ctypes pointer, or anything with data_ptr()."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    return ctypes.cast(x, ctypes.c_void_p).value


def vs_version() -> int:
    return lib().vs_version()


def vs_strerror(code: int) -> str:
    return lib().vs_strerror(code).decode()


def vs_status_string(code: int) -> str:
    return lib().vs_status_string(code).decode()


def vs_tree_validate_host(parent, T: int) -> int:
    """parent: host int32 array (numpy) of T entries."""
    return lib().vs_tree_validate_host(_ptr(parent), T)


def vs_tree_mask_build(parent, B, T, mask, depth, status=None, stream=None) -> int:
    return lib().vs_tree_mask_build(_ptr(parent), B, T, _ptr(mask), _ptr(depth), _ptr(status), _ptr(stream))


def vs_attention_plan(desc: AttnDesc):
    plan = AttnPlan()
    rc = lib().vs_attention_plan(ctypes.byref(desc), ctypes.byref(plan))
    return rc, plan


def vs_attention_workspace_bytes(desc: AttnDesc) -> int:
    return lib().vs_attention_workspace_bytes(ctypes.byref(desc))


def vs_tree_verify_attention(desc: AttnDesc, q, k_cache, v_cache, prefix_len, tree_parent, tree_mask, out,
                             status=None, workspace=None, workspace_bytes=0, stream=None) -> int:
    return lib().vs_tree_verify_attention(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                          _ptr(prefix_len), _ptr(tree_parent), _ptr(tree_mask), _ptr(out),
                                          _ptr(status), _ptr(workspace), workspace_bytes, _ptr(stream))


def vs_compress_attention_workspace_bytes(desc: AttnDesc) -> int:
    return lib().vs_compress_attention_workspace_bytes(ctypes.byref(desc))


def vs_compress_attention(desc: AttnDesc, q, k, v, kv_len, out, status=None, workspace=None, workspace_bytes=0,
                          stream=None) -> int:
    return lib().vs_compress_attention(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(kv_len), _ptr(out),
                                       _ptr(status), _ptr(workspace), workspace_bytes, _ptr(stream))


def vs_accept_workspace_bytes(B: int, T: int, V: int) -> int:
    return lib().vs_accept_workspace_bytes(B, T, V)


def vs_tree_accept(logits, ld_logits, V, draft_tokens, parent, B, T, accepted_len, path, bonus_token,
                   row_argmax=None, status=None, workspace=None, workspace_bytes=0, stream=None) -> int:
    return lib().vs_tree_accept(_ptr(logits), ld_logits, V, _ptr(draft_tokens), _ptr(parent), B, T,
                                _ptr(accepted_len), _ptr(path), _ptr(bonus_token), _ptr(row_argmax),
                                _ptr(status), _ptr(workspace), workspace_bytes, _ptr(stream))


def vs_tree_accept_noalloc(logits, ld_logits, V, draft_tokens, parent, B, T, accepted_len, path, bonus_token,
                           row_argmax=None, status=None, stream=None) -> int:
    return lib().vs_tree_accept_noalloc(_ptr(logits), ld_logits, V, _ptr(draft_tokens), _ptr(parent), B, T,
                                        _ptr(accepted_len), _ptr(path), _ptr(bonus_token), _ptr(row_argmax),
                                        _ptr(status), _ptr(stream))


def vs_accept_sample_workspace_bytes(B: int, T: int, V: int) -> int:
    return lib().vs_accept_sample_workspace_bytes(B, T, V)


def vs_tree_accept_sample(logits, ld_logits, V, temperature, draft_tokens, parent, u_accept, u_bonus, B, T,
                          accepted_len, path, bonus_token, status=None, workspace=None, workspace_bytes=0,
                          stream=None) -> int:
    return lib().vs_tree_accept_sample(_ptr(logits), ld_logits, V, temperature, _ptr(draft_tokens), _ptr(parent),
                                       _ptr(u_accept), _ptr(u_bonus), B, T, _ptr(accepted_len), _ptr(path),
                                       _ptr(bonus_token), _ptr(status), _ptr(workspace), workspace_bytes,
                                       _ptr(stream))


def vs_draft_expand_workspace_bytes(B: int, F: int, V: int, K: int) -> int:
    return lib().vs_draft_expand_workspace_bytes(B, F, V, K)


def vs_draft_expand(logits, ld_logits, V, cum_in, frontier_cand, B, F, K, cand_base, cand_capacity, cand_token,
                    cand_score, cand_parent, next_frontier_cand, next_cum, workspace=None, workspace_bytes=0,
                    stream=None) -> int:
    return lib().vs_draft_expand(_ptr(logits), ld_logits, V, _ptr(cum_in), _ptr(frontier_cand), B, F, K, cand_base,
                                 cand_capacity, _ptr(cand_token), _ptr(cand_score), _ptr(cand_parent),
                                 _ptr(next_frontier_cand), _ptr(next_cum), _ptr(workspace), workspace_bytes,
                                 _ptr(stream))


def vs_draft_tree_build(cand_token, cand_score, cand_parent, B, M, cand_capacity, N, root_token, parent,
                        draft_tokens, node_cand, num_nodes, status=None, stream=None) -> int:
    return lib().vs_draft_tree_build(_ptr(cand_token), _ptr(cand_score), _ptr(cand_parent), B, M, cand_capacity, N,
                                     _ptr(root_token), _ptr(parent), _ptr(draft_tokens), _ptr(node_cand),
                                     _ptr(num_nodes), _ptr(status), _ptr(stream))


def vs_tree_kv_commit(desc: KVDesc, k_cache, v_cache, prefix_len, path, accepted_len, new_prefix_len,
                      status=None, stream=None) -> int:
    return lib().vs_tree_kv_commit(ctypes.byref(desc), _ptr(k_cache), _ptr(v_cache), _ptr(prefix_len), _ptr(path),
                                   _ptr(accepted_len), _ptr(new_prefix_len), _ptr(status), _ptr(stream))


def vs_peak_hbm_read(src, nbytes: int, sink, workgroups: int, stream=None) -> int:
    return lib().vs_peak_hbm_read(_ptr(src), nbytes, _ptr(sink), workgroups, _ptr(stream))


def vs_peak_hbm_copy(dst, src, nbytes: int, workgroups: int, stream=None) -> int:
    return lib().vs_peak_hbm_copy(_ptr(dst), _ptr(src), nbytes, workgroups, _ptr(stream))


def vs_peak_mfma_bf16(operands, iters: int, sink, workgroups: int, stream=None) -> int:
    return lib().vs_peak_mfma_bf16(_ptr(operands), iters, _ptr(sink), workgroups, _ptr(stream))


def vs_peak_mfma_flops(iters: int, workgroups: int) -> float:
    return lib().vs_peak_mfma_flops(iters, workgroups)
