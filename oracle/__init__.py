"""Python face of the CPU oracle (oracle.c) — TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package. It shares no code with the HIP library and never imports it. The arithmetic
lives in oracle.c (plain C, fp64); this file only marshals numpy arrays through ctypes
and loops over batch entries.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OK, BAD_ROOT, BAD_PARENT, BAD_SIZE, BAD_PATH = 0, 1, 2, 3, 4


# ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (any finding aborts). Python itself is not instrumented, so the
# sanitizer runtime has to be preloaded:
#   ORACLE_SANITIZE=1 ASAN_OPTIONS=detect_leaks=0 LD_PRELOAD=$(gcc -print-file-name=libasan.so) \
#       python -m pytest tests -m "not gpu"
_SANITIZE = os.environ.get("ORACLE_SANITIZE", "") not in ("", "0")
if _SANITIZE:
    _LIB = os.path.join(_HERE, "liboracle_san.so")


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc into liboracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O2"]
        if _SANITIZE:
            flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                     "-fno-sanitize-recover=all"]
        subprocess.check_call(["gcc", *flags, "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.oracle_tree_validate.argtypes = [i32p, ctypes.c_int32]
        lib.oracle_tree_validate.restype = ctypes.c_int
        lib.oracle_tree_mask.argtypes = [i32p, ctypes.c_int32, ctypes.POINTER(ctypes.c_uint64), i32p]
        lib.oracle_tree_mask.restype = ctypes.c_int
        lib.oracle_tree_attention.argtypes = [
            f32p, f32p, f32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_double, i32p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
            i32p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
            ctypes.POINTER(ctypes.c_double)]
        lib.oracle_tree_attention.restype = ctypes.c_int
        lib.oracle_row_argmax.argtypes = [f32p, ctypes.c_int64]
        lib.oracle_row_argmax.restype = ctypes.c_int64
        lib.oracle_tree_accept.argtypes = [i32p, i32p, i32p, ctypes.c_int32, i32p, i32p, i32p]
        lib.oracle_tree_accept.restype = ctypes.c_int
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_tree_accept_sample.argtypes = [
            f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, i32p, i32p, ctypes.c_int32, f64p, ctypes.c_double,
            i32p, i32p, i32p, f64p]
        lib.oracle_tree_accept_sample.restype = ctypes.c_int
        lib.oracle_tree_accept_sample_check.argtypes = [
            f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, i32p, i32p, ctypes.c_int32, f64p, ctypes.c_double,
            ctypes.c_int32, i32p, ctypes.c_int32, ctypes.c_double, f64p]
        lib.oracle_tree_accept_sample_check.restype = ctypes.c_int
        lib.oracle_draft_expand.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, f32p, ctypes.c_int32, ctypes.c_int32,
                                            i32p, f64p, i32p, f64p]
        lib.oracle_draft_expand.restype = ctypes.c_int
        lib.oracle_draft_tree_build.argtypes = [i32p, f32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                i32p, i32p, i32p, i32p]
        lib.oracle_draft_tree_build.restype = ctypes.c_int
        lib.oracle_compress_attention.argtypes = [
            f32p, f32p, f32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_double, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int32, ctypes.c_int64, f64p]
        lib.oracle_compress_attention.restype = ctypes.c_int
        lib.oracle_kv_commit.argtypes = [
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int32,
            ctypes.c_int64, i32p]
        lib.oracle_kv_commit.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def tree_validate(parent) -> int:
    parent = _i32(parent)
    return int(_load().oracle_tree_validate(_p(parent, ctypes.c_int32), len(parent)))


def tree_mask(parent):
    """(rc, mask uint64[T], depth int32[T]) for one tree."""
    parent = _i32(parent)
    T = len(parent)
    mask = np.zeros(T, dtype=np.uint64)
    depth = np.zeros(T, dtype=np.int32)
    rc = _load().oracle_tree_mask(_p(parent, ctypes.c_int32), T, _p(mask, ctypes.c_uint64),
                                  _p(depth, ctypes.c_int32))
    return int(rc), mask, depth


def tree_attention_seq(q, k_cache, v_cache, S, parent, scale, Hkv, *, block_table=None,
                       block_size=16, threads=1):
    """One sequence. q f32 [T, Hq, d]. Contiguous: k_cache/v_cache f32 [Hkv, cap, d].
    Paged: k_cache/v_cache f32 [n_blocks, Hkv, block_size, d] and block_table int32[...].
    Returns float64 [T, Hq, d]."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    k_cache = np.ascontiguousarray(k_cache, dtype=np.float32)
    v_cache = np.ascontiguousarray(v_cache, dtype=np.float32)
    parent = _i32(parent)
    T, Hq, d = q.shape
    out = np.zeros((T, Hq, d), dtype=np.float64)
    if block_table is None:
        assert k_cache.shape[0] == Hkv and k_cache.shape[2] == d
        cap = k_cache.shape[1]
        assert S + T <= cap
        paged, sh, st, sb = 0, cap * d, d, 0
        bt = np.zeros(1, dtype=np.int32)
    else:
        bt = _i32(block_table)
        assert k_cache.shape[1] == Hkv and k_cache.shape[2] == block_size and k_cache.shape[3] == d
        nb = (S + T + block_size - 1) // block_size
        assert nb <= len(bt) and (bt[:nb] >= 0).all() and (bt[:nb] < k_cache.shape[0]).all()
        paged, sh, st, sb = 1, block_size * d, d, Hkv * block_size * d

    def run(h0, h1):
        return lib.oracle_tree_attention(
            _p(q, ctypes.c_float), _p(k_cache, ctypes.c_float), _p(v_cache, ctypes.c_float),
            T, Hq, Hkv, d, int(S), float(scale), _p(parent, ctypes.c_int32), paged, sh, st,
            _p(bt, ctypes.c_int32), block_size, sb, h0, h1, _p(out, ctypes.c_double))

    if threads <= 1:
        rcs = [run(0, Hq)]
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            rcs = list(ex.map(lambda h: run(h, h + 1), range(Hq)))
    rc = max(int(r) for r in rcs)
    if rc != OK:
        raise ValueError(f"oracle_tree_attention failed with code {rc}")
    return out


def tree_attention(inp, threads=1, seqs=None):
    """Whole batch from a gen.AttnInputs-like object (fields: cfg, prefix_len, parent, q,
    k_cache, v_cache, block_table, scale). Returns float64 [B, T, Hq, d]."""
    cfg = inp.cfg
    B = inp.q.shape[0]
    out = np.zeros(inp.q.shape, dtype=np.float64)
    for b in (range(B) if seqs is None else seqs):
        if inp.block_table is None:
            out[b] = tree_attention_seq(inp.q[b], inp.k_cache[b], inp.v_cache[b], int(inp.prefix_len[b]),
                                        inp.parent[b], inp.scale, cfg.Hkv, threads=threads)
        else:
            out[b] = tree_attention_seq(inp.q[b], inp.k_cache, inp.v_cache, int(inp.prefix_len[b]),
                                        inp.parent[b], inp.scale, cfg.Hkv,
                                        block_table=inp.block_table[b], block_size=cfg.block_size,
                                        threads=threads)
    return out


def row_argmax(logits) -> np.ndarray:
    """int32 argmax of every row of a float32 [..., V] array (first maximum)."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    V = lg.shape[-1]
    flat = lg.reshape(-1, V)
    out = np.empty(flat.shape[0], dtype=np.int32)
    lib = _load()
    for r in range(flat.shape[0]):
        out[r] = lib.oracle_row_argmax(_p(flat[r], ctypes.c_float), V)
    return out.reshape(lg.shape[:-1])


def tree_accept_from_argmax(amax, draft, parent):
    """(rc, accepted_len, path int32[T], bonus) for one tree given per-node argmax."""
    amax, draft, parent = _i32(amax), _i32(draft), _i32(parent)
    T = len(parent)
    alen = ctypes.c_int32(0)
    bonus = ctypes.c_int32(0)
    path = np.full(T, -1, dtype=np.int32)
    rc = _load().oracle_tree_accept(_p(amax, ctypes.c_int32), _p(draft, ctypes.c_int32),
                                    _p(parent, ctypes.c_int32), T, ctypes.byref(alen),
                                    _p(path, ctypes.c_int32), ctypes.byref(bonus))
    return int(rc), int(alen.value), path, int(bonus.value)


def tree_accept(logits, draft, parent):
    """Batch: logits f32 [B, T, V], draft/parent int32 [B, T] →
    (amax [B,T], accepted_len [B], path [B,T], bonus [B])."""
    lg = np.asarray(logits)
    B, T, _ = lg.shape
    amax = row_argmax(lg)
    alen = np.zeros(B, dtype=np.int32)
    path = np.full((B, T), -1, dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    for b in range(B):
        rc, alen[b], path[b], bonus[b] = tree_accept_from_argmax(amax[b], draft[b], parent[b])
        if rc != OK:
            raise ValueError(f"oracle_tree_accept failed with code {rc}")
    return amax, alen, path, bonus


def kv_commit_seq(cache, S, path, accepted_len, *, block_table=None, block_size=16):
    """Moves the accepted path's rows of ONE sequence inside `cache` IN PLACE and returns
    (rc, new_prefix). Contiguous: cache [Hkv, cap, d]; paged: cache [n_blocks, Hkv, block_size, d]
    (the whole pool) with that sequence's block_table row. Any dtype; rows move as bytes."""
    assert cache.flags["C_CONTIGUOUS"]
    path = _i32(path)
    T = len(path)
    d = cache.shape[-1]
    if block_table is None:
        Hkv, cap = cache.shape[0], cache.shape[1]
        assert S + T <= cap
        paged, sh, st, sb = 0, cap * d, d, 0
        bt = np.zeros(1, dtype=np.int32)
    else:
        bt = _i32(block_table)
        Hkv = cache.shape[1]
        assert cache.shape[2] == block_size
        paged, sh, st, sb = 1, block_size * d, d, Hkv * block_size * d
    newp = np.zeros(1, dtype=np.int32)
    rc = _load().oracle_kv_commit(cache.ctypes.data_as(ctypes.c_void_p), cache.dtype.itemsize, Hkv, d, int(S), T,
                                  _p(path, ctypes.c_int32), int(accepted_len), paged, sh, st,
                                  _p(bt, ctypes.c_int32), block_size, sb, _p(newp, ctypes.c_int32))
    return int(rc), int(newp[0])


def tree_accept_sample_seq(logits, draft, parent, temperature, u_accept, u_bonus):
    """One sequence: logits f32 [T, V]; u_accept [T] and u_bonus in [0, 1).
    Returns (rc, accepted_len, path int32[T], bonus, margin)."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    T, V = lg.shape
    draft, parent = _i32(draft), _i32(parent)
    ua = np.ascontiguousarray(u_accept, dtype=np.float64)
    alen, bonus, margin = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_double(0)
    path = np.full(T, -1, dtype=np.int32)
    rc = _load().oracle_tree_accept_sample(_p(lg, ctypes.c_float), V, V, float(temperature), _p(draft, ctypes.c_int32),
                                           _p(parent, ctypes.c_int32), T, _p(ua, ctypes.c_double), float(u_bonus),
                                           ctypes.byref(alen), _p(path, ctypes.c_int32), ctypes.byref(bonus),
                                           ctypes.byref(margin))
    return int(rc), int(alen.value), path, int(bonus.value), float(margin.value)


def tree_accept_sample_check_seq(logits, draft, parent, temperature, u_accept, u_bonus, accepted_len, path, bonus,
                                 eps):
    """Is the claimed outcome one the rule can produce when each uniform-vs-threshold comparison
    may be off by eps? Returns (rc, worst): rc 0 = yes; worst = largest wrong-side distance."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    T, V = lg.shape
    draft, parent, path = _i32(draft), _i32(parent), _i32(path)
    ua = np.ascontiguousarray(u_accept, dtype=np.float64)
    worst = ctypes.c_double(0)
    rc = _load().oracle_tree_accept_sample_check(_p(lg, ctypes.c_float), V, V, float(temperature),
                                                 _p(draft, ctypes.c_int32), _p(parent, ctypes.c_int32), T,
                                                 _p(ua, ctypes.c_double), float(u_bonus), int(accepted_len),
                                                 _p(path, ctypes.c_int32), int(bonus), float(eps), ctypes.byref(worst))
    return int(rc), float(worst.value)


def tree_accept_sample(logits, draft, parent, temperature, u_accept, u_bonus):
    """Batch: logits [B,T,V], u_accept [B,T], u_bonus [B] -> (accepted_len [B], path [B,T], bonus [B], margin [B])."""
    B, T, _ = np.asarray(logits).shape
    alen = np.zeros(B, dtype=np.int32)
    path = np.full((B, T), -1, dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    margin = np.zeros(B)
    for b in range(B):
        rc, alen[b], path[b], bonus[b], margin[b] = tree_accept_sample_seq(logits[b], draft[b], parent[b], temperature,
                                                                           u_accept[b], u_bonus[b])
        if rc != OK:
            raise ValueError(f"oracle_tree_accept_sample failed with code {rc}")
    return alen, path, bonus, margin


def draft_expand_seq(logits, cum_in, K):
    """One expansion step of one sequence: logits f32 [F,V], cum_in f32 [F].
    Returns (rc, cand_token int32[F*K], cand_score f64[F*K], frontier int32[min(K,F*K)], cut_gap)."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    F, V = lg.shape
    cum = np.ascontiguousarray(cum_in, dtype=np.float32)
    tok = np.full(F * K, -1, dtype=np.int32)
    sc = np.zeros(F * K, dtype=np.float64)
    fr = np.full(min(K, F * K), -1, dtype=np.int32)
    gap = ctypes.c_double(0)
    rc = _load().oracle_draft_expand(_p(lg, ctypes.c_float), V, V, _p(cum, ctypes.c_float), F, K,
                                     _p(tok, ctypes.c_int32), _p(sc, ctypes.c_double), _p(fr, ctypes.c_int32),
                                     ctypes.byref(gap))
    return int(rc), tok, sc, fr, float(gap.value)


def draft_tree_build_seq(cand_token, cand_score, cand_parent, N, root_token=-1):
    """Final selection of one sequence. Returns (rc, parent int32[T], tokens int32[T], node_cand int32[T])."""
    tok, par = _i32(cand_token), _i32(cand_parent)
    sc = np.ascontiguousarray(cand_score, dtype=np.float32)
    M = len(tok)
    parent = np.full(N + 1, -1, dtype=np.int32)
    tokens = np.full(N + 1, -1, dtype=np.int32)
    node_cand = np.full(N + 1, -1, dtype=np.int32)
    T = ctypes.c_int32(0)
    rc = _load().oracle_draft_tree_build(_p(tok, ctypes.c_int32), _p(sc, ctypes.c_float), _p(par, ctypes.c_int32), M, N,
                                         int(root_token), _p(parent, ctypes.c_int32), _p(tokens, ctypes.c_int32),
                                         _p(node_cand, ctypes.c_int32), ctypes.byref(T))
    t = int(T.value) if rc == OK else 0
    return int(rc), parent[:t], tokens[:t], node_cand[:t]


def compress_attention_seq(q, k_cache, v_cache, r, scale, Hkv, *, block_table=None, block_size=16):
    """Vision-adaptor compression attention for one image: q f32 [nq, Hq, d] (the learnable
    queries), K / V f32 [Hkv, cap, d] (contiguous) or [n_blocks, Hkv, block_size, d] (paged), of
    which the first r logical tokens are the image embeddings. Returns float64 [nq, Hq, d]."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    k_cache = np.ascontiguousarray(k_cache, dtype=np.float32)
    v_cache = np.ascontiguousarray(v_cache, dtype=np.float32)
    nq, Hq, d = q.shape
    out = np.zeros((nq, Hq, d), dtype=np.float64)
    if block_table is None:
        cap = k_cache.shape[1]
        assert k_cache.shape[0] == Hkv and r <= cap
        paged, sh, st, sb = 0, cap * d, d, 0
        bt = np.zeros(1, dtype=np.int32)
    else:
        bt = _i32(block_table)
        assert k_cache.shape[1] == Hkv and k_cache.shape[2] == block_size
        paged, sh, st, sb = 1, block_size * d, d, Hkv * block_size * d
    rc = _load().oracle_compress_attention(_p(q, ctypes.c_float), _p(k_cache, ctypes.c_float),
                                           _p(v_cache, ctypes.c_float), nq, Hq, Hkv, d, int(r), float(scale), paged,
                                           sh, st, _p(bt, ctypes.c_int32), block_size, sb, _p(out, ctypes.c_double))
    if rc != OK:
        raise ValueError(f"oracle_compress_attention failed with code {rc}")
    return out
