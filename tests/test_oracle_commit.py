"""Pins for the oracle's KV-cache commit of the accepted path (no GPU)."""
import dataclasses
import json
import os

import numpy as np
import pytest

import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _gather_expected(orig, S, path, alen):
    """Out-of-place statement of the result: destination rows gathered from a pristine copy."""
    exp = orig.copy()
    ks = np.arange(1, alen + 1)
    exp[:, S + ks] = orig[:, S + path[ks]]
    return exp


def test_hand_worked_example(oracle_mod):
    g = json.load(open(os.path.join(GOLDEN, "kv_commit_tiny.json")))
    cache = np.array(g["cache_before"], dtype=np.float32)[None]        # [Hkv=1, cap, d]
    rc, newp = oracle_mod.kv_commit_seq(cache, g["S"], g["path"], g["accepted_len"])
    assert rc == 0 and newp == g["new_prefix"]
    assert np.array_equal(cache[0], np.array(g["cache_after"], dtype=np.float32))


@pytest.mark.parametrize("dtype", [np.uint16, np.float32])
@pytest.mark.parametrize("seed", range(12))
def test_equals_gather_from_pristine_copy(oracle_mod, dtype, seed):
    g = gen.rng(seed, gen.STREAM_PATH)
    T = int(g.integers(1, 65))
    parent = gen.random_tree(gen.rng(seed, gen.STREAM_TREE), T, max_depth=min(8, max(1, T - 1)), max_children=4)
    path, alen = gen.random_accept_path(g, parent, full=(seed % 3 == 0))
    Hkv, d, S = int(g.integers(1, 5)), int(g.choice([8, 64, 128])), int(g.integers(0, 40))
    cap = S + T + int(g.integers(0, 5))
    orig = g.integers(0, 60000, size=(Hkv, cap, d)).astype(dtype)
    cache = orig.copy()
    rc, newp = oracle_mod.kv_commit_seq(cache, S, path, alen)
    assert rc == 0 and newp == S + alen + 1
    assert np.array_equal(cache, _gather_expected(orig, S, path, alen))
    # the new context, in order, is the old prefix followed by the accepted nodes' rows
    ctx = np.concatenate([orig[:, :S], orig[:, S + path[:alen + 1]]], axis=1)
    assert np.array_equal(cache[:, :newp], ctx)


def test_paged_equals_contiguous(oracle_mod):
    g = gen.rng(5, gen.STREAM_PATH)
    T, Hkv, d, S, bs = 33, 2, 16, 37, 16
    parent = gen.random_tree(gen.rng(5, gen.STREAM_TREE), T, 6, 3)
    path, alen = gen.random_accept_path(g, parent, full=True)
    assert alen >= 3
    nb = (S + T + bs - 1) // bs
    cont = g.integers(0, 60000, size=(Hkv, nb * bs, d)).astype(np.uint16)
    table = g.permutation(nb + 3)[:nb].astype(np.int32)
    pool = np.full((nb + 3, Hkv, bs, d), 7, dtype=np.uint16)
    for i, blk in enumerate(table):
        pool[blk] = cont[:, i * bs:(i + 1) * bs]
    pool0 = pool.copy()
    rc1, n1 = oracle_mod.kv_commit_seq(cont, S, path, alen)
    rc2, n2 = oracle_mod.kv_commit_seq(pool, S, path, alen, block_table=table, block_size=bs)
    assert rc1 == rc2 == 0 and n1 == n2
    for i, blk in enumerate(table):
        assert np.array_equal(pool[blk], cont[:, i * bs:(i + 1) * bs])
    unused = [b for b in range(nb + 3) if b not in set(table.tolist())]
    assert np.array_equal(pool[unused], pool0[unused])                  # blocks of other sequences untouched


def test_chain_path_and_zero_acceptance_are_identities(oracle_mod):
    T, S = 9, 4
    orig = gen.rng(2, gen.STREAM_K).integers(0, 9999, size=(3, S + T, 8)).astype(np.uint16)
    path = np.arange(T, dtype=np.int32)                                  # chain tree fully accepted
    c = orig.copy()
    assert oracle_mod.kv_commit_seq(c, S, path, T - 1) == (0, S + T)
    assert np.array_equal(c, orig)
    c = orig.copy()
    assert oracle_mod.kv_commit_seq(c, S, [0] + [-1] * (T - 1), 0) == (0, S + 1)
    assert np.array_equal(c, orig)


@pytest.mark.parametrize("path,alen", [([1, 2, 3], 1), ([0, 2, 2], 2), ([0, 2, 1], 2), ([0, 1, 3], 2), ([0, 1, 2], 3),
                                        ([0, 1, 2], -1)])
def test_malformed_paths_are_rejected_and_nothing_moves(oracle_mod, path, alen):
    orig = np.arange(2 * 8 * 4, dtype=np.uint16).reshape(2, 8, 4)
    c = orig.copy()
    rc, _ = oracle_mod.kv_commit_seq(c, 2, path, alen)
    assert rc == oracle_mod.BAD_PATH
    assert np.array_equal(c, orig)


def test_closed_loop_next_step_sees_prefix_plus_accepted_tokens(oracle_mod):
    """What the commit is for: the next verify step over the committed cache must equal a verify
    step over a cache assembled directly from the old prefix and the accepted tokens' rows."""
    cfg = gen.Config("loop", 1, 4, 2, 64, 24, 5, 3, 100, 0.5, 1, "bf16", prefix=[50])
    inp = gen.attention_inputs(cfg, 77, poison_tail=False)
    S, T = 50, cfg.T
    path, alen = gen.random_accept_path(gen.rng(77, gen.STREAM_PATH), inp.parent[0], full=True)
    k, v = inp.k_cache[0].copy(), inp.v_cache[0].copy()                 # [Hkv, cap, d]
    k0, v0 = k.copy(), v.copy()
    assert oracle_mod.kv_commit_seq(k, S, path, alen)[0] == 0
    rc, newS = oracle_mod.kv_commit_seq(v, S, path, alen)
    # the next step: a fresh small tree whose rows go to slots newS .. newS + T2 - 1
    T2 = 6
    parent2 = gen.random_tree(gen.rng(78, gen.STREAM_TREE), T2, 3, 2)
    g = gen.rng(78, gen.STREAM_K)
    newk = g.standard_normal((cfg.Hkv, T2, cfg.d)).astype(np.float32)
    newv = g.standard_normal((cfg.Hkv, T2, cfg.d)).astype(np.float32)
    q2 = g.standard_normal((T2, cfg.Hq, cfg.d)).astype(np.float32)
    k[:, newS:newS + T2] = newk
    v[:, newS:newS + T2] = newv
    got = oracle_mod.tree_attention_seq(q2, k, v, newS, parent2, inp.scale, cfg.Hkv)
    rows = np.concatenate([np.arange(S), S + path[:alen + 1]])
    k_ref = np.concatenate([k0[:, rows], newk], axis=1)
    v_ref = np.concatenate([v0[:, rows], newv], axis=1)
    ref = oracle_mod.tree_attention_seq(q2, np.ascontiguousarray(k_ref), np.ascontiguousarray(v_ref), newS, parent2,
                                        inp.scale, cfg.Hkv)
    assert np.array_equal(got, ref)
