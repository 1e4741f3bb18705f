"""GPU parity of vs_tree_kv_commit against the oracle: every byte of every layer's cache."""
import dataclasses

import numpy as np
import pytest

import gen
import paper_2509_15235_amd as vs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def _layers(cfg, seed, L, poison=True):
    """L layers of one configuration's caches, stacked; bf16 as uint16 bits, fp32 as float32."""
    ins = [gen.attention_inputs(cfg, seed, layer=l, poison_tail=poison) for l in range(L)]
    bf = cfg.dtype == "bf16"
    k = np.stack([i.k_bits if bf else i.k_cache for i in ins])
    v = np.stack([i.v_bits if bf else i.v_cache for i in ins])
    return ins[0], np.ascontiguousarray(k), np.ascontiguousarray(v)


def _paths(parent, seed, full_every=3):
    B, T = parent.shape
    path = np.empty((B, T), dtype=np.int32)
    alen = np.empty(B, dtype=np.int32)
    for b in range(B):
        path[b], alen[b] = gen.random_accept_path(gen.rng(seed, gen.STREAM_PATH, b), parent[b], full=(b % full_every == 0))
    return path, alen


def _oracle_commit(oracle_mod, inp, k, v, path, alen, skip=()):
    k, v = k.copy(), v.copy()
    B = len(alen)
    newp = inp.prefix_len.copy()
    for b in range(B):
        if b in skip:
            continue
        for arr in (k, v):
            for l in range(arr.shape[0]):
                if inp.block_table is None:
                    rc, n = oracle_mod.kv_commit_seq(arr[l, b], int(inp.prefix_len[b]), path[b], int(alen[b]))
                else:
                    rc, n = oracle_mod.kv_commit_seq(arr[l], int(inp.prefix_len[b]), path[b], int(alen[b]),
                                                     block_table=inp.block_table[b], block_size=inp.cfg.block_size)
                assert rc == 0
        newp[b] = n
    return k, v, newp


def _same_bytes(a, b):
    return np.array_equal(a.view(np.uint8), b.view(np.uint8))           # NaN-poisoned tails compare as bytes


@pytest.mark.parametrize("name,L", [("C1", 2), ("C2", 2), ("C3", 3), ("C4", 2), ("C5", 2)])
def test_configurations_bit_exact(gu, oracle_mod, name, L):
    cfg = gen.CONFIGS[name]
    inp, k, v = _layers(cfg, 60 + int(name[1]), L)
    path, alen = _paths(inp.parent, 61)
    dc = gu.DeviceCommit(cfg, k, v, inp.prefix_len, path, alen, inp.block_table)
    gk, gv, newp, status = dc.run()
    ek, ev, enp = _oracle_commit(oracle_mod, inp, k, v, path, alen)
    assert (status == 0).all()
    assert np.array_equal(newp, enp)
    assert _same_bytes(gk, ek) and _same_bytes(gv, ev)
    assert not _same_bytes(gk, k) or (alen == 0).all() or all((path[b, :alen[b] + 1] == np.arange(alen[b] + 1)).all() for b in range(len(alen)))


def _fuzz():
    cases = []
    k = 0
    for dtype, d in (("bf16", 64), ("bf16", 128), ("f32", 8), ("f32", 64), ("bf16", 8)):
        for paged in (False, True):
            for T in (1, 2, 17, 64):
                cases.append((dtype, d, paged, T, 1 + k % 4, 1 + k % 3, [0, 5, 16, 31, 100][k % 5], k))
                k += 1
    return cases


@pytest.mark.parametrize("dtype,d,paged,T,B,hkv,S,k", _fuzz())
def test_fuzz_bit_exact(gu, oracle_mod, dtype, d, paged, T, B, hkv, S, k):
    depth = min(7, max(1, T - 1))
    cfg = gen.Config(f"cf{k}", B, hkv, hkv, d, T, depth, 4, 100, 0.5, 1, dtype,
                     prefix=None if paged else [S + b for b in range(B)],
                     prefix_range=(S, S + 20) if paged else None, paged=paged)
    inp, kk, vv = _layers(cfg, 2000 + k, 1 + k % 3)
    path, alen = _paths(inp.parent, 3000 + k, full_every=2)
    if k % 5 == 0:
        alen[0] = 0
        path[0, 1:] = -1
    gk, gv, newp, status = gu.DeviceCommit(cfg, kk, vv, inp.prefix_len, path, alen, inp.block_table).run()
    ek, ev, enp = _oracle_commit(oracle_mod, inp, kk, vv, path, alen)
    assert (status == 0).all() and np.array_equal(newp, enp)
    assert _same_bytes(gk, ek) and _same_bytes(gv, ev)


def test_long_paths_cross_the_batch_of_eight(gu, oracle_mod):
    """Chain-like trees: up to 63 accepted tokens, several batches of moves per thread."""
    T, B = 64, 3
    parent = np.stack([gen.chain_tree(T), gen.random_tree(gen.rng(1, gen.STREAM_TREE), T, 40, 2),
                       gen.random_tree(gen.rng(2, gen.STREAM_TREE), T, 63, 2)])
    cfg = gen.Config("long", B, 2, 2, 128, T, 63, 2, 100, 0.5, 1, "bf16", prefix=[7, 300, 33])
    ins = gen.attention_inputs(cfg, 70, parent=parent)
    k, v = ins.k_bits[None].copy(), ins.v_bits[None].copy()
    path, alen = _paths(parent, 71, full_every=1)
    assert alen.max() >= 20
    gk, gv, newp, status = gu.DeviceCommit(cfg, k, v, ins.prefix_len, path, alen).run()
    ek, ev, enp = _oracle_commit(oracle_mod, ins, k, v, path, alen)
    assert (status == 0).all() and np.array_equal(newp, enp) and _same_bytes(gk, ek) and _same_bytes(gv, ev)


def test_bad_sequences_are_reported_and_left_alone(gu, oracle_mod):
    cfg = gen.Config("bad", 6, 2, 2, 64, 8, 4, 3, 10, 0.5, 1, "bf16", prefix_range=(20, 60), paged=True)
    inp, k, v = _layers(cfg, 80, 2)
    path, alen = _paths(inp.parent, 81, full_every=1)
    assert (alen >= 2).all()
    path[1, 0] = 1                                      # does not start at the root
    path[2, 2] = path[2, 1]                             # not increasing
    alen[3] = cfg.T                                     # accepted_len out of range
    prefix = inp.prefix_len.copy()
    prefix[4] = 10 ** 6                                 # beyond the cache
    table = inp.block_table.copy()
    table[5, int(inp.prefix_len[5]) // cfg.block_size] = 10 ** 7   # block id outside the pool
    inp2 = dataclasses.replace(inp, prefix_len=prefix, block_table=table)
    gk, gv, newp, status = gu.DeviceCommit(cfg, k, v, prefix, path, alen, table).run()
    assert list(status) == [0, 5, 5, 5, 3, 4], status
    ek, ev, enp = _oracle_commit(oracle_mod, inp2, k, v, path, alen, skip=(1, 2, 3, 4, 5))
    assert np.array_equal(newp, enp)                    # failed sequences keep their prefix length
    assert _same_bytes(gk, ek) and _same_bytes(gv, ev)  # ... and their rows


def test_accept_commit_verify_chain(gu, oracle_mod):
    """accept -> commit -> next verify step on the device equals the oracle's closed loop."""
    import torch
    cfg = gen.Config("chain", 2, 8, 2, 128, 24, 5, 3, 500, 0.8, 1, "bf16", prefix=[300, 77])
    inp = gen.attention_inputs(cfg, 90, poison_tail=False, extra_cap=40)
    acc = gen.accept_inputs(cfg, 90, parent=inp.parent)
    amax, alen, path, bonus, st = gu.run_accept(acc.logits, acc.tokens, acc.parent)
    assert (st == 0).all() and alen.max() >= 1
    dc = gu.DeviceCommit(cfg, inp.k_bits[None].copy(), inp.v_bits[None].copy(), inp.prefix_len, path, alen)
    gk, gv, newp, status = dc.run()
    assert (status == 0).all() and np.array_equal(newp, inp.prefix_len + alen + 1)
    # next step: a fresh tree of T2 nodes whose rows the "forward pass" writes behind the new prefix
    T2 = 9
    cfg2 = dataclasses.replace(cfg, T=T2, max_depth=3)
    nxt = gen.attention_inputs(cfg2, 91, prefix_len=newp, poison_tail=False, extra_cap=inp.k_cache.shape[2] - int(newp.max()) - T2)
    kb, vb = gk[0].copy(), gv[0].copy()
    for b in range(cfg.B):
        s = int(newp[b])
        kb[b, :, s:s + T2] = nxt.k_bits[b, :, s:s + T2]
        vb[b, :, s:s + T2] = nxt.v_bits[b, :, s:s + T2]
    dev_in = dataclasses.replace(nxt, k_bits=kb, v_bits=vb, k_cache=gen.bf16_bits_to_f32(kb), v_cache=gen.bf16_bits_to_f32(vb))
    got = gu.DeviceAttn(dev_in).run()
    # reference: context assembled from the ORIGINAL cache rows (old prefix + accepted nodes), never committed
    for b in range(cfg.B):
        S = int(inp.prefix_len[b])
        rows = np.concatenate([np.arange(S), S + path[b, :alen[b] + 1]])
        s = int(newp[b])
        kr = np.concatenate([inp.k_cache[b][:, rows], nxt.k_cache[b][:, s:s + T2]], axis=1)
        vr = np.concatenate([inp.v_cache[b][:, rows], nxt.v_cache[b][:, s:s + T2]], axis=1)
        ref = oracle_mod.tree_attention_seq(nxt.q[b], np.ascontiguousarray(kr), np.ascontiguousarray(vr), s, nxt.parent[b],
                                            nxt.scale, cfg.Hkv)
        gu.check_close(got[b], ref, 1.5e-3, 6e-3, what=f"sequence {b} after commit")
