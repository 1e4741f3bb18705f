"""Pins for the oracle's tree-masked attention (no GPU).

Each test ties oracle_tree_attention to something it does not compute itself: a library
causal-attention routine, a closed form from the paper, hand-worked numbers, or an
invariant that a plausible mistake (wrong mask bit, dropped scale, transposed operand,
wrong GQA mapping, wrong paging arithmetic) would break."""
import json
import math
import os

import numpy as np
import pytest
import torch

import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, *shape):
    return gen.rng(seed, 99).standard_normal(shape).astype(np.float32)


def test_hand_worked_tree(oracle_mod):
    g = json.load(open(os.path.join(GOLDEN, "tiny_tree_attention.json")))
    kp = np.log(np.array(g["prefix_keys_exp"]))
    kt = np.log(np.array(g["tree_keys_exp"]))
    k = np.concatenate([kp, kt]).astype(np.float64)
    v = np.array(g["prefix_values"] + g["tree_values"], dtype=np.float32)
    k32 = k.astype(np.float32)
    T = len(g["parent"])
    q = np.ones((T, 1, 1), dtype=np.float32)
    out = oracle_mod.tree_attention_seq(q, k32.reshape(1, -1, 1), v.reshape(1, -1, 1), len(kp),
                                        g["parent"], 1.0, 1)
    exp = np.array([n / d for n, d in g["expected_num_den"]])
    # keys are fp32 roundings of ln(.), so weights carry ~1e-7 relative error
    np.testing.assert_allclose(out[:, 0, 0], exp, rtol=5e-7)
    # the sibling must not leak: with node 1 visible to node 2 the answer would be 370/11
    assert abs(out[2, 0, 0] - 370.0 / 11.0) > 1.0


@pytest.mark.parametrize("S,T,Hq,Hkv,d", [(37, 9, 4, 2, 16), (0, 12, 2, 2, 8), (100, 1, 3, 1, 32)])
def test_chain_tree_is_causal_attention(oracle_mod, S, T, Hq, Hkv, d):
    """A chain-shaped tree sees prefix + all earlier tree nodes + itself: the last T rows
    of ordinary causal attention over S+T tokens (torch's fp64 SDPA, is_causal)."""
    n = S + T
    k = _rand(1, Hkv, n, d)
    v = _rand(2, Hkv, n, d)
    q_all = _rand(3, n, Hq, d)
    scale = 0.37
    out = oracle_mod.tree_attention_seq(q_all[S:], k, v, S, gen.chain_tree(T), scale, Hkv)
    g = Hq // Hkv
    tq = torch.from_numpy(q_all).double().permute(1, 0, 2)                 # [Hq, n, d]
    tk = torch.from_numpy(k).double().repeat_interleave(g, dim=0)
    tv = torch.from_numpy(v).double().repeat_interleave(g, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    ref = ref.permute(1, 0, 2).numpy()[S:]
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)


def test_single_node_is_decode_attention(oracle_mod):
    S, Hq, Hkv, d = 77, 6, 3, 16
    k = _rand(4, Hkv, S + 1, d)
    v = _rand(5, Hkv, S + 1, d)
    q = _rand(6, 1, Hq, d)
    scale = 1.0 / math.sqrt(d)
    out = oracle_mod.tree_attention_seq(q, k, v, S, [-1], scale, Hkv)
    tq = torch.from_numpy(q).double()[0]                                    # [Hq, d]
    for h in range(Hq):
        kv = h // (Hq // Hkv)
        w = torch.softmax(torch.from_numpy(k[kv]).double() @ tq[h] * scale, dim=0)
        ref = (w[:, None] * torch.from_numpy(v[kv]).double()).sum(0).numpy()
        np.testing.assert_allclose(out[0, h], ref, rtol=1e-10, atol=1e-12)


def test_eq3_redundant_keys_closed_form(oracle_mod):
    """Paper Eq. 3-4: R identical keys (score A) and one unique key (score B)."""
    cases = json.load(open(os.path.join(GOLDEN, "eq3_cases.json")))["cases"]
    d = 4
    for c in cases:
        R = c["R"]
        A = math.log(c["A_is_ln"]) if "A_is_ln" in c else c["A"]
        B = math.log(c["B_is_ln"]) if "B_is_ln" in c else c["B"]
        # q = e_0; redundant key s = A e_0, unique key t = B e_0 + junk on other axes
        q = np.zeros((1, 1, d)); q[0, 0, 0] = 1.0
        s = np.zeros(d); s[0] = A
        t = np.array([B, 3.0, -2.0, 0.5])
        v_s = np.array([1.0, -1.0, 2.0, 0.0])
        v_t = np.array([-4.0, 8.0, 0.5, 16.0])
        # R redundant = R-1 prefix copies + the single tree node's own key; unique in prefix
        pos_u = (R - 1) // 2
        keys = [s] * (R - 1)
        vals = [v_s] * (R - 1)
        keys.insert(pos_u, t)
        vals.insert(pos_u, v_t)
        keys.append(s)
        vals.append(v_s)
        k = np.array(keys, dtype=np.float64)[None]
        v = np.array(vals, dtype=np.float64)[None]
        k32 = k.astype(np.float32)
        out = oracle_mod.tree_attention_seq(q.astype(np.float32), k32, v.astype(np.float32), R, [-1], 1.0, 1)
        a = c["alpha_unique"]
        # fp32 storage of ln(.) perturbs the weights by ~1e-7 relative
        np.testing.assert_allclose(out[0, 0], a * v_t + (1 - a) * v_s, rtol=1e-6, atol=1e-6)
    # Eq. 4: output tends to the redundant value as R grows
    prev = None
    for R in (1, 10, 100, 1000, 10000):
        k = np.zeros((1, R + 1, d), dtype=np.float32)
        v = np.tile(v_s.astype(np.float32), (R + 1, 1))[None].copy()
        k[0, 0] = [1.0, 0, 0, 0]
        v[0, 0] = v_t
        out = oracle_mod.tree_attention_seq(q.astype(np.float32), k, v, R, [-1], 1.0, 1)
        err = np.abs(out[0, 0] - v_s).max()
        assert prev is None or err < prev
        prev = err
    assert prev < 1e-2


def test_zero_keys_give_mean_of_visible_values(oracle_mod):
    """With all scores equal the output is the plain mean over exactly the visible set:
    S prefix tokens plus depth+1 tree tokens (pins the visible count and which V rows)."""
    S, T, Hq, Hkv, d = 13, 10, 2, 1, 5
    parent = gen.random_tree(gen.rng(7, 1), T, 4, 3)
    _, mask, depth = oracle_mod.tree_mask(parent)
    k = np.zeros((Hkv, S + T, d), dtype=np.float32)
    v = _rand(8, Hkv, S + T, d)
    q = _rand(9, T, Hq, d)
    out = oracle_mod.tree_attention_seq(q, k, v, S, parent, 0.3, Hkv)
    for i in range(T):
        anc = []
        j = i
        while j != -1:
            anc.append(j)
            j = int(parent[j])
        rows = list(range(S)) + [S + a for a in anc]
        assert len(rows) == S + depth[i] + 1
        ref = v[0, rows].astype(np.float64).mean(0)
        for h in range(Hq):
            np.testing.assert_allclose(out[i, h], ref, rtol=1e-12, atol=1e-13)


def _needle_setup(seed=11):
    S, T, Hq, Hkv, d = 5, 9, 2, 1, 8
    parent = np.array([-1, 0, 0, 1, 1, 2, 3, 3, 5], dtype=np.int32)
    k = _rand(seed, Hkv, S + T, d)
    v = _rand(seed + 1, Hkv, S + T, d)
    q = _rand(seed + 2, T, Hq, d)
    return S, T, Hq, Hkv, d, parent, q, k, v


def test_needle_on_non_ancestor_is_invisible(oracle_mod):
    S, T, Hq, Hkv, d, parent, q, k, v = _needle_setup()
    base = oracle_mod.tree_attention_seq(q, k, v, S, parent, 0.5, Hkv)
    _, mask, _ = oracle_mod.tree_mask(parent)
    for i in range(T):
        for j in range(T):
            if int(mask[i]) >> j & 1:
                continue
            k2, v2 = k.copy(), v.copy()
            k2[0, S + j] = 50.0 * q[i, 0]
            v2[0, S + j] = 1e3
            out = oracle_mod.tree_attention_seq(q, k2, v2, S, parent, 0.5, Hkv)
            assert np.array_equal(out[i], base[i])
            k2[0, S + j] = np.nan
            v2[0, S + j] = np.inf
            out = oracle_mod.tree_attention_seq(q, k2, v2, S, parent, 0.5, Hkv)
            assert np.array_equal(out[i], base[i])


def test_needle_on_ancestor_dominates(oracle_mod):
    S, T, Hq, Hkv, d, parent, q, k, v = _needle_setup()
    _, mask, _ = oracle_mod.tree_mask(parent)
    for i in range(T):
        for j in range(T):
            if not (int(mask[i]) >> j & 1):
                continue
            k2, v2 = k.copy(), v.copy()
            k2[0, S + j] = 50.0 * q[i, 0]
            v2[0, S + j] = 1e3
            out = oracle_mod.tree_attention_seq(q, k2, v2, S, parent, 0.5, Hkv)
            np.testing.assert_allclose(out[i, 0], 1e3, rtol=1e-6)
    # a prefix needle is seen by every node
    k2, v2 = k.copy(), v.copy()
    k2[0, 2] = 50.0 * q[4, 1]
    v2[0, 2] = -7.0
    out = oracle_mod.tree_attention_seq(q, k2, v2, S, parent, 0.5, Hkv)
    np.testing.assert_allclose(out[4, 1], -7.0, rtol=1e-6)


def test_cache_beyond_tree_is_never_read(oracle_mod):
    inp = gen.attention_inputs(gen.CONFIGS["C1"], 5, poison_tail=True)
    assert np.isnan(inp.k_cache[0, 0, int(inp.prefix_len[0]) + inp.cfg.T:]).all()
    out = oracle_mod.tree_attention(inp)
    assert np.isfinite(out).all()


def test_output_in_convex_hull_of_visible_values(oracle_mod):
    S, T, Hq, Hkv, d, parent, q, k, v = _needle_setup(21)
    out = oracle_mod.tree_attention_seq(q, k, v, S, parent, 0.5, Hkv)
    _, mask, _ = oracle_mod.tree_mask(parent)
    for i in range(T):
        rows = list(range(S)) + [S + j for j in range(T) if int(mask[i]) >> j & 1]
        lo, hi = v[0, rows].min(0), v[0, rows].max(0)
        for h in range(Hq):
            assert (out[i, h] >= lo - 1e-12).all() and (out[i, h] <= hi + 1e-12).all()


def test_gqa_equals_mha_with_repeated_heads(oracle_mod):
    S, T, Hq, Hkv, d = 19, 7, 8, 2, 8
    parent = gen.random_tree(gen.rng(31, 1), T, 3, 3)
    k, v, q = _rand(32, Hkv, S + T, d), _rand(33, Hkv, S + T, d), _rand(34, T, Hq, d)
    out = oracle_mod.tree_attention_seq(q, k, v, S, parent, 0.4, Hkv)
    g = Hq // Hkv
    out2 = oracle_mod.tree_attention_seq(q, np.repeat(k, g, axis=0), np.repeat(v, g, axis=0), S, parent, 0.4, Hq)
    assert np.array_equal(out, out2)
    # heads of different groups must differ (would catch h % g instead of h / g)
    assert not np.allclose(out[:, 0], out[:, g])


def test_prefix_permutation_invariance(oracle_mod):
    S, T, Hq, Hkv, d = 23, 6, 2, 1, 8
    parent = gen.random_tree(gen.rng(41, 1), T, 3, 3)
    k, v, q = _rand(42, Hkv, S + T, d), _rand(43, Hkv, S + T, d), _rand(44, T, Hq, d)
    out = oracle_mod.tree_attention_seq(q, k, v, S, parent, 0.4, Hkv)
    perm = np.concatenate([gen.rng(45, 1).permutation(S), np.arange(S, S + T)])
    out2 = oracle_mod.tree_attention_seq(q, k[:, perm], v[:, perm], S, parent, 0.4, Hkv)
    np.testing.assert_allclose(out, out2, rtol=1e-12, atol=1e-14)


def test_tree_relabelling_permutes_rows(oracle_mod):
    S, T, Hq, Hkv, d = 9, 8, 2, 1, 8
    parent = np.array([-1, 0, 0, 1, 1, 2, 2, 3], dtype=np.int32)
    # swap labels of the sibling pair (1,2) together with their subtrees' parents
    relabel = np.array([0, 2, 1, 5, 6, 3, 4, 7])             # new index of old node
    # keep topological order: new parent array
    newp = np.empty(T, dtype=np.int32)
    for old in range(T):
        newp[relabel[old]] = -1 if parent[old] < 0 else relabel[parent[old]]
    assert all(newp[i] < i for i in range(1, T))
    k, v, q = _rand(52, Hkv, S + T, d), _rand(53, Hkv, S + T, d), _rand(54, T, Hq, d)
    out = oracle_mod.tree_attention_seq(q, k, v, S, parent, 0.4, Hkv)
    inv = np.argsort(relabel)                                    # old index at new position
    k2, v2 = k.copy(), v.copy()
    k2[:, S:] = k[:, S + inv]
    v2[:, S:] = v[:, S + inv]
    out2 = oracle_mod.tree_attention_seq(q[inv], k2, v2, S, newp, 0.4, Hkv)
    np.testing.assert_allclose(out2, out[inv], rtol=1e-12, atol=1e-14)


def test_paged_equals_contiguous(oracle_mod):
    cfg = gen.Config("p", 3, 4, 2, 16, 11, 4, 3, 100, 0.5, 1, "f32", prefix_range=(5, 70), paged=True)
    inp = gen.attention_inputs(cfg, 3)
    out = oracle_mod.tree_attention(inp)
    bs = cfg.block_size
    for b in range(cfg.B):
        n = int(inp.prefix_len[b]) + cfg.T
        nb = (n + bs - 1) // bs
        ids = inp.block_table[b, :nb]
        kc = inp.k_cache[ids].transpose(1, 0, 2, 3).reshape(cfg.Hkv, nb * bs, cfg.d)
        vc = inp.v_cache[ids].transpose(1, 0, 2, 3).reshape(cfg.Hkv, nb * bs, cfg.d)
        ref = oracle_mod.tree_attention_seq(inp.q[b], kc, vc, int(inp.prefix_len[b]), inp.parent[b],
                                            inp.scale, cfg.Hkv)
        assert np.array_equal(out[b], ref)
    assert np.isfinite(out).all()


def test_scale_and_operand_orientation(oracle_mod):
    """Doubling K equals doubling the scale (pins that scale multiplies q.k), and a
    one-hot query picks out one key coordinate (pins the dot product's orientation)."""
    S, T, Hq, Hkv, d = 6, 3, 1, 1, 4
    parent = gen.chain_tree(T)
    k, v = _rand(61, Hkv, S + T, d), _rand(62, Hkv, S + T, d)
    q = np.zeros((T, Hq, d), dtype=np.float32)
    q[:, 0, 2] = 1.0
    a = oracle_mod.tree_attention_seq(q, 2 * k, v, S, parent, 0.7, Hkv)
    b = oracle_mod.tree_attention_seq(q, k, v, S, parent, 1.4, Hkv)
    np.testing.assert_allclose(a, b, rtol=1e-12)
    n = S + 1
    w = np.exp(1.4 * k[0, :n, 2].astype(np.float64))
    ref = (w[:, None] * v[0, :n]).sum(0) / w.sum()
    np.testing.assert_allclose(b[0, 0], ref, rtol=1e-12)
