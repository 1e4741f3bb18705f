"""Pins for the oracle's vision-adaptor compression attention (no GPU)."""
import json
import math
import os

import numpy as np
import pytest
import torch

import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_example(oracle_mod):
    g = json.load(open(os.path.join(GOLDEN, "compress_attention_tiny.json")))
    k = np.stack([np.log(np.array(g["k_first_component_is_ln_of"], dtype=np.float64)),
                  np.array(g["k_second_component"])], axis=1)[None]            # [Hkv=1, 3, 2]
    q = np.array(g["q"])[:, None, :]                                            # [2, 1, 2]
    v = np.array(g["v"])[None]
    out = oracle_mod.compress_attention_seq(q, k, v, 3, 1.0, 1)
    np.testing.assert_allclose(out[:, 0], g["out"], rtol=1e-6)                  # ln(.) is stored in fp32


@pytest.mark.parametrize("nq,Hq,Hkv,d,r", [(1, 2, 2, 8, 5), (16, 8, 2, 16, 77), (64, 4, 4, 32, 300), (7, 14, 2, 64, 129)])
def test_against_an_independent_softmax_attention(oracle_mod, nq, Hq, Hkv, d, r):
    g = gen.rng(nq * 1000 + r, gen.STREAM_Q)
    cap = r + 9
    q = g.standard_normal((nq, Hq, d), dtype=np.float32)
    k = g.standard_normal((Hkv, cap, d), dtype=np.float32)
    v = g.standard_normal((Hkv, cap, d), dtype=np.float32)
    k[:, r:] = np.nan                                                           # slots beyond r are never read
    v[:, r:] = np.nan
    scale = 1.0 / math.sqrt(d)
    out = oracle_mod.compress_attention_seq(q, k, v, r, scale, Hkv)
    grp = Hq // Hkv
    tq = torch.from_numpy(q.astype(np.float64)).permute(1, 0, 2)                # [Hq, nq, d]
    tk = torch.from_numpy(k[:, :r].astype(np.float64)).repeat_interleave(grp, dim=0)
    tv = torch.from_numpy(v[:, :r].astype(np.float64)).repeat_interleave(grp, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)
    # weights are a convex combination: every output channel lies inside the hull of the values
    for h in range(Hq):
        vv = v[h // grp, :r].astype(np.float64)
        assert (out[:, h] <= vv.max(axis=0) + 1e-12).all() and (out[:, h] >= vv.min(axis=0) - 1e-12).all()


def test_eq3_redundant_image_embeddings_closed_form(oracle_mod):
    """Paper Eq. 3-4 in the setting it is written for: R identical (redundant) image embeddings
    scoring A and one unique embedding scoring B; the unique one gets e^B / (R e^A + e^B)."""
    cases = json.load(open(os.path.join(GOLDEN, "eq3_cases.json")))["cases"]
    d = 4
    for c in cases:
        R = c["R"]
        A = math.log(c["A_is_ln"]) if "A_is_ln" in c else c["A"]
        B = math.log(c["B_is_ln"]) if "B_is_ln" in c else c["B"]
        q = np.zeros((1, 1, d)); q[0, 0, 0] = 1.0
        s = np.zeros(d); s[0] = A
        t = np.array([B, 3.0, -2.0, 0.5])
        v_s = np.array([1.0, -1.0, 2.0, 0.0])
        v_t = np.array([-4.0, 8.0, 0.5, 16.0])
        keys, vals = [s] * R, [v_s] * R
        keys.insert(R // 3, t)
        vals.insert(R // 3, v_t)
        out = oracle_mod.compress_attention_seq(q, np.array(keys)[None], np.array(vals)[None], R + 1, 1.0, 1)
        a = c["alpha_unique"]
        np.testing.assert_allclose(out[0, 0], a * v_t + (1 - a) * v_s, rtol=1e-6, atol=1e-6)


def test_zero_keys_average_exactly_r_values(oracle_mod):
    g = gen.rng(5, gen.STREAM_V)
    for r in (1, 2, 31, 100):
        v = g.standard_normal((1, r + 4, 3), dtype=np.float32)
        k = np.zeros_like(v)
        out = oracle_mod.compress_attention_seq(np.ones((2, 1, 3), np.float32), k, v, r, 0.7, 1)
        np.testing.assert_allclose(out[0, 0], v[0, :r].astype(np.float64).mean(axis=0), rtol=1e-12, atol=1e-14)


def test_paged_equals_contiguous_and_rejects_empty_images(oracle_mod):
    g = gen.rng(9, gen.STREAM_K)
    Hkv, d, r, bs = 2, 8, 45, 16
    k = g.standard_normal((Hkv, 48, d), dtype=np.float32)
    v = g.standard_normal((Hkv, 48, d), dtype=np.float32)
    q = g.standard_normal((3, 4, d), dtype=np.float32)
    table = np.array([2, 0, 3], dtype=np.int32)
    pool_k = np.full((5, Hkv, bs, d), np.nan, dtype=np.float32)
    pool_v = np.full((5, Hkv, bs, d), np.nan, dtype=np.float32)
    for i, blk in enumerate(table):
        pool_k[blk] = k[:, i * bs:(i + 1) * bs]
        pool_v[blk] = v[:, i * bs:(i + 1) * bs]
    a = oracle_mod.compress_attention_seq(q, k, v, r, 0.3, Hkv)
    b = oracle_mod.compress_attention_seq(q, pool_k, pool_v, r, 0.3, Hkv, block_table=table, block_size=bs)
    assert np.array_equal(a, b)
    with pytest.raises(ValueError):
        oracle_mod.compress_attention_seq(q, k, v, 0, 0.3, Hkv)
