"""GPU parity: tree masks, row argmax and acceptance must match the oracle bit for bit."""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def test_mask_matches_oracle(gu, oracle_mod):
    rows = [gen.chain_tree(64), gen.star_tree(64)]
    for s in range(30):
        g = gen.rng(s, gen.STREAM_TREE)
        rows.append(gen.random_tree(g, 64, int(g.integers(1, 9)), 64))
    parent = np.stack(rows)
    mask, depth, status, _ = gu.run_mask(parent)
    assert (status == 0).all()
    for b in range(parent.shape[0]):
        rc, m, d = oracle_mod.tree_mask(parent[b])
        assert rc == 0
        np.testing.assert_array_equal(mask[b], m)
        np.testing.assert_array_equal(depth[b], d)


@pytest.mark.parametrize("T", [1, 2, 7, 31, 60])
def test_mask_small_trees(gu, oracle_mod, T):
    parent = np.stack([gen.random_tree(gen.rng(s, 1), T, 6, 4) if T > 1 else np.array([-1], dtype=np.int32)
                       for s in range(5)])
    mask, depth, status, _ = gu.run_mask(parent)
    assert (status == 0).all()
    for b in range(5):
        _, m, d = oracle_mod.tree_mask(parent[b])
        np.testing.assert_array_equal(mask[b], m)
        np.testing.assert_array_equal(depth[b], d)


def test_mask_invalid_trees_report_status(gu, oracle_mod):
    parent = np.array([[-1, 0, 1, 2], [0, 0, 1, 2], [-1, 0, 2, 1], [-1, -1, 0, 0], [-1, 0, 0, 7]], dtype=np.int32)
    mask, depth, status, _ = gu.run_mask(parent)
    exp = [oracle_mod.tree_validate(p) for p in parent]
    assert exp == [0, oracle_mod.BAD_ROOT, oracle_mod.BAD_PARENT, oracle_mod.BAD_PARENT, oracle_mod.BAD_PARENT]
    np.testing.assert_array_equal(status, exp)          # the two code sets coincide by value
    assert (mask[1:] == 0).all() and (depth[1:] == 0).all()
    assert int(mask[0][3]) == 0b1111


def _check_accept(gu, oracle_mod, logits, tokens, parent, **kw):
    amax, alen, path, bonus, status = gu.run_accept(logits, tokens, parent, **kw)
    o_amax, o_alen, o_path, o_bonus = oracle_mod.tree_accept(logits, tokens, parent)
    assert (status == 0).all()
    np.testing.assert_array_equal(amax, o_amax)
    np.testing.assert_array_equal(alen, o_alen)
    np.testing.assert_array_equal(path, o_path)
    np.testing.assert_array_equal(bonus, o_bonus)
    return alen


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_accept_configs(gu, oracle_mod, name):
    """All five configurations at their stated sizes (C4: its own seed and planted-match
    probability 0.6; C5: 16 independent trees over the full 152064-token vocabulary, 584 MB of logits)."""
    cfg = gen.CONFIGS[name]
    ai = gen.accept_inputs(cfg, 100 + int(name[1]))
    assert ai.logits.shape == (cfg.B, cfg.T, cfg.V)
    alen = _check_accept(gu, oracle_mod, ai.logits, ai.tokens, ai.parent)
    assert alen.shape == (cfg.B,)
    if cfg.B >= 8:
        assert alen.max() >= 1 and len(set(alen.tolist())) > 1


def test_accept_huge_vocab(gu, oracle_mod):
    """More than 64 chunks per row: the walk kernel fetches a second batch of chunk results."""
    import dataclasses
    cfg = dataclasses.replace(gen.CONFIGS["C1"], V=300001, T=9, B=2, max_depth=4, prefix=[4, 4])
    ai = gen.accept_inputs(cfg, 321)
    _check_accept(gu, oracle_mod, ai.logits, ai.tokens, ai.parent)


@pytest.mark.parametrize("V,ld,off", [(1, 1, 0), (5, 5, 0), (1000, 1000, 0), (1000, 1003, 0), (1000, 1000, 1),
                                      (8192, 8192, 0), (8193, 8196, 0), (20001, 20004, 0), (33000, 33000, 3)])
def test_accept_shapes_strides_alignment(gu, oracle_mod, V, ld, off):
    import dataclasses
    cfg = dataclasses.replace(gen.CONFIGS["C1"], V=V, T=13, B=3, max_depth=4, prefix=[4, 4, 4])
    ai = gen.accept_inputs(cfg, 7 + V)
    _check_accept(gu, oracle_mod, ai.logits, ai.tokens, ai.parent, ld=ld, offset_elems=off)


def test_argmax_ties_zeros_nan(gu, oracle_mod):
    V, T = 20000, 16
    parent = gen.random_tree(gen.rng(5, 1), T, 4, 4)[None]
    tokens = gen.draft_tokens(gen.rng(5, 2), parent[0], V)[None]
    lg = -np.abs(gen.rng(5, 3).standard_normal((1, T, V)).astype(np.float32)) - 1.0
    lg[0, 0, 100] = 3.0; lg[0, 0, 19000] = 3.0                     # equal maxima far apart
    lg[0, 1, 9000] = -0.0; lg[0, 1, 17000] = 0.0                   # signed zeros
    lg[0, 2, 9000] = 0.0; lg[0, 2, 17000] = -0.0
    lg[0, 3, :] = 2.5                                              # constant row
    lg[0, 4, V - 1] = 9.0                                          # last element
    lg[0, 5, 0] = np.nan; lg[0, 5, 77] = 50.0                      # NaN in column 0 is never displaced
    lg[0, 6, 5] = np.nan; lg[0, 6, 8191] = 4.0; lg[0, 6, 8192] = 4.0   # tie across a chunk boundary
    lg[0, 7, :] = np.nan
    lg[0, 8, :] = -np.inf
    lg[0, 9, :] = -np.inf; lg[0, 9, 12345] = -1e30
    lg[0, 10, 1::2] = np.nan; lg[0, 10, 4000] = 7.0
    lg[0, 11, 8191] = np.inf; lg[0, 11, 16000] = np.inf
    _check_accept(gu, oracle_mod, lg, tokens, parent)


def test_accept_duplicate_siblings_and_forced_paths(gu, oracle_mod):
    parent = np.array([[-1, 0, 0, 1, 2, 3, 4]], dtype=np.int32)
    tokens = np.array([[0, 5, 5, 9, 9, 3, 3]], dtype=np.int32)
    V = 64
    lg = np.zeros((1, 7, V), dtype=np.float32)
    lg[0, 0, 5] = 1; lg[0, 1, 9] = 1; lg[0, 2, 9] = 1; lg[0, 3, 3] = 1; lg[0, 4, 3] = 1; lg[0, 5, 11] = 1; lg[0, 6, 12] = 1
    amax, alen, path, bonus, status = gu.run_accept(lg, tokens, parent)
    assert alen[0] == 3 and list(path[0][:4]) == [0, 1, 3, 5] and bonus[0] == 11
    _check_accept(gu, oracle_mod, lg, tokens, parent)
    lg[0, 0, 5] = 0; lg[0, 0, 6] = 1                                # nothing matches at the root
    amax, alen, path, bonus, status = gu.run_accept(lg, tokens, parent)
    assert alen[0] == 0 and path[0][0] == 0 and (path[0][1:] == -1).all() and bonus[0] == 6


def test_accept_invalid_tree_status(gu):
    parent = np.array([[-1, 0, 0], [-1, 0, 2], [1, 0, 0]], dtype=np.int32)
    tokens = np.zeros((3, 3), dtype=np.int32)
    lg = gen.rng(1, 1).standard_normal((3, 3, 50)).astype(np.float32)
    amax, alen, path, bonus, status = gu.run_accept(lg, tokens, parent)
    assert list(status) == [0, 2, 1]
    np.testing.assert_array_equal(amax, np.argmax(lg, axis=2))
    assert (path[1:] == -1).all() and (bonus[1:] == -1).all()
