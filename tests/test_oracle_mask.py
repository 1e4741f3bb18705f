"""Pins for the oracle's tree validation and ancestor masks (no GPU)."""
import numpy as np
import pytest

import gen
from oracle import bruteforce


def test_chain_closed_form(oracle_mod):
    for T in (1, 2, 7, 33, 64):
        rc, mask, depth = oracle_mod.tree_mask(gen.chain_tree(T))
        assert rc == oracle_mod.OK
        for i in range(T):
            assert int(mask[i]) == (1 << (i + 1)) - 1
            assert depth[i] == i


def test_star_closed_form(oracle_mod):
    for T in (2, 9, 64):
        rc, mask, depth = oracle_mod.tree_mask(gen.star_tree(T))
        assert rc == oracle_mod.OK
        assert int(mask[0]) == 1 and depth[0] == 0
        for i in range(1, T):
            assert int(mask[i]) == (1 | (1 << i))
            assert depth[i] == 1


def test_structural_invariants_and_reachability(oracle_mod):
    for seed in range(40):
        g = gen.rng(seed, gen.STREAM_TREE)
        T = int(g.integers(1, 65)) if seed % 2 else int(g.integers(1, 13))
        D = int(g.integers(1, 8))
        parent = gen.random_tree(g, T, D, 64 if D < 3 else 4 + T // 8)
        rc, mask, depth = oracle_mod.tree_mask(parent)
        assert rc == oracle_mod.OK
        brute = bruteforce.reachability_mask(parent)
        for i in range(T):
            m = int(mask[i])
            assert m == brute[i]
            assert bin(m).count("1") == depth[i] + 1
            assert m >> i & 1
            assert m >> (i + 1) == 0          # only earlier nodes can be ancestors
            if i:
                p = int(parent[i])
                assert m >> p & 1
                assert m & ~(1 << i) == int(mask[p])
                assert depth[i] == depth[p] + 1


def test_paper_shaped_tree(oracle_mod):
    # Appendix A: 30 draft tokens, depth 3, 8 nodes per expansion
    for seed in range(5):
        parent = gen.topk_tree(gen.rng(seed, gen.STREAM_TREE))
        assert len(parent) == 31
        rc, mask, depth = oracle_mod.tree_mask(parent)
        assert rc == oracle_mod.OK
        assert depth.max() <= 3
        assert np.bincount(parent[1:], minlength=31).max() <= 8


@pytest.mark.parametrize("parent,code", [
    ([0], "BAD_ROOT"), ([-2], "BAD_ROOT"), ([-1, -1], "BAD_PARENT"), ([-1, 1], "BAD_PARENT"),
    ([-1, 0, 2], "BAD_PARENT"), ([-1, 0, 5], "BAD_PARENT"), ([-1, 0, -3], "BAD_PARENT"),
])
def test_invalid_trees(oracle_mod, parent, code):
    assert oracle_mod.tree_validate(np.array(parent, dtype=np.int32)) == getattr(oracle_mod, code)
    rc, _, _ = oracle_mod.tree_mask(np.array(parent, dtype=np.int32))
    assert rc == getattr(oracle_mod, code)
