"""Pins for the oracle's argmax and greedy acceptance (no GPU)."""
import itertools

import numpy as np
import pytest

import gen
from oracle import bruteforce


# ------------------------------------------------------------------ argmax

def test_argmax_planted_and_ties(oracle_mod):
    V = 1000
    row = -np.abs(gen.rng(1, 5).standard_normal(V).astype(np.float32)) - 1.0
    r = row.copy(); r[617] = 3.0
    assert oracle_mod.row_argmax(r) == 617
    r = row.copy(); r[100] = 3.0; r[900] = 3.0
    assert oracle_mod.row_argmax(r) == 100
    r = row.copy(); r[7] = -0.0; r[500] = 0.0
    assert oracle_mod.row_argmax(r) == 7
    r = row.copy(); r[7] = 0.0; r[500] = -0.0
    assert oracle_mod.row_argmax(r) == 7
    assert oracle_mod.row_argmax(np.full(V, 2.5, dtype=np.float32)) == 0
    r = row.copy(); r[V - 1] = 9.0
    assert oracle_mod.row_argmax(r) == V - 1
    r = row.copy(); r[0] = 9.0
    assert oracle_mod.row_argmax(r) == 0


def test_argmax_nan_rule(oracle_mod):
    """NaN never wins a strict '>' comparison; a NaN incumbent at index 0 is never
    replaced (this is what a plain left-to-right scan does)."""
    r = np.array([1.0, np.nan, 5.0, np.nan, 5.0], dtype=np.float32)
    assert oracle_mod.row_argmax(r) == 2
    r = np.array([np.nan, 1.0, 5.0], dtype=np.float32)
    assert oracle_mod.row_argmax(r) == 0
    r = np.full(9, np.nan, dtype=np.float32)
    assert oracle_mod.row_argmax(r) == 0
    r = np.array([-np.inf, -np.inf, -np.inf], dtype=np.float32)
    assert oracle_mod.row_argmax(r) == 0
    r = np.array([-np.inf, np.inf, np.inf], dtype=np.float32)
    assert oracle_mod.row_argmax(r) == 1


def test_argmax_matches_numpy_on_finite_rows(oracle_mod):
    lg = gen.rng(2, 5).standard_normal((50, 4099)).astype(np.float32)
    lg[:, ::7] = np.round(lg[:, ::7])                         # many exact ties
    lg[3, :] = np.round(lg[3, :])
    np.testing.assert_array_equal(oracle_mod.row_argmax(lg), np.argmax(lg, axis=1))


# ------------------------------------------------------------------ accept

def _all_trees(T):
    for tail in itertools.product(*[range(i) for i in range(1, T)]):
        yield np.array((-1,) + tail, dtype=np.int32)


def test_accept_equals_bruteforce_on_all_small_trees(oracle_mod):
    """Exhaustive over every tree with T <= 6 and random over T <= 12, with a tiny vocab
    so matches, mismatches and duplicate sibling tokens all occur."""
    g = gen.rng(3, 5)
    count = 0
    for T in range(1, 7):
        for parent in _all_trees(T):
            for _ in range(3):
                amax = g.integers(0, 3, T).astype(np.int32)
                draft = g.integers(0, 3, T).astype(np.int32)
                rc, alen, path, bonus = oracle_mod.tree_accept_from_argmax(amax, draft, parent)
                assert rc == oracle_mod.OK
                bl, bp, bb = bruteforce.accept_bruteforce(amax, draft, parent)
                assert (alen, list(path[:alen + 1]), bonus) == (bl, bp, bb)
                assert (path[alen + 1:] == -1).all()
                count += 1
    for seed in range(300):
        gg = gen.rng(seed, 6)
        T = int(gg.integers(7, 13))
        parent = gen.random_tree(gg, T, int(gg.integers(2, 6)), 4)
        amax = gg.integers(0, 2, T).astype(np.int32)
        draft = gg.integers(0, 2, T).astype(np.int32)
        rc, alen, path, bonus = oracle_mod.tree_accept_from_argmax(amax, draft, parent)
        bl, bp, bb = bruteforce.accept_bruteforce(amax, draft, parent)
        assert (alen, list(path[:alen + 1]), bonus) == (bl, bp, bb)
    assert count > 400


def test_accept_forced_full_path_and_zero(oracle_mod):
    for seed in range(20):
        g = gen.rng(seed, 7)
        T = 40
        parent = gen.random_tree(g, T, 6, 4)
        _, _, depth = oracle_mod.tree_mask(parent)
        draft = gen.draft_tokens(g, parent, 5000)
        leaf = int(np.argmax(depth))                        # first deepest node
        chain = []
        j = leaf
        while j != -1:
            chain.append(j); j = int(parent[j])
        chain.reverse()
        amax = np.full(T, 6000, dtype=np.int32)            # matches no draft token
        for a, b in zip(chain[:-1], chain[1:]):
            amax[a] = draft[b]
        amax[leaf] = 4242
        rc, alen, path, bonus = oracle_mod.tree_accept_from_argmax(amax, draft, parent)
        assert alen == depth[leaf] and list(path[:alen + 1]) == chain and bonus == 4242
        amax[:] = 6000
        amax[0] = 77
        rc, alen, path, bonus = oracle_mod.tree_accept_from_argmax(amax, draft, parent)
        assert alen == 0 and path[0] == 0 and (path[1:] == -1).all() and bonus == 77


def test_accept_structural_invariants_on_generated_inputs(oracle_mod):
    cfg = gen.Config("a", 6, 1, 1, 8, 30, 5, 4, 500, 0.7, 1, "f32", prefix=[4] * 6)
    ai = gen.accept_inputs(cfg, 9)
    amax, alen, path, bonus = oracle_mod.tree_accept(ai.logits, ai.tokens, ai.parent)
    np.testing.assert_array_equal(amax, np.argmax(ai.logits, axis=2))
    assert alen.max() > 0
    for b in range(cfg.B):
        p = path[b]
        L = alen[b]
        assert p[0] == 0
        for k in range(L):
            assert ai.parent[b][p[k + 1]] == p[k]
            assert ai.tokens[b][p[k + 1]] == amax[b][p[k]]
        best = p[L]
        assert bonus[b] == amax[b][best]
        kids = [i for i in range(cfg.T) if ai.parent[b][i] == best]
        assert all(ai.tokens[b][c] != amax[b][best] for c in kids)


def test_accept_duplicate_sibling_tokens_tie_goes_to_lowest_index(oracle_mod):
    parent = np.array([-1, 0, 0, 1, 2], dtype=np.int32)
    draft = np.array([0, 5, 5, 9, 9], dtype=np.int32)       # siblings 1,2 share a token
    amax = np.array([5, 9, 9, 1, 2], dtype=np.int32)
    rc, alen, path, bonus = oracle_mod.tree_accept_from_argmax(amax, draft, parent)
    assert alen == 2 and list(path[:3]) == [0, 1, 3] and bonus == 1


def test_accept_chain_mean_length_statistic(oracle_mod):
    """On a chain where each link matches independently with probability pi the expected
    accepted length is sum_{k=1..D} pi^k (loose statistical check of the generator's
    planting rule together with the walk)."""
    D, pi, V, n = 6, 0.7, 64, 600
    parent = gen.chain_tree(D + 1)
    tot = 0
    for s in range(n):
        tok = gen.draft_tokens(gen.rng(s, gen.STREAM_TOKENS), parent, V)
        lg = gen.logits_with_plants(gen.rng(s, gen.STREAM_LOGITS), gen.rng(s, gen.STREAM_PLANT),
                                    parent, tok, V, pi)
        _, alen, _, _ = oracle_mod.tree_accept(lg[None], tok[None], parent[None])
        tot += int(alen[0])
    # an unplanted link still matches by chance with probability 1/V
    pe = pi + (1 - pi) / V
    expect = sum(pe ** k for k in range(1, D + 1))
    assert abs(tot / n - expect) < 0.2


def test_accept_rejects_invalid_tree(oracle_mod):
    rc, *_ = oracle_mod.tree_accept_from_argmax([0, 0], [0, 0], [-1, 1])
    assert rc == oracle_mod.BAD_PARENT
