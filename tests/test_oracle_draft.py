"""Pins for the oracle's draft-tree construction (no GPU)."""
import itertools
import json
import math
import os

import numpy as np
import pytest

import gen
from oracle import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _log_softmax64(rows):
    z = np.asarray(rows, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))


def test_hand_worked_example(oracle_mod):
    g = json.load(open(os.path.join(GOLDEN, "draft_tree_tiny.json")))
    K, N = g["K"], g["N"]
    l0 = np.log(np.array(g["level0_probs"])).astype(np.float32)
    rc, tok, sc, fr, gap = oracle_mod.draft_expand_seq(l0, np.zeros(1, np.float32), K)
    assert rc == 0 and tok.tolist() == g["level0_tokens"] and fr.tolist() == g["level0_frontier"]
    np.testing.assert_allclose(np.exp(sc), g["level0_scores_exp"], rtol=1e-6)
    assert gap == math.inf                                      # nothing dropped at the first level
    l1 = np.log(np.array(g["level1_probs"])).astype(np.float32)
    rc, tok1, sc1, fr1, gap1 = oracle_mod.draft_expand_seq(l1, sc[fr].astype(np.float32), K)
    assert rc == 0 and tok1.tolist() == g["level1_tokens"] and fr1.tolist() == g["level1_frontier"]
    np.testing.assert_allclose(np.exp(sc1), g["level1_scores_exp"], rtol=1e-6)
    assert abs(gap1 - (math.log(0.2) - math.log(0.15))) < 1e-6
    rc, parent, tokens, node_cand = oracle_mod.draft_tree_build_seq(
        g["all_tokens"], np.log(g["all_scores_exp"]).astype(np.float32), g["all_parent"], N, root_token=9)
    assert rc == 0
    assert parent.tolist() == g["tree_parent"] and tokens.tolist() == g["tree_tokens"]
    assert node_cand.tolist() == g["tree_node_cand"]


@pytest.mark.parametrize("seed", range(6))
def test_expand_against_numpy_and_bruteforce(oracle_mod, seed):
    F, V, K = [(1, 50, 4), (3, 200, 3), (8, 1000, 8), (5, 37, 5), (2, 9, 9), (8, 64, 1)][seed]
    lg = gen.draft_logits(seed, 0, 1, F, V)
    if seed % 2:                                                # equal logits: lower token id first
        lg[:, ::3] = np.float32(1.25)
    cum = (-gen.rng(seed, gen.STREAM_DRAFT, 999).random(F) * 3).astype(np.float32)
    rc, tok, sc, fr, gap = oracle_mod.draft_expand_seq(lg, cum, K)
    assert rc == 0
    # tokens: numpy's stable argsort of the negated logits; scores: an independent log-softmax
    want_tok = np.argsort(-lg.astype(np.float64), axis=1, kind="stable")[:, :K]
    np.testing.assert_array_equal(tok.reshape(F, K), want_tok)
    lsm = _log_softmax64(lg)
    want_sc = cum.astype(np.float64)[:, None] + np.take_along_axis(lsm, want_tok, axis=1)
    np.testing.assert_allclose(sc.reshape(F, K), want_sc, rtol=0, atol=1e-12)
    # frontier: pure-Python sort
    b_tok, b_sc, b_keep = bruteforce.expand_frontier_bruteforce([list(map(float, r)) for r in lg],
                                                                [float(c) for c in cum], K)
    assert tok.tolist() == b_tok and fr.tolist() == b_keep
    kept = set(fr.tolist())
    dropped = [sc[c] for c in range(F * K) if c not in kept]
    if dropped:
        assert abs(gap - (min(sc[c] for c in kept) - max(dropped))) < 1e-12 and gap >= 0
    else:
        assert gap == math.inf
    # log-probabilities: every candidate scores below its frontier node, rows sum to <= 1
    assert (sc.reshape(F, K) <= cum[:, None] + 1e-12).all()
    assert (np.exp(sc.reshape(F, K) - cum[:, None].astype(np.float64)).sum(axis=1) <= 1 + 1e-12).all()


def test_expand_ties_between_frontier_nodes_keep_the_lower_candidate(oracle_mod):
    lg = np.zeros((2, 4), dtype=np.float32)                     # all candidates score ln(1/4)
    rc, tok, sc, fr, gap = oracle_mod.draft_expand_seq(lg, np.zeros(2, np.float32), 2)
    assert tok.tolist() == [0, 1, 0, 1] and fr.tolist() == [0, 1] and gap == 0.0


def test_expand_rejects_bad_sizes(oracle_mod):
    lg = np.zeros((2, 4), dtype=np.float32)
    assert oracle_mod.draft_expand_seq(lg, np.zeros(2, np.float32), 5)[0] == oracle_mod.BAD_SIZE    # K > V
    assert oracle_mod.draft_expand_seq(lg, np.zeros(2, np.float32), 0)[0] == oracle_mod.BAD_SIZE


def _grow(oracle_mod, seed, V, K, D):
    """Runs D expansion steps with the oracle; returns the candidate arrays of all levels."""
    toks, scs, pars = [], [], []
    frontier_cand, cum = [-1], np.zeros(1, np.float32)
    for level in range(D):
        F = len(frontier_cand)
        lg = gen.draft_logits(seed, 0, level, F, V)
        rc, tok, sc, fr, _ = oracle_mod.draft_expand_seq(lg, cum, K)
        assert rc == 0
        base = len(toks)
        toks += tok.tolist()
        scs += sc.astype(np.float32).tolist()
        pars += [frontier_cand[c // K] for c in range(F * K)]
        frontier_cand = [base + int(c) for c in fr]
        cum = sc[fr].astype(np.float32)
    return np.array(toks, np.int32), np.array(scs, np.float32), np.array(pars, np.int32)


@pytest.mark.parametrize("seed", range(10))
def test_tree_build_maximises_total_probability_over_closed_subsets(oracle_mod, seed):
    """The claim behind the rule (EAGLE-2): the N best-scored candidates form the parent-closed
    set of N nodes with the largest total probability. Checked by exhaustive search."""
    V, K, D, N = [(6, 2, 3, 4), (8, 3, 2, 5), (5, 2, 4, 6), (7, 2, 3, 3), (9, 3, 2, 7)][seed % 5]
    tok, sc, par = _grow(oracle_mod, 100 + seed, V, K, D)
    M = len(tok)
    assert M == K + (D - 1) * K * K and M <= 14
    rc, parent, tokens, node_cand = oracle_mod.draft_tree_build_seq(tok, sc, par, N, root_token=5)
    assert rc == 0 and len(parent) == N + 1
    assert tuple(node_cand[1:].tolist()) == bruteforce.best_closed_subset(sc.astype(np.float64).tolist(), par.tolist(), N)
    # structure: a valid tree in parent-before-child order whose edges are the candidates' edges
    assert oracle_mod.tree_validate(parent) == 0 and tokens[0] == 5 and node_cand[0] == -1
    assert (np.diff(node_cand[1:]) > 0).all()
    for t in range(1, N + 1):
        c = node_cand[t]
        assert tokens[t] == tok[c]
        assert (parent[t] == 0 and par[c] == -1) or node_cand[parent[t]] == par[c]


def test_tree_build_paper_shape(oracle_mod):
    """Appendix A's configuration: 8 kept per expansion, depth 3, 30 draft tokens -> 8 + 2*64 = 136
    candidates, a 31-node tree of depth <= 3 that the mask oracle accepts."""
    tok, sc, par = _grow(oracle_mod, 7, 5000, 8, 3)
    assert len(tok) == 136
    rc, parent, tokens, node_cand = oracle_mod.draft_tree_build_seq(tok, sc, par, 30, root_token=1)
    assert rc == 0 and len(parent) == 31
    rc, mask, depth = oracle_mod.tree_mask(parent)
    assert rc == 0 and depth.max() <= 3 and (np.diff(depth) >= 0).all()       # level order
    order = np.argsort(-sc, kind="stable")[:30]
    assert sorted(order.tolist()) == node_cand[1:].tolist()


def test_tree_build_single_candidate_per_step_is_a_chain(oracle_mod):
    tok, sc, par = _grow(oracle_mod, 3, 40, 1, 6)
    rc, parent, tokens, node_cand = oracle_mod.draft_tree_build_seq(tok, sc, par, 6)
    assert rc == 0 and parent.tolist() == [-1, 0, 1, 2, 3, 4, 5] and tokens[1:].tolist() == tok.tolist()


def test_tree_build_fewer_candidates_than_requested(oracle_mod):
    rc, parent, tokens, node_cand = oracle_mod.draft_tree_build_seq([4, 5], [-0.1, -2.0], [-1, 0], 10)
    assert rc == 0 and parent.tolist() == [-1, 0, 1] and tokens.tolist() == [-1, 4, 5]


def test_tree_build_ties_prefer_the_earlier_candidate_hence_the_parent(oracle_mod):
    # child (cand 2) has probability 1 under its parent (cand 1): equal scores; N = 2 must keep the parent
    rc, parent, tokens, node_cand = oracle_mod.draft_tree_build_seq([7, 8, 9], [-1.0, -0.5, -0.5], [-1, -1, 1], 2)
    assert rc == 0 and node_cand.tolist() == [-1, 1, 2] and parent.tolist() == [-1, 0, 1]


def test_tree_build_rejects_malformed_candidates(oracle_mod):
    assert oracle_mod.draft_tree_build_seq([1, 2], [-1.0, -2.0], [-1, 1], 2)[0] == oracle_mod.BAD_PARENT   # self parent
    assert oracle_mod.draft_tree_build_seq([1, 2], [-1.0, -2.0], [-2, 0], 2)[0] == oracle_mod.BAD_PARENT
    # a child scoring above its parent (not a sum of log-probabilities) leaves the set unclosed
    assert oracle_mod.draft_tree_build_seq([1, 2, 3], [-3.0, -1.0, -0.5], [-1, -1, 0], 2)[0] == oracle_mod.BAD_PARENT
    assert oracle_mod.draft_tree_build_seq([1], [-1.0], [-1], 64)[0] == oracle_mod.BAD_SIZE
