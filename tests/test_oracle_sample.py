"""Pins for the oracle's stochastic tree acceptance (no GPU)."""
import json
import math
import os

import numpy as np
import pytest

import gen
from oracle import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _softmax64(row, temperature=1.0):
    z = np.asarray(row, dtype=np.float64) / temperature
    e = np.exp(z - z.max())
    return e / e.sum()


def _small_case(seed, T, V, max_children=3):
    g = gen.rng(seed, gen.STREAM_LOGITS)
    parent = gen.random_tree(gen.rng(seed, gen.STREAM_TREE), T, max_depth=min(4, max(1, T - 1)), max_children=max_children)
    draft = gen.draft_tokens(gen.rng(seed, gen.STREAM_TOKENS), parent, V)
    logits = (1.5 * g.standard_normal((T, V))).astype(np.float32)
    return parent, draft, logits


def test_hand_worked_example(oracle_mod):
    g = json.load(open(os.path.join(GOLDEN, "accept_sample_tiny.json")))
    logits = np.log(np.array(g["weights"], dtype=np.float64)).astype(np.float32)
    for c in g["cases"]:
        rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(logits, g["draft"], g["parent"], g["temperature"],
                                                                     c["u_accept"], c["u_bonus"])
        assert rc == 0 and alen == c["accepted_len"] and list(path) == c["path"] and bonus == c["bonus"], c["_why"]


@pytest.mark.parametrize("seed", range(8))
def test_rule_preserves_the_target_distribution_exactly(seed):
    """Enumerating every accept / reject outcome (bruteforce.py, independent of oracle.c): whatever
    node the walk stands on, the next emitted token - an accepted child's or the bonus - is
    distributed as the target's softmax at that node."""
    T, V = 7, 5
    parent, draft, logits = _small_case(seed, T, V)
    if seed % 2:                                        # duplicate sibling tokens must not break it
        kids = [c for c in range(1, T) if parent[c] == 0]
        if len(kids) >= 2:
            draft[kids[1]] = draft[kids[0]]
    p_rows = [_softmax64(logits[i]) for i in range(T)]
    dist = bruteforce.sample_output_distribution([list(p) for p in p_rows], draft, parent)
    assert abs(sum(dist.values()) - 1.0) < 1e-12

    def node_of(prefix):
        cur = 0
        for tok in prefix:
            nxt = [c for c in range(cur + 1, T) if parent[c] == cur and draft[c] == tok]
            cur = nxt[0]                                 # first sibling with that token (later duplicates have mass 0)
        return cur

    prefixes = {seq[:k] for seq in dist for k in range(len(seq))}
    for pre in prefixes:
        reach = sum(pr for seq, pr in dist.items() if seq[:len(pre)] == pre)
        node = node_of(pre)
        for y in range(V):
            got = sum(pr for seq, pr in dist.items() if seq[:len(pre) + 1] == pre + (y,))
            assert abs(got / reach - p_rows[node][y]) < 1e-12, (pre, y)


def test_oracle_agrees_with_enumeration_by_monte_carlo(oracle_mod):
    """The C oracle driven by random uniforms reproduces the enumerated sequence distribution
    (chi-square over every emitted sequence with expected count >= 20)."""
    T, V, N = 6, 5, 60000
    parent, draft, logits = _small_case(3, T, V)
    dist = bruteforce.sample_output_distribution([list(_softmax64(logits[i])) for i in range(T)], draft, parent)
    g = gen.rng(11, gen.STREAM_PATH)
    ua = g.random((N, T))
    ub = g.random(N)
    counts = {}
    for n in range(N):
        rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(logits, draft, parent, 1.0, ua[n], ub[n])
        key = tuple(int(draft[c]) for c in path[1:alen + 1]) + (bonus,)
        counts[key] = counts.get(key, 0) + 1
    assert set(counts) <= set(dist)
    chi2, dof = 0.0, 0
    for seq, pr in dist.items():
        if pr * N >= 20:
            chi2 += (counts.get(seq, 0) - pr * N) ** 2 / (pr * N)
            dof += 1
    assert dof >= 10
    assert chi2 < dof + 5 * math.sqrt(2 * dof), (chi2, dof)    # five sigma


@pytest.mark.parametrize("seed", range(10))
def test_cold_temperature_is_the_greedy_rule(oracle_mod, seed):
    cfg = gen.Config("cold", 1, 1, 1, 64, 20, 5, 3, 300, 0.7, 1, "bf16", prefix=[1])
    acc = gen.accept_inputs(cfg, seed)
    amax, alen_g, path_g, bonus_g = oracle_mod.tree_accept(acc.logits, acc.tokens, acc.parent)
    g = gen.rng(seed, gen.STREAM_PATH)
    ua = 0.01 + 0.98 * g.random(cfg.T)
    rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(acc.logits[0], acc.tokens[0], acc.parent[0], 1e-4, ua,
                                                                 0.01 + 0.98 * g.random())
    assert rc == 0 and alen == alen_g[0] and bonus == bonus_g[0]
    # the greedy oracle reports the deepest accepted node; the walk follows the first accepted child:
    # with distinct sibling tokens at most one child matches, so the paths coincide
    assert list(path) == list(path_g[0])


def test_uniform_extremes_and_duplicates(oracle_mod):
    parent = np.array([-1, 0, 0, 1, 1], dtype=np.int32)
    draft = np.array([0, 3, 3, 2, 1], dtype=np.int32)          # nodes 1 and 2 repeat token 3
    logits = np.zeros((5, 6), dtype=np.float32)
    # u = 0 accepts the first child with positive probability at every level
    rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(logits, draft, parent, 1.0, np.zeros(5), 0.0)
    assert (alen, list(path), bonus) == (2, [0, 1, 3, -1, -1], 0)
    # u just below 1 rejects everything (all probabilities are 1/6 .. 1/4); tokens 3 is removed once
    rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(logits, draft, parent, 1.0, np.full(5, 0.999), 0.999)
    assert (alen, list(path)) == (0, [0, -1, -1, -1, -1]) and bonus == 5
    # node 1 rejected, its duplicate node 2 can never be accepted, not even with u = 0
    ua = np.array([0, 0.9, 0.0, 0, 0])
    rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(logits, draft, parent, 1.0, ua, 0.5)
    assert alen == 0 and bonus != 3
    # a certain token (probability 1 in fp64) is accepted for every u < 1
    hot = logits.copy(); hot[0, 3] = 800.0
    rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(hot, draft, parent, 1.0, np.full(5, 0.999999), 0.3)
    assert alen >= 1 and path[1] == 1


@pytest.mark.parametrize("seed", range(6))
def test_bonus_is_the_inverse_cdf_in_index_order(oracle_mod, seed):
    V = 1000
    g = gen.rng(seed, gen.STREAM_LOGITS)
    logits = (2.0 * g.standard_normal((1, V))).astype(np.float32)
    tau = [1.0, 0.5, 2.0][seed % 3]
    for u in (0.0, 0.25, 0.5, 0.987, 0.999999):
        rc, alen, path, bonus, margin = oracle_mod.tree_accept_sample_seq(logits, [0], [-1], tau, [0.0], u)
        p = _softmax64(logits[0], tau)
        want = int(np.searchsorted(np.cumsum(p), u * p.sum(), side="right"))
        assert alen == 0 and (bonus == min(want, V - 1) or margin < 1e-12)


def test_margin_flags_knife_edges(oracle_mod):
    logits = np.log(np.array([[4, 2, 1, 1], [1, 1, 1, 1]], dtype=np.float64)).astype(np.float32)
    rc, alen, path, bonus, margin = oracle_mod.tree_accept_sample_seq(logits, [0, 1], [-1, 0], 1.0, [0, 0.25 + 1e-9], 0.3)
    assert margin < 1e-6
    rc, alen, path, bonus, margin = oracle_mod.tree_accept_sample_seq(logits, [0, 1], [-1, 0], 1.0, [0, 0.6], 0.3)
    assert alen == 0 and 0.02 < margin < 0.36


def test_malformed_inputs(oracle_mod):
    logits = np.zeros((3, 4), dtype=np.float32)
    assert oracle_mod.tree_accept_sample_seq(logits, [0, 1, 2], [0, 0, 0], 1.0, np.zeros(3), 0.5)[0] == oracle_mod.BAD_ROOT
    assert oracle_mod.tree_accept_sample_seq(logits, [0, 1, 2], [-1, 0, 0], 0.0, np.zeros(3), 0.5)[0] == oracle_mod.BAD_SIZE
    # a draft token outside the vocabulary has probability 0
    rc, alen, path, bonus, _ = oracle_mod.tree_accept_sample_seq(logits, [0, 9, -4], [-1, 0, 0], 1.0, np.zeros(3), 0.5)
    assert rc == 0 and alen == 0


@pytest.mark.parametrize("seed", range(12))
def test_outcome_check_admits_exactly_the_rule_s_outcome(oracle_mod, seed):
    """oracle_tree_accept_sample_check with eps = 0: the walk's own result passes, every
    neighbouring claim (another bonus token, a shorter or longer path, a sibling) fails."""
    T, V = 9, 40
    parent, draft, logits = _small_case(50 + seed, T, V)
    g = gen.rng(seed, gen.STREAM_PATH)
    ua, ub = g.random(T), float(g.random())
    rc, alen, path, bonus, margin = oracle_mod.tree_accept_sample_seq(logits, draft, parent, 1.0, ua, ub)
    chk = lambda a, p, bo, eps=0.0: oracle_mod.tree_accept_sample_check_seq(logits, draft, parent, 1.0, ua, ub, a, p,
                                                                           bo, eps)
    rc, worst = chk(alen, path, bonus)
    assert rc == 0 and worst <= 0.0 and abs(-worst - margin) < 1e-12   # the closest call is the margin
    for other in range(V):
        if other != bonus:
            assert chk(alen, path, other)[0] != 0
    if alen > 0:                                                # stopping early: the accepted child was "rejected"
        short = path.copy(); short[alen] = -1
        for bo in range(V):
            assert chk(alen - 1, short, bo)[0] != 0
    kids = [c for c in range(T) if parent[c] == path[alen]]
    for c in kids:                                              # going further: a rejected child was "accepted"
        longer = path.copy(); longer[alen + 1] = c
        assert all(chk(alen + 1, longer, bo)[0] != 0 for bo in range(V))
    bad = path.copy(); bad[0] = 1
    assert chk(alen, bad, bonus)[0] != 0
    stray = path.copy(); stray[T - 1] = 3 if alen < T - 1 else stray[T - 1]
    if alen < T - 1:
        assert chk(alen, stray, bonus)[0] != 0                  # entries past the path must be -1


def test_outcome_check_tolerance_admits_only_knife_edges(oracle_mod):
    """Root row weights 4:2:1:1 (probabilities .5 .25 .125 .125), child token 1 (p = .25)."""
    logits = np.log(np.array([[4, 2, 1, 1], [1, 1, 1, 1]], dtype=np.float64)).astype(np.float32)
    draft, parent = [0, 1], [-1, 0]
    acc, rej = np.array([0, 1, -1], dtype=np.int32)[:2], np.array([0, -1], dtype=np.int32)
    chk = lambda ua1, ub, a, p, bo, eps: oracle_mod.tree_accept_sample_check_seq(
        logits, draft, parent, 1.0, [0.0, ua1], ub, a, p, bo, eps)[0]
    # u = .25 + 1e-7 rejects exactly; "accepted" is admitted with eps = 1e-6 but not with 1e-8
    assert chk(0.25 + 1e-7, 0.1, 0, rej, 0, 0.0) == 0
    assert chk(0.25 + 1e-7, 0.1, 1, acc, 0, 0.0) != 0
    assert chk(0.25 + 1e-7, 0.1, 1, acc, 0, 1e-6) == 0
    assert chk(0.25 + 1e-7, 0.1, 1, acc, 0, 1e-8) != 0
    # a clear rejection is never admitted as accepted, whatever small eps
    assert chk(0.6, 0.1, 1, acc, 0, 1e-3) != 0
    # bonus after the rejection: residual 4:0:1:1 -> cumulative 2/3, 2/3, 5/6, 1; token 1 has no weight
    assert chk(0.6, 0.5, 0, rej, 0, 0.0) == 0
    assert chk(0.6, 0.7, 0, rej, 2, 0.0) == 0
    assert chk(0.6, 0.7, 0, rej, 1, 1.0) != 0                   # removed token: never, whatever eps
    assert chk(0.6, 2 / 3 + 1e-7, 0, rej, 0, 0.0) != 0
    assert chk(0.6, 2 / 3 + 1e-7, 0, rej, 0, 1e-6) == 0         # within eps of token 0's bracket
    assert chk(0.6, 2 / 3 + 1e-7, 0, rej, 3, 1e-6) != 0
