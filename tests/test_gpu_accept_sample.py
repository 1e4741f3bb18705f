"""GPU parity: stochastic tree acceptance (vs_tree_accept_sample) against the oracle.

The decisions compare a probability - fp32 on the GPU, fp64 in the oracle - with a uniform
that both sides receive as input, so an outcome is unique only where no uniform lies within
the fp32 path's error of its threshold. Every GPU outcome must pass the oracle's outcome check
(oracle_tree_accept_sample_check: the walk replayed along the claimed path in fp64, each
comparison allowed to be off by EPS), and where the oracle's `margin` (the closest call of its
own walk) exceeds EPS the outcome must equal the oracle's exactly. EPS bounds the fp32 error of
a probability or of a normalised cumulative sum: hardware exp2 of an argument known to ~2e-6
relative, sums of <= 2^23 terms in chunks of 4096 merged pairwise, ~5e-6 in all; EPS is twice
that. Every test prints the largest deviation any comparison actually needed (`worst`).
With a large vocabulary single tokens weigh less than EPS (1 / 152064 = 6.6e-6), so the bonus
token may legitimately be a neighbour of the oracle's: there the exact-match floor is the number
of sequences whose margin exceeds EPS - which are checked one by one - and nothing more can be
demanded.
"""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu

EPS = 1e-5


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def _check(gu, oracle_mod, logits, tokens, parent, temperature, ua, ub, min_exact_frac=0.9, **kw):
    alen, path, bonus, status = gu.run_accept_sample(logits, tokens, parent, temperature, ua, ub, **kw)
    again = gu.run_accept_sample(logits, tokens, parent, temperature, ua, ub, **kw)     # nothing may depend on timing
    assert (again[0] == alen).all() and (again[1] == path).all() and (again[2] == bonus).all()
    ua64, ub64 = ua.astype(np.float64), ub.astype(np.float64)
    o_alen, o_path, o_bonus, margin = oracle_mod.tree_accept_sample(logits, tokens, parent, temperature, ua64, ub64)
    assert (status == 0).all()
    B, T, V = logits.shape
    exact, clear, worst_all = 0, 0, 0.0
    for b in range(B):
        rc, worst = oracle_mod.tree_accept_sample_check_seq(logits[b], tokens[b], parent[b], temperature, ua64[b],
                                                            ub64[b], alen[b], path[b], bonus[b], EPS)
        assert rc == 0, (b, alen[b], path[b], bonus[b], o_alen[b], o_path[b], o_bonus[b], worst, margin[b])
        worst_all = max(worst_all, float(worst))
        same = alen[b] == o_alen[b] and (path[b] == o_path[b]).all() and bonus[b] == o_bonus[b]
        if margin[b] > EPS:
            clear += 1
            assert same, (b, alen[b], o_alen[b], bonus[b], o_bonus[b], margin[b])
        exact += bool(same)
    print(f"accept_sample B={B} T={T} V={V} temperature={temperature}: worst deviation {worst_all:.3g} (EPS {EPS}), "
          f"{exact} of {B} equal the oracle's outcome, {clear} have a margin above EPS")
    assert exact >= max(clear, min_exact_frac * B - 1), f"only {exact} of {B} sequences equal the oracle's outcome"
    return alen, path, bonus, o_alen


def _case(seed, B, T, V, max_depth=6, max_children=4, spread=1.5):
    parent = np.stack([gen.random_tree(gen.rng(seed, gen.STREAM_TREE, b), T, min(max_depth, max(1, T - 1)),
                                       max_children) if T > 1 else np.array([-1], dtype=np.int32) for b in range(B)])
    tokens = np.stack([gen.draft_tokens(gen.rng(seed, gen.STREAM_TOKENS, b), parent[b], V) for b in range(B)])
    logits = np.stack([gen.logits_with_candidates(gen.rng(seed, gen.STREAM_LOGITS, b),
                                                  gen.rng(seed, gen.STREAM_CANDIDATE, b), parent[b], tokens[b], V,
                                                  spread) for b in range(B)])
    ua, ub = gen.uniforms(seed, B, T)
    return parent, tokens, logits, ua, ub


@pytest.mark.parametrize("temperature", [0.7, 1.0, 1.6])
@pytest.mark.parametrize("T,V", [(8, 1000), (13, 4096), (31, 4097), (60, 8191), (7, 40000)])
def test_matches_oracle_small_vocab(gu, oracle_mod, T, V, temperature):
    parent, tokens, logits, ua, ub = _case(100 + T, 24, T, V)
    alen, _, _, _ = _check(gu, oracle_mod, logits, tokens, parent, temperature, ua, ub)
    if temperature <= 1.0:                                     # (a hot softmax leaves the candidates little mass)
        assert alen.max() >= 1                                 # some candidate was accepted


def test_matches_oracle_qwen_vocab(gu, oracle_mod):
    """C3's acceptance shape: 60-node trees over a 152064-token vocabulary (several sequences)."""
    cfg = gen.CONFIGS["C3"]
    parent, tokens, logits, ua, ub = _case(3, 6, cfg.T, cfg.V)
    alen, _, _, _ = _check(gu, oracle_mod, logits, tokens, parent, 1.0, ua, ub, min_exact_frac=0.5)
    assert alen.max() >= 1


@pytest.mark.parametrize("T,V", [(8, 300000), (64, 270001)])
def test_matches_oracle_huge_vocab(gu, oracle_mod, T, V):
    """More than 64 chunks per row (a second batch of chunk statistics per thread), and - with 64
    nodes - more chunk statistics than the walk kernel keeps in LDS (it reads them from memory again)."""
    parent, tokens, logits, ua, ub = _case(200 + T, 2, T, V)
    _check(gu, oracle_mod, logits, tokens, parent, 1.0, ua, ub, min_exact_frac=0.5)


def test_single_node_tree_is_plain_sampling(gu, oracle_mod):
    parent, tokens, logits, ua, ub = _case(5, 16, 1, 5000)
    alen, path, _, _ = _check(gu, oracle_mod, logits, tokens, parent, 1.0, ua, ub)
    assert (alen == 0).all() and (path[:, 0] == 0).all()


def test_rejecting_a_dominant_token_resums_its_chunk(gu, oracle_mod):
    """A child whose token holds ~all of the mass is rejected (u above its probability): the
    subtraction cancels the chunk sum and the kernel has to sum the chunk afresh. Siblings that
    repeat the removed token or name a token outside the vocabulary have probability 0."""
    T, V, B = 6, 20000, 16
    parent = np.tile(np.array([-1, 0, 0, 0, 0, 1], dtype=np.int32), (B, 1))
    tokens = np.tile(np.array([0, 7000, 7000, V + 5, 123, 9], dtype=np.int32), (B, 1))
    logits = np.stack([gen.rng(11, gen.STREAM_LOGITS, b).standard_normal((T, V), dtype=np.float32) for b in range(B)])
    logits[:, 0, 7000] = 15.0           # p ~ 0.99 (background mass ~ V*sqrt(e)), and 99.8 % of its chunk
    logits[:, 0, 123] = 9.0             # after the removal: a real share of what is left
    ua, ub = gen.uniforms(11, B, T)
    ua[:, 1] = np.float32(0.9975)       # rejected all the same
    ua[:, 2] = 0.0                      # duplicate of the removed token: never accepted, even with u = 0
    ua[:, 3] = 0.0                      # outside the vocabulary: never accepted
    alen, path, bonus, _ = _check(gu, oracle_mod, logits, tokens, parent, 1.0, ua, ub, min_exact_frac=0.7)
    assert (path[:, 1] != 1).all() and (path[:, 1] != 2).all() and (path[:, 1] != 3).all()
    assert (bonus != 7000).all()
    assert (alen == 1).any() and (alen == 0).any()


def test_uniform_extremes(gu, oracle_mod):
    """u = 0 accepts the first child at every node (any positive probability passes) and draws the
    first token that has weight; the largest fp32 below 1 rejects every child here. These sit on
    the thresholds by construction, so the expected results are spelled out rather than gated
    by the oracle's margin."""
    parent, tokens, logits, ua, ub = _case(21, 12, 20, 6000)
    B, T, V = logits.shape
    alen, path, bonus, status = gu.run_accept_sample(logits, tokens, parent, 1.0, np.zeros_like(ua), np.zeros_like(ub))
    o_alen, o_path, o_bonus, _ = oracle_mod.tree_accept_sample(logits, tokens, parent, 1.0, np.zeros((B, T)),
                                                               np.zeros(B))
    assert (status == 0).all()
    np.testing.assert_array_equal(alen, o_alen)
    np.testing.assert_array_equal(path, o_path)
    np.testing.assert_array_equal(bonus, o_bonus)
    for b in range(B):
        for k in range(alen[b]):
            kids = np.nonzero(parent[b] == path[b][k])[0]
            assert path[b][k + 1] == kids.min()
        assert not (parent[b] == path[b][alen[b]]).any()      # the walk ended at a leaf
        assert bonus[b] == 0
    top = np.float32(1.0 - 2.0 ** -24)
    alen, _, bonus, status = gu.run_accept_sample(logits, tokens, parent, 1.0, np.full_like(ua, top),
                                                  np.full_like(ub, top))
    assert (status == 0).all() and (alen == 0).all()
    assert (bonus >= V - 64).all()      # the cumulative sum reaches 1 - 6e-8 of the mass in the last few tokens


def test_cold_temperature_is_the_greedy_rule(gu, oracle_mod):
    cfg = gen.CONFIGS["C1"]
    ai = gen.accept_inputs(cfg, 9, B=16, parent=np.stack([gen.draw_trees(cfg, 9 + b)[0] for b in range(16)]))
    ua, ub = gen.uniforms(9, 16, cfg.T)
    alen, path, bonus, status = gu.run_accept_sample(ai.logits, ai.tokens, ai.parent, 1e-6, ua, ub)
    _, g_alen, g_path, g_bonus, _ = gu.run_accept(ai.logits, ai.tokens, ai.parent)
    np.testing.assert_array_equal(alen, g_alen)
    np.testing.assert_array_equal(path, g_path)
    np.testing.assert_array_equal(bonus, g_bonus)
    o = oracle_mod.tree_accept(ai.logits, ai.tokens, ai.parent)
    np.testing.assert_array_equal(alen, o[1])


@pytest.mark.parametrize("ld,offset", [(1003, 0), (1000, 1), (1008, 4)])
def test_unaligned_rows_and_padding(gu, oracle_mod, ld, offset):
    parent, tokens, logits, ua, ub = _case(31, 8, 9, 1000)
    _check(gu, oracle_mod, logits, tokens, parent, 1.0, ua, ub, ld=ld, offset_elems=offset)


def test_banned_tokens_are_never_drawn(gu, oracle_mod):
    parent, tokens, logits, ua, ub = _case(41, 32, 5, 9000)
    banned = gen.rng(41, gen.STREAM_PLANT).random((9000,)) < 0.5
    logits[:, :, banned] = -np.inf
    _, _, bonus, _ = _check(gu, oracle_mod, logits, tokens, parent, 1.0, ua, ub)
    assert not banned[bonus].any()


def test_bonus_distribution_is_the_softmax(gu):
    """Independent of the oracle: with a root-only tree the call is plain sampling, so over many
    uniforms the drawn tokens follow softmax(logits / temperature) (chi-square, 49 dof)."""
    V, B, temperature = 50, 40000, 1.3
    row = (1.2 * gen.rng(51, gen.STREAM_LOGITS).standard_normal(V)).astype(np.float32)
    logits = np.broadcast_to(row, (B, 1, V)).copy()
    parent = np.full((B, 1), -1, dtype=np.int32)
    tokens = np.zeros((B, 1), dtype=np.int32)
    ua, ub = gen.uniforms(51, B, 1)
    alen, path, bonus, status = gu.run_accept_sample(logits, tokens, parent, temperature, ua, ub)
    assert (status == 0).all() and (alen == 0).all()
    z = row.astype(np.float64) / temperature
    p = np.exp(z - z.max())
    p /= p.sum()
    counts = np.bincount(bonus, minlength=V)
    chi2 = float(((counts - B * p) ** 2 / (B * p)).sum())
    assert chi2 < 95.0, chi2            # 49 dof: P(chi2 > 95) < 1e-4
    # and the draw is the inverse of the cumulative sum: monotone in u
    order = np.argsort(ub, kind="stable")
    assert (np.diff(bonus[order]) >= 0).all()


def test_accepted_child_distribution(gu):
    """Independent of the oracle: a root with three children; over many uniforms the first emitted
    token (an accepted child's, or the bonus) follows the root's softmax."""
    V, B = 12, 60000
    row = gen.rng(52, gen.STREAM_LOGITS).standard_normal((4, V)).astype(np.float32)
    logits = np.broadcast_to(row, (B, 4, V)).copy()
    parent = np.tile(np.array([-1, 0, 0, 0], dtype=np.int32), (B, 1))
    tokens = np.tile(np.array([0, 3, 8, 5], dtype=np.int32), (B, 1))
    ua, ub = gen.uniforms(52, B, 4)
    alen, path, bonus, status = gu.run_accept_sample(logits, tokens, parent, 1.0, ua, ub)
    assert (status == 0).all() and alen.max() == 1
    first = np.where(alen == 1, tokens[0][np.maximum(path[:, 1], 0)], bonus)
    z = row[0].astype(np.float64)
    p = np.exp(z - z.max())
    p /= p.sum()
    counts = np.bincount(first, minlength=V)
    chi2 = float(((counts - B * p) ** 2 / (B * p)).sum())
    assert chi2 < 40.0, chi2            # 11 dof: P(chi2 > 40) < 1e-4


def test_malformed_trees_report_status(gu):
    parent = np.array([[-1, 0, 1, 2], [0, 0, 1, 2], [-1, 0, 2, 1]], dtype=np.int32)
    tokens = np.zeros((3, 4), dtype=np.int32)
    logits = gen.rng(61, gen.STREAM_LOGITS).standard_normal((3, 4, 300), dtype=np.float32)
    ua, ub = gen.uniforms(61, 3, 4)
    alen, path, bonus, status = gu.run_accept_sample(logits, tokens, parent, 1.0, ua, ub)
    assert status.tolist() == [0, 1, 2]
    assert (path[1:] == -1).all() and (alen[1:] == 0).all() and (bonus[1:] == -1).all()


def test_repeated_calls_are_deterministic(gu):
    parent, tokens, logits, ua, ub = _case(71, 8, 30, 30000)
    a = gu.run_accept_sample(logits, tokens, parent, 1.0, ua, ub)
    b = gu.run_accept_sample(logits, tokens, parent, 1.0, ua, ub)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
