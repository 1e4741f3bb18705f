"""GPU parity: draft-tree construction (vs_draft_expand, vs_draft_tree_build) against the oracle.

Tokens, parents and the final tree are integer work and must match bit for bit. Scores are
fp32 on the GPU (log-sum-exp merged from 4096-entry chunks) and fp64 in the oracle: they must
agree to SCORE_TOL, derived from |score| <= ~40 with a relative error of a few fp32 ulps
(2^-23 * 40 * 4 ~ 2e-5). The next frontier is decided by comparing scores: where the oracle's
gap at the cut exceeds 2 * SCORE_TOL the kept set must be the oracle's; closer than that, the
two sets may differ only by candidates within the tolerance of the cut.
"""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu

SCORE_TOL = 3e-5


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def _grow_both(gu, oracle_mod, seed, B, V, K, D, mutate=None, **kw):
    """D expansion steps on the GPU, each checked against the oracle run on the GPU's own frontier
    (so a knife-edge swap at one level cannot cascade into a spurious mismatch at the next)."""
    cap = K + (D - 1) * K * K
    dd = gu.DeviceDraft(B, K, cap)
    nf = nc = None
    for level in range(D):
        F = 1 if level == 0 else nf.shape[1]
        logits = np.stack([gen.draft_logits(seed, b, level, F, V) for b in range(B)])
        if mutate is not None:
            mutate(level, logits)
        base = dd.M
        cum_h = np.zeros((B, F), np.float32) if nc is None else nc.cpu().numpy()
        fc_h = np.full((B, F), -1, np.int32) if nf is None else nf.cpu().numpy()
        nf, nc = dd.expand(logits, nc, nf, **kw)
        tok = dd.tok.cpu().numpy()[:, base:base + F * K]
        sc = dd.score.cpu().numpy()[:, base:base + F * K]
        par = dd.par.cpu().numpy()[:, base:base + F * K]
        nf_h, nc_h = nf.cpu().numpy(), nc.cpu().numpy()
        for b in range(B):
            rc, o_tok, o_sc, o_fr, gap = oracle_mod.draft_expand_seq(logits[b], cum_h[b], K)
            assert rc == 0
            np.testing.assert_array_equal(tok[b], o_tok)
            np.testing.assert_allclose(sc[b], o_sc, rtol=0, atol=SCORE_TOL)
            np.testing.assert_array_equal(par[b], np.repeat(fc_h[b], K))
            got = nf_h[b] - base
            assert (np.diff(got) > 0).all() and got.min() >= 0 and got.max() < F * K
            np.testing.assert_array_equal(nc_h[b], sc[b][got])           # the scores handed on are the stored ones
            if gap > 2 * SCORE_TOL:
                np.testing.assert_array_equal(got, o_fr)
            else:
                cut = o_sc[o_fr].min()
                for c in set(got.tolist()) ^ set(o_fr.tolist()):
                    assert abs(o_sc[c] - cut) <= 2 * SCORE_TOL
    return dd


def _check_build(gu, oracle_mod, dd, N, root_token=None):
    parent, tokens, node_cand, num, status = dd.build(N, root_token)
    again = dd.build(N, root_token)                                                     # nothing may depend on timing
    assert all((a == b).all() for a, b in zip(again, (parent, tokens, node_cand, num, status)))
    tok, sc, par = dd.tok.cpu().numpy(), dd.score.cpu().numpy(), dd.par.cpu().numpy()
    for b in range(dd.B):
        rc, o_parent, o_tokens, o_cand = oracle_mod.draft_tree_build_seq(
            tok[b, :dd.M], sc[b, :dd.M], par[b, :dd.M], N, -1 if root_token is None else root_token[b])
        assert rc == 0 and status[b] == 0 and num[b] == len(o_parent)
        T = num[b]
        np.testing.assert_array_equal(parent[b, :T], o_parent)
        np.testing.assert_array_equal(tokens[b, :T], o_tokens)
        np.testing.assert_array_equal(node_cand[b, :T], o_cand)
        assert (parent[b, T:] == -1).all() and (tokens[b, T:] == -1).all() and (node_cand[b, T:] == -1).all()
    return parent, tokens, num


def test_paper_configuration(gu, oracle_mod):
    """Appendix A: K = 8 kept per expansion, depth 3, N = 30 draft tokens; Qwen-sized vocabulary."""
    dd = _grow_both(gu, oracle_mod, 1, 3, 152064, 8, 3)
    assert dd.M == 136
    parent, tokens, num = _check_build(gu, oracle_mod, dd, 30, root_token=[11, 12, 13])
    assert (num == 31).all() and (tokens[:, 0] == [11, 12, 13]).all()
    mask, depth, status, _ = gu.run_mask(parent)                        # feeds the verification path as is
    assert (status == 0).all() and depth.max() <= 3 and (np.diff(depth, axis=1) >= 0).all()


@pytest.mark.parametrize("V,K,D,N", [(1000, 4, 4, 20), (4096, 8, 2, 63), (4097, 16, 2, 40), (8191, 1, 6, 6),
                                     (32000, 10, 3, 59), (50, 16, 3, 30), (16, 16, 2, 63)])
def test_shapes(gu, oracle_mod, V, K, D, N):
    dd = _grow_both(gu, oracle_mod, 10 + K, 4, V, K, D)
    _check_build(gu, oracle_mod, dd, N)


@pytest.mark.parametrize("V,K", [(152064, 16), (300000, 8), (270001, 16)])
def test_long_rows(gu, oracle_mod, V, K):
    """Rows whose merged chunk lists do not fit a wave's registers (chunks x K > 512: the lists are
    re-read per extracted entry) and rows of more than 64 chunks (chunk statistics in several passes)."""
    dd = _grow_both(gu, oracle_mod, 40 + K, 2, V, K, 2)
    _check_build(gu, oracle_mod, dd, 30)


def test_equal_logits_take_the_lower_token_id(gu, oracle_mod):
    def plateau(level, logits):
        logits[:, :, ::5] = np.float32(20.0)                            # many equal maxima, across chunks too
    dd = _grow_both(gu, oracle_mod, 21, 3, 9000, 8, 3, mutate=plateau)
    tok = dd.tok.cpu().numpy()
    assert (tok[:, :8] == np.arange(0, 40, 5)).all()
    _check_build(gu, oracle_mod, dd, 30)


def test_minus_infinity_logits(gu, oracle_mod):
    def ban(level, logits):
        logits[:, :, 100:] = -np.inf                                    # only 100 tokens allowed
        logits[:, :, :3] = -np.inf
    dd = _grow_both(gu, oracle_mod, 22, 2, 6000, 8, 2, mutate=ban)
    tok = dd.tok.cpu().numpy()[:, :dd.M]
    assert (tok >= 3).all() and (tok < 100).all()


@pytest.mark.parametrize("ld,offset", [(1003, 0), (1000, 1), (1008, 4)])
def test_unaligned_rows_and_padding(gu, oracle_mod, ld, offset):
    dd = _grow_both(gu, oracle_mod, 31, 3, 1000, 8, 3, ld=ld, offset_elems=offset)
    _check_build(gu, oracle_mod, dd, 30)


def test_build_on_handmade_candidates(gu, oracle_mod):
    """Ties between a parent and a child with probability 1, fewer candidates than N, prefixes of M."""
    import torch
    dd = gu.DeviceDraft(2, 2, 8)
    dd.tok[:] = torch.tensor([[7, 8, 9, 1, 2, 3, 4, 5]] * 2, dtype=torch.int32)
    dd.score[:] = torch.tensor([[-1.0, -0.5, -0.5, -1.0, -3.0, -0.75, -9.0, -0.75],
                                [-0.1, -0.2, -0.3, -0.4, -0.5, -0.6, -0.7, -0.8]])
    dd.par[:] = torch.tensor([[-1, -1, 1, 0, 0, 2, 2, 5]] * 2, dtype=torch.int32)
    for M in (1, 3, 8):
        dd.M = M
        for N in (1, 2, 5, 63):
            _check_build(gu, oracle_mod, dd, N)


@pytest.mark.parametrize("M,N", [(2048, 63), (2047, 40), (1025, 63), (257, 30), (66, 63), (65, 5)])
def test_build_at_large_candidate_counts(gu, oracle_mod, M, N):
    """Up to the maximum the build accepts: random forests whose scores fall along every parent
    chain (as cumulative log-probabilities do), with many exactly equal scores, at counts that are
    not multiples of the kernel's group sizes (4 scores per read, 64 candidates per ballot, 256 per
    round)."""
    import torch
    r = np.random.default_rng(M * 131 + N)
    B = 2
    tok = r.integers(0, 50000, size=(B, M)).astype(np.int32)
    par = np.empty((B, M), np.int32)
    sc = np.empty((B, M), np.float32)
    for b in range(B):
        for c in range(M):
            pc = -1 if (c == 0 or r.random() < 0.02) else int(r.integers(max(0, c - 300), c))
            par[b, c] = pc
            base = 0.0 if pc < 0 else float(sc[b, pc])
            sc[b, c] = np.float32(base - float(r.choice([0.0, 0.25, 0.5, 1.0, 3.0])))   # ties, also with the parent
    dd = gu.DeviceDraft(B, 16, M)
    dd.tok[:] = torch.from_numpy(tok)
    dd.score[:] = torch.from_numpy(sc)
    dd.par[:] = torch.from_numpy(par)
    dd.M = M
    _check_build(gu, oracle_mod, dd, N)


def test_build_reports_malformed_candidates(gu, oracle_mod):
    import torch
    dd = gu.DeviceDraft(4, 2, 3)
    dd.M = 3
    dd.tok[:] = 1
    dd.score[:] = torch.tensor([[-1.0, -2.0, -3.0], [-1.0, -2.0, -3.0], [-3.0, -1.0, -0.5], [-1.0, -2.0, -3.0]])
    dd.par[:] = torch.tensor([[-1, 0, 1], [-1, 1, 0], [-1, -1, 0], [-2, 0, 0]], dtype=torch.int32)
    parent, tokens, node_cand, num, status = dd.build(2)
    exp = [oracle_mod.draft_tree_build_seq([1, 1, 1], dd.score[b].cpu().numpy(), dd.par[b].cpu().numpy(), 2)[0]
           for b in range(4)]
    assert exp == [0, oracle_mod.BAD_PARENT, oracle_mod.BAD_PARENT, oracle_mod.BAD_PARENT]
    assert status.tolist() == [0, 6, 6, 6] and num.tolist() == [3, 0, 0, 0]
    assert (parent[1:] == -1).all()


def test_draft_then_verify_closed_loop(gu, oracle_mod):
    """The built tree and tokens go straight into greedy acceptance: with target logits that put
    their maximum on one child's token along a chosen path, that path is what gets accepted."""
    dd = _grow_both(gu, oracle_mod, 41, 2, 3000, 4, 3)
    parent, tokens, num = _check_build(gu, oracle_mod, dd, 20, root_token=[5, 6])
    B, T = parent.shape
    V = 3000
    logits = np.stack([gen.rng(41, gen.STREAM_LOGITS, b).standard_normal((T, V), dtype=np.float32) for b in range(B)])
    want = []
    for b in range(B):
        node, path = 0, [0]
        while True:
            kids = np.nonzero(parent[b] == node)[0]
            if len(kids) == 0:
                break
            nxt = int(kids[-1])
            logits[b, node, tokens[b, nxt]] = 50.0
            node = nxt
            path.append(node)
        want.append(path)
    amax, alen, path, bonus, status = gu.run_accept(logits, tokens, parent)
    o = oracle_mod.tree_accept(logits, tokens, parent)
    np.testing.assert_array_equal(alen, o[1])
    np.testing.assert_array_equal(path, o[2])
    for b in range(B):
        assert path[b, :alen[b] + 1].tolist() == want[b]
