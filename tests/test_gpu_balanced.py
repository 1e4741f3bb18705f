"""GPU parity of the balanced schedule (ragged batches: every workgroup takes an equal share of all
sequences' keys, shares may cross sequence boundaries) against the fp64 oracle."""
import dataclasses

import numpy as np
import pytest

import gen
import paper_2509_15235_amd as vs

pytestmark = pytest.mark.gpu

CONTRACT = (2e-2, 1e-2)
TIGHT_LONG = (1.5e-3, 6e-3)
TIGHT_SHORT = (1.2e-2, 6e-3)


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def _cfg(**kw):
    base = dict(B=5, Hq=8, Hkv=2, d=128, T=13, max_depth=4, V=100, layers=1, dtype="bf16", prefix=None,
                prefix_range=(1, 2), paged=False, segments=None)
    base.update(kw)
    return dataclasses.replace(gen.CONFIGS["C3"], **base)


def _check(gu, oracle_mod, inp, ref, **kw):
    da = gu.DeviceAttn(inp, schedule=vs.VS_SCHED_BALANCED, **kw)
    pl = da.plan()
    assert pl.schedule == vs.VS_SCHED_BALANCED and pl.combine == 1 and pl.keys_per_split == 0
    got = da.run()
    assert (da.status.cpu().numpy() == 0).all()
    gu.check_close(got, ref, *CONTRACT, what="contract")
    tight = TIGHT_LONG if int(inp.prefix_len.min()) >= 256 else TIGHT_SHORT
    worst = gu.check_close(got, ref, *tight, what=f"tight {kw}")
    return got, worst, da


@pytest.mark.parametrize("paged", [False, True])
def test_ragged_batch_every_share_count(gu, oracle_mod, paged):
    """Five sequences of very different lengths; shares from fewer than sequences to more than 64-key steps."""
    lens = np.array([700, 64, 1500, 130, 999], dtype=np.int32)
    inp = gen.attention_inputs(_cfg(paged=paged), 501, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    for shares in (1, 2, 3, 7, 16, 33, 64):
        for waves in (4, 8):
            _, worst, da = _check(gu, oracle_mod, inp, ref, num_splits=shares, waves_per_group=waves)
            assert da.plan().num_splits == shares
    print(f"ragged paged={paged}: worst {worst:.3e}")


def test_whole_sequences_match_the_unsplit_plan(gu, oracle_mod):
    """A batch of equal lengths and one share per sequence: every share is one whole sequence, the rows leave
    the main kernel as final output, and they equal the pipelined kernel's without key splits bit for bit."""
    lens = np.full(4, 2 * 640 - 13, dtype=np.int32)            # 20 steps of 64 keys per sequence with T = 13
    inp = gen.attention_inputs(_cfg(B=4), 502, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    got_b, _, _ = _check(gu, oracle_mod, inp, ref, num_splits=4)
    dp = gu.DeviceAttn(inp, schedule=vs.VS_SCHED_PIPELINED, num_splits=1, waves_per_group=4)
    got_p = dp.run()
    np.testing.assert_array_equal(got_b, got_p)                 # same key ranges, same arithmetic
    # two shares per sequence: the regular cut (halves, as equal splits would be) is no worse than any other
    got_b, _, _ = _check(gu, oracle_mod, inp, ref, num_splits=8)
    got_p = gu.DeviceAttn(inp, schedule=vs.VS_SCHED_PIPELINED, num_splits=2, waves_per_group=4).run()
    np.testing.assert_array_equal(got_b, got_p)
    _check(gu, oracle_mod, inp, ref, num_splits=7)              # shares that do not line up with the sequences


def test_tiny_sequences_and_more_shares_than_steps(gu, oracle_mod):
    lens = np.array([10, 3, 70, 1, 55, 200], dtype=np.int32)
    inp = gen.attention_inputs(_cfg(B=6, T=7, Hq=4, Hkv=4, max_depth=3), 503, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    for shares in (1, 5, 16, 64):
        _check(gu, oracle_mod, inp, ref, num_splits=shares, waves_per_group=4)


def test_single_sequence_and_head_dim_64(gu, oracle_mod):
    inp = gen.attention_inputs(_cfg(B=1, T=60, Hq=28, Hkv=4, max_depth=6), 504, prefix_len=np.array([1696], dtype=np.int32))
    ref = oracle_mod.tree_attention(inp, threads=8)
    _check(gu, oracle_mod, inp, ref, num_splits=9)
    inp = gen.attention_inputs(_cfg(B=3, d=64, T=30, Hq=16, Hkv=4, max_depth=5), 505,
                               prefix_len=np.array([900, 100, 2000], dtype=np.int32))
    ref = oracle_mod.tree_attention(inp, threads=8)
    for waves in (4, 8):
        _check(gu, oracle_mod, inp, ref, num_splits=11, waves_per_group=waves)


def test_sixty_four_sequences(gu, oracle_mod):
    g = gen.rng(506, 1)
    lens = g.integers(1, 400, size=64).astype(np.int32)
    inp = gen.attention_inputs(_cfg(B=64, T=5, Hq=4, Hkv=2, max_depth=3), 506, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    _check(gu, oracle_mod, inp, ref, num_splits=37, waves_per_group=4)
    _check(gu, oracle_mod, inp, ref)                              # the planner's own share count


def test_bad_prefix_and_bad_tree_are_reported_and_isolated(gu, oracle_mod):
    lens = np.array([300, 120, 500, 77], dtype=np.int32)
    inp = gen.attention_inputs(_cfg(B=4), 507, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    bad = dataclasses.replace(inp, prefix_len=np.array([300, 9999, 500, -4], dtype=np.int32), parent=inp.parent.copy())
    bad.parent[2, 3] = 7                                           # parent after child: malformed tree of sequence 2
    da = gu.DeviceAttn(bad, schedule=vs.VS_SCHED_BALANCED, num_splits=6, max_prefix_len=500)
    got = da.run()
    st = da.status.cpu().numpy()
    assert list(st) == [0, 3, 2, 3]                                # ok, bad prefix, bad parent, bad prefix
    gu.check_close(got[0], ref[0], *TIGHT_LONG, what="the good sequence next to the bad ones")


def test_masks_given_and_repeated_runs(gu, oracle_mod):
    """The caller's masks instead of the parent rows; two runs give the same bits."""
    import torch
    lens = np.array([1300, 257, 640, 2100, 33, 900, 1500], dtype=np.int32)
    inp = gen.attention_inputs(_cfg(B=7, T=20, Hq=14, Hkv=2, max_depth=5, paged=True), 508, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    got, _, da = _check(gu, oracle_mod, inp, ref, num_splits=13)
    mask, _, st, _ = gu.run_mask(inp.parent)
    assert (st == 0).all()
    got_m = da.run(tree_mask=torch.from_numpy(mask.astype(np.int64)).cuda())
    np.testing.assert_array_equal(got, got_m)
    np.testing.assert_array_equal(got, da.run())


def test_bad_block_is_reported(gu, oracle_mod):
    lens = np.array([500, 300, 800], dtype=np.int32)
    inp = gen.attention_inputs(_cfg(B=3, paged=True), 510, prefix_len=lens)
    ref = oracle_mod.tree_attention(inp, threads=8)
    bad = dataclasses.replace(inp, block_table=inp.block_table.copy())
    bad.block_table[1, 2] = inp.n_blocks + 5
    da = gu.DeviceAttn(bad, schedule=vs.VS_SCHED_BALANCED, num_splits=5)
    got = da.run()
    assert list(da.status.cpu().numpy()) == [0, 4, 0]
    gu.check_close(got[0], ref[0], *TIGHT_LONG, what="sequence 0")
    gu.check_close(got[2], ref[2], *TIGHT_LONG, what="sequence 2")


def test_random_batches_and_share_counts(gu, oracle_mod):
    """Seeded random batch sizes, lengths (some a single token, some a few thousand) and share counts."""
    g = gen.rng(511, 1)
    worst = 0.0
    for case in range(14):
        B = int(g.integers(1, 25))
        hi = int(g.choice([40, 300, 3000]))
        lens = g.integers(1, hi + 1, size=B).astype(np.int32)
        shares = int(g.choice([0, 1, 2, 3, 5, 8, 13, 21, 32, 47, 64]))
        waves = int(g.choice([4, 8]))
        d = int(g.choice([64, 128]))
        inp = gen.attention_inputs(_cfg(B=B, T=6, Hq=4, Hkv=2, d=d, max_depth=3, paged=bool(case % 2)), 600 + case, prefix_len=lens)
        ref = oracle_mod.tree_attention(inp, threads=8)
        _, w, _ = _check(gu, oracle_mod, inp, ref, num_splits=shares, waves_per_group=waves)
        worst = max(worst, w)
    print(f"random batches: worst {worst:.3e}")
