"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2509_15235_amd as vs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "vispec_verify.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(vs_[a-z_]+)\s*\(", hdr))
    assert declared == set(vs.EXPORTED_SYMBOLS)
    L = ctypes.CDLL(vs.lib_path())
    for name in declared:
        assert hasattr(L, name), name
    assert vs.vs_version() == 100
    # the measurement helpers' header
    hdr = open(os.path.join(ROOT, "include", "vispec_peaks.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(vs_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(vs.PEAK_SYMBOLS)
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["vispec_peaks.h", "vispec_verify.h"]
    g = 4096
    assert vs.vs_peak_hbm_read(None, 1 << 20, g, 256) == -1 and vs.vs_peak_hbm_read(g + 4, 1 << 20, g, 256) == -2
    assert vs.vs_peak_hbm_copy(g, g, 8, 256) == -2 and vs.vs_peak_mfma_bf16(g, 0, g, 256) == -2
    assert vs.vs_peak_mfma_flops(10, 256) == 8 * 256 * 10 * 16 * 32768


def test_error_strings():
    assert vs.vs_strerror(0) == "ok"
    for code in range(-7, 0):
        assert vs.vs_strerror(code) not in ("ok", "unknown error")
    assert vs.vs_strerror(-99) == "unknown error"
    assert vs.vs_status_string(2).startswith("a parent")


@pytest.mark.parametrize("parent,exp", [([-1], 0), ([-1, 0, 1, 1], 0), ([0], 1), ([-1, 1], 2), ([-1, 0, 2], 2),
                                        ([-1, -1], 2), ([-1, 0, -5], 2)])
def test_tree_validate_host(parent, exp):
    a = np.array(parent, dtype=np.int32)
    assert vs.vs_tree_validate_host(a, len(a)) == exp


def test_tree_validate_host_matches_oracle_on_random_arrays(oracle_mod):
    g = np.random.default_rng(0)
    for _ in range(300):
        T = int(g.integers(1, 10))
        a = g.integers(-2, T, T).astype(np.int32)
        if g.random() < 0.5:
            a[0] = -1
        assert vs.vs_tree_validate_host(a, T) == oracle_mod.tree_validate(a)
    assert vs.vs_tree_validate_host(None, 3) == -1
    assert vs.vs_tree_validate_host(np.array([-1], dtype=np.int32), 0) == -2
    assert vs.vs_tree_validate_host(np.zeros(65, dtype=np.int32), 65) == -2


def _desc(**kw):
    d = vs.AttnDesc(B=1, T=60, Hq=28, Hkv=4, d=128, dtype=vs.VS_BF16, softmax_scale=0.1, max_prefix_len=1696,
                    capacity=1800, stride_seq=4 * 1800 * 128, stride_head=1800 * 128, stride_tok=128)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


@pytest.mark.parametrize("kw,code", [
    ({}, 0),
    ({"T": 0}, -2), ({"T": 65}, -2), ({"B": 0}, -2), ({"Hq": 30}, -2), ({"d": 96}, -2),
    ({"softmax_scale": 0.0}, -2), ({"softmax_scale": float("nan")}, -2), ({"max_prefix_len": -1}, -2),
    ({"dtype": 7}, -3), ({"dtype": vs.VS_F32, "impl": vs.VS_IMPL_MFMA}, -3), ({"impl": 9}, -2),
    ({"stride_tok": 64}, -6), ({"stride_tok": 132}, -6), ({"capacity": 1700}, -6),
    ({"paged": 1, "block_size": 16, "max_blocks": 200, "num_blocks": 300, "stride_block": 4 * 16 * 128,
      "stride_head": 16 * 128, "block_table": None}, -1),
    ({"paged": 1, "block_size": 24, "max_blocks": 200, "num_blocks": 300, "block_table": 4096}, -6),
    ({"paged": 1, "block_size": 16, "max_blocks": 10, "num_blocks": 300, "block_table": 4096}, -6),
    ({"num_splits": -1}, -2),
    ({"schedule": 5}, -2), ({"schedule": vs.VS_SCHED_PIPELINED, "rows_per_wave": 2}, -2),
    ({"schedule": vs.VS_SCHED_BALANCED}, 0), ({"schedule": vs.VS_SCHED_BALANCED, "num_splits": 64}, 0),
    ({"schedule": vs.VS_SCHED_BALANCED, "num_splits": 65}, -2), ({"schedule": vs.VS_SCHED_BALANCED, "B": 65}, -2),
    ({"schedule": vs.VS_SCHED_BALANCED, "rows_per_wave": 2}, -2), ({"schedule": vs.VS_SCHED_BALANCED, "waves_per_group": 2}, -2),
    ({"schedule": vs.VS_SCHED_BALANCED, "impl": vs.VS_IMPL_GENERIC}, -2),
    ({"schedule": vs.VS_SCHED_RESIDENT}, 0), ({"schedule": vs.VS_SCHED_RESIDENT, "rows_per_wave": 2}, -2),
    ({"schedule": vs.VS_SCHED_RESIDENT, "waves_per_group": 4}, -2),
    ({"schedule": vs.VS_SCHED_PIPELINED, "waves_per_group": 2}, -2),
    ({"schedule": vs.VS_SCHED_PIPELINED, "waves_per_group": 4}, 0), ({"schedule": vs.VS_SCHED_LOOP}, 0),
])
def test_attention_descriptor_validation(kw, code):
    rc, plan = vs.vs_attention_plan(_desc(**kw))
    assert rc == code
    if code != 0:
        assert vs.vs_attention_workspace_bytes(_desc(**kw)) == 0


def test_plan_and_workspace_sizes():
    # one layer of one short sequence: LDS-resident splits of 128 keys, four row blocks per workgroup
    rc, plan = vs.vs_attention_plan(_desc())
    assert rc == 0 and plan.impl == vs.VS_IMPL_MFMA and plan.schedule == vs.VS_SCHED_RESIDENT
    assert plan.rows_per_wave == 1 and plan.waves_per_group == 8 and plan.row_groups == 4
    assert plan.keys_per_split == 128 and plan.num_splits == 14
    assert plan.workgroups == 4 * plan.row_groups * plan.num_splits and plan.combine == 1
    ws = vs.vs_attention_workspace_bytes(_desc())
    assert ws >= 4 * plan.num_splits * 448 * (128 * 2 + 2 * 4)          # bf16 partial rows + fp32 (max, sum)
    # ... the streaming loop when asked for, or when the caller's knobs rule the resident kernel out
    rc, plan = vs.vs_attention_plan(_desc(schedule=vs.VS_SCHED_LOOP))
    assert plan.schedule == vs.VS_SCHED_LOOP and plan.rows_per_wave == 1 and plan.waves_per_group == 4 and plan.row_groups == 4
    assert plan.keys_per_split % 64 == 0 and plan.num_splits * plan.keys_per_split >= 1696 + 60
    assert plan.workgroups == 4 * plan.row_groups * plan.num_splits and plan.combine == 1
    assert vs.vs_attention_plan(_desc(waves_per_group=4))[1].schedule == vs.VS_SCHED_LOOP
    assert vs.vs_attention_plan(_desc(num_splits=2))[1].schedule == vs.VS_SCHED_LOOP
    # ... for more sequences than fit in one round of its workgroups (one per CU): two sequences
    # take the loop with one workgroup per CU
    rc, two = vs.vs_attention_plan(_desc(B=2))
    assert two.schedule == vs.VS_SCHED_LOOP and two.num_splits == 7 and two.workgroups == 224
    # ... and for long sequences
    one_long = _desc(max_prefix_len=6684, capacity=6800, stride_head=6800 * 128)
    assert vs.vs_attention_plan(one_long)[1].schedule == vs.VS_SCHED_LOOP
    # from twelve (sequence, KV head) units on the pipelined kernel: three GQA sequences, one MHA layer
    rc, three = vs.vs_attention_plan(_desc(B=3))
    assert three.schedule == vs.VS_SCHED_PIPELINED and three.waves_per_group == 8 and three.workgroups <= 256
    rc, one_mha = vs.vs_attention_plan(_desc(Hq=32, Hkv=32, stride_seq=32 * 1800 * 128))
    assert one_mha.schedule == vs.VS_SCHED_PIPELINED and one_mha.waves_per_group == 4 and one_mha.workgroups <= 256
    # an explicit resident schedule caps a split at 192 keys whatever split count is asked for
    rc, pr = vs.vs_attention_plan(_desc(schedule=vs.VS_SCHED_RESIDENT, num_splits=1, max_prefix_len=6684, capacity=6800,
                                        stride_head=6800 * 128))
    assert pr.keys_per_split == 192 and pr.num_splits == 36
    # many units: pipelined kernel, eight waves, rows split over two workgroups, no key split, no combine
    big = _desc(B=28, stride_seq=4 * 1800 * 128)
    rc, pb = vs.vs_attention_plan(big)
    assert pb.schedule == vs.VS_SCHED_PIPELINED
    assert pb.rows_per_wave == 1 and pb.waves_per_group == 8 and pb.row_groups == 2
    assert pb.num_splits == 1 and pb.workgroups == 224 and pb.combine == 0
    assert vs.vs_attention_workspace_bytes(big) == 0
    long_ = _desc(B=28, max_prefix_len=6684, capacity=6800, stride_seq=4 * 6800 * 128, stride_head=6800 * 128)
    rc, pl = vs.vs_attention_plan(long_)
    assert pl.schedule == vs.VS_SCHED_PIPELINED and pl.row_groups == 2 and pl.num_splits == 1 and pl.workgroups == 224
    # fewer units than CUs: key splits fill the machine
    mid = _desc(B=16, max_prefix_len=8192, capacity=8300, stride_seq=4 * 8300 * 128, stride_head=8300 * 128)
    rc, pm5 = vs.vs_attention_plan(mid)
    # ... by equal shares of the whole batch's keys, since the sequences of a batch may differ in length
    assert pm5.schedule == vs.VS_SCHED_BALANCED and pm5.num_splits == 32 and pm5.keys_per_split == 0
    assert pm5.workgroups == 256 and pm5.combine == 1 and pm5.waves_per_group == 8 and pm5.row_groups == 2
    # 4 KV heads x (32 shares + 16 sequences) slots of 448 rows: bf16 rows plus (max, sum) pairs
    assert vs.vs_attention_workspace_bytes(mid) == 4 * 48 * 448 * (128 * 2 + 8) + 256
    mid.schedule = vs.VS_SCHED_PIPELINED
    rc, pm5 = vs.vs_attention_plan(mid)
    assert pm5.schedule == vs.VS_SCHED_PIPELINED and pm5.num_splits == 2 and pm5.workgroups == 256 and pm5.combine == 1
    # the caller's split count, short sequences, or a single sequence keep the equal splits
    assert vs.vs_attention_plan(_desc(B=16, max_prefix_len=8192, capacity=8300, stride_seq=4 * 8300 * 128,
                                      stride_head=8300 * 128, num_splits=3))[1].schedule == vs.VS_SCHED_PIPELINED
    assert vs.vs_attention_plan(_desc(B=8, stride_seq=4 * 1800 * 128))[1].schedule == vs.VS_SCHED_PIPELINED
    # more than one round of whole sequences and less than two: shares instead of a second, partly filled round;
    # one or two full rounds stay as they are
    big40 = _desc(B=40, max_prefix_len=8192, capacity=8300, stride_seq=4 * 8300 * 128, stride_head=8300 * 128)
    rc, p40 = vs.vs_attention_plan(big40)
    assert p40.schedule == vs.VS_SCHED_BALANCED and p40.num_splits == 32 and p40.workgroups == 256
    assert vs.vs_attention_workspace_bytes(big40) == 4 * 72 * 448 * (128 * 2 + 8) + 256
    for B in (32, 64):
        assert vs.vs_attention_plan(_desc(B=B, max_prefix_len=8192, capacity=8300, stride_seq=4 * 8300 * 128,
                                          stride_head=8300 * 128))[1].schedule == vs.VS_SCHED_PIPELINED
    # four-wave workgroups (MHA): two per CU, hence 512 places and 16 shares per KV head
    rc, pm8 = vs.vs_attention_plan(_desc(B=8, Hq=32, Hkv=32, max_prefix_len=8192, capacity=8300, stride_seq=32 * 8300 * 128,
                                         stride_head=8300 * 128))
    assert pm8.schedule == vs.VS_SCHED_BALANCED and pm8.waves_per_group == 4 and pm8.num_splits == 16 and pm8.workgroups == 512
    # few row blocks per unit (MHA): four waves
    mha = _desc(B=32, Hq=32, Hkv=32, max_prefix_len=3136, capacity=3300, stride_seq=32 * 3300 * 128, stride_head=3300 * 128)
    rc, pm2 = vs.vs_attention_plan(mha)
    assert pm2.schedule == vs.VS_SCHED_PIPELINED and pm2.waves_per_group == 4 and pm2.row_groups == 1 and pm2.num_splits == 1
    # two row blocks per wave exist in the straight loop only
    rc, p2 = vs.vs_attention_plan(_desc(B=28, stride_seq=4 * 1800 * 128, rows_per_wave=2))
    assert p2.schedule == vs.VS_SCHED_LOOP and p2.rows_per_wave == 2 and p2.waves_per_group == 8 and p2.num_splits == 2
    rc, pf = vs.vs_attention_plan(_desc(schedule=vs.VS_SCHED_PIPELINED))
    assert pf.schedule == vs.VS_SCHED_PIPELINED and pf.waves_per_group == 8 and pf.num_splits * pf.keys_per_split >= 1756
    # explicit knobs
    rc, plan1 = vs.vs_attention_plan(_desc(num_splits=1))
    assert plan1.num_splits == 1 and plan1.combine == 0 and vs.vs_attention_workspace_bytes(_desc(num_splits=1)) == 0
    rc, pk = vs.vs_attention_plan(_desc(rows_per_wave=2, waves_per_group=8, num_splits=3))
    assert pk.rows_per_wave == 2 and pk.waves_per_group == 8 and pk.row_groups == 1 and pk.num_splits == 3
    assert vs.vs_attention_plan(_desc(rows_per_wave=3))[0] == -2
    assert vs.vs_attention_plan(_desc(waves_per_group=3))[0] == -2
    rc, pg = vs.vs_attention_plan(_desc(dtype=vs.VS_F32))
    assert pg.impl == vs.VS_IMPL_GENERIC and vs.vs_attention_workspace_bytes(_desc(dtype=vs.VS_F32)) == 0
    # MHA: two row blocks per unit; the loop uses two waves, the pipelined kernel four
    rc, pm = vs.vs_attention_plan(_desc(Hq=32, Hkv=32, max_prefix_len=3136, capacity=3300, schedule=vs.VS_SCHED_LOOP))
    assert pm.waves_per_group == 2 and pm.rows_per_wave == 1 and pm.num_splits > 1 and pm.workgroups <= 256
    rc, pm = vs.vs_attention_plan(_desc(Hq=32, Hkv=32, max_prefix_len=3136, capacity=3300))
    assert pm.schedule == vs.VS_SCHED_PIPELINED and pm.waves_per_group == 4 and pm.num_splits == 8 and pm.workgroups == 256


def test_calls_reject_bad_arguments_before_any_launch():
    d = _desc()
    good = 4096  # never dereferenced: every call below fails validation first
    assert vs.vs_tree_verify_attention(d, None, good, good, good, good, None, good) == -1
    assert vs.vs_tree_verify_attention(d, good, good, good, good, good, None, None) == -1
    assert vs.vs_tree_verify_attention(d, good + 2, good, good, good, good, None, good) == -6     # misaligned q
    assert vs.vs_tree_verify_attention(d, good, good, good, good, good, None, good, None, None, 0) == -4
    assert vs.vs_tree_verify_attention(d, good, good, good, good, good, None, good, None, good, 16) == -4
    assert vs.vs_tree_verify_attention(_desc(T=99), good, good, good, good, good, None, good) == -2
    assert vs.vs_tree_mask_build(None, 1, 4, good, good) == -1
    assert vs.vs_tree_mask_build(good, 1, 65, good, good) == -2
    assert vs.vs_tree_mask_build(good, 0, 4, good, good) == -2
    n = vs.vs_accept_workspace_bytes(1, 60, 152064)
    assert n >= 60 * 19 * 8
    assert vs.vs_accept_workspace_bytes(1, 65, 10) == 0
    assert vs.vs_tree_accept(None, 10, 10, good, good, 1, 4, good, good, good) == -1
    assert vs.vs_tree_accept(good, 9, 10, good, good, 1, 4, good, good, good, None, None, good, 1 << 20) == -2
    assert vs.vs_tree_accept(good, 10, 10, good, good, 1, 4, good, good, good, None, None, None, 0) == -4
    assert vs.vs_tree_accept(good, 10, 10, good, good, 1, 4, good, good, good, None, None, good, 8) == -4


def test_sizes_beyond_a_grid_dimension_are_shape_errors():
    """The logits scans launch one workgroup per (row, 4096-logit chunk) and the split combine one
    grid row per (sequence, KV head): more than a grid dimension holds is reported as a shape error
    on the host, not left to the launch to refuse."""
    g = 4096
    B = 1 << 20                                            # x 64 rows x 38 chunks > 2^31
    assert vs.vs_tree_accept(g, 152064, 152064, g, g, B, 64, g, g, g, None, None, g, 1 << 40) == -2
    assert vs.vs_tree_accept_sample(g, 152064, 152064, 1.0, g, g, g, g, B, 64, g, g, g, None, g, 1 << 40) == -2
    assert vs.vs_draft_expand(g, 152064, 152064, None, None, B, 64, 8, 0, 512, g, g, g, g, g, g, 1 << 40) == -2
    assert vs.vs_attention_plan(_desc(B=65535 // 4 + 1))[0] == -2


def test_no_device_is_reported_after_the_argument_checks():
    """On a machine without a GPU a call whose arguments are all acceptable ends in VS_ERR_NO_DEVICE
    before anything is enqueued (bad arguments still get their own codes, as above)."""
    import torch
    if torch.cuda.device_count() > 0:
        pytest.skip("a GPU is visible")
    g = 4096
    assert vs.vs_tree_mask_build(g, 1, 4, g, g) == -7
    assert vs.vs_tree_accept(g, 10, 10, g, g, 1, 4, g, g, g, None, None, g, 1 << 20) == -7
    assert vs.vs_tree_verify_attention(_desc(num_splits=1), g, g, g, g, g, None, g) == -7
    assert vs.vs_strerror(-7) == "no usable gfx950 device"


def test_accept_sample_rejects_bad_arguments_before_any_launch():
    g = 4096  # never dereferenced
    n = vs.vs_accept_sample_workspace_bytes(1, 60, 152064)
    assert n >= 2 * 60 * 38 * 4
    assert vs.vs_accept_sample_workspace_bytes(1, 65, 10) == 0
    assert vs.vs_accept_sample_workspace_bytes(1, 4, 8388608) > 0
    assert vs.vs_accept_sample_workspace_bytes(1, 4, 8388609) == 0            # more chunks than the walk keeps
    ok = dict(workspace=g, workspace_bytes=1 << 20)
    assert vs.vs_tree_accept_sample(None, 10, 10, 1.0, g, g, g, g, 1, 4, g, g, g, **ok) == -1
    assert vs.vs_tree_accept_sample(g, 10, 10, 1.0, g, g, None, g, 1, 4, g, g, g, **ok) == -1   # uniforms are required
    assert vs.vs_tree_accept_sample(g, 10, 10, 1.0, g, g, g, None, 1, 4, g, g, g, **ok) == -1
    assert vs.vs_tree_accept_sample(g, 9, 10, 1.0, g, g, g, g, 1, 4, g, g, g, **ok) == -2
    assert vs.vs_tree_accept_sample(g, 10, 10, 1.0, g, g, g, g, 1, 65, g, g, g, **ok) == -2
    assert vs.vs_tree_accept_sample(g, 10, 10, 0.0, g, g, g, g, 1, 4, g, g, g, **ok) == -2       # temperature 0: greedy call
    assert vs.vs_tree_accept_sample(g, 10, 10, -1.0, g, g, g, g, 1, 4, g, g, g, **ok) == -2
    assert vs.vs_tree_accept_sample(g, 10, 10, float("nan"), g, g, g, g, 1, 4, g, g, g, **ok) == -2
    assert vs.vs_tree_accept_sample(g, 10, 10, float("inf"), g, g, g, g, 1, 4, g, g, g, **ok) == -2
    assert vs.vs_tree_accept_sample(g, 1 << 24, 8388609, 1.0, g, g, g, g, 1, 4, g, g, g, **ok) == -2
    assert vs.vs_tree_accept_sample(g, 10, 10, 1.0, g, g, g, g, 1, 4, g, g, g) == -4
    assert vs.vs_tree_accept_sample(g, 10, 10, 1.0, g, g, g, g, 1, 4, g, g, g, None, g, 8) == -4
    assert vs.vs_tree_accept_sample(g, 10, 10, 1.0, g, g, g, g, 1, 4, g, g, g, None, g + 8, 1 << 20) == -4


def test_draft_calls_reject_bad_arguments_before_any_launch():
    g = 4096  # never dereferenced
    assert vs.vs_draft_expand_workspace_bytes(1, 8, 152064, 8) >= 8 * 38 * (8 + 8 * 8)
    assert vs.vs_draft_expand_workspace_bytes(1, 8, 152064, 17) == 0
    assert vs.vs_draft_expand_workspace_bytes(1, 65, 152064, 8) == 0
    assert vs.vs_draft_expand_workspace_bytes(1, 1, 4, 8) == 0                   # K > V
    ws = dict(workspace=g, workspace_bytes=1 << 24)
    ex = lambda **kw: vs.vs_draft_expand(**{**dict(logits=g, ld_logits=100, V=100, cum_in=None, frontier_cand=None,
                                                  B=1, F=1, K=8, cand_base=0, cand_capacity=136, cand_token=g,
                                                  cand_score=g, cand_parent=g, next_frontier_cand=g, next_cum=g,
                                                  **ws), **kw})
    assert ex(logits=None) == -1 and ex(cand_score=None) == -1 and ex(next_cum=None) == -1
    assert ex(K=0) == -2 and ex(K=17) == -2 and ex(F=0) == -2 and ex(F=65) == -2 and ex(V=7) == -2
    assert ex(ld_logits=99) == -2
    assert ex(cand_base=130) == -2 and ex(cand_base=-1) == -2 and ex(F=8, cand_base=73) == -2
    assert ex(workspace=None) == -4 and ex(workspace_bytes=64) == -4 and ex(workspace=g + 16) == -4
    bd = lambda **kw: vs.vs_draft_tree_build(**{**dict(cand_token=g, cand_score=g, cand_parent=g, B=1, M=136,
                                                      cand_capacity=136, N=30, root_token=None, parent=g,
                                                      draft_tokens=g, node_cand=g, num_nodes=g), **kw})
    assert bd(cand_token=None) == -1 and bd(num_nodes=None) == -1
    assert bd(M=0) == -2 and bd(M=2049, cand_capacity=4096) == -2 and bd(M=137) == -2
    assert bd(N=0) == -2 and bd(N=64) == -2 and bd(B=0) == -2


def test_compress_attention_rejects_bad_arguments_before_any_launch():
    g = 4096  # never dereferenced
    d = _desc(T=16)
    assert vs.vs_compress_attention(d, None, g, g, g, g) == -1
    assert vs.vs_compress_attention(d, g, g, g, None, g) == -1
    assert vs.vs_compress_attention(_desc(T=65), g, g, g, g, g) == -2
    assert vs.vs_compress_attention(_desc(T=16, max_prefix_len=0), g, g, g, g, g) == -2       # no image embeddings at all
    assert vs.vs_compress_attention(d, g + 2, g, g, g, g) == -6                              # misaligned q
    assert vs.vs_compress_attention(_desc(T=16, num_splits=4), g, g, g, g, g, None, None, 0) == -4
    # the queries' own K/V are not in the cache: a cache of exactly max_prefix_len tokens is enough
    tight = _desc(T=16, max_prefix_len=1800)
    assert vs.vs_compress_attention_workspace_bytes(tight) > 0 and vs.vs_attention_workspace_bytes(tight) == 0
    assert vs.vs_compress_attention_workspace_bytes(_desc(T=0)) == 0


def test_kv_commit_rejects_bad_arguments_before_any_launch():
    def kd(**kw):
        d = vs.KVDesc(B=2, T=8, Hkv=2, d=64, dtype=vs.VS_BF16, num_layers=3, stride_layer=2 * 2 * 100 * 64,
                      capacity=100, stride_seq=2 * 100 * 64, stride_head=100 * 64, stride_tok=64)
        for k, v in kw.items():
            setattr(d, k, v)
        return d
    g = 4096  # never dereferenced: every call below fails validation first
    assert vs.vs_tree_kv_commit(kd(), None, g, g, g, g, g + 64) == -1
    assert vs.vs_tree_kv_commit(kd(), g, g, g, g, g, None) == -1
    assert vs.vs_tree_kv_commit(kd(T=0), g, g, g, g, g, g + 64) == -2
    assert vs.vs_tree_kv_commit(kd(T=65), g, g, g, g, g, g + 64) == -2
    assert vs.vs_tree_kv_commit(kd(num_layers=0), g, g, g, g, g, g + 64) == -2
    assert vs.vs_tree_kv_commit(kd(dtype=3), g, g, g, g, g, g + 64) == -3
    assert vs.vs_tree_kv_commit(kd(d=4), g, g, g, g, g, g + 64) == -6            # 8-byte rows
    assert vs.vs_tree_kv_commit(kd(stride_tok=68), g, g, g, g, g, g + 64) == -6   # 136-byte row pitch
    assert vs.vs_tree_kv_commit(kd(capacity=4), g, g, g, g, g, g + 64) == -6
    assert vs.vs_tree_kv_commit(kd(), g + 2, g, g, g, g, g + 64) == -6            # misaligned cache
    assert vs.vs_tree_kv_commit(kd(), g, g, g, g, g, g) == -6                     # new_prefix_len aliases prefix_len
    assert vs.vs_tree_kv_commit(kd(paged=1, block_size=16, max_blocks=8, num_blocks=9, stride_block=2 * 16 * 64,
                                   stride_head=16 * 64), g, g, g, g, g, g + 64) == -1   # no block table
    assert vs.vs_tree_kv_commit(kd(paged=1, block_size=24, max_blocks=8, num_blocks=9, block_table=g), g, g, g, g, g,
                                g + 64) == -6
    assert "accepted path" in vs.vs_status_string(5)
