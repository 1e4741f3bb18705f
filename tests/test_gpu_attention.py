"""GPU parity of tree_verify_attention against the fp64 oracle.

Contract tolerance (bf16 inputs, fp32 accumulation): |gpu - ref| <= 2e-2 + 1e-2 |ref|.
Because that bound is loose next to outputs of rms ~0.04, every case also has to meet a
tight bound derived from the arithmetic: the bf16 rounding of the output (2^-9 relative)
plus the bf16 rounding of the probabilities (at most 2^-9 of the largest visible |V|, far
less once hundreds of keys share the weight)."""
import dataclasses

import numpy as np
import pytest

import gen
import paper_2509_15235_amd as vs

pytestmark = pytest.mark.gpu

CONTRACT = (2e-2, 1e-2)
TIGHT_LONG = (1.5e-3, 6e-3)    # hundreds of visible keys
TIGHT_SHORT = (1.2e-2, 6e-3)   # a handful of keys: P's rounding is not averaged away
TIGHT_F32 = (2e-5, 2e-5)


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def _tight(inp):
    if inp.cfg.dtype == "f32":
        return TIGHT_F32
    return TIGHT_LONG if int(inp.prefix_len.min()) >= 256 else TIGHT_SHORT


def _run_and_check(gu, oracle_mod, inp, ref=None, **kw):
    if ref is None:
        ref = oracle_mod.tree_attention(inp, threads=8)
    da = gu.DeviceAttn(inp, **kw)
    got = da.run()
    assert (da.status.cpu().numpy() == 0).all()
    if inp.cfg.dtype == "bf16":
        gu.check_close(got, ref, *CONTRACT, what="contract")
    gu.check_close(got, ref, *_tight(inp), what=f"tight {kw}")
    return got, ref, da


# ---------------------------------------------------------------- the five configurations

def test_c1_tiny_fp32(gu, oracle_mod):
    inp = gen.attention_inputs(gen.CONFIGS["C1"], 11)
    _run_and_check(gu, oracle_mod, inp)


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_full_size_single_sequence(gu, oracle_mod, name):
    inp = gen.attention_inputs(gen.CONFIGS[name], 20 + int(name[1]))
    ref = oracle_mod.tree_attention(inp, threads=8)
    got, _, da = _run_and_check(gu, oracle_mod, inp, ref=ref)                       # launch shape of the bench
    assert da.plan().impl == vs.VS_IMPL_MFMA
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=1)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=7)
    # every kernel shape: row blocks per wave x waves per workgroup
    for rpw in (1, 2):
        for nw in (1, 2, 4, 8):
            _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=3, rows_per_wave=rpw, waves_per_group=nw)
    # the software-pipelined schedule: both wave counts, no split / few / many splits
    for nw in (4, 8):
        for sp in (1, 3, 0):
            got_p, _, dp = _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=sp, waves_per_group=nw,
                                          schedule=vs.VS_SCHED_PIPELINED)
            assert dp.plan().schedule == vs.VS_SCHED_PIPELINED
    # the LDS-resident schedule: planner's split count (three 64-key tiles each), splits of one, two and three (the most) 64-key tiles
    for sp in (0, 10 ** 6, (inp.cfg.prefix[0] + inp.cfg.T + 127) // 128, 1):
        _, _, dr = _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=sp, schedule=vs.VS_SCHED_RESIDENT)
        assert dr.plan().schedule == vs.VS_SCHED_RESIDENT and dr.plan().keys_per_split <= 192
    _run_and_check(gu, oracle_mod, inp, ref=ref, impl=vs.VS_IMPL_GENERIC)


def test_c5_ragged_paged_batch(gu, oracle_mod):
    inp = gen.attention_inputs(gen.CONFIGS["C5"], 25)
    ref = oracle_mod.tree_attention(inp, threads=8)
    _, _, da = _run_and_check(gu, oracle_mod, inp, ref=ref)            # launch shape of the bench: balanced shares
    assert da.plan().schedule == vs.VS_SCHED_BALANCED and da.plan().workgroups == 256
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=4)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=3, rows_per_wave=2, waves_per_group=8)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=2, rows_per_wave=1, waves_per_group=4)
    for nw, sp in ((8, 1), (8, 2), (4, 5)):   # paged copies in the pipelined kernel
        _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=sp, waves_per_group=nw, schedule=vs.VS_SCHED_PIPELINED)
    for sp in (0, 11):                        # ... and in the resident one
        _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=sp, schedule=vs.VS_SCHED_RESIDENT)


def test_layers_folded_into_batch(gu, oracle_mod):
    """The bench's roofline launch: the layers of one C3 step as independent batch entries."""
    cfg = dataclasses.replace(gen.CONFIGS["C3"], B=4, prefix=[1696] * 4)
    inp = gen.attention_inputs(cfg, 26)
    ref = oracle_mod.tree_attention(inp, threads=8)
    _run_and_check(gu, oracle_mod, inp, ref=ref)
    # the launch shape the planner picks for 28 layers: pipelined, eight waves, rows split over
    # two workgroups, no key split
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=1, waves_per_group=8, schedule=vs.VS_SCHED_PIPELINED)
    # and the straight-loop alternatives
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=1, rows_per_wave=1, waves_per_group=8, schedule=vs.VS_SCHED_LOOP)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=2, rows_per_wave=2, waves_per_group=8)
    _run_and_check(gu, oracle_mod, inp, ref=ref, schedule=vs.VS_SCHED_RESIDENT)


@pytest.mark.parametrize("name,seqs,wgs", [("C3", None, 224), ("C4", [0, 13, 27], 224), ("C2", [0, 31], 1024)])
def test_folded_launch_at_full_size(gu, oracle_mod, name, seqs, wgs):
    """bench.py's roofline launch exactly as it is timed: every layer of one step as a batch entry (28 or 32 x
    the configuration's sequence), the planner's choice - pipelined, no key split, 224 workgroups of eight waves
    (GQA) or 1024 of four (MHA). C3: every entry against the oracle; C4 (6684-token prefixes) and C2: sampled
    entries."""
    base = gen.CONFIGS[name]
    cfg = dataclasses.replace(base, B=base.layers, prefix=[base.prefix[0]] * base.layers)
    inp = gen.attention_inputs(cfg, 40 + int(name[1]))
    da = gu.DeviceAttn(inp)
    pl = da.plan()
    assert pl.schedule == vs.VS_SCHED_PIPELINED and pl.num_splits == 1 and pl.workgroups == wgs and pl.combine == 0
    got = da.run()
    assert (da.status.cpu().numpy() == 0).all()
    which = list(range(cfg.B)) if seqs is None else seqs
    ref = oracle_mod.tree_attention(inp, threads=8, seqs=which)
    worst = 0.0
    for b in which:
        gu.check_close(got[b], ref[b], *CONTRACT, what=f"{name} entry {b} contract")
        worst = max(worst, gu.check_close(got[b], ref[b], *TIGHT_LONG, what=f"{name} entry {b} tight"))
    print(f"{name} folded, {len(which)} of {cfg.B} entries: worst {worst:.3e}")


# ---------------------------------------------------------------- fuzz over shapes

def _fuzz_cases():
    cases = []
    prefixes = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 257, 700]
    k = 0
    for d in (64, 128):
        for g, hkv in ((1, 2), (2, 1), (4, 2), (7, 1), (8, 1)):
            for paged in (False, True):
                T = [1, 5, 33, 60, 64, 17, 2][k % 7]
                S = prefixes[(3 * k) % len(prefixes)]
                splits = [0, 1, 2, 3][k % 4]
                B = 1 + k % 3
                cases.append((d, g, hkv, paged, T, S, splits, B, k))
                k += 1
    return cases


@pytest.mark.parametrize("d,g,hkv,paged,T,S,splits,B,k", _fuzz_cases())
def test_fuzz_shapes(gu, oracle_mod, d, g, hkv, paged, T, S, splits, B, k):
    depth = min(6, max(1, T - 1))
    cfg = gen.Config(f"fuzz{k}", B, g * hkv, hkv, d, T, depth, 8, 100, 0.5, 1, "bf16",
                     prefix=None if paged else [max(0, S - b) for b in range(B)],
                     prefix_range=(max(0, S - 3), S + 40) if paged else None, paged=paged)
    inp = gen.attention_inputs(cfg, 1000 + k)
    ref = oracle_mod.tree_attention(inp, threads=4)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=splits)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=splits, rows_per_wave=1 + k % 2, waves_per_group=[8, 1, 4, 2][k % 4])
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=splits, waves_per_group=[4, 8][k % 2], schedule=vs.VS_SCHED_PIPELINED)
    _run_and_check(gu, oracle_mod, inp, ref=ref, num_splits=splits, schedule=vs.VS_SCHED_RESIDENT)
    _run_and_check(gu, oracle_mod, inp, ref=ref, impl=vs.VS_IMPL_GENERIC)


def test_paper_shaped_tree(gu, oracle_mod):
    """Appendix A's tree: 30 draft tokens (31 nodes), depth 3, 8 nodes per expansion."""
    parent = np.stack([gen.topk_tree(gen.rng(s, gen.STREAM_TREE)) for s in range(2)])
    cfg = gen.Config("paper-tree", 2, 28, 4, 128, 31, 3, 8, 100, 0.5, 1, "bf16", prefix=[600, 333])
    inp = gen.attention_inputs(cfg, 31, parent=parent)
    _run_and_check(gu, oracle_mod, inp)


# ---------------------------------------------------------------- mask-sensitive cases

def test_tree_dominated_no_prefix(gu, oracle_mod):
    """S = 0: every weight sits on tree keys, so a wrong mask bit cannot hide."""
    for g, T in ((7, 60), (1, 64), (4, 9)):
        cfg = gen.Config("nopre", 2, g, 1, 128, T, 6, 4, 100, 0.5, 1, "bf16", prefix=[0, 0])
        inp = gen.attention_inputs(cfg, 40 + T)
        _run_and_check(gu, oracle_mod, inp)
        _run_and_check(gu, oracle_mod, inp, schedule=vs.VS_SCHED_PIPELINED)
        _run_and_check(gu, oracle_mod, inp, schedule=vs.VS_SCHED_RESIDENT)
        _run_and_check(gu, oracle_mod, inp, impl=vs.VS_IMPL_GENERIC)


def test_mask_from_mask_build_equals_internal(gu, oracle_mod):
    import torch
    inp = gen.attention_inputs(dataclasses.replace(gen.CONFIGS["C3"], prefix=[50]), 41)
    da = gu.DeviceAttn(inp)
    a = da.run().copy()
    _, _, _, mask_dev = gu.run_mask(inp.parent)
    b = da.run(tree_mask=mask_dev)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("impl,sched", [(vs.VS_IMPL_MFMA, vs.VS_SCHED_LOOP), (vs.VS_IMPL_MFMA, vs.VS_SCHED_PIPELINED),
                                        (vs.VS_IMPL_MFMA, vs.VS_SCHED_RESIDENT), (vs.VS_IMPL_GENERIC, 0)])
def test_needles(gu, oracle_mod, impl, sched):
    """A huge key on a NON-ancestor tree slot must not move a node's output; the same key
    on an ancestor slot must pull the output to that slot's value."""
    S, T = 300, 24
    cfg = gen.Config("needle", 1, 7, 1, 128, T, 5, 3, 100, 0.5, 1, "bf16", prefix=[S])
    base = gen.attention_inputs(cfg, 42)
    _, mask, _ = oracle_mod.tree_mask(base.parent[0])
    node, head = T - 1, 3
    non_anc = [j for j in range(T) if not (int(mask[node]) >> j & 1)]
    anc = [j for j in range(T) if (int(mask[node]) >> j & 1)]
    assert non_anc and len(anc) >= 2
    ref_base = oracle_mod.tree_attention(base)

    def planted(slot, val):
        inp = gen.attention_inputs(cfg, 42)
        kq = 4.0 * inp.q[0, node, head]                       # score ~ 4*|q|^2/sqrt(d) ~ 45
        inp.k_cache[0, 0, S + slot] = kq
        inp.v_cache[0, 0, S + slot] = val
        inp.k_bits = gen.f32_to_bf16_bits(inp.k_cache)
        inp.v_bits = gen.f32_to_bf16_bits(inp.v_cache)
        inp.k_cache = gen.bf16_bits_to_f32(inp.k_bits)
        inp.v_cache = gen.bf16_bits_to_f32(inp.v_bits)
        return inp

    inp = planted(non_anc[0], 100.0)
    got = gu.DeviceAttn(inp, impl=impl, schedule=sched).run()
    gu.check_close(got[0, node, head], ref_base[0, node, head], *TIGHT_LONG, what="non-ancestor needle leaked")
    inp = planted(anc[1], 100.0)
    got = gu.DeviceAttn(inp, impl=impl, schedule=sched).run()
    ref = oracle_mod.tree_attention(inp)
    assert abs(ref[0, node, head, 0] - 100.0) < 1.0
    gu.check_close(got[0, node, head], ref[0, node, head], 0.5, 1e-2, what="ancestor needle")


def _scaled_values(cfg, seed, factor):
    """Inputs whose V rows are N(0,1) times a power of two (exact in bf16), K and q unchanged."""
    inp = gen.attention_inputs(cfg, seed)
    inp.v_cache = (inp.v_cache.astype(np.float64) * factor).astype(np.float32)
    inp.v_bits = gen.f32_to_bf16_bits(inp.v_cache)
    assert np.array_equal(gen.bf16_bits_to_f32(inp.v_bits)[np.isfinite(inp.v_cache)], inp.v_cache[np.isfinite(inp.v_cache)])
    return inp


@pytest.mark.parametrize("exp2", [-20, 10, 17, 100])       # |V| around 1e-6, 1e3, 1.3e5 (beyond fp16's 65504), 1.3e30
def test_value_range_on_every_split_schedule(gu, oracle_mod, exp2):
    """bf16 values keep fp32's exponent range, and so must everything between the kernels: the
    partial results of key splits travel through the workspace and may not narrow it. Every
    schedule with more than one split, the in-kernel merge of key parts, and the unsplit forms."""
    factor = 2.0 ** exp2
    cfg = dataclasses.replace(gen.CONFIGS["C3"], B=2, prefix=[1100, 700])
    inp = _scaled_values(cfg, 49, factor)
    ref = oracle_mod.tree_attention(inp, threads=8)
    assert np.isfinite(ref).all() and np.abs(ref).max() > 0.05 * factor
    cases = [dict(schedule=vs.VS_SCHED_LOOP, num_splits=5), dict(schedule=vs.VS_SCHED_LOOP, num_splits=3, rows_per_wave=2, waves_per_group=8),
             dict(schedule=vs.VS_SCHED_LOOP, num_splits=7, waves_per_group=1),
             dict(schedule=vs.VS_SCHED_PIPELINED, num_splits=4, waves_per_group=8), dict(schedule=vs.VS_SCHED_PIPELINED, num_splits=2, waves_per_group=4),
             dict(schedule=vs.VS_SCHED_RESIDENT), dict(schedule=vs.VS_SCHED_RESIDENT, num_splits=10 ** 6),
             dict(), dict(num_splits=1), dict(schedule=vs.VS_SCHED_PIPELINED, num_splits=1), dict(impl=vs.VS_IMPL_GENERIC)]
    for kw in cases:
        da = gu.DeviceAttn(inp, **kw)
        got = da.run()
        assert (da.status.cpu().numpy() == 0).all()
        if kw.get("num_splits", 0) not in (1,) and kw.get("impl") is None and kw:
            assert da.plan().num_splits > 1, kw
        gu.check_close(got, ref, CONTRACT[0] * factor, CONTRACT[1], what=f"contract, V x 2^{exp2}, {kw}")
        gu.check_close(got, ref, TIGHT_LONG[0] * factor, TIGHT_LONG[1], what=f"tight, V x 2^{exp2}, {kw}")


def test_channels_of_very_different_size_keep_their_relative_accuracy(gu, oracle_mod):
    """One channel of V is 2^40 times larger than its neighbours: the small channels must still come
    out to bf16 accuracy relative to their own size (a partial-result format with one exponent per
    row would flush them)."""
    cfg = dataclasses.replace(gen.CONFIGS["C3"], prefix=[900])
    inp = gen.attention_inputs(cfg, 50)
    scale_c = np.ones(cfg.d, dtype=np.float64)
    scale_c[5::16] = 2.0 ** 40
    inp.v_cache = (inp.v_cache.astype(np.float64) * scale_c).astype(np.float32)
    inp.v_bits = gen.f32_to_bf16_bits(inp.v_cache)
    ref = oracle_mod.tree_attention(inp, threads=8)
    for kw in (dict(schedule=vs.VS_SCHED_RESIDENT), dict(schedule=vs.VS_SCHED_LOOP, num_splits=6),
               dict(schedule=vs.VS_SCHED_PIPELINED, num_splits=3, waves_per_group=8)):
        got = gu.DeviceAttn(inp, **kw).run()
        err = np.abs(got - ref) / scale_c
        bound = TIGHT_LONG[0] + TIGHT_LONG[1] * np.abs(ref) / scale_c
        assert (err <= bound).all(), (kw, float((err - bound).max()))


def test_non_finite_value_in_a_masked_tree_slot(gu, oracle_mod):
    """Where the two sides differ by contract: K/V in every slot that is read must be finite. The
    oracle skips a key a node may not see, so an Inf or NaN planted in a non-ancestor's V row leaves
    that node's reference finite. The matrix-core kernels multiply such a row by a zero probability
    instead (0 x Inf = NaN), so rows that mask the slot come out non-finite there, while rows whose
    tile does not hold the slot, and the generic kernel (which skips like the oracle), stay exact."""
    S, T = 300, 24
    cfg = gen.Config("r19", 1, 7, 1, 128, T, 5, 3, 100, 0.5, 1, "bf16", prefix=[S])
    inp = gen.attention_inputs(cfg, 51)
    _, mask, _ = oracle_mod.tree_mask(inp.parent[0])
    slot = T - 2
    hides = [i for i in range(T) if not (int(mask[i]) >> slot & 1)]
    sees = [i for i in range(T) if (int(mask[i]) >> slot & 1)]
    assert hides and sees
    inp.v_cache[0, 0, S + slot, 7] = np.inf
    inp.v_bits = gen.f32_to_bf16_bits(inp.v_cache)
    ref = oracle_mod.tree_attention(inp)
    assert np.isfinite(ref[0, hides]).all() and not np.isfinite(ref[0, sees][..., 7]).any()
    got = gu.DeviceAttn(inp, impl=vs.VS_IMPL_GENERIC).run()
    gu.check_close(got[0, hides], ref[0, hides], *TIGHT_LONG, what="generic kernel skips masked keys")
    assert not np.isfinite(got[0, sees][..., 7]).any()
    for sched in (vs.VS_SCHED_LOOP, vs.VS_SCHED_PIPELINED, vs.VS_SCHED_RESIDENT):
        got = gu.DeviceAttn(inp, impl=vs.VS_IMPL_MFMA, schedule=sched, num_splits=1).run()
        assert not np.isfinite(got[0, sees][..., 7]).any()
        # documented restriction: the masked rows' channel 7 is NaN here, every other channel is right
        other = [c for c in range(cfg.d) if c != 7]
        gu.check_close(got[0, hides][..., other], ref[0, hides][..., other], *TIGHT_LONG, what=f"other channels, schedule {sched}")
        assert np.isnan(got[0, hides][..., 7]).all(), "the restriction documented for non-finite K/V no longer holds: compare with the oracle instead"


def test_redundant_image_keys_closed_form(gu):
    """Paper Eq. 3-4 on the device: R identical keys + one unique key, T = 1."""
    import math
    d, R = 128, 2048
    A, B = 0.0, math.log(512.0)
    cfg = gen.Config("eq3", 1, 1, 1, d, 1, 1, 1, 10, 0.5, 1, "bf16", prefix=[R])
    inp = gen.attention_inputs(cfg, 43)
    q = np.zeros(d, dtype=np.float32); q[0] = 1.0
    s = np.zeros(d, dtype=np.float32); s[0] = A
    t = np.zeros(d, dtype=np.float32); t[0] = 6.25; t[5] = 3.0         # 6.25 is exact in bf16
    B = 6.25
    v_s = np.full(d, 0.5, dtype=np.float32)
    v_t = np.full(d, -8.0, dtype=np.float32)
    inp.q[0, 0, 0] = q
    inp.k_cache[0, 0, :R + 1] = s
    inp.v_cache[0, 0, :R + 1] = v_s
    inp.k_cache[0, 0, 777] = t
    inp.v_cache[0, 0, 777] = v_t
    inp.scale = 1.0
    for nm in ("q", "k", "v"):
        arr = getattr(inp, nm if nm == "q" else nm + "_cache")
        setattr(inp, nm + "_bits", gen.f32_to_bf16_bits(arr))
    alpha = math.exp(B) / (R * math.exp(A) + math.exp(B))               # R redundant incl. the node's own key
    expect = alpha * (-8.0) + (1 - alpha) * 0.5
    for impl in (vs.VS_IMPL_MFMA, vs.VS_IMPL_GENERIC):
        got = gu.DeviceAttn(inp, impl=impl, num_splits=3 if impl == vs.VS_IMPL_MFMA else 0).run()
        np.testing.assert_allclose(got[0, 0, 0], expect, rtol=1e-2, atol=1e-2)


# ---------------------------------------------------------------- layout and determinism

def test_paged_equals_contiguous_bitwise(gu, oracle_mod):
    cfg = dataclasses.replace(gen.CONFIGS["C5"], B=3, prefix_range=(900, 1400))
    inp = gen.attention_inputs(cfg, 44)
    da = gu.DeviceAttn(inp, num_splits=2)
    paged = da.run().copy()
    bs = cfg.block_size
    # same tokens, gathered into a contiguous cache
    cap = int(inp.prefix_len.max()) + cfg.T + 3
    kb = np.full((cfg.B, cfg.Hkv, cap, cfg.d), gen.BF16_NAN_BITS, dtype=np.uint16)
    vb = kb.copy()
    for b in range(cfg.B):
        n = int(inp.prefix_len[b]) + cfg.T
        nb = (n + bs - 1) // bs
        ids = inp.block_table[b, :nb]
        kb[b, :, :n] = inp.k_bits[ids].transpose(1, 0, 2, 3).reshape(cfg.Hkv, nb * bs, cfg.d)[:, :n]
        vb[b, :, :n] = inp.v_bits[ids].transpose(1, 0, 2, 3).reshape(cfg.Hkv, nb * bs, cfg.d)[:, :n]
    cfg2 = dataclasses.replace(cfg, paged=False)
    inp2 = gen.AttnInputs(cfg2, inp.prefix_len, inp.parent, inp.q, gen.bf16_bits_to_f32(kb), gen.bf16_bits_to_f32(vb),
                          cap=cap, scale=inp.scale, q_bits=inp.q_bits, k_bits=kb, v_bits=vb)
    cont = gu.DeviceAttn(inp2, num_splits=2).run()
    assert np.array_equal(paged, cont)
    # the pipelined kernel: paged copies take the general path, contiguous ones the fast path
    kw = dict(num_splits=2, waves_per_group=8, schedule=vs.VS_SCHED_PIPELINED)
    assert np.array_equal(gu.DeviceAttn(inp, **kw).run(), gu.DeviceAttn(inp2, **kw).run())
    # the resident kernel: the contiguous cache is NaN past each sequence's end, which its
    # copies read (they start before the sequence's length is known) and must discard
    kw = dict(num_splits=0, schedule=vs.VS_SCHED_RESIDENT)
    assert np.array_equal(gu.DeviceAttn(inp, **kw).run(), gu.DeviceAttn(inp2, **kw).run())


def test_deterministic_and_untouched_guards(gu):
    import torch
    inp = gen.attention_inputs(gen.CONFIGS["C3"], 45)
    da = gu.DeviceAttn(inp)
    a = da.run().copy()
    da.out.fill_(float("nan"))
    b = da.run()
    assert np.array_equal(a, b)
    assert np.isfinite(b).all()


@pytest.mark.parametrize("sched,kw", [
    (vs.VS_SCHED_LOOP, {}), (vs.VS_SCHED_LOOP, {"rows_per_wave": 2, "waves_per_group": 8, "num_splits": 2}),
    (vs.VS_SCHED_PIPELINED, {"waves_per_group": 8}), (vs.VS_SCHED_PIPELINED, {"waves_per_group": 4, "num_splits": 3}),
    (vs.VS_SCHED_RESIDENT, {}), (vs.VS_SCHED_RESIDENT, {"num_splits": 10 ** 6}),
])
@pytest.mark.parametrize("B,S", [(1, 50), (1, 1696), (4, 700)])
def test_repeated_runs_bit_identical(gu, sched, kw, B, S):
    """Nothing in a kernel may depend on timing: the same launch gives the same bits every time
    (plain tiles, masked tiles, the merge of key parts and the split combine all take part)."""
    cfg = dataclasses.replace(gen.CONFIGS["C3"], B=B, prefix=[S - 13 * b for b in range(B)])
    da = gu.DeviceAttn(gen.attention_inputs(cfg, 48), schedule=sched, **kw)
    first = da.run().copy()
    assert np.isfinite(first).all()
    for rep in range(5):
        assert np.array_equal(da.run(), first), f"run {rep + 2} differs from the first"


def test_max_prefix_bound_larger_than_actual(gu, oracle_mod):
    """The host bound only sizes the launch: splits past a sequence's end are empty."""
    cfg = dataclasses.replace(gen.CONFIGS["C3"], prefix=[130])
    inp = gen.attention_inputs(cfg, 46, extra_cap=4000)
    _run_and_check(gu, oracle_mod, inp, max_prefix_len=3000, num_splits=9)
    _run_and_check(gu, oracle_mod, inp, max_prefix_len=3000, num_splits=9, schedule=vs.VS_SCHED_PIPELINED)
    _run_and_check(gu, oracle_mod, inp, max_prefix_len=3000, schedule=vs.VS_SCHED_RESIDENT)


# ---------------------------------------------------------------- data-dependent errors

def test_status_reports_bad_inputs_without_faulting(gu):
    import torch
    cfg = gen.Config("bad", 4, 4, 2, 64, 6, 3, 3, 10, 0.5, 1, "bf16", prefix_range=(20, 60), paged=True)
    inp = gen.attention_inputs(cfg, 47)
    inp.parent[1] = [-1, 0, 2, 1, 0, 0]            # parent[2] = 2 is not < 2
    inp.prefix_len[2] = 10 ** 6                    # beyond the cache
    inp.block_table[3, 0] = 10 ** 7                # outside the pool
    for impl, sched in ((vs.VS_IMPL_MFMA, vs.VS_SCHED_LOOP), (vs.VS_IMPL_MFMA, vs.VS_SCHED_PIPELINED),
                        (vs.VS_IMPL_MFMA, vs.VS_SCHED_RESIDENT), (vs.VS_IMPL_GENERIC, 0)):
        da = gu.DeviceAttn(inp, impl=impl, max_prefix_len=60, schedule=sched)
        da.run()
        st = da.status.cpu().numpy()
        assert list(st) == [0, 2, 3, 4], st
        good = da.out[0].float().cpu().numpy()
        assert np.isfinite(good).all()
