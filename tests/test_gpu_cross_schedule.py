"""Randomised cross-check of every MFMA schedule against the generic kernel (fp32 arithmetic on the
same bf16 inputs; itself checked against the oracle elsewhere), with every launch repeated: shapes
the fixed parity cases do not list - odd group sizes, ragged batches, paged caches with small
blocks, key ranges that end anywhere inside a tile, host bounds far above the actual lengths."""
import numpy as np
import pytest

import gen
import paper_2509_15235_amd as vs

pytestmark = pytest.mark.gpu


def _cases(n):
    r = np.random.default_rng(20240917)
    out = []
    for k in range(n):
        d = int(r.choice([64, 128]))
        hkv = int(r.choice([1, 2, 3, 4]))
        g = int(r.choice([1, 2, 3, 4, 5, 7, 8]))
        T = int(r.choice([1, 2, 7, 16, 31, 32, 33, 48, 60, 63, 64]))
        B = int(r.integers(1, 5))
        paged = bool(r.integers(0, 2))
        smax = int(r.choice([40, 130, 300, 700, 1500, 2600]))
        lo = int(r.integers(0, smax))
        bound_slack = int(r.choice([0, 0, 17, 900]))
        splits = int(r.choice([0, 0, 1, 2, 5, 13]))
        block = int(r.choice([16, 32, 128]))
        out.append((k, d, hkv, g, T, B, paged, lo, smax, bound_slack, splits, block))
    return out


@pytest.mark.parametrize("k,d,hkv,g,T,B,paged,lo,smax,slack,splits,block", _cases(48))
def test_schedules_agree_with_generic_kernel(k, d, hkv, g, T, B, paged, lo, smax, slack, splits, block):
    import gpu_util as gu
    depth = min(6, max(1, T - 1))
    if paged:
        cfg = gen.Config(f"x{k}", B, g * hkv, hkv, d, T, depth, 8, 100, 0.5, 1, "bf16", prefix_range=(lo, smax + 1),
                         paged=True, block_size=block)
    else:
        pre = [int(v) for v in np.random.default_rng(k).integers(lo, smax + 1, size=B)]
        cfg = gen.Config(f"x{k}", B, g * hkv, hkv, d, T, depth, 8, 100, 0.5, 1, "bf16", prefix=pre)
    inp = gen.attention_inputs(cfg, 3000 + k, extra_cap=slack + 5)
    bound = int(inp.prefix_len.max()) + slack
    if paged:   # the table's row length caps what the host may claim
        bound = min(bound, inp.block_table.shape[1] * block - T)
    ref = gu.DeviceAttn(inp, impl=vs.VS_IMPL_GENERIC, max_prefix_len=bound).run().copy()
    assert np.isfinite(ref).all()
    tol = (1.5e-3, 6e-3) if int(inp.prefix_len.min()) >= 256 else (1.2e-2, 6e-3)
    variants = [dict(schedule=vs.VS_SCHED_LOOP, rows_per_wave=1 + k % 2, waves_per_group=[1, 2, 4, 8][k % 4]),
                dict(schedule=vs.VS_SCHED_LOOP),
                dict(schedule=vs.VS_SCHED_PIPELINED, waves_per_group=[4, 8][k % 2]),
                dict(schedule=vs.VS_SCHED_RESIDENT),
                dict()]
    for kw in variants:
        da = gu.DeviceAttn(inp, max_prefix_len=bound, num_splits=splits, **kw)
        got = da.run().copy()
        assert (da.status.cpu().numpy() == 0).all()
        gu.check_close(got, ref, *tol, what=f"case {k} {kw} plan splits {da.plan().num_splits}")
        da.out.fill_(float("nan"))
        assert np.array_equal(da.run(), got), f"case {k} {kw}: second run differs"
