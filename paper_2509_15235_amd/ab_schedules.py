"""A/B timing of tree-verify attention launch plans on one GPU.

Times `vs_tree_verify_attention` per call for several (schedule, key splits) choices of one shape,
the way a model would issue the calls: `--layers` dependent calls per buffer set, every set with its
own K/V (so that a call's K/V is cold in the caches once `--sets x --layers` layers exceed them), all
replayed from one HIP graph per variant. The variants alternate inside one process and every
variant is timed `--reps` times, so differences of a fraction of a percent are visible; numbers
from different processes or boxes differ by more than that.

    python -m paper_2509_15235_amd.ab_schedules --variants 0:0,1:0,2:0,3:0
    python -m paper_2509_15235_amd.ab_schedules --B 8 --layers 8 --sets 4 --variants 1:0,1:4,2:0

A variant is `schedule:num_splits` with schedule 0 = AUTO, 1 = LOOP, 2 = PIPELINED, 3 = RESIDENT and
num_splits 0 = the planner's choice. The launch planner's thresholds were set from such runs.
"""
from __future__ import annotations

import argparse
import sys


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--B", type=int, default=1, help="sequences per call")
    ap.add_argument("--S", type=int, default=1696, help="prefix length of every sequence")
    ap.add_argument("--T", type=int, default=60, help="tree nodes")
    ap.add_argument("--Hq", type=int, default=28)
    ap.add_argument("--Hkv", type=int, default=4)
    ap.add_argument("--d", type=int, default=128, choices=[64, 128])
    ap.add_argument("--layers", type=int, default=28, help="calls per buffer set")
    ap.add_argument("--sets", type=int, default=8, help="buffer sets (sets x layers x K/V of a layer should exceed 256 MB)")
    ap.add_argument("--variants", default="0:0,1:0,2:0,3:0")
    ap.add_argument("--reps", type=int, default=6)
    ap.add_argument("--no-mask", action="store_true", help="let every call derive the ancestor masks itself")
    a = ap.parse_args(argv)

    import torch
    import paper_2509_15235_amd as vs
    if not torch.cuda.is_available():
        print("ab_schedules: no GPU", file=sys.stderr)
        return 3
    vs.lib()
    dev = torch.device("cuda:0")
    B, S, T, Hq, Hkv, d, L = a.B, a.S, a.T, a.Hq, a.Hkv, a.d, a.layers
    cap = S + T + 4
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    sets = []
    for _ in range(a.sets):
        q = torch.randn((L, B, T, Hq, d), generator=g, device=dev).to(torch.bfloat16)
        k = torch.randn((L, B, Hkv, cap, d), generator=g, device=dev).to(torch.bfloat16)
        v = torch.randn((L, B, Hkv, cap, d), generator=g, device=dev).to(torch.bfloat16)
        sets.append((q, k, v, torch.empty_like(q)))
    # a ternary tree in level order: node i's parent is (i - 1) // 3
    parent = torch.tensor([[-1] + [(i - 1) // 3 for i in range(1, T)]] * B, device=dev, dtype=torch.int32)
    prefix = torch.full((B,), S, device=dev, dtype=torch.int32)
    status = torch.zeros(B, device=dev, dtype=torch.int32)
    mask = torch.zeros((B, T), device=dev, dtype=torch.int64)
    depth = torch.zeros((B, T), device=dev, dtype=torch.int32)
    rc = vs.vs_tree_mask_build(parent, B, T, mask, depth, status, torch.cuda.current_stream().cuda_stream)
    assert rc == 0, vs.vs_strerror(rc)
    torch.cuda.synchronize()
    mk = None if a.no_mask else mask

    graphs = {}
    stream = torch.cuda.Stream()
    for var in a.variants.split(","):
        sched, sp = (int(x) for x in var.split(":"))
        desc = vs.AttnDesc(B=B, T=T, Hq=Hq, Hkv=Hkv, d=d, dtype=vs.VS_BF16, softmax_scale=d ** -0.5, max_prefix_len=S,
                           capacity=cap, stride_seq=Hkv * cap * d, stride_head=cap * d, stride_tok=d, num_splits=sp,
                           schedule=sched)
        rc, plan = vs.vs_attention_plan(desc)
        if rc != 0:
            print(f"{var}: {vs.vs_strerror(rc)}")
            continue
        nb = vs.vs_attention_workspace_bytes(desc)
        ws = torch.empty(max(nb, 256), device=dev, dtype=torch.uint8)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=stream):
            st = torch.cuda.current_stream().cuda_stream
            for (q, k, v, o) in sets:
                for l in range(L):
                    rc = vs.vs_tree_verify_attention(desc, q[l], k[l], v[l], prefix, parent, mk, o[l], status, ws, nb, st)
                    assert rc == 0, vs.vs_strerror(rc)
        graphs[var] = (gr, plan, ws)
    ncalls = a.sets * L
    res = {v: [] for v in graphs}
    for _ in range(a.reps):
        for var, (gr, plan, ws) in graphs.items():
            for _ in range(3):
                gr.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            res[var].append(e0.elapsed_time(e1) / (10 * ncalls) * 1e3)
    names = {vs.VS_SCHED_LOOP: "loop", vs.VS_SCHED_PIPELINED: "pipelined", vs.VS_SCHED_RESIDENT: "resident"}
    for var, (gr, plan, ws) in graphs.items():
        r = sorted(res[var])
        print(f"{var:6s} {names.get(plan.schedule, '?'):9s} splits={plan.num_splits:3d} keys/split={plan.keys_per_split:5d} "
              f"workgroups={plan.workgroups:5d} waves={plan.waves_per_group}  us/call: min {r[0]:.2f} median {r[len(r) // 2]:.2f} "
              f"max {r[-1]:.2f}", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
