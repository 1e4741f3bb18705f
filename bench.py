#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

A step = one pass of the whole path for one speculative cycle of the named workload:
    1 x vs_tree_mask_build  +  L x vs_tree_verify_attention (one per decoder layer)
    +  1 x vs_tree_accept
over synthetic inputs already resident in HBM (seeded N(0,1) Q/K/V, logits with planted
matches; they stand in for the paper's benchmark prompts and model weights). Projections,
RoPE, MLPs and the LM head are not part of the step.

Prints ONE JSON line: verify steps/s as `value`, plus
  roofline      the attention kernel with the step's L layers folded into one launch as
                independent batch entries (same per-layer shape), timed with HIP events
  per_layer_call  the same kernel launched for a single layer (B = 1), launch-bound
  argmax        the logits scan of vs_tree_accept against HBM bandwidth
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C3", choices=["C2", "C3", "C4"])
    ap.add_argument("--sets", type=int, default=0, help="distinct buffer sets to rotate over (0 = enough to exceed 512 MB)")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every launch from Python instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the attention legs of the other configurations (C2 / C4 folded, C5 ragged batch)")
    ap.add_argument("--only-leg", default="", choices=["", "C2", "C4", "C5"],
                    help="run nothing but this configuration's attention leg and print its block (for profiler runs)")
    ap.add_argument("--leg-schedule", type=int, default=0, help="vs_attn_schedule of --only-leg (0: the planner's choice)")
    ap.add_argument("--leg-splits", type=int, default=0, help="num_splits of --only-leg")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--folded-splits", type=int, default=0)
    ap.add_argument("--seed", type=int, default=2024)
    return ap.parse_args()


def other_config_leg(vs, gen, torch, dev, stream, gtorch, name, seed, check, num_splits=0, schedule=0):
    """Attention of one of the other configurations on device-generated data; returns a roofline block.
    C2 / C4: the L layers folded into one launch (contiguous caches); C5: one layer of the ragged batch
    over a paged cache with a shuffled block table."""
    import numpy as np
    cfg = gen.CONFIGS[name]
    T, Hq, Hkv, d, eb = cfg.T, cfg.Hq, cfg.Hkv, cfg.d, 2
    scale = 1.0 / np.sqrt(d)
    sp = stream.cuda_stream
    if cfg.paged:
        S_b, _ = gen.draw_prefix(cfg, seed)
        B = cfg.B
        parent_h = gen.draw_trees(cfg, seed)
        bs = cfg.block_size
        nblk = (S_b.astype(np.int64) + T + bs - 1) // bs
        n_blocks = int(nblk.sum()) + 3
        perm = gen.rng(seed, gen.STREAM_BLOCKS).permutation(n_blocks).astype(np.int32)
        max_blocks = int(nblk.max()) + 1
        table_h = np.zeros((B, max_blocks), dtype=np.int32)
        at = 0
        for b in range(B):
            table_h[b, :nblk[b]] = perm[at:at + nblk[b]]
            at += int(nblk[b])
        table = torch.from_numpy(table_h).to(dev)
        kv_shape = (n_blocks, Hkv, bs, d)
        launch = f"one layer of the ragged batch: B={B}, prefixes {int(S_b.min())}..{int(S_b.max())}, paged cache"
        layers_per_call = 1
    else:
        B = cfg.layers
        S_b = np.full(B, cfg.prefix[0], dtype=np.int32)
        parent_h = np.repeat(gen.draw_trees(cfg, seed), B, axis=0)
        cap = int(S_b[0]) + T + 4
        kv_shape = (B, Hkv, cap, d)
        table = None
        launch = f"B={B} proxy: {B} layers folded into one launch as independent batch entries"
        layers_per_call = B
    kv_bytes = 2 * int(np.prod(kv_shape)) * eb
    nsets = max(2, int(np.ceil(600e6 / kv_bytes)))
    sets = []
    for _ in range(nsets):
        sets.append(dict(
            q=torch.randn((B, T, Hq, d), generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16),
            k=torch.randn(kv_shape, generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16),
            v=torch.randn(kv_shape, generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16),
            out=torch.empty((B, T, Hq, d), device=dev, dtype=torch.bfloat16)))
    desc = vs.AttnDesc(B=B, T=T, Hq=Hq, Hkv=Hkv, d=d, dtype=vs.VS_BF16, softmax_scale=float(scale),
                       max_prefix_len=int(S_b.max()), impl=vs.VS_IMPL_AUTO, num_splits=num_splits, schedule=schedule)
    if cfg.paged:
        desc.paged, desc.block_size, desc.max_blocks, desc.num_blocks = 1, bs, max_blocks, n_blocks
        desc.stride_block, desc.stride_head, desc.stride_tok = Hkv * bs * d, bs * d, d
        desc.block_table = table.data_ptr()
    else:
        desc.paged, desc.capacity = 0, cap
        desc.stride_seq, desc.stride_head, desc.stride_tok = Hkv * cap * d, cap * d, d
    rc, plan = vs.vs_attention_plan(desc)
    assert rc == 0
    ws_bytes = max(vs.vs_attention_workspace_bytes(desc), 256)
    ws = torch.empty(ws_bytes, device=dev, dtype=torch.uint8)
    parent = torch.from_numpy(parent_h.astype(np.int32)).to(dev)
    prefix = torch.from_numpy(S_b.astype(np.int32)).to(dev)
    mask = torch.zeros((B, T), device=dev, dtype=torch.int64)
    depth = torch.zeros((B, T), device=dev, dtype=torch.int32)
    status = torch.zeros((B,), device=dev, dtype=torch.int32)
    check(vs.vs_tree_mask_build(parent, B, T, mask, depth, status, sp))
    stream.synchronize()
    depth_h = depth.cpu().numpy()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for st in sets:
            check(vs.vs_tree_verify_attention(desc, st["q"], st["k"], st["v"], prefix, parent, mask, st["out"], status,
                                              ws, ws_bytes, torch.cuda.current_stream().cuda_stream))
    with torch.cuda.stream(stream):
        t_end = time.perf_counter() + 0.15                                               # let the clocks settle
        while time.perf_counter() < t_end:
            g.replay()
            stream.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        reps = 40
        e0.record(stream)
        for _ in range(reps):
            g.replay()
        e1.record(stream)
        stream.synchronize()
    ms = e0.elapsed_time(e1) / reps / nsets
    assert int(status.abs().max().item()) == 0
    vis_pairs = int(sum(int(S_b[b]) + int(dd) + 1 for b in range(B) for dd in depth_h[b]))
    flops = 4.0 * d * Hq * vis_pairs
    nbytes = float(sum(2.0 * Hkv * (int(S_b[b]) + T) * d * eb for b in range(B)) + 2.0 * B * T * Hq * d * eb)
    t_mfma, t_hbm = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
    tf, gbs = flops / (ms * 1e-3) / 1e12, nbytes / (ms * 1e-3) / 1e9
    blk = {"bound": "mfma" if t_mfma >= t_hbm else "hbm"}
    if blk["bound"] == "mfma":
        blk.update({"achieved": round(tf, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)})
    else:
        blk.update({"achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)})
    sched = {vs.VS_SCHED_PIPELINED: "attn_mfma_pipe_kernel", vs.VS_SCHED_BALANCED: "attn_mfma_pipe_kernel (balanced shares)",
             vs.VS_SCHED_RESIDENT: "attn_mfma_resident_kernel"}.get(plan.schedule, "attn_mfma_kernel")
    blk.update({"traffic": None, "workload": cfg.name, "launch": launch, "us_per_launch": round(ms * 1e3, 2),
                "tflops": round(tf, 2), "hbm_gbs": round(gbs, 1), "workgroups": plan.workgroups, "num_splits": plan.num_splits,
                "kernel": sched + (" + attn_combine_kernel" if plan.combine else ""),
                "layers_per_launch": layers_per_call, "buffer_sets": nsets, "data": "device-generated N(0,1)"})
    del sets
    torch.cuda.empty_cache()
    return blk


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no cross-GPU part); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import gen
    import paper_2509_15235_amd as vs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    vs.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.only_leg:
        def check_rc(rc):
            if rc != 0:
                raise RuntimeError(f"libvispec_verify: {vs.vs_strerror(rc)} ({rc})")
        gleg = torch.Generator(device=dev)
        gleg.manual_seed(args.seed)
        blk = other_config_leg(vs, gen, torch, dev, torch.cuda.Stream(device=dev), gleg, args.only_leg, args.seed, check_rc,
                               num_splits=args.leg_splits, schedule=args.leg_schedule)
        print(json.dumps({"leg": args.only_leg, **blk}))
        return

    cfg = gen.CONFIGS[args.config]
    L, T, Hq, Hkv, d, V = cfg.layers, cfg.T, cfg.Hq, cfg.Hkv, cfg.d, cfg.V
    S = int(cfg.prefix[0])
    group = Hq // Hkv
    cap = S + T + 4
    scale = 1.0 / np.sqrt(d)
    eb = 2

    # ---------------------------------------------------------------- inputs
    parent_h = gen.draw_trees(cfg, args.seed)                       # [1, T]
    host_layers = [gen.attention_inputs(cfg, args.seed, layer=l, poison_tail=False, parent=parent_h, extra_cap=4)
                   for l in range(L)]
    acc_h = gen.accept_inputs(cfg, args.seed, parent=parent_h)

    kv_bytes_set = 2 * L * Hkv * cap * d * eb
    logit_bytes = T * V * 4
    nsets = args.sets if args.sets > 0 else max(2, int(np.ceil(600e6 / (kv_bytes_set + logit_bytes))))

    def bf16_dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    gtorch = torch.Generator(device=dev)
    gtorch.manual_seed(args.seed)
    sets = []
    for s in range(nsets):
        if s == 0:
            q = bf16_dev(np.concatenate([h.q_bits for h in host_layers], axis=0))          # [L,T,Hq,d]
            k = bf16_dev(np.concatenate([h.k_bits for h in host_layers], axis=0))          # [L,Hkv,cap,d]
            v = bf16_dev(np.concatenate([h.v_bits for h in host_layers], axis=0))
            logits = torch.from_numpy(acc_h.logits[0]).to(dev)                             # [T,V]
        else:
            q = torch.randn((L, T, Hq, d), generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16)
            k = torch.randn((L, Hkv, cap, d), generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16)
            v = torch.randn((L, Hkv, cap, d), generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16)
            logits = torch.randn((T, V), generator=gtorch, device=dev, dtype=torch.float32)
        out = torch.empty((L, T, Hq, d), device=dev, dtype=torch.bfloat16)
        sets.append(dict(q=q, k=k, v=v, out=out, logits=logits))

    parent1 = torch.from_numpy(parent_h.astype(np.int32)).to(dev)                          # [1,T]
    parentL = parent1.repeat(L, 1).contiguous()                                            # [L,T]
    prefix1 = torch.full((1,), S, device=dev, dtype=torch.int32)
    prefixL = torch.full((L,), S, device=dev, dtype=torch.int32)
    tokens = torch.from_numpy(acc_h.tokens.astype(np.int32)).to(dev)
    mask = torch.zeros((1, T), device=dev, dtype=torch.int64)
    maskL = torch.zeros((L, T), device=dev, dtype=torch.int64)
    depth = torch.zeros((L, T), device=dev, dtype=torch.int32)
    status = torch.zeros((L,), device=dev, dtype=torch.int32)
    alen = torch.zeros((1,), device=dev, dtype=torch.int32)
    path = torch.zeros((1, T), device=dev, dtype=torch.int32)
    bonus = torch.zeros((1,), device=dev, dtype=torch.int32)
    amax = torch.zeros((1, T), device=dev, dtype=torch.int32)

    def make_desc(B, num_splits):
        dsc = vs.AttnDesc(B=B, T=T, Hq=Hq, Hkv=Hkv, d=d, dtype=vs.VS_BF16, softmax_scale=float(scale),
                          max_prefix_len=S, paged=0, capacity=cap, stride_seq=Hkv * cap * d,
                          stride_head=cap * d, stride_tok=d, impl=vs.VS_IMPL_AUTO, num_splits=num_splits)
        return dsc

    desc1 = make_desc(1, args.num_splits)
    descL = make_desc(L, args.folded_splits)
    rc1, plan1 = vs.vs_attention_plan(desc1)
    rcL, planL = vs.vs_attention_plan(descL)
    assert rc1 == 0 and rcL == 0
    ws_bytes = max(vs.vs_attention_workspace_bytes(desc1), vs.vs_attention_workspace_bytes(descL), 256)
    ws = torch.empty(ws_bytes, device=dev, dtype=torch.uint8)
    aws_bytes = vs.vs_accept_workspace_bytes(1, T, V)
    aws = torch.empty(aws_bytes, device=dev, dtype=torch.uint8)
    lay_q = T * Hq * d * eb
    lay_kv = Hkv * cap * d * eb

    def check(rc):
        if rc != 0:
            raise vs.VSError(rc, "libvispec_verify")

    def enqueue_step(st, stream):
        check(vs.vs_tree_mask_build(parent1, 1, T, mask, depth, status, stream))
        qp, kp, vp, op = st["q"].data_ptr(), st["k"].data_ptr(), st["v"].data_ptr(), st["out"].data_ptr()
        for l in range(L):
            check(vs.vs_tree_verify_attention(desc1, qp + l * lay_q, kp + l * lay_kv, vp + l * lay_kv, prefix1,
                                              parent1, mask, op + l * lay_q, status, ws, ws_bytes, stream))
        check(vs.vs_tree_accept(st["logits"], V, V, tokens, parent1, 1, T, alen, path, bonus, amax, status,
                                aws, aws_bytes, stream))

    def enqueue_folded(st, stream):
        check(vs.vs_tree_verify_attention(descL, st["q"], st["k"], st["v"], prefixL, parentL, maskL, st["out"],
                                          status, ws, ws_bytes, stream))

    kvdesc = vs.KVDesc(B=1, T=T, Hkv=Hkv, d=d, dtype=vs.VS_BF16, num_layers=L, stride_layer=Hkv * cap * d, paged=0,
                       capacity=cap, stride_seq=Hkv * cap * d, stride_head=cap * d, stride_tok=d)
    new_prefix = torch.zeros((1,), device=dev, dtype=torch.int32)

    def enqueue_commit(st, stream):
        check(vs.vs_tree_kv_commit(kvdesc, st["k"], st["v"], prefix1, path, alen, new_prefix, status, stream))

    def enqueue_accept(st, stream):
        check(vs.vs_tree_accept(st["logits"], V, V, tokens, parent1, 1, T, alen, path, bonus, amax, status,
                                aws, aws_bytes, stream))

    # stochastic acceptance (temperature 1) and draft-tree construction (Appendix A: K = 8, depth 3, N = 30):
    # the rows built beyond the greedy step; timed separately, not part of `value`
    ua_h, ub_h = gen.uniforms(args.seed, 1, T)
    u_acc, u_bon = torch.from_numpy(ua_h).to(dev), torch.from_numpy(ub_h).to(dev)
    sws_bytes = vs.vs_accept_sample_workspace_bytes(1, T, V)
    sws = torch.empty(sws_bytes, device=dev, dtype=torch.uint8)
    s_alen, s_path, s_bonus = torch.zeros_like(alen), torch.zeros_like(path), torch.zeros_like(bonus)

    def enqueue_sample(st, stream):
        check(vs.vs_tree_accept_sample(st["logits"], V, V, 1.0, tokens, parent1, u_acc, u_bon, 1, T, s_alen, s_path,
                                       s_bonus, status, sws, sws_bytes, stream))

    DK, DD, DN = 8, 3, 30
    dcap = DK + (DD - 1) * DK * DK
    d_tok = torch.zeros((1, dcap), device=dev, dtype=torch.int32)
    d_par = torch.zeros((1, dcap), device=dev, dtype=torch.int32)
    d_score = torch.zeros((1, dcap), device=dev, dtype=torch.float32)
    d_front = [torch.zeros((1, DK), device=dev, dtype=torch.int32) for _ in range(DD)]
    d_cum = [torch.zeros((1, DK), device=dev, dtype=torch.float32) for _ in range(DD)]
    d_parent = torch.zeros((1, DN + 1), device=dev, dtype=torch.int32)
    d_tokens, d_cand = torch.zeros_like(d_parent), torch.zeros_like(d_parent)
    d_num = torch.zeros((1,), device=dev, dtype=torch.int32)
    dws_bytes = vs.vs_draft_expand_workspace_bytes(1, DK, V, DK)
    dws = torch.empty(dws_bytes, device=dev, dtype=torch.uint8)
    draft_rows = 1 + (DD - 1) * DK                                                        # logits rows one tree reads

    def enqueue_draft(st, stream):
        # the target's logits rows stand in for the draft model's (same shape and distribution)
        lg = st["logits"].data_ptr()
        row, base = 0, 0
        for level in range(DD):
            F = 1 if level == 0 else DK
            check(vs.vs_draft_expand(lg + row * V * 4, V, V, None if level == 0 else d_cum[level - 1],
                                     None if level == 0 else d_front[level - 1], 1, F, DK, base, dcap, d_tok, d_score,
                                     d_par, d_front[level], d_cum[level], dws, dws_bytes, stream))
            row += F
            base += F * DK
        check(vs.vs_draft_tree_build(d_tok, d_score, d_par, 1, dcap, dcap, DN, None, d_parent, d_tokens, d_cand, d_num,
                                     status, stream))

    # the vision adaptor's compression attention on the same buffers: T query vectors over the image's
    # embeddings (C3: 1296 image tokens), one image, one (adaptor) layer
    n_img = min(1296, S)
    desc_c = vs.AttnDesc(B=1, T=T, Hq=Hq, Hkv=Hkv, d=d, dtype=vs.VS_BF16, softmax_scale=float(scale),
                         max_prefix_len=n_img, paged=0, capacity=cap, stride_seq=Hkv * cap * d, stride_head=cap * d,
                         stride_tok=d)
    len_c = torch.full((1,), n_img, device=dev, dtype=torch.int32)
    cws_bytes = vs.vs_compress_attention_workspace_bytes(desc_c)
    cws = torch.empty(max(cws_bytes, 256), device=dev, dtype=torch.uint8)
    out_c = torch.empty((1, T, Hq, d), device=dev, dtype=torch.bfloat16)

    def enqueue_compress(st, stream):
        check(vs.vs_compress_attention(desc_c, st["q"], st["k"], st["v"], len_c, out_c, status, cws, cws_bytes, stream))

    stream = torch.cuda.Stream(device=dev)
    sp = stream.cuda_stream
    check(vs.vs_tree_mask_build(parentL, L, T, maskL, depth, status, sp))
    stream.synchronize()

    # ---------------------------------------------------------------- parity spot check (layer 0 of set 0)
    import oracle
    with torch.cuda.stream(stream):
        enqueue_step(sets[0], sp)
    stream.synchronize()
    ref0 = oracle.tree_attention(host_layers[0], threads=min(os.cpu_count() or 1, 16))
    got0 = sets[0]["out"][0].float().cpu().numpy()
    err0 = float(np.abs(got0 - ref0[0]).max())
    o_amax, o_alen, o_path, o_bonus = oracle.tree_accept(acc_h.logits, acc_h.tokens, acc_h.parent)
    accept_ok = bool((amax.cpu().numpy() == o_amax).all() and alen.item() == o_alen[0] and bonus.item() == o_bonus[0]
                     and (path.cpu().numpy() == o_path).all())
    # commit of the accepted path: every layer of set 0 against the oracle, byte for byte
    with torch.cuda.stream(stream):
        enqueue_commit(sets[0], sp)
    stream.synchronize()
    commit_ok = int(new_prefix.item()) == S + int(o_alen[0]) + 1
    for name, bits in (("k", "k_bits"), ("v", "v_bits")):
        got = sets[0][name].view(torch.int16).cpu().numpy().view(np.uint16)                # [L,Hkv,cap,d]
        for l in range(L):
            want = getattr(host_layers[l], bits)[0].copy()
            oracle.kv_commit_seq(want, S, o_path[0], int(o_alen[0]))
            commit_ok = commit_ok and bool(np.array_equal(got[l], want))
    # stochastic acceptance: the GPU's outcome must be one the rule allows within the fp32 error bound
    with torch.cuda.stream(stream):
        enqueue_sample(sets[0], sp)
        enqueue_draft(sets[0], sp)
    stream.synchronize()
    rc_s, _ = oracle.tree_accept_sample_check_seq(acc_h.logits[0], acc_h.tokens[0], acc_h.parent[0], 1.0,
                                                  ua_h[0].astype(np.float64), float(ub_h[0]), int(s_alen.item()),
                                                  s_path.cpu().numpy()[0], int(s_bonus.item()), 2e-5)
    sample_ok = rc_s == 0
    # draft tree: the final selection, bit for bit, from the candidates the GPU produced; first level against the oracle
    rc_d, o_par, o_tok, o_cand = oracle.draft_tree_build_seq(d_tok.cpu().numpy()[0], d_score.cpu().numpy()[0],
                                                             d_par.cpu().numpy()[0], DN)
    rc_e, e_tok, e_sc, _, _ = oracle.draft_expand_seq(acc_h.logits[0][:1], np.zeros(1, np.float32), DK)
    draft_ok = bool(rc_d == 0 and rc_e == 0 and int(d_num.item()) == DN + 1
                    and (d_parent.cpu().numpy()[0] == o_par).all() and (d_tokens.cpu().numpy()[0] == o_tok).all()
                    and (d_tok.cpu().numpy()[0, :DK] == e_tok).all()
                    and np.abs(d_score.cpu().numpy()[0, :DK] - e_sc).max() <= 3e-5)
    with torch.cuda.stream(stream):
        enqueue_compress(sets[0], sp)
    stream.synchronize()
    ref_c = oracle.compress_attention_seq(host_layers[0].q[0], host_layers[0].k_cache[0], host_layers[0].v_cache[0],
                                          n_img, scale, Hkv)
    err_c = float(np.abs(out_c[0].float().cpu().numpy() - ref_c).max())
    if not (err0 <= 2e-2 and accept_ok and commit_ok and sample_ok and draft_ok and err_c <= 2e-2):
        print(f"bench.py: parity check failed (attention max|err| {err0}, accept ok {accept_ok}, commit ok {commit_ok}, "
              f"sample ok {sample_ok}, draft ok {draft_ok}, compression attention max|err| {err_c})", file=sys.stderr)
        sys.exit(4)

    # ---------------------------------------------------------------- runners (HIP graphs or eager)
    def build_runner(enq):
        if args.no_graph:
            return [(lambda st=st: enq(st, sp)) for st in sets]
        graphs = []
        for st in sets:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                enq(st, torch.cuda.current_stream().cuda_stream)
            graphs.append(g)
        return [g.replay for g in graphs]

    def timed(runner, iters, warmup):
        with torch.cuda.stream(stream):
            for i in range(warmup):
                runner[i % nsets]()
            stream.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record(stream)
            for i in range(iters):
                runner[i % nsets]()
            e1.record(stream)
            stream.synchronize()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
        return e0.elapsed_time(e1) / iters, wall / iters * 1e3            # ms per iteration (events, wall clock)

    step_runner = build_runner(enqueue_step)
    ms_step, ms_step_wall = timed(step_runner, args.steps, args.warmup)
    ms_step = max(ms_step, ms_step_wall) if args.no_graph else ms_step

    # kernel-level legs: one graph holds one call per buffer set, back to back, so that the event
    # time per call is the duration of the call's kernels and not the gap between graph launches
    def per_call(enq, iters, warmup):
        def enqueue_all(_st, stream_):
            for st in sets:
                enq(st, stream_)
        ms, _ = timed(build_runner(enqueue_all), iters, warmup)
        return ms / nsets

    # The folded launch is the one heavy kernel here, and the GPU needs about 100 ms of sustained
    # heavy work before its clocks settle (idle sclk 157 MHz; the same kernel measures 70 - 75 us
    # per launch over the first few milliseconds and 62 us from ~150 ms on): warm up for >= 150 ms,
    # then time >= 100 ms of back-to-back launches.
    ms_folded = per_call(enqueue_folded, max(args.steps // 4, 320), 480)

    def enqueue_one_layer(st, stream_):
        check(vs.vs_tree_verify_attention(desc1, st["q"], st["k"], st["v"], prefix1, parent1, mask, st["out"],
                                          status, ws, ws_bytes, stream_))
    ms_single = per_call(enqueue_one_layer, max(args.steps, 50), max(args.warmup, 5))
    ms_accept = per_call(enqueue_accept, max(args.steps // 2, 25), max(args.warmup, 5))
    ms_sample = per_call(enqueue_sample, max(args.steps // 2, 25), max(args.warmup, 5))
    ms_draft = per_call(enqueue_draft, max(args.steps // 2, 25), max(args.warmup, 5))
    ms_commit = per_call(enqueue_commit, max(args.steps // 2, 25), max(args.warmup, 5))
    ms_compress = per_call(enqueue_compress, max(args.steps // 2, 25), max(args.warmup, 5))

    # ---------------------------------------------------------------- what the machine delivers (measured peaks)
    # Trivial kernels of the library (include/vispec_peaks.h), timed like the legs above. The copy of
    # known size is also the reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters when
    # the HBM traffic of the kernels above is derived from a --pmc run.
    peak_bytes = 1 << 30
    cal_src = torch.randint(0, 255, (peak_bytes,), device=dev, dtype=torch.uint8)
    cal_dst = torch.empty_like(cal_src)
    sink = torch.zeros(65536 * 512, device=dev, dtype=torch.float32)
    ops_const = torch.full((8 * 128 * 8,), 1.0, device=dev, dtype=torch.bfloat16)
    ops_rand = torch.randn((8 * 128 * 8,), generator=gtorch, device=dev, dtype=torch.float32).to(torch.bfloat16)
    mfma_iters, mfma_wgs = 2000, 256

    def time_calls(fn, reps, warm):
        with torch.cuda.stream(stream):
            for _ in range(warm):
                fn()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            stream.synchronize()
        return e0.elapsed_time(e1) / reps                                              # ms per call

    ms_read = time_calls(lambda: check(vs.vs_peak_hbm_read(cal_src, peak_bytes, sink, 8192, sp)), 20, 5)
    ms_copy = time_calls(lambda: check(vs.vs_peak_hbm_copy(cal_dst, cal_src, peak_bytes // 2, 8192, sp)), 20, 5)
    # the matrix-core loops run ~100 ms each so that the clocks settle (see the folded leg)
    ms_mc = time_calls(lambda: check(vs.vs_peak_mfma_bf16(ops_const, mfma_iters, sink, mfma_wgs, sp)), 60, 60)
    ms_mr = time_calls(lambda: check(vs.vs_peak_mfma_bf16(ops_rand, mfma_iters, sink, mfma_wgs, sp)), 60, 60)
    mfma_flops = vs.vs_peak_mfma_flops(mfma_iters, mfma_wgs)
    measured_peaks = {
        "hbm_read_gbs": round(peak_bytes / (ms_read * 1e-3) / 1e9, 1),
        "hbm_copy_gbs": round(2 * (peak_bytes // 2) / (ms_copy * 1e-3) / 1e9, 1),
        "mfma_bf16_const_tflops": round(mfma_flops / (ms_mc * 1e-3) / 1e12, 1),
        "mfma_bf16_random_tflops": round(mfma_flops / (ms_mr * 1e-3) / 1e12, 1),
        "note": "vs_peak_* kernels: 1 GiB streaming read, 512 MiB copy (read + write counted), 2048 waves of "
                "v_mfma_f32_32x32x16_bf16 on all-ones / on N(0,1) operands; nominal peaks 8000 GB/s and 2500 TFLOP/s",
    }
    del cal_dst

    # ---------------------------------------------------------------- the other configurations' attention
    # Shapes of the benchmark's other configurations on device-generated N(0,1) data (their parity is
    # the GPU tests' business): C2 and C4 with their layers folded into one launch like `roofline`,
    # C5 as it is (16 ragged sequences over a paged cache need no folding: one layer is one launch).
    others = {}
    if not args.no_other_configs:
        for name in ("C2", "C4", "C5"):
            if name == args.config:
                continue
            others[name] = other_config_leg(vs, gen, torch, dev, stream, gtorch, name, args.seed, check)

    # ---------------------------------------------------------------- algorithmic work
    _, _, depth_h = oracle.tree_mask(parent_h[0])
    vis_pairs = int(sum(S + int(dd) + 1 for dd in depth_h))                      # visible (query, key) pairs per head
    flops_layer = 4.0 * d * Hq * vis_pairs
    bytes_layer = 2.0 * Hkv * (S + T) * d * eb + 2.0 * T * Hq * d * eb
    t_mfma = flops_layer / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    t_hbm = bytes_layer / (HBM_PEAK_GBS * 1e9)
    bound = "mfma" if t_mfma >= t_hbm else "hbm"

    def roof(ms_call, layers_per_call):
        sec = ms_call * 1e-3
        if bound == "mfma":
            ach = flops_layer * layers_per_call / sec / 1e12
            return {"bound": "mfma", "achieved": round(ach, 3), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None}
        ach = bytes_layer * layers_per_call / sec / 1e9
        return {"bound": "hbm", "achieved": round(ach, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None}

    roofline = roof(ms_folded, L)
    # HBM bytes per folded launch measured with rocprofv3 counters (a separate --pmc run of this
    # same command; the summary and its scaling are under profiles/)
    try:
        with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")) as f:
            traffic = json.load(f)
        roofline["traffic"] = traffic.get(args.config, {}).get("folded_attention_call_bytes")
        roofline["traffic_source"] = "profiles/hbm_traffic.json: " + traffic.get("_source", "rocprofv3 --pmc runs of this command")
    except OSError:
        traffic = {}
        roofline["traffic_source"] = "not measured"
    def kernel_name(pl):
        k = {vs.VS_SCHED_PIPELINED: "attn_mfma_pipe_kernel", vs.VS_SCHED_RESIDENT: "attn_mfma_resident_kernel"}.get(
            pl.schedule, "attn_mfma_kernel")
        return k + (" + attn_combine_kernel" if pl.combine else "")

    roofline.update({"kernel": kernel_name(planL),
                     "launch": f"B={L} proxy: the step's {L} layers folded into one launch as independent batch entries "
                               "(same per-layer shape; layers of a real model are sequentially dependent, so the timed "
                               "step issues `per_layer_call` instead)",
                     "us_per_launch": round(ms_folded * 1e3, 2), "workgroups": planL.workgroups,
                     "num_splits": planL.num_splits,
                     "tflops": round(flops_layer * L / (ms_folded * 1e-3) / 1e12, 2),
                     "hbm_gbs": round(bytes_layer * L / (ms_folded * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak": round(bytes_layer * L / (ms_folded * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
    per_layer = roof(ms_single, 1)
    per_layer.update({"launch": "one layer, B=1: the call the timed step issues once per layer", "us_per_launch": round(ms_single * 1e3, 2),
                      "workgroups": plan1.workgroups, "num_splits": plan1.num_splits, "kernel": kernel_name(plan1),
                      "algorithmic_bytes": int(bytes_layer), "workspace_bytes": int(vs.vs_attention_workspace_bytes(desc1))})
    per_layer["traffic"] = traffic.get(args.config, {}).get("per_layer_call_bytes")
    per_layer["traffic_source"] = roofline["traffic_source"]
    for blk in (roofline, per_layer):
        blk["frac_of_measured_mfma_random"] = round(blk["achieved"] / measured_peaks["mfma_bf16_random_tflops"], 4) if bound == "mfma" else None
    argmax_gbs = logit_bytes / (ms_accept * 1e-3) / 1e9
    argmax = {"bound": "hbm", "achieved": round(argmax_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
              "frac": round(argmax_gbs / HBM_PEAK_GBS, 4), "us_per_launch": round(ms_accept * 1e3, 2),
              "bytes": logit_bytes, "note": "whole vs_tree_accept call: logits scan + tree walk (two dependent kernels)"}

    sample_gbs = logit_bytes / (ms_sample * 1e-3) / 1e9
    sample = {"bound": "hbm", "achieved": round(sample_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
              "frac": round(sample_gbs / HBM_PEAK_GBS, 4), "us_per_launch": round(ms_sample * 1e3, 2),
              "bytes": logit_bytes, "note": "vs_tree_accept_sample at temperature 1 (scan + walk); not part of the step"}
    draft_bytes = draft_rows * V * 4
    draft = {"bound": "latency", "us_per_tree": round(ms_draft * 1e3, 2), "bytes": draft_bytes,
             "gbs": round(draft_bytes / (ms_draft * 1e-3) / 1e9, 1),
             "note": f"{DD} x vs_draft_expand (K={DK}) + vs_draft_tree_build (N={DN}) = 7 dependent kernels over "
                     f"{draft_rows} logits rows; the draft model between the expansions is not included"}

    compress = {"bound": "latency", "us_per_launch": round(ms_compress * 1e3, 2), "queries": T, "image_embeddings": n_img,
                "note": "vs_compress_attention (vision adaptor): one image, one layer; not part of the step"}

    commit_bytes = 2 * 2 * L * Hkv * int(o_alen[0]) * d * eb                               # rows read + rows written, K and V
    commit = {"bound": "latency", "us_per_launch": round(ms_commit * 1e3, 2), "accepted_len": int(o_alen[0]),
              "bytes": commit_bytes, "note": "after the step (not part of it): moves accepted rows of all layers"}

    # ---------------------------------------------------------------- CPU baseline: the oracle, one full step
    cpu = None
    if not args.no_cpu_baseline:
        threads = min(os.cpu_count() or 1, 16, Hq)
        t0 = time.perf_counter()
        for l in range(L):
            oracle.tree_attention(host_layers[l], threads=threads)
        oracle.tree_accept(acc_h.logits, acc_h.tokens, acc_h.parent)
        tc = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.tree_attention(host_layers[0], threads=1)
        t1 = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.tree_accept(acc_h.logits, acc_h.tokens, acc_h.parent)
        ta = time.perf_counter() - t0
        cpu = {"value": round(1.0 / tc, 4), "unit": "steps/s", "cores": threads, "kind": "oracle",
               "sample": f"one full step of {cfg.name}: {L} layers of fp64 attention + one accept, {tc:.2f} s",
               "one_thread_s": round(L * t1 + ta, 2),
               "one_thread_sample": f"one layer of attention on one thread ({t1:.2f} s) x {L} + one accept ({ta:.3f} s), extrapolated"}

    line = {
        "metric": "verify steps/sec (tree-verify attention TFLOP/s and HBM GB/s as % of roofline in `roofline`)",
        "value": round(1e3 / ms_step, 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B=1 Hq={Hq} Hkv={Hkv} d={d} prefix={S} tree={T} nodes depth<={cfg.max_depth} "
                               f"layers={L} vocab={V}; step = mask_build + {L} x attention + accept",
                   "hip_graph": not args.no_graph, "buffer_sets": nsets},
        "roofline": roofline, "per_layer_call": per_layer, "argmax": argmax, "accept_sample": sample, "draft_tree": draft, "compress_attention": compress, "kv_commit": commit, "cpu_baseline": cpu,
        "measured_peaks": measured_peaks, "other_configs": others,
        "parity": {"attention_max_abs_err_layer0": err0, "accept_bit_exact": accept_ok, "commit_bit_exact": commit_ok,
                   "sample_outcome_valid": sample_ok, "draft_tree_bit_exact": draft_ok,
                   "compress_attention_max_abs_err": err_c},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
