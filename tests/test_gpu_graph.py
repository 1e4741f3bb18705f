"""A verify step captured in a HIP graph must replay to the same bits as eager launches."""
import numpy as np
import pytest

import gen
import paper_2509_15235_amd as vs

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    import torch
    import gpu_util as gu
    import dataclasses
    cfg = dataclasses.replace(gen.CONFIGS["C3"], prefix=[700], V=30000)
    inp = gen.attention_inputs(cfg, 77)
    ai = gen.accept_inputs(cfg, 77, parent=inp.parent)
    da = gu.DeviceAttn(inp, num_splits=4)
    eager = da.run().copy()
    e_acc = gu.run_accept(ai.logits, ai.tokens, ai.parent)

    T, V = cfg.T, cfg.V
    logits = gu.dev(ai.logits.reshape(T, V))
    tok, par = gu.dev(ai.tokens), gu.dev(ai.parent)
    alen = torch.zeros(1, device="cuda", dtype=torch.int32)
    path = torch.zeros((1, T), device="cuda", dtype=torch.int32)
    bonus = torch.zeros(1, device="cuda", dtype=torch.int32)
    amax = torch.zeros((1, T), device="cuda", dtype=torch.int32)
    mask = torch.zeros((1, T), device="cuda", dtype=torch.int64)
    depth = torch.zeros((1, T), device="cuda", dtype=torch.int32)
    nb = vs.vs_accept_workspace_bytes(1, T, V)
    aws = torch.empty(nb, device="cuda", dtype=torch.uint8)

    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        sp = torch.cuda.current_stream().cuda_stream
        assert vs.vs_tree_mask_build(par, 1, T, mask, depth, da.status, sp) == 0
        assert vs.vs_tree_verify_attention(da.desc, da.q, da.k, da.v, da.prefix, da.parent, mask, da.out, da.status,
                                           da.ws, da.ws_bytes, sp) == 0
        assert vs.vs_tree_accept(logits, V, V, tok, par, 1, T, alen, path, bonus, amax, da.status, aws, nb, sp) == 0
    for rep in range(4):
        da.out.fill_(float("nan"))
        da.ws.fill_(0xFF)
        alen.fill_(-5); path.fill_(-5); bonus.fill_(-5); amax.fill_(-5)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = da.out.float().cpu().numpy().astype(np.float64)
        assert np.array_equal(got, eager), f"replay {rep}"
        assert (amax.cpu().numpy() == e_acc[0]).all() and alen.item() == e_acc[1][0]
        assert (path.cpu().numpy() == e_acc[2]).all() and bonus.item() == e_acc[3][0]
        # eager work of the program between replays
        again = da.run()
        assert np.array_equal(again, eager)


def test_graph_replays_of_the_speculative_cycle_match_eager():
    """Draft-tree construction followed by stochastic acceptance of that tree, captured in one
    graph: every replay gives the bits of the eager calls (the workspaces are scribbled on in
    between, so nothing may depend on what a previous call left there)."""
    import torch
    import gpu_util as gu
    V, K, D, N, B = 20000, 4, 3, 20, 2
    T = N + 1
    cap = K + (D - 1) * K * K
    levels = [np.stack([gen.draft_logits(5, b, lv, 1 if lv == 0 else K, V) for b in range(B)]) for lv in range(D)]
    # eager reference
    dd = gu.DeviceDraft(B, K, cap)
    nf = nc = None
    for lv in range(D):
        nf, nc = dd.expand(levels[lv], nc, nf)
    e_parent, e_tokens, e_cand, e_num, e_st = dd.build(N)
    assert (e_st == 0).all() and (e_num == T).all()
    tl = np.stack([gen.logits_with_candidates(gen.rng(5, gen.STREAM_LOGITS, b), gen.rng(5, gen.STREAM_CANDIDATE, b),
                                              e_parent[b], e_tokens[b], V) for b in range(B)])
    ua, ub = gen.uniforms(5, B, T)
    e_alen, e_path, e_bonus, _ = gu.run_accept_sample(tl, e_tokens, e_parent, 1.0, ua, ub)

    # the same calls on fresh buffers inside a graph
    lg = [gu.dev(x.reshape(-1, V)) for x in levels]
    c_tok = torch.zeros((B, cap), device="cuda", dtype=torch.int32)
    c_par = torch.zeros_like(c_tok)
    c_score = torch.zeros((B, cap), device="cuda", dtype=torch.float32)
    fr = [torch.zeros((B, K), device="cuda", dtype=torch.int32) for _ in range(D)]
    cu = [torch.zeros((B, K), device="cuda", dtype=torch.float32) for _ in range(D)]
    parent = torch.zeros((B, T), device="cuda", dtype=torch.int32)
    tokens, ncand = torch.zeros_like(parent), torch.zeros_like(parent)
    num = torch.zeros(B, device="cuda", dtype=torch.int32)
    status = torch.zeros(B, device="cuda", dtype=torch.int32)
    dws_n = vs.vs_draft_expand_workspace_bytes(B, K, V, K)
    dws = torch.empty(dws_n, device="cuda", dtype=torch.uint8)
    tlog = gu.dev(tl.reshape(B * T, V))
    d_ua, d_ub = gu.dev(ua), gu.dev(ub)
    alen = torch.zeros(B, device="cuda", dtype=torch.int32)
    path = torch.zeros((B, T), device="cuda", dtype=torch.int32)
    bonus = torch.zeros(B, device="cuda", dtype=torch.int32)
    sws_n = vs.vs_accept_sample_workspace_bytes(B, T, V)
    sws = torch.empty(sws_n, device="cuda", dtype=torch.uint8)
    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        sp = torch.cuda.current_stream().cuda_stream
        base = 0
        for lv in range(D):
            F = 1 if lv == 0 else K
            assert vs.vs_draft_expand(lg[lv], V, V, None if lv == 0 else cu[lv - 1], None if lv == 0 else fr[lv - 1], B, F,
                                      K, base, cap, c_tok, c_score, c_par, fr[lv], cu[lv], dws, dws_n, sp) == 0
            base += F * K
        assert vs.vs_draft_tree_build(c_tok, c_score, c_par, B, cap, cap, N, None, parent, tokens, ncand, num, status,
                                      sp) == 0
        assert vs.vs_tree_accept_sample(tlog, V, V, 1.0, tokens, parent, d_ua, d_ub, B, T, alen, path, bonus, status,
                                        sws, sws_n, sp) == 0
    for rep in range(3):
        for t in (c_tok, c_par, parent, tokens, ncand, num, alen, path, bonus):
            t.fill_(-9)
        c_score.fill_(float("nan"))
        dws.fill_(0xFF)
        sws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert (parent.cpu().numpy() == e_parent).all() and (tokens.cpu().numpy() == e_tokens).all(), f"replay {rep}"
        assert (alen.cpu().numpy() == e_alen).all() and (path.cpu().numpy() == e_path).all()
        assert (bonus.cpu().numpy() == e_bonus).all()
        again = gu.run_accept_sample(tl, e_tokens, e_parent, 1.0, ua, ub)     # eager work between replays
        assert (again[0] == e_alen).all() and (again[2] == e_bonus).all()
