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
