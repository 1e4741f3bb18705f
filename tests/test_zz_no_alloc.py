"""GPU test of vs_tree_accept_noalloc, the acceptance call that keeps its scratch in a static
device array: its outputs must equal vs_tree_accept's bit for bit (which the other tests hold
to the oracle), on two calls in a row, the second with a smaller input that leaves most of the
array holding the first call's results. Runs last so that a failure here hides no other test."""
import numpy as np
import pytest

import gen
import paper_2509_15235_amd as vs

pytestmark = pytest.mark.gpu


def _run(gu, torch, logits, tokens, parent, noalloc):
    B, T, V = logits.shape
    lg = gu.dev(logits.reshape(B * T, V))
    tok, par = gu.dev(tokens.astype(np.int32)), gu.dev(parent.astype(np.int32))
    alen = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    path = torch.full((B, T), -7, device="cuda", dtype=torch.int32)
    bonus = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    amax = torch.full((B, T), -7, device="cuda", dtype=torch.int32)
    status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
    if noalloc:
        rc = vs.vs_tree_accept_noalloc(lg, V, V, tok, par, B, T, alen, path, bonus, amax, status, gu.stream_ptr())
    else:
        n = vs.vs_accept_workspace_bytes(B, T, V)
        ws = torch.empty(n, device="cuda", dtype=torch.uint8)
        rc = vs.vs_tree_accept(lg, V, V, tok, par, B, T, alen, path, bonus, amax, status, ws, n, gu.stream_ptr())
    assert rc == 0, vs.vs_strerror(rc)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (amax, alen, path, bonus, status)]


def test_noalloc_equals_workspace_call_twice_in_a_row(oracle_mod):
    import torch
    assert torch.cuda.is_available()
    import gpu_util as gu
    import dataclasses
    big = dataclasses.replace(gen.CONFIGS["C3"], B=3, V=152064)          # 3 x 60 rows x 38 chunks
    small = dataclasses.replace(gen.CONFIGS["C1"], B=2, T=9, V=5000, max_depth=4, prefix=[4, 4])
    for cfg, seed in ((big, 71), (small, 72)):                              # the second call is the smaller one
        ai = gen.accept_inputs(cfg, seed)
        want = _run(gu, torch, ai.logits, ai.tokens, ai.parent, noalloc=False)
        got = _run(gu, torch, ai.logits, ai.tokens, ai.parent, noalloc=True)
        for w, g, name in zip(want, got, ("row_argmax", "accepted_len", "path", "bonus_token", "status")):
            np.testing.assert_array_equal(g, w, err_msg=f"{cfg.name}: {name}")
        o_amax, o_alen, o_path, o_bonus = oracle_mod.tree_accept(ai.logits, ai.tokens, ai.parent)
        np.testing.assert_array_equal(got[0], o_amax)
        np.testing.assert_array_equal(got[1], o_alen)
        np.testing.assert_array_equal(got[2], o_path)
        np.testing.assert_array_equal(got[3], o_bonus)
        assert (got[4] == 0).all()


def test_noalloc_rejects_sizes_beyond_its_scratch():
    import torch
    g = 4096
    # 64 sequences x 64 rows x 38 chunks = 155648 pairs: more than the static array holds
    assert vs.vs_accept_workspace_bytes(64, 64, 152064) > (1 << 20)
    assert vs.vs_tree_accept_noalloc(g, 152064, 152064, g, g, 64, 64, g, g, g) == -4
    assert vs.vs_tree_accept_noalloc(None, 10, 10, g, g, 1, 4, g, g, g) == -1
    assert vs.vs_tree_accept_noalloc(g, 9, 10, g, g, 1, 4, g, g, g) == -2
