"""GPU parity: the vision adaptor's compression attention (vs_compress_attention) against the oracle.
Same arithmetic and the same bounds as the tree-verification attention: bf16 storage, fp32
accumulation, |err| <= 2e-2 + 1e-2 |ref| (contract) and the tighter derived bound
1.5e-3 + 6e-3 |ref| for >= 256 keys (1.2e-2 + 6e-3 |ref| for fewer); fp32 storage 2e-5 + 2e-5 |ref|."""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available()
    import gpu_util
    return gpu_util


def _run(gu, inp, Hq, Hkv, d, nq, dtype="bf16", impl=0, schedule=0, num_splits=0, waves=0, max_len=None):
    import torch
    import paper_2509_15235_amd as vs
    bf = dtype == "bf16"
    q = gu.dev_bf16(inp["q_bits"]) if bf else gu.dev(inp["q"])
    k = gu.dev_bf16(inp["k_bits"]) if bf else gu.dev(inp["k"])
    v = gu.dev_bf16(inp["v_bits"]) if bf else gu.dev(inp["v"])
    lens = gu.dev(inp["lens"])
    B, cap = len(inp["lens"]), inp["cap"]
    out = torch.full((B, nq, Hq, d), float("nan"), device="cuda", dtype=torch.bfloat16 if bf else torch.float32)
    status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
    desc = vs.AttnDesc(B=B, T=nq, Hq=Hq, Hkv=Hkv, d=d, dtype=vs.VS_BF16 if bf else vs.VS_F32,
                       softmax_scale=float(inp["scale"]),
                       max_prefix_len=int(inp["lens"].max()) if max_len is None else max_len, capacity=cap,
                       stride_seq=Hkv * cap * d, stride_head=cap * d, stride_tok=d, impl=impl, schedule=schedule,
                       num_splits=num_splits, waves_per_group=waves)
    nbytes = vs.vs_compress_attention_workspace_bytes(desc)
    ws = torch.empty(max(nbytes, 256), device="cuda", dtype=torch.uint8)
    rc = vs.vs_compress_attention(desc, q, k, v, lens, out, status, ws, nbytes, gu.stream_ptr())
    assert rc == 0, vs.vs_strerror(rc)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), status.cpu().numpy()


def _ref(oracle_mod, inp, Hkv):
    return np.stack([oracle_mod.compress_attention_seq(inp["q"][b], inp["k"][b], inp["v"][b], int(inp["lens"][b]),
                                                       inp["scale"], Hkv) for b in range(len(inp["lens"]))])


def _bounds(gu, got, ref, lens, what):
    gu.check_close(got, ref, 2e-2, 1e-2, what=what + " (contract)")
    for b, r in enumerate(lens):
        a = 1.5e-3 if r >= 256 else 1.2e-2
        gu.check_close(got[b], ref[b], a, 6e-3, what=f"{what} image {b} r={r} (derived bound)")


@pytest.mark.parametrize("nq,Hq,Hkv,lens", [
    (1, 32, 32, [2880]),                 # one query (the paper's smallest setting), LLaVA-1.6-sized image
    (16, 32, 32, [576, 300]),            # MHA
    (64, 28, 4, [1296, 1, 77]),          # the paper's largest query count, Qwen-sized image, GQA group of 7
    (32, 8, 2, [64, 65, 63, 31, 32, 33]),  # tile boundaries
])
def test_matches_oracle_every_kernel(gu, oracle_mod, nq, Hq, Hkv, lens):
    import paper_2509_15235_amd as vs
    d = 128
    inp = gen.compress_inputs(nq + len(lens), len(lens), nq, Hq, Hkv, d, lens)
    ref = _ref(oracle_mod, inp, Hkv)
    for impl, sched, splits, waves in ((vs.VS_IMPL_MFMA, vs.VS_SCHED_LOOP, 0, 0), (vs.VS_IMPL_MFMA, vs.VS_SCHED_LOOP, 1, 0),
                                       (vs.VS_IMPL_MFMA, vs.VS_SCHED_LOOP, 3, 8), (vs.VS_IMPL_MFMA, vs.VS_SCHED_PIPELINED, 0, 0),
                                       (vs.VS_IMPL_MFMA, vs.VS_SCHED_PIPELINED, 2, 4), (vs.VS_IMPL_MFMA, vs.VS_SCHED_RESIDENT, 0, 0),
                                       (vs.VS_IMPL_MFMA, vs.VS_SCHED_RESIDENT, 40, 8), (vs.VS_IMPL_MFMA, vs.VS_SCHED_BALANCED, 5, 0),
                                       (vs.VS_IMPL_MFMA, vs.VS_SCHED_BALANCED, 0, 8), (vs.VS_IMPL_GENERIC, 0, 0, 0)):
        got, status = _run(gu, inp, Hq, Hkv, d, nq, impl=impl, schedule=sched, num_splits=splits, waves=waves)
        assert (status == 0).all()
        _bounds(gu, got, ref, lens, f"impl {impl} schedule {sched} splits {splits} waves {waves}")


def test_fp32_storage_and_head_dim_64(gu, oracle_mod):
    inp = gen.compress_inputs(3, 2, 8, 4, 1, 64, [64, 40], dtype="f32")
    got, status = _run(gu, inp, 4, 1, 64, 8, dtype="f32")
    assert (status == 0).all()
    gu.check_close(got, _ref(oracle_mod, inp, 1), 2e-5, 2e-5, what="fp32 compression attention")
    inp = gen.compress_inputs(4, 2, 8, 4, 2, 64, [300, 129])
    got, status = _run(gu, inp, 4, 2, 64, 8)
    _bounds(gu, got, _ref(oracle_mod, inp, 2), [300, 129], "d = 64")


def test_redundant_image_embeddings(gu, oracle_mod):
    """The situation Section 4.1 argues from: most image embeddings are copies of a few patterns.
    With R copies of one embedding and one unique embedding the queries' outputs follow Eq. 3."""
    nq, H, d, R = 4, 2, 128, 900
    inp = gen.compress_inputs(7, 1, nq, H, H, d, [R + 1])
    for name in ("k", "v"):
        row = inp[name][0, :, 0].copy()
        inp[name][0, :, :R] = row[:, None, :]
        inp[name + "_bits"][0, :, :R] = gen.f32_to_bf16_bits(row)[:, None, :]
    ref = _ref(oracle_mod, inp, H)
    got, status = _run(gu, inp, H, H, d, nq)
    _bounds(gu, got, ref, [R + 1], "redundant embeddings")
    # closed form (Eq. 3): weight of the unique embedding = e^B / (R e^A + e^B)
    for i in range(nq):
        for h in range(H):
            A = inp["scale"] * float(inp["q"][0, i, h].astype(np.float64) @ inp["k"][0, h, 0].astype(np.float64))
            Bs = inp["scale"] * float(inp["q"][0, i, h].astype(np.float64) @ inp["k"][0, h, R].astype(np.float64))
            a = 1.0 / (1.0 + R * np.exp(A - Bs))
            want = a * inp["v"][0, h, R] + (1 - a) * inp["v"][0, h, 0]
            np.testing.assert_allclose(ref[0, i, h], want, rtol=1e-9, atol=1e-12)


def test_bad_lengths_report_status(gu, oracle_mod):
    inp = gen.compress_inputs(9, 3, 4, 4, 4, 128, [100, 50, 70], cap=130)
    inp["lens"] = np.array([100, 0, 121], dtype=np.int32)        # empty image; longer than the descriptor's bound
    got, status = _run(gu, inp, 4, 4, 128, 4, max_len=120)
    assert status.tolist() == [0, 3, 3]
    inp["lens"] = np.array([100], dtype=np.int32)
    ref = oracle_mod.compress_attention_seq(inp["q"][0], inp["k"][0], inp["v"][0], 100, inp["scale"], 4)
    gu.check_close(got[0], ref, 1.2e-2, 6e-3, what="valid image next to invalid ones")
