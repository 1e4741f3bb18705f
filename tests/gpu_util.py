"""Helpers for the GPU tests: move generated inputs to the device and call the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_2509_15235_amd as vs


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


class DeviceAttn:
    """Device copies of a gen.AttnInputs plus the matching descriptor."""

    def __init__(self, inp, impl=vs.VS_IMPL_AUTO, num_splits=0, max_prefix_len=None, rows_per_wave=0,
                 waves_per_group=0, schedule=0):
        cfg = inp.cfg
        self.inp = inp
        bf = cfg.dtype == "bf16"
        self.q = dev_bf16(inp.q_bits) if bf else dev(inp.q)
        self.k = dev_bf16(inp.k_bits) if bf else dev(inp.k_cache)
        self.v = dev_bf16(inp.v_bits) if bf else dev(inp.v_cache)
        self.prefix = dev(inp.prefix_len.astype(np.int32))
        self.parent = dev(inp.parent.astype(np.int32))
        B, T = inp.parent.shape
        self.out = torch.full((B, T, cfg.Hq, cfg.d), float("nan"), device="cuda",
                              dtype=torch.bfloat16 if bf else torch.float32)
        self.status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
        d = vs.AttnDesc()
        d.B, d.T, d.Hq, d.Hkv, d.d = B, T, cfg.Hq, cfg.Hkv, cfg.d
        d.dtype = vs.VS_BF16 if bf else vs.VS_F32
        d.softmax_scale = float(inp.scale)
        d.max_prefix_len = int(inp.prefix_len.max()) if max_prefix_len is None else max_prefix_len
        d.impl = impl
        d.num_splits = num_splits
        d.rows_per_wave = rows_per_wave
        d.waves_per_group = waves_per_group
        d.schedule = schedule
        if inp.block_table is None:
            cap = inp.k_cache.shape[2]
            d.paged = 0
            d.capacity = cap
            d.stride_seq = cfg.Hkv * cap * cfg.d
            d.stride_head = cap * cfg.d
            d.stride_tok = cfg.d
            self.table = None
        else:
            self.table = dev(inp.block_table.astype(np.int32))
            d.paged = 1
            d.block_size = cfg.block_size
            d.max_blocks = inp.block_table.shape[1]
            d.num_blocks = inp.k_cache.shape[0]
            d.stride_block = cfg.Hkv * cfg.block_size * cfg.d
            d.stride_head = cfg.block_size * cfg.d
            d.stride_tok = cfg.d
            d.block_table = self.table.data_ptr()
        self.desc = d
        self.ws_bytes = vs.vs_attention_workspace_bytes(d)
        self.ws = torch.empty(max(self.ws_bytes, 256), device="cuda", dtype=torch.uint8)

    def plan(self):
        rc, pl = vs.vs_attention_plan(self.desc)
        assert rc == 0, vs.vs_strerror(rc)
        return pl

    def run(self, tree_mask=None, sync=True):
        rc = vs.vs_tree_verify_attention(self.desc, self.q, self.k, self.v, self.prefix, self.parent, tree_mask,
                                         self.out, self.status, self.ws, self.ws_bytes, stream_ptr())
        assert rc == 0, vs.vs_strerror(rc)
        if sync:
            torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64)


def check_close(got, ref, abs_tol, rel_tol, what=""):
    err = np.abs(got - ref)
    bound = abs_tol + rel_tol * np.abs(ref)
    bad = ~(err <= bound)          # NaN-safe
    if bad.any():
        idx = np.unravel_index(np.argmax(np.where(np.isnan(err), np.inf, err - bound)), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements outside |err| <= {abs_tol} + {rel_tol}|ref|; "
                             f"worst at {idx}: got {got[idx]} ref {ref[idx]}; max|err| {np.nanmax(err)}")
    return float(err.max())


def run_mask(parent: np.ndarray):
    B, T = parent.shape
    p = dev(parent.astype(np.int32))
    mask = torch.zeros((B, T), device="cuda", dtype=torch.int64)
    depth = torch.zeros((B, T), device="cuda", dtype=torch.int32)
    status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
    rc = vs.vs_tree_mask_build(p, B, T, mask, depth, status, stream_ptr())
    assert rc == 0, vs.vs_strerror(rc)
    torch.cuda.synchronize()
    return mask.cpu().numpy().view(np.uint64), depth.cpu().numpy(), status.cpu().numpy(), mask


def run_accept(logits: np.ndarray, tokens: np.ndarray, parent: np.ndarray, ld=None, offset_elems=0):
    """logits [B,T,V]; optional row stride ld >= V and a start offset (in elements) to
    exercise the unaligned path."""
    B, T, V = logits.shape
    ld = V if ld is None else ld
    buf = torch.full((B * T * ld + offset_elems + 8,), float("nan"), device="cuda", dtype=torch.float32)
    view = buf[offset_elems:offset_elems + B * T * ld].view(B * T, ld)
    view[:, :V] = dev(logits.reshape(B * T, V))
    tok = dev(tokens.astype(np.int32))
    par = dev(parent.astype(np.int32))
    alen = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    path = torch.full((B, T), -7, device="cuda", dtype=torch.int32)
    bonus = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    amax = torch.full((B, T), -7, device="cuda", dtype=torch.int32)
    status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
    nbytes = vs.vs_accept_workspace_bytes(B, T, V)
    ws = torch.empty(nbytes, device="cuda", dtype=torch.uint8)
    rc = vs.vs_tree_accept(view.data_ptr(), ld, V, tok, par, B, T, alen, path, bonus, amax, status, ws, nbytes,
                           stream_ptr())
    assert rc == 0, vs.vs_strerror(rc)
    torch.cuda.synchronize()
    return (amax.cpu().numpy(), alen.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy(), status.cpu().numpy())


def run_accept_sample(logits: np.ndarray, tokens: np.ndarray, parent: np.ndarray, temperature: float,
                      u_accept: np.ndarray, u_bonus: np.ndarray, ld=None, offset_elems=0):
    """logits [B,T,V]; uniforms f32 [B,T] and [B]; optional row stride and start offset as in run_accept."""
    B, T, V = logits.shape
    ld = V if ld is None else ld
    buf = torch.full((B * T * ld + offset_elems + 8,), float("nan"), device="cuda", dtype=torch.float32)
    view = buf[offset_elems:offset_elems + B * T * ld].view(B * T, ld)
    view[:, :V] = dev(logits.reshape(B * T, V))
    tok = dev(tokens.astype(np.int32))
    par = dev(parent.astype(np.int32))
    ua = dev(np.asarray(u_accept, dtype=np.float32))
    ub = dev(np.asarray(u_bonus, dtype=np.float32))
    alen = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    path = torch.full((B, T), -7, device="cuda", dtype=torch.int32)
    bonus = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
    nbytes = vs.vs_accept_sample_workspace_bytes(B, T, V)
    ws = torch.empty(nbytes, device="cuda", dtype=torch.uint8)
    rc = vs.vs_tree_accept_sample(view.data_ptr(), ld, V, float(temperature), tok, par, ua, ub, B, T, alen, path,
                                  bonus, status, ws, nbytes, stream_ptr())
    assert rc == 0, vs.vs_strerror(rc)
    torch.cuda.synchronize()
    return alen.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy(), status.cpu().numpy()


class DeviceDraft:
    """Candidate arrays of B sequences on the device plus the calls that fill them."""

    def __init__(self, B, K, capacity):
        self.B, self.K, self.cap = B, K, capacity
        self.tok = torch.full((B, capacity), -7, device="cuda", dtype=torch.int32)
        self.score = torch.full((B, capacity), float("nan"), device="cuda", dtype=torch.float32)
        self.par = torch.full((B, capacity), -7, device="cuda", dtype=torch.int32)
        self.M = 0

    def expand(self, logits: np.ndarray, cum_in, frontier_cand, ld=None, offset_elems=0):
        """logits [B,F,V] numpy; cum_in / frontier_cand device tensors [B,F] or None.
        Returns device tensors (next_frontier_cand [B,keep], next_cum [B,keep])."""
        B, F, V = logits.shape
        K = self.K
        ld = V if ld is None else ld
        buf = torch.full((B * F * ld + offset_elems + 8,), float("nan"), device="cuda", dtype=torch.float32)
        view = buf[offset_elems:offset_elems + B * F * ld].view(B * F, ld)
        view[:, :V] = dev(logits.reshape(B * F, V))
        keep = min(K, F * K)
        nf = torch.full((B, keep), -7, device="cuda", dtype=torch.int32)
        nc = torch.full((B, keep), float("nan"), device="cuda", dtype=torch.float32)
        nbytes = vs.vs_draft_expand_workspace_bytes(B, F, V, K)
        assert nbytes > 0
        ws = torch.empty(nbytes, device="cuda", dtype=torch.uint8)
        rc = vs.vs_draft_expand(view.data_ptr(), ld, V, cum_in, frontier_cand, B, F, K, self.M, self.cap, self.tok,
                                self.score, self.par, nf, nc, ws, nbytes, stream_ptr())
        assert rc == 0, vs.vs_strerror(rc)
        torch.cuda.synchronize()
        self.M += F * K
        return nf, nc

    def build(self, N, root_token=None, M=None):
        B = self.B
        M = self.M if M is None else M
        parent = torch.full((B, N + 1), -7, device="cuda", dtype=torch.int32)
        tokens = torch.full((B, N + 1), -7, device="cuda", dtype=torch.int32)
        node_cand = torch.full((B, N + 1), -7, device="cuda", dtype=torch.int32)
        num = torch.full((B,), -7, device="cuda", dtype=torch.int32)
        status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
        rt = None if root_token is None else dev(np.asarray(root_token, dtype=np.int32))
        rc = vs.vs_draft_tree_build(self.tok, self.score, self.par, B, M, self.cap, N, rt, parent, tokens, node_cand,
                                    num, status, stream_ptr())
        assert rc == 0, vs.vs_strerror(rc)
        torch.cuda.synchronize()
        return (parent.cpu().numpy(), tokens.cpu().numpy(), node_cand.cpu().numpy(), num.cpu().numpy(),
                status.cpu().numpy())


class DeviceCommit:
    """Device copies of L layers of K/V caches (stacked along a leading layer axis) plus the
    descriptor of vs_tree_kv_commit. `k_layers` / `v_layers`: numpy [L, ...one layer's cache...]
    of uint16 (bf16 storage) or float32."""

    def __init__(self, cfg, k_layers, v_layers, prefix_len, path, accepted_len, block_table=None):
        bf = k_layers.dtype == np.uint16
        self.k = dev_bf16(k_layers) if bf else dev(k_layers)
        self.v = dev_bf16(v_layers) if bf else dev(v_layers)
        self.bf = bf
        B, T = path.shape
        self.prefix = dev(prefix_len.astype(np.int32))
        self.path = dev(path.astype(np.int32))
        self.alen = dev(accepted_len.astype(np.int32))
        self.newp = torch.full((B,), -7, device="cuda", dtype=torch.int32)
        self.status = torch.full((B,), -99, device="cuda", dtype=torch.int32)
        d = vs.KVDesc()
        d.B, d.T, d.Hkv, d.d = B, T, cfg.Hkv, cfg.d
        d.dtype = vs.VS_BF16 if bf else vs.VS_F32
        d.num_layers = k_layers.shape[0]
        d.stride_layer = int(np.prod(k_layers.shape[1:]))
        if block_table is None:
            cap = k_layers.shape[3]
            d.paged, d.capacity = 0, cap
            d.stride_seq, d.stride_head, d.stride_tok = cfg.Hkv * cap * cfg.d, cap * cfg.d, cfg.d
            self.table = None
        else:
            self.table = dev(block_table.astype(np.int32))
            d.paged, d.block_size = 1, cfg.block_size
            d.max_blocks, d.num_blocks = block_table.shape[1], k_layers.shape[1]
            d.stride_block, d.stride_head, d.stride_tok = cfg.Hkv * cfg.block_size * cfg.d, cfg.block_size * cfg.d, cfg.d
            d.block_table = self.table.data_ptr()
        self.desc = d

    def run(self):
        rc = vs.vs_tree_kv_commit(self.desc, self.k, self.v, self.prefix, self.path, self.alen, self.newp, self.status,
                                  stream_ptr())
        assert rc == 0, vs.vs_strerror(rc)
        torch.cuda.synchronize()
        host = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if self.bf else (lambda t: t.cpu().numpy())
        return host(self.k), host(self.v), self.newp.cpu().numpy(), self.status.cpu().numpy()
