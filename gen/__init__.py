"""Seeded synthetic inputs for the tree-verification path.

This module only *draws inputs* (trees, Q/K/V, block tables, logits). It holds none of
the method's arithmetic: no masks, no softmax, no argmax, no acceptance. Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so that the two
sides see bit-identical data.

Randomness: numpy's Philox counter-based generator keyed by (seed, stream id), so every
tensor has its own reproducible sub-stream.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

# ----------------------------------------------------------------------------- rng

STREAM_TREE = 1
STREAM_Q = 2
STREAM_K = 3
STREAM_V = 4
STREAM_LOGITS = 5
STREAM_TOKENS = 6
STREAM_PLANT = 7
STREAM_PREFIX = 8
STREAM_BLOCKS = 9
STREAM_PATH = 10
STREAM_UNIFORM = 11
STREAM_CANDIDATE = 12


def rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    """Independent generator for (seed, stream, sub)."""
    return np.random.Generator(np.random.Philox(key=[(seed << 20) ^ sub, stream]))


# ----------------------------------------------------------------------------- bf16 storage

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 storage (round-to-nearest-even), returned as uint16 bit patterns.
    Inputs are finite or NaN; NaN stays NaN (quiet bit forced)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


BF16_NAN_BITS = np.uint16(0x7FC1)


# ----------------------------------------------------------------------------- trees

def chain_tree(T: int) -> np.ndarray:
    p = np.arange(-1, T - 1, dtype=np.int32)
    return p


def star_tree(T: int) -> np.ndarray:
    p = np.zeros(T, dtype=np.int32)
    p[0] = -1
    return p


def _level_order(parent_list: List[int], depth_list: List[int]) -> np.ndarray:
    """Relabel nodes so depth is non-decreasing (stable in creation order)."""
    n = len(parent_list)
    order = sorted(range(n), key=lambda i: (depth_list[i], i))
    new_of_old = {old: new for new, old in enumerate(order)}
    parent = np.empty(n, dtype=np.int32)
    for new, old in enumerate(order):
        p = parent_list[old]
        parent[new] = -1 if p < 0 else new_of_old[p]
    return parent


def random_tree(g: np.random.Generator, T: int, max_depth: int, max_children: int) -> np.ndarray:
    """Draft tree in the style of a top-k expansion: a root, a spine that reaches
    `max_depth` (when T allows), and the remaining nodes attached to uniformly chosen
    nodes that still have room (depth < max_depth, children < max_children). Nodes are
    returned in level order, so parent[i] < i. Node 0 is the root (parent -1)."""
    assert T >= 1
    parent = [-1]
    depth = [0]
    nchild = [0]
    spine = min(max_depth, T - 1)
    for k in range(spine):
        parent.append(k)
        depth.append(k + 1)
        nchild.append(0)
        nchild[k] += 1
    while len(parent) < T:
        elig = [i for i in range(len(parent)) if depth[i] < max_depth and nchild[i] < max_children]
        if not elig:
            raise ValueError("tree cannot hold T nodes under the depth/branching limits")
        p = elig[int(g.integers(0, len(elig)))]
        parent.append(p)
        depth.append(depth[p] + 1)
        nchild.append(0)
        nchild[p] += 1
    return _level_order(parent, depth)


def topk_tree(g: np.random.Generator, n_draft: int = 30, depth: int = 3, topk: int = 8) -> np.ndarray:
    """Tree with the paper's inference hyper-parameters (Appendix A, implementation
    details: 30 draft tokens, depth 3, 8 nodes selected per expansion). Every node gets a
    pseudo-confidence (its parent's times a uniform draw, so it decreases along a path);
    at each level the `topk` most confident new nodes are expanded into `topk` children
    each; finally the `n_draft` most confident candidates are kept, which is closed under
    ancestors because confidence decreases along paths. Returns parent[] for n_draft + 1
    nodes in level order."""
    parent = [-1]
    dep = [0]
    conf = [1.0]
    frontier = [0]
    for lv in range(1, depth + 1):
        new_nodes = []
        for o in frontier:
            for _ in range(topk):
                parent.append(o)
                dep.append(lv)
                conf.append(conf[o] * float(g.random()))
                new_nodes.append(len(parent) - 1)
        frontier = sorted(new_nodes, key=lambda i: -conf[i])[:topk]
    cand = sorted(range(1, len(parent)), key=lambda i: -conf[i])[:n_draft]
    keep = sorted([0] + cand)
    remap = {old: new for new, old in enumerate(keep)}
    p2 = [(-1 if parent[i] < 0 else remap[parent[i]]) for i in keep]
    d2 = [dep[i] for i in keep]
    return _level_order(p2, d2)


def draft_tokens(g: np.random.Generator, parent: np.ndarray, V: int) -> np.ndarray:
    """One token id per node, uniform in [0, V); siblings get distinct tokens (a top-k
    expansion never proposes the same token twice under one parent)."""
    T = len(parent)
    tok = np.zeros(T, dtype=np.int32)
    used = {}
    for i in range(T):
        p = int(parent[i])
        s = used.setdefault(p, set())
        while True:
            t = int(g.integers(0, V))
            if t not in s or len(s) >= V:     # a vocabulary smaller than the fan-out must repeat
                break
        s.add(t)
        tok[i] = t
    return tok


PLANT_VALUE = np.float32(20.0)  # far above any N(0,1) draw at these vocab sizes


def logits_with_plants(g_logits: np.random.Generator, g_plant: np.random.Generator,
                       parent: np.ndarray, tokens: np.ndarray, V: int, pi: float) -> np.ndarray:
    """fp32 logits [T, V] ~ N(0,1). For every node p that has children, with probability
    `pi` one child c is drawn uniformly and logits[p, tokens[c]] is raised to PLANT_VALUE,
    which makes the target's greedy choice at p equal to that child's draft token."""
    T = len(parent)
    lg = g_logits.standard_normal((T, V), dtype=np.float32)
    children = [[] for _ in range(T)]
    for i in range(1, T):
        children[int(parent[i])].append(i)
    for p in range(T):
        if not children[p]:
            continue
        u = g_plant.random()
        c = children[p][int(g_plant.integers(0, len(children[p])))]
        if u < pi:
            lg[p, tokens[c]] = PLANT_VALUE
    return lg


# ----------------------------------------------------------------------------- configs

@dataclass
class Config:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    T: int
    max_depth: int
    max_children: int
    V: int
    pi: float
    layers: int
    dtype: str                      # "bf16" | "f32"
    prefix: Optional[List[int]] = None   # fixed prefix lengths; None → drawn (ragged)
    prefix_range: Optional[tuple] = None
    paged: bool = False
    block_size: int = 16
    segments: Optional[list] = None      # metadata: [("text"|"image", n), ...] for B == 1


CONFIGS = {
    # tiny fp32 case the oracle finishes in milliseconds
    "C1": Config("C1-tiny", 1, 4, 1, 64, 8, 3, 4, 1000, 0.7, 1, "f32", prefix=[64],
                 segments=[("text", 4), ("image", 48), ("text", 12)]),
    # LLaVA-1.6-7B-shaped MHA
    "C2": Config("C2-llava7b-mha", 1, 32, 32, 128, 60, 6, 4, 32000, 0.7, 32, "bf16", prefix=[3136],
                 segments=[("text", 32), ("image", 2880), ("text", 224)]),
    # Qwen2.5-VL-7B-shaped GQA
    "C3": Config("C3-qwen7b-gqa", 1, 28, 4, 128, 60, 6, 4, 152064, 0.7, 28, "bf16", prefix=[1696],
                 segments=[("text", 16), ("image", 1296), ("text", 384)]),
    # four images interleaved with text
    "C4": Config("C4-multi-image", 1, 28, 4, 128, 60, 6, 4, 152064, 0.6, 28, "bf16", prefix=[6684],
                 segments=[("text", 300), ("image", 1296), ("text", 300), ("image", 1296),
                           ("text", 300), ("image", 1296), ("text", 300), ("image", 1296),
                           ("text", 300)]),
    # ragged batch over a paged cache
    "C5": Config("C5-ragged-paged", 16, 28, 4, 128, 60, 6, 4, 152064, 0.7, 28, "bf16",
                 prefix_range=(1024, 8192), paged=True),
}


@dataclass
class AttnInputs:
    """One layer's attention inputs for a batch. Float arrays hold the values *after*
    rounding to the storage dtype (so they are exactly what the device reads);
    for bf16 the *_bits arrays hold the storage itself."""
    cfg: Config
    prefix_len: np.ndarray            # int32 [B]
    parent: np.ndarray                # int32 [B, T]
    q: np.ndarray                     # f32 [B, T, Hq, d]
    k_cache: np.ndarray               # f32, contiguous [B, Hkv, cap, d] or paged [nblk, Hkv, bs, d]
    v_cache: np.ndarray
    cap: int = 0
    block_table: Optional[np.ndarray] = None   # int32 [B, max_blocks]
    n_blocks: int = 0
    scale: float = 1.0
    q_bits: Optional[np.ndarray] = None
    k_bits: Optional[np.ndarray] = None
    v_bits: Optional[np.ndarray] = None
    n_images: Optional[np.ndarray] = None


def draw_prefix(cfg: Config, seed: int) -> (np.ndarray, np.ndarray):
    """Prefix lengths and image counts (metadata only: image and text positions are the
    same kind of cache entry for the target model)."""
    if cfg.prefix is not None:
        S = np.array(cfg.prefix, dtype=np.int32)
        nimg = np.array([sum(1 for s in (cfg.segments or []) if s[0] == "image")] * cfg.B, dtype=np.int32)
        return S, nimg
    g = rng(seed, STREAM_PREFIX)
    lo, hi = cfg.prefix_range
    S = g.integers(lo, hi + 1, size=cfg.B).astype(np.int32)
    nimg = np.zeros(cfg.B, dtype=np.int32)
    for b in range(cfg.B):
        cap_img = min(4, (int(S[b]) - 16) // 1296)
        nimg[b] = 0 if cap_img <= 0 else int(g.integers(1, cap_img + 1))
    return S, nimg


def draw_trees(cfg: Config, seed: int) -> np.ndarray:
    out = np.empty((cfg.B, cfg.T), dtype=np.int32)
    for b in range(cfg.B):
        out[b] = random_tree(rng(seed, STREAM_TREE, b), cfg.T, cfg.max_depth, cfg.max_children)
    return out


def _store(x: np.ndarray, dtype: str):
    """Round to the storage dtype; returns (values as f32, bf16 bits or None)."""
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return bf16_bits_to_f32(bits), bits
    return np.ascontiguousarray(x, dtype=np.float32), None


def attention_inputs(cfg: Config, seed: int, layer: int = 0, poison_tail: bool = True,
                     prefix_len: Optional[np.ndarray] = None, parent: Optional[np.ndarray] = None,
                     extra_cap: int = 5) -> AttnInputs:
    """Q/K/V ~ N(0,1) rounded once to the storage dtype. The cache of each sequence
    holds prefix_len + T tokens (the T tree nodes' K/V sit in slots S..S+T-1, as a
    verify forward leaves them). With `poison_tail`, every cache slot that holds no
    token (capacity beyond S+T, unused slots of a sequence's last block, unused pool
    blocks) is filled with NaN so that any read of it shows up in the output."""
    B, T, Hq, Hkv, d = cfg.B, cfg.T, cfg.Hq, cfg.Hkv, cfg.d
    if prefix_len is None:
        prefix_len, nimg = draw_prefix(cfg, seed)
    else:
        prefix_len = np.asarray(prefix_len, dtype=np.int32)
        nimg = None
    if parent is None:
        parent = draw_trees(cfg, seed)
    sub = layer
    q = rng(seed, STREAM_Q, sub).standard_normal((B, T, Hq, d), dtype=np.float32)
    qv, qb = _store(q, cfg.dtype)
    fill = np.float32(np.nan) if poison_tail else np.float32(0.0)
    gk = rng(seed, STREAM_K, sub)
    gv = rng(seed, STREAM_V, sub)
    ntok = prefix_len.astype(np.int64) + T
    if not cfg.paged:
        cap = int(ntok.max()) + extra_cap
        k = np.full((B, Hkv, cap, d), fill, dtype=np.float32)
        v = np.full((B, Hkv, cap, d), fill, dtype=np.float32)
        for b in range(B):
            n = int(ntok[b])
            k[b, :, :n, :] = gk.standard_normal((Hkv, n, d), dtype=np.float32)
            v[b, :, :n, :] = gv.standard_normal((Hkv, n, d), dtype=np.float32)
        kv_, kb = _store(k, cfg.dtype)
        vv_, vb = _store(v, cfg.dtype)
        return AttnInputs(cfg, prefix_len, parent, qv, kv_, vv_, cap=cap, scale=1.0 / np.sqrt(d),
                          q_bits=qb, k_bits=kb, v_bits=vb, n_images=nimg)
    bs = cfg.block_size
    nblk_seq = (ntok + bs - 1) // bs
    n_used = int(nblk_seq.sum())
    n_blocks = n_used + 3                       # a few pool blocks nobody owns
    perm = rng(seed, STREAM_BLOCKS).permutation(n_blocks).astype(np.int32)
    max_blocks = int(nblk_seq.max()) + 1
    table = np.full((B, max_blocks), -1, dtype=np.int32)
    k = np.full((n_blocks, Hkv, bs, d), fill, dtype=np.float32)
    v = np.full((n_blocks, Hkv, bs, d), fill, dtype=np.float32)
    at = 0
    for b in range(B):
        nb = int(nblk_seq[b])
        ids = perm[at:at + nb]
        at += nb
        table[b, :nb] = ids
        n = int(ntok[b])
        kk = gk.standard_normal((Hkv, nb * bs, d), dtype=np.float32)
        vv = gv.standard_normal((Hkv, nb * bs, d), dtype=np.float32)
        kk[:, n:, :] = fill
        vv[:, n:, :] = fill
        k[ids] = kk.reshape(Hkv, nb, bs, d).transpose(1, 0, 2, 3)
        v[ids] = vv.reshape(Hkv, nb, bs, d).transpose(1, 0, 2, 3)
    kv_, kb = _store(k, cfg.dtype)
    vv_, vb = _store(v, cfg.dtype)
    return AttnInputs(cfg, prefix_len, parent, qv, kv_, vv_, block_table=table, n_blocks=n_blocks,
                      scale=1.0 / np.sqrt(d), q_bits=qb, k_bits=kb, v_bits=vb, n_images=nimg)


@dataclass
class AcceptInputs:
    cfg: Config
    parent: np.ndarray      # int32 [B, T]
    tokens: np.ndarray      # int32 [B, T]
    logits: np.ndarray      # f32 [B, T, V]


def accept_inputs(cfg: Config, seed: int, parent: Optional[np.ndarray] = None,
                  B: Optional[int] = None) -> AcceptInputs:
    if parent is None:
        parent = draw_trees(cfg, seed)
    nb = parent.shape[0] if B is None else B
    tok = np.empty((nb, cfg.T), dtype=np.int32)
    lg = np.empty((nb, cfg.T, cfg.V), dtype=np.float32)
    for b in range(nb):
        tok[b] = draft_tokens(rng(seed, STREAM_TOKENS, b), parent[b], cfg.V)
        lg[b] = logits_with_plants(rng(seed, STREAM_LOGITS, b), rng(seed, STREAM_PLANT, b),
                                   parent[b], tok[b], cfg.V, cfg.pi)
    return AcceptInputs(cfg, parent[:nb], tok, lg)


def random_accept_path(g: np.random.Generator, parent: np.ndarray, full: bool = False):
    """A root-to-node path of one tree, as tree_accept reports it: (path int32[T] padded with
    -1, accepted_len). The end node is drawn uniformly (the deepest node of lowest index if
    `full`)."""
    T = len(parent)
    depth = np.zeros(T, dtype=np.int32)
    for i in range(1, T):
        depth[i] = depth[parent[i]] + 1
    end = int(np.argmax(depth)) if full else int(g.integers(0, T))
    path = np.full(T, -1, dtype=np.int32)
    j = end
    while j != -1:
        path[depth[j]] = j
        j = int(parent[j])
    return path, int(depth[end])


def uniforms(seed: int, B: int, T: int):
    """The random numbers a stochastic acceptance consumes, as inputs: u_accept f32 [B,T] and
    u_bonus f32 [B], uniform in [0, 1) (24 random bits each, so the fp32 value is exact)."""
    g = rng(seed, STREAM_UNIFORM)
    ua = (g.integers(0, 1 << 24, size=(B, T)).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
    ub = (g.integers(0, 1 << 24, size=(B,)).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
    return ua, ub


def logits_with_candidates(g_logits: np.random.Generator, g_cand: np.random.Generator, parent: np.ndarray,
                           tokens: np.ndarray, V: int, spread: float = 1.5) -> np.ndarray:
    """Logits for stochastic acceptance: N(0,1) rows in which every child's token is raised to
    about the level where one candidate holds a sizeable share of its parent's softmax mass
    (log of the row's expected background mass V*sqrt(e), plus N(0, spread^2)), the way a draft
    model's top-k candidates sit among the target's likely tokens. f32 [T, V]."""
    T = len(parent)
    lg = g_logits.standard_normal((T, V), dtype=np.float32)
    level = np.log(V) + 0.5
    for c in range(1, T):
        lg[parent[c], tokens[c]] = np.float32(level + spread * g_cand.standard_normal())
    return lg


STREAM_DRAFT = 13


def draft_logits(seed: int, b: int, level: int, F: int, V: int, sharp: float = 3.0) -> np.ndarray:
    """Stand-in for a draft model's output at the F frontier nodes of one expansion step:
    f32 [F, V], N(0, sharp^2) so that a handful of tokens hold most of each row's mass, as a
    trained draft head's logits do."""
    g = rng(seed, STREAM_DRAFT, b * 64 + level)
    return (sharp * g.standard_normal((F, V), dtype=np.float32)).astype(np.float32)


STREAM_ADAPTOR = 14


def compress_inputs(seed: int, B: int, nq: int, Hq: int, Hkv: int, d: int, lens, dtype: str = "bf16",
                    cap: Optional[int] = None):
    """Inputs of the vision adaptor's compression attention: nq query vectors per image (stand-ins
    for the learnable queries after their projection), K / V of lens[b] image embeddings per image
    in a contiguous [B, Hkv, cap, d] cache whose slots beyond lens[b] are NaN. Values N(0,1),
    rounded once to the storage dtype. Returns a dict of f32 values (and bf16 bits when dtype is
    bf16)."""
    lens = np.asarray(lens, dtype=np.int32)
    cap = int(lens.max()) + 5 if cap is None else cap
    g = rng(seed, STREAM_ADAPTOR)
    q = g.standard_normal((B, nq, Hq, d), dtype=np.float32)
    k = g.standard_normal((B, Hkv, cap, d), dtype=np.float32)
    v = g.standard_normal((B, Hkv, cap, d), dtype=np.float32)
    qv, qb = _store(q, dtype)
    kv, kb = _store(k, dtype)
    vv, vb = _store(v, dtype)
    for b in range(B):
        for arr, bits in ((kv, kb), (vv, vb)):
            arr[b, :, lens[b]:] = np.nan
            if bits is not None:
                bits[b, :, lens[b]:] = 0x7FC0
    return dict(q=qv, k=kv, v=vv, q_bits=qb, k_bits=kb, v_bits=vb, lens=lens, cap=cap, scale=1.0 / np.sqrt(d))
