"""Seeded synthetic inputs for the tree-masked Mamba2 SSD verification pass.

This module only *draws* data: token trees as parent-index arrays and random
tensors of the workload shapes.  It holds none of the method's arithmetic (no
decay, no recurrence, no convolution) so that it can feed both the HIP path and
the independent CPU oracle without the two sharing any computation.

The paper's experiments feed real model activations (MT-Bench, HumanEval,
GSM8K prompts through Mamba2 / MambaInLlama); kernel cost depends only on the
shapes and the tree topology, so seeded synthetic tensors of the same shapes
stand in for them.  Tree sizes follow the paper's own workloads: full binary
trees of 15/31/63 tokens (Sec. 5.1), beam-search trees of M tokens per layer
for N layers (Table "tree-decoding-gen"), and static trees of 13-29 tokens
(Table "static-configs").

bf16 tensors are carried as numpy ``uint16`` bit patterns (numpy has no
bfloat16); the *rounded* values are what both consumers receive.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 20250514 * 10

# --------------------------------------------------------------------------- #
# bf16 <-> fp32 bit manipulation (data format handling only)
# --------------------------------------------------------------------------- #


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen uint16 bf16 bit patterns to fp32 exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# --------------------------------------------------------------------------- #
# trees
# --------------------------------------------------------------------------- #


def full_binary_tree(levels: int) -> np.ndarray:
    """Full binary tree with ``levels`` levels: parent[i] = (i-1)//2, root -1."""
    n = (1 << levels) - 1
    parent = (np.arange(n, dtype=np.int64) - 1) // 2
    parent[0] = -1
    return parent.astype(np.int32)


def chain_tree(n: int) -> np.ndarray:
    """Linear chain: parent[i] = i-1 (the lower-triangular mask case)."""
    return (np.arange(n, dtype=np.int32) - 1).astype(np.int32)


def star_tree(n: int) -> np.ndarray:
    """Root with n-1 leaf children."""
    parent = np.zeros(n, dtype=np.int32)
    parent[0] = -1
    return parent


def _children_lists(parent: np.ndarray) -> List[List[int]]:
    kids: List[List[int]] = [[] for _ in range(len(parent))]
    for i, p in enumerate(parent):
        if p >= 0:
            kids[int(p)].append(i)
    return kids


def relabel_bfs(parent: np.ndarray) -> np.ndarray:
    """Relabel a rooted tree (any labelling, root = the node with parent -1) in
    breadth-first order, children in increasing old label.  Result has
    parent[0] = -1 and parent[i] < i."""
    kids = _children_lists(parent)
    root = int(np.flatnonzero(np.asarray(parent) < 0)[0])
    order = [root]
    head = 0
    while head < len(order):
        order.extend(kids[order[head]])
        head += 1
    return _apply_order(parent, order)


def relabel_dfs(parent: np.ndarray) -> np.ndarray:
    """Relabel in depth-first pre-order (children in increasing old label)."""
    kids = _children_lists(parent)
    root = int(np.flatnonzero(np.asarray(parent) < 0)[0])
    order: List[int] = []
    stack = [root]
    while stack:
        u = stack.pop()
        order.append(u)
        stack.extend(reversed(kids[u]))
    return _apply_order(parent, order)


def _apply_order(parent: np.ndarray, order: List[int]) -> np.ndarray:
    new_of_old = np.empty(len(parent), dtype=np.int64)
    new_of_old[np.asarray(order)] = np.arange(len(order))
    out = np.empty(len(parent), dtype=np.int32)
    for old, p in enumerate(parent):
        out[new_of_old[old]] = -1 if p < 0 else new_of_old[int(p)]
    return out


def relabel_permutation(parent: np.ndarray, relabel) -> np.ndarray:
    """perm[new] = old for the relabelling function ``relabel`` (bfs or dfs)."""
    kids = _children_lists(parent)
    root = int(np.flatnonzero(np.asarray(parent) < 0)[0])
    if relabel is relabel_bfs:
        order = [root]
        head = 0
        while head < len(order):
            order.extend(kids[order[head]])
            head += 1
    else:
        order = []
        stack = [root]
        while stack:
            u = stack.pop()
            order.append(u)
            stack.extend(reversed(kids[u]))
    return np.asarray(order, dtype=np.int64)


def gen_tree(n: int, depth: int, cmax: int, rng: np.random.Generator) -> np.ndarray:
    """Random tree with exactly ``n`` nodes and exactly ``depth`` edges on its
    longest root path.  A spine of depth+1 nodes fixes the depth; further
    nodes attach to a uniformly chosen open node, where a node at level l is
    open while it has fewer than cap(l) children and l < depth, with
    cap(l) = max(1, cmax - (l*(cmax-1))//depth): the child budget shrinks with
    the level (root up to ``cmax``).  Returned in breadth-first labelling."""
    if n < depth + 1:
        raise ValueError("n must be at least depth+1")
    par = [-1] + list(range(depth))
    lev = list(range(depth + 1))
    nkid = [1] * depth + [0]

    def cap(l: int) -> int:
        return max(1, cmax - (l * (cmax - 1)) // max(depth, 1))

    while len(par) < n:
        open_nodes = [u for u in range(len(par)) if lev[u] < depth and nkid[u] < cap(lev[u])]
        if not open_nodes:
            raise ValueError("tree capacity exhausted: raise cmax or depth")
        u = open_nodes[int(rng.integers(len(open_nodes)))]
        par.append(u)
        lev.append(lev[u] + 1)
        nkid.append(0)
        nkid[u] += 1
    return relabel_bfs(np.asarray(par, dtype=np.int32))


def beam_tree(m: int, steps: int, rng: np.random.Generator) -> np.ndarray:
    """Beam-search shaped tree: a root, then ``steps`` layers of ``m`` tokens,
    each token's parent uniform in the previous layer."""
    par = [-1]
    prev = [0]
    for _ in range(steps):
        cur = []
        for _ in range(m):
            par.append(prev[int(rng.integers(len(prev)))])
            cur.append(len(par) - 1)
        prev = cur
    return np.asarray(par, dtype=np.int32)


def static_tree(width: int, depth: int) -> np.ndarray:
    """A root followed by ``depth`` layers of ``width`` tokens, where the
    first token of each layer is the parent of the whole next layer (sizes
    1 + width*depth = 13 for width 3, depth 4: the paper's static tree)."""
    par = [-1]
    anchor = 0
    for _ in range(depth):
        first = len(par)
        par.extend([anchor] * width)
        anchor = first
    return np.asarray(par, dtype=np.int32)


def tree_depths(parent: np.ndarray) -> np.ndarray:
    """Edges from the root, by the topological order parent[i] < i."""
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


# --------------------------------------------------------------------------- #
# workloads
# --------------------------------------------------------------------------- #


@dataclass
class Workload:
    """One seeded problem instance.  fp32 arrays hold the exact values both the
    HIP path and the oracle consume (already rounded to bf16 where
    io_dtype == 'bf16')."""

    name: str
    io_dtype: str                    # 'f32' | 'bf16'
    batch: int
    nnodes: int
    nheads: int
    headdim: int
    dstate: int
    ngroups: int
    conv_width: int                  # 0 = no conv
    parent: np.ndarray               # int32 [B,N]
    dt: np.ndarray                   # f32 [B,N,H]
    A: np.ndarray                    # f32 [H]
    D: np.ndarray                    # f32 [H]
    h0: Optional[np.ndarray]         # f32 [B,H,P,S] (None = drawn elsewhere)
    # without conv: x,B,C drawn directly
    x: Optional[np.ndarray] = None   # f32 [B,N,H,P]
    Bm: Optional[np.ndarray] = None  # f32 [B,N,G,S]
    Cm: Optional[np.ndarray] = None  # f32 [B,N,G,S]
    # with conv: pre-conv activations; x|B|C are channel ranges of the conv output
    xbc_pre: Optional[np.ndarray] = None     # f32 [B,N,Cc]
    conv_state: Optional[np.ndarray] = None  # f32 [B,W-1,Cc], oldest row first
    conv_w: Optional[np.ndarray] = None      # f32 [Cc,W]
    conv_b: Optional[np.ndarray] = None      # f32 [Cc]
    accepted: Optional[np.ndarray] = None    # int32 [B]
    extras: Dict[str, np.ndarray] = field(default_factory=dict)

    @property
    def conv_channels(self) -> int:
        return self.nheads * self.headdim + 2 * self.ngroups * self.dstate


def _softplus(z: np.ndarray) -> np.ndarray:
    return np.logaddexp(0.0, z)


def _streams(config_id: int, n: int = 12) -> List[np.random.Generator]:
    ss = np.random.SeedSequence(BASE_SEED + config_id)
    return [np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(n)]


def draw_tensors(name: str, io_dtype: str, parent: np.ndarray, nheads: int, headdim: int,
                 dstate: int, ngroups: int, conv_width: int, config_id: int,
                 with_accept: bool = False, with_h0: bool = True) -> Workload:
    """Draw every tensor of one call in a fixed stream order:
    (trees), xBC | x,B,C, dt, A, D, h0, conv_w, conv_b, conv_state, accepted.
    x,B,C (or the pre-conv xBC) ~ N(0,1); dt = softplus(N(0,1) - 2);
    A_h = -exp(U(0,2)); D ~ N(0,1); h0 ~ N(0, std 0.1);
    conv_w, conv_b ~ U(-0.5,0.5); conv_state ~ N(0,1)."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    B, N = parent.shape
    H, P, S, G, W = nheads, headdim, dstate, ngroups, conv_width
    st = _streams(config_id)
    rnd = (lambda a: round_to_bf16(a)) if io_dtype == "bf16" else (lambda a: a.astype(np.float32))
    wl = Workload(name=name, io_dtype=io_dtype, batch=B, nnodes=N, nheads=H, headdim=P,
                  dstate=S, ngroups=G, conv_width=W, parent=parent,
                  dt=_softplus(st[2].standard_normal((B, N, H)) - 2.0).astype(np.float32),
                  A=(-np.exp(st[3].uniform(0.0, 2.0, H))).astype(np.float32),
                  D=st[4].standard_normal(H).astype(np.float32),
                  h0=(0.1 * st[5].standard_normal((B, H, P, S))).astype(np.float32) if with_h0 else None)
    if W > 0:
        Cc = H * P + 2 * G * S
        wl.xbc_pre = rnd(st[1].standard_normal((B, N, Cc)).astype(np.float32))
        wl.conv_w = rnd(st[6].uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
        wl.conv_b = rnd(st[7].uniform(-0.5, 0.5, Cc).astype(np.float32))
        wl.conv_state = rnd(st[8].standard_normal((B, W - 1, Cc)).astype(np.float32))
    else:
        g = st[1]
        wl.x = rnd(g.standard_normal((B, N, H, P)).astype(np.float32))
        wl.Bm = rnd(g.standard_normal((B, N, G, S)).astype(np.float32))
        wl.Cm = rnd(g.standard_normal((B, N, G, S)).astype(np.float32))
    if with_accept:
        wl.accepted = st[9].integers(0, N, size=B).astype(np.int32)
    return wl


def direct_xbc(wl: Workload, seed_offset: int = 100) -> Workload:
    """Variant of a conv workload whose x,B,C are drawn N(0,1) directly (so the
    SSD sees the same input statistics as the no-conv configuration)."""
    g = _streams(seed_offset + zlib.crc32(wl.name.encode()) % 89, 2)[0]
    rnd = (lambda a: round_to_bf16(a)) if wl.io_dtype == "bf16" else (lambda a: a.astype(np.float32))
    B, N, H, P, S, G = wl.batch, wl.nnodes, wl.nheads, wl.headdim, wl.dstate, wl.ngroups
    out = Workload(**{**wl.__dict__})
    out.conv_width = 0
    out.xbc_pre = out.conv_state = out.conv_w = out.conv_b = None
    out.x = rnd(g.standard_normal((B, N, H, P)).astype(np.float32))
    out.Bm = rnd(g.standard_normal((B, N, G, S)).astype(np.float32))
    out.Cm = rnd(g.standard_normal((B, N, G, S)).astype(np.float32))
    return out


def config(config_id: int, scale: Optional[dict] = None) -> Workload:
    """The five benchmark configurations.  ``scale`` may override batch/nheads
    (e.g. {"batch": 2, "nheads": 8}) to get a small instance with the same
    recipe for CPU-only tests."""
    scale = scale or {}
    st = _streams(config_id)
    tr = st[0]
    if config_id == 0:
        parent = full_binary_tree(4)[None, :]
        return draw_tensors("cfg0_binary15_f32", "f32", parent, scale.get("nheads", 4), 64, 64, 1, 0, 0)
    if config_id == 1:
        parent = gen_tree(64, 6, 4, tr)[None, :]
        return draw_tensors("cfg1_tree64_b1", "bf16", parent, scale.get("nheads", 80), 64, 128, 1, 4, 1)
    if config_id == 2:
        B = scale.get("batch", 16)
        trees = []
        for _ in range(B):
            d = 4 + int(tr.integers(0, 5))
            trees.append(gen_tree(64, d, 4, tr))
        return draw_tensors("cfg2_tree64_b16", "bf16", np.stack(trees), scale.get("nheads", 80), 64, 128, 1, 4, 2,
                            with_accept=True)
    if config_id == 3:
        B = scale.get("batch", 4)
        trees = [gen_tree(256, 10, 8, tr) for _ in range(B - 1)] + [chain_tree(256)]
        H = scale.get("nheads", 128)
        return draw_tensors("cfg3_tree256_g8", "bf16", np.stack(trees), H, 64, 128, scale.get("ngroups", 8), 0, 3)
    if config_id == 4:
        B = scale.get("batch", 8)
        H = scale.get("nheads", 80)
        T = scale.get("prefix", 4096)
        trees = np.stack([gen_tree(128, 8, 4, tr) for _ in range(B)])
        wl = draw_tensors("cfg4_prefix_tree128", "bf16", trees, H, 64, 128, 1, 4, 4, with_h0=False)
        # accepted node: path length l ~ U{1..8} nodes, a uniform node of depth l-1
        acc = np.empty(B, dtype=np.int32)
        for b in range(B):
            l = int(st[9].integers(1, 9))
            dep = tree_depths(trees[b])
            cand = np.flatnonzero(dep == l - 1)
            acc[b] = cand[int(st[9].integers(len(cand)))]
        wl.accepted = acc
        # prefix activations (post-conv x,B,C drawn directly) and its dt
        g = st[10]
        wl.extras["prefix_x"] = round_to_bf16(g.standard_normal((B, T, H, 64)).astype(np.float32))
        wl.extras["prefix_B"] = round_to_bf16(g.standard_normal((B, T, 1, 128)).astype(np.float32))
        wl.extras["prefix_C"] = round_to_bf16(g.standard_normal((B, T, 1, 128)).astype(np.float32))
        wl.extras["prefix_dt"] = _softplus(g.standard_normal((B, T, H)) - 2.0).astype(np.float32)
        return wl
    raise ValueError("config_id must be 0..4")


def sweep_trees(rng: np.random.Generator) -> Dict[str, np.ndarray]:
    """Tree shapes of the paper's own workloads (sizes only; connectivity of the
    static trees is in figures that are not available, so ``static_tree`` is a
    stand-in with the printed token counts)."""
    out = {f"binary{(1 << l) - 1}": full_binary_tree(l) for l in (4, 5, 6)}
    for m in (2, 3, 4, 5):
        for n in (4, 8, 16):
            out[f"beam_m{m}_n{n}"] = beam_tree(m, n, rng)
    out["static13"] = static_tree(3, 4)
    out["static16"] = static_tree(3, 5)
    return out
