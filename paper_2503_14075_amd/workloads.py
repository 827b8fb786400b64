"""Seeded synthetic workloads with the shapes of the paper's models.

This module only *generates inputs*: counter-based random tensors, ragged
lengths, draft-tree topologies, page tables and token ids.  It contains none
of the method's arithmetic (no attention, no top-k, no gather, no acceptance
walk), so that both the CPU oracle's tests and the HIP path's tests can be fed
byte-identical buffers from here without sharing any computation.

Shapes follow the models the paper evaluates (Sec. 6.1 and Tables 1-2):
576 visual tokens for LLaVA-1.5, 2880 (5 tiles x 576) for LLaVA-NeXT,
32 heads x 128, 32 layers, and draft trees bounded by the tree-SSD defaults
of App. A (at most 60 candidates plus the root, depth 4-6).

Randomness: every tensor element is a pure function of (seed, stream, index)
through the public splitmix64 finaliser, turned into a normal deviate by
Box-Muller in fp64 and then rounded to the storage type.  Host-side structure
(lengths, parents, page order) uses the same generator one value at a time.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


# --------------------------------------------------------------------------
# scalar generator (host-side structure)
# --------------------------------------------------------------------------
def mix64(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _C1) & _MASK64
    z = ((z ^ (z >> 27)) * _C2) & _MASK64
    return z ^ (z >> 31)


class HostRng:
    """splitmix64 sequence for lengths, tree topologies and page orders."""

    def __init__(self, seed: int, stream: int = 0):
        self.state = mix64((seed * 0x1000003 + stream * _GOLDEN + 0x5851F42D4C957F2D) & _MASK64)

    def next_u64(self) -> int:
        self.state = (self.state + _GOLDEN) & _MASK64
        return mix64(self.state)

    def randint(self, lo: int, hi: int) -> int:
        """Uniform integer in [lo, hi], both ends included."""
        return lo + self.next_u64() % (hi - lo + 1)

    def uniform(self) -> float:
        return ((self.next_u64() >> 11) + 0.5) * (1.0 / (1 << 53))

    def shuffle(self, xs: List[int]) -> None:
        for i in range(len(xs) - 1, 0, -1):
            j = self.next_u64() % (i + 1)
            xs[i], xs[j] = xs[j], xs[i]


# --------------------------------------------------------------------------
# tensor generator (counter based; runs on whatever device it is given)
# --------------------------------------------------------------------------
def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64_t(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _stream_key(seed: int, stream: int) -> int:
    return mix64((seed & 0xFFFFFFFF) * 0x100000001B3 + (stream + 1) * _GOLDEN)


def _u64_at(seed: int, stream: int, start: int, count: int, device) -> torch.Tensor:
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    key = _s64(_stream_key(seed, stream))
    return _mix64_t(idx * _s64(_GOLDEN) + key)


def _unit(x: torch.Tensor) -> torch.Tensor:
    return (_lsr(x, 11).to(torch.float64) + 0.5) * (1.0 / (1 << 53))


_CHUNK = 1 << 23


def normal(seed: int, stream: int, shape: Sequence[int], std: float, dtype: torch.dtype,
           device="cpu") -> torch.Tensor:
    """N(0, std^2) deviates rounded (to nearest even) to `dtype`."""
    n = int(math.prod(shape))
    out = torch.empty(n, dtype=dtype, device=device)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        u1 = _unit(_u64_at(seed, stream, 2 * s, 2 * c, device))
        r = torch.sqrt(-2.0 * torch.log(u1[0::2]))
        z = r * torch.cos((2.0 * math.pi) * u1[1::2])
        out[s:s + c] = (z * std).to(dtype)
    return out.view(*shape)


def integers(seed: int, stream: int, shape: Sequence[int], lo: int, hi: int,
             device="cpu") -> torch.Tensor:
    """Uniform int32 in [lo, hi]."""
    n = int(math.prod(shape))
    x = _lsr(_u64_at(seed, stream, 0, n, device), 11) % (hi - lo + 1) + lo
    return x.to(torch.int32).view(*shape)


# --------------------------------------------------------------------------
# draft-tree topologies
# --------------------------------------------------------------------------
def random_parent_tree(rng: HostRng, T: int, max_depth: int) -> List[int]:
    """Node 0 is the root (parent -1); node i>0 hangs under a uniformly drawn
    earlier node whose depth is still below the cap."""
    parent, depth = [-1], [0]
    for i in range(1, T):
        cands = [j for j in range(i) if depth[j] < max_depth]
        p = cands[rng.next_u64() % len(cands)]
        parent.append(p)
        depth.append(depth[p] + 1)
    return parent


def fanout_tree(rng: HostRng, T: int, fanout: Sequence[int]) -> List[int]:
    """Expand the full tree whose nodes at depth d have fanout[d] children,
    give every node a confidence (product of seeded, rank-decaying sibling
    probabilities along its path) and keep the root plus the T-1 most
    confident nodes.  Confidence shrinks along a path, so the kept set is
    closed under taking parents.  Nodes are renumbered breadth first.  This
    mirrors how App. A bounds a drafted tree to N_max candidates."""
    par, dep, conf = [-1], [0], [1.0]
    frontier = [0]
    for d, f in enumerate(fanout):
        nxt = []
        for u in frontier:
            w = [(0.55 ** r) * (0.75 + 0.5 * rng.uniform()) for r in range(f)]
            tot = sum(w) * 1.02
            for r in range(f):
                par.append(u)
                dep.append(d + 1)
                conf.append(conf[u] * w[r] / tot)
                nxt.append(len(par) - 1)
        frontier = nxt
    order = sorted(range(1, len(par)), key=lambda i: (-conf[i], i))
    keep = sorted([0] + order[:T - 1], key=lambda i: (dep[i], i))
    if len(keep) != T:
        raise ValueError("fan-out tree smaller than the requested node count")
    new_id = {old: k for k, old in enumerate(keep)}
    return [-1 if par[old] < 0 else new_id[par[old]] for old in keep]


def tree_depths(parent: Sequence[int]) -> List[int]:
    d = []
    for i, p in enumerate(parent):
        d.append(0 if p < 0 else d[p] + 1)
    return d


def plant_tokens(rng: HostRng, parent: Sequence[int], vocab: int = 32000,
                 p_match: float = 0.6) -> Tuple[List[int], List[int]]:
    """Draft ids and target-argmax ids uniform in [0, vocab); then, with
    probability p_match per node (close to the token acceptance rate the
    paper reports), one of the node's children is given the node's argmax id
    so that acceptance paths of non-trivial length occur."""
    T = len(parent)
    draft = [rng.randint(0, vocab - 1) for _ in range(T)]
    argmx = [rng.randint(0, vocab - 1) for _ in range(T)]
    kids: Dict[int, List[int]] = {}
    for i, p in enumerate(parent):
        if p >= 0:
            kids.setdefault(p, []).append(i)
    for u in range(T):
        if u in kids and rng.uniform() < p_match:
            c = kids[u][rng.next_u64() % len(kids[u])]
            draft[c] = argmx[u]
    return draft, argmx


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    dtype: str                 # "f32" or "bf16"
    H: int
    d_h: int
    hidden: int
    M: int                     # visual tokens
    N: Tuple[int, int]         # text tokens, inclusive range
    n_q: Optional[int]         # scoring rows (last n_q text rows); None = all text rows
    R: int                     # kept visual tokens
    P: Tuple[int, int]         # generated-prefix rows, inclusive range
    T: int                     # tree rows, root included
    tree: Tuple                # ("random", depth_cap) or ("fanout", (f0, f1, ...))
    B: int = 1                 # sequences
    L: int = 1                 # independent per-layer caches verified per sequence
    compact_layers: int = 1    # layers whose K and V are compacted (hidden is always)
    paged: bool = False
    page_rows: int = 16
    kv_std: float = 1.0
    q_std: float = 1.0

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d_h)


_LLAVA = dict(dtype="bf16", H=32, d_h=128, hidden=4096, kv_std=0.5, q_std=1.0 / math.sqrt(128.0))

CONFIGS: Dict[str, Config] = {
    "cfg0": Config("cfg0", 0, "f32", 4, 64, 256, 576, (32, 32), 8, 64, (0, 0), 8, ("random", 4)),
    "cfg1": Config("cfg1", 1, M=576, N=(64, 64), n_q=None, R=64, P=(128, 128), T=26,
                   tree=("fanout", (4, 3, 2, 1, 1)), **_LLAVA),
    "cfg2_p0": Config("cfg2_p0", 2, M=576, N=(64, 64), n_q=None, R=64, P=(0, 0), T=64,
                      tree=("random", 6), L=32, compact_layers=30, **_LLAVA),
    "cfg2_p256": Config("cfg2_p256", 2, M=576, N=(64, 64), n_q=None, R=64, P=(256, 256), T=64,
                        tree=("random", 6), L=32, compact_layers=30, **_LLAVA),
    "cfg2_p1024": Config("cfg2_p1024", 2, M=576, N=(64, 64), n_q=None, R=64, P=(1024, 1024), T=64,
                         tree=("random", 6), L=32, compact_layers=30, **_LLAVA),
    "cfg3": Config("cfg3", 3, M=576, N=(32, 128), n_q=None, R=64, P=(0, 512), T=32,
                   tree=("random", 5), B=16, paged=True, **_LLAVA),
    "cfg4": Config("cfg4", 4, M=2880, N=(128, 128), n_q=16, R=320, P=(2048, 2048), T=64,
                   tree=("fanout", (8, 4, 2, 2, 1, 1)), B=4, **_LLAVA),
}


def replicate(cfg: Config, B: int, name: Optional[str] = None) -> Config:
    """The same shapes with B independent sequences (different values each)."""
    d = dict(cfg.__dict__)
    d.update(B=B, name=name or f"{cfg.name}x{B}")
    return Config(**d)


@dataclass
class Workload:
    cfg: Config
    # ---- per sequence (B) ----
    n_text: List[int]
    n_tot: List[int]
    n_q: List[int]
    n_q_max: int
    q_pos0: List[int]                  # absolute position of the first scoring row
    score_row_off: List[int]           # first row of sequence b in k_score
    q_sel: torch.Tensor                # [B][n_q_max][H][d_h]
    k_score: torch.Tensor              # [sum n_tot][H][d_h]
    compact_src: List[torch.Tensor]    # [n_tensors] pools [sum n_tot][row_elems]; sequence b at score_row_off[b]
    compact_dst_off: List[int]         # first destination row of sequence b (sum of kept rows before it)
    # ---- per verified instance (B*L, sequence-major: inst = b*L + layer) ----
    ctx_len: List[int]
    n_nodes: List[int]
    parent: List[List[int]]            # [B*L][T]
    q_tree: torch.Tensor               # [B*L][T][H][d_h]
    k_pool: torch.Tensor               # [pool_rows][H][d_h]
    v_pool: torch.Tensor
    row_off: Optional[List[int]]       # contiguous mode: first pool row of instance
    page_table: Optional[List[List[int]]]   # paged mode: [B*L][max_pages]
    max_pages: int
    # ---- per sequence acceptance ----
    draft: List[List[int]]             # [B][T]
    argmax: List[List[int]]
    tree_seq: List[List[int]]          # [B][T] parent of the sequence's tree
    extras: Dict[str, object] = field(default_factory=dict)


# stream ids for the tensor generator
_ST_QSEL, _ST_KSCORE, _ST_QTREE, _ST_KPOOL, _ST_VPOOL, _ST_COMPACT = 1, 2, 3, 4, 5, 16


def make_workload(cfg: Config, device="cpu", with_compact: bool = True,
                  with_score: bool = True) -> Workload:
    rng = HostRng(cfg.seed, 0)
    B, L, T, H, d_h = cfg.B, cfg.L, cfg.T, cfg.H, cfg.d_h
    dt = cfg.torch_dtype
    n_text = [rng.randint(*cfg.N) for _ in range(B)]
    p_len = [rng.randint(*cfg.P) for _ in range(B)]
    n_tot = [cfg.M + n for n in n_text]
    n_q = [n if cfg.n_q is None else min(cfg.n_q, n) for n in n_text]
    n_q_max = max(n_q)
    q_pos0 = [nt - q for nt, q in zip(n_tot, n_q)]

    # trees: one per sequence, shared by that sequence's layers
    trees = []
    for b in range(B):
        trng = HostRng(cfg.seed, 100 + b)
        if cfg.tree[0] == "random":
            trees.append(random_parent_tree(trng, T, cfg.tree[1]))
        else:
            trees.append(fanout_tree(trng, T, cfg.tree[1]))
    draft, argmx = [], []
    for b in range(B):
        d, a = plant_tokens(HostRng(cfg.seed, 200 + b), trees[b])
        draft.append(d)
        argmx.append(a)

    # scoring inputs
    score_row_off, acc = [], 0
    for b in range(B):
        score_row_off.append(acc)
        acc += n_tot[b]
    if with_score:
        q_sel = normal(cfg.seed, _ST_QSEL, (B, n_q_max, H, d_h), cfg.q_std, dt, device)
        k_score = normal(cfg.seed, _ST_KSCORE, (acc, H, d_h), cfg.kv_std, dt, device)
    else:
        q_sel = torch.empty(0, dtype=dt, device=device)
        k_score = torch.empty(0, dtype=dt, device=device)

    # compaction sources: hidden, then K and V of each compacted layer; every tensor is
    # one pool holding all sequences back to back (same row offsets as k_score)
    compact_src: List[torch.Tensor] = []
    compact_dst_off, dacc = [], 0
    for b in range(B):
        compact_dst_off.append(dacc)
        dacc += cfg.R + n_text[b]
    if with_compact:
        compact_src.append(normal(cfg.seed, _ST_COMPACT, (acc, cfg.hidden), 1.0, dt, device))
        for l in range(cfg.compact_layers):
            for kv in range(2):
                compact_src.append(normal(cfg.seed, _ST_COMPACT + 1 + 2 * l + kv, (acc, H * d_h),
                                          cfg.kv_std, dt, device))

    # verification caches: instance = (sequence, layer)
    n_keep = [cfg.R + n for n in n_text]
    ctx_len, n_nodes, parent = [], [], []
    for b in range(B):
        for _ in range(L):
            ctx_len.append(n_keep[b] + p_len[b])
            n_nodes.append(T)
            parent.append(list(trees[b]))
    n_inst = B * L
    rows = [c + T for c in ctx_len]
    row_off: Optional[List[int]] = None
    page_table: Optional[List[List[int]]] = None
    max_pages = 0
    if cfg.paged:
        pr = cfg.page_rows
        n_pages = [(r + pr - 1) // pr for r in rows]
        max_pages = max(n_pages)
        ids = list(range(sum(n_pages)))
        HostRng(cfg.seed, 300).shuffle(ids)
        page_table, k = [], 0
        for i in range(n_inst):
            page_table.append(ids[k:k + n_pages[i]] + [0] * (max_pages - n_pages[i]))
            k += n_pages[i]
        pool_rows = sum(n_pages) * pr
    else:
        row_off, acc = [], 0
        for i in range(n_inst):
            row_off.append(acc)
            acc += rows[i]
        pool_rows = acc
    q_tree = normal(cfg.seed, _ST_QTREE, (n_inst, T, H, d_h), cfg.q_std, dt, device)
    k_pool = normal(cfg.seed, _ST_KPOOL, (pool_rows, H, d_h), cfg.kv_std, dt, device)
    v_pool = normal(cfg.seed, _ST_VPOOL, (pool_rows, H, d_h), cfg.kv_std, dt, device)

    return Workload(cfg=cfg, n_text=n_text, n_tot=n_tot, n_q=n_q, n_q_max=n_q_max, q_pos0=q_pos0,
                    score_row_off=score_row_off, q_sel=q_sel, k_score=k_score,
                    compact_src=compact_src, compact_dst_off=compact_dst_off, ctx_len=ctx_len, n_nodes=n_nodes, parent=parent,
                    q_tree=q_tree, k_pool=k_pool, v_pool=v_pool, row_off=row_off,
                    page_table=page_table, max_pages=max_pages, draft=draft, argmax=argmx,
                    tree_seq=trees)


def instance_rows(w: Workload, inst: int) -> torch.Tensor:
    """Pool row index of every cache row (context then tree rows) of one
    verified instance, as an int64 tensor on the CPU."""
    n = w.ctx_len[inst] + w.n_nodes[inst]
    r = torch.arange(n, dtype=torch.int64)
    if w.page_table is None:
        return r + w.row_off[inst]
    pr = w.cfg.page_rows
    pt = torch.tensor(w.page_table[inst], dtype=torch.int64)
    return pt[r // pr] * pr + r % pr
