"""ctypes front end of the fp64 CPU oracle (oracle/twig_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU package never imports this, and
this never imports the GPU package.

Tensors cross as CPU torch tensors (fp32, or bf16 viewed as 16-bit patterns);
results come back as torch tensors.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "twig_oracle.c")
_LIB = os.path.join(_HERE, "libtwig_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_max_threads.restype = ctypes.c_int
        _lib.orc_rbar.restype = ctypes.c_int
    return _lib


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


def max_threads() -> int:
    return int(lib().orc_max_threads())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError(f"oracle takes fp32 or bf16 inputs, got {t.dtype}")


def _p(t: torch.Tensor):
    assert t.device.type == "cpu" and t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def _i32(xs) -> torch.Tensor:
    return torch.as_tensor(xs, dtype=torch.int32).contiguous()


def _i64(xs) -> torch.Tensor:
    return torch.as_tensor(xs, dtype=torch.int64).contiguous()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid argument (code {rc})")


def ttp_score(q_sel: torch.Tensor, k: torch.Tensor, n_q: Sequence[int], q_pos0: Sequence[int],
              n_tot: Sequence[int], k_row_off: Sequence[int], v_start: int, M: int, scale: float,
              causal: bool = True) -> torch.Tensor:
    """scores [B][M] in fp64.  k may hold fewer heads than q_sel (grouped-query attention: query
    head h reads key head h // (H // H_kv))."""
    B, n_q_max, H, d_h = q_sel.shape
    H_kv = k.shape[1]
    assert k.shape[2] == d_h and H % H_kv == 0 and k.dtype == q_sel.dtype
    out = torch.zeros(B, M, dtype=torch.float64)
    a, b_, c, d = _i32(n_q), _i32(q_pos0), _i32(n_tot), _i64(k_row_off)
    rc = lib().orc_ttp_score(_p(q_sel), _p(k), _dtype_code(k), B, H, H_kv, d_h, n_q_max, _p(a), _p(b_),
                             _p(c), _p(d), int(v_start), int(M), ctypes.c_double(scale),
                             int(bool(causal)), _p(out))
    _check(rc, "ttp_score")
    return out


def ttp_select(scores: torch.Tensor, R: int) -> torch.Tensor:
    """kept [B][R] int32, ascending; scores fp32 [B][M]."""
    assert scores.dtype == torch.float32 and scores.dim() == 2
    B, M = scores.shape
    kept = torch.empty(B, max(R, 0), dtype=torch.int32)
    rc = lib().orc_ttp_select(_p(scores.contiguous()), B, M, int(R), _p(kept))
    _check(rc, "ttp_select")
    return kept


def ttp_compact(kept: torch.Tensor, v_start: int, M: int, src: torch.Tensor) -> torch.Tensor:
    """src [n_tot][...] of any dtype -> dst [v_start + R + n_tot - v_start - M][...]."""
    kept = _i32(kept)
    R, n_tot = int(kept.numel()), int(src.shape[0])
    src = src.contiguous()
    row_bytes = src[0].numel() * src.element_size() if n_tot else 0
    n_out = n_tot - M + R
    # (one row more than needed: an empty result still gets a buffer to point at)
    dst = torch.empty((max(n_out, 0) + 1,) + tuple(src.shape[1:]), dtype=src.dtype)
    rc = lib().orc_ttp_compact(_p(kept), R, int(v_start), int(M), n_tot, _p(src), _p(dst),
                               ctypes.c_size_t(row_bytes))
    _check(rc, "ttp_compact")
    return dst[:max(n_out, 0)]


def tree_ancestors(parent: Sequence[int]) -> List[int]:
    par = _i32(parent)
    T = int(par.numel())
    anc = torch.zeros(max(T, 1), dtype=torch.int64)
    rc = lib().orc_tree_ancestors(_p(par), T, _p(anc))
    _check(rc, "tree_ancestors")
    return [int(x) & ((1 << 64) - 1) for x in anc[:T].tolist()]


def cache_rows(ctx_len: Sequence[int], n_nodes: Sequence[int], row_off: Optional[Sequence[int]],
               page_table: Optional[Sequence[Sequence[int]]], page_rows: int):
    """Pool row of each cache row of each instance.  Contiguous: instance b
    starts at row_off[b].  Paged: cache row r lives in page
    page_table[b][r // page_rows] at slot r % page_rows."""
    rows, offs = [], []
    for b, (c, t) in enumerate(zip(ctx_len, n_nodes)):
        offs.append(len(rows))
        for r in range(c + t):
            if page_table is None:
                rows.append(row_off[b] + r)
            else:
                rows.append(page_table[b][r // page_rows] * page_rows + r % page_rows)
    return _i64(rows), _i64(offs)


def tree_verify_attn(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                     ctx_len: Sequence[int], n_nodes: Sequence[int], parent, scale: float,
                     row_off: Optional[Sequence[int]] = None, page_table=None,
                     page_rows: int = 16) -> torch.Tensor:
    """out [B][T_max][H][d_h] fp64 (rows past n_nodes[b] are zero).  The pools may hold fewer heads
    than q (grouped-query attention: query head h reads key/value head h // (H // H_kv))."""
    B, T_max, H, d_h = q.shape
    H_kv = k_pool.shape[1]
    assert k_pool.shape[2] == d_h and H % H_kv == 0 and v_pool.shape == k_pool.shape
    assert k_pool.dtype == q.dtype == v_pool.dtype
    rows, offs = cache_rows(ctx_len, n_nodes, row_off, page_table, page_rows)
    if rows.numel() and int(rows.max()) >= k_pool.shape[0]:
        raise ValueError("oracle tree_verify_attn: cache row outside the pool")
    par = _i32(parent).view(B, T_max)
    out = torch.zeros(B, T_max, H, d_h, dtype=torch.float64)
    a, c = _i32(n_nodes), _i32(ctx_len)
    rc = lib().orc_tree_verify_attn(_p(q), _p(k_pool), _p(v_pool), _dtype_code(q), B, H, H_kv, d_h, T_max,
                                    _p(a), _p(c), _p(rows), _p(offs), _p(par),
                                    ctypes.c_double(scale), _p(out))
    _check(rc, "tree_verify_attn")
    return out


def tree_accept(draft, argmax, parent, n_nodes: Sequence[int]):
    """(n_acc [B], path [B][T_max], bonus [B]) int32."""
    d, a, p = _i32(draft), _i32(argmax), _i32(parent)
    B, T_max = d.shape
    assert a.shape == d.shape == p.shape
    n = _i32(n_nodes)
    n_acc = torch.empty(B, dtype=torch.int32)
    path = torch.empty(B, T_max, dtype=torch.int32)
    bonus = torch.empty(B, dtype=torch.int32)
    rc = lib().orc_tree_accept(_p(d), _p(a), _p(p), _p(n), T_max, B, _p(n_acc), _p(path), _p(bonus))
    _check(rc, "tree_accept")
    return n_acc, path, bonus


def chain_draft_len(prob, theta: float, delta: int) -> int:
    """Tokens drafted by one sequence under the early exit (prob: fp32 [delta] or None)."""
    if prob is None:
        rc = lib().orc_chain_draft_len(None, ctypes.c_float(theta), int(delta))
    else:
        pr = torch.as_tensor(prob, dtype=torch.float32).contiguous()
        if pr.numel() != delta:
            raise ValueError("chain_draft_len: one probability per draft position")
        rc = lib().orc_chain_draft_len(_p(pr), ctypes.c_float(theta), int(delta))
    _check(0 if rc >= 0 else rc, "chain_draft_len")
    return int(rc)


def chain_accept(draft, argmax, n_draft: int):
    """(n_acc, next_token) of one sequence; draft[0] is the last accepted token."""
    d, a = _i32(draft), _i32(argmax)
    if d.numel() <= n_draft or a.numel() <= n_draft:
        raise ValueError("chain_accept: arrays shorter than the draft")
    nxt = ctypes.c_int32(0)
    rc = lib().orc_chain_accept(_p(d), _p(a), int(n_draft), ctypes.byref(nxt))
    _check(0 if rc >= 0 else rc, "chain_accept")
    return int(rc), int(nxt.value)


def rbar(M: int, K: int, R: int, K_f: int, L: int) -> int:
    return int(lib().orc_rbar(int(M), int(K), int(R), int(K_f), int(L)))


def kv_commit(pool: torch.Tensor, ctx_len: Sequence[int], n_nodes: Sequence[int], path, n_acc,
              row_off: Optional[Sequence[int]] = None, page_table=None, page_rows: int = 16):
    """Moves the accepted rows of every sequence in place inside `pool` ([rows][...]) and
    returns the new context lengths."""
    assert pool.device.type == "cpu" and pool.is_contiguous()
    row_bytes = pool[0].numel() * pool.element_size()
    p = _i32(path)
    new_len = []
    for b, (c, t) in enumerate(zip(ctx_len, n_nodes)):
        rows, _ = cache_rows([c], [t], None if row_off is None else [row_off[b]],
                             None if page_table is None else [page_table[b]], page_rows)
        pb = p[b].contiguous()
        rc = lib().orc_kv_commit(_p(pool), ctypes.c_size_t(row_bytes), _p(rows), int(rows.numel()), int(c),
                                 _p(pb), int(n_acc[b]), int(t))
        if rc < 0:
            raise ValueError(f"oracle kv_commit: invalid argument (code {rc})")
        new_len.append(rc)
    return new_len


def ttp_score_phead(q: torch.Tensor, gq: torch.Tensor, k: torch.Tensor, gk: torch.Tensor,
                    k_row_off: Sequence[int], gk_row_off: Sequence[int], v_start: int, M: int,
                    scale: float) -> torch.Tensor:
    """scores [B][M] fp64; q, gq [B][H][d_h]; k, gk [rows][H][d_h]."""
    B, H, d_h = q.shape
    assert gq.shape == q.shape and k.shape[1:] == (H, d_h) and gk.shape[1:] == (H, d_h)
    assert q.dtype == gq.dtype == k.dtype == gk.dtype
    out = torch.zeros(B, M, dtype=torch.float64)
    a, b_ = _i64(k_row_off), _i64(gk_row_off)
    rc = lib().orc_ttp_score_phead(_p(q), _p(gq), _p(k), _p(gk), _dtype_code(q), B, H, d_h, _p(a), _p(b_),
                                   int(v_start), int(M), ctypes.c_double(scale), _p(out))
    _check(rc, "ttp_score_phead")
    return out


def draft_topk(probs: torch.Tensor, E: int):
    """(ids [n][E] int32, vals [n][E] fp32), larger first, ties lower index first."""
    assert probs.dtype == torch.float32 and probs.dim() == 2
    n, V = probs.shape
    ids = torch.empty(n, E, dtype=torch.int32)
    vals = torch.empty(n, E, dtype=torch.float32)
    _check(lib().orc_draft_topk(_p(probs.contiguous()), n, V, int(E), _p(ids), _p(vals)), "draft_topk")
    return ids, vals


def draft_topk_logits(logits: torch.Tensor, E: int):
    """(ids [n][E] int32, probs [n][E] fp64) of softmax(logits) per row: larger logit first, ties
    lower index first."""
    assert logits.dtype == torch.float32 and logits.dim() == 2
    n, V = logits.shape
    ids = torch.empty(n, E, dtype=torch.int32)
    probs = torch.empty(n, E, dtype=torch.float64)
    _check(lib().orc_draft_topk_logits(_p(logits.contiguous()), n, V, int(E), _p(ids), _p(probs)),
           "draft_topk_logits")
    return ids, probs


def draft_tree(logits: torch.Tensor, E: int, K: int, D: int):
    """The level-wise drafting loop on a logits table [1 + N][V] (row 0: after the root, row 1 + c: after
    candidate c).  Returns (parent [n] int32, token [n] int32, prob [n] fp64, conf [n] fp64,
    expanded [D-1][K] int32, margin [D-1] fp64)."""
    assert logits.dtype == torch.float32 and logits.dim() == 2
    N = E + (D - 1) * K * E
    V = logits.shape[1]
    if logits.shape[0] != 1 + N or E > V:
        raise ValueError(f"oracle draft_tree: logits must be [1 + {N}][V >= E], got {tuple(logits.shape)}")
    par = torch.empty(N, dtype=torch.int32)
    tok = torch.empty(N, dtype=torch.int32)
    prob = torch.empty(N, dtype=torch.float64)
    conf = torch.empty(N, dtype=torch.float64)
    exp = torch.full((max(D - 1, 1), K), -1, dtype=torch.int32)
    margin = torch.ones(max(D - 1, 1), dtype=torch.float64)
    n = lib().orc_draft_tree(_p(logits.contiguous()), V, int(E), int(K), int(D), _p(par), _p(tok), _p(prob), _p(conf),
                             _p(exp), _p(margin))
    if n < 0:
        raise ValueError(f"oracle draft_tree: invalid argument (code {n})")
    return par[:n], tok[:n], prob[:n], conf[:n], exp[:D - 1], margin[:D - 1]


def tree_confidence(cand_parent: Sequence[int], cand_prob: Sequence[float]) -> torch.Tensor:
    """fp64 confidence (product of draft probabilities along the path) of every candidate."""
    cp = _i32(cand_parent)
    pb = torch.as_tensor(cand_prob, dtype=torch.float32).contiguous()
    conf = torch.empty(cp.numel(), dtype=torch.float64)
    _check(lib().orc_tree_confidence(_p(cp), _p(pb), int(cp.numel()), _p(conf)), "tree_confidence")
    return conf


def tree_build(cand_parent: Sequence[int], cand_token: Sequence[int], cand_prob: Sequence[float],
               root_token: int, T_max: int):
    """(n_nodes, parent [T_max], token [T_max], src [T_max]) for one sequence."""
    cp, ct = _i32(cand_parent), _i32(cand_token)
    pb = torch.as_tensor(cand_prob, dtype=torch.float32).contiguous()
    par = torch.empty(T_max, dtype=torch.int32)
    tok = torch.empty(T_max, dtype=torch.int32)
    src = torch.empty(T_max, dtype=torch.int32)
    n = lib().orc_tree_build(_p(cp), _p(ct), _p(pb), int(cp.numel()), int(root_token), int(T_max), _p(par),
                             _p(tok), _p(src))
    if n < 0:
        raise ValueError(f"oracle tree_build: invalid argument (code {n})")
    return int(n), par, tok, src
