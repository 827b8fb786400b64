"""Thin ctypes binding of libtwigpath.so: one Python function per C-ABI entry
point, same names without the tw_ prefix.  Argument marshalling only -- every
step of the path runs in the HIP kernels.  torch provides device memory and
the current stream, nothing else.

Importing this module loads the library and raises if it has not been built
(`python -m paper_2503_14075_amd.build`); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TWIGPATH_LIB names another build of the same library (the diagnostic build of build.py --trace)
LIB_PATH = os.environ.get("TWIGPATH_LIB") or os.path.join(_HERE, "libtwigpath.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_14075_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)

TW_OK, TW_ERR_INVALID_ARG, TW_ERR_UNSUPPORTED, TW_ERR_WORKSPACE, TW_ERR_LAUNCH = 0, -1, -2, -3, -4
TW_F32, TW_BF16 = 0, 1
TW_CALL_TTP_SCORE, TW_CALL_TREE_VERIFY_ATTN = 1, 2
TW_STATIC_SCRATCH_BYTES = 16 << 20
_STATUS = {0: "TW_OK", -1: "TW_ERR_INVALID_ARG", -2: "TW_ERR_UNSUPPORTED", -3: "TW_ERR_WORKSPACE",
           -4: "TW_ERR_LAUNCH"}

EXPORTS = ["tw_version", "tw_workspace_bytes", "tw_ttp_score", "tw_ttp_score_gqa", "tw_ttp_score_select", "tw_ttp_score_phead", "tw_ttp_select", "tw_ttp_compact",
           "tw_ttp_compact_batched",
           "tw_tree_ancestor_masks", "tw_tree_verify_attn", "tw_tree_verify_attn_gqa", "tw_tree_verify_attn_static", "tw_tree_accept", "tw_chain_tree", "tw_chain_accept", "tw_kv_commit", "tw_draft_topk", "tw_draft_topk_logits", "tw_draft_expand",
           "tw_tree_build_workspace_bytes", "tw_tree_build", "tw_validate_tree",
           "tw_rbar"]


class KvView(ctypes.Structure):
    _fields_ = [("base", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("H", ctypes.c_int32),
                ("d_h", ctypes.c_int32), ("pool_rows", ctypes.c_int64), ("row_off", ctypes.c_void_p),
                ("page_table", ctypes.c_void_p), ("max_pages", ctypes.c_int32),
                ("page_rows", ctypes.c_int32)]


_vp, _i32, _i64, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
_lib.tw_version.restype = _i32
_lib.tw_workspace_bytes.restype = _sz
_lib.tw_workspace_bytes.argtypes = [_i32] * 6
_lib.tw_ttp_score.restype = _i32
_lib.tw_ttp_score.argtypes = [_vp, _i32, _vp, _vp, ctypes.POINTER(KvView), _vp, _i32, _i32, _i32, _i32,
                              _f32, _i32, _vp, _vp, _sz, _vp]
_lib.tw_ttp_score_gqa.restype = _i32
_lib.tw_ttp_score_gqa.argtypes = [_vp, _i32, _vp, _vp, ctypes.POINTER(KvView), _i32, _vp, _i32, _i32, _i32, _i32,
                                  _f32, _i32, _vp, _vp, _sz, _vp]
_lib.tw_ttp_score_select.restype = _i32
_lib.tw_ttp_score_select.argtypes = [_vp, _i32, _vp, _vp, ctypes.POINTER(KvView), _vp, _i32, _i32, _i32, _i32,
                                     _f32, _i32, _vp, _i32, _vp, _vp, _sz, _vp]
_lib.tw_ttp_score_phead.restype = _i32
_lib.tw_ttp_score_phead.argtypes = [_vp, _vp, ctypes.POINTER(KvView), ctypes.POINTER(KvView), _i32, _i32, _i32,
                                    _f32, _vp, _vp, _sz, _vp]
_lib.tw_ttp_select.restype = _i32
_lib.tw_ttp_select.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp]
_lib.tw_ttp_compact.restype = _i32
_lib.tw_ttp_compact.argtypes = [_vp, _i32, _i32, _i32, _i32, ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                _i32, _sz, _vp]
_lib.tw_ttp_compact_batched.restype = _i32
_lib.tw_ttp_compact_batched.argtypes = [_vp, _i32, _i32, _i32, _vp, _i32, _vp, _vp, _i32,
                                        ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i32, _sz, _vp]
_lib.tw_tree_ancestor_masks.restype = _i32
_lib.tw_tree_ancestor_masks.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp]
_lib.tw_tree_verify_attn.restype = _i32
_lib.tw_tree_verify_attn.argtypes = [_vp, ctypes.POINTER(KvView), ctypes.POINTER(KvView), _vp, _i32, _vp,
                                     _vp, _i32, _i32, _f32, _vp, _i32, _vp, _sz, _vp]
_lib.tw_tree_verify_attn_gqa.restype = _i32
_lib.tw_tree_verify_attn_gqa.argtypes = [_vp, ctypes.POINTER(KvView), ctypes.POINTER(KvView), _i32, _vp, _i32, _vp,
                                         _vp, _i32, _i32, _f32, _vp, _i32, _vp, _sz, _vp]
_lib.tw_tree_verify_attn_static.restype = _i32
_lib.tw_tree_verify_attn_static.argtypes = [_vp, ctypes.POINTER(KvView), ctypes.POINTER(KvView), _vp, _i32, _vp,
                                            _vp, _i32, _i32, _f32, _vp, _i32, _vp]
_lib.tw_tree_accept.restype = _i32
_lib.tw_tree_accept.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.tw_chain_tree.restype = _i32
_lib.tw_chain_tree.argtypes = [_vp, _f32, _i32, _i32, _vp, _vp, _vp]
_lib.tw_chain_accept.restype = _i32
_lib.tw_chain_accept.argtypes = [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.tw_kv_commit.restype = _i32
_lib.tw_kv_commit.argtypes = [_vp, _vp, _i32, ctypes.POINTER(KvView), _i32, _vp, _i32, _vp, _vp]
_lib.tw_draft_topk.restype = _i32
_lib.tw_draft_topk.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.tw_draft_topk_logits.restype = _i32
_lib.tw_draft_topk_logits.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.tw_draft_expand.restype = _i32
_lib.tw_draft_expand.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.tw_tree_build_workspace_bytes.restype = _sz
_lib.tw_tree_build_workspace_bytes.argtypes = [_i32, _i32, _i32]
_lib.tw_tree_build.restype = _i32
_lib.tw_tree_build.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.tw_validate_tree.restype = _i32
_lib.tw_validate_tree.argtypes = [ctypes.POINTER(_i32), _i32]
_lib.tw_rbar.restype = _i32
_lib.tw_rbar.argtypes = [_i32] * 5


class TwigError(RuntimeError):
    def __init__(self, call: str, status: int):
        super().__init__(f"{call} returned {_STATUS.get(status, status)}")
        self.status = status


def _check(call: str, status: int) -> None:
    if status != TW_OK:
        raise TwigError(call, status)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors passed to twigpath must be contiguous")
    return t.data_ptr()


def _stream() -> Optional[int]:
    return torch.cuda.current_stream().cuda_stream or None


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TW_F32
    if t.dtype == torch.bfloat16:
        return TW_BF16
    raise TwigError("dtype", TW_ERR_UNSUPPORTED)


def kv_view(pool: torch.Tensor, row_off: Optional[torch.Tensor] = None,
            page_table: Optional[torch.Tensor] = None, page_rows: int = 0) -> KvView:
    """pool [rows][H][d_h]; row_off int32 [B] (contiguous) or page_table int32 [B][max_pages]."""
    rows, H, d_h = pool.shape
    view = KvView(_ptr(pool), _dtype_code(pool), H, d_h, rows, _ptr(row_off), _ptr(page_table),
                  0 if page_table is None else page_table.shape[1], page_rows)
    view._keep = (pool, row_off, page_table)   # the struct holds raw pointers: keep their tensors alive with it
    return view


def version() -> int:
    return int(_lib.tw_version())


def workspace_bytes(which: int, B: int, rows: int, H: int, d_h: int, max_rows: int) -> int:
    return int(_lib.tw_workspace_bytes(which, B, rows, H, d_h, max_rows))


def ttp_score(q_sel: torch.Tensor, k: KvView, n_q: Optional[torch.Tensor], q_pos0: torch.Tensor,
              n_tot: torch.Tensor, n_tot_max: int, v_start: int, M: int, scale: float, causal: bool,
              scores: torch.Tensor, ws: Optional[torch.Tensor]) -> None:
    B, n_q_max = q_sel.shape[0], q_sel.shape[1]
    _check("tw_ttp_score", _lib.tw_ttp_score(
        _ptr(q_sel), n_q_max, _ptr(n_q), _ptr(q_pos0), ctypes.byref(k), _ptr(n_tot), n_tot_max, B,
        v_start, M, scale, int(causal), _ptr(scores), _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def ttp_score_select(q_sel: torch.Tensor, k: KvView, n_q: Optional[torch.Tensor], q_pos0: torch.Tensor,
                     n_tot: torch.Tensor, n_tot_max: int, v_start: int, M: int, scale: float, causal: bool,
                     scores: torch.Tensor, R: int, kept: torch.Tensor, ws: Optional[torch.Tensor]) -> None:
    B, n_q_max = q_sel.shape[0], q_sel.shape[1]
    _check("tw_ttp_score_select", _lib.tw_ttp_score_select(
        _ptr(q_sel), n_q_max, _ptr(n_q), _ptr(q_pos0), ctypes.byref(k), _ptr(n_tot), n_tot_max, B,
        v_start, M, scale, int(causal), _ptr(scores), R, _ptr(kept), _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def ttp_score_gqa(q_sel: torch.Tensor, k: KvView, q_heads_per_kv: int, n_q: Optional[torch.Tensor],
                  q_pos0: torch.Tensor, n_tot: torch.Tensor, n_tot_max: int, v_start: int, M: int, scale: float,
                  causal: bool, scores: torch.Tensor, ws: Optional[torch.Tensor]) -> None:
    B, n_q_max = q_sel.shape[0], q_sel.shape[1]
    _check("tw_ttp_score_gqa", _lib.tw_ttp_score_gqa(
        _ptr(q_sel), n_q_max, _ptr(n_q), _ptr(q_pos0), ctypes.byref(k), q_heads_per_kv, _ptr(n_tot), n_tot_max, B,
        v_start, M, scale, int(causal), _ptr(scores), _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def ttp_score_phead(q: torch.Tensor, gq: torch.Tensor, k: KvView, gk: KvView, v_start: int, M: int,
                    scale: float, scores: torch.Tensor, ws: torch.Tensor) -> None:
    _check("tw_ttp_score_phead", _lib.tw_ttp_score_phead(
        _ptr(q), _ptr(gq), ctypes.byref(k), ctypes.byref(gk), q.shape[0], v_start, M, scale, _ptr(scores),
        _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def ttp_select(scores: torch.Tensor, R: int, kept: torch.Tensor) -> None:
    B, M = scores.shape
    _check("tw_ttp_select", _lib.tw_ttp_select(_ptr(scores), B, M, R, _ptr(kept), _stream()))


def ttp_compact(kept: Optional[torch.Tensor], R: int, v_start: int, M: int, n_tot: int,
                src: Sequence[torch.Tensor], dst: Sequence[torch.Tensor], row_bytes: int) -> None:
    n = len(src)
    s_arr = (_vp * max(n, 1))(*[_ptr(t) for t in src])
    d_arr = (_vp * max(n, 1))(*[_ptr(t) for t in dst])
    _check("tw_ttp_compact", _lib.tw_ttp_compact(_ptr(kept), R, v_start, M, n_tot, s_arr, d_arr, n,
                                                 row_bytes, _stream()))


def ttp_compact_batched(kept: torch.Tensor, R: int, v_start: int, M: int, n_tot: torch.Tensor,
                        n_tot_max: int, src_row_off: torch.Tensor, dst_row_off: torch.Tensor,
                        src: Sequence[torch.Tensor], dst: Sequence[torch.Tensor], row_bytes: int) -> None:
    n, B = len(src), n_tot.numel()
    s_arr = (_vp * max(n, 1))(*[_ptr(t) for t in src])
    d_arr = (_vp * max(n, 1))(*[_ptr(t) for t in dst])
    _check("tw_ttp_compact_batched", _lib.tw_ttp_compact_batched(
        _ptr(kept), R, v_start, M, _ptr(n_tot), n_tot_max, _ptr(src_row_off), _ptr(dst_row_off), B,
        s_arr, d_arr, n, row_bytes, _stream()))


def tree_ancestor_masks(parent: torch.Tensor, n_nodes: torch.Tensor, masks: torch.Tensor) -> None:
    B, T_max = parent.shape
    _check("tw_tree_ancestor_masks", _lib.tw_tree_ancestor_masks(_ptr(parent), _ptr(n_nodes), T_max, B,
                                                                 _ptr(masks), _stream()))


def tree_verify_attn(q: torch.Tensor, k: KvView, v: KvView, ctx_len: torch.Tensor, max_ctx_len: int,
                     parent: torch.Tensor, n_nodes: torch.Tensor, scale: float, out: torch.Tensor,
                     ws: Optional[torch.Tensor]) -> None:
    B, T_max = q.shape[0], q.shape[1]
    _check("tw_tree_verify_attn", _lib.tw_tree_verify_attn(
        _ptr(q), ctypes.byref(k), ctypes.byref(v), _ptr(ctx_len), max_ctx_len, _ptr(parent),
        _ptr(n_nodes), T_max, B, scale, _ptr(out), _dtype_code(out), _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def tree_verify_attn_static(q: torch.Tensor, k: KvView, v: KvView, ctx_len: torch.Tensor, max_ctx_len: int,
                            parent: torch.Tensor, n_nodes: torch.Tensor, scale: float, out: torch.Tensor) -> None:
    B, T_max = q.shape[0], q.shape[1]
    _check("tw_tree_verify_attn_static", _lib.tw_tree_verify_attn_static(
        _ptr(q), ctypes.byref(k), ctypes.byref(v), _ptr(ctx_len), max_ctx_len, _ptr(parent),
        _ptr(n_nodes), T_max, B, scale, _ptr(out), _dtype_code(out), _stream()))


def tree_verify_attn_gqa(q: torch.Tensor, k: KvView, v: KvView, q_heads_per_kv: int, ctx_len: torch.Tensor,
                         max_ctx_len: int, parent: torch.Tensor, n_nodes: torch.Tensor, scale: float,
                         out: torch.Tensor, ws: Optional[torch.Tensor]) -> None:
    B, T_max = q.shape[0], q.shape[1]
    _check("tw_tree_verify_attn_gqa", _lib.tw_tree_verify_attn_gqa(
        _ptr(q), ctypes.byref(k), ctypes.byref(v), q_heads_per_kv, _ptr(ctx_len), max_ctx_len, _ptr(parent),
        _ptr(n_nodes), T_max, B, scale, _ptr(out), _dtype_code(out), _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def tree_accept(draft: torch.Tensor, argmax: torch.Tensor, parent: torch.Tensor, n_nodes: torch.Tensor,
                n_acc: torch.Tensor, path: torch.Tensor, bonus: torch.Tensor) -> None:
    B, T_max = draft.shape
    _check("tw_tree_accept", _lib.tw_tree_accept(_ptr(draft), _ptr(argmax), _ptr(parent), _ptr(n_nodes),
                                                 T_max, B, _ptr(n_acc), _ptr(path), _ptr(bonus),
                                                 _stream()))


def chain_tree(prob: Optional[torch.Tensor], theta: float, delta: int, parent: torch.Tensor,
               n_nodes: torch.Tensor) -> None:
    B = n_nodes.shape[0]
    _check("tw_chain_tree", _lib.tw_chain_tree(_ptr(prob), theta, delta, B, _ptr(parent), _ptr(n_nodes), _stream()))


def chain_accept(draft: torch.Tensor, argmax: torch.Tensor, n_nodes: torch.Tensor, n_acc: torch.Tensor,
                 path: torch.Tensor, bonus: torch.Tensor) -> None:
    B, T_max = draft.shape
    _check("tw_chain_accept", _lib.tw_chain_accept(_ptr(draft), _ptr(argmax), _ptr(n_nodes), T_max, B,
                                                   _ptr(n_acc), _ptr(path), _ptr(bonus), _stream()))


def kv_commit(path: torch.Tensor, n_acc: torch.Tensor, views: Sequence[KvView], ctx_len: torch.Tensor,
              new_ctx_len: Optional[torch.Tensor]) -> None:
    B, T_max = path.shape
    arr = (KvView * max(len(views), 1))(*views)
    _check("tw_kv_commit", _lib.tw_kv_commit(_ptr(path), _ptr(n_acc), T_max, arr, len(views), _ptr(ctx_len),
                                             B, _ptr(new_ctx_len), _stream()))


def draft_topk(probs: torch.Tensor, E: int, ids: torch.Tensor, vals: torch.Tensor) -> None:
    n, V = probs.shape
    _check("tw_draft_topk", _lib.tw_draft_topk(_ptr(probs), n, V, E, _ptr(ids), _ptr(vals), _stream()))


def draft_topk_logits(logits: torch.Tensor, E: int, ids: torch.Tensor, probs: torch.Tensor) -> None:
    n, V = logits.shape
    _check("tw_draft_topk_logits",
           _lib.tw_draft_topk_logits(_ptr(logits), n, V, E, _ptr(ids), _ptr(probs), _stream()))


def draft_expand(sel: Optional[torch.Tensor], prev_off: int, out_off: int, ids: torch.Tensor, probs: torch.Tensor,
                 cand_parent: torch.Tensor, cand_token: torch.Tensor, cand_prob: torch.Tensor,
                 cand_conf: torch.Tensor, level_conf: torch.Tensor) -> None:
    B, n_exp, E = ids.shape
    _check("tw_draft_expand", _lib.tw_draft_expand(
        _ptr(sel), n_exp, prev_off, out_off, _ptr(ids), _ptr(probs), E, cand_parent.shape[1], B, _ptr(cand_parent),
        _ptr(cand_token), _ptr(cand_prob), _ptr(cand_conf), _ptr(level_conf), _stream()))


def tree_build_workspace_bytes(B: int, N: int, T_max: int) -> int:
    return int(_lib.tw_tree_build_workspace_bytes(B, N, T_max))


def tree_build(cand_parent: torch.Tensor, cand_token: torch.Tensor, cand_prob: torch.Tensor,
               n_cand: torch.Tensor, root_token: torch.Tensor, T_max: int, parent_out: torch.Tensor,
               token_out: torch.Tensor, src_out: torch.Tensor, n_nodes_out: torch.Tensor,
               ws: Optional[torch.Tensor]) -> None:
    B, N = cand_parent.shape
    _check("tw_tree_build", _lib.tw_tree_build(
        _ptr(cand_parent), _ptr(cand_token), _ptr(cand_prob), _ptr(n_cand), _ptr(root_token), N, B, T_max,
        _ptr(parent_out), _ptr(token_out), _ptr(src_out), _ptr(n_nodes_out), _ptr(ws),
        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def validate_tree(parent: Sequence[int]) -> int:
    arr = (_i32 * max(len(parent), 1))(*parent)
    return int(_lib.tw_validate_tree(arr, len(parent)))


def rbar(M: int, K: int, R: int, K_f: int, L: int) -> int:
    return int(_lib.tw_rbar(M, K, R, K_f, L))


def raw():
    """The ctypes library handle (error-path tests call entry points with hand-made arguments)."""
    return _lib
