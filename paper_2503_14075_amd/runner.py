"""Device-side staging of a synthetic Workload and one-call-per-step drivers.

This is plumbing for the tests and the benchmark: it places the generated
tensors in HBM, allocates outputs and workspaces with torch, and calls the
library through `binding`.  No step of the method is computed here.
"""
from __future__ import annotations

from typing import List, Optional

import torch

from . import binding as tw
from .workloads import Workload


def _i32(xs, device) -> torch.Tensor:
    return torch.tensor(xs, dtype=torch.int32, device=device)


class DeviceWorkload:
    def __init__(self, w: Workload, device="cuda:0"):
        cfg = w.cfg
        self.w, self.cfg, self.device = w, cfg, device
        dev = device
        B, L, T, H, d_h = cfg.B, cfg.L, cfg.T, cfg.H, cfg.d_h
        self.B, self.n_inst = B, B * L
        # ---- pruning side -------------------------------------------------------
        self.q_sel = w.q_sel.to(dev)
        self.k_score = w.k_score.to(dev)
        self.has_score = self.k_score.numel() > 0
        self.n_q = _i32(w.n_q, dev)
        self.q_pos0 = _i32(w.q_pos0, dev)
        self.n_tot = _i32(w.n_tot, dev)
        self.n_tot_max = max(w.n_tot)
        self.score_row_off = _i32(w.score_row_off, dev)
        self.scores = torch.zeros(B, cfg.M, dtype=torch.float32, device=dev)
        self.kept = torch.zeros(B, cfg.R, dtype=torch.int32, device=dev)
        if self.has_score:
            self.k_score_view = tw.kv_view(self.k_score, row_off=self.score_row_off)
            nbytes = tw.workspace_bytes(tw.TW_CALL_TTP_SCORE, B, w.n_q_max, H, d_h, self.n_tot_max)
            self.score_ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device=dev)
        self.compact_src = [t.to(dev) for t in w.compact_src]
        n_keep_total = sum(cfg.R + n for n in w.n_text)
        self.compact_dst = [torch.empty((n_keep_total,) + tuple(t.shape[1:]), dtype=t.dtype, device=dev)
                            for t in self.compact_src]
        self.compact_dst_off = _i32(w.compact_dst_off, dev)
        # ---- verification side --------------------------------------------------
        self.q_tree = w.q_tree.to(dev)
        self.k_pool = w.k_pool.to(dev)
        self.v_pool = w.v_pool.to(dev)
        self.ctx_len = _i32(w.ctx_len, dev)
        self.max_ctx_len = max(w.ctx_len)
        self.n_nodes = _i32(w.n_nodes, dev)
        self.parent = _i32(w.parent, dev)
        self.row_off = None if w.row_off is None else _i32(w.row_off, dev)
        self.page_table = None if w.page_table is None else _i32(w.page_table, dev)
        self.k_view = tw.kv_view(self.k_pool, self.row_off, self.page_table, cfg.page_rows)
        self.v_view = tw.kv_view(self.v_pool, self.row_off, self.page_table, cfg.page_rows)
        self.out = torch.zeros(self.n_inst, T, H, d_h, dtype=torch.float32, device=dev)
        nbytes = tw.workspace_bytes(tw.TW_CALL_TREE_VERIFY_ATTN, self.n_inst, T, H, d_h,
                                    self.max_ctx_len + T)
        # zeroed once: the arrival counters at its start must be zero before the first call and are left zero by every call
        self.verify_ws = torch.zeros(max(nbytes, 4) // 4, dtype=torch.float32, device=dev) if nbytes else None
        # ---- acceptance -----------------------------------------------------------
        self.draft = _i32(w.draft, dev)
        self.argmax = _i32(w.argmax, dev)
        self.tree_seq = _i32(w.tree_seq, dev)
        self.n_nodes_seq = _i32([T] * B, dev)
        self.n_acc = torch.zeros(B, dtype=torch.int32, device=dev)
        self.path = torch.zeros(B, T, dtype=torch.int32, device=dev)
        self.bonus = torch.zeros(B, dtype=torch.int32, device=dev)

    # one call per step of the path ------------------------------------------------
    def run_score(self) -> None:
        cfg = self.cfg
        tw.ttp_score(self.q_sel, self.k_score_view, self.n_q, self.q_pos0, self.n_tot, self.n_tot_max,
                     0, cfg.M, cfg.scale, True, self.scores, self.score_ws)

    def run_score_select(self) -> None:
        """Score and top-R keep in one call (the head reduction and the select share a launch)."""
        cfg = self.cfg
        tw.ttp_score_select(self.q_sel, self.k_score_view, self.n_q, self.q_pos0, self.n_tot, self.n_tot_max,
                            0, cfg.M, cfg.scale, True, self.scores, cfg.R, self.kept, self.score_ws)

    def run_select(self) -> None:
        tw.ttp_select(self.scores, self.cfg.R, self.kept)

    def run_compact(self) -> None:
        cfg = self.cfg
        # hidden rows and KV rows may differ in width: one batched call per row width
        groups = {}
        for s, d in zip(self.compact_src, self.compact_dst):
            groups.setdefault(s[0].numel() * s.element_size(), []).append((s, d))
        for row_bytes, pairs in groups.items():
            tw.ttp_compact_batched(self.kept, cfg.R, 0, cfg.M, self.n_tot, self.n_tot_max,
                                   self.score_row_off, self.compact_dst_off, [p[0] for p in pairs],
                                   [p[1] for p in pairs], row_bytes)

    def run_verify(self) -> None:
        tw.tree_verify_attn(self.q_tree, self.k_view, self.v_view, self.ctx_len, self.max_ctx_len,
                            self.parent, self.n_nodes, self.cfg.scale, self.out, self.verify_ws)

    def run_accept(self) -> None:
        tw.tree_accept(self.draft, self.argmax, self.tree_seq, self.n_nodes_seq, self.n_acc, self.path,
                       self.bonus)

    def step(self) -> None:
        """One pass of the whole path: score -> select -> compact -> verify -> accept."""
        if self.has_score:
            self.run_score_select()
        else:
            self.run_select()
        if self.compact_src:
            self.run_compact()
        self.run_verify()
        self.run_accept()

    def step_two_streams(self, side: torch.cuda.Stream) -> None:
        """The same pass with its two independent chains on two streams: verify -> accept on `side`,
        score -> select -> compact on the current stream, which waits for `side` at the end.  The
        chains share no buffer (each has its own workspace)."""
        cur = torch.cuda.current_stream()
        side.wait_stream(cur)
        with torch.cuda.stream(side):
            self.run_verify()
            self.run_accept()
        if self.has_score:
            self.run_score_select()
        else:
            self.run_select()
        if self.compact_src:
            self.run_compact()
        cur.wait_stream(side)
