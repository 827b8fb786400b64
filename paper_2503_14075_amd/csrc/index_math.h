// Index arithmetic of the kernels on values that come from device memory and
// cannot be checked on the host (lengths, offsets, page ids, tree sizes, kept
// indices, accepted paths).  Every function maps arbitrary 32-bit contents to
// row numbers inside the buffers that the call's host arguments describe, so a
// violated precondition gives an unspecified result but never an access
// outside them.  Plain C++ without any HIP type: the same source is compiled
// into the kernels and into a host program that sweeps hostile values.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define TW_HD __host__ __device__ __forceinline__
#else
#define TW_HD inline
#endif

namespace tw {

TW_HD int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }
TW_HD int64_t clampl(int64_t x, int64_t lo, int64_t hi) { return x < lo ? lo : (x > hi ? hi : x); }

// --- tree verification ----------------------------------------------------------------------------
// Tree size T, context length C and the cache rows [r_begin, r_end) of split `split` of a sequence.
// A split is split_rows rows long (a positive multiple of 32 with n_splits * split_rows >= max_rows);
// a sequence of n_rows = C + T rows has n_b = ceil(n_rows / split_rows) non-empty splits, the later
// ones are empty (r_begin == r_end).  max_rows = max_ctx_len + T_max on the host, so C + T <= max_rows.
struct SeqInfo {
    int T, C, n_rows, n_b, r_begin, r_end;
};
TW_HD SeqInfo seq_info_from(int n_nodes_raw, int ctx_len_raw, int T_max, int max_rows, int split_rows,
                            int n_splits, int split) {
    SeqInfo s;
    s.T = clampi(n_nodes_raw, 1, T_max);
    s.C = clampi(ctx_len_raw, 0, max_rows - T_max);
    s.n_rows = s.C + s.T;
    s.n_b = clampi((int)(((int64_t)s.n_rows + split_rows - 1) / split_rows), 1, n_splits);
    const int64_t rb = (int64_t)split * split_rows;
    s.r_begin = rb < s.n_rows ? (int)rb : s.n_rows;
    const int64_t re = (int64_t)s.r_begin + split_rows;
    s.r_end = re < s.n_rows ? (int)re : s.n_rows;
    return s;
}

// Parent of tree node i > 0 from unchecked contents: some node before i.
TW_HD int clamp_parent(int p, int i) { return p < 0 ? 0 : (p >= i ? i - 1 : p); }

// --- key/value pools ------------------------------------------------------------------------------
// Contiguous view: first pool row of a sequence, and how many rows past it stay inside the pool.
TW_HD int64_t seq_first_row(int row_off_raw, int64_t pool_rows) { return clampl(row_off_raw, 0, pool_rows - 1); }
// Contiguous view, streaming kernels: the last cache row a workgroup may touch (its piece's last row,
// cut off at the end of the pool), and the cache row of row r of the chunk that starts at `base`
// (loads past the last row read it again), 0 <= result <= last_row.
TW_HD int seq_last_row(int last, int64_t first_row, int64_t pool_rows) {
    const int64_t room = pool_rows - 1 - first_row;
    const int l = last < room ? last : (int)room;
    return l < 0 ? 0 : l;
}
TW_HD int chunk_start(int base, int last_row) { return base < last_row ? (base < 0 ? 0 : base) : last_row; }
TW_HD int chunk_row_offset(int r, int start, int last_row) {
    const int lim = last_row - start;
    return r < lim ? (r < 0 ? 0 : r) : lim;
}
// Paged view: page-table slot of cache row r (r >= 0), and the pool row of (page id, r).
TW_HD int page_slot(int r, int page_rows, int page_shift, int max_pages) {
    const int pi = page_shift >= 0 ? r >> page_shift : r / page_rows;
    return pi < max_pages ? pi : max_pages - 1;
}
TW_HD int64_t paged_pool_row(int page_id_raw, int r, int page_rows, int page_shift, int64_t pool_rows) {
    const int slot = page_shift >= 0 ? r & (page_rows - 1) : r % page_rows;
    return clampl((int64_t)page_id_raw * page_rows + slot, 0, pool_rows - 1);
}
// Pool row of cache row r of a contiguous sequence.
TW_HD int64_t contiguous_pool_row(int row_off_raw, int r, int64_t pool_rows) {
    return clampl((int64_t)row_off_raw + r, 0, pool_rows - 1);
}

// --- compaction -----------------------------------------------------------------------------------
// Length of a sequence for the compaction: between the end of the visual span and the host's bound.
TW_HD int compact_n_tot(int n_tot_raw, int v_start, int M, int n_tot_max) {
    return clampi(n_tot_raw, v_start + M, n_tot_max);
}
// Source row of destination row r (0 <= r < n_tot - M + R) given the kept index read for it
// (kept_raw is only used for v_start <= r < v_start + R); inside [0, n_tot).
TW_HD int compact_src_row_from(int kept_raw, int R, int v_start, int M, int n_tot, int r) {
    int sr;
    if (r < v_start) sr = r;
    else if (r < v_start + R) sr = v_start + clampi(kept_raw, 0, M - 1);
    else sr = r - R + M;
    return sr < n_tot ? sr : n_tot - 1;
}

// --- commit of the accepted path -------------------------------------------------------------------
// Number of accepted nodes and the context length, held where C + T_max cannot wrap.
TW_HD int commit_n_acc(int n_acc_raw, int T_max) { return clampi(n_acc_raw, 0, T_max - 1); }
TW_HD int commit_ctx(int ctx_raw) { return clampi(ctx_raw, 0, 1 << 30); }
// Tree node whose row moves to the next slot of the accepted path, given the previous one (0 before
// the first): strictly increasing and inside the tree whatever the contents, so that a move never
// writes a row that a later move reads.
TW_HD int commit_next_node(int prev, int path_raw, int T_max) {
    const int p = path_raw <= prev ? prev + 1 : path_raw;
    return p > T_max - 1 ? T_max - 1 : p;
}
// Tree size of a sequence for the integer kernels (ancestor masks, acceptance walk).
TW_HD int tree_nodes(int n_nodes_raw, int T_max) { return clampi(n_nodes_raw, 1, T_max); }
// Candidates of a drafted tree: their number inside [0, N]; the next step of a walk from candidate
// u towards the root: an earlier candidate, or -1 (a child of the root; also what a parent entry
// that does not precede u is taken for), so every walk ends after at most u + 1 steps.
TW_HD int cand_count(int n_cand_raw, int N) { return clampi(n_cand_raw, 0, N); }
TW_HD int cand_walk_parent(int parent_raw, int u) { return parent_raw < u ? (parent_raw < 0 ? -1 : parent_raw) : -1; }
// The node that a level of the drafting loop expands: entry `sel_raw` of the previous level's slice
// [prev_off, out_off) of the candidate arrays (out_off > prev_off >= 0).
TW_HD int expand_parent(int sel_raw, int prev_off, int out_off) {
    return prev_off + clampi(sel_raw, 0, out_off - prev_off - 1);
}
// Kept candidate number r of the select, inside [0, N).
TW_HD int kept_candidate(int kept_raw, int N) { return clampi(kept_raw, 0, N - 1); }

// --- pruning score ----------------------------------------------------------------------------------
// Scoring rows, prompt length and first scoring position of a sequence: 0 <= n_q <= n_q_max rows of
// this launch's window [row0, row0 + n_q_max) of the q_rows rows that q_sel holds per sequence,
// 0 <= n_tot <= n_tot_max, and a first position for which pos0 + (row index < 2 * n_q_max) cannot wrap.
struct ScoreSeq {
    int n_q, n_tot, pos0;
};
TW_HD ScoreSeq score_seq_from(int n_q_raw, int n_tot_raw, int q_pos0_raw, int q_rows, int row0, int n_q_max,
                              int n_tot_max) {
    ScoreSeq s;
    const int n_all = clampi(n_q_raw, 1, q_rows);
    s.n_q = clampi(n_all - row0, 0, n_q_max);
    s.n_tot = clampi(n_tot_raw, 0, n_tot_max);
    s.pos0 = clampi(q_pos0_raw, 0, n_tot_max) + row0;
    return s;
}

}  // namespace tw
