// Host-side sweep of the kernels' index arithmetic (index_math.h) over hostile device contents:
// every row or slot number it produces must lie inside the buffers that the host arguments
// describe, and no step may overflow (built with -fsanitize=address,undefined by its test).
#include <cassert>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "index_math.h"

using namespace tw;

#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); \
            std::exit(1);                                                         \
        }                                                                         \
    } while (0)

static const int kHostile[] = {INT32_MIN, INT32_MIN + 1, -(1 << 30), -100000, -65, -64, -2, -1, 0, 1, 2, 5, 25, 31, 32,
                               33, 63, 64, 65, 255, 256, 257, 1000, 4095, 4096, 1 << 20, (1 << 30) - 1, 1 << 30,
                               (1 << 30) + 1, INT32_MAX - 1, INT32_MAX};

static void sweep_seq_info() {
    for (int T_max : {1, 2, 26, 32, 33, 64})
        for (int max_ctx : {0, 1, 31, 255, 256, 4097, 100000, (1 << 30) - 64}) {
            const int max_rows = max_ctx + T_max;
            for (int want : {1, 2, 3, 7, 64}) {
                // the host's plan: pieces of whole 32-row chunks, as few as cover the longest sequence
                const int per = (max_rows + want - 1) / want;
                const int split_rows = (per + 31) / 32 * 32;
                const int n_splits = (int)(((int64_t)max_rows + split_rows - 1) / split_rows);
                CHECK(split_rows >= 32 && (int64_t)n_splits * split_rows >= max_rows);
                for (int nn : kHostile)
                    for (int cc : kHostile) {
                        int covered = 0, n_b = -1;
                        for (int s = 0; s < n_splits; ++s) {
                            const SeqInfo q = seq_info_from(nn, cc, T_max, max_rows, split_rows, n_splits, s);
                            CHECK(q.T >= 1 && q.T <= T_max && q.C >= 0 && q.C + q.T == q.n_rows && q.n_rows <= max_rows);
                            CHECK(q.n_b >= 1 && q.n_b <= n_splits);
                            CHECK(n_b < 0 || n_b == q.n_b);
                            n_b = q.n_b;
                            CHECK(q.r_begin >= 0 && q.r_begin <= q.r_end && q.r_end <= q.n_rows);
                            CHECK(q.r_begin == covered || q.r_begin == q.n_rows);   // consecutive pieces
                            if (s < q.n_b) CHECK(q.r_end > q.r_begin);              // pieces that are counted are not empty
                            else CHECK(q.r_end == q.r_begin);
                            covered = q.r_end;
                            if (s == n_splits - 1) CHECK(covered == q.n_rows);
                        }
                    }
            }
        }
}

static void sweep_pool_rows() {
    for (int64_t pool_rows : {(int64_t)1, (int64_t)17, (int64_t)4096, (int64_t)INT32_MAX, (int64_t)5 << 30})
        for (int off : kHostile) {
            const int64_t first = seq_first_row(off, pool_rows);
            CHECK(first >= 0 && first < pool_rows);
            for (int last : kHostile) {
                const int last_row = seq_last_row(last, first, pool_rows);
                CHECK(last_row >= 0 && first + last_row < pool_rows);
                for (int base : kHostile) {
                    const int start = chunk_start(base, last_row);
                    CHECK(start >= 0 && start <= last_row);
                    for (int r : {INT32_MIN, -1, 0, 1, 31, 32, INT32_MAX}) {
                        const int ro = chunk_row_offset(r, start, last_row);
                        CHECK(ro >= 0 && start + ro <= last_row);
                    }
                }
            }
            for (int r : kHostile) {
                if (r < 0) continue;   // callers pass rows >= 0 (pool_row clamps before)
                const int64_t row = contiguous_pool_row(off, r, pool_rows);
                CHECK(row >= 0 && row < pool_rows);
            }
        }
    for (int page_rows : {1, 3, 16, 64, 1000})
        for (int max_pages : {1, 2, 47, 1 << 20}) {
            int shift = -1;
            for (int sh = 0; sh < 31; ++sh)
                if (page_rows == (1 << sh)) shift = sh;
            for (int64_t pool_rows : {(int64_t)page_rows, (int64_t)page_rows * 47, (int64_t)5 << 30})
                for (int r : kHostile) {
                    if (r < 0) continue;
                    const int pi = page_slot(r, page_rows, shift, max_pages);
                    CHECK(pi >= 0 && pi < max_pages);
                    for (int page : kHostile) {
                        const int64_t row = paged_pool_row(page, r, page_rows, shift, pool_rows);
                        CHECK(row >= 0 && row < pool_rows);
                    }
                }
        }
}

static void sweep_compact() {
    for (int v_start : {0, 3, 100})
        for (int M : {1, 30, 576})
            for (int R : {0, 1, 5, 30}) {
                if (R > M) continue;
                for (int extra : {0, 1, 64}) {
                    const int n_tot_max = v_start + M + extra;
                    for (int nt : kHostile) {
                        const int n_tot = compact_n_tot(nt, v_start, M, n_tot_max);
                        CHECK(n_tot >= v_start + M && n_tot <= n_tot_max);
                        const int n_out = n_tot - M + R;
                        for (int r = 0; r < n_out; ++r)
                            for (int kept : kHostile) {
                                const int sr = compact_src_row_from(kept, R, v_start, M, n_tot, r);
                                CHECK(sr >= 0 && sr < n_tot);
                                if (r < v_start) CHECK(sr == r);
                                if (r >= v_start + R) CHECK(sr == r - R + M);
                            }
                    }
                }
            }
}

static void sweep_commit_and_trees() {
    for (int T_max : {1, 2, 3, 26, 64}) {
        for (int na : kHostile) {
            const int n = commit_n_acc(na, T_max);
            CHECK(n >= 0 && n <= T_max - 1);
        }
        for (int c : kHostile) {
            const int C = commit_ctx(c);
            CHECK(C >= 0 && (int64_t)C + T_max + 1 < INT32_MAX);
        }
        // any sequence of path entries: move i reads a node >= i + 1 inside the tree, never below the
        // previous one, so no move writes a row that a later move reads
        for (int a : kHostile)
            for (int b : kHostile) {
                int prev = 0;
                for (int i = 0; i < T_max - 1; ++i) {
                    const int p = commit_next_node(prev, (i & 1) ? a : b, T_max);
                    CHECK(p >= i + 1 && p <= T_max - 1 && p >= prev);
                    prev = p;
                }
            }
        for (int nn : kHostile) {
            const int T = tree_nodes(nn, T_max);
            CHECK(T >= 1 && T <= T_max);
        }
        for (int i = 1; i < T_max; ++i)
            for (int p : kHostile) {
                const int q = clamp_parent(p, i);
                CHECK(q >= 0 && q < i);
            }
    }
    for (int N : {0, 1, 310, 8192})
        for (int nc : kHostile) {
            const int n = cand_count(nc, N);
            CHECK(n >= 0 && n <= N);
            for (int u : {0, 1, 7, N - 1}) {
                if (u < 0 || u >= N) continue;
                for (int p : kHostile) {
                    const int q = cand_walk_parent(p, u);
                    CHECK(q >= -1 && q < u);
                }
                for (int k : kHostile) {
                    const int c = kept_candidate(k, N);
                    CHECK(c >= 0 && c < N);
                }
            }
        }
}

static void sweep_score() {
    for (int n_q_max : {1, 8, 32, 64})
        for (int q_rows : {n_q_max, 128})
            for (int row0 : {0, 64})
                for (int n_tot_max : {1, 640, 3008, 1 << 30})
                    for (int nq : kHostile)
                        for (int nt : kHostile)
                            for (int pos : kHostile) {
                                const ScoreSeq s = score_seq_from(nq, nt, pos, q_rows, row0, n_q_max, n_tot_max);
                                CHECK(s.n_q >= 0 && s.n_q <= n_q_max);
                                CHECK(s.n_tot >= 0 && s.n_tot <= n_tot_max);
                                CHECK(s.pos0 >= 0);
                                const int last_pos = s.pos0 + 2 * n_q_max + 1;   // what the kernels add to it
                                CHECK(last_pos > s.pos0);
                            }
}

int main() {
    sweep_seq_info();
    sweep_pool_rows();
    sweep_compact();
    sweep_commit_and_trees();
    sweep_score();
    std::puts("index_math sweep: ok");
    return 0;
}
