/*
 * CPU oracle for the pruned-cache decode path of TwigVLM / TwigVLM++.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library must compute.  It is used by the tests, by the smoke
 * check and by the CPU-baseline leg of the benchmark, never by the product
 * path, and it shares no source with the HIP kernels.
 *
 * Every function takes host pointers.  Floating-point inputs are either fp32
 * (dtype 0) or bf16 bit patterns in uint16 (dtype 1); both are widened exactly
 * to fp64 and all arithmetic is fp64.  Rows of a key/value tensor are
 * token-major: row r holds H heads of d_h contiguous elements.
 *
 * Parity pins (tests/test_oracle_*.py): every function below is checked
 * against closed forms, library attention routines, brute force and
 * exhaustive enumeration; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen(const void* base, int dtype, int64_t idx) {
    if (dtype == 0) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Pruning score (Sec. 3.1 Eq. 2 attention map; Sec. 3.1 Eq. 3 text-to-visual
 * column sums; head averaging as in Sec. 5.1 Eq. 7).
 *
 * For sequence b, head h and scoring row i (absolute position p = q_pos0[b]+i)
 * the attention row is softmax_j(scale * q . k_j) over keys j <= p when causal,
 * over all n_tot[b] keys otherwise.  score[b][m] is the mean over heads and
 * scoring rows of the attention weight on visual key v_start + m.
 *
 *   q_sel  [B][n_q_max][H][d_h]   rows beyond n_q[b] unused
 *   k      rows of H_kv heads; rows of sequence b start at row k_row_off[b].  H_kv == H is
 *          ordinary multi-head attention; H = g * H_kv is the grouped-query attention of the
 *          Qwen2.5-VL base model among those of Sec. 6: query head h reads key head h / g.
 *   scores [B][M] fp64
 */
int orc_ttp_score(const void* q_sel, const void* k, int dtype, int B, int H, int H_kv, int d_h, int n_q_max,
                  const int32_t* n_q, const int32_t* q_pos0, const int32_t* n_tot,
                  const int64_t* k_row_off, int v_start, int M, double scale, int causal,
                  double* scores) {
    if (!q_sel || !k || !scores || B < 0 || M < 0) return -1;
    if (H < 1 || H_kv < 1 || H % H_kv) return -1;
    const int group = H / H_kv;   /* grouped-query attention: query head h reads key head h / group */
    for (int b = 0; b < B; ++b) {
        if (v_start < 0 || v_start + M > n_tot[b] || n_q[b] < 1 || n_q[b] > n_q_max) return -1;
        if (q_pos0[b] < 0 || q_pos0[b] + n_q[b] > n_tot[b]) return -1;
    }
    int nthr = orc_max_threads();
    for (int b = 0; b < B; ++b) {
        int nt = n_tot[b];
        double* part = (double*)calloc((size_t)nthr * (size_t)M, sizeof(double));
        if (!part) return -3;
#pragma omp parallel
        {
#ifdef _OPENMP
            int tid = omp_get_thread_num();
#else
            int tid = 0;
#endif
            double* acc = part + (size_t)tid * M;
            double* s = (double*)malloc((size_t)nt * sizeof(double));
#pragma omp for collapse(2) schedule(static)
            for (int h = 0; h < H; ++h) {
                for (int i = 0; i < n_q[b]; ++i) {
                    int p = q_pos0[b] + i;
                    int nvis = causal ? p + 1 : nt;
                    int64_t qo = (((int64_t)b * n_q_max + i) * H + h) * d_h;
                    double mx = -INFINITY;
                    for (int j = 0; j < nvis; ++j) {
                        int64_t ko = ((k_row_off[b] + j) * H_kv + h / group) * (int64_t)d_h;
                        double dot = 0.0;
                        for (int c = 0; c < d_h; ++c)
                            dot += widen(q_sel, dtype, qo + c) * widen(k, dtype, ko + c);
                        s[j] = scale * dot;
                        if (s[j] > mx) mx = s[j];
                    }
                    double l = 0.0;
                    for (int j = 0; j < nvis; ++j) {
                        s[j] = exp(s[j] - mx);
                        l += s[j];
                    }
                    for (int m = 0; m < M; ++m) {
                        int j = v_start + m;
                        if (j < nvis) acc[m] += s[j] / l;
                    }
                }
            }
            free(s);
        }
        for (int m = 0; m < M; ++m) {
            double t = 0.0;
            for (int th = 0; th < nthr; ++th) t += part[(size_t)th * M + m];
            scores[(size_t)b * M + m] = t / ((double)H * (double)n_q[b]);
        }
        free(part);
    }
    return 0;
}

/*
 * Top-R keep (the TopR operator of Sec. 3.1 Eq. 3).  Order: higher score
 * first, equal scores (fp32 ==, so -0 equals +0) lower index first.  The R
 * best indices are returned in ascending index order.  kept [B][R].
 */
typedef struct { float s; int32_t m; } orc_pair;

static int pair_cmp(const void* a, const void* b) {
    const orc_pair* x = (const orc_pair*)a;
    const orc_pair* y = (const orc_pair*)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->m > y->m) - (x->m < y->m);
}

static int int_cmp(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

int orc_ttp_select(const float* scores, int B, int M, int R, int32_t* kept) {
    if (B < 0 || M < 0 || R < 0 || R > M) return -1;
    if ((B > 0 && M > 0 && !scores) || (B > 0 && R > 0 && !kept)) return -1;
    orc_pair* pr = (orc_pair*)malloc(sizeof(orc_pair) * (size_t)(M > 0 ? M : 1));
    if (!pr) return -3;
    for (int b = 0; b < B; ++b) {
        for (int m = 0; m < M; ++m) {
            pr[m].s = scores[(size_t)b * M + m];
            pr[m].m = m;
        }
        /* the comparator is a total order on (score, index), so any sort is stable here */
        qsort(pr, (size_t)M, sizeof(orc_pair), pair_cmp);
        for (int r = 0; r < R; ++r) kept[(size_t)b * R + r] = pr[r].m;
        qsort(kept + (size_t)b * R, (size_t)R, sizeof(int32_t), int_cmp);
    }
    free(pr);
    return 0;
}

/*
 * Stable compaction (Sec. 3.1 Eq. 3: the kept visual rows, in their original
 * order, followed by every text row; rows in front of the visual span are
 * kept like text).  dst has v_start + R + (n_tot - v_start - M) rows.
 */
int orc_ttp_compact(const int32_t* kept, int R, int v_start, int M, int n_tot, const void* src,
                    void* dst, size_t row_bytes) {
    if (R < 0 || R > M || v_start < 0 || v_start + M > n_tot) return -1;
    if (!src || !dst || (R > 0 && !kept)) return -1;
    for (int r = 0; r < R; ++r)
        if (kept[r] < 0 || kept[r] >= M) return -1;
    const char* s = (const char*)src;
    char* d = (char*)dst;
    int64_t o = 0;
    for (int r = 0; r < v_start; ++r) memcpy(d + (o++) * row_bytes, s + (int64_t)r * row_bytes, row_bytes);
    for (int r = 0; r < R; ++r)
        memcpy(d + (o++) * row_bytes, s + (int64_t)(v_start + kept[r]) * row_bytes, row_bytes);
    for (int r = v_start + M; r < n_tot; ++r)
        memcpy(d + (o++) * row_bytes, s + (int64_t)r * row_bytes, row_bytes);
    return 0;
}

/*
 * Ancestor-or-self sets of a draft tree as bit masks (tree attention of
 * Sec. 5.4 / App. A: a node sees its ancestors; the diagonal is included as
 * in any causal mask).  Node 0 is the root with parent -1, parent[i] < i.
 */
int orc_tree_ancestors(const int32_t* parent, int T, uint64_t* anc) {
    if (!parent || !anc || T < 1 || T > 64 || parent[0] != -1) return -1;
    for (int i = 1; i < T; ++i)
        if (parent[i] < 0 || parent[i] >= i) return -1;
    for (int i = 0; i < T; ++i) {
        uint64_t m = 0;
        for (int u = i; u >= 0; u = parent[u]) m |= (uint64_t)1 << u;
        anc[i] = m;
    }
    return 0;
}

/*
 * Tree verification attention (Sec. 3.1 Eq. 2 restricted by the
 * topology-aware mask of Sec. 5.4 / App. A).  For instance b, tree row t and
 * head h the visible keys are the ctx_len[b] committed rows plus the tree rows
 * of t's ancestors and t itself; tree row u's key/value is cache row
 * ctx_len[b] + u.  Cache row r of instance b is pool row rows[rows_off[b] + r].
 *
 *   q   [B][T_max][H][d_h]       out [B][T_max][H][d_h] fp64 (rows >= n_nodes[b] untouched)
 *   k_pool, v_pool  rows of H_kv heads (H_kv == H, or grouped-query attention as in orc_ttp_score)
 */
int orc_tree_verify_attn(const void* q, const void* k_pool, const void* v_pool, int dtype, int B,
                         int H, int H_kv, int d_h, int T_max, const int32_t* n_nodes, const int32_t* ctx_len,
                         const int64_t* rows, const int64_t* rows_off, const int32_t* parent,
                         double scale, double* out) {
    if (!q || !k_pool || !v_pool || !out || !parent || T_max < 1 || T_max > 64) return -1;
    if (H < 1 || H_kv < 1 || H % H_kv) return -1;
    const int group = H / H_kv;   /* query head h reads key/value head h / group */
    for (int b = 0; b < B; ++b) {
        if (n_nodes[b] < 1 || n_nodes[b] > T_max || ctx_len[b] < 0) return -1;
        uint64_t tmp[64];
        if (orc_tree_ancestors(parent + (size_t)b * T_max, n_nodes[b], tmp)) return -1;
    }
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int T = n_nodes[b], C = ctx_len[b];
            uint64_t anc[64];
            orc_tree_ancestors(parent + (size_t)b * T_max, T, anc);
            const int64_t* rw = rows + rows_off[b];
            double* s = (double*)malloc((size_t)(C + T) * sizeof(double));
            for (int t = 0; t < T; ++t) {
                int64_t qo = (((int64_t)b * T_max + t) * H + h) * d_h;
                double mx = -INFINITY;
                for (int j = 0; j < C + T; ++j) {
                    int vis = j < C || ((anc[t] >> (j - C)) & 1);
                    if (!vis) { s[j] = -INFINITY; continue; }
                    int64_t ko = (rw[j] * H_kv + h / group) * (int64_t)d_h;
                    double dot = 0.0;
                    for (int c = 0; c < d_h; ++c)
                        dot += widen(q, dtype, qo + c) * widen(k_pool, dtype, ko + c);
                    s[j] = scale * dot;
                    if (s[j] > mx) mx = s[j];
                }
                double l = 0.0;
                for (int j = 0; j < C + T; ++j) {
                    s[j] = (s[j] == -INFINITY) ? 0.0 : exp(s[j] - mx);
                    l += s[j];
                }
                double* o = out + qo;
                for (int c = 0; c < d_h; ++c) o[c] = 0.0;
                for (int j = 0; j < C + T; ++j) {
                    if (s[j] == 0.0) continue;
                    int64_t vo = (rw[j] * H_kv + h / group) * (int64_t)d_h;
                    double w = s[j] / l;
                    for (int c = 0; c < d_h; ++c) o[c] += w * widen(v_pool, dtype, vo + c);
                }
            }
            free(s);
        }
    }
    return 0;
}

/*
 * Greedy acceptance walk (Sec. 5.4, App. A and the last steps of Alg. 2; a
 * chain is the sequence case of Alg. 1).  argmax[i] is the target model's
 * prediction for the token that follows node i.  Starting from the root, a
 * child is accepted when its draft id equals the argmax id of the node it
 * hangs under.  When several children of one node carry the matching id the
 * walk explores each and keeps the deepest end point, ties toward the lower
 * node index.  n_acc counts accepted draft nodes (root excluded), path lists
 * them root-side first (unused slots -1), bonus is argmax at the end point.
 */
static void walk(const int32_t* draft, const int32_t* argmx, const int32_t* parent, int T, int cur,
                 int depth, int* best, int* best_depth) {
    if (depth > *best_depth || (depth == *best_depth && cur < *best)) {
        *best = cur;
        *best_depth = depth;
    }
    for (int c = cur + 1; c < T; ++c)
        if (parent[c] == cur && draft[c] == argmx[cur])
            walk(draft, argmx, parent, T, c, depth + 1, best, best_depth);
}

int orc_tree_accept(const int32_t* draft, const int32_t* argmx, const int32_t* parent,
                    const int32_t* n_nodes, int T_max, int B, int32_t* n_acc, int32_t* path,
                    int32_t* bonus) {
    if (!draft || !argmx || !parent || !n_nodes || !n_acc || !path || !bonus) return -1;
    if (T_max < 1 || T_max > 64) return -1;
    for (int b = 0; b < B; ++b) {
        const int32_t* par = parent + (size_t)b * T_max;
        int T = n_nodes[b];
        uint64_t tmp[64];
        if (T < 1 || T > T_max || orc_tree_ancestors(par, T, tmp)) return -1;
        int best = 0, best_depth = -1;
        walk(draft + (size_t)b * T_max, argmx + (size_t)b * T_max, par, T, 0, 0, &best, &best_depth);
        n_acc[b] = best_depth;
        bonus[b] = argmx[(size_t)b * T_max + best];
        int32_t* p = path + (size_t)b * T_max;
        for (int i = 0; i < T_max; ++i) p[i] = -1;
        for (int u = best, d = best_depth; u > 0; u = par[u]) p[--d] = u;
    }
    return 0;
}

/*
 * Sequence-based self-speculative decoding (Sec. 3.1; App. A, SSD paragraph;
 * Alg. 1), one sequence.
 *
 * orc_chain_draft_len: how many tokens the draft model produces.  It stops
 * after delta tokens, or earlier, right after a token whose probability is
 * below theta (Alg. 1 tests the token it has just appended, so that token is
 * part of the draft).  prob may be NULL: no early exit.
 *
 * orc_chain_accept: draft[i], i = 1..n_draft, are the draft tokens (draft[0] is
 * the last accepted token and is not read); argmx[i] is the target model's
 * prediction for the token after position i.  Accepted are the draft tokens
 * that match the target's predictions up to the first mismatch; the target's
 * prediction at that point is the next token.  Returns the number accepted and
 * stores the next token.
 */
int orc_chain_draft_len(const float* prob, float theta, int delta) {
    if (delta < 1) return -1;
    if (!prob) return delta;
    int len = 0;
    while (len < delta) {
        const float p = prob[len];
        ++len;                   /* the token is appended ... */
        if (p < theta) break;    /* ... then tested */
    }
    return len;
}

int orc_chain_accept(const int32_t* draft, const int32_t* argmx, int n_draft, int32_t* next_token) {
    if (!draft || !argmx || !next_token || n_draft < 0) return -1;
    int n = 0;
    for (int i = 1; i <= n_draft; ++i) {
        if (draft[i] != argmx[i - 1]) break;
        n = i;
    }
    *next_token = argmx[n];
    return n;
}

/*
 * Average number of retained visual tokens with FinalWipe (Sec. 4.2 Eq. 6;
 * Eq. 4 is the case K_f = L), rounded to the nearest integer.
 */
int orc_rbar(int M, int K, int R, int K_f, int L) {
    double x = ((double)M * K + (double)R * (K_f - K)) / (double)L;
    return (int)floor(x + 0.5);
}

/*
 * Commit of the accepted path into one cache tensor (the step that follows the
 * acceptance walk in Alg. 2; KV append of Sec. 3.1).  The tree root already
 * sits at cache row C; accepted node path[i] (cache row C + path[i]) becomes
 * cache row C + 1 + i.  Stated as a gather from a snapshot of the old rows, so
 * the order of the moves cannot matter.  rows[r] is the pool row of cache row r
 * of this sequence (n_rows_known entries).  Returns the new context length
 * C + 1 + n_acc, or -1 for invalid arguments.
 */
int orc_kv_commit(void* pool, size_t row_bytes, const int64_t* rows, int n_rows_known, int C,
                  const int32_t* path, int n_acc, int T) {
    if (!pool || !rows || C < 0 || n_acc < 0 || n_acc > T - 1 || C + T > n_rows_known) return -1;
    for (int i = 0; i < n_acc; ++i) {
        if (path[i] < 1 || path[i] >= T) return -1;
        if (i > 0 && path[i] <= path[i - 1]) return -1;
    }
    char* p = (char*)pool;
    char* snap = (char*)malloc((size_t)(n_acc > 0 ? n_acc : 1) * row_bytes);
    if (!snap) return -3;
    for (int i = 0; i < n_acc; ++i) memcpy(snap + (size_t)i * row_bytes, p + (size_t)rows[C + path[i]] * row_bytes, row_bytes);
    for (int i = 0; i < n_acc; ++i) memcpy(p + (size_t)rows[C + 1 + i] * row_bytes, snap + (size_t)i * row_bytes, row_bytes);
    free(snap);
    return C + 1 + n_acc;
}

/*
 * Pruning score in the P-Head form (Sec. 5.1 Eq. 7): for each head the single
 * query (last text token) and every visual key are first multiplied
 * element-wise by their gate vectors, the scaled dot products are normalised by
 * a softmax over the M visual keys only, and the heads are averaged.
 *
 *   q, gq   [B][H][d_h]      k, gk  token-major rows; visual key m of sequence b is row
 *   k_row_off[b] + v_start + m (gk_row_off for the gates).   scores [B][M] fp64
 */
int orc_ttp_score_phead(const void* q, const void* gq, const void* k, const void* gk, int dtype, int B,
                        int H, int d_h, const int64_t* k_row_off, const int64_t* gk_row_off, int v_start,
                        int M, double scale, double* scores) {
    if (!q || !gq || !k || !gk || !scores || B < 0 || M < 1 || v_start < 0) return -1;
    double* s = (double*)malloc((size_t)M * sizeof(double));
    if (!s) return -3;
    for (int b = 0; b < B; ++b) {
        for (int m = 0; m < M; ++m) scores[(size_t)b * M + m] = 0.0;
        for (int h = 0; h < H; ++h) {
            int64_t qo = ((int64_t)b * H + h) * d_h;
            double mx = -INFINITY;
            for (int m = 0; m < M; ++m) {
                int64_t ko = ((k_row_off[b] + v_start + m) * H + h) * (int64_t)d_h;
                int64_t go = ((gk_row_off[b] + v_start + m) * H + h) * (int64_t)d_h;
                double dot = 0.0;
                for (int c = 0; c < d_h; ++c)
                    dot += (widen(gq, dtype, qo + c) * widen(q, dtype, qo + c)) *
                           (widen(gk, dtype, go + c) * widen(k, dtype, ko + c));
                s[m] = scale * dot;
                if (s[m] > mx) mx = s[m];
            }
            double l = 0.0;
            for (int m = 0; m < M; ++m) {
                s[m] = exp(s[m] - mx);
                l += s[m];
            }
            for (int m = 0; m < M; ++m) scores[(size_t)b * M + m] += s[m] / l / (double)H;
        }
    }
    free(s);
    return 0;
}

/*
 * Rank-ordered top-E of a row (per-node expansion of the draft tree, Sec. 5.4 /
 * App. A): the E largest values, larger first, equal values lower index first.
 */
int orc_draft_topk(const float* probs, int n, int V, int E, int32_t* ids, float* vals) {
    if (n < 0 || V < 0 || E < 0 || E > V) return -1;
    if (n > 0 && E > 0 && (!probs || !ids || !vals)) return -1;
    orc_pair* pr = (orc_pair*)malloc(sizeof(orc_pair) * (size_t)(V > 0 ? V : 1));
    if (!pr) return -3;
    for (int r = 0; r < n; ++r) {
        for (int m = 0; m < V; ++m) {
            pr[m].s = probs[(size_t)r * V + m];
            pr[m].m = m;
        }
        qsort(pr, (size_t)V, sizeof(orc_pair), pair_cmp);
        for (int e = 0; e < E; ++e) {
            ids[(size_t)r * E + e] = pr[e].m;
            vals[(size_t)r * E + e] = pr[e].s;
        }
    }
    free(pr);
    return 0;
}

/*
 * The same expansion taken from the logits of the draft head (Sec. 5.4 / App. A):
 * the E most probable tokens of softmax(logits[r]) and their probabilities.  The
 * order is decided on the logits themselves (softmax is monotone): larger logit
 * first, equal logits lower index first.  The probabilities are fp64,
 * exp(l - max) / sum over the whole row.
 */
int orc_draft_topk_logits(const float* logits, int n, int V, int E, int32_t* ids, double* probs) {
    if (n < 0 || V < 0 || E < 0 || E > V) return -1;
    if (n > 0 && E > 0 && (!logits || !ids || !probs)) return -1;
    orc_pair* pr = (orc_pair*)malloc(sizeof(orc_pair) * (size_t)(V > 0 ? V : 1));
    if (!pr) return -3;
    for (int r = 0; r < n; ++r) {
        const float* row = logits + (size_t)r * V;
        double mx = -INFINITY, sum = 0.0;
        for (int m = 0; m < V; ++m)
            if ((double)row[m] > mx) mx = (double)row[m];
        for (int m = 0; m < V; ++m) sum += exp((double)row[m] - mx);
        for (int m = 0; m < V; ++m) {
            pr[m].s = row[m];
            pr[m].m = m;
        }
        qsort(pr, (size_t)V, sizeof(orc_pair), pair_cmp);
        for (int e = 0; e < E; ++e) {
            ids[(size_t)r * E + e] = pr[e].m;
            probs[(size_t)r * E + e] = exp((double)pr[e].s - mx) / sum;
        }
    }
    free(pr);
    return 0;
}

typedef struct { double s; int32_t m; } orc_pair_d;

static int pair_d_cmp(const void* a, const void* b) {
    const orc_pair_d* x = (const orc_pair_d*)a;
    const orc_pair_d* y = (const orc_pair_d*)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->m > y->m) - (x->m < y->m);
}

/*
 * The level-wise drafting loop of tree-based self-speculative decoding (Sec. 5.4 / App. A) on given
 * logits: level 1 holds the E most probable tokens after the root; every later level, up to D,
 * expands the K most confident nodes of the level before it (confidence = product of the draft
 * probabilities along the path, fp64; ties toward the lower candidate index; all of them when
 * the level has fewer than K) by their E most probable tokens, the expanded nodes taken in ascending
 * candidate index.  logits is [1 + N][V] fp32 with N = E + (D - 1) * K * E: row 0 holds the logits
 * after the root, row 1 + c those after candidate c (only the rows of expanded nodes are read: they
 * stand for the draft model's forward passes).  Candidates come out in generation order:
 * cand_parent (-1 under the root), cand_token, cand_prob and cand_conf [N]; expanded [(D - 1) * K]
 * lists the nodes expanded at levels 2..D (-1 for unused slots); margin [D - 1] is the relative gap
 * between the least confident expanded node and the most confident node left out (1 when none is
 * left out), which tells a test how far a selection is from a tie.  Composes orc_draft_topk_logits.
 * Returns the number of candidates, -1 on invalid arguments, -3 when out of memory.
 */
int orc_draft_topk_logits(const float* logits, int n, int V, int E, int32_t* ids, double* probs);

int orc_draft_tree(const float* logits, int V, int E, int K, int D, int32_t* cand_parent, int32_t* cand_token,
                   double* cand_prob, double* cand_conf, int32_t* expanded, double* margin) {
    if (V < 1 || E < 1 || E > V || K < 1 || D < 1 || !logits || !cand_parent || !cand_token || !cand_prob || !cand_conf)
        return -1;
    if (D > 1 && (!expanded || !margin)) return -1;
    int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
    double* pr = (double*)malloc(sizeof(double) * (size_t)E);
    orc_pair_d* order = (orc_pair_d*)malloc(sizeof(orc_pair_d) * (size_t)(K * E > E ? K * E : E));
    int32_t* chosen = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
    if (!ids || !pr || !order || !chosen) return -3;
    for (int i = 0; i < (D - 1) * K; ++i) expanded[i] = -1;
    /* level 1: the root's E most probable tokens */
    orc_draft_topk_logits(logits, 1, V, E, ids, pr);
    for (int e = 0; e < E; ++e) {
        cand_parent[e] = -1;
        cand_token[e] = ids[e];
        cand_prob[e] = pr[e];
        cand_conf[e] = pr[e];
    }
    int prev_off = 0, prev_n = E, n = E;
    for (int level = 2; level <= D; ++level) {
        /* the K most confident nodes of the previous level, then in ascending candidate index */
        for (int i = 0; i < prev_n; ++i) {
            order[i].s = cand_conf[prev_off + i];
            order[i].m = prev_off + i;
        }
        qsort(order, (size_t)prev_n, sizeof(orc_pair_d), pair_d_cmp);
        const int k = prev_n < K ? prev_n : K;
        margin[level - 2] = k < prev_n ? (order[k - 1].s - order[k].s) / order[k - 1].s : 1.0;
        for (int j = 0; j < k; ++j) chosen[j] = order[j].m;
        qsort(chosen, (size_t)k, sizeof(int32_t), int_cmp);
        const int out_off = n;
        for (int j = 0; j < k; ++j) {
            const int u = chosen[j];
            expanded[(level - 2) * K + j] = u;
            orc_draft_topk_logits(logits + (size_t)(1 + u) * V, 1, V, E, ids, pr);
            for (int e = 0; e < E; ++e) {
                cand_parent[n] = u;
                cand_token[n] = ids[e];
                cand_prob[n] = pr[e];
                cand_conf[n] = cand_conf[u] * pr[e];
                ++n;
            }
        }
        prev_off = out_off;
        prev_n = k * E;
    }
    free(ids);
    free(pr);
    free(order);
    free(chosen);
    return n;
}

/*
 * Confidence of drafted candidates (App. A): the product of the draft
 * probabilities along the path from the root to the candidate, in fp64.  A
 * candidate's parent precedes it (cand_parent[i] < i, -1 for a child of the
 * root), so one pass in generation order gives conf[i] = conf[parent] * prob[i].
 * Returns 0, -1 on invalid arguments.
 */
int orc_tree_confidence(const int32_t* cand_parent, const float* cand_prob, int n_cand, double* conf) {
    if (n_cand < 0 || (n_cand > 0 && (!cand_parent || !cand_prob || !conf))) return -1;
    for (int i = 0; i < n_cand; ++i) {
        if (cand_parent[i] < -1 || cand_parent[i] >= i) return -1;
        conf[i] = (cand_parent[i] < 0 ? 1.0 : conf[cand_parent[i]]) * (double)cand_prob[i];
    }
    return 0;
}

/*
 * Pruning of a drafted tree to its most confident candidates (App. A).  The
 * confidence of candidate i is orc_tree_confidence (fp64 product along the
 * path); the T_max - 1 most confident candidates are kept, ties toward the
 * lower index (a product with a factor <= 1 never exceeds its parent's, so the
 * kept set holds every ancestor of a kept candidate); node 0 is the root, kept
 * candidates follow in ascending candidate index.
 * One sequence per call.  Returns the number of nodes (root included), -1 on
 * invalid arguments.
 */
int orc_tree_build(const int32_t* cand_parent, const int32_t* cand_token, const float* cand_prob, int n_cand,
                   int32_t root_token, int T_max, int32_t* parent_out, int32_t* token_out, int32_t* src_out) {
    if (n_cand < 0 || T_max < 1 || T_max > 64 || !parent_out || !token_out || !src_out) return -1;
    for (int i = 0; i < n_cand; ++i)
        if (cand_parent[i] < -1 || cand_parent[i] >= i) return -1;
    int n_keep = n_cand < T_max - 1 ? n_cand : T_max - 1;
    orc_pair_d* pr = (orc_pair_d*)malloc(sizeof(orc_pair_d) * (size_t)(n_cand > 0 ? n_cand : 1));
    int32_t* node_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_cand > 0 ? n_cand : 1));
    double* conf = (double*)malloc(sizeof(double) * (size_t)(n_cand > 0 ? n_cand : 1));
    if (!pr || !node_of || !conf) return -3;
    orc_tree_confidence(cand_parent, cand_prob, n_cand, conf);
    for (int i = 0; i < n_cand; ++i) {
        pr[i].s = conf[i];
        pr[i].m = i;
        node_of[i] = 0;
    }
    free(conf);
    qsort(pr, (size_t)n_cand, sizeof(orc_pair_d), pair_d_cmp);
    int32_t keep[64];
    for (int r = 0; r < n_keep; ++r) keep[r] = pr[r].m;
    qsort(keep, (size_t)n_keep, sizeof(int32_t), int_cmp);
    for (int t = 0; t < T_max; ++t) {
        parent_out[t] = 0;
        token_out[t] = 0;
        src_out[t] = -1;
    }
    parent_out[0] = -1;
    token_out[0] = root_token;
    for (int r = 0; r < n_keep; ++r) node_of[keep[r]] = 1 + r;
    for (int r = 0; r < n_keep; ++r) {
        int c = keep[r];
        parent_out[1 + r] = cand_parent[c] < 0 ? 0 : node_of[cand_parent[c]];
        token_out[1 + r] = cand_token[c];
        src_out[1 + r] = c;
    }
    free(pr);
    free(node_of);
    return 1 + n_keep;
}
