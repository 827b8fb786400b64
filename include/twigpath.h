/*
 * twigpath -- C ABI of the MI355X (gfx950) decode hot path of TwigVLM /
 * TwigVLM++: twig-guided token pruning (score, top-R select, stable
 * compaction) and tree-based self-speculative verification (ancestor masks,
 * tree-masked attention, greedy acceptance walk).
 *
 * Conventions for every call
 *   - Pointers marked [dev] are device memory owned by the caller; pointers
 *     marked [host] are read on the host during the call and not retained.
 *   - The library allocates no device memory and keeps no results between calls
 *     (it remembers only, per device, which kernels already had their
 *     shared-memory limit raised).  Scratch space comes in through (ws,
 *     ws_bytes); tw_workspace_bytes() tells how much a call needs.
 *   - A call only enqueues work on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and returns.  Nothing synchronises, nothing is
 *     read back.  Outputs are valid once the caller has synchronised the stream.
 *   - The return value is a tw_status.  No exception crosses the boundary and
 *     nothing is printed.  Contents of device arrays cannot be checked without
 *     a synchronisation, so they are preconditions; when one is violated the
 *     kernels stay inside the buffers described by the arguments (indices are
 *     clamped) but the result is unspecified.
 *   - Same inputs give bit-identical outputs from run to run (no
 *     order-dependent floating-point atomics anywhere).
 *   - A call may be recorded into a HIP graph (stream capture): it consists of
 *     kernel launches only, no memset or copy nodes.  The first launch of some
 *     kernels on a device also raises that kernel's shared-memory limit (a
 *     function attribute, not a stream operation); callers that want nothing
 *     but launches inside a capture make one eager call of the same shape first.
 *
 * Tensor layout: token-major rows.  A row of a key, value or query tensor is H
 * heads of d_h contiguous elements (bf16 or fp32).  d_h must be a multiple of
 * 8 and at most 128; the matrix-core path is taken for bf16 with d_h 64 or 128.
 */
#ifndef TWIGPATH_H
#define TWIGPATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; these are its only exported symbols. */
#if defined(__GNUC__) || defined(__clang__)
#define TW_API __attribute__((visibility("default")))
#else
#define TW_API
#endif

typedef enum {
    TW_OK = 0,
    TW_ERR_INVALID_ARG = -1, /* null pointer, negative size, R > M, span outside the sequence ... */
    TW_ERR_UNSUPPORTED = -2, /* T_max > 64, d_h not supported, dtype combination not built */
    TW_ERR_WORKSPACE = -3,   /* ws is NULL or ws_bytes too small */
    TW_ERR_LAUNCH = -4       /* the HIP runtime reported an error for a launch */
} tw_status;

typedef enum { TW_F32 = 0, TW_BF16 = 1 } tw_dtype;

typedef enum { TW_CALL_TTP_SCORE = 1, TW_CALL_TREE_VERIFY_ATTN = 2 } tw_call;

#define TW_MAX_TREE 64 /* tree rows per sequence, root included */

/*
 * One layer's K (or V) for a batch of B sequences, living in one pool of
 * pool_rows rows.  Contiguous mode (page_table == NULL): cache row r of
 * sequence b is pool row row_off[b] + r.  Paged mode: it is slot r % page_rows
 * of page page_table[b * max_pages + r / page_rows].  The struct itself is
 * host memory; base, row_off and page_table point to device memory.  base, and
 * every query/gate tensor passed beside a view, is 16-byte aligned (checked:
 * INVALID_ARG otherwise); rows are read with 16-byte accesses.
 */
typedef struct tw_kv_view {
    const void* base;          /* [dev] pool_rows * H * d_h elements */
    int32_t dtype;             /* tw_dtype */
    int32_t H, d_h;
    int64_t pool_rows;
    const int32_t* row_off;    /* [dev] [B], contiguous mode */
    const int32_t* page_table; /* [dev] [B][max_pages], paged mode, else NULL */
    int32_t max_pages, page_rows;
} tw_kv_view;

/* Library version, 1000*major + minor (2.0: the verification workspace carries counters that start at zero;
 * 2.1: they take the first 1024 bytes whatever the shape of the launch). */
TW_API int32_t tw_version(void);

/*
 * Scratch bytes needed by a call.  `which` is a tw_call.  For
 * TW_CALL_TTP_SCORE: rows = n_q_max, max_rows = n_tot_max.  For
 * TW_CALL_TREE_VERIFY_ATTN: rows = T_max, max_rows = max_ctx_len + T_max.
 * H = heads of the query tensor (the view's H, times q_heads_per_kv for the
 * grouped-query entry points).  Returns 0 for calls that need none or for invalid arguments.  The buffer
 * handed to the call is device memory, 16-byte aligned, and not shared with a call that may run
 * at the same time.
 * TW_CALL_TTP_SCORE: its contents on entry do not matter and are undefined on return.
 * TW_CALL_TREE_VERIFY_ATTN: the first 1024 bytes of the buffer are arrival counters, one per
 * (sequence, head) of a launch that cuts sequences into pieces (only launches with fewer than 256
 * such units do); the launch needs them at zero and puts them back to zero as its last action.
 * Partial results lie behind them, in whole 128-byte lines per workgroup when the buffer is
 * 128-byte aligned (recommended).  Zero the buffer once, after allocating it (hipMemset); from
 * then on it serves any number of calls of any shape, one after the other: whatever the shapes,
 * no call writes partial results where another keeps counters.  With counters that are not zero
 * the output is unspecified (still memory-safe, and no kernel waits for another).  After
 * TW_ERR_LAUNCH zero it again.
 */
TW_API size_t tw_workspace_bytes(int32_t which, int32_t B, int32_t rows, int32_t H, int32_t d_h,
                          int32_t max_rows);

/*
 * Pruning score (Sec. 3.1 Eq. 2 and Eq. 3; head mean as in Sec. 5.1 Eq. 7).
 * For sequence b, the n_q[b] scoring rows are query rows at absolute positions
 * q_pos0[b] .. q_pos0[b]+n_q[b]-1 (the last text rows).  Each row's attention
 * is softmax_j(scale * q.k_j) over keys j <= its position (causal != 0) or over
 * all n_tot[b] keys (causal == 0).  scores[b][m] is the mean over heads and
 * scoring rows of the weight on visual key v_start + m.
 *
 *   q_sel   [dev] [B][n_q_max][H][d_h], same dtype as k
 *   k       [host struct] contiguous view of the scoring layer's keys
 *   n_q     [dev] [B] or NULL (= n_q_max for every sequence)
 *   q_pos0  [dev] [B];  n_tot [dev] [B];  n_tot_max = host upper bound of n_tot
 *   scores  [dev] [B][M] fp32 out
 * Preconditions on device contents: 1 <= n_q[b] <= n_q_max,
 * q_pos0[b] + n_q[b] <= n_tot[b] <= n_tot_max, v_start + M <= n_tot[b].
 * Accuracy: logits are fp32 sums of exact bf16 (or fp32) products; exponentials, normalisers,
 * weights and the sums over rows and heads are fp32.  A score is within 1e-6 of the exact mean.
 * The result does not depend on launch order (fixed summation order).
 * Errors: INVALID_ARG for null pointers, negative sizes, v_start + M > n_tot_max,
 * paged k view; UNSUPPORTED for d_h; WORKSPACE.
 */
TW_API int32_t tw_ttp_score(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                     const tw_kv_view* k, const int32_t* n_tot, int32_t n_tot_max, int32_t B,
                     int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * The same score for a base model with grouped-query attention (Qwen2.5-VL
 * among the base VLMs of Sec. 6): q_sel holds H_q = q_heads_per_kv * k->H heads,
 * the view's rows k->H key heads, query head h reads key head h / q_heads_per_kv,
 * and the mean is over the H_q query heads.  q_heads_per_kv = 1 is tw_ttp_score.
 * The workspace is sized by tw_workspace_bytes with H = H_q.
 * Errors as tw_ttp_score, plus INVALID_ARG (q_heads_per_kv < 1) and UNSUPPORTED
 * (q_heads_per_kv > 64, H_q > 65535).
 */
TW_API int32_t tw_ttp_score_gqa(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                         const tw_kv_view* k, int32_t q_heads_per_kv, const int32_t* n_tot, int32_t n_tot_max,
                         int32_t B, int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * tw_ttp_score followed by tw_ttp_select in one call, with one launch fewer: the launch that adds
 * the heads also keeps the R best visual tokens of every row (rows of up to 1024 scores; longer
 * rows get the separate select launch).  scores and kept come out bit-identical to the two
 * separate calls.  kept [dev] [B][R] int32 out; R == 0 leaves it untouched.
 * Errors: those of tw_ttp_score and tw_ttp_select.
 */
TW_API int32_t tw_ttp_score_select(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                                   const tw_kv_view* k, const int32_t* n_tot, int32_t n_tot_max, int32_t B,
                                   int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                                   int32_t R, int32_t* kept, void* ws, size_t ws_bytes, void* stream);

/*
 * Pruning score in the P-Head form (Sec. 5.1 Eq. 7).  One query per sequence
 * (the last text token).  For head h and visual key m the logit is
 *   scale * sum_c (gq[b][h][c] * q[b][h][c]) * (gk[key][h][c] * K[key][h][c]),   key = v_start + m,
 * the softmax runs over the M visual keys only, and scores[b][m] is the mean
 * over heads (so every scores[b] sums to one).  gq / gk are the outputs of the
 * gating projections G_q, G_k, laid out like q and K.
 *   q, gq   [dev] [B][H][d_h], dtype of the views
 *   k, gk   [host structs] contiguous views with the same dtype/H/d_h
 *   scores  [dev] [B][M] fp32 out
 *   ws      at least B*H*M*4 bytes (tw_workspace_bytes(TW_CALL_TTP_SCORE, B, 1, H, d_h, M))
 * Errors: INVALID_ARG (null pointers, paged views, span outside the pools),
 * UNSUPPORTED (d_h, view mismatch, M > 32768), WORKSPACE.
 */
TW_API int32_t tw_ttp_score_phead(const void* q, const void* gq, const tw_kv_view* k, const tw_kv_view* gk,
                           int32_t B, int32_t v_start, int32_t M, float scale, float* scores, void* ws,
                           size_t ws_bytes, void* stream);

/*
 * Top-R keep (TopR of Sec. 3.1 Eq. 3).  kept[b] receives the indices of the R
 * largest scores[b][.], ties toward the lower index, in ascending index order.
 * -0.0 and +0.0 compare equal; scores must be finite.
 *   scores [dev] [B][M] fp32;  kept [dev] [B][R] int32 out.
 * R == M returns 0..M-1, R == 0 writes nothing.  Errors: INVALID_ARG for
 * R < 0, R > M, null pointers with non-empty sizes; UNSUPPORTED for M > 2^20.
 */
TW_API int32_t tw_ttp_select(const float* scores, int32_t B, int32_t M, int32_t R, int32_t* kept,
                      void* stream);

/*
 * Stable compaction (Sec. 3.1 Eq. 3, Sec. 4.2 Eq. 5: kept visual rows in their
 * original order, then every text row; rows before the visual span are kept
 * like text).  Destination row r takes source row
 *   r                          for r < v_start,
 *   v_start + kept[r-v_start]  for v_start <= r < v_start + R,
 *   r - R + M                  otherwise,
 * for each of n_tensors (src, dst) pairs with rows of row_bytes bytes; src has
 * n_tot rows, dst has n_tot - M + R rows and must not overlap src.  R = 0 is
 * FinalWipe (Sec. 4.2).
 *   kept [dev] [R] ascending, values in [0, M);  src, dst [host] tables of
 *   n_tensors device pointers.
 * Errors: INVALID_ARG for null tables or entries, R > M, v_start + M > n_tot,
 * row_bytes == 0.
 */
TW_API int32_t tw_ttp_compact(const int32_t* kept, int32_t R, int32_t v_start, int32_t M, int32_t n_tot,
                       const void* const* src, void* const* dst, int32_t n_tensors,
                       size_t row_bytes, void* stream);

/*
 * The same compaction for a batch of B sequences whose rows live in shared
 * pools (one launch for the whole batch).  Sequence b owns source rows
 * src_row_off[b] .. +n_tot[b] and destination rows dst_row_off[b] ..
 * +n_tot[b]-M+R of every (src[t], dst[t]) pair; kept is [dev] [B][R];
 * n_tot, src_row_off, dst_row_off are [dev] [B]; n_tot_max is a host upper bound
 * of n_tot.  Precondition on device contents: v_start + M <= n_tot[b] <= n_tot_max
 * (a length outside that range is moved into it; the row offsets say where the
 * caller's rows are and are taken as they come).
 * Errors as tw_ttp_compact, plus UNSUPPORTED for B > 65535.
 */
TW_API int32_t tw_ttp_compact_batched(const int32_t* kept, int32_t R, int32_t v_start, int32_t M,
                               const int32_t* n_tot, int32_t n_tot_max, const int32_t* src_row_off,
                               const int32_t* dst_row_off, int32_t B, const void* const* src,
                               void* const* dst, int32_t n_tensors, size_t row_bytes, void* stream);

/*
 * Ancestor-or-self bit masks of draft trees (tree attention, Sec. 5.4 and
 * App. A).  Node 0 is the root (parent -1); parent[i] < i for i > 0.
 *   parent [dev] [B][T_max];  n_nodes [dev] [B];  masks [dev] [B][T_max] uint64 out
 * (entries past n_nodes[b] are written as 0).
 */
TW_API int32_t tw_tree_ancestor_masks(const int32_t* parent, const int32_t* n_nodes, int32_t T_max,
                               int32_t B, uint64_t* masks, void* stream);

/*
 * Tree verification attention (Sec. 3.1 Eq. 2 under the topology-aware causal
 * mask of Sec. 5.4 / App. A; verification step of Alg. 2).  For sequence b,
 * tree row t and head h:
 *   out[b][t][h][:] = sum_j softmax_j(scale * q[b][t][h].K[j][h]) * V[j][h][:]
 * over the ctx_len[b] committed cache rows plus the tree rows of t's ancestors
 * and t itself; tree row u's key/value sit at cache row ctx_len[b] + u.
 *
 *   q        [dev] [B][T_max][H][d_h], dtype of the views
 *   k, v     [host structs] same dtype/H/d_h/paging mode
 *   ctx_len  [dev] [B];  max_ctx_len = host upper bound
 *   parent   [dev] [B][T_max];  n_nodes [dev] [B], 1 <= n_nodes[b] <= T_max
 *   out      [dev] [B][T_max][H][d_h], 16-byte aligned, dtype out_dtype: TW_F32, or TW_BF16
 *            (the fp32 result rounded to nearest even once, at the store; what a following
 *            bf16 projection consumes, and half the bytes written).  Rows past n_nodes[b]
 *            are not written.
 * Accuracy for bf16 inputs: fp32 accumulation; the softmax weights enter the value
 * product as bf16, normalised by their rounded sum: max-abs error <= 2e-3 for fp32 out,
 * plus half a bf16 unit in the last place of the result for bf16 out.
 * Errors: INVALID_ARG, UNSUPPORTED (T_max > 64, d_h, view mismatch, out_dtype), WORKSPACE.
 */
TW_API int32_t tw_tree_verify_attn(const void* q, const tw_kv_view* k, const tw_kv_view* v,
                            const int32_t* ctx_len, int32_t max_ctx_len, const int32_t* parent,
                            const int32_t* n_nodes, int32_t T_max, int32_t B, float scale,
                            void* out, int32_t out_dtype, void* ws, size_t ws_bytes, void* stream);

/*
 * The same attention for a base model with grouped-query attention (Qwen2.5-VL
 * among the base VLMs of Sec. 6): q and out hold H_q = q_heads_per_kv * k->H
 * heads, the views' rows hold k->H key/value heads, and query head h reads
 * key/value head h / q_heads_per_kv.  q_heads_per_kv = 1 is tw_tree_verify_attn.
 * The workspace is sized by tw_workspace_bytes with H = H_q.
 * Errors as tw_tree_verify_attn, plus INVALID_ARG (q_heads_per_kv < 1) and
 * UNSUPPORTED (q_heads_per_kv > 64, H_q > 65535).
 */
TW_API int32_t tw_tree_verify_attn_gqa(const void* q, const tw_kv_view* k, const tw_kv_view* v,
                                int32_t q_heads_per_kv, const int32_t* ctx_len, int32_t max_ctx_len,
                                const int32_t* parent, const int32_t* n_nodes, int32_t T_max, int32_t B,
                                float scale, void* out, int32_t out_dtype, void* ws, size_t ws_bytes,
                                void* stream);

/*
 * tw_tree_verify_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * computation, arguments and errors as tw_tree_verify_attn, with the scratch of a split launch
 * (arrival counters, partial results) in a device array of TW_STATIC_SCRATCH_BYTES that the
 * library holds on every GPU it runs on until the process ends.  The call allocates nothing and
 * frees nothing.  A launch that would need more scratch than that returns TW_ERR_WORKSPACE (ask
 * tw_workspace_bytes; a launch with at least 256 (sequence, head) units needs none and always fits).
 * All calls on one GPU share that GPU's array: two of them must not overlap in time (put them on
 * one stream, or order them with events), or they race on it.  The counters in it are zero when
 * the library is loaded and every launch returns them to zero as its last action, so calls of
 * different shapes may follow each other freely.
 */
#define TW_STATIC_SCRATCH_BYTES (16u << 20)
TW_API int32_t tw_tree_verify_attn_static(const void* q, const tw_kv_view* k, const tw_kv_view* v,
                                   const int32_t* ctx_len, int32_t max_ctx_len, const int32_t* parent,
                                   const int32_t* n_nodes, int32_t T_max, int32_t B, float scale,
                                   void* out, int32_t out_dtype, void* stream);

/*
 * Greedy acceptance walk with bonus token (Sec. 5.4, App. A, last steps of
 * Alg. 2; a chain is the sequence case of Alg. 1).  argmax[b][i] is the target
 * model's prediction for the token after node i.  A non-root node is matched
 * when draft[node] == argmax[parent[node]]; the accepted end point is the
 * deepest node whose whole path from the root is matched (ties toward the
 * lower node index; with distinct sibling tokens this is the walk from the
 * root).  n_acc[b] = accepted draft nodes (root excluded), path[b][0..n_acc)
 * = their node indices from the root side, remaining slots -1,
 * bonus[b] = argmax at the end point.  All arrays [dev] int32.
 */
TW_API int32_t tw_tree_accept(const int32_t* draft, const int32_t* argmax, const int32_t* parent,
                       const int32_t* n_nodes, int32_t T_max, int32_t B, int32_t* n_acc,
                       int32_t* path, int32_t* bonus, void* stream);

/*
 * Sequence-based self-speculative decoding (Sec. 3.1, "Decoding acceleration via
 * self-speculation"; App. A, SSD paragraph: delta = 5, theta = 0.6; Alg. 1) as
 * the chain case of the tree calls: node 0 is the last accepted token, node i
 * the i-th draft token, parent[i] = i - 1, T_max = delta + 1.
 *
 * tw_chain_tree -- the draft model's early exit.  prob [dev] fp32 [B][delta]:
 * the draft model's probability of its i-th draft token (NULL: no early exit).
 * Drafting stops after the first token whose probability is below theta (that
 * token stays in the draft) or after delta tokens:
 * n_nodes[b] = 1 + min(delta, 1 + first i with prob[b][i] < theta); the
 * comparison is made in fp32.  parent [dev] int32 [B][delta + 1] receives the
 * chain (all entries, parent[b][0] = -1).  Both outputs are what
 * tw_tree_verify_attn and tw_chain_accept take.  1 <= delta < TW_MAX_TREE.
 *
 * tw_chain_accept -- draft[b][i] is the token of node i (entry 0 is not read),
 * argmax[b][i] the target model's prediction for the token after node i.
 * n_acc[b] = length of the longest prefix of the n_nodes[b] - 1 draft tokens
 * with draft[b][i] == argmax[b][i - 1]; path[b][j] = j + 1 for j < n_acc[b],
 * -1 after; bonus[b] = argmax[b][n_acc[b]], the target model's own next token.
 * Same result as tw_tree_accept on the chain; the outputs are what
 * tw_kv_commit takes.  All arrays [dev] int32, [B][T_max] or [B].
 */
TW_API int32_t tw_chain_tree(const float* prob, float theta, int32_t delta, int32_t B, int32_t* parent,
                      int32_t* n_nodes, void* stream);
TW_API int32_t tw_chain_accept(const int32_t* draft, const int32_t* argmax, const int32_t* n_nodes,
                        int32_t T_max, int32_t B, int32_t* n_acc, int32_t* path, int32_t* bonus,
                        void* stream);

/*
 * Commit of the accepted path into the KV cache (the step after the acceptance
 * walk in Alg. 2; KV append of Sec. 3.1), so that the next draft-verify
 * iteration can run on the same cache.  For every sequence b and every view
 * (one layer's K or V, each with its own row mapping): the tree root stays at
 * cache row C = ctx_len[b]; accepted node path[b][i] (cache row C + path[b][i])
 * is moved to cache row C + 1 + i for i < n_acc[b]; other rows are untouched;
 * new_ctx_len[b] = C + 1 + n_acc[b] (may be NULL; must not alias ctx_len).
 * In place.  path/n_acc are the outputs of tw_tree_accept.
 *   path [dev] [B][T_max], n_acc [dev] [B], ctx_len [dev] [B], views [host] n_views
 *   structs, new_ctx_len [dev] [B] out.
 * Precondition on device contents: path strictly increasing, 1 <= path[b][i] < T_max.
 * Errors: INVALID_ARG (null pointers, malformed views), UNSUPPORTED (T_max > 64, B > 65535).
 */
TW_API int32_t tw_kv_commit(const int32_t* path, const int32_t* n_acc, int32_t T_max, const tw_kv_view* views,
                     int32_t n_views, const int32_t* ctx_len, int32_t B, int32_t* new_ctx_len,
                     void* stream);

/*
 * Rank-ordered top-E of each row (the per-node expansion of the draft tree by
 * its E most probable tokens, Sec. 5.4 / App. A).  ids[r] / vals[r] receive the
 * E largest entries of probs[r][0..V), larger value first, equal values lower
 * index first.  probs [dev] [n][V] fp32 finite; ids [dev] [n][E] int32; vals [dev]
 * [n][E] fp32.  Errors: INVALID_ARG (E > V, null pointers), UNSUPPORTED (E > 256,
 * V > 2^20).
 */
TW_API int32_t tw_draft_topk(const float* probs, int32_t n, int32_t V, int32_t E, int32_t* ids, float* vals,
                      void* stream);

/*
 * The same expansion taken straight from the logits of the draft head (Sec. 5.4
 * / App. A): ids[r] receives the E most probable tokens of softmax(logits[r][0..V)),
 * larger logit first, equal logits lower index first; probs[r] their
 * probabilities exp(l - max) / sum over the whole row, computed in fp32 in the
 * same single read of the row (relative error below 2e-5).
 *   logits [dev] [n][V] fp32 finite; ids [dev] [n][E] int32; probs [dev] [n][E] fp32.
 * Rows that are 16-byte aligned and a multiple of four long are read with
 * 16-byte loads; any other shape is accepted and read element by element.
 * Errors: INVALID_ARG (E > V, null pointers), UNSUPPORTED (E > 256, V > 2^20).
 */
TW_API int32_t tw_draft_topk_logits(const float* logits, int32_t n, int32_t V, int32_t E, int32_t* ids, float* probs,
                             void* stream);

/*
 * One level of the drafting loop (Sec. 5.4 / App. A: level 1 holds the E most probable tokens after
 * the root; every later level expands the K most confident nodes of the level before it by E tokens
 * each).  The candidates of sequence b live in arrays [B][N] in generation order, in the format
 * tw_tree_build takes.  This call writes one level: candidate out_off + j * E + e is token e of
 * expanded node j,
 *   cand_parent = prev_off + sel[b][j]   (-1 when sel is NULL: the root is the one expanded node),
 *   cand_token = ids[b][j][e],  cand_prob = probs[b][j][e],
 *   cand_conf = cand_conf[parent] * cand_prob   (fp32; 1 * cand_prob under the root),
 * and level_conf[b][j * E + e] = cand_conf of the same candidate, the row that tw_ttp_select takes
 * to pick the next level's expanded nodes (their indices inside this level, ascending).
 *   sel        [dev] [B][n_exp] indices into the previous level's slice [prev_off, out_off), or NULL
 *   ids, probs [dev] [B][n_exp][E], as tw_draft_topk_logits writes them for the expanded nodes' rows
 *   cand_parent, cand_token [dev] [B][N] int32;  cand_prob, cand_conf [dev] [B][N] fp32
 *   level_conf [dev] [B][n_exp * E] fp32 out
 * Errors: INVALID_ARG (negative sizes, out_off + n_exp * E > N, sel with prev_off >= out_off, no sel
 * with n_exp > 1, null pointers), UNSUPPORTED (n_exp * E > 65536, B > 65535).
 */
TW_API int32_t tw_draft_expand(const int32_t* sel, int32_t n_exp, int32_t prev_off, int32_t out_off,
                               const int32_t* ids, const float* probs, int32_t E, int32_t N, int32_t B,
                               int32_t* cand_parent, int32_t* cand_token, float* cand_prob, float* cand_conf,
                               float* level_conf, void* stream);

/*
 * Pruning of a drafted token tree to its most confident candidates (App. A:
 * the completed tree keeps at most N_max candidate nodes, highest confidence
 * first, together with their ancestors).  Candidates 0..n_cand[b)-1 of sequence
 * b are the drafted nodes in generation order: cand_parent < own index, or -1
 * for a child of the root; cand_prob in [0, 1] is the draft probability of the
 * token given its parent.  The confidence of a candidate is the product of
 * cand_prob along its path; the T_max-1 most confident candidates are kept
 * (ties toward the lower index; the kept set is closed under taking parents
 * because confidence never grows along a path).  Output, in the format the
 * verification calls take: node 0 = root (parent -1, token root_token[b]); kept
 * candidates follow in ascending candidate index (a topological order);
 * parent_out / token_out / src_out (the candidate index, -1 for the root) are
 * [dev] [B][T_max], unused slots hold parent 0, token 0, src -1;
 * n_nodes_out[b] = 1 + min(T_max - 1, n_cand[b]).
 * ws: tw_tree_build_workspace_bytes(B, N, T_max).  Errors: INVALID_ARG,
 * UNSUPPORTED (T_max > 64, N > 8192, B > 65535), WORKSPACE.
 */
TW_API size_t tw_tree_build_workspace_bytes(int32_t B, int32_t N, int32_t T_max);
TW_API int32_t tw_tree_build(const int32_t* cand_parent, const int32_t* cand_token, const float* cand_prob,
                      const int32_t* n_cand, const int32_t* root_token, int32_t N, int32_t B, int32_t T_max,
                      int32_t* parent_out, int32_t* token_out, int32_t* src_out, int32_t* n_nodes_out,
                      void* ws, size_t ws_bytes, void* stream);

/* Host helper: TW_OK when parent[0] == -1 and 0 <= parent[i] < i for 0 < i < T <= 64. */
TW_API int32_t tw_validate_tree(const int32_t* parent_host, int32_t T);

/* Host helper: average retained visual tokens with FinalWipe (Sec. 4.2 Eq. 6;
 * K_f = L gives Sec. 3.1 Eq. 4), rounded to the nearest integer. */
TW_API int32_t tw_rbar(int32_t M, int32_t K, int32_t R, int32_t K_f, int32_t L);

#ifdef __cplusplus
}
#endif
#endif /* TWIGPATH_H */
