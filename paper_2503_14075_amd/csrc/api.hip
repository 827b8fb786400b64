// C-ABI entry points of libtwigpath: argument validation, launch planning and
// dispatch.  Every call enqueues on the caller's stream and returns.
#include "twig_internal.h"
#ifdef TW_TRACE
#include <cstdlib>
#endif

using namespace tw;

#ifdef TW_TRACE
static unsigned long long* g_trace = nullptr;   // timeline buffer of the diagnostic build (tw_debug_set_trace)
#endif

namespace {

bool dh_ok(int d_h) { return d_h >= 8 && d_h <= 128 && d_h % 8 == 0; }

int view_status(const tw_kv_view* v, bool allow_paged) {
    if (!v || !v->base || v->pool_rows <= 0 || v->H <= 0) return TW_ERR_INVALID_ARG;
    if ((uintptr_t)v->base % 16) return TW_ERR_INVALID_ARG;
    if (v->dtype != TW_F32 && v->dtype != TW_BF16) return TW_ERR_UNSUPPORTED;
    if (!dh_ok(v->d_h)) return TW_ERR_UNSUPPORTED;
    if (v->page_table) {
        if (!allow_paged || v->max_pages <= 0 || v->page_rows <= 0) return TW_ERR_INVALID_ARG;
    } else if (!v->row_off) {
        return TW_ERR_INVALID_ARG;
    }
    return TW_OK;
}

}  // namespace

namespace tw {

// Wavefront layout and row split of tree verification.  A node block is 32 tree rows.  With at
// least 768 (sequence, head, node block) units every wavefront takes its own unit (four heads,
// or two heads x two blocks, per workgroup) and the cache is never split; with fewer, a workgroup
// takes one head and its wavefronts share the head's rows round-robin.  Then the cache rows are
// additionally cut into pieces of split_rows rows, one workgroup each, while the launch has fewer
// than 256 workgroups (one per compute unit), never below 256 rows per piece.  The pieces have one
// length for the whole launch (the host knows the longest sequence only): a shorter sequence
// simply has fewer of them, and one that fits a single piece is finished by its workgroup alone.
VerifyPlan verify_plan(int B, int H, int T_max, int max_rows) {
    VerifyPlan p;
    p.n_blk = T_max > 32 ? 2 : 1;
    const long units = (long)B * H * p.n_blk;
    p.n_splits = 1;
    p.split_rows = (int)(((int64_t)max_rows + 31) / 32 * 32);
    if (units >= 768) {
        p.heads_per_wg = 4 / p.n_blk;
        p.n_phase = 1;
        return p;
    }
    p.heads_per_wg = 1;
    p.n_phase = 4 / p.n_blk;
    const long wgs = (long)B * H;
    long want = wgs >= 256 || wgs <= 0 ? 1 : (256 + wgs - 1) / wgs;
    long cap = max_rows / 256;
    if (cap < 1) cap = 1;
    if (cap > 64) cap = 64;
    int n = (int)(want < cap ? want : cap);
#ifdef TW_TRACE
    if (const char* f = getenv("TW_FORCE_SPLITS")) n = atoi(f) > 0 ? atoi(f) : n;   // diagnostic build: plan sweeps
#endif
    if (n > 1) {
        // whole 32-row chunks per piece, then as few pieces as cover the longest sequence
        const int per = (max_rows + n - 1) / n;
        p.split_rows = (per + 31) / 32 * 32;
        p.n_splits = (int)(((int64_t)max_rows + p.split_rows - 1) / p.split_rows);
    }
    return p;
}


size_t verify_workspace_bytes(int B, int H, int T_max, int d_h, int max_rows) {
    const int ns = verify_plan(B, H, T_max, max_rows).n_splits;
    if (ns == 1) return 0;
    return kVerifyCounterBytes +
           (size_t)ns * B * H * (partial_stride(T_max * d_h) + partial_stride(T_max * 2)) * sizeof(float);
}

}  // namespace tw

#ifdef TW_TRACE
// Diagnostic build only (build.py --trace): the timeline buffer of the verification kernels, and a bare
// read-only stream over `bytes` of memory (16-byte non-temporal loads, eight in flight per lane, `wgs`
// workgroups of 256 lanes) -- what the memory system gives a kernel that does nothing but read.
extern "C" TW_API void tw_debug_set_trace(void* p) { g_trace = (unsigned long long*)p; }

typedef __attribute__((ext_vector_type(4))) unsigned int dbg_u32x4;
__global__ __launch_bounds__(256) void debug_stream_read_kernel(const dbg_u32x4* __restrict__ src, size_t n16,
                                                                unsigned* sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    dbg_u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += 8 * stride) {
        dbg_u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t j = i + u * stride;
            v[u] = __builtin_nontemporal_load(src + (j < n16 ? j : n16 - 1));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1u;   // never true in practice: keeps the loads
}
extern "C" TW_API int32_t tw_debug_stream_read(const void* src, size_t bytes, int32_t wgs, void* sink, void* stream) {
    if (!src || !sink || bytes < 16 || wgs < 1) return TW_ERR_INVALID_ARG;
    hipLaunchKernelGGL(debug_stream_read_kernel, dim3(wgs), dim3(256), 0, (hipStream_t)stream,
                       (const dbg_u32x4*)src, bytes / 16, (unsigned*)sink);
    return hipGetLastError() == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}
#endif

extern "C" {

int32_t tw_version(void) { return 2001; }

size_t tw_workspace_bytes(int32_t which, int32_t B, int32_t rows, int32_t H, int32_t d_h,
                          int32_t max_rows) {
    if (B <= 0 || rows <= 0 || H <= 0 || d_h <= 0 || max_rows <= 0) return 0;
    if (which == TW_CALL_TTP_SCORE) return score_workspace_bytes(B, H, rows, max_rows);
    if (which == TW_CALL_TREE_VERIFY_ATTN) return verify_workspace_bytes(B, H, rows, d_h, max_rows);
    return 0;
}

int32_t tw_ttp_score(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                     const tw_kv_view* k, const int32_t* n_tot, int32_t n_tot_max, int32_t B,
                     int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                     void* ws, size_t ws_bytes, void* stream) {
    return tw_ttp_score_gqa(q_sel, n_q_max, n_q, q_pos0, k, 1, n_tot, n_tot_max, B, v_start, M, scale, causal,
                            scores, ws, ws_bytes, stream);
}

// score, and with kept != NULL the top-R keep of every row inside the last launch
static int32_t score_impl(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                          const tw_kv_view* k, int32_t q_heads_per_kv, const int32_t* n_tot, int32_t n_tot_max,
                          int32_t B, int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                          int32_t R, int32_t* kept, void* ws, size_t ws_bytes, void* stream);

int32_t tw_ttp_score_gqa(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                         const tw_kv_view* k, int32_t q_heads_per_kv, const int32_t* n_tot, int32_t n_tot_max,
                         int32_t B, int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                         void* ws, size_t ws_bytes, void* stream) {
    return score_impl(q_sel, n_q_max, n_q, q_pos0, k, q_heads_per_kv, n_tot, n_tot_max, B, v_start, M, scale, causal,
                      scores, 0, nullptr, ws, ws_bytes, stream);
}

int32_t tw_ttp_score_select(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                            const tw_kv_view* k, const int32_t* n_tot, int32_t n_tot_max, int32_t B, int32_t v_start,
                            int32_t M, float scale, int32_t causal, float* scores, int32_t R, int32_t* kept, void* ws,
                            size_t ws_bytes, void* stream) {
    if (R < 0 || R > M) return TW_ERR_INVALID_ARG;
    if (M > (1 << 20)) return TW_ERR_UNSUPPORTED;
    if (R > 0 && B > 0 && !kept) return TW_ERR_INVALID_ARG;
    return score_impl(q_sel, n_q_max, n_q, q_pos0, k, 1, n_tot, n_tot_max, B, v_start, M, scale, causal, scores, R,
                      R > 0 ? kept : nullptr, ws, ws_bytes, stream);
}

static int32_t score_impl(const void* q_sel, int32_t n_q_max, const int32_t* n_q, const int32_t* q_pos0,
                          const tw_kv_view* k, int32_t q_heads_per_kv, const int32_t* n_tot, int32_t n_tot_max,
                          int32_t B, int32_t v_start, int32_t M, float scale, int32_t causal, float* scores,
                          int32_t R, int32_t* kept, void* ws, size_t ws_bytes, void* stream) {
    if (B < 0 || M < 0 || n_q_max < 1 || n_tot_max < 1 || v_start < 0 || q_heads_per_kv < 1)
        return TW_ERR_INVALID_ARG;
    if (q_heads_per_kv > 64) return TW_ERR_UNSUPPORTED;
    if (B == 0 || M == 0) return TW_OK;
    if (!q_sel || !q_pos0 || !n_tot || !scores || (uintptr_t)q_sel % 16) return TW_ERR_INVALID_ARG;
    const int vs = view_status(k, false);
    if (vs != TW_OK) return vs;
    if ((int64_t)v_start + M > n_tot_max || n_q_max > n_tot_max) return TW_ERR_INVALID_ARG;
    if ((int64_t)k->H * q_heads_per_kv > 65535) return TW_ERR_UNSUPPORTED;
    const int H_q = k->H * q_heads_per_kv;
    const size_t need = score_workspace_bytes(B, H_q, n_q_max, n_tot_max);
    if (!ws || ws_bytes < need) return TW_ERR_WORKSPACE;
    if ((uintptr_t)ws % 16) return TW_ERR_INVALID_ARG;
    ScoreArgs a;
    a.q_sel = q_sel;
    a.k = to_dev(*k);
    a.n_q = n_q;
    a.q_pos0 = q_pos0;
    a.n_tot = n_tot;
    a.scores = scores;
    a.ws = (float*)ws;
    a.n_q_max = n_q_max;
    a.n_tot_max = n_tot_max;
    a.B = B;
    a.H = H_q;
    a.group = q_heads_per_kv;
    a.d_h = k->d_h;
    a.v_start = v_start;
    a.M = M;
    a.causal = causal != 0;
    a.scale = scale;
    a.kept = kept;
    a.R = R;
#ifdef TW_TRACE
    a.trace = g_trace;
    if (const char* d = getenv("TW_SCORE_DRY")) a.dry = atoi(d);
#endif
    return launch_score(a, k->dtype, (hipStream_t)stream) == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}

int32_t tw_ttp_score_phead(const void* q, const void* gq, const tw_kv_view* k, const tw_kv_view* gk,
                           int32_t B, int32_t v_start, int32_t M, float scale, float* scores, void* ws,
                           size_t ws_bytes, void* stream) {
    if (B < 0 || M < 0 || v_start < 0) return TW_ERR_INVALID_ARG;
    if (B == 0 || M == 0) return TW_OK;
    if (!q || !gq || !scores || (uintptr_t)q % 16 || (uintptr_t)gq % 16) return TW_ERR_INVALID_ARG;
    int vs = view_status(k, false);
    if (vs != TW_OK) return vs;
    vs = view_status(gk, false);
    if (vs != TW_OK) return vs;
    if (k->dtype != gk->dtype || k->H != gk->H || k->d_h != gk->d_h) return TW_ERR_UNSUPPORTED;
    if (M > 32768) return TW_ERR_UNSUPPORTED;   // logits of one head are kept in LDS
    if ((int64_t)v_start + M > k->pool_rows || (int64_t)v_start + M > gk->pool_rows) return TW_ERR_INVALID_ARG;
    const size_t need = (size_t)B * k->H * M * sizeof(float);
    if (!ws || ws_bytes < need) return TW_ERR_WORKSPACE;
    PheadArgs a;
    a.q = q;
    a.gq = gq;
    a.k = to_dev(*k);
    a.gk = to_dev(*gk);
    a.scores = scores;
    a.ws = (float*)ws;
    a.B = B;
    a.H = k->H;
    a.d_h = k->d_h;
    a.v_start = v_start;
    a.M = M;
    a.scale = scale;
    return launch_phead(a, k->dtype, (hipStream_t)stream) == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}

int32_t tw_ttp_select(const float* scores, int32_t B, int32_t M, int32_t R, int32_t* kept,
                      void* stream) {
    if (B < 0 || M < 0 || R < 0 || R > M) return TW_ERR_INVALID_ARG;
    if (M > (1 << 20)) return TW_ERR_UNSUPPORTED;
    if (B == 0 || R == 0) return TW_OK;
    if (!scores || !kept) return TW_ERR_INVALID_ARG;
    return launch_select(scores, B, M, R, kept, (hipStream_t)stream) == hipSuccess ? TW_OK
                                                                                   : TW_ERR_LAUNCH;
}

static int32_t compact_tables(const CompactBatch& cb, int B, int n_out_max, const void* const* src,
                              void* const* dst, int n_tensors, size_t row_bytes, hipStream_t s) {
    for (int t0 = 0; t0 < n_tensors; t0 += kCompactMaxTensors) {
        const int n = n_tensors - t0 < kCompactMaxTensors ? n_tensors - t0 : kCompactMaxTensors;
        CompactTable tab;
        for (int t = 0; t < kCompactMaxTensors; ++t) {
            tab.src[t] = t < n ? src[t0 + t] : nullptr;
            tab.dst[t] = t < n ? dst[t0 + t] : nullptr;
        }
        if (launch_compact(cb, B, n_out_max, tab, n, row_bytes, s) != hipSuccess) return TW_ERR_LAUNCH;
    }
    return TW_OK;
}

int32_t tw_ttp_compact(const int32_t* kept, int32_t R, int32_t v_start, int32_t M, int32_t n_tot,
                       const void* const* src, void* const* dst, int32_t n_tensors,
                       size_t row_bytes, void* stream) {
    if (R < 0 || M < 0 || R > M || v_start < 0 || n_tot < 0 || n_tensors < 0) return TW_ERR_INVALID_ARG;
    if ((int64_t)v_start + M > n_tot) return TW_ERR_INVALID_ARG;
    if (n_tensors == 0) return TW_OK;
    if (!src || !dst || row_bytes == 0 || (R > 0 && !kept)) return TW_ERR_INVALID_ARG;
    for (int t = 0; t < n_tensors; ++t)
        if (!src[t] || !dst[t]) return TW_ERR_INVALID_ARG;
    const CompactBatch cb = {kept, nullptr, nullptr, nullptr, n_tot, R, v_start, M};
    return compact_tables(cb, 1, n_tot - M + R, src, dst, n_tensors, row_bytes, (hipStream_t)stream);
}

int32_t tw_ttp_compact_batched(const int32_t* kept, int32_t R, int32_t v_start, int32_t M,
                               const int32_t* n_tot, int32_t n_tot_max, const int32_t* src_row_off,
                               const int32_t* dst_row_off, int32_t B, const void* const* src,
                               void* const* dst, int32_t n_tensors, size_t row_bytes, void* stream) {
    if (R < 0 || M < 0 || R > M || v_start < 0 || n_tot_max < 0 || n_tensors < 0 || B < 0)
        return TW_ERR_INVALID_ARG;
    if ((int64_t)v_start + M > n_tot_max) return TW_ERR_INVALID_ARG;
    if (B > 65535) return TW_ERR_UNSUPPORTED;
    if (n_tensors == 0 || B == 0) return TW_OK;
    if (!src || !dst || row_bytes == 0 || (R > 0 && !kept) || !n_tot || !src_row_off || !dst_row_off)
        return TW_ERR_INVALID_ARG;
    for (int t = 0; t < n_tensors; ++t)
        if (!src[t] || !dst[t]) return TW_ERR_INVALID_ARG;
    const CompactBatch cb = {kept, n_tot, src_row_off, dst_row_off, n_tot_max, R, v_start, M};
    return compact_tables(cb, B, n_tot_max - M + R, src, dst, n_tensors, row_bytes, (hipStream_t)stream);
}

int32_t tw_tree_ancestor_masks(const int32_t* parent, const int32_t* n_nodes, int32_t T_max,
                               int32_t B, uint64_t* masks, void* stream) {
    if (B < 0 || T_max < 1) return TW_ERR_INVALID_ARG;
    if (T_max > TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (!parent || !n_nodes || !masks) return TW_ERR_INVALID_ARG;
    return launch_ancestor_masks(parent, n_nodes, T_max, B, masks, (hipStream_t)stream) == hipSuccess
               ? TW_OK
               : TW_ERR_LAUNCH;
}

int32_t tw_tree_verify_attn(const void* q, const tw_kv_view* k, const tw_kv_view* v,
                            const int32_t* ctx_len, int32_t max_ctx_len, const int32_t* parent,
                            const int32_t* n_nodes, int32_t T_max, int32_t B, float scale,
                            void* out, int32_t out_dtype, void* ws, size_t ws_bytes, void* stream) {
    return tw_tree_verify_attn_gqa(q, k, v, 1, ctx_len, max_ctx_len, parent, n_nodes, T_max, B, scale, out,
                                   out_dtype, ws, ws_bytes, stream);
}

int32_t tw_tree_verify_attn_gqa(const void* q, const tw_kv_view* k, const tw_kv_view* v,
                                int32_t q_heads_per_kv, const int32_t* ctx_len, int32_t max_ctx_len,
                                const int32_t* parent, const int32_t* n_nodes, int32_t T_max, int32_t B,
                                float scale, void* out, int32_t out_dtype, void* ws, size_t ws_bytes,
                                void* stream) {
    if (B < 0 || T_max < 1 || max_ctx_len < 0 || q_heads_per_kv < 1) return TW_ERR_INVALID_ARG;
    if (q_heads_per_kv > 64) return TW_ERR_UNSUPPORTED;
    if (T_max > TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (out_dtype != TW_F32 && out_dtype != TW_BF16) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (!q || !ctx_len || !parent || !n_nodes || !out) return TW_ERR_INVALID_ARG;
    if ((uintptr_t)q % 16 || (uintptr_t)out % 16) return TW_ERR_INVALID_ARG;
    int vs = view_status(k, true);
    if (vs != TW_OK) return vs;
    vs = view_status(v, true);
    if (vs != TW_OK) return vs;
    if (k->dtype != v->dtype || k->H != v->H || k->d_h != v->d_h) return TW_ERR_UNSUPPORTED;
    if ((k->page_table == nullptr) != (v->page_table == nullptr)) return TW_ERR_UNSUPPORTED;
    const int64_t max_rows64 = (int64_t)max_ctx_len + T_max;
    if (max_rows64 > (1ll << 30)) return TW_ERR_UNSUPPORTED;
    const int max_rows = (int)max_rows64;
    VerifyArgs a;
    a.q = q;
    a.out = out;
    a.out_bf16 = out_dtype == TW_BF16;
    a.k = to_dev(*k);
    a.v = to_dev(*v);
    a.ctx_len = ctx_len;
    a.parent = parent;
    a.n_nodes = n_nodes;
    a.T_max = T_max;
    a.B = B;
    if ((int64_t)k->H * q_heads_per_kv > 65535) return TW_ERR_UNSUPPORTED;
    a.H = k->H * q_heads_per_kv;
    a.group = q_heads_per_kv;
    a.d_h = k->d_h;
    a.max_rows = max_rows;
    a.scale = scale;
    const VerifyPlan plan = verify_plan(B, a.H, T_max, max_rows);
    a.n_splits = plan.n_splits;
    a.split_rows = plan.split_rows;
    a.n_blk = plan.n_blk;
    a.n_phase = plan.n_phase;
    a.heads_per_wg = plan.heads_per_wg;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    a.arrive = nullptr;
    a.o_stride = a.ml_stride = 0;
#ifdef TW_TRACE
    a.trace = g_trace;
#endif
    if (a.n_splits > 1) {
        const size_t need = verify_workspace_bytes(B, a.H, T_max, a.d_h, max_rows);
        if (!ws || ws_bytes < need) return TW_ERR_WORKSPACE;
        if ((uintptr_t)ws % 16) return TW_ERR_INVALID_ARG;
        a.arrive = (int32_t*)ws;
        a.o_stride = partial_stride(T_max * a.d_h);
        a.ml_stride = partial_stride(T_max * 2);
        a.part_o = (float*)((char*)ws + kVerifyCounterBytes);
        a.part_ml = a.part_o + (size_t)a.n_splits * B * a.H * a.o_stride;
    }
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (verify_mfma_supported(a, k->dtype))
        e = launch_verify_mfma(a, s);
    else
        e = launch_verify_generic(a, k->dtype, s);
    return e == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}

int32_t tw_tree_accept(const int32_t* draft, const int32_t* argmax, const int32_t* parent,
                       const int32_t* n_nodes, int32_t T_max, int32_t B, int32_t* n_acc,
                       int32_t* path, int32_t* bonus, void* stream) {
    if (B < 0 || T_max < 1) return TW_ERR_INVALID_ARG;
    if (T_max > TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (!draft || !argmax || !parent || !n_nodes || !n_acc || !path || !bonus) return TW_ERR_INVALID_ARG;
    return launch_accept(draft, argmax, parent, n_nodes, T_max, B, n_acc, path, bonus,
                         (hipStream_t)stream) == hipSuccess
               ? TW_OK
               : TW_ERR_LAUNCH;
}

int32_t tw_chain_tree(const float* prob, float theta, int32_t delta, int32_t B, int32_t* parent,
                      int32_t* n_nodes, void* stream) {
    if (B < 0 || delta < 1 || !(theta == theta)) return TW_ERR_INVALID_ARG;
    if (delta >= TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (!parent || !n_nodes) return TW_ERR_INVALID_ARG;
    return launch_chain_tree(prob, theta, delta, B, parent, n_nodes, (hipStream_t)stream) == hipSuccess
               ? TW_OK
               : TW_ERR_LAUNCH;
}

int32_t tw_chain_accept(const int32_t* draft, const int32_t* argmax, const int32_t* n_nodes, int32_t T_max,
                        int32_t B, int32_t* n_acc, int32_t* path, int32_t* bonus, void* stream) {
    if (B < 0 || T_max < 1) return TW_ERR_INVALID_ARG;
    if (T_max > TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (!draft || !argmax || !n_nodes || !n_acc || !path || !bonus) return TW_ERR_INVALID_ARG;
    return launch_chain_accept(draft, argmax, n_nodes, T_max, B, n_acc, path, bonus, (hipStream_t)stream) ==
                   hipSuccess
               ? TW_OK
               : TW_ERR_LAUNCH;
}

int32_t tw_kv_commit(const int32_t* path, const int32_t* n_acc, int32_t T_max, const tw_kv_view* views,
                     int32_t n_views, const int32_t* ctx_len, int32_t B, int32_t* new_ctx_len,
                     void* stream) {
    if (B < 0 || n_views < 0 || T_max < 1) return TW_ERR_INVALID_ARG;
    if (T_max > TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (B > 65535) return TW_ERR_UNSUPPORTED;
    if (!path || !n_acc || !ctx_len || (n_views > 0 && !views)) return TW_ERR_INVALID_ARG;
    for (int v = 0; v < n_views; ++v) {
        if (!views[v].base || views[v].pool_rows <= 0 || views[v].H <= 0 || views[v].d_h <= 0)
            return TW_ERR_INVALID_ARG;
        if (views[v].dtype != TW_F32 && views[v].dtype != TW_BF16) return TW_ERR_UNSUPPORTED;
        if (views[v].page_table ? (views[v].max_pages <= 0 || views[v].page_rows <= 0) : !views[v].row_off)
            return TW_ERR_INVALID_ARG;
    }
    hipStream_t s = (hipStream_t)stream;
    // 32 views per launch; the first launch also writes the new lengths.  With no views at all a
    // launch over one empty view still writes them.
    const int n_launch_views = n_views > 0 ? n_views : (new_ctx_len ? 1 : 0);
    for (int v0 = 0; v0 < n_launch_views; v0 += kCommitMaxViews) {
        CommitArgs a;
        const int n = n_launch_views - v0 < kCommitMaxViews ? n_launch_views - v0 : kCommitMaxViews;
        size_t max_row = 16;
        for (int v = 0; v < kCommitMaxViews; ++v) {
            a.views[v] = KvDev{};
            a.elem_bytes[v] = 0;
            if (v < n && v0 + v < n_views) {
                a.views[v] = to_dev(views[v0 + v]);
                a.elem_bytes[v] = views[v0 + v].dtype == TW_F32 ? 4 : 2;
                const size_t rb = (size_t)views[v0 + v].H * views[v0 + v].d_h * a.elem_bytes[v];
                if (rb > max_row) max_row = rb;
            }
        }
        a.path = path;
        a.n_acc = n_acc;
        a.ctx_len = ctx_len;
        a.new_ctx_len = v0 == 0 ? new_ctx_len : nullptr;
        a.T_max = T_max;
        if (launch_kv_commit(a, n, B, max_row, s) != hipSuccess) return TW_ERR_LAUNCH;
    }
    return TW_OK;
}

int32_t tw_draft_topk(const float* probs, int32_t n, int32_t V, int32_t E, int32_t* ids, float* vals,
                      void* stream) {
    if (n < 0 || V < 0 || E < 0 || E > V) return TW_ERR_INVALID_ARG;
    if (E > 256 || V > (1 << 20)) return TW_ERR_UNSUPPORTED;
    if (n == 0 || E == 0) return TW_OK;
    if (!probs || !ids || !vals) return TW_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    // vocabulary-sized rows with a small E: one read of the row and a short candidate list
    hipError_t err = hipSuccess;
    if (launch_topk_rows(probs, n, V, E, ids, vals, false, s, &err)) return err == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
    // otherwise: radix select of the survivors, then their rank order inside the same workgroup
    return launch_select(probs, n, V, E, ids, s, vals) == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}

int32_t tw_draft_topk_logits(const float* logits, int32_t n, int32_t V, int32_t E, int32_t* ids, float* probs,
                             void* stream) {
    if (n < 0 || V < 0 || E < 0 || E > V) return TW_ERR_INVALID_ARG;
    if (E > 256 || V > (1 << 20)) return TW_ERR_UNSUPPORTED;
    if (n == 0 || E == 0) return TW_OK;
    if (!logits || !ids || !probs) return TW_ERR_INVALID_ARG;
    hipError_t err = hipSuccess;
    if (!launch_topk_rows(logits, n, V, E, ids, probs, true, (hipStream_t)stream, &err)) return TW_ERR_UNSUPPORTED;
    return err == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}

int32_t tw_draft_expand(const int32_t* sel, int32_t n_exp, int32_t prev_off, int32_t out_off, const int32_t* ids,
                        const float* probs, int32_t E, int32_t N, int32_t B, int32_t* cand_parent,
                        int32_t* cand_token, float* cand_prob, float* cand_conf, float* level_conf, void* stream) {
    if (B < 0 || n_exp < 0 || E < 0 || N < 0 || prev_off < 0 || out_off < 0) return TW_ERR_INVALID_ARG;
    if ((int64_t)n_exp * E > 65536 || B > 65535) return TW_ERR_UNSUPPORTED;
    if ((int64_t)out_off + (int64_t)n_exp * E > N) return TW_ERR_INVALID_ARG;
    if (sel ? prev_off >= out_off : n_exp > 1) return TW_ERR_INVALID_ARG;   // a slice to pick from, or the root alone
    if (B == 0 || n_exp == 0 || E == 0) return TW_OK;
    if (!ids || !probs || !cand_parent || !cand_token || !cand_prob || !cand_conf || !level_conf)
        return TW_ERR_INVALID_ARG;
    return launch_draft_expand(sel, n_exp, prev_off, out_off, ids, probs, E, N, B, cand_parent, cand_token, cand_prob,
                               cand_conf, level_conf, (hipStream_t)stream) == hipSuccess
               ? TW_OK
               : TW_ERR_LAUNCH;
}

size_t tw_tree_build_workspace_bytes(int32_t B, int32_t N, int32_t T_max) {
    if (B <= 0 || N <= 0 || T_max <= 1) return 0;
    const int R = T_max - 1 < N ? T_max - 1 : N;
    return (size_t)B * N * sizeof(float) + (size_t)B * R * sizeof(int32_t);
}

int32_t tw_tree_build(const int32_t* cand_parent, const int32_t* cand_token, const float* cand_prob,
                      const int32_t* n_cand, const int32_t* root_token, int32_t N, int32_t B, int32_t T_max,
                      int32_t* parent_out, int32_t* token_out, int32_t* src_out, int32_t* n_nodes_out,
                      void* ws, size_t ws_bytes, void* stream) {
    if (B < 0 || N < 0 || T_max < 1) return TW_ERR_INVALID_ARG;
    if (T_max > TW_MAX_TREE || N > 8192) return TW_ERR_UNSUPPORTED;
    if (B == 0) return TW_OK;
    if (B > 65535) return TW_ERR_UNSUPPORTED;
    if (!n_cand || !root_token || !parent_out || !token_out || !src_out || !n_nodes_out) return TW_ERR_INVALID_ARG;
    if (N > 0 && (!cand_parent || !cand_token || !cand_prob)) return TW_ERR_INVALID_ARG;
    const int R = T_max - 1 < N ? T_max - 1 : N;
    const size_t need = tw_tree_build_workspace_bytes(B, N, T_max);
    if (need > 0 && (!ws || ws_bytes < need)) return TW_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    float* conf = (float*)ws;
    int32_t* kept = (int32_t*)((char*)ws + (size_t)B * N * sizeof(float));
    TreeBuildArgs a;
    a.cand_parent = cand_parent;
    a.cand_token = cand_token;
    a.n_cand = n_cand;
    a.root_token = root_token;
    a.kept = kept;
    a.parent_out = parent_out;
    a.token_out = token_out;
    a.src_out = src_out;
    a.n_nodes_out = n_nodes_out;
    a.N = N;
    a.R = R;
    a.T_max = T_max;
    hipError_t e = hipSuccess;
    if (R > 0 && launch_tree_build_fused(a, cand_prob, conf, B, s, &e)) return e == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
    if (R > 0) {
        if (launch_tree_conf(cand_parent, cand_prob, n_cand, B, N, conf, s) != hipSuccess) return TW_ERR_LAUNCH;
        if (launch_select(conf, B, N, R, kept, s) != hipSuccess) return TW_ERR_LAUNCH;
    }
    return launch_tree_emit(a, B, s) == hipSuccess ? TW_OK : TW_ERR_LAUNCH;
}

int32_t tw_validate_tree(const int32_t* parent_host, int32_t T) {
    if (!parent_host || T < 1) return TW_ERR_INVALID_ARG;
    if (T > TW_MAX_TREE) return TW_ERR_UNSUPPORTED;
    if (parent_host[0] != -1) return TW_ERR_INVALID_ARG;
    for (int i = 1; i < T; ++i)
        if (parent_host[i] < 0 || parent_host[i] >= i) return TW_ERR_INVALID_ARG;
    return TW_OK;
}

int32_t tw_rbar(int32_t M, int32_t K, int32_t R, int32_t K_f, int32_t L) {
    if (L <= 0) return -1;
    const long num = (long)M * K + (long)R * (K_f - K);
    // nearest integer of num / L for non-negative num: floor((2*num + L) / (2*L))
    return (int32_t)((2 * num + L) / (2L * L));
}

}  // extern "C"
