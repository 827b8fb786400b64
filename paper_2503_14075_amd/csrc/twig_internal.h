// Internal declarations shared by the HIP translation units of libtwigpath.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "index_math.h"
#include "twigpath.h"

namespace tw {

// Device-side copy of a tw_kv_view.
struct KvDev {
    const void* base;
    const int32_t* row_off;
    const int32_t* page_table;
    int64_t pool_rows;
    int32_t max_pages, page_rows;
    int32_t page_shift;   // log2(page_rows) when that is a power of two, else -1
    int32_t H, d_h;
};

inline KvDev to_dev(const tw_kv_view& v) {
    KvDev d;
    d.base = v.base;
    d.row_off = v.row_off;
    d.page_table = v.page_table;
    d.pool_rows = v.pool_rows;
    d.max_pages = v.max_pages;
    d.page_rows = v.page_rows > 0 ? v.page_rows : 1;
    d.page_shift = -1;
    for (int sh = 0; sh < 31; ++sh)
        if (d.page_rows == (1 << sh)) d.page_shift = sh;
    d.H = v.H;
    d.d_h = v.d_h;
    return d;
}

// Pool row of cache row r of sequence b, clamped into the pool.
__device__ __forceinline__ int64_t pool_row(const KvDev& kv, int b, int r) {
    r = r < 0 ? 0 : r;   // a row index made from unchecked device contents may have wrapped
    if (kv.page_table) {
        const int pi = page_slot(r, kv.page_rows, kv.page_shift, kv.max_pages);
        return paged_pool_row(kv.page_table[(int64_t)b * kv.max_pages + pi], r, kv.page_rows, kv.page_shift, kv.pool_rows);
    }
    return contiguous_pool_row(kv.row_off[b], r, kv.pool_rows);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }

// fp32 -> bf16, round to nearest even (the hardware conversion), two values in one word
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf2_t __attribute__((ext_vector_type(2)));
    const bf2_t p = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, p);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float x) { return (uint16_t)(pack_bf16x2(x, 0.f) & 0xFFFFu); }

// Four consecutive elements of an attention output (element index i, a multiple of 4) in its dtype.
// `streaming` marks data this kernel does not read again.
__device__ __forceinline__ void store_out4(void* out, int out_bf16, int64_t i, float x, float y, float z, float w,
                                           bool streaming) {
    typedef __attribute__((ext_vector_type(4))) float f4_t;
    typedef __attribute__((ext_vector_type(2))) unsigned int u2_t;
    if (out_bf16) {
        const u2_t v = {pack_bf16x2(x, y), pack_bf16x2(z, w)};
        u2_t* p = (u2_t*)((uint16_t*)out + i);
        if (streaming) __builtin_nontemporal_store(v, p);
        else *p = v;
    } else {
        const f4_t v = {x, y, z, w};
        f4_t* p = (f4_t*)((float*)out + i);
        if (streaming) __builtin_nontemporal_store(v, p);
        else *p = v;
    }
}

// Raw buffer access (buffer_load / buffer_store through a descriptor built in scalar registers):
// the way to give a vector memory instruction all three cache-policy bits of gfx950.  `aux` of the
// builtins: sc0 = 1, nt = 2, sc1 = 16.  Offsets past `bytes` are dropped by the hardware.
constexpr int kAuxSc0 = 1, kAuxNt = 2, kAuxSc1 = 16;
// system scope + streaming: bulk data a kernel touches once (4 % faster row copies than nt alone,
// and, unlike stores without nt, no dirty lines left behind for the next kernel to pay for)
constexpr int kAuxStream = kAuxSc0 | kAuxSc1 | kAuxNt;
// system scope, cached: a modest output written once at the end of a workgroup's life
constexpr int kAuxThrough = kAuxSc0 | kAuxSc1;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void* base, uint32_t bytes) {
    // last descriptor word: untyped 32-bit data (raw dword accesses ignore the format)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// Raises a kernel's dynamic LDS limit to `bytes`, once per device (bit d of `done` = device d has
// it; the limit of a kernel is a per-device attribute).  Devices past 31 set it on every call.  The
// bitmap is the only thing the library remembers between calls; threads may race to set the same
// attribute to the same value, which is harmless, and the bit is published after the attribute.
inline hipError_t raise_lds_limit_once(const void* kernel, int bytes, std::atomic<uint32_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 32 && ((done.load(std::memory_order_acquire) >> dev) & 1u)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 32) done.fetch_or(1u << dev, std::memory_order_release);
    return e;
}

// Ancestor-or-self mask of node i from a parent array held in shared memory.
// Parents are clamped to [0, i) so the walk always ends at the root.
__device__ __forceinline__ uint64_t ancestor_mask(const int* s_parent, int i) {
    uint64_t m = 1ull << i;
    int u = i;
    while (u > 0) {
        const int p = clamp_parent(s_parent[u], u);
        m |= 1ull << p;
        u = p;
    }
    return m;
}

// --- verification attention -------------------------------------------------
struct VerifyArgs {
    const void* q;
    void* out;        // [B][T_max][H][d_h], fp32 or bf16
    int32_t out_bf16;
    KvDev k, v;
    const int32_t* ctx_len;
    const int32_t* parent;
    const int32_t* n_nodes;
    // Partial results of split launches, one slot per (piece, sequence, head).  A slot is a whole number of
    // 128-byte lines (o_stride, ml_stride floats): no line of it is shared with another workgroup's slot.
    float* part_o;   // [n_splits][B][H] slots of [T_max][d_h] unnormalised partial outputs
    float* part_ml;  // [n_splits][B][H] slots of [T_max][2]: running max (natural-log units), running sum
    int32_t o_stride, ml_stride;
    int32_t* arrive; // [B][H] pieces of the unit that have written their partial; zero between launches
    int32_t T_max, B, H, d_h;   // H: query heads = group * (heads of a cache row, k.H)
    int32_t group;              // query heads per key/value head (1: multi-head attention)
    int32_t n_splits, split_rows, max_rows;   // grid.z pieces of split_rows rows (a multiple of 32) each
    int32_t n_blk, n_phase, heads_per_wg;   // wavefront layout of the matrix-core kernel
    float scale;
#ifdef TW_TRACE
    unsigned long long* trace;   // diagnostic build: 8 timestamps / hardware ids per workgroup
#endif
};

// Diagnostic build (-DTW_TRACE, `python -m paper_2503_14075_amd.build --trace`): thread 0 of every
// workgroup of the verification kernels records the 100 MHz wall clock at a few points of its life
// into the buffer handed to tw_debug_set_trace; slot 6 / 7 hold the hardware and XCD ids.
#ifdef TW_TRACE
#define TW_TRACE_MARK(a, slot)                                                                             \
    do {                                                                                                   \
        if ((a).trace && threadIdx.x == 0)                                                                 \
            (a).trace[(blockIdx.x + gridDim.x * (blockIdx.y + (size_t)gridDim.y * blockIdx.z)) * 8 + (slot)] = \
                (slot) == 6 ? (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4)                \
                : (slot) == 7 ? (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20)             \
                              : __builtin_amdgcn_s_memrealtime();                                          \
    } while (0)
#else
#define TW_TRACE_MARK(a, slot)
#endif

// Launch shape of tree verification: heads_per_wg * n_blk * n_phase == 4 wavefronts.
struct VerifyPlan {
    int n_splits, split_rows, n_blk, n_phase, heads_per_wg;
};
VerifyPlan verify_plan(int B, int H, int T_max, int max_rows);
size_t verify_workspace_bytes(int B, int H, int T_max, int d_h, int max_rows);
hipError_t launch_verify_generic(const VerifyArgs& a, int dtype, hipStream_t s);
bool verify_mfma_supported(const VerifyArgs& a, int dtype);
hipError_t launch_verify_mfma(const VerifyArgs& a, hipStream_t s);
// The arrival counters at the start of the workspace: the same 1 KB whatever the shape of the launch (a launch is
// only cut into pieces while it has fewer than 256 (sequence, head) units), so that launches of different
// shapes may share a workspace: none of them writes partial results where another one keeps counters.
constexpr size_t kVerifyCounterBytes = 256 * sizeof(int32_t);
constexpr int kPartialLineFloats = 32;
inline int partial_stride(int floats) { return (floats + kPartialLineFloats - 1) / kPartialLineFloats * kPartialLineFloats; }

// Partial results of a piece travel between workgroups on different XCDs, whose L2s are not kept
// coherent with each other: they are written and read with system-scope accesses (sc0 sc1: written
// through to memory, read from memory), which is cheaper by far than the cache-wide write-back and
// invalidate of a release / acquire fence pair (measured: 40 us of fences on a 36 us launch).
// Addressed through a descriptor over one (piece, sequence, head) slot.
__device__ __forceinline__ void store_partial4(float* slot_base, uint32_t slot_bytes, uint32_t byte_off, float4 v) {
    typedef __attribute__((ext_vector_type(4))) unsigned int u4_t;
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4_t, v), raw_buffer(slot_base, slot_bytes), (int)byte_off,
                                           0, kAuxThrough);
}
__device__ __forceinline__ void store_partial2(float* slot_base, uint32_t slot_bytes, uint32_t byte_off, float2 v) {
    typedef __attribute__((ext_vector_type(2))) unsigned int u2_t;
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u2_t, v), raw_buffer(slot_base, slot_bytes), (int)byte_off,
                                          0, kAuxThrough);
}

// A (sequence, head) unit whose cache rows were cut into n_b > 1 pieces: called by every thread of a
// workgroup (n_threads of them) after it has issued the stores of its piece's partial result
// (store_partial*).  Every thread waits for its own stores to be acknowledged, the workgroup meets,
// and one thread counts the piece in at the unit's counter.  The workgroup that arrives last merges
// the n_b partials in piece order -- the result does not depend on which one that is -- normalises,
// stores, and puts the counter back to zero for the next launch.  No workgroup waits for another.
__device__ inline void finish_split_unit(const VerifyArgs& a, int b, int h, int T, int n_b, int tid, int n_threads) {
    __shared__ int s_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's write-through stores have reached memory
    __syncthreads();
    if (tid == 0) {
        int32_t* cnt = a.arrive + (int64_t)b * a.H + h;
        const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = old == n_b - 1;
        if (s_last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;
    // d_h/4 lanes per node, four output columns each.  A thread owns up to kItems such items and
    // requests the partials of two pieces for all of them before it uses any (the merge is a few
    // microseconds of memory latency: every round of dependent loads counts); the merge itself is
    // the online-softmax update, one piece at a time, in piece order.
    constexpr int kItems = 4, kBatch = 2;
    const int lanes = a.d_h / 4;
    const int64_t split_stride = (int64_t)a.B * a.H;      // slots per piece
    const int64_t unit0 = (int64_t)b * a.H + h;
    const uint32_t o_bytes = (uint32_t)(a.T_max * a.d_h * 4), ml_bytes = (uint32_t)(a.T_max * 8);
    const int n_items = T * lanes;
    for (int idx0 = tid; idx0 < n_items; idx0 += n_threads * kItems) {
        float m[kItems], l[kItems];
        float4 acc[kItems];
#pragma unroll
        for (int u = 0; u < kItems; ++u) {
            m[u] = -INFINITY;
            l[u] = 0.f;
            acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int s0 = 0; s0 < n_b; s0 += kBatch) {
            float2 ml[kBatch][kItems];
            float4 v[kBatch][kItems];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int s = s0 + i < n_b ? s0 + i : n_b - 1;   // past the last piece: re-read it, unused
                const int64_t slot = unit0 + s * split_stride;
                const __amdgpu_buffer_rsrc_t rml = raw_buffer(a.part_ml + slot * a.ml_stride, ml_bytes);
                const __amdgpu_buffer_rsrc_t ro = raw_buffer(a.part_o + slot * a.o_stride, o_bytes);
#pragma unroll
                for (int u = 0; u < kItems; ++u) {
                    // items past the end fall outside the descriptors and read zeros
                    const int idx = idx0 + u * n_threads, t = idx / lanes, c4 = idx - t * lanes;
                    ml[i][u] = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(rml, t * 8, 0, kAuxThrough));
                    v[i][u] = __builtin_bit_cast(
                        float4, __builtin_amdgcn_raw_buffer_load_b128(ro, (t * a.d_h + 4 * c4) * 4, 0, kAuxThrough));
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
#pragma unroll
                for (int u = 0; u < kItems; ++u) {
                    // a piece in which this node saw no key carries max = -inf and is skipped
                    if (s0 + i < n_b && ml[i][u].x != -INFINITY) {
                        const float m_new = fmaxf(m[u], ml[i][u].x);
                        const float keep = expf(m[u] - m_new), w = expf(ml[i][u].x - m_new);
                        l[u] = l[u] * keep + ml[i][u].y * w;
                        acc[u].x = acc[u].x * keep + v[i][u].x * w;
                        acc[u].y = acc[u].y * keep + v[i][u].y * w;
                        acc[u].z = acc[u].z * keep + v[i][u].z * w;
                        acc[u].w = acc[u].w * keep + v[i][u].w * w;
                        m[u] = m_new;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kItems; ++u) {
            const int idx = idx0 + u * n_threads, t = idx / lanes, c4 = idx - t * lanes;
            if (idx < n_items) {
                const float inv = 1.f / l[u];
                store_out4(a.out, a.out_bf16, ((((int64_t)b * a.T_max + t) * a.H + h) * a.d_h) + 4 * c4, acc[u].x * inv,
                           acc[u].y * inv, acc[u].z * inv, acc[u].w * inv, false);
            }
        }
    }
}

// --- pruning score -----------------------------------------------------------
struct ScoreArgs {
    const void* q_sel;
    KvDev k;
    const int32_t* n_q;
    const int32_t* q_pos0;
    const int32_t* n_tot;
    float* scores;
    float* ws;
    float* stats = nullptr;    // per-split row statistics, inside ws (set by the launcher)
    float* rtab = nullptr;     // long-prompt kernel: per-chunk reference maxima, inside ws
    float* etab = nullptr;     // long-prompt kernel: per-chunk exponentials, inside ws
    int32_t n_splits = 1;
    // Scoring rows taken in two launches (rows 0..63, then the rest) by the shared-memory one-pass
    // kernel: a launch covers rows row0 .. row0 + n_q_max - 1 of the q_stride rows that q_sel holds
    // per sequence (q_stride == 0: n_q_max), and n_halves partial planes are added at the end.
    int32_t row0 = 0, q_stride = 0, n_halves = 1;
    int32_t n_q_max, n_tot_max, B, H, d_h, v_start, M, causal;   // H: query heads = group * k.H
    int32_t group = 1;   // query heads per key head (1: multi-head attention)
    float scale;
    // tw_ttp_score_select: the head reduction also keeps the R best of every row (kept [B][R])
    int32_t* kept = nullptr;
    int32_t R = 0;
#ifdef TW_TRACE
    // diagnostic build: per-wavefront timestamps of the register-resident kernel, and how much of its
    // work is switched off at run time (0 nothing; 1 the matrix products and row maxima; 2 also the
    // exponentials; 3 also the column sums; 4 also the Q traffic: the bare K stream and its staging)
    unsigned long long* trace = nullptr;
    int32_t dry = 0;
#endif
};
int score_key_splits(int B, int H, int n_tot_max);
size_t score_workspace_bytes(int B, int H, int n_q_max, int n_tot_max);
hipError_t launch_score(const ScoreArgs& a, int dtype, hipStream_t s);
hipError_t launch_score_reduce(const ScoreArgs& a, hipStream_t s);
bool score_resident_supported(const ScoreArgs& a, int dtype);
bool score_stream_supported(const ScoreArgs& a, int dtype);
size_t score_stream_workspace_floats(int B, int H, int n_q_max, int n_tot_max);
hipError_t launch_score_stream(const ScoreArgs& a, float* tables, hipStream_t s);
hipError_t launch_score_resident(const ScoreArgs& a, hipStream_t s);

// --- pruning score, P-Head form ------------------------------------------------
struct PheadArgs {
    const void* q;    // [B][H][d_h]
    const void* gq;   // [B][H][d_h]
    KvDev k, gk;      // keys and their gates, same layout
    float* scores;    // [B][M]
    float* ws;        // [B][H][M]
    int32_t B, H, d_h, v_start, M;
    float scale;
};
hipError_t launch_phead(const PheadArgs& a, int dtype, hipStream_t s);

// --- select / compact / tree -------------------------------------------------
// ranked_vals non-null (R <= 256): kept comes out in rank order (larger value first, equal values
// lower index first) with the values beside it; null: ascending index order.
hipError_t launch_select(const float* scores, int B, int M, int R, int32_t* kept, hipStream_t s,
                         float* ranked_vals = nullptr);
// Rank-ordered top-E of long rows for small E in one read of the row; false when the shape is
// not one it covers (nothing launched), otherwise *err holds the launch status.
// With `logits` the rows are logits and vals receives the winners' softmax probabilities.
bool launch_topk_rows(const float* x, int n, int V, int E, int32_t* ids, float* vals, bool logits, hipStream_t s,
                      hipError_t* err);

constexpr int kCompactMaxTensors = 64;
struct CompactTable {
    const void* src[kCompactMaxTensors];
    void* dst[kCompactMaxTensors];
};
// One sequence: n_tot/src_off/dst_off null and n_tot_all set.  Batch: device arrays [B].
struct CompactBatch {
    const int32_t* kept;     // [B][R]
    const int32_t* n_tot;    // [B] or null
    const int32_t* src_off;  // [B] first source row of sequence b, or null
    const int32_t* dst_off;  // [B] first destination row, or null
    int32_t n_tot_all, R, v_start, M;   // n_tot_all: the length (n_tot null) or its upper bound
};
hipError_t launch_compact(const CompactBatch& cb, int B, int n_out_max, const CompactTable& tab,
                          int n_tensors, size_t row_bytes, hipStream_t s);

// --- draft-side tree build ------------------------------------------------------
struct TreeBuildArgs {
    const int32_t* cand_parent;  // [B][N]
    const int32_t* cand_token;   // [B][N]
    const int32_t* n_cand;       // [B]
    const int32_t* root_token;   // [B]
    const int32_t* kept;         // [B][R] ascending
    int32_t* parent_out;         // [B][T_max]
    int32_t* token_out;          // [B][T_max]
    int32_t* src_out;            // [B][T_max]
    int32_t* n_nodes_out;        // [B]
    int32_t N, R, T_max;
};
hipError_t launch_tree_conf(const int32_t* cand_parent, const float* cand_prob, const int32_t* n_cand, int B,
                            int N, float* conf, hipStream_t s);
bool launch_tree_build_fused(const TreeBuildArgs& a, const float* cand_prob, float* conf, int B, hipStream_t s,
                             hipError_t* err);
hipError_t launch_tree_emit(const TreeBuildArgs& a, int B, hipStream_t s);
hipError_t launch_draft_expand(const int32_t* sel, int n_exp, int prev_off, int out_off, const int32_t* ids,
                               const float* probs, int E, int N, int B, int32_t* cand_parent, int32_t* cand_token,
                               float* cand_prob, float* cand_conf, float* level_conf, hipStream_t s);

// --- commit of the accepted path ------------------------------------------------
constexpr int kCommitMaxViews = 32;
struct CommitArgs {
    KvDev views[kCommitMaxViews];
    int32_t elem_bytes[kCommitMaxViews];
    const int32_t* path;      // [B][T_max]
    const int32_t* n_acc;     // [B]
    const int32_t* ctx_len;   // [B]
    int32_t* new_ctx_len;     // [B] or null
    int32_t T_max;
};
hipError_t launch_kv_commit(const CommitArgs& a, int n_views, int B, size_t max_row_bytes, hipStream_t s);

hipError_t launch_chain_tree(const float* prob, float theta, int delta, int B, int32_t* parent, int32_t* n_nodes,
                             hipStream_t s);
hipError_t launch_chain_accept(const int32_t* draft, const int32_t* argmx, const int32_t* n_nodes, int T_max, int B,
                               int32_t* n_acc, int32_t* path, int32_t* bonus, hipStream_t s);
hipError_t launch_ancestor_masks(const int32_t* parent, const int32_t* n_nodes, int T_max, int B,
                                 uint64_t* masks, hipStream_t s);
hipError_t launch_accept(const int32_t* draft, const int32_t* argmax, const int32_t* parent,
                         const int32_t* n_nodes, int T_max, int B, int32_t* n_acc, int32_t* path,
                         int32_t* bonus, hipStream_t s);

}  // namespace tw
