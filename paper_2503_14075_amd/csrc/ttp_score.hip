// Pruning score of twig-guided token pruning (Sec. 3.1 Eq. 2-3, head mean as
// in Sec. 5.1 Eq. 7): attention rows of the last text queries, averaged over
// heads and rows, restricted to the visual columns.
//
// The attention map is never materialised.  A (sequence, head) is handled in
// two passes over its keys:
//   pass 1  logits of every scoring row against every visible key -> per-row
//           running (max, sum) only;
//   pass 2  logits against the visual keys again (re-read from cache, not
//           stored), weights exp(logit - max)/sum, summed over the scoring rows
//           per key -> partial[b][h][m] in the workspace.
// score_reduce then adds the heads in a fixed order.  No floating-point
// atomics: results are bit-identical from run to run.
//
// A launch with few (sequence, head) pairs and long sequences splits the keys
// over workgroups instead, in two launches: the first leaves per-row
// (max, sum) of every key split in the workspace, the second merges them in
// split order and takes one share of the visual columns per workgroup.
//
// bf16 with d_h 64/128 and at most 128 scoring rows runs on the matrix cores:
// one wavefront per head, 32-key chunks staged through LDS exactly as in the
// verification kernel.  Pass 1 forms K.Q^T (a lane owns one scoring row, so
// the row statistics need no cross-lane traffic inside the loop); pass 2 forms
// Q.K^T with the same register fragments swapped (a lane owns one key, so the
// sum over scoring rows is in-lane).  Everything else takes the generic fp32
// vector path.
#include "mfma_util.h"
#include "select_block.h"
#include "twig_internal.h"

namespace tw {

// ============================================================================
// matrix-core path
// ============================================================================
constexpr int kScMfThreads = 256;
constexpr int kScChunk = 32;

template <int DH>
struct ScCfg {
    static constexpr int kRowB = DH * 2;
    static constexpr int kKStride = kRowB + 16;
    static constexpr int kLanesPerRow = kRowB / 16;
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;
    static constexpr int kLoads = kScChunk / kRowsPerLoad;
    static constexpr int kDC = DH / 16;
    static constexpr int kWaveLds = kScChunk * kKStride + 128 * 4;   // K chunk + per-row statistics
};

// MODE 0: both passes, one wavefront per (sequence, head).  MODE 1: row statistics of key split
// blockIdx.z only.  MODE 2: merge the statistics of all splits, then the weights of column split
// blockIdx.z.
template <int DH, int NB, int MODE>
__global__ __launch_bounds__(kScMfThreads, (NB <= 2 ? 2 : 1)) void score_mfma_kernel(ScoreArgs a) {
    using Cf = ScCfg<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, li = lane & 31;
    const int b = blockIdx.y, h = blockIdx.x * 4 + wave;
    if (h >= a.H) return;
    const ScoreSeq sq = score_seq_from(a.n_q ? a.n_q[b] : a.n_q_max, a.n_tot[b], a.q_pos0[b], a.n_q_max, 0, a.n_q_max,
                                       a.n_tot_max);
    const int n_q = sq.n_q, n_tot = sq.n_tot, pos0 = sq.pos0;
    float* partial = a.ws + ((int64_t)b * a.H + h) * a.M;
    const int split = MODE == 0 ? 0 : blockIdx.z;
    float2* stats = (float2*)a.stats + (((int64_t)b * a.H + h) * a.n_splits) * (32 * NB);   // [split][row]
    if (n_tot == 0) {
        if (MODE != 1 && split == 0)
            for (int m = lane; m < a.M; m += 64) partial[m] = 0.f;
        return;
    }
    unsigned char* ldsK = lds + wave * Cf::kWaveLds;
    float* s_stat = (float*)(ldsK + kScChunk * Cf::kKStride);

    // Q fragments: lane (i, g) holds Q[row 32nb+i][16c + 8g .. +7]; rows past n_q are zero
    bf16x8 qf[NB][Cf::kDC];
    const uint16_t* qb = (const uint16_t*)a.q_sel;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int i = 32 * nb + li;
        const int ic = i < n_q ? i : n_q - 1;
        const u32x4* src = (const u32x4*)(qb + (((int64_t)b * a.n_q_max + ic) * a.H + h) * DH + 8 * g);
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            u32x4 v = src[2 * c];
            if (i >= n_q) v = (u32x4){0u, 0u, 0u, 0u};
            qf[nb][c] = as_bf16x8(v);
        }
    }
    const float sl2 = a.scale * kLog2e;

    const int ld_row = lane / Cf::kLanesPerRow, ld_col = lane % Cf::kLanesPerRow;
    // a cache row holds the key heads; query head h reads key head h / group
    const unsigned char* kbase = (const unsigned char*)a.k.base + (int64_t)(h / a.group) * Cf::kRowB + ld_col * 16;
    const int64_t pool_stride = (int64_t)a.k.H * Cf::kRowB;
    const int64_t last_pool_row = a.k.pool_rows - 1;
    const int64_t row0 = (int64_t)a.k.row_off[b];
    u32x4 pk[Cf::kLoads];
    auto issue_loads = [&](int base, int end) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            int r = base + ld_row + Cf::kRowsPerLoad * j;
            r = r < end - 1 ? r : end - 1;   // past the end: re-read the last key (cached), masked below
            const int64_t prow = clampl(row0 + r, 0, last_pool_row);
            // streaming hint on both passes: 13-23 % faster on 4..64 prompts of 3008 keys
            pk[j] = __builtin_nontemporal_load((const u32x4*)(kbase + prow * pool_stride));
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j)
            *(u32x4*)(ldsK + (ld_row + Cf::kRowsPerLoad * j) * Cf::kKStride + ld_col * 16) = pk[j];
    };
    auto lds_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // keys visible to scoring row i: j < vis_end(i)
    const int vis_all = a.causal ? min(pos0 + 1, n_tot) : n_tot;   // visible to every row

    // ---- pass 1: per-row (max, sum) over all visible keys ----------------------
    float run_m[NB], run_l[NB];
    int vis_end[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        run_m[nb] = -INFINITY;
        run_l[nb] = 0.f;
        vis_end[nb] = a.causal ? min(pos0 + 32 * nb + li + 1, n_tot) : n_tot;
    }
    // key range of pass 1: everything, or this split's share in whole chunks
    int k_begin = 0, k_end = n_tot;
    if (MODE == 1) {
        const int per = ((n_tot + a.n_splits - 1) / a.n_splits + kScChunk - 1) / kScChunk * kScChunk;
        k_begin = min(split * per, n_tot);
        k_end = min(k_begin + per, n_tot);
    }
    // column range of pass 2: the chunks that cover the visual span, or this split's share of them
    const int span_end = a.v_start + a.M;
    int c_begin = a.v_start / kScChunk * kScChunk, c_end = span_end;
    if (MODE == 2) {
        const int chunks = (span_end - c_begin + kScChunk - 1) / kScChunk;
        const int per = (chunks + a.n_splits - 1) / a.n_splits * kScChunk;
        c_begin = min(c_begin + split * per, span_end);
        c_end = min(c_begin + per, span_end);
    }
    const int c_load_end = max(1, min(c_end, n_tot));
    if (MODE != 2) issue_loads(k_begin, k_end);   // k_end >= 1 here
    for (int base = k_begin; MODE != 2 && base < k_end; base += kScChunk) {
        stage();
        issue_loads(base + kScChunk, k_end);
        lds_sync();
        floatx16 s[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[nb][r] = 0.f;
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            const bf16x8 kf = as_bf16x8(*(const u32x4*)(ldsK + li * Cf::kKStride + 32 * c + 16 * g));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nb][c], s[nb], 0, 0, 0);
        }
        const bool need_mask = base + kScChunk > vis_all;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float x[16], mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                x[r] = s[nb][r] * sl2;
                if (need_mask && base + acc_row(r, g) >= vis_end[nb]) x[r] = -INFINITY;
                mx = fmaxf(mx, x[r]);
            }
            const float m_new = fmaxf(run_m[nb], mx);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) psum += fast_exp2(x[r] - m_safe);
            run_l[nb] = run_l[nb] * fast_exp2(run_m[nb] - m_safe) + psum;
            run_m[nb] = m_new;
        }
    }
    if (MODE == 2) {
        issue_loads(c_begin, c_load_end);   // in flight while the statistics are merged
        // (max, sum) of row i over all key splits, merged in split order; both lane groups compute it
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float2* st = stats + 32 * nb + li;
            float m = -INFINITY, l = 0.f;
            for (int s0 = 0; s0 < a.n_splits; s0 += 4) {
                float2 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = st[(int64_t)min(s0 + u, a.n_splits - 1) * (32 * NB)];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (s0 + u >= a.n_splits) continue;
                    const float m_new = fmaxf(m, v[u].x);
                    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                    l = l * fast_exp2(m - m_safe) + v[u].y * fast_exp2(v[u].x - m_safe);
                    m = m_new;
                }
            }
            run_m[nb] = m;
            run_l[nb] = g == 0 ? l : 0.f;   // the lane-group merge below adds the two halves
        }
    }
    // merge the two lane groups of a row; publish max + log2(sum) per row
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float om = __shfl_xor(run_m[nb], 32, 64), ol = __shfl_xor(run_l[nb], 32, 64);
        const float m = fmaxf(run_m[nb], om);
        const float m_safe = m == -INFINITY ? 0.f : m;
        const float l = run_l[nb] * fast_exp2(run_m[nb] - m_safe) + ol * fast_exp2(om - m_safe);
        const int i = 32 * nb + li;
        if (MODE == 1) {
            if (g == 0) stats[(int64_t)split * (32 * NB) + i] = make_float2(m, l);
        } else if (g == 0) {
            s_stat[i] = (i < n_q && l > 0.f) ? m + log2f(l) : INFINITY;   // +inf: row contributes nothing
        }
    }
    if (MODE == 1) return;
    lds_sync();
    float mc[NB][16];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mc[nb][r] = s_stat[32 * nb + acc_row(r, g)];

    // ---- pass 2: weights on the visual keys, summed over scoring rows -----------
    if (MODE != 2) issue_loads(c_begin, c_load_end);
    for (int base = c_begin; base < c_end; base += kScChunk) {
        lds_sync();   // fragment reads of the previous chunk are complete before it is overwritten
        stage();
        issue_loads(base + kScChunk, c_load_end);
        lds_sync();
        floatx16 d[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) d[nb][r] = 0.f;
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            const bf16x8 kf = as_bf16x8(*(const u32x4*)(ldsK + li * Cf::kKStride + 32 * c + 16 * g));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                d[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[nb][c], kf, d[nb], 0, 0, 0);
        }
        const int j = base + li;   // this lane's key
        const bool need_mask = base + kScChunk > vis_all;
        float acc = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float x = fmaf(d[nb][r], sl2, -mc[nb][r]);
                if (need_mask) {
                    const int i = 32 * nb + acc_row(r, g);
                    const int ve = a.causal ? min(pos0 + i + 1, n_tot) : n_tot;
                    if (j >= ve) x = -INFINITY;
                }
                acc += fast_exp2(x);
            }
        }
        acc += __shfl_xor(acc, 32, 64);
        if (g == 0 && j >= a.v_start && j < span_end) partial[j - a.v_start] = acc;
    }
}

// ============================================================================
// generic path (fp32 inputs, other head sizes, more than 128 scoring rows)
// ============================================================================
constexpr int kScThreads = 256;
constexpr int kScRows = 16;   // scoring rows per block of the inner loop
constexpr int kScKeys = 64;   // keys per tile

template <typename TIn>
__device__ __forceinline__ void load8(const TIn* p, float* dst);

template <>
__device__ __forceinline__ void load8<float>(const float* p, float* dst) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w;
    dst[4] = b.x; dst[5] = b.y; dst[6] = b.z; dst[7] = b.w;
}

template <>
__device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, float* dst) {
    const uint4 a = *(const uint4*)p;
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        dst[2 * e] = __uint_as_float(w[e] << 16);
        dst[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
    }
}

// grid (H, B).  The workgroup walks the scoring rows of its (sequence, head) in
// blocks of 16; lane (i, kg) = (tid / 16, tid % 16) owns row i and keys kg + 16*jj
// of each 64-key tile.
template <typename TIn>
__global__ __launch_bounds__(kScThreads) void score_generic_kernel(ScoreArgs a) {
    extern __shared__ float smem[];
    const int d_h = a.d_h, ld = d_h + 1;
    float* sQ = smem;                    // [kScRows][ld], pre-multiplied by scale
    float* sK = sQ + kScRows * ld;       // [kScKeys][ld]
    float* sP = sK + kScKeys * ld;       // [kScRows][kScKeys + 1]
    __shared__ float s_m[kScRows], s_l[kScRows];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const ScoreSeq sq = score_seq_from(a.n_q ? a.n_q[b] : a.n_q_max, a.n_tot[b], a.q_pos0[b], a.n_q_max, 0, a.n_q_max,
                                       a.n_tot_max);
    const int n_q = sq.n_q, n_tot = sq.n_tot, pos0 = sq.pos0;
    const TIn* q = (const TIn*)a.q_sel;
    const TIn* kbase = (const TIn*)a.k.base;
    const int c8n = d_h / 8;
    float* partial = a.ws + ((int64_t)b * a.H + h) * a.M;
    const int i = tid / 16, kg = tid % 16;
    const int span_end = a.v_start + a.M;

    auto load_keys = [&](int base) {
        for (int idx = tid; idx < kScKeys * c8n; idx += kScThreads) {
            const int r = idx / c8n, c8 = idx % c8n;
            float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (base + r < n_tot)
                load8<TIn>(kbase + (pool_row(a.k, b, base + r) * a.k.H + h / a.group) * d_h + c8 * 8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) sK[r * ld + c8 * 8 + e] = v[e];
        }
    };

    for (int row0 = 0; row0 < n_q; row0 += kScRows) {
        __syncthreads();
        for (int idx = tid; idx < kScRows * c8n; idx += kScThreads) {
            const int ii = idx / c8n, c8 = idx % c8n;
            float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (row0 + ii < n_q)
                load8<TIn>(q + (((int64_t)b * a.n_q_max + row0 + ii) * a.H + h) * d_h + c8 * 8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) sQ[ii * ld + c8 * 8 + e] = v[e] * a.scale;
        }
        const int i_abs = row0 + i;
        const bool row_ok = i_abs < n_q;
        const int n_vis = !row_ok ? 0 : (a.causal ? min(pos0 + i_abs + 1, n_tot) : n_tot);
        // ---- pass 1 ----
        float run_m = -INFINITY, run_l = 0.f;
        for (int base = 0; base < n_tot; base += kScKeys) {
            __syncthreads();
            load_keys(base);
            __syncthreads();
            float dot[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
            for (int c = 0; c < d_h; ++c) {
                const float qv = sQ[i * ld + c];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) dot[jj] = fmaf(qv, sK[(kg + 16 * jj) * ld + c], dot[jj]);
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if (base + kg + 16 * jj < n_vis) {
                    const float m_new = fmaxf(run_m, dot[jj]);
                    run_l = run_l * expf(run_m - m_new) + expf(dot[jj] - m_new);
                    run_m = m_new;
                }
            }
        }
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            const float om = __shfl_xor(run_m, off, 64), ol = __shfl_xor(run_l, off, 64);
            const float m_new = fmaxf(run_m, om);
            const float sa = run_m == -INFINITY ? 0.f : expf(run_m - m_new);
            const float sb = om == -INFINITY ? 0.f : expf(om - m_new);
            run_l = run_l * sa + ol * sb;
            run_m = m_new;
        }
        if (kg == 0) {
            s_m[i] = run_m;
            s_l[i] = run_l;
        }
        // ---- pass 2 over the tiles that touch the visual span ----
        for (int base = a.v_start / kScKeys * kScKeys; base < span_end; base += kScKeys) {
            __syncthreads();
            load_keys(base);
            __syncthreads();
            float dot[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
            for (int c = 0; c < d_h; ++c) {
                const float qv = sQ[i * ld + c];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) dot[jj] = fmaf(qv, sK[(kg + 16 * jj) * ld + c], dot[jj]);
            }
            const float m = s_m[i], l = s_l[i];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int j = base + kg + 16 * jj;
                sP[i * (kScKeys + 1) + kg + 16 * jj] = j < n_vis ? expf(dot[jj] - m) / l : 0.f;
            }
            __syncthreads();
            if (tid < kScKeys) {
                const int j = base + tid;
                if (j >= a.v_start && j < span_end) {
                    float sum = 0.f;
#pragma unroll
                    for (int ii = 0; ii < kScRows; ++ii) sum += sP[ii * (kScKeys + 1) + tid];
                    // this lane is the only writer of the slot for the whole kernel
                    partial[j - a.v_start] = row0 == 0 ? sum : partial[j - a.v_start] + sum;
                }
            }
        }
    }
}

// scores[b][m] = mean over heads and scoring rows; the planes of partial sums (one per head, and
// per half of the scoring rows when they were taken in two launches) are added in index order.
__global__ __launch_bounds__(256) void score_reduce_kernel(ScoreArgs a) {
    const int b = blockIdx.y, m = blockIdx.x * 256 + threadIdx.x;
    if (m >= a.M) return;
    const int q_rows = a.q_stride ? a.q_stride : a.n_q_max;
    int n_q = a.n_q ? a.n_q[b] : q_rows;
    n_q = n_q < 1 ? 1 : (n_q > q_rows ? q_rows : n_q);
    float acc = 0.f;
    for (int half = 0; half < a.n_halves; ++half) {
        const float* p = a.ws + ((int64_t)half * a.B + b) * a.H * a.M + m;
        int h = 0;
        for (; h + 8 <= a.H; h += 8) {   // eight independent loads in flight, added in head order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = p[(int64_t)(h + u) * a.M];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; h < a.H; ++h) acc += p[(int64_t)h * a.M];
    }
    a.scores[(int64_t)b * a.M + m] = acc / ((float)a.H * (float)n_q);
}

// The same head reduction followed, inside the launch, by the top-R keep of the row (TopR of
// Sec. 3.1 Eq. 3) for rows of up to 1024 scores: one workgroup of 1024 lanes per sequence, a lane
// per column (all loads of a batch in flight together, heads added in the order of
// score_reduce_kernel so the scores are bit-identical).  Each lane writes its score and the select
// reads it back through the same lane, so no other lane's write is ever read.
constexpr int kFusedSelectMaxM = 1024;
__global__ __launch_bounds__(1024) void score_reduce_select_kernel(ScoreArgs a) {
    const int b = blockIdx.x, m = threadIdx.x;
    if (m < a.M) {
        const int q_rows = a.q_stride ? a.q_stride : a.n_q_max;
        const int n_q = clampi(a.n_q ? a.n_q[b] : q_rows, 1, q_rows);
        float acc = 0.f;
        for (int half = 0; half < a.n_halves; ++half) {
            const float* p = a.ws + ((int64_t)half * a.B + b) * a.H * a.M + m;
            int h = 0;
            for (; h + 8 <= a.H; h += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = p[(int64_t)(h + u) * a.M];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += v[u];
            }
            for (; h < a.H; ++h) acc += p[(int64_t)h * a.M];
        }
        a.scores[(int64_t)b * a.M + m] = acc / ((float)a.H * (float)n_q);
    }
    select_block<1, 1024>(a.scores + (int64_t)b * a.M, a.M, a.R, a.kept + (int64_t)b * a.R, nullptr);
}

// Key splits of the two-pass matrix-core kernel: up to 256 workgroups in all (more brought
// nothing in timing sweeps over 1..16 sequences of 700..3000 keys, and cost time with 128
// scoring rows, where a compute unit holds one workgroup), at least two 32-key chunks per split.
int score_key_splits(int B, int H, int n_tot_max) {
    const long wgs = (long)B * ((H + 3) / 4);
    if (wgs <= 0 || wgs >= 256) return 1;
    long want = (256 + wgs - 1) / wgs, cap = n_tot_max / 64;
    want = want < cap ? want : cap;
    return (int)(want < 1 ? 1 : (want > 32 ? 32 : want));
}

// Workspace layout, in floats: per-head partial sums (at most n_tot_max visual keys) | (max, sum)
// of up to 128 scoring rows per (sequence, head, key split) | tables of the long-prompt kernel.
// Every part starts 16-byte aligned.
constexpr int kLongPrompt = 768;   // longest prompt the shared-memory one-pass kernel takes
static size_t score_partial_floats(int B, int H, int n_tot_max, int n_q_max = 0) {
    // two planes per head when 65..128 scoring rows may be taken in two launches
    const size_t planes = n_q_max > 64 && n_tot_max <= kLongPrompt ? 2 : 1;
    return (planes * B * H * n_tot_max + 3) / 4 * 4;
}
static size_t score_stats_floats(int B, int H, int n_tot_max) {
    return (size_t)B * H * score_key_splits(B, H, n_tot_max) * 128 * 2;
}

size_t score_workspace_bytes(int B, int H, int n_q_max, int n_tot_max) {
    size_t n = score_partial_floats(B, H, n_tot_max, n_q_max) + score_stats_floats(B, H, n_tot_max);
    if (n_q_max <= 32 && n_tot_max > kLongPrompt) n += score_stream_workspace_floats(B, H, n_q_max, n_tot_max);
    return n * sizeof(float);
}

template <int DH, int NB>
static hipError_t launch_score_mfma(const ScoreArgs& a0, hipStream_t s) {
    ScoreArgs a = a0;
    const size_t lds = 4 * (size_t)ScCfg<DH>::kWaveLds;
    a.n_splits = score_key_splits(a.B, a.H, a.n_tot_max);
    a.stats = a.ws + score_partial_floats(a.B, a.H, a.n_tot_max, a.n_q_max);
    const dim3 grid((a.H + 3) / 4, a.B, a.n_splits);
    if (a.n_splits == 1) {
        hipLaunchKernelGGL((score_mfma_kernel<DH, NB, 0>), grid, dim3(kScMfThreads), lds, s, a);
    } else {
        hipLaunchKernelGGL((score_mfma_kernel<DH, NB, 1>), grid, dim3(kScMfThreads), lds, s, a);
        hipLaunchKernelGGL((score_mfma_kernel<DH, NB, 2>), grid, dim3(kScMfThreads), lds, s, a);
    }
    return hipGetLastError();
}

template <int DH>
static hipError_t launch_score_mfma_rows(const ScoreArgs& a, hipStream_t s) {
    if (a.n_q_max <= 32) return launch_score_mfma<DH, 1>(a, s);
    if (a.n_q_max <= 64) return launch_score_mfma<DH, 2>(a, s);
    return launch_score_mfma<DH, 4>(a, s);
}

hipError_t launch_score_reduce(const ScoreArgs& a, hipStream_t s) {
    if (a.kept && a.R > 0 && a.M <= kFusedSelectMaxM) {
        hipLaunchKernelGGL(score_reduce_select_kernel, dim3(a.B), dim3(1024), 0, s, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(score_reduce_kernel, dim3((a.M + 255) / 256, a.B), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.kept && a.R > 0) e = launch_select(a.scores, a.B, a.M, a.R, a.kept, s);
    return e;
}

hipError_t launch_score(const ScoreArgs& a, int dtype, hipStream_t s) {
    if (a.B == 0 || a.M == 0) return hipSuccess;
    hipError_t e;
    ScoreArgs lo = a;   // rows 0..63 of a 65..128-row request
    lo.n_q_max = 64;
    lo.q_stride = a.n_q_max;
    if (score_resident_supported(a, dtype)) {
        e = launch_score_resident(a, s);
    } else if (a.n_q_max > 64 && a.n_q_max <= 128 && score_resident_supported(lo, dtype)) {
        // the shared-memory one-pass kernel twice: rows 0..63, then rows 64.. into a second plane
        ScoreArgs hi = lo;
        hi.row0 = 64;
        hi.n_q_max = a.n_q_max - 64;
        hi.ws = a.ws + (size_t)a.B * a.H * a.M;
        e = launch_score_resident(lo, s);
        if (e == hipSuccess) e = launch_score_resident(hi, s);
        if (e != hipSuccess) return e;
        ScoreArgs all = a;
        all.n_halves = 2;
        return launch_score_reduce(all, s);
    } else if (score_stream_supported(a, dtype) && a.n_tot_max > kLongPrompt) {
        ScoreArgs al = a;
        al.n_splits = score_key_splits(a.B, a.H, a.n_tot_max);
        al.stats = a.ws + score_partial_floats(a.B, a.H, a.n_tot_max);
        e = launch_score_stream(al, al.stats + score_stats_floats(a.B, a.H, a.n_tot_max), s);
    } else if (dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.n_q_max <= 128) {
        e = a.d_h == 128 ? launch_score_mfma_rows<128>(a, s) : launch_score_mfma_rows<64>(a, s);
    } else {
        const size_t lds = ((size_t)(kScRows + kScKeys) * (a.d_h + 1) + (size_t)kScRows * (kScKeys + 1)) *
                           sizeof(float);
        if (dtype == TW_F32)
            hipLaunchKernelGGL(score_generic_kernel<float>, dim3(a.H, a.B), dim3(kScThreads), lds, s, a);
        else
            hipLaunchKernelGGL(score_generic_kernel<uint16_t>, dim3(a.H, a.B), dim3(kScThreads), lds, s, a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    return launch_score_reduce(a, s);
}

}  // namespace tw
