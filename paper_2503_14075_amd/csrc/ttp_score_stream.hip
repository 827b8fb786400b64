// Pruning score for long prompts (Sec. 3.1 Eq. 2-3, head mean as in Sec. 5.1 Eq. 7): one read of
// the keys, at most 32 scoring rows, any prompt length.
//
// The normaliser of a scoring row is known only after its last key, and a score is a sum over
// rows, so the weights cannot be summed while the keys stream by.  Instead of reading the keys a
// second time, the stream kernel leaves, per 32-key chunk of the visual span, the exponentials
// exp2(logit - m) in fp32 (m = the row's running maximum after that chunk, kept beside them),
// 4 bytes per (row, key) against the 2 * d_h bytes of a key.  The weights kernel then scales
// each chunk by exp2(m - final maximum) / final sum and adds the rows.
//
//   score_stream_kernel          grid (ceil(H / 4), B, key splits), one wavefront per head:
//                                K chunk -> LDS -> K.Q^T on the matrix cores (a lane owns one
//                                scoring row), online (max, sum), table rows out through an LDS
//                                transpose as whole 128-byte lines; per-split (max, sum) per row.
//   score_stream_weights_kernel  grid (ceil(span chunks / 8), H, B): merges the splits'
//                                statistics in split order; a lane owns 4 keys of one chunk and
//                                adds the table rows in row order.
//   score_reduce_kernel          adds the heads in index order (shared with the other kernels).
//
// Every weight is fp32 from the logit to the column sum.
#include "mfma_util.h"
#include "twig_internal.h"

namespace tw {

constexpr int kStThreads = 256;
constexpr int kStChunk = 32;
constexpr int kStTrStride = 144;  // bytes per row of the transpose area (32 floats, padded): 16-byte aligned

template <int DH>
struct StCfg {
    static constexpr int kRowB = DH * 2;
    static constexpr int kKStride = kRowB + 16;
    static constexpr int kLanesPerRow = kRowB / 16;
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;
    static constexpr int kLoads = kStChunk / kRowsPerLoad;
    static constexpr int kDC = DH / 16;
    static constexpr int kWaveLds = kStChunk * kKStride + 32 * kStTrStride;   // K chunk + transpose area
};

// Rows of the table kept per chunk: the scoring rows rounded up to a multiple of 8.
__host__ __device__ inline int stream_table_rows(int n_q_max) { return (n_q_max + 7) / 8 * 8; }
// Chunks that can touch a visual span inside n_tot_max keys.
__host__ __device__ inline int stream_max_chunks(int n_tot_max) { return n_tot_max / kStChunk + 2; }

template <int DH>
__global__ __launch_bounds__(kStThreads, 2) void score_stream_kernel(ScoreArgs a) {
    using Cf = StCfg<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, li = lane & 31;
    const int b = blockIdx.y, h = blockIdx.x * 4 + wave, split = blockIdx.z;
    if (h >= a.H) return;
    const ScoreSeq sq = score_seq_from(a.n_q ? a.n_q[b] : a.n_q_max, a.n_tot[b], a.q_pos0[b], a.n_q_max, 0, a.n_q_max,
                                       a.n_tot_max);
    const int n_q = sq.n_q, n_tot = sq.n_tot, pos0 = sq.pos0;
    if (n_tot == 0) return;   // the weights kernel writes zeros without looking at the table
    unsigned char* ldsK = lds + wave * Cf::kWaveLds;
    unsigned char* s_tr = ldsK + kStChunk * Cf::kKStride;

    // Q fragments: lane (i, g) holds Q[row i][16c + 8g .. +7]; rows past n_q are zero
    bf16x8 qf[Cf::kDC];
    {
        const int ic = li < n_q ? li : n_q - 1;
        const u32x4* src =
            (const u32x4*)((const uint16_t*)a.q_sel + (((int64_t)b * a.n_q_max + ic) * a.H + h) * DH + 8 * g);
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            u32x4 v = src[2 * c];
            if (li >= n_q) v = (u32x4){0u, 0u, 0u, 0u};
            qf[c] = as_bf16x8(v);
        }
    }
    const float sl2 = a.scale * kLog2e;

    const int ld_row = lane / Cf::kLanesPerRow, ld_col = lane % Cf::kLanesPerRow;
    // a cache row holds the key heads; query head h reads key head h / group
    const unsigned char* kbase = (const unsigned char*)a.k.base + (int64_t)(h / a.group) * Cf::kRowB + ld_col * 16;
    const int64_t pool_stride = (int64_t)a.k.H * Cf::kRowB;
    const int64_t last_pool_row = a.k.pool_rows - 1;
    const int64_t row0 = (int64_t)a.k.row_off[b];
    // this split's share of the keys, in whole chunks
    const int per = ((n_tot + a.n_splits - 1) / a.n_splits + kStChunk - 1) / kStChunk * kStChunk;
    const int k_begin = min(split * per, n_tot), k_end = min(k_begin + per, n_tot);   // k_end >= 1
    u32x4 pk[Cf::kLoads];
    auto issue_loads = [&](int base) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            int r = base + ld_row + Cf::kRowsPerLoad * j;
            r = r < k_end - 1 ? r : k_end - 1;   // past the end: re-read the last key (cached), masked below
            const int64_t prow = clampl(row0 + r, 0, last_pool_row);
            pk[j] = __builtin_nontemporal_load((const u32x4*)(kbase + prow * pool_stride));   // streamed once
        }
    };
    auto lds_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    const int vis_all = a.causal ? min(pos0 + 1, n_tot) : n_tot;            // keys visible to every row
    const int vis_end = a.causal ? min(pos0 + li + 1, n_tot) : n_tot;       // keys visible to row li
    const int span_end = a.v_start + a.M, c_base = a.v_start / kStChunk * kStChunk;
    const int e_rows = stream_table_rows(a.n_q_max), max_chunks = stream_max_chunks(a.n_tot_max);
    const int64_t unit = (int64_t)b * a.H + h;
    float* etab = a.etab + unit * max_chunks * e_rows * kStChunk;
    float* rtab = a.rtab + unit * max_chunks * 32;

    float run_m = -INFINITY, run_l = 0.f;   // run_l: this lane group's share of the row sum
    issue_loads(k_begin);
    for (int base = k_begin; base < k_end; base += kStChunk) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j)
            *(u32x4*)(ldsK + (ld_row + Cf::kRowsPerLoad * j) * Cf::kKStride + ld_col * 16) = pk[j];
        issue_loads(base + kStChunk);
        lds_sync();
        floatx16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            const bf16x8 kf = as_bf16x8(*(const u32x4*)(ldsK + li * Cf::kKStride + 32 * c + 16 * g));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], s, 0, 0, 0);
        }
        // register r of lane (row li, group g) is key base + acc_row(r, g)
        const bool need_mask = base + kStChunk > vis_all;
        float x[16], mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            x[r] = s[r] * sl2;
            if (need_mask && base + acc_row(r, g) >= vis_end) x[r] = -INFINITY;
            mx = fmaxf(mx, x[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));   // both lane groups of a row keep the same maximum
        const float m_new = fmaxf(run_m, mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        float e[16], psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            e[r] = fast_exp2(x[r] - m_safe);
            psum += e[r];
        }
        run_l = run_l * fast_exp2(run_m - m_safe) + psum;
        run_m = m_new;
        if (base + kStChunk > a.v_start && base < span_end) {
            // rows x 32 keys through the transpose area, out as 128-byte lines: registers 4q .. 4q+3 of
            // lane (row li, group g) are the keys 8q + 4g .. + 3 of the chunk
            const int cid = (base - c_base) / kStChunk;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4*)(s_tr + li * kStTrStride + (8 * q + 4 * g) * 4) =
                    make_float4(e[4 * q], e[4 * q + 1], e[4 * q + 2], e[4 * q + 3]);
            lds_sync();
            const int row = lane >> 1, half = lane & 1;
            const f32x4* src = (const f32x4*)(s_tr + row * kStTrStride + half * 64);
            const f32x4 p0 = src[0], p1 = src[1], p2 = src[2], p3 = src[3];
            if (row < e_rows) {
                f32x4* dst = (f32x4*)(etab + ((int64_t)cid * e_rows + row) * kStChunk + half * 16);
                __builtin_nontemporal_store(p0, dst);
                __builtin_nontemporal_store(p1, dst + 1);
                __builtin_nontemporal_store(p2, dst + 2);
                __builtin_nontemporal_store(p3, dst + 3);
            }
            if (g == 0) rtab[cid * 32 + li] = m_safe;
        }
        lds_sync();   // fragment and transpose reads are complete before the areas are written again
    }
    const float l = run_l + __shfl_xor(run_l, 32, 64);
    if (g == 0) ((float2*)a.stats)[(unit * a.n_splits + split) * 32 + li] = make_float2(run_m, l);
}

// grid (ceil(span chunks / 8), H, B), one wavefront per workgroup.  A lane owns 4 consecutive keys
// of one chunk: chunk 8 * blockIdx.x + lane / 8, keys 4 * (lane % 8) .. + 3, and walks the table
// rows of that chunk with one 16-byte load per row, adding them in row order.
// ER = table rows per chunk.  The table and reference loads are requested before the statistics
// are merged, so the kernel is three memory latencies long, not five.
template <int ER>
__global__ __launch_bounds__(64) void score_stream_weights_kernel(ScoreArgs a) {
    __shared__ float s_msum[32];
    const int lane = threadIdx.x;
    const int jj = lane & 31;
    const int h = blockIdx.y, b = blockIdx.z;
    const ScoreSeq sq = score_seq_from(a.n_q ? a.n_q[b] : a.n_q_max, a.n_tot[b], 0, a.n_q_max, 0, a.n_q_max, a.n_tot_max);
    const int n_q = sq.n_q, n_tot = sq.n_tot;
    const int span_end = a.v_start + a.M, c_base = a.v_start / kStChunk * kStChunk;
    const int span_chunks = (span_end - c_base + kStChunk - 1) / kStChunk;
    constexpr int e_rows = ER;
    const int max_chunks = stream_max_chunks(a.n_tot_max);
    const int64_t unit = (int64_t)b * a.H + h;
    const float* etab = a.etab + unit * max_chunks * e_rows * kStChunk;
    const float* rtab = a.rtab + unit * max_chunks * 32;
    float* partial = a.ws + unit * a.M;

    const int cid = 8 * blockIdx.x + (lane >> 3), kq = lane & 7;
    const int base = c_base + cid * kStChunk;
    const bool in_span = cid < span_chunks;
    const bool valid = in_span && base < n_tot;   // the stream kernel has written this chunk

    const int cc = valid ? cid : 0;   // lanes without a chunk read chunk 0 of the unit and drop it
    const f32x4* blk = (const f32x4*)(etab + (int64_t)cc * e_rows * kStChunk + 4 * kq);
    const float* ref = rtab + cc * 32;
    f32x4 w[ER];
    float rf[ER];
#pragma unroll
    for (int r = 0; r < ER; ++r) {
        w[r] = blk[r * (kStChunk / 4)];
        rf[r] = ref[r];
    }

    // final max + log2(sum) of scoring row jj, from the splits' statistics in split order
    float msum = INFINITY;   // +inf: the row contributes nothing
    if (n_tot > 0) {
        const float2* st = (const float2*)a.stats + unit * a.n_splits * 32 + jj;
        float m = -INFINITY, l = 0.f;
        for (int s0 = 0; s0 < a.n_splits; s0 += 8) {
            float2 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = st[(int64_t)min(s0 + u, a.n_splits - 1) * 32];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (s0 + u >= a.n_splits) continue;
                const float m_new = fmaxf(m, v[u].x);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                l = l * fast_exp2(m - m_safe) + v[u].y * fast_exp2(v[u].x - m_safe);
                m = m_new;
            }
        }
        if (jj < n_q && l > 0.f) msum = m + log2f(l);
    }
    if (lane < 32) s_msum[jj] = msum;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < ER; ++r) {
        const float f = valid ? fast_exp2(rf[r] - s_msum[r]) : 0.f;
        acc.x = fmaf(w[r].x, f, acc.x);
        acc.y = fmaf(w[r].y, f, acc.y);
        acc.z = fmaf(w[r].z, f, acc.z);
        acc.w = fmaf(w[r].w, f, acc.w);
    }
    if (in_span) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = base + 4 * kq + k;
            if (j >= a.v_start && j < span_end) partial[j - a.v_start] = j < n_tot ? acc[k] : 0.f;
        }
    }
}

bool score_stream_supported(const ScoreArgs& a, int dtype) {
    return dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.n_q_max <= 32;
}

size_t score_stream_workspace_floats(int B, int H, int n_q_max, int n_tot_max) {
    const size_t units = (size_t)B * H, chunks = (size_t)stream_max_chunks(n_tot_max);
    const size_t rtab = units * chunks * 32;
    const size_t etab = units * chunks * stream_table_rows(n_q_max) * kStChunk;
    return rtab + etab;
}

hipError_t launch_score_stream(const ScoreArgs& a0, float* tables, hipStream_t s) {
    ScoreArgs a = a0;
    a.rtab = tables;
    a.etab = tables + (size_t)a.B * a.H * stream_max_chunks(a.n_tot_max) * 32;
    const dim3 grid((a.H + 3) / 4, a.B, a.n_splits);
    if (a.d_h == 128)
        hipLaunchKernelGGL(score_stream_kernel<128>, grid, dim3(kStThreads), 4 * (size_t)StCfg<128>::kWaveLds, s, a);
    else
        hipLaunchKernelGGL(score_stream_kernel<64>, grid, dim3(kStThreads), 4 * (size_t)StCfg<64>::kWaveLds, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int c_base = a.v_start / kStChunk * kStChunk;
    const int span_chunks = (a.v_start + a.M - c_base + kStChunk - 1) / kStChunk;
    const dim3 wgrid((span_chunks + 7) / 8, a.H, a.B);
    switch (stream_table_rows(a.n_q_max)) {
        case 8: hipLaunchKernelGGL(score_stream_weights_kernel<8>, wgrid, dim3(64), 0, s, a); break;
        case 16: hipLaunchKernelGGL(score_stream_weights_kernel<16>, wgrid, dim3(64), 0, s, a); break;
        case 24: hipLaunchKernelGGL(score_stream_weights_kernel<24>, wgrid, dim3(64), 0, s, a); break;
        default: hipLaunchKernelGGL(score_stream_weights_kernel<32>, wgrid, dim3(64), 0, s, a); break;
    }
    return hipGetLastError();
}

}  // namespace tw
