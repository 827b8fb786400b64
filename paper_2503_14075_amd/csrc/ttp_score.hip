// Pruning score of twig-guided token pruning (Sec. 3.1 Eq. 2-3, head mean as
// in Sec. 5.1 Eq. 7): attention rows of the last text queries, averaged over
// heads and rows, restricted to the visual columns.
//
// Two kernels, both with a fixed summation order (bit-identical run to run):
//   1. score_logits: one workgroup per (head, 16 scoring rows, sequence) walks
//      the keys in tiles of 64 staged in LDS, writes the masked logits to the
//      workspace and keeps an online (max, sum) per row.
//   2. score_reduce: one lane per visual key sums exp(logit - max) / sum over
//      heads and rows in a fixed order.
#include "twig_internal.h"

namespace tw {

constexpr int kScThreads = 256;
constexpr int kScRows = 16;   // scoring rows per workgroup
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

template <typename TIn>
__global__ __launch_bounds__(kScThreads) void score_logits_kernel(ScoreArgs a) {
    extern __shared__ float smem[];
    const int d_h = a.d_h, ld = d_h + 1;
    float* sQ = smem;                 // [kScRows][ld], pre-multiplied by scale
    float* sK = sQ + kScRows * ld;    // [kScKeys][ld]
    const int h = blockIdx.x, b = blockIdx.z, row0 = blockIdx.y * kScRows;
    const int tid = threadIdx.x;
    int n_q = a.n_q ? a.n_q[b] : a.n_q_max;
    n_q = n_q < 1 ? 1 : (n_q > a.n_q_max ? a.n_q_max : n_q);
    if (row0 >= n_q) return;
    int n_tot = a.n_tot[b];
    n_tot = n_tot < 0 ? 0 : (n_tot > a.n_tot_max ? a.n_tot_max : n_tot);
    const int pos0 = a.q_pos0[b];
    const TIn* q = (const TIn*)a.q_sel;
    const TIn* kbase = (const TIn*)a.k.base;
    const int c8n = d_h / 8;

    for (int idx = tid; idx < kScRows * c8n; idx += kScThreads) {
        const int i = idx / c8n, c8 = idx % c8n;
        float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (row0 + i < n_q)
            load8<TIn>(q + (((int64_t)b * a.n_q_max + row0 + i) * a.H + h) * d_h + c8 * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) sQ[i * ld + c8 * 8 + e] = v[e] * a.scale;
    }

    const int i = tid / 16, kg = tid % 16;
    const int i_abs = row0 + i;
    const bool row_ok = i_abs < n_q;
    const int n_vis = !row_ok ? 0 : (a.causal ? min(pos0 + i_abs + 1, n_tot) : n_tot);
    float* logit_row = a.ws + (((int64_t)b * a.H + h) * a.n_q_max + i_abs) * (int64_t)a.n_tot_max;
    float run_m = -INFINITY, run_l = 0.f;

    for (int base = 0; base < n_tot; base += kScKeys) {
        __syncthreads();
        for (int idx = tid; idx < kScKeys * c8n; idx += kScThreads) {
            const int r = idx / c8n, c8 = idx % c8n;
            float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (base + r < n_tot) {
                const int64_t prow = pool_row(a.k, b, base + r);
                load8<TIn>(kbase + (prow * a.H + h) * d_h + c8 * 8, v);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sK[r * ld + c8 * 8 + e] = v[e];
        }
        __syncthreads();
        float dot[4] = {0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < d_h; ++c) {
            const float qv = sQ[i * ld + c];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) dot[jj] = fmaf(qv, sK[(kg + 16 * jj) * ld + c], dot[jj]);
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int j = base + kg + 16 * jj;
            if (row_ok && j < n_tot) {
                const bool vis = j < n_vis;
                const float s = vis ? dot[jj] : -INFINITY;
                logit_row[j] = s;
                if (vis) {
                    const float m_new = fmaxf(run_m, s);
                    run_l = run_l * expf(run_m - m_new) + expf(s - m_new);
                    run_m = m_new;
                }
            }
        }
    }
    // merge the 16 lanes that share a scoring row
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        const float om = __shfl_xor(run_m, off, 64), ol = __shfl_xor(run_l, off, 64);
        const float m_new = fmaxf(run_m, om);
        const float sa = run_m == -INFINITY ? 0.f : expf(run_m - m_new);
        const float sb = om == -INFINITY ? 0.f : expf(om - m_new);
        run_l = run_l * sa + ol * sb;
        run_m = m_new;
    }
    if (row_ok && kg == 0) {
        float* st = a.ws + (int64_t)a.B * a.H * a.n_q_max * a.n_tot_max +
                    (((int64_t)b * a.H + h) * a.n_q_max + i_abs) * 2;
        st[0] = run_m;
        st[1] = run_l;
    }
}

__global__ __launch_bounds__(kScThreads) void score_reduce_kernel(ScoreArgs a) {
    const int b = blockIdx.y, m = blockIdx.x * kScThreads + threadIdx.x;
    if (m >= a.M) return;
    int n_q = a.n_q ? a.n_q[b] : a.n_q_max;
    n_q = n_q < 1 ? 1 : (n_q > a.n_q_max ? a.n_q_max : n_q);
    const int j = a.v_start + m;
    const float* stats = a.ws + (int64_t)a.B * a.H * a.n_q_max * a.n_tot_max;
    float acc = 0.f;
    for (int h = 0; h < a.H; ++h) {
        for (int i = 0; i < n_q; ++i) {
            const int64_t row = ((int64_t)b * a.H + h) * a.n_q_max + i;
            const float s = a.ws[row * a.n_tot_max + j];
            const float mx = stats[row * 2], l = stats[row * 2 + 1];
            if (s != -INFINITY) acc += expf(s - mx) / l;
        }
    }
    a.scores[(int64_t)b * a.M + m] = acc / ((float)a.H * (float)n_q);
}

size_t score_workspace_bytes(int B, int H, int n_q_max, int n_tot_max) {
    return ((size_t)B * H * n_q_max * n_tot_max + (size_t)B * H * n_q_max * 2) * sizeof(float);
}

hipError_t launch_score(const ScoreArgs& a, int dtype, hipStream_t s) {
    if (a.B == 0 || a.M == 0) return hipSuccess;
    const dim3 grid(a.H, (a.n_q_max + kScRows - 1) / kScRows, a.B);
    const size_t lds = (size_t)(kScRows + kScKeys) * (a.d_h + 1) * sizeof(float);
    if (dtype == TW_F32)
        hipLaunchKernelGGL(score_logits_kernel<float>, grid, dim3(kScThreads), lds, s, a);
    else
        hipLaunchKernelGGL(score_logits_kernel<uint16_t>, grid, dim3(kScThreads), lds, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(score_reduce_kernel, dim3((a.M + kScThreads - 1) / kScThreads, a.B),
                       dim3(kScThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace tw
