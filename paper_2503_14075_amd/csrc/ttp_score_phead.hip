// Pruning score in the P-Head form (Sec. 5.1 Eq. 7): one query (the last text
// token) per sequence, query and keys modulated element-wise by gate vectors,
// softmax over the M visual keys only, mean over heads.
//
// One workgroup per (head, sequence).  Sixteen lanes share a key (16-byte
// pieces of the key row and of its gate row), so a wavefront consumes four
// keys per step with fully coalesced 256-byte segments; logits go to LDS, the
// softmax runs over LDS, the per-head weights go to partial[b][h][m] and
// score_reduce_kernel adds the heads in index order.  With one query the work
// is a pure stream over K and its gates: HBM-bound, plain fp32 vector math.
#include "twig_internal.h"

namespace tw {

constexpr int kPhThreads = 256;

template <typename TIn>
__device__ __forceinline__ void ph_load8(const TIn* p, float* dst);
template <>
__device__ __forceinline__ void ph_load8<float>(const float* p, float* dst) {
    typedef __attribute__((ext_vector_type(4))) float f4;
    const f4 a = __builtin_nontemporal_load((const f4*)p), b = __builtin_nontemporal_load((const f4*)(p + 4));
    dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w;
    dst[4] = b.x; dst[5] = b.y; dst[6] = b.z; dst[7] = b.w;
}
template <>
__device__ __forceinline__ void ph_load8<uint16_t>(const uint16_t* p, float* dst) {
    // keys and gates are read once: the streaming hint is worth 11 % on the 128-sequence launch
    typedef __attribute__((ext_vector_type(4))) unsigned int u4;
    const u4 a = __builtin_nontemporal_load((const u4*)p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        dst[2 * e] = __uint_as_float(w[e] << 16);
        dst[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* s_red, int tid) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off, 64);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    __syncthreads();
    if ((tid & 63) == 0) s_red[tid >> 6] = v;
    __syncthreads();
    float r = s_red[0];
    for (int w = 1; w < kPhThreads / 64; ++w) r = is_max ? fmaxf(r, s_red[w]) : r + s_red[w];
    return r;
}

// kUnroll = independent key/gate load pairs in flight per lane: 4 when the launch is too small to
// hide the load latency by occupancy (measured: 8 sequences 44 -> 29 us), 1 when it is not (128
// sequences: 219 us, against 231 us with 4).
template <typename TIn, int kUnroll>
__global__ __launch_bounds__(kPhThreads) void phead_kernel(PheadArgs a) {
    extern __shared__ float s_logit[];   // [M]
    __shared__ float s_red[kPhThreads / 64];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int l16 = tid & 15, slot = tid >> 4;   // 16 lanes per key, 16 keys per step
    const int d_h = a.d_h, c0 = l16 * 8;
    const bool col_ok = c0 < d_h;
    float qg[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col_ok) {
        float qv[8], gv[8];
        ph_load8<TIn>((const TIn*)a.q + ((int64_t)b * a.H + h) * d_h + c0, qv);
        ph_load8<TIn>((const TIn*)a.gq + ((int64_t)b * a.H + h) * d_h + c0, gv);
#pragma unroll
        for (int e = 0; e < 8; ++e) qg[e] = a.scale * (qv[e] * gv[e]);
    }
    const TIn* kb = (const TIn*)a.k.base;
    const TIn* gb = (const TIn*)a.gk.base;
    // 16 * kUnroll keys per step (keys past M re-read the last key and are dropped)
    for (int j0 = 0; j0 < a.M; j0 += 16 * kUnroll) {
        float kv[kUnroll][8], gv[kUnroll][8];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + 16 * u + slot;
            const int jc = j < a.M ? j : a.M - 1;
            const int cc = col_ok ? c0 : 0;
            ph_load8<TIn>(kb + (pool_row(a.k, b, a.v_start + jc) * a.H + h) * d_h + cc, kv[u]);
            ph_load8<TIn>(gb + (pool_row(a.gk, b, a.v_start + jc) * a.H + h) * d_h + cc, gv[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + 16 * u + slot;
            float dot = 0.f;
            if (col_ok) {
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(qg[e], kv[u][e] * gv[u][e], dot);
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) dot += __shfl_xor(dot, off, 64);
            if (l16 == 0 && j < a.M) s_logit[j] = dot;
        }
    }
    __syncthreads();
    float mx = -INFINITY;
    for (int j = tid; j < a.M; j += kPhThreads) mx = fmaxf(mx, s_logit[j]);
    mx = block_reduce(mx, true, s_red, tid);
    float sum = 0.f;
    for (int j = tid; j < a.M; j += kPhThreads) {
        const float e = expf(s_logit[j] - mx);
        s_logit[j] = e;
        sum += e;
    }
    sum = block_reduce(sum, false, s_red, tid);
    float* partial = a.ws + ((int64_t)b * a.H + h) * a.M;
    const float inv = 1.f / sum;
    for (int j = tid; j < a.M; j += kPhThreads) partial[j] = s_logit[j] * inv;
}

hipError_t launch_phead(const PheadArgs& a, int dtype, hipStream_t s) {
    if (a.B == 0 || a.M == 0) return hipSuccess;
    const size_t lds = (size_t)a.M * sizeof(float);
    const bool small = (long)a.B * a.H <= 512;
    const void* fn = dtype == TW_F32 ? (small ? (const void*)phead_kernel<float, 4> : (const void*)phead_kernel<float, 1>)
                                     : (small ? (const void*)phead_kernel<uint16_t, 4>
                                              : (const void*)phead_kernel<uint16_t, 1>);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const dim3 grid(a.H, a.B), block(kPhThreads);
    if (dtype == TW_F32) {
        if (small) hipLaunchKernelGGL((phead_kernel<float, 4>), grid, block, lds, s, a);
        else hipLaunchKernelGGL((phead_kernel<float, 1>), grid, block, lds, s, a);
    } else {
        if (small) hipLaunchKernelGGL((phead_kernel<uint16_t, 4>), grid, block, lds, s, a);
        else hipLaunchKernelGGL((phead_kernel<uint16_t, 1>), grid, block, lds, s, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // head mean: the same reduction as the attention-map form, one scoring row per sequence
    ScoreArgs r = {};
    r.n_q = nullptr;
    r.n_q_max = 1;
    r.scores = a.scores;
    r.ws = a.ws;
    r.B = a.B;
    r.H = a.H;
    r.M = a.M;
    return launch_score_reduce(r, s);
}

}  // namespace tw
