// Top-R keep of the pruning function (TopR of Sec. 3.1 Eq. 3): radix select on
// order-preserving 32-bit keys, ties toward the lower index, ascending output.
// One workgroup per sequence; inputs are a few KB so this is latency work.
#include "twig_internal.h"

namespace tw {

constexpr int kSelThreads = 256;

// Larger float <=> larger key.  -0.0 is folded into +0.0 first so the two tie.
__device__ __forceinline__ uint32_t order_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores, int M,
                                                             int R, int32_t* __restrict__ kept) {
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_prefix, s_need;
    __shared__ uint32_t s_wave_eq[kSelThreads / 64], s_wave_sel[kSelThreads / 64];
    __shared__ uint32_t s_run_eq, s_run_sel;
    const int tid = threadIdx.x;
    const float* sc = scores + (int64_t)blockIdx.x * M;
    int32_t* out = kept + (int64_t)blockIdx.x * R;
    if (R <= 0) return;

    if (tid == 0) {
        s_prefix = 0u;
        s_need = (uint32_t)R;
    }
    // Four passes, most significant byte first.  After a pass the key prefix of
    // the R-th largest element is known down to that byte, and s_need is its
    // rank among the elements sharing the prefix.
    for (int shift = 24; shift >= 0; shift -= 8) {
        s_hist[tid] = 0u;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
        for (int m = tid; m < M; m += kSelThreads) {
            const uint32_t key = order_key(sc[m]);
            if ((key & hi_mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 0xFFu], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t need = s_need, above = 0u;
            int bucket = 255;
            for (; bucket > 0; --bucket) {
                if (above + s_hist[bucket] >= need) break;
                above += s_hist[bucket];
            }
            s_prefix = prefix | ((uint32_t)bucket << shift);
            s_need = need - above;
        }
        __syncthreads();
    }
    const uint32_t thr = s_prefix;   // key of the R-th largest score
    const uint32_t need = s_need;    // how many elements equal to it are kept (lowest indices)
    if (tid == 0) {
        s_run_eq = 0u;
        s_run_sel = 0u;
    }
    __syncthreads();
    const int lane = tid & 63, wave = tid >> 6;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int m0 = 0; m0 < M; m0 += kSelThreads) {
        const int m = m0 + tid;
        uint32_t key = 0u;
        bool eq = false, gt = false;
        if (m < M) {
            key = order_key(sc[m]);
            eq = key == thr;
            gt = key > thr;
        }
        // rank of this element among the equal keys, in index order
        const uint64_t eq_ballot = __ballot(eq);
        if (lane == 0) s_wave_eq[wave] = (uint32_t)__popcll(eq_ballot);
        __syncthreads();
        uint32_t eq_rank = s_run_eq + (uint32_t)__popcll(eq_ballot & below);
        for (int w = 0; w < wave; ++w) eq_rank += s_wave_eq[w];
        const bool sel = gt || (eq && eq_rank < need);
        const uint64_t sel_ballot = __ballot(sel);
        if (lane == 0) s_wave_sel[wave] = (uint32_t)__popcll(sel_ballot);
        __syncthreads();
        uint32_t pos = s_run_sel + (uint32_t)__popcll(sel_ballot & below);
        for (int w = 0; w < wave; ++w) pos += s_wave_sel[w];
        if (sel && pos < (uint32_t)R) out[pos] = m;
        __syncthreads();
        if (tid == 0) {
            uint32_t e = 0u, s = 0u;
            for (int w = 0; w < kSelThreads / 64; ++w) {
                e += s_wave_eq[w];
                s += s_wave_sel[w];
            }
            s_run_eq += e;
            s_run_sel += s;
        }
        __syncthreads();
    }
}

hipError_t launch_select(const float* scores, int B, int M, int R, int32_t* kept, hipStream_t s) {
    if (B == 0 || R == 0) return hipSuccess;
    hipLaunchKernelGGL(select_kernel, dim3(B), dim3(kSelThreads), 0, s, scores, M, R, kept);
    return hipGetLastError();
}

}  // namespace tw
