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

// Keys of one sequence are loaded once into registers (KPT per lane) when the
// row fits, otherwise (KPT == 0) every pass re-reads them from memory.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores, int M,
                                                             int R, int32_t* __restrict__ kept) {
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_prefix, s_need;
    __shared__ uint32_t s_wave_a[kSelThreads / 64], s_wave_b[kSelThreads / 64];
    __shared__ uint32_t s_run_eq, s_run_sel;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* sc = scores + (int64_t)blockIdx.x * M;
    int32_t* out = kept + (int64_t)blockIdx.x * R;
    if (R <= 0) return;

    uint32_t keys[KPT > 0 ? KPT : 1];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
        const int m = tid + u * kSelThreads;
        keys[u] = m < M ? order_key(sc[m]) : 0u;
    }
    auto key_at = [&](int u, int m) -> uint32_t { return KPT > 0 ? keys[u] : order_key(sc[m]); };
    const int n_iter = (M + kSelThreads - 1) / kSelThreads;

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
        const uint32_t prefix = s_prefix, need = s_need;
        const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
        if (KPT > 0) {
#pragma unroll
            for (int u = 0; u < KPT; ++u) {
                const int m = tid + u * kSelThreads;
                if (m < M && (keys[u] & hi_mask) == prefix) atomicAdd(&s_hist[(keys[u] >> shift) & 0xFFu], 1u);
            }
        } else {
            for (int u = 0; u < n_iter; ++u) {
                const int m = tid + u * kSelThreads;
                if (m < M) {
                    const uint32_t key = key_at(u, m);
                    if ((key & hi_mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 0xFFu], 1u);
                }
            }
        }
        __syncthreads();
        // lane tid owns bucket 255 - tid; inclusive scan from the largest bucket down
        const uint32_t mine = s_hist[255 - tid];
        uint32_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        if (lane == 63) s_wave_a[wave] = incl;
        __syncthreads();
        for (int w = 0; w < wave; ++w) incl += s_wave_a[w];
        // exactly one bucket has  (count above it) < need <= (count above it) + (its own count)
        if (incl >= need && incl - mine < need) {
            s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
            s_need = need - (incl - mine);
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
    const uint64_t below = (1ull << lane) - 1ull;
    for (int u = 0; u < n_iter; ++u) {
        const int m = u * kSelThreads + tid;
        bool eq = false, gt = false;
        if (m < M) {
            const uint32_t key = key_at(u, m);
            eq = key == thr;
            gt = key > thr;
        }
        // rank of this element among the equal keys, in index order
        const uint64_t eq_ballot = __ballot(eq);
        if (lane == 0) s_wave_a[wave] = (uint32_t)__popcll(eq_ballot);
        __syncthreads();
        uint32_t eq_rank = s_run_eq + (uint32_t)__popcll(eq_ballot & below);
        for (int w = 0; w < wave; ++w) eq_rank += s_wave_a[w];
        const bool sel = gt || (eq && eq_rank < need);
        const uint64_t sel_ballot = __ballot(sel);
        if (lane == 0) s_wave_b[wave] = (uint32_t)__popcll(sel_ballot);
        __syncthreads();
        uint32_t pos = s_run_sel + (uint32_t)__popcll(sel_ballot & below);
        for (int w = 0; w < wave; ++w) pos += s_wave_b[w];
        if (sel && pos < (uint32_t)R) out[pos] = m;
        __syncthreads();
        if (tid == 0) {
            uint32_t e = 0u, s2 = 0u;
            for (int w = 0; w < kSelThreads / 64; ++w) {
                e += s_wave_a[w];
                s2 += s_wave_b[w];
            }
            s_run_eq += e;
            s_run_sel += s2;
        }
        __syncthreads();
    }
}

hipError_t launch_select(const float* scores, int B, int M, int R, int32_t* kept, hipStream_t s) {
    if (B == 0 || R == 0) return hipSuccess;
    if (M <= 4 * kSelThreads)
        hipLaunchKernelGGL(select_kernel<4>, dim3(B), dim3(kSelThreads), 0, s, scores, M, R, kept);
    else if (M <= 12 * kSelThreads)
        hipLaunchKernelGGL(select_kernel<12>, dim3(B), dim3(kSelThreads), 0, s, scores, M, R, kept);
    else
        hipLaunchKernelGGL(select_kernel<0>, dim3(B), dim3(kSelThreads), 0, s, scores, M, R, kept);
    return hipGetLastError();
}

}  // namespace tw
