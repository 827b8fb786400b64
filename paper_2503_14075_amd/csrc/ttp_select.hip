// Top-R keep of the pruning function (TopR of Sec. 3.1 Eq. 3): radix select on
// order-preserving 32-bit keys, ties toward the lower index, ascending output.
// One workgroup per sequence; inputs are a few KB so this is latency work.
#include "select_block.h"

namespace tw {


template <int KPT, int THREADS>
__global__ __launch_bounds__(THREADS) void select_kernel(const float* __restrict__ scores, int M, int R,
                                                         int32_t* __restrict__ kept, float* __restrict__ ranked_vals) {
    select_block<KPT, THREADS>(scores + (int64_t)blockIdx.x * M, M, R, kept + (int64_t)blockIdx.x * R,
                               ranked_vals ? ranked_vals + (int64_t)blockIdx.x * R : nullptr);
}

hipError_t launch_select(const float* scores, int B, int M, int R, int32_t* kept, hipStream_t s,
                         float* ranked_vals) {
    if (B == 0 || R == 0) return hipSuccess;
    if (ranked_vals && R > 256) return hipErrorInvalidValue;
    // rows up to 32768 scores (a vocabulary) are held in registers: 4 or 12 per lane of 256, or 32
    // per lane of 1024 (one row of 32000: 147 us with a re-read per pass, measured, against this)
    if (M <= 4 * 256)
        hipLaunchKernelGGL((select_kernel<4, 256>), dim3(B), dim3(256), 0, s, scores, M, R, kept, ranked_vals);
    else if (M <= 12 * 256)
        hipLaunchKernelGGL((select_kernel<12, 256>), dim3(B), dim3(256), 0, s, scores, M, R, kept, ranked_vals);
    else if (M <= 32 * 1024)
        hipLaunchKernelGGL((select_kernel<32, 1024>), dim3(B), dim3(1024), 0, s, scores, M, R, kept, ranked_vals);
    else
        hipLaunchKernelGGL((select_kernel<0, 256>), dim3(B), dim3(256), 0, s, scores, M, R, kept, ranked_vals);
    return hipGetLastError();
}

}  // namespace tw
