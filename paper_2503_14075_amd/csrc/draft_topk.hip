// Rank-ordered top-E of vocabulary-sized rows for small E (the per-node expansion of the draft
// tree by its E most probable tokens, Sec. 5.4 / App. A).  One workgroup per row, the row read
// once with 16-byte loads and held in registers.
//
// The lanes form 64 groups that partition the row.  The E-th largest of the 64 group maxima is a
// lower bound of the E-th largest value of the row (E groups hold a value at least that large), so
// every winner, and every value tied with the last winner, is among the values not below that
// bound.  For a row without massive ties those are about E values; they go to a short list in LDS
// and are ranked there (larger value first, equal values lower index first).  A row whose list
// overflows (many values tied at the bound) is handed to the general radix select.
#include "select_block.h"

namespace tw {

constexpr int kTkCap = 1024;   // list entries
typedef __attribute__((ext_vector_type(4))) float f32x4t;

template <int NV, int THREADS>   // 16-byte pieces per lane, lanes per row
__global__ __launch_bounds__(THREADS) void topk_rows_kernel(const float* __restrict__ probs, int V, int E,
                                                            int32_t* __restrict__ ids, float* __restrict__ vals) {
    constexpr int kWaves = THREADS / 64;
    __shared__ float s_max[THREADS];
    __shared__ uint32_t s_key[kTkCap];
    __shared__ uint32_t s_idx[kTkCap];
    __shared__ uint32_t s_n;
    const int tid = threadIdx.x, lane = tid & 63;
    const float* row = probs + (int64_t)blockIdx.x * V;
    int32_t* out = ids + (int64_t)blockIdx.x * E;
    float* out_v = vals + (int64_t)blockIdx.x * E;
    const int n_pieces = V >> 2;   // V is a multiple of four here

    // slots past the row hold -inf: below every finite value, and kept off the list by index too
    f32x4t raw[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int piece = tid + u * THREADS;
        raw[u] = f32x4t{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (piece < n_pieces) raw[u] = __builtin_nontemporal_load((const f32x4t*)row + piece);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < NV; ++u) mx = fmaxf(fmaxf(mx, fmaxf(raw[u][0], raw[u][1])), fmaxf(raw[u][2], raw[u][3]));
    s_max[tid] = mx;
    if (tid == 0) s_n = 0u;
    __syncthreads();
    // Lane l of every wavefront takes the maximum of the lanes l, l + 64, ... (64 groups that
    // partition the row) and counts the group maxima above and not below its own: the E-th largest
    // group maximum is the one with (above) < E <= (not below).  Every wavefront finds it for itself.
    float gmax = s_max[lane];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) gmax = fmaxf(gmax, s_max[lane + 64 * w]);
    int above = 0, not_below = 0;
#pragma unroll
    for (int j = 0; j < 64; ++j) {
        const float o = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(gmax), j));
        above += o > gmax;
        not_below += o >= gmax;
    }
    const uint64_t is_bound = __ballot(above < E && E <= not_below);
    // finite input always has such a lane; lane 0 stands in otherwise, which only lengthens the list
    const int src = is_bound ? __ffsll((unsigned long long)is_bound) - 1 : 0;
    const float tau = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(gmax), src));
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const float pm = fmaxf(fmaxf(raw[u][0], raw[u][1]), fmaxf(raw[u][2], raw[u][3]));
        if (pm >= tau && tid + u * THREADS < n_pieces) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (raw[u][c] >= tau) {
                    const uint32_t pos = atomicAdd(&s_n, 1u);
                    if (pos < (uint32_t)kTkCap) {
                        s_key[pos] = order_key(raw[u][c]);
                        s_idx[pos] = (uint32_t)((tid + u * THREADS) * 4 + c);
                    }
                }
            }
        }
    }
    __syncthreads();
    const int L = (int)s_n;
    if (L > kTkCap) {   // the same for every lane of the workgroup
        select_block<0, THREADS>(row, V, E, out, out_v);
        return;
    }
    for (int e = tid; e < L; e += THREADS) {
        const uint32_t key = s_key[e], idx = s_idx[e];
        int rank = 0;
        for (int j = 0; j < L; ++j) rank += (s_key[j] > key) || (s_key[j] == key && s_idx[j] < idx);
        if (rank < E) {
            out[rank] = (int32_t)idx;
            out_v[rank] = row[idx];
        }
    }
}

bool launch_topk_rows(const float* probs, int n, int V, int E, int32_t* ids, float* vals, hipStream_t s,
                      hipError_t* err) {
    // rows shorter than this are served as fast by the radix select; every group of lanes must
    // own a value, the row must fit the registers, and the bound is only tight while E is far
    // below the number of groups
    if (E < 1 || E > 32 || V <= 3072 || V > 32768 || (V & 3) || ((uintptr_t)probs & 15)) return false;
    // 512 lanes with 16 pieces each: measured against 256 x 32 and 1024 x 8 (30.7 / 33.0 / 34.3 us
    // for 1280 rows of 32000)
    hipLaunchKernelGGL((topk_rows_kernel<16, 512>), dim3(n), dim3(512), 0, s, probs, V, E, ids, vals);
    *err = hipGetLastError();
    return true;
}

}  // namespace tw
