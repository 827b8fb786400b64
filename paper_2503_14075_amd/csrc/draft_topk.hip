// Rank-ordered top-E of vocabulary-sized rows for small E (the per-node expansion of the draft
// tree by its E most probable tokens, Sec. 5.4 / App. A), from probabilities or from logits.  One
// workgroup per row; the row is read once, in chunks of 32768 values held in registers.
//
// The lanes form 64 groups that partition the row.  The E-th largest of the 64 group maxima is a
// lower bound of the E-th largest value of the row (E groups hold a value at least that large), so
// every winner, and every value tied with the last winner, is among the values not below that
// bound.  For a row without massive ties those are about E values; they go to a short list in LDS
// and are ranked there (larger value first, equal values lower index first).  With several chunks
// the group maxima run on from chunk to chunk, so the bound only rises and the list stays a
// superset of the winners.  A row whose list overflows (many values tied at the bound) is handed
// to the general radix select, and so is every row when E is above 32.
//
// From logits, every lane keeps a running maximum of its own values and the sum of exp(l - that
// maximum), updated 16 bytes at a time in the order the loads return, so the exponentials are
// taken while the rest of the row is still on its way; the lanes' sums are brought to the row
// maximum once at the end, and the winners leave as probabilities.
#include "select_block.h"

namespace tw {

constexpr int kTkCap = 1024;   // list entries
constexpr int kTkListE = 32;   // the bound of the group maxima is used up to this E (far below the 64 groups)
typedef __attribute__((ext_vector_type(4))) float f32x4t;

// NV 16-byte pieces per lane and chunk, THREADS lanes per row; kLogits: softmax of the row on the
// way; kVec: rows are 16-byte aligned and a multiple of four long
template <int NV, int THREADS, bool kLogits, bool kVec>
// (held to 128 registers: two workgroups of 512 per compute unit)
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(4))) void topk_rows_kernel(
    const float* __restrict__ x, int V, int E, int32_t* __restrict__ ids, float* __restrict__ vals) {
    constexpr int kWaves = THREADS / 64;
    constexpr int kChunk = THREADS * NV * 4;
    __shared__ float s_max[THREADS];
    __shared__ uint32_t s_key[kTkCap];
    __shared__ uint32_t s_idx[kTkCap];
    __shared__ float s_val[kTkCap];
    __shared__ float s_sum[kWaves];
    __shared__ uint32_t s_n;
    const int tid = threadIdx.x, lane = tid & 63;
    const float* row = x + (int64_t)blockIdx.x * V;
    int32_t* out = ids + (int64_t)blockIdx.x * E;
    float* out_v = vals + (int64_t)blockIdx.x * E;

    float G = -INFINITY;                        // group maximum over the chunks so far (lane l: group l)
    float lane_m = -INFINITY, lane_sum = 0.f;   // kLogits: this lane's maximum so far, its sum of exp(l - lane_m)
    if (tid == 0) s_n = 0u;
    for (int c0 = 0; c0 < V; c0 += kChunk) {
        // slots past the row hold -inf: below every finite value, and kept off the list by index too
        f32x4t raw[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int first = c0 + (tid + u * THREADS) * 4;
            raw[u] = f32x4t{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (kVec) {
                // no load inside a branch: a piece past the row reads the row's first piece and is replaced
                // by -inf where it is used, so the wait for piece u waits for piece u, not for all of them
                raw[u] = __builtin_nontemporal_load((const f32x4t*)(row + (first < V ? first : 0)));
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (first + c < V) raw[u][c] = __builtin_nontemporal_load(row + first + c);
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the chunk is issued before the first is waited for
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (kVec) {
                // (the choice is made on the bits, which keeps the compiler from moving the load back
                // under the condition)
                const uint32_t keep = c0 + (tid + u * THREADS) * 4 < V ? 0xFFFFFFFFu : 0u;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    raw[u][c] = __uint_as_float((__float_as_uint(raw[u][c]) & keep) | (0xFF800000u & ~keep));
            }
            const float pm = fmaxf(fmaxf(raw[u][0], raw[u][1]), fmaxf(raw[u][2], raw[u][3]));
            mx = fmaxf(mx, pm);
            if (kLogits) {
                // (a piece of empty slots, -inf throughout, adds nothing and must not produce inf - inf)
                const float m_new = fmaxf(lane_m, pm);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                lane_sum = lane_sum * __expf(lane_m - m_safe) +
                           ((__expf(raw[u][0] - m_safe) + __expf(raw[u][1] - m_safe)) +
                            (__expf(raw[u][2] - m_safe) + __expf(raw[u][3] - m_safe)));
                lane_m = m_new;
                // one piece at a time, in the order the loads return: the sums are pinned here, or the
                // exponentials (needed only at the end) would all be moved behind the wait for the last load
                if (kVec) asm volatile("" : "+v"(lane_sum), "+v"(lane_m));
            }
        }
        if (c0 > 0) __syncthreads();   // every wavefront has read the maxima of the chunk before
        s_max[tid] = mx;
        __syncthreads();
        // Lane l of every wavefront folds the lanes l, l + 64, ... into its group maximum and counts
        // the group maxima above and not below its own: the E-th largest group maximum is the one
        // with (above) < E <= (not below).  Every wavefront finds it for itself.
        float gmax = s_max[lane];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) gmax = fmaxf(gmax, s_max[lane + 64 * w]);
        G = fmaxf(G, gmax);
        if (E <= kTkListE) {
            int above = 0, not_below = 0;
#pragma unroll
            for (int j = 0; j < 64; ++j) {
                const float o = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(G), j));
                above += o > G;
                not_below += o >= G;
            }
            const uint64_t is_bound = __ballot(above < E && E <= not_below);
            // finite input always has such a lane; lane 0 stands in otherwise, which only lengthens the list
            const int src = is_bound ? __ffsll((unsigned long long)is_bound) - 1 : 0;
            const float tau = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(G), src));
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                const float pm = fmaxf(fmaxf(raw[u][0], raw[u][1]), fmaxf(raw[u][2], raw[u][3]));
                if (pm >= tau) {
                    const int first = c0 + (tid + u * THREADS) * 4;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (raw[u][c] >= tau && first + c < V) {
                            const uint32_t pos = atomicAdd(&s_n, 1u);
                            if (pos < (uint32_t)kTkCap) {
                                s_key[pos] = order_key(raw[u][c]);
                                s_idx[pos] = (uint32_t)(first + c);
                                s_val[pos] = raw[u][c];
                            }
                        }
                    }
                }
            }
        }
    }
    float run_m = G;   // kLogits: the row maximum, the largest group maximum
    if (kLogits) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) run_m = fmaxf(run_m, __shfl_xor(run_m, off, 64));
        lane_sum *= __expf(lane_m - (run_m == -INFINITY ? 0.f : run_m));   // a lane without values: 0 * 0
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) lane_sum += __shfl_xor(lane_sum, off, 64);
        if (lane == 0) s_sum[tid >> 6] = lane_sum;
    }
    __syncthreads();
    float total = 0.f;
    if (kLogits) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += s_sum[w];
    }
    const int L = (int)s_n;
    if (L > kTkCap || E > kTkListE) {   // the same for every lane of the workgroup
        select_block<0, THREADS>(row, V, E, out, out_v);
        if (kLogits) {
            __syncthreads();   // the winners' logits are in out_v
            if (tid < E) out_v[tid] = __expf(out_v[tid] - run_m) / total;
        }
        return;
    }
    // rank of a list entry = the entries ahead of it; eight lanes share an entry, each counts every
    // eighth of the list (the trip count is the same for every lane, the shuffles see all of them)
    for (int e0 = 0; e0 < L; e0 += THREADS / 8) {
        const int e = e0 + (tid >> 3);
        uint32_t key = 0u, idx = 0u;
        int rank = 0;
        if (e < L) {
            key = s_key[e];
            idx = s_idx[e];
            for (int j = tid & 7; j < L; j += 8) rank += (s_key[j] > key) || (s_key[j] == key && s_idx[j] < idx);
        }
        rank += __shfl_xor(rank, 1, 64);
        rank += __shfl_xor(rank, 2, 64);
        rank += __shfl_xor(rank, 4, 64);
        if (e < L && (tid & 7) == 0 && rank < E) {
            out[rank] = (int32_t)idx;
            const float v = s_val[e];
            out_v[rank] = kLogits ? __expf(v - run_m) / total : v;
        }
    }
}

bool launch_topk_rows(const float* x, int n, int V, int E, int32_t* ids, float* vals, bool logits, hipStream_t s,
                      hipError_t* err) {
    // the bound is only tight while E is far below the number of groups; probability rows shorter
    // than this are served as fast by the radix select
    // (a larger E from logits still takes this kernel for its softmax sums, with the radix select inside)
    if (E < 1 || E > 256 || (!logits && (E > kTkListE || V <= 3072))) return false;
    const bool vec = (V & 3) == 0 && ((uintptr_t)x & 15) == 0;
    // 512 lanes with 16 pieces each: measured against 256 x 32 and 1024 x 8 (30.7 / 33.0 / 34.3 us
    // for 1280 rows of 32000)
    const dim3 grid(n), block(512);
    if (logits) {
        if (vec) hipLaunchKernelGGL((topk_rows_kernel<16, 512, true, true>), grid, block, 0, s, x, V, E, ids, vals);
        else hipLaunchKernelGGL((topk_rows_kernel<16, 512, true, false>), grid, block, 0, s, x, V, E, ids, vals);
    } else {
        if (vec) hipLaunchKernelGGL((topk_rows_kernel<16, 512, false, true>), grid, block, 0, s, x, V, E, ids, vals);
        else hipLaunchKernelGGL((topk_rows_kernel<16, 512, false, false>), grid, block, 0, s, x, V, E, ids, vals);
    }
    *err = hipGetLastError();
    return true;
}

}  // namespace tw
