// Ancestor masks and the greedy acceptance walk of tree-based self-speculative
// decoding (Sec. 5.4, App. A, Alg. 2).  One 64-lane wavefront per sequence:
// lane i owns tree node i, the tree fits a single uint64 per node.
#include "twig_internal.h"

namespace tw {

__global__ __launch_bounds__(64) void ancestor_masks_kernel(const int32_t* __restrict__ parent,
                                                            const int32_t* __restrict__ n_nodes,
                                                            int T_max, uint64_t* __restrict__ masks) {
    __shared__ int s_parent[TW_MAX_TREE];
    const int b = blockIdx.x, i = threadIdx.x;
    const int T = tree_nodes(n_nodes[b], T_max);
    s_parent[i] = i < T ? parent[(int64_t)b * T_max + i] : 0;
    __syncthreads();
    if (i < T_max) masks[(int64_t)b * T_max + i] = i < T ? ancestor_mask(s_parent, i) : 0ull;
}

// A node is matched when its draft id equals the target argmax of its parent.
// A node is reachable by the walk when every non-root node on its path is
// matched, i.e. (ancestors-or-self minus the root) is a subset of the matched
// set.  The deepest reachable node wins, ties toward the lower index: the key
// depth*64 + (63-i) is maximised over the wavefront.
__global__ __launch_bounds__(64) void accept_kernel(const int32_t* __restrict__ draft,
                                                    const int32_t* __restrict__ argmx,
                                                    const int32_t* __restrict__ parent,
                                                    const int32_t* __restrict__ n_nodes, int T_max,
                                                    int32_t* __restrict__ n_acc,
                                                    int32_t* __restrict__ path,
                                                    int32_t* __restrict__ bonus) {
    __shared__ int s_parent[TW_MAX_TREE];
    __shared__ unsigned long long s_best_anc;
    const int b = blockIdx.x, i = threadIdx.x;
    const int64_t base = (int64_t)b * T_max;
    const int T = tree_nodes(n_nodes[b], T_max);
    int par = 0;
    if (i < T) par = i == 0 ? -1 : clamp_parent(parent[base + i], i);
    s_parent[i] = par;
    __syncthreads();
    const uint64_t anc = i < T ? ancestor_mask(s_parent, i) : 0ull;
    const bool matched = i > 0 && i < T && draft[base + i] == argmx[base + par];
    const uint64_t matched_set = __ballot(matched);
    const bool reachable = i < T && ((anc & ~1ull) & ~matched_set) == 0ull;
    const int depth = __popcll(anc) - 1;
    int key = reachable ? depth * 64 + (63 - i) : -1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        int other = __shfl_xor(key, off, 64);
        key = other > key ? other : key;
    }
    const int best = 63 - (key & 63);
    if (i == best) s_best_anc = anc;
    __syncthreads();
    const uint64_t on_path = s_best_anc & ~1ull;  // accepted draft nodes
    if (i < T_max) {
        // parent[i] < i, so ascending node index along a path is root-to-leaf order
        const int n = __popcll(on_path);
        if ((on_path >> i) & 1ull) path[base + __popcll(on_path & ((1ull << i) - 1ull))] = i;
        if (i >= n) path[base + i] = -1;
        if (i == 0) {
            n_acc[b] = n;
            bonus[b] = argmx[base + best];
        }
    }
}

hipError_t launch_ancestor_masks(const int32_t* parent, const int32_t* n_nodes, int T_max, int B,
                                 uint64_t* masks, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(ancestor_masks_kernel, dim3(B), dim3(64), 0, s, parent, n_nodes, T_max, masks);
    return hipGetLastError();
}

hipError_t launch_accept(const int32_t* draft, const int32_t* argmx, const int32_t* parent,
                         const int32_t* n_nodes, int T_max, int B, int32_t* n_acc, int32_t* path,
                         int32_t* bonus, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, s, draft, argmx, parent, n_nodes, T_max,
                       n_acc, path, bonus);
    return hipGetLastError();
}

}  // namespace tw
