// Sequence-based self-speculative decoding as the chain case of the tree calls
// (Sec. 3.1 "Decoding acceleration via self-speculation"; App. A, SSD paragraph;
// Alg. 1): the early exit of the draft model shapes the chain, and acceptance is
// the longest prefix of the draft that the target model predicts itself, plus
// the target's own next token.  A few integers per sequence: one lane each.
#include "twig_internal.h"

namespace tw {

__global__ __launch_bounds__(256) void chain_tree_kernel(const float* __restrict__ prob, float theta, int delta,
                                                         int B, int32_t* __restrict__ parent,
                                                         int32_t* __restrict__ n_nodes) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int T_max = delta + 1;
    int n = delta;
    if (prob) {
        for (int i = delta - 1; i >= 0; --i)
            if (prob[(int64_t)b * delta + i] < theta) n = i + 1;   // the token that falls below theta is kept
    }
    n_nodes[b] = 1 + n;
    for (int i = 0; i < T_max; ++i) parent[(int64_t)b * T_max + i] = i - 1;
}

__global__ __launch_bounds__(256) void chain_accept_kernel(const int32_t* __restrict__ draft,
                                                           const int32_t* __restrict__ argmx,
                                                           const int32_t* __restrict__ n_nodes, int T_max, int B,
                                                           int32_t* __restrict__ n_acc, int32_t* __restrict__ path,
                                                           int32_t* __restrict__ bonus) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int64_t base = (int64_t)b * T_max;
    const int T = tree_nodes(n_nodes[b], T_max);
    int n = 0;
    while (n + 1 < T && draft[base + n + 1] == argmx[base + n]) ++n;
    for (int i = 0; i < T_max; ++i) path[base + i] = i < n ? i + 1 : -1;
    n_acc[b] = n;
    bonus[b] = argmx[base + n];
}

hipError_t launch_chain_tree(const float* prob, float theta, int delta, int B, int32_t* parent, int32_t* n_nodes,
                             hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(chain_tree_kernel, dim3((B + 255) / 256), dim3(256), 0, s, prob, theta, delta, B, parent,
                       n_nodes);
    return hipGetLastError();
}

hipError_t launch_chain_accept(const int32_t* draft, const int32_t* argmx, const int32_t* n_nodes, int T_max, int B,
                               int32_t* n_acc, int32_t* path, int32_t* bonus, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(chain_accept_kernel, dim3((B + 255) / 256), dim3(256), 0, s, draft, argmx, n_nodes, T_max, B,
                       n_acc, path, bonus);
    return hipGetLastError();
}

}  // namespace tw
