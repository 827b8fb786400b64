// Draft-side tree construction of tree-based self-speculative decoding
// (Sec. 5.4, App. A): cumulative path confidence of every drafted candidate,
// and the final pruning of the drafted tree to its N_max most confident
// candidates with a topological renumbering that the verification calls take
// as parent[].  (The per-node top-E tokens in rank order come from the select
// kernel.)
#include "select_block.h"

namespace tw {

constexpr int kTbThreads = 256;

// Confidence of candidate i of sequence b: product of prob along the path root -> candidate;
// -1 for slots past n (the number of valid candidates).
__device__ __forceinline__ float path_confidence(const int32_t* __restrict__ cand_parent,
                                                 const float* __restrict__ cand_prob, int64_t row, int i, int n,
                                                 int N) {
    if (i >= n) return -1.f;
    // multiply from the node up to the root; parents precede children so the walk ends
    float c = 1.f;
    int u = i;
    for (int step = 0; step < N && u >= 0; ++step) {
        c *= cand_prob[row + u];
        u = cand_walk_parent(cand_parent[row + u], u);
    }
    return c;
}

__global__ __launch_bounds__(kTbThreads) void tree_conf_kernel(const int32_t* __restrict__ cand_parent,
                                                               const float* __restrict__ cand_prob,
                                                               const int32_t* __restrict__ n_cand, int N,
                                                               float* __restrict__ conf) {
    const int b = blockIdx.y, i = blockIdx.x * kTbThreads + threadIdx.x;
    if (i >= N) return;
    const int n = cand_count(n_cand[b], N);
    conf[(int64_t)b * N + i] = path_confidence(cand_parent, cand_prob, (int64_t)b * N, i, n, N);
}

// kept [B][R] ascending candidate indices (radix select on conf).  Node 0 is the root; kept
// candidate number r becomes node 1 + r (valid candidates precede the -1 padding slots).
// s_inv: N ints of LDS, candidate index -> node id, 0 = not kept.
__device__ __forceinline__ void emit_tree(const TreeBuildArgs& a, int b, int32_t* s_inv) {
    const int tid = threadIdx.x;
    const int n = cand_count(a.n_cand[b], a.N);
    const int n_keep = n < a.R ? n : a.R;
    for (int i = tid; i < a.N; i += kTbThreads) s_inv[i] = 0;
    __syncthreads();
    for (int r = tid; r < n_keep; r += kTbThreads) {
        const int c = a.kept[(int64_t)b * a.R + r];
        if (c >= 0 && c < a.N) s_inv[c] = 1 + r;
    }
    __syncthreads();
    const int64_t o = (int64_t)b * a.T_max;
    for (int t = tid; t < a.T_max; t += kTbThreads) {
        int32_t par = 0, tok = 0, src = -1;
        if (t == 0) {
            par = -1;
            tok = a.root_token[b];
        } else if (t <= n_keep) {
            const int c = kept_candidate(a.kept[(int64_t)b * a.R + t - 1], a.N);
            const int p = a.cand_parent[(int64_t)b * a.N + c];
            par = (p >= 0 && p < c) ? s_inv[p] : 0;   // a child of the root, or of a kept candidate
            par = par < t ? par : 0;
            tok = a.cand_token[(int64_t)b * a.N + c];
            src = c;
        }
        a.parent_out[o + t] = par;
        a.token_out[o + t] = tok;
        a.src_out[o + t] = src;
    }
    if (tid == 0) a.n_nodes_out[b] = 1 + n_keep;
}

__global__ __launch_bounds__(kTbThreads) void tree_emit_kernel(TreeBuildArgs a) {
    extern __shared__ int32_t s_inv[];
    emit_tree(a, blockIdx.x, s_inv);
}

// The three steps in one launch, one workgroup per sequence, when the candidates of a sequence
// fit the registers of the select (N <= 256 * KPT): confidences to the workspace, select from
// them in place, emit.  Each step reads what the same workgroup wrote before a barrier.
template <int KPT>
__global__ __launch_bounds__(kTbThreads) void tree_build_fused_kernel(TreeBuildArgs a, const float* cand_prob,
                                                                      float* conf) {
    extern __shared__ int32_t s_inv[];
    const int b = blockIdx.x;
    const int n = cand_count(a.n_cand[b], a.N);
    const int64_t row = (int64_t)b * a.N;
    for (int i = threadIdx.x; i < a.N; i += kTbThreads)
        conf[row + i] = path_confidence(a.cand_parent, cand_prob, row, i, n, a.N);
    __syncthreads();
    select_block<KPT, kTbThreads>(conf + row, a.N, a.R, const_cast<int32_t*>(a.kept) + (int64_t)b * a.R, nullptr);
    __syncthreads();
    emit_tree(a, b, s_inv);
}

hipError_t launch_tree_conf(const int32_t* cand_parent, const float* cand_prob, const int32_t* n_cand, int B,
                            int N, float* conf, hipStream_t s) {
    if (B == 0 || N == 0) return hipSuccess;
    hipLaunchKernelGGL(tree_conf_kernel, dim3((N + kTbThreads - 1) / kTbThreads, B), dim3(kTbThreads), 0, s,
                       cand_parent, cand_prob, n_cand, N, conf);
    return hipGetLastError();
}

hipError_t launch_tree_emit(const TreeBuildArgs& a, int B, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(tree_emit_kernel, dim3(B), dim3(kTbThreads), (size_t)a.N * sizeof(int32_t), s, a);
    return hipGetLastError();
}

// false: the candidates do not fit the fused kernel, the caller launches the three steps
bool launch_tree_build_fused(const TreeBuildArgs& a, const float* cand_prob, float* conf, int B, hipStream_t s,
                             hipError_t* err) {
    if (a.N > 12 * kTbThreads || B == 0) return false;
    const size_t lds = (size_t)a.N * sizeof(int32_t);
    if (a.N <= 4 * kTbThreads)
        hipLaunchKernelGGL(tree_build_fused_kernel<4>, dim3(B), dim3(kTbThreads), lds, s, a, cand_prob, conf);
    else
        hipLaunchKernelGGL(tree_build_fused_kernel<12>, dim3(B), dim3(kTbThreads), lds, s, a, cand_prob, conf);
    *err = hipGetLastError();
    return true;
}

}  // namespace tw
