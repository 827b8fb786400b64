// Draft-side tree construction of tree-based self-speculative decoding
// (Sec. 5.4, App. A): per-node top-E tokens in rank order, cumulative path
// confidence of every drafted candidate, and the final pruning of the drafted
// tree to its N_max most confident candidates with a topological renumbering
// that the verification calls take as parent[].
#include "twig_internal.h"

namespace tw {

constexpr int kTbThreads = 256;

__device__ __forceinline__ uint32_t tb_order_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Rank order of the E survivors of a row: larger value first, equal values lower index first.
// kept [n][E] holds the survivors' indices in ascending order (output of the radix select).
__global__ __launch_bounds__(kTbThreads) void rank_sort_kernel(const float* __restrict__ vals, int V, int E,
                                                               int32_t* __restrict__ ids,
                                                               float* __restrict__ out_vals) {
    __shared__ uint32_t s_key[kTbThreads];
    __shared__ int32_t s_idx[kTbThreads];
    const int row = blockIdx.x, i = threadIdx.x;
    int32_t idx = 0;
    uint32_t key = 0u;
    float v = 0.f;
    if (i < E) {
        idx = ids[(int64_t)row * E + i];
        idx = idx < 0 ? 0 : (idx >= V ? V - 1 : idx);
        v = vals[(int64_t)row * V + idx];
        key = tb_order_key(v);
    }
    s_key[i] = key;
    s_idx[i] = idx;
    __syncthreads();
    if (i < E) {
        int rank = 0;
        for (int j = 0; j < E; ++j) rank += (s_key[j] > key) || (s_key[j] == key && s_idx[j] < idx);
        ids[(int64_t)row * E + rank] = idx;   // every slot is written exactly once: the order is total
        out_vals[(int64_t)row * E + rank] = v;
    }
}

// conf[b][i] = product of prob along the path root -> candidate i; -1 for slots past n_cand[b].
__global__ __launch_bounds__(kTbThreads) void tree_conf_kernel(const int32_t* __restrict__ cand_parent,
                                                               const float* __restrict__ cand_prob,
                                                               const int32_t* __restrict__ n_cand, int N,
                                                               float* __restrict__ conf) {
    const int b = blockIdx.y, i = blockIdx.x * kTbThreads + threadIdx.x;
    if (i >= N) return;
    int n = n_cand[b];
    n = n < 0 ? 0 : (n > N ? N : n);
    float c = -1.f;
    if (i < n) {
        // multiply from the node up to the root; parents precede children so the walk ends
        c = 1.f;
        int u = i;
        for (int step = 0; step < N && u >= 0; ++step) {
            c *= cand_prob[(int64_t)b * N + u];
            int p = cand_parent[(int64_t)b * N + u];
            u = p < u ? p : -1;
        }
    }
    conf[(int64_t)b * N + i] = c;
}

// kept [B][R] ascending candidate indices (radix select on conf).  Node 0 is the root; kept
// candidate number r becomes node 1 + r (valid candidates precede the -1 padding slots).
__global__ __launch_bounds__(kTbThreads) void tree_emit_kernel(TreeBuildArgs a) {
    extern __shared__ int32_t s_inv[];   // candidate index -> node id, 0 = not kept
    const int b = blockIdx.x, tid = threadIdx.x;
    int n = a.n_cand[b];
    n = n < 0 ? 0 : (n > a.N ? a.N : n);
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
            int c = a.kept[(int64_t)b * a.R + t - 1];
            c = c < 0 ? 0 : (c >= a.N ? a.N - 1 : c);
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

hipError_t launch_rank_sort(const float* vals, int n, int V, int E, int32_t* ids, float* out_vals,
                            hipStream_t s) {
    if (n == 0 || E == 0) return hipSuccess;
    hipLaunchKernelGGL(rank_sort_kernel, dim3(n), dim3(kTbThreads), 0, s, vals, V, E, ids, out_vals);
    return hipGetLastError();
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

}  // namespace tw
