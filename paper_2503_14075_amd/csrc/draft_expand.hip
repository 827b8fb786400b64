// One level of the tree-based drafting loop (Sec. 5.4 / App. A): the E most probable tokens of
// every expanded node become candidates of the drafted tree.  Pure bookkeeping -- parent, token,
// probability and cumulative confidence (parent's confidence x own probability) of this level's
// candidates, written into the per-sequence candidate arrays in generation order, plus the level's
// confidences as a contiguous row for the top-K select of the next level.  Latency-bound: a few
// hundred candidates per sequence.
#include "twig_internal.h"

namespace tw {

constexpr int kExpandThreads = 256;

struct ExpandArgs {
    const int32_t* sel;     // [B][n_exp] expanded nodes, indices into the previous level's slice; null = the root
    const int32_t* ids;     // [B][n_exp][E]
    const float* probs;     // [B][n_exp][E]
    int32_t* cand_parent;   // [B][N]
    int32_t* cand_token;    // [B][N]
    float* cand_prob;       // [B][N]
    float* cand_conf;       // [B][N]
    float* level_conf;      // [B][n_exp * E]
    int32_t n_exp, prev_off, out_off, E, N;
};

// grid (ceil(n_exp * E / 256), B)
__global__ __launch_bounds__(kExpandThreads) void draft_expand_kernel(ExpandArgs a) {
    const int b = blockIdx.y, i = blockIdx.x * kExpandThreads + threadIdx.x;
    const int n_new = a.n_exp * a.E;
    if (i >= n_new) return;
    const int j = i / a.E;
    const int64_t row = (int64_t)b * a.N;
    int parent = -1;
    float parent_conf = 1.f;
    if (a.sel) {
        // the expanded node: inside the previous level's slice [prev_off, out_off) whatever the contents
        parent = expand_parent(a.sel[(int64_t)b * a.n_exp + j], a.prev_off, a.out_off);
        parent_conf = a.cand_conf[row + parent];
    }
    const float p = a.probs[(int64_t)b * n_new + i];
    const float conf = parent_conf * p;
    const int c = a.out_off + i;
    a.cand_parent[row + c] = parent;
    a.cand_token[row + c] = a.ids[(int64_t)b * n_new + i];
    a.cand_prob[row + c] = p;
    a.cand_conf[row + c] = conf;
    a.level_conf[(int64_t)b * n_new + i] = conf;
}

hipError_t launch_draft_expand(const int32_t* sel, int n_exp, int prev_off, int out_off, const int32_t* ids,
                               const float* probs, int E, int N, int B, int32_t* cand_parent, int32_t* cand_token,
                               float* cand_prob, float* cand_conf, float* level_conf, hipStream_t s) {
    const ExpandArgs a = {sel, ids, probs, cand_parent, cand_token, cand_prob, cand_conf, level_conf,
                          n_exp, prev_off, out_off, E, N};
    hipLaunchKernelGGL(draft_expand_kernel, dim3((n_exp * E + kExpandThreads - 1) / kExpandThreads, B),
                       dim3(kExpandThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace tw
