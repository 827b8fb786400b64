// Commit of the accepted draft path into the KV cache (the step after the
// acceptance walk of Alg. 2, needed before the next draft-verify iteration; KV
// append of Sec. 3.1).  The root of the verified tree already sits at cache row
// C; accepted node path[i] (tree row C + path[i]) moves to cache row C + 1 + i,
// the rejected rows are simply left behind, and the new context length is
// C + 1 + n_acc.
//
// In place and race free without barriers: path[] is strictly increasing with
// path[i] >= i + 1, so a move never writes a row that a LATER move reads, and a
// row that an EARLIER move reads may only be overwritten by a later move.  Each
// lane owns a 16-byte column of the row and performs the moves in ascending
// order, so its own loads precede its own conflicting stores in program order.
#include "twig_internal.h"

namespace tw {

constexpr int kCommitThreads = 256;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4c;

// grid (column blocks, views, B)
__global__ __launch_bounds__(kCommitThreads) void kv_commit_kernel(CommitArgs a) {
    const int b = blockIdx.z;
    const KvDev& kv = a.views[blockIdx.y];
    const size_t row_bytes = (size_t)kv.H * kv.d_h * (a.elem_bytes[blockIdx.y]);
    const size_t col = ((size_t)blockIdx.x * kCommitThreads + threadIdx.x) * 16;
    const int n = commit_n_acc(a.n_acc[b], a.T_max);
    // held where C + T_max cannot wrap; rows past the pool are clamped by pool_row
    const int C = commit_ctx(a.ctx_len[b]);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && a.new_ctx_len) a.new_ctx_len[b] = C + 1 + n;
    if (col >= row_bytes) return;
    char* base = (char*)kv.base;
    int prev = 0;
    for (int i = 0; i < n; ++i) {
        // keeps the order property even on malformed input: strictly increasing, inside the tree
        const int p = commit_next_node(prev, a.path[(int64_t)b * a.T_max + i], a.T_max);
        prev = p;
        if (p == i + 1) continue;   // already in place
        const char* src = base + (size_t)pool_row(kv, b, C + p) * row_bytes + col;
        char* dst = base + (size_t)pool_row(kv, b, C + 1 + i) * row_bytes + col;
        if (row_bytes - col >= 16) {
            *(u32x4c*)dst = *(const u32x4c*)src;
        } else {
            for (size_t e = 0; e < row_bytes - col; ++e) dst[e] = src[e];
        }
    }
}

hipError_t launch_kv_commit(const CommitArgs& a, int n_views, int B, size_t max_row_bytes, hipStream_t s) {
    if (n_views <= 0 || B <= 0) return hipSuccess;
    const int col_blocks = (int)((max_row_bytes + 16 * kCommitThreads - 1) / (16 * kCommitThreads));
    hipLaunchKernelGGL(kv_commit_kernel, dim3(col_blocks, n_views, B), dim3(kCommitThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace tw
