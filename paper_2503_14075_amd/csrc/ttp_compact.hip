// Stable compaction of hidden-state and KV rows after token pruning
// (Sec. 3.1 Eq. 3, Sec. 4.2 Eq. 5; R = 0 is FinalWipe).  A pure row gather:
// one workgroup moves one destination row of one tensor with 16-byte lanes
// (as many lanes as the row has 16-byte pieces, up to 1024: one load and one
// store per lane for rows up to 16 KB, measured 6 % faster than two per lane),
// one launch covers every tensor of the pointer table and every sequence of a
// batch.
#include "twig_internal.h"

namespace tw {

constexpr int kCompactMaxThreads = 1024;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

template <bool kVec16>
__global__ __launch_bounds__(kCompactMaxThreads) void compact_kernel(CompactBatch cb, CompactTable tab,
                                                                  size_t row_bytes) {
    const int r = blockIdx.x, b = blockIdx.z;
    // a sequence length from device memory is held between the end of the visual span and the host's
    // upper bound, so every row index below stays inside [0, n_tot_all) of the sequence
    const int n_tot = cb.n_tot ? compact_n_tot(cb.n_tot[b], cb.v_start, cb.M, cb.n_tot_all) : cb.n_tot_all;
    if (r >= n_tot - cb.M + cb.R) return;
    const int64_t s0 = cb.src_off ? cb.src_off[b] : 0, d0 = cb.dst_off ? cb.dst_off[b] : 0;
    const bool in_kept = r >= cb.v_start && r < cb.v_start + cb.R;
    const int sr = compact_src_row_from(in_kept ? cb.kept[(int64_t)b * cb.R + r - cb.v_start] : 0, cb.R, cb.v_start,
                                        cb.M, n_tot, r);
    const char* src = (const char*)tab.src[blockIdx.y] + (size_t)(s0 + sr) * row_bytes;
    char* dst = (char*)tab.dst[blockIdx.y] + (size_t)(d0 + r) * row_bytes;
    if (kVec16) {
        // one descriptor per row and side; system-scope streaming loads and stores
        const __amdgpu_buffer_rsrc_t rs = raw_buffer(src, (uint32_t)row_bytes);
        const __amdgpu_buffer_rsrc_t rd = raw_buffer(dst, (uint32_t)row_bytes);
        const uint32_t n = (uint32_t)row_bytes;
        // rows longer than the workgroup: two independent 16-byte loads in flight per lane
        uint32_t o = threadIdx.x * 16u;
        const uint32_t kStep = blockDim.x * 16u;
        for (; o + kStep < n; o += 2 * kStep) {
            const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)o, 0, kAuxStream);
            const u32x4 c = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(o + kStep), 0, kAuxStream);
            __builtin_amdgcn_raw_buffer_store_b128(a, rd, (int)o, 0, kAuxStream);
            __builtin_amdgcn_raw_buffer_store_b128(c, rd, (int)(o + kStep), 0, kAuxStream);
        }
        if (o < n)
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_amdgcn_raw_buffer_load_b128(rs, (int)o, 0, kAuxStream), rd,
                                                   (int)o, 0, kAuxStream);
    } else {
        for (size_t i = threadIdx.x; i < row_bytes; i += blockDim.x) dst[i] = src[i];
    }
}

hipError_t launch_compact(const CompactBatch& cb, int B, int n_out_max, const CompactTable& tab,
                          int n_tensors, size_t row_bytes, hipStream_t s) {
    if (n_out_max <= 0 || n_tensors <= 0 || B <= 0) return hipSuccess;
    bool vec = (row_bytes % 16) == 0 && row_bytes < (1ull << 31);   // 32-bit offsets inside a row
    for (int t = 0; t < n_tensors; ++t)
        vec = vec && ((uintptr_t)tab.src[t] % 16 == 0) && ((uintptr_t)tab.dst[t] % 16 == 0);
    dim3 grid(n_out_max, n_tensors, B);
    // one lane per 16-byte piece (per byte on the unaligned path), in whole wavefronts
    const size_t pieces = vec ? (row_bytes + 15) / 16 : row_bytes;
    size_t threads = (pieces + 63) / 64 * 64;
    threads = threads < 64 ? 64 : (threads > kCompactMaxThreads ? kCompactMaxThreads : threads);
    if (vec)
        hipLaunchKernelGGL(compact_kernel<true>, grid, dim3((unsigned)threads), 0, s, cb, tab, row_bytes);
    else
        hipLaunchKernelGGL(compact_kernel<false>, grid, dim3((unsigned)threads), 0, s, cb, tab, row_bytes);
    return hipGetLastError();
}

}  // namespace tw
