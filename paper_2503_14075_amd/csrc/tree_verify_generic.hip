// Tree verification attention, generic path (fp32 or bf16 inputs, any
// supported d_h): plain fp32 vector arithmetic with LDS-staged K/V tiles.
// This is the path for fp32 caches and unusual head sizes; bf16 caches with
// d_h 64/128 take the matrix-core kernel in tree_verify_mfma.hip.
//
// Work split: grid (H, B, n_splits).  A workgroup owns one (sequence, head)
// and one contiguous range of cache rows; four lanes share a tree node (each
// owns every fourth output column).  Softmax is the usual online form; when
// the cache rows of a sequence are cut into several pieces the unnormalised
// partial (max, sum, output) triples go to the workspace and the workgroup
// that finishes last merges them in piece order (finish_split_unit).
#include "twig_internal.h"

namespace tw {

constexpr int kGenThreads = 256;
constexpr int kGenTile = 16;

// four consecutive elements (d_h is a multiple of 8 and the tensors are 16-byte aligned)
template <typename TIn>
__device__ __forceinline__ float4 ld4(const TIn* p);
template <>
__device__ __forceinline__ float4 ld4<float>(const float* p) { return *(const float4*)p; }
template <>
__device__ __forceinline__ float4 ld4<uint16_t>(const uint16_t* p) {
    const uint2 w = *(const uint2*)p;
    return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u),
                       __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xFFFF0000u));
}

// kCq = output columns a lane can own: 16 serves d_h <= 64, 32 serves d_h <= 128.
template <typename TIn, int kCq>
__global__ __launch_bounds__(kGenThreads) void verify_generic_kernel(VerifyArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ int s_parent[TW_MAX_TREE];
    __shared__ unsigned long long s_anc[TW_MAX_TREE];
    const int d_h = a.d_h, ld = d_h + 1, cq = d_h / 4;
    float* sQ = smem;                        // [64][ld]   pre-multiplied by scale
    float* sK = sQ + TW_MAX_TREE * ld;       // [kGenTile][ld]
    float* sV = sK + kGenTile * ld;          // [kGenTile][d_h]
    float* sP = sV + kGenTile * d_h;         // [64][kGenTile + 1]
    const int h = blockIdx.x, b = blockIdx.y, split = blockIdx.z;
    const int h_kv = h / a.group;   // the key/value head this query head reads
    const int tid = threadIdx.x;
    const SeqInfo sq = seq_info_from(a.n_nodes[b], a.ctx_len[b], a.T_max, a.max_rows, a.split_rows, a.n_splits, split);
    if (split >= sq.n_b) return;   // a piece past the end of this sequence (whole workgroup)
    const int T = sq.T, C = sq.C, r_begin = sq.r_begin, r_end = sq.r_end;

    if (tid < TW_MAX_TREE) s_parent[tid] = tid < T ? a.parent[(int64_t)b * a.T_max + tid] : 0;
    __syncthreads();
    if (tid < TW_MAX_TREE) s_anc[tid] = tid < T ? ancestor_mask(s_parent, tid) : 0ull;
    const TIn* q = (const TIn*)a.q;
    {
        // Q rows in pieces of four elements, all requested before the first is stored
        constexpr int kQLd = TW_MAX_TREE * 32 / kGenThreads;   // d_h <= 128: at most 32 pieces per row
        float4 qreg[kQLd];
#pragma unroll
        for (int u = 0; u < kQLd; ++u) {
            const int idx = tid + u * kGenThreads;
            const int t = idx / cq, c4 = idx - t * cq;
            qreg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (t < T) qreg[u] = ld4<TIn>(q + (((int64_t)b * a.T_max + t) * a.H + h) * d_h + 4 * c4);
        }
#pragma unroll
        for (int u = 0; u < kQLd; ++u) {
            const int idx = tid + u * kGenThreads;
            const int t = idx / cq, c4 = idx - t * cq;
            if (t < TW_MAX_TREE) {
                float* dst = sQ + t * ld + 4 * c4;
                dst[0] = a.scale * qreg[u].x;
                dst[1] = a.scale * qreg[u].y;
                dst[2] = a.scale * qreg[u].z;
                dst[3] = a.scale * qreg[u].w;
            }
        }
    }
    __syncthreads();

    const int t = tid >> 2, qd = tid & 3;   // node, column phase
    const uint64_t anc = s_anc[t];
    float run_m = -INFINITY, run_l = 0.f;   // run_l: this lane's share of the row sum
    float o[kCq];
#pragma unroll
    for (int cc = 0; cc < kCq; ++cc) o[cc] = 0.f;
    const TIn* kb = (const TIn*)a.k.base;
    const TIn* vb = (const TIn*)a.v.base;

    // A tile's K and V go through registers in pieces of four elements: all loads of the next tile
    // are requested before the current one is consumed (d_h <= 128: at most kGenLd pieces per thread).
    constexpr int kGenLd = kGenTile * 32 / kGenThreads;
    float4 kreg[kGenLd], vreg[kGenLd];
    auto load_tile = [&](int base) {
#pragma unroll
        for (int u = 0; u < kGenLd; ++u) {
            const int idx = tid + u * kGenThreads;
            const int r = idx / cq, c4 = idx - r * cq;
            kreg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            vreg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < kGenTile && base + r < r_end) {
                kreg[u] = ld4<TIn>(kb + (pool_row(a.k, b, base + r) * a.k.H + h_kv) * d_h + 4 * c4);
                vreg[u] = ld4<TIn>(vb + (pool_row(a.v, b, base + r) * a.k.H + h_kv) * d_h + 4 * c4);
            }
        }
    };
    load_tile(r_begin);
    for (int base = r_begin; base < r_end; base += kGenTile) {
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kGenLd; ++u) {
            const int idx = tid + u * kGenThreads;
            const int r = idx / cq, c4 = idx - r * cq;
            if (r < kGenTile) {
                float* dk = sK + r * ld + 4 * c4;
                dk[0] = kreg[u].x;
                dk[1] = kreg[u].y;
                dk[2] = kreg[u].z;
                dk[3] = kreg[u].w;
                *(float4*)(sV + r * d_h + 4 * c4) = vreg[u];
            }
        }
        load_tile(base + kGenTile);
        __syncthreads();
        float s[4], tile_m = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int jr = qd + 4 * jj, r = base + jr;
            float dot = 0.f;
#pragma unroll 8
            for (int c = 0; c < d_h; ++c) dot = fmaf(sQ[t * ld + c], sK[jr * ld + c], dot);
            const bool vis = r < r_end && (r < C || ((anc >> (r - C)) & 1ull));
            s[jj] = vis ? dot : -INFINITY;
            tile_m = fmaxf(tile_m, s[jj]);
        }
        tile_m = fmaxf(tile_m, __shfl_xor(tile_m, 1, 64));
        tile_m = fmaxf(tile_m, __shfl_xor(tile_m, 2, 64));
        const float m_new = fmaxf(run_m, tile_m);
        const float alpha = m_new == -INFINITY ? 1.f : expf(run_m - m_new);   // exp(-inf) = 0 on first hit
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const float p = s[jj] == -INFINITY ? 0.f : expf(s[jj] - m_new);
            sP[t * (kGenTile + 1) + qd + 4 * jj] = p;
            run_l = (jj == 0 ? run_l * alpha : run_l) + p;
        }
        run_m = m_new;
        __syncthreads();
#pragma unroll
        for (int cc = 0; cc < kCq; ++cc) o[cc] *= alpha;
        // columns past d_h re-read the row's last element and are never stored: no branch sits
        // between the shared-memory reads, so they are requested together
#pragma unroll 4
        for (int jr = 0; jr < kGenTile; ++jr) {
            const float p = sP[t * (kGenTile + 1) + jr];
#pragma unroll
            for (int cc = 0; cc < kCq; ++cc) {
                const int col = qd + 4 * cc;
                o[cc] = fmaf(p, sV[jr * d_h + (col < d_h ? col : d_h - 1)], o[cc]);
            }
        }
    }
    float l = run_l;
    l += __shfl_xor(l, 1, 64);
    l += __shfl_xor(l, 2, 64);
    if (sq.n_b == 1) {
        if (t >= T) return;
        const int64_t row = (((int64_t)b * a.T_max + t) * a.H + h) * d_h;
        const float inv = 1.f / l;
#pragma unroll
        for (int cc = 0; cc < kCq; ++cc) {
            if (cc < cq) {
                if (a.out_bf16) ((uint16_t*)a.out)[row + qd + 4 * cc] = f32_to_bf16(o[cc] * inv);
                else ((float*)a.out)[row + qd + 4 * cc] = o[cc] * inv;
            }
        }
    } else {
        if (t < T) {
            const int64_t slot = ((int64_t)split * a.B + b) * a.H + h;   // this piece's slot
            const __amdgpu_buffer_rsrc_t ro = raw_buffer(a.part_o + slot * a.o_stride, (uint32_t)(a.T_max * d_h * 4));
#pragma unroll
            for (int cc = 0; cc < kCq; ++cc)
                if (cc < cq)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, o[cc]), ro,
                                                          (t * d_h + qd + 4 * cc) * 4, 0, kAuxThrough);
            if (qd == 0)
                store_partial2(a.part_ml + slot * a.ml_stride, (uint32_t)(a.T_max * 8), (uint32_t)(t * 8),
                               make_float2(run_m, l));
        }
        finish_split_unit(a, b, h, T, sq.n_b, tid, kGenThreads);
    }
}

hipError_t launch_verify_generic(const VerifyArgs& a, int dtype, hipStream_t s) {
    const dim3 grid(a.H, a.B, a.n_splits);
    const size_t lds = ((size_t)TW_MAX_TREE * (a.d_h + 1) + (size_t)kGenTile * (a.d_h + 1) +
                        (size_t)kGenTile * a.d_h + (size_t)TW_MAX_TREE * (kGenTile + 1)) * sizeof(float);
    const bool narrow = a.d_h <= 64;
    if (dtype == TW_F32) {
        if (narrow) hipLaunchKernelGGL((verify_generic_kernel<float, 16>), grid, dim3(kGenThreads), lds, s, a);
        else hipLaunchKernelGGL((verify_generic_kernel<float, 32>), grid, dim3(kGenThreads), lds, s, a);
    } else {
        if (narrow) hipLaunchKernelGGL((verify_generic_kernel<uint16_t, 16>), grid, dim3(kGenThreads), lds, s, a);
        else hipLaunchKernelGGL((verify_generic_kernel<uint16_t, 32>), grid, dim3(kGenThreads), lds, s, a);
    }
    return hipGetLastError();
}

}  // namespace tw
