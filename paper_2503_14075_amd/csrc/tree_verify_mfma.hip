// Tree verification attention on the CDNA4 matrix cores (bf16 caches, d_h 64 or
// 128): the verification step of Alg. 2 -- Sec. 3.1 Eq. 2 under the
// topology-aware mask of Sec. 5.4 / App. A.  Every K/V byte of a (sequence,
// head) is fetched from HBM once and shared by all tree rows.
//
// Decomposition
//   grid (ceil(H/4), B, n_splits), 256 threads.  Wavefront w of a workgroup owns
//   head 4*blockIdx.x + w and walks the split's cache rows in chunks of 32.  The
//   four wavefronts never synchronise after the prologue; each has a private LDS
//   staging area.  Per chunk a wavefront
//     1. stores the prefetched K and V rows (16-byte lanes, fully coalesced
//        256-byte row segments) into LDS and issues the loads of the next chunk,
//     2. S^T[row][node] = K . Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows read
//        back from LDS as 16-byte fragments, B = Q fragments kept in registers),
//     3. online softmax per node: the 32x32 accumulator layout gives every lane
//        16 rows of one node, so the row maximum needs one cross-lane exchange,
//     4. O^T[col][node] += V^T . P^T with the same instruction: the accumulator
//        layout of step 2 is exactly a B-operand layout once the reduction index
//        is permuted, so P never leaves registers; V^T fragments are gathered
//        from LDS (one 8-byte read per row, regrouped with byte permutes).
//   Exponentials run in base 2 with scale*log2(e) folded into the logits.
//
// MFMA operand layouts used (lane l, g = l/32, i = l%32):
//   A[i][8g+e], B[8g+e][i] for e = 0..7;  D[8*(r/4) + 4g + r%4][i] for r = 0..15.
#include "mfma_util.h"
#include "twig_internal.h"

namespace tw {

constexpr int kMfThreads = 256;
constexpr int kChunk = 32;

template <int DH>
struct MfCfg {
    static constexpr int kRowB = DH * 2;            // bytes of one (row, head) segment
    static constexpr int kKStride = kRowB + 16;     // padded K row in LDS
    static constexpr int kVStride = kRowB;          // V row in LDS
    static constexpr int kLanesPerRow = kRowB / 16; // 16-byte lanes covering a segment
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;
    static constexpr int kLoads = kChunk / kRowsPerLoad;  // 16-byte loads per lane per tensor
    static constexpr int kDC = DH / 16;             // reduction chunks of QK^T
    static constexpr int kNQ = DH / 32;             // output column blocks of PV
    static constexpr int kWaveLds = kChunk * (kKStride + kVStride);
};

// K and V share one row mapping (same row_off / page_table) on this path.
template <int DH, int NB, bool PAGED>
__global__ __launch_bounds__(kMfThreads, (NB == 1 ? 2 : 1)) void verify_mfma_kernel(VerifyArgs a) {
    using Cf = MfCfg<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int s_parent[TW_MAX_TREE];
    __shared__ unsigned long long s_anc[TW_MAX_TREE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, li = lane & 31;
    const int b = blockIdx.y, split = blockIdx.z;
    const int h = blockIdx.x * 4 + wave;
    int T = a.n_nodes[b];
    T = T < 1 ? 1 : (T > a.T_max ? a.T_max : T);
    int C = a.ctx_len[b];
    C = C < 0 ? 0 : (C > a.max_rows - a.T_max ? a.max_rows - a.T_max : C);
    const int n_rows = C + T;
    int per = (n_rows + a.n_splits - 1) / a.n_splits;
    per = (per + kChunk - 1) / kChunk * kChunk;
    const int r_begin = min(split * per, n_rows), r_end = min(r_begin + per, n_rows);

    if (tid < TW_MAX_TREE) s_parent[tid] = tid < T ? a.parent[(int64_t)b * a.T_max + tid] : 0;
    __syncthreads();
    if (tid < TW_MAX_TREE) s_anc[tid] = tid < T ? ancestor_mask(s_parent, tid) : 0ull;
    __syncthreads();
    if (h >= a.H) return;

    unsigned char* ldsK = lds + wave * Cf::kWaveLds;
    unsigned char* ldsV = ldsK + kChunk * Cf::kKStride;

    // Q fragments (B operand): lane (i, g) holds Q[node 32nb+i][16c + 8g .. +7]; padding nodes are zero
    bf16x8 qf[NB][Cf::kDC];
    uint64_t anc[NB];
    const uint16_t* qb = (const uint16_t*)a.q;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int t = 32 * nb + li;
        const int tc = t < T ? t : T - 1;
        anc[nb] = s_anc[t];
        const u32x4* src = (const u32x4*)(qb + (((int64_t)b * a.T_max + tc) * a.H + h) * DH + 8 * g);
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            u32x4 v = src[2 * c];
            if (t >= T) v = (u32x4){0u, 0u, 0u, 0u};
            qf[nb][c] = as_bf16x8(v);
        }
    }

    floatx16 o[NB][Cf::kNQ];
    float run_m[NB], run_l[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        run_m[nb] = -INFINITY;
        run_l[nb] = 0.f;
#pragma unroll
        for (int q = 0; q < Cf::kNQ; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[nb][q][r] = 0.f;
    }
    const float sl2 = a.scale * kLog2e;

    // lane's share of a chunk load: row (lane / lanes_per_row) + rows_per_load * j,
    // 16-byte column lane % lanes_per_row of the head's segment
    const int ld_row = lane / Cf::kLanesPerRow, ld_col = lane % Cf::kLanesPerRow;
    const unsigned char* kbase = (const unsigned char*)a.k.base + (int64_t)h * Cf::kRowB + ld_col * 16;
    const unsigned char* vbase = (const unsigned char*)a.v.base + (int64_t)h * Cf::kRowB + ld_col * 16;
    const int64_t pool_stride = (int64_t)a.H * Cf::kRowB;
    const int64_t last_pool_row = a.k.pool_rows - 1;
    const int32_t* ptab = PAGED ? a.k.page_table + (int64_t)b * a.k.max_pages : nullptr;
    const int64_t row0 = PAGED ? 0 : (int64_t)a.k.row_off[b];
    const int last_row = r_end - 1;   // loads past the split re-read its last row (cached) and are masked

    // Paged caches: the page of every row this lane loads, looked up two chunks ahead
    // so the dependent data loads never wait on a table read.
    int pg[Cf::kLoads];
    auto lookup_pages = [&](int base) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            int r = base + ld_row + Cf::kRowsPerLoad * j;
            r = r < last_row ? r : last_row;
            int pi = r / a.k.page_rows;
            pi = pi < a.k.max_pages ? pi : a.k.max_pages - 1;
            pg[j] = ptab[pi];
        }
    };
    u32x4 pk[Cf::kLoads], pv[Cf::kLoads];
    auto issue_loads = [&](int base) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            int r = base + ld_row + Cf::kRowsPerLoad * j;
            r = r < last_row ? r : last_row;
            int64_t prow;
            if (PAGED)
                prow = (int64_t)pg[j] * a.k.page_rows + (r % a.k.page_rows);
            else
                prow = row0 + r;
            prow = prow < 0 ? 0 : (prow > last_pool_row ? last_pool_row : prow);
            pk[j] = __builtin_nontemporal_load((const u32x4*)(kbase + prow * pool_stride));   // streamed once
            pv[j] = __builtin_nontemporal_load((const u32x4*)(vbase + prow * pool_stride));
        }
    };

    if (r_begin >= r_end) {
        // empty split: nothing visible, the combine kernel skips it
        if (a.n_splits > 1 && g == 0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int t = 32 * nb + li;
                if (t < T) {
                    const int64_t slot = (((int64_t)split * a.B + b) * a.H + h) * a.T_max + t;
                    a.part_ml[slot * 2] = -INFINITY;
                    a.part_ml[slot * 2 + 1] = 0.f;
                }
            }
        }
        return;
    }
    if (PAGED) lookup_pages(r_begin);
    issue_loads(r_begin);
    if (PAGED) lookup_pages(r_begin + kChunk);
    for (int base = r_begin; base < r_end; base += kChunk) {
        // ---- 1. stage the prefetched chunk, start the next one -----------------
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            const int r = ld_row + Cf::kRowsPerLoad * j;
            *(u32x4*)(ldsK + r * Cf::kKStride + ld_col * 16) = pk[j];
            *(u32x4*)(ldsV + r * Cf::kVStride + ld_col * 16) = pv[j];
        }
        issue_loads(base + kChunk);
        if (PAGED) lookup_pages(base + 2 * kChunk);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- 2. S^T = K . Q^T ---------------------------------------------------
        floatx16 s[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[nb][r] = 0.f;
#pragma unroll
        for (int c = 0; c < Cf::kDC; ++c) {
            const bf16x8 kf = as_bf16x8(*(const u32x4*)(ldsK + li * Cf::kKStride + 32 * c + 16 * g));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nb][c], s[nb], 0, 0, 0);
        }

        // ---- 3. online softmax ---------------------------------------------------
        const bool need_mask = base + kChunk > C;
        bf16x8 pf[NB][2];
        float alpha[NB];
        bool any_rescale = false;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float x[16], mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                x[r] = s[nb][r] * sl2;
                if (need_mask) {
                    const int row = base + acc_row(r, g);
                    const bool vis = row < C || (row < n_rows && ((anc[nb] >> (row - C)) & 1ull));
                    x[r] = vis ? x[r] : -INFINITY;
                }
                mx = fmaxf(mx, x[r]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(run_m[nb], mx);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            alpha[nb] = fast_exp2(run_m[nb] - m_safe);   // 0 on the first visible chunk, 1 when the maximum holds
            any_rescale = any_rescale || (alpha[nb] != 1.f);
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // the row sum is taken over the bf16-rounded weights that enter the PV
                // product, so the normalised weights still sum to one
                const __bf16 pb = (__bf16)fast_exp2(x[r] - m_safe);
                psum += (float)pb;
                pf[nb][r >> 3][r & 7] = pb;
            }
            run_l[nb] = run_l[nb] * alpha[nb] + psum;
            run_m[nb] = m_new;
        }
        if (__any(any_rescale)) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int q = 0; q < Cf::kNQ; ++q)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[nb][q][r] *= alpha[nb];
        }

        // ---- 4. O^T += V^T . P^T -------------------------------------------------
        // reduction slot (g, e) of half c2 is chunk row acc_row(8*c2 + e, g); output
        // column block q holds columns kNQ*i + q.
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
            uint32_t w[8][Cf::kNQ / 2];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned char* p = ldsV + acc_row(8 * c2 + e, g) * Cf::kVStride + li * (Cf::kNQ * 2);
                if (Cf::kNQ == 4) {
                    const uint2 t2 = *(const uint2*)p;
                    w[e][0] = t2.x;
                    w[e][Cf::kNQ / 2 - 1] = t2.y;
                } else {
                    w[e][0] = *(const uint32_t*)p;
                }
            }
#pragma unroll
            for (int q = 0; q < Cf::kNQ; ++q) {
                u32x4 av;
                const uint32_t sel = (q & 1) ? 0x07060302u : 0x05040100u;
                av.x = __builtin_amdgcn_perm(w[1][q >> 1], w[0][q >> 1], sel);
                av.y = __builtin_amdgcn_perm(w[3][q >> 1], w[2][q >> 1], sel);
                av.z = __builtin_amdgcn_perm(w[5][q >> 1], w[4][q >> 1], sel);
                av.w = __builtin_amdgcn_perm(w[7][q >> 1], w[6][q >> 1], sel);
                const bf16x8 vf = as_bf16x8(av);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    o[nb][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nb][c2], o[nb][q], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: normalise or hand the partial to the combine kernel ----------
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int t = 32 * nb + li;
        const float l = run_l[nb] + __shfl_xor(run_l[nb], 32, 64);
        if (t >= T) continue;
        float* dst;
        float mul;
        if (a.n_splits == 1) {
            dst = a.out + (((int64_t)b * a.T_max + t) * a.H + h) * DH;
            mul = 1.f / l;
        } else {
            const int64_t slot = (((int64_t)split * a.B + b) * a.H + h) * a.T_max + t;
            dst = a.part_o + slot * DH;
            mul = 1.f;
            if (g == 0) {
                a.part_ml[slot * 2] = run_m[nb] * kLn2;   // natural-log units for the combine
                a.part_ml[slot * 2 + 1] = l;
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float* p = dst + Cf::kNQ * acc_row(r, g);
            if (Cf::kNQ == 4) {
                *(float4*)p = make_float4(o[nb][0][r] * mul, o[nb][1][r] * mul,
                                          o[nb][Cf::kNQ - 2][r] * mul, o[nb][Cf::kNQ - 1][r] * mul);
            } else {
                *(float2*)p = make_float2(o[nb][0][r] * mul, o[nb][1][r] * mul);
            }
        }
    }
}

template <int DH, int NB, bool PAGED>
static hipError_t launch_one(const VerifyArgs& a, hipStream_t s) {
    const dim3 grid((a.H + 3) / 4, a.B, a.n_splits);
    const size_t lds = 4 * (size_t)MfCfg<DH>::kWaveLds;
    hipError_t e = hipFuncSetAttribute((const void*)verify_mfma_kernel<DH, NB, PAGED>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((verify_mfma_kernel<DH, NB, PAGED>), grid, dim3(kMfThreads), lds, s, a);
    return hipGetLastError();
}

template <int DH, int NB>
static hipError_t launch_paging(const VerifyArgs& a, hipStream_t s) {
    return a.k.page_table ? launch_one<DH, NB, true>(a, s) : launch_one<DH, NB, false>(a, s);
}

bool verify_mfma_supported(const VerifyArgs& a, int dtype) {
    return dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.k.page_table == a.v.page_table &&
           a.k.row_off == a.v.row_off && a.k.page_rows == a.v.page_rows &&
           a.k.max_pages == a.v.max_pages && a.k.pool_rows == a.v.pool_rows;
}

hipError_t launch_verify_mfma(const VerifyArgs& a, hipStream_t s) {
    const bool wide = a.T_max > 32;
    if (a.d_h == 128) return wide ? launch_paging<128, 2>(a, s) : launch_paging<128, 1>(a, s);
    return wide ? launch_paging<64, 2>(a, s) : launch_paging<64, 1>(a, s);
}

}  // namespace tw
