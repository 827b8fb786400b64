// Pruning score (Sec. 3.1 Eq. 2-3, head mean as in Sec. 5.1 Eq. 7), fast path
// for prompts whose logits fit the register file: bf16, d_h 64/128, at most 64
// scoring rows and at most 8*CPW*32 = 768 keys.
//
// One 8-wavefront workgroup per compute unit loops over (sequence, head) pairs.
// Wavefront w owns key chunks w, w+8, w+16, ... of the pair (32 keys each):
// The pair's Q rows sit in LDS (double-buffered across pairs), shared by all waves.
//   pass 1  K chunk -> LDS -> K.Q^T on the matrix cores; per-row running
//           (max, sum); the exponentials 2^(logit - running max) of the chunk
//           STAY in registers (16-bit fixed point) with that reference maximum.
//   merge   the eight wavefronts exchange their row statistics through LDS
//           -> max + log2(sum) per row.
//   pass 2  weights = stored exponential * 2^(reference - that), transposed through
//           the wavefront's LDS stage so that a lane owns a key, summed over the
//           scoring rows in a fixed order -> partial[b][h][m].
// K is read from HBM exactly once and nothing of size rows x keys is stored.
// Two chunks per wavefront are always in flight: a prefetch slot is refilled
// (with the pair's third chunk, then with the next pair's chunks) as soon as its
// contents have been staged, so the memory pipe stays busy across pairs.  The loop count of every workgroup
// is fixed by the grid; there are no waits on other workgroups.
#include "mfma_util.h"
#include "twig_internal.h"

namespace tw {

constexpr int kRsWaves = 8;
constexpr int kRsThreads = kRsWaves * 64;
constexpr int kRsChunk = 32;
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// Two weights in (0, 1] as 16-bit fixed point (v_cvt_pknorm_u16_f32): absolute step 2^-16.
__device__ __forceinline__ uint32_t pack_unorm16(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pknorm_u16(a, b));
}
__device__ __forceinline__ float unorm16_lo(uint32_t v) { return (float)(v & 0xFFFFu); }
__device__ __forceinline__ float unorm16_hi(uint32_t v) { return (float)(v >> 16); }

template <int DH>
struct RsCfg {
    static constexpr int kRowB = DH * 2;
    static constexpr int kKStride = 272;   // bytes; K rows (<= 256 B) padded, and 68 floats per key in pass 2
    static constexpr int kLanesPerRow = kRowB / 16;
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;
    static constexpr int kLoads = kRsChunk / kRowsPerLoad;
    static constexpr int kDC = DH / 16;
    static constexpr int kWaveLds = kRsChunk * kKStride;
};

template <int DH, int NB, int CPW>
__global__ __launch_bounds__(kRsThreads, 2) void score_resident_kernel(ScoreArgs a, int n_pairs) {
    using Cf = RsCfg<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, li = lane & 31;
    unsigned char* stage = lds + wave * Cf::kWaveLds;
    // row statistics of the eight wavefronts, double-buffered by pair parity: [2][waves][64 rows][2]
    float* s_part = (float*)(lds + kRsWaves * Cf::kWaveLds);
    // Q rows of the pair, 272-byte rows like the K stage, double-buffered: [2][32*NB rows]
    unsigned char* s_q = lds + kRsWaves * Cf::kWaveLds + 2 * kRsWaves * 64 * 2 * sizeof(float);
    constexpr int kQBuf = 32 * NB * Cf::kKStride;
    // per-key sums of the pair being finished, written out (coalesced) at the top of the next pair
    float* s_keys = (float*)(s_q + 2 * kQBuf);
    // parked exponentials of chunk 0: [wave][NB*2 pieces][64 lanes] 16-byte vectors
    unsigned char* s_park = (unsigned char*)(s_keys + kRsWaves * CPW * kRsChunk) + wave * (NB * 2 * 64 * 16);
    constexpr int kQLoads = (32 * NB * Cf::kLanesPerRow + kRsThreads - 1) / kRsThreads;   // 16-byte pieces per thread

    const int ld_row = lane / Cf::kLanesPerRow, ld_col = lane % Cf::kLanesPerRow;
    const int64_t pool_stride = (int64_t)a.H * Cf::kRowB;
    const int64_t last_pool_row = a.k.pool_rows - 1;
    const float sl2 = a.scale * kLog2e;
    const int span_end = a.v_start + a.M;
    const uint16_t* qb = (const uint16_t*)a.q_sel;

    // Two prefetch slots: chunk 0 and 2 of a pair use slot 0, chunk 1 uses slot 1.
    static_assert(CPW == 3, "the prefetch schedule below is written for three chunks per wavefront");
    u32x4 pk[2][Cf::kLoads];
    // Per-pair scalars.  The pair index is uniform across the workgroup; readfirstlane makes that
    // visible to the compiler so the small table reads are scalar loads and never sit in the
    // vector-memory queue in front of (or behind) the K prefetches.
    struct PairInfo {
        int b, h, n_q, n_tot, pos0;
        int64_t row0;
    };
    auto pair_info = [&](int pr) {
        PairInfo p;
        p.b = __builtin_amdgcn_readfirstlane(pr / a.H);
        p.h = __builtin_amdgcn_readfirstlane(pr - p.b * a.H);
        // constant address space: these tables are not written while the kernel runs
        typedef const int32_t __attribute__((address_space(4))) * ctab;
        int n_q = a.n_q ? ((ctab)a.n_q)[p.b] : a.n_q_max;
        p.n_q = n_q < 1 ? 1 : (n_q > a.n_q_max ? a.n_q_max : n_q);
        int n_tot = ((ctab)a.n_tot)[p.b];
        p.n_tot = n_tot < 0 ? 0 : (n_tot > a.n_tot_max ? a.n_tot_max : n_tot);
        p.pos0 = ((ctab)a.q_pos0)[p.b];
        p.row0 = (int64_t)((ctab)a.k.row_off)[p.b];
        return p;
    };
    // loads of owned chunk c of a pair (32 keys x one head segment, 16 bytes per lane per load)
    auto issue_chunk = [&](const PairInfo& p, int c, int slot) {
        const unsigned char* kbase = (const unsigned char*)a.k.base + (int64_t)p.h * Cf::kRowB + ld_col * 16;
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            int r = kRsChunk * (wave + kRsWaves * c) + ld_row + Cf::kRowsPerLoad * j;
            r = r < p.n_tot - 1 ? r : p.n_tot - 1;   // past the end: the last key again (cached), masked later
            int64_t prow = p.row0 + r;
            prow = prow < 0 ? 0 : (prow > last_pool_row ? last_pool_row : prow);
            // pool rows and the row pitch both fit 32 bits: one 32x32->64 multiply-add per address
            pk[slot][j] = __builtin_nontemporal_load(
                (const u32x4*)(kbase + (uint64_t)(uint32_t)prow * (uint32_t)pool_stride));
        }
    };
    // this thread's 16-byte pieces of the pair's Q rows (zero past n_q)
    u32x4 qn[kQLoads];
    auto issue_q = [&](const PairInfo& p) {
        const int b = p.b, h = p.h, n_q = p.n_q;
#pragma unroll
        for (int u = 0; u < kQLoads; ++u) {
            const int piece = tid + u * kRsThreads;
            const int i = piece / Cf::kLanesPerRow, col = piece % Cf::kLanesPerRow;
            const int ic = i < n_q ? i : n_q - 1;
            u32x4 v = *(const u32x4*)(qb + (((int64_t)b * a.n_q_max + ic) * a.H + h) * DH + 8 * col);
            if (i >= n_q) v = (u32x4){0u, 0u, 0u, 0u};
            qn[u] = v;
        }
    };
    auto store_q = [&](int parity) {
#pragma unroll
        for (int u = 0; u < kQLoads; ++u) {
            const int piece = tid + u * kRsThreads;
            const int i = piece / Cf::kLanesPerRow, col = piece % Cf::kLanesPerRow;
            if (i < 32 * NB) *(u32x4*)(s_q + parity * kQBuf + i * Cf::kKStride + col * 16) = qn[u];
        }
    };
    auto lds_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    int pair = blockIdx.x;
    if (pair >= n_pairs) return;
    PairInfo cur = pair_info(pair);
    issue_chunk(cur, 0, 0);
    issue_chunk(cur, 1, 1);
    issue_q(cur);
    store_q(0);
    float* prev_partial = nullptr;
    auto write_out = [&](float* dst) {
        for (int m = tid; m < a.M; m += kRsThreads) dst[m] = s_keys[a.v_start + m];
    };
    for (int it = 0; pair < n_pairs; ++it) {
        __syncthreads();   // Q rows of this pair are in LDS; pass 2 of the previous pair is complete
        if (it > 0) write_out(prev_partial);
        const int next = pair + gridDim.x;
        const bool has_next = next < n_pairs;
        const PairInfo nxt = pair_info(has_next ? next : pair);
        const int n_q = cur.n_q, n_tot = cur.n_tot, pos0 = cur.pos0;
        float* partial = a.ws + ((int64_t)cur.b * a.H + cur.h) * a.M;

        const unsigned char* qbuf = s_q + (it & 1) * kQBuf;
        const int vis_all = a.causal ? min(pos0 + 1, n_tot) : n_tot;   // keys visible to every row
        int vis_end[NB];
        float run_m[NB], run_l[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            vis_end[nb] = a.causal ? min(pos0 + 32 * nb + li + 1, n_tot) : n_tot;
            run_m[nb] = -INFINITY;
            run_l[nb] = 0.f;
        }

        // after chunk 0 is staged its slot takes chunk 2 of this pair; after chunks 1 and 2 the
        // slots take chunks 1 and 0 of the next pair
        auto refill = [&](int c) {
            if (c == 0) issue_chunk(cur, 2, 0);
            else if (has_next) issue_chunk(nxt, c == 1 ? 1 : 0, c == 1 ? 1 : 0);
        };
        // ---- pass 1: logits of the owned chunks into registers, row statistics -----
        // es[c][nb][r/2] = the pair 2^(logit - ref[c][nb]) for r, r+1; values in (0, 1], ref = the
        // row's running maximum after chunk c.  Stored as 16-bit fixed point: half the registers
        // of fp32.  A stored value is off by at most 2^-17, so a weight (stored value times
        // 2^(ref - max)/sum <= 1/sum) is off by at most 2^-17/sum and a score, a mean of weights,
        // by at most 2^-17 * mean(1/sum) <= 3.8e-6 if every rounding went the same way; with
        // roundings of mixed sign the error is that divided by about sqrt(H * n_q), and for the
        // near-uniform attention of real prompts (sum ~ n_tot) it is below 1e-8.
        // Chunks 1 and 2 live in registers; chunk 0 is parked in a private LDS area (s_park) so that
        // the kernel fits 256 registers without scratch spills -- a scratch reload would wait on
        // the vector-memory counter and with it on every K prefetch in flight.
        uint32_t es[CPW][NB][8];
        float ref[CPW][NB];
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int base = kRsChunk * (wave + kRsWaves * c);
            if (base < n_tot) {
#pragma unroll
                for (int j = 0; j < Cf::kLoads; ++j)
                    *(u32x4*)(stage + (ld_row + Cf::kRowsPerLoad * j) * Cf::kKStride + ld_col * 16) = pk[c & 1][j];
                refill(c);   // the slot's registers are free again: keep the memory pipe full
                lds_sync();
                const bool need_mask = base + kRsChunk > vis_all;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    // one 32-row block at a time keeps a single accumulator tile live
                    floatx16 s;
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                    for (int dc = 0; dc < Cf::kDC; ++dc) {
                        // A: lane (j, g) takes K[key j][16dc + 8g .. +7];  B: Q[row 32nb+i][same columns]
                        const bf16x8 kf = as_bf16x8(*(const u32x4*)(stage + li * Cf::kKStride + 32 * dc + 16 * g));
                        const bf16x8 qf = as_bf16x8(
                            *(const u32x4*)(qbuf + (32 * nb + li) * Cf::kKStride + 32 * dc + 16 * g));
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf, s, 0, 0, 0);
                    }
                    float x[16], mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        x[r] = s[r] * sl2;
                        if (need_mask && base + acc_row(r, g) >= vis_end[nb]) x[r] = -INFINITY;
                        mx = fmaxf(mx, x[r]);
                    }
                    const float m_new = fmaxf(run_m[nb], mx);
                    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                    float psum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        const float e0 = fast_exp2(x[r] - m_safe), e1 = fast_exp2(x[r + 1] - m_safe);
                        psum += e0;
                        psum += e1;
                        es[c][nb][r >> 1] = pack_unorm16(e0, e1);
                    }
                    if (c == 0) {
                        *(u32x4*)(s_park + ((nb * 2 + 0) * 64 + lane) * 16) =
                            (u32x4){es[0][nb][0], es[0][nb][1], es[0][nb][2], es[0][nb][3]};
                        *(u32x4*)(s_park + ((nb * 2 + 1) * 64 + lane) * 16) =
                            (u32x4){es[0][nb][4], es[0][nb][5], es[0][nb][6], es[0][nb][7]};
                    }
                    ref[c][nb] = m_safe;
                    run_l[nb] = run_l[nb] * fast_exp2(run_m[nb] - m_safe) + psum;
                    run_m[nb] = m_new;
                }
                lds_sync();   // fragment reads done before the stage is reused
            } else {
                refill(c);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    ref[c][nb] = 0.f;
#pragma unroll
                    for (int r = 0; r < 8; ++r) es[c][nb][r] = 0u;
                    if (c == 0) {
                        *(u32x4*)(s_park + ((nb * 2 + 0) * 64 + lane) * 16) = (u32x4){0u, 0u, 0u, 0u};
                        *(u32x4*)(s_park + ((nb * 2 + 1) * 64 + lane) * 16) = (u32x4){0u, 0u, 0u, 0u};
                    }
                }
            }
        }
        // ---- merge: lane groups, then wavefronts ------------------------------------
        float* part = s_part + (size_t)(it & 1) * kRsWaves * 64 * 2;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float om = __shfl_xor(run_m[nb], 32, 64), ol = __shfl_xor(run_l[nb], 32, 64);
            const float m = fmaxf(run_m[nb], om);
            const float m_safe = m == -INFINITY ? 0.f : m;
            const float l = run_l[nb] * fast_exp2(run_m[nb] - m_safe) + ol * fast_exp2(om - m_safe);
            if (g == 0) {
                part[(wave * 64 + 32 * nb + li) * 2] = m;
                part[(wave * 64 + 32 * nb + li) * 2 + 1] = l;
            }
        }
        __syncthreads();
        if (has_next) issue_q(nxt);
        float mc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int i = 32 * nb + li;
            float wm[kRsWaves], wl[kRsWaves], m = -INFINITY;
#pragma unroll
            for (int w = 0; w < kRsWaves; ++w) {
                wm[w] = part[(w * 64 + i) * 2];
                wl[w] = part[(w * 64 + i) * 2 + 1];
                m = fmaxf(m, wm[w]);
            }
            const float m_safe = m == -INFINITY ? 0.f : m;
            float l = 0.f;
#pragma unroll
            for (int w = 0; w < kRsWaves; ++w) l += wl[w] * fast_exp2(wm[w] - m_safe);
            mc[nb] = (i < n_q && l > 0.f) ? m + log2f(l) : INFINITY;   // +inf: the row contributes nothing
        }
        // ---- pass 2: weights from registers, per-key sums over the scoring rows -----
        float* stage_f = (float*)stage;   // [32 keys][68] floats
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int base = kRsChunk * (wave + kRsWaves * c);
            if (base < span_end && base + kRsChunk > a.v_start) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    // one exponential per (chunk, row); 1/65535 undoes the fixed-point scale
                    const float w = fast_exp2(ref[c][nb] - mc[nb]) * (1.f / 65535.f);
                    uint32_t e[8];
                    if (c == 0) {
                        const u32x4 lo = *(const u32x4*)(s_park + ((nb * 2 + 0) * 64 + lane) * 16);
                        const u32x4 hi = *(const u32x4*)(s_park + ((nb * 2 + 1) * 64 + lane) * 16);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            e[r] = lo[r];
                            e[4 + r] = hi[r];
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 8; ++r) e[r] = es[c][nb][r];
                    }
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        stage_f[acc_row(r, g) * 68 + 32 * nb + li] = unorm16_lo(e[r >> 1]) * w;
                        stage_f[acc_row(r + 1, g) * 68 + 32 * nb + li] = unorm16_hi(e[r >> 1]) * w;
                    }
                }
                lds_sync();
                // lane (key li, half g) adds rows [16*NB*g, 16*NB*(g+1)) in index order
                float sum = 0.f;
#pragma unroll
                for (int q = 0; q < 4 * NB; ++q) {
                    const float4 v = *(const float4*)(stage_f + li * 68 + 16 * NB * g + 4 * q);
                    sum += v.x;
                    sum += v.y;
                    sum += v.z;
                    sum += v.w;
                }
                const float other = __shfl_xor(sum, 32, 64);
                const int j = base + li;
                if (g == 0) s_keys[j] = sum + other;
                lds_sync();
            }
        }
        if (has_next) store_q((it + 1) & 1);   // that buffer was last read before this pair's barrier
        prev_partial = partial;
        pair = next;
        cur = nxt;
    }
    __syncthreads();
    write_out(prev_partial);
}

static int resident_grid(int n_pairs) {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            v = 256;
        n_cu = v;
    }
    return n_pairs < n_cu ? n_pairs : n_cu;
}

template <int DH, int NB, int CPW>
static hipError_t launch_rs(const ScoreArgs& a, hipStream_t s) {
    const int n_pairs = a.B * a.H;
    const size_t lds = (size_t)kRsWaves * RsCfg<DH>::kWaveLds + 2 * kRsWaves * 64 * 2 * sizeof(float) +
                       2 * (size_t)32 * NB * RsCfg<DH>::kKStride + (size_t)kRsWaves * CPW * kRsChunk * sizeof(float) +
                       (size_t)kRsWaves * NB * 2 * 64 * 16;
    hipError_t e = hipFuncSetAttribute((const void*)score_resident_kernel<DH, NB, CPW>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((score_resident_kernel<DH, NB, CPW>), dim3(resident_grid(n_pairs)), dim3(kRsThreads), lds,
                       s, a, n_pairs);
    return hipGetLastError();
}

// up to 64 scoring rows x 768 keys per (sequence, head)
bool score_resident_supported(const ScoreArgs& a, int dtype) {
    return dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.n_q_max <= 64 &&
           a.n_tot_max <= kRsWaves * 3 * kRsChunk;
}

hipError_t launch_score_resident(const ScoreArgs& a, hipStream_t s) {
    if (a.n_q_max <= 32) return a.d_h == 128 ? launch_rs<128, 1, 3>(a, s) : launch_rs<64, 1, 3>(a, s);
    return a.d_h == 128 ? launch_rs<128, 2, 3>(a, s) : launch_rs<64, 2, 3>(a, s);
}

}  // namespace tw
