// Pruning score (Sec. 3.1 Eq. 2-3, head mean as in Sec. 5.1 Eq. 7), fast path
// for prompts whose weights fit on chip: bf16, d_h 64/128, at most 64 scoring
// rows, at most 768 keys, a visual span that fits the LDS table.
//
// One 8-wavefront workgroup per compute unit loops over (sequence, head) pairs.
// Wavefront w owns key chunks w, w+8, w+16 of the pair (32 keys each).
//   pass 1  K chunk: coalesced loads -> registers (two chunks always in flight
//           per wavefront, across pair boundaries) -> a 16-row LDS stage ->
//           matrix-core operand registers.  K.Q^T with Q read from LDS; per-row
//           running (max, sum); the exponentials 2^(logit - running max), as
//           16-bit fixed point, go to an LDS table [key pair][row]; the reference
//           maximum of each (chunk, row) stays in a register.
//   merge   the eight wavefronts publish their row statistics -> max + log2(sum)
//           per scoring row.
//   pass 2  each wavefront, for its own chunks: stored exponential * 2^(reference
//           - that), summed over the scoring rows in a fixed order by four lanes
//           per key pair -> partial[b][h][m].
// K is read from HBM exactly once, nothing of size rows x keys leaves the chip.
// Per-pair table reads are scalar loads, no load sits inside a branch and the
// kernel has no scratch spills: any of these would make a wavefront wait for
// every K load in flight instead of the one it needs.  The loop count of every
// workgroup is fixed by the grid; there are no waits on other workgroups.
#include "mfma_util.h"
#include "twig_internal.h"

namespace tw {

constexpr int kRsWaves = 8;
constexpr int kRsThreads = kRsWaves * 64;
constexpr int kRsChunk = 32;
constexpr int kRsCpw = 3;                                  // chunks per wavefront
constexpr int kRsMaxKeys = kRsWaves * kRsCpw * kRsChunk;   // 768
constexpr int kRsLdsBytes = 160 * 1024;                    // LDS of a compute unit

// Value of the lane's neighbour inside its group of four (DPP quad_perm control: 0xB1 swaps lanes
// 0<->1 and 2<->3, 0x4E swaps 0<->2 and 1<->3).
template <int CTRL>
__device__ __forceinline__ float quad_swap(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int DH, int NB>
struct RsCfg {
    static constexpr int kRowB = DH * 2;
    static constexpr int kDC = DH / 16;
    static constexpr int kRows = 32 * NB;             // scoring rows held
    static constexpr int kStride = 272;               // bytes per K or Q row in LDS (padded)
    static constexpr int kPieces = kRowB / 16;        // 16-byte pieces per row = lanes per row of a load
    static constexpr int kRowsPerLoad = 64 / kPieces;
    static constexpr int kLoads = kRsChunk / kRowsPerLoad;   // loads per chunk (per lane)
    static constexpr int kHalf = kLoads / 2;                  // loads per 16-row half
    static constexpr int kEsStride = kRows + 4;       // dwords per key pair in the table (padded)
    static constexpr int kWStride = kRows + 4;        // floats per lane group of factors (padded)
    // LDS layout (bytes); the table of exponentials comes last and is sized by the visual span
    static constexpr int kOffQ = 0;
    static constexpr int kOffStage = kOffQ + kRows * kStride;
    static constexpr int kWaveStage = 16 * kStride;
    static constexpr int kOffPart = kOffStage + kRsWaves * kWaveStage;
    static constexpr int kOffW = kOffPart + kRsWaves * kRows * 2 * 4;
    static constexpr int kOffEs = kOffW + kRsWaves * 2 * kWStride * 4;
    static constexpr int kEsChunk = 16 * kEsStride * 4;        // bytes of table per 32-key chunk
    static constexpr int kMaxSpanChunks = (kRsLdsBytes - kOffEs) / kEsChunk;
};

template <int DH, int NB>
__global__ __launch_bounds__(kRsThreads, 2) void score_resident_kernel(ScoreArgs a, int n_pairs) {
    using Cf = RsCfg<DH, NB>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    // the wavefront index in a scalar register: branches on it are real branches, not lane masks
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, li = lane & 31;
    const int ld_row = lane / Cf::kPieces, ld_col = lane % Cf::kPieces;
    unsigned char* s_q = lds + Cf::kOffQ;                              // Q rows of the pair
    unsigned char* stage = lds + Cf::kOffStage + wave * Cf::kWaveStage;   // 16 K rows of this wavefront
    float* s_part = (float*)(lds + Cf::kOffPart);    // [wave][row][2]: running max and sum of each wavefront
    float* w_tab = (float*)(lds + Cf::kOffW) + wave * (2 * Cf::kWStride);   // [lane group][row] factors
    // [chunk of the span][key pair][kEsStride]: two 16-bit exponentials per scoring row
    uint32_t* s_es = (uint32_t*)(lds + Cf::kOffEs);

    const uint32_t pool_stride = (uint32_t)(a.k.H * Cf::kRowB);   // a cache row holds the key heads
    const int64_t last_pool_row = a.k.pool_rows - 1;
    const float sl2 = a.scale * kLog2e;
    const int span_end = a.v_start + a.M;
    const int first_chunk = a.v_start / kRsChunk;
    const uint16_t* qb = (const uint16_t*)a.q_sel;

    // Per-pair scalars.  The pair index is uniform across the workgroup; readfirstlane makes that
    // visible to the compiler, and the constant address space says the tables are not written
    // while the kernel runs, so the reads become scalar loads.
    struct PairInfo {
        int b, h, n_q, n_tot, pos0;
        int64_t row0;
    };
    auto pair_info = [&](int pr) {
        typedef const int32_t __attribute__((address_space(4))) * ctab;
        PairInfo p;
        p.b = __builtin_amdgcn_readfirstlane(pr / a.H);
        p.h = __builtin_amdgcn_readfirstlane(pr - p.b * a.H);
        // rows of the sequence that fall into this launch's window (none: every row is masked out
        // and the pair's partial sums come out as zeros)
        const int q_rows = a.q_stride ? a.q_stride : a.n_q_max;
        int n_q = a.n_q ? ((ctab)a.n_q)[p.b] : q_rows;
        n_q = (n_q < 1 ? 1 : (n_q > q_rows ? q_rows : n_q)) - a.row0;
        p.n_q = n_q < 0 ? 0 : (n_q > a.n_q_max ? a.n_q_max : n_q);
        int n_tot = ((ctab)a.n_tot)[p.b];
        p.n_tot = n_tot < 0 ? 0 : (n_tot > a.n_tot_max ? a.n_tot_max : n_tot);
        p.pos0 = ((ctab)a.q_pos0)[p.b] + a.row0;
        p.row0 = (int64_t)((ctab)a.k.row_off)[p.b];
        return p;
    };
    // Two prefetch slots: chunks 0 and 2 of a pair use slot 0, chunk 1 uses slot 1.  A load moves 16
    // bytes per lane, kPieces lanes per key row.  Every call issues the same number of loads on every
    // path; `live` false (no further pair) points all lanes at one row instead of skipping them.
    u32x4 pk[2][Cf::kLoads];
    auto issue_chunk = [&](const PairInfo& p, int c, int slot, bool live) {
        // scalar part of the address: the sequence's first row (kept inside the pool) and the head
        const int64_t row0 = p.row0 < 0 ? 0 : (p.row0 > last_pool_row ? last_pool_row : p.row0);
        const unsigned char* sbase =
            (const unsigned char*)a.k.base + (uint64_t)row0 * pool_stride + (int64_t)(p.h / a.group) * Cf::kRowB;
        // lane part, 32 bits: its key row, held below the sequence's end and the pool's end
        const int64_t room = last_pool_row - row0;
        int last = live ? p.n_tot - 1 : 0;   // past the end: the last key again (cached), masked later
        last = last < room ? last : (int)room;
        last = last < 0 ? 0 : last;
        const int rbase = kRsChunk * (wave + kRsWaves * c) + ld_row;
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            int r = rbase + Cf::kRowsPerLoad * j;
            r = r < last ? r : last;
            pk[slot][j] = __builtin_nontemporal_load(
                (const u32x4*)(sbase + ((uint32_t)r * pool_stride + 16u * (uint32_t)ld_col)));
        }
    };
    // The thread index as a value the compiler must take as new at each use: addresses derived from
    // it are recomputed where they are needed instead of being kept (and spilled) across pass 1.
    auto fresh_tid = [&]() {
        int t = tid;
        asm volatile("" : "+v"(t));
        return t;
    };
    // this thread's 16-byte pieces of the pair's Q rows (zeroed past n_q when they are stored)
    constexpr int kQLoads = (Cf::kRows * Cf::kPieces + kRsThreads - 1) / kRsThreads;
    u32x4 qn[kQLoads];
    auto issue_q = [&](const PairInfo& p) {
        const int t = fresh_tid();
#pragma unroll
        for (int u = 0; u < kQLoads; ++u) {
            const int piece = t + u * kRsThreads;
            const int i = piece / Cf::kPieces, col = piece % Cf::kPieces;
            const int ic = a.row0 + (i < p.n_q ? i : (p.n_q > 0 ? p.n_q - 1 : 0));
            const uint16_t* sbase =
                qb + ((int64_t)p.b * (a.q_stride ? a.q_stride : a.n_q_max) * a.H + p.h) * DH;   // scalar part
            qn[u] = __builtin_nontemporal_load((const u32x4*)(sbase + (uint32_t)(ic * a.H * DH + 8 * col)));
        }
    };
    auto store_q = [&](const PairInfo& p) {
        const int t = fresh_tid();
#pragma unroll
        for (int u = 0; u < kQLoads; ++u) {
            const int piece = t + u * kRsThreads;
            const int i = piece / Cf::kPieces, col = piece % Cf::kPieces;
            if (i < Cf::kRows)
                *(u32x4*)(s_q + i * Cf::kStride + col * 16) = i < p.n_q ? qn[u] : (u32x4){0u, 0u, 0u, 0u};
        }
    };
    auto lds_sync = [&]() {   // orders this wavefront's LDS writes before its later reads (and back)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    int pair = blockIdx.x;   // (numbering the pairs so that an XCD takes whole sequences changes nothing here)
    if (pair >= n_pairs) return;
    PairInfo cur = pair_info(pair);
    issue_chunk(cur, 0, 0, true);
    issue_chunk(cur, 1, 1, true);
    issue_q(cur);
    store_q(cur);
    while (pair < n_pairs) {
        __syncthreads();   // Q rows of this pair are in LDS; every wavefront is done with the previous pair
        const int next = pair + gridDim.x;
        const bool has_next = next < n_pairs;
        const PairInfo nxt = pair_info(has_next ? next : pair);
        issue_q(nxt);
        const int n_q = cur.n_q, n_tot = cur.n_tot, pos0 = cur.pos0;
        const int vis_all = a.causal ? min(pos0 + 1, n_tot) : n_tot;   // keys visible to every row

        // ---- pass 1: logits of the owned chunks, row statistics, table of exponentials ----------
        // A table entry is 2^(logit - ref) in (0, 1], ref = the row's running maximum after the
        // chunk, as 16-bit fixed point.  A stored value is off by at most 2^-17, so a weight (stored
        // value times 2^(ref - max)/sum <= 1/sum) is off by at most 2^-17/sum and a score, a mean of
        // weights, by at most 2^-17 * mean(1/sum) <= 3.8e-6 if every rounding went the same way; with
        // roundings of mixed sign the error is that divided by about sqrt(H * n_q), and for the
        // near-uniform attention of real prompts (sum ~ n_tot) it is below 1e-8.
        float run_m[NB], run_l[NB], ref[kRsCpw][NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            run_m[nb] = -INFINITY;
            run_l[nb] = 0.f;
        }
#pragma unroll
        for (int c = 0; c < kRsCpw; ++c) {
            const int chunk = wave + kRsWaves * c, base = kRsChunk * chunk, slot = c & 1;
            // The refill of the slot runs for every chunk, also one past the end of the sequence (its
            // loads point at the last key; its staging and arithmetic are skipped): no load sits inside
            // a branch.  The 16-row stage takes the chunk in two halves; lane (j, g) of the half that
            // holds key j reads its operand fragments K[key base+j][16dc + 8g .. +7].
            const bool live = base < n_tot;
            u32x4 kf[Cf::kDC];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                if (live) {
#pragma unroll
                    for (int jj = 0; jj < Cf::kHalf; ++jj)
                        *(u32x4*)(stage + (ld_row + Cf::kRowsPerLoad * jj) * Cf::kStride + ld_col * 16) =
                            pk[slot][half * Cf::kHalf + jj];
                }
                if (half == 1) {
                    // the slot's registers are free again: chunk 2 of this pair after chunk 0, then
                    // chunks 1 and 0 of the next pair
                    if (c == 0) issue_chunk(cur, 2, 0, true);
                    else issue_chunk(nxt, c == 1 ? 1 : 0, slot, has_next);
                }
                if (live) {
                    lds_sync();
                    if ((li >> 4) == half) {
#pragma unroll
                        for (int dc = 0; dc < Cf::kDC; ++dc)
                            kf[dc] = *(const u32x4*)(stage + (li & 15) * Cf::kStride + 32 * dc + 16 * g);
                    }
                    lds_sync();   // fragment reads done before the stage is written again
                }
            }
            const bool in_span = base < span_end && base + kRsChunk > a.v_start;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) ref[c][nb] = 0.f;
            if (live) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    // one 32-row block at a time keeps a single accumulator tile live
                    floatx16 s;
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                    for (int dc = 0; dc < Cf::kDC; ++dc) {
                        // B operand: lane (i, g) takes Q[row 32nb+i][16dc + 8g .. +7]
                        const bf16x8 qf =
                            as_bf16x8(*(const u32x4*)(s_q + (32 * nb + li) * Cf::kStride + 32 * dc + 16 * g));
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[dc]), qf, s, 0, 0, 0);
                    }
                    if (base + kRsChunk > vis_all) {
                        const int vis_end = a.causal ? min(pos0 + 32 * nb + li + 1, n_tot) : n_tot;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (base + acc_row(r, g) >= vis_end) s[r] = -INFINITY;
                    }
                    // scale > 0: the maximum of the scaled logits is the scaled maximum
                    float mx = s[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
                    const float m_new = fmaxf(run_m[nb], mx * sl2);
                    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                    float psum = 0.f;
                    if (in_span) {
                        // lane (row, g) holds keys acc_row(r, g); r and r+1 (r even) are neighbouring keys
                        // and share a table entry; the 32 lanes of a group write 32 consecutive words
                        uint32_t* es_row =
                            s_es + ((chunk - first_chunk) * 16 + 2 * g) * Cf::kEsStride + 32 * nb + li;
#pragma unroll
                        for (int r = 0; r < 16; r += 2) {
                            const float e0 = fast_exp2(__builtin_fmaf(s[r], sl2, -m_safe));
                            const float e1 = fast_exp2(__builtin_fmaf(s[r + 1], sl2, -m_safe));
                            psum += e0;
                            psum += e1;
                            es_row[(4 * (r >> 2) + ((r & 3) >> 1)) * Cf::kEsStride] = pack_unorm16(e0, e1);
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) psum += fast_exp2(__builtin_fmaf(s[r], sl2, -m_safe));
                    }
                    ref[c][nb] = m_safe;
                    run_l[nb] = run_l[nb] * fast_exp2(run_m[nb] - m_safe) + psum;
                    run_m[nb] = m_new;
                    // keep the blocks apart: interleaving two of them costs more registers than there are
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // the two lane groups of a row hold different keys of the same chunks: merge, then publish
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float om = __shfl_xor(run_m[nb], 32, 64), ol = __shfl_xor(run_l[nb], 32, 64);
            const float m = fmaxf(run_m[nb], om);
            const float m_safe = m == -INFINITY ? 0.f : m;
            const float l = run_l[nb] * fast_exp2(run_m[nb] - m_safe) + ol * fast_exp2(om - m_safe);
            const int t1 = fresh_tid() & 63;
            if (t1 < 32) {
                s_part[(wave * Cf::kRows + 32 * nb + t1) * 2] = m;
                s_part[(wave * Cf::kRows + 32 * nb + t1) * 2 + 1] = l;
            }
        }
        __syncthreads();   // row statistics of all wavefronts are complete
        store_q(nxt);      // every wavefront is past its last read of the Q rows

        // From here to the end of the pair a wavefront works on its own chunks only.
        // ---- merge: max + log2(sum) over the eight wavefronts for the lane's rows ------------------
        const int ln = fresh_tid() & 63, l5 = ln & 31, gg = ln >> 5;
        float mc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int row = 32 * nb + l5;
            float m = -INFINITY;
#pragma unroll
            for (int w = 0; w < kRsWaves; ++w) m = fmaxf(m, s_part[(w * Cf::kRows + row) * 2]);
            const float m_safe = m == -INFINITY ? 0.f : m;
            float l = 0.f;
#pragma unroll
            for (int w = 0; w < kRsWaves; ++w)
                l += s_part[(w * Cf::kRows + row) * 2 + 1] * fast_exp2(s_part[(w * Cf::kRows + row) * 2] - m_safe);
            // log2(65535) undoes the fixed-point scale; a row past n_q, or one that saw no key, gets
            // +inf and so the factor 2^-inf = 0
            mc[nb] = (row < n_q && l > 0.f) ? m + log2f(l) + 15.99997798f : INFINITY;
        }
        // ---- pass 2: four lanes per key pair, each adds a quarter of the rows in index order ------
        float* partial = a.ws + ((int64_t)cur.b * a.H + cur.h) * a.M;
        const int kpl = ln >> 2, quarter = ln & 3;   // key pair within the chunk, quarter of the rows
        constexpr int kRQ = Cf::kRows / 4;
#pragma unroll
        for (int c = 0; c < kRsCpw; ++c) {
            const int chunk = wave + kRsWaves * c, base = kRsChunk * chunk;
            if (base < span_end && base + kRsChunk > a.v_start) {
                float sum0 = 0.f, sum1 = 0.f;
                if (base < n_tot) {
                    // factor of every (lane group, row) of this chunk: 2^(reference - mc)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        w_tab[gg * Cf::kWStride + 32 * nb + l5] = fast_exp2(ref[c][nb] - mc[nb]);
                    lds_sync();
                    const uint32_t* es = s_es + ((chunk - first_chunk) * 16 + kpl) * Cf::kEsStride + kRQ * quarter;
                    // the lane group that wrote the pair: key pairs 2g, 2g+1 of every four
                    const float* w = w_tab + ((kpl >> 1) & 1) * Cf::kWStride + kRQ * quarter;
#pragma unroll
                    for (int q = 0; q < kRQ / 4; ++q) {
                        const u32x4 v = *(const u32x4*)(es + 4 * q);
                        const float4 f = *(const float4*)(w + 4 * q);
                        sum0 += (float)(v.x & 0xFFFFu) * f.x;
                        sum1 += (float)(v.x >> 16) * f.x;
                        sum0 += (float)(v.y & 0xFFFFu) * f.y;
                        sum1 += (float)(v.y >> 16) * f.y;
                        sum0 += (float)(v.z & 0xFFFFu) * f.z;
                        sum1 += (float)(v.z >> 16) * f.z;
                        sum0 += (float)(v.w & 0xFFFFu) * f.w;
                        sum1 += (float)(v.w >> 16) * f.w;
                    }
                    lds_sync();   // reads of the factors done before the next chunk overwrites them
                    // (q0 + q1) + (q2 + q3), the same in all four lanes
                    sum0 += quad_swap<0xB1>(sum0);
                    sum1 += quad_swap<0xB1>(sum1);
                    sum0 += quad_swap<0x4E>(sum0);
                    sum1 += quad_swap<0x4E>(sum1);
                }
                // lane 0 of the four writes the even key, lane 1 the odd one
                const int j = base + 2 * kpl + quarter;
                if (quarter < 2 && j >= a.v_start && j < span_end)
                    partial[j - a.v_start] = j < n_tot ? (quarter == 0 ? sum0 : sum1) : 0.f;
            }
        }
        pair = next;
        cur = nxt;
    }
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

template <int DH, int NB>
static hipError_t launch_rs(const ScoreArgs& a, hipStream_t s) {
    const int n_pairs = a.B * a.H;
    using Cf = RsCfg<DH, NB>;
    const int span_chunks = (a.v_start + a.M - 1) / kRsChunk - a.v_start / kRsChunk + 1;
    const size_t lds = Cf::kOffEs + (size_t)span_chunks * Cf::kEsChunk;
    // the table grows with the visual span: raise the limit to a compute unit's LDS once per kernel and device
    static uint32_t raised = 0u;
    const hipError_t e = raise_lds_limit_once((const void*)score_resident_kernel<DH, NB>, kRsLdsBytes, raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((score_resident_kernel<DH, NB>), dim3(resident_grid(n_pairs)), dim3(kRsThreads), lds, s, a,
                       n_pairs);
    return hipGetLastError();
}

// up to 64 scoring rows x 768 keys per (sequence, head), and a table of exponentials (one 32-key
// chunk of it per chunk that the visual span touches) that fits beside the other LDS buffers
bool score_resident_supported(const ScoreArgs& a, int dtype) {
    if (a.M <= 0) return false;
    const int span_chunks = (a.v_start + a.M - 1) / kRsChunk - a.v_start / kRsChunk + 1;
    const int max_chunks = a.n_q_max <= 32 ? (a.d_h == 128 ? RsCfg<128, 1>::kMaxSpanChunks : RsCfg<64, 1>::kMaxSpanChunks)
                                           : (a.d_h == 128 ? RsCfg<128, 2>::kMaxSpanChunks : RsCfg<64, 2>::kMaxSpanChunks);
    return dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.n_q_max <= 64 && a.n_tot_max <= kRsMaxKeys &&
           a.k.pool_rows <= 0x7FFFFFFFll && a.scale > 0.f && span_chunks <= max_chunks;
}

hipError_t launch_score_resident(const ScoreArgs& a, hipStream_t s) {
    if (a.n_q_max <= 32) return a.d_h == 128 ? launch_rs<128, 1>(a, s) : launch_rs<64, 1>(a, s);
    return a.d_h == 128 ? launch_rs<128, 2>(a, s) : launch_rs<64, 2>(a, s);
}

}  // namespace tw
