// Pruning score (Sec. 3.1 Eq. 2-3, head mean as in Sec. 5.1 Eq. 7), fast path
// for prompts whose attention rows fit in registers: bf16, d_h 64/128, at most
// 64 scoring rows, at most 768 keys.
//
// One 8-wavefront workgroup per compute unit loops over (sequence, head) pairs.
// Wavefront w owns key chunks w, w+8, w+16 of the pair (32 keys each).
//   pass 1  K chunk: coalesced loads -> registers (two chunks always in flight
//           per wavefront, across pair boundaries) -> a 32-row LDS stage ->
//           matrix-core operand registers.  K.Q^T with Q read from LDS; the
//           logits of the wavefront's three chunks stay in its registers as fp32
//           accumulator tiles (lane = scoring row, registers = keys).  Row maximum
//           over the wavefront's keys, exponentials in place, row sum.
//   merge   the eight wavefronts publish (max, sum) per row; one workgroup barrier
//           (the only one of the pair: the Q rows and the statistics area are
//           double-buffered); every lane turns the statistics into the factor
//           2^(own max - row max) / row sum of its rows.
//   pass 2  each wavefront, for its own chunks of the visual span: weights =
//           exponentials * factor, summed over the scoring rows -- over the row
//           blocks inside the lane, over the 32 lanes by a reduce-scatter of
//           lane exchanges (no shared memory) -> partial[b][h][m].
// K is read from HBM exactly once, nothing of size rows x keys leaves the
// registers, and every weight is fp32 from the logit to the column sum.
// Per-pair table reads are scalar loads, no load sits inside a branch and the
// kernel has no scratch spills: any of these would make a wavefront wait for
// every K load in flight instead of the one it needs.  The loop count of every
// workgroup is fixed by the grid; there are no waits on other workgroups.
#include "mfma_util.h"
#include "twig_internal.h"

namespace tw {

// Diagnostic build: lane 0 of every wavefront records the 100 MHz wall clock at eight points of each of
// its first 16 pairs: [workgroup][wavefront][pair][mark].
#ifdef TW_TRACE
#define RS_MARK(slot)                                                                                  \
    do {                                                                                               \
        asm volatile("" ::: "memory");                                                                 \
        const unsigned long long t_ = __builtin_amdgcn_s_memrealtime();                                \
        if (a.trace && lane == 0 && iter < 16)                                                         \
            a.trace[(((size_t)blockIdx.x * kRsWaves + wave) * 16 + iter) * 8 + (slot)] = t_;           \
        asm volatile("" ::: "memory");                                                                 \
    } while (0)
#define RS_DRY(level) (a.dry >= (level))
#else
#define RS_MARK(slot)
#define RS_DRY(level) false
#endif

constexpr int kRsWaves = 8;
constexpr int kRsThreads = kRsWaves * 64;
constexpr int kRsChunk = 32;
constexpr int kRsCpw = 3;                                  // chunks per wavefront
constexpr int kRsMaxKeys = kRsWaves * kRsCpw * kRsChunk;   // 768

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// keep + (the partner lane's send) for one step of the reduce-scatter inside a row of 16 lanes
template <int CTRL>
__device__ __forceinline__ float rs_step(bool upper, float a, float b) {
    const float keep = upper ? b : a, send = upper ? a : b;
    return keep + dpp_move<CTRL>(send);
}

// Sums over the 32 lanes of each half of the wavefront, for 16 registers at once: on return the
// lane with index li inside its half holds the total of v[li >> 1] (both lanes of a pair hold it).
// Every step halves the registers: a lane keeps one half of them and receives its partner's
// contribution to that half -- across the two 16-lane rows with v_permlane16_swap, inside a row
// with the mirror and quad permutations of the DPP modifier.  31 additions per lane, in an order
// fixed by the lane index.
__device__ __forceinline__ float reduce_scatter_32x16(const floatx16& v, int li) {
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
    float u[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        // afterwards .x holds (v[r] of row 0, v[r + 8] of row 0) in the rows 0 and 1 of each half and .y the
        // same of row 1: their sum is v[r] over both rows in row 0 and v[r + 8] over both rows in row 1
        // (elements copied out first: a bit cast applied to a vector element reads element 0)
        const float lo = v[r], hi = v[r + 8];
        const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
        u[r] = __uint_as_float(sw.x) + __uint_as_float(sw.y);
    }
    const bool b3 = (li & 8) != 0, b2 = (li & 4) != 0, b1 = (li & 2) != 0;
    float w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = rs_step<0x140>(b3, u[j], u[j + 4]);   // row_mirror: lane l <-> 15 - l
    const float x0 = rs_step<0x141>(b2, w[0], w[2]), x1 = rs_step<0x141>(b2, w[1], w[3]);   // row_half_mirror
    const float y = rs_step<0x4E>(b1, x0, x1);                                             // lanes l <-> l ^ 2
    return y + dpp_move<0xB1>(y);                                                          // lanes l <-> l ^ 1
}

template <int DH, int NB>
struct RsCfg {
    static constexpr int kRowB = DH * 2;
    static constexpr int kDC = DH / 16;
    static constexpr int kRows = 32 * NB;             // scoring rows held
    static constexpr int kStride = kRowB + 16;        // bytes per K or Q row in LDS (padded)
    static constexpr int kPieces = kRowB / 16;        // 16-byte pieces per row = lanes per row of a load
    static constexpr int kRowsPerLoad = 64 / kPieces;
    static constexpr int kLoads = kRsChunk / kRowsPerLoad;   // loads per chunk (per lane)
    // LDS layout (bytes)
    static constexpr int kQBytes = kRows * kStride;
    static constexpr int kOffQ = 0;
    static constexpr int kOffStage = kOffQ + 2 * kQBytes;
    static constexpr int kWaveStage = kRsChunk * kStride;     // one whole chunk per wavefront
    static constexpr int kOffPart = kOffStage + kRsWaves * kWaveStage;
    static constexpr int kPartBytes = kRsWaves * kRows * 2 * 4;
    static constexpr int kLds = kOffPart + 2 * kPartBytes;
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
    unsigned char* stage = lds + Cf::kOffStage + wave * Cf::kWaveStage;   // one K chunk of this wavefront

    const uint32_t pool_stride = (uint32_t)(a.k.H * Cf::kRowB);   // a cache row holds the key heads
    const int64_t last_pool_row = a.k.pool_rows - 1;
    const float sl2 = a.scale * kLog2e;
    const int span_end = a.v_start + a.M;
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
        // rows of the sequence that fall into this launch's window (none: every row gets the factor
        // zero and the pair's partial sums come out as zeros)
        const int q_rows = a.q_stride ? a.q_stride : a.n_q_max;
        const ScoreSeq sq = score_seq_from(a.n_q ? ((ctab)a.n_q)[p.b] : q_rows, ((ctab)a.n_tot)[p.b],
                                           ((ctab)a.q_pos0)[p.b], q_rows, a.row0, a.n_q_max, a.n_tot_max);
        p.n_q = sq.n_q;
        p.n_tot = sq.n_tot;
        p.pos0 = sq.pos0;
        p.row0 = seq_first_row(((ctab)a.k.row_off)[p.b], a.k.pool_rows);
        return p;
    };
    // Two prefetch slots: chunks 0 and 2 of a pair use slot 0, chunk 1 uses slot 1.  A load moves 16
    // bytes per lane, kPieces lanes per key row.  Every call issues the same number of loads on every
    // path; `live` false (no further pair) points all lanes at one row instead of skipping them.
    u32x4 pk[2][Cf::kLoads];
    auto issue_chunk = [&](const PairInfo& p, int c, int slot, bool live) {
        // scalar part of the address: the sequence's first row (inside the pool) and the head
        const unsigned char* sbase =
            (const unsigned char*)a.k.base + (uint64_t)p.row0 * pool_stride + (int64_t)(p.h / a.group) * Cf::kRowB;
        // lane part, 32 bits: its key row, held below the sequence's end and the pool's end
        const int64_t room = last_pool_row - p.row0;
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
    auto store_q = [&](const PairInfo& p, int buf) {
        unsigned char* s_q = lds + Cf::kOffQ + buf * Cf::kQBytes;
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
    store_q(cur, 0);
    __syncthreads();
    int par = 0;
#ifdef TW_TRACE
    int iter = 0;
#endif
    while (pair < n_pairs) {
        RS_MARK(0);   // top of the pair
        const unsigned char* s_q = lds + Cf::kOffQ + par * Cf::kQBytes;
        float* s_part = (float*)(lds + Cf::kOffPart + par * Cf::kPartBytes);
        const int next = pair + gridDim.x;
        const bool has_next = next < n_pairs;
        const PairInfo nxt = pair_info(has_next ? next : pair);
        if (!RS_DRY(4)) issue_q(nxt);
        const int n_q = cur.n_q, n_tot = cur.n_tot, pos0 = cur.pos0;
        const int vis_all = a.causal ? min(pos0 + 1, n_tot) : n_tot;   // keys visible to every row

        // ---- pass 1: logits of the owned chunks into registers, row maxima ---------------------------
        // st[c][nb]: lane (row 32nb + li, g) holds the 16 keys base + acc_row(r, g) of chunk c
        floatx16 st[kRsCpw][NB];
        float row_m[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) row_m[nb] = -INFINITY;
#pragma unroll
        for (int c = 0; c < kRsCpw; ++c) {
            const int chunk = wave + kRsWaves * c, base = kRsChunk * chunk, slot = c & 1;
            // The refill of the slot runs for every chunk, also one past the end of the sequence (its
            // loads point at the last key; its staging and arithmetic are skipped): no load sits inside
            // a branch.
            const bool live = base < n_tot;
            if (live) {
#pragma unroll
                for (int j = 0; j < Cf::kLoads; ++j)
                    *(u32x4*)(stage + (ld_row + Cf::kRowsPerLoad * j) * Cf::kStride + ld_col * 16) = pk[slot][j];
            }
            // the slot's registers are free again: chunk 2 of this pair after chunk 0, then chunks 1
            // and 0 of the next pair
            if (c == 0) RS_MARK(1);        // chunk 0 has arrived and is staged
            else if (c == 1) RS_MARK(3);   // chunk 1
            else RS_MARK(4);               // chunk 2
            if (c == 0) issue_chunk(cur, 2, 0, true);
            else issue_chunk(nxt, c == 1 ? 1 : 0, slot, has_next);
            if (live && !RS_DRY(1)) {
                lds_sync();
                // A operand: lane (j, g) takes K[key base + j][16dc + 8g .. +7]
                u32x4 kf[Cf::kDC];
#pragma unroll
                for (int dc = 0; dc < Cf::kDC; ++dc)
                    kf[dc] = *(const u32x4*)(stage + li * Cf::kStride + 32 * dc + 16 * g);
                lds_sync();   // fragment reads done before the stage is written again
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
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
                    float mx = s[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
                    row_m[nb] = fmaxf(row_m[nb], mx);
                    st[c][nb] = s;
                }
                if (c == 0) RS_MARK(2);   // logits of chunk 0 done
            } else {
                // no key: the weights are zero as they stand (the exponentials below skip the chunk)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st[c][nb][r] = 0.f;
            }
        }
        // ---- exponentials in place, relative to the wavefront's own row maximum; publish (max, sum) ----
        // scale > 0: the maximum of the scaled logits is the scaled maximum.  Base-2 units throughout.
        float own_m[NB], m_safe[NB], row_l[NB];
        RS_MARK(5);   // pass 1 done
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            own_m[nb] = fmaxf(row_m[nb], __shfl_xor(row_m[nb], 32, 64)) * sl2;
            m_safe[nb] = own_m[nb] == -INFINITY ? 0.f : own_m[nb];
            row_l[nb] = 0.f;
        }
#pragma unroll
        for (int c = 0; c < kRsCpw; ++c) {
            // a wavefront whose last chunk lies past the end of the sequence saves a third of the work
            if (kRsChunk * (wave + kRsWaves * c) < n_tot && !RS_DRY(2)) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = fast_exp2(__builtin_fmaf(st[c][nb][r], sl2, -m_safe[nb]));
                        st[c][nb][r] = e;
                        row_l[nb] += e;
                    }
            }
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float m = own_m[nb];
            const float l = row_l[nb] + __shfl_xor(row_l[nb], 32, 64);
            const int t1 = fresh_tid() & 63;
            if (t1 < 32) {
                s_part[(wave * Cf::kRows + 32 * nb + t1) * 2] = m;
                s_part[(wave * Cf::kRows + 32 * nb + t1) * 2 + 1] = l;
            }
        }
        if (!RS_DRY(4)) store_q(nxt, par ^ 1);
        RS_MARK(6);   // exponentials done, statistics published
        __syncthreads();
        RS_MARK(7);   // through the barrier   // row statistics of all wavefronts are complete; next pair's Q rows in place

        // From here to the end of the pair a wavefront works on its own registers only.
        // ---- merge: factor 2^(own max - row max) / row sum for the lane's rows ----------------------
        const int ln = fresh_tid() & 63, l5 = ln & 31, gg = ln >> 5;
        float fac[NB];
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
            // a row past n_q, or one that saw no key at all, weighs nothing; a wavefront whose keys were
            // all hidden from the row holds zeros and its own maximum -inf
            fac[nb] = (row < n_q && l > 0.f && own_m[nb] != -INFINITY) ? fast_exp2(own_m[nb] - m_safe) / l : 0.f;
        }
        // ---- pass 2: column sums of the weights over the scoring rows -------------------------------
        float* partial = a.ws + ((int64_t)cur.b * a.H + cur.h) * a.M;
#pragma unroll
        for (int c = 0; c < kRsCpw; ++c) {
            const int chunk = wave + kRsWaves * c, base = kRsChunk * chunk;
            if (base < span_end && base + kRsChunk > a.v_start && !RS_DRY(3)) {
                floatx16 col;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = st[c][0][r] * fac[0];
#pragma unroll
                    for (int nb = 1; nb < NB; ++nb) v = __builtin_fmaf(st[c][nb][r], fac[nb], v);
                    col[r] = v;
                }
                const float total = reduce_scatter_32x16(col, l5);
                // the lane pair (2r, 2r + 1) of half g holds key base + acc_row(r, g); keys past the end of
                // the sequence were never visible and come out as zeros
                const int j = base + acc_row(l5 >> 1, gg);
                if ((l5 & 1) == 0 && j >= a.v_start && j < span_end) partial[j - a.v_start] = total;
            }
        }
        pair = next;
        cur = nxt;
        par ^= 1;
#ifdef TW_TRACE
        ++iter;
#endif
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
    // more than the default 64 KB of LDS: raise the limit once per kernel and device
    static std::atomic<uint32_t> raised{0u};
    const hipError_t e = raise_lds_limit_once((const void*)score_resident_kernel<DH, NB>, Cf::kLds, raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((score_resident_kernel<DH, NB>), dim3(resident_grid(n_pairs)), dim3(kRsThreads), Cf::kLds, s, a,
                       n_pairs);
    return hipGetLastError();
}

// up to 64 scoring rows x 768 keys per (sequence, head): what eight wavefronts hold in registers
bool score_resident_supported(const ScoreArgs& a, int dtype) {
    return a.M > 0 && dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.n_q_max <= 64 &&
           a.n_tot_max <= kRsMaxKeys && a.k.pool_rows <= 0x7FFFFFFFll && a.scale > 0.f;
}

hipError_t launch_score_resident(const ScoreArgs& a, hipStream_t s) {
    if (a.n_q_max <= 32) return a.d_h == 128 ? launch_rs<128, 1>(a, s) : launch_rs<64, 1>(a, s);
    return a.d_h == 128 ? launch_rs<128, 2>(a, s) : launch_rs<64, 2>(a, s);
}

}  // namespace tw
