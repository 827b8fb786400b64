// Tree verification attention on the CDNA4 matrix cores (bf16 caches, d_h 64 or
// 128): the verification step of Alg. 2 -- Sec. 3.1 Eq. 2 under the
// topology-aware mask of Sec. 5.4 / App. A.  Every K/V byte of a (sequence,
// head) is fetched from HBM once and shared by all tree rows.
//
// Decomposition
//   A wavefront owns one work unit = (head, block of 32 tree nodes, row phase).
//   The four wavefronts of a workgroup split as  heads_per_wg x n_blk x n_phase = 4:
//     T <= 32, many units   4 heads x 1 block x 1 phase       verify_mfma_kernel
//     T <= 32, few units    1 head  x 1 block x 4 phases      verify_mfma_kernel
//     T <= 64, many units   2 heads x 2 blocks x 1 phase      verify_mfma_pair_kernel
//     T <= 64, few units    1 head  x 2 blocks x 2 phases     verify_mfma_pair_kernel
//   Phases take the 32-row chunks of a head round-robin and merge through LDS at the end.
//   In the pair kernel the two node blocks of a head need the same K/V rows: one wavefront
//   loads the K chunk, its partner the V chunk, into a stage they share (double-buffered,
//   one workgroup barrier per chunk, loads two chunks ahead).
//   grid (ceil(H / heads_per_wg), B, n_splits); n_splits > 1 additionally cuts the cache rows
//   into pieces of split_rows rows, one workgroup each (a workgroup past the end of its
//   sequence leaves at once).  A sequence in one piece is finished by its workgroup; otherwise
//   partial (max, sum, O) go to the workspace and the workgroup that arrives last at the
//   unit's counter merges them in split order (finish_split_unit).
//
// Per 32-row chunk a wavefront
//     1. stores prefetched K/V rows (16-byte lanes, fully coalesced 256-byte row segments)
//        into the LDS stage and issues the loads of a later chunk,
//     2. S^T[row][node] = K . Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows read
//        back from LDS as 16-byte fragments, B = Q fragments kept in registers),
//     3. online softmax per node: the 32x32 accumulator layout gives every lane
//        16 rows of one node, so the row maximum needs one cross-lane exchange,
//     4. O^T[col][node] += V^T . P^T with the same instruction: the accumulator
//        layout of step 2 is exactly a B-operand layout once the reduction index
//        is permuted, so P never leaves registers; V^T fragments are gathered
//        from LDS (one 8-byte read per row, regrouped with byte permutes).
//   Exponentials run in base 2 with scale*log2(e) folded into the logits.
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
    static constexpr int kStage = kChunk * (kKStride + kVStride);   // one K+V chunk
    static constexpr int kOStride = DH + 4;         // floats per node row in the merge buffer
    static constexpr int kMergeLds = 4 * 32 * kOStride * 4 + 4 * 32 * 2 * 4;   // O tiles + (max, sum)
    static constexpr int kLds = 4 * kStage > kMergeLds ? 4 * kStage : kMergeLds;
};

// Per-wavefront attention state of one (head, node block).
template <int DH>
struct WaveState {
    bf16x8 qf[MfCfg<DH>::kDC];      // Q fragments (B operand): lane (i, g) holds Q[node][16c + 8g .. +7]
    floatx16 o[MfCfg<DH>::kNQ];     // O^T accumulators, column block q holds columns kNQ*i + q
    float run_m, run_l;             // running maximum (base-2 units) and this lane's share of the row sum
    uint64_t anc;                   // ancestor-or-self mask of the lane's node
};

// Q fragments of tree node t: the loads depend on nothing but the unit, so they are issued at the very top
// of the kernel (node clamped into the T_max rows the tensor holds); padding nodes are zeroed afterwards.
template <int DH>
__device__ __forceinline__ void issue_q(u32x4 (&raw)[MfCfg<DH>::kDC], const VerifyArgs& a, int b, int h, int t, int g) {
    const int tc = t < a.T_max ? t : a.T_max - 1;
    const u32x4* src = (const u32x4*)((const uint16_t*)a.q + (((int64_t)b * a.T_max + tc) * a.H + h) * DH + 8 * g);
#pragma unroll
    for (int c = 0; c < MfCfg<DH>::kDC; ++c) raw[c] = src[2 * c];
}
template <int DH>
__device__ __forceinline__ void init_state(WaveState<DH>& w, const u32x4 (&raw)[MfCfg<DH>::kDC], int t, int T) {
    using Cf = MfCfg<DH>;
#pragma unroll
    for (int c = 0; c < Cf::kDC; ++c) w.qf[c] = as_bf16x8(t < T ? raw[c] : (u32x4){0u, 0u, 0u, 0u});
#pragma unroll
    for (int q = 0; q < Cf::kNQ; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) w.o[q][r] = 0.f;
    w.run_m = -INFINITY;
    w.run_l = 0.f;
}

// Ancestor-or-self masks of a tree of up to 64 nodes inside one wavefront, lane = node, no shared
// memory and no barrier: pointer doubling, six rounds of (mask |= mask of the jump target; jump
// target = its jump target) cover every depth below 64.  `par_raw` is the lane's parent entry as
// read; lanes past T return 0.
__device__ __forceinline__ uint64_t wave_ancestor_mask(int par_raw, int node, int T) {
    int j = node > 0 ? clamp_parent(par_raw, node) : 0;
    uint32_t lo = node < 32 ? 1u << node : 0u, hi = node >= 32 ? 1u << (node - 32) : 0u;
#pragma unroll
    for (int round = 0; round < 6; ++round) {
        const uint32_t jl = __shfl(lo, j, 64), jh = __shfl(hi, j, 64);
        const int jj = __shfl(j, j, 64);
        lo |= jl;
        hi |= jh;
        j = jj;
    }
    return node < T ? ((uint64_t)hi << 32) | lo : 0ull;
}

// Steps 2-4 for the chunk staged at (ldsK, ldsV) whose first cache row is `base`.
template <int DH>
__device__ __forceinline__ void process_chunk(WaveState<DH>& w, const unsigned char* ldsK,
                                              const unsigned char* ldsV, int base, int C, int n_rows,
                                              float sl2, int g, int li) {
    using Cf = MfCfg<DH>;
    floatx16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int c = 0; c < Cf::kDC; ++c) {
        const bf16x8 kf = as_bf16x8(*(const u32x4*)(ldsK + li * Cf::kKStride + 32 * c + 16 * g));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, w.qf[c], s, 0, 0, 0);
    }
    if (base + kChunk > C) {   // only chunks that touch tree rows test the ancestor masks
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = base + acc_row(r, g);
            const bool vis = row < C || (row < n_rows && ((w.anc >> (row - C)) & 1ull));
            s[r] = vis ? s[r] : -INFINITY;
        }
    }
    // scale > 0: the maximum of the scaled logits is the scaled maximum of the raw ones
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sl2;
    const float m_new = fmaxf(w.run_m, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(w.run_m - m_safe);   // 0 on the first visible chunk, 1 when the maximum holds
    float psum = 0.f;
    uint32_t pw[8];
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
        // the row sum is taken over the bf16-rounded weights that enter the PV product (a two-term
        // dot product with ones adds a rounded pair), so the normalised weights still sum to one
        const bf16x2 p2 = {(__bf16)fast_exp2(__builtin_fmaf(s[r], sl2, -m_safe)),
                           (__bf16)fast_exp2(__builtin_fmaf(s[r + 1], sl2, -m_safe))};
        psum = __builtin_amdgcn_fdot2_f32_bf16(p2, ones, psum, false);
        pw[r >> 1] = __builtin_bit_cast(uint32_t, p2);
    }
    const bf16x8 pf[2] = {as_bf16x8((u32x4){pw[0], pw[1], pw[2], pw[3]}),
                          as_bf16x8((u32x4){pw[4], pw[5], pw[6], pw[7]})};
    w.run_l = w.run_l * alpha + psum;
    w.run_m = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
        for (int q = 0; q < Cf::kNQ; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.o[q][r] *= alpha;
    }
    // reduction slot (g, e) of half c2 is chunk row acc_row(8*c2 + e, g)
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2) {
        uint32_t v[8][Cf::kNQ / 2];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned char* p = ldsV + acc_row(8 * c2 + e, g) * Cf::kVStride + li * (Cf::kNQ * 2);
            if (Cf::kNQ == 4) {
                const uint2 t2 = *(const uint2*)p;
                v[e][0] = t2.x;
                v[e][Cf::kNQ / 2 - 1] = t2.y;
            } else {
                v[e][0] = *(const uint32_t*)p;
            }
        }
#pragma unroll
        for (int q = 0; q < Cf::kNQ; ++q) {
            u32x4 av;
            const uint32_t sel = (q & 1) ? 0x07060302u : 0x05040100u;
            av.x = __builtin_amdgcn_perm(v[1][q >> 1], v[0][q >> 1], sel);
            av.y = __builtin_amdgcn_perm(v[3][q >> 1], v[2][q >> 1], sel);
            av.z = __builtin_amdgcn_perm(v[5][q >> 1], v[4][q >> 1], sel);
            av.w = __builtin_amdgcn_perm(v[7][q >> 1], v[6][q >> 1], sel);
            w.o[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), pf[c2], w.o[q], 0, 0, 0);
        }
    }
}

// One unit per wavefront (n_phase == 1, never split): normalise and store.
// The accumulators hold, per lane, 16 scattered 16-byte pieces of one node's output row; stored
// from there every store instruction would touch 64 different 128-byte lines (measured: 25 us for
// the 55 MB of the bench launch).  The tile goes through `tile` (32 x kOStride floats of LDS that
// this wavefront owns and no longer reads) so that a store instruction writes whole rows.
template <int DH>
__device__ __forceinline__ void epilogue_direct(const WaveState<DH>& w, const VerifyArgs& a, float* tile, int b,
                                                int h, int T, int lane, int node0 = 0) {
    // T = nodes of this wavefront's block (may be <= 0), node0 = tree index of its first node
    static_assert(32 * MfCfg<DH>::kOStride * 4 <= MfCfg<DH>::kStage, "the tile fits one K+V stage");
    using Cf = MfCfg<DH>;
    const int g = lane >> 5, li = lane & 31;
    const float l = w.run_l + __shfl_xor(w.run_l, 32, 64);
    const float mul = 1.f / l;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // earlier reads of this LDS area are done
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        float* p = tile + li * Cf::kOStride + Cf::kNQ * acc_row(r, g);
        if (Cf::kNQ == 4)
            *(float4*)p = make_float4(w.o[0][r] * mul, w.o[1][r] * mul, w.o[Cf::kNQ - 2][r] * mul,
                                      w.o[Cf::kNQ - 1][r] * mul);
        else
            *(float2*)p = make_float2(w.o[0][r] * mul, w.o[1][r] * mul);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lanes_per_row consecutive lanes store one node's row as consecutive 16-byte pieces
    constexpr int kLanesPerRow = DH / 4, kRowsPerStore = 64 / kLanesPerRow;
    const int sub = lane / kLanesPerRow, c4 = lane % kLanesPerRow;
    // Written once at the end of the wavefront's life: system-scope stores through a descriptor
    // over the block's 32 rows of `out` (2 % faster than streaming stores on the bench launch).
    const int64_t first = (((int64_t)b * a.T_max + node0) * a.H + h) * DH;   // node 0 of the block
    const uint32_t node_stride = (uint32_t)a.H * DH;
    if (a.out_bf16) {
        typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
        const __amdgpu_buffer_rsrc_t ro = raw_buffer((const uint16_t*)a.out + first, 32u * node_stride * 2u);
#pragma unroll
        for (int n0 = 0; n0 < 32; n0 += kRowsPerStore) {
            const int node = n0 + sub;
            if (node < T) {
                const f32x4 v = *(const f32x4*)(tile + node * Cf::kOStride + 4 * c4);
                const u32x2 p = {pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
                __builtin_amdgcn_raw_buffer_store_b64(p, ro, (int)((node * node_stride + 4 * c4) * 2u), 0, kAuxThrough);
            }
        }
    } else {
        const __amdgpu_buffer_rsrc_t ro = raw_buffer((const float*)a.out + first, 32u * node_stride * 4u);
#pragma unroll
        for (int n0 = 0; n0 < 32; n0 += kRowsPerStore) {
            const int node = n0 + sub;
            if (node < T) {
                const f32x4 v = *(const f32x4*)(tile + node * Cf::kOStride + 4 * c4);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), ro,
                                                       (int)((node * node_stride + 4 * c4) * 4u), 0, kAuxThrough);
            }
        }
    }
}

// Row phases of one head merge through LDS.  Merge slot of a wavefront = blk * n_phase + phase.
// Must be entered by the whole workgroup after its last use of the stages.
template <int DH>
__device__ __forceinline__ void epilogue_merge(const WaveState<DH>& w, const VerifyArgs& a, unsigned char* lds,
                                               int b, int h, int T, int split, int n_b, int slot_w, int n_blk,
                                               int n_phase, int g, int li, int tid) {
    using Cf = MfCfg<DH>;
    __syncthreads();
    float* mo = (float*)lds;                      // [4 slots][32 nodes][kOStride]
    float* mstat = mo + 4 * 32 * Cf::kOStride;    // [4 slots][32 nodes][2]
    const float l_wave = w.run_l + __shfl_xor(w.run_l, 32, 64);
    float* mine = mo + (slot_w * 32 + li) * Cf::kOStride;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        float* p = mine + Cf::kNQ * acc_row(r, g);
        if (Cf::kNQ == 4)
            *(float4*)p = make_float4(w.o[0][r], w.o[1][r], w.o[Cf::kNQ - 2][r], w.o[Cf::kNQ - 1][r]);
        else
            *(float2*)p = make_float2(w.o[0][r], w.o[1][r]);
    }
    if (g == 0) {
        mstat[(slot_w * 32 + li) * 2] = w.run_m;
        mstat[(slot_w * 32 + li) * 2 + 1] = l_wave;
    }
    __syncthreads();
    // thread -> (node, 4 output columns); phases are added in index order
    constexpr int kPerRow = DH / 4;
    for (int idx = tid; idx < n_blk * 32 * kPerRow; idx += kMfThreads) {
        const int node = idx / kPerRow, d4 = idx % kPerRow;
        const int nblk = node >> 5, nl = node & 31;
        if (node >= T) continue;
        float m = -INFINITY;
        for (int p = 0; p < n_phase; ++p) m = fmaxf(m, mstat[((nblk * n_phase + p) * 32 + nl) * 2]);
        const float m_safe = m == -INFINITY ? 0.f : m;
        float l = 0.f;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int p = 0; p < n_phase; ++p) {
            const int s = nblk * n_phase + p;
            const float sc = fast_exp2(mstat[(s * 32 + nl) * 2] - m_safe);
            l += mstat[(s * 32 + nl) * 2 + 1] * sc;
            const float4 v = *(const float4*)(mo + (s * 32 + nl) * Cf::kOStride + 4 * d4);
            acc.x += v.x * sc;
            acc.y += v.y * sc;
            acc.z += v.z * sc;
            acc.w += v.w * sc;
        }
        if (n_b == 1) {
            const float inv = 1.f / l;
            store_out4(a.out, a.out_bf16, (((int64_t)b * a.T_max + node) * a.H + h) * DH + 4 * d4, acc.x * inv,
                       acc.y * inv, acc.z * inv, acc.w * inv, false);
        } else {
            const int64_t slot = ((int64_t)split * a.B + b) * a.H + h;   // this piece's slot
            store_partial4(a.part_o + slot * a.o_stride, (uint32_t)(a.T_max * DH * 4), (uint32_t)((node * DH + 4 * d4) * 4),
                           acc);
            if (d4 == 0)
                store_partial2(a.part_ml + slot * a.ml_stride, (uint32_t)(a.T_max * 8), (uint32_t)(node * 8),
                               make_float2(m * kLn2, l));
        }
    }
    if (n_b > 1) finish_split_unit(a, b, h, T, n_b, tid, kMfThreads);
}

// Tree, context length and this split's rows of a sequence, common to both kernels.
__device__ __forceinline__ SeqInfo seq_info(const VerifyArgs& a, int b, int split) {
    return seq_info_from(a.n_nodes[b], a.ctx_len[b], a.T_max, a.max_rows, a.split_rows, a.n_splits, split);
}

// (head group, sequence) of a workgroup.  The hardware hands consecutive workgroups to the eight
// XCDs (each with its own L2) round-robin; taken in grid order, XCD x would get head group x of
// every sequence, i.e. one eighth of every cache row.  Renumbered, an XCD gets whole sequences: its
// workgroups read complete 8 KB rows at about the same time (1.5 % faster on the bench launch, A/B on
// one machine; the opposite order, sequences fastest, is 4 % slower).  Grids that are not a multiple of 8 keep
// grid order, and so does the one-head-per-workgroup layout of small launches: there a batch of unequal
// sequences must not hand whole (long or short) sequences to single XCDs, and in grid order every XCD gets
// an eighth of the heads of every sequence (ragged batch of 16, measured: the XCDs ended between 21 and
// 38 us with whole sequences each).
__device__ __forceinline__ void unit_of_block(const VerifyArgs& a, int& hg, int& b) {
    const int total = gridDim.x * gridDim.y, id = blockIdx.x + gridDim.x * blockIdx.y;
    hg = blockIdx.x;
    b = blockIdx.y;
    if ((total & 7) == 0 && a.heads_per_wg > 1) {
        const int u = (id & 7) * (total >> 3) + (id >> 3);
        hg = u % gridDim.x;
        b = u / gridDim.x;
    }
}

// Addresses of the K/V rows of one (sequence, head).  A load takes cache row base + r of a chunk,
// 16-byte column `col` of the head's segment; rows past `last_row` read that row again.
//   contiguous: everything up to the chunk is scalar (sequence start and chunk start, both kept
//               inside the pool); a lane adds a 32-bit offset of at most 32 rows.
//   paged:      the pool row comes from the page table, per lane, in 64 bits.
struct ChunkAddr {
    const unsigned char* base;   // contiguous: first row of the chunk; paged: row 0 of the pool
    int lim;                     // contiguous: last_row - chunk start (>= 0)
};
template <bool PAGED>
struct SeqAddr {
    const unsigned char *k_seq, *v_seq;   // head segment of the sequence's first row (paged: of pool row 0)
    const int32_t* ptab;
    uint32_t stride;
    int last_row;                          // contiguous: also kept inside the pool
    __device__ __forceinline__ SeqAddr(const VerifyArgs& a, int b, int hc, int row_bytes, uint32_t pool_stride,
                                       int last) {
        stride = pool_stride;
        int64_t row0 = 0;
        if (PAGED) {
            ptab = a.k.page_table + (int64_t)b * a.k.max_pages;
            last_row = last;
        } else {
            ptab = nullptr;
            row0 = seq_first_row(a.k.row_off[b], a.k.pool_rows);
            last_row = seq_last_row(last, row0, a.k.pool_rows);
        }
        k_seq = (const unsigned char*)a.k.base + (uint64_t)row0 * pool_stride + (int64_t)hc * row_bytes;
        v_seq = (const unsigned char*)a.v.base + (uint64_t)row0 * pool_stride + (int64_t)hc * row_bytes;
    }
    __device__ __forceinline__ int page(const VerifyArgs& a, int r) const {
        r = r < last_row ? r : last_row;
        return ptab[page_slot(r, a.k.page_rows, a.k.page_shift, a.k.max_pages)];
    }
    __device__ __forceinline__ ChunkAddr chunk(const unsigned char* seq, int base) const {
        ChunkAddr c;
        if (PAGED) {
            c.base = seq;
            c.lim = 0;
        } else {
            const int cb = chunk_start(base, last_row);
            c.base = seq + (uint64_t)(uint32_t)cb * stride;
            c.lim = last_row - cb;
        }
        return c;
    }
    __device__ __forceinline__ const u32x4* at(const VerifyArgs& a, const ChunkAddr& c, int base, int r, int col,
                                               int page) const {
        if (PAGED) {
            int row = base + r;
            row = row < last_row ? row : last_row;
            const int64_t prow = paged_pool_row(page, row, a.k.page_rows, a.k.page_shift, a.k.pool_rows);
            return (const u32x4*)(c.base + (uint64_t)(uint32_t)prow * stride + 16 * col);
        }
        const int rr = r < c.lim ? r : c.lim;   // chunk_row_offset with the chunk's limit precomputed; r >= 0
        return (const u32x4*)(c.base + ((uint32_t)rr * stride + 16u * (uint32_t)col));
    }
};

// A 16-byte piece of a K/V row.  STREAM: with the non-temporal hint, for multi-head attention where
// every byte is used once (the bench launch: 108 against 130 us).  With grouped-query attention the
// query heads of a group read the same rows at about the same time, and the hint would push the lines
// out of L2 before the next head of the group arrives (Qwen2.5-VL heads, 128 sequences: 51 against 68 us).
template <bool STREAM>
__device__ __forceinline__ u32x4 load_kv(const u32x4* p) {
    return STREAM ? __builtin_nontemporal_load(p) : *p;
}

// ---------------------------------------------------------------------------------------------
// T <= 32: every wavefront stages its own chunks (K and V) in a private LDS area; no workgroup
// barrier inside the loop.  K and V share one row mapping (same row_off / page_table).
// ---------------------------------------------------------------------------------------------
template <int DH, bool PAGED, bool STREAM>
__global__ __launch_bounds__(kMfThreads, 2) void verify_mfma_kernel(VerifyArgs a) {
    using Cf = MfCfg<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    TW_TRACE_MARK(a, 0);
    TW_TRACE_MARK(a, 6);
    TW_TRACE_MARK(a, 7);
    // the wavefront index in a scalar register: head, phase and chunk base are then scalars, branches
    // on them real branches, and the addresses below a scalar base plus a 32-bit lane offset
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, li = lane & 31;
    const int split = blockIdx.z;
    int hg, b;
    unit_of_block(a, hg, b);
    const int n_phase = a.n_phase;               // 1 (four heads per workgroup) or 4 (one head)
    const int phase = wave % n_phase;
    const int h = hg * a.heads_per_wg + wave / n_phase;
    const bool active = h < a.H;
    const int hc = active ? h : a.H - 1;
    const int t = li;                            // this lane's tree node
    // What depends on nothing but the unit is requested first: the lane's parent entry and its Q
    // fragments travel while the lengths and offsets of the sequence are still being read.
    const int par_raw = a.parent[(int64_t)b * a.T_max + (t < a.T_max ? t : a.T_max - 1)];
    u32x4 q_raw[Cf::kDC];
    issue_q<DH>(q_raw, a, b, hc, t, g);
    const SeqInfo sq = seq_info(a, b, split);
    if (split >= sq.n_b) return;                 // a piece past the end of this sequence (whole workgroup)

    unsigned char* ldsK = lds + wave * Cf::kStage;
    unsigned char* ldsV = ldsK + kChunk * Cf::kKStride;
    const float sl2 = a.scale * kLog2e;

    // lane's share of a chunk load: row (lane / lanes_per_row) + rows_per_load * j,
    // 16-byte column lane % lanes_per_row of the head's segment
    const int ld_row = lane / Cf::kLanesPerRow, ld_col = lane % Cf::kLanesPerRow;
    const uint32_t pool_stride = (uint32_t)(a.k.H * Cf::kRowB);   // a cache row holds the key/value heads
    // loads past the split re-read its last row (cached) and are masked
    const int last_row = sq.r_end > sq.r_begin ? sq.r_end - 1 : sq.r_begin;
    const int step = kChunk * n_phase;
    const SeqAddr<PAGED> ad(a, b, hc / a.group, Cf::kRowB, pool_stride, last_row);   // query head -> its key/value head

    // Paged caches: the page of every row this lane loads, looked up two chunks ahead
    // so the dependent data loads never wait on a table read.
    int pg[Cf::kLoads];
    auto lookup_pages = [&](int base) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) pg[j] = ad.page(a, base + ld_row + Cf::kRowsPerLoad * j);
    };
    u32x4 pk[Cf::kLoads], pv[Cf::kLoads];
    auto issue_loads = [&](int base) {
        const ChunkAddr ck = ad.chunk(ad.k_seq, base), cv = ad.chunk(ad.v_seq, base);
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            const int r = ld_row + Cf::kRowsPerLoad * j;
            pk[j] = load_kv<STREAM>(ad.at(a, ck, base, r, ld_col, PAGED ? pg[j] : 0));
            pv[j] = load_kv<STREAM>(ad.at(a, cv, base, r, ld_col, PAGED ? pg[j] : 0));
        }
    };

    const int first = sq.r_begin + kChunk * phase;
    if (active && first < sq.r_end) {
        if (PAGED) lookup_pages(first);
        issue_loads(first);
        if (PAGED) lookup_pages(first + step);
    }
    // the first chunk is in flight; now the tree masks (inside the wavefront) and the Q fragments
    TW_TRACE_MARK(a, 1);
    WaveState<DH> w;
    w.anc = wave_ancestor_mask(par_raw, t, sq.T);
    init_state<DH>(w, q_raw, t, sq.T);
    TW_TRACE_MARK(a, 2);
    for (int base = first; active && base < sq.r_end; base += step) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            const int r = ld_row + Cf::kRowsPerLoad * j;
            *(u32x4*)(ldsK + r * Cf::kKStride + ld_col * 16) = pk[j];
            *(u32x4*)(ldsV + r * Cf::kVStride + ld_col * 16) = pv[j];
        }
        issue_loads(base + step);
        if (PAGED) lookup_pages(base + 2 * step);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        process_chunk<DH>(w, ldsK, ldsV, base, sq.C, sq.n_rows, sl2, g, li);
        if (base == first) TW_TRACE_MARK(a, 3);
    }
    TW_TRACE_MARK(a, 4);
    if (n_phase == 1) {
        if (active) epilogue_direct<DH>(w, a, (float*)ldsK, b, h, sq.T, lane);
    } else {
        epilogue_merge<DH>(w, a, lds, b, h, sq.T, split, sq.n_b, phase, 1, n_phase, g, li, tid);
    }
    TW_TRACE_MARK(a, 5);
}

// ---------------------------------------------------------------------------------------------
// 32 < T <= 64: wavefronts 2p and 2p+1 hold node blocks 0 and 1 of the same (head, phase) and
// share one double-buffered stage: the even one loads the K chunk, the odd one the V chunk, two
// chunks ahead; one workgroup barrier per chunk makes the stage visible.  Every wavefront runs
// the same number of iterations so the barriers match.
// ---------------------------------------------------------------------------------------------
template <int DH, bool PAGED, bool STREAM>
__global__ __launch_bounds__(kMfThreads, 2) void verify_mfma_pair_kernel(VerifyArgs a) {
    using Cf = MfCfg<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    TW_TRACE_MARK(a, 0);
    TW_TRACE_MARK(a, 6);
    TW_TRACE_MARK(a, 7);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar, as in the kernel above
    const int g = lane >> 5, li = lane & 31;
    const int split = blockIdx.z;
    int hg, b;
    unit_of_block(a, hg, b);
    const int blk = wave & 1, pair = wave >> 1;
    const int n_phase = a.n_phase;               // 1 (two heads per workgroup) or 2 (one head)
    const int phase = n_phase == 1 ? 0 : pair;
    const int h = hg * a.heads_per_wg + (n_phase == 1 ? pair : 0);
    const bool active = h < a.H;
    const int hc = active ? h : a.H - 1;
    const int t = 32 * blk + li;
    // requested before anything else (see the kernel above); here lane = node for the masks
    const int par_raw = a.parent[(int64_t)b * a.T_max + (lane < a.T_max ? lane : a.T_max - 1)];
    u32x4 q_raw[Cf::kDC];
    issue_q<DH>(q_raw, a, b, hc, t, g);
    const SeqInfo sq = seq_info(a, b, split);
    if (split >= sq.n_b) return;                 // a piece past the end of this sequence (whole workgroup)

    unsigned char* stage = lds + pair * 2 * Cf::kStage;   // two buffers of one K+V chunk
    const float sl2 = a.scale * kLog2e;

    const int ld_row = lane / Cf::kLanesPerRow, ld_col = lane % Cf::kLanesPerRow;
    const int dst_off = blk == 0 ? 0 : kChunk * Cf::kKStride;
    const int dst_stride = blk == 0 ? Cf::kKStride : Cf::kVStride;
    const uint32_t pool_stride = (uint32_t)(a.k.H * Cf::kRowB);   // a cache row holds the key/value heads
    const int last_row = sq.r_end > sq.r_begin ? sq.r_end - 1 : sq.r_begin;
    const int step = kChunk * n_phase;
    const SeqAddr<PAGED> ad(a, b, hc / a.group, Cf::kRowB, pool_stride, last_row);   // query head -> its key/value head
    // the even wavefront of a pair streams K, the odd one V
    const unsigned char* seq_base = blk == 0 ? ad.k_seq : ad.v_seq;

    u32x4 pld[2][Cf::kLoads];
    // Paged caches: the pages of the chunk that a slot takes next are looked up when the slot's
    // current chunk is issued (four chunks ahead of its use), so data loads never wait on a table.
    int pg[2][PAGED ? Cf::kLoads : 1];
    auto lookup_pages = [&](int base, int slot) {
        if (PAGED) {
#pragma unroll
            for (int j = 0; j < Cf::kLoads; ++j) pg[slot][j] = ad.page(a, base + ld_row + Cf::kRowsPerLoad * j);
        }
    };
    auto issue_loads = [&](int base, int slot) {
        const ChunkAddr cc = ad.chunk(seq_base, base);
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j) {
            const int r = ld_row + Cf::kRowsPerLoad * j;
            pld[slot][j] = load_kv<STREAM>(ad.at(a, cc, base, r, ld_col, PAGED ? pg[slot][j] : 0));
        }
    };
    auto stage_chunk = [&](int slot, unsigned char* buf) {
#pragma unroll
        for (int j = 0; j < Cf::kLoads; ++j)
            *(u32x4*)(buf + dst_off + (ld_row + Cf::kRowsPerLoad * j) * dst_stride + ld_col * 16) = pld[slot][j];
    };

    const int n_chunks = (sq.r_end - sq.r_begin + kChunk - 1) / kChunk;
    const int n_iter = (n_chunks + n_phase - 1) / n_phase;   // the same for every wavefront of the workgroup
    const int first = sq.r_begin + kChunk * phase;
    lookup_pages(first, 0);
    lookup_pages(first + step, 1);
    issue_loads(first, 0);
    issue_loads(first + step, 1);
    lookup_pages(first + 2 * step, 0);
    lookup_pages(first + 3 * step, 1);
    // two chunks are in flight; now the tree masks (inside the wavefront) and the Q fragments
    TW_TRACE_MARK(a, 1);
    WaveState<DH> w;
    {
        const uint64_t m = wave_ancestor_mask(par_raw, lane, sq.T);   // of node `lane`; this lane's node is t
        w.anc = ((uint64_t)__shfl((uint32_t)(m >> 32), t, 64) << 32) | __shfl((uint32_t)m, t, 64);
    }
    init_state<DH>(w, q_raw, t, sq.T);
    TW_TRACE_MARK(a, 2);
    for (int it = 0; it < n_iter; it += 2) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int base = first + (it + half) * step;
            unsigned char* buf = stage + half * Cf::kStage;
            stage_chunk(half, buf);
            issue_loads(base + 2 * step, half);
            lookup_pages(base + 4 * step, half);
            __syncthreads();   // the partner's half of the chunk is staged; the other buffer is free again
            if (active && it + half < n_iter && base < sq.r_end)
                process_chunk<DH>(w, buf, buf + kChunk * Cf::kKStride, base, sq.C, sq.n_rows, sl2, g, li);
            if (it == 0 && half == 0) TW_TRACE_MARK(a, 3);
        }
    }
    TW_TRACE_MARK(a, 4);
    if (n_phase == 1) {
        __syncthreads();   // the partner is done with the shared stage; each wavefront takes one buffer of it
        if (active)
            epilogue_direct<DH>(w, a, (float*)(stage + blk * Cf::kStage), b, h, sq.T - 32 * blk, lane, 32 * blk);
    } else {
        epilogue_merge<DH>(w, a, lds, b, h, sq.T, split, sq.n_b, blk * n_phase + phase, 2, n_phase, g, li, tid);
    }
    TW_TRACE_MARK(a, 5);
}

template <int DH, bool PAGED, bool STREAM>
static hipError_t launch_one(const VerifyArgs& a, hipStream_t s) {
    const dim3 grid((a.H + a.heads_per_wg - 1) / a.heads_per_wg, a.B, a.n_splits);
    const size_t lds = MfCfg<DH>::kLds;
    const void* fn = a.n_blk == 1 ? (const void*)verify_mfma_kernel<DH, PAGED, STREAM>
                                  : (const void*)verify_mfma_pair_kernel<DH, PAGED, STREAM>;
    // the kernels' LDS need is a constant: raise the limit once per kernel and device, not on every launch
    static std::atomic<uint32_t> raised[2];
    const hipError_t e = raise_lds_limit_once(fn, (int)lds, raised[a.n_blk - 1]);
    if (e != hipSuccess) return e;
    if (a.n_blk == 1)
        hipLaunchKernelGGL((verify_mfma_kernel<DH, PAGED, STREAM>), grid, dim3(kMfThreads), lds, s, a);
    else
        hipLaunchKernelGGL((verify_mfma_pair_kernel<DH, PAGED, STREAM>), grid, dim3(kMfThreads), lds, s, a);
    return hipGetLastError();
}

template <int DH, bool PAGED>
static hipError_t launch_kv_policy(const VerifyArgs& a, hipStream_t s) {
    return a.group == 1 ? launch_one<DH, PAGED, true>(a, s) : launch_one<DH, PAGED, false>(a, s);
}

bool verify_mfma_supported(const VerifyArgs& a, int dtype) {
    return dtype == TW_BF16 && (a.d_h == 64 || a.d_h == 128) && a.k.page_table == a.v.page_table &&
           a.k.row_off == a.v.row_off && a.k.page_rows == a.v.page_rows &&
           a.k.max_pages == a.v.max_pages && a.k.pool_rows == a.v.pool_rows &&
           a.k.pool_rows <= 0x7FFFFFFFll && a.scale > 0.f;
}

hipError_t launch_verify_mfma(const VerifyArgs& a, hipStream_t s) {
    if (a.d_h == 128) return a.k.page_table ? launch_kv_policy<128, true>(a, s) : launch_kv_policy<128, false>(a, s);
    return a.k.page_table ? launch_kv_policy<64, true>(a, s) : launch_kv_policy<64, false>(a, s);
}

}  // namespace tw
