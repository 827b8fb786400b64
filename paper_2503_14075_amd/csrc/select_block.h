// Top-R keep of one row by one workgroup (TopR of Sec. 3.1 Eq. 3): radix select on
// order-preserving 32-bit keys, ties toward the lower index, ascending output (or rank order on
// request).  A device function so that kernels which produce a row can select from it in place.
#pragma once

#include "twig_internal.h"

namespace tw {

// Larger float <=> larger key.  -0.0 is folded into +0.0 first so the two tie.
__device__ __forceinline__ uint32_t order_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Keys of one sequence are loaded once into registers (KPT per lane, THREADS lanes) when the
// row fits, otherwise (KPT == 0) every pass re-reads them from memory.
// sc: the row; out: its R output slots; ranked_row: NULL, or R slots for the values in rank order.
// Every thread of the THREADS-wide workgroup calls it (it contains workgroup barriers).
template <int KPT, int THREADS>
__device__ __forceinline__ void select_block(const float* __restrict__ sc, int M, int R, int32_t* __restrict__ out,
                                             float* __restrict__ ranked_row) {
    constexpr int kWaves = THREADS / 64;
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_prefix, s_need, s_eq_total;
    __shared__ uint32_t s_wave_a[4];   // the bucket scan is done by the first 256 lanes
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (R <= 0) return;

    uint32_t keys[KPT > 0 ? KPT : 1];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
        const int m = tid + u * THREADS;
        keys[u] = m < M ? order_key(sc[m]) : 0u;
    }
    const int n_iter = (M + THREADS - 1) / THREADS;

    if (tid == 0) {
        s_prefix = 0u;
        s_need = (uint32_t)R;
    }
    // Four passes, most significant byte first.  After a pass the key prefix of
    // the R-th largest element is known down to that byte, and s_need is its
    // rank among the elements sharing the prefix.
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) s_hist[tid] = 0u;
        __syncthreads();
        const uint32_t prefix = s_prefix, need = s_need;
        const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
        // Scores of one row share most of their leading bits, so in the first passes a wavefront's
        // keys fall into very few buckets: the lanes that share the first lane's bucket add their
        // count with one atomic, the others add one each.
        auto count = [&](bool valid, uint32_t key) {
            const uint32_t bucket = (key >> shift) & 0xFFu;
            const uint64_t vmask = __ballot(valid);
            if (vmask == 0ull) return;
            const int leader = __ffsll((unsigned long long)vmask) - 1;
            const uint32_t b0 = __builtin_amdgcn_readlane(bucket, leader);   // leader is wavefront-uniform
            const uint64_t same = __ballot(valid && bucket == b0);
            if (lane == leader) atomicAdd(&s_hist[b0], (uint32_t)__popcll(same));
            if (valid && bucket != b0) atomicAdd(&s_hist[bucket], 1u);
        };
        if (KPT > 0) {
#pragma unroll
            for (int u = 0; u < KPT; ++u) {
                const int m = tid + u * THREADS;
                count(m < M && (keys[u] & hi_mask) == prefix, keys[u]);
            }
        } else {
            for (int u = 0; u < n_iter; ++u) {
                const int m = tid + u * THREADS;
                const uint32_t key = m < M ? order_key(sc[m]) : 0u;
                count(m < M && (key & hi_mask) == prefix, key);
            }
        }
        __syncthreads();
        // lane tid < 256 owns bucket 255 - tid; inclusive scan from the largest bucket down
        uint32_t mine = 0u, incl = 0u;
        if (tid < 256) {
            mine = s_hist[255 - tid];
            incl = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off, 64);
                if (lane >= off) incl += up;
            }
            if (lane == 63) s_wave_a[wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = 0; w < wave; ++w) incl += s_wave_a[w];
            // exactly one bucket has  (count above it) < need <= (count above it) + (its own count)
            if (incl >= need && incl - mine < need) {
                s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
                s_need = need - (incl - mine);
                s_eq_total = mine;   // after the last pass: how many keys equal the R-th largest
            }
        }
        __syncthreads();
    }
    const uint32_t thr = s_prefix;   // key of the R-th largest score
    const uint32_t need = s_need;    // how many elements equal to it are kept (lowest indices)
    // Output in ascending index order.  Element m = u * THREADS + tid belongs to (round u,
    // wavefront): rounds, and wavefronts inside a round, are in index order, so an element's rank
    // among the equal keys and its output position are a count inside its wavefront (ballot) plus
    // the totals of all earlier (round, wavefront) cells, which every wavefront scans for itself,
    // one lane per cell.  A sweep covers as many rounds as 64 cells hold; the running totals are
    // carried from sweep to sweep.
    constexpr int kSweep = (KPT > 0 && KPT < 64 / kWaves) ? KPT : 64 / kWaves;   // rounds per sweep
    __shared__ uint32_t s_cell[64];
    // Long rows with few survivors (the top few of a vocabulary): instead of sweeping every round,
    // the survivors and the keys equal to the threshold are appended to a short list in any order
    // and ranked by index there.  Taken when the row needs several sweeps and the list fits.
    constexpr int kListCap = 1024;
    constexpr bool kManySweeps = KPT == 0 || KPT > kSweep;
    __shared__ uint32_t s_list[kManySweeps ? kListCap : 1];
    __shared__ uint32_t s_n_list;
    if (kManySweeps && (uint32_t)R - need + s_eq_total <= (uint32_t)kListCap) {
        if (tid == 0) s_n_list = 0u;
        __syncthreads();
        auto append = [&](uint32_t key, int m) {
            if (m < M && key >= thr) s_list[atomicAdd(&s_n_list, 1u)] = (uint32_t)m | (key == thr ? 0x80000000u : 0u);
        };
        if (KPT > 0) {
#pragma unroll
            for (int u = 0; u < KPT; ++u) append(keys[u], tid + u * THREADS);
        } else {
            for (int u = 0; u < n_iter; ++u) {
                const int m = tid + u * THREADS;
                append(m < M ? order_key(sc[m]) : 0u, m);
            }
        }
        __syncthreads();
        const int L = (int)s_n_list;
        constexpr uint32_t kEq = 0x80000000u, kKeep = 0x40000000u, kIdx = 0x3FFFFFFFu;   // indices are below 2^20
        // kept: every key above the threshold, and the `need` lowest indices among the equal ones.
        // The decisions are made on the list as appended, then written as a flag after a barrier.
        bool keep[(kListCap + THREADS - 1) / THREADS];
#pragma unroll
        for (int k = 0; k < (kListCap + THREADS - 1) / THREADS; ++k) {
            const int e = tid + k * THREADS;
            keep[k] = false;
            if (e < L) {
                const uint32_t me = s_list[e], idx = me & kIdx;
                keep[k] = true;
                if (me & kEq) {
                    uint32_t eq_rank = 0u;
                    for (int j = 0; j < L; ++j) eq_rank += (s_list[j] & kEq) && (s_list[j] & kIdx) < idx;
                    keep[k] = eq_rank < need;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < (kListCap + THREADS - 1) / THREADS; ++k) {
            const int e = tid + k * THREADS;
            if (e < L && keep[k]) s_list[e] |= kKeep;
        }
        __syncthreads();
        // output position of a kept entry: the kept entries with a lower index
#pragma unroll
        for (int k = 0; k < (kListCap + THREADS - 1) / THREADS; ++k) {
            const int e = tid + k * THREADS;
            if (e < L && keep[k]) {
                const uint32_t idx = s_list[e] & kIdx;
                uint32_t pos = 0u;
                for (int j = 0; j < L; ++j) pos += (s_list[j] & kKeep) && (s_list[j] & kIdx) < idx;
                if (pos < (uint32_t)R) out[pos] = (int32_t)idx;
            }
        }
    } else {
    const uint64_t below = (1ull << lane) - 1ull;
    uint32_t run_eq = 0u, run_sel = 0u;   // totals of the sweeps before this one (same in every thread)
    auto sweep = [&](int u0, auto key_of) {
        const int nu = min(kSweep, n_iter - u0);
        uint64_t eq_b[kSweep], gt_b[kSweep];
#pragma unroll
        for (int du = 0; du < kSweep; ++du) {
            const int m = (u0 + du) * THREADS + tid;
            bool eq = false, gt = false;
            if (du < nu && m < M) {
                const uint32_t key = key_of(du, m);
                eq = key == thr;
                gt = key > thr;
            }
            eq_b[du] = __ballot(eq);
            gt_b[du] = __ballot(gt);
            if (lane == 0) s_cell[du * kWaves + wave] = (uint32_t)__popcll(eq_b[du]);
        }
        __syncthreads();
        // exclusive scan of the equal-key counts over the cells
        uint32_t c = lane < nu * kWaves ? s_cell[lane] : 0u, incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        const uint32_t eq_total = __shfl(incl, 63, 64);
        const uint32_t eq_excl = incl - c;
        __syncthreads();   // every wavefront has read the equal-key counts
        uint64_t sel_b[kSweep];
#pragma unroll
        for (int du = 0; du < kSweep; ++du) {
            const uint32_t cell_base = __shfl(eq_excl, du * kWaves + wave, 64);
            const uint32_t eq_rank = run_eq + cell_base + (uint32_t)__popcll(eq_b[du] & below);
            const bool eq = (eq_b[du] >> lane) & 1ull, gt = (gt_b[du] >> lane) & 1ull;
            sel_b[du] = __ballot(gt || (eq && eq_rank < need));
            if (lane == 0) s_cell[du * kWaves + wave] = (uint32_t)__popcll(sel_b[du]);
        }
        __syncthreads();
        c = lane < nu * kWaves ? s_cell[lane] : 0u;
        incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        const uint32_t sel_total = __shfl(incl, 63, 64);
        const uint32_t sel_excl = incl - c;
#pragma unroll
        for (int du = 0; du < kSweep; ++du) {
            const uint32_t pos = run_sel + __shfl(sel_excl, du * kWaves + wave, 64) +
                                 (uint32_t)__popcll(sel_b[du] & below);
            if (((sel_b[du] >> lane) & 1ull) && pos < (uint32_t)R) out[pos] = (u0 + du) * THREADS + tid;
        }
        run_eq += eq_total;
        run_sel += sel_total;
        __syncthreads();   // the cells are rewritten by the next sweep
    };
    if (KPT > 0) {
        // register-held keys: the sweeps are unrolled so that keys[] is indexed by constants
#pragma unroll
        for (int u0 = 0; u0 < KPT; u0 += kSweep) {
            if (u0 < n_iter)
                sweep(u0, [&](int du, int) { return keys[(u0 + du) < KPT ? (u0 + du) : 0]; });
        }
    } else {
        for (int u0 = 0; u0 < n_iter; u0 += kSweep) sweep(u0, [&](int, int m) { return order_key(sc[m]); });
    }
    }
    // Rank order on request (R <= 256): larger value first, equal values lower index first, with
    // the values beside the indices.  The survivors were just written in index order by this
    // workgroup; the order is total, so every output slot is written exactly once.
    if (ranked_row) {
        __shared__ uint32_t s_rk_key[256];
        __shared__ int32_t s_rk_idx[256];
        __syncthreads();   // the survivors are in `out`
        int32_t idx = 0;
        uint32_t key = 0u;
        float v = 0.f;
        if (tid < R) {
            idx = out[tid];
            idx = idx < 0 ? 0 : (idx >= M ? M - 1 : idx);
            v = sc[idx];
            key = order_key(v);
            s_rk_key[tid] = key;
            s_rk_idx[tid] = idx;
        }
        __syncthreads();
        if (tid < R) {
            int rank = 0;
            for (int j = 0; j < R; ++j) rank += (s_rk_key[j] > key) || (s_rk_key[j] == key && s_rk_idx[j] < idx);
            out[rank] = idx;
            ranked_row[rank] = v;
        }
    }
}


}  // namespace tw
