// Exact top-K selection fused behind a matrix-core contraction, shared by the scan kernels and the seed
// selection kernel.  Each tile row has a queue of pending candidates and a sorted list of its K best so far in
// LDS; the wave merges queues into lists with bitonic networks over its 64 lanes (or over aligned segments of
// 16 / 32 lanes, several rows at a time).  Keys are (distance bits << 32 | entry index): unsigned order is
// (distance, index) order.  One-wave workgroups only.
#pragma once

#include "vf_device.h"

namespace vf {

// Ascending bitonic sort of the keys held one per lane, independently inside every
// aligned segment of SEG lanes (SEG = 16, 32 or 64).
template <int SEG> __device__ __forceinline__ uint64_t wave_sort_segments(uint64_t v, int lane)
{
#pragma unroll
    for (int k = 2; k <= SEG; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)v, j), hi = __shfl_xor((uint32_t)(v >> 32), j);
            const uint64_t o = ((uint64_t)hi << 32) | lo;
            const bool up = k == SEG ? true : (lane & k) == 0;
            const bool take_min = ((lane & j) == 0) == up;
            const uint64_t mn = v < o ? v : o, mx = v < o ? o : v;
            v = take_min ? mn : mx;
        }
    }
    return v;
}

// Ascending sort of a bitonic sequence held one key per lane (last stage of the network above).
__device__ __forceinline__ uint64_t wave_bitonic_merge64(uint64_t v, int lane)
{
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, j), hi = __shfl_xor((uint32_t)(v >> 32), j);
        const uint64_t o = ((uint64_t)hi << 32) | lo;
        const uint64_t mn = v < o ? v : o, mx = v < o ? o : v;
        v = (lane & j) == 0 ? mn : mx;
    }
    return v;
}

// The same two networks over NR independent key sets at once: the chains of dependent
// cross-lane moves of the NR sets interleave, which hides their latency.
template <int NR> __device__ __forceinline__ void wave_sort64_multi(uint64_t (&v)[NR], int lane)
{
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const bool up = k == 64 ? true : (lane & k) == 0;
            const bool take_min = ((lane & j) == 0) == up;
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                const uint32_t lo = __shfl_xor((uint32_t)v[u], j), hi = __shfl_xor((uint32_t)(v[u] >> 32), j);
                const uint64_t o = ((uint64_t)hi << 32) | lo;
                const uint64_t mn = v[u] < o ? v[u] : o, mx = v[u] < o ? o : v[u];
                v[u] = take_min ? mn : mx;
            }
        }
    }
}

template <int NR> __device__ __forceinline__ void wave_bitonic_merge64_multi(uint64_t (&v)[NR], int lane)
{
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) {
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const uint32_t lo = __shfl_xor((uint32_t)v[u], j), hi = __shfl_xor((uint32_t)(v[u] >> 32), j);
            const uint64_t o = ((uint64_t)hi << 32) | lo;
            const uint64_t mn = v[u] < o ? v[u] : o, mx = v[u] < o ? o : v[u];
            v[u] = (lane & j) == 0 ? mn : mx;
        }
    }
}

// Orders the LDS accesses of a one-wave workgroup without waiting for outstanding global loads
// (a wave's DS instructions execute in issue order; only the compiler must not reorder them).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Merge the pending queues of all tile rows into their sorted K best, NR rows at a time with
// the whole wave.  Lane r (r < 32) holds row r's pending count `pcv` (<= 2 * 64) and its K-th
// best key `row_kth`; pend is [rows][PC], best is [rows][KS] ascending, KEY_MAX padded.
// A row's 64 pending keys are sorted, the 64 smallest of them and the row's reversed best list
// form a bitonic sequence (element-wise minimum), and one merge network sorts that.
template <int NR>
__device__ __forceinline__ void wave_drain_rows(uint64_t *pend, int PC, uint64_t *best, int KS, int K, int &pcv,
                                                uint64_t &row_kth, int lane)
{
    uint32_t todo = (uint32_t)__ballot(lane < 32 && pcv > 0);
    while (todo != 0) {
        int rr[NR];
        bool on[NR];
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            on[u] = todo != 0;
            rr[u] = on[u] ? __builtin_ctz(todo) : rr[0];
            todo &= todo - 1;
        }
        int pc_max = 0;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int pc = on[u] ? __builtin_amdgcn_readlane(pcv, rr[u]) : 0;
            pc_max = pc > pc_max ? pc : pc_max;
        }
        for (int off = 0; off < pc_max; off += 64) {
            uint64_t v[NR];
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                const int pc = __builtin_amdgcn_readlane(pcv, rr[u]);
                const uint64_t kth = readlane64(row_kth, rr[u]);
                const uint64_t x = (on[u] && off + lane < pc) ? pend[rr[u] * PC + off + lane] : KEY_MAX;
                v[u] = x < kth ? x : KEY_MAX;
            }
            wave_sort64_multi<NR>(v, lane);
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                const uint64_t w = lane < K ? best[rr[u] * KS + lane] : KEY_MAX;
                const uint32_t lo = __shfl((uint32_t)v[u], 63 - lane), hi = __shfl((uint32_t)(v[u] >> 32), 63 - lane);
                const uint64_t vr = ((uint64_t)hi << 32) | lo;
                v[u] = w < vr ? w : vr;
            }
            wave_bitonic_merge64_multi<NR>(v, lane);
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                if (on[u]) {   // wave uniform
                    if (lane < K) best[rr[u] * KS + lane] = v[u];
                    const uint64_t nk = readlane64(v[u], K - 1);
                    if (lane == rr[u]) row_kth = nk;
                }
            }
            if (off + 64 < pc_max) wave_lds_sync();   // the next round reads the lists just written
        }
    }
    pcv = 0;
}

// The rows whose queue holds at most SEG keys (K <= SEG), 64 / SEG of them at a time: one row per
// aligned segment of SEG lanes, the sort and merge networks confined to the segment.  After the
// first drain of an item almost every row is of this kind (a handful of keys passed the row's
// threshold), and a 16-lane network has 10 + 4 stages for four rows where the 64-lane one has
// 21 + 6 for each.  Rows it has merged leave with pcv = 0.
template <int SEG>
__device__ __forceinline__ void wave_drain_rows_packed(const uint64_t *pend, int PC, uint64_t *best, int KS, int K,
                                                       int &pcv, uint64_t &row_kth, int lane)
{
    constexpr int NSEG = 64 / SEG;
    const int seg = lane / SEG, ls = lane % SEG;
    uint32_t todo = (uint32_t)__ballot(lane < 32 && pcv > 0 && pcv <= SEG);
    const uint32_t merged = todo;
    while (todo != 0) {
        int r = -1;   // the row of this lane's segment
#pragma unroll
        for (int u = 0; u < NSEG; ++u) {
            const int ru = todo != 0 ? __builtin_ctz(todo) : -1;
            if (u == seg) r = ru;
            todo &= todo - 1;
        }
        const int rs = r >= 0 ? r : 0;
        const int pc_rs = __shfl(pcv, rs);   // outside any condition: a cross-lane read needs its source lane active
        const int pc = r >= 0 ? pc_rs : 0;
        const uint32_t klo = __shfl((uint32_t)row_kth, rs), khi = __shfl((uint32_t)(row_kth >> 32), rs);
        const uint64_t kth = ((uint64_t)khi << 32) | klo;
        uint64_t x = ls < pc ? pend[rs * PC + ls] : KEY_MAX;
        x = x < kth ? x : KEY_MAX;
        x = wave_sort_segments<SEG>(x, lane);
        const int bi = SEG - 1 - ls;   // the row's best list, reversed
        const uint64_t w = (r >= 0 && bi < K) ? best[rs * KS + bi] : KEY_MAX;
        x = w < x ? w : x;             // ascending min descending: the SEG smallest, bitonic
#pragma unroll
        for (int j = SEG / 2; j > 0; j >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)x, j), hi = __shfl_xor((uint32_t)(x >> 32), j);
            const uint64_t o = ((uint64_t)hi << 32) | lo;
            const uint64_t mn = x < o ? x : o, mx = x < o ? o : x;
            x = (lane & j) == 0 ? mn : mx;
        }
        if (r >= 0 && ls < K) best[rs * KS + ls] = x;
    }
    if (merged != 0) {
        wave_lds_sync();
        if (lane < 32 && ((merged >> lane) & 1u)) { row_kth = best[lane * KS + K - 1]; pcv = 0; }
    }
}

}  // namespace vf
