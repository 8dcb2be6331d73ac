// Device-side helpers shared by the gfx950 kernels.
#pragma once

#include "vf_internal.h"

#pragma clang fp contract(off)

namespace vf {

// Membership test "global id g carries label l" (the predicate of Section 4.3.2).
// Graph labels answer from their bitset; scan labels by binary search in their
// ascending posting list.
__device__ __forceinline__ bool has_label(const LabelMeta &m, int32_t l, int32_t g)
{
    const int32_t slot = m.hs_slot[l];
    if (slot >= 0) return (m.bitsets[(int64_t)slot * m.bitset_words + (g >> 5)] >> (g & 31)) & 1u;
    const int64_t off = m.O_LS[l];
    if (off < 0) return false;
    int32_t lo = 0, hi = m.S[l] - 1;
    while (lo <= hi) {
        const int32_t mid = (lo + hi) >> 1;
        const int32_t v = m.M_LS[off + mid];
        if (v == g) return true;
        if (v < g) lo = mid + 1; else hi = mid - 1;
    }
    return false;
}

// The barrier of a one-wave workgroup; or (WAVE_ONLY), for a wave that works by itself inside a larger workgroup
// (the serving kernel's workers), only what a one-wave barrier is needed for: the ordering of the wave's own LDS
// traffic -- without the workgroup barrier the other waves would have to join.
template <bool WAVE_ONLY> __device__ __forceinline__ void wave_sync()
{
    if constexpr (WAVE_ONLY) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    } else {
        __syncthreads();
    }
}
template <bool WAVE_ONLY> __device__ __forceinline__ int wave_lane() { return WAVE_ONLY ? (int)(threadIdx.x & 63u) : (int)threadIdx.x; }

// float -> bfloat16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_rn_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---------------------------------------------------------------- 8-lane teams

// Sum over the 8 lanes of a team in the fixed tree ((a0+a1)+(a2+a3)) + ((a4+a5)+(a6+a7));
// every lane of the team receives the result.
__device__ __forceinline__ float team_sum_f(float v)
{
    v = v + __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));  // quad_perm [1,0,3,2]
    v = v + __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true));  // quad_perm [2,3,0,1]
    v = v + __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x141, 0xF, 0xF, true)); // row_half_mirror
    return v;
}
__device__ __forceinline__ int team_sum_i(int v)
{
    v = v + __builtin_amdgcn_mov_dpp(v, 0xB1, 0xF, 0xF, true);
    v = v + __builtin_amdgcn_mov_dpp(v, 0x4E, 0xF, 0xF, true);
    v = v + __builtin_amdgcn_mov_dpp(v, 0x141, 0xF, 0xF, true);
    return v;
}

// Squared L2 distance between the query (16-byte chunks in qv) and the row at xrow,
// computed by one 8-lane team; tl = lane within the team.  Lane tl handles chunks
// tl, tl+8, ... .  fp32: lane-sequential acc = fma(d, d, acc) with d = q-x rounded, then
// team_sum_f -- an order that a CPU evaluation (C fmaf) reproduces bit for bit.
__device__ __forceinline__ uint32_t team_dist_bits_f32(const uint4 *qv, const char *xrow, int nchunks, int tl)
{
    const int steps = (nchunks + 7) >> 3;
    float acc = 0.0f;
    for (int st0 = 0; st0 < steps; st0 += 4) {
        uint4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {   // all loads of the batch are issued before the first use
            const int ci = (st0 + u) * 8 + tl;
            x[u] = make_uint4(0, 0, 0, 0);
            if (ci < nchunks) x[u] = *(const uint4 *)(xrow + ci * kChunkBytes);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ci = (st0 + u) * 8 + tl;
            if (ci < nchunks) {
                const uint4 q = qv[ci];
                float d;
                d = __uint_as_float(q.x) - __uint_as_float(x[u].x); acc = __builtin_fmaf(d, d, acc);
                d = __uint_as_float(q.y) - __uint_as_float(x[u].y); acc = __builtin_fmaf(d, d, acc);
                d = __uint_as_float(q.z) - __uint_as_float(x[u].z); acc = __builtin_fmaf(d, d, acc);
                d = __uint_as_float(q.w) - __uint_as_float(x[u].w); acc = __builtin_fmaf(d, d, acc);
            }
        }
    }
    return __float_as_uint(team_sum_f(acc));
}

// uint8: exact integer sum of (q-x)^2 = q.q + x.x - 2 q.x on the packed dot-product unit.
// qq_lane = sum of q^2 over the bytes this lane handles.
__device__ __forceinline__ int lane_qq_u8(const uint4 *qv, int nchunks, int tl)
{
    uint32_t qq = 0;
    for (int ci = tl; ci < nchunks; ci += 8) {
        const uint4 q = qv[ci];
        qq = __builtin_amdgcn_udot4(q.x, q.x, qq, false);
        qq = __builtin_amdgcn_udot4(q.y, q.y, qq, false);
        qq = __builtin_amdgcn_udot4(q.z, q.z, qq, false);
        qq = __builtin_amdgcn_udot4(q.w, q.w, qq, false);
    }
    return (int)qq;
}
__device__ __forceinline__ uint32_t team_dist_bits_u8(const uint4 *qv, int qq_lane, const char *xrow, int nchunks, int tl)
{
    const int steps = (nchunks + 7) >> 3;
    uint32_t xx = 0, qx = 0;
#pragma unroll 2
    for (int st = 0; st < steps; ++st) {
        const int ci = st * 8 + tl;
        if (ci < nchunks) {
            const uint4 x = *(const uint4 *)(xrow + ci * kChunkBytes);
            const uint4 q = qv[ci];
            xx = __builtin_amdgcn_udot4(x.x, x.x, xx, false); qx = __builtin_amdgcn_udot4(q.x, x.x, qx, false);
            xx = __builtin_amdgcn_udot4(x.y, x.y, xx, false); qx = __builtin_amdgcn_udot4(q.y, x.y, qx, false);
            xx = __builtin_amdgcn_udot4(x.z, x.z, xx, false); qx = __builtin_amdgcn_udot4(q.z, x.z, qx, false);
            xx = __builtin_amdgcn_udot4(x.w, x.w, xx, false); qx = __builtin_amdgcn_udot4(q.w, x.w, qx, false);
        }
    }
    return (uint32_t)team_sum_i(qq_lane + (int)xx - 2 * (int)qx);
}

__device__ __forceinline__ uint64_t shfl64(uint64_t v, int src)
{
    const uint32_t lo = __shfl((uint32_t)v, src), hi = __shfl((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t shfl_up64(uint64_t v)
{
    const uint32_t lo = __shfl_up((uint32_t)v, 1), hi = __shfl_up((uint32_t)(v >> 32), 1);
    return ((uint64_t)hi << 32) | lo;
}

// value of lane `src` (wave-uniform index) in every lane
__device__ __forceinline__ uint64_t readlane64(uint64_t v, int src)
{
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, src), hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}
// lane i receives the value of lane i - 1 (lane 0 keeps its own): DPP wave_shr:1
__device__ __forceinline__ uint64_t wave_shr1_64(uint64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, 0x138, 0xF, 0xF, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32), 0x138, 0xF, 0xF, false);
    return ((uint64_t)hi << 32) | lo;
}

// Ascending bitonic sort of the 64 values held one per lane.
__device__ __forceinline__ uint32_t wave_sort_u32(uint32_t v, int lane)
{
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)v, j);
            const bool up = k == 64 ? true : (lane & k) == 0;
            const bool take_min = ((lane & j) == 0) == up;
            const uint32_t mn = v < o ? v : o, mx = v < o ? o : v;
            v = take_min ? mn : mx;
        }
    }
    return v;
}

// Ascending sort of a bitonic sequence of 64 values held one per lane.
__device__ __forceinline__ uint32_t wave_merge_u32(uint32_t v, int lane)
{
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, j);
        const uint32_t mn = v < o ? v : o, mx = v < o ? o : v;
        v = (lane & j) == 0 ? mn : mx;
    }
    return v;
}

// The same two networks for 64-bit keys.
__device__ __forceinline__ uint64_t wave_sort64(uint64_t v, int lane)
{
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)v, j), hi = __shfl_xor((uint32_t)(v >> 32), j);
            const uint64_t o = ((uint64_t)hi << 32) | lo;
            const bool up = k == 64 ? true : (lane & k) == 0;
            const bool take_min = ((lane & j) == 0) == up;
            const uint64_t mn = v < o ? v : o, mx = v < o ? o : v;
            v = take_min ? mn : mx;
        }
    }
    return v;
}

__device__ __forceinline__ uint64_t wave_merge64(uint64_t v, int lane)
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

// Bitonic sort of keys[0..n) ascending in LDS by one wave; n a power of two.
__device__ __forceinline__ void wave_bitonic_sort(uint64_t *keys, int n, int lane)
{
    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = lane; i < n / 2; i += 64) {
                const int a = ((i & ~(j - 1)) << 1) | (i & (j - 1)), b = a | j;
                const bool up = (a & k) == 0;
                const uint64_t x = keys[a], y = keys[b];
                if ((x > y) == up) { keys[a] = y; keys[b] = x; }
            }
            __syncthreads();
        }
}

}  // namespace vf
