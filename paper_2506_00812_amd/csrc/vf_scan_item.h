// The work of one scan item -- a tile of queries against a segment of an interleaved list, with the exact top-K
// selection fused in -- as device functions, so that the launch-per-batch kernels and the resident serving kernel
// share them: scan_topk_item (32-row matrix-core tiles, uint8 and float32) and scan_valu_item (float32 on plain
// FMAs, one list entry per lane).  One-wave workgroups; smem is the workgroup's dynamic LDS.
#pragma once

#include "vf_select.h"

namespace vf {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
template <int DT> struct Acc;
template <> struct Acc<0> { using type = v16i; };
template <> struct Acc<1> { using type = v16f; };

constexpr int kDrainRows = 4;   // rows merged at a time by the 64-lane networks

// WAVE_ONLY: the wave works by itself inside a larger workgroup (the serving kernel), see wave_sync
template <int DT, int NCP, bool WAVE_ONLY = false>
__device__ __forceinline__ void scan_topk_item(const ScanParams &p, const ScanItem &it, uint4 *smem)
{
    const int lane = wave_lane<WAVE_ONLY>(), n32 = lane & 31, h = lane >> 5;
    const int ncp = NCP > 0 ? NCP : p.ncp;
    const int nchunks = 2 * ncp, K = p.K;
    const int row_bytes = p.dim * (DT == 0 ? 1 : 4);
    const int real_chunks = row_bytes / kChunkBytes;

    const int TR = p.tile_rows;                                  // rows the LDS buffers hold (16 or 32)
    uint4 *qtile = smem;                                         // [nchunks][TR]
    const int KS = K | 1;                                        // row stride of `best` (odd: spreads LDS banks)
    constexpr int PC = 64;                                       // pending slots per row: drained before a group could overflow them
    uint64_t *pend = (uint64_t *)(smem + nchunks * TR);          // [tile_rows][PC] candidates not yet merged
    uint64_t *best = pend + p.tile_rows * PC;                    // [tile_rows][KS] K best so far, ascending, KEY_MAX padded
    int32_t *qrow_s = (int32_t *)(best + p.tile_rows * KS);      // [32]
    uint32_t *qnorm_s = (uint32_t *)(qrow_s + 32);               // [32] float bits / int
    uint32_t *pcnt = qnorm_s + 32;                               // [32] keys waiting in pend[r]

    if (lane < 32) { qrow_s[lane] = lane < it.q_count ? p.qrow[it.q_begin + lane] : -1; pcnt[lane] = 0; }
    for (int i = lane; i < p.tile_rows * KS; i += 64) best[i] = KEY_MAX;
    wave_sync<WAVE_ONLY>();

    // ---- stage the query tile, chunk-major, and its norms
    {
        // lane (r = n32, h) copies chunks h, h+2, ... of query row r; eight loads are issued
        // before the first is stored so that their latencies overlap
        const int qr = qrow_s[n32];
        const char *qp = (const char *)p.qsrc + (int64_t)(qr >= 0 ? qr : 0) * row_bytes;
        for (int c0 = h; c0 < nchunks; c0 += 16) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 2 * u;
                v[u] = make_uint4(0, 0, 0, 0);
                if (qr >= 0 && c < real_chunks) v[u] = *(const uint4 *)(qp + c * kChunkBytes);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 2 * u;
                if (c < nchunks && n32 < TR) {
                    uint4 w = v[u];
                    if (DT == 0 && qr >= 0 && c < real_chunks) {
                        w.x ^= 0x80808080u; w.y ^= 0x80808080u; w.z ^= 0x80808080u; w.w ^= 0x80808080u;
                    }
                    qtile[c * TR + n32] = w;
                }
            }
        }
    }
    wave_sync<WAVE_ONLY>();
    {
        // row n32, chunks h, h+2, ...
        if (DT == 0) {
            int acc = 0;
            for (int c = h; c < nchunks && n32 < TR; c += 2) {
                const uint4 v = qtile[c * TR + n32];
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int e = (int)(int8_t)(w[i] >> (8 * b));
                        acc += e * e;
                    }
            }
            acc += __shfl_xor(acc, 32);
            if (h == 0) qnorm_s[n32] = (uint32_t)acc;
        } else {
            float acc = 0.f;
            for (int c = h; c < nchunks && n32 < TR; c += 2) {
                const uint4 v = qtile[c * TR + n32];
                const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
#pragma unroll
                for (int i = 0; i < 4; ++i) acc += f[i] * f[i];
            }
            acc += __shfl_xor(acc, 32);
            if (h == 0) qnorm_s[n32] = __float_as_uint(acc);
        }
    }
    wave_sync<WAVE_ONLY>();

    // per-lane constants for its 16 accumulator rows: row(j) = 8*(j/4) + 4*h + (j%4)
    uint32_t qn[16], thr[16];
    uint32_t and_rows = 0;  // bit j: row(j) is an AND query
    uint32_t live_rows = 0; // bit j: row(j) holds a query
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int row = 8 * (j >> 2) + 4 * h + (j & 3);
        qn[j] = qnorm_s[row];
        thr[j] = 0xFFFFFFFFu;
        if (row < it.q_count) live_rows |= 1u << j;
        if (p.others_off != nullptr && row < it.q_count) {
            const int qr = qrow_s[row];
            if (p.others_off[qr + 1] > p.others_off[qr]) and_rows |= 1u << j;
        }
    }
    const bool any_and = __any(and_rows != 0);
    // state of tile row r, held by lane r (r < 32)
    int pcv = 0;                  // keys waiting in pend[r] (copy of pcnt[r])
    uint64_t row_kth = KEY_MAX;   // K-th best key of row r so far; a candidate must be smaller to enter

    // Merge the pending queue of every row into its sorted K best, one row at a time with the whole
    // wave, then broadcast the thresholds to the accumulator layout (thr[j] of lane (n32, h)
    // belongs to row 8*(j/4) + 4*h + (j%4)).
    auto drain = [&]() {
        wave_lds_sync();
        if (K <= 16) wave_drain_rows_packed<16>(pend, PC, best, KS, K, pcv, row_kth, lane);
        if (K <= 32) wave_drain_rows_packed<32>(pend, PC, best, KS, K, pcv, row_kth, lane);
        wave_drain_rows<kDrainRows>(pend, PC, best, KS, K, pcv, row_kth, lane);
        if (lane < 32) pcnt[lane] = 0;
        wave_lds_sync();
        const uint32_t t = (uint32_t)(row_kth >> 32);
#pragma unroll
        for (int j = 0; j < 16; ++j) thr[j] = __shfl(t, 8 * (j >> 2) + 4 * h + (j & 3));
    };

    const int n_groups = (it.n + kGroup - 1) / kGroup;
    // B operand registers: the whole group is resident; each half is refilled with the next
    // group's chunks right after its own MFMAs have been issued, so the loads have the other
    // half's MFMAs and the selection to complete in -- a full group of prefetch distance for
    // one group's worth of registers.
    constexpr int NB = NCP > 0 ? NCP : 1;
    constexpr int H0 = (NB + 1) / 2;
    uint4 breg[NB];
    if constexpr (NCP > 0) {
        const uint4 *blk0 = p.xblk + it.group0 * (int64_t)(nchunks * 32);
#pragma unroll
        for (int cp = 0; cp < NCP; ++cp) breg[cp] = blk0[(2 * cp + h) * 32 + n32];
    }
    // norm (and, for AND tiles, global id) of this lane's entry, fetched one group ahead as well
    uint32_t xn_next = ((const uint32_t *)p.xnorm)[it.group0 * kGroup + n32];
    int32_t gid_next = -1;
    if (any_and && n32 < it.n) gid_next = p.map[it.map_off + it.entry0 + n32];
    // graph build: the entry that is the query itself is skipped (entry == self0 + row base)
    const int self0 = it.self_base >= 0 ? it.self_base + 4 * h : -0x40000000;
    for (int grp = 0; grp < n_groups; ++grp) {
        const uint4 *blk = p.xblk + (it.group0 + grp) * (int64_t)(nchunks * 32);
        typename Acc<DT>::type acc;
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0;
        const uint32_t xn = xn_next;
        const int32_t gid = gid_next;
        if (grp + 1 < n_groups) {
            xn_next = ((const uint32_t *)p.xnorm)[(it.group0 + grp + 1) * kGroup + n32];
            if (any_and && (grp + 1) * kGroup + n32 < it.n)
                gid_next = p.map[it.map_off + it.entry0 + (grp + 1) * kGroup + n32];
        }
        auto contract = [&](int cp, uint4 b) {
            // rows the tile does not hold contribute zeros without touching LDS
            uint4 a = make_uint4(0, 0, 0, 0);
            if (n32 < TR) a = qtile[(2 * cp + h) * TR + n32];
            if constexpr (DT == 0) {
                b.x ^= 0x80808080u; b.y ^= 0x80808080u; b.z ^= 0x80808080u; b.w ^= 0x80808080u;
                const v4i av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w};
                const v4i bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w};
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, acc, 0, 0, 0);
            } else {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
            }
        };
        if constexpr (NCP > 0) {
            const bool more = grp + 1 < n_groups;
            const uint4 *nblk = blk + nchunks * 32;
#pragma unroll
            for (int cp = 0; cp < H0; ++cp) contract(cp, breg[cp]);
            if (more) {
#pragma unroll
                for (int cp = 0; cp < H0; ++cp) breg[cp] = nblk[(2 * cp + h) * 32 + n32];
            }
#pragma unroll
            for (int cp = H0; cp < NCP; ++cp) contract(cp, breg[cp]);
            if (more) {
#pragma unroll
                for (int cp = H0; cp < NCP; ++cp) breg[cp] = nblk[(2 * cp + h) * 32 + n32];
            }
        } else {
            for (int cp = 0; cp < ncp; ++cp) contract(cp, blk[(2 * cp + h) * 32 + n32]);
        }
        const int entry = it.entry0 + grp * kGroup + n32;   // list-relative
        const bool col_ok = grp * kGroup + n32 < it.n;

        // phase 1 (pure VALU, branch-free): distances and threshold tests of this lane's 16 rows
        uint32_t bitsv[16];
        uint32_t pm = 0;   // bit j: the entry of this lane is a candidate for row(j)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if constexpr (DT == 0) {
                bitsv[j] = (uint32_t)((int)qn[j] + (int)xn - 2 * acc[j]);
            } else {
                const float d = (__uint_as_float(qn[j]) + __uint_as_float(xn)) - 2.0f * acc[j];
                bitsv[j] = __float_as_uint(fmaxf(d, 0.0f));
            }
            const uint32_t below = bitsv[j] <= thr[j] ? 1u : 0u;
            const uint32_t not_self = entry != self0 + 8 * (j >> 2) + (j & 3) ? 1u : 0u;
            pm |= (below & not_self) << j;
        }
        pm &= col_ok ? live_rows : 0u;
        if (any_and && pm != 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (((pm & and_rows) >> j) & 1u) {
                    // partner labels of the row's query (looked up on demand: few pairs get here)
                    const int qr = qrow_s[8 * (j >> 2) + 4 * h + (j & 3)];
                    const int o_begin = p.others_off[qr], o_end = p.others_off[qr + 1];
                    bool ok = true;
                    for (int o = o_begin; o < o_end && ok; ++o) ok = has_label(p.meta, p.others[o], gid);
                    if (!ok) pm &= ~(1u << j);
                }
            }
        }
        // phase 2: every lane queues its candidates (slot from the row's LDS counter)
        if (pm != 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if ((pm >> j) & 1u) {
                    const int row = 8 * (j >> 2) + 4 * h + (j & 3);
                    const uint32_t slot = atomicAdd(&pcnt[row], 1u);
                    pend[row * PC + slot] = ((uint64_t)bitsv[j] << 32) | (uint32_t)entry;
                }
            }
        }
        if (__any(pm != 0)) {
            wave_lds_sync();
            pcv = lane < 32 ? (int)pcnt[lane] : 0;
        }
        if (__any(pcv > PC - 32) || (grp + 1 == n_groups && __any(pcv != 0))) drain();
    }
    wave_sync<WAVE_ONLY>();

    // ---- results: every row's K best are already in ascending order
    for (int r = 0; r < it.q_count; ++r) {
        if (lane >= K) continue;
        const uint64_t key = best[r * KS + lane];
        const bool none = key == KEY_MAX;
        const uint32_t hi = (uint32_t)(key >> 32), idx = (uint32_t)key;
        if (it.part_row < 0) {
            const int64_t o = (int64_t)qrow_s[r] * K + lane;
            p.out_ids[o] = none ? -1 : (int64_t)p.map[it.map_off + idx];
            p.out_dists[o] = none ? __builtin_inff() : (DT == 0 ? (float)(int)hi : __uint_as_float(hi));
        } else {
            const int64_t o = (int64_t)(it.part_row + r) * K + lane;
            p.res_idx[o] = none ? -1 : (int32_t)idx;
            p.res_bits[o] = hi;
        }
    }
}


// QLDS: the tile's single query is read from LDS (q_lds, NCH * 4 floats) instead of through scalar loads from
// global memory.  A resident kernel needs that: its queries arrive in memory that is rewritten while the kernel
// runs, and the scalar data cache is never invalidated inside a kernel.
template <int NCH, bool QLDS = false>
__device__ __forceinline__ void scan_valu_item(const ScanParams &p, const ScanItem &it, uint4 *smem, const float *q_lds = nullptr)
{
    const int lane = wave_lane<QLDS>(), n32 = lane & 31, h = lane >> 5;
    const int K = p.K, KS = K | 1, TR = p.tile_rows;
    constexpr int PC = 96;   // a step adds <= 64 keys to a row and rows above 32 are drained after every step
    constexpr int row_bytes = NCH * kChunkBytes;
    uint64_t *pend = (uint64_t *)smem;                  // [TR][PC]
    uint64_t *best = pend + TR * PC;                    // [TR][KS]
    int32_t *qrow_s = (int32_t *)(best + TR * KS);      // [32]
    float *qnorm_s = (float *)(qrow_s + 32);            // [32]

    if (lane < 32) qrow_s[lane] = lane < it.q_count ? p.qrow[it.q_begin + lane] : -1;
    for (int i = lane; i < TR * KS; i += 64) best[i] = KEY_MAX;
    wave_sync<QLDS>();
    for (int r = 0; r < it.q_count; ++r) {
        float acc = 0.f;
        if (lane < NCH) {
            const uint4 v = *(const uint4 *)((const char *)p.qsrc + (int64_t)qrow_s[r] * row_bytes + lane * kChunkBytes);
            const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
            acc = (f[0] * f[0] + f[1] * f[1]) + (f[2] * f[2] + f[3] * f[3]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) qnorm_s[r] = acc;
    }
    wave_sync<QLDS>();

    // state of tile row r, held by lane r
    int pcv = 0;
    uint64_t row_kth = KEY_MAX;
    const float qn_lane = lane < it.q_count ? qnorm_s[lane] : 0.f;
    const int qr_lane = lane < 32 ? qrow_s[lane] : -1;
    uint32_t and_rows = 0;
    if (p.others_off != nullptr)
        and_rows = (uint32_t)__ballot(lane < it.q_count && p.others_off[qr_lane >= 0 ? qr_lane + 1 : 0] > p.others_off[qr_lane >= 0 ? qr_lane : 0]);

    const int n_groups = (it.n + kGroup - 1) / kGroup;
    const int n_steps = (n_groups + 1) / 2;
    for (int step = 0; step < n_steps; ++step) {
        const int grp = 2 * step + h;
        const int g_eff = grp < n_groups ? grp : n_groups - 1;   // the odd tail group does not exist: re-read the last one, masked
        const int rel = grp * kGroup + n32;
        const bool col_ok = rel < it.n;
        const int entry = it.entry0 + rel;
        const uint4 *blk = p.xblk + (it.group0 + g_eff) * (int64_t)(NCH * 32);
        uint32_t x[NCH * 4];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const uint4 v = blk[c * 32 + n32];
            x[4 * c] = v.x; x[4 * c + 1] = v.y; x[4 * c + 2] = v.z; x[4 * c + 3] = v.w;
        }
        const float xn = ((const float *)p.xnorm)[(it.group0 + g_eff) * kGroup + n32];
        int32_t gid = -1;
        if (and_rows != 0 && col_ok) gid = p.map[it.map_off + entry];

        for (int r = 0; r < it.q_count; ++r) {
            const int qr = __builtin_amdgcn_readlane(qr_lane, r);
            // the queries are not written while the kernel runs: reading them through the constant
            // address space makes these wave-uniform loads scalar loads
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
            if constexpr (QLDS) {
#pragma unroll
                for (int e = 0; e < NCH * 4; e += 4) {
                    const float4 qv = *(const float4 *)(q_lds + e);   // every lane reads the same address: a broadcast
                    a0 = __builtin_fmaf(__uint_as_float(x[e]), qv.x, a0);
                    a1 = __builtin_fmaf(__uint_as_float(x[e + 1]), qv.y, a1);
                    a2 = __builtin_fmaf(__uint_as_float(x[e + 2]), qv.z, a2);
                    a3 = __builtin_fmaf(__uint_as_float(x[e + 3]), qv.w, a3);
                }
            } else {
                typedef const float __attribute__((address_space(4))) *const_f32;
                const const_f32 qp = (const_f32)(uintptr_t)((const char *)p.qsrc + (int64_t)qr * row_bytes);
#pragma unroll
                for (int e = 0; e < NCH * 4; e += 4) {
                    a0 = __builtin_fmaf(__uint_as_float(x[e]), qp[e], a0);
                    a1 = __builtin_fmaf(__uint_as_float(x[e + 1]), qp[e + 1], a1);
                    a2 = __builtin_fmaf(__uint_as_float(x[e + 2]), qp[e + 2], a2);
                    a3 = __builtin_fmaf(__uint_as_float(x[e + 3]), qp[e + 3], a3);
                }
            }
            const float dot = (a0 + a1) + (a2 + a3);
            const float qn = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(qn_lane), r));
            const uint32_t bits = __float_as_uint(fmaxf((qn + xn) - 2.0f * dot, 0.0f));
            const uint32_t thr = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(row_kth >> 32), r);
            bool pass = col_ok && bits <= thr;
            if ((and_rows >> r) & 1u) {
                if (pass) {
                    const int o_begin = p.others_off[qr], o_end = p.others_off[qr + 1];
                    for (int o = o_begin; o < o_end && pass; ++o) pass = has_label(p.meta, p.others[o], gid);
                }
            }
            const uint64_t m = __ballot(pass);
            if (m != 0) {
                const int base = __builtin_amdgcn_readlane(pcv, r);
                if (pass) pend[r * PC + base + __popcll(m & ((1ull << lane) - 1ull))] = ((uint64_t)bits << 32) | (uint32_t)entry;
                if (lane == r) pcv = base + __popcll(m);
            }
        }
        if (__any(pcv > PC - 64) || (step + 1 == n_steps && __any(pcv != 0))) {
            wave_lds_sync();
            if (K <= 16) wave_drain_rows_packed<16>(pend, PC, best, KS, K, pcv, row_kth, lane);
            if (K <= 32) wave_drain_rows_packed<32>(pend, PC, best, KS, K, pcv, row_kth, lane);
            wave_drain_rows<4>(pend, PC, best, KS, K, pcv, row_kth, lane);
            wave_lds_sync();
        }
    }
    wave_sync<QLDS>();

    for (int r = 0; r < it.q_count; ++r) {
        if (lane >= K) continue;
        const uint64_t key = best[r * KS + lane];
        const bool none = key == KEY_MAX;
        const uint32_t hi = (uint32_t)(key >> 32), idx = (uint32_t)key;
        if (it.part_row < 0) {
            const int64_t o = (int64_t)qrow_s[r] * K + lane;
            p.out_ids[o] = none ? -1 : (int64_t)p.map[it.map_off + idx];
            p.out_dists[o] = none ? __builtin_inff() : __uint_as_float(hi);
        } else {
            const int64_t o = (int64_t)(it.part_row + r) * K + lane;
            p.res_idx[o] = none ? -1 : (int32_t)idx;
            p.res_bits[o] = hi;
        }
    }
}


}  // namespace vf
