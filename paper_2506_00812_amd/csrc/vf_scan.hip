// IVF-BFS (Section 4.2.2, Alg. 2): distances of a tile of up to 32 queries that
// share a label against every vector of that label's posting list, fused with an
// exact top-K selection.  The same contraction builds the per-label kNN graphs
// (queries = the list itself) and the exact ground truth.
//
// Mapping to CDNA4.  One wave64 per (query tile, list).  The list is stored in
// the paper's interleaved layout -- groups of 32 vectors, 16-byte chunks -- which
// is exactly the B-operand layout of a 32x32 MFMA on a 64-wide wave: lanes 0..31
// read chunk 2c of vectors 0..31 (512 contiguous bytes), lanes 32..63 chunk 2c+1.
// So list tiles go HBM -> registers -> MFMA with fully coalesced 1 KiB loads and
// no LDS round trip; the query tile (A operand) is staged once in LDS in the same
// chunk-major layout.  uint8 data is shifted by -128 on the fly and contracted on
// the int8 MFMA (exact int32); float data uses the fp32 MFMA.  Distances are
// |q|^2 + |x|^2 - 2 q.x.
//
// Top-K.  Each lane ends up with the distances of 16 query rows to one list entry
// (the MFMA accumulator layout).  A per-row threshold (the current K-th best) is
// kept in registers; a lane appends its survivors to the rows' pending queues in LDS
// (slot from an LDS atomic counter -- no cross-lane step).  When a queue could
// overflow, the wave merges queue after queue into the row's sorted K best: bitonic
// sort of the 64 pending keys in registers, element-wise minimum against the reversed
// sorted list, bitonic merge -- and broadcasts the tightened thresholds.  The result
// does not depend on the order in which candidates were queued.  Keys are
// (distance bits << 32 | entry index): unsigned order == (distance, id) order.
//
// Three kernels share that selection.  scan_topk_kernel: 32-row tiles (uint8 search, and for
// both types the kNN self-joins of the index build and the ground truth).  scan_topk16_kernel:
// float32 search tiles, which hold at most 16 queries, on the 16x16x4 MFMA.  scan_valu_kernel:
// float32 tiles of small batches on plain FMAs.
#include <type_traits>

#include "vf_select.h"

namespace vf {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

#ifndef VF_SCAN_WAVES
#define VF_SCAN_WAVES 2
#endif
#ifndef VF_SCAN16_WAVES
#define VF_SCAN16_WAVES 2
#endif
#ifndef VF_DRAIN_ROWS
#define VF_DRAIN_ROWS 4
#endif
template <int DT> struct Acc;
template <> struct Acc<0> { using type = v16i; };
template <> struct Acc<1> { using type = v16f; };

// NCP > 0: the number of chunk pairs per vector is known at compile time; the B
// operand of the NEXT group (NCP 1-KiB loads) is then fetched into registers while
// the MFMAs of the current group run, which is what keeps HBM busy at the skinny
// shapes of the search (a handful of queries per list).  NCP == 0: any p.ncp, no
// prefetch.
template <int DT, int NCP>
__global__ __launch_bounds__(64, VF_SCAN_WAVES) void scan_topk_kernel(ScanParams p)
{
    extern __shared__ uint4 smem[];
    const ScanItem it = p.items[blockIdx.x];
    const int lane = threadIdx.x, n32 = lane & 31, h = lane >> 5;
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
    __syncthreads();

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
    __syncthreads();
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
    __syncthreads();

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
        wave_drain_rows<VF_DRAIN_ROWS>(pend, PC, best, KS, K, pcv, row_kth, lane);
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
    __syncthreads();

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

// float32 search tiles of <= 16 queries: the same selection around v_mfma_f32_16x16x4_f32, which
// spends half the matrix-core time of a 32-row tile on them.  Lane (c = lane % 16, kq = lane / 16):
//   A operand  row c of the query tile, the 16-byte chunks 4 s + kq (s = 0 .. chunks / 4 - 1), read
//              from global memory once and kept in registers for the whole item (two waves per SIMD
//              leave room for it without spills; the workgroup's LDS holds only queues and lists);
//   B operand  list entries c (column block 0) and 16 + c (block 1) of the group, the same chunks;
//              the four components of a chunk feed four consecutive MFMAs, so the contraction
//              index runs over (s, kq, component) on both operands alike;
//   D          rows 4 kq + i (i = 0..3) x entry c of each column block.
template <int NCP, bool AND, int SLOTS>
__global__ __launch_bounds__(64, VF_SCAN16_WAVES) void scan_topk16_kernel(ScanParams p)
{
    extern __shared__ uint4 smem[];
    typedef float v4f __attribute__((ext_vector_type(4)));
    constexpr int NCH = 2 * NCP, NS = NCH / 4, row_bytes = NCH * kChunkBytes, PC = 64;
    static_assert(NCH % 4 == 0, "the chunk count must be a multiple of four");
    ScanItem it = p.items[blockIdx.x];
    if (p.panel_n > 0) {
        const int rem = it.n - p.panel_entry0;
        if (rem <= 0) return;   // the item's list ends before this panel (the whole workgroup leaves)
        it.group0 += p.panel_entry0 / kGroup;
        it.entry0 += p.panel_entry0;
        it.n = rem < p.panel_n ? rem : p.panel_n;
    }
    const int lane = threadIdx.x, n32 = lane & 31, h = lane >> 5, c16 = lane & 15, kq = lane >> 4;
    const int K = p.K, KS = K | 1, TR = p.tile_rows;   // TR <= 16

    uint64_t *pend = (uint64_t *)smem;                           // [TR][PC]
    uint64_t *best = pend + TR * PC;                             // [TR][KS]
    int32_t *qrow_s = (int32_t *)(best + TR * KS);               // [32]
    uint32_t *qnorm_s = (uint32_t *)(qrow_s + 32);               // [32]
    uint32_t *pcnt = qnorm_s + 32;                               // [32]

    if (lane < 32) { qrow_s[lane] = lane < it.q_count ? p.qrow[it.q_begin + lane] : -1; pcnt[lane] = 0; }
    for (int i = lane; i < TR * KS; i += 64) best[i] = KEY_MAX;
    __syncthreads();
    const bool carry = p.carry != 0 && it.part_row >= 0;
    if (carry) {   // the K best so far of every row, left by the launch over the previous panel
        for (int r = 0; r < it.q_count; ++r) {
            if (lane < K) {
                const int64_t o = (int64_t)(it.part_row + r) * K + lane;
                const int32_t idx = p.res_idx[o];
                if (idx >= 0) best[r * KS + lane] = ((uint64_t)p.res_bits[o] << 32) | (uint32_t)idx;
            }
        }
    }
    // A operand, resident in registers for the whole item: lane (c16, kq) holds chunks 4 sq + kq of
    // query row c16 (zeros for a row the tile does not have); the row's squared norm is summed over
    // the four lanes that share it
    uint4 areg[NS];
    {
        const int qr = c16 < it.q_count ? qrow_s[c16] : -1;
        const char *qp = (const char *)p.qsrc + (int64_t)(qr >= 0 ? qr : 0) * row_bytes;
        float acc = 0.f;
#pragma unroll
        for (int sq = 0; sq < NS; ++sq) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (qr >= 0) v = *(const uint4 *)(qp + (4 * sq + kq) * kChunkBytes);
            areg[sq] = v;
            const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
#pragma unroll
            for (int i = 0; i < 4; ++i) acc += f[i] * f[i];
        }
        acc += __shfl_xor(acc, 16);
        acc += __shfl_xor(acc, 32);
        if (kq == 0) qnorm_s[c16] = __float_as_uint(acc);
    }
    __syncthreads();

    // this lane's four rows: 4 kq + i
    float qn[4];
    uint32_t thr[4];
    uint32_t live = 0, and_rows = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 4 * kq + i;
        qn[i] = __uint_as_float(qnorm_s[row]);
        thr[i] = 0xFFFFFFFFu;
        if (row < it.q_count) {
            live |= 1u << i;
            if (AND) {
                const int qr = qrow_s[row];
                if (p.others_off[qr + 1] > p.others_off[qr]) and_rows |= 1u << i;
            }
        }
    }
    int pcv = 0;                  // state of tile row r, held by lane r
    uint64_t row_kth = KEY_MAX;
    if (carry) {
        if (lane < it.q_count) row_kth = best[lane * KS + K - 1];
        const uint32_t t = (uint32_t)(row_kth >> 32);
#pragma unroll
        for (int i = 0; i < 4; ++i) thr[i] = __shfl(t, 4 * kq + i);
    }

    auto drain = [&]() {
        wave_lds_sync();
        if (K <= 16) wave_drain_rows_packed<16>(pend, PC, best, KS, K, pcv, row_kth, lane);
        if (K <= 32) wave_drain_rows_packed<32>(pend, PC, best, KS, K, pcv, row_kth, lane);
        wave_drain_rows<4>(pend, PC, best, KS, K, pcv, row_kth, lane);
        if (lane < 32) pcnt[lane] = 0;
        wave_lds_sync();
        const uint32_t t = (uint32_t)(row_kth >> 32);
#pragma unroll
        for (int i = 0; i < 4; ++i) thr[i] = __shfl(t, 4 * kq + i);
    };

    const int n_groups = (it.n + kGroup - 1) / kGroup;
    // segment-relative index of the entry that equals this lane's row 4 kq (graph build), else never matched
    const int self0 = it.self_base >= 0 ? it.self_base + 4 * kq - it.entry0 : -0x40000000;
    // B registers: two groups (slots 0 and 1, even and odd groups), each of two column blocks.  A slot is
    // refilled with the chunks of the group after next right after its own MFMAs have been issued, so a
    // wave keeps up to two groups (32 KiB at dim 128) of list in flight (kNN self-joins of the index
    // build: 12 % faster than with one group of distance; search tiles: unchanged).
    // Nothing else is prefetched: a scalar carried from one step to the next gets copied at the top of the
    // loop, and that copy would wait for every load issued before it.  The entries' norms are summed from
    // the B registers (in the shadow of the MFMAs) and the AND predicate fetches global ids on demand.
    uint4 breg[SLOTS][2][NS];
    auto fetch_block = [&](int slot, int g, int cb) {   // group g (exists), column block cb -> slot
        const uint4 *blk = p.xblk + (it.group0 + g) * (int64_t)(NCH * 32);
#pragma unroll
        for (int sq = 0; sq < NS; ++sq) breg[slot][cb][sq] = blk[(4 * sq + kq) * 32 + cb * 16 + c16];
    };
    // Every fetch is unconditional (past the end the last group is fetched again, from L2): with a fetch
    // under a condition the compiler cannot tell which loads are outstanding where the paths meet, and
    // its waits then cover all of them, the block just requested included.
    const int last_group = n_groups - 1;
#pragma unroll
    for (int slot = 0; slot < SLOTS; ++slot) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) fetch_block(slot, slot < last_group ? slot : last_group, cb);
        __builtin_amdgcn_sched_barrier(0);   // the loads stay in this order, here and in the loop
    }
    for (int grp0 = 0; grp0 < n_groups; grp0 += SLOTS) {
#pragma unroll
      for (int slot = 0; slot < SLOTS; ++slot) {
        // (an odd number of groups ends with a phantom step on the re-fetched last group, every column
        // masked: a way out between the two steps would be one more path into the loop's end, one on
        // which slot 0 holds the newest loads, and the waits at the top would cover slot 1's as well)
        const int grp = grp0 + slot;
        const int refill = grp + SLOTS < last_group ? grp + SLOTS : last_group;
        v4f acc[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) acc[cb] = (v4f){0.f, 0.f, 0.f, 0.f};
        // the two column blocks are two independent accumulation chains: issued alternately they keep the
        // matrix core busy (one chain alone issues every 52 cycles, two every 32)
#pragma unroll
        for (int sq = 0; sq < NS; ++sq) {
            const uint4 a = areg[sq], b0 = breg[slot][0][sq], b1 = breg[slot][1][sq];
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b0.x), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b1.x), acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b0.y), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b1.y), acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b0.z), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b1.z), acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b0.w), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b1.w), acc[1], 0, 0, 0);
        }
        // |x|^2 of this lane's two entries: its own chunks, then the four lanes that share an entry
        float xn[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int sq = 0; sq < NS; ++sq) {
                const uint4 b = breg[slot][cb][sq];
                const float f[4] = {__uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w)};
                s0 += f[0] * f[0]; s1 += f[1] * f[1]; s0 += f[2] * f[2]; s1 += f[3] * f[3];
            }
            float t = s0 + s1;
            t += __shfl_xor(t, 16);
            t += __shfl_xor(t, 32);
            xn[cb] = t;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) fetch_block(slot, refill, cb);
        __builtin_amdgcn_sched_barrier(0);

        // phase 1 (branch-free): distances and threshold tests of this lane's 4 rows x 2 entries
        uint32_t bitsv[8];
        uint32_t pm = 0;   // bit cb * 4 + i
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const uint32_t col_ok = grp * kGroup + cb * 16 + c16 < it.n ? live : 0u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float d = (qn[i] + xn[cb]) - 2.0f * acc[cb][i];
                bitsv[cb * 4 + i] = __float_as_uint(fmaxf(d, 0.0f));
                const uint32_t below = bitsv[cb * 4 + i] <= thr[i] ? 1u : 0u;
                // graph build: the list entry that is the query row itself is skipped
                const uint32_t not_self = grp * kGroup + cb * 16 + c16 != self0 + i ? 1u : 0u;
                pm |= (below & not_self & (col_ok >> i) & 1u) << (cb * 4 + i);
            }
        }
        if (AND && pm != 0) {
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                if (((pm >> b) & 1u) && ((and_rows >> (b & 3)) & 1u)) {
                    const int qr = qrow_s[4 * kq + (b & 3)];
                    const int o_begin = p.others_off[qr], o_end = p.others_off[qr + 1];
                    bool ok = true;
                    const int32_t gid = p.map[it.map_off + it.entry0 + grp * kGroup + (b >> 2) * 16 + c16];
                    for (int o = o_begin; o < o_end && ok; ++o) ok = has_label(p.meta, p.others[o], gid);
                    if (!ok) pm &= ~(1u << b);
                }
            }
        }
        // phase 2: queue the candidates (slot from the row's LDS counter)
        if (pm != 0) {
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                if ((pm >> b) & 1u) {
                    const int row = 4 * kq + (b & 3);
                    const int entry = it.entry0 + grp * kGroup + (b >> 2) * 16 + c16;
                    const uint32_t slot = atomicAdd(&pcnt[row], 1u);
                    pend[row * PC + slot] = ((uint64_t)bitsv[b] << 32) | (uint32_t)entry;
                }
            }
        }
        if (__any(pm != 0)) {
            wave_lds_sync();
            pcv = lane < 32 ? (int)pcnt[lane] : 0;
        }
        if (__any(pcv >= PC - 32) || (grp + 1 == n_groups && __any(pcv != 0))) drain();
      }
    }
    __syncthreads();

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

// float32 lists with few queries per tile.  The fp32 matrix core runs at only twice the VALU
// FMA rate and a 32-row tile with a handful of queries wastes most of it, so below ~16 queries
// per tile plain FMAs are faster: a lane holds one list entry's whole vector in registers (two
// 32-vector groups per step), the tile's queries are walked one after the other, and a query
// row -- the same for all lanes -- comes in through scalar loads and feeds the FMAs as a scalar
// operand.  Distances are |q|^2 + |x|^2 - 2 q.x as in the MFMA kernel; selection uses the same
// per-row queues and merge.  Lane r (r < 32) holds the state of tile row r.
template <int NCH>
__global__ __launch_bounds__(64) void scan_valu_kernel(ScanParams p)
{
    extern __shared__ uint4 smem[];
    const ScanItem it = p.items[blockIdx.x];
    const int lane = threadIdx.x, n32 = lane & 31, h = lane >> 5;
    const int K = p.K, KS = K | 1, TR = p.tile_rows;
    constexpr int PC = 96;   // a step adds <= 64 keys to a row and rows above 32 are drained after every step
    constexpr int row_bytes = NCH * kChunkBytes;
    uint64_t *pend = (uint64_t *)smem;                  // [TR][PC]
    uint64_t *best = pend + TR * PC;                    // [TR][KS]
    int32_t *qrow_s = (int32_t *)(best + TR * KS);      // [32]
    float *qnorm_s = (float *)(qrow_s + 32);            // [32]

    if (lane < 32) qrow_s[lane] = lane < it.q_count ? p.qrow[it.q_begin + lane] : -1;
    for (int i = lane; i < TR * KS; i += 64) best[i] = KEY_MAX;
    __syncthreads();
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
    __syncthreads();

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
            typedef const float __attribute__((address_space(4))) *const_f32;
            const const_f32 qp = (const_f32)(uintptr_t)((const char *)p.qsrc + (int64_t)qr * row_bytes);
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
            for (int e = 0; e < NCH * 4; e += 4) {
                a0 = __builtin_fmaf(__uint_as_float(x[e]), qp[e], a0);
                a1 = __builtin_fmaf(__uint_as_float(x[e + 1]), qp[e + 1], a1);
                a2 = __builtin_fmaf(__uint_as_float(x[e + 2]), qp[e + 2], a2);
                a3 = __builtin_fmaf(__uint_as_float(x[e + 3]), qp[e + 3], a3);
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
    __syncthreads();

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

// Final top-K of a query whose list was scanned in several segments: sort the
// segments' candidates by (distance, entry) and keep the first K.  One wave per query.
template <int DT>
__global__ __launch_bounds__(64) void scan_merge_kernel(const MergeItem *items, const int32_t *res_idx,
                                                        const uint32_t *res_bits, int32_t K, int32_t P,
                                                        const int32_t *map, int64_t *out_ids, float *out_dists)
{
    extern __shared__ uint4 smem[];
    uint64_t *keys = (uint64_t *)smem;  // [P], P a power of two >= nseg * K
    const MergeItem it = items[blockIdx.x];
    const int lane = threadIdx.x;
    const int total = it.nseg * K;
    for (int i = lane; i < P; i += 64) {
        uint64_t key = KEY_MAX;
        if (i < total) {
            const int64_t o = (int64_t)(it.part_row + (i / K) * it.stride) * K + (i % K);
            const int32_t idx = res_idx[o];
            if (idx >= 0) key = ((uint64_t)res_bits[o] << 32) | (uint32_t)idx;
        }
        keys[i] = key;
    }
    __syncthreads();
    wave_bitonic_sort(keys, P, lane);
    if (lane < K) {
        const uint64_t key = keys[lane];
        const bool none = key == KEY_MAX;
        const uint32_t hi = (uint32_t)(key >> 32);
        const int64_t o = (int64_t)it.qrow * K + lane;
        out_ids[o] = none ? -1 : (int64_t)map[it.map_off + (uint32_t)key];
        out_dists[o] = none ? __builtin_inff() : (DT == 0 ? (float)(int)hi : __uint_as_float(hi));
    }
}

// LDS of the 32-row form: the query tile (chunk-major), per row a 64-slot queue and the sorted best list
size_t scan_lds_bytes(int32_t ncp, int32_t tile_rows, int32_t K)
{
    return (size_t)2 * ncp * tile_rows * 16 + (size_t)tile_rows * (64 + (K | 1)) * 8 + 3 * 32 * 4;
}

template <int DT> static void launch_scan_dt(const ScanParams &p, int n_items, hipStream_t s)
{
    const size_t lds = scan_lds_bytes(p.ncp, p.tile_rows, p.K);
    const dim3 grid(n_items), block(64);
    if (DT == 0) {
        switch (p.ncp) {
        case 4: hipLaunchKernelGGL((scan_topk_kernel<DT, 4>), grid, block, lds, s, p); break;   // uint8 dim 128
        case 6: hipLaunchKernelGGL((scan_topk_kernel<DT, 6>), grid, block, lds, s, p); break;   // uint8 dim 192
        default: hipLaunchKernelGGL((scan_topk_kernel<DT, 0>), grid, block, lds, s, p); break;
        }
    } else {
        switch (p.ncp) {
        case 12: hipLaunchKernelGGL((scan_topk_kernel<DT, 12>), grid, block, lds, s, p); break; // float dim 96
        case 16: hipLaunchKernelGGL((scan_topk_kernel<DT, 16>), grid, block, lds, s, p); break; // float dim 128
        default: hipLaunchKernelGGL((scan_topk_kernel<DT, 0>), grid, block, lds, s, p); break;
        }
    }
}

bool scan16_supported(int dtype, int dim, int tile_rows)
{
    return dtype == 1 && (dim == 128 || dim == 96) && tile_rows <= 16;
}

// float32 tiles of <= 16 queries: see scan_topk16_kernel
void launch_scan16(const ScanParams &p, int n_items, hipStream_t s)
{
    if (n_items <= 0) return;
    const size_t lds = (size_t)p.tile_rows * (64 + (p.K | 1)) * 8 + 3 * 32 * 4;   // no query tile: it lives in registers
    // Instantiations.  AND: with loads of the AND predicate inside the loop the compiler can no longer count
    // which outstanding loads a wait must cover, and every wait becomes a wait for all of them.  SLOTS: the
    // kNN self-joins of the index build (alone on the chip) prefetch two groups ahead; search
    // tiles one group, with 70 registers less per wave, which leaves room for the waves of the graph kernels
    // that run beside them.
    const bool with_and = p.others_off != nullptr;
    const bool deep = p.K > 16;   // the self-joins keep 48 or 64 candidates per row, searches k
    const dim3 grid(n_items), block(64);
#define VF_LAUNCH16(NCP_) \
    do { \
        if (deep) { \
            if (with_and) hipLaunchKernelGGL((scan_topk16_kernel<NCP_, true, 2>), grid, block, lds, s, p); \
            else hipLaunchKernelGGL((scan_topk16_kernel<NCP_, false, 2>), grid, block, lds, s, p); \
        } else { \
            if (with_and) hipLaunchKernelGGL((scan_topk16_kernel<NCP_, true, 1>), grid, block, lds, s, p); \
            else hipLaunchKernelGGL((scan_topk16_kernel<NCP_, false, 1>), grid, block, lds, s, p); \
        } \
    } while (0)
    if (p.dim == 128) VF_LAUNCH16(16);
    else VF_LAUNCH16(12);
#undef VF_LAUNCH16
}

bool scan_valu_supported(int dtype, int dim, int tile_rows)
{
    return dtype == 1 && (dim == 128 || dim == 96) && tile_rows <= 16;
}

// float32 search tiles (no self exclusion): see scan_valu_kernel
void launch_scan_valu(const ScanParams &p, int n_items, hipStream_t s)
{
    if (n_items <= 0) return;
    const size_t lds = (size_t)p.tile_rows * (96 + (p.K | 1)) * 8 + 2 * 32 * 4;
    if (p.dim == 128) hipLaunchKernelGGL((scan_valu_kernel<32>), dim3(n_items), dim3(64), lds, s, p);
    else hipLaunchKernelGGL((scan_valu_kernel<24>), dim3(n_items), dim3(64), lds, s, p);
}

void launch_scan_merge(int dtype, const MergeItem *items, int n_items, const int32_t *res_idx, const uint32_t *res_bits,
                       int32_t K, int32_t max_keys, const int32_t *map, int64_t *out_ids, float *out_dists, hipStream_t s)
{
    if (n_items <= 0) return;
    int32_t P = 64;
    while (P < max_keys) P <<= 1;
    if (dtype == 0)
        hipLaunchKernelGGL(scan_merge_kernel<0>, dim3(n_items), dim3(64), (size_t)P * 8, s, items, res_idx, res_bits, K, P,
                           map, out_ids, out_dists);
    else
        hipLaunchKernelGGL(scan_merge_kernel<1>, dim3(n_items), dim3(64), (size_t)P * 8, s, items, res_idx, res_bits, K, P,
                           map, out_ids, out_dists);
}

void launch_scan(int dtype, const ScanParams &p, int n_items, hipStream_t s)
{
    if (n_items <= 0) return;
    if (dtype == 0) launch_scan_dt<0>(p, n_items, s);
    else launch_scan_dt<1>(p, n_items, s);
}

}  // namespace vf
