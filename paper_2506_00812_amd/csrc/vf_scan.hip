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

#include "vf_scan_item.h"

namespace vf {

constexpr int kScanWaves = 2;     // waves per SIMD the 32-row kernel is compiled for
constexpr int kScan16Waves = 2;   // and the 16-row kernel

// NCP > 0: the number of chunk pairs per vector is known at compile time; the B
// operand of the NEXT group (NCP 1-KiB loads) is then fetched into registers while
// the MFMAs of the current group run, which is what keeps HBM busy at the skinny
// shapes of the search (a handful of queries per list).  NCP == 0: any p.ncp, no
// prefetch.
template <int DT, int NCP>
__global__ __launch_bounds__(64, kScanWaves) void scan_topk_kernel(ScanParams p)
{
    extern __shared__ uint4 smem[];
    const ScanItem it = p.items[blockIdx.x];
    scan_topk_item<DT, NCP>(p, it, smem);
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
__global__ __launch_bounds__(64, kScan16Waves) void scan_topk16_kernel(ScanParams p)
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
    scan_valu_item<NCH>(p, it, smem);
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
