// Graph-search initialisation (Section 4.2.1: the initial candidates are sampled
// inside the label's list): distances from every graph query to the seeds of its
// label, computed densely.
//
// The seeds of a label -- local ids floor(j * n / ns) -- do not depend on the query,
// so all queries of a label score the same vectors: a dense queries x seeds block per label
// instead of every query gathering its seeds from HBM.  Three kernels fill that block:
//
//   seed_mfma_kernel    the default wherever it has an instantiation.  The block is a contraction,
//                       |q|^2 + |x|^2 - 2 q.x on the matrix cores: exact for uint8, an approximation
//                       for float32 that the beam kernel re-ranks under a proof (see below).
//   seed_select_kernel  the same scoring with the selection fused in: per (query, seed segment) only a
//                       run of the K smallest keys leaves the kernel (off by default: slower than the
//                       unfused pair except on long uint8 seed lists).
//   seed_dist_kernel    the ordered distance itself on the vector ALU, for dimensions and list sizes the
//                       matrix-core kernels do not cover and as the reference route of the tests: one wave
//                       takes up to 64 queries of one label (one query per lane, the query vector held in
//                       registers) and a chunk of kSeedChunk seeds; a seed vector is the same for all lanes,
//                       so it is fetched with scalar loads and used as a scalar operand -- no LDS or
//                       cross-lane traffic in the inner loop.  A lane evaluates the distance in exactly the
//                       order the 8-lane teams of the beam kernel use (partial sum t takes the 16-byte
//                       chunks 8s + t, fused multiply-add, fixed tree), so the bits are identical to a
//                       gathered evaluation and to the CPU evaluation.
//
// Output of the unfused kernels: dseed[gq][j] = distance bits of graph query gq to seed j, consumed by the
// beam kernel, which keeps the best itopk.
#include "vf_select.h"

namespace vf {

template <int DT, int NCH>
__global__ __launch_bounds__(64) void seed_dist_kernel(SeedParams p)
{
    constexpr int SC = kSeedChunk;
    __shared__ uint32_t outb[64 * (SC + 1)];
    const int lane = threadIdx.x;
    const int tile = blockIdx.x / p.max_chunks, chunk = blockIdx.x % p.max_chunks;
    const SeedTile t = p.tiles[tile];
    const int n = p.meta.S[t.label];
    const int64_t base = p.meta.O_HS[t.label];
    const int ns = p.n_seeds < n ? p.n_seeds : n;
    const int j0 = chunk * SC;
    if (j0 >= ns) return;
    const int cnt = ns - j0 < SC ? ns - j0 : SC;
    constexpr int row_bytes = NCH * kChunkBytes;

    // seeds of this chunk -> global ids (lane i holds seed j0 + i)
    int g = 0;
    if (lane < cnt) g = p.meta.M_HS[base + (int64_t)(((uint64_t)(j0 + lane) * (uint64_t)n) / (uint64_t)ns)];

    // this lane's query
    uint32_t q[NCH * 4];
    {
        const int qi = p.gq_query[t.gq_begin + (lane < t.q_count ? lane : 0)];
        const uint4 *qrow = (const uint4 *)((const char *)p.Q + (int64_t)qi * row_bytes);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const uint4 v = qrow[ch];
            q[ch * 4] = v.x; q[ch * 4 + 1] = v.y; q[ch * 4 + 2] = v.z; q[ch * 4 + 3] = v.w;
        }
    }
    uint32_t qq = 0;
    if (DT == 0) {
#pragma unroll
        for (int w = 0; w < NCH * 4; ++w) qq = __builtin_amdgcn_udot4(q[w], q[w], qq, false);
    }

    for (int i = 0; i < cnt; ++i) {
        // the seed vector is wave uniform: it comes in through scalar loads and feeds the VALU
        // as a scalar operand -- no LDS staging, no cross-lane traffic
        const int gi = __builtin_amdgcn_readlane(g, i);
        const uint32_t *__restrict__ xp = (const uint32_t *)((const char *)p.X + (int64_t)gi * row_bytes);
        uint32_t bits;
        if (DT == 0) {
            uint32_t xx = 0, qx = 0;
#pragma unroll
            for (int w = 0; w < NCH * 4; ++w) {
                const uint32_t x = xp[w];
                xx = __builtin_amdgcn_udot4(x, x, xx, false);
                qx = __builtin_amdgcn_udot4(q[w], x, qx, false);
            }
            bits = (uint32_t)((int)qq + (int)xx - 2 * (int)qx);
        } else {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = 0.0f;
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float d = __uint_as_float(q[ch * 4 + c]) - __uint_as_float(xp[ch * 4 + c]);
                    a[ch & 7] = __builtin_fmaf(d, d, a[ch & 7]);
                }
            }
            const float b0 = a[0] + a[1], b1 = a[2] + a[3], b2 = a[4] + a[5], b3 = a[6] + a[7];
            const float c0 = b0 + b1, c1 = b2 + b3;
            bits = __float_as_uint(c0 + c1);
        }
        outb[lane * (SC + 1) + i] = bits;
    }
    __syncthreads();

    // rows of dseed: SC consecutive seeds per query
    for (int r0 = 0; r0 < t.q_count; r0 += 64 / SC) {
        const int r = r0 + lane / SC, col = lane % SC;
        if (r < t.q_count && col < cnt)
            p.dseed[(int64_t)(t.gq_begin + r) * p.ns_stride + j0 + col] = outb[r * (SC + 1) + col];
    }
}

// ---------------------------------------------------------------------------------------------
// float32, matrix cores.  queries x seeds of one label is a dense contraction, so the bulk of the
// work can run on MFMA as |q|^2 + |x|^2 - 2 q.x.  That value is rounded differently from the
// ordered distance the search is defined with, so it is used as a filter only: the beam kernel
// keeps the itopk + margin best approximations per query (at most 64), re-scores those with the
// ordered distance, and accepts the list only if its worst entry lies below the last kept approximation
// by more than the rounding-error bound (else it scores every seed itself).  One wave: a tile of <= 32 queries (A operand, staged in LDS) against kSeedMfmaChunk
// seeds in groups of 32 (B operand gathered row-wise from X: lane (v, h) reads the 16-byte
// chunks 2c + h of seed v, the operand layout of v_mfma_f32_32x32x2_f32).
// uint8 data go through the same kernel with v_mfma_i32_32x32x32_i8 on the vectors shifted by -128
// (the shift cancels in q - x): the int32 result is the exact distance, so nothing is approximate
// there and the rows of dseed are used as they are.
typedef float v16f_seed __attribute__((ext_vector_type(16)));
typedef int v16i_seed __attribute__((ext_vector_type(16)));
typedef int v4i_seed __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf_seed __attribute__((ext_vector_type(8)));

// CACHED: the B operand comes from the interleaved copy of the seeds (coalesced 1-KiB loads, lane (v, h)
// taking chunk 2 c + h of seed v of the group); otherwise every lane pair gathers its seed's row from X
// (32 rows of 32 bytes per load instruction).  NG = 32-seed groups per wave (fully unrolled: a loop with a
// run-time trip count needs both operand buffers live at once and spills): few long waves for large
// batches, many short ones for small batches.
// DT = 2: float32 data whose interleaved seed copy holds bfloat16 (16-byte chunks of 8 components, NCH of
// them per seed, CACHED only).  The queries are split into a bfloat16 high part and the bfloat16 rounding
// of the rest (|q - hi - lo| <= 2^-16 |q| per component), both multiplied with the seeds by
// v_mfma_f32_32x32x16_bf16 into one float32 accumulator: half the operand bytes and a quarter of the
// matrix-core time of the float32 form (two products per component at sixteen times the rate).  The norms stay those of the unrounded vectors, so the only new
// error is 2 q.(x - bf16(x)), which the beam kernel's bound carries as err_q * |q|.
template <int DT, int NCP, bool CACHED, int NG>
__global__ __launch_bounds__(64) void seed_mfma_kernel(SeedParams p)
{
    static_assert(DT != 2 || CACHED, "bfloat16 seeds exist only as the interleaved copy");
    constexpr int NCH = 2 * NCP, row_bytes = (DT == 2 ? 2 : 1) * NCH * kChunkBytes;   // row_bytes: of a query
    __shared__ uint4 qtile[(DT == 2 ? 2 : 1) * NCH * 32];   // DT 2: high parts, then low parts
    __shared__ uint32_t qnorm_s[32];   // float bits / int
    const int lane = threadIdx.x, n32 = lane & 31, h = lane >> 5;
    const int tile = blockIdx.x / p.max_chunks, chunk = blockIdx.x % p.max_chunks;
    const SeedTile t = p.tiles[tile];
    const int n = p.meta.S[t.label];
    const int64_t base = p.meta.O_HS[t.label];
    const int ns = p.n_seeds < n ? p.n_seeds : n;
    const int j0 = chunk * (NG * 32);
    if (j0 >= ns) return;

    constexpr bool cached = CACHED;
    const int64_t grp0 = cached ? p.seed_goff[p.meta.hs_slot[t.label]] + j0 / 32 : 0;
    // global ids and norms of this lane's seed in each group (issued first: the longest dependent chain)
    int gid[NG];
    uint32_t xn[NG];
    if (cached) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            gid[g] = 0;
            xn[g] = j0 + g * 32 < ns ? p.seed_norm[(grp0 + g) * 32 + n32] : 0u;
        }
    } else {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int j = j0 + g * 32 + n32;
            const int c = j < ns ? (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns) : 0;
            gid[g] = p.meta.M_HS[base + c];
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) xn[g] = p.xnorm_all[gid[g]];
    }

    // query tile, chunk-major; rows without a query are zero
    {
        const int qr = n32 < t.q_count ? p.gq_query[t.gq_begin + n32] : -1;
        const char *qp = (const char *)p.Q + (int64_t)(qr >= 0 ? qr : 0) * row_bytes;
        float facc = 0.f;
        int iacc = 0;
#pragma unroll
        for (int c0 = 0; c0 < NCP; ++c0) {
            const int c = 2 * c0 + h;
            if constexpr (DT == 2) {   // components 8 c .. 8 c + 7
                uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
                if (qr >= 0) {
                    v0 = *(const uint4 *)(qp + (2 * c) * kChunkBytes);
                    v1 = *(const uint4 *)(qp + (2 * c + 1) * kChunkBytes);
                }
                const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                uint32_t hi[8], lo[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float f = __uint_as_float(w[i]);
                    facc += f * f;
                    hi[i] = bf16_rn_bits(f);
                    lo[i] = bf16_rn_bits(f - __uint_as_float(hi[i] << 16));
                }
                qtile[c * 32 + n32] = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
                qtile[NCH * 32 + c * 32 + n32] =
                    make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
                continue;
            }
            uint4 v = make_uint4(0, 0, 0, 0);
            if (qr >= 0) {
                v = *(const uint4 *)(qp + c * kChunkBytes);
                if (DT == 0) { v.x ^= 0x80808080u; v.y ^= 0x80808080u; v.z ^= 0x80808080u; v.w ^= 0x80808080u; }
            }
            qtile[c * 32 + n32] = v;
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (DT == 0) {
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) {
                        const int e = (int)(int8_t)(w[i] >> (8 * bb));
                        iacc += e * e;
                    }
                } else {
                    facc += __uint_as_float(w[i]) * __uint_as_float(w[i]);
                }
            }
        }
        if (DT == 0) {
            iacc += __shfl_xor(iacc, 32);
            if (h == 0) qnorm_s[n32] = (uint32_t)iacc;
        } else {
            facc += __shfl_xor(facc, 32);
            if (h == 0) qnorm_s[n32] = __float_as_uint(facc);
        }
    }
    __syncthreads();
    uint32_t qn[16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) qn[jj] = qnorm_s[8 * (jj >> 2) + 4 * h + (jj & 3)];

    uint4 bnext[NCP];
    auto fetch_group = [&](int g) {   // group g of this wave's seeds (exists)
        if (cached) {
            const uint4 *blk = p.seed_blk + (grp0 + g) * (int64_t)(NCH * 32);
#pragma unroll
            for (int cp = 0; cp < NCP; ++cp) bnext[cp] = blk[(2 * cp + h) * 32 + n32];
        } else {
            const char *xrow = (const char *)p.X + (int64_t)gid[g] * row_bytes;
#pragma unroll
            for (int cp = 0; cp < NCP; ++cp) bnext[cp] = *(const uint4 *)(xrow + (2 * cp + h) * kChunkBytes);
        }
    };
    fetch_group(0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        if (j0 + g * 32 >= ns) break;   // wave uniform
        uint4 b[NCP];
#pragma unroll
        for (int cp = 0; cp < NCP; ++cp) b[cp] = bnext[cp];
        if (g + 1 < NG && j0 + (g + 1) * 32 < ns) fetch_group(g + 1 < NG ? g + 1 : g);
        uint32_t bits[16];
        if constexpr (DT == 0) {
            v16i_seed acc;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = 0;
#pragma unroll
            for (int cp = 0; cp < NCP; ++cp) {
                const uint4 a = qtile[(2 * cp + h) * 32 + n32];
                uint4 bb = b[cp];
                bb.x ^= 0x80808080u; bb.y ^= 0x80808080u; bb.z ^= 0x80808080u; bb.w ^= 0x80808080u;
                const v4i_seed av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w};
                const v4i_seed bv = {(int)bb.x, (int)bb.y, (int)bb.z, (int)bb.w};
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, acc, 0, 0, 0);
            }
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) bits[jj] = (uint32_t)((int)qn[jj] + (int)xn[g] - 2 * acc[jj]);
        } else if constexpr (DT == 2) {
            v16f_seed acc;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = 0.f;
#pragma unroll
            for (int cp = 0; cp < NCP; ++cp) {
                const v8bf_seed bv = __builtin_bit_cast(v8bf_seed, b[cp]);
                const uint4 ah = qtile[(2 * cp + h) * 32 + n32], al = qtile[NCH * 32 + (2 * cp + h) * 32 + n32];
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_seed, ah), bv, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_seed, al), bv, acc, 0, 0, 0);
            }
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float d = (__uint_as_float(qn[jj]) + __uint_as_float(xn[g])) - 2.0f * acc[jj];
                bits[jj] = __float_as_uint(fmaxf(d, 0.0f));
            }
        } else {
            v16f_seed acc;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = 0.f;
#pragma unroll
            for (int cp = 0; cp < NCP; ++cp) {
                const uint4 a = qtile[(2 * cp + h) * 32 + n32];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b[cp].x), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b[cp].y), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b[cp].z), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b[cp].w), acc, 0, 0, 0);
            }
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float d = (__uint_as_float(qn[jj]) + __uint_as_float(xn[g])) - 2.0f * acc[jj];
                bits[jj] = __float_as_uint(fmaxf(d, 0.0f));
            }
        }
        // Every lane stores every value, those without a (query, seed) pair into a dump area behind the
        // matrix: with the stores under conditions the compiler cannot count them, and its wait for the next
        // group's operand loads becomes a wait for these stores to be acknowledged as well.  The dump area has
        // a slot per workgroup index (mod 1024): one shared slot is a single hot cache line when many tiles
        // are partly filled.
        const int j = j0 + g * 32 + n32;
        uint32_t *dump = p.dseed + p.dump_off + (((int64_t)(blockIdx.x & (unsigned)p.dump_mask)) << 6) + lane;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int row = 8 * (jj >> 2) + 4 * h + (jj & 3);
            const bool ok = j < ns && row < t.q_count;
            uint32_t *dst = ok ? p.dseed + (int64_t)(t.gq_begin + row) * p.ns_stride + j : dump;
            *dst = bits[jj];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Seed scoring with the selection fused in.  The beam search starts from the best `itopk` of a query's
// seeds, a few dozen out of thousands, so nothing but those needs to leave the kernel that scores them.
// One wave takes a tile of <= 32 same-label queries and a SEGMENT of the label's seeds (seg_seeds of them,
// whole 32-seed groups of the interleaved copy), contracts them on the matrix cores group by group like
// seed_mfma_kernel, and keeps per query row the K smallest (value, seed index) pairs with the queue-and-merge
// selection of the scan kernels: a row's threshold tightens as the segment streams by, so after the first
// groups only a few values per group reach a queue.  Output: one sorted run of K keys
// (value bits << 32 | seed index) per (query, segment); the beam kernel merges a query's runs.
// Why that is enough.  uint8 values are the exact distances, and the order of keys is the order of
// (distance, local id) since the local id floor(j n / ns) grows with j: the K best of the union of the runs are
// the K best seeds.  float32 values are approximations: the beam kernel keeps the K best of the union, re-scores
// them with the ordered distance and needs a lower bound T on the approximation of every seed it did NOT keep.
// A seed missing from the union was rejected in its segment by K values that all are in the union, so its
// approximation is at least the union's K-th smallest value, which is T as before.
// A operand (queries) in registers for the whole segment; LDS holds only the queues and the lists.
// DT = 0: uint8 data (v_mfma_i32_32x32x32_i8 on the -128 shifted bytes).  DT = 2: float32 data, seeds from the
// bfloat16 copy, queries split into a bfloat16 high and low part (see seed_mfma_kernel).
template <int DT, int NCP>
__global__ __launch_bounds__(64, 2) void seed_select_kernel(SeedSelParams p)
{
    static_assert(DT == 0 || DT == 2, "uint8, or float32 data with a bfloat16 seed copy");
    extern __shared__ uint4 smem[];
    constexpr int NCH = 2 * NCP, PC = 64;
    constexpr int row_bytes = (DT == 2 ? 2 : 1) * NCH * kChunkBytes;   // of a query
    const int K = p.K, KS = K | 1;
    uint64_t *pend = (uint64_t *)smem;               // [32][PC] candidates not yet merged
    uint64_t *best = pend + 32 * PC;                 // [32][KS] K best so far, ascending, KEY_MAX padded
    uint32_t *qnorm_s = (uint32_t *)(best + 32 * KS); // [32] float bits / int
    uint32_t *pcnt = qnorm_s + 32;                   // [32] keys waiting in pend[r]
    int32_t *qrow_s = (int32_t *)(pcnt + 32);        // [32] query index of the row, -1: none
    int32_t *pslot_s = qrow_s + 32;                  // [32] bitset row of the row's AND partner, see below

    const int lane = threadIdx.x, n32 = lane & 31, h = lane >> 5;
    const int tile = blockIdx.x / p.max_segs, seg = blockIdx.x % p.max_segs;
    const SeedTile t = p.tiles[tile];
    const int n = p.meta.S[t.label];
    const int ns = p.n_seeds < n ? p.n_seeds : n;
    const int j0 = seg * p.seg_seeds;
    if (j0 >= ns) return;   // the label has fewer segments than the grid allows for (the whole workgroup leaves)
    const int nj = ns - j0 < p.seg_seeds ? ns - j0 : p.seg_seeds;
    const int n_groups = (nj + 31) >> 5;
    const int64_t grp0 = p.seed_goff[p.meta.hs_slot[t.label]] + (j0 >> 5);

    if (lane < 32) {
        const int qr = lane < t.q_count ? p.gq_query[t.gq_begin + lane] : -1;
        qrow_s[lane] = qr;
        pcnt[lane] = 0;
        // the common AND query has one partner label, a graph label: its predicate is one bit of that label's
        // bitset, which can be fetched for all of a lane's rows at once (pslot_s >= 0); other rows evaluate the
        // general predicate pair by pair
        int ps = -1;
        if (qr >= 0 && p.others_off != nullptr && p.others_off[qr + 1] - p.others_off[qr] == 1)
            ps = p.meta.hs_slot[p.others[p.others_off[qr]]];
        pslot_s[lane] = ps;
    }
    for (int i = lane; i < 32 * KS; i += 64) best[i] = KEY_MAX;
    __syncthreads();

    // ---- A operand: lane (n32, h) holds chunks 2 cp + h of query row n32 (zeros for a row without a query)
    uint4 areg[NCP], alo[DT == 2 ? NCP : 1];
    {
        const int qr = qrow_s[n32];
        const char *qp = (const char *)p.Q + (int64_t)(qr >= 0 ? qr : 0) * row_bytes;
        float facc = 0.f;
        int iacc = 0;
#pragma unroll
        for (int cp = 0; cp < NCP; ++cp) {
            const int c = 2 * cp + h;
            if constexpr (DT == 2) {   // components 8 c .. 8 c + 7
                uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
                if (qr >= 0) {
                    v0 = *(const uint4 *)(qp + (2 * c) * kChunkBytes);
                    v1 = *(const uint4 *)(qp + (2 * c + 1) * kChunkBytes);
                }
                const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                uint32_t hi[8], lo[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float f = __uint_as_float(w[i]);
                    facc += f * f;
                    hi[i] = bf16_rn_bits(f);
                    lo[i] = bf16_rn_bits(f - __uint_as_float(hi[i] << 16));
                }
                areg[cp] = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
                alo[cp] = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
            } else {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (qr >= 0) {
                    v = *(const uint4 *)(qp + c * kChunkBytes);
                    v.x ^= 0x80808080u; v.y ^= 0x80808080u; v.z ^= 0x80808080u; v.w ^= 0x80808080u;
                }
                areg[cp] = v;
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) {
                        const int e = (int)(int8_t)(w[i] >> (8 * bb));
                        iacc += e * e;
                    }
            }
        }
        if (DT == 0) {
            iacc += __shfl_xor(iacc, 32);
            if (h == 0) qnorm_s[n32] = (uint32_t)iacc;
        } else {
            facc += __shfl_xor(facc, 32);
            if (h == 0) qnorm_s[n32] = __float_as_uint(facc);
        }
    }
    __syncthreads();

    // per-lane constants for its 16 accumulator rows: row(j) = 8 * (j / 4) + 4 * h + (j % 4)
    uint32_t qn[16], thr[16];
    uint32_t live_rows = 0, and_rows = 0, fast_rows = 0;   // and_rows: general predicate; fast_rows: one bitset bit
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int row = 8 * (j >> 2) + 4 * h + (j & 3);
        qn[j] = qnorm_s[row];
        thr[j] = 0xFFFFFFFFu;
        if (row < t.q_count) {
            live_rows |= 1u << j;
            if (p.others_off != nullptr) {
                const int qr = qrow_s[row];
                if (pslot_s[row] >= 0) fast_rows |= 1u << j;
                else if (p.others_off[qr + 1] > p.others_off[qr]) and_rows |= 1u << j;
            }
        }
    }
    const bool any_and = __any((and_rows | fast_rows) != 0);
    int pcv = 0;                  // state of tile row r, held by lane r (r < 32)
    uint64_t row_kth = KEY_MAX;

    // Merge queues into lists: only the rows whose queue could overflow on the next group (more than PC - 32
    // keys), or every row with a key at the end of the segment.  A drain costs a sort and a merge per row
    // whatever the queue holds, so a row is left alone until its queue is worth it.
    auto drain = [&](bool all) {
        wave_lds_sync();
        const bool mine = lane < 32 && pcv > (all ? 0 : PC - 32);
        int pcv_sel = mine ? pcv : 0;
        if (K <= 32) wave_drain_rows_packed<32>(pend, PC, best, KS, K, pcv_sel, row_kth, lane);
        wave_drain_rows<4>(pend, PC, best, KS, K, pcv_sel, row_kth, lane);
        if (mine) { pcnt[lane] = 0; pcv = 0; }
        wave_lds_sync();
        const uint32_t tk = (uint32_t)(row_kth >> 32);
#pragma unroll
        for (int j = 0; j < 16; ++j) thr[j] = __shfl(tk, 8 * (j >> 2) + 4 * h + (j & 3));
    };

    // B operand: the whole group in registers, each half refilled with the next group's chunks right after its
    // own MFMAs have been issued
    constexpr int H0 = (NCP + 1) / 2;
    uint4 breg[NCP];
    {
        const uint4 *blk0 = p.seed_blk + grp0 * (int64_t)(NCH * 32);
#pragma unroll
        for (int cp = 0; cp < NCP; ++cp) breg[cp] = blk0[(2 * cp + h) * 32 + n32];
    }
    uint32_t xn_next = p.seed_norm[grp0 * 32 + n32];
    int32_t gid_next = -1;
    if (any_and) gid_next = p.seed_map[grp0 * 32 + n32];
    for (int grp = 0; grp < n_groups; ++grp) {
        const uint4 *nblk = p.seed_blk + (grp0 + grp + 1) * (int64_t)(NCH * 32);
        const bool more = grp + 1 < n_groups;
        const uint32_t xn = xn_next;
        const int32_t gid = gid_next;
        if (more) {
            xn_next = p.seed_norm[(grp0 + grp + 1) * 32 + n32];
            if (any_and) gid_next = p.seed_map[(grp0 + grp + 1) * 32 + n32];
        }
        uint32_t bitsv[16];
        if constexpr (DT == 0) {
            v16i_seed acc;
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[j] = 0;
            auto contract = [&](int cp) {
                uint4 b = breg[cp];
                b.x ^= 0x80808080u; b.y ^= 0x80808080u; b.z ^= 0x80808080u; b.w ^= 0x80808080u;
                const uint4 a = areg[cp];
                const v4i_seed av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w};
                const v4i_seed bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w};
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, acc, 0, 0, 0);
            };
#pragma unroll
            for (int cp = 0; cp < H0; ++cp) contract(cp);
            if (more) {
#pragma unroll
                for (int cp = 0; cp < H0; ++cp) breg[cp] = nblk[(2 * cp + h) * 32 + n32];
            }
#pragma unroll
            for (int cp = H0; cp < NCP; ++cp) contract(cp);
            if (more) {
#pragma unroll
                for (int cp = H0; cp < NCP; ++cp) breg[cp] = nblk[(2 * cp + h) * 32 + n32];
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) bitsv[j] = (uint32_t)((int)qn[j] + (int)xn - 2 * acc[j]);
        } else {
            v16f_seed acc;
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[j] = 0.f;
            auto contract = [&](int cp) {
                const v8bf_seed bv = __builtin_bit_cast(v8bf_seed, breg[cp]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_seed, areg[cp]), bv, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_seed, alo[cp]), bv, acc, 0, 0, 0);
            };
#pragma unroll
            for (int cp = 0; cp < H0; ++cp) contract(cp);
            if (more) {
#pragma unroll
                for (int cp = 0; cp < H0; ++cp) breg[cp] = nblk[(2 * cp + h) * 32 + n32];
            }
#pragma unroll
            for (int cp = H0; cp < NCP; ++cp) contract(cp);
            if (more) {
#pragma unroll
                for (int cp = H0; cp < NCP; ++cp) breg[cp] = nblk[(2 * cp + h) * 32 + n32];
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float d = (__uint_as_float(qn[j]) + __uint_as_float(xn)) - 2.0f * acc[j];
                bitsv[j] = __float_as_uint(fmaxf(d, 0.0f));
            }
        }
        // phase 1 (branch-free): threshold tests of this lane's 16 rows against its seed of the group
        const int jrel = grp * 32 + n32;
        uint32_t pm = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) pm |= (bitsv[j] <= thr[j] ? 1u : 0u) << j;
        pm &= jrel < nj ? live_rows : 0u;
        if (any_and && __any((pm & fast_rows) != 0)) {
            // one bitset word per candidate pair, all requested before the first is looked at (pairs that are
            // no candidates read the table's first word: one cached address for the whole wave)
            const uint32_t *bs = p.meta.bitsets;
            const int64_t wi = gid >> 5;
#pragma unroll
            for (int j0 = 0; j0 < 16; j0 += 8) {
                uint32_t wv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = j0 + u;
                    const bool c = ((pm & fast_rows) >> j) & 1u;
                    const int ps = pslot_s[8 * (j >> 2) + 4 * h + (j & 3)];
                    wv[u] = bs[c ? (int64_t)ps * p.meta.bitset_words + wi : 0];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = j0 + u;
                    if ((((pm & fast_rows) >> j) & 1u) && !((wv[u] >> (gid & 31)) & 1u)) pm &= ~(1u << j);
                }
            }
        }
        if (any_and && (pm & and_rows) != 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (((pm & and_rows) >> j) & 1u) {
                    const int qr = qrow_s[8 * (j >> 2) + 4 * h + (j & 3)];
                    const int o_begin = p.others_off[qr], o_end = p.others_off[qr + 1];
                    bool ok = true;
                    for (int o = o_begin; o < o_end && ok; ++o) ok = has_label(p.meta, p.others[o], gid);
                    if (!ok) pm &= ~(1u << j);
                }
            }
        }
        // phase 2: queue the candidates (slot from the row's LDS counter)
        if (pm != 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if ((pm >> j) & 1u) {
                    const int row = 8 * (j >> 2) + 4 * h + (j & 3);
                    const uint32_t slot = atomicAdd(&pcnt[row], 1u);
                    pend[row * PC + slot] = ((uint64_t)bitsv[j] << 32) | (uint32_t)(j0 + jrel);
                }
            }
        }
        if (__any(pm != 0)) {
            wave_lds_sync();
            pcv = lane < 32 ? (int)pcnt[lane] : 0;
        }
        const bool last = grp + 1 == n_groups;
        if (__any(pcv > PC - 32) || (last && __any(pcv != 0))) drain(last);
    }
    __syncthreads();

    // ---- one sorted run of K keys per (query, segment)
    for (int r = 0; r < t.q_count; ++r)
        if (lane < K) p.runs[((int64_t)(t.gq_begin + r) * p.max_segs + seg) * K + lane] = best[r * KS + lane];
}

bool seed_select_supported(int dtype, int dim, bool bf16_copy)
{
    return dtype == 0 ? (dim == 128 || dim == 192) : (bf16_copy && (dim == 96 || dim == 128));
}

size_t seed_select_lds_bytes(int32_t K) { return (size_t)32 * 64 * 8 + (size_t)32 * (K | 1) * 8 + 4 * 32 * 4; }

void launch_seed_select(int dtype, const SeedSelParams &p, int n_tiles, hipStream_t s)
{
    if (n_tiles <= 0) return;
    const dim3 grid((unsigned)n_tiles * (unsigned)p.max_segs), block(64);
    const size_t lds = seed_select_lds_bytes(p.K);
    if (dtype == 0 && p.dim == 128) hipLaunchKernelGGL((seed_select_kernel<0, 4>), grid, block, lds, s, p);
    else if (dtype == 0 && p.dim == 192) hipLaunchKernelGGL((seed_select_kernel<0, 6>), grid, block, lds, s, p);
    else if (dtype == 1 && p.dim == 128) hipLaunchKernelGGL((seed_select_kernel<2, 8>), grid, block, lds, s, p);
    else if (dtype == 1 && p.dim == 96) hipLaunchKernelGGL((seed_select_kernel<2, 6>), grid, block, lds, s, p);
}

// Profiling only: how many of a graph query's seeds pass its AND predicate (the "distances computed" figure the
// search is accounted with counts them; the selection kernel tests only the seeds that reach a queue).
__global__ __launch_bounds__(64) void seed_pass_count_kernel(const int32_t *gq_query, const int32_t *gq_label, LabelMeta meta,
                                                             int32_t n_seeds, const int32_t *others_off,
                                                             const int32_t *others, int32_t *pass_count)
{
    const int gq = blockIdx.x, lane = threadIdx.x;
    const int qi = gq_query[gq], label = gq_label[gq];
    const int n = meta.S[label];
    const int ns = n_seeds < n ? n_seeds : n;
    const int64_t base = meta.O_HS[label];
    const int o_begin = others_off[qi], o_end = others_off[qi + 1];
    int cnt = 0;
    for (int j = lane; j < ns; j += 64) {
        const int g = meta.M_HS[base + (int64_t)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns)];
        bool ok = true;
        for (int o = o_begin; o < o_end && ok; ++o) ok = has_label(meta, others[o], g);
        cnt += ok ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
    if (lane == 0) pass_count[gq] = cnt;
}

void launch_seed_pass_count(const int32_t *gq_query, const int32_t *gq_label, const LabelMeta &meta, int32_t n_seeds,
                            const int32_t *others_off, const int32_t *others, int32_t *pass_count, int n_gq, hipStream_t s)
{
    if (n_gq <= 0) return;
    hipLaunchKernelGGL(seed_pass_count_kernel, dim3(n_gq), dim3(64), 0, s, gq_query, gq_label, meta, n_seeds, others_off,
                       others, pass_count);
}

bool seed_mfma_supported(int dtype, int dim)
{
    return dtype == 1 ? (dim == 96 || dim == 128) : (dim == 128 || dim == 192);
}

void launch_seed_mfma(int dtype, const SeedParams &p, int n_tiles, hipStream_t s)
{
    if (n_tiles <= 0) return;
    const dim3 grid((unsigned)n_tiles * (unsigned)p.max_chunks), block(64);
    // separate instantiations for the two operand sources (one kernel holding both paths needs so many
    // registers that a SIMD takes a single wave of it) and for the seeds per wave (p.chunk_seeds: 128,
    // or 512 with the interleaved copy)
    const bool cached = p.seed_blk != nullptr;
    const bool wide = cached && p.chunk_seeds == 4 * kSeedMfmaChunk;
#define VF_LAUNCH_SEED(DT_, NCP_) \
    do { \
        if (wide) hipLaunchKernelGGL((seed_mfma_kernel<DT_, NCP_, true, 16>), grid, block, 0, s, p); \
        else if (cached) hipLaunchKernelGGL((seed_mfma_kernel<DT_, NCP_, true, 4>), grid, block, 0, s, p); \
        else hipLaunchKernelGGL((seed_mfma_kernel<DT_, NCP_, false, 4>), grid, block, 0, s, p); \
    } while (0)
    if (dtype == 1 && p.seed_bf16 && cached) {
        if (p.dim == 128) {
            if (wide) hipLaunchKernelGGL((seed_mfma_kernel<2, 8, true, 16>), grid, block, 0, s, p);
            else hipLaunchKernelGGL((seed_mfma_kernel<2, 8, true, 4>), grid, block, 0, s, p);
        } else if (p.dim == 96) {
            if (wide) hipLaunchKernelGGL((seed_mfma_kernel<2, 6, true, 16>), grid, block, 0, s, p);
            else hipLaunchKernelGGL((seed_mfma_kernel<2, 6, true, 4>), grid, block, 0, s, p);
        }
    } else if (dtype == 1 && p.dim == 128) VF_LAUNCH_SEED(1, 16);
    else if (dtype == 1 && p.dim == 96) VF_LAUNCH_SEED(1, 12);
    else if (dtype == 0 && p.dim == 128) VF_LAUNCH_SEED(0, 4);
    else if (dtype == 0 && p.dim == 192) VF_LAUNCH_SEED(0, 6);
#undef VF_LAUNCH_SEED
}

// The interleaved float32 copy of the seeds (groups of 32, 2 * nch16 chunks of 4 components) rounded to
// bfloat16 (nch16 chunks of 8 components); err2[group * 32 + v] = |x - bf16(x)|^2.  One thread per seed.
__global__ void seed_pack_bf16_kernel(const uint4 *blk32, int64_t n_vec, int32_t nch16, uint4 *blk16, float *err2)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_vec) return;
    const int64_t g = t >> 5;
    const int v = (int)(t & 31);
    float e2 = 0.f;
    for (int c = 0; c < nch16; ++c) {
        const uint4 a = blk32[(g * (2 * nch16) + 2 * c) * 32 + v], b = blk32[(g * (2 * nch16) + 2 * c + 1) * 32 + v];
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float f = __uint_as_float(w[i]);
            r[i] = bf16_rn_bits(f);
            const float d = f - __uint_as_float(r[i] << 16);
            e2 += d * d;
        }
        blk16[(g * nch16 + c) * 32 + v] = make_uint4(r[0] | (r[1] << 16), r[2] | (r[3] << 16), r[4] | (r[5] << 16), r[6] | (r[7] << 16));
    }
    err2[t] = e2;
}

void launch_seed_pack_bf16(const uint4 *blk32, int64_t n_groups, int32_t nch16, uint4 *blk16, float *err2, hipStream_t s)
{
    if (n_groups <= 0) return;
    hipLaunchKernelGGL(seed_pack_bf16_kernel, dim3((unsigned)((n_groups * 32 + 255) / 256)), dim3(256), 0, s, blk32,
                       n_groups * 32, nch16, blk16, err2);
}

__global__ void seed_map_kernel(const int32_t *M_HS, const int64_t *slot_base, const int32_t *slot_n, int32_t n_seeds,
                                const int32_t *grp_slot, const int32_t *grp_j0, int64_t n_groups, int32_t *seed_map)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_groups * 32) return;
    const int64_t g = t >> 5;
    const int slot = grp_slot[g];
    const int n = slot_n[slot];
    const int ns = n_seeds < n ? n_seeds : n;
    const int j = grp_j0[g] + (int)(t & 31);
    seed_map[t] = j < ns ? M_HS[slot_base[slot] + (int64_t)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns)] : 0;
}

void launch_seed_map(const int32_t *M_HS, const int64_t *slot_base, const int32_t *slot_n, int32_t n_seeds,
                     const int32_t *grp_slot, const int32_t *grp_j0, int64_t n_groups, int32_t *seed_map, hipStream_t s)
{
    if (n_groups <= 0) return;
    hipLaunchKernelGGL(seed_map_kernel, dim3((unsigned)((n_groups * 32 + 255) / 256)), dim3(256), 0, s, M_HS, slot_base,
                       slot_n, n_seeds, grp_slot, grp_j0, n_groups, seed_map);
}

// One thread per row, elements in ascending order.  float32: sum of squares (float bits);
// uint8: sum of (x - 128)^2 (int32).
template <int DT> __global__ void row_norm_kernel(const void *X, int32_t dim, int64_t n, uint32_t *out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (DT == 1) {
        const float4 *x = (const float4 *)((const float *)X + i * dim);
        float acc = 0.f;
        for (int e = 0; e < dim / 4; ++e) {
            const float4 v = x[e];
            acc += v.x * v.x; acc += v.y * v.y; acc += v.z * v.z; acc += v.w * v.w;
        }
        out[i] = __float_as_uint(acc);
    } else {
        const uint4 *x = (const uint4 *)((const uint8_t *)X + i * dim);
        int acc = 0;
        for (int e = 0; e < dim / 16; ++e) {
            const uint4 v = x[e];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int d = (int)((w[a] >> (8 * b)) & 0xFFu) - 128;
                    acc += d * d;
                }
        }
        out[i] = (uint32_t)acc;
    }
}

void launch_row_norms(int dtype, const void *X, int32_t dim, int64_t n, uint32_t *out, hipStream_t s)
{
    if (n <= 0) return;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (dtype == 1) hipLaunchKernelGGL(row_norm_kernel<1>, grid, block, 0, s, X, dim, n, out);
    else hipLaunchKernelGGL(row_norm_kernel<0>, grid, block, 0, s, X, dim, n, out);
}

bool seed_dist_supported(int dtype, int dim)
{
    const int nch = dim * (dtype == 0 ? 1 : 4) / kChunkBytes;
    return nch == 8 || nch == 12 || nch == 16 || nch == 24 || nch == 32;
}

template <int DT> static void launch_seed_dt(const SeedParams &p, int nch, unsigned grid, hipStream_t s)
{
    switch (nch) {
    case 8: hipLaunchKernelGGL((seed_dist_kernel<DT, 8>), dim3(grid), dim3(64), 0, s, p); break;
    case 12: hipLaunchKernelGGL((seed_dist_kernel<DT, 12>), dim3(grid), dim3(64), 0, s, p); break;
    case 16: hipLaunchKernelGGL((seed_dist_kernel<DT, 16>), dim3(grid), dim3(64), 0, s, p); break;
    case 24: hipLaunchKernelGGL((seed_dist_kernel<DT, 24>), dim3(grid), dim3(64), 0, s, p); break;
    case 32: hipLaunchKernelGGL((seed_dist_kernel<DT, 32>), dim3(grid), dim3(64), 0, s, p); break;
    default: break;
    }
}

void launch_seed_dist(int dtype, const SeedParams &p, int n_tiles, hipStream_t s)
{
    if (n_tiles <= 0) return;
    const int nch = p.dim * (dtype == 0 ? 1 : 4) / kChunkBytes;
    const unsigned grid = (unsigned)n_tiles * (unsigned)p.max_chunks;
    if (dtype == 0) launch_seed_dt<0>(p, nch, grid, s);
    else launch_seed_dt<1>(p, nch, grid, s);
}

}  // namespace vf
