// IVF-BFS (Section 4.2.2, Alg. 2) on float32 lists in two steps that read half the bytes of the plain scan:
// a filter over a bfloat16 copy of the interleaved lists, then an exact re-ranking of the few candidates it
// keeps.  The scan of a batch is bound by the bytes of the lists it streams (a handful of queries share a list),
// so the copy's 2 bytes per component are what counts; the result is still the exact filtered top-k, because a
// query whose filtered result cannot be proven complete is scanned again with the exact distance.
//
// scan_bf16_kernel.  The tile and selection of scan_topk16_kernel around v_mfma_f32_16x16x32_bf16: lane
// (c = lane % 16, kq = lane / 16) holds, of query row c, the 16-byte chunks 4 s + kq (8 components each) as a
// bfloat16 high part and the bfloat16 rounding of the rest (|q - hi - lo| <= 2^-16 |q| per component), and of
// list entries c and 16 + c of a group the same chunks of the bfloat16 copy; both parts go into one float32
// accumulator.  Norms are those of the unrounded vectors, so an approximation |q|^2 + |x|^2 - 2 (hi + lo).bf16(x)
// differs from the ordered float32 distance by at most
//     B = err_bound (|q|^2 + max |x|^2) + 2 |q| max |x - bf16(x)|.
// Per (query, segment) the Kc = k + margin smallest approximations are kept.
//
// scan_rerank_kernel.  One wave per query: the Kc smallest approximations over all its segments (T = the largest
// of them), their vectors gathered from the vector table and scored with the ordered float32 distance by 8-lane
// teams, sorted, the k best written.  Every candidate that was dropped anywhere has an approximation >= T, hence
// an ordered distance >= T - B: if the k-th re-ranked distance is below T - B (or nothing was dropped) the result
// is the exact one.  Otherwise (rare: counted, and reported by the profile) the wave scans the query's whole list
// itself with the ordered distance, 64 entries a step: predicate, gather, score, merge into the k best.
#include "vf_beam.h"
#include "vf_select.h"

namespace vf {

typedef __bf16 v8bf_scan __attribute__((ext_vector_type(8)));
typedef float v4f_scan __attribute__((ext_vector_type(4)));

constexpr int kScanBf16Waves = 2;   // waves per SIMD the kernel is compiled for

template <int NCH16, bool AND, int SLOTS>
__global__ __launch_bounds__(64, kScanBf16Waves) void scan_bf16_kernel(ScanParams p)
{
    extern __shared__ uint4 smem[];
    constexpr int NS = NCH16 / 4, PC = 64;
    static_assert(NCH16 % 4 == 0, "the chunk count must be a multiple of four");
    const ScanItem it = p.items[blockIdx.x];
    const int lane = threadIdx.x, c16 = lane & 15, kq = lane >> 4;
    const int K = p.K, KS = K | 1, TR = p.tile_rows;   // K: candidates kept per row; TR <= 16

    uint64_t *pend = (uint64_t *)smem;                           // [TR][PC]
    uint64_t *best = pend + TR * PC;                             // [TR][KS]
    int32_t *qrow_s = (int32_t *)(best + TR * KS);               // [32]
    uint32_t *qnorm_s = (uint32_t *)(qrow_s + 32);               // [32]
    uint32_t *pcnt = qnorm_s + 32;                               // [32]

    if (lane < 32) { qrow_s[lane] = lane < it.q_count ? p.qrow[it.q_begin + lane] : -1; pcnt[lane] = 0; }
    for (int i = lane; i < TR * KS; i += 64) best[i] = KEY_MAX;
    __syncthreads();

    // A operand, resident in registers: the chunks 4 sq + kq of query row c16, split into two bfloat16 parts;
    // the row's squared norm (of the float32 values) is summed over the four lanes that share it
    uint4 ahi[NS], alo[NS];
    {
        const int qr = c16 < it.q_count ? qrow_s[c16] : -1;
        const float *qp = (const float *)p.qsrc + (int64_t)(qr >= 0 ? qr : 0) * p.dim;
        float acc = 0.f;
#pragma unroll
        for (int sq = 0; sq < NS; ++sq) {
            float f[8];
            if (qr >= 0) {
                const float4 a = *(const float4 *)(qp + 8 * (4 * sq + kq)), b = *(const float4 *)(qp + 8 * (4 * sq + kq) + 4);
                f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) f[i] = 0.f;
            }
            uint32_t hi[8], lo[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                hi[i] = bf16_rn_bits(f[i]);
                lo[i] = bf16_rn_bits(f[i] - __uint_as_float(hi[i] << 16));
                acc += f[i] * f[i];
            }
            ahi[sq] = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
            alo[sq] = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
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
    const float *xnorm = (const float *)p.xnorm;
    // B registers: SLOTS groups in flight, each of two column blocks (entries c16 and 16 + c16) with their norms.
    // Every fetch is unconditional (past the end the last group is fetched again, from L2), so that the compiler
    // can count the outstanding loads at every wait.
    uint4 breg[SLOTS][2][NS];
    float xnr[SLOTS][2];
    auto fetch_block = [&](int slot, int g, int cb) {
        const uint4 *blk = p.xblk + (it.group0 + g) * (int64_t)(NCH16 * 32);
#pragma unroll
        for (int sq = 0; sq < NS; ++sq) breg[slot][cb][sq] = blk[(4 * sq + kq) * 32 + cb * 16 + c16];
        xnr[slot][cb] = xnorm[(it.group0 + g) * 32 + cb * 16 + c16];
    };
    const int last_group = n_groups - 1;
#pragma unroll
    for (int slot = 0; slot < SLOTS; ++slot) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) fetch_block(slot, slot < last_group ? slot : last_group, cb);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int grp0 = 0; grp0 < n_groups; grp0 += SLOTS) {
#pragma unroll
      for (int slot = 0; slot < SLOTS; ++slot) {
        // (a group count that is no multiple of SLOTS ends with phantom steps on the re-fetched last group,
        // every column masked)
        const int grp = grp0 + slot;
        const int refill = grp + SLOTS < last_group ? grp + SLOTS : last_group;
        v4f_scan acc[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) acc[cb] = (v4f_scan){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sq = 0; sq < NS; ++sq) {
            const v8bf_scan ah = __builtin_bit_cast(v8bf_scan, ahi[sq]), al = __builtin_bit_cast(v8bf_scan, alo[sq]);
            const v8bf_scan b0 = __builtin_bit_cast(v8bf_scan, breg[slot][0][sq]), b1 = __builtin_bit_cast(v8bf_scan, breg[slot][1][sq]);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, b1, acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, b1, acc[1], 0, 0, 0);
        }
        const float xn[2] = {xnr[slot][0], xnr[slot][1]};
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) fetch_block(slot, refill, cb);
        __builtin_amdgcn_sched_barrier(0);

        // phase 1 (branch-free): approximations and threshold tests of this lane's 4 rows x 2 entries
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
                pm |= (below & (col_ok >> i) & 1u) << (cb * 4 + i);
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
                    const uint32_t at = atomicAdd(&pcnt[row], 1u);
                    pend[row * PC + at] = ((uint64_t)bitsv[b] << 32) | (uint32_t)entry;
                }
            }
        }
        if (__any(pm != 0)) {
            wave_lds_sync();
            pcv = lane < 32 ? (int)pcnt[lane] : 0;
        }
        if (__any(pcv >= PC - 32) || (grp + 1 >= n_groups && __any(pcv != 0))) drain();
      }
    }
    __syncthreads();

    // every item leaves its rows' kept candidates as a partial row (ascending, -1 = none)
    for (int r = 0; r < it.q_count; ++r) {
        if (lane >= K) continue;
        const uint64_t key = best[r * KS + lane];
        const int64_t o = (int64_t)(it.part_row + r) * K + lane;
        p.res_idx[o] = key == KEY_MAX ? -1 : (int32_t)(uint32_t)key;
        p.res_bits[o] = (uint32_t)(key >> 32);
    }
}

__global__ __launch_bounds__(64) void scan_rerank_kernel(RerankParams p)
{
    __shared__ uint4 qv[64];          // the query, 16-byte chunks (dim <= 256)
    __shared__ int32_t cand_g[64];
    __shared__ int32_t cand_e[64];
    __shared__ uint32_t cand_d[64];
    const MergeItem it = p.items[blockIdx.x];
    const int lane = threadIdx.x, team = lane >> 3, tl = lane & 7;
    const int row_bytes = p.dim * 4, nchunks = row_bytes / kChunkBytes;
    const int Kc = p.Kc;
    for (int i = lane; i < nchunks; i += 64) qv[i] = *(const uint4 *)((const char *)p.Q + (int64_t)it.qrow * row_bytes + i * kChunkBytes);

    // the Kc smallest approximations over the segments' runs (each ascending)
    TopM<1> list;
    list.init(Kc);
    auto load_run = [&](int sg) -> uint64_t {
        if (lane >= Kc) return KEY_MAX;
        const int64_t o = (int64_t)(it.part_row + sg * it.stride) * Kc + lane;
        const int32_t idx = p.res_idx[o];
        return idx >= 0 ? ((uint64_t)p.res_bits[o] << 32) | (uint32_t)idx : KEY_MAX;
    };
    uint64_t next = load_run(0);
    for (int sg = 0; sg < it.nseg; ++sg) {
        const uint64_t key = next;
        if (sg + 1 < it.nseg) next = load_run(sg + 1);
        merge_sorted_run(list, key, lane);
    }
    const uint64_t kept = list.cur[0];
    const bool valid = kept != KEY_MAX;
    const uint32_t idx = (uint32_t)kept;
    const int cnt = __popcll(__ballot(valid));   // the kept candidates sit in lanes 0 .. cnt - 1
    if (valid) cand_g[lane] = p.map[it.map_off + idx];
    __syncthreads();
    // ordered distances of cand_g[lo .. n) into cand_d, eight at a time (one per 8-lane team); lo a multiple of 8
    auto score = [&](int n, int lo = 0) {
#pragma unroll 2
        for (int r0 = lo; r0 < n; r0 += 8) {
            const int my = r0 + team;
            const int g = cand_g[my < n ? my : 0];
            const uint32_t bits = team_dist_bits_f32(qv, (const char *)p.X + (int64_t)g * row_bytes, nchunks, tl);
            if (tl == 0 && my < n) cand_d[my] = bits;
        }
    };
    float qn = 0.f;
    for (int i = lane; i < nchunks; i += 64) {
        const uint4 v = qv[i];
        const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        qn += f[0] * f[0] + f[1] * f[1] + f[2] * f[2] + f[3] * f[3];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) qn += __shfl_xor(qn, o);
    const float B = p.err_bound * (qn + p.xn_max) + p.err_q * sqrtf(qn);
    const bool all_kept = list.worst == KEY_MAX;   // fewer than Kc candidates in all: no segment dropped one
    // The kept candidates are re-scored in the order of their approximations, first k and a few to spare, then eight
    // at a time, until everything not re-scored is provably worse than the k-th result: those candidates have
    // approximations >= T, the approximation of the first one not re-scored (the last one kept, once all are),
    // hence ordered distances >= T - B.  Most queries stop after the first step.
    int done_to = (p.K + 6 + 7) & ~7;
    done_to = done_to < cnt ? done_to : cnt;
    int scored_to = 0;
    uint64_t key = KEY_MAX;
    bool proven = false;
    while (true) {
        score(done_to, scored_to);
        scored_to = done_to;
        __syncthreads();
        key = (valid && lane < done_to) ? ((uint64_t)cand_d[lane] << 32) | idx : KEY_MAX;
        key = wave_sort64(key, lane);
        const uint64_t rest = done_to < cnt ? readlane64(kept, done_to) : list.worst;
        const uint64_t kth = readlane64(key, p.K - 1);
        proven = (all_kept && done_to == cnt) ||
                 (kth != KEY_MAX && rest != KEY_MAX &&
                  __uint_as_float((uint32_t)(kth >> 32)) < __uint_as_float((uint32_t)(rest >> 32)) - B);
        if (proven || done_to == cnt) break;
        done_to = done_to + 8 < cnt ? done_to + 8 : cnt;
    }
    if (!proven) {   // (wave-uniform) the definition itself: every entry of the list that passes the predicate
        if (lane == 0) atomicAdd(p.fail_count, 1u);
        int o_begin = 0, o_end = 0;
        if (p.others_off != nullptr) { o_begin = p.others_off[it.qrow]; o_end = p.others_off[it.qrow + 1]; }
        TopM<1> ex;
        ex.init(p.K);
        for (int e0 = 0; e0 < it.n; e0 += 64) {
            const int e = e0 + lane;
            bool ok = e < it.n;
            int g = 0;
            if (ok) {
                g = p.map[it.map_off + e];
                for (int o = o_begin; o < o_end && ok; ++o) ok = has_label(p.meta, p.others[o], g);
            }
            const uint64_t m = __ballot(ok);
            const int n_ok = __popcll(m);
            __syncthreads();
            if (ok) {
                const int at = __popcll(m & ((1ull << lane) - 1ull));
                cand_g[at] = g;
                cand_e[at] = e;
            }
            __syncthreads();
            score(n_ok);
            __syncthreads();
            merge_batch(ex, lane < n_ok ? ((uint64_t)cand_d[lane] << 32) | (uint32_t)cand_e[lane] : KEY_MAX, lane);
        }
        key = ex.cur[0];
    }
    if (lane < p.K) {
        const bool none = key == KEY_MAX;
        const int64_t o = (int64_t)it.qrow * p.K + lane;
        p.out_ids[o] = none ? -1 : (int64_t)p.map[it.map_off + (uint32_t)key];
        p.out_dists[o] = none ? __builtin_inff() : __uint_as_float((uint32_t)(key >> 32));
    }
}

bool scan_bf16_supported(int dtype, int dim, int tile_rows, int keep)
{
    return dtype == 1 && (dim == 128 || dim == 96) && tile_rows <= 16 && keep >= 1 && keep <= 64;
}

size_t scan_bf16_lds_bytes(int tile_rows, int keep)
{
    return (size_t)tile_rows * (64 + (keep | 1)) * 8 + 3 * 32 * 4;
}

void launch_scan_bf16(const ScanParams &p, int n_items, int slots, hipStream_t s)
{
    if (n_items <= 0) return;
    const size_t lds = scan_bf16_lds_bytes(p.tile_rows, p.K);
    const bool with_and = p.others_off != nullptr;
    const dim3 grid(n_items), block(64);
    // AND: as in scan_topk16_kernel (the predicate's loads inside the loop turn every wait into a wait for all
    // outstanding loads).  SLOTS: list groups a wave keeps in flight (8 KiB each at dim 128).
#define VF_LAUNCH_BF16(NCH16_) \
    do { \
        if (slots >= 2) { \
            if (with_and) hipLaunchKernelGGL((scan_bf16_kernel<NCH16_, true, 2>), grid, block, lds, s, p); \
            else hipLaunchKernelGGL((scan_bf16_kernel<NCH16_, false, 2>), grid, block, lds, s, p); \
        } else { \
            if (with_and) hipLaunchKernelGGL((scan_bf16_kernel<NCH16_, true, 1>), grid, block, lds, s, p); \
            else hipLaunchKernelGGL((scan_bf16_kernel<NCH16_, false, 1>), grid, block, lds, s, p); \
        } \
    } while (0)
    if (p.dim == 128) VF_LAUNCH_BF16(16);
    else VF_LAUNCH_BF16(12);
#undef VF_LAUNCH_BF16
}

void launch_scan_rerank(const RerankParams &p, int n_items, hipStream_t s)
{
    if (n_items <= 0) return;
    hipLaunchKernelGGL(scan_rerank_kernel, dim3(n_items), dim3(64), 0, s, p);
}

}  // namespace vf
