// IVF-Graph search (Section 4.2.1, Alg. 2): beam search of one query inside the
// virtual graph G_l of its label, with the greedy AND policy of Section 4.3.2.
//
// Mapping to CDNA4.  One wave64 per query (a one-wave workgroup: every step is
// wave-synchronous and up to 32 queries are resident per CU, so many independent
// gathers are in flight).  The top-M list ("itopk") lives in REGISTERS, sorted, one
// slot per lane and E = ceil(itopk / 64) registers: a candidate that beats the
// current worst entry is inserted by the whole wave with a ballot, a population
// count and a DPP wave shift -- no sort, no LDS traffic, and the list is always
// ordered, so picking the next parents is a ballot over the "unexpanded" bits.
// LDS only holds the query vector, the visited hash and the candidate staging area.
// A wave is split into eight 8-lane teams; a team fetches one candidate vector with
// 16-byte loads (128 contiguous bytes per team and step) and reduces its partial
// sums with DPP adds, so eight candidate rows are gathered at a time.
//
// Keys are (distance bits << 32 | local id << 1 | unexpanded): unsigned order is
// (distance, local id) order with ties to the lower id.  The visited table may
// forget (bounded probing); a forgotten vertex is scored again and then either loses
// against the worst entry (the list only tightens) or is recognised as a duplicate
// of an entry at insertion, so forgetting changes the number of distances computed,
// never the result.
//
// fp32 distances are evaluated in a fixed order so that results can be compared
// bit for bit with a CPU evaluation: lane t of a team sums (q_e - x_e)^2 over
// e = 32 s + 4 t + c (s ascending, c = 0..3) as acc = fma(d, d, acc), d = q - x, and the
// team combines ((a0+a1)+(a2+a3)) + ((a4+a5)+(a6+a7)).
#pragma once
#include "vf_device.h"

#ifndef VF_SEED_BLOCKS
#define VF_SEED_BLOCKS 16
#endif

namespace vf {

// true: id was not in the table (it is now, unless the probe budget ran out)
__device__ __forceinline__ bool visit(uint32_t *tab, int bits, uint32_t id)
{
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t slot = (id * 0x9E3779B1u) >> (32 - bits);
    for (int pr = 0; pr < 16; ++pr) {
        const uint32_t old = atomicCAS(&tab[slot], 0xFFFFFFFFu, id);
        if (old == 0xFFFFFFFFu) return true;
        if (old == id) return false;
        slot = (slot + 1) & mask;
    }
    return true;
}

// Is local id c one of the ns stratified seeds floor(j * n / ns), j < ns?  (ns <= n.)
// Seeds are scored up front, so a child that is a seed has been visited already;
// answering this arithmetically keeps the seeds out of the visited table.
// c is a seed iff some multiple of n lies in [c * ns, c * ns + ns), i.e. iff
// r = (c * ns) mod n is 0 or larger than n - ns.  The quotient comes from a double-precision
// multiplication by 1 / n (for n * ns < 2^52 the product is exact in a double and the estimate is off by at most
// one, which the two corrections absorb); the remainder is exact integer arithmetic.
__device__ __forceinline__ bool is_seed(uint32_t c, uint32_t n, uint32_t ns, double inv_n)
{
    if (ns >= n) return true;
    if (((uint64_t)n * ns) >> 52) {   // (not reached with realistic seed counts) plain integer division
        const uint64_t j = ((uint64_t)c * ns + n - 1) / n;
        return j < ns && (uint32_t)((j * n) / ns) == c;
    }
    const uint64_t prod = (uint64_t)c * ns;
    const uint32_t q = (uint32_t)((double)c * (double)ns * inv_n);
    int64_t r = (int64_t)prod - (int64_t)((uint64_t)q * n);
    if (r < 0) r += n;
    if (r >= (int64_t)n) r -= n;
    return r == 0 || r > (int64_t)(n - ns);
}

// floor(j * n / ns) for j < ns <= n: quotient estimated in double precision (exact product below 2^52, the
// estimate off by at most one), corrected with the exact remainder.
__device__ __forceinline__ int seed_local_id(uint32_t j, uint32_t n, uint32_t ns)
{
    const uint64_t prod = (uint64_t)j * n;
    if (((uint64_t)n * ns) >> 52) return (int)(prod / ns);
    uint32_t q = (uint32_t)((double)j * (double)n / (double)ns);
    int64_t r = (int64_t)prod - (int64_t)((uint64_t)q * ns);
    if (r < 0) { r += ns; --q; }
    if (r >= (int64_t)ns) { r -= ns; ++q; }
    return (int)q;
}

// The sorted top-M list: element i sits in register i / 64 of lane i % 64.
template <int E> struct TopM {
    uint64_t cur[E];
    int itopk;
    uint64_t worst;  // key of element itopk - 1 (KEY_MAX while the list is not full)

    __device__ __forceinline__ void init(int itopk_)
    {
        itopk = itopk_;
        worst = KEY_MAX;
#pragma unroll
        for (int r = 0; r < E; ++r) cur[r] = KEY_MAX;
    }

    // Insert a key (wave-uniform value).  Rejects keys that do not beat the worst entry
    // and keys whose (distance, id) the list already holds.
    __device__ __forceinline__ void insert(uint64_t key, int lane)
    {
        if (key >= worst) return;
        int pos = 0;
        bool dup = false;
#pragma unroll
        for (int r = 0; r < E; ++r) {
            dup = dup || __any((cur[r] >> 1) == (key >> 1));
            pos += __popcll(__ballot(cur[r] < key));
        }
        if (dup) return;
#pragma unroll
        for (int r = E - 1; r >= 0; --r) {
            uint64_t up = wave_shr1_64(cur[r]);
            if (r > 0) {
                const uint64_t carry = readlane64(cur[r - 1], 63);
                if (lane == 0) up = carry;
            }
            const int idx = r * 64 + lane;
            uint64_t nw = idx < pos ? cur[r] : (idx == pos ? key : up);
            if (idx >= itopk) nw = KEY_MAX;
            cur[r] = nw;
        }
        const int wl = (itopk - 1) & 63, wr = (itopk - 1) >> 6;
#pragma unroll
        for (int r = 0; r < E; ++r)
            if (r == wr) worst = readlane64(cur[r], wl);
    }
};

// A batch of up to 64 keys, one per lane (KEY_MAX = none), none of them in the list yet, into a list of at
// most 64 entries: sort the batch, take the 64 smallest of batch and list (element-wise minimum against
// the reversed batch), sort that bitonic sequence.  The same list as inserting the keys one by one, in
// about 330 wave instructions whatever the batch holds (one insertion: about 30).
__device__ __forceinline__ void merge_batch(TopM<1> &list, uint64_t key, int lane)
{
    uint64_t v = key < list.worst ? key : KEY_MAX;
    if (!__any(v != KEY_MAX)) return;
    v = wave_sort64(v, lane);
    const uint64_t vr = shfl64(v, 63 - lane);
    uint64_t m = list.cur[0] < vr ? list.cur[0] : vr;
    m = wave_merge64(m, lane);
    if (lane >= list.itopk) m = KEY_MAX;
    list.cur[0] = m;
    list.worst = readlane64(m, list.itopk - 1);
}

// The same for a batch that arrives sorted (ascending by lane, KEY_MAX at the end): the keys at or above the
// list's worst entry are a suffix, so the batch stays sorted after they are dropped and needs no sort.
__device__ __forceinline__ void merge_sorted_run(TopM<1> &list, uint64_t key, int lane)
{
    const uint64_t v = key < list.worst ? key : KEY_MAX;
    if (!__any(v != KEY_MAX)) return;
    const uint64_t vr = shfl64(v, 63 - lane);
    uint64_t m = list.cur[0] < vr ? list.cur[0] : vr;
    m = wave_merge64(m, lane);
    if (lane >= list.itopk) m = KEY_MAX;
    list.cur[0] = m;
    list.worst = readlane64(m, list.itopk - 1);
}

// Offers the keys held one per lane (distance bits, id; distinct and none of them in the list yet) to a
// one-register list: many at once through a sort and merge, a few one by one.
__device__ __forceinline__ void offer_distinct(TopM<1> &list, bool valid, uint32_t bits, int id, int lane)
{
    const bool in = valid && bits <= (uint32_t)(list.worst >> 32);
    uint64_t m = __ballot(in);
    if (__popcll(m) >= 10) {
        merge_batch(list, in ? ((uint64_t)bits << 32) | ((uint64_t)(uint32_t)id << 1) | 1ull : KEY_MAX, lane);
        return;
    }
    while (m) {
        const int b = __builtin_ctzll(m);
        m &= m - 1;
        const uint32_t kb = __builtin_amdgcn_readlane(bits, b);
        const uint32_t kc = (uint32_t)__builtin_amdgcn_readlane(id, b);
        list.insert(((uint64_t)kb << 32) | ((uint64_t)kc << 1) | 1ull, lane);
    }
}

// A wave scores seeds [j_lo, j_hi) of a list itself from the interleaved copy of the seeds (p.sblk; a wave that
// serves one query at a time has no tile of queries to share a dense kernel with) and offers them to `list`: one
// seed per lane, 64 seeds a step, every load a coalesced 16-byte chunk, the query (qv, LDS) a broadcast.  A lane
// walks its seed's chunks in the order of the 8-lane teams (partial sum t takes chunks t, t + 8, ...; fused
// multiply-add; the fixed tree), so the bits are those of a gathered evaluation.  Seeds that fail the predicate
// (others / o_cnt) are left out.  as_index: the list stores the seed index j instead of the local id.
template <int DT>
__device__ __forceinline__ void stream_seed_segment(const BeamParams &p, int label, const int32_t *others, int o_cnt,
                                                    const uint4 *qv, int nchunks, int j_lo, int j_hi, bool as_index,
                                                    TopM<1> &list, int lane)
{
    const int n = p.meta.S[label];
    const int ns = p.n_seeds < n ? p.n_seeds : n;
    const int64_t base = p.meta.O_HS[label];
    const int64_t g0 = p.sgoff[p.meta.hs_slot[label]];
    int qq_all = 0;
    if (DT == 0) {
        for (int ci = 0; ci < nchunks; ++ci) {
            const uint4 q = qv[ci];
            qq_all = (int)__builtin_amdgcn_udot4(q.x, q.x, (uint32_t)qq_all, false);
            qq_all = (int)__builtin_amdgcn_udot4(q.y, q.y, (uint32_t)qq_all, false);
            qq_all = (int)__builtin_amdgcn_udot4(q.z, q.z, (uint32_t)qq_all, false);
            qq_all = (int)__builtin_amdgcn_udot4(q.w, q.w, (uint32_t)qq_all, false);
        }
    }
    for (int j0 = j_lo; j0 < j_hi; j0 += 64) {
        const int j = j0 + lane;
        const bool valid = j < j_hi;
        const int je = valid ? j : j_hi - 1;   // lanes past the end re-read the last seed (in bounds), masked below
        const uint4 *col = p.sblk + (g0 + (je >> 5)) * (int64_t)(p.sblk_chunks * 32) + (je & 31);
        uint32_t bits;
        if (DT == 0) {
            uint32_t xx = 0, qx = 0;
            for (int c0 = 0; c0 < nchunks; c0 += 8) {
                uint4 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = col[(int64_t)((c0 + u < nchunks) ? c0 + u : nchunks - 1) * 32];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (c0 + u < nchunks) {
                        const uint4 q = qv[c0 + u];
                        xx = __builtin_amdgcn_udot4(x[u].x, x[u].x, xx, false); qx = __builtin_amdgcn_udot4(q.x, x[u].x, qx, false);
                        xx = __builtin_amdgcn_udot4(x[u].y, x[u].y, xx, false); qx = __builtin_amdgcn_udot4(q.y, x[u].y, qx, false);
                        xx = __builtin_amdgcn_udot4(x[u].z, x[u].z, xx, false); qx = __builtin_amdgcn_udot4(q.z, x[u].z, qx, false);
                        xx = __builtin_amdgcn_udot4(x[u].w, x[u].w, xx, false); qx = __builtin_amdgcn_udot4(q.w, x[u].w, qx, false);
                    }
                }
            }
            bits = (uint32_t)(qq_all + (int)xx - 2 * (int)qx);
        } else {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = 0.0f;
            if (nchunks <= 32) {
                // every chunk of the lane's seed is requested before the first is used (128 registers of loads in
                // flight): a step of 64 seeds then costs one memory latency, not one per eight chunks -- the wave has
                // a SIMD to itself and nothing else hides that latency.  Same order of operations as below.
                uint4 x[32];
#pragma unroll
                for (int c = 0; c < 32; ++c)
                    if (c < nchunks) x[c] = col[(int64_t)c * 32];   // (wave-uniform)
#pragma unroll
                for (int c = 0; c < 32; ++c) {
                    if (c < nchunks) {
                        const uint4 q = qv[c];
                        float d;
                        d = __uint_as_float(q.x) - __uint_as_float(x[c].x); a[c & 7] = __builtin_fmaf(d, d, a[c & 7]);
                        d = __uint_as_float(q.y) - __uint_as_float(x[c].y); a[c & 7] = __builtin_fmaf(d, d, a[c & 7]);
                        d = __uint_as_float(q.z) - __uint_as_float(x[c].z); a[c & 7] = __builtin_fmaf(d, d, a[c & 7]);
                        d = __uint_as_float(q.w) - __uint_as_float(x[c].w); a[c & 7] = __builtin_fmaf(d, d, a[c & 7]);
                    }
                }
            } else
            for (int c0 = 0; c0 < nchunks; c0 += 8) {   // chunk c0 + u belongs to partial sum u
                uint4 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = col[(int64_t)((c0 + u < nchunks) ? c0 + u : nchunks - 1) * 32];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (c0 + u < nchunks) {
                        const uint4 q = qv[c0 + u];
                        float d;
                        d = __uint_as_float(q.x) - __uint_as_float(x[u].x); a[u] = __builtin_fmaf(d, d, a[u]);
                        d = __uint_as_float(q.y) - __uint_as_float(x[u].y); a[u] = __builtin_fmaf(d, d, a[u]);
                        d = __uint_as_float(q.z) - __uint_as_float(x[u].z); a[u] = __builtin_fmaf(d, d, a[u]);
                        d = __uint_as_float(q.w) - __uint_as_float(x[u].w); a[u] = __builtin_fmaf(d, d, a[u]);
                    }
                }
            }
            const float b0 = a[0] + a[1], b1 = a[2] + a[3], b2 = a[4] + a[5], b3 = a[6] + a[7];
            const float c0s = b0 + b1, c1s = b2 + b3;
            bits = __float_as_uint(c0s + c1s);
        }
        const int c = valid ? seed_local_id((uint32_t)j, (uint32_t)n, (uint32_t)ns) : 0;
        bool pass = valid;
        if (o_cnt > 0 && valid) {
            const int g = p.meta.M_HS[base + c];
            for (int o = 0; o < o_cnt && pass; ++o) pass = has_label(p.meta, others[o], g);
        }
        offer_distinct(list, pass, bits, as_index ? j : c, lane);
    }
}

// One query of a beam search launch: where its inputs and outputs are.
struct BeamQuery {
    const void *q;             // the query vector (16-byte aligned)
    int32_t label;             // the graph list that is searched
    const int32_t *others;     // AND partner labels
    int32_t o_cnt;
    int64_t *out_ids;          // [k]
    float *out_dists;          // [k]
    int32_t *counters;         // optional [4]: distances computed, rows expanded, predicate tests, mode word
    int32_t *gathered;         // optional [1]
    const uint32_t *dseed_row; // optional: the query's row of the seed distance matrix
    const uint64_t *runs;      // optional: the query's runs from the selecting seed kernel
    int32_t seed_pass;         // seeds that pass the predicate (profiling, AND), -1: not counted
};

// The search of one query by one wave: a one-wave workgroup, or (STREAM_SEEDS, the serving kernel) one wave of a
// larger workgroup working by itself (wave_sync orders the wave's LDS traffic either way).
// smem: beam_lds_bytes of LDS.
// AND = false: compiled for batches without predicate labels (none of the predicate's code and registers).
// LAT: for launches of so few waves that each has a SIMD to itself (small batches, serving workers): the vectors of up
// to 64 candidates are requested before the first distance is computed (128 registers of loads in flight), so a
// batch of children costs one memory latency instead of one per 16 candidates.
template <int DT, int E, bool STREAM_SEEDS = false, bool AND = true, bool LAT = false>
__device__ __forceinline__ void beam_search_wave(const BeamParams &p, const BeamQuery &bq, uint4 *smem)
{
    const int lane = wave_lane<STREAM_SEEDS>(), team = lane >> 3, tl = lane & 7;
    const int label = bq.label;
    const int n = p.meta.S[label];
    const int64_t base = p.meta.O_HS[label];
    const int itopk = p.itopk, R = p.R;
    const int row_bytes = p.dim * (DT == 0 ? 1 : 4);
    const int nchunks = row_bytes / kChunkBytes;

    uint4 *qv = smem;                                  // [nchunks]
    int32_t *cand_c = (int32_t *)(smem + nchunks);     // [128] local ids
    int32_t *cand_g = cand_c + 128;                    // [128] global ids
    uint32_t *cand_d = (uint32_t *)(cand_g + 128);     // [128] distance bits
    int32_t *parents = (int32_t *)(cand_d + 128);      // [8]
    uint32_t *hash = (uint32_t *)(parents + 8);        // [1 << hash_bits]

    for (int i = lane; i < nchunks; i += 64)
        qv[i] = *(const uint4 *)((const char *)bq.q + i * kChunkBytes);
    for (int i = lane; i < (1 << p.hash_bits); i += 64) hash[i] = 0xFFFFFFFFu;
    wave_sync<STREAM_SEEDS>();

    const int o_cnt = AND ? bq.o_cnt : 0;
    const int qq_lane = DT == 0 ? lane_qq_u8(qv, nchunks, tl) : 0;

    // The AND predicate of global id g.  One partner label with a bitset -- every two-label query whose searched
    // list is its smallest: the partner's list is at least as long, so it is a graph list too -- is one word of
    // that bitset; the general form walks the partner labels (bitset or binary search each).
    const uint32_t *bits0 = nullptr;
    if (AND && o_cnt == 1) {
        const int32_t slot = p.meta.hs_slot[bq.others[0]];
        if (slot >= 0) bits0 = p.meta.bitsets + (int64_t)slot * p.meta.bitset_words;
    }
    auto passes = [&](int g) -> bool {
        if (bits0 != nullptr) return (bits0[g >> 5] >> (g & 31)) & 1u;
        bool ok = true;
        for (int o = 0; o < o_cnt && ok; ++o) ok = has_label(p.meta, bq.others[o], g);
        return ok;
    };
    // global ids of this list's seeds in seed order, when the call has them (else M_HS[base + floor(j n / ns)])
    const int32_t *smap = nullptr;
    if (AND && o_cnt > 0 && p.seed_map != nullptr) smap = p.seed_map + p.seed_goff[p.meta.hs_slot[label]] * 32;
    auto seed_gid = [&](int j) -> int {   // (ns as below: the number of seeds of this list)
        const int ns_ = p.n_seeds < n ? p.n_seeds : n;
        return smap != nullptr ? smap[j] : p.meta.M_HS[base + (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns_)];
    };

    TopM<E> top;
    top.init(itopk);
    int n_scored = 0, n_expanded = 0, n_tested = 0;  // work counters (uniform across the wave)
    int n_gathered = 0;                              // distances whose vector this wave fetched itself

    // Offer the candidates held one per lane (valid lanes, distance bits, local id) to the list.
    auto offer_to = [&](auto &list, bool valid, uint32_t bits, int c) {
        uint64_t m = __ballot(valid && bits <= (uint32_t)(list.worst >> 32));
        while (m) {
            const int b = __builtin_ctzll(m);
            m &= m - 1;
            const uint32_t kb = __builtin_amdgcn_readlane(bits, b);
            const uint32_t kc = (uint32_t)__builtin_amdgcn_readlane(c, b);
            list.insert(((uint64_t)kb << 32) | ((uint64_t)kc << 1) | 1ull, lane);
        }
    };
    auto offer = [&](bool valid, uint32_t bits, int c) { offer_to(top, valid, bits, c); };
    // Seeds are distinct and offered once, so many of them can enter a list in one merge.
    auto offer_seeds_to = [&](TopM<1> &list, bool valid, uint32_t bits, int c) {
        const bool in = valid && bits <= (uint32_t)(list.worst >> 32);
        if (__popcll(__ballot(in)) < 10) { offer_to(list, valid, bits, c); return; }
        merge_batch(list, in ? ((uint64_t)bits << 32) | ((uint64_t)(uint32_t)c << 1) | 1ull : KEY_MAX, lane);
    };

    // Distances of cand[0..cnt) (eight at a time, one per team) into cand_d.
    // (lo: a multiple of 8, the entries before it have been dealt with)
    auto score = [&](int cnt, bool distinct_new = false, int lo = 0) {   // distinct_new: seeds (see offer_seeds_to)
        n_scored += cnt - lo;
        n_gathered += cnt - lo;
        int lo_rest = lo;
        if constexpr (LAT) {
            if (nchunks <= 32) {   // at most four 16-byte chunks per lane of a team
                constexpr int NR = 8;
                for (int r0 = lo; r0 < cnt; r0 += 8 * NR) {
                    uint4 x[NR][4];
#pragma unroll
                    for (int u = 0; u < NR; ++u) {
                        const int my = r0 + 8 * u + team;
#pragma unroll
                        for (int w = 0; w < 4; ++w) x[u][w] = make_uint4(0, 0, 0, 0);
                        if (r0 + 8 * u < cnt) {   // (wave-uniform)
                            const char *xrow = (const char *)p.X + (int64_t)cand_g[my < cnt ? my : 0] * row_bytes;
#pragma unroll
                            for (int w = 0; w < 4; ++w)
                                if (w * 8 + tl < nchunks) x[u][w] = *(const uint4 *)(xrow + (w * 8 + tl) * kChunkBytes);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < NR; ++u) {
                        const int my = r0 + 8 * u + team;
                        if (r0 + 8 * u >= cnt) break;   // (wave-uniform)
                        uint32_t bits;
                        if constexpr (DT == 0) {
                            uint32_t xx = 0, qx = 0;
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
                                if (w * 8 + tl < nchunks) {
                                    const uint4 q = qv[w * 8 + tl], xv = x[u][w];
                                    xx = __builtin_amdgcn_udot4(xv.x, xv.x, xx, false); qx = __builtin_amdgcn_udot4(q.x, xv.x, qx, false);
                                    xx = __builtin_amdgcn_udot4(xv.y, xv.y, xx, false); qx = __builtin_amdgcn_udot4(q.y, xv.y, qx, false);
                                    xx = __builtin_amdgcn_udot4(xv.z, xv.z, xx, false); qx = __builtin_amdgcn_udot4(q.z, xv.z, qx, false);
                                    xx = __builtin_amdgcn_udot4(xv.w, xv.w, xx, false); qx = __builtin_amdgcn_udot4(q.w, xv.w, qx, false);
                                }
                            }
                            bits = (uint32_t)team_sum_i(qq_lane + (int)xx - 2 * (int)qx);
                        } else {   // the order of team_dist_bits_f32
                            float acc = 0.0f;
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
                                if (w * 8 + tl < nchunks) {
                                    const uint4 q = qv[w * 8 + tl], xv = x[u][w];
                                    float d;
                                    d = __uint_as_float(q.x) - __uint_as_float(xv.x); acc = __builtin_fmaf(d, d, acc);
                                    d = __uint_as_float(q.y) - __uint_as_float(xv.y); acc = __builtin_fmaf(d, d, acc);
                                    d = __uint_as_float(q.z) - __uint_as_float(xv.z); acc = __builtin_fmaf(d, d, acc);
                                    d = __uint_as_float(q.w) - __uint_as_float(xv.w); acc = __builtin_fmaf(d, d, acc);
                                }
                            }
                            bits = __float_as_uint(team_sum_f(acc));
                        }
                        if (tl == 0 && my < cnt) cand_d[my] = bits;
                    }
                }
                lo_rest = cnt;
            }
        }
#pragma unroll 2
        for (int r0 = lo_rest; r0 < cnt; r0 += 8) {
            const int my = r0 + team;
            const int g = cand_g[my < cnt ? my : 0];
            const char *xrow = (const char *)p.X + (int64_t)g * row_bytes;
            uint32_t bits;
            if (DT == 0) bits = team_dist_bits_u8(qv, qq_lane, xrow, nchunks, tl);
            else bits = team_dist_bits_f32(qv, xrow, nchunks, tl);
            if (tl == 0 && my < cnt) cand_d[my] = bits;
        }
        wave_sync<STREAM_SEEDS>();
        for (int i0 = 0; i0 < cnt; i0 += 64) {
            const int i = i0 + lane;
            const bool valid = i < cnt && i >= lo;
            if constexpr (E == 1) {
                if (distinct_new) { offer_seeds_to(top, valid, valid ? cand_d[i] : 0u, valid ? cand_c[i] : 0); continue; }
            }
            offer(valid, valid ? cand_d[i] : 0u, valid ? cand_c[i] : 0);
        }
    };

    // Keep the candidates that pass the AND predicate, compacted into cand[].
    // g_known: the global id of c if the caller has it already (>= 0), else it is looked up in M.
    auto filter_and_compact = [&](bool valid, int c, int cnt, int g_known = -1) -> int {
        int g = g_known;
        if (o_cnt > 0) n_tested += __popcll(__ballot(valid));
        if (valid) {
            if (g < 0) g = p.meta.M_HS[base + c];
            valid = passes(g);
        }
        const uint64_t m = __ballot(valid);
        if (valid) {
            const int at = cnt + __popcll(m & ((1ull << lane) - 1ull));
            cand_c[at] = c;
            cand_g[at] = g;
        }
        return cnt + __popcll(m);
    };

    // ---- InitializeSearch: stratified seeds floor(j * n / ns)
    const int ns = p.n_seeds < n ? p.n_seeds : n;
    const double inv_n = 1.0 / (double)n;
    int j_begin = 0;   // seeds below j_begin have been dealt with

    // Selection from a dense row of seed distances in two passes over chunks of 64 * NBLK seeds
    // held in registers: an upper bound of the M-th smallest distance of the chunk (M = list
    // capacity <= 64) comes from the lanes' own two smallest values, and only the few seeds at or
    // below it (and below the list's worst entry) are offered to the list.  Same result as offering
    // every seed, at a fraction of the insertions.  as_index: the list stores the seed index j
    // instead of the local id floor(j * n / ns).  Returns the number of seeds dealt with (a chunk
    // whose bound lets more than 128 seeds through ends the selection early).
    bool lazy_used = false, lazy_ok = true;
    auto select_seeds = [&](TopM<1> &list, const uint32_t *drow, bool as_index) -> int {
        constexpr int NBLK = VF_SEED_BLOCKS;
        int done_to = 0;
        for (int jc = 0; jc < ns; jc += 64 * NBLK) {
            uint32_t v[NBLK];
#pragma unroll
            for (int i = 0; i < NBLK; ++i) {
                const int j = jc + i * 64 + lane;
                v[i] = j < ns ? drow[j] : 0xFFFFFFFFu;
            }
            const int chunk_n = ns - jc < 64 * NBLK ? ns - jc : 64 * NBLK;
            int chunk_scored = chunk_n, chunk_tested = o_cnt > 0 ? chunk_n : 0;   // every seed counts as tested
            // AND: a seed that fails the predicate is taken out before the selection (its value becomes +inf).
            // Without the seeds' own id map the local id floor(j n / ns) advances by (64 n) / ns per step of 64 seeds:
            // one division per lane and chunk, then quotient / remainder increments.
            auto apply_predicate = [&]() {
                chunk_scored = 0;
                if (smap != nullptr) {
#pragma unroll
                    for (int i = 0; i < NBLK; ++i) {
                        const int j = jc + i * 64 + lane;
                        bool pass = j < ns;
                        if (pass) pass = passes(smap[j]);
                        if (!pass) v[i] = 0xFFFFFFFFu;
                        chunk_scored += __popcll(__ballot(pass));
                    }
                    return;
                }
                const uint64_t t64 = 64ull * (uint64_t)n;
                const uint32_t Q64 = (uint32_t)(t64 / (uint64_t)ns), R64 = (uint32_t)(t64 % (uint64_t)ns);
                const uint64_t t0 = (uint64_t)(jc + lane) * (uint64_t)n;
                uint32_t cq = (uint32_t)(t0 / (uint64_t)ns), cr = (uint32_t)(t0 % (uint64_t)ns);
#pragma unroll
                for (int i = 0; i < NBLK; ++i) {
                    const int j = jc + i * 64 + lane;
                    bool pass = j < ns;
                    if (pass) pass = passes(p.meta.M_HS[base + cq]);
                    if (!pass) v[i] = 0xFFFFFFFFu;
                    chunk_scored += __popcll(__ballot(pass));
                    cr += R64; cq += Q64;
                    if (cr >= (uint32_t)ns) { cr -= (uint32_t)ns; cq += 1; }
                }
            };
            // With a full list the predicate is only evaluated for the few seeds at or below the list's worst entry
            // (a predicate test is a 4-byte read from a bitset of n / 8 bytes: a cache line each).  Not for queries
            // whose predicate passes so few seeds that most values stay below that entry (lazy_ok, sticky).
            bool lazy = lazy_ok && o_cnt > 0 && list.worst != KEY_MAX;
            // seeds at or below the bound, compacted into cand[] (those beyond its 128 slots only counted)
            auto compact = [&](uint32_t tau) -> int {
                wave_sync<STREAM_SEEDS>();
                int cnt = 0;
#pragma unroll
                for (int i = 0; i < NBLK; ++i) {
                    const int j = jc + i * 64 + lane;
                    const bool pass = v[i] <= tau && v[i] != 0xFFFFFFFFu && j < ns;
                    const uint64_t m = __ballot(pass);
                    if (m == 0) continue;   // (wave-uniform; with a full list most blocks of 64 hold no candidate)
                    const int at = cnt + __popcll(m & ((1ull << lane) - 1ull));
                    if (pass && at < 128) {
                        cand_d[at] = v[i];
                        cand_c[at] = j;
                    }
                    cnt += __popcll(m);
                }
                wave_sync<STREAM_SEEDS>();
                return cnt;
            };
            int cnt;
            for (;;) {
                if (o_cnt > 0 && !lazy) apply_predicate();
                // the two smallest values of every lane; the M-th smallest of those 128 bounds the M-th
                // smallest of the chunk: sort both sets across the wave, take the 64 smallest of their
                // union (element-wise minimum against the reversed other set), sort those
                // (a full list bounds the chunk as well as that, or better from the third chunk on: its worst
                // entry is the M-th smallest of everything before)
                uint32_t tau = (uint32_t)(list.worst >> 32);
                // (a chunk whose passing seeds all fit into the list's free entries needs no bound: AND queries
                // whose predicate passes few seeds spend most of their chunks in this state)
                const bool all_fit = list.worst == KEY_MAX && o_cnt > 0 &&
                                     __popcll(__ballot(list.cur[0] != KEY_MAX)) + chunk_scored <= list.itopk;
                if (all_fit) tau = 0xFFFFFFFEu;
                if (list.worst == KEY_MAX && !all_fit) {
                    uint32_t m1 = v[0], m2 = 0xFFFFFFFFu;
#pragma unroll
                    for (int i = 1; i < NBLK; ++i) {
                        const uint32_t hi = v[i] > m1 ? v[i] : m1;
                        m2 = hi < m2 ? hi : m2;
                        m1 = v[i] < m1 ? v[i] : m1;
                    }
                    const uint32_t s1 = wave_sort_u32(m1, lane), s2 = wave_sort_u32(m2, lane);
                    const uint32_t s2r = (uint32_t)__shfl((int)s2, 63 - lane);
                    const uint32_t sorted = wave_merge_u32(s1 < s2r ? s1 : s2r, lane);
                    tau = (uint32_t)__builtin_amdgcn_readlane((int)sorted, list.itopk - 1);
                }
                cnt = compact(tau);
                if (!(lazy && cnt > 128)) break;
                lazy = false;      // too many for the candidate area: the predicate first after all
                lazy_ok = false;
            }
            if (lazy) lazy_used = true;
            if (cnt > 128) break;
            n_scored += chunk_scored;
            n_tested += chunk_tested;
            for (int i0 = 0; i0 < cnt; i0 += 64) {
                const int i = i0 + lane;
                bool valid = i < cnt;
                int c = valid ? cand_c[i] : 0;
                if (lazy || !as_index) {
                    const int cl = (int)(((uint64_t)c * (uint64_t)n) / (uint64_t)ns);
                    if (lazy && valid) valid = passes(seed_gid(c));
                    if (!as_index) c = cl;
                }
                offer_seeds_to(list, valid, valid ? cand_d[i] : 0u, c);
            }
            done_to = jc + 64 * NBLK < ns ? jc + 64 * NBLK : ns;
        }
        return done_to;
    };

    bool seeds_done = false;
    int n_rescored = 0, seed_fallback = 0;   // profiling only
    // After a seed phase that skipped predicate tests the number of seeds that pass (the definition's count of
    // distances computed) is not known to the wave; while profiling a small kernel has counted them beforehand.
    auto fix_seed_count = [&]() {
        if (lazy_used && bq.seed_pass >= 0) n_scored = bq.seed_pass;
    };
    // The runs the selection kernel left for this query: one per seed segment, sorted, keys
    // (value bits << 32 | seed index).  as_index as in select_seeds.
    auto merge_runs = [&](TopM<1> &list, bool as_index) {
        const int nseg = (ns + p.seg_seeds - 1) / p.seg_seeds;
        const uint64_t *runs = bq.runs;
        uint64_t next = lane < p.run_K ? runs[lane] : KEY_MAX;
        for (int sg = 0; sg < nseg; ++sg) {
            const uint64_t raw = next;
            if (sg + 1 < nseg) next = lane < p.run_K ? runs[(sg + 1) * p.run_K + lane] : KEY_MAX;
            uint64_t key = KEY_MAX;
            if (raw != KEY_MAX) {
                const uint32_t j = (uint32_t)raw;
                const uint32_t c = as_index ? j : (uint32_t)seed_local_id(j, (uint32_t)n, (uint32_t)ns);
                key = (raw & 0xFFFFFFFF00000000ull) | ((uint64_t)c << 1) | 1ull;
            }
            merge_sorted_run(list, key, lane);
        }
        n_tested += o_cnt > 0 ? ns : 0;
        n_scored += (o_cnt > 0 && bq.seed_pass >= 0) ? bq.seed_pass : ns;
    };

    if constexpr (E == 1 && DT == 1) {
        if ((bq.dseed_row != nullptr || bq.runs != nullptr) && p.seed_approx != 0) {
            // The seeds were scored approximately on the matrix cores.  Keep the seed_keep best of them, re-score
            // those with the ordered distance, and accept the result only if every other seed is provably
            // worse than the list's worst entry: its approximation is at least T (the last one kept),
            // its ordered distance therefore at least T - B.
            TopM<1> tmp;
            tmp.init(p.seed_keep);
            int got = ns;
            if (bq.runs != nullptr) merge_runs(tmp, true);
            else got = select_seeds(tmp, bq.dseed_row, true);
            if (got == ns) {
                fix_seed_count();
                const uint64_t key = tmp.cur[0];
                const bool valid = key != KEY_MAX;
                const int c = valid ? seed_local_id((uint32_t)(key >> 1) & 0x7FFFFFFFu, (uint32_t)n, (uint32_t)ns) : 0;
                // the kept seeds sit in lanes 0 .. cnt - 1 (sorted list) and have passed the predicate already
                wave_sync<STREAM_SEEDS>();
                const int cnt = __popcll(__ballot(valid));
                if (valid) { cand_c[lane] = c; cand_g[lane] = p.meta.M_HS[base + c]; }
                wave_sync<STREAM_SEEDS>();
                float qn = 0.f;
                for (int i = lane; i < nchunks; i += 64) {
                    const uint4 v = qv[i];
                    const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
                    qn += f[0] * f[0] + f[1] * f[1] + f[2] * f[2] + f[3] * f[3];
                }
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) qn += __shfl_xor(qn, o);
                const float B = p.err_bound * (qn + p.xn_max) + p.err_q * sqrtf(qn);
                const bool all_kept = tmp.worst == KEY_MAX;
                // The kept seeds are re-scored in the order of their approximations, first enough to fill the list and
                // eight to spare, then eight at a time, until everything not re-scored yet is provably worse than the
                // list's worst entry: those seeds have approximations >= T, the approximation of the first one not
                // re-scored (the last one kept, once all are), hence ordered distances >= T - B.  Most queries stop
                // after the first step; the spare candidates beyond it are for the few that need them.
                int done_to = (itopk + 8 + 7) & ~7;
                done_to = done_to < cnt ? done_to : cnt;
                score(done_to, true);
                bool proven = false;
                while (true) {
                    const uint64_t next = done_to < cnt ? readlane64(key, done_to) : tmp.worst;
                    proven = top.worst != KEY_MAX && next != KEY_MAX &&
                             __uint_as_float((uint32_t)(top.worst >> 32)) < __uint_as_float((uint32_t)(next >> 32)) - B;
                    if (proven || done_to == cnt) break;
                    const int upto = done_to + 8 < cnt ? done_to + 8 : cnt;
                    score(upto, true, done_to);
                    done_to = upto;
                }
                if (proven || (all_kept && done_to == cnt)) {
                    seeds_done = true;
                    n_scored -= done_to;   // the re-scored seeds were counted when they were selected
                    n_rescored = done_to;
                }
            }
            if (!seeds_done) {   // start over; the gather path below scores every seed
                top.init(itopk);
                n_scored = 0;
                n_tested = 0;
                seed_fallback = 1;
                if (p.fallback_count != nullptr && lane == 0) atomicAdd(p.fallback_count, 1u);
            }
        }
    }
    if constexpr (E == 1) {
        if (!seeds_done && bq.runs != nullptr && p.seed_approx == 0) {   // exact distances (uint8)
            merge_runs(top, false);
            seeds_done = true;
        }
        if (!seeds_done && bq.dseed_row != nullptr && p.seed_approx == 0)
            j_begin = select_seeds(top, bq.dseed_row, false);
    }
    if (seeds_done) {
    } else if (bq.dseed_row != nullptr && p.seed_approx == 0) {
        // plain path (AND queries, long lists of candidates): stream the row and offer every seed
        const uint32_t *drow = bq.dseed_row;
        for (int j0 = j_begin; j0 < ns; j0 += 64) {
            const int j = j0 + lane;
            const bool valid = j < ns;
            const uint32_t bits = valid ? drow[j] : 0u;
            bool pass = valid;
            int c = 0;
            if (o_cnt > 0) {
                n_tested += __popcll(__ballot(valid));
                // (a seed above the list's worst entry cannot enter it: its predicate is not evaluated)
                const bool full = top.worst != KEY_MAX;
                if (full) { lazy_used = true; pass = valid && bits <= (uint32_t)(top.worst >> 32); }
                if (pass) {
                    c = (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns);
                    pass = passes(seed_gid(j));
                }
                n_scored += __popcll(__ballot(pass));
            } else {
                n_scored += __popcll(__ballot(valid));
                if (pass && bits <= (uint32_t)(top.worst >> 32)) c = (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns);
            }
            offer(pass, bits, c);
        }
        fix_seed_count();
    } else if (STREAM_SEEDS && E == 1 && p.sblk != nullptr) {
        if constexpr (E == 1) stream_seed_segment<DT>(p, label, bq.others, o_cnt, qv, nchunks, 0, ns, false, top, lane);
    } else {
        for (int j0 = 0; j0 < ns; j0 += 64) {
            const int j = j0 + lane;
            const bool valid = j < ns;
            const int c = valid ? (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns) : 0;
            wave_sync<STREAM_SEEDS>();
            const int cnt = filter_and_compact(valid, c, 0);
            wave_sync<STREAM_SEEDS>();
            score(cnt);
        }
    }

    // ---- iterations: expand the best unexpanded entries, score their unvisited children, merge
    // child slot j = j0 + lane (j0 = 0 or 64, width * R <= 128) is edge j % R of parent j / R
    const int jq0 = lane / R, jr0 = lane - jq0 * R, jq1 = (lane + 64) / R, jr1 = lane + 64 - jq1 * R;
    for (int it = 0; it < p.iters; ++it) {
        int np = 0;
#pragma unroll
        for (int r = 0; r < E; ++r) {
            uint64_t m = __ballot(top.cur[r] != KEY_MAX && (top.cur[r] & 1ull));
            while (m && np < p.width) {
                const int b = __builtin_ctzll(m);
                m &= m - 1;
                if (lane == b) {
                    parents[np] = (int32_t)((top.cur[r] >> 1) & 0x7FFFFFFFu);
                    top.cur[r] &= ~1ull;
                }
                ++np;
            }
        }
        // clearing the flag lowers a key by one: refresh the cached worst key
        {
            const int wl = (itopk - 1) & 63, wr = (itopk - 1) >> 6;
#pragma unroll
            for (int r = 0; r < E; ++r)
                if (r == wr) top.worst = readlane64(top.cur[r], wl);
        }
        wave_sync<STREAM_SEEDS>();
        if (np == 0) break;
        n_expanded += np;
        int cnt = 0;
        for (int j0 = 0; j0 < np * R; j0 += 64) {
            const int j = j0 + lane;
            bool valid = j < np * R;
            int c = -1, g = -1;
            if (valid) {
                // the row as local ids (list bookkeeping) and as global ids (where the vector is): two
                // independent coalesced loads instead of a lookup in M that depends on the first
                const int pa = parents[j0 == 0 ? jq0 : jq1];
                const int64_t at = (base + pa) * R + (j0 == 0 ? jr0 : jr1);
                c = p.G[at];
                g = p.Gg[at];
                valid = c >= 0 && !is_seed((uint32_t)c, (uint32_t)n, (uint32_t)ns, inv_n) &&
                        visit(hash, p.hash_bits, (uint32_t)c);
            }
            cnt = filter_and_compact(valid, c, cnt, g);
        }
        wave_sync<STREAM_SEEDS>();
        score(cnt);
    }

    if (bq.counters != nullptr && lane == 0) {
        int32_t *cn = bq.counters;
        cn[0] = n_scored; cn[1] = n_expanded; cn[2] = n_tested; cn[3] = 2 + seed_fallback + (n_rescored << 8);
        if (bq.gathered != nullptr) *bq.gathered = n_gathered;
    }

    // ---- first k entries (k <= 64: register 0), local -> global through M
    if (lane < p.k) {
        const uint64_t key = top.cur[0];
        const int o = lane;
        if (key == KEY_MAX) {
            bq.out_ids[o] = -1;
            bq.out_dists[o] = __builtin_inff();
        } else {
            const uint32_t hi = (uint32_t)(key >> 32);
            bq.out_ids[o] = (int64_t)p.meta.M_HS[base + ((uint32_t)(key >> 1) & 0x7FFFFFFFu)];
            bq.out_dists[o] = DT == 0 ? (float)(int)hi : __uint_as_float(hi);
        }
    }
}

}  // namespace vf
