// IVF-Graph search (Section 4.2.1, Alg. 2): beam search of one query inside the
// virtual graph G_l of its label, with the greedy AND policy of Section 4.3.2.
//
// Mapping to CDNA4.  One wave64 per query (a one-wave workgroup: every step is
// wave-synchronous, barriers cost nothing, and up to 32 queries are resident per
// CU so that many independent gathers are in flight).  The top-M list ("itopk"),
// the pending candidates and the visited hash live in LDS.  A wave is split into
// eight 8-lane teams; a team fetches one candidate vector with 16-byte loads
// (128 contiguous bytes per team and step) and reduces its partial sums with
// DPP adds, so eight candidate rows are gathered at a time.
//
// Keys are (distance bits << 32 | local id << 1 | unexpanded): unsigned order is
// (distance, local id) order with ties to the lower id; an expanded entry sorts
// before an unexpanded duplicate of itself, which the merge then drops.  The
// visited table may forget (bounded probing); by construction this changes the
// number of distances computed, never the result.
//
// fp32 distances are evaluated in a fixed order so that results can be compared
// bit for bit with a CPU evaluation: lane t of a team sums (q_e - x_e)^2 over
// e = 32 s + 4 t + c (s ascending, c = 0..3) as acc = fma(d, d, acc), d = q - x, and the
// team combines ((a0+a1)+(a2+a3)) + ((a4+a5)+(a6+a7)).
#include "vf_device.h"

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
__device__ __forceinline__ bool is_seed(uint32_t c, uint32_t n, uint32_t ns)
{
    if (ns >= n) return true;
    const uint64_t j = ((uint64_t)c * ns + n - 1) / n;  // smallest j with floor(j * n / ns) >= c
    return j < ns && (uint32_t)((j * n) / ns) == c;
}

struct BeamLds {
    uint64_t *list;   // [LP]
    int32_t *cand_c;  // [128]
    int32_t *cand_g;  // [128]
    int32_t *parents; // [8]
    uint32_t *hash;   // [1 << hash_bits]
    uint4 *qv;        // [row_bytes / 16]
};

// Sort list[0..LP) ascending, drop duplicates of (distance, id) -- they sit next to
// each other, the expanded copy first -- and everything beyond itopk.  LP <= 512.
__device__ void sort_list(uint64_t *list, int LP, int itopk, int lane)
{
    for (;;) {
        wave_bitonic_sort(list, LP, lane);
        uint32_t dups = 0;
        for (int i0 = 0, w = 0; i0 < LP; i0 += 64, ++w) {
            const int i = i0 + lane;
            const uint64_t cur = list[i], prev = i > 0 ? list[i - 1] : KEY_MAX;
            if (i > 0 && cur != KEY_MAX && (cur >> 1) == (prev >> 1)) dups |= 1u << w;
        }
        __syncthreads();
        if (!__any(dups != 0)) break;
        for (int i0 = 0, w = 0; i0 < LP; i0 += 64, ++w)
            if ((dups >> w) & 1u) list[i0 + lane] = KEY_MAX;
        __syncthreads();
    }
    for (int i = itopk + lane; i < LP; i += 64) list[i] = KEY_MAX;
    __syncthreads();
}

template <int DT>
__global__ __launch_bounds__(64) void beam_kernel(BeamParams p)
{
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x, team = lane >> 3, tl = lane & 7;
    const int gq = blockIdx.x;
    const int qi = p.gq_query[gq], label = p.gq_label[gq];
    const int n = p.meta.S[label];
    const int64_t base = p.meta.O_HS[label];
    const int itopk = p.itopk, LP = p.LP, CB = LP - itopk, R = p.R;
    const int row_bytes = p.dim * (DT == 0 ? 1 : 4);
    const int nchunks = row_bytes / kChunkBytes;

    BeamLds s;
    s.qv = smem;
    s.list = (uint64_t *)(smem + nchunks);
    s.cand_c = (int32_t *)(s.list + LP);
    s.cand_g = s.cand_c + 128;
    s.parents = s.cand_g + 128;
    s.hash = (uint32_t *)(s.parents + 8);

    for (int i = lane; i < nchunks; i += 64)
        s.qv[i] = *(const uint4 *)((const char *)p.Q + (int64_t)qi * row_bytes + i * kChunkBytes);
    for (int i = lane; i < LP; i += 64) s.list[i] = KEY_MAX;
    for (int i = lane; i < (1 << p.hash_bits); i += 64) s.hash[i] = 0xFFFFFFFFu;
    __syncthreads();

    int o_begin = 0, o_cnt = 0;
    if (p.others_off != nullptr) { o_begin = p.others_off[qi]; o_cnt = p.others_off[qi + 1] - o_begin; }

    const int qq_lane = DT == 0 ? lane_qq_u8(s.qv, nchunks, tl) : 0;

    uint64_t thr = KEY_MAX;  // key of list[itopk-1] after the last sort
    int pc = 0;              // pending candidates appended behind the list
    int n_scored = 0, n_expanded = 0, n_tested = 0;  // work counters (uniform across the wave)

    // Score cand[0..cnt) (eight at a time, one per team) and append those that beat thr.
    auto score_and_append = [&](int cnt) {
        n_scored += cnt;
        for (int r0 = 0; r0 < cnt; r0 += 8) {
            const int my = r0 + team;
            const bool valid = my < cnt;
            const int c = s.cand_c[valid ? my : 0];
            const int g = s.cand_g[valid ? my : 0];
            const char *xrow = (const char *)p.X + (int64_t)g * row_bytes;
            uint32_t bits;
            if (DT == 0) bits = team_dist_bits_u8(s.qv, qq_lane, xrow, nchunks, tl);
            else bits = team_dist_bits_f32(s.qv, xrow, nchunks, tl);
            const uint64_t key = ((uint64_t)bits << 32) | ((uint64_t)(uint32_t)c << 1) | 1ull;
            const bool pass = valid && tl == 0 && key < thr;
            const uint64_t m = __ballot(pass);
            if (pass) s.list[itopk + pc + __popcll(m & ((1ull << lane) - 1ull))] = key;
            pc += __popcll(m);
        }
    };

    // Keep the candidates that pass the AND predicate, compacted into cand[].
    auto filter_and_compact = [&](bool valid, int c, int cnt) -> int {
        int g = 0;
        if (o_cnt > 0) n_tested += __popcll(__ballot(valid));
        if (valid) {
            g = p.meta.M_HS[base + c];
            for (int o = 0; o < o_cnt && valid; ++o) valid = has_label(p.meta, p.others[o_begin + o], g);
        }
        const uint64_t m = __ballot(valid);
        if (valid) {
            const int at = cnt + __popcll(m & ((1ull << lane) - 1ull));
            s.cand_c[at] = c;
            s.cand_g[at] = g;
        }
        return cnt + __popcll(m);
    };

    auto flush = [&]() {
        __syncthreads();
        sort_list(s.list, LP, itopk, lane);
        thr = s.list[itopk - 1];
        pc = 0;
    };

    // ---- InitializeSearch: stratified seeds floor(j * n / ns)
    const int ns = p.n_seeds < n ? p.n_seeds : n;
    if (p.dseed != nullptr) {
        // distances were computed densely per label; stream this query's row and keep the best
        const uint32_t *drow = p.dseed + (int64_t)gq * p.ns_stride;
        for (int j0 = 0; j0 < ns; j0 += 64) {
            if (pc + 64 > CB) flush();
            const int j = j0 + lane;
            const bool valid = j < ns;
            const uint32_t bits = valid ? drow[j] : 0u;
            bool pass = valid;
            int c = 0;
            if (o_cnt > 0) {
                n_tested += __popcll(__ballot(valid));
                if (valid) {
                    c = (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns);
                    const int g = p.meta.M_HS[base + c];
                    for (int o = 0; o < o_cnt && pass; ++o) pass = has_label(p.meta, p.others[o_begin + o], g);
                }
                n_scored += __popcll(__ballot(pass));
            } else {
                n_scored += __popcll(__ballot(valid));
            }
            pass = pass && bits <= (uint32_t)(thr >> 32);
            if (pass && o_cnt == 0) c = (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns);
            const uint64_t key = ((uint64_t)bits << 32) | ((uint64_t)(uint32_t)c << 1) | 1ull;
            pass = pass && key < thr;
            const uint64_t m = __ballot(pass);
            if (pass) s.list[itopk + pc + __popcll(m & ((1ull << lane) - 1ull))] = key;
            pc += __popcll(m);
        }
    } else
    for (int j0 = 0; j0 < ns; j0 += 64) {
        if (pc + 64 > CB) flush();
        const int j = j0 + lane;
        const bool valid = j < ns;
        const int c = valid ? (int)(((uint64_t)j * (uint64_t)n) / (uint64_t)ns) : 0;
        __syncthreads();
        const int cnt = filter_and_compact(valid, c, 0);
        __syncthreads();
        score_and_append(cnt);
    }
    flush();

    // ---- iterations: expand the best unexpanded entries, score their unvisited children, merge
    for (int it = 0; it < p.iters; ++it) {
        int np = 0;
        for (int blk = 0; blk < itopk && np < p.width; blk += 64) {
            const int i = blk + lane;
            const uint64_t key = i < itopk ? s.list[i] : KEY_MAX;
            uint64_t m = __ballot(key != KEY_MAX && (key & 1ull));
            while (m && np < p.width) {
                const int b = __builtin_ctzll(m);
                m &= m - 1;
                if (lane == b) {
                    s.list[i] = key & ~1ull;
                    s.parents[np] = (int32_t)((key >> 1) & 0x7FFFFFFFu);
                }
                ++np;
            }
        }
        __syncthreads();
        if (np == 0) break;
        n_expanded += np;
        int cnt = 0;
        for (int j0 = 0; j0 < np * R; j0 += 64) {
            const int j = j0 + lane;
            bool valid = j < np * R;
            int c = -1;
            if (valid) {
                const int pa = s.parents[j / R];
                c = p.G[(base + pa) * R + (j % R)];
                valid = c >= 0 && !is_seed((uint32_t)c, (uint32_t)n, (uint32_t)ns) &&
                        visit(s.hash, p.hash_bits, (uint32_t)c);
            }
            cnt = filter_and_compact(valid, c, cnt);
        }
        __syncthreads();
        score_and_append(cnt);
        if (pc > 0) flush();
    }
    __syncthreads();

    if (p.counters != nullptr && lane == 0) {
        int32_t *cn = p.counters + (int64_t)qi * 4;
        cn[0] = n_scored; cn[1] = n_expanded; cn[2] = n_tested; cn[3] = 2;
    }

    // ---- first k entries, local -> global through M
    if (lane < p.k) {
        const uint64_t key = s.list[lane];
        const int64_t o = (int64_t)qi * p.k + lane;
        if (key == KEY_MAX) {
            p.out_ids[o] = -1;
            p.out_dists[o] = __builtin_inff();
        } else {
            const uint32_t hi = (uint32_t)(key >> 32);
            p.out_ids[o] = (int64_t)p.meta.M_HS[base + ((uint32_t)(key >> 1) & 0x7FFFFFFFu)];
            p.out_dists[o] = DT == 0 ? (float)(int)hi : __uint_as_float(hi);
        }
    }
}

size_t beam_lds_bytes(const BeamParams &p, int dtype)
{
    const size_t row_bytes = (size_t)p.dim * (dtype == 0 ? 1 : 4);
    return row_bytes + (size_t)p.LP * 8 + 128 * 4 * 2 + 8 * 4 + ((size_t)4 << p.hash_bits);
}

void launch_beam(int dtype, const BeamParams &p, int n_gq, hipStream_t s)
{
    if (n_gq <= 0) return;
    const size_t lds = beam_lds_bytes(p, dtype);
    if (dtype == 0) hipLaunchKernelGGL(beam_kernel<0>, dim3(n_gq), dim3(64), lds, s, p);
    else hipLaunchKernelGGL(beam_kernel<1>, dim3(n_gq), dim3(64), lds, s, p);
}

}  // namespace vf
