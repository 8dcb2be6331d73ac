// Graph-search initialisation (Section 4.2.1: the initial candidates are sampled
// inside the label's list): distances from every graph query to the seeds of its
// label, computed densely.
//
// The seeds of a label -- local ids floor(j * n / ns) -- do not depend on the query,
// so all queries of a label score the same vectors.  Instead of every query gathering
// its seeds from HBM, one wave takes up to 64 queries of one label (one query per lane,
// the query vector held in registers) and a chunk of kSeedChunk seeds; a seed vector is the
// same for all lanes, so it is fetched with scalar loads and used as a scalar operand: the
// seed vectors are fetched once per 64 queries and the inner loop is pure VALU work with
// no LDS or cross-lane traffic.  A lane evaluates the
// distance in exactly the order the 8-lane teams of the beam kernel use (partial sum t
// takes the 16-byte chunks 8s + t, fused multiply-add, fixed tree), so the bits are
// identical to a gathered evaluation and to the CPU evaluation.
//
// Output: dseed[gq][j] = distance bits of graph query gq to seed j, consumed by the
// beam kernel, which keeps the best itopk.
#include "vf_device.h"

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
