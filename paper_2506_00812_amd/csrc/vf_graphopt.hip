// Graph optimisation of the per-list graphs (index build, optional): a degree-D exact kNN graph is
// reduced to degree R by rank-based pruning and reverse edges, the graph optimisation of the CAGRA
// paper (Ootomo et al. 2023, Section 3.2) that the paper's BuildCAGRAGraph (Alg. 1) stands for.
// All of it is integer work on ranks and ids; the rules, fixed where that description leaves
// freedom so that the result is unique:
//   1. pruning    edge x -> y_j (rank j of x's row) has c_j detours: pairs (i, r), i < j, r < j, with
//                 y_j at rank r of y_i's row.  The R edges with the smallest (c_j, j) are kept in that
//                 order: the forward row F[x].
//   2. reverse    every edge x -> y at position p of F[x] proposes x to y; the R proposals with the
//                 smallest (p, x) form B[y].
//   3. merge      row of y = F[y][0 .. R/2), then the first R - R/2 entries of B[y] not among those,
//                 then the remaining entries of F[y], in order, not yet in the row.
// Vertices are addressed by their position g in the compacted graph partition (all lists one after
// the other); node_base[g] is the position of the first vertex of g's list, so local id = g - base.
#include "vf_device.h"

namespace vf {

// ---------------------------------------------------------------- step 1: one wave per vertex

__global__ __launch_bounds__(64) void graph_prune_kernel(const int32_t *knn, const int32_t *node_base, int32_t D,
                                                         int32_t R, int32_t *F)
{
    __shared__ int32_t tab_key[128];   // open-addressing table: local id -> rank in this vertex's row
    __shared__ int32_t tab_pos[128];
    __shared__ int32_t cnt[64];
    const int lane = threadIdx.x;
    const int64_t g = blockIdx.x;
    const int64_t base = node_base[g];
    const int32_t y = lane < D ? knn[g * D + lane] : -1;
    tab_key[lane] = -1; tab_key[lane + 64] = -1;
    cnt[lane] = 0;
    __syncthreads();
    if (y >= 0) {   // the ids of a row are distinct: every insertion claims a slot of its own
        uint32_t h = ((uint32_t)y * 2654435761u) >> 25;
        while (atomicCAS(&tab_key[h], -1, y) != -1) h = (h + 1) & 127;
        tab_pos[h] = lane;
    }
    __syncthreads();
    // rows of the D neighbours, four at a time (their loads are issued before the first is used)
    for (int i0 = 0; i0 < D; i0 += 4) {
        int32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u;
            const int32_t yi = __shfl(y, i < D ? i : 0);
            v[u] = (i < D && yi >= 0 && lane < D) ? knn[(base + yi) * D + lane] : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u;
            if (v[u] < 0) continue;
            uint32_t h = ((uint32_t)v[u] * 2654435761u) >> 25;
            int j = -1;
            for (;;) {
                const int32_t k = tab_key[h];
                if (k == v[u]) { j = tab_pos[h]; break; }
                if (k == -1) break;
                h = (h + 1) & 127;
            }
            if (j > i && j > lane) atomicAdd(&cnt[j], 1);   // lane = rank r of v in y_i's row
        }
    }
    __syncthreads();
    uint32_t key = (lane < D && y >= 0) ? ((uint32_t)cnt[lane] << 8) | (uint32_t)lane : 0xFFFFFFFFu;
    key = wave_sort_u32(key, lane);
    const int32_t kept = __shfl(y, key == 0xFFFFFFFFu ? 0 : (int)(key & 0xFFu));
    if (lane < R) F[g * R + lane] = key == 0xFFFFFFFFu ? -1 : kept;
}

// ---------------------------------------------------------------- step 2: proposals grouped by target

__global__ void graph_indegree_kernel(const int32_t *F, const int32_t *node_base, int64_t n_nodes, int32_t R,
                                      int32_t *deg)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_nodes * R) return;
    const int32_t y = F[t];
    if (y >= 0) atomicAdd(&deg[node_base[t / R] + y], 1);
}

// seg[off[y] + slot] = (p << 32 | local id of x): the slot order is arbitrary, step 3 selects by key
__global__ void graph_reverse_fill_kernel(const int32_t *F, const int32_t *node_base, int64_t n_nodes, int32_t R,
                                          const int64_t *off, int32_t *cursor, uint64_t *seg)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_nodes * R) return;
    const int32_t y = F[t];
    if (y < 0) return;
    const int64_t g = t / R;
    const int32_t base = node_base[g];
    const int64_t gy = (int64_t)base + y;
    const int32_t slot = atomicAdd(&cursor[gy], 1);
    seg[off[gy] + slot] = ((uint64_t)(uint32_t)(t % R) << 32) | (uint32_t)(g - base);
}

// ---------------------------------------------------------------- step 3: one wave per vertex

__global__ __launch_bounds__(64) void graph_reverse_merge_kernel(const int32_t *F, const int64_t *off,
                                                                 const uint64_t *seg, int32_t R, int32_t *G)
{
    const int lane = threadIdx.x;
    const int64_t y = blockIdx.x;
    const int64_t beg = off[y], end = off[y + 1];
    // the R smallest proposals, ascending, one per lane (lanes >= R hold KEY_MAX)
    uint64_t best = KEY_MAX;
    for (int64_t c = beg; c < end; c += 64) {
        uint64_t v = c + lane < end ? seg[c + lane] : KEY_MAX;
        const uint64_t kth = shfl64(best, R - 1);
        if (!__any(v < kth)) continue;
        v = wave_sort64(v, lane);
        const uint64_t vr = shfl64(v, 63 - lane);      // descending
        const uint64_t m = best < vr ? best : vr;      // the 64 smallest of both, bitonic
        best = wave_merge64(m, lane);
        if (lane >= R) best = KEY_MAX;
    }
    const int32_t b = (lane < R && best != KEY_MAX) ? (int32_t)(uint32_t)best : -1;
    const int32_t f = lane < R ? F[y * R + lane] : -1;
    const int half = R / 2, quota = R - half;
    bool in_p = false;
    for (int t = 0; t < half; ++t) {
        const int32_t ft = __shfl(f, t);
        in_p = in_p || (b >= 0 && b == ft);
    }
    const bool keep_b = b >= 0 && !in_p;
    const uint64_t mb = __ballot(keep_b);
    const int rank_b = __popcll(mb & ((1ull << lane) - 1ull));
    const bool sel_b = keep_b && rank_b < quota;
    const int nb = min(__popcll(mb), quota);
    const int32_t b_sel = sel_b ? b : -1;
    bool in_b = false;
    for (int t = 0; t < R; ++t) {
        const int32_t bt = __shfl(b_sel, t);
        in_b = in_b || (bt >= 0 && bt == f);
    }
    const bool keep_f = lane >= half && lane < R && f >= 0 && !in_b;
    const uint64_t mf = __ballot(keep_f);
    const int rank_f = __popcll(mf & ((1ull << lane) - 1ull));
    const int need = R - half - nb;
    const bool sel_f = keep_f && rank_f < need;
    const int total = half + nb + min(__popcll(mf), need);
    int32_t *row = G + y * R;
    if (lane < half) row[lane] = f;
    if (sel_b) row[half + rank_b] = b;
    if (sel_f) row[half + nb + rank_f] = f;
    if (lane >= total && lane < R) row[lane] = -1;
}

// out[g][e] = M[node_base[g] + rows[g][e]] (-1 stays -1): graph rows as global ids
__global__ void graph_global_ids_based_kernel(const int32_t *rows, const int32_t *node_base, const int32_t *M,
                                              int64_t n_nodes, int32_t R, int32_t *out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_nodes * R) return;
    const int32_t c = rows[t];
    out[t] = c >= 0 ? M[(int64_t)node_base[t / R] + c] : -1;
}

// ---------------------------------------------------------------- launchers

void launch_graph_prune(const int32_t *knn, const int32_t *node_base, int64_t n_nodes, int32_t D, int32_t R, int32_t *F,
                        hipStream_t s)
{
    if (n_nodes <= 0) return;
    hipLaunchKernelGGL(graph_prune_kernel, dim3((unsigned)n_nodes), dim3(64), 0, s, knn, node_base, D, R, F);
}

void launch_graph_indegree(const int32_t *F, const int32_t *node_base, int64_t n_nodes, int32_t R, int32_t *deg,
                           hipStream_t s)
{
    if (n_nodes <= 0) return;
    hipLaunchKernelGGL(graph_indegree_kernel, dim3((unsigned)((n_nodes * R + 255) / 256)), dim3(256), 0, s, F, node_base,
                       n_nodes, R, deg);
}

void launch_graph_reverse_fill(const int32_t *F, const int32_t *node_base, int64_t n_nodes, int32_t R, const int64_t *off,
                               int32_t *cursor, uint64_t *seg, hipStream_t s)
{
    if (n_nodes <= 0) return;
    hipLaunchKernelGGL(graph_reverse_fill_kernel, dim3((unsigned)((n_nodes * R + 255) / 256)), dim3(256), 0, s, F,
                       node_base, n_nodes, R, off, cursor, seg);
}

void launch_graph_reverse_merge(const int32_t *F, const int64_t *off, const uint64_t *seg, int64_t n_nodes, int32_t R,
                                int32_t *G, hipStream_t s)
{
    if (n_nodes <= 0) return;
    hipLaunchKernelGGL(graph_reverse_merge_kernel, dim3((unsigned)n_nodes), dim3(64), 0, s, F, off, seg, R, G);
}

void launch_graph_global_ids_based(const int32_t *rows, const int32_t *node_base, const int32_t *M, int64_t n_nodes,
                                   int32_t R, int32_t *out, hipStream_t s)
{
    if (n_nodes <= 0) return;
    hipLaunchKernelGGL(graph_global_ids_based_kernel, dim3((unsigned)((n_nodes * R + 255) / 256)), dim3(256), 0, s, rows,
                       node_base, M, n_nodes, R, out);
}

}  // namespace vf
