// Build-time kernels for Alg. 1: the interleaved list layout of Section 4.2.2
// (StoreInterleaved), per-label membership bitsets for the AND predicate of
// Section 4.3.2, and the final ordering of graph rows.
#include "vf_beam.h"

namespace vf {

// One thread per 16-byte chunk slot: xblk[(g * nchunks + c) * 32 + v].
template <int DT>
__global__ void interleave_kernel(const char *X, int32_t row_bytes, const int32_t *map, const int64_t *grp_src,
                                  const int32_t *grp_cnt, int64_t n, int64_t n_groups, int32_t nchunks, uint4 *xblk)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = n_groups * nchunks * 32;
    if (t >= total) return;
    const int v = (int)(t & 31);
    const int64_t gc = t >> 5;
    const int c = (int)(gc % nchunks);
    const int64_t g = gc / nchunks;
    int64_t src;
    int cnt;
    if (grp_src != nullptr) { src = grp_src[g]; cnt = grp_cnt[g]; }
    else { src = g * 32; cnt = (int)(n - src < 32 ? n - src : 32); }
    uint4 val = make_uint4(0, 0, 0, 0);
    if (v < cnt && c * kChunkBytes < row_bytes)
        val = *(const uint4 *)(X + (int64_t)map[src + v] * row_bytes + c * kChunkBytes);
    xblk[t] = val;
}

// One thread per slot: squared norm of the vector (uint8 after the -128 shift), 0 for padding.
template <int DT>
__global__ void norm_kernel(const char *X, int32_t dim, const int32_t *map, const int64_t *grp_src,
                            const int32_t *grp_cnt, int64_t n, int64_t n_groups, void *xnorm)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_groups * 32) return;
    const int v = (int)(t & 31);
    const int64_t g = t >> 5;
    int64_t src;
    int cnt;
    if (grp_src != nullptr) { src = grp_src[g]; cnt = grp_cnt[g]; }
    else { src = g * 32; cnt = (int)(n - src < 32 ? n - src : 32); }
    if (DT == 0) {
        int acc = 0;
        if (v < cnt) {
            const uint8_t *x = (const uint8_t *)X + (int64_t)map[src + v] * dim;
            for (int e = 0; e < dim; ++e) { const int d = (int)x[e] - 128; acc += d * d; }
        }
        ((int32_t *)xnorm)[t] = acc;
    } else {
        float acc = 0.f;
        if (v < cnt) {
            const float *x = (const float *)X + (int64_t)map[src + v] * dim;
            for (int e = 0; e < dim; ++e) acc += x[e] * x[e];
        }
        ((float *)xnorm)[t] = acc;
    }
}

void launch_interleave(int dtype, const void *X, int32_t dim, const int32_t *map, const int64_t *grp_src,
                       const int32_t *grp_cnt, int64_t n, int64_t n_groups, int32_t ncp, uint4 *xblk, void *xnorm,
                       hipStream_t s)
{
    if (n_groups <= 0) return;
    const int32_t row_bytes = dim * (dtype == 0 ? 1 : 4);
    const int64_t total = n_groups * 2 * ncp * 32;
    const unsigned b1 = (unsigned)((total + 255) / 256), b2 = (unsigned)((n_groups * 32 + 255) / 256);
    if (dtype == 0) {
        hipLaunchKernelGGL(interleave_kernel<0>, dim3(b1), dim3(256), 0, s, (const char *)X, row_bytes, map, grp_src,
                           grp_cnt, n, n_groups, 2 * ncp, xblk);
        hipLaunchKernelGGL(norm_kernel<0>, dim3(b2), dim3(256), 0, s, (const char *)X, dim, map, grp_src, grp_cnt, n,
                           n_groups, xnorm);
    } else {
        hipLaunchKernelGGL(interleave_kernel<1>, dim3(b1), dim3(256), 0, s, (const char *)X, row_bytes, map, grp_src,
                           grp_cnt, n, n_groups, 2 * ncp, xblk);
        hipLaunchKernelGGL(norm_kernel<1>, dim3(b2), dim3(256), 0, s, (const char *)X, dim, map, grp_src, grp_cnt, n,
                           n_groups, xnorm);
    }
}

__global__ void bitset_fill_kernel(const int32_t *map, int64_t n, uint32_t *bits)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    const int32_t g = map[t];
    atomicOr(&bits[g >> 5], 1u << (g & 31));
}

void launch_bitset_fill(const int32_t *map, int64_t n, uint32_t *bits, hipStream_t s)
{
    if (n <= 0) return;
    hipLaunchKernelGGL(bitset_fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, map, n, bits);
}

// uint8: candidates come out of the int8 contraction exact and ordered; copy R of them.
__global__ void graph_rows_copy_kernel(const int32_t *cand_idx, int64_t n, int32_t K, int32_t R, int32_t *G_rows)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * R) return;
    const int64_t j = t / R;
    const int e = (int)(t % R);
    G_rows[t] = cand_idx[j * K + e];
}

// float32: the contraction's |q|^2+|x|^2-2q.x distances are rounded differently from
// the ordered fp32 distance the search uses, so the K > R best candidates are scored
// again with that distance and the R best by (distance, local id) become the row -- if that is provably the
// exact row: every list member the self-join dropped has an approximation >= T (the largest one kept), hence an
// ordered distance >= T - B with B = err_bound (|x_v|^2 + max |x|^2); the row stands when its R-th distance is
// below T - B or nothing was dropped.  Otherwise (near-ties at rank R beyond the K - R spare candidates, data far
// from the origin) the wave scores every member of the list itself.  err_bound < 0: no check (no norms).
// One wave per vertex.
__global__ __launch_bounds__(64) void graph_rows_rerank_kernel(const char *X, int32_t row_bytes, const int32_t *map,
                                                               int64_t n, const int32_t *cand_idx, const uint32_t *cand_bits,
                                                               int32_t K, int32_t R, int32_t *G_rows, float err_bound,
                                                               float xn_max, uint32_t *rescanned)
{
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x, team = lane >> 3, tl = lane & 7;
    const int64_t j = blockIdx.x;
    const int nchunks = row_bytes / kChunkBytes;
    uint4 *qv = smem;
    uint64_t *keys = (uint64_t *)(smem + nchunks);  // [64]
    const char *self = X + (int64_t)map[j] * row_bytes;
    for (int i = lane; i < nchunks; i += 64) qv[i] = *(const uint4 *)(self + i * kChunkBytes);
    keys[lane] = KEY_MAX;
    __syncthreads();
    for (int r0 = 0; r0 < K; r0 += 8) {
        const int my = r0 + team;
        const int c = my < K ? cand_idx[j * K + my] : -1;
        const char *xrow = X + (int64_t)map[c >= 0 ? c : 0] * row_bytes;
        const uint32_t bits = team_dist_bits_f32(qv, xrow, nchunks, tl);
        if (tl == 0 && c >= 0) keys[my] = ((uint64_t)bits << 32) | (uint32_t)c;
    }
    __syncthreads();
    wave_bitonic_sort(keys, 64, lane);
    uint64_t key = keys[lane];
    if (err_bound >= 0.f && n - 1 > K) {   // members were dropped: can one of them belong to the row?
        float vn = 0.f;
        for (int i = lane; i < nchunks; i += 64) {
            const uint4 v = qv[i];
            const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
            vn += f[0] * f[0] + f[1] * f[1] + f[2] * f[2] + f[3] * f[3];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) vn += __shfl_xor(vn, o);
        const float B = err_bound * (vn + xn_max);
        const float T = __uint_as_float(cand_bits[j * K + K - 1]);
        const uint64_t rth = readlane64(key, R - 1);
        const bool proven = rth != KEY_MAX && __uint_as_float((uint32_t)(rth >> 32)) < T - B;
        if (!proven) {   // (wave-uniform) the definition itself
            if (lane == 0 && rescanned != nullptr) atomicAdd(rescanned, 1u);
            uint32_t *dist = (uint32_t *)keys;   // [64]
            TopM<1> ex;
            ex.init(R);
            for (int64_t e0 = 0; e0 < n; e0 += 64) {
                __syncthreads();
                for (int r0 = 0; r0 < 64; r0 += 8) {
                    const int64_t e = e0 + r0 + team;
                    const char *xrow = X + (int64_t)map[e < n ? e : 0] * row_bytes;
                    const uint32_t bits = team_dist_bits_f32(qv, xrow, nchunks, tl);
                    if (tl == 0) dist[r0 + team] = bits;
                }
                __syncthreads();
                const int64_t e = e0 + lane;
                merge_batch(ex, (e < n && e != j) ? ((uint64_t)dist[lane] << 32) | (uint32_t)e : KEY_MAX, lane);
            }
            key = ex.cur[0];
        }
    }
    if (lane < R) G_rows[j * R + lane] = key == KEY_MAX ? -1 : (int32_t)(uint32_t)key;
}

void launch_graph_rows(int dtype, const void *X, int32_t dim, const int32_t *map, int64_t n, const int32_t *cand_idx,
                       const uint32_t *cand_bits, int32_t K, int32_t R, int32_t *G_rows, float err_bound, float xn_max,
                       uint32_t *rescanned, hipStream_t s)
{
    if (n <= 0) return;
    if (dtype == 0) {
        hipLaunchKernelGGL(graph_rows_copy_kernel, dim3((unsigned)((n * R + 255) / 256)), dim3(256), 0, s, cand_idx, n, K,
                           R, G_rows);
    } else {
        const int32_t row_bytes = dim * 4;
        hipLaunchKernelGGL(graph_rows_rerank_kernel, dim3((unsigned)n), dim3(64), (size_t)row_bytes + 64 * 8, s,
                           (const char *)X, row_bytes, map, n, cand_idx, cand_bits, K, R, G_rows, err_bound, xn_max,
                           rescanned);
    }
}

__global__ void graph_global_ids_kernel(const int32_t *rows, const int32_t *map, int64_t count, int32_t *out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const int32_t c = rows[t];
    out[t] = c >= 0 ? map[c] : -1;
}

void launch_graph_global_ids(const int32_t *rows, const int32_t *map, int64_t count, int32_t *out, hipStream_t s)
{
    if (count <= 0) return;
    hipLaunchKernelGGL(graph_global_ids_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, rows, map, count, out);
}

__global__ void fill_out_kernel(int64_t *ids, float *dists, int64_t count)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    ids[t] = -1;
    dists[t] = __builtin_inff();
}

void launch_fill_out(int64_t *ids, float *dists, int64_t count, hipStream_t s)
{
    if (count <= 0) return;
    hipLaunchKernelGGL(fill_out_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, ids, dists, count);
}

__global__ void fill_rows_kernel(int64_t *ids, float *dists, const int32_t *rows, int64_t n_rows, int32_t k)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_rows * k) return;
    const int64_t o = (int64_t)rows[t / k] * k + t % k;
    ids[o] = -1;
    dists[o] = __builtin_inff();
}

void launch_fill_rows(int64_t *ids, float *dists, const int32_t *rows, int64_t n_rows, int32_t k, hipStream_t s)
{
    if (n_rows <= 0) return;
    hipLaunchKernelGGL(fill_rows_kernel, dim3((unsigned)((n_rows * k + 255) / 256)), dim3(256), 0, s, ids, dists, rows,
                       n_rows, k);
}

__global__ void gather_rows_kernel(const uint4 *rows, int32_t chunks, const int32_t *parent, int64_t n, uint4 *out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * chunks) return;
    const int64_t i = t / chunks;
    const int c = (int)(t % chunks);
    out[t] = rows[(int64_t)parent[i] * chunks + c];
}

void launch_gather_rows(const void *rows, int32_t row_bytes, const int32_t *parent, int64_t n, void *out, hipStream_t s)
{
    if (n <= 0) return;
    const int32_t chunks = row_bytes / kChunkBytes;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((n * chunks + 255) / 256)), dim3(256), 0, s, (const uint4 *)rows,
                       chunks, parent, n, (uint4 *)out);
}

// One wave per query.  Keys (id << 32 | distance bits) sorted: equal ids become neighbours with the
// smallest distance first; the survivors, re-keyed (distance bits << 32 | id), are sorted again.
// Distances are non-negative floats, whose bit patterns order like the values.
__global__ __launch_bounds__(64) void multi_merge_kernel(const int32_t *first, const int64_t *sub_ids, const float *sub_dists,
                                                         int32_t k, int32_t P, int64_t *out_ids, float *out_dists)
{
    extern __shared__ uint4 smem[];
    uint64_t *keys = (uint64_t *)smem;        // [P]
    uint64_t *keys2 = keys + P;               // [P]
    const int lane = threadIdx.x;
    const int64_t q = blockIdx.x;
    const int64_t lo = first[q], hi = first[q + 1];
    const int total = (int)(hi - lo) * k;
    for (int i = lane; i < P; i += 64) {
        uint64_t key = KEY_MAX;
        if (i < total) {
            const int64_t id = sub_ids[lo * k + i];
            if (id >= 0) key = ((uint64_t)id << 32) | __float_as_uint(sub_dists[lo * k + i]);
        }
        keys[i] = key;
    }
    __syncthreads();
    wave_bitonic_sort(keys, P, lane);
    for (int i = lane; i < P; i += 64) {
        const uint64_t key = keys[i];
        const bool keep = key != KEY_MAX && (i == 0 || (keys[i - 1] >> 32) != (key >> 32));
        keys2[i] = keep ? ((key << 32) | (key >> 32)) : KEY_MAX;
    }
    __syncthreads();
    wave_bitonic_sort(keys2, P, lane);
    if (lane < k) {
        const uint64_t key = lane < P ? keys2[lane] : KEY_MAX;
        const bool none = key == KEY_MAX;
        out_ids[q * k + lane] = none ? -1 : (int64_t)(uint32_t)key;
        out_dists[q * k + lane] = none ? __builtin_inff() : __uint_as_float((uint32_t)(key >> 32));
    }
}

void launch_multi_merge(const int32_t *first, int64_t nq, const int64_t *sub_ids, const float *sub_dists, int32_t k,
                        int64_t *out_ids, float *out_dists, hipStream_t s)
{
    if (nq <= 0) return;
    int32_t P = 64;
    while (P < (kMaxOthers + 1) * k) P <<= 1;
    hipLaunchKernelGGL(multi_merge_kernel, dim3((unsigned)nq), dim3(64), (size_t)P * 16, s, first, sub_ids, sub_dists, k, P,
                       out_ids, out_dists);
}

}  // namespace vf
