// Internal declarations shared by the host code and the gfx950 kernels.
// Nothing here is part of the C ABI (see include/vecflow.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

namespace vf {

constexpr uint64_t KEY_MAX = ~0ull;
constexpr int kGroup = 32;       // vectors per interleaved group (Section 4.2.2)
constexpr int kChunkBytes = 16;  // bytes per interleaved chunk  (Section 4.2.2)
constexpr int kMaxOthers = 7;    // AND partners per query besides the searched label
constexpr int kSeedChunk = 16;   // seeds per wave of the dense seed kernel

// Per-label metadata on the device, used by the predicate and by the kernels to
// slice a label's part of the compacted arrays (S, O, M of Alg. 1).
struct LabelMeta {
    const int32_t *S;        // [n_labels] |C_l|
    const int64_t *O_HS;     // [n_labels] start in M_HS / graph rows, -1 if none
    const int64_t *O_LS;     // [n_labels] start in M_LS, -1 if none
    const int32_t *hs_slot;  // [n_labels] rank among graph labels (bitset row), -1 if none
    const int32_t *M_HS;
    const int32_t *M_LS;
    const uint32_t *bitsets; // [n_graph_labels][bitset_words]
    int64_t bitset_words;
};

// ---------------------------------------------------------------- scan / contraction kernel

// One wave's work: a tile of <= 32 queries against one segment of a list.
struct ScanItem {
    int64_t group0;    // first 32-vector group of the segment in the interleaved buffer
    int64_t map_off;   // start of the list in `map` (local -> global id)
    int32_t entry0;    // list-relative index of the segment's first entry
    int32_t n;         // entries in the segment
    int32_t q_begin;   // first tile row in qrow[]
    int32_t q_count;   // tile rows, 1..32
    int32_t self_base; // >= 0: list entry self_base + r is skipped for tile row r (graph build)
    int32_t part_row;  // >= 0: K candidates of tile row r go to partial row part_row + r; < 0: final output
};

// Merge of the per-segment candidates of one query into its final top-k.
struct MergeItem {
    int64_t map_off;   // start of the list in `map`
    int32_t qrow;      // query index (output row)
    int32_t part_row;  // partial row of segment 0
    int32_t stride;    // partial rows between consecutive segments
    int32_t nseg;
    int32_t n;         // entries of the list
    int32_t pad;
};

struct ScanParams {
    const uint4 *xblk;      // [group][2*ncp][32] 16-byte chunks
    const void *xnorm;      // per slot (group*32 + lane): float (f32) / int32 (u8, after -128 shift)
    const int32_t *map;
    const void *qsrc;       // row-major [*][dim] query rows
    const int32_t *qrow;    // row of qsrc for each tile row
    const ScanItem *items;
    int32_t dim, ncp, K;
    int32_t tile_rows;      // rows of the largest tile (LDS buffers are sized for it), <= 32
    // Panel mode (scan_topk16_kernel, panel_n > 0): every item of the launch covers only list entries
    // [panel_entry0, panel_entry0 + panel_n) of its list (multiples of 32); with carry != 0 a row's K best
    // start from the partial row a previous launch left in res_idx / res_bits.  Launching the panels of a
    // long list one after the other keeps all resident waves on the same few megabytes, which every XCD's L2
    // then serves: the kNN self-join of a 400,000-vector list is otherwise bound by HBM bandwidth.
    int32_t panel_entry0, panel_n, carry;
    int64_t *out_ids;       // final output [*][K] (items with part_row < 0): row = qrow value
    float *out_dists;
    int32_t *res_idx;       // partial output [*][K]: list-relative entry index, -1 = none
    uint32_t *res_bits;     //                        distance bits (float bits / integer)
    const int32_t *others_off; // [*] per query row value: AND partner labels (mode 0 only), may be null
    const int32_t *others;
    LabelMeta meta;
};

void launch_scan(int dtype, const ScanParams &p, int n_items, hipStream_t s);
// float32, dim 96 / 128, <= 16 queries per tile, no self exclusion: 16-row matrix-core tiles
bool scan16_supported(int dtype, int dim, int tile_rows);
void launch_scan16(const ScanParams &p, int n_items, hipStream_t s);
// float32, dim 96 / 128, <= 16 queries per tile, no self exclusion: FMAs with scalar query operands
bool scan_valu_supported(int dtype, int dim, int tile_rows);
void launch_scan_valu(const ScanParams &p, int n_items, hipStream_t s);
void launch_scan_merge(int dtype, const MergeItem *items, int n_items, const int32_t *res_idx, const uint32_t *res_bits,
                       int32_t K, int32_t max_keys, const int32_t *map, int64_t *out_ids, float *out_dists,
                       hipStream_t s);

// float32 lists filtered from their bfloat16 copy (scan_bf16_kernel: xblk holds chunks of 8 bfloat16 components,
// xnorm the norms of the unrounded vectors, K = candidates kept per query and segment, every item writes partial
// rows), then re-ranked: per query the Kc best approximations of all its segments are re-scored with the ordered
// float32 distance from the vector table; the k best of them are the result if the proof holds that no dropped
// candidate can be among them, else the query's wave scans the whole list with the ordered distance.
struct RerankParams {
    const MergeItem *items;
    const int32_t *res_idx;     // partial rows [*][Kc]
    const uint32_t *res_bits;
    const int32_t *map;         // local -> global id of the scan partition
    const void *X;              // vector table, row-major
    const void *Q;
    int32_t dim, Kc, K;
    float err_bound, xn_max, err_q;   // |approximation - ordered distance| <= err_bound (|q|^2 + xn_max) + err_q |q|
    uint32_t *fail_count;       // incremented once per query whose proof failed
    const int32_t *others_off;  // AND partner labels per query; null when the batch has none
    const int32_t *others;
    LabelMeta meta;
    int64_t *out_ids;
    float *out_dists;
};
bool scan_bf16_supported(int dtype, int dim, int tile_rows, int keep);
size_t scan_bf16_lds_bytes(int tile_rows, int keep);
void launch_scan_bf16(const ScanParams &p, int n_items, int slots, hipStream_t s);
void launch_scan_rerank(const RerankParams &p, int n_items, hipStream_t s);

// ---------------------------------------------------------------- beam search kernel

struct BeamParams {
    const void *X;           // global vectors, row-major [n][dim]
    const void *Q;           // queries, row-major [nq][dim]
    const int32_t *G;        // [n_HS][R] local ids
    const int32_t *Gg;       // [n_HS][R] the same rows as global ids (-1 where G is -1)
    const int32_t *gq_query; // [n_gq] query index
    const int32_t *gq_label; // [n_gq] searched label
    const int32_t *others_off;
    const int32_t *others;
    LabelMeta meta;
    int32_t dim, R, k, itopk, width, iters, n_seeds;
    int32_t LP;        // list slots (power of two >= itopk + width*R)
    int32_t hash_bits; // visited table has 1 << hash_bits slots
    int64_t *out_ids;
    float *out_dists;
    int32_t *counters; // optional [nq][4]: distances computed, rows expanded, predicate tests, method
    int32_t *gathered; // optional [nq]: distances whose vector the kernel fetched itself
    const uint32_t *dseed; // optional [n_gq][ns_stride]: seed distance bits from seed_dist_kernel / seed_mfma_kernel
    int32_t ns_stride;
    // dseed holds MFMA approximations (float32 only): the kernel re-scores the best of them with the
    // ordered distance and proves, with B = err_bound * (|q|^2 + xn_max) + err_q * |q|, that no other seed can matter
    int32_t seed_approx;
    int32_t seed_keep;  // approximations kept for re-ranking (itopk < seed_keep <= 64)
    float err_bound, xn_max;
    uint32_t *fallback_count;  // optional: incremented once per query whose proof failed
    float err_q;        // 0 unless the seeds were scored from their bfloat16 copy: 2 * max |x - bf16(x)| over the seeds
    // seeds scored with the selection fused in (seed_select_kernel; itopk <= 64): per query run_segs runs of run_K
    // keys, of which the first ceil(min(n_seeds, |C_l|) / seg_seeds) exist.  uint8: exact distances; float32:
    // approximations (seed_approx != 0, run_K == seed_keep)
    const uint64_t *seed_runs;
    int32_t run_K, run_segs, seg_seeds;
    const int32_t *seed_pass;  // optional (profiling, AND batches): seeds of the query that pass its predicate
    // optional (AND batches with a dense seed distance matrix): global ids of the seeds of every graph list in seed
    // order, 32-seed groups, first group of a list at seed_goff[rank of the list among graph lists] -- consecutive
    // seeds at consecutive addresses, where M_HS holds them floor(n / n_seeds) entries apart
    const int32_t *seed_map;
    const int64_t *seed_goff;
    int32_t lat_waves;         // launches of at most this many graph queries (itopk <= 64) run the latency instantiation
    // optional: an interleaved copy of the seeds (uint8 or float32, never bfloat16) from which a wave scores its
    // seeds itself when no dense seed kernel ran (the serving kernel); sgoff: first group of each graph list
    const uint4 *sblk;
    const int64_t *sgoff;
    int32_t sblk_chunks;       // 16-byte chunks per vector in that copy (the even count of the interleaved layout)
};

// ---------------------------------------------------------------- dense seed distances

struct SeedTile {
    int32_t label;
    int32_t gq_begin;  // first graph query (position in gq_query) of the tile
    int32_t q_count;   // queries, all searching `label`: 1..64 (seed_dist_kernel), 1..32 (seed_mfma_kernel)
};

struct SeedParams {
    const void *X;
    const void *Q;
    const int32_t *gq_query;
    const SeedTile *tiles;
    LabelMeta meta;
    int32_t dim, n_seeds, ns_stride, max_chunks;  // max_chunks = seed chunks per tile (kSeedChunk or kSeedMfmaChunk seeds each)
    uint32_t *dseed;
    const uint32_t *xnorm_all;  // [n] squared norms of the rows of X, float bits / int32 of the -128 shifted bytes (seed_mfma_kernel only)
    // seed_mfma_kernel, optional: the seeds of every graph list for this n_seeds as an interleaved copy
    // ([group][chunk][32] 16-byte chunks like a scan list, 32 seeds per group in seed order, zero padded)
    const uint4 *seed_blk;
    int32_t seed_bf16;          // float32 data: seed_blk holds the seeds rounded to bfloat16 (chunks of 8 components)
    const uint32_t *seed_norm;  // [group * 32 + v] squared norms as in xnorm_all
    const int64_t *seed_goff;   // [n_graph_labels] first group of each graph list, by rank among graph labels
    int32_t chunk_seeds;        // seeds per wave: kSeedMfmaChunk, or four times that (interleaved copy only); max_chunks matches it
    int64_t dump_off;           // seed_mfma_kernel: dseed[dump_off .. dump_off + 64 * (dump_mask + 1)) takes the stores of
    int32_t dump_mask;          // lanes without a pair, 64 entries per workgroup index & dump_mask (2^k - 1)
};

// Seed scoring with fused selection (seed_select_kernel): one run of K keys per (graph query, seed segment)
struct SeedSelParams {
    const void *Q;
    const int32_t *gq_query;
    const SeedTile *tiles;      // tiles of <= 32 graph queries of one label
    LabelMeta meta;
    int32_t dim, n_seeds;
    int32_t K;                  // keys kept per (query, segment), <= 64
    int32_t seg_seeds;          // seeds per segment, a multiple of 32
    int32_t max_segs;           // segments per tile in the grid: ceil(min(n_seeds, longest list of the batch) / seg_seeds)
    const uint4 *seed_blk;      // interleaved copy of the seeds: uint8, or bfloat16 for float32 data
    const uint32_t *seed_norm;  // [group * 32 + v] squared norms (int32 of the -128 shifted bytes / float bits)
    const int64_t *seed_goff;   // [n_graph_labels] first group of each graph list
    const int32_t *seed_map;    // [group * 32 + v] global id of the seed (AND predicate)
    const int32_t *others_off;  // AND partner labels per query; null when the batch has none
    const int32_t *others;
    uint64_t *runs;             // [n_gq][max_segs][K]: (value bits << 32 | seed index), ascending, KEY_MAX = none
};
bool seed_select_supported(int dtype, int dim, bool bf16_copy);
size_t seed_select_lds_bytes(int32_t K);
void launch_seed_select(int dtype, const SeedSelParams &p, int n_tiles, hipStream_t s);
void launch_seed_pass_count(const int32_t *gq_query, const int32_t *gq_label, const LabelMeta &meta, int32_t n_seeds,
                            const int32_t *others_off, const int32_t *others, int32_t *pass_count, int n_gq, hipStream_t s);

// seed_map[g * 32 + v] = global id of seed j = grp_j0[g] + v of graph list grp_slot[g] (local id floor(j n / ns)),
// 0 for v beyond the list's seeds
void launch_seed_pack_bf16(const uint4 *blk32, int64_t n_groups, int32_t nch16, uint4 *blk16, float *err2, hipStream_t s);
void launch_seed_map(const int32_t *M_HS, const int64_t *slot_base, const int32_t *slot_n, int32_t n_seeds,
                     const int32_t *grp_slot, const int32_t *grp_j0, int64_t n_groups, int32_t *seed_map, hipStream_t s);

constexpr int kSeedMfmaChunk = 128;  // seeds per wave of the MFMA seed kernel when it gathers rows (four 32-seed groups)

bool seed_dist_supported(int dtype, int dim);
void launch_seed_dist(int dtype, const SeedParams &p, int n_tiles, hipStream_t s);
// |q|^2 + |x|^2 - 2 q.x through the matrix cores: approximate for float32, exact for uint8
bool seed_mfma_supported(int dtype, int dim);
void launch_seed_mfma(int dtype, const SeedParams &p, int n_tiles, hipStream_t s);
// squared norms of all rows of a table (float bits, or int32 of the -128 shifted bytes)
void launch_row_norms(int dtype, const void *X, int32_t dim, int64_t n, uint32_t *out, hipStream_t s);

size_t beam_lds_bytes(const BeamParams &p, int dtype);
void launch_beam(int dtype, const BeamParams &p, int n_gq, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);

// ---------------------------------------------------------------- build-time kernels

// Interleave `n_groups` groups of 32 vectors gathered through `map` (Section 4.2.2
// layout) and compute their norms.  grp_src/grp_cnt give, per group, the first
// position in `map` and the number of valid vectors; with grp_src == nullptr group
// g covers map[g*32 .. min(n, g*32+32)).
void launch_interleave(int dtype, const void *X, int32_t dim, const int32_t *map, const int64_t *grp_src,
                       const int32_t *grp_cnt, int64_t n, int64_t n_groups, int32_t ncp, uint4 *xblk, void *xnorm,
                       hipStream_t s);

void launch_bitset_fill(const int32_t *map, int64_t n, uint32_t *bits, hipStream_t s);

// Graph rows from candidate lists: u8 copies the first R candidates (already exact);
// f32 re-scores K candidates with the ordered fp32 distance and keeps the best R, provided that no member the
// self-join dropped can belong to the row (cand_bits: the candidates' approximate distances; err_bound, xn_max:
// |approximation - ordered distance| <= err_bound (|x_v|^2 + xn_max); err_bound < 0: unchecked); a row without
// that proof is computed from every member of the list and counted in *rescanned (optional).
void launch_graph_rows(int dtype, const void *X, int32_t dim, const int32_t *map, int64_t n, const int32_t *cand_idx,
                       const uint32_t *cand_bits, int32_t K, int32_t R, int32_t *G_rows, float err_bound, float xn_max,
                       uint32_t *rescanned, hipStream_t s);

// out[i] = map[rows[i]] (rows[i] >= 0), -1 otherwise: graph rows as global ids
void launch_graph_global_ids(const int32_t *rows, const int32_t *map, int64_t count, int32_t *out, hipStream_t s);
void launch_fill_out(int64_t *ids, float *dists, int64_t count, hipStream_t s);
// rows[i] of the [*][k] outputs := (-1, +inf)
void launch_fill_rows(int64_t *ids, float *dists, const int32_t *rows, int64_t n_rows, int32_t k, hipStream_t s);

// ---------------------------------------------------------------- graph optimisation (vf_graphopt.hip)

// Vertices are positions g in the compacted graph partition; node_base[g] = position of the first vertex of
// g's list.  knn: [n_nodes][D] local ids in rank order; F, G: [n_nodes][R] local ids.
void launch_graph_prune(const int32_t *knn, const int32_t *node_base, int64_t n_nodes, int32_t D, int32_t R, int32_t *F,
                        hipStream_t s);
void launch_graph_indegree(const int32_t *F, const int32_t *node_base, int64_t n_nodes, int32_t R, int32_t *deg,
                           hipStream_t s);
void launch_graph_reverse_fill(const int32_t *F, const int32_t *node_base, int64_t n_nodes, int32_t R, const int64_t *off,
                               int32_t *cursor, uint64_t *seg, hipStream_t s);
void launch_graph_reverse_merge(const int32_t *F, const int64_t *off, const uint64_t *seg, int64_t n_nodes, int32_t R,
                                int32_t *G, hipStream_t s);
void launch_graph_global_ids_based(const int32_t *rows, const int32_t *node_base, const int32_t *M, int64_t n_nodes,
                                   int32_t R, int32_t *out, hipStream_t s);

// ---------------------------------------------------------------- multi-label queries (OR, parallel AND)

// out[i] = row parent[i] of a row-major table (rows of row_bytes, a multiple of 16)
void launch_gather_rows(const void *rows, int32_t row_bytes, const int32_t *parent, int64_t n, void *out, hipStream_t s);
// Query j owns the sub-search results first[j] .. first[j+1] (<= 8 rows of k (id, distance) pairs, id -1 = none):
// an id found more than once keeps its smallest distance; the k best by (distance, id) are written.
void launch_multi_merge(const int32_t *first, int64_t nq, const int64_t *sub_ids, const float *sub_dists, int32_t k,
                        int64_t *out_ids, float *out_dists, hipStream_t s);

// ---------------------------------------------------------------- errors

void set_error(const std::string &msg);
const char *last_error();

}  // namespace vf
