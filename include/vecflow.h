/*
 * vecflow.h -- C ABI of the MI355X (gfx950) label-filtered top-k search library.
 *
 * The library implements the query hot path of the dual-structured
 * label-centric inverted index of arXiv 2506.00812: every label l owns a
 * posting list C_l of vector ids (Section 4.1.2); lists with |C_l| >= T are
 * searched by beam search over a per-label proximity graph ("IVF-Graph",
 * Section 4.2.1, Alg. 2), smaller lists are scanned exhaustively ("IVF-BFS",
 * Section 4.2.2); multi-label AND queries search the smallest of their lists and
 * test the remaining labels with a predicate (Section 4.3.2).
 *
 * Conventions
 *   - Every function returns VF_OK (0) or a negative error code and never throws
 *     or aborts.  vf_last_error() returns a thread-local message for the last
 *     failing call of the calling thread.
 *   - "device" pointers are HIP device memory on the current device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes.
 *   - Distances are squared Euclidean (no square root).
 *   - dtype VF_U8: uint8 vectors, integer-exact distances (exactly representable in
 *     the float output for dim <= 258).  dtype VF_F32: float32 vectors.
 *   - Supported shapes: VF_U8 needs dim % 16 == 0, VF_F32 needs dim % 4 == 0;
 *     16 <= dim*sizeof(elem) <= 992 (a 32-row tile of the contraction kernel, its query rows and its
 *     candidate queues, must fit the 64 KiB of LDS a workgroup may use); n < 2^31.
 */
#ifndef VECFLOW_H
#define VECFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VF_OK 0
#define VF_EINVAL (-1) /* bad shape / dtype / parameter / label id            */
#define VF_ENOMEM (-2) /* host or device allocation failed                     */
#define VF_EHIP (-3)   /* a HIP runtime call failed; text in vf_last_error()   */
#define VF_EINTERNAL (-4) /* an unexpected failure inside the library (a C++ exception caught at the boundary) */
#define VF_EBUSY (-5)  /* vf_serve_submit: the job ring is full, try again                */

#define VF_U8 0
#define VF_F32 1

typedef struct vf_index vf_index; /* opaque; owned by the library */

/*
 * Device allocator supplied by the caller (for instance PyTorch's caching allocator), so that the index and
 * its workspaces live in memory the caller's framework accounts for.
 *   alloc   returns `bytes` of device memory on the current device, aligned to at least 256 bytes, or NULL
 *           when it has none (the call in progress then fails with VF_ENOMEM); must not throw
 *   free    takes back a pointer alloc returned; the library calls it only after all work that used the
 *           memory has completed on the device
 *   ctx     passed through to both
 * The struct is copied by vf_build_index; the functions and ctx must stay valid until vf_index_free returns.
 * Every device allocation of the index goes through it: the arrays of Alg. 1 at build time, and the
 * per-stream workspaces and seed copies that searches create or grow on demand.  Pinned host staging buffers
 * are the library's own (hipHostMalloc).
 */
typedef struct vf_allocator {
    void *(*alloc)(size_t bytes, void *ctx);
    void (*free)(void *ptr, void *ctx);
    void *ctx;
} vf_allocator;

/*
 * Index construction (Alg. 1; layout of Section 4.2.1 "redundancy bypassing" and
 * Section 4.2.2 "interleaved" lists).
 *
 *   vectors        device, row-major [n][dim], dtype as given.  NOT copied: the
 *                  index references this single global table X and the caller must
 *                  keep it alive and unmodified for the index's lifetime.
 *   label_offsets  host, [n+1], CSR over label_ids
 *   label_ids      host, labels of each vector in any order; duplicates allowed
 *   n_labels       vocabulary size; every id must lie in [0, n_labels)
 *   T              specificity threshold on the posting-list size: |C_l| >= T ->
 *                  graph list, 0 < |C_l| < T -> scan list (Section 4.1.1-4.1.2)
 *   graph_degree   R, out-degree of each per-label graph; needs 1 <= R <= 64 and
 *                  T >= R + 1
 *   allocator      device allocator for everything the index holds (see vf_allocator);
 *                  NULL = hipMalloc / hipFree
 *   hip_stream     hipStream_t (NULL = default stream); the call returns after the
 *                  build has completed on it
 *   out            receives the index
 *
 * Per label the library keeps S (size), O (offset) and M (local -> global id map),
 * separately for the graph ("HS") and scan ("LS") partitions, both compacted in
 * ascending label id.  Posting lists are in ascending global id.  A graph list's
 * rows are the exact R nearest other members of the list, as local ids, ordered by
 * (distance, local id); for float32 data, distance is the ordered float32 distance the search uses (a row taken
 * from the matrix-core self-join's candidates is kept only with a proof that no other member can belong to it,
 * and is otherwise computed from every member of the list).
 */
int vf_build_index(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                   const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                   const vf_allocator *allocator, void *hip_stream, vf_index **out);

/*
 * The same index with the per-list graphs the paper's BuildCAGRAGraph (Alg. 1) stands for in its second
 * half: graph optimisation as in the CAGRA paper (Ootomo et al. 2023, Section 3.2).  Every graph list gets
 * an exact kNN graph of degree knn_degree = D, which is then reduced to graph_degree = R using ranks only:
 *   1. the edge x -> y_j (rank j in x's row) is detourable through y_i, i < j, when y_j stands at a rank
 *      r < j in y_i's row; the R edges with the fewest such (i, r) pairs (ties: lower rank) are kept, in
 *      that order;
 *   2. every kept edge x -> y at position p proposes the reverse edge y -> x; a vertex keeps the R
 *      proposals with the smallest (p, x);
 *   3. row = the first R/2 kept edges, then up to R - R/2 reverse edges not among them, then the
 *      remaining kept edges, in order, until the row holds R entries.
 *
 *   graph_kind   VF_GRAPH_KNN: exactly vf_build_index (knn_degree must be 0);
 *                VF_GRAPH_PRUNED: as described above
 *   knn_degree   D; 0 = min(2 R, 64) for uint8, min(2 R, 48) for float32, which are also the largest
 *                values accepted (the self-join keeps 64 candidates per vertex and float32 rows are
 *                re-ranked out of 16 more candidates than they keep).  Needs R <= D and T >= D + 1.
 * All other arguments, ownership and errors as for vf_build_index.  Searches do not depend on graph_kind.
 */
#define VF_GRAPH_KNN 0
#define VF_GRAPH_PRUNED 1
int vf_build_index_opt(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                       const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                       int32_t graph_kind, int32_t knn_degree, const vf_allocator *allocator, void *hip_stream,
                       vf_index **out);

/*
 * Batched label-filtered top-k search (Alg. 2; AND semantics of Section 4.3.2).
 *
 *   queries         device, row-major [nq][dim], same dtype as the index
 *   qlabel_offsets  host, [nq+1]; every query needs at least one label
 *   qlabel_ids      host; a query with several labels is an AND query.  Duplicates
 *                   are ignored.  At most 8 distinct labels per query.
 *   k               results per query, 1 <= k <= itopk
 *   itopk           capacity of the top-M list of the graph search, <= 256
 *   width           parents expanded per iteration, width * R <= 128
 *   iters           number of graph iterations (fixed; the loop also ends when the
 *                   top-M list holds no unexpanded entry)
 *   n_seeds         initial candidates per graph query: min(n_seeds, |C_l|) local ids
 *                   floor(j * |C_l| / n_seeds); 0 means itopk
 *   out_ids         device [nq][k] global vector ids, ascending by (distance, id);
 *                   -1 where fewer than k vectors qualify
 *   out_dists       device [nq][k] squared distances; +inf where out_ids is -1.  uint8: exact integers.
 *                   float32: graph-searched queries, and scan-routed queries of batches with more than 256
 *                   of them, carry the ordered float32 distance (eight partial sums over 16-byte chunks,
 *                   fused multiply-add, a fixed tree); other scan-routed queries |q|^2 + |x|^2 - 2 q.x in
 *                   float32, within 1e-4 relative of the exact value on data whose norms are comparable
 *                   to the distances
 *   hip_stream      the search is enqueued on this stream and the call returns
 *                   without waiting; outputs are valid once the stream has been
 *                   synchronised.  Calls on one stream run in order.  Calls on
 *                   different streams may be issued without waiting for one another,
 *                   from one host thread or several (the host side of a call is
 *                   serialised inside the library), and overlap on the GPU: the index
 *                   keeps a workspace per calling stream, eight of them; a ninth stream
 *                   takes over the workspace of a stream that is idle, else it waits on
 *                   the host until one has drained.  This is how
 *                   small batches that arrive faster than one call completes are
 *                   served by plain calls (the paper's own answer to that case, a resident
 *                   kernel, Section 4.2.3, is vf_serve_begin below).  vf_search_multi follows the same rule; profiled calls
 *                   and vf_search_exact must not overlap with other calls on the index.
 *
 * A query whose label (any of its labels) has an empty posting list, or whose
 * labels have an empty intersection, yields a row of (-1, +inf); that is not an
 * error.
 */
int vf_search(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
              const int32_t *qlabel_ids, int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds,
              int64_t *out_ids, float *out_dists, void *hip_stream);

/*
 * vf_search with its parameters in a struct, and one more routing option (selectivity-aware routing of AND queries,
 * the remedy for the recall ceiling of the greedy policy that Section 5.3 reports):
 *   and_scan_limit   > 0: an AND query (two or more distinct labels) whose smallest list is a graph list of at most
 *                    this many vectors is answered exactly -- every member of that list is tested with the predicate
 *                    (Section 4.3.2) and the members that pass are scored: the filtered scan of Section 4.3.2's LS
 *                    case applied to a short HS list -- instead of by the greedy graph search.  0: vf_search's routing.
 * Everything else as in vf_search (reserved must be zero).
 */
typedef struct vf_search_params {
    int32_t k, itopk, width, iters, n_seeds;
    int32_t and_scan_limit;
    int32_t reserved[2];
} vf_search_params;
int vf_search_ex(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                 const int32_t *qlabel_ids, const vf_search_params *params, int64_t *out_ids, float *out_dists,
                 void *hip_stream);

/*
 * vf_search for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Arguments, results and error behaviour are those of vf_search, and so are the kernels; the
 * call creates nothing (no device or pinned memory, no stream, no event): its device-side temporaries (routing
 * tables, partial results of segmented scan lists, seed distances) live in one fixed array of
 * VF_NOALLOC_SCRATCH_BYTES of device memory per GPU, which the library holds from its first use on that GPU until
 * the process ends, and the routing tables travel as kernel arguments.  Every launch goes to hip_stream, one
 * after the other.  A call with more than VF_NOALLOC_MAX_QUERIES queries, or whose temporaries would not fit the
 * array (the message says how many bytes it needs), fails with VF_EINVAL before anything is launched.  The
 * interleaved seed copy of vf_search is used when an earlier vf_search call with the same n_seeds has left one;
 * otherwise the seed kernel gathers the seeds' rows.  All calls on one GPU share the array, whatever their
 * index or stream: two calls that overlap on the device race; the caller keeps them in stream order or waits
 * in between.
 */
#define VF_NOALLOC_SCRATCH_BYTES (8u << 20)
#define VF_NOALLOC_MAX_QUERIES 1024
int vf_search_noalloc(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                      const int32_t *qlabel_ids, int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds,
                      int64_t *out_ids, float *out_dists, void *hip_stream);

/*
 * Queue-driven serving of single queries (the persistent kernel of Section 4.2.3).  vf_serve_begin launches ONE
 * kernel that stays resident for the session: a dispatcher wave watches a job ring in pinned host memory and
 * feeds a ring in device memory; worker waves (one per query, as many queries in flight as there are workers)
 * claim jobs from it with an atomic compare-and-swap, route them (smallest list; graph search for |C_l| >= T,
 * scan otherwise; the other labels as AND predicate) and write the k results and a done flag straight into a
 * result ring in host memory.  A query costs no kernel launch and no HIP call: vf_serve_submit and
 * vf_serve_poll only touch pinned memory.  Results are those of vf_search for the same query and parameters
 * (uint8 and graph-searched float32 queries bit for bit).
 *
 *   k, itopk, width, iters, n_seeds   as in vf_search, fixed for the session; itopk <= 64.  A worker scores its
 *                  query's seeds itself (no batch to share a dense seed kernel with), its waves each a share
 *   n_workers      worker workgroups, 0 = 240 (every workgroup of the kernel must fit on the chip at once)
 *   waves_per_worker  waves of a worker, 1, 4 or 8; 0 = 8.  All of them score seeds, the first one searches
 *   ring_slots     jobs that may be in flight or unread, 0 = 1024
 *   max_jobs       the kernel ends after this many jobs, 0 = no limit
 *   idle_polls     the kernel ends after this many consecutive polls of the job ring without a new job
 *                  (a poll takes about a microsecond), 0 = 2,000,000: every wave leaves on its own, the
 *                  session need not be ended for the GPU to become free again
 * The index must outlive the session and must not be freed before vf_serve_end.  One host thread at a time may
 * submit; any thread may poll.
 *
 * vf_serve_submit  query: HOST pointer, dim elements of the index's dtype; labels: 1..8 label ids (AND).  *job
 *                  receives the job's id (0, 1, 2, ... in submission order).  VF_EBUSY when ring_slots jobs
 *                  before it are not finished yet; VF_EINVAL once the kernel has ended.
 * vf_serve_poll    *done = 1 and the k (id, distance) pairs (host arrays; -1 / +inf padded) once the job has
 *                  completed, else *done = 0.  A result stays readable until ring_slots further jobs have
 *                  been submitted.
 * vf_serve_end     asks the kernel to stop, waits for it (bounded: see idle_polls), reports how many jobs it
 *                  completed and why it ended (1 asked to, 2 max_jobs, 3 idle), and releases the session.
 */
typedef struct vf_server vf_server;
typedef struct vf_serve_params {
    int32_t k, itopk, width, iters, n_seeds;
    int32_t n_workers, ring_slots;
    int32_t waves_per_worker;
    int64_t max_jobs, idle_polls;
} vf_serve_params;
int vf_serve_begin(vf_index *index, const vf_serve_params *params, vf_server **out);
int vf_serve_submit(vf_server *server, const void *query, const int32_t *labels, int32_t n_labels, int64_t *job);
int vf_serve_poll(vf_server *server, int64_t job, int64_t *out_ids, float *out_dists, int32_t *done);
int vf_serve_end(vf_server *server, int64_t *jobs_done, int32_t *exit_reason);
/*
 * A batch of host queries through a session, one job per query: submits them in order with at most in_flight
 * (<= ring_slots) jobs outstanding and collects the results in order.  queries: HOST, row-major [nq][dim]; label
 * arrays as in vf_search; out_ids / out_dists: HOST [nq][k]; latency_us: optional HOST [nq], microseconds from a
 * job's submission until its result was seen.  Returns when every job is done (an error if the kernel ends first).
 */
int vf_serve_run(vf_server *server, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                 const int32_t *qlabel_ids, int32_t in_flight, int64_t *out_ids, float *out_dists, float *latency_us);

/*
 * Multi-label queries through one search per label and a merge.
 *   mode VF_AND_GREEDY    the same as vf_search (smallest list + predicate, Section 4.3.2).
 *   mode VF_AND_PARALLEL  the parallel policy at the end of Section 4.3.2: when every query label
 *                         is a graph label, each label's list is searched with the other labels
 *                         as the predicate and the results are merged.  When the smallest list
 *                         is below T its filtered scan is exact already and is the answer.
 *   mode VF_OR            Section 4.3.1: one plain single-label search per distinct query label
 *                         (graph or scan by its size), merged: the nearest vectors that carry ANY
 *                         of the labels.
 * Merge: an id found by several searches keeps its smallest distance; the k best by
 * (distance, id).  Other arguments, layout and error behaviour as in vf_search; the searches of
 * all queries run as one batch of up to 8 * nq single-list searches.
 */
#define VF_AND_GREEDY 0
#define VF_AND_PARALLEL 1
#define VF_OR 2
#define VF_MULTI_EXACT 0x100 /* or-ed into mode: every search is the exact scan of its list (ground truth; synchronises) */
int vf_search_multi(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                    const int32_t *qlabel_ids, int32_t mode, int32_t k, int32_t itopk, int32_t width, int32_t iters,
                    int32_t n_seeds, int64_t *out_ids, float *out_dists, void *hip_stream);

/*
 * Exact filtered top-k (Section 3, Def. 1) for every query, graph lists included,
 * by exhaustive scan of the smallest list with the predicate applied: the ground
 * truth against which recall (Section 3, Eq. 1) is measured.  Arguments as in
 * vf_search.  Synchronises the stream before returning.
 */
int vf_search_exact(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                    const int32_t *qlabel_ids, int32_t k, int64_t *out_ids, float *out_dists, void *hip_stream);

/* Arrays that vf_index_export can copy to the host (names follow Alg. 1). */
#define VF_ARR_S 0      /* int64 [n_labels]      |C_l|                                            */
#define VF_ARR_O_HS 1   /* int64 [n_labels]      start of l in M_HS / G_HS rows, -1 if not a graph label */
#define VF_ARR_O_LS 2   /* int64 [n_labels]      start of l in M_LS, -1 if not a scan label        */
#define VF_ARR_M_HS 3   /* int32 [n_HS]          local -> global id, graph partition               */
#define VF_ARR_M_LS 4   /* int32 [n_LS]          local -> global id, scan partition                */
#define VF_ARR_G_HS 5   /* int32 [n_HS][R]       compacted label graphs, local ids                 */
#define VF_ARR_GO_LS 6  /* int64 [n_labels]      first 32-vector group of l in X_LS, -1 if none    */
#define VF_ARR_X_LS 7   /* bytes                 interleaved scan lists: [group][chunk][32][16 B]  */
#define VF_ARR_BITSET 8 /* uint32 [n_graph_labels][ceil(n/32)]  membership bitsets, graph labels in label order */

/*
 * Copy one index array to host memory.  With host_dst == NULL only *bytes is set
 * (the size needed); otherwise *bytes must be at least that size on entry.
 */
int vf_index_export(const vf_index *index, int which, void *host_dst, size_t *bytes);

/*
 * Sizes of an index, in the terms of the memory model of Section 4.2.4 (N points, F_HS / F_LS average number
 * of graph / scan labels per point, so that n_HS = N F_HS and n_LS = N F_LS, out-degree R, b bytes per
 * element, D elements per vector).  The base table X (N D b) is the caller's and is not counted.
 *   bytes_graph    neighbour lists of the HS partition, the model's N F_HS R b with b = 4 (ids are int32),
 *                  stored twice: as local ids (G_HS of Alg. 1) and once more as global ids (a copy the search
 *                  reads instead of a lookup in M_HS)
 *   bytes_x_ls     vectors of the LS partition, the model's N D F_LS b, in the interleaved layout of Section
 *                  4.2.2: every list is padded to whole groups of 32 vectors (n_groups_LS groups in all) and to
 *                  an even number of 16-byte chunks per vector (chunks_per_vector), plus one 4-byte squared
 *                  norm per slot
 *   bytes_maps     local -> global index mappings M_HS and M_LS, the model's N F b with b = 4
 *   bytes_bitsets  membership bitsets of the graph labels (the AND predicate of Section 4.3.2 as this library
 *                  stores it): n_graph_labels ceil(N / 32) 4
 *   bytes_meta     per-label sizes and offsets ("label metadata" of Section 4.2.4): 24 bytes per label
 *   bytes_x_ls_bf16  float32 data: the vectors of the LS partition once more, rounded to bfloat16 in the same
 *                  interleaved layout (half of bytes_x_ls without its norms); the scan of large batches streams
 *                  this copy and re-ranks what it keeps.  0 for uint8 data.  Not in the paper's model
 *   bytes_total    the sum of the six
 */
typedef struct vf_stats {
    int64_t n, n_HS, n_LS, n_groups_LS;
    int32_t dim, dtype, n_labels, T, graph_degree, n_graph_labels, n_scan_labels, chunks_per_vector;
    int64_t bytes_graph, bytes_maps, bytes_x_ls, bytes_bitsets, bytes_meta, bytes_total;
    int64_t bytes_x_ls_bf16;
} vf_stats;

int vf_index_stats(const vf_index *index, vf_stats *out);

/*
 * Experiment and test switches (not part of the paper's method): launch geometry, which kernels serve which
 * batch sizes, the error-bound scale of the float32 seed proofs.  With index == NULL the process-wide
 * defaults change, which indexes built afterwards start from (the build-time switches "build16",
 * "build_panel_kb" and "build_progress" only act that way); with an index, that index's own copy changes, and
 * no call on it may be in flight.  Names: "seg_groups", "seg_groups_heavy", "heavy_rows", "tile_rows",
 * "zero_copy_bytes", "scan_valu", "scan16", "scan_bf16", "scan_bf16_margin", "scan_bf16_slots", "scan_bf16_seg_groups", "beam_lat_waves", "overlap", "seed_exact", "seed_slack", "seed_margin",
 * "seed_margin_bf16", "seed_cache", "seed_bf16", "seed_bf16_min_batch", "seed_fb_window", "seed_select",
 * "seed_seg_seeds", "build16",
 * "build_panel_kb", "build_progress".  Returns VF_EINVAL for an unknown name or a value out of range.
 * Results never depend on any of them.
 */
int vf_tune(vf_index *index, const char *name, double value);

/*
 * Measurement support (not part of the paper's method).  While profiling is on,
 * every vf_search / vf_search_exact call brackets its IVF-BFS launch and its IVF-Graph launch with HIP
 * events on the caller's stream and has the graph kernel record, per query, how
 * many distances it computed, rows it expanded and predicate tests it made.
 * vf_profile_read waits for the last profiled call and reports it, together with
 * the duration sums over all calls since vf_profile_enable(index, 1).  (Up to 64 profiled
 * calls can be outstanding; a further one first waits for the oldest.)
 * on = 1 leaves the launch schedule as it is (IVF-BFS runs on a second stream beside
 * IVF-Graph, so the two intervals overlap and each kernel shares the chip); on = 2 also
 * puts every launch on the caller's stream, one after the other, so each interval is
 * that kernel's duration with the chip to itself; on = 0 switches both off.
 * on | 4: batches with AND queries also run a small kernel before each call that counts, per graph query, the
 * seeds that pass its predicate, so that "distances computed" is exact for them; without it that count
 * includes, for such a query, the seeds whose predicate the search never had to evaluate (seeds that could not
 * enter a full list).
 *   per_query   optional host buffer [nq][4] int32 of the last call:
 *               distances computed, rows expanded, predicate tests, and a mode word:
 *               0 = scan path (the first three are then 0); low byte 2 = graph path,
 *               3 = graph path whose matrix-core seed scores could not be proven
 *               sufficient (the kernel then scored every seed itself); bits 8 and up =
 *               seeds re-scored with the ordered distance after matrix-core scoring
 */
typedef struct vf_profile {
    float scan_ms, seed_ms, beam_ms;   /* durations of the last call: the IVF-BFS scan kernel (vf_search_exact: all its
                                          scan and merge launches), dense seed scoring, beam search */
    double scan_ms_sum, seed_ms_sum, beam_ms_sum; /* sums over all calls since profiling was enabled */
    int64_t calls;                     /* number of calls in those sums                */
    int64_t nq, n_scan_queries, n_graph_queries, n_scan_items;
    int64_t scan_list_entries;         /* sum over scan items of the list length       */
    int64_t scan_pairs;                /* sum over scan items of queries x list length */
    int64_t beam_scored, beam_expanded, beam_tested;
    int64_t n_seed_tiles;              /* tiles of same-label graph queries scored densely (<= 32 queries on the matrix cores,
                                          <= 64 with the ordered-distance kernel; 0: seeds were gathered)                  */
    int64_t seed_pairs;                /* sum over graph queries of the seeds scored for them                            */
    int64_t seed_tile_seeds;           /* sum over seed tiles of the seeds they read                                     */
    int64_t seeds_on_matrix_cores;     /* 1: the seeds were scored on MFMA (float32: approximations, re-ranked by the beam
                                          kernel); 2: the same from the bfloat16 copy of the seeds (float32 data)         */
    int64_t seed_rescored;             /* ordered distances computed for that re-ranking                                 */
    int64_t seed_fallbacks;            /* queries whose proof failed and that scored every seed themselves               */
    int64_t beam_gathered;             /* distances whose vector the beam kernel fetched itself (children, re-ranked seeds, seeds when not scored densely) */
    int64_t scan_kernel;               /* IVF-BFS kernel of the call: 0 = 32-row matrix-core tiles, 1 = 16-row matrix-core tiles, 2 = FMA,
                                          3 = filter from the bfloat16 copy of the lists + exact re-ranking (float32 data)         */
    int64_t seed_selected;             /* 1: the seed kernel also selected (a few keys per query and seed segment instead of every distance) */
    int64_t seed_run_keys;             /* 8-byte keys that kernel left for the beam kernel (sum over graph queries of segments x keys per run) */
    int64_t scan_fallbacks;            /* scan queries since profiling was enabled whose filtered result (scan_kernel 3) could not
                                          be proven complete and that the exact kernels scanned again                         */
    double host_plan_ms_sum, host_blob_ms_sum, host_launch_ms_sum; /* host time inside the calls since profiling was enabled:
                                          routing and work lists; assembling the routing blob; everything else (HIP calls)   */
    double host_wait_ms_sum;           /* ... and time the host waited for a staging buffer (two calls ahead of the device) */
} vf_profile;

int vf_profile_enable(vf_index *index, int on);
int vf_profile_read(vf_index *index, vf_profile *out, int32_t *per_query);

/*
 * Test support, host only (no device call): routes a batch the way vf_search does -- per query the searched label
 * (the smallest of its lists, ties to the lower label id, Section 4.3.2; -1 when one of its lists is empty),
 * the method (0 = empty result, 1 = scan, |C_l| < T, 2 = graph, Section 4.1.2) and the number of predicate
 * labels -- and builds the work list of the scan path for posting-list sizes S alone (scan lists laid out in
 * ascending label id, as vf_build_index does).
 *   items_out   [items_cap][8] int64: first 32-vector group, start in M_LS, first entry, entries, first tile row,
 *               tile rows, -1, partial row of tile row 0 (-1: the item writes final results)
 *   merges_out  [merges_cap][5] int64: start in M_LS, query, partial row of segment 0, stride, segments
 *   qrow_out    [nq] int32: the query of every scan tile row, then the graph queries grouped by label
 *   counts      [6] int64: graph queries, scan tile rows, items, merges, partial rows, largest segment count
 * Output arrays may be NULL except searched, method, n_others and counts (a first call with NULL arrays gives the
 * sizes).
 */
int vf_debug_route(const int32_t *S, int32_t n_labels, int32_t T, int64_t nq, const int64_t *qlabel_offsets,
                   const int32_t *qlabel_ids, int32_t tile_rows, int32_t seg_groups, int32_t *searched, int32_t *method,
                   int32_t *n_others, int64_t *items_out, int64_t items_cap, int64_t *merges_out, int64_t merges_cap,
                   int32_t *qrow_out, int64_t *counts);

/* Releases the index and its workspace.  NULL is allowed. */
void vf_index_free(vf_index *index);

/* Message of the calling thread's last failing call; valid until its next call. */
const char *vf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
