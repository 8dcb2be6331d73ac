// Host side of the C ABI declared in include/vecflow.h: index construction
// (Alg. 1), query routing and grouping (ClassifyQueries of Alg. 2, list choice of
// Section 4.3.2), kernel launches, export.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <ctime>
#include <mutex>
#include <new>
#include <numeric>

#include "../../include/vecflow.h"
#include "vf_internal.h"

namespace vf {

static thread_local std::string g_err;
void set_error(const std::string &msg) { g_err = msg; }

#define VF_HIP(expr)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) {                                                                        \
            set_error(std::string(#expr) + ": " + hipGetErrorString(e_));                              \
            return e_ == hipErrorOutOfMemory ? VF_ENOMEM : VF_EHIP;                                    \
        }                                                                                              \
    } while (0)

#define VF_REQUIRE(cond, msg)                 \
    do {                                      \
        if (!(cond)) {                        \
            set_error(msg);                   \
            return VF_EINVAL;                 \
        }                                     \
    } while (0)

static int env_int_early(const char *name, int dflt)
{
    const char *e = getenv(name);
    return (e && *e) ? atoi(e) : dflt;
}

struct DevBuf {
    void *p = nullptr;
    size_t cap = 0;
    int reserve(size_t bytes)
    {
        if (bytes <= cap) return VF_OK;
        if (p) { (void)hipFree(p); p = nullptr; cap = 0; }
        const size_t want = bytes + bytes / 4 + 256;
        VF_HIP(hipMalloc(&p, want));
        cap = want;
        return VF_OK;
    }
    void release()
    {
        if (p) (void)hipFree(p);
        p = nullptr; cap = 0;
    }
    template <class T> T *as() const { return (T *)p; }
};

struct Staging {  // pinned host blob + the event that says its last upload has finished
    void *p = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool pending = false;
};

// Result of routing one batch (host side) and the scratch it reuses between calls.
struct Routed {
    std::vector<int32_t> gq_query, gq_label;          // graph queries, grouped by label (ascending), stable in query order
    std::vector<int32_t> others_off, others;          // [nq+1], AND partner labels per query
    std::vector<uint64_t> scan_pairs;                 // (label << 32 | query) of scan queries, ascending
    bool any_and = false;
    // scratch kept between calls
    std::vector<int32_t> q_best;                      // searched label of each query, -1: empty result
    std::vector<int32_t> empty_q;                     // queries with q_best == -1
    std::vector<int32_t> cnt;                         // [n_labels] queries per searched label (zero between calls)
    std::vector<int32_t> touched;                     // labels with cnt > 0
};

}  // namespace vf

using namespace vf;

// Everything a call writes besides its outputs.  An index has kWorkspaces of them and hands one to each
// stream that calls it, so that calls on different streams can overlap on the GPU (small batches leave most
// of the chip idle); calls on one stream share one workspace and run in order as before.
struct Workspace {
    DevBuf ws_blob, ws_blob_b, part_idx, part_bits, dseed;
    // vf_search_multi: gathered query rows, results of the sub-searches, their parents
    DevBuf multi_q, multi_ids, multi_dists, multi_meta;
    std::vector<int32_t> multi_host;      // [n_sub parents | nq + 1 first sub-search of each query], alive until the next call
    std::vector<int64_t> multi_qoff;
    std::vector<int32_t> multi_qids;
    // the scan path runs beside the graph path on a second stream of the same (default) priority
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_copy = nullptr;
    hipEvent_t ev_blob_done[2] = {nullptr, nullptr};   // recorded on the caller's stream when a call that read blob b ends
    bool blob_used[2] = {false, false};
    int blob_next = 0;   // the device blob alternates between two buffers
    Staging stage[2];
    int stage_next = 0;
    Routed routed;
    bool ready = false;          // stream and events exist
    bool owned = false;
    hipStream_t owner = nullptr; // the stream whose calls use this workspace
};

struct vf_index {
    int dtype = 0;
    int64_t n = 0;
    int32_t dim = 0, n_labels = 0, T = 0, R = 0, ncp = 0;
    int32_t graph_kind = 0, knn_degree = 0;
    const void *X = nullptr;
    // host metadata
    std::vector<int32_t> S, hs_slot;
    std::vector<int64_t> O_HS, O_LS, GO_LS;
    std::vector<int32_t> graph_labels;
    int64_t n_HS = 0, n_LS = 0, n_groups_LS = 0, bitset_words = 0;
    int32_t n_scan_labels = 0;
    // device
    DevBuf d_S, d_O_HS, d_O_LS, d_hs_slot, d_M_HS, d_M_LS, d_G, d_X_LS, d_xnorm_LS, d_bitsets;
    DevBuf d_Gg;   // [n_HS][R] the graph rows once more with global ids: saves the search one dependent load per expansion
    // float32 indexes with graph labels: squared norm of every row of X and the largest of them,
    // for the matrix-core seed scoring (its error bound needs the largest norm)
    DevBuf d_xnorm_all;
    float xn_max = 0.f;
    float seed_err_bound = 0.f;  // relative to |q|^2 + xn_max; VF_SEED_SLACK in the environment scales it (tests)
    bool seed_mfma = false;      // VF_SEED_EXACT=1 in the environment keeps the exact VALU seed kernel
    // search workspaces (see Workspace); profiled calls and vf_search_exact must not overlap with other calls
    static constexpr int kWorkspaces = 8;
    Workspace ws[kWorkspaces];
    int ws_steal = 0;
    std::recursive_mutex mu;     // host side of every call
    DevBuf tmp_blk, tmp_norm, counters;
    // the seeds of every graph list for the last n_seeds used, interleaved like a scan list, so that the
    // matrix-core seed kernel reads its B operand with coalesced loads (rebuilt when n_seeds changes)
    DevBuf seed_blk, seed_norm, seed_goff;
    DevBuf seed_blk16;           // the same seeds rounded to bfloat16 (float32 data only)
    bool seed_bf16 = false;      // seed_blk16 is valid
    bool seed_f32 = false;       // float32 data: seed_blk was kept beside seed_blk16 (small copies only)
    // Watch on the bfloat16 form: queries whose proof failed are counted on the device; the count is fetched
    // every kFallbackWindow graph queries and read at a later call, and a window with more than 1/64 failures
    // switches this index back to the float32 copy (a failed proof costs its query a gather of every seed).
    bool seed_bf16_off = false;
    DevBuf d_fb_count;
    uint32_t *h_fb = nullptr;    // pinned
    hipEvent_t ev_fb = nullptr;
    bool fb_pending = false;
    uint32_t fb_last = 0;
    int64_t fb_window_q = 0, fb_sent_q = 0;
    float seed_bf16_delta = 0.f; // upper bound of |x - bf16(x)| over the seeds of the copy
    int32_t seed_cache_ns = -1;      // n_seeds the copy was built for
    bool seed_cache_ok = false;      // false: it did not fit, the kernel gathers rows from the vector table
    // profiling
    bool profiling = false, prof_valid = false;
    // a ring of event sets (scan begin/end, graph begin, seeds end, beam end), one set per profiled call:
    // a call never waits for an earlier one unless kProfRing calls are still unread
    static constexpr int kProfRing = 64;
    hipEvent_t prof_ring[kProfRing][5] = {};
    hipEvent_t *prof_ev = prof_ring[0];   // the set of the call being issued
    int prof_next = 0, prof_unfolded = 0; // next ring slot; recorded sets whose durations are not in the sums yet
    bool overlap = true;  // VF_NO_OVERLAP=1 in the environment serialises the two paths (for per-kernel timing)
    bool prof_serial = false;  // vf_profile_enable(index, 2): same, switched at run time
    vf_profile prof{};
    std::vector<int32_t> prof_graph_queries;   // graph-routed queries of the last profiled call
    double prof_scan_sum = 0, prof_seed_sum = 0, prof_beam_sum = 0;
    int64_t prof_calls = 0;
    LabelMeta meta() const
    {
        LabelMeta m;
        m.S = d_S.as<int32_t>(); m.O_HS = d_O_HS.as<int64_t>(); m.O_LS = d_O_LS.as<int64_t>();
        m.hs_slot = d_hs_slot.as<int32_t>(); m.M_HS = d_M_HS.as<int32_t>(); m.M_LS = d_M_LS.as<int32_t>();
        m.bitsets = d_bitsets.as<uint32_t>(); m.bitset_words = bitset_words;
        return m;
    }
    size_t elem() const { return dtype == VF_U8 ? 1 : 4; }
    size_t group_bytes() const { return (size_t)2 * ncp * 32 * 16; }
};

static void free_index(vf_index *ix)
{
    if (!ix) return;
    DevBuf *bufs[] = {&ix->d_S, &ix->d_O_HS, &ix->d_O_LS, &ix->d_hs_slot, &ix->d_M_HS, &ix->d_M_LS, &ix->d_G, &ix->d_Gg,
                      &ix->d_X_LS, &ix->d_xnorm_LS, &ix->d_bitsets, &ix->d_xnorm_all, &ix->tmp_blk, &ix->tmp_norm, &ix->counters, &ix->seed_blk, &ix->seed_blk16, &ix->seed_norm, &ix->seed_goff};
    for (DevBuf *b : bufs) b->release();
    for (auto &set : ix->prof_ring)
        for (hipEvent_t e : set)
            if (e) (void)hipEventDestroy(e);
    if (ix->ev_fb) (void)hipEventDestroy(ix->ev_fb);
    if (ix->h_fb) (void)hipHostFree(ix->h_fb);
    ix->d_fb_count.release();
    for (Workspace &w : ix->ws) {
        DevBuf *wb[] = {&w.ws_blob, &w.ws_blob_b, &w.part_idx, &w.part_bits, &w.dseed, &w.multi_q, &w.multi_ids, &w.multi_dists, &w.multi_meta};
        for (DevBuf *b : wb) b->release();
        if (w.ev_fork) (void)hipEventDestroy(w.ev_fork);
        if (w.ev_join) (void)hipEventDestroy(w.ev_join);
        if (w.ev_copy) (void)hipEventDestroy(w.ev_copy);
        for (hipEvent_t e : w.ev_blob_done)
            if (e) (void)hipEventDestroy(e);
        if (w.side) { (void)hipStreamSynchronize(w.side); (void)hipStreamDestroy(w.side); }
        for (Staging &s : w.stage) {
            if (s.pending) (void)hipEventSynchronize(s.done);
            if (s.done) (void)hipEventDestroy(s.done);
            if (s.p) (void)hipHostFree(s.p);
        }
    }
    delete ix;
}

template <class T> static int upload(DevBuf &b, const std::vector<T> &v, hipStream_t s)
{
    int rc = b.reserve(std::max<size_t>(v.size() * sizeof(T), 16));
    if (rc != VF_OK) return rc;
    if (!v.empty()) VF_HIP(hipMemcpyAsync(b.p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, s));
    return VF_OK;
}

// Exact kNN rows of label l's list: interleave the list, contract it against itself, keep K candidates per
// vertex, order `deg` of them into rows_out ([|C_l|][deg] local ids); with global_ids the same rows also go
// to the index's global-id table (deg == R).
static int build_graph_for_label(vf_index *ix, int32_t l, int32_t K, int32_t deg, int32_t *rows_out, bool global_ids,
                                 DevBuf &cand_idx, DevBuf &cand_dist, DevBuf &d_items, hipStream_t s)
{
    const int64_t base = ix->O_HS[l];
    const int32_t nl = ix->S[l];
    const int64_t n_groups = (nl + 31) / 32;
    const int32_t *map = ix->d_M_HS.as<int32_t>() + base;
    launch_interleave(ix->dtype, ix->X, ix->dim, map, nullptr, nullptr, nl, n_groups, ix->ncp, ix->tmp_blk.as<uint4>(),
                      ix->tmp_norm.p, s);
    // float32: 16-row tiles on the 16x16x4 MFMA (their smaller LDS footprint more than doubles the resident
    // waves); uint8: 32-row tiles
    static const int build16 = env_int_early("VF_BUILD16", 1);
    const int32_t TR = (build16 && scan16_supported(ix->dtype, ix->dim, 16)) ? 16 : 32;
    const int64_t n_tiles = (nl + TR - 1) / TR;
    std::vector<ScanItem> items((size_t)n_tiles);
    for (int64_t t = 0; t < n_tiles; ++t) {
        ScanItem &it = items[(size_t)t];
        it.group0 = 0; it.map_off = 0; it.entry0 = 0; it.n = nl;
        it.q_begin = (int32_t)(t * TR);
        it.q_count = (int32_t)std::min<int64_t>(TR, nl - t * TR);
        it.self_base = it.q_begin;
        it.part_row = it.q_begin;
    }
    int rc = upload(d_items, items, s);
    if (rc != VF_OK) return rc;
    VF_HIP(hipStreamSynchronize(s));  // `items` is pageable host memory
    ScanParams p{};
    p.xblk = ix->tmp_blk.as<uint4>(); p.xnorm = ix->tmp_norm.p; p.map = map;
    p.qsrc = ix->X; p.qrow = map; p.items = d_items.as<ScanItem>();
    p.dim = ix->dim; p.ncp = ix->ncp; p.K = K; p.tile_rows = TR;
    p.res_idx = cand_idx.as<int32_t>(); p.res_bits = cand_dist.as<uint32_t>();
    p.others_off = nullptr; p.others = nullptr; p.meta = ix->meta();
    if (TR == 16) {
        // long lists go panel by panel so that the resident waves share L2
        // (VF_BUILD_PANEL_KB: panel size, 4096 by default -- the measured optimum, one XCD's L2; lists of
        // up to 4 panels are not cut)
        static const int64_t panel_bytes = (int64_t)std::max(1, env_int_early("VF_BUILD_PANEL_KB", 4096)) << 10;
        const int64_t list_bytes = n_groups * (int64_t)ix->group_bytes();
        if (list_bytes <= 4 * panel_bytes) {
            launch_scan16(p, (int)n_tiles, s);
        } else {
            const int32_t panel = (int32_t)std::max<int64_t>(32, panel_bytes / ((int64_t)ix->group_bytes() / 32) / 32 * 32);
            for (int64_t e0 = 0; e0 < nl; e0 += panel) {
                p.panel_entry0 = (int32_t)e0; p.panel_n = panel; p.carry = e0 > 0;
                launch_scan16(p, (int)n_tiles, s);
            }
        }
    } else {
        launch_scan(ix->dtype, p, (int)n_tiles, s);
    }
    launch_graph_rows(ix->dtype, ix->X, ix->dim, map, nl, cand_idx.as<int32_t>(), K, deg, rows_out, s);
    if (global_ids)
        launch_graph_global_ids(rows_out, map, (int64_t)nl * deg, ix->d_Gg.as<int32_t>() + base * ix->R, s);
    VF_HIP(hipGetLastError());
    return VF_OK;
}

// Reduces the degree-D rows of all lists (knn, [n_HS][D]) to the index's degree-R rows: rank-based pruning,
// reverse edges, merge (vf_graphopt.hip).  d_Gg serves as the forward rows' storage until the end.
static int optimize_graphs(vf_index *ix, const int32_t *d_knn, int32_t D, hipStream_t s)
{
    const int64_t nn = ix->n_HS;
    const int32_t R = ix->R;
    int rc;
    DevBuf d_base, d_deg, d_off, d_seg;
    struct Rel { DevBuf &a, &b, &c, &d; ~Rel() { a.release(); b.release(); c.release(); d.release(); } } rel{d_base, d_deg, d_off, d_seg};
    std::vector<int32_t> base((size_t)nn);
    for (int32_t l : ix->graph_labels)
        std::fill(base.begin() + ix->O_HS[(size_t)l], base.begin() + ix->O_HS[(size_t)l] + ix->S[(size_t)l],
                  (int32_t)ix->O_HS[(size_t)l]);
    if ((rc = upload(d_base, base, s)) != VF_OK) return rc;
    if ((rc = d_deg.reserve((size_t)nn * 4)) != VF_OK) return rc;
    if ((rc = d_off.reserve((size_t)(nn + 1) * 8)) != VF_OK) return rc;
    int32_t *F = ix->d_Gg.as<int32_t>();
    launch_graph_prune(d_knn, d_base.as<int32_t>(), nn, D, R, F, s);
    VF_HIP(hipMemsetAsync(d_deg.p, 0, (size_t)nn * 4, s));
    launch_graph_indegree(F, d_base.as<int32_t>(), nn, R, d_deg.as<int32_t>(), s);
    std::vector<int32_t> deg((size_t)nn);
    VF_HIP(hipMemcpyAsync(deg.data(), d_deg.p, (size_t)nn * 4, hipMemcpyDeviceToHost, s));
    VF_HIP(hipStreamSynchronize(s));   // also: `base` is pageable host memory
    std::vector<int64_t> off((size_t)nn + 1);
    off[0] = 0;
    for (int64_t g = 0; g < nn; ++g) off[(size_t)g + 1] = off[(size_t)g] + deg[(size_t)g];
    VF_REQUIRE(off[(size_t)nn] <= nn * (int64_t)R, "internal: more proposals than forward edges");
    if ((rc = upload(d_off, off, s)) != VF_OK) return rc;
    if ((rc = d_seg.reserve((size_t)std::max<int64_t>(1, off[(size_t)nn]) * 8)) != VF_OK) return rc;
    VF_HIP(hipMemsetAsync(d_deg.p, 0, (size_t)nn * 4, s));   // now the per-target cursors
    launch_graph_reverse_fill(F, d_base.as<int32_t>(), nn, R, d_off.as<int64_t>(), d_deg.as<int32_t>(),
                              d_seg.as<uint64_t>(), s);
    launch_graph_reverse_merge(F, d_off.as<int64_t>(), d_seg.as<uint64_t>(), nn, R, ix->d_G.as<int32_t>(), s);
    launch_graph_global_ids_based(ix->d_G.as<int32_t>(), d_base.as<int32_t>(), ix->d_M_HS.as<int32_t>(), nn, R,
                                  ix->d_Gg.as<int32_t>(), s);
    VF_HIP(hipGetLastError());
    VF_HIP(hipStreamSynchronize(s));   // `off` is pageable host memory; the temporaries are freed on return
    return VF_OK;
}

static int build_index_impl(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                            const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                            int32_t graph_kind, int32_t knn_degree, void *hip_stream, vf_index **out);

extern "C" int vf_build_index(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                              const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                              void *hip_stream, vf_index **out)
{
    return build_index_impl(vectors, dtype, n, dim, label_offsets, label_ids, n_labels, T, graph_degree, VF_GRAPH_KNN, 0,
                            hip_stream, out);
}

extern "C" int vf_build_index_opt(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                                  const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                                  int32_t graph_kind, int32_t knn_degree, void *hip_stream, vf_index **out)
{
    return build_index_impl(vectors, dtype, n, dim, label_offsets, label_ids, n_labels, T, graph_degree, graph_kind,
                            knn_degree, hip_stream, out);
}

static int build_index_impl(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                            const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                            int32_t graph_kind, int32_t knn_degree, void *hip_stream, vf_index **out)
{
    VF_REQUIRE(out != nullptr, "out is NULL");
    *out = nullptr;
    VF_REQUIRE(vectors && label_offsets && label_ids, "NULL input pointer");
    VF_REQUIRE(dtype == VF_U8 || dtype == VF_F32, "dtype must be VF_U8 or VF_F32");
    VF_REQUIRE(n > 0 && n < ((int64_t)1 << 31), "n must be in [1, 2^31)");
    const int64_t row_bytes = (int64_t)dim * (dtype == VF_U8 ? 1 : 4);
    VF_REQUIRE(dim > 0 && row_bytes % 16 == 0 && row_bytes >= 16 && row_bytes <= 2048,
               "dim: uint8 needs dim % 16 == 0, float32 dim % 4 == 0, 16 <= bytes per vector <= 2048");
    VF_REQUIRE(((uintptr_t)vectors & 15) == 0, "vectors must be 16-byte aligned");
    VF_REQUIRE(n_labels > 0, "n_labels must be positive");
    VF_REQUIRE(graph_degree >= 1 && graph_degree <= 64, "graph_degree must be in [1, 64]");
    VF_REQUIRE(T >= graph_degree + 1, "T must be at least graph_degree + 1");
    VF_REQUIRE(graph_kind == VF_GRAPH_KNN || graph_kind == VF_GRAPH_PRUNED, "graph_kind must be VF_GRAPH_KNN or VF_GRAPH_PRUNED");
    // degree of the kNN graph a pruned graph starts from: 2 R, as far as the self-join's 64 candidates per
    // row reach (float32 rows are re-ranked out of 16 candidates more than they keep)
    const int32_t knn_max = dtype == VF_U8 ? 64 : 48;
    int32_t D = graph_degree;
    if (graph_kind == VF_GRAPH_PRUNED) {
        D = knn_degree > 0 ? knn_degree : std::min(2 * graph_degree, knn_max);
        VF_REQUIRE(D >= graph_degree && D <= knn_max,
                   "knn_degree must lie in [graph_degree, 64] (uint8) or [graph_degree, 48] (float32)");
        VF_REQUIRE(T >= D + 1, "T must be at least knn_degree + 1");
    } else {
        VF_REQUIRE(knn_degree == 0, "knn_degree is only used with VF_GRAPH_PRUNED");
    }
    VF_REQUIRE(label_offsets[0] == 0, "label_offsets[0] must be 0");
    for (int64_t i = 0; i < n; ++i) VF_REQUIRE(label_offsets[i + 1] >= label_offsets[i], "label_offsets must not decrease");
    const int64_t n_raw = label_offsets[n];
    for (int64_t p = 0; p < n_raw; ++p)
        VF_REQUIRE(label_ids[p] >= 0 && label_ids[p] < n_labels, "label id outside [0, n_labels)");

    hipStream_t s = (hipStream_t)hip_stream;
    vf_index *ix = new (std::nothrow) vf_index();
    if (!ix) { set_error("out of host memory"); return VF_ENOMEM; }
    struct Guard { vf_index *ix; ~Guard() { if (ix) free_index(ix); } } guard{ix};
    ix->dtype = dtype; ix->n = n; ix->dim = dim; ix->n_labels = n_labels; ix->T = T; ix->R = graph_degree;
    ix->X = vectors;
    ix->ncp = (int32_t)((row_bytes / 16 + 1) / 2);

    try {
        // ---- pass 1 (Alg. 1): posting-list sizes over sorted, duplicate-free label sets
        std::vector<int32_t> uniq((size_t)n_raw);
        std::vector<int64_t> uoff((size_t)n + 1, 0);
        int64_t w = 0;
        for (int64_t i = 0; i < n; ++i) {
            const int64_t b = label_offsets[i], e = label_offsets[i + 1], start = w;
            for (int64_t p = b; p < e; ++p) uniq[(size_t)w++] = label_ids[p];
            std::sort(uniq.begin() + start, uniq.begin() + w);
            w = std::unique(uniq.begin() + start, uniq.begin() + w) - uniq.begin();
            uoff[(size_t)i + 1] = w;
        }
        ix->S.assign((size_t)n_labels, 0);
        for (int64_t p = 0; p < w; ++p) ix->S[(size_t)uniq[(size_t)p]]++;

        // ---- split by T; S/O/M per partition, compacted in ascending label id
        ix->O_HS.assign((size_t)n_labels, -1); ix->O_LS.assign((size_t)n_labels, -1);
        ix->GO_LS.assign((size_t)n_labels, -1); ix->hs_slot.assign((size_t)n_labels, -1);
        for (int32_t l = 0; l < n_labels; ++l) {
            const int32_t sz = ix->S[(size_t)l];
            if (sz >= T) {
                ix->O_HS[(size_t)l] = ix->n_HS; ix->n_HS += sz;
                ix->hs_slot[(size_t)l] = (int32_t)ix->graph_labels.size();
                ix->graph_labels.push_back(l);
            } else if (sz > 0) {
                ix->O_LS[(size_t)l] = ix->n_LS; ix->n_LS += sz;
                ix->GO_LS[(size_t)l] = ix->n_groups_LS; ix->n_groups_LS += (sz + 31) / 32;
                ix->n_scan_labels++;
            }
        }
        std::vector<int32_t> M_HS((size_t)ix->n_HS), M_LS((size_t)ix->n_LS);
        {
            std::vector<int32_t> fill((size_t)n_labels, 0);
            for (int64_t i = 0; i < n; ++i)
                for (int64_t p = uoff[(size_t)i]; p < uoff[(size_t)i + 1]; ++p) {
                    const int32_t l = uniq[(size_t)p];
                    if (ix->O_HS[(size_t)l] >= 0) M_HS[(size_t)(ix->O_HS[(size_t)l] + fill[(size_t)l]++)] = (int32_t)i;
                    else M_LS[(size_t)(ix->O_LS[(size_t)l] + fill[(size_t)l]++)] = (int32_t)i;
                }
        }
        std::vector<int32_t>().swap(uniq);
        std::vector<int64_t>().swap(uoff);

        int rc;
        if ((rc = upload(ix->d_S, ix->S, s)) != VF_OK) return rc;
        if ((rc = upload(ix->d_O_HS, ix->O_HS, s)) != VF_OK) return rc;
        if ((rc = upload(ix->d_O_LS, ix->O_LS, s)) != VF_OK) return rc;
        if ((rc = upload(ix->d_hs_slot, ix->hs_slot, s)) != VF_OK) return rc;
        if ((rc = upload(ix->d_M_HS, M_HS, s)) != VF_OK) return rc;
        if ((rc = upload(ix->d_M_LS, M_LS, s)) != VF_OK) return rc;
        VF_HIP(hipStreamSynchronize(s));

        // ---- scan partition: StoreInterleaved over every scan list (Section 4.2.2)
        if (ix->n_groups_LS > 0) {
            std::vector<int64_t> grp_src((size_t)ix->n_groups_LS);
            std::vector<int32_t> grp_cnt((size_t)ix->n_groups_LS);
            for (int32_t l = 0; l < n_labels; ++l) {
                if (ix->GO_LS[(size_t)l] < 0) continue;
                const int32_t sz = ix->S[(size_t)l];
                for (int32_t g = 0; g < (sz + 31) / 32; ++g) {
                    grp_src[(size_t)(ix->GO_LS[(size_t)l] + g)] = ix->O_LS[(size_t)l] + (int64_t)g * 32;
                    grp_cnt[(size_t)(ix->GO_LS[(size_t)l] + g)] = std::min(32, sz - g * 32);
                }
            }
            DevBuf d_src, d_cnt;
            struct R2 { DevBuf &a, &b; ~R2() { a.release(); b.release(); } } r2{d_src, d_cnt};
            if ((rc = upload(d_src, grp_src, s)) != VF_OK) return rc;
            if ((rc = upload(d_cnt, grp_cnt, s)) != VF_OK) return rc;
            if ((rc = ix->d_X_LS.reserve((size_t)ix->n_groups_LS * ix->group_bytes())) != VF_OK) return rc;
            if ((rc = ix->d_xnorm_LS.reserve((size_t)ix->n_groups_LS * 32 * 4)) != VF_OK) return rc;
            launch_interleave(dtype, vectors, dim, ix->d_M_LS.as<int32_t>(), d_src.as<int64_t>(), d_cnt.as<int32_t>(),
                              ix->n_LS, ix->n_groups_LS, ix->ncp, ix->d_X_LS.as<uint4>(), ix->d_xnorm_LS.p, s);
            VF_HIP(hipGetLastError());
            VF_HIP(hipStreamSynchronize(s));
        }

        // ---- graph partition: membership bitsets and one exact kNN graph per list
        const int32_t n_gl = (int32_t)ix->graph_labels.size();
        ix->bitset_words = (n + 31) / 32;
        if (n_gl > 0) {
            const size_t bs_bytes = (size_t)n_gl * ix->bitset_words * 4;
            if ((rc = ix->d_bitsets.reserve(bs_bytes)) != VF_OK) return rc;
            VF_HIP(hipMemsetAsync(ix->d_bitsets.p, 0, bs_bytes, s));
            if ((rc = ix->d_G.reserve((size_t)ix->n_HS * ix->R * 4)) != VF_OK) return rc;
            if ((rc = ix->d_Gg.reserve((size_t)ix->n_HS * ix->R * 4)) != VF_OK) return rc;
            int32_t max_list = 0;
            for (int32_t l : ix->graph_labels) max_list = std::max(max_list, ix->S[(size_t)l]);
            const bool pruned = graph_kind == VF_GRAPH_PRUNED;
            const int32_t K = dtype == VF_U8 ? D : std::min(64, D + 16);
            DevBuf d_knn;
            struct RK { DevBuf &a; ~RK() { a.release(); } } rk{d_knn};
            if (pruned && (rc = d_knn.reserve((size_t)ix->n_HS * D * 4)) != VF_OK) return rc;
            DevBuf cand_idx, cand_dist, d_items;
            struct R3 { DevBuf &a, &b, &c; ~R3() { a.release(); b.release(); c.release(); } } r3{cand_idx, cand_dist, d_items};
            const int64_t max_groups = (max_list + 31) / 32;
            if ((rc = ix->tmp_blk.reserve((size_t)max_groups * ix->group_bytes())) != VF_OK) return rc;
            if ((rc = ix->tmp_norm.reserve((size_t)max_groups * 32 * 4)) != VF_OK) return rc;
            if ((rc = cand_idx.reserve((size_t)max_groups * 32 * K * 4)) != VF_OK) return rc;
            if ((rc = cand_dist.reserve((size_t)max_groups * 32 * K * 4)) != VF_OK) return rc;
            // VF_BUILD_PROGRESS=1: a line on stderr every few seconds (index builds of 10^7 vectors take minutes)
            const char *prog_env = getenv("VF_BUILD_PROGRESS");
            const bool progress = prog_env && prog_env[0] == '1';
            time_t last_print = time(nullptr);
            size_t done = 0;
            for (int32_t l : ix->graph_labels) {
                if (progress && time(nullptr) - last_print >= 10) {
                    fprintf(stderr, "[vf_build_index] %zu of %zu label graphs built, next list holds %d vectors\n", done,
                            ix->graph_labels.size(), ix->S[(size_t)l]);
                    fflush(stderr);
                    last_print = time(nullptr);
                }
                ++done;
                launch_bitset_fill(ix->d_M_HS.as<int32_t>() + ix->O_HS[(size_t)l], ix->S[(size_t)l],
                                   ix->d_bitsets.as<uint32_t>() + (int64_t)ix->hs_slot[(size_t)l] * ix->bitset_words, s);
                const int64_t base = ix->O_HS[(size_t)l];
                int32_t *rows = pruned ? d_knn.as<int32_t>() + base * D : ix->d_G.as<int32_t>() + base * ix->R;
                if ((rc = build_graph_for_label(ix, l, K, D, rows, !pruned, cand_idx, cand_dist, d_items, s)) != VF_OK)
                    return rc;
            }
            VF_HIP(hipStreamSynchronize(s));
            if (pruned) {
                cand_idx.release(); cand_dist.release();
                if ((rc = optimize_graphs(ix, d_knn.as<int32_t>(), D, s)) != VF_OK) return rc;
            }
            ix->graph_kind = graph_kind; ix->knn_degree = pruned ? D : 0;
            ix->tmp_blk.release();
            ix->tmp_norm.release();
            if (seed_mfma_supported(ix->dtype, ix->dim)) {
                const char *ex = getenv("VF_SEED_EXACT");
                if (!(ex && ex[0] == '1')) {
                    if ((rc = ix->d_xnorm_all.reserve((size_t)n * 4)) != VF_OK) return rc;
                    launch_row_norms(ix->dtype, ix->X, ix->dim, n, ix->d_xnorm_all.as<uint32_t>(), s);
                    float mx = 0.f;
                    bool finite = true;
                    if (ix->dtype == VF_F32) {
                        std::vector<float> hn((size_t)n);
                        VF_HIP(hipMemcpyAsync(hn.data(), ix->d_xnorm_all.p, (size_t)n * 4, hipMemcpyDeviceToHost, s));
                        VF_HIP(hipStreamSynchronize(s));
                        for (float v : hn) { finite = finite && v == v && v <= 3.0e38f; mx = v > mx ? v : mx; }
                    }
                    // a table with NaN or overflowing norms keeps the exact kernel, and so does one whose largest
                    // squared norm is outside [1e-24, 1e30]: the bound below is relative to that norm and assumes
                    // that what the matrix cores flush (products under 1.2e-38) is negligible beside it
                    if (ix->dtype == VF_F32 && !(mx >= 1e-24f && mx <= 1e30f)) finite = false;
                    if (finite) {
                        ix->xn_max = mx;
                        // |approximation - ordered distance| <= 300 u (|q|^2 + |x|^2), u = 2^-24 (dot product of
                        // <= 512 terms in any order, two norms, the final additions, the ordered sum's own
                        // error); 512 u = 2^-15 is used
                        float slack = 1.0f;
                        if (const char *e = getenv("VF_SEED_SLACK")) slack = (float)atof(e);
                        ix->seed_err_bound = slack * 3.0517578125e-05f;
                        ix->seed_mfma = true;
                    }
                }
            }
        }
        VF_HIP(hipGetLastError());
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return VF_ENOMEM;
    }
    {
        const char *e = getenv("VF_NO_OVERLAP");
        ix->overlap = !(e && e[0] == '1');
    }
    guard.ix = nullptr;
    *out = ix;
    return VF_OK;
}

// ---------------------------------------------------------------- routing

// Add the durations of the last profiled call to the running sums (waits for it).
// Adds the durations of the oldest `count` unread profiled calls to the sums (waits for them).
static int fold_profile(vf_index *ix, int count)
{
    for (; count > 0 && ix->prof_unfolded > 0; --count, --ix->prof_unfolded) {
        const int slot = (ix->prof_next - ix->prof_unfolded + 2 * vf_index::kProfRing) % vf_index::kProfRing;
        hipEvent_t *ev = ix->prof_ring[slot];
        VF_HIP(hipEventSynchronize(ev[4]));
        VF_HIP(hipEventSynchronize(ev[1]));
        VF_HIP(hipEventElapsedTime(&ix->prof.scan_ms, ev[0], ev[1]));
        VF_HIP(hipEventElapsedTime(&ix->prof.seed_ms, ev[2], ev[3]));
        VF_HIP(hipEventElapsedTime(&ix->prof.beam_ms, ev[3], ev[4]));
        ix->prof_scan_sum += ix->prof.scan_ms;
        ix->prof_seed_sum += ix->prof.seed_ms;
        ix->prof_beam_sum += ix->prof.beam_ms;
        ix->prof_calls++;
    }
    return VF_OK;
}

namespace {

// ClassifyQueries (Alg. 2) + smallest-list choice (Section 4.3.2).  Queries are grouped by the
// label they search with a counting sort: O(nq + labels touched), no comparison sort of the batch.
int route_queries(const vf_index *ix, int64_t nq, const int64_t *qoff, const int32_t *qids, bool all_scan,
                  bool first_is_searched, Routed &r)
{
    VF_REQUIRE(qoff && qids, "NULL query label arrays");
    VF_REQUIRE(qoff[0] >= 0, "qlabel_offsets[0] must be >= 0");
    r.others_off.assign((size_t)nq + 1, 0);
    r.others.clear();
    r.any_and = false;
    r.empty_q.clear();
    r.q_best.resize((size_t)nq);
    if (r.cnt.size() != (size_t)ix->n_labels) r.cnt.assign((size_t)ix->n_labels, 0);
    r.touched.clear();
    struct Reset {   // the counters must be zero again on every exit path
        Routed &r;
        ~Reset() { for (int32_t l : r.touched) r.cnt[(size_t)l] = 0; }
    } reset{r};
    int32_t labs[kMaxOthers + 1];
    for (int64_t j = 0; j < nq; ++j) {
        const int64_t b = qoff[j], e = qoff[j + 1];
        VF_REQUIRE(e > b, "every query needs at least one label");
        int32_t nl = 0;
        for (int64_t p = b; p < e; ++p) {
            const int32_t l = qids[p];
            VF_REQUIRE(l >= 0 && l < ix->n_labels, "query label outside [0, n_labels)");
            bool seen = false;
            for (int32_t i = 0; i < nl; ++i) seen = seen || labs[i] == l;
            if (seen) continue;
            VF_REQUIRE(nl <= kMaxOthers, "more than 8 distinct labels in one query");
            labs[nl++] = l;
        }
        int32_t best = labs[0];
        bool empty = false;
        for (int32_t i = 0; i < nl; ++i) {
            const int32_t l = labs[i];
            const int32_t sl = ix->S[(size_t)l], sb = ix->S[(size_t)best];
            if (sl == 0) empty = true;
            if (!first_is_searched && (sl < sb || (sl == sb && l < best))) best = l;
        }
        if (!empty) {
            for (int32_t i = 0; i < nl; ++i)
                if (labs[i] != best) r.others.push_back(labs[i]);
            if (nl > 1) r.any_and = true;
            if (r.cnt[(size_t)best]++ == 0) r.touched.push_back(best);
        }
        r.q_best[(size_t)j] = empty ? -1 : best;
        if (empty) r.empty_q.push_back((int32_t)j);
        r.others_off[(size_t)j + 1] = (int32_t)r.others.size();
    }
    // offsets per touched label, graph labels and scan labels in separate outputs, each by ascending label
    std::sort(r.touched.begin(), r.touched.end());
    size_t n_g = 0, n_s = 0;
    for (int32_t l : r.touched) {
        const bool graph = !all_scan && ix->S[(size_t)l] >= ix->T;
        const int32_t c = r.cnt[(size_t)l];
        // reuse the counter as "next free position" (graph positions are stored negated - 1)
        if (graph) { r.cnt[(size_t)l] = -(int32_t)n_g - 1; n_g += (size_t)c; }
        else { r.cnt[(size_t)l] = (int32_t)n_s + 1; n_s += (size_t)c; }
    }
    r.gq_query.resize(n_g); r.gq_label.resize(n_g); r.scan_pairs.resize(n_s);
    for (int64_t j = 0; j < nq; ++j) {
        const int32_t l = r.q_best[(size_t)j];
        if (l < 0) continue;
        int32_t &c = r.cnt[(size_t)l];
        if (c < 0) {
            const size_t at = (size_t)(-c - 1);
            r.gq_query[at] = (int32_t)j; r.gq_label[at] = l;
            --c;
        } else {
            const size_t at = (size_t)(c - 1);
            r.scan_pairs[at] = ((uint64_t)(uint32_t)l << 32) | (uint32_t)j;
            ++c;
        }
    }
    return VF_OK;
}

struct BlobLayout {
    size_t off_gq_query, off_gq_label, off_others_off, off_others, off_qrow, off_items, off_merges, off_tiles, off_empty, total;
};

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

// The workspace of the calls on stream s: the one the stream has used before, else a free one, else one taken
// from another stream once that stream has drained.
static int workspace_for(vf_index *ix, hipStream_t s, Workspace **out)
{
    Workspace *w = nullptr;
    for (Workspace &c : ix->ws)
        if (c.owned && c.owner == s) { w = &c; break; }
    if (!w)
        for (Workspace &c : ix->ws)
            if (!c.owned) { w = &c; break; }
    if (!w) {
        // every workspace has an owner: take one whose streams are idle, else the next in turn once its streams
        // have drained (a stream its owner has destroyed meanwhile has drained; the error that reports it is dropped)
        for (Workspace &c : ix->ws) {
            const hipError_t qo = hipStreamQuery(c.owner), qs = hipStreamQuery(c.side);
            if (qo != hipSuccess || qs != hipSuccess) (void)hipGetLastError();
            if (qo != hipErrorNotReady && qs == hipSuccess) { w = &c; break; }
        }
        if (!w) {
            w = &ix->ws[ix->ws_steal];
            ix->ws_steal = (ix->ws_steal + 1) % vf_index::kWorkspaces;
            if (hipStreamSynchronize(w->owner) != hipSuccess) (void)hipGetLastError();
            VF_HIP(hipStreamSynchronize(w->side));
        }
    }
    w->owned = true;
    w->owner = s;
    if (!w->ready) {
        VF_HIP(hipStreamCreateWithFlags(&w->side, hipStreamNonBlocking));
        VF_HIP(hipEventCreateWithFlags(&w->ev_fork, hipEventDisableTiming));
        VF_HIP(hipEventCreateWithFlags(&w->ev_join, hipEventDisableTiming));
        VF_HIP(hipEventCreateWithFlags(&w->ev_copy, hipEventDisableTiming));
        for (hipEvent_t &e : w->ev_blob_done) VF_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        w->ready = true;
    }
    *out = w;
    return VF_OK;
}

static int get_staging(Workspace *W, size_t bytes, Staging **out)
{
    Staging &st = W->stage[W->stage_next];
    W->stage_next ^= 1;
    if (st.pending) { VF_HIP(hipEventSynchronize(st.done)); st.pending = false; }
    if (!st.done) VF_HIP(hipEventCreateWithFlags(&st.done, hipEventDisableTiming));
    if (bytes > st.cap) {
        if (st.p) { (void)hipHostFree(st.p); st.p = nullptr; st.cap = 0; }
        const size_t want = bytes + bytes / 2 + 4096;
        VF_HIP(hipHostMalloc(&st.p, want, hipHostMallocDefault));
        st.cap = want;
    }
    *out = &st;
    return VF_OK;
}

static int check_search_args(const vf_index *ix, const void *queries, int64_t nq, int32_t k, const int64_t *out_ids,
                             const float *out_dists)
{
    VF_REQUIRE(ix != nullptr, "index is NULL");
    VF_REQUIRE(nq >= 0 && nq < ((int64_t)1 << 31), "nq out of range");
    VF_REQUIRE(nq == 0 || (queries && out_ids && out_dists), "NULL query or output pointer");
    VF_REQUIRE(((uintptr_t)queries & 15) == 0, "queries must be 16-byte aligned");
    VF_REQUIRE(k >= 1 && k <= 64, "k must be in [1, 64]");
    return VF_OK;
}

// Work list of the scan path.  The (label, query) pairs of one label are cut into
// tiles of <= 32 queries; a long list is cut into segments of whole 32-vector groups
// so that many waves share it, and a merge item per query then combines the segments.
constexpr int kMaxSegs = 64;

static int env_int(const char *name, int dflt, int lo, int hi)
{
    const char *e = getenv(name);
    if (!e || !*e) return dflt;
    const int v = atoi(e);
    return v < lo ? lo : (v > hi ? hi : v);
}
// tuning knobs (the environment overrides exist for experiments)
static const int kSegGroups = env_int("VF_SEG_GROUPS", 16, 1, 4096);  // 32-vector groups per list segment
static const int kSegGroupsHeavy = env_int("VF_SEG_GROUPS_HEAVY", 16, 1, 4096);  // the same for tiles of >= kHeavyRows queries
static const int kHeavyRows = env_int("VF_SEG_HEAVY_ROWS", 9, 1, 33);
static const int kZeroCopyBytes = env_int("VF_ZERO_COPY_BYTES", 8192, 0, 1 << 20);  // blobs up to this size are read in place
static const int kFallbackWindow = env_int("VF_SEED_FB_WINDOW", 131072, 1, 1 << 30);  // graph queries between two looks at the failed proofs
static const int kSeedMargin = env_int("VF_SEED_MARGIN", 8, 1, 32);  // matrix-core seed scores kept beyond itopk for re-ranking
static const int kScanValu = env_int("VF_SCAN_VALU", 1, 0, 2);      // float32 FMA scan kernel: 0 never, 1 for small batches, 2 always
static const int kScan16 = env_int("VF_SCAN16", 1, 0, 1);          // 0: float32 search tiles keep the 32-row matrix-core kernel
static const int kTileRows = env_int("VF_TILE_ROWS", 16, 1, 32);      // queries per scan tile

struct ItemBuilder {
    std::vector<int32_t> qrow;
    std::vector<ScanItem> items;
    std::vector<MergeItem> merges;
    int64_t part_rows = 0;
    int32_t max_nseg = 1;
    int32_t tile_rows = kTileRows;

    // pairs[lo, hi) all carry the same label, whose list is (group0, map_off, n)
    void add_label(const std::vector<uint64_t> &pairs, size_t lo, size_t hi, int64_t group0, int64_t map_off, int32_t n)
    {
        const int32_t n_groups = (n + 31) / 32;
        for (size_t t = lo; t < hi; t += (size_t)tile_rows) {
            const int32_t q_begin = (int32_t)qrow.size();
            const int32_t q_count = (int32_t)std::min<size_t>((size_t)tile_rows, hi - t);
            // a tile's work item is a serial chain whose cost per group grows with its queries (selection):
            // tiles with many queries get shorter segments, so that the items of a launch end together
            const int32_t want = q_count >= kHeavyRows ? kSegGroupsHeavy : kSegGroups;
            const int32_t seg_groups = std::max(want, (n_groups + kMaxSegs - 1) / kMaxSegs);
            const int32_t nseg = (n_groups + seg_groups - 1) / seg_groups;
            max_nseg = std::max(max_nseg, nseg);
            for (size_t u = t; u < t + (size_t)q_count; ++u) qrow.push_back((int32_t)(uint32_t)pairs[u]);
            for (int32_t sg = 0; sg < nseg; ++sg) {
                ScanItem it{};
                it.group0 = group0 + (int64_t)sg * seg_groups;
                it.map_off = map_off;
                it.entry0 = sg * seg_groups * 32;
                it.n = std::min(seg_groups * 32, n - it.entry0);
                it.q_begin = q_begin; it.q_count = q_count; it.self_base = -1;
                it.part_row = nseg == 1 ? -1 : (int32_t)(part_rows + (int64_t)sg * q_count);
                items.push_back(it);
            }
            if (nseg > 1) {
                for (int32_t r = 0; r < q_count; ++r)
                    merges.push_back(MergeItem{map_off, qrow[(size_t)q_begin + r], (int32_t)(part_rows + r), q_count, nseg});
                part_rows += (int64_t)nseg * q_count;
            }
        }
    }
};

// Interleaved copy of the seeds (local ids floor(j n / ns), j < ns = min(n_seeds, n)) of every graph list.
// Depends on the index and on n_seeds only; rebuilt on the caller's stream when n_seeds changes, skipped
// (seed_cache_ok = false) when it would need more than half of the free device memory.
static int ensure_seed_cache(vf_index *ix, int32_t n_seeds, hipStream_t s)
{
    static const int enabled = env_int_early("VF_SEED_CACHE", 1);
    if (ix->seed_cache_ns == n_seeds) return VF_OK;
    ix->seed_cache_ns = n_seeds;
    ix->seed_cache_ok = false;
    if (!enabled) return VF_OK;
    const size_t n_gl = ix->graph_labels.size();
    std::vector<int64_t> goff(n_gl), slot_base(n_gl);
    std::vector<int32_t> slot_n(n_gl), grp_slot, grp_j0, grp_cnt;
    std::vector<int64_t> grp_src;
    int64_t n_groups = 0;
    for (size_t t = 0; t < n_gl; ++t) {
        const int32_t l = ix->graph_labels[t];
        const int32_t n = ix->S[(size_t)l], ns = std::min(n_seeds, n);
        goff[t] = n_groups; slot_base[t] = ix->O_HS[(size_t)l]; slot_n[t] = n;
        for (int32_t j0 = 0; j0 < ns; j0 += 32) {
            grp_slot.push_back((int32_t)t); grp_j0.push_back(j0);
            grp_src.push_back(n_groups * 32); grp_cnt.push_back(std::min(32, ns - j0));
            ++n_groups;
        }
    }
    if (n_groups == 0) return VF_OK;
    const size_t need = (size_t)n_groups * (ix->group_bytes() * 3 / 2 + 32 * 4 + 32 * 4 + 32 * 4 + 32);
    if (need > ix->seed_blk.cap) {
        size_t free_b = 0, total_b = 0;
        VF_HIP(hipMemGetInfo(&free_b, &total_b));
        if (need + need / 4 > (free_b + ix->seed_blk.cap) / 2) return VF_OK;
    }
    int rc;
    DevBuf d_map, d_base, d_n, d_slot, d_j0, d_src, d_cnt;
    struct Rel { DevBuf *b[7]; ~Rel() { for (DevBuf *x : b) x->release(); } } rel{{&d_map, &d_base, &d_n, &d_slot, &d_j0, &d_src, &d_cnt}};
    if ((rc = ix->seed_blk.reserve((size_t)n_groups * ix->group_bytes())) != VF_OK) return rc;
    if ((rc = ix->seed_norm.reserve((size_t)n_groups * 32 * 4)) != VF_OK) return rc;
    if ((rc = d_map.reserve((size_t)n_groups * 32 * 4)) != VF_OK) return rc;
    if ((rc = upload(ix->seed_goff, goff, s)) != VF_OK) return rc;
    if ((rc = upload(d_base, slot_base, s)) != VF_OK) return rc;
    if ((rc = upload(d_n, slot_n, s)) != VF_OK) return rc;
    if ((rc = upload(d_slot, grp_slot, s)) != VF_OK) return rc;
    if ((rc = upload(d_j0, grp_j0, s)) != VF_OK) return rc;
    if ((rc = upload(d_src, grp_src, s)) != VF_OK) return rc;
    if ((rc = upload(d_cnt, grp_cnt, s)) != VF_OK) return rc;
    launch_seed_map(ix->d_M_HS.as<int32_t>(), d_base.as<int64_t>(), d_n.as<int32_t>(), n_seeds, d_slot.as<int32_t>(),
                    d_j0.as<int32_t>(), n_groups, d_map.as<int32_t>(), s);
    launch_interleave(ix->dtype, ix->X, ix->dim, d_map.as<int32_t>(), d_src.as<int64_t>(), d_cnt.as<int32_t>(),
                      n_groups * 32, n_groups, ix->ncp, ix->seed_blk.as<uint4>(), ix->seed_norm.p, s);
    VF_HIP(hipGetLastError());
    VF_HIP(hipStreamSynchronize(s));   // the tables above are pageable host memory and temporaries
    ix->seed_bf16 = false;
    ix->seed_f32 = true;
    ix->seed_blk16.release();
    static const int want_bf16 = env_int_early("VF_SEED_BF16", 1);
    if (ix->dtype == VF_F32 && want_bf16 && !ix->seed_bf16_off) {
        // float32 data: a second copy in bfloat16; the largest rounding error of a seed goes into the
        // beam kernel's proof (zero for integer-valued data up to 256, SIFT's kind)
        DevBuf d_err2;
        struct Rel2 { DevBuf *b[1]; ~Rel2() { for (DevBuf *x : b) x->release(); } } rel2{{&d_err2}};
        if ((rc = ix->seed_blk16.reserve((size_t)n_groups * ix->group_bytes() / 2)) != VF_OK) return rc;
        if ((rc = d_err2.reserve((size_t)n_groups * 32 * 4)) != VF_OK) return rc;
        launch_seed_pack_bf16(ix->seed_blk.as<uint4>(), n_groups, ix->ncp, ix->seed_blk16.as<uint4>(), d_err2.as<float>(), s);
        std::vector<float> e2((size_t)n_groups * 32);
        VF_HIP(hipMemcpyAsync(e2.data(), d_err2.p, e2.size() * 4, hipMemcpyDeviceToHost, s));
        VF_HIP(hipStreamSynchronize(s));
        double mx = 0.0;
        bool finite = true;
        for (float v : e2) { finite = finite && v == v && v <= 3.0e38f; mx = v > mx ? v : mx; }
        if (!finite) ix->seed_blk16.release();
        if (finite) {
            // small batches are served from the float32 copy (its proofs need fewer re-scored seeds, which
            // is what a latency-bound call notices), so a copy of up to 128 MiB stays
            if ((size_t)n_groups * ix->group_bytes() > ((size_t)128 << 20)) {
                ix->seed_blk.release();
                ix->seed_f32 = false;
            }
            ix->seed_bf16 = true;
            ix->seed_bf16_delta = (float)(std::sqrt(mx) * 1.001);
            if (!ix->h_fb) {
                if ((rc = ix->d_fb_count.reserve(4)) != VF_OK) return rc;
                VF_HIP(hipMemsetAsync(ix->d_fb_count.p, 0, 4, s));
                VF_HIP(hipStreamSynchronize(s));
                VF_HIP(hipHostMalloc((void **)&ix->h_fb, 4, hipHostMallocDefault));
                *ix->h_fb = 0;
                VF_HIP(hipEventCreateWithFlags(&ix->ev_fb, hipEventDisableTiming));
            }
        }
    }
    ix->seed_cache_ok = true;
    return VF_OK;
}

// first_is_searched: every query searches the list of its first label (the others are the
// predicate) instead of its smallest list -- the sub-searches of vf_search_multi.
static int search_impl(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids, int32_t k,
                       int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds, bool exact, int64_t *out_ids,
                       float *out_dists, hipStream_t s, bool first_is_searched = false)
{
    int rc = check_search_args(ix, queries, nq, k, out_ids, out_dists);
    if (rc != VF_OK) return rc;
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    Workspace *W = nullptr;
    if ((rc = workspace_for(ix, s, &W)) != VF_OK) return rc;
    if (!exact) {
        VF_REQUIRE(itopk >= k && itopk >= 1 && itopk <= 256, "itopk must be in [k, 256]");
        VF_REQUIRE(width >= 1 && width <= 8 && width * ix->R <= 128, "width must be >= 1 with width * R <= 128");
        VF_REQUIRE(iters >= 0, "iters must be >= 0");
        VF_REQUIRE(n_seeds >= 0, "n_seeds must be >= 0");
        if (n_seeds == 0) n_seeds = itopk;
    }
    // beam kernel geometry: list slots and visited-table size; checked before anything is launched
    int32_t beam_LP = 128, beam_hb = 9;
    if (!exact) {
        while (beam_LP < itopk + std::max(64, width * ix->R)) beam_LP <<= 1;
        const int64_t visits = (int64_t)iters * width * ix->R;
        while (beam_hb < 13 && ((int64_t)1 << beam_hb) < 2 * visits) ++beam_hb;
        BeamParams chk{};
        chk.dim = ix->dim; chk.LP = beam_LP; chk.hash_bits = beam_hb;
        VF_REQUIRE(beam_lds_bytes(chk, ix->dtype) <= 64 * 1024, "search parameters need more than 64 KiB of LDS");
    }
    if (nq == 0) return VF_OK;
    try {
        Routed &r = W->routed;
        if ((rc = route_queries(ix, nq, qoff, qids, exact, first_is_searched, r)) != VF_OK) return rc;

        // scan items over the stored interleaved lists (scan labels); in exact mode graph labels follow
        ItemBuilder ib;
        size_t first_hs = r.scan_pairs.size();
        if (exact) {
            // scan labels first, graph labels after them (both still ordered by label)
            std::stable_partition(r.scan_pairs.begin(), r.scan_pairs.end(), [&](uint64_t pr) {
                return ix->O_LS[(size_t)(pr >> 32)] >= 0;
            });
            first_hs = 0;
            while (first_hs < r.scan_pairs.size() && ix->O_LS[(size_t)(r.scan_pairs[first_hs] >> 32)] >= 0) ++first_hs;
        }
        for (size_t i = 0; i < first_hs;) {
            const int32_t l = (int32_t)(r.scan_pairs[i] >> 32);
            size_t e = i;
            while (e < first_hs && (int32_t)(r.scan_pairs[e] >> 32) == l) ++e;
            ib.add_label(r.scan_pairs, i, e, ix->GO_LS[(size_t)l], ix->O_LS[(size_t)l], ix->S[(size_t)l]);
            i = e;
        }
        const size_t n_ls_items = ib.items.size(), n_ls_merges = ib.merges.size();
        // exact mode: one temporary interleaved copy per graph label, used right after it is made
        struct HsRun { int32_t label; size_t item_lo, item_hi; };
        std::vector<HsRun> hs_runs;
        int32_t max_hs_list = 0;
        for (size_t i = first_hs; i < r.scan_pairs.size();) {
            const int32_t l = (int32_t)(r.scan_pairs[i] >> 32);
            size_t e = i;
            while (e < r.scan_pairs.size() && (int32_t)(r.scan_pairs[e] >> 32) == l) ++e;
            const size_t lo = ib.items.size();
            ib.add_label(r.scan_pairs, i, e, 0, ix->O_HS[(size_t)l], ix->S[(size_t)l]);
            hs_runs.push_back({l, lo, ib.items.size()});
            max_hs_list = std::max(max_hs_list, ix->S[(size_t)l]);
            i = e;
        }
        std::vector<int32_t> &qrow = ib.qrow;
        std::vector<ScanItem> &items = ib.items;

        const size_t n_gq = r.gq_query.size();
        // dense seed scoring: tiles of <= 64 graph queries that search the same label
        std::vector<SeedTile> tiles;
        const int32_t ns_stride = (n_seeds + 31) & ~31;
        // the seed distance matrix must fit: reuse what is allocated, or grow into at most half of the free memory
        bool dseed_fits = true;
        {
            const uint64_t need = (uint64_t)n_gq * (uint64_t)ns_stride * 4;
            if (need > W->dseed.cap) {
                size_t free_b = 0, total_b = 0;
                VF_HIP(hipMemGetInfo(&free_b, &total_b));
                dseed_fits = need + need / 4 + 256 <= (free_b + W->dseed.cap) / 2;
            }
        }
        const bool dense_seeds = !exact && n_gq > 0 && seed_dist_supported(ix->dtype, ix->dim) && dseed_fits;
        // uint8: the matrix cores give the exact integer distances, nothing else changes.
        // float32: approximations, re-ranked by the beam kernel (its proof needs a list of at most 48 entries).
        const bool seeds_mfma = dense_seeds && ix->seed_mfma && n_seeds > 64 &&
                                (ix->dtype == VF_U8 || itopk <= 48);
        if (dense_seeds) {
            const size_t tile_q = seeds_mfma ? 32 : 64;
            for (size_t i = 0; i < n_gq;) {
                size_t e = i;
                while (e < n_gq && r.gq_label[e] == r.gq_label[i]) ++e;
                for (size_t t = i; t < e; t += tile_q)
                    tiles.push_back(SeedTile{r.gq_label[i], (int32_t)t, (int32_t)std::min<size_t>(tile_q, e - t)});
                i = e;
            }
        }
        BlobLayout L;
        size_t o = 0;
        L.off_gq_query = o; o = align_up(o + n_gq * 4);
        L.off_gq_label = o; o = align_up(o + n_gq * 4);
        L.off_others_off = o; o = align_up(o + r.others_off.size() * 4);
        L.off_others = o; o = align_up(o + std::max<size_t>(r.others.size(), 1) * 4);
        L.off_qrow = o; o = align_up(o + std::max<size_t>(qrow.size(), 1) * 4);
        L.off_items = o; o = align_up(o + std::max<size_t>(items.size(), 1) * sizeof(ScanItem));
        L.off_merges = o; o = align_up(o + std::max<size_t>(ib.merges.size(), 1) * sizeof(MergeItem));
        L.off_tiles = o; o = align_up(o + std::max<size_t>(tiles.size(), 1) * sizeof(SeedTile));
        L.off_empty = o; o = align_up(o + std::max<size_t>(r.empty_q.size(), 1) * 4);
        L.total = o;

        Staging *st = nullptr;
        if ((rc = get_staging(W, L.total, &st)) != VF_OK) return rc;
        char *hp = (char *)st->p;
        if (n_gq) {
            memcpy(hp + L.off_gq_query, r.gq_query.data(), n_gq * 4);
            memcpy(hp + L.off_gq_label, r.gq_label.data(), n_gq * 4);
        }
        memcpy(hp + L.off_others_off, r.others_off.data(), r.others_off.size() * 4);
        if (!r.others.empty()) memcpy(hp + L.off_others, r.others.data(), r.others.size() * 4);
        if (!qrow.empty()) memcpy(hp + L.off_qrow, qrow.data(), qrow.size() * 4);
        if (!items.empty()) memcpy(hp + L.off_items, items.data(), items.size() * sizeof(ScanItem));
        if (!ib.merges.empty()) memcpy(hp + L.off_merges, ib.merges.data(), ib.merges.size() * sizeof(MergeItem));
        if (!tiles.empty()) memcpy(hp + L.off_tiles, tiles.data(), tiles.size() * sizeof(SeedTile));
        if (!r.empty_q.empty()) memcpy(hp + L.off_empty, r.empty_q.data(), r.empty_q.size() * 4);
        if (dense_seeds && (rc = W->dseed.reserve(((size_t)n_gq * ns_stride + 64 * 1024) * 4)) != VF_OK) return rc;
        if (ib.part_rows > 0) {
            VF_REQUIRE(ib.part_rows < ((int64_t)1 << 31), "too many partial result rows in one call");
            if ((rc = W->part_idx.reserve((size_t)ib.part_rows * k * 4)) != VF_OK) return rc;
            if ((rc = W->part_bits.reserve((size_t)ib.part_rows * k * 4)) != VF_OK) return rc;
        }
        // The scan path runs on the side stream beside the graph path on the caller's stream.
        const bool forked = ix->overlap && !ix->prof_serial && !exact && n_gq > 0 && !items.empty();
        // Two device blobs alternate.  When the call forks, its blob is uploaded on the side stream: there it
        // follows the previous call's scan, not the previous call's beam search, so the upload is off the
        // critical path.  The buffer was last read two calls ago; the upload waits for that call's end.
        // A small blob (small batches) is not copied at all: the kernels read the few hundred bytes they need
        // straight from the pinned staging buffer, which saves the copy's submission and its latency; the
        // staging buffer then stays untouched until the call's last kernel has ended.
        const bool zero_copy = kZeroCopyBytes > 0 && L.total <= (size_t)kZeroCopyBytes;
        const int bsel = W->blob_next;
        DevBuf &blob = bsel ? W->ws_blob_b : W->ws_blob;
        char *dp = nullptr;
        if (zero_copy) {
            void *dev_view = nullptr;
            VF_HIP(hipHostGetDevicePointer(&dev_view, st->p, 0));
            dp = (char *)dev_view;
        } else {
            W->blob_next ^= 1;
            if ((rc = blob.reserve(L.total)) != VF_OK) return rc;
            dp = blob.as<char>();
            hipStream_t cs = forked ? W->side : s;
            if (forked && W->blob_used[bsel]) VF_HIP(hipStreamWaitEvent(cs, W->ev_blob_done[bsel], 0));
            VF_HIP(hipMemcpyAsync(dp, hp, L.total, hipMemcpyHostToDevice, cs));
            VF_HIP(hipEventRecord(st->done, cs));
            st->pending = true;
            if (forked) {
                VF_HIP(hipEventRecord(W->ev_copy, cs));
                VF_HIP(hipStreamWaitEvent(s, W->ev_copy, 0));
            }
        }

        // every routed query's kernel writes all k entries of its row; only queries without any match are padded here
        launch_fill_rows(out_ids, out_dists, (const int32_t *)(dp + L.off_empty), (int64_t)r.empty_q.size(), k, s);

        const bool prof = ix->profiling;
        if (prof) {
            if (ix->prof_unfolded == vf_index::kProfRing && (rc = fold_profile(ix, 1)) != VF_OK) return rc;
            ix->prof_ev = ix->prof_ring[ix->prof_next];
            // [nq][4] counters, then [nq] gathered; written by the beam kernel for graph queries only (no clearing
            // pass: the rows of the other queries are never read)
            if ((rc = ix->counters.reserve((size_t)nq * 20)) != VF_OK) return rc;
            ix->prof_graph_queries = r.gq_query;
            vf_profile &pf = ix->prof;
            pf = vf_profile{};
            pf.nq = nq; pf.n_graph_queries = (int64_t)r.gq_query.size(); pf.n_scan_queries = (int64_t)qrow.size();
            pf.n_scan_items = (int64_t)items.size();
            for (const ScanItem &it : items) { pf.scan_list_entries += it.n; pf.scan_pairs += (int64_t)it.n * it.q_count; }
            pf.n_seed_tiles = (int64_t)tiles.size();
            pf.seeds_on_matrix_cores = seeds_mfma ? 1 : 0;
            for (const SeedTile &t : tiles) {
                const int64_t ns_l = std::min<int64_t>(n_seeds, ix->S[(size_t)t.label]);
                pf.seed_pairs += ns_l * t.q_count;
                pf.seed_tile_seeds += ns_l;
            }
        }
        hipStream_t ss = s;
        const int32_t *d_others_off = r.any_and ? (const int32_t *)(dp + L.off_others_off) : nullptr;
        const int32_t *d_others = (const int32_t *)(dp + L.off_others);

        BeamParams bp{};
        if (n_gq) {
            bp.X = ix->X; bp.Q = queries; bp.G = ix->d_G.as<int32_t>(); bp.Gg = ix->d_Gg.as<int32_t>();
            bp.gq_query = (const int32_t *)(dp + L.off_gq_query);
            bp.gq_label = (const int32_t *)(dp + L.off_gq_label);
            bp.others_off = d_others_off; bp.others = d_others; bp.meta = ix->meta();
            bp.dim = ix->dim; bp.R = ix->R; bp.k = k; bp.itopk = itopk; bp.width = width; bp.iters = iters;
            bp.n_seeds = n_seeds;
            bp.LP = beam_LP;
            bp.hash_bits = beam_hb;
            bp.out_ids = out_ids; bp.out_dists = out_dists;
            bp.counters = prof ? ix->counters.as<int32_t>() : nullptr;
            bp.gathered = prof ? ix->counters.as<int32_t>() + (size_t)nq * 4 : nullptr;
            bp.dseed = nullptr; bp.ns_stride = ns_stride;
        }
        auto run_seeds = [&]() -> int {
            if (prof) VF_HIP(hipEventRecord(ix->prof_ev[2], s));
            if (n_gq) {
                if (dense_seeds) {
                    SeedParams sd{};
                    sd.X = ix->X; sd.Q = queries; sd.gq_query = bp.gq_query;
                    sd.tiles = (const SeedTile *)(dp + L.off_tiles); sd.meta = bp.meta;
                    sd.dim = ix->dim; sd.n_seeds = n_seeds; sd.ns_stride = ns_stride;
                    sd.dseed = W->dseed.as<uint32_t>();
                    sd.dump_off = (int64_t)n_gq * ns_stride;
                    sd.dump_mask = 1023;
                    if (seeds_mfma) {
                        sd.chunk_seeds = kSeedMfmaChunk;
                        sd.max_chunks = (ns_stride + kSeedMfmaChunk - 1) / kSeedMfmaChunk;
                        sd.xnorm_all = ix->d_xnorm_all.as<uint32_t>();
                        if (ix->fb_pending && hipEventQuery(ix->ev_fb) == hipSuccess) {
                            const uint32_t now = *ix->h_fb, failed = now - ix->fb_last;
                            ix->fb_last = now;
                            ix->fb_pending = false;
                            if ((int64_t)failed * 64 > ix->fb_sent_q) {
                                ix->seed_bf16_off = true;
                                ix->seed_cache_ns = -1;   // the copy is rebuilt in float32 below
                            }
                        } else if (ix->fb_pending) {
                            (void)hipGetLastError();      // "not ready" is no error
                        }
                        if ((rc = ensure_seed_cache(ix, n_seeds, s)) != VF_OK) return rc;
                        if (ix->seed_cache_ok) {
                            static const int min16 = env_int_early("VF_SEED_BF16_MIN_BATCH", 512);
                            const bool use16 = ix->seed_bf16 && (!ix->seed_f32 || (int64_t)n_gq >= min16);
                            sd.seed_blk = use16 ? ix->seed_blk16.as<uint4>() : ix->seed_blk.as<uint4>();
                            sd.seed_norm = ix->seed_norm.as<uint32_t>();
                            sd.seed_goff = ix->seed_goff.as<int64_t>();
                            sd.seed_bf16 = use16 ? 1 : 0;
                            if (prof && sd.seed_bf16) ix->prof.seeds_on_matrix_cores = 2;
                            // seeds per wave: few long waves share the chip better with the scan (512 seeds:
                            // step 0.374 -> 0.340 ms on 10,000-query batches), small batches need many short ones
                            sd.chunk_seeds = 4 * kSeedMfmaChunk;
                            if ((int64_t)tiles.size() * ((ns_stride + sd.chunk_seeds - 1) / sd.chunk_seeds) < 512)
                                sd.chunk_seeds = kSeedMfmaChunk;
                            sd.max_chunks = (ns_stride + sd.chunk_seeds - 1) / sd.chunk_seeds;
                        }
                        launch_seed_mfma(ix->dtype, sd, (int)tiles.size(), s);
                        if (ix->dtype == VF_F32) {
                            bp.seed_approx = 1; bp.err_bound = ix->seed_err_bound; bp.xn_max = ix->xn_max;
                            bp.seed_keep = std::min(64, itopk + kSeedMargin);
                            if (sd.seed_bf16) {
                                // two bfloat16 products per component (<= 256 terms, <= 2 u each: 512 u), the
                                // query's split (2^-16 = 256 u), norms and final additions (< 200 u): under
                                // 1024 u; 4096 u = 2^-12 relative to |q|^2 + xn_max is used, plus
                                // 2 |q| max |x - bf16(x)|
                                bp.err_bound = ix->seed_err_bound * 8.0f;
                                bp.err_q = 2.0f * ix->seed_bf16_delta;
                                bp.fallback_count = ix->d_fb_count.as<uint32_t>();
                                // the wider bound needs a wider gap: more approximations are kept for re-ranking
                                // (a failed proof costs the query a gather of every seed)
                                static const int margin16 = env_int_early("VF_SEED_MARGIN_BF16", 24);
                                bp.seed_keep = std::min(64, itopk + std::max(margin16, kSeedMargin));
                            }
                        }
                    } else {
                        sd.max_chunks = ns_stride / kSeedChunk;
                        launch_seed_dist(ix->dtype, sd, (int)tiles.size(), s);
                    }
                    bp.dseed = sd.dseed;
                }
            }
            if (prof) VF_HIP(hipEventRecord(ix->prof_ev[3], s));
            return VF_OK;
        };
        auto run_scan = [&]() -> int {
            if (forked) {
                VF_HIP(hipEventRecord(W->ev_fork, s));
                VF_HIP(hipStreamWaitEvent(W->side, W->ev_fork, 0));
                ss = W->side;
            }
            if (prof) VF_HIP(hipEventRecord(ix->prof_ev[0], ss));

            ScanParams sp{};
            sp.qsrc = queries; sp.qrow = (const int32_t *)(dp + L.off_qrow);
            sp.dim = ix->dim; sp.ncp = ix->ncp; sp.K = k; sp.tile_rows = ib.tile_rows;
            sp.out_ids = out_ids; sp.out_dists = out_dists;
            sp.res_idx = W->part_idx.as<int32_t>(); sp.res_bits = W->part_bits.as<uint32_t>();
            const MergeItem *d_merges = (const MergeItem *)(dp + L.off_merges);
            sp.others_off = d_others_off; sp.others = d_others; sp.meta = ix->meta();
            if (n_ls_items) {
                sp.xblk = ix->d_X_LS.as<uint4>(); sp.xnorm = ix->d_xnorm_LS.p; sp.map = ix->d_M_LS.as<int32_t>();
                sp.items = (const ScanItem *)(dp + L.off_items);
                // small batches are latency-bound: the FMA kernel finishes a one-query tile three times sooner;
                // large batches keep the matrix-core kernel, which leaves the vector ALU to the beam search
                const bool small_batch = kScanValu == 2 || (kScanValu == 1 && qrow.size() <= 256);
                if (!exact && small_batch && scan_valu_supported(ix->dtype, ix->dim, sp.tile_rows)) {
                    launch_scan_valu(sp, (int)n_ls_items, ss);
                    if (prof) ix->prof.scan_kernel = 2;
                } else if (!exact && kScan16 && scan16_supported(ix->dtype, ix->dim, sp.tile_rows)) {
                    launch_scan16(sp, (int)n_ls_items, ss);
                    if (prof) ix->prof.scan_kernel = 1;
                } else {
                    launch_scan(ix->dtype, sp, (int)n_ls_items, ss);
                }
                // a search times its scan kernel by itself (the merge of the segments' candidates follows it)
                if (prof && hs_runs.empty()) VF_HIP(hipEventRecord(ix->prof_ev[1], ss));
                launch_scan_merge(ix->dtype, d_merges, (int)n_ls_merges, sp.res_idx, sp.res_bits, k, ib.max_nseg * k,
                                  ix->d_M_LS.as<int32_t>(), out_ids, out_dists, ss);
            }
            if (!hs_runs.empty()) {
                const int64_t max_groups = (max_hs_list + 31) / 32;
                if ((rc = ix->tmp_blk.reserve((size_t)max_groups * ix->group_bytes())) != VF_OK) return rc;
                if ((rc = ix->tmp_norm.reserve((size_t)max_groups * 32 * 4)) != VF_OK) return rc;
                for (const HsRun &run : hs_runs) {
                    const int32_t nl = ix->S[(size_t)run.label];
                    launch_interleave(ix->dtype, ix->X, ix->dim, ix->d_M_HS.as<int32_t>() + ix->O_HS[(size_t)run.label], nullptr,
                                      nullptr, nl, (nl + 31) / 32, ix->ncp, ix->tmp_blk.as<uint4>(), ix->tmp_norm.p, s);
                    sp.xblk = ix->tmp_blk.as<uint4>(); sp.xnorm = ix->tmp_norm.p; sp.map = ix->d_M_HS.as<int32_t>();
                    sp.items = (const ScanItem *)(dp + L.off_items) + run.item_lo;
                    launch_scan(ix->dtype, sp, (int)(run.item_hi - run.item_lo), s);
                }
                launch_scan_merge(ix->dtype, d_merges + n_ls_merges, (int)(ib.merges.size() - n_ls_merges), sp.res_idx,
                                  sp.res_bits, k, ib.max_nseg * k, ix->d_M_HS.as<int32_t>(), out_ids, out_dists, s);
            }
            if (prof && !(hs_runs.empty() && n_ls_items)) VF_HIP(hipEventRecord(ix->prof_ev[1], ss));
            if (forked) VF_HIP(hipEventRecord(W->ev_join, ss));
            return VF_OK;
        };
        // the scan goes first: its longest work items decide when it ends (measured: forking it
        // after the seed kernel costs 6 to 20 % of the step)
        if ((rc = run_scan()) != VF_OK) return rc;
        if ((rc = run_seeds()) != VF_OK) return rc;
        if (n_gq) launch_beam(ix->dtype, bp, (int)n_gq, s);
        if (bp.fallback_count != nullptr) {
            ix->fb_window_q += (int64_t)n_gq;
            if (!ix->fb_pending && ix->fb_window_q >= kFallbackWindow) {
                VF_HIP(hipMemcpyAsync(ix->h_fb, bp.fallback_count, 4, hipMemcpyDeviceToHost, s));
                VF_HIP(hipEventRecord(ix->ev_fb, s));
                ix->fb_pending = true;
                ix->fb_sent_q = ix->fb_window_q;
                ix->fb_window_q = 0;
            }
        }
        if (prof) {
            VF_HIP(hipEventRecord(ix->prof_ev[4], s));
            ix->prof_valid = true;
            ix->prof_next = (ix->prof_next + 1) % vf_index::kProfRing;
            ++ix->prof_unfolded;
        }
        if (forked) VF_HIP(hipStreamWaitEvent(s, W->ev_join, 0));
        if (zero_copy) {
            VF_HIP(hipEventRecord(st->done, s));
            st->pending = true;
        } else {
            VF_HIP(hipEventRecord(W->ev_blob_done[bsel], s));
            W->blob_used[bsel] = true;
        }
        VF_HIP(hipGetLastError());
        if (exact) {
            VF_HIP(hipStreamSynchronize(s));
            ix->tmp_blk.release();
            ix->tmp_norm.release();
        }
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return VF_ENOMEM;
    }
    return VF_OK;
}

extern "C" int vf_search(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                         const int32_t *qlabel_ids, int32_t k, int32_t itopk, int32_t width, int32_t iters,
                         int32_t n_seeds, int64_t *out_ids, float *out_dists, void *hip_stream)
{
    return search_impl(index, queries, nq, qlabel_offsets, qlabel_ids, k, itopk, width, iters, n_seeds, false, out_ids,
                       out_dists, (hipStream_t)hip_stream);
}

extern "C" int vf_search_exact(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                               const int32_t *qlabel_ids, int32_t k, int64_t *out_ids, float *out_dists, void *hip_stream)
{
    return search_impl(index, queries, nq, qlabel_offsets, qlabel_ids, k, 0, 0, 0, 0, true, out_ids, out_dists,
                       (hipStream_t)hip_stream);
}

// OR queries (Section 4.3.1) and the parallel AND policy (end of Section 4.3.2): every query becomes
// one search per label, the searches run as one ordinary batch, and a merge kernel combines them.
extern "C" int vf_search_multi(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids,
                               int32_t mode, int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds,
                               int64_t *out_ids, float *out_dists, void *hip_stream)
{
    hipStream_t s = (hipStream_t)hip_stream;
    const bool exact = (mode & VF_MULTI_EXACT) != 0;
    mode &= ~VF_MULTI_EXACT;
    VF_REQUIRE(mode == VF_AND_GREEDY || mode == VF_AND_PARALLEL || mode == VF_OR, "mode must be VF_AND_GREEDY, VF_AND_PARALLEL or VF_OR");
    if (mode == VF_AND_GREEDY)
        return search_impl(ix, queries, nq, qoff, qids, k, itopk, width, iters, n_seeds, exact, out_ids, out_dists, s);
    int rc = check_search_args(ix, queries, nq, k, out_ids, out_dists);
    if (rc != VF_OK) return rc;
    VF_REQUIRE(qoff && qids, "NULL query label arrays");
    if (nq == 0) return VF_OK;
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    Workspace *W = nullptr;
    if ((rc = workspace_for(ix, s, &W)) != VF_OK) return rc;
    try {
        std::vector<int32_t> &host = W->multi_host;
        std::vector<int64_t> &sqoff = W->multi_qoff;
        std::vector<int32_t> &sqids = W->multi_qids;
        host.clear(); sqoff.assign(1, 0); sqids.clear();
        std::vector<int32_t> first((size_t)nq + 1, 0);
        int32_t labs[kMaxOthers + 1];
        for (int64_t j = 0; j < nq; ++j) {
            const int64_t b = qoff[j], e = qoff[j + 1];
            VF_REQUIRE(e > b, "every query needs at least one label");
            int32_t nl = 0;
            for (int64_t p = b; p < e; ++p) {
                const int32_t l = qids[p];
                VF_REQUIRE(l >= 0 && l < ix->n_labels, "query label outside [0, n_labels)");
                bool seen = false;
                for (int32_t i = 0; i < nl; ++i) seen = seen || labs[i] == l;
                if (seen) continue;
                VF_REQUIRE(nl <= kMaxOthers, "more than 8 distinct labels in one query");
                labs[nl++] = l;
            }
            auto add = [&](int32_t searched, bool with_others) {
                host.push_back((int32_t)j);
                sqids.push_back(searched);
                if (with_others)
                    for (int32_t i = 0; i < nl; ++i)
                        if (labs[i] != searched) sqids.push_back(labs[i]);
                sqoff.push_back((int64_t)sqids.size());
            };
            if (mode == VF_OR) {
                for (int32_t i = 0; i < nl; ++i)
                    if (ix->S[(size_t)labs[i]] > 0) add(labs[i], false);
            } else {
                int32_t best = labs[0];
                bool empty = false;
                for (int32_t i = 0; i < nl; ++i) {
                    const int32_t sl = ix->S[(size_t)labs[i]], sb = ix->S[(size_t)best];
                    if (sl == 0) empty = true;
                    if (sl < sb || (sl == sb && labs[i] < best)) best = labs[i];
                }
                if (!empty) {
                    if (ix->S[(size_t)best] < ix->T) add(best, true);   // the filtered scan of the smallest list is exact
                    else for (int32_t i = 0; i < nl; ++i) add(labs[i], true);
                }
            }
            first[(size_t)j + 1] = (int32_t)host.size();
        }
        const int64_t n_sub = (int64_t)host.size();
        if (n_sub == 0) {
            launch_fill_out(out_ids, out_dists, nq * (int64_t)k, s);
            VF_HIP(hipGetLastError());
            return VF_OK;
        }
        host.insert(host.end(), first.begin(), first.end());
        const size_t row_bytes = (size_t)ix->dim * ix->elem();
        if ((rc = W->multi_meta.reserve(host.size() * 4)) != VF_OK) return rc;
        if ((rc = W->multi_q.reserve((size_t)n_sub * row_bytes)) != VF_OK) return rc;
        if ((rc = W->multi_ids.reserve((size_t)n_sub * k * 8)) != VF_OK) return rc;
        if ((rc = W->multi_dists.reserve((size_t)n_sub * k * 4)) != VF_OK) return rc;
        VF_HIP(hipMemcpyAsync(W->multi_meta.p, host.data(), host.size() * 4, hipMemcpyHostToDevice, s));
        const int32_t *d_parent = W->multi_meta.as<int32_t>();
        const int32_t *d_first = d_parent + n_sub;
        launch_gather_rows(queries, (int32_t)row_bytes, d_parent, n_sub, W->multi_q.p, s);
        rc = search_impl(ix, W->multi_q.p, n_sub, sqoff.data(), sqids.data(), k, itopk, width, iters, n_seeds, exact,
                         W->multi_ids.as<int64_t>(), W->multi_dists.as<float>(), s, true);
        if (rc != VF_OK) return rc;
        launch_multi_merge(d_first, nq, W->multi_ids.as<int64_t>(), W->multi_dists.as<float>(), k, out_ids, out_dists, s);
        VF_HIP(hipGetLastError());
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return VF_ENOMEM;
    }
    return VF_OK;
}

// ---------------------------------------------------------------- export / stats

extern "C" int vf_index_export(const vf_index *ix, int which, void *host_dst, size_t *bytes)
{
    VF_REQUIRE(ix && bytes, "NULL argument");
    const void *hsrc = nullptr, *dsrc = nullptr;
    size_t need = 0;
    std::vector<int64_t> s64;
    switch (which) {
    case VF_ARR_S:
        s64.assign(ix->S.begin(), ix->S.end()); hsrc = s64.data(); need = s64.size() * 8; break;
    case VF_ARR_O_HS: hsrc = ix->O_HS.data(); need = ix->O_HS.size() * 8; break;
    case VF_ARR_O_LS: hsrc = ix->O_LS.data(); need = ix->O_LS.size() * 8; break;
    case VF_ARR_GO_LS: hsrc = ix->GO_LS.data(); need = ix->GO_LS.size() * 8; break;
    case VF_ARR_M_HS: dsrc = ix->d_M_HS.p; need = (size_t)ix->n_HS * 4; break;
    case VF_ARR_M_LS: dsrc = ix->d_M_LS.p; need = (size_t)ix->n_LS * 4; break;
    case VF_ARR_G_HS: dsrc = ix->d_G.p; need = (size_t)ix->n_HS * ix->R * 4; break;
    case VF_ARR_X_LS: dsrc = ix->d_X_LS.p; need = (size_t)ix->n_groups_LS * ix->group_bytes(); break;
    case VF_ARR_BITSET: dsrc = ix->d_bitsets.p; need = ix->graph_labels.size() * (size_t)ix->bitset_words * 4; break;
    default: VF_REQUIRE(false, "unknown array id");
    }
    if (host_dst == nullptr) { *bytes = need; return VF_OK; }
    VF_REQUIRE(*bytes >= need, "destination buffer too small");
    *bytes = need;
    if (need == 0) return VF_OK;
    if (hsrc) memcpy(host_dst, hsrc, need);
    else VF_HIP(hipMemcpy(host_dst, dsrc, need, hipMemcpyDeviceToHost));
    return VF_OK;
}

extern "C" int vf_index_stats(const vf_index *ix, vf_stats *out)
{
    VF_REQUIRE(ix && out, "NULL argument");
    memset(out, 0, sizeof(*out));
    out->n = ix->n; out->n_HS = ix->n_HS; out->n_LS = ix->n_LS; out->n_groups_LS = ix->n_groups_LS;
    out->dim = ix->dim; out->dtype = ix->dtype; out->n_labels = ix->n_labels; out->T = ix->T; out->graph_degree = ix->R;
    out->n_graph_labels = (int32_t)ix->graph_labels.size(); out->n_scan_labels = ix->n_scan_labels;
    out->chunks_per_vector = 2 * ix->ncp;
    out->bytes_graph = 2 * ix->n_HS * ix->R * 4;   // local ids + global ids
    out->bytes_maps = (ix->n_HS + ix->n_LS) * 4;
    out->bytes_x_ls = ix->n_groups_LS * (int64_t)ix->group_bytes() + ix->n_groups_LS * 32 * 4;
    out->bytes_bitsets = (int64_t)ix->graph_labels.size() * ix->bitset_words * 4;
    out->bytes_meta = (int64_t)ix->n_labels * (4 + 8 + 8 + 4);
    out->bytes_total = out->bytes_graph + out->bytes_maps + out->bytes_x_ls + out->bytes_bitsets + out->bytes_meta;
    return VF_OK;
}

extern "C" int vf_profile_enable(vf_index *ix, int on)
{
    VF_REQUIRE(ix != nullptr, "index is NULL");
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    if (on)
        for (auto &set : ix->prof_ring)
            for (hipEvent_t &e : set)
                if (!e) VF_HIP(hipEventCreate(&e));
    ix->profiling = on != 0;
    ix->prof_serial = on == 2;
    ix->prof_valid = false;
    ix->prof_next = 0; ix->prof_unfolded = 0;
    ix->prof_scan_sum = ix->prof_seed_sum = ix->prof_beam_sum = 0;
    ix->prof_calls = 0;
    return VF_OK;
}

extern "C" int vf_profile_read(vf_index *ix, vf_profile *out, int32_t *per_query)
{
    VF_REQUIRE(ix && out, "NULL argument");
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    VF_REQUIRE(ix->prof_valid, "no profiled vf_search call to report");
    int rc = fold_profile(ix, vf_index::kProfRing);
    if (rc != VF_OK) return rc;
    vf_profile pf = ix->prof;
    pf.scan_ms_sum = ix->prof_scan_sum; pf.seed_ms_sum = ix->prof_seed_sum; pf.beam_ms_sum = ix->prof_beam_sum;
    pf.calls = ix->prof_calls;
    try {
        std::vector<int32_t> cn((size_t)pf.nq * 4);
        VF_HIP(hipMemcpy(cn.data(), ix->counters.p, cn.size() * 4, hipMemcpyDeviceToHost));
        std::vector<int32_t> gathered((size_t)pf.nq);
        VF_HIP(hipMemcpy(gathered.data(), ix->counters.as<int32_t>() + (size_t)pf.nq * 4, gathered.size() * 4, hipMemcpyDeviceToHost));
        if (per_query) memset(per_query, 0, cn.size() * 4);
        for (int32_t j : ix->prof_graph_queries) {   // the other rows of the device arrays hold nothing
            const int32_t *row = &cn[(size_t)j * 4];
            pf.beam_scored += row[0]; pf.beam_expanded += row[1]; pf.beam_tested += row[2];
            pf.seed_fallbacks += (row[3] & 0xFF) == 3;
            pf.seed_rescored += row[3] >> 8;
            pf.beam_gathered += gathered[(size_t)j];
            if (per_query) memcpy(per_query + (size_t)j * 4, row, 16);
        }
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return VF_ENOMEM;
    }
    *out = pf;
    return VF_OK;
}

extern "C" void vf_index_free(vf_index *ix) { free_index(ix); }

extern "C" const char *vf_last_error(void) { return g_err.c_str(); }
