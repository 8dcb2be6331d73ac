// Host-side state of the library: the index object behind the C ABI of include/vecflow.h, its
// per-stream workspaces, the tuning switches, and the functions the host source files share.
// Nothing here is part of the C ABI.
#pragma once

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/vecflow.h"
#include "vf_internal.h"

namespace vf {

#define VF_HIP(expr)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) {                                                                        \
            ::vf::set_error(std::string(#expr) + ": " + hipGetErrorString(e_));                        \
            return e_ == hipErrorOutOfMemory ? VF_ENOMEM : VF_EHIP;                                    \
        }                                                                                              \
    } while (0)

#define VF_REQUIRE(cond, msg)                 \
    do {                                      \
        if (!(cond)) {                        \
            ::vf::set_error(msg);             \
            return VF_EINVAL;                 \
        }                                     \
    } while (0)

// Runs the body of an extern "C" entry point: no exception crosses the ABI.
template <class F> int guarded(F &&body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return VF_ENOMEM;
    } catch (const std::exception &e) {
        set_error(std::string("internal error: ") + e.what());
        return VF_EINTERNAL;
    } catch (...) {
        set_error("internal error (unknown exception)");
        return VF_EINTERNAL;
    }
}

// Where the index's device memory comes from: the allocator the caller gave to vf_build_index, or
// hipMalloc / hipFree.
struct DeviceAllocator {
    vf_allocator user{};   // user.alloc == nullptr: hipMalloc / hipFree
    int64_t live_bytes = 0, peak_bytes = 0;
    int alloc(void **p, size_t bytes);
    void release(void *p, size_t bytes);
};

struct DevBuf {
    void *p = nullptr;
    size_t cap = 0;
    DeviceAllocator *al = nullptr;   // nullptr: hipMalloc / hipFree
    DevBuf() = default;
    explicit DevBuf(DeviceAllocator *a) : al(a) {}
    DevBuf(const DevBuf &) = delete;
    DevBuf &operator=(const DevBuf &) = delete;
    // Grows the buffer to at least `bytes` (contents are not kept); never shrinks.
    int reserve(size_t bytes);
    void release();
    template <class T> T *as() const { return (T *)p; }
};

// Releases temporaries on every exit path of a function.
struct DevBufGuard {
    std::vector<DevBuf *> bufs;
    DevBufGuard(std::initializer_list<DevBuf *> b) : bufs(b) {}
    ~DevBufGuard() { for (DevBuf *b : bufs) b->release(); }
};

// Switches and sizes that experiments and tests may change (vf_tune); the defaults are the measured optima.
// An index copies the process-wide defaults when it is built; afterwards it has its own.
struct Tuning {
    int seg_groups = 16;          // 32-vector groups per scan-list segment
    int seg_groups_heavy = 16;    // the same for tiles of >= heavy_rows queries
    int heavy_rows = 9;
    int tile_rows = 16;           // queries per scan tile
    int zero_copy_bytes = 8192;   // a per-call routing blob up to this size is read in place from pinned host memory
    int scan_valu = 1;            // float32 FMA scan kernel: 0 never, 1 for batches of <= 256 scan queries, 2 always
    int scan16 = 1;               // 0: float32 search tiles keep the 32-row matrix-core kernel
    int scan_bf16 = 1;            // float32 lists of large batches: filter from the bfloat16 copy, re-rank exactly (0: off)
    int scan_bf16_margin = 22;    // approximations kept beyond k per query and segment by that filter
    int scan_bf16_slots = 1;      // list groups a wave of that filter keeps in flight (1 or 2)
    int scan_bf16_seg_groups = 24;   // 32-vector groups per list segment when that filter runs (half the bytes per group)
    int beam_lat_waves = 1024;    // beam launches of up to this many graph queries use the latency instantiation (a wave per SIMD); 0: never
    int overlap = 1;              // 0: the scan path runs on the caller's stream, before the graph path
    int seed_exact = 0;           // 1: seeds are scored by the ordered-distance kernel, never on the matrix cores
    double seed_slack = 1.0;      // scales the rounding-error bound of the float32 seed proofs
    int seed_margin = 8;          // approximations kept beyond itopk for re-ranking (float32 copy of the seeds)
    int seed_margin_bf16 = 24;    // the same from the bfloat16 copy
    int seed_cache = 1;           // 0: no interleaved copy of the seeds, the seed kernel gathers rows
    int seed_bf16 = 1;            // 0: float32 data keep only the float32 copy of the seeds
    int seed_bf16_min_batch = 512;   // calls with fewer graph queries use the float32 copy when it is resident
    int seed_fb_window = 131072;  // graph queries between two looks at the failed-proof counter
    int seed_select = 0;          // 1: the seed kernel also selects (runs of keys instead of every distance; itopk <= 64)
    int seed_seg_seeds = 0;       // seeds per wave of the selecting seed kernel; 0: chosen per call (512 .. 16384)
    int build16 = 1;              // float32 kNN self-joins on 16-row tiles
    int build_panel_kb = 4096;    // self-joins of long lists go panel by panel, this much of the list per launch
    int build_progress = 0;       // 1: a line on stderr every ten seconds while graphs are built
    // returns false for an unknown name or a value out of range
    bool set(const char *name, double value);
};
Tuning &default_tuning();
std::mutex &default_tuning_mutex();

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
    std::vector<int32_t> xq_query, xq_label;          // AND queries on short graph lists that are answered exactly
    bool any_and = false;
    // scratch kept between calls
    std::vector<int32_t> q_best;                      // searched label of each query, -1: empty result
    std::vector<int32_t> empty_q;                     // queries with q_best == -1
    std::vector<int32_t> cnt;                         // [n_labels] queries per searched label (zero between calls)
    std::vector<int32_t> touched;                     // labels with cnt > 0
};

// What routing needs to know of an index (a view, so that routing can be exercised without a device).
struct RouteView {
    const int32_t *S;     // [n_labels] posting-list sizes
    int32_t n_labels, T;
};

// ClassifyQueries (Alg. 2) + smallest-list choice (Section 4.3.2).  all_scan: every list is scanned (exact
// mode); first_is_searched: a query searches the list of its first label, the others are the predicate.
int route_queries(const RouteView &ix, int64_t nq, const int64_t *qoff, const int32_t *qids, bool all_scan,
                  bool first_is_searched, Routed &r);

// Work list of the scan path: the (label, query) pairs of one label are cut into tiles of <= tile_rows
// queries; a long list is cut into segments of whole 32-vector groups so that many waves share it, and a
// merge item per query then combines the segments.
constexpr int kMaxSegs = 64;
struct ItemBuilder {
    std::vector<int32_t> qrow;
    std::vector<ScanItem> items;
    std::vector<MergeItem> merges;
    int64_t part_rows = 0;
    int32_t max_nseg = 1;
    int32_t tile_rows = 16, seg_groups = 16, seg_groups_heavy = 16, heavy_rows = 9;
    bool all_partial = false;   // every item writes partial rows and every query gets a merge item (one-segment lists too)
    explicit ItemBuilder(const Tuning &t)
        : tile_rows(t.tile_rows), seg_groups(t.seg_groups), seg_groups_heavy(t.seg_groups_heavy), heavy_rows(t.heavy_rows) {}
    // pairs[lo, hi) all carry the same label, whose list is (group0, map_off, n)
    void add_label(const std::vector<uint64_t> &pairs, size_t lo, size_t hi, int64_t group0, int64_t map_off, int32_t n);
};

// Everything a call writes besides its outputs.  An index has kWorkspaces of them and hands one to each
// stream that calls it, so that calls on different streams can overlap on the GPU (small batches leave most
// of the chip idle); calls on one stream share one workspace and run in order.
struct Workspace {
    DevBuf ws_blob, ws_blob_b, part_idx, part_bits, dseed;
    // vf_search_multi: gathered query rows, results of the sub-searches, their parents
    DevBuf multi_q, multi_ids, multi_dists, multi_meta;
    std::vector<int32_t> multi_host;      // [n_sub parents | nq + 1 first sub-search of each query], alive until the next call
    std::vector<int64_t> multi_qoff;
    std::vector<int32_t> multi_qids;
    // the scan path runs beside the graph path on a second stream of the same (default) priority
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    bool prev_forked = false;   // the previous call on this workspace ran its scan path on the side stream
    int blob_next = 0;   // the device blob alternates between two buffers
    Staging stage[2];
    int stage_next = 0;
    Routed routed;
    bool ready = false;          // stream and events exist
    bool owned = false;
    hipStream_t owner = nullptr; // the stream whose calls use this workspace
    std::vector<DevBuf *> bufs()
    {
        return {&ws_blob, &ws_blob_b, &part_idx, &part_bits, &dseed, &multi_q, &multi_ids, &multi_dists, &multi_meta};
    }
};

// The seeds of every graph list for one n_seeds (local ids floor(j n / ns)), interleaved like a scan list, so
// that the matrix-core seed kernel reads its B operand with coalesced loads.  Derived from the index and
// n_seeds alone.  An index keeps a few of them (calls on different streams may use different seed counts at
// the same time); a copy is only rebuilt or dropped after the whole device has drained.
struct SeedCopy {
    int32_t n_seeds = -1;        // -1: slot unused
    bool ok = false;             // false: the copy did not fit, the kernel gathers rows from the vector table
    bool has_f32 = false;        // blk is valid
    bool has_bf16 = false;       // blk16 is valid (float32 data only)
    float bf16_delta = 0.f;      // upper bound of |x - bf16(x)| over the seeds of the copy
    uint64_t last_use = 0;
    DevBuf blk, blk16, norm, goff;
    DevBuf map;                  // [group * 32 + v] global id of the seed (AND predicate inside the seed kernel)
    std::vector<DevBuf *> bufs() { return {&blk, &blk16, &norm, &goff, &map}; }
};

}  // namespace vf

struct vf_index {
    vf::DeviceAllocator alloc;
    vf::Tuning tune;
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
    vf::DevBuf d_S, d_O_HS, d_O_LS, d_hs_slot, d_M_HS, d_M_LS, d_G, d_X_LS, d_xnorm_LS, d_bitsets;
    // float32 data: the scan lists once more in bfloat16 (16-byte chunks of 8 components, half the bytes), which the
    // filtering scan kernel streams; ls_bf16_delta = max |x - bf16(x)| over the lists' vectors (its error bound)
    vf::DevBuf d_X_LS16, d_scan_fb;
    bool has_ls16 = false;
    float ls_bf16_delta = 0.f, ls_xn_max = 0.f;   // ... and the largest squared norm of a list vector
    uint32_t scan_fb_seen = 0;   // failed proofs already reported (d_scan_fb counts them on the device)
    vf::DevBuf d_Gg;   // [n_HS][R] the graph rows once more with global ids: saves the search one dependent load per expansion
    // indexes with graph labels: squared norm of every row of X and the largest of them, for the matrix-core
    // seed scoring (its error bound needs the largest norm)
    vf::DevBuf d_xnorm_all;
    float xn_max = 0.f;
    bool seed_mfma_ok = false;   // the norms exist and are finite: seeds may be scored on the matrix cores
    // search workspaces (see Workspace); profiled calls and vf_search_exact must not overlap with other calls
    static constexpr int kWorkspaces = 8;
    vf::Workspace ws[kWorkspaces];
    int ws_steal = 0;
    std::recursive_mutex mu;     // host side of every call
    vf::Routed noalloc_routed;   // host-side scratch of vf_search_noalloc (kept between calls)
    std::vector<char> noalloc_blob;
    vf::DevBuf tmp_blk, tmp_norm, counters;
    static constexpr int kSeedCopies = 4;
    vf::SeedCopy seed_copies[kSeedCopies];
    uint64_t seed_tick = 0;
    // Watch on the bfloat16 form of the seed copies: queries whose proof failed are counted on the device; the
    // count is fetched every tune.seed_fb_window graph queries and read at a later call, and a window with more
    // than 1/64 failures switches this index back to float32 copies (a failed proof costs its query a gather of
    // every seed).
    bool seed_bf16_off = false;
    vf::DevBuf d_fb_count;
    uint32_t *h_fb = nullptr;    // pinned
    hipEvent_t ev_fb = nullptr;
    bool fb_pending = false;
    uint32_t fb_last = 0;
    int64_t fb_window_q = 0, fb_sent_q = 0;
    // profiling
    bool profiling = false, prof_valid = false;
    // a ring of event sets (scan begin/end, graph begin, seeds end, beam end), one set per profiled call:
    // a call never waits for an earlier one unless kProfRing calls are still unread
    static constexpr int kProfRing = 64;
    hipEvent_t prof_ring[kProfRing][5] = {};
    hipEvent_t *prof_ev = prof_ring[0];   // the set of the call being issued
    int prof_next = 0, prof_unfolded = 0; // next ring slot; recorded sets whose durations are not in the sums yet
    bool prof_serial = false;  // vf_profile_enable(index, 2): every launch on the caller's stream
    bool prof_exact_counts = false;   // ... | 4: count the seeds that pass each AND query's predicate before every call
    vf_profile prof{};
    std::vector<int32_t> prof_graph_queries;   // graph-routed queries of the last profiled call
    double prof_scan_sum = 0, prof_seed_sum = 0, prof_beam_sum = 0;
    double prof_host_plan = 0, prof_host_blob = 0, prof_host_launch = 0, prof_host_wait = 0;   // host milliseconds inside profiled calls
    int64_t prof_calls = 0;

    vf_index();
    std::vector<vf::DevBuf *> bufs()
    {
        return {&d_S, &d_O_HS, &d_O_LS, &d_hs_slot, &d_M_HS, &d_M_LS, &d_G, &d_Gg, &d_X_LS, &d_xnorm_LS, &d_bitsets,
                &d_xnorm_all, &tmp_blk, &tmp_norm, &counters, &d_fb_count, &d_X_LS16, &d_scan_fb};
    }
    vf::LabelMeta meta() const
    {
        vf::LabelMeta m;
        m.S = d_S.as<int32_t>(); m.O_HS = d_O_HS.as<int64_t>(); m.O_LS = d_O_LS.as<int64_t>();
        m.hs_slot = d_hs_slot.as<int32_t>(); m.M_HS = d_M_HS.as<int32_t>(); m.M_LS = d_M_LS.as<int32_t>();
        m.bitsets = d_bitsets.as<uint32_t>(); m.bitset_words = bitset_words;
        return m;
    }
    vf::RouteView route_view() const { return vf::RouteView{S.data(), n_labels, T}; }
    size_t elem() const { return dtype == VF_U8 ? 1 : 4; }
    size_t group_bytes() const { return (size_t)2 * ncp * 32 * 16; }
    // float32 seed proofs: |approximation - ordered distance| <= seed_err_bound() (|q|^2 + xn_max)
    float seed_err_bound() const { return (float)(tune.seed_slack * 3.0517578125e-05); }
};

namespace vf {

template <class T> int upload(DevBuf &b, const std::vector<T> &v, hipStream_t s)
{
    int rc = b.reserve(std::max<size_t>(v.size() * sizeof(T), 16));
    if (rc != VF_OK) return rc;
    if (!v.empty()) VF_HIP(hipMemcpyAsync(b.p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, s));
    return VF_OK;
}

// vf_search.hip: the pieces of one search call
struct BlobLayout {
    size_t off_gq_query, off_gq_label, off_xq_query, off_xq_label, off_others_off, off_others, off_qrow, off_items, off_merges, off_tiles, off_empty, total;
};

// Everything the host decides about a call before anything is launched.
struct HsRun { int32_t label; size_t item_lo, item_hi; };   // exact mode: the scan items of one graph list
struct CallPlan {
    int64_t nq = 0;
    int32_t k = 0, itopk = 0, width = 0, iters = 0, n_seeds = 0;
    bool exact = false;
    int32_t beam_LP = 128, beam_hb = 9;   // beam kernel geometry: list slots and visited-table size
    int32_t ns_stride = 0;                // row length of the seed distance matrix
    ItemBuilder ib;
    size_t n_ls_items = 0, n_ls_merges = 0;
    std::vector<HsRun> hs_runs;
    int32_t max_hs_list = 0;
    std::vector<SeedTile> tiles;          // dense seed scoring: tiles of <= 64 (32) graph queries of one label
    size_t n_gq = 0;
    size_t n_xq = 0;                      // AND queries answered by the exact predicate scan of a short graph list
    bool dense_seeds = false, seeds_mfma = false;
    // seeds_mfma with the selection fused into the seed kernel: runs of sel_K keys per (query, segment)
    bool seed_select = false, sel_bf16 = false;
    int32_t sel_K = 0, seg_seeds = 0, max_segs = 0;
    BlobLayout L{};
    size_t dseed_words = 0;               // seed distance matrix + the dump area behind it
    size_t part_words = 0;                // partial result rows x k (x scan_keep with the bfloat16 filter)
    // float32 scan lists filtered from their bfloat16 copy and re-ranked
    bool scan_bf16 = false;
    int32_t scan_keep = 0;                // approximations kept per (query, segment)
    explicit CallPlan(const Tuning &t) : ib(t) {}
};

// Where a call's device-side temporaries live (a workspace's buffers, or the static scratch array of the entry
// point that allocates nothing).
struct CallMem {
    char *blob = nullptr;          // device address of the routing blob
    uint32_t *dseed = nullptr;
    int32_t *part_idx = nullptr;
    uint32_t *part_bits = nullptr;
};

int check_search_args(const vf_index *ix, const void *queries, int64_t nq, int32_t k, const int64_t *out_ids,
                      const float *out_dists);
int check_search_params(const vf_index *ix, bool exact, int32_t k, int32_t &itopk, int32_t width, int32_t iters,
                        int32_t &n_seeds);
int plan_call(const vf_index *ix, Routed &r, int64_t nq, const int64_t *qoff, const int32_t *qids, bool exact,
              bool first_is_searched, int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds,
              int32_t and_scan_limit, uint64_t dseed_budget_words, const SeedCopy *sc, CallPlan &P);
// May this call's seeds be scored on the matrix cores (so that an interleaved seed copy is worth having)?
bool wants_seed_copy(const vf_index *ix, bool exact, int32_t itopk, int32_t n_seeds);
// The resident copy for n_seeds, or (build = true) a new one; *out stays null when there is none.
int seed_copy_for(vf_index *ix, int32_t n_seeds, hipStream_t s, bool build, SeedCopy **out);
int build_seed_copy(vf_index *ix, int32_t n_seeds, hipStream_t s, bool want_bf16, SeedCopy *c);
void fill_blob(const CallPlan &P, const Routed &r, char *hp);
int launch_call(vf_index *ix, const CallPlan &P, const Routed &r, const CallMem &M, const SeedCopy *sc, const void *queries,
                int64_t *out_ids, float *out_dists, hipStream_t s, hipStream_t side, hipEvent_t ev_fork,
                hipEvent_t ev_join, bool may_allocate);

// vf_index_build.hip
int build_index_impl(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                     const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree, int32_t graph_kind,
                     int32_t knn_degree, const vf_allocator *allocator, void *hip_stream, vf_index **out);
void free_index(vf_index *ix);

// vf_search.hip
int search_impl(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids, int32_t k,
                int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds, bool exact, int64_t *out_ids,
                float *out_dists, hipStream_t s, bool first_is_searched = false, int32_t and_scan_limit = 0);
int search_multi_impl(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids,
                      int32_t mode, int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds,
                      int64_t *out_ids, float *out_dists, hipStream_t s);
int fold_profile(vf_index *ix, int count);
// Drops every interleaved seed copy (after the device has drained): they are rebuilt on demand.
int drop_seed_copies(vf_index *ix);

// LDS bytes of the scan kernels for a tile (host-side check before a launch)
size_t scan_lds_bytes(int32_t ncp, int32_t tile_rows, int32_t K);

}  // namespace vf
