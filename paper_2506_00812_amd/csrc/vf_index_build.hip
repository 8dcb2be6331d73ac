// Index construction (Alg. 1): posting lists, the HS / LS split at threshold T, the compacted S / O / M arrays
// of each partition, the interleaved scan lists of Section 4.2.2, membership bitsets for the AND predicate of
// Section 4.3.2, and one proximity graph per graph list (Section 4.2.1).  Also the index's memory management.
#include <ctime>

#include "vf_host.h"

namespace vf {

int DeviceAllocator::alloc(void **p, size_t bytes)
{
    *p = nullptr;
    if (user.alloc != nullptr) {
        void *q = user.alloc(bytes, user.ctx);
        if (q == nullptr) {
            set_error("the caller's device allocator returned NULL for " + std::to_string(bytes) + " bytes");
            return VF_ENOMEM;
        }
        if (((uintptr_t)q & 255) != 0) {
            user.free(q, user.ctx);
            set_error("the caller's device allocator returned memory that is not 256-byte aligned");
            return VF_EINVAL;
        }
        *p = q;
    } else {
        VF_HIP(hipMalloc(p, bytes));
    }
    live_bytes += (int64_t)bytes;
    peak_bytes = std::max(peak_bytes, live_bytes);
    return VF_OK;
}

void DeviceAllocator::release(void *p, size_t bytes)
{
    if (p == nullptr) return;
    if (user.alloc != nullptr) {
        // the allocator may hand the block to someone else at once: everything that used it must have completed
        // (hipFree waits for the device by itself)
        (void)hipDeviceSynchronize();
        user.free(p, user.ctx);
    } else {
        (void)hipFree(p);
    }
    live_bytes -= (int64_t)bytes;
}

int DevBuf::reserve(size_t bytes)
{
    if (bytes <= cap) return VF_OK;
    // a first allocation is exact (index arrays are sized once); a buffer that grows takes a quarter more than
    // asked, so that a workspace settles after a few calls
    const bool grows = p != nullptr;
    release();
    const size_t want = grows ? bytes + bytes / 4 + 256 : ((bytes + 255) & ~(size_t)255);
    if (al != nullptr) {
        int rc = al->alloc(&p, want);
        if (rc != VF_OK) return rc;
    } else {
        VF_HIP(hipMalloc(&p, want));
    }
    cap = want;
    return VF_OK;
}

void DevBuf::release()
{
    if (p != nullptr) {
        if (al != nullptr) al->release(p, cap);
        else (void)hipFree(p);
    }
    p = nullptr;
    cap = 0;
}

}  // namespace vf

using namespace vf;

vf_index::vf_index()
{
    for (DevBuf *b : bufs()) b->al = &alloc;
    for (Workspace &w : ws)
        for (DevBuf *b : w.bufs()) b->al = &alloc;
    for (SeedCopy &c : seed_copies)
        for (DevBuf *b : c.bufs()) b->al = &alloc;
}

namespace vf {

void free_index(vf_index *ix)
{
    if (!ix) return;
    // memory goes back to the allocator only after everything that used it has completed
    (void)hipDeviceSynchronize();
    for (DevBuf *b : ix->bufs()) b->release();
    for (SeedCopy &c : ix->seed_copies)
        for (DevBuf *b : c.bufs()) b->release();
    for (auto &set : ix->prof_ring)
        for (hipEvent_t e : set)
            if (e) (void)hipEventDestroy(e);
    if (ix->ev_fb) (void)hipEventDestroy(ix->ev_fb);
    if (ix->h_fb) (void)hipHostFree(ix->h_fb);
    for (Workspace &w : ix->ws) {
        for (DevBuf *b : w.bufs()) b->release();
        if (w.ev_fork) (void)hipEventDestroy(w.ev_fork);
        if (w.ev_join) (void)hipEventDestroy(w.ev_join);
        if (w.side) (void)hipStreamDestroy(w.side);
        for (Staging &s : w.stage) {
            if (s.done) (void)hipEventDestroy(s.done);
            if (s.p) (void)hipHostFree(s.p);
        }
    }
    delete ix;
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
    const int32_t TR = (ix->tune.build16 && scan16_supported(ix->dtype, ix->dim, 16)) ? 16 : 32;
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
        // long lists go panel by panel so that the resident waves share L2 (4 MiB of list per launch by
        // default -- the measured optimum, one XCD's L2; lists of up to 4 panels are not cut)
        const int64_t panel_bytes = (int64_t)std::max(1, ix->tune.build_panel_kb) << 10;
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
    // float32 rows are accepted only with a proof that the self-join's K candidates contain them (the bound of the
    // float32 matrix-core approximations, relative to the largest squared norm of the table)
    const bool checked = ix->dtype == VF_F32 && ix->xn_max > 0.f;
    launch_graph_rows(ix->dtype, ix->X, ix->dim, map, nl, cand_idx.as<int32_t>(), cand_dist.as<uint32_t>(), K, deg, rows_out,
                      checked ? ix->seed_err_bound() : -1.f, ix->xn_max, nullptr, s);
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
    DevBuf d_base(&ix->alloc), d_deg(&ix->alloc), d_off(&ix->alloc), d_seg(&ix->alloc);
    DevBufGuard rel{&d_base, &d_deg, &d_off, &d_seg};
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

int build_index_impl(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                     const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree, int32_t graph_kind,
                     int32_t knn_degree, const vf_allocator *allocator, void *hip_stream, vf_index **out)
{
    VF_REQUIRE(out != nullptr, "out is NULL");
    *out = nullptr;
    VF_REQUIRE(vectors && label_offsets && label_ids, "NULL input pointer");
    VF_REQUIRE(dtype == VF_U8 || dtype == VF_F32, "dtype must be VF_U8 or VF_F32");
    VF_REQUIRE(n > 0 && n < ((int64_t)1 << 31), "n must be in [1, 2^31)");
    const int64_t row_bytes = (int64_t)dim * (dtype == VF_U8 ? 1 : 4);
    VF_REQUIRE(dim > 0 && row_bytes % 16 == 0 && row_bytes >= 16 && row_bytes <= 2048,
               "dim: uint8 needs dim % 16 == 0, float32 dim % 4 == 0, 16 <= bytes per vector <= 992");
    // a 32-row tile of the contraction kernel with the 64 candidates per row of a graph build must fit in LDS
    VF_REQUIRE(scan_lds_bytes((int32_t)((row_bytes / 16 + 1) / 2), 32, 64) <= 64 * 1024,
               "dim: vectors of more than 992 bytes are not supported (LDS of the contraction kernel)");
    VF_REQUIRE(allocator == nullptr || (allocator->alloc != nullptr && allocator->free != nullptr),
               "allocator: both functions must be given");
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
    if (allocator != nullptr) ix->alloc.user = *allocator;
    {
        std::lock_guard<std::mutex> lock(default_tuning_mutex());
        ix->tune = default_tuning();
    }

    {
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
            DevBuf d_src(&ix->alloc), d_cnt(&ix->alloc);
            DevBufGuard r2{&d_src, &d_cnt};
            if ((rc = upload(d_src, grp_src, s)) != VF_OK) return rc;
            if ((rc = upload(d_cnt, grp_cnt, s)) != VF_OK) return rc;
            if ((rc = ix->d_X_LS.reserve((size_t)ix->n_groups_LS * ix->group_bytes())) != VF_OK) return rc;
            if ((rc = ix->d_xnorm_LS.reserve((size_t)ix->n_groups_LS * 32 * 4)) != VF_OK) return rc;
            launch_interleave(dtype, vectors, dim, ix->d_M_LS.as<int32_t>(), d_src.as<int64_t>(), d_cnt.as<int32_t>(),
                              ix->n_LS, ix->n_groups_LS, ix->ncp, ix->d_X_LS.as<uint4>(), ix->d_xnorm_LS.p, s);
            VF_HIP(hipGetLastError());
            VF_HIP(hipStreamSynchronize(s));
            // float32 lists once more in bfloat16, for the filtering scan kernel.  Its proofs need the largest
            // rounding error |x - bf16(x)| and the largest squared norm of a list vector; a table with NaN or
            // overflowing values, or norms outside [1e-24, 1e30] (the bound is relative to the norm and assumes
            // that what the matrix cores flush is negligible beside it), keeps the exact kernels only.
            if (dtype == VF_F32 && ix->tune.scan_bf16 && scan_bf16_supported(dtype, dim, 16, 32)) {
                const size_t n_slots = (size_t)ix->n_groups_LS * 32;
                DevBuf d_err2(&ix->alloc);
                DevBufGuard r4{&d_err2};
                if ((rc = ix->d_X_LS16.reserve((size_t)ix->n_groups_LS * ix->group_bytes() / 2)) != VF_OK) return rc;
                if ((rc = d_err2.reserve(n_slots * 4)) != VF_OK) return rc;
                launch_seed_pack_bf16(ix->d_X_LS.as<uint4>(), ix->n_groups_LS, ix->ncp, ix->d_X_LS16.as<uint4>(),
                                      d_err2.as<float>(), s);
                std::vector<float> e2(n_slots), nr(n_slots);
                VF_HIP(hipMemcpyAsync(e2.data(), d_err2.p, n_slots * 4, hipMemcpyDeviceToHost, s));
                VF_HIP(hipMemcpyAsync(nr.data(), ix->d_xnorm_LS.p, n_slots * 4, hipMemcpyDeviceToHost, s));
                VF_HIP(hipStreamSynchronize(s));
                double mx_e = 0.0;
                float mx_n = 0.f;
                bool finite = true;
                for (size_t i = 0; i < n_slots; ++i) {
                    finite = finite && e2[i] == e2[i] && e2[i] <= 3.0e38f && nr[i] == nr[i] && nr[i] <= 3.0e38f;
                    mx_e = e2[i] > mx_e ? e2[i] : mx_e;
                    mx_n = nr[i] > mx_n ? nr[i] : mx_n;
                }
                if (finite && mx_n >= 1e-24f && mx_n <= 1e30f) {
                    if ((rc = ix->d_scan_fb.reserve(4)) != VF_OK) return rc;
                    VF_HIP(hipMemsetAsync(ix->d_scan_fb.p, 0, 4, s));
                    VF_HIP(hipStreamSynchronize(s));
                    ix->has_ls16 = true;
                    ix->ls_bf16_delta = (float)(std::sqrt(mx_e) * 1.001);
                    ix->ls_xn_max = mx_n;
                } else {
                    ix->d_X_LS16.release();
                }
            }
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
            DevBuf d_knn(&ix->alloc);
            DevBufGuard rk{&d_knn};
            if (pruned && (rc = d_knn.reserve((size_t)ix->n_HS * D * 4)) != VF_OK) return rc;
            DevBuf cand_idx(&ix->alloc), cand_dist(&ix->alloc), d_items(&ix->alloc);
            DevBufGuard r3{&cand_idx, &cand_dist, &d_items};
            const int64_t max_groups = (max_list + 31) / 32;
            if ((rc = ix->tmp_blk.reserve((size_t)max_groups * ix->group_bytes())) != VF_OK) return rc;
            if ((rc = ix->tmp_norm.reserve((size_t)max_groups * 32 * 4)) != VF_OK) return rc;
            if ((rc = cand_idx.reserve((size_t)max_groups * 32 * K * 4)) != VF_OK) return rc;
            if ((rc = cand_dist.reserve((size_t)max_groups * 32 * K * 4)) != VF_OK) return rc;
            // squared norm of every row of X and the largest of them: the matrix-core seed scoring reads the norms,
            // its proofs and those of the float32 graph rows need the largest
            if (ix->dtype == VF_F32 || seed_mfma_supported(ix->dtype, ix->dim)) {
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
                // squared norm is outside [1e-24, 1e30]: the proofs' bound is relative to that norm and assumes
                // that what the matrix cores flush (products under 1.2e-38) is negligible beside it.
                // The bound itself: |approximation - ordered distance| <= 300 u (|q|^2 + |x|^2), u = 2^-24 (dot
                // product of <= 512 terms in any order, two norms, the final additions, the ordered sum's own
                // error); 512 u = 2^-15 is used (vf_index::seed_err_bound).
                if (ix->dtype == VF_F32 && !(mx >= 1e-24f && mx <= 1e30f)) finite = false;
                if (finite) {
                    ix->xn_max = mx;
                    ix->seed_mfma_ok = seed_mfma_supported(ix->dtype, ix->dim);
                }
                if (!finite || !ix->seed_mfma_ok) ix->d_xnorm_all.release();
            }
            // optionally a line on stderr every few seconds (index builds of 10^7 vectors take minutes)
            const bool progress = ix->tune.build_progress != 0;
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
        }
        VF_HIP(hipGetLastError());
    }
    guard.ix = nullptr;
    *out = ix;
    return VF_OK;
}

}  // namespace vf
