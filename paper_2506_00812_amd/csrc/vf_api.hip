// The C ABI declared in include/vecflow.h.  Every entry point runs its body under a guard, so that no C++
// exception crosses the boundary; the work itself is in vf_index_build.hip (Alg. 1), vf_route.hip (routing and
// grouping, host only) and vf_search.hip (Alg. 2).
#include "vf_host.h"

using namespace vf;

extern "C" int vf_build_index(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                              const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                              const vf_allocator *allocator, void *hip_stream, vf_index **out)
{
    return guarded([&] {
        return build_index_impl(vectors, dtype, n, dim, label_offsets, label_ids, n_labels, T, graph_degree, VF_GRAPH_KNN,
                                0, allocator, hip_stream, out);
    });
}

extern "C" int vf_build_index_opt(const void *vectors, int dtype, int64_t n, int32_t dim, const int64_t *label_offsets,
                                  const int32_t *label_ids, int32_t n_labels, int32_t T, int32_t graph_degree,
                                  int32_t graph_kind, int32_t knn_degree, const vf_allocator *allocator, void *hip_stream,
                                  vf_index **out)
{
    return guarded([&] {
        return build_index_impl(vectors, dtype, n, dim, label_offsets, label_ids, n_labels, T, graph_degree, graph_kind,
                                knn_degree, allocator, hip_stream, out);
    });
}

extern "C" int vf_search(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                         const int32_t *qlabel_ids, int32_t k, int32_t itopk, int32_t width, int32_t iters,
                         int32_t n_seeds, int64_t *out_ids, float *out_dists, void *hip_stream)
{
    return guarded([&] {
        return search_impl(index, queries, nq, qlabel_offsets, qlabel_ids, k, itopk, width, iters, n_seeds, false, out_ids,
                           out_dists, (hipStream_t)hip_stream);
    });
}

extern "C" int vf_search_ex(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                            const int32_t *qlabel_ids, const vf_search_params *params, int64_t *out_ids, float *out_dists,
                            void *hip_stream)
{
    return guarded([&]() -> int {
        VF_REQUIRE(params != nullptr, "params is NULL");
        VF_REQUIRE(params->reserved[0] == 0 && params->reserved[1] == 0, "params: reserved fields must be zero");
        return search_impl(index, queries, nq, qlabel_offsets, qlabel_ids, params->k, params->itopk, params->width,
                           params->iters, params->n_seeds, false, out_ids, out_dists, (hipStream_t)hip_stream, false,
                           params->and_scan_limit);
    });
}

extern "C" int vf_search_exact(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                               const int32_t *qlabel_ids, int32_t k, int64_t *out_ids, float *out_dists, void *hip_stream)
{
    return guarded([&] {
        return search_impl(index, queries, nq, qlabel_offsets, qlabel_ids, k, 0, 0, 0, 0, true, out_ids, out_dists,
                           (hipStream_t)hip_stream);
    });
}

extern "C" int vf_search_multi(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                               const int32_t *qlabel_ids, int32_t mode, int32_t k, int32_t itopk, int32_t width,
                               int32_t iters, int32_t n_seeds, int64_t *out_ids, float *out_dists, void *hip_stream)
{
    return guarded([&] {
        return search_multi_impl(index, queries, nq, qlabel_offsets, qlabel_ids, mode, k, itopk, width, iters, n_seeds,
                                 out_ids, out_dists, (hipStream_t)hip_stream);
    });
}

extern "C" int vf_tune(vf_index *index, const char *name, double value)
{
    return guarded([&]() -> int {
        VF_REQUIRE(name != nullptr, "name is NULL");
        if (index == nullptr) {
            std::lock_guard<std::mutex> lock(default_tuning_mutex());
            VF_REQUIRE(default_tuning().set(name, value), std::string("unknown tuning name or value out of range: ") + name);
            return VF_OK;
        }
        std::lock_guard<std::recursive_mutex> lock(index->mu);
        Tuning t = index->tune;
        VF_REQUIRE(t.set(name, value), std::string("unknown tuning name or value out of range: ") + name);
        // the seed copies depend on these two: drop them (after the device has drained), they are rebuilt on demand
        if (t.seed_cache != index->tune.seed_cache || t.seed_bf16 != index->tune.seed_bf16) {
            int rc = drop_seed_copies(index);
            if (rc != VF_OK) return rc;
        }
        index->tune = t;
        return VF_OK;
    });
}

// ---------------------------------------------------------------- export / stats

// ---------------------------------------------------------------- export / stats

static int export_impl(const vf_index *ix, int which, void *host_dst, size_t *bytes)
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

extern "C" int vf_index_export(const vf_index *index, int which, void *host_dst, size_t *bytes)
{
    return guarded([&] { return export_impl(index, which, host_dst, bytes); });
}

static int stats_impl(const vf_index *ix, vf_stats *out)
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
    out->bytes_x_ls_bf16 = ix->has_ls16 ? ix->n_groups_LS * (int64_t)ix->group_bytes() / 2 : 0;
    out->bytes_total = out->bytes_graph + out->bytes_maps + out->bytes_x_ls + out->bytes_bitsets + out->bytes_meta +
                       out->bytes_x_ls_bf16;
    return VF_OK;
}

extern "C" int vf_index_stats(const vf_index *index, vf_stats *out)
{
    return guarded([&] { return stats_impl(index, out); });
}

static int profile_enable_impl(vf_index *ix, int on)
{
    VF_REQUIRE(ix != nullptr, "index is NULL");
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    if (on)
        for (auto &set : ix->prof_ring)
            for (hipEvent_t &e : set)
                if (!e) VF_HIP(hipEventCreate(&e));
    VF_REQUIRE(on >= 0 && on <= 7 && (on & 3) != 3, "on must be 0, 1 or 2, optionally | 4");
    ix->profiling = (on & 3) != 0;
    ix->prof_serial = (on & 3) == 2;
    ix->prof_exact_counts = (on & 4) != 0;
    ix->prof_valid = false;
    ix->prof_next = 0; ix->prof_unfolded = 0;
    ix->prof_scan_sum = ix->prof_seed_sum = ix->prof_beam_sum = 0;
    ix->prof_host_plan = ix->prof_host_blob = ix->prof_host_launch = ix->prof_host_wait = 0;
    ix->prof_calls = 0;
    if (on && ix->has_ls16) {   // failed scan proofs are counted from here on
        VF_HIP(hipDeviceSynchronize());
        VF_HIP(hipMemcpy(&ix->scan_fb_seen, ix->d_scan_fb.p, 4, hipMemcpyDeviceToHost));
    }
    return VF_OK;
}

static int profile_read_impl(vf_index *ix, vf_profile *out, int32_t *per_query)
{
    VF_REQUIRE(ix && out, "NULL argument");
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    VF_REQUIRE(ix->prof_valid, "no profiled vf_search call to report");
    int rc = fold_profile(ix, vf_index::kProfRing);
    if (rc != VF_OK) return rc;
    vf_profile pf = ix->prof;
    pf.scan_ms_sum = ix->prof_scan_sum; pf.seed_ms_sum = ix->prof_seed_sum; pf.beam_ms_sum = ix->prof_beam_sum;
    pf.calls = ix->prof_calls;
    pf.host_plan_ms_sum = ix->prof_host_plan; pf.host_blob_ms_sum = ix->prof_host_blob; pf.host_launch_ms_sum = ix->prof_host_launch; pf.host_wait_ms_sum = ix->prof_host_wait;
    {
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
    }
    if (ix->has_ls16) {
        uint32_t now = 0;
        VF_HIP(hipMemcpy(&now, ix->d_scan_fb.p, 4, hipMemcpyDeviceToHost));
        pf.scan_fallbacks = (int64_t)(uint32_t)(now - ix->scan_fb_seen);
    }
    *out = pf;
    return VF_OK;
}

extern "C" int vf_profile_enable(vf_index *index, int on)
{
    return guarded([&] { return profile_enable_impl(index, on); });
}

extern "C" int vf_profile_read(vf_index *index, vf_profile *out, int32_t *per_query)
{
    return guarded([&] { return profile_read_impl(index, out, per_query); });
}

extern "C" void vf_index_free(vf_index *index)
{
    (void)guarded([&] { free_index(index); return VF_OK; });
}
