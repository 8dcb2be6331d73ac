// Search calls (Alg. 2): per-stream workspaces, the interleaved seed copies, and the launch schedule of one
// batch -- route on the host, IVF-BFS scan beside IVF-Graph seed scoring and beam search, finalise.
#include <chrono>

#include "vf_host.h"

namespace vf {

// Adds the durations of the oldest `count` unread profiled calls to the sums (waits for them).
int fold_profile(vf_index *ix, int count)
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

static size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }


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
    if (!w->owned || w->owner != s) w->prev_forked = false;
    w->owned = true;
    w->owner = s;
    if (!w->ready) {
        VF_HIP(hipStreamCreateWithFlags(&w->side, hipStreamNonBlocking));
        VF_HIP(hipEventCreateWithFlags(&w->ev_fork, hipEventDisableTiming));
        VF_HIP(hipEventCreateWithFlags(&w->ev_join, hipEventDisableTiming));
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

int check_search_args(const vf_index *ix, const void *queries, int64_t nq, int32_t k, const int64_t *out_ids,
                             const float *out_dists)
{
    VF_REQUIRE(ix != nullptr, "index is NULL");
    VF_REQUIRE(nq >= 0 && nq < ((int64_t)1 << 31), "nq out of range");
    VF_REQUIRE(nq == 0 || (queries && out_ids && out_dists), "NULL query or output pointer");
    VF_REQUIRE(((uintptr_t)queries & 15) == 0, "queries must be 16-byte aligned");
    VF_REQUIRE(k >= 1 && k <= 64, "k must be in [1, 64]");
    return VF_OK;
}

// Drops every interleaved seed copy.  Other streams may still be reading them: the device drains first.
int drop_seed_copies(vf_index *ix)
{
    VF_HIP(hipDeviceSynchronize());
    for (SeedCopy &c : ix->seed_copies) {
        for (DevBuf *b : c.bufs()) b->release();
        c.n_seeds = -1;
        c.ok = c.has_f32 = c.has_bf16 = false;
    }
    return VF_OK;
}

// The interleaved copy of the seeds of every graph list for n_seeds (see SeedCopy): the resident one, or a new
// one built on the caller's stream (the call returns after it is complete, so later calls on any stream may
// read it).  The index keeps kSeedCopies of them; the least recently used one makes room, after the device
// has drained, since calls on other streams may still be reading it.  (*out)->ok is false when a copy would need
// more than half of the free device memory: the seed kernel then gathers rows from the vector table.
bool wants_seed_copy(const vf_index *ix, bool exact, int32_t itopk, int32_t n_seeds)
{
    return !exact && !ix->graph_labels.empty() && ix->seed_mfma_ok && !ix->tune.seed_exact && n_seeds > 64 &&
           (ix->dtype == VF_U8 || itopk <= 48);
}

int seed_copy_for(vf_index *ix, int32_t n_seeds, hipStream_t s, bool build, SeedCopy **out)
{
    SeedCopy *c = nullptr;
    *out = nullptr;
    for (SeedCopy &x : ix->seed_copies)
        if (x.n_seeds == n_seeds) c = &x;
    if (c != nullptr) {
        c->last_use = ++ix->seed_tick;
        *out = c;
        return VF_OK;
    }
    if (!build) return VF_OK;
    for (SeedCopy &x : ix->seed_copies)
        if (x.n_seeds < 0) { c = &x; break; }
    if (c == nullptr) {
        c = &ix->seed_copies[0];
        for (SeedCopy &x : ix->seed_copies)
            if (x.last_use < c->last_use) c = &x;
        VF_HIP(hipDeviceSynchronize());
        for (DevBuf *b : c->bufs()) b->release();
    }
    c->last_use = ++ix->seed_tick;
    *out = c;
    return build_seed_copy(ix, n_seeds, s, ix->dtype == VF_F32 && ix->tune.seed_bf16 && !ix->seed_bf16_off, c);
}

// Fills *c for n_seeds on stream s (complete when the call returns).  want_bf16: float32 data also get the
// bfloat16 form (and lose the float32 one when it is larger than 128 MiB).
int build_seed_copy(vf_index *ix, int32_t n_seeds, hipStream_t s, bool want_bf16, SeedCopy *c)
{
    c->n_seeds = n_seeds;
    c->ok = c->has_f32 = c->has_bf16 = false;
    c->bf16_delta = 0.f;
    if (!ix->tune.seed_cache) return VF_OK;
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
    {
        const size_t need = (size_t)n_groups * (ix->group_bytes() * 3 / 2 + 32 * 4 + 32 * 4 + 32 * 4 + 32 * 4 + 32);
        size_t free_b = 0, total_b = 0;
        VF_HIP(hipMemGetInfo(&free_b, &total_b));
        if (need + need / 4 > free_b / 2) return VF_OK;
    }
    int rc;
    DevBuf d_base(&ix->alloc), d_n(&ix->alloc), d_slot(&ix->alloc), d_j0(&ix->alloc), d_src(&ix->alloc), d_cnt(&ix->alloc),
        d_err2(&ix->alloc);
    DevBufGuard rel{&d_base, &d_n, &d_slot, &d_j0, &d_src, &d_cnt, &d_err2};
    DevBuf &d_map = c->map;
    if ((rc = c->blk.reserve((size_t)n_groups * ix->group_bytes())) != VF_OK) return rc;
    if ((rc = c->norm.reserve((size_t)n_groups * 32 * 4)) != VF_OK) return rc;
    if ((rc = d_map.reserve((size_t)n_groups * 32 * 4)) != VF_OK) return rc;
    if ((rc = upload(c->goff, goff, s)) != VF_OK) return rc;
    if ((rc = upload(d_base, slot_base, s)) != VF_OK) return rc;
    if ((rc = upload(d_n, slot_n, s)) != VF_OK) return rc;
    if ((rc = upload(d_slot, grp_slot, s)) != VF_OK) return rc;
    if ((rc = upload(d_j0, grp_j0, s)) != VF_OK) return rc;
    if ((rc = upload(d_src, grp_src, s)) != VF_OK) return rc;
    if ((rc = upload(d_cnt, grp_cnt, s)) != VF_OK) return rc;
    launch_seed_map(ix->d_M_HS.as<int32_t>(), d_base.as<int64_t>(), d_n.as<int32_t>(), n_seeds, d_slot.as<int32_t>(),
                    d_j0.as<int32_t>(), n_groups, d_map.as<int32_t>(), s);
    launch_interleave(ix->dtype, ix->X, ix->dim, d_map.as<int32_t>(), d_src.as<int64_t>(), d_cnt.as<int32_t>(),
                      n_groups * 32, n_groups, ix->ncp, c->blk.as<uint4>(), c->norm.p, s);
    VF_HIP(hipGetLastError());
    VF_HIP(hipStreamSynchronize(s));   // the tables above are pageable host memory and temporaries
    c->has_f32 = true;
    if (want_bf16) {
        // float32 data: a second copy in bfloat16; the largest rounding error of a seed goes into the
        // beam kernel's proof (zero for integer-valued data up to 256, SIFT's kind)
        if ((rc = c->blk16.reserve((size_t)n_groups * ix->group_bytes() / 2)) != VF_OK) return rc;
        if ((rc = d_err2.reserve((size_t)n_groups * 32 * 4)) != VF_OK) return rc;
        launch_seed_pack_bf16(c->blk.as<uint4>(), n_groups, ix->ncp, c->blk16.as<uint4>(), d_err2.as<float>(), s);
        std::vector<float> e2((size_t)n_groups * 32);
        VF_HIP(hipMemcpyAsync(e2.data(), d_err2.p, e2.size() * 4, hipMemcpyDeviceToHost, s));
        VF_HIP(hipStreamSynchronize(s));
        double mx = 0.0;
        bool finite = true;
        for (float v : e2) { finite = finite && v == v && v <= 3.0e38f; mx = v > mx ? v : mx; }
        if (!finite) c->blk16.release();
        if (finite) {
            // small batches are served from the float32 copy (its proofs need fewer re-scored seeds, which
            // is what a latency-bound call notices), so a copy of up to 128 MiB stays
            if ((size_t)n_groups * ix->group_bytes() > ((size_t)128 << 20)) {
                c->blk.release();
                c->has_f32 = false;
            }
            c->has_bf16 = true;
            c->bf16_delta = (float)(std::sqrt(mx) * 1.001);
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
    c->ok = true;
    return VF_OK;
}

// ---------------------------------------------------------------- one search call: plan, blob, launches

int check_search_params(const vf_index *ix, bool exact, int32_t k, int32_t &itopk, int32_t width, int32_t iters,
                               int32_t &n_seeds)
{
    if (exact) return VF_OK;
    VF_REQUIRE(itopk >= k && itopk >= 1 && itopk <= 256, "itopk must be in [k, 256]");
    VF_REQUIRE(width >= 1 && width <= 8 && width * ix->R <= 128, "width must be >= 1 with width * R <= 128");
    VF_REQUIRE(iters >= 0, "iters must be >= 0");
    VF_REQUIRE(n_seeds >= 0, "n_seeds must be >= 0");
    if (n_seeds == 0) n_seeds = itopk;
    return VF_OK;
}

// Routing, work lists, blob layout.  dseed_budget_words: how large a seed distance matrix may be (beyond it the
// beam kernel gathers the seeds itself).
int plan_call(const vf_index *ix, Routed &r, int64_t nq, const int64_t *qoff, const int32_t *qids, bool exact,
                     bool first_is_searched, int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds,
                     int32_t and_scan_limit, uint64_t dseed_budget_words, const SeedCopy *sc, CallPlan &P)
{
    int rc;
    P.nq = nq; P.k = k; P.itopk = itopk; P.width = width; P.iters = iters; P.n_seeds = n_seeds; P.exact = exact;
    if (!exact) {
        while (P.beam_LP < itopk + std::max(64, width * ix->R)) P.beam_LP <<= 1;
        const int64_t visits = (int64_t)iters * width * ix->R;
        while (P.beam_hb < 13 && ((int64_t)1 << P.beam_hb) < 2 * visits) ++P.beam_hb;
        BeamParams chk{};
        chk.dim = ix->dim; chk.LP = P.beam_LP; chk.hash_bits = P.beam_hb;
        VF_REQUIRE(beam_lds_bytes(chk, ix->dtype) <= 64 * 1024, "search parameters need more than 64 KiB of LDS");
    }
    VF_REQUIRE(scan_lds_bytes(ix->ncp, exact ? 32 : std::max(P.ib.tile_rows, 16), k) <= 64 * 1024,
               "the scan tile of this dim and k needs more than 64 KiB of LDS");
    if ((rc = route_queries(ix->route_view(), nq, qoff, qids, exact, first_is_searched, r)) != VF_OK) return rc;

    // scan items over the stored interleaved lists (scan labels); in exact mode graph labels follow
    ItemBuilder &ib = P.ib;
    size_t first_hs = r.scan_pairs.size();
    // float32 lists of large batches are filtered from their bfloat16 copy and re-ranked (every item then leaves
    // partial rows of scan_keep candidates and every scan query gets a merge item); small batches keep the FMA kernel
    {
        const Tuning &tn = ix->tune;
        const int32_t keep = std::min(64, k + tn.scan_bf16_margin);
        const bool small_batch = tn.scan_valu == 2 || (tn.scan_valu == 1 && r.scan_pairs.size() <= 256);
        if (!exact && ix->has_ls16 && tn.scan_bf16 && tn.scan16 && !small_batch && keep > k &&
            !r.scan_pairs.empty() && scan_bf16_supported(ix->dtype, ix->dim, ib.tile_rows, keep) &&
            scan_bf16_lds_bytes(std::max(ib.tile_rows, 16), keep) <= 64 * 1024) {
            P.scan_bf16 = true;
            P.scan_keep = keep;
            ib.all_partial = true;
            ib.seg_groups = ib.seg_groups_heavy = tn.scan_bf16_seg_groups;
        }
    }
    if (exact) {
        // scan labels first, graph labels after them (both still ordered by label)
        std::stable_partition(r.scan_pairs.begin(), r.scan_pairs.end(), [&](uint64_t pr) {
            return ix->O_LS[(size_t)(pr >> 32)] >= 0;
        });
        first_hs = 0;
        while (first_hs < r.scan_pairs.size() && ix->O_LS[(size_t)(r.scan_pairs[first_hs] >> 32)] >= 0) ++first_hs;
    }
    ib.qrow.reserve(r.scan_pairs.size());     // (no regrowth while the work lists are built)
    ib.items.reserve(r.scan_pairs.size());
    ib.merges.reserve(r.scan_pairs.size());
    for (size_t i = 0; i < first_hs;) {
        const int32_t l = (int32_t)(r.scan_pairs[i] >> 32);
        size_t e = i;
        while (e < first_hs && (int32_t)(r.scan_pairs[e] >> 32) == l) ++e;
        ib.add_label(r.scan_pairs, i, e, ix->GO_LS[(size_t)l], ix->O_LS[(size_t)l], ix->S[(size_t)l]);
        i = e;
    }
    P.n_ls_items = ib.items.size(); P.n_ls_merges = ib.merges.size();
    // exact mode: one temporary interleaved copy per graph label, used right after it is made
    for (size_t i = first_hs; i < r.scan_pairs.size();) {
        const int32_t l = (int32_t)(r.scan_pairs[i] >> 32);
        size_t e = i;
        while (e < r.scan_pairs.size() && (int32_t)(r.scan_pairs[e] >> 32) == l) ++e;
        const size_t lo = ib.items.size();
        ib.add_label(r.scan_pairs, i, e, 0, ix->O_HS[(size_t)l], ix->S[(size_t)l]);
        P.hs_runs.push_back({l, lo, ib.items.size()});
        P.max_hs_list = std::max(P.max_hs_list, ix->S[(size_t)l]);
        i = e;
    }
    VF_REQUIRE(ib.part_rows < ((int64_t)1 << 31), "too many partial result rows in one call");
    P.part_words = (size_t)ib.part_rows * (P.scan_bf16 ? P.scan_keep : k);

    // selectivity-aware routing: AND queries whose (smallest) graph list is short leave the graph path
    r.xq_query.clear(); r.xq_label.clear();
    if (!exact && and_scan_limit > 0 && r.any_and) {
        size_t w = 0;
        for (size_t i = 0; i < r.gq_query.size(); ++i) {
            const int32_t q = r.gq_query[i], l = r.gq_label[i];
            if (r.others_off[(size_t)q + 1] > r.others_off[(size_t)q] && ix->S[(size_t)l] <= and_scan_limit) {
                r.xq_query.push_back(q); r.xq_label.push_back(l);
            } else {
                r.gq_query[w] = q; r.gq_label[w] = l; ++w;
            }
        }
        r.gq_query.resize(w); r.gq_label.resize(w);
    }
    P.n_xq = r.xq_query.size();
    P.n_gq = r.gq_query.size();
    P.ns_stride = (n_seeds + 31) & ~31;
    // Seeds on the matrix cores.  uint8: they give the exact integer distances, nothing else changes.
    // float32: approximations, re-ranked by the beam kernel (its proof needs a list of at most 48 entries).
    const bool mfma_ok = wants_seed_copy(ix, exact, itopk, n_seeds) && P.n_gq > 0;
    // With an interleaved seed copy the seed kernel also selects (itopk <= 64: the beam kernel's one-register
    // list): it leaves sel_K keys per (query, seed segment) instead of every distance.  float32 data: from the
    // bfloat16 copy; calls with few graph queries keep the float32 copy and the unfused kernel (their proofs
    // need fewer re-scored seeds, which a latency-bound call notices).
    const Tuning &tune = ix->tune;
    if (mfma_ok && sc != nullptr && sc->ok && tune.seed_select && itopk <= 64 &&
        seed_select_supported(ix->dtype, ix->dim, sc->has_bf16) &&
        (ix->dtype == VF_U8 || !sc->has_f32 || (int64_t)P.n_gq >= tune.seed_bf16_min_batch)) {
        P.sel_bf16 = ix->dtype == VF_F32;
        P.sel_K = ix->dtype == VF_U8 ? itopk : std::min(64, itopk + std::max(tune.seed_margin_bf16, tune.seed_margin));
        int32_t longest = 0;
        size_t n_tiles = 0;
        for (size_t i = 0; i < P.n_gq;) {
            size_t e = i;
            while (e < P.n_gq && r.gq_label[e] == r.gq_label[i]) ++e;
            longest = std::max(longest, std::min(n_seeds, ix->S[(size_t)r.gq_label[i]]));
            n_tiles += (e - i + 31) / 32;
            i = e;
        }
        // seeds per wave: long segments select better (a row's threshold tightens as the segment streams by) but
        // the launch needs a few thousand waves
        int32_t seg = tune.seed_seg_seeds;
        if (seg <= 0) {
            const int64_t want_segs = std::max<int64_t>(1, (2048 + (int64_t)n_tiles - 1) / (int64_t)n_tiles);
            seg = (int32_t)std::min<int64_t>(16384, std::max<int64_t>(512, (longest / want_segs) / 32 * 32));
        }
        seg = std::max(32, seg / 32 * 32);
        P.seg_seeds = seg;
        P.max_segs = (longest + seg - 1) / seg;
        const uint64_t need = (uint64_t)P.n_gq * (uint64_t)P.max_segs * (uint64_t)P.sel_K * 2;   // 8-byte keys
        if (need <= dseed_budget_words) {
            P.seed_select = true;
            P.dense_seeds = P.seeds_mfma = true;
            P.dseed_words = (size_t)need;
        }
    }
    if (!P.seed_select) {
        // every distance goes through the seed distance matrix, which must fit
        const uint64_t need = (uint64_t)P.n_gq * (uint64_t)P.ns_stride + 64 * 1024;
        P.dense_seeds = !exact && P.n_gq > 0 && seed_dist_supported(ix->dtype, ix->dim) && need <= dseed_budget_words;
        P.seeds_mfma = P.dense_seeds && mfma_ok;
        if (P.dense_seeds) P.dseed_words = (size_t)need;
    }
    if (P.dense_seeds) {
        const size_t tile_q = P.seeds_mfma ? 32 : 64;
        for (size_t i = 0; i < P.n_gq;) {
            size_t e = i;
            while (e < P.n_gq && r.gq_label[e] == r.gq_label[i]) ++e;
            for (size_t t = i; t < e; t += tile_q)
                P.tiles.push_back(SeedTile{r.gq_label[i], (int32_t)t, (int32_t)std::min<size_t>(tile_q, e - t)});
            i = e;
        }
    }
    BlobLayout &L = P.L;
    size_t o = 0;
    L.off_gq_query = o; o = align_up(o + P.n_gq * 4);
    L.off_gq_label = o; o = align_up(o + P.n_gq * 4);
    L.off_xq_query = o; o = align_up(o + P.n_xq * 4);
    L.off_xq_label = o; o = align_up(o + P.n_xq * 4);
    L.off_others_off = o; o = align_up(o + (r.any_and ? r.others_off.size() : 1) * 4);   // (not sent when no query has partners)
    L.off_others = o; o = align_up(o + std::max<size_t>(r.others.size(), 1) * 4);
    L.off_qrow = o; o = align_up(o + std::max<size_t>(ib.qrow.size(), 1) * 4);
    L.off_items = o; o = align_up(o + std::max<size_t>(ib.items.size(), 1) * sizeof(ScanItem));
    L.off_merges = o; o = align_up(o + std::max<size_t>(ib.merges.size(), 1) * sizeof(MergeItem));
    L.off_tiles = o; o = align_up(o + std::max<size_t>(P.tiles.size(), 1) * sizeof(SeedTile));
    L.off_empty = o; o = align_up(o + std::max<size_t>(r.empty_q.size(), 1) * 4);
    L.total = o;
    return VF_OK;
}

// The routing blob in host memory (hp holds P.L.total bytes).
void fill_blob(const CallPlan &P, const Routed &r, char *hp)
{
    const BlobLayout &L = P.L;
    const ItemBuilder &ib = P.ib;
    if (P.n_gq) {
        memcpy(hp + L.off_gq_query, r.gq_query.data(), P.n_gq * 4);
        memcpy(hp + L.off_gq_label, r.gq_label.data(), P.n_gq * 4);
    }
    if (P.n_xq) {
        memcpy(hp + L.off_xq_query, r.xq_query.data(), P.n_xq * 4);
        memcpy(hp + L.off_xq_label, r.xq_label.data(), P.n_xq * 4);
    }
    if (r.any_and) memcpy(hp + L.off_others_off, r.others_off.data(), r.others_off.size() * 4);
    if (!r.others.empty()) memcpy(hp + L.off_others, r.others.data(), r.others.size() * 4);
    if (!ib.qrow.empty()) memcpy(hp + L.off_qrow, ib.qrow.data(), ib.qrow.size() * 4);
    if (!ib.items.empty()) memcpy(hp + L.off_items, ib.items.data(), ib.items.size() * sizeof(ScanItem));
    if (!ib.merges.empty()) memcpy(hp + L.off_merges, ib.merges.data(), ib.merges.size() * sizeof(MergeItem));
    if (!P.tiles.empty()) memcpy(hp + L.off_tiles, P.tiles.data(), P.tiles.size() * sizeof(SeedTile));
    if (!r.empty_q.empty()) memcpy(hp + L.off_empty, r.empty_q.data(), r.empty_q.size() * 4);
}

// The launches of one call.  s: the caller's stream; side: the stream the scan path runs on beside the graph path
// (ev_fork / ev_join tie it to s), or nullptr: everything on s.  may_allocate = false (the entry point that
// allocates nothing): no seed copy is built, no profiling, no failed-proof watch.
int launch_call(vf_index *ix, const CallPlan &P, const Routed &r, const CallMem &M, const SeedCopy *sc, const void *queries,
                int64_t *out_ids, float *out_dists, hipStream_t s, hipStream_t side, hipEvent_t ev_fork, hipEvent_t ev_join,
                bool may_allocate)
{
    int rc;
    const Tuning &tune = ix->tune;
    const BlobLayout &L = P.L;
    const ItemBuilder &ib = P.ib;
    char *dp = M.blob;
    const int32_t k = P.k;
    const size_t n_gq = P.n_gq;
    const bool forked = side != nullptr;
    const bool exact = P.exact;

    // every routed query's kernel writes all k entries of its row; only queries without any match are padded here
    launch_fill_rows(out_ids, out_dists, (const int32_t *)(dp + L.off_empty), (int64_t)r.empty_q.size(), k, s);

    const bool prof = may_allocate && ix->profiling;
    if (prof) {
        if (ix->prof_unfolded == vf_index::kProfRing && (rc = fold_profile(ix, 1)) != VF_OK) return rc;
        ix->prof_ev = ix->prof_ring[ix->prof_next];
        // [nq][4] counters, then [nq] gathered; written by the beam kernel for graph queries only (no clearing
        // pass: the rows of the other queries are never read)
        if ((rc = ix->counters.reserve((size_t)P.nq * 24)) != VF_OK) return rc;
        ix->prof_graph_queries = r.gq_query;
        ix->prof_graph_queries.insert(ix->prof_graph_queries.end(), r.xq_query.begin(), r.xq_query.end());
        vf_profile &pf = ix->prof;
        pf = vf_profile{};
        pf.nq = P.nq; pf.n_graph_queries = (int64_t)r.gq_query.size(); pf.n_scan_queries = (int64_t)ib.qrow.size();
        pf.n_scan_items = (int64_t)ib.items.size();
        for (const ScanItem &it : ib.items) { pf.scan_list_entries += it.n; pf.scan_pairs += (int64_t)it.n * it.q_count; }
        pf.n_seed_tiles = (int64_t)P.tiles.size();
        pf.seeds_on_matrix_cores = P.seeds_mfma ? 1 : 0;
        for (const SeedTile &t : P.tiles) {
            const int64_t ns_l = std::min<int64_t>(P.n_seeds, ix->S[(size_t)t.label]);
            pf.seed_pairs += ns_l * t.q_count;
            pf.seed_tile_seeds += ns_l;
        }
    }
    hipStream_t ss = s;
    const int32_t *d_others_off = r.any_and ? (const int32_t *)(dp + L.off_others_off) : nullptr;
    const int32_t *d_others = (const int32_t *)(dp + L.off_others);

    BeamParams bp{};
    if (n_gq || P.n_xq) {
        bp.X = ix->X; bp.Q = queries; bp.G = ix->d_G.as<int32_t>(); bp.Gg = ix->d_Gg.as<int32_t>();
        bp.gq_query = (const int32_t *)(dp + L.off_gq_query);
        bp.gq_label = (const int32_t *)(dp + L.off_gq_label);
        bp.others_off = d_others_off; bp.others = d_others; bp.meta = ix->meta();
        bp.dim = ix->dim; bp.R = ix->R; bp.k = k; bp.itopk = P.itopk; bp.width = P.width; bp.iters = P.iters;
        bp.n_seeds = P.n_seeds;
        bp.lat_waves = ix->tune.beam_lat_waves;
        bp.LP = P.beam_LP;
        bp.hash_bits = P.beam_hb;
        bp.out_ids = out_ids; bp.out_dists = out_dists;
        bp.counters = prof ? ix->counters.as<int32_t>() : nullptr;
        bp.gathered = prof ? ix->counters.as<int32_t>() + (size_t)P.nq * 4 : nullptr;
        bp.dseed = nullptr; bp.ns_stride = P.ns_stride;
    }
    // While profiling, the beam kernel's launch takes the two events that bracket it (end of seed scoring = its begin,
    // and its end) as the kernel's own begin and end times: events recorded around it would each put a barrier packet
    // on the stream, and the timed kernels a few microseconds apart.
    const bool attach = prof && n_gq > 0 && P.n_xq == 0;
    auto count_passing_seeds = [&]() {
        if (prof && ix->prof_exact_counts && n_gq && (P.seed_select || P.dense_seeds) && r.any_and) {
            // profiling only, outside the timed interval: the counters report the seeds that pass the predicate as
            // distances computed, and neither the selecting seed kernel nor the beam kernel's selection from a
            // row of seed distances tests the seeds that cannot enter a full list
            launch_seed_pass_count(bp.gq_query, bp.gq_label, bp.meta, P.n_seeds, d_others_off, d_others,
                                   ix->counters.as<int32_t>() + (size_t)P.nq * 5, (int)n_gq, s);
        }
    };
    auto run_seeds = [&]() -> int {
        // (a profiled call that forks has recorded this event already: it is its fork event)
        if (prof && !forked) VF_HIP(hipEventRecord(ix->prof_ev[2], s));
        if (n_gq && P.seed_select) {
            // scoring and selection in one kernel: runs of sel_K keys per (query, seed segment)
            SeedSelParams sl{};
            sl.Q = queries; sl.gq_query = bp.gq_query;
            sl.tiles = (const SeedTile *)(dp + L.off_tiles); sl.meta = bp.meta;
            sl.dim = ix->dim; sl.n_seeds = P.n_seeds; sl.K = P.sel_K; sl.seg_seeds = P.seg_seeds; sl.max_segs = P.max_segs;
            sl.seed_blk = P.sel_bf16 ? sc->blk16.as<uint4>() : sc->blk.as<uint4>();
            sl.seed_norm = sc->norm.as<uint32_t>();
            sl.seed_goff = sc->goff.as<int64_t>();
            sl.seed_map = sc->map.as<int32_t>();
            sl.others_off = d_others_off; sl.others = d_others;
            sl.runs = (uint64_t *)M.dseed;
            launch_seed_select(ix->dtype, sl, (int)P.tiles.size(), s);
            bp.seed_runs = sl.runs; bp.run_K = P.sel_K; bp.run_segs = P.max_segs; bp.seg_seeds = P.seg_seeds;
            if (prof) {
                ix->prof.seeds_on_matrix_cores = P.sel_bf16 ? 2 : 1;
                ix->prof.seed_selected = 1;
                for (const SeedTile &t : P.tiles) {
                    const int64_t ns_l = std::min<int64_t>(P.n_seeds, ix->S[(size_t)t.label]);
                    ix->prof.seed_run_keys += (int64_t)t.q_count * ((ns_l + P.seg_seeds - 1) / P.seg_seeds) * P.sel_K;
                }
                if (ix->prof_exact_counts && r.any_and) bp.seed_pass = ix->counters.as<int32_t>() + (size_t)P.nq * 5;   // filled before the timed interval
            }
            if (ix->dtype == VF_F32) {
                // two bfloat16 products per component (<= 256 terms, <= 2 u each: 512 u), the query's split
                // (2^-16 = 256 u), norms and final additions (< 200 u): under 1024 u; 4096 u = 2^-12 relative to
                // |q|^2 + xn_max is used, plus 2 |q| max |x - bf16(x)|
                bp.seed_approx = 1; bp.xn_max = ix->xn_max;
                bp.err_bound = ix->seed_err_bound() * 8.0f;
                bp.err_q = 2.0f * sc->bf16_delta;
                bp.seed_keep = P.sel_K;
                if (may_allocate) bp.fallback_count = ix->d_fb_count.as<uint32_t>();
            }
        } else if (n_gq && P.dense_seeds) {
            SeedParams sd{};
            sd.X = ix->X; sd.Q = queries; sd.gq_query = bp.gq_query;
            sd.tiles = (const SeedTile *)(dp + L.off_tiles); sd.meta = bp.meta;
            sd.dim = ix->dim; sd.n_seeds = P.n_seeds; sd.ns_stride = P.ns_stride;
            sd.dseed = M.dseed;
            sd.dump_off = (int64_t)n_gq * P.ns_stride;
            sd.dump_mask = 1023;
            if (P.seeds_mfma) {
                sd.chunk_seeds = kSeedMfmaChunk;
                sd.max_chunks = (P.ns_stride + kSeedMfmaChunk - 1) / kSeedMfmaChunk;
                sd.xnorm_all = ix->d_xnorm_all.as<uint32_t>();
                float seed_bf16_delta = 0.f;
                if (sc != nullptr && sc->ok) {
                    // without the watch on failed proofs (it needs a pinned counter) the bfloat16 form is used only
                    // where it is the only one
                    const bool use16 = sc->has_bf16 &&
                                       (!sc->has_f32 || (may_allocate && (int64_t)n_gq >= tune.seed_bf16_min_batch));
                    sd.seed_blk = use16 ? sc->blk16.as<uint4>() : sc->blk.as<uint4>();
                    sd.seed_norm = sc->norm.as<uint32_t>();
                    sd.seed_goff = sc->goff.as<int64_t>();
                    sd.seed_bf16 = use16 ? 1 : 0;
                    seed_bf16_delta = sc->bf16_delta;
                    if (prof && sd.seed_bf16) ix->prof.seeds_on_matrix_cores = 2;
                    // seeds per wave: few long waves share the chip better with the scan (512 seeds:
                    // step 0.374 -> 0.340 ms on 10,000-query batches), small batches need many short ones
                    sd.chunk_seeds = 4 * kSeedMfmaChunk;
                    if ((int64_t)P.tiles.size() * ((P.ns_stride + sd.chunk_seeds - 1) / sd.chunk_seeds) < 512)
                        sd.chunk_seeds = kSeedMfmaChunk;
                    sd.max_chunks = (P.ns_stride + sd.chunk_seeds - 1) / sd.chunk_seeds;
                }
                launch_seed_mfma(ix->dtype, sd, (int)P.tiles.size(), s);
                if (ix->dtype == VF_F32) {
                    bp.seed_approx = 1; bp.err_bound = ix->seed_err_bound(); bp.xn_max = ix->xn_max;
                    bp.seed_keep = std::min(64, P.itopk + tune.seed_margin);
                    if (sd.seed_bf16) {
                        // the bfloat16 bound (see above) and its wider margin: more approximations are kept for
                        // re-ranking (a failed proof costs the query a gather of every seed)
                        bp.err_bound = ix->seed_err_bound() * 8.0f;
                        bp.err_q = 2.0f * seed_bf16_delta;
                        if (may_allocate) bp.fallback_count = ix->d_fb_count.as<uint32_t>();
                        bp.seed_keep = std::min(64, P.itopk + std::max(tune.seed_margin_bf16, tune.seed_margin));
                    }
                }
            } else {
                sd.max_chunks = P.ns_stride / kSeedChunk;
                launch_seed_dist(ix->dtype, sd, (int)P.tiles.size(), s);
            }
            bp.dseed = sd.dseed;
            if (r.any_and && sc != nullptr && sc->ok) { bp.seed_map = sc->map.as<int32_t>(); bp.seed_goff = sc->goff.as<int64_t>(); }
            if (prof && ix->prof_exact_counts && r.any_and) bp.seed_pass = ix->counters.as<int32_t>() + (size_t)P.nq * 5;   // filled before the timed interval
        }
        if (prof && !attach) VF_HIP(hipEventRecord(ix->prof_ev[3], s));
        return VF_OK;
    };
    auto run_scan = [&]() -> int {
        if (forked) {
            // (while profiling the event that marks the start of the graph path serves as the fork event: every
            // event recorded on the caller's stream delays the kernel behind it by a few microseconds)
            hipEvent_t fork = prof ? ix->prof_ev[2] : ev_fork;
            VF_HIP(hipEventRecord(fork, s));
            VF_HIP(hipStreamWaitEvent(side, fork, 0));
            ss = side;
        }
        if (prof) VF_HIP(hipEventRecord(ix->prof_ev[0], ss));

        ScanParams sp{};
        sp.qsrc = queries; sp.qrow = (const int32_t *)(dp + L.off_qrow);
        sp.dim = ix->dim; sp.ncp = ix->ncp; sp.K = k; sp.tile_rows = ib.tile_rows;
        sp.out_ids = out_ids; sp.out_dists = out_dists;
        sp.res_idx = M.part_idx; sp.res_bits = M.part_bits;
        const MergeItem *d_merges = (const MergeItem *)(dp + L.off_merges);
        sp.others_off = d_others_off; sp.others = d_others; sp.meta = ix->meta();
        if (P.n_ls_items) {
            sp.xblk = ix->d_X_LS.as<uint4>(); sp.xnorm = ix->d_xnorm_LS.p; sp.map = ix->d_M_LS.as<int32_t>();
            sp.items = (const ScanItem *)(dp + L.off_items);
            // small batches are latency-bound: the FMA kernel finishes a one-query tile three times sooner;
            // large batches keep the matrix-core kernel, which leaves the vector ALU to the beam search
            const bool small_batch = tune.scan_valu == 2 || (tune.scan_valu == 1 && ib.qrow.size() <= 256);
            if (P.scan_bf16) {
                // filter from the bfloat16 copy, then re-rank (a query whose result is not proven complete is
                // scanned exactly by its re-ranking wave)
                ScanParams sb = sp;
                sb.xblk = ix->d_X_LS16.as<uint4>(); sb.K = P.scan_keep;
                launch_scan_bf16(sb, (int)P.n_ls_items, tune.scan_bf16_slots, ss);
                if (prof) { ix->prof.scan_kernel = 3; VF_HIP(hipEventRecord(ix->prof_ev[1], ss)); }
                RerankParams rp{};
                rp.items = d_merges; rp.res_idx = sp.res_idx; rp.res_bits = sp.res_bits; rp.map = sp.map;
                rp.X = ix->X; rp.Q = queries; rp.dim = ix->dim; rp.Kc = P.scan_keep; rp.K = k;
                // the bound of the bfloat16 seed proofs (same arithmetic: two bfloat16 products per component into a
                // float32 accumulator, norms of the unrounded vectors), with the lists' own largest norm and rounding error
                rp.err_bound = ix->seed_err_bound() * 8.0f; rp.xn_max = ix->ls_xn_max; rp.err_q = 2.0f * ix->ls_bf16_delta;
                rp.fail_count = ix->d_scan_fb.as<uint32_t>();
                rp.others_off = sp.others_off; rp.others = sp.others; rp.meta = sp.meta;
                rp.out_ids = out_ids; rp.out_dists = out_dists;
                launch_scan_rerank(rp, (int)P.n_ls_merges, ss);
            } else if (!exact && small_batch && scan_valu_supported(ix->dtype, ix->dim, sp.tile_rows)) {
                launch_scan_valu(sp, (int)P.n_ls_items, ss);
                if (prof) ix->prof.scan_kernel = 2;
            } else if (!exact && tune.scan16 && scan16_supported(ix->dtype, ix->dim, sp.tile_rows)) {
                launch_scan16(sp, (int)P.n_ls_items, ss);
                if (prof) ix->prof.scan_kernel = 1;
            } else {
                launch_scan(ix->dtype, sp, (int)P.n_ls_items, ss);
            }
            // a search times its scan kernel by itself (the merge of the segments' candidates follows it)
            if (!P.scan_bf16) {
                if (prof && P.hs_runs.empty()) VF_HIP(hipEventRecord(ix->prof_ev[1], ss));
                launch_scan_merge(ix->dtype, d_merges, (int)P.n_ls_merges, sp.res_idx, sp.res_bits, k, ib.max_nseg * k,
                                  ix->d_M_LS.as<int32_t>(), out_ids, out_dists, ss);
            }
        }
        if (!P.hs_runs.empty()) {
            const int64_t max_groups = (P.max_hs_list + 31) / 32;
            if ((rc = ix->tmp_blk.reserve((size_t)max_groups * ix->group_bytes())) != VF_OK) return rc;
            if ((rc = ix->tmp_norm.reserve((size_t)max_groups * 32 * 4)) != VF_OK) return rc;
            for (const HsRun &run : P.hs_runs) {
                const int32_t nl = ix->S[(size_t)run.label];
                launch_interleave(ix->dtype, ix->X, ix->dim, ix->d_M_HS.as<int32_t>() + ix->O_HS[(size_t)run.label], nullptr,
                                  nullptr, nl, (nl + 31) / 32, ix->ncp, ix->tmp_blk.as<uint4>(), ix->tmp_norm.p, s);
                sp.xblk = ix->tmp_blk.as<uint4>(); sp.xnorm = ix->tmp_norm.p; sp.map = ix->d_M_HS.as<int32_t>();
                sp.items = (const ScanItem *)(dp + L.off_items) + run.item_lo;
                launch_scan(ix->dtype, sp, (int)(run.item_hi - run.item_lo), s);
            }
            launch_scan_merge(ix->dtype, d_merges + P.n_ls_merges, (int)(ib.merges.size() - P.n_ls_merges), sp.res_idx,
                              sp.res_bits, k, ib.max_nseg * k, ix->d_M_HS.as<int32_t>(), out_ids, out_dists, s);
        }
        if (prof && !(P.hs_runs.empty() && P.n_ls_items)) VF_HIP(hipEventRecord(ix->prof_ev[1], ss));
        if (forked) VF_HIP(hipEventRecord(ev_join, ss));
        return VF_OK;
    };
    // the scan goes first: its longest work items decide when it ends (measured: forking it
    // after the seed kernel costs 6 to 20 % of the step)
    count_passing_seeds();
    if ((rc = run_scan()) != VF_OK) return rc;
    if ((rc = run_seeds()) != VF_OK) return rc;
    if (n_gq) launch_beam(ix->dtype, bp, (int)n_gq, s, attach ? ix->prof_ev[3] : nullptr, attach ? ix->prof_ev[4] : nullptr);
    if (P.n_xq) {
        // the exact route of short AND queries: the beam kernel with every member of the list as a seed, no
        // iteration and a list of k entries -- each member is tested with the predicate, the members that pass
        // are gathered and scored, the k best stay
        BeamParams bx = bp;
        bx.gq_query = (const int32_t *)(dp + L.off_xq_query);
        bx.gq_label = (const int32_t *)(dp + L.off_xq_label);
        bx.n_seeds = 0x7FFFFFFF; bx.iters = 0; bx.itopk = k; bx.LP = 128; bx.hash_bits = 9;
        bx.dseed = nullptr; bx.seed_runs = nullptr; bx.seed_pass = nullptr; bx.seed_approx = 0; bx.fallback_count = nullptr;
        launch_beam(ix->dtype, bx, (int)P.n_xq, s);
    }
    if (bp.fallback_count != nullptr) {
        ix->fb_window_q += (int64_t)n_gq;
        if (!ix->fb_pending && ix->fb_window_q >= tune.seed_fb_window) {
            VF_HIP(hipMemcpyAsync(ix->h_fb, bp.fallback_count, 4, hipMemcpyDeviceToHost, s));
            VF_HIP(hipEventRecord(ix->ev_fb, s));
            ix->fb_pending = true;
            ix->fb_sent_q = ix->fb_window_q;
            ix->fb_window_q = 0;
        }
    }
    if (prof) {
        if (!attach) VF_HIP(hipEventRecord(ix->prof_ev[4], s));
        ix->prof_valid = true;
        ix->prof_next = (ix->prof_next + 1) % vf_index::kProfRing;
        ++ix->prof_unfolded;
    }
    if (forked) VF_HIP(hipStreamWaitEvent(s, ev_join, 0));
    return VF_OK;
}

// first_is_searched: every query searches the list of its first label (the others are the
// predicate) instead of its smallest list -- the sub-searches of vf_search_multi.
int search_impl(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids, int32_t k,
                int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds, bool exact, int64_t *out_ids,
                float *out_dists, hipStream_t s, bool first_is_searched, int32_t and_scan_limit)
{
    int rc = check_search_args(ix, queries, nq, k, out_ids, out_dists);
    if (rc != VF_OK) return rc;
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    const auto t_enter = std::chrono::steady_clock::now();
    if ((rc = check_search_params(ix, exact, k, itopk, width, iters, n_seeds)) != VF_OK) return rc;
    Workspace *W = nullptr;
    if ((rc = workspace_for(ix, s, &W)) != VF_OK) return rc;
    if (nq == 0) return VF_OK;
    const Tuning &tune = ix->tune;
    // the seed distance matrix reuses what is allocated, or grows into at most half of the free memory
    uint64_t dseed_budget = W->dseed.cap / 4;
    // (the driver is only asked when the buffer at hand may be too small for this call: the query is slow)
    if ((uint64_t)nq * (uint64_t)((std::max(n_seeds, itopk) + 31) & ~31) + 64 * 1024 > dseed_budget) {
        size_t free_b = 0, total_b = 0;
        VF_HIP(hipMemGetInfo(&free_b, &total_b));
        dseed_budget = std::max<uint64_t>(dseed_budget, (uint64_t)((free_b + W->dseed.cap) / 2) / 5);   // / 4 bytes, / 1.25 growth
    }
    // the interleaved copy of the seeds for this seed count (built on first use), after a look at the watch
    // on failed float32 proofs
    SeedCopy *sc = nullptr;
    if (wants_seed_copy(ix, exact, itopk, n_seeds)) {
        if (ix->fb_pending && hipEventQuery(ix->ev_fb) == hipSuccess) {
            const uint32_t now = *ix->h_fb, failed = now - ix->fb_last;
            ix->fb_last = now;
            ix->fb_pending = false;
            if ((int64_t)failed * 64 > ix->fb_sent_q) {
                ix->seed_bf16_off = true;   // the copies are rebuilt in float32
                if ((rc = drop_seed_copies(ix)) != VF_OK) return rc;
            }
        } else if (ix->fb_pending) {
            (void)hipGetLastError();      // "not ready" is no error
        }
        if ((rc = seed_copy_for(ix, n_seeds, s, true, &sc)) != VF_OK) return rc;
    }
    CallPlan P(tune);
    Routed &r = W->routed;
    VF_REQUIRE(and_scan_limit >= 0, "and_scan_limit must be >= 0");
    if ((rc = plan_call(ix, r, nq, qoff, qids, exact, first_is_searched, k, itopk, width, iters, n_seeds, and_scan_limit,
                        dseed_budget, sc, P)) != VF_OK)
        return rc;
    const BlobLayout &L = P.L;
    const auto t_planned = std::chrono::steady_clock::now();
    Staging *st = nullptr;
    if ((rc = get_staging(W, L.total, &st)) != VF_OK) return rc;
    const auto t_staged = std::chrono::steady_clock::now();   // (waiting for the staging buffer is the GPU's time, not the host's)
    char *hp = (char *)st->p;
    fill_blob(P, r, hp);
    const auto t_blob = std::chrono::steady_clock::now();
    if (P.dense_seeds && (rc = W->dseed.reserve(P.dseed_words * 4)) != VF_OK) return rc;
    if (P.part_words > 0) {
        if ((rc = W->part_idx.reserve(P.part_words * 4)) != VF_OK) return rc;
        if ((rc = W->part_bits.reserve(P.part_words * 4)) != VF_OK) return rc;
    }
    // The scan path runs on the side stream beside the graph path on the caller's stream.
    const bool forked = tune.overlap && !ix->prof_serial && !exact && P.n_gq > 0 && !P.ib.items.empty();
    // Two device blobs alternate.  When the call forks, its blob is uploaded on the side stream: there it
    // follows the previous call's scan, not the previous call's beam search, so the upload is off the
    // critical path.  The buffer was last read two calls ago, by kernels on the side stream (which precede the
    // upload there) and on the caller's stream: those precede the fork event of the previous call, which the
    // side stream has waited for -- if that call forked; if not, the upload first waits for the caller's stream.
    // A small blob (small batches) is not copied at all: the kernels read the few hundred bytes they need
    // straight from the pinned staging buffer, which saves the copy's submission and its latency; the
    // staging buffer then stays untouched until the call's last kernel has ended.
    const bool zero_copy = tune.zero_copy_bytes > 0 && L.total <= (size_t)tune.zero_copy_bytes;
    const int bsel = W->blob_next;
    DevBuf &blob = bsel ? W->ws_blob_b : W->ws_blob;
    CallMem M;
    if (zero_copy) {
        void *dev_view = nullptr;
        VF_HIP(hipHostGetDevicePointer(&dev_view, st->p, 0));
        M.blob = (char *)dev_view;
    } else {
        W->blob_next ^= 1;
        if ((rc = blob.reserve(L.total)) != VF_OK) return rc;
        M.blob = blob.as<char>();
        hipStream_t cs = forked ? W->side : s;
        if (forked && !W->prev_forked) {
            VF_HIP(hipEventRecord(W->ev_fork, s));
            VF_HIP(hipStreamWaitEvent(cs, W->ev_fork, 0));
        }
        VF_HIP(hipMemcpyAsync(M.blob, hp, L.total, hipMemcpyHostToDevice, cs));
        VF_HIP(hipEventRecord(st->done, cs));
        st->pending = true;
        if (forked) VF_HIP(hipStreamWaitEvent(s, st->done, 0));
    }
    W->prev_forked = forked;
    M.dseed = W->dseed.as<uint32_t>();
    M.part_idx = W->part_idx.as<int32_t>();
    M.part_bits = W->part_bits.as<uint32_t>();
    if ((rc = launch_call(ix, P, r, M, sc, queries, out_ids, out_dists, s, forked ? W->side : nullptr, W->ev_fork,
                          W->ev_join, true)) != VF_OK)
        return rc;
    if (zero_copy) {
        VF_HIP(hipEventRecord(st->done, s));
        st->pending = true;
    }
    VF_HIP(hipGetLastError());
    if (ix->profiling) {
        const auto t_end = std::chrono::steady_clock::now();
        auto ms = [](auto a, auto b) { return std::chrono::duration<double, std::milli>(b - a).count(); };
        ix->prof_host_plan += ms(t_enter, t_planned);
        ix->prof_host_wait += ms(t_planned, t_staged);
        ix->prof_host_blob += ms(t_staged, t_blob);
        ix->prof_host_launch += ms(t_blob, t_end);
    }
    if (exact) {
        VF_HIP(hipStreamSynchronize(s));
        ix->tmp_blk.release();
        ix->tmp_norm.release();
    }
    return VF_OK;
}

// OR queries (Section 4.3.1) and the parallel AND policy (end of Section 4.3.2): every query becomes
// one search per label, the searches run as one ordinary batch, and a merge kernel combines them.
int search_multi_impl(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids, int32_t mode,
                      int32_t k, int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds, int64_t *out_ids,
                      float *out_dists, hipStream_t s)
{
    const bool exact = (mode & VF_MULTI_EXACT) != 0;
    mode &= ~VF_MULTI_EXACT;
    VF_REQUIRE(mode == VF_AND_GREEDY || mode == VF_AND_PARALLEL || mode == VF_OR, "mode must be VF_AND_GREEDY, VF_AND_PARALLEL or VF_OR");
    if (mode == VF_AND_GREEDY)
        return search_impl(ix, queries, nq, qoff, qids, k, itopk, width, iters, n_seeds, exact, out_ids, out_dists, s, false);
    int rc = check_search_args(ix, queries, nq, k, out_ids, out_dists);
    if (rc != VF_OK) return rc;
    VF_REQUIRE(qoff && qids, "NULL query label arrays");
    if (nq == 0) return VF_OK;
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    Workspace *W = nullptr;
    if ((rc = workspace_for(ix, s, &W)) != VF_OK) return rc;
    {
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
    }
    return VF_OK;
}

}  // namespace vf
