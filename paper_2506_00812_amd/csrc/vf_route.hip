// Host-only part of a search call: ClassifyQueries of Alg. 2 (graph or scan by the size of the list against
// T, Section 4.1.2), the smallest-list choice of Section 4.3.2, the grouping of the batch by searched label and
// the work list of the scan path.  No device call is made here, so all of it can be exercised without a GPU
// (vf_debug_route).  Also here: the tuning switches and the thread-local error text.
#include "vf_host.h"

namespace vf {

static thread_local std::string g_err;

void set_error(const std::string &msg)
{
    try {
        g_err = msg;
    } catch (...) {
        g_err.clear();
    }
}

const char *last_error() { return g_err.c_str(); }

Tuning &default_tuning()
{
    static Tuning t;
    return t;
}

std::mutex &default_tuning_mutex()
{
    static std::mutex m;
    return m;
}

bool Tuning::set(const char *name, double value)
{
    if (!name || !(value == value)) return false;
    struct IntKnob { const char *name; int Tuning::*field; int lo, hi; };
    static const IntKnob knobs[] = {
        {"seg_groups", &Tuning::seg_groups, 1, 4096},
        {"seg_groups_heavy", &Tuning::seg_groups_heavy, 1, 4096},
        {"heavy_rows", &Tuning::heavy_rows, 1, 33},
        {"tile_rows", &Tuning::tile_rows, 1, 32},
        {"zero_copy_bytes", &Tuning::zero_copy_bytes, 0, 1 << 20},
        {"scan_valu", &Tuning::scan_valu, 0, 2},
        {"scan16", &Tuning::scan16, 0, 1},
        {"scan_bf16", &Tuning::scan_bf16, 0, 1},
        {"scan_bf16_margin", &Tuning::scan_bf16_margin, 0, 54},
        {"scan_bf16_slots", &Tuning::scan_bf16_slots, 1, 2},
        {"scan_bf16_seg_groups", &Tuning::scan_bf16_seg_groups, 1, 1024},
        {"beam_lat_waves", &Tuning::beam_lat_waves, 0, 1 << 20},
        {"overlap", &Tuning::overlap, 0, 1},
        {"seed_exact", &Tuning::seed_exact, 0, 1},
        {"seed_margin", &Tuning::seed_margin, 1, 32},
        {"seed_margin_bf16", &Tuning::seed_margin_bf16, 1, 32},
        {"seed_cache", &Tuning::seed_cache, 0, 1},
        {"seed_bf16", &Tuning::seed_bf16, 0, 1},
        {"seed_bf16_min_batch", &Tuning::seed_bf16_min_batch, 0, 1 << 30},
        {"seed_fb_window", &Tuning::seed_fb_window, 1, 1 << 30},
        {"seed_select", &Tuning::seed_select, 0, 1},
        {"seed_seg_seeds", &Tuning::seed_seg_seeds, 0, 1 << 20},
        {"build16", &Tuning::build16, 0, 1},
        {"build_panel_kb", &Tuning::build_panel_kb, 1, 1 << 22},
        {"build_progress", &Tuning::build_progress, 0, 1},
    };
    if (strcmp(name, "seed_slack") == 0) {
        if (!(value > 0.0 && value <= 1e30)) return false;
        seed_slack = value;
        return true;
    }
    for (const IntKnob &k : knobs) {
        if (strcmp(name, k.name) != 0) continue;
        if (value < (double)k.lo || value > (double)k.hi || value != (double)(int)value) return false;
        this->*(k.field) = (int)value;
        return true;
    }
    return false;
}

// Queries are grouped by the label they search with a counting sort: O(nq + labels touched), no comparison
// sort of the batch.
int route_queries(const RouteView &ix, int64_t nq, const int64_t *qoff, const int32_t *qids, bool all_scan,
                  bool first_is_searched, Routed &r)
{
    VF_REQUIRE(qoff && qids, "NULL query label arrays");
    VF_REQUIRE(qoff[0] >= 0, "qlabel_offsets[0] must be >= 0");
    r.others_off.assign((size_t)nq + 1, 0);
    r.others.clear();
    r.any_and = false;
    r.empty_q.clear();
    r.q_best.resize((size_t)nq);
    if (r.cnt.size() != (size_t)ix.n_labels) r.cnt.assign((size_t)ix.n_labels, 0);
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
            VF_REQUIRE(l >= 0 && l < ix.n_labels, "query label outside [0, n_labels)");
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
            const int32_t sl = ix.S[l], sb = ix.S[best];
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
        const bool graph = !all_scan && ix.S[l] >= ix.T;
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

void ItemBuilder::add_label(const std::vector<uint64_t> &pairs, size_t lo, size_t hi, int64_t group0, int64_t map_off,
                            int32_t n)
{
    const int32_t n_groups = (n + 31) / 32;
    for (size_t t = lo; t < hi; t += (size_t)tile_rows) {
        const int32_t q_begin = (int32_t)qrow.size();
        const int32_t q_count = (int32_t)std::min<size_t>((size_t)tile_rows, hi - t);
        // a tile's work item is a serial chain whose cost per group grows with its queries (selection):
        // tiles with many queries may get shorter segments, so that the items of a launch end together
        const int32_t want = q_count >= heavy_rows ? seg_groups_heavy : seg_groups;
        const int32_t sg_len = std::max(want, (n_groups + kMaxSegs - 1) / kMaxSegs);
        const int32_t nseg = (n_groups + sg_len - 1) / sg_len;
        max_nseg = std::max(max_nseg, nseg);
        for (size_t u = t; u < t + (size_t)q_count; ++u) qrow.push_back((int32_t)(uint32_t)pairs[u]);
        for (int32_t sg = 0; sg < nseg; ++sg) {
            ScanItem it{};
            it.group0 = group0 + (int64_t)sg * sg_len;
            it.map_off = map_off;
            it.entry0 = sg * sg_len * 32;
            it.n = std::min(sg_len * 32, n - it.entry0);
            it.q_begin = q_begin; it.q_count = q_count; it.self_base = -1;
            it.part_row = (nseg == 1 && !all_partial) ? -1 : (int32_t)(part_rows + (int64_t)sg * q_count);
            items.push_back(it);
        }
        if (nseg > 1 || all_partial) {
            for (int32_t r = 0; r < q_count; ++r)
                merges.push_back(MergeItem{map_off, qrow[(size_t)q_begin + r], (int32_t)(part_rows + r), q_count, nseg, n, 0});
            part_rows += (int64_t)nseg * q_count;
        }
    }
}

}  // namespace vf

using namespace vf;

extern "C" const char *vf_last_error(void) { return vf::last_error(); }

extern "C" int vf_debug_route(const int32_t *S, int32_t n_labels, int32_t T, int64_t nq, const int64_t *qoff,
                              const int32_t *qids, int32_t tile_rows, int32_t seg_groups, int32_t *searched,
                              int32_t *method, int32_t *n_others, int64_t *items_out, int64_t items_cap,
                              int64_t *merges_out, int64_t merges_cap, int32_t *qrow_out, int64_t *counts)
{
    return guarded([&]() -> int {
        VF_REQUIRE(S && n_labels > 0 && T > 0 && nq >= 0 && searched && method && n_others && counts, "bad argument");
        VF_REQUIRE(nq < ((int64_t)1 << 31), "nq out of range");
        Tuning tune;
        VF_REQUIRE(tune.set("tile_rows", tile_rows) && tune.set("seg_groups", seg_groups) &&
                       tune.set("seg_groups_heavy", seg_groups),
                   "tile_rows or seg_groups out of range");
        Routed r;
        const RouteView view{S, n_labels, T};
        int rc = route_queries(view, nq, qoff, qids, false, false, r);
        if (rc != VF_OK) return rc;
        // offsets of the scan partition as the index build lays them out (ascending label id)
        std::vector<int64_t> O_LS((size_t)n_labels, -1), GO_LS((size_t)n_labels, -1);
        int64_t n_LS = 0, n_groups = 0;
        for (int32_t l = 0; l < n_labels; ++l)
            if (S[l] > 0 && S[l] < T) {
                O_LS[(size_t)l] = n_LS; n_LS += S[l];
                GO_LS[(size_t)l] = n_groups; n_groups += (S[l] + 31) / 32;
            }
        for (int64_t j = 0; j < nq; ++j) {
            const int32_t l = r.q_best[(size_t)j];
            searched[j] = l;
            method[j] = l < 0 ? 0 : (S[l] >= T ? 2 : 1);
            n_others[j] = r.others_off[(size_t)j + 1] - r.others_off[(size_t)j];
        }
        ItemBuilder ib(tune);
        for (size_t i = 0; i < r.scan_pairs.size();) {
            const int32_t l = (int32_t)(r.scan_pairs[i] >> 32);
            size_t e = i;
            while (e < r.scan_pairs.size() && (int32_t)(r.scan_pairs[e] >> 32) == l) ++e;
            ib.add_label(r.scan_pairs, i, e, GO_LS[(size_t)l], O_LS[(size_t)l], S[l]);
            i = e;
        }
        counts[0] = (int64_t)r.gq_query.size();
        counts[1] = (int64_t)ib.qrow.size();
        counts[2] = (int64_t)ib.items.size();
        counts[3] = (int64_t)ib.merges.size();
        counts[4] = ib.part_rows;
        counts[5] = ib.max_nseg;
        VF_REQUIRE((items_out == nullptr || (int64_t)ib.items.size() <= items_cap) &&
                       (merges_out == nullptr || (int64_t)ib.merges.size() <= merges_cap),
                   "output arrays too small (the counts are set)");
        if (items_out)
            for (size_t i = 0; i < ib.items.size(); ++i) {
                const ScanItem &it = ib.items[i];
                int64_t *o = items_out + i * 8;
                o[0] = it.group0; o[1] = it.map_off; o[2] = it.entry0; o[3] = it.n; o[4] = it.q_begin; o[5] = it.q_count;
                o[6] = it.self_base; o[7] = it.part_row;
            }
        if (merges_out)
            for (size_t i = 0; i < ib.merges.size(); ++i) {
                const MergeItem &m = ib.merges[i];
                int64_t *o = merges_out + i * 5;
                o[0] = m.map_off; o[1] = m.qrow; o[2] = m.part_row; o[3] = m.stride; o[4] = m.nseg;
            }
        if (qrow_out && !ib.qrow.empty()) memcpy(qrow_out, ib.qrow.data(), ib.qrow.size() * 4);
        // graph queries follow the scan tile rows in qrow_out: grouped by label, stable in query order
        if (qrow_out && !r.gq_query.empty()) memcpy(qrow_out + ib.qrow.size(), r.gq_query.data(), r.gq_query.size() * 4);
        return VF_OK;
    });
}
