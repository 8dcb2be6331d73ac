// Queue-driven serving of small batches (Section 4.2.3): one kernel stays resident for a whole session and pulls
// single queries from a job queue, so a query costs neither a kernel launch nor a host-side synchronisation.
//
// Shape on this machine.  The host writes a job (query vector + labels) into a ring in pinned host memory and
// bumps a counter.  Workgroup 0 of the resident kernel is the DISPATCHER: it alone polls that counter across
// PCIe, copies new jobs into a ring in device memory and publishes them by advancing a device-side tail.  The
// other workgroups are WORKERS (one query at a time, as in the paper's one block per query; NW waves each: all of
// them score a share of the query's seeds, then the first wave searches while the others wait at the workgroup's
// barrier): a worker claims the next job with a compare-and-swap on the device-side head -- the atomic ring buffer of
// the paper's figure; "which worker is free" needs no queue of its own, a free worker is one that is polling --
// routes it (smallest list, graph or scan by T, Section 4.1.2 / 4.3.2), runs the same beam search or list
// scan the batched kernels run (the device functions are shared), writes the k results straight into the
// result ring in host memory and releases a per-job done flag there.
//
// Every wave exits on its own.  The dispatcher leaves when the host asks it to, when max_jobs jobs have been
// published, or after idle_polls consecutive polls without a new job; leaving, it raises the device-side stop
// flag.  A worker leaves when it sees that flag and the queue is drained, and in any case after
// 16 * idle_polls consecutive empty polls.  So a session that is never ended ends by itself, and
// vf_serve_end always returns.
#include <atomic>
#include <chrono>

#include "vf_beam.h"
#include "vf_host.h"
#include "vf_scan_item.h"

namespace vf {

constexpr int kServeHdr = 64;   // bytes of a job slot before the query vector

struct ServeJobHdr {            // first kServeHdr bytes of a job slot (host ring and device ring)
    int32_t n_labels;
    int32_t labels[kMaxOthers + 1];
    int32_t pad[7];
};
static_assert(sizeof(ServeJobHdr) == kServeHdr, "job header size");

struct ServeResult {            // one slot of the result ring (pinned host memory)
    uint64_t done;              // job id + 1 once ids / dists of that job are complete
    int64_t ids[64];
    float dists[64];
};

struct ServeHostCtrl {          // pinned host memory, both sides read and write
    uint64_t tail;              // host: jobs submitted so far
    uint32_t stop;              // host: 1 = end the session
    uint32_t pad0;
    uint64_t published;         // device: jobs copied to the device ring (their host slots may be reused)
    uint64_t jobs_done;         // device: jobs completed (written at exit)
    uint32_t exit_reason;       // device: 0 while running; 1 host asked, 2 max_jobs reached, 3 idle bound
    uint32_t pad1;
};

struct ServeDevCtrl {           // device memory
    uint64_t head;              // next job to claim
    uint64_t tail;              // jobs published
    uint32_t stop;
    uint32_t pad;
    uint64_t jobs_done;
};

struct ServeParams {
    BeamParams bp;              // static part: tables, dim, R, k, itopk, width, iters, n_seeds, LP, hash_bits
    ScanParams sp;              // static part: scan lists, norms, map, dim, ncp, K, tile_rows, meta
    const int64_t *GO_LS;       // [n_labels] first 32-vector group of a scan list
    int32_t T, n_labels;
    int32_t ring_slots, slot_stride, row_bytes;
    const char *host_ring;      // device view of the pinned job ring
    char *dev_ring;
    ServeResult *results;       // device view of the pinned result ring
    ServeHostCtrl *hctrl;       // device view
    ServeDevCtrl *dctrl;
    int64_t max_jobs, idle_polls;
    int32_t lds_kernels;        // bytes of LDS the search functions use; the worker's own words follow (lds_own bytes)
    int32_t lds_own;
};

template <class T> __device__ __forceinline__ T load_sys(const T *p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM); }
template <class T> __device__ __forceinline__ T load_dev(const T *p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT); }

// DT: 0 uint8, 1 float32.  NC: compile-time chunk count of the scan function (chunk pairs for scan_topk_item,
// chunks for scan_valu_item), 0 = generic.
template <int DT, int NC, int NW>
__global__ __launch_bounds__(64 * NW) void serve_kernel(ServeParams p)
{
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;

    if (blockIdx.x == 0) {
        // ---------------- dispatcher (the first wave; it never meets a workgroup barrier)
        if (wv != 0) return;
        uint64_t published = 0;
        int64_t idle = 0;
        uint32_t reason = 0;
        while (reason == 0) {
            const uint64_t t = load_sys(&p.hctrl->tail);
            const uint32_t stop = load_sys(&p.hctrl->stop);
            uint64_t upto = t;
            if ((int64_t)upto > p.max_jobs) upto = (uint64_t)p.max_jobs;
            if (upto > published) {
                for (uint64_t j = published; j < upto; ++j) {   // at most ring_slots jobs: the host waits for `published`
                    const size_t off = (size_t)(j % (uint64_t)p.ring_slots) * (size_t)p.slot_stride;
                    const uint4 *src = (const uint4 *)(p.host_ring + off);
                    uint4 *dst = (uint4 *)(p.dev_ring + off);
                    for (int i = lane; i < p.slot_stride / 16; i += 64) dst[i] = src[i];
                }
                __threadfence();
                published = upto;
                if (lane == 0) {
                    __hip_atomic_store(&p.dctrl->tail, published, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&p.hctrl->published, published, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
                }
                idle = 0;
            } else {
                ++idle;
                __builtin_amdgcn_s_sleep(32);
            }
            if (stop != 0) reason = 1;
            else if ((int64_t)published >= p.max_jobs) reason = 2;
            else if (idle > p.idle_polls) reason = 3;
        }
        if (lane == 0) __hip_atomic_store(&p.dctrl->stop, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        // the session's exit record is complete once every published job is done: bounded wait for the workers
        int64_t spins = 0;
        while (load_dev(&p.dctrl->jobs_done) < published && spins < 16 * p.idle_polls + 1024) { ++spins; __builtin_amdgcn_s_sleep(32); }
        if (lane == 0) {
            p.hctrl->jobs_done = load_dev(&p.dctrl->jobs_done);
            __hip_atomic_store(&p.hctrl->exit_reason, reason, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        return;
    }

    // ---------------- worker
    // Every wave of the workgroup passes the same four barriers per job.  LDS: the search functions' area (first
    // wave), then [0..7] others, [8..9] others_off, [10] qrow, [11..12] job, [16..] the query (FMA scan only), then
    // per wave a copy of the query and a run of 64 seed keys.
    int32_t *own = (int32_t *)((char *)smem + p.lds_kernels);
    char *share = (char *)smem + p.lds_kernels + p.lds_own;
    const int q_bytes = (p.row_bytes + 15) & ~15;
    uint4 *hq = (uint4 *)(share + (size_t)wv * q_bytes);                         // this wave's copy of the query
    uint64_t *runs = (uint64_t *)(share + (size_t)NW * q_bytes);                 // [NW][64]
    int64_t idle = 0;
    while (true) {
        if (wv == 0 && lane == 0) {
            int64_t job = -1;
            while (true) {
                const uint64_t h = load_dev(&p.dctrl->head), t = load_dev(&p.dctrl->tail);
                if (h < t) {
                    uint64_t expect = h;
                    if (__hip_atomic_compare_exchange_strong(&p.dctrl->head, &expect, h + 1, __ATOMIC_ACQ_REL, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT)) { job = (int64_t)h; break; }
                    continue;   // another worker took it: look again (progress: the head moved)
                }
                if (load_dev(&p.dctrl->stop) != 0) break;      // drained and stopping
                if (++idle > 16 * p.idle_polls) break;          // nothing for very long: the dispatcher must be gone
                __builtin_amdgcn_s_sleep(32);
            }
            idle = 0;
            own[11] = (int32_t)(job & 0xFFFFFFFFll);
            own[12] = (int32_t)(job >> 32);
        }
        __syncthreads();
        const int64_t job = ((int64_t)own[12] << 32) | (uint32_t)own[11];
        if (job < 0) return;   // (the whole workgroup: every wave reads the same word)
        // an acquire by every lane: the job's slot may sit in this CU's cache from an earlier trip round the ring
        (void)load_dev(&p.dctrl->tail);
        const size_t soff = (size_t)((uint64_t)job % (uint64_t)p.ring_slots);
        const char *slot = p.dev_ring + soff * (size_t)p.slot_stride;
        const ServeJobHdr *hdr = (const ServeJobHdr *)slot;
        const void *qvec = slot + kServeHdr;
        ServeResult *res = p.results + soff;

        // route (ClassifyQueries of Alg. 2, smallest list of Section 4.3.2): every lane computes the same
        // (the slot is rewritten while this kernel runs: its header is read with coherent loads, never through
        // the scalar cache, which nothing invalidates inside a kernel)
        int nl = 0;
        int32_t labs[kMaxOthers + 1];
        const int n_hdr = __hip_atomic_load(&hdr->n_labels, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int n_in = n_hdr < kMaxOthers + 1 ? n_hdr : kMaxOthers + 1;
        for (int i = 0; i < n_in; ++i) {
            const int32_t l = __hip_atomic_load(&hdr->labels[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool seen = l < 0 || l >= p.n_labels;   // (the host has checked the range; never trust a ring)
            for (int u = 0; u < nl; ++u) seen = seen || labs[u] == l;
            if (!seen) labs[nl++] = l;
        }
        int32_t best = nl > 0 ? labs[0] : -1;
        bool empty = nl == 0;
        for (int i = 0; i < nl; ++i) {
            const int32_t sl = p.bp.meta.S[labs[i]], sb = p.bp.meta.S[best];
            if (sl == 0) empty = true;
            if (sl < sb || (sl == sb && labs[i] < best)) best = labs[i];
        }
        int o_cnt = 0;
        if (wv == 0 && lane == 0) {
            for (int i = 0; i < nl; ++i)
                if (labs[i] != best) own[o_cnt++] = labs[i];
            own[8] = 0; own[9] = o_cnt; own[10] = 0;
        }
        o_cnt = nl > 0 ? nl - 1 : 0;
        __syncthreads();

        const int k = p.bp.k;
        const bool graph = !empty && p.bp.meta.S[best] >= p.T;
        // the seeds of a graph job are shared out over the workgroup's waves: each scores its share from the
        // interleaved seed copy into a list of its own and leaves that list as a sorted run of keys
        const bool shared_seeds = graph && p.bp.sblk != nullptr;
        int seg = 64;
        if (shared_seeds) {
            const int n = p.bp.meta.S[best];
            const int ns = p.bp.n_seeds < n ? p.bp.n_seeds : n;
            const int nchunks = p.row_bytes / kChunkBytes;
            seg = (((ns + NW - 1) / NW) + 63) & ~63;
            const int j_lo = wv * seg, j_hi = j_lo + seg < ns ? j_lo + seg : ns;
            for (int i = lane; i < nchunks; i += 64) hq[i] = ((const uint4 *)qvec)[i];
            wave_sync<true>();
            TopM<1> part;
            part.init(p.bp.itopk);
            if (j_lo < j_hi) stream_seed_segment<DT>(p.bp, best, own, o_cnt, hq, nchunks, j_lo, j_hi, true, part, lane);
            const uint64_t key = part.cur[0];   // (distance bits << 32 | seed index << 1 | 1), ascending
            runs[wv * 64 + lane] = key == KEY_MAX ? KEY_MAX : (key & 0xFFFFFFFF00000000ull) | ((key >> 1) & 0x7FFFFFFFull);
        }
        __syncthreads();

        if (wv == 0) {
            if (empty) {
                if (lane < k) { res->ids[lane] = -1; res->dists[lane] = __builtin_inff(); }
            } else if (graph) {
                BeamQuery bq;
                bq.q = qvec; bq.label = best; bq.others = own; bq.o_cnt = o_cnt;
                bq.out_ids = res->ids; bq.out_dists = res->dists;
                bq.counters = nullptr; bq.gathered = nullptr; bq.dseed_row = nullptr; bq.runs = nullptr; bq.seed_pass = -1;
                BeamParams bp = p.bp;
                if (shared_seeds) {   // the waves' runs, merged by the search as the runs of a selecting seed kernel would be
                    bq.runs = runs;
                    bp.run_K = 64; bp.run_segs = NW; bp.seg_seeds = seg; bp.seed_approx = 0;
                }
                beam_search_wave<DT, 1, true>(bp, bq, smem);
            } else {
                ScanParams sp = p.sp;
                sp.qsrc = qvec; sp.qrow = own + 10;
                sp.others_off = o_cnt > 0 ? own + 8 : nullptr; sp.others = own;
                sp.out_ids = res->ids; sp.out_dists = res->dists;
                ScanItem it;
                it.group0 = p.GO_LS[best]; it.map_off = p.bp.meta.O_LS[best]; it.entry0 = 0; it.n = p.bp.meta.S[best];
                it.q_begin = 0; it.q_count = 1; it.self_base = -1; it.part_row = -1;
                if constexpr (DT == 1 && (NC == 24 || NC == 32)) {
                    // the FMA scan takes its query as a wave-uniform operand: from LDS here (see scan_valu_item)
                    float *q_lds = (float *)(own + 16);
                    for (int i = lane; i < NC; i += 64) ((uint4 *)q_lds)[i] = ((const uint4 *)qvec)[i];
                    wave_sync<true>();
                    scan_valu_item<NC, true>(sp, it, smem, q_lds);
                } else {
                    scan_topk_item<DT, NC, true>(sp, it, smem);
                }
            }
            wave_sync<true>();
            __threadfence_system();
            if (lane == 0) {
                __hip_atomic_store(&res->done, (uint64_t)job + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_fetch_add(&p.dctrl->jobs_done, (uint64_t)1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
    }
}

}  // namespace vf

using namespace vf;

struct vf_server {
    vf_index *ix = nullptr;
    hipStream_t stream = nullptr;
    char *h_ring = nullptr;               // pinned
    ServeResult *h_results = nullptr;     // pinned
    ServeHostCtrl *h_ctrl = nullptr;      // pinned
    DevBuf d_ring, d_ctrl, d_GO_LS;
    SeedCopy seeds;                       // the session's own interleaved copy of the seeds (workers score from it)
    int32_t ring_slots = 0, slot_stride = 0, row_bytes = 0, k = 0;
    int64_t max_jobs = 0;
    uint64_t next_job = 0;
    bool launched = false;
    std::mutex mu;
};

static void free_server(vf_server *sv)
{
    if (!sv) return;
    if (sv->stream) { (void)hipStreamSynchronize(sv->stream); (void)hipStreamDestroy(sv->stream); }
    sv->d_ring.release(); sv->d_ctrl.release(); sv->d_GO_LS.release();
    for (DevBuf *b : sv->seeds.bufs()) b->release();
    if (sv->h_ring) (void)hipHostFree(sv->h_ring);
    if (sv->h_results) (void)hipHostFree(sv->h_results);
    if (sv->h_ctrl) (void)hipHostFree(sv->h_ctrl);
    delete sv;
}

template <int DT, int NC> static void launch_serve(const ServeParams &p, int n_workers, int waves, size_t lds, hipStream_t s)
{
    const dim3 grid(1 + n_workers);
    if (waves == 1) hipLaunchKernelGGL((serve_kernel<DT, NC, 1>), grid, dim3(64), lds, s, p);
    else if (waves == 4) hipLaunchKernelGGL((serve_kernel<DT, NC, 4>), grid, dim3(256), lds, s, p);
    else hipLaunchKernelGGL((serve_kernel<DT, NC, 8>), grid, dim3(512), lds, s, p);
}

static int serve_begin_impl(vf_index *ix, const vf_serve_params *prm, vf_server **out)
{
    VF_REQUIRE(out != nullptr, "out is NULL");
    *out = nullptr;
    VF_REQUIRE(ix != nullptr && prm != nullptr, "NULL argument");
    int32_t k = prm->k, itopk = prm->itopk, width = prm->width, iters = prm->iters, n_seeds = prm->n_seeds;
    VF_REQUIRE(k >= 1 && k <= 64, "k must be in [1, 64]");
    int rc = check_search_params(ix, false, k, itopk, width, iters, n_seeds);
    if (rc != VF_OK) return rc;
    VF_REQUIRE(itopk <= 64, "vf_serve_begin: itopk must be at most 64");
    const int32_t n_workers = prm->n_workers > 0 ? prm->n_workers : 240;
    const int32_t waves = prm->waves_per_worker > 0 ? prm->waves_per_worker : 8;
    VF_REQUIRE(waves == 1 || waves == 4 || waves == 8, "waves_per_worker must be 1, 4 or 8 (0 = 8)");
    const int32_t ring_slots = prm->ring_slots > 0 ? prm->ring_slots : 1024;
    // every workgroup must be resident at once (a CU takes several)
    VF_REQUIRE(n_workers >= 1 && n_workers <= 1023, "n_workers must be in [1, 1023]");
    VF_REQUIRE(ring_slots >= 1 && ring_slots <= (1 << 20), "ring_slots must be in [1, 2^20]");
    const int64_t max_jobs = prm->max_jobs > 0 ? prm->max_jobs : ((int64_t)1 << 62);
    const int64_t idle_polls = prm->idle_polls > 0 ? prm->idle_polls : 2000000;
    VF_REQUIRE(idle_polls <= ((int64_t)1 << 32), "idle_polls must be at most 2^32");

    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    vf_server *sv = new vf_server();
    struct Guard { vf_server *sv; ~Guard() { if (sv) free_server(sv); } } guard{sv};
    sv->ix = ix; sv->k = k; sv->ring_slots = ring_slots; sv->max_jobs = max_jobs;
    sv->row_bytes = (int32_t)((size_t)ix->dim * ix->elem());
    sv->slot_stride = kServeHdr + ((sv->row_bytes + 63) & ~63);
    sv->d_ring.al = sv->d_ctrl.al = sv->d_GO_LS.al = &ix->alloc;
    for (DevBuf *b : sv->seeds.bufs()) b->al = &ix->alloc;
    const size_t ring_bytes = (size_t)ring_slots * sv->slot_stride;
    const unsigned flags = hipHostMallocMapped | hipHostMallocCoherent;
    VF_HIP(hipHostMalloc((void **)&sv->h_ring, ring_bytes, flags));
    VF_HIP(hipHostMalloc((void **)&sv->h_results, (size_t)ring_slots * sizeof(ServeResult), flags));
    VF_HIP(hipHostMalloc((void **)&sv->h_ctrl, sizeof(ServeHostCtrl), flags));
    memset(sv->h_ring, 0, ring_bytes);
    memset(sv->h_results, 0, (size_t)ring_slots * sizeof(ServeResult));
    memset(sv->h_ctrl, 0, sizeof(ServeHostCtrl));
    VF_HIP(hipStreamCreateWithFlags(&sv->stream, hipStreamNonBlocking));
    if ((rc = sv->d_ring.reserve(ring_bytes)) != VF_OK) return rc;
    if ((rc = sv->d_ctrl.reserve(sizeof(ServeDevCtrl))) != VF_OK) return rc;
    if ((rc = upload(sv->d_GO_LS, ix->GO_LS, sv->stream)) != VF_OK) return rc;
    VF_HIP(hipMemsetAsync(sv->d_ctrl.p, 0, sizeof(ServeDevCtrl), sv->stream));
    VF_HIP(hipStreamSynchronize(sv->stream));
    // the seeds of every graph list, interleaved, in the data's own type (exact distances): a worker streams its
    // query's seeds from it, one seed per lane.  The session owns the copy (the index's copies may be dropped
    // while the kernel runs).  When it does not fit, workers gather the seeds' rows from the vector table.
    if (!ix->graph_labels.empty() && (rc = build_seed_copy(ix, n_seeds, sv->stream, false, &sv->seeds)) != VF_OK) return rc;

    ServeParams p{};
    // beam search: geometry as vf_search computes it
    int32_t LP = 128, hb = 9;
    while (LP < itopk + std::max(64, width * ix->R)) LP <<= 1;
    const int64_t visits = (int64_t)iters * width * ix->R;
    while (hb < 13 && ((int64_t)1 << hb) < 2 * visits) ++hb;
    p.bp.X = ix->X; p.bp.G = ix->d_G.as<int32_t>(); p.bp.Gg = ix->d_Gg.as<int32_t>(); p.bp.meta = ix->meta();
    p.bp.dim = ix->dim; p.bp.R = ix->R; p.bp.k = k; p.bp.itopk = itopk; p.bp.width = width; p.bp.iters = iters;
    p.bp.n_seeds = n_seeds; p.bp.LP = LP; p.bp.hash_bits = hb;
    if (sv->seeds.ok && sv->seeds.has_f32) {
        p.bp.sblk = sv->seeds.blk.as<uint4>(); p.bp.sgoff = sv->seeds.goff.as<int64_t>(); p.bp.sblk_chunks = 2 * ix->ncp;
    }
    const size_t beam_lds = beam_lds_bytes(p.bp, ix->dtype);
    // scan: one query against a whole list
    p.sp.xblk = ix->d_X_LS.as<uint4>(); p.sp.xnorm = ix->d_xnorm_LS.p; p.sp.map = ix->d_M_LS.as<int32_t>();
    p.sp.dim = ix->dim; p.sp.ncp = ix->ncp; p.sp.K = k; p.sp.tile_rows = 16; p.sp.meta = ix->meta();
    const bool valu = scan_valu_supported(ix->dtype, ix->dim, 16);
    const size_t scan_lds = valu ? (size_t)16 * (96 + (k | 1)) * 8 + 2 * 32 * 4 : scan_lds_bytes(ix->ncp, 16, k);
    const size_t lds_kernels = (std::max(beam_lds, scan_lds) + 63) & ~(size_t)63;
    const size_t lds_own = (64 + (valu ? (size_t)sv->row_bytes : 0) + 63) & ~(size_t)63;
    // per wave a copy of the query and a run of 64 seed keys
    const size_t lds_share = (size_t)waves * ((((size_t)sv->row_bytes + 15) & ~(size_t)15) + 64 * 8);
    VF_REQUIRE(lds_kernels + lds_own + lds_share <= 64 * 1024, "search parameters need more than 64 KiB of LDS");
    p.GO_LS = sv->d_GO_LS.as<int64_t>(); p.T = ix->T; p.n_labels = ix->n_labels;
    p.ring_slots = ring_slots; p.slot_stride = sv->slot_stride; p.row_bytes = sv->row_bytes;
    void *dv = nullptr;
    VF_HIP(hipHostGetDevicePointer(&dv, sv->h_ring, 0)); p.host_ring = (const char *)dv;
    VF_HIP(hipHostGetDevicePointer(&dv, sv->h_results, 0)); p.results = (ServeResult *)dv;
    VF_HIP(hipHostGetDevicePointer(&dv, sv->h_ctrl, 0)); p.hctrl = (ServeHostCtrl *)dv;
    p.dev_ring = sv->d_ring.as<char>(); p.dctrl = sv->d_ctrl.as<ServeDevCtrl>();
    p.max_jobs = max_jobs; p.idle_polls = idle_polls; p.lds_kernels = (int32_t)lds_kernels; p.lds_own = (int32_t)lds_own;
    const size_t lds = lds_kernels + lds_own + lds_share;
    if (ix->dtype == VF_U8) {
        if (ix->dim == 128) launch_serve<0, 4>(p, n_workers, waves, lds, sv->stream);
        else if (ix->dim == 192) launch_serve<0, 6>(p, n_workers, waves, lds, sv->stream);
        else launch_serve<0, 0>(p, n_workers, waves, lds, sv->stream);
    } else {
        if (ix->dim == 128) launch_serve<1, 32>(p, n_workers, waves, lds, sv->stream);
        else if (ix->dim == 96) launch_serve<1, 24>(p, n_workers, waves, lds, sv->stream);
        else launch_serve<1, 0>(p, n_workers, waves, lds, sv->stream);
    }
    VF_HIP(hipGetLastError());
    sv->launched = true;
    guard.sv = nullptr;
    *out = sv;
    return VF_OK;
}

static int serve_submit_impl(vf_server *sv, const void *query, const int32_t *labels, int32_t n_labels, int64_t *job)
{
    VF_REQUIRE(sv && query && labels && job, "NULL argument");
    VF_REQUIRE(n_labels >= 1 && n_labels <= kMaxOthers + 1, "a query needs 1 to 8 labels");
    for (int32_t i = 0; i < n_labels; ++i)
        VF_REQUIRE(labels[i] >= 0 && labels[i] < sv->ix->n_labels, "query label outside [0, n_labels)");
    std::lock_guard<std::mutex> lock(sv->mu);
    std::atomic_thread_fence(std::memory_order_acquire);
    VF_REQUIRE(__atomic_load_n(&sv->h_ctrl->exit_reason, __ATOMIC_ACQUIRE) == 0,
               "the serving kernel has ended (stop requested, max_jobs reached, or idle for too long): begin a new session");
    VF_REQUIRE((int64_t)sv->next_job < sv->max_jobs, "max_jobs of this session have been submitted");
    const uint64_t j = sv->next_job;
    if (j >= (uint64_t)sv->ring_slots) {
        // the slot's previous job must have left the host ring (copied to the device) and be done (its result slot is
        // about to be reused)
        const uint64_t prev = j - (uint64_t)sv->ring_slots;
        const uint64_t pub = __atomic_load_n(&sv->h_ctrl->published, __ATOMIC_ACQUIRE);
        const uint64_t done = __atomic_load_n(&sv->h_results[prev % (uint64_t)sv->ring_slots].done, __ATOMIC_ACQUIRE);
        if (pub <= prev || done < prev + 1) {
            set_error("the job ring is full");
            return VF_EBUSY;
        }
    }
    char *slot = sv->h_ring + (size_t)(j % (uint64_t)sv->ring_slots) * sv->slot_stride;
    ServeJobHdr hdr{};
    hdr.n_labels = n_labels;
    for (int32_t i = 0; i < n_labels; ++i) hdr.labels[i] = labels[i];
    memcpy(slot, &hdr, sizeof(hdr));
    memcpy(slot + kServeHdr, query, (size_t)sv->row_bytes);
    __atomic_store_n(&sv->h_ctrl->tail, j + 1, __ATOMIC_RELEASE);
    sv->next_job = j + 1;
    *job = (int64_t)j;
    return VF_OK;
}

static int serve_poll_impl(vf_server *sv, int64_t job, int64_t *out_ids, float *out_dists, int32_t *done)
{
    VF_REQUIRE(sv && done, "NULL argument");
    *done = 0;
    VF_REQUIRE(job >= 0 && (uint64_t)job < sv->next_job, "no such job");
    const ServeResult *res = sv->h_results + (size_t)((uint64_t)job % (uint64_t)sv->ring_slots);
    const uint64_t d = __atomic_load_n(&res->done, __ATOMIC_ACQUIRE);
    VF_REQUIRE(d <= (uint64_t)job + 1, "the job's result has been overwritten by a later job (the result ring wrapped)");
    if (d < (uint64_t)job + 1) {
        // not done: say so, unless the kernel has ended and never will be
        if (__atomic_load_n(&sv->h_ctrl->exit_reason, __ATOMIC_ACQUIRE) != 0 &&
            __atomic_load_n(&res->done, __ATOMIC_ACQUIRE) < (uint64_t)job + 1) {
            set_error("the serving kernel ended before this job was processed");
            return VF_EINVAL;
        }
        return VF_OK;
    }
    if (out_ids) memcpy(out_ids, res->ids, (size_t)sv->k * 8);
    if (out_dists) memcpy(out_dists, res->dists, (size_t)sv->k * 4);
    *done = 1;
    return VF_OK;
}

static int serve_end_impl(vf_server *sv, int64_t *jobs_done, int32_t *exit_reason)
{
    VF_REQUIRE(sv != nullptr, "server is NULL");
    {
        std::lock_guard<std::mutex> lock(sv->mu);
        __atomic_store_n(&sv->h_ctrl->stop, 1u, __ATOMIC_RELEASE);
    }
    VF_HIP(hipStreamSynchronize(sv->stream));   // every wave of the kernel exits by itself
    if (jobs_done) *jobs_done = (int64_t)__atomic_load_n(&sv->h_ctrl->jobs_done, __ATOMIC_ACQUIRE);
    if (exit_reason) *exit_reason = (int32_t)__atomic_load_n(&sv->h_ctrl->exit_reason, __ATOMIC_ACQUIRE);
    free_server(sv);
    return VF_OK;
}

// A host batch through the session: submit in order with at most in_flight jobs outstanding, collect in order.
static int serve_run_impl(vf_server *sv, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids,
                          int32_t in_flight, int64_t *out_ids, float *out_dists, float *latency_us)
{
    VF_REQUIRE(sv && queries && qoff && qids && out_ids && out_dists, "NULL argument");
    VF_REQUIRE(nq >= 0 && in_flight >= 1 && in_flight <= sv->ring_slots, "in_flight must be in [1, ring_slots]");
    using clock = std::chrono::steady_clock;
    std::vector<clock::time_point> t_sub((size_t)nq);
    std::vector<int64_t> job_of((size_t)nq);
    int64_t next = 0, head = 0;   // next query to submit, oldest query not collected yet
    const auto deadline = clock::now() + std::chrono::seconds(120);
    while (head < nq) {
        bool moved = false;
        if (next < nq && next - head < in_flight) {
            const int64_t b = qoff[next], e = qoff[next + 1];
            VF_REQUIRE(e > b && e - b <= kMaxOthers + 1, "a query needs 1 to 8 labels");
            int64_t job = -1;
            const int rc = serve_submit_impl(sv, (const char *)queries + (size_t)next * sv->row_bytes, qids + b, (int32_t)(e - b), &job);
            if (rc == VF_OK) {
                t_sub[(size_t)next] = clock::now();
                job_of[(size_t)next] = job;
                ++next;
                moved = true;
            } else if (rc != VF_EBUSY) {
                return rc;
            }
        }
        if (head < next) {
            int32_t done = 0;
            const int rc = serve_poll_impl(sv, job_of[(size_t)head], out_ids + head * sv->k, out_dists + head * sv->k, &done);
            if (rc != VF_OK) return rc;
            if (done) {
                if (latency_us)
                    latency_us[head] = std::chrono::duration<float, std::micro>(clock::now() - t_sub[(size_t)head]).count();
                ++head;
                moved = true;
            }
        }
        if (!moved && clock::now() > deadline) {
            set_error("vf_serve_run: no progress for two minutes");
            return VF_EHIP;
        }
    }
    return VF_OK;
}

extern "C" int vf_serve_run(vf_server *server, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                            const int32_t *qlabel_ids, int32_t in_flight, int64_t *out_ids, float *out_dists,
                            float *latency_us)
{
    return guarded([&] { return serve_run_impl(server, queries, nq, qlabel_offsets, qlabel_ids, in_flight, out_ids, out_dists, latency_us); });
}

extern "C" int vf_serve_begin(vf_index *index, const vf_serve_params *params, vf_server **out)
{
    return guarded([&] { return serve_begin_impl(index, params, out); });
}

extern "C" int vf_serve_submit(vf_server *server, const void *query, const int32_t *labels, int32_t n_labels, int64_t *job)
{
    return guarded([&] { return serve_submit_impl(server, query, labels, n_labels, job); });
}

extern "C" int vf_serve_poll(vf_server *server, int64_t job, int64_t *out_ids, float *out_dists, int32_t *done)
{
    return guarded([&] { return serve_poll_impl(server, job, out_ids, out_dists, done); });
}

extern "C" int vf_serve_end(vf_server *server, int64_t *jobs_done, int32_t *exit_reason)
{
    return guarded([&] { return serve_end_impl(server, jobs_done, exit_reason); });
}
