// vf_search for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
// that forbid hipMalloc.  Same routing, same kernels and the same results as vf_search; what differs is where the
// call's device-side temporaries live -- in a file-scope array of device memory instead of a workspace the
// library allocates and grows -- and that nothing is created on the way: no stream, no event, no pinned staging
// buffer, no seed copy.  The routing tables reach the device as kernel arguments.
#include "vf_host.h"

namespace vf {

// Device-side temporaries of one call: routing blob | partial rows of the scan lists' segments (index, distance
// bits) | seed distance matrix.  One array per GPU the library runs on, held until the process ends; every call
// on a GPU shares it and finds the last call's contents in it (no part of it needs to start at zero: every word
// a kernel reads has been written earlier in the same call).
constexpr size_t kScratchBytes = (size_t)VF_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// The array's device address, per device: the name `scratch` is only a host-side handle of the symbol.
constexpr int kMaxDevices = 64;
static unsigned char *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mu;

static int scratch_for_current_device(unsigned char **out)
{
    int dev = -1;
    VF_HIP(hipGetDevice(&dev));
    VF_REQUIRE(dev >= 0 && dev < kMaxDevices, "device ordinal out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        VF_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        VF_REQUIRE(ptr != nullptr, "no device address for the scratch array");
        g_scratch_ptr[dev] = (unsigned char *)ptr;
    }
    *out = g_scratch_ptr[dev];
    return VF_OK;
}

// A piece of the routing blob travels as a kernel argument (no host buffer the device could read exists).
constexpr int kChunkWords = 960;   // 3840 bytes: the argument block of a kernel holds 4096
struct BlobChunk { uint32_t w[kChunkWords]; };

__global__ __launch_bounds__(256) void blob_put_kernel(BlobChunk c, uint32_t *dst, int n_words)
{
    for (int i = threadIdx.x; i < n_words; i += 256) dst[i] = c.w[i];
}

int search_noalloc_impl(vf_index *ix, const void *queries, int64_t nq, const int64_t *qoff, const int32_t *qids, int32_t k,
                        int32_t itopk, int32_t width, int32_t iters, int32_t n_seeds, int64_t *out_ids, float *out_dists,
                        hipStream_t s)
{
    int rc = check_search_args(ix, queries, nq, k, out_ids, out_dists);
    if (rc != VF_OK) return rc;
    VF_REQUIRE(nq <= VF_NOALLOC_MAX_QUERIES, "vf_search_noalloc: more than VF_NOALLOC_MAX_QUERIES queries in one call");
    std::lock_guard<std::recursive_mutex> lock(ix->mu);
    if ((rc = check_search_params(ix, false, k, itopk, width, iters, n_seeds)) != VF_OK) return rc;
    unsigned char *base = nullptr;
    if ((rc = scratch_for_current_device(&base)) != VF_OK) return rc;
    if (nq == 0) return VF_OK;

    Routed &r = ix->noalloc_routed;
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    // First with room for the seed distance matrix (dense seed scoring); if the call does not fit that way,
    // without it (the beam kernel then gathers its seeds itself).
    SeedCopy *sc = nullptr;   // a copy is used when a regular call has left one
    if (wants_seed_copy(ix, false, itopk, n_seeds) && (rc = seed_copy_for(ix, n_seeds, s, false, &sc)) != VF_OK) return rc;
    CallPlan P(ix->tune);
    size_t off_idx = 0, off_bits = 0, off_dseed = 0, total = 0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        P = CallPlan(ix->tune);
        const uint64_t budget_words = attempt == 0 ? kScratchBytes / 4 : 0;
        if ((rc = plan_call(ix, r, nq, qoff, qids, false, false, k, itopk, width, iters, n_seeds, 0, budget_words, sc, P)) != VF_OK)
            return rc;
        off_idx = up(P.L.total);
        off_bits = up(off_idx + P.part_words * 4);
        off_dseed = up(off_bits + P.part_words * 4);
        total = off_dseed + (P.dense_seeds ? P.dseed_words * 4 : 0);
        if (total <= kScratchBytes || !P.dense_seeds) break;
    }
    if (total > kScratchBytes) {
        set_error("vf_search_noalloc: this call needs " + std::to_string(total) + " bytes of scratch memory, the fixed array holds " +
                  std::to_string(kScratchBytes) + " (fewer queries or a smaller k per call; or vf_search)");
        return VF_EINVAL;
    }
    const size_t off_blob = 0;
    // routing blob: assembled in host memory the index keeps, sent in pieces of kChunkWords words
    std::vector<char> &hb = ix->noalloc_blob;
    hb.assign((P.L.total + 3) & ~(size_t)3, 0);
    fill_blob(P, r, hb.data());
    const size_t n_words = hb.size() / 4;
    for (size_t w0 = 0; w0 < n_words; w0 += kChunkWords) {
        BlobChunk c;
        const size_t nw = std::min<size_t>(kChunkWords, n_words - w0);
        memcpy(c.w, hb.data() + w0 * 4, nw * 4);
        hipLaunchKernelGGL(blob_put_kernel, dim3(1), dim3(256), 0, s, c, (uint32_t *)(base + off_blob) + w0, (int)nw);
    }
    CallMem M;
    M.blob = (char *)(base + off_blob);
    M.part_idx = (int32_t *)(base + off_idx);
    M.part_bits = (uint32_t *)(base + off_bits);
    M.dseed = (uint32_t *)(base + off_dseed);
    // everything on the caller's stream, one launch after the other
    if ((rc = launch_call(ix, P, r, M, sc, queries, out_ids, out_dists, s, nullptr, nullptr, nullptr, false)) != VF_OK) return rc;
    VF_HIP(hipGetLastError());
    return VF_OK;
}

}  // namespace vf

extern "C" int vf_search_noalloc(vf_index *index, const void *queries, int64_t nq, const int64_t *qlabel_offsets,
                                 const int32_t *qlabel_ids, int32_t k, int32_t itopk, int32_t width, int32_t iters,
                                 int32_t n_seeds, int64_t *out_ids, float *out_dists, void *hip_stream)
{
    return vf::guarded([&] {
        return vf::search_noalloc_impl(index, queries, nq, qlabel_offsets, qlabel_ids, k, itopk, width, iters, n_seeds,
                                       out_ids, out_dists, (hipStream_t)hip_stream);
    });
}
