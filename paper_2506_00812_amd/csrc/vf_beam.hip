// Launch of the IVF-Graph beam search (Section 4.2.1, Alg. 2): one wave64 per graph query of the batch.
#include <hip/hip_ext.h>

#include "vf_beam.h"

namespace vf {

// Waves per SIMD the register budget is set for: the one-register-list kernels (E = 1) are the ones whose every
// wave should be resident at once.  float32 without predicate 7 (<= 72 VGPRs), with predicate 6 (80, a few values
// spilled: measured faster on 100,000 two-label queries than 5 waves without spills); uint8 with predicate 7.
// LAT: the instantiation for launches of at most BeamParams::lat_waves queries (every wave on a SIMD of its own): two waves per
// SIMD's worth of registers, the candidates' vectors requested 64 at a time.
template <int DT, int E, bool AND, bool LAT = false>
__global__ __launch_bounds__(64, LAT ? 2 : (DT == 1 && E == 1) ? (AND ? 6 : 7) : (E == 1 && AND) ? 7 : 8) void beam_kernel(BeamParams p)
{
    extern __shared__ uint4 smem[];
    const int gq = blockIdx.x;
    const int qi = p.gq_query[gq];
    const int row_bytes = p.dim * (DT == 0 ? 1 : 4);
    BeamQuery bq;
    bq.q = (const char *)p.Q + (int64_t)qi * row_bytes;
    bq.label = p.gq_label[gq];
    bq.others = nullptr; bq.o_cnt = 0;
    if (AND && p.others_off != nullptr) {
        const int o_begin = p.others_off[qi];
        bq.others = p.others + o_begin;
        bq.o_cnt = p.others_off[qi + 1] - o_begin;
    }
    bq.out_ids = p.out_ids + (int64_t)qi * p.k;
    bq.out_dists = p.out_dists + (int64_t)qi * p.k;
    bq.counters = p.counters != nullptr ? p.counters + (int64_t)qi * 4 : nullptr;
    bq.gathered = p.gathered != nullptr ? p.gathered + qi : nullptr;
    bq.dseed_row = p.dseed != nullptr ? p.dseed + (int64_t)gq * p.ns_stride : nullptr;
    bq.runs = p.seed_runs != nullptr ? p.seed_runs + (int64_t)gq * p.run_segs * p.run_K : nullptr;
    bq.seed_pass = p.seed_pass != nullptr ? p.seed_pass[gq] : -1;
    beam_search_wave<DT, E, false, AND, LAT>(p, bq, smem);
}

size_t beam_lds_bytes(const BeamParams &p, int dtype)
{
    const size_t row_bytes = (size_t)p.dim * (dtype == 0 ? 1 : 4);
    return row_bytes + 128 * 4 * 3 + 8 * 4 + ((size_t)4 << p.hash_bits);
}

template <int DT, bool AND>
static void launch_beam_dt(const BeamParams &p, int n_gq, size_t lds, hipStream_t s, hipEvent_t start, hipEvent_t stop)
{
    const dim3 grid(n_gq), block(64);
    if (p.itopk <= 64 && n_gq <= p.lat_waves) hipExtLaunchKernelGGL((beam_kernel<DT, 1, AND, true>), grid, block, (uint32_t)lds, s, start, stop, 0, p);
    else if (p.itopk <= 64) hipExtLaunchKernelGGL((beam_kernel<DT, 1, AND>), grid, block, (uint32_t)lds, s, start, stop, 0, p);
    else if (p.itopk <= 128) hipExtLaunchKernelGGL((beam_kernel<DT, 2, AND>), grid, block, (uint32_t)lds, s, start, stop, 0, p);
    else hipExtLaunchKernelGGL((beam_kernel<DT, 4, AND>), grid, block, (uint32_t)lds, s, start, stop, 0, p);
}

// start / stop (optional): events that take the kernel's own begin and end times.  Recording events around the
// launch instead puts a barrier packet of their own before and behind the kernel, each of which delays the next
// kernel on the stream by a few microseconds.
void launch_beam(int dtype, const BeamParams &p, int n_gq, hipStream_t s, hipEvent_t start, hipEvent_t stop)
{
    if (n_gq <= 0) return;
    const size_t lds = beam_lds_bytes(p, dtype);
    // batches without predicate labels run an instantiation without the predicate's code
    const bool with_and = p.others_off != nullptr;
    if (dtype == 0) {
        if (with_and) launch_beam_dt<0, true>(p, n_gq, lds, s, start, stop);
        else launch_beam_dt<0, false>(p, n_gq, lds, s, start, stop);
    } else {
        if (with_and) launch_beam_dt<1, true>(p, n_gq, lds, s, start, stop);
        else launch_beam_dt<1, false>(p, n_gq, lds, s, start, stop);
    }
}

}  // namespace vf
