// Device kernels of the majority-voting vote step for gfx950 (MI355X).
//
// The step is bound by HBM traffic: the only work that touches all N*d
// coordinates is the error compensation a = g + e (Algorithm 1) and finding
// each worker's K largest |a| (its vote).  Nothing here is a dense
// contraction, so no MFMA; the design goal is ONE streaming pass over g and e.
//
// How the per-worker top-K is found without re-reading the row:
//   1. mv_sample_hist     histogram of the magnitude bit patterns of a strided
//      mv_pick_threshold  sample of each row (cache-line sized chunks), turned
//                         into a bin edge tau that about 2K coordinates of the
//                         row exceed (an ESTIMATE, never trusted); also resets
//                         the row's per-step counters
//   2. mv_stream_collect  the streaming pass: a = g + e is written over e, and
//                         every coordinate with |a| >= tau is appended to the
//                         row's candidate list; each wavefront's 1024-coordinate
//                         segment records where its run of candidates went
//   3. mv_row_select      per row: EXACT select of the K-th largest magnitude
//                         among the candidates (their number is known exactly;
//                         if it is < K or overflowed the list, the row is
//                         selected exactly from memory instead), and of the
//                         largest coordinate taken among its ties.  Long lists
//                         (large K) go through mv_sel_hist / mv_sel_split /
//                         mv_sel_rank, many workgroups per row
//   4. mv_row_votes       one thread per candidate: the taken ones cast their vote
//   5. mv_mask_count /    counting-sort selection of the K most voted
//      mv_mask_emit       coordinates, ties to the lowest coordinate.  Extra
//                         workgroups of the same two launches write each row's
//                         vote in ascending coordinate order (segment tallies
//                         scanned, then one thread per candidate), off the
//                         critical path
//   6. mv_gather_update   masked gather, sum over workers in order, mean, and
//                         the error update (zero on the mask)
//   7. mv_ad_*            majority voting with add-drop (Algorithm 2): replaces
//                         step 4 by the update of the workers' standing votes
//   8. mv_rs_*            majority voting with random selection (Algorithm 1,
//                         S_rand-weighted): replaces the mask of step 5
//
// Two things measured on this machine shape much of the code: a returning
// atomic completes only after the previous one on the same cache line (so
// list space is reserved once per workgroup and hot counters sit on lines of
// their own), and a load issued inside a divergent per-thread loop pays its
// full latency every time (so sparse work is first compacted into LDS and then
// fetched by all lanes together).
#pragma once

#include "mv_common.hpp"
#include "mv_stream.hpp"
#include "mv_select.hpp"
#include "mv_mask.hpp"
#include "mv_add_drop.hpp"
#include "mv_random_select.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// measurement aid: a plain streaming copy (n16 units of 16 bytes), the yardstick
// for the HBM bandwidth a kernel of this shape can reach and for scaling the
// profiler's byte counters
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mv_probe_copy_kernel(const u32x4* __restrict__ src,
                                                            u32x4* __restrict__ dst, uint64_t n16)
{
    const uint64_t base = (uint64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint64_t i = base + (uint64_t)u * 256;
        if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    }
}

}  // namespace mvk
