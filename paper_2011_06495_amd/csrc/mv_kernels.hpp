// Device kernels of the majority-voting vote step for gfx950 (MI355X).
//
// The step is bound by HBM traffic: the only work that touches all N*d
// coordinates is the error compensation a = g + e (Algorithm 1) and finding
// each worker's K largest |a| (its vote).  Nothing here is a dense
// contraction, so no MFMA; the design goal is ONE streaming pass over g and e.
//
// How the per-worker top-K is found without re-reading the row:
//   1. mv_stream_collect  ONE launch holds the threshold estimate and the
//                         streaming pass.  The first workgroups of the grid take
//                         a histogram of the magnitude bit patterns of a strided
//                         sample of each row; the last of a row's samplers turns
//                         it into a bin edge tau that somewhat more than K
//                         coordinates of the row exceed (an ESTIMATE, never
//                         trusted) and publishes it.  The other workgroups
//                         stream: a = g + e is written over e, and every
//                         coordinate with |a| >= tau is appended to the row's
//                         candidate list; each wavefront's 1024-coordinate
//                         segment records where its run of candidates went.  A
//                         streaming wavefront looks for its row's tau while its
//                         loads are in flight and polls a bounded number of
//                         times; a row whose wavefronts did not all see tau is
//                         selected from memory instead
//   2. mv_row_select      per row, a few workgroups: EXACT select of the K-th
//                         largest magnitude among the candidates (their number
//                         is known exactly; if it is < K or overflowed the list,
//                         the row is selected exactly from memory instead) and of
//                         the largest coordinate taken among its ties; then every
//                         workgroup casts the votes of its share of the list.
//                         Long lists (large K) go through mv_sel_hist /
//                         mv_sel_split / mv_sel_rank and mv_row_votes, many
//                         workgroups per row
//   3. mv_mask_count      counting-sort selection of the K most voted
//                         coordinates, ties to the lowest coordinate: the vote
//                         threshold from the level counters, the counts of every
//                         block of the vote bytes, their sums across blocks
//                         (published between the workgroups), and the mask's
//                         coordinates written in place.  Extra workgroups scan
//                         the segment tallies for the sorted vote lists
//   4. mv_gather_update   masked gather, sum over workers in order, mean, and
//                         the error update (zero on the mask); extra workgroups
//                         write each row's vote in ascending coordinate order
//   5. mv_ad_*            majority voting with add-drop (Algorithm 2): replaces
//                         the vote casting by the update of the workers'
//                         standing votes
//   6. mv_rs_*            majority voting with random selection (Algorithm 1,
//                         S_rand-weighted): replaces the mask of step 3
//
// Things measured on this machine that shape much of the code: a returning
// atomic completes only after the previous one on the same cache line (so
// list space is reserved once per workgroup and hot counters sit on lines of
// their own); a load issued inside a divergent per-thread loop pays its full
// latency every time (so sparse work is first compacted into LDS and then
// fetched by all lanes together); a kernel boundary costs about 2 us and a
// small dependent kernel at least 4 us (so short steps share a launch, with
// words published between workgroups where one step feeds the next); a
// workgroup of 1024 threads with more than 64 VGPRs or more than 80 KB of LDS has
// a compute unit to itself, two fit otherwise (so the grids of the small kernels
// are sized to about one workgroup per each of the chip's 256 units).
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
