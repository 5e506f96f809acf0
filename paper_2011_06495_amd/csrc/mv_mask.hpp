// Vote casting for long lists, the global mask (counting sort over the vote levels,
// ordered emission), the sorted vote lists, and the masked gather / mean / error update.
//
// These kernels are short (a few dependent memory round trips each), and the chip
// starts only a few hundred workgroups per microsecond: they use workgroups of 1024
// threads and grids of a few hundred workgroups.
#pragma once

#include "mv_common.hpp"
#include "mv_select.hpp"

namespace mvk {

constexpr int kMaskThreads = 1024;   // mv_mask_count / mv_gather_update
constexpr int kLookBack = 256;       // earlier blocks whose totals a block of mv_mask_count adds up itself

// ----------------------------------------------------------------------------
// 4. vote casting for long candidate lists (the rows' select ran in the mv_sel_*
//    kernels): many workgroups per row, each casting the votes of its share
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(kRowThreads) void mv_row_votes(
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count, uint32_t nseg,
    const uint32_t* __restrict__ kth_in, const uint32_t* __restrict__ tie_cut_in,
    const uint32_t* __restrict__ slow_flag, uint32_t* __restrict__ seg_sel,
    uint32_t* __restrict__ votes32, uint32_t* __restrict__ lvl_sets)
{
    __shared__ uint32_t lvl[257];
    const uint32_t row = blockIdx.y;
    const uint32_t kth = kth_in[row], tie_cut = tie_cut_in[row];
    if (slow_flag[row] == 1u) return;                              // whole workgroup
    const uint32_t C = row_count[row];
    for (int i = threadIdx.x; i < 257; i += kRowThreads) lvl[i] = 0;
    __syncthreads();
    cast_votes_of_share<kRowThreads, true>(cand + (size_t)row * cap, C, kth, tie_cut, blockIdx.x, gridDim.x, votes32, lvl,
                                     seg_sel ? seg_sel + (size_t)row * nseg : nullptr);
    __syncthreads();
    merge_levels(lvl, lvl_sets, blockIdx.y * gridDim.x + blockIdx.x);
}

// ----------------------------------------------------------------------------
// 5. global mask = the K most voted coordinates, ties to the lowest coordinate
// ----------------------------------------------------------------------------
// Counting sort over the vote levels 0..N in two kernels.  The level counters (summed
// over their sets) say how many coordinates hold at least v votes (plain voting: filled
// while the votes were cast) or exactly v votes (add-drop voting: a histogram of the
// vote sum).  The threshold v* is the level at which K coordinates are covered walking
// down from N: all coordinates above v* are taken, and the first K - (#above)
// coordinates, in coordinate order, with exactly v* votes.  A block is the 16384 Q
// coordinates of one workgroup (Q = 1 to 8 quads of 16 vote bytes per thread, chosen
// so that the grid stays at a few hundred workgroups).  mv_mask_count counts, per
// wavefront's stretch of the vote bytes, the coordinates above and at v*;
// mv_gather_update turns the counts of the earlier stretches into positions: each of
// its workgroups emits the part of the mask it gathers.

// All threads of the workgroup: vstar / take_eq from the level counters.
__device__ __forceinline__ void vote_threshold(const uint32_t* __restrict__ lvl_sets, uint32_t N, uint32_t K,
                                               uint32_t* lvl /*LDS, 256*/, uint32_t* thr /*LDS, 2*/,
                                               uint32_t& vstar, uint32_t& take_eq, int exact_levels)
{
    if (threadIdx.x < 256) {                      // thread v adds up level v's sets, all loads in flight together
        uint32_t c[kLvlSets];
        const uint32_t v = threadIdx.x;
#pragma unroll
        for (int q = 0; q < kLvlSets; ++q) c[q] = (v <= N) ? lvl_sets[(size_t)q * 256 + v] : 0u;
        uint32_t sum = 0;
#pragma unroll
        for (int q = 0; q < kLvlSets; ++q) sum += c[q];
        lvl[v] = sum;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (exact_levels) {
            // coordinates with EXACTLY v votes, v = 1..N: walk down from N until K coordinates are
            // covered; level 0 (every other coordinate) covers whatever is left
            uint32_t above = 0, v = N;
            while (v > 0 && above + lvl[v] < K) {
                above += lvl[v];
                --v;
            }
            thr[0] = v;
            thr[1] = K - above;
        } else {
            // coordinates with AT LEAST v votes; at least K coordinates hold a vote
            uint32_t v = N;
            while (v > 1 && lvl[v] < K) --v;
            thr[0] = v;
            thr[1] = K - ((v < N) ? lvl[v + 1] : 0u);
        }
    }
    __syncthreads();
    vstar = thr[0];
    take_eq = thr[1];
}

// The thread's coordinates with more than / exactly vstar votes among its 16 Q bytes from j0
// on.  Must be called by all lanes of a wavefront together: a word that holds no vote in
// any lane is passed over by the whole wavefront (most words, where votes are sparse);
// with vstar == 0 the coordinates without a vote count too and nothing is passed over.
template <int Q>
__device__ __forceinline__ void count_above_and_at(const uint32_t (&ww)[4 * Q], int64_t j0, int64_t d,
                                                   uint32_t vstar, uint32_t& gt, uint32_t& eq)
{
    gt = 0;
    eq = 0;
#pragma unroll
    for (int q = 0; q < 4 * Q; ++q) {
        if (vstar != 0u && __ballot(ww[q] != 0u) == 0ull) continue;   // wave-uniform
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t v = (ww[q] >> (8 * b)) & 255u;
            const bool inside = j0 + 4 * q + b < d;                   // matters when v* is 0
            gt += (inside && v > vstar);
            eq += (inside && v == vstar);
        }
    }
}

// Exclusive scan of a row's segment tallies for the sorted vote lists, 4096 segments
// at a time: seg_pre[s] = taken candidates in the earlier segments of s's block of
// 1024 segments, and blk_total[blk] = taken candidates in the whole block.
__device__ __forceinline__ void seg_scan_part(const uint32_t* __restrict__ ssel, uint32_t nseg,
                                              uint32_t part, uint32_t* __restrict__ spre,
                                              uint32_t* __restrict__ blk_total, uint64_t* scan_lds,
                                              uint32_t* bound /*LDS, 5*/)
{
    const uint32_t t = threadIdx.x;
    const uint32_t s0 = part * 4096u + t * 4u;
    uint32_t v[4];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v[q] = (s0 + q < nseg) ? ssel[s0 + q] : 0u;
        sum += v[q];
    }
    uint64_t total;
    uint64_t ex = block_excl_scan64<kMaskThreads>(sum, scan_lds, total);
    if ((t & 255u) == 0u) bound[t >> 8] = (uint32_t)ex;      // threads 256 k .. 256 k + 255 hold block k of the four
    if (t == 0) bound[4] = (uint32_t)total;
    __syncthreads();
    const uint32_t k = t >> 8;
    ex -= bound[k];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (s0 + q < nseg) spre[s0 + q] = (uint32_t)ex;
        ex += v[q];
    }
    if ((t & 255u) == 0u && part * 4u + k < (nseg + 1023u) / 1024u) blk_total[part * 4u + k] = bound[k + 1] - bound[k];
    __syncthreads();                              // the LDS scratch is free for the next part
}

// Workgroups [0, n_vote_blocks): count the block's coordinates above and at the vote
// threshold (also per wavefront's stretch of 1024 Q coordinates), exchange the counts
// with the other blocks and write the block's part of the mask; optionally copy the vote
// bytes to the caller.  Workgroups beyond (only launched when the sorted vote lists are
// wanted): one per row, scanning the row's segment tallies.
template <int Q>
__global__ __launch_bounds__(kMaskThreads) void mv_mask_count(const uint32_t* __restrict__ votes32,
                                                              int64_t d, uint32_t N, uint32_t K,
                                                              const uint32_t* __restrict__ lvl_sets,
                                                              u32x2* __restrict__ sub_cnt,
                                                              u32x2* __restrict__ block_cnt,
                                                              uint32_t* __restrict__ vote_thr,
                                                              uint8_t* __restrict__ votes_out,
                                                              uint32_t n_vote_blocks, uint32_t scan_parts,
                                                              uint32_t scan_blocks, uint32_t nseg,
                                                              const uint32_t* __restrict__ slow_flag,
                                                              const uint32_t* __restrict__ seg_sel,
                                                              uint32_t* __restrict__ seg_pre,
                                                              uint32_t* __restrict__ blk_total,
                                                              int exact_levels,
                                                              unsigned long long* __restrict__ lookback,
                                                              uint32_t* __restrict__ emit_fail, uint32_t spin_limit,
                                                              uint32_t* __restrict__ mask_idx)
{
    __shared__ uint32_t lvl[256];
    __shared__ uint32_t thr[2];
    __shared__ uint64_t scan_lds[kMaskThreads / kWave + 1];
    __shared__ uint32_t bound[5];
    __shared__ uint64_t before_sh;
    if (blockIdx.x >= n_vote_blocks) {
        const uint32_t row = blockIdx.x - n_vote_blocks;       // one workgroup per row
        if (slow_flag[row] == 1u) return;
        for (uint32_t part = 0; part < scan_parts; ++part)
            seg_scan_part(seg_sel + (size_t)row * nseg, nseg, part, seg_pre + (size_t)row * nseg,
                          blk_total + (size_t)row * scan_blocks, scan_lds, bound);
        return;
    }
    // the block's vote words first: their latency overlaps the level counters' loads.
    // Thread t owns the block's bytes [16 Q t, 16 Q t + 16 Q).
    const int64_t j0 = ((int64_t)blockIdx.x * kMaskThreads + threadIdx.x) * (16 * Q);
    u32x4 w[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int64_t j = j0 + q * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        w[q] = (j < d) ? *reinterpret_cast<const u32x4*>(votes32 + (j >> 2)) : z;   // padded to 16 bytes with zeros
    }
    uint32_t vstar, take_eq;
    vote_threshold(lvl_sets, N, K, lvl, thr, vstar, take_eq, exact_levels);
    uint32_t ww[4 * Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        ww[4 * q + 0] = w[q].x; ww[4 * q + 1] = w[q].y; ww[4 * q + 2] = w[q].z; ww[4 * q + 3] = w[q].w;
        if (votes_out) {
            const int64_t j = j0 + q * 16;
            if (j + 16 <= d && ((reinterpret_cast<uintptr_t>(votes_out) & 15) == 0)) {
                *reinterpret_cast<u32x4*>(votes_out + j) = w[q];
            } else {
                for (int b = 0; b < 16; ++b)
                    if (j + b < d) votes_out[j + b] = (uint8_t)((ww[4 * q + (b >> 2)] >> (8 * (b & 3))) & 255u);
            }
        }
    }
    uint32_t gt, eq;
    count_above_and_at<Q>(ww, j0, d, vstar, gt, eq);
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    const uint64_t both = pack2(gt, eq);
    uint64_t block_total;
    const uint64_t ex = block_excl_scan64<kMaskThreads>(both, scan_lds, block_total);   // before this thread, in the block
    {
        // the counts per wavefront stretch and per block: what mv_gather_update scans when the
        // mask could not be written here
        const uint64_t stretch = (uint64_t)__shfl((unsigned long long)(ex + both), kWave - 1, kWave) -
                                 (uint64_t)__shfl((unsigned long long)ex, 0, kWave);
        if (lane == 0) {
            u32x2 r;
            r.x = (uint32_t)(stretch >> 32);
            r.y = (uint32_t)stretch;
            sub_cnt[(size_t)blockIdx.x * (kMaskThreads / kWave) + wave] = r;
        }
        if (threadIdx.x == 0) {
            u32x2 r;
            r.x = (uint32_t)(block_total >> 32);
            r.y = (uint32_t)block_total;
            block_cnt[blockIdx.x] = r;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {    // the threshold, for the kernel that follows
        vote_thr[0] = vstar;
        vote_thr[1] = take_eq;
    }
    if (!mask_idx) return;                        // random selection writes the mask elsewhere

    // The counts of the earlier blocks, without another kernel: every block publishes its own
    // totals at once (word 0 of its pair); its first wavefront then reads the totals of the
    // kLookBack blocks before it, all loads in flight together, and the sum over everything
    // up to the block before those (word 1 of that block's pair, published by that block once
    // it has summed up itself), polling until every word is there.  A word holds a "present"
    // bit and both counts (each below 2^31), so one 64-bit store publishes it whole.  Blocks
    // are dispatched in the order of their numbers and publish their totals before they wait,
    // so the wait ends; were a word still missing after spin_limit polls, the block gives up,
    // says so in emit_fail, and mv_gather_update finds the mask from the counts instead.
    constexpr unsigned long long kPresent = 1ull << 63, kCountMask = 0x7FFFFFFFull;
    constexpr int kPer = kLookBack / kWave;
    auto word_of = [&](uint64_t counts) { return kPresent | ((counts >> 32) << 31) | (counts & kCountMask); };
    auto counts_of = [&](unsigned long long w) {
        return pack2((uint32_t)((w >> 31) & kCountMask), (uint32_t)(w & kCountMask));
    };
    if (wave == 0) {
        const int64_t me = blockIdx.x;
        if (lane == 0)
            __hip_atomic_store(&lookback[2 * me], word_of(block_total), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // lane l: the totals of blocks me - 1 - l - 64 r; lane 0 also the sum up to block me - kLookBack - 1
        const unsigned long long* src[kPer + 1];
        unsigned long long w[kPer + 1];
#pragma unroll
        for (int r = 0; r < kPer; ++r) {
            const int64_t b = me - 1 - (int64_t)lane - (int64_t)kWave * r;
            src[r] = b >= 0 ? &lookback[2 * b] : nullptr;
        }
        src[kPer] = (lane == 0 && me - kLookBack - 1 >= 0) ? &lookback[2 * (me - kLookBack - 1) + 1] : nullptr;
#pragma unroll
        for (int r = 0; r <= kPer; ++r) w[r] = src[r] ? 0ull : kPresent;
        bool found = true;
        for (uint32_t polls = 0;; ++polls) {
            bool all = true;
#pragma unroll
            for (int r = 0; r <= kPer; ++r)
                if (!(w[r] & kPresent)) w[r] = __hip_atomic_load(src[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int r = 0; r <= kPer; ++r) all = all && (w[r] & kPresent);
            if (__ballot(!all) == 0ull) break;
            if (polls >= spin_limit) {                                // uniform
                found = false;
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        uint64_t before = 0;
#pragma unroll
        for (int r = 0; r <= kPer; ++r) before += counts_of(w[r]);
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) before += (uint64_t)__shfl_xor((unsigned long long)before, o, kWave);
        if (lane == 0) {
            if (found)
                __hip_atomic_store(&lookback[2 * me + 1], word_of(before + block_total), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            else
                __hip_atomic_store(emit_fail, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            before_sh = before;
            bound[0] = found ? 1u : 0u;
        }
    }
    __syncthreads();
    if (bound[0] == 0u) return;                   // whole workgroup
    const uint64_t before = before_sh;
    if ((uint32_t)(before >> 32) + min((uint32_t)before, take_eq) >= K) return;   // the mask is full before this block
    uint32_t g0 = (uint32_t)((before + ex) >> 32), e0 = (uint32_t)(before + ex);
#pragma unroll
    for (int q = 0; q < 4 * Q; ++q) {
        if (vstar != 0u && __ballot(ww[q] != 0u) == 0ull) continue;   // wave-uniform: no vote in this word
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t v = (ww[q] >> (8 * b)) & 255u;
            const int64_t j = j0 + 4 * q + b;
            const bool inside = j < d;
            const bool is_gt = inside && v > vstar, is_eq = inside && v == vstar;
            if (is_gt || (is_eq && e0 < take_eq)) {
                const uint32_t pos = g0 + min(e0, take_eq);
                if (pos < K) mask_idx[pos] = (uint32_t)j;
            }
            g0 += is_gt;
            e0 += is_eq;
        }
    }
}

// ----------------------------------------------------------------------------
// 6. masked gather, ordered sum over workers, mean, error update; beside it, the
//    sorted vote lists
// ----------------------------------------------------------------------------

// A row's vote list in ascending coordinate order, without a sort: a taken
// candidate's rank is (taken candidates in earlier blocks of 1024 segments, from
// blk_total) + (in earlier segments of its block, from seg_pre) + (before it in its
// own segment's run; runs are ascending).
__device__ __forceinline__ void row_emit_block(const u32x2* __restrict__ crow, uint32_t C,
                                               const u32x2* __restrict__ srow,
                                               const uint32_t* __restrict__ prow,
                                               const uint32_t* __restrict__ blk_total, uint32_t scan_blocks,
                                               uint32_t K, uint32_t kth, uint32_t tie_cut, uint32_t blk,
                                               uint32_t nblk, uint32_t* __restrict__ out,
                                               uint32_t* blk_pre /*LDS, kMaxScanBlocks*/, uint64_t* scan_lds)
{
    if ((uint64_t)blk * 4 * kMaskThreads >= C) return;       // whole workgroup
    // exclusive prefix of the blocks' totals, once per workgroup
    {
        constexpr int per = kMaxScanBlocks / kMaskThreads;
        uint32_t v[per];
        uint32_t sum = 0;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            const uint32_t b = threadIdx.x * per + q;
            v[q] = (b < scan_blocks) ? blk_total[b] : 0u;
            sum += v[q];
        }
        uint64_t total;
        uint64_t ex = block_excl_scan64<kMaskThreads>(sum, scan_lds, total);
#pragma unroll
        for (int q = 0; q < per; ++q) {
            blk_pre[threadIdx.x * per + q] = (uint32_t)ex;
            ex += v[q];
        }
        __syncthreads();
    }
    // Lanes of a wavefront hold consecutive list entries, so the entries of one run
    // sit in neighbouring lanes: the rank inside the run comes from a ballot; only
    // the part of the first lane's run that lies before the wavefront is counted
    // from memory, by the whole wavefront together.  kU entries per thread are in
    // flight at a time, each followed by the loads that depend on it.
    constexpr int kU = 4;
    const uint32_t lane = lane_id();
    for (uint64_t i0 = (uint64_t)blk * kU * kMaskThreads; i0 < C; i0 += (uint64_t)nblk * kU * kMaskThreads) {
        u32x2 c[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const uint64_t i = i0 + (uint64_t)u * kMaskThreads + threadIdx.x;
            const u32x2 none = {0u, 0xFFFFFFFFu};
            c[u] = (i < C) ? crow[i] : none;
        }
        uint32_t seg_before[kU], run0[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const uint32_t sg = c[u].y / kSeg;                // 0x3FFFFF for lanes past the end
            const bool there = c[u].y != 0xFFFFFFFFu;
            seg_before[u] = there ? prow[sg] + blk_pre[sg / 1024u] : 0u;
            run0[u] = there ? srow[sg].x : 0u;
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const uint64_t i = i0 + (uint64_t)u * kMaskThreads + threadIdx.x;
            const uint64_t wave_first = i - lane;
            if (wave_first >= C) break;                           // wave-uniform
            const bool taken = c[u].y != 0xFFFFFFFFu && is_taken(c[u], kth, tie_cut);
            const uint32_t sg = c[u].y / kSeg;
            const uint32_t prev = __shfl_up(sg, 1, kWave);
            const uint64_t heads = __ballot(lane == 0 || sg != prev);
            const uint64_t tk = __ballot(taken);
            if (tk == 0ull) continue;                             // wave-uniform
            const uint64_t upto = (lane == 63) ? ~0ull : ((2ull << lane) - 1);      // lanes 0..lane
            const uint32_t head_lane = 63u - (uint32_t)__clzll((long long)(heads & upto));
            const uint64_t in_run_before = ((1ull << lane) - 1) & ~((1ull << head_lane) - 1);
            uint32_t rank = (uint32_t)__popcll(tk & in_run_before);
            // the run of lane 0 may have started before this wavefront
            const uint32_t first_run = __shfl(run0[u], 0, kWave);
            uint32_t carry = 0;
            for (uint64_t j0 = first_run; j0 < wave_first; j0 += kWave) {
                const uint64_t j = j0 + lane;
                const bool tj = (j < wave_first) && is_taken(crow[j], kth, tie_cut);
                carry += (uint32_t)__popcll(__ballot(tj));
            }
            if (head_lane == 0) rank += carry;
            if (taken) {
                const uint32_t pos = seg_before[u] + rank;
                if (pos < K) out[pos] = c[u].y;
            }
        }
    }
}

// Workgroups [0, n_gather_blocks): each owns `rounds` times kb = 1024 / N consecutive
// positions of the mask.
// (a) Unless the mask is given (random selection writes it elsewhere), the workgroup
//     first finds its own positions' coordinates: the counts per block of the vote bytes
//     and, inside the few blocks that matter, per wavefront stretch (from mv_mask_count)
//     are scanned, which says where in the mask each stretch's coordinates go; the few
//     stretches that reach into the workgroup's positions are read again, one wavefront each, and their coordinates above the
//     vote threshold, and the first take_eq at it, go to their positions -- in LDS for
//     the gather, and in mask_idx for the caller.  No kernel of its own emits the mask.
// (b) Thread (kl, n) reads a[n][mask[k]] (held in e), stores +0.0 there (the error
//     update: the residual of a transmitted coordinate is zero), and parks the value in
//     LDS; one thread per coordinate then adds the N values in worker order 0..N-1 in
//     fp32 and applies the 1/N of the mean once.
// Workgroups beyond (only launched when the sorted vote lists are wanted): write
// row (b / emit_blocks)'s vote list; they start after the gather's workgroups and
// run beside them.
constexpr int kGatherRounds = 4;                  // at most this many rounds of kb positions per workgroup

struct GatherLds {
    float    tile[kMaskThreads + kMaskThreads / 2 + 8];
    uint32_t slice[kGatherRounds * kMaskThreads];              // the workgroup's positions' coordinates
    uint32_t need[3 * (kMaskThreads + 2)];                     // stretches to read: (stretch, above before, at before)
    uint32_t blocks[3 * (kMaskThreads + 2)];                   // blocks whose stretches are looked at
    uint32_t n_need, n_blocks;
    uint32_t blk_pre[kMaxScanBlocks];
    uint64_t scan[kMaskThreads / kWave + 1];
};

template <int Q>
__global__ __launch_bounds__(kMaskThreads) void mv_gather_update(float* __restrict__ e, int64_t ld_e,
                                                                 int64_t d, uint32_t N, uint32_t K,
                                                                 const uint32_t* __restrict__ votes32,
                                                                 const u32x2* __restrict__ sub_cnt,
                                                                 const u32x2* __restrict__ block_cnt, uint32_t n_blocks,
                                                                 const uint32_t* __restrict__ vote_thr,
                                                                 uint32_t* __restrict__ mask_idx, int mask_given,
                                                                 const uint32_t* __restrict__ emit_fail,
                                                                 float scale, int apply_scale,
                                                                 float* __restrict__ agg, uint32_t rounds,
                                                                 uint32_t n_gather_blocks, uint32_t emit_blocks,
                                                                 const u32x2* __restrict__ cand, uint32_t cap,
                                                                 const uint32_t* __restrict__ row_count,
                                                                 const u32x2* __restrict__ seg, uint32_t nseg,
                                                                 const uint32_t* __restrict__ seg_pre,
                                                                 const uint32_t* __restrict__ blk_total,
                                                                 uint32_t scan_blocks,
                                                                 const uint32_t* __restrict__ kth_in,
                                                                 const uint32_t* __restrict__ tie_cut_in,
                                                                 const uint32_t* __restrict__ slow_flag,
                                                                 uint32_t* __restrict__ worker_idx,
                                                                 uint32_t* __restrict__ step_no)
{
    __shared__ GatherLds lds;
    if (blockIdx.x >= n_gather_blocks) {
        const uint32_t b = blockIdx.x - n_gather_blocks;
        const uint32_t row = b / emit_blocks;
        if (slow_flag[row] == 1u) return;
        row_emit_block(cand + (size_t)row * cap, row_count[row], seg + (size_t)row * nseg,
                       seg_pre + (size_t)row * nseg, blk_total + (size_t)row * scan_blocks, scan_blocks, K,
                       kth_in[row], tie_cut_in[row], b % emit_blocks, emit_blocks,
                       worker_idx + (size_t)row * K, lds.blk_pre, lds.scan);
        return;
    }
    const uint32_t kb = kMaskThreads / N;             // N <= 255, so kb >= 4
    const uint32_t t = threadIdx.x, lane = lane_id(), wave = t / kWave;
    // This is the step's last kernel and nothing in it reads the step's number: the next step
    // gets the next number (kept on the device, so that a captured step can be replayed).
    if (blockIdx.x == 0 && t == 0) step_no[0] = step_no[0] + 1u;
    const uint32_t k0 = blockIdx.x * kb * rounds;     // the workgroup's positions: [k0, k1)
    const uint32_t k1 = min(K, k0 + kb * rounds);

    if (!mask_given && emit_fail[0] != 0u) {          // uniform over the grid; not expected
        const uint32_t vstar = vote_thr[0], take_eq = vote_thr[1];
        // one round of at most kb <= 1024 positions [q0, q1) at a time: that bounds the lists in LDS
        for (uint32_t r = 0; r < rounds; ++r) {
            const uint32_t q0 = k0 + r * kb, q1 = min(k1, q0 + kb);
            if (q0 >= q1) break;                          // uniform
            if (t == 0) {
                lds.n_need = 0;
                lds.n_blocks = 0;
            }
            // position of a stretch's (a block's) first mask coordinate = (coordinates above the threshold
            // before it) + min(coordinates at the threshold before it, take_eq)
            auto reaches_in = [&](uint32_t g, uint32_t q, u32x2 c) {
                const uint32_t q_taken = min(q, take_eq);                  // of the earlier ones at the threshold
                const uint32_t first = g + q_taken;
                const uint32_t n_in = c.x + min(c.y, take_eq - q_taken);
                return n_in != 0u && first < q1 && first + n_in > q0;
            };
            // first level: the blocks' totals
            uint32_t gt_before = 0, eq_before = 0;        // over the blocks of the earlier passes
            for (uint32_t b0 = 0; b0 < n_blocks; b0 += kMaskThreads) {
                const u32x2 none = {0u, 0u};
                const u32x2 c = b0 + t < n_blocks ? block_cnt[b0 + t] : none;
                uint64_t total;
                const uint64_t ex = block_excl_scan64<kMaskThreads>(pack2(c.x, c.y), lds.scan, total);
                const uint32_t g = gt_before + (uint32_t)(ex >> 32), q = eq_before + (uint32_t)ex;
                if (reaches_in(g, q, c)) {
                    const uint32_t at = atomicAdd(&lds.n_blocks, 1u);
                    lds.blocks[3 * at + 0] = b0 + t;
                    lds.blocks[3 * at + 1] = g;
                    lds.blocks[3 * at + 2] = q;
                }
                gt_before += (uint32_t)(total >> 32);
                eq_before += (uint32_t)total;
                __syncthreads();                          // lds.scan is reused by the next pass
                if (gt_before + min(eq_before, take_eq) >= q1) break;   // uniform: the rest lies behind these positions
            }
            __syncthreads();
            // second level: the stretches of those blocks (16 each), one wavefront per block
            constexpr uint32_t kSubs = kMaskThreads / kWave;
            const uint32_t n_blk = lds.n_blocks;
            for (uint32_t i = wave; i < n_blk; i += kSubs) {
                const uint32_t b = lds.blocks[3 * i];
                const u32x2 none = {0u, 0u};
                const u32x2 c = lane < kSubs ? sub_cnt[(size_t)b * kSubs + lane] : none;
                const uint64_t both = pack2(c.x, c.y);
                const uint64_t ex = wave_incl_scan64(both) - both;
                const uint32_t g = lds.blocks[3 * i + 1] + (uint32_t)(ex >> 32), q = lds.blocks[3 * i + 2] + (uint32_t)ex;
                if (lane < kSubs && reaches_in(g, q, c)) {
                    const uint32_t at = atomicAdd(&lds.n_need, 1u);
                    lds.need[3 * at + 0] = b * kSubs + lane;
                    lds.need[3 * at + 1] = g;
                    lds.need[3 * at + 2] = q;
                }
            }
            __syncthreads();
            // one wavefront per needed stretch: its 1024 Q vote bytes, lane l owning bytes [16 Q l, 16 Q l + 16 Q)
            const uint32_t n_need = lds.n_need;
            for (uint32_t i = wave; i < n_need; i += kSubs) {
                const uint32_t sidx = lds.need[3 * i];
                const int64_t j0 = ((int64_t)sidx * kWave + lane) * (16 * Q);
                uint32_t ww[4 * Q];
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const int64_t j = j0 + q * 16;
                    const u32x4 z = {0u, 0u, 0u, 0u};
                    const u32x4 w = (j < d) ? *reinterpret_cast<const u32x4*>(votes32 + (j >> 2)) : z;
                    ww[4 * q + 0] = w.x; ww[4 * q + 1] = w.y; ww[4 * q + 2] = w.z; ww[4 * q + 3] = w.w;
                }
                uint32_t gt, eq;
                count_above_and_at<Q>(ww, j0, d, vstar, gt, eq);
                const uint64_t both = pack2(gt, eq);
                const uint64_t ex = wave_incl_scan64(both) - both;
                uint32_t g0 = lds.need[3 * i + 1] + (uint32_t)(ex >> 32), e0 = lds.need[3 * i + 2] + (uint32_t)ex;
#pragma unroll
                for (int q = 0; q < 4 * Q; ++q) {
                    if (vstar != 0u && __ballot(ww[q] != 0u) == 0ull) continue;   // wave-uniform: no vote in this word
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const uint32_t v = (ww[q] >> (8 * b)) & 255u;
                        const int64_t j = j0 + 4 * q + b;
                        const bool inside = j < d;
                        const bool is_gt = inside && v > vstar, is_eq = inside && v == vstar;
                        if (is_gt || (is_eq && e0 < take_eq)) {
                            const uint32_t pos = g0 + min(e0, take_eq);
                            if (pos >= q0 && pos < q1) {
                                lds.slice[pos - k0] = (uint32_t)j;
                                mask_idx[pos] = (uint32_t)j;
                            }
                        }
                        g0 += is_gt;
                        e0 += is_eq;
                    }
                }
            }
            __syncthreads();                          // the lists are reused by the next round
        }
    } else {
        for (uint32_t k = k0 + t; k < k1; k += kMaskThreads) lds.slice[k - k0] = mask_idx[k];
    }
    __syncthreads();

    const uint32_t kl = t / N, n = t % N;
    const uint32_t pitch = N + 1;                     // kb * (N + 1) <= 1024 + kb <= 1536
    // a thread's loads of all rounds are in flight together
    float v[kGatherRounds];
#pragma unroll
    for (int r = 0; r < kGatherRounds; ++r) {
        const uint32_t k = k0 + (uint32_t)r * kb + kl;
        const uint32_t j = ((uint32_t)r < rounds && kl < kb && k < k1) ? lds.slice[k - k0] : 0xFFFFFFFFu;
        v[r] = 0.0f;
        if ((int64_t)j < d) {                         // always true for a mask built above
            float* p = e + (int64_t)n * ld_e + j;
            v[r] = *p;
            *p = 0.0f;
        }
    }
#pragma unroll
    for (int r = 0; r < kGatherRounds; ++r) {
        if ((uint32_t)r >= rounds) break;             // uniform over the workgroup
        if (kl < kb) lds.tile[kl * pitch + n] = v[r];
        __syncthreads();
        if (t < kb) {
            const uint32_t kk = k0 + (uint32_t)r * kb + t;
            if (kk < k1) {
                float s = lds.tile[t * pitch];        // worker 0
                for (uint32_t m = 1; m < N; ++m) s = s + lds.tile[t * pitch + m];
                agg[kk] = apply_scale ? s * scale : s;
            }
        }
        __syncthreads();
    }
}

}  // namespace mvk
