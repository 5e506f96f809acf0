// Vote casting, the global mask (counting sort over the vote levels, ordered emission),
// the sorted vote lists, and the masked gather / mean / error update.
#pragma once

#include "mv_common.hpp"
#include "mv_select.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// 4. vote casting
// ----------------------------------------------------------------------------
// One thread per candidate: a taken candidate casts its vote and, when the
// sorted vote lists are wanted (seg_sel != nullptr), is tallied in its
// 1024-coordinate segment (seg_sel was zeroed by the streaming pass).
__global__ __launch_bounds__(kVoteThreads) void mv_row_votes(
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count, uint32_t nseg,
    const uint32_t* __restrict__ kth_in, const uint32_t* __restrict__ tie_cut_in,
    const uint32_t* __restrict__ slow_flag, uint32_t* __restrict__ seg_sel,
    uint32_t* __restrict__ votes32, uint32_t* __restrict__ cnt_ge)
{
    __shared__ uint32_t lvl[257];
    const uint32_t row = blockIdx.y, t = threadIdx.x;
    // the thread's first list entry is fetched together with the row's counters, not after
    // them (the list's storage holds cap entries; an entry at or beyond the count is ignored)
    const u32x2* crow = cand + (size_t)row * cap;
    const uint64_t i_first = (uint64_t)blockIdx.x * kVoteThreads + t;
    const u32x2 c_first = crow[min(i_first, (uint64_t)cap - 1)];
    const uint32_t kth = kth_in[row], tie_cut = tie_cut_in[row];
    if (slow_flag[row] == 1u) return;                              // whole workgroup
    const uint32_t C = row_count[row * kCounterStride];
    if ((uint64_t)blockIdx.x * kVoteThreads >= C) return;    // whole workgroup
    for (int i = t; i < 257; i += kVoteThreads) lvl[i] = 0;
    __syncthreads();
    uint32_t*    ssel = seg_sel ? seg_sel + (size_t)row * nseg : nullptr;
    const uint32_t lane = lane_id();
    for (uint64_t i0 = (uint64_t)blockIdx.x * kVoteThreads; i0 < C; i0 += (uint64_t)gridDim.x * kVoteThreads) {
        const uint64_t i = i0 + t;
        u32x2 c = {0u, 0xFFFFFFFFu};
        bool taken = false;
        if (i < C) {
            c = (i == i_first) ? c_first : crow[i];
            taken = is_taken(c, kth, tie_cut);
        }
        if (taken) cast_vote(votes32, c.y, lvl);
        if (ssel) {
            // neighbouring list entries mostly share a segment (they are one run):
            // the first lane of each group of equal segments adds the group's count
            const uint32_t sg = c.y / kSeg;
            const uint32_t prev = __shfl_up(sg, 1, kWave);
            const uint64_t heads = __ballot(lane == 0 || sg != prev);
            const uint64_t tk = __ballot(taken);
            if (heads & (1ull << lane)) {
                const uint64_t above = (lane == kWave - 1) ? 0ull : (heads >> (lane + 1));
                const uint32_t len = above ? (uint32_t)__ffsll((long long)above) : (kWave - lane);
                const uint64_t span = (len >= 64 ? ~0ull : ((1ull << len) - 1)) << lane;
                const uint32_t n = (uint32_t)__popcll(tk & span);
                if (n) atomicAdd(&ssel[sg], n);
            }
        }
    }
    __syncthreads();
    for (int i = t; i < 256; i += kVoteThreads) {
        const uint32_t c = lvl[i];
        if (c) atomicAdd(&cnt_ge[(size_t)row * 256 + i], c);
    }
}

// ----------------------------------------------------------------------------
// 5. global mask = the K most voted coordinates, ties to the lowest coordinate;
//    beside it, the sorted vote lists
// ----------------------------------------------------------------------------
// cnt_ge[v] = number of coordinates with at least v votes (v = 1..N).  The
// threshold v* is the largest v with cnt_ge[v] >= K: all cnt_ge[v*+1]
// coordinates above it are taken, and the first K - cnt_ge[v*+1] coordinates
// (in coordinate order) with exactly v* votes.
__device__ __forceinline__ void vote_threshold(const uint32_t* __restrict__ cnt_ge, uint32_t N,
                                               uint32_t K, uint32_t* lds_lvl /*256*/, uint32_t* lds2,
                                               uint32_t& vstar, uint32_t& take_eq, int exact_levels)
{
    // cnt_ge holds one set of 256 level counters per worker row (the rows only spread the
    // atomics that filled them over as many cache lines); add the rows up (levels 0..N),
    // all loads of a thread in flight together
    for (uint32_t v = threadIdx.x; v < 256; v += blockDim.x) lds_lvl[v] = 0;
    __syncthreads();
    const uint32_t per_row = N + 1, n_vals = N * per_row;
    for (uint32_t i0 = threadIdx.x; i0 < n_vals; i0 += blockDim.x * 4) {
        uint32_t c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i = i0 + u * blockDim.x;
            c[u] = (i < n_vals) ? cnt_ge[(size_t)(i / per_row) * 256 + (i % per_row)] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i = i0 + u * blockDim.x;
            if (i < n_vals && c[u]) atomicAdd(&lds_lvl[i % per_row], c[u]);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (exact_levels) {
            // the sums are the numbers of coordinates with EXACTLY v votes, v = 0..N:
            // walk down from N until K coordinates are covered
            uint32_t above = 0, v = N;
            while (v > 0 && above + lds_lvl[v] < K) {
                above += lds_lvl[v];
                --v;
            }
            lds2[0] = v;
            lds2[1] = K - above;
        } else {
            uint32_t v = N;
            while (v > 1 && lds_lvl[v] < K) --v;
            lds2[0] = v;
            lds2[1] = K - ((v < N) ? lds_lvl[v + 1] : 0u);
        }
    }
    __syncthreads();
    vstar = lds2[0];
    take_eq = lds2[1];
}

// Exclusive scan of a row's segment tallies, in blocks of 1024 segments:
// seg_pre[s] = taken candidates in the earlier segments of s's block, and
// blk_total[blk] = taken candidates in the whole block.
__device__ __forceinline__ void seg_scan_block(const uint32_t* __restrict__ ssel, uint32_t nseg,
                                               uint32_t blk, uint32_t* __restrict__ spre,
                                               uint32_t* __restrict__ blk_total, uint64_t* scan_lds)
{
    const uint32_t t = threadIdx.x;
    const uint32_t s0 = blk * 1024u;
    uint32_t v[4];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t s = s0 + t * 4 + q;
        v[q] = (s < nseg) ? ssel[s] : 0u;
        sum += v[q];
    }
    uint64_t total;
    uint64_t ex = block_excl_scan64<kVoteThreads>(sum, scan_lds, total);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t s = s0 + t * 4 + q;
        if (s < nseg) spre[s] = (uint32_t)ex;
        ex += v[q];
    }
    if (t == 0) blk_total[blk] = (uint32_t)total;
}

// Workgroups [0, n_vote_blocks): count, per block of kVoteBlock coordinates, how
// many have votes > v* and == v*; optionally copy the vote bytes to the caller.
// Workgroups beyond (only launched when the sorted vote lists are wanted): scan
// the segment tallies of row (b / scan_blocks), block (b % scan_blocks).
__global__ __launch_bounds__(kVoteThreads) void mv_mask_count(const uint32_t* __restrict__ votes32,
                                                              int64_t d, uint32_t N, uint32_t K,
                                                              const uint32_t* __restrict__ cnt_ge,
                                                              u32x2* __restrict__ block_cnt,
                                                              uint8_t* __restrict__ votes_out,
                                                              uint32_t n_vote_blocks, uint32_t scan_blocks,
                                                              uint32_t nseg,
                                                              const uint32_t* __restrict__ slow_flag,
                                                              const uint32_t* __restrict__ seg_sel,
                                                              uint32_t* __restrict__ seg_pre,
                                                              uint32_t* __restrict__ blk_total,
                                                              uint32_t* __restrict__ vote_thr,
                                                              int exact_levels)
{
    __shared__ uint32_t lds2[2];
    __shared__ uint32_t lds_lvl[256];
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    if (blockIdx.x >= n_vote_blocks) {
        const uint32_t b = blockIdx.x - n_vote_blocks;
        const uint32_t row = b / scan_blocks;
        if (slow_flag[row] == 1u) return;
        seg_scan_block(seg_sel + (size_t)row * nseg, nseg, b % scan_blocks, seg_pre + (size_t)row * nseg,
                       blk_total + (size_t)row * scan_blocks, scan_lds);
        return;
    }
    // the block's vote words first: their latency overlaps the threshold's loads
    constexpr int kIt = kVoteBlock / (kVoteThreads * 16);
    const int64_t base = (int64_t)blockIdx.x * kVoteBlock;
    u32x4 w[kIt];
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        w[it] = (j < d) ? *reinterpret_cast<const u32x4*>(votes32 + (j >> 2)) : z;   // padded to 16 bytes with zeros
    }
    uint32_t vstar, take_eq;
    vote_threshold(cnt_ge, N, K, lds_lvl, lds2, vstar, take_eq, exact_levels);
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        if (j < d) {
            const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t v = (ww[q] >> (8 * b)) & 255u;
                    const bool inside = j + q * 4 + b < d;      // matters when v* is 0
                    gt += (inside && v > vstar);
                    eq += (inside && v == vstar);
                }
            if (votes_out) {
                if (j + 16 <= d && ((reinterpret_cast<uintptr_t>(votes_out) & 15) == 0)) {
                    *reinterpret_cast<u32x4*>(votes_out + j) = w[it];
                } else {
                    for (int q = 0; q < 16; ++q)
                        if (j + q < d) votes_out[j + q] = (uint8_t)((ww[q >> 2] >> (8 * (q & 3))) & 255u);
                }
            }
        }
    }
    uint64_t total;
    (void)block_excl_scan64<kVoteThreads>(pack2(gt, eq), scan_lds, total);
    if (threadIdx.x == 0) {
        u32x2 r;
        r.x = (uint32_t)(total >> 32);
        r.y = (uint32_t)total;
        block_cnt[blockIdx.x] = r;
        if (blockIdx.x == 0) {                   // the threshold, for mv_mask_emit
            vote_thr[0] = vstar;
            vote_thr[1] = take_eq;
        }
    }
}

// One thread per candidate of a row: a taken candidate's rank in the row's
// ascending vote list is (taken candidates in earlier blocks of 1024 segments,
// from blk_total) + (in earlier segments of its block, from seg_pre) + (before
// it in its own segment's run; runs are ascending), so the list comes out
// sorted without a sort.
__device__ __forceinline__ void row_emit_block(const u32x2* __restrict__ crow, uint32_t C,
                                               const u32x2* __restrict__ srow,
                                               const uint32_t* __restrict__ prow,
                                               const uint32_t* __restrict__ blk_total, uint32_t scan_blocks,
                                               uint32_t K, uint32_t kth, uint32_t tie_cut, uint32_t blk,
                                               uint32_t nblk, uint32_t* __restrict__ out,
                                               uint32_t* blk_pre /*LDS, kMaxScanBlocks*/, uint64_t* scan_lds)
{
    if ((uint64_t)blk * kVoteThreads >= C) return;           // whole workgroup
    // exclusive prefix of the blocks' totals, once per workgroup
    {
        constexpr int per = kMaxScanBlocks / kVoteThreads;
        uint32_t v[per];
        uint32_t sum = 0;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            const uint32_t b = threadIdx.x * per + q;
            v[q] = (b < scan_blocks) ? blk_total[b] : 0u;
            sum += v[q];
        }
        uint64_t total;
        uint64_t ex = block_excl_scan64<kVoteThreads>(sum, scan_lds, total);
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
    // from memory, by the whole wavefront together.
    const uint32_t lane = lane_id();
    for (uint64_t i0 = (uint64_t)blk * kVoteThreads; i0 < C; i0 += (uint64_t)nblk * kVoteThreads) {
        const uint64_t i = i0 + threadIdx.x;
        const uint64_t wave_first = i - lane;
        u32x2 c = {0u, 0xFFFFFFFFu};
        bool taken = false;
        if (i < C) {
            c = crow[i];
            taken = is_taken(c, kth, tie_cut);
        }
        const uint32_t sg = c.y / kSeg;                       // 0x3FFFFF for lanes past the end
        const uint32_t prev = __shfl_up(sg, 1, kWave);
        const uint64_t heads = __ballot(lane == 0 || sg != prev);
        const uint64_t tk = __ballot(taken);
        if (tk == 0ull) continue;                             // wave-uniform
        const uint64_t upto = (lane == 63) ? ~0ull : ((2ull << lane) - 1);      // lanes 0..lane
        const uint32_t head_lane = 63u - (uint32_t)__clzll((long long)(heads & upto));
        const uint64_t in_run_before = ((1ull << lane) - 1) & ~((1ull << head_lane) - 1);
        uint32_t rank = (uint32_t)__popcll(tk & in_run_before);
        // the run of lane 0 may have started before this wavefront
        const uint32_t sg0 = __shfl(sg, 0, kWave);
        uint32_t carry = 0;
        if (wave_first < C) {                                 // wave-uniform
            const uint32_t run0 = srow[sg0].x;
            for (uint64_t j0 = run0; j0 < wave_first; j0 += kWave) {
                const uint64_t j = j0 + lane;
                const bool tj = (j < wave_first) && is_taken(crow[j], kth, tie_cut);
                carry += (uint32_t)__popcll(__ballot(tj));
            }
        }
        if (head_lane == 0) rank += carry;
        if (taken) {
            const uint32_t pos = prow[sg] + blk_pre[sg / 1024u] + rank;
            if (pos < K) out[pos] = c.y;
        }
    }
}

// Workgroups [0, n_vote_blocks): emit the mask in ascending order and clear the
// vote words for the next step.  Workgroups beyond (only launched when the
// sorted vote lists are wanted): write row (b / emit_blocks)'s vote list.
__global__ __launch_bounds__(kVoteThreads) void mv_mask_emit(uint32_t* __restrict__ votes32,
                                                             int64_t d, uint32_t K,
                                                             const uint32_t* __restrict__ vote_thr,
                                                             const u32x2* __restrict__ block_cnt,
                                                             uint32_t* __restrict__ mask_idx,
                                                             uint32_t n_vote_blocks, uint32_t emit_blocks,
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
                                                             int clear_votes)
{
    __shared__ uint32_t blk_pre[kMaxScanBlocks];
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    if (blockIdx.x >= n_vote_blocks) {
        const uint32_t b = blockIdx.x - n_vote_blocks;
        const uint32_t row = b / emit_blocks;
        if (slow_flag[row] == 1u) return;
        row_emit_block(cand + (size_t)row * cap, row_count[row * kCounterStride], seg + (size_t)row * nseg,
                       seg_pre + (size_t)row * nseg, blk_total + (size_t)row * scan_blocks, scan_blocks, K,
                       kth_in[row], tie_cut_in[row], b % emit_blocks, emit_blocks,
                       worker_idx + (size_t)row * K, blk_pre, scan_lds);
        return;
    }
    // the block's vote words first (cleared behind for the next step): their latency
    // overlaps the loads of the prefix below
    constexpr int kIt = kVoteBlock / (kVoteThreads * 16);
    const int64_t base = (int64_t)blockIdx.x * kVoteBlock;
    u32x4 w[kIt];
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        w[it] = z;
        if (j < d) {
            u32x4* p = reinterpret_cast<u32x4*>(votes32 + (j >> 2));
            w[it] = *p;
            if (clear_votes && (w[it].x | w[it].y | w[it].z | w[it].w) != 0u) *p = z;
        }
    }
    const uint32_t vstar = vote_thr[0], take_eq = vote_thr[1];   // found by mv_mask_count

    // coordinates selected / tied before this block
    uint64_t mine = 0;
    for (uint32_t b = threadIdx.x; b < blockIdx.x; b += kVoteThreads) {
        const u32x2 r = block_cnt[b];
        mine += pack2(r.x, r.y);
    }
    uint64_t before;
    (void)block_excl_scan64<kVoteThreads>(mine, scan_lds, before);
    __syncthreads();
    uint32_t gt_before = (uint32_t)(before >> 32), eq_before = (uint32_t)before;

#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
        uint32_t gt = 0, eq = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
            const bool inside = j + q < d;                             // matters when v* is 0
            gt += (inside && v > vstar);
            eq += (inside && v == vstar);
        }
        uint64_t total;
        const uint64_t ex = block_excl_scan64<kVoteThreads>(pack2(gt, eq), scan_lds, total);
        if (gt | eq) {
            uint32_t g0 = gt_before + (uint32_t)(ex >> 32), e0 = eq_before + (uint32_t)ex;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                const bool inside = j + q < d;
                const bool is_gt = inside && v > vstar, is_eq = inside && v == vstar;
                if (is_gt || (is_eq && e0 < take_eq)) {
                    const uint32_t pos = g0 + min(e0, take_eq);
                    if (mask_idx && pos < K) mask_idx[pos] = (uint32_t)(j + q);
                }
                g0 += is_gt;
                e0 += is_eq;
            }
        }
        gt_before += (uint32_t)(total >> 32);
        eq_before += (uint32_t)total;
        __syncthreads();
    }
}

// ----------------------------------------------------------------------------
// 6. masked gather, ordered sum over workers, mean, error update
// ----------------------------------------------------------------------------
// A workgroup handles kb = 256 / N mask coordinates.  Thread (kl, n) reads
// a[n][mask[k]] (held in e), stores +0.0 there (the error update: the residual
// of a transmitted coordinate is zero), and parks the value in LDS; one thread
// per coordinate then adds the N values in worker order 0..N-1 in fp32 and
// applies the 1/N of the mean once.
__global__ __launch_bounds__(kGatherThreads) void mv_gather_update(float* __restrict__ e, int64_t ld_e,
                                                                   int64_t d, uint32_t N, uint32_t K,
                                                                   const uint32_t* __restrict__ mask_idx,
                                                                   float scale, int apply_scale,
                                                                   float* __restrict__ agg)
{
    __shared__ float tile[2 * kGatherThreads];
    const uint32_t kb = kGatherThreads / N;          // N <= 255, so kb >= 1
    const uint32_t t = threadIdx.x;
    const uint32_t kl = t / N, n = t % N;
    const uint32_t k = blockIdx.x * kb + kl;
    const uint32_t pitch = N + 1;                     // kb * (N + 1) <= 256 + kb <= 512
    if (kl < kb && k < K) {
        const uint32_t j = mask_idx[k];
        float v = 0.0f;
        if ((int64_t)j < d) {                         // always true for a mask built by mv_mask_emit
            float* p = e + (int64_t)n * ld_e + j;
            v = *p;
            *p = 0.0f;
        }
        tile[kl * pitch + n] = v;
    }
    __syncthreads();
    if (t < kb) {
        const uint32_t kk = blockIdx.x * kb + t;
        if (kk < K) {
            float s = tile[t * pitch];                // worker 0
            for (uint32_t m = 1; m < N; ++m) s = s + tile[t * pitch + m];
            agg[kk] = apply_scale ? s * scale : s;
        }
    }
}

}  // namespace mvk
