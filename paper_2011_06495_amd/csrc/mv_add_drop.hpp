// Majority voting with add-drop (Algorithm 2): candidate lists, K_ad-selects, update of the
// standing votes and of their sum, ordered compaction of the scratch bitmaps.
#pragma once

#include "mv_common.hpp"
#include "mv_select.hpp"
#include "mv_mask.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// 7. majority voting with add-drop (Algorithm 2)
// ----------------------------------------------------------------------------
// State, owned by the caller: vote_bits (row n = the bitmap of M~_n, the worker's
// standing vote) and msum (one byte per coordinate, M^sum = the sum of the
// standing votes).  After mv_row_select, membership of coordinate j in a row's
// plain top-K is a local test on (|a[n][j]|, j) against (kth, tie_cut), so
//   A = top-K and not in the standing vote   -> candidates for addition
//   D = in the standing vote and not top-K   -> candidates for removal
// are gathered into two lists per row; the K_ad largest of A and the K_ad
// smallest of D are selected exactly (ties to the lowest coordinate), applied to
// scratch bitmaps and to msum, and the scratch bitmaps are compacted in
// coordinate order into the sorted add / drop lists while the standing vote is
// updated.

// One workgroup-wide reservation: every thread brings `n_mine` entries; returns the
// position of the thread's first entry in the row's list (the list counter is bumped
// once per workgroup).  All threads of the workgroup must call it.
__device__ __forceinline__ uint32_t reserve_in_list(uint32_t n_mine, uint32_t* __restrict__ counter,
                                                    uint64_t* scan_lds, uint32_t* bcast)
{
    uint64_t total;
    const uint64_t ex = block_excl_scan64<kVoteThreads>(n_mine, scan_lds, total);
    if (threadIdx.x == 0) bcast[0] = total ? atomicAdd(counter, (uint32_t)total) : 0u;
    __syncthreads();
    const uint32_t base = bcast[0];
    __syncthreads();
    return base + (uint32_t)ex;
}

__device__ __forceinline__ bool vote_bit(const uint32_t* __restrict__ bits_row, uint32_t j)
{
    return (bits_row[j >> 5] >> (j & 31u)) & 1u;
}

// A-lists.  Rows whose top-K came from the candidate list: one thread per candidate.
// Rows selected from memory (slow_flag == 1): the whole row is read.
__device__ __forceinline__ void ad_collect_add_block(
    uint32_t bx, uint32_t nbx, uint64_t* scan_lds, uint32_t* bcast,
    const float* __restrict__ e, int64_t ld_e, int64_t d,
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count,
    const uint32_t* __restrict__ kth_in, const uint32_t* __restrict__ tie_cut_in,
    const uint32_t* __restrict__ slow_flag, const uint32_t* __restrict__ vote_bits, int64_t ld_bits,
    u32x2* __restrict__ a_list, uint32_t* __restrict__ ad_count)
{
    const uint32_t row = blockIdx.y, t = threadIdx.x;
    const uint32_t kth = kth_in[row], tie_cut = tie_cut_in[row];
    const uint32_t* bits = vote_bits + (int64_t)row * ld_bits;
    u32x2* arow = a_list + (size_t)row * cap;
    uint32_t* counter = ad_count + ad_counter(row, 0);
    if (slow_flag[row] == 1u) {
        const float* xrow = e + (int64_t)row * ld_e;
        for (int64_t j0 = (int64_t)bx * kVoteThreads; j0 < d; j0 += (int64_t)nbx * kVoteThreads) {
            const int64_t j = j0 + t;
            u32x2 c = {0u, 0u};
            bool in_a = false;
            if (j < d) {
                c.x = __float_as_uint(xrow[j]) & kAbsMask;
                c.y = (uint32_t)j;
                in_a = is_taken(c, kth, tie_cut) && !vote_bit(bits, c.y);
            }
            const uint32_t pos = reserve_in_list(in_a ? 1u : 0u, counter, scan_lds, bcast);
            if (in_a && pos < cap) arow[pos] = c;
        }
        return;
    }
    const uint32_t C = row_count[row];
    const u32x2* crow = cand + (size_t)row * cap;
    for (uint64_t i0 = (uint64_t)bx * kVoteThreads; i0 < C; i0 += (uint64_t)nbx * kVoteThreads) {
        const uint64_t i = i0 + t;
        u32x2 c = {0u, 0u};
        bool in_a = false;
        if (i < C) {
            c = crow[i];
            in_a = is_taken(c, kth, tie_cut) && !vote_bit(bits, c.y);
        }
        const uint32_t pos = reserve_in_list(in_a ? 1u : 0u, counter, scan_lds, bcast);
        if (in_a && pos < cap) arow[pos] = c;
    }
}

// D-lists: the standing vote's bitmap is scanned, 4 words per thread; a set
// coordinate that is not in the row's top-K goes to the list with the
// complemented magnitude, so that "largest first" selects the smallest magnitudes.
constexpr int kDropStage = 1024;   // set bits of one workgroup's stretch staged in LDS per round
constexpr int kBitIt = 1;          // quads of bitmap words per thread in the bitmap kernels (more per thread measured no faster)
constexpr int kBitBlockWords = kVoteThreads * 4 * kBitIt;   // bitmap words per workgroup
__device__ __forceinline__ void ad_collect_drop_block(
    uint32_t bx, uint64_t* scan_lds, uint32_t* bcast, uint32_t* stage,
    const float* __restrict__ e, int64_t ld_e, int64_t d,
    const uint32_t* __restrict__ kth_in, const uint32_t* __restrict__ tie_cut_in,
    const uint32_t* __restrict__ vote_bits, int64_t ld_bits, uint32_t nwords,
    u32x2* __restrict__ d_list, uint32_t cap_d, uint32_t* __restrict__ ad_count)
{
    const uint32_t row = blockIdx.y, t = threadIdx.x;
    const uint32_t kth = kth_in[row], tie_cut = tie_cut_in[row];
    const float* xrow = e + (int64_t)row * ld_e;
    // the workgroup's stretch of the bitmap: kBitIt quads of words per thread
    uint32_t w[kBitIt][4];
    uint32_t n_bits = 0;
#pragma unroll
    for (int it = 0; it < kBitIt; ++it) {
        const uint32_t w0 = bx * kBitBlockWords + ((uint32_t)it * kVoteThreads + t) * 4;
        w[it][0] = w[it][1] = w[it][2] = w[it][3] = 0;
        if (w0 < nwords) {                        // rows are padded to a multiple of 4 words
            const u32x4 v = *reinterpret_cast<const u32x4*>(vote_bits + (int64_t)row * ld_bits + w0);
            w[it][0] = v.x; w[it][1] = v.y; w[it][2] = v.z; w[it][3] = v.w;
            if ((uint64_t)w0 * 32 + 128 > (uint64_t)d) {        // bits at or beyond d do not exist
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    for (int b = 0; b < 32; ++b)
                        if ((int64_t)(w0 + q) * 32 + b >= d) w[it][q] &= ~(1u << b);
            }
        }
        n_bits += __popc(w[it][0]) + __popc(w[it][1]) + __popc(w[it][2]) + __popc(w[it][3]);
    }
    uint64_t total;
    const uint64_t ex = block_excl_scan64<kVoteThreads>(n_bits, scan_lds, total);
    if (total == 0) return;                                  // whole workgroup
    u32x2* drow = d_list + (size_t)row * cap_d;
    // The members' coordinates are parked in LDS (kDropStage at a time; one round unless the
    // stretch is crowded with votes) and their values then fetched by all lanes together,
    // instead of one dependent load per set bit inside each thread's own loop.
    auto one_round = [&](const uint32_t c0) {
        uint32_t sp = (uint32_t)ex;
#pragma unroll
        for (int it = 0; it < kBitIt; ++it) {
            const uint32_t w0 = bx * kBitBlockWords + ((uint32_t)it * kVoteThreads + t) * 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t m = w[it][q];
                while (m) {
                    const uint32_t b = __ffs((int)m) - 1;
                    m &= m - 1;
                    if (sp - c0 < (uint32_t)kDropStage) stage[sp - c0] = (w0 + q) * 32 + b;   // sp < c0 wraps: not staged
                    ++sp;
                }
            }
        }
        __syncthreads();
        const uint32_t cnt = min((uint32_t)kDropStage, (uint32_t)total - c0);
        constexpr int kRounds = kDropStage / kVoteThreads;
        u32x2 c[kRounds];
        uint32_t n_keep = 0, keep = 0;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const uint32_t i = (uint32_t)r * kVoteThreads + t;
            if (i < cnt) {
                const uint32_t j = stage[i];
                c[r].x = __float_as_uint(xrow[j]) & kAbsMask;
                c[r].y = j;
                if (!is_taken(c[r], kth, tie_cut)) {         // left the top-K: a drop candidate
                    keep |= 1u << r;
                    ++n_keep;
                }
            }
        }
        uint32_t pos = reserve_in_list(n_keep, ad_count + ad_counter(row, 1), scan_lds, bcast);
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            if (keep & (1u << r)) {
                if (pos < cap_d) {
                    u32x2 o;
                    o.x = kAbsMask - c[r].x;
                    o.y = c[r].y;
                    drow[pos] = o;
                }
                ++pos;
            }
        }
    };
    if (total <= (uint64_t)kDropStage) {                     // uniform; the usual case
        one_round(0u);
    } else {
        for (uint32_t c0 = 0; c0 < (uint32_t)total; c0 += kDropStage) one_round(c0);
    }
}

// One launch for both lists: the first add_blocks workgroups of a row walk its
// candidate list (A-list), the others its standing vote's bitmap (D-list).
__global__ __launch_bounds__(kVoteThreads) void mv_ad_collect(
    const float* __restrict__ e, int64_t ld_e, int64_t d,
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count,
    const uint32_t* __restrict__ kth_in, const uint32_t* __restrict__ tie_cut_in,
    const uint32_t* __restrict__ slow_flag, const uint32_t* __restrict__ vote_bits, int64_t ld_bits,
    uint32_t nwords, u32x2* __restrict__ a_list, u32x2* __restrict__ d_list, uint32_t cap_d,
    uint32_t* __restrict__ ad_count, uint32_t add_blocks)
{
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    __shared__ uint32_t bcast[1];
    __shared__ uint32_t stage[kDropStage];
    if (blockIdx.x < add_blocks)
        ad_collect_add_block(blockIdx.x, add_blocks, scan_lds, bcast, e, ld_e, d, cand, cap, row_count, kth_in,
                             tie_cut_in, slow_flag, vote_bits, ld_bits, a_list, ad_count);
    else
        ad_collect_drop_block(blockIdx.x - add_blocks, scan_lds, bcast, stage, e, ld_e, d, kth_in, tie_cut_in,
                              vote_bits, ld_bits, nwords, d_list, cap_d, ad_count);
}

// Workgroup (0, n): the K_ad first of row n's A-list under (magnitude desc,
// coordinate asc); workgroup (1, n): the same for the D-list, whose keys are the
// complemented magnitudes.  Result: ad_thr[n][2*which] = key threshold,
// [2*which+1] = tie cut (membership test as for the top-K), and
// counts_out[2n + which] = how many are taken = min(K_ad, list length).
__global__ __launch_bounds__(kRowThreads) void mv_ad_select(
    const u32x2* __restrict__ a_list, uint32_t cap_a, const u32x2* __restrict__ d_list, uint32_t cap_d,
    const uint32_t* __restrict__ ad_count, uint32_t k_ad, const uint32_t* __restrict__ tau_bits,
    const uint32_t* __restrict__ slow_flag, uint32_t* __restrict__ ad_thr, uint32_t* __restrict__ counts_out)
{
    __shared__ SelectLds lds;
    const uint32_t which = blockIdx.x, row = blockIdx.y, t = threadIdx.x;
    const u32x2* list = which ? d_list + (size_t)row * cap_d : a_list + (size_t)row * cap_a;
    const uint32_t len = min(ad_count[ad_counter(row, which)], which ? cap_d : cap_a);
    uint32_t kth, tie_cut;
    if (len == 0) {
        kth = 0xFFFFFFFFu;                        // nothing passes the membership test
        tie_cut = 0;
    } else if (len <= k_ad) {
        kth = 0;                                  // everything passes
        tie_cut = 0xFFFFFFFFu;
    } else {
        uint32_t path;
        auto at = [list](uint64_t i) { return list[i].x; };
        const KeysInMemory<decltype(at)> src{at, len};
        // every A-list magnitude is at least the row's estimate tau when the row's top-K
        // came from its candidate list; the D-list has no such bound
        const uint32_t tau = (which || slow_flag[row] == 1u) ? 0u : tau_bits[row];
        select_among_candidates(src, list, len, k_ad, tau, lds, kth, tie_cut, path);
    }
    if (t == 0) {
        ad_thr[4 * row + 2 * which] = kth;
        ad_thr[4 * row + 2 * which + 1] = tie_cut;
        counts_out[2 * row + which] = min(len, k_ad);
    }
}

// Applies the selected additions and removals: marks them in the row's scratch
// bitmap (one bitmap for both: a marked coordinate that is in the standing vote is a
// removal, one that is not is an addition) and moves msum by +1 / -1 (bytes packed four
// to a word; a byte never carries because 0 <= msum <= N <= 255 holds before and after).
__global__ __launch_bounds__(kVoteThreads) void mv_ad_apply(
    const u32x2* __restrict__ a_list, uint32_t cap_a, const u32x2* __restrict__ d_list, uint32_t cap_d,
    const uint32_t* __restrict__ ad_count, const uint32_t* __restrict__ ad_thr,
    uint32_t* __restrict__ ad_bits, uint32_t nwords_pad, uint32_t* __restrict__ msum32)
{
    const uint32_t row = blockIdx.y;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const u32x2* list = which ? d_list + (size_t)row * cap_d : a_list + (size_t)row * cap_a;
        const uint32_t len = min(ad_count[ad_counter(row, which)], which ? cap_d : cap_a);
        const uint32_t kth = ad_thr[4 * row + 2 * which], tie_cut = ad_thr[4 * row + 2 * which + 1];
        uint32_t* bits = ad_bits + (size_t)row * nwords_pad;   // additions and removals share the row's bitmap
        for (uint32_t i = blockIdx.x * kVoteThreads + threadIdx.x; i < len; i += gridDim.x * kVoteThreads) {
            const u32x2 c = list[i];
            if (is_taken(c, kth, tie_cut)) {
                atomicOr(&bits[c.y >> 5], 1u << (c.y & 31u));
                const uint32_t one = 1u << ((c.y & 3u) * 8u);
                if (which) atomicSub(&msum32[c.y >> 2], one);
                else       atomicAdd(&msum32[c.y >> 2], one);
            }
        }
    }
}

// Ordered compaction of the N scratch bitmaps, in two kernels: marked additions and
// removals per block of kBitBlockWords words, then (prefix over the blocks before + scan
// inside the block) each thread writes its marked coordinates in ascending order to the
// add list or the drop list.  The second kernel also clears the scratch words and folds
// them into the standing vote.  Without a standing vote (vote_bits == nullptr) every
// marked coordinate counts as an addition: a plain ordered compaction.
__device__ __forceinline__ void compact_count_block(const uint32_t* __restrict__ ad_bits, uint32_t nwords_pad,
                                                    uint32_t nblk, u32x2* __restrict__ blk_cnt,
                                                    const uint32_t* __restrict__ vote_bits, int64_t ld_bits,
                                                    uint32_t r, uint32_t bx, uint64_t* scan_lds)
{
    const uint32_t* vrow = vote_bits ? vote_bits + (int64_t)r * ld_bits : nullptr;
    uint32_t n_add = 0, n_drop = 0;
#pragma unroll
    for (int it = 0; it < kBitIt; ++it) {
        const uint32_t w0 = bx * kBitBlockWords + ((uint32_t)it * kVoteThreads + threadIdx.x) * 4;
        if (w0 < nwords_pad) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(ad_bits + (size_t)r * nwords_pad + w0);
            const uint32_t m[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (m[q]) {                       // rare: the standing vote's word decides which is which
                    const uint32_t in_vote = vrow ? vrow[w0 + q] : 0u;
                    n_add += __popc(m[q] & ~in_vote);
                    n_drop += __popc(m[q] & in_vote);
                }
            }
        }
    }
    uint64_t total;
    (void)block_excl_scan64<kVoteThreads>(pack2(n_add, n_drop), scan_lds, total);
    if (threadIdx.x == 0) {
        u32x2 c;
        c.x = (uint32_t)(total >> 32);
        c.y = (uint32_t)total;
        blk_cnt[(size_t)r * nblk + bx] = c;
    }
}
// Histogram of the vote levels of msum (one byte per coordinate, values 0..N) over a
// block of kVoteBlock coordinates: lvl_sets[set][v] += coordinates with exactly v votes.
__device__ __forceinline__ void ad_levels_block(const uint32_t* __restrict__ msum32, int64_t d,
                                                uint32_t* __restrict__ lvl_sets, uint32_t bx, uint32_t* h /*256*/)
{
    // all of the block's words first: a load placed after the LDS atomics of the previous
    // round would wait for its full latency every round
    constexpr int kIt = kVoteBlock / (kVoteThreads * 16);
    const int64_t base = (int64_t)bx * kVoteBlock;
    u32x4 w[kIt];
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        w[it] = (j < d) ? *reinterpret_cast<const u32x4*>(msum32 + (j >> 2)) : z;
    }
    h[threadIdx.x] = 0;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        if (j < d) {
            const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
            if ((ww[0] | ww[1] | ww[2] | ww[3]) != 0u) {     // most coordinates have no vote
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                    if (v && j + q < d) atomicAdd(&h[v], 1u);
                }
            }
        }
    }
    __syncthreads();
    const uint32_t c = h[threadIdx.x];
    if (c && threadIdx.x) atomicAdd(&lvl_sets[(size_t)(bx % kLvlSets) * 256 + threadIdx.x], c);
}

// One launch after mv_ad_apply: the first n_count_blocks workgroups count the additions
// and removals marked in the scratch bitmaps per block (row = id / nblk), the others take
// the histogram of msum's levels.
__global__ __launch_bounds__(kVoteThreads) void mv_ad_compact_count(const uint32_t* __restrict__ ad_bits,
                                                                    uint32_t nwords_pad, uint32_t nblk,
                                                                    u32x2* __restrict__ blk_cnt,
                                                                    const uint32_t* __restrict__ vote_bits,
                                                                    int64_t ld_bits, uint32_t n_count_blocks,
                                                                    const uint32_t* __restrict__ msum32, int64_t d,
                                                                    uint32_t* __restrict__ lvl_sets)
{
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    __shared__ uint32_t h[256];
    if (blockIdx.x < n_count_blocks)
        compact_count_block(ad_bits, nwords_pad, nblk, blk_cnt, vote_bits, ld_bits, blockIdx.x / nblk,
                            blockIdx.x % nblk, scan_lds);
    else
        ad_levels_block(msum32, d, lvl_sets, blockIdx.x - n_count_blocks, h);
}

__global__ __launch_bounds__(kVoteThreads) void mv_ad_compact_emit(uint32_t* __restrict__ ad_bits,
                                                                   uint32_t nwords_pad, uint32_t nblk,
                                                                   const u32x2* __restrict__ blk_cnt,
                                                                   uint32_t k_ad,
                                                                   uint32_t* __restrict__ add_idx,
                                                                   uint32_t* __restrict__ drop_idx,
                                                                   uint32_t* __restrict__ vote_bits,
                                                                   int64_t ld_bits)
{
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    const uint32_t row = blockIdx.y;
    uint32_t* vrow = vote_bits ? vote_bits + (int64_t)row * ld_bits : nullptr;   // null: compaction only, all additions
    // the block's words first (cleared behind): their latency overlaps the prefix's loads
    uint32_t w[kBitIt][4], in_vote[kBitIt][4];
#pragma unroll
    for (int it = 0; it < kBitIt; ++it) {
        const uint32_t w0 = blockIdx.x * kBitBlockWords + ((uint32_t)it * kVoteThreads + threadIdx.x) * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) w[it][q] = in_vote[it][q] = 0;
        if (w0 < nwords_pad) {
            u32x4* p = reinterpret_cast<u32x4*>(ad_bits + (size_t)row * nwords_pad + w0);
            const u32x4 v = *p;
            w[it][0] = v.x; w[it][1] = v.y; w[it][2] = v.z; w[it][3] = v.w;
            if ((v.x | v.y | v.z | v.w) != 0u) {
                const u32x4 z = {0u, 0u, 0u, 0u};
                *p = z;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (w[it][q] && vrow) in_vote[it][q] = vrow[w0 + q];
            }
        }
    }
    uint64_t mine = 0;
    for (uint32_t b = threadIdx.x; b < blockIdx.x; b += kVoteThreads) {
        const u32x2 c = blk_cnt[(size_t)row * nblk + b];
        mine += pack2(c.x, c.y);
    }
    uint64_t before;
    (void)block_excl_scan64<kVoteThreads>(mine, scan_lds, before);
    __syncthreads();
    uint32_t* out_add = add_idx + (size_t)row * k_ad;
    uint32_t* out_drop = drop_idx ? drop_idx + (size_t)row * k_ad : nullptr;
    uint64_t done = before;                       // (additions, removals) before the current quad row
#pragma unroll
    for (int it = 0; it < kBitIt; ++it) {
        const uint32_t w0 = blockIdx.x * kBitBlockWords + ((uint32_t)it * kVoteThreads + threadIdx.x) * 4;
        uint32_t n_add = 0, n_drop = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            n_add += __popc(w[it][q] & ~in_vote[it][q]);
            n_drop += __popc(w[it][q] & in_vote[it][q]);
        }
        uint64_t total;
        const uint64_t at = done + block_excl_scan64<kVoteThreads>(pack2(n_add, n_drop), scan_lds, total);
        uint32_t pos_add = (uint32_t)(at >> 32), pos_drop = (uint32_t)at;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t m = w[it][q];
            if (m && vrow) atomicXor(&vrow[w0 + q], m);     // additions enter the standing vote, removals leave it
            while (m) {
                const uint32_t b = __ffs((int)m) - 1;
                m &= m - 1;
                const uint32_t j = (w0 + q) * 32 + b;
                if ((in_vote[it][q] >> b) & 1u) {
                    if (out_drop && pos_drop < k_ad) out_drop[pos_drop] = j;
                    ++pos_drop;
                } else {
                    if (pos_add < k_ad) out_add[pos_add] = j;
                    ++pos_add;
                }
            }
        }
        done += total;
        __syncthreads();
    }
}

}  // namespace mvk
