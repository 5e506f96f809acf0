// Majority voting with random selection (Algorithm 1, the S_rand-weighted line).
#pragma once

#include "mv_common.hpp"
#include "mv_select.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// 8. majority voting with random selection (Algorithm 1, the S_rand-weighted line;
//    Sec. 2, paragraph after Algorithm 1; Sec. 4.2)
// ----------------------------------------------------------------------------
// Winners are drawn in proportion to their votes until K distinct ones are
// selected.  Stated without an order of draws: every voted coordinate j gets an
// exponential clock of rate votes[j], i.e. the time rand_exp[j] / votes[j] with
// rand_exp[j] ~ Exp(1) from the caller, and the K clocks that ring first win
// (equal times: lowest coordinate first).  The time is one correctly rounded fp32
// division; its bit pattern, complemented, is a key for the same exact select
// that serves the rows: list of (key, coordinate), a histogram of the key's 11
// leading bits, the members of the bin that holds the K-th, their exact ranking.
// Selected coordinates are marked in a bitmap that an ordered compaction turns
// into the ascending mask.

// Scan of the packed vote bytes (grid as for the mask kernels): every voted
// coordinate is appended to the list with its key.  rs_count[0] = list length.
__device__ __forceinline__ u32x2 rs_entry(const float* __restrict__ rand_exp, uint32_t j, uint32_t v)
{
    const float time = __fdiv_rn(rand_exp[j], (float)v);
    u32x2 c;
    c.x = kAbsMask - (__float_as_uint(time) & kAbsMask);            // sooner = larger key
    c.y = j;
    return c;
}
__global__ __launch_bounds__(kVoteThreads) void mv_rs_keys(const uint32_t* __restrict__ votes32, int64_t d,
                                                           const float* __restrict__ rand_exp,
                                                           u32x2* __restrict__ list, uint32_t list_cap,
                                                           uint32_t* __restrict__ rs_count)
{
    constexpr int kIt = kVoteBlock / (kVoteThreads * 16);
    constexpr int kPerIt = kVoteThreads * 16;                      // coordinates per round: all may hold a vote
    __shared__ uint32_t stage[kPerIt];
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    __shared__ uint32_t base_sh;
    const int64_t base = (int64_t)blockIdx.x * kVoteBlock;
    u32x4 w[kIt];
    uint32_t n = 0;
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        w[it] = (j < d) ? *reinterpret_cast<const u32x4*>(votes32 + (j >> 2)) : z;   // bytes past d are zero
    }
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
#pragma unroll
        for (int q = 0; q < 16; ++q) n += ((ww[q >> 2] >> (8 * (q & 3))) & 255u) != 0u;
    }
    uint64_t total;
    const uint64_t ex = block_excl_scan64<kVoteThreads>(n, scan_lds, total);
    if (total == 0) return;                                        // whole workgroup
    if (threadIdx.x == 0) base_sh = atomicAdd(&rs_count[0], (uint32_t)total);
    if (total <= (uint64_t)kPerIt) {                               // uniform; usual case: one round for the whole block
        uint32_t sp = (uint32_t)ex;
        if (n) {
#pragma unroll
            for (int it = 0; it < kIt; ++it) {
                if ((w[it].x | w[it].y | w[it].z | w[it].w) == 0u) continue;
                const uint32_t off0 = ((uint32_t)it * kVoteThreads + threadIdx.x) * 16;
                const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
                for (int q = 0; q < 16; ++q) {
                    const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                    if (v) stage[sp++] = ((off0 + (uint32_t)q) << 8) | v;
                }
            }
        }
        __syncthreads();
        const uint32_t at = base_sh;
        for (uint32_t i = threadIdx.x; i < (uint32_t)total; i += kVoteThreads) {
            const uint32_t s = stage[i];
            if (at + i < list_cap) list[at + i] = rs_entry(rand_exp, (uint32_t)base + (s >> 8), s & 255u);
        }
        return;
    }
    __syncthreads();
    uint32_t first = base_sh;                                      // list position of the round's first entry
    // A block crowded with votes (the mask concentrates in few tensors), round by round of
    // 4096 coordinates.  Either way the voted coordinates are parked in LDS as (offset,
    // votes) and their random numbers then fetched by all lanes together: one dependent load
    // per entry inside each thread's own loop made this kernel 2.5x slower, and 8x slower
    // on crowded blocks.
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
        uint32_t n_it = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) n_it += ((ww[q >> 2] >> (8 * (q & 3))) & 255u) != 0u;
        uint64_t round_total;
        uint32_t sp = (uint32_t)block_excl_scan64<kVoteThreads>(n_it, scan_lds, round_total);
        if (n_it) {
            const uint32_t off0 = ((uint32_t)it * kVoteThreads + threadIdx.x) * 16;   // offset in the block
            for (int q = 0; q < 16; ++q) {
                const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                if (v) stage[sp++] = ((off0 + (uint32_t)q) << 8) | v;
            }
        }
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < (uint32_t)round_total; i += kVoteThreads) {
            const uint32_t s = stage[i];
            if (first + i < list_cap) list[first + i] = rs_entry(rand_exp, (uint32_t)base + (s >> 8), s & 255u);
        }
        first += (uint32_t)round_total;
        __syncthreads();
    }
}

// ---- random selection: one list (row 0); winners are marked in the bitmap
__global__ __launch_bounds__(kRowThreads) void mv_rs_hist(ListSelect a)
{
    __shared__ uint32_t hist[kSelBins];
    list_hist_body(a, 0, hist);
}
__global__ __launch_bounds__(kRowThreads) void mv_rs_split(ListSelect a, uint32_t* __restrict__ rs_bits)
{
    __shared__ ListSplitLds lds;
    list_split_body(a, 0, lds, rs_bits);
}
// Also leaves the list's length at zero for the next step.
__global__ __launch_bounds__(kRowThreads) void mv_rs_rank(ListSelect a, uint32_t* __restrict__ rs_count,
                                                          uint32_t* __restrict__ rs_bits)
{
    __shared__ SelectLds lds;
    uint32_t kth, tie_cut, path;
    const uint32_t C = min(a.count2[0], a.cap);
    const bool ranked = list_rank_body(a, 0, lds, kth, tie_cut, path);
    __syncthreads();
    if (threadIdx.x == 0) rs_count[0] = 0;
    if (!ranked) return;
    const u32x2* list2 = a.list2;
    for (uint32_t i = threadIdx.x; i < C; i += kRowThreads) {
        const u32x2 c = list2[i];
        if (is_taken(c, kth, tie_cut)) atomicOr(&rs_bits[c.y >> 5], 1u << (c.y & 31u));
    }
}

}  // namespace mvk
