// Threshold estimate (sample histogram, pick) and the one streaming pass over g and e.
#pragma once

#include "mv_common.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// 1. sample histogram and threshold estimate
// ----------------------------------------------------------------------------
// Chunk c of a row is the coordinates [32c, 32c+32); chunk c is sampled when
// c % stride == 0.  bin = (bits(|g+e|)) >> kHistShift.  Workgroups of a row add
// their LDS histograms into the row's global one.
constexpr int kSampleThreads = 1024;
template <typename GT>
__global__ __launch_bounds__(kSampleThreads) void mv_sample_hist(const GT* __restrict__ g, int64_t ld_g,
                                                                 const float* __restrict__ e, int64_t ld_e,
                                                                 int64_t d, uint32_t stride,
                                                                 uint32_t n_sampled_chunks,
                                                                 uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[kHistBins];
    const uint32_t row = blockIdx.y, t = threadIdx.x;
    for (int b = t; b < kHistBins; b += kSampleThreads) h[b] = 0;
    __syncthreads();

    const GT*    grow = g + (int64_t)row * ld_g;
    const float* erow = e + (int64_t)row * ld_e;
    const uint64_t nquads = (uint64_t)n_sampled_chunks * (kChunk / 4);
    const uint64_t step = (uint64_t)gridDim.x * kSampleThreads;
    auto start_of = [stride](uint64_t q) {
        return (int64_t)(q / (kChunk / 4)) * stride * kChunk + (int64_t)(q % (kChunk / 4)) * 4;
    };
    auto tally = [&](float a) { atomicAdd(&h[(__float_as_uint(a) & kAbsMask) >> kHistShift], 1u); };
    // The samples lie far apart in memory and every load pays the full latency: two
    // quads' loads are in flight per thread and the grid is sized for one or two rounds.
    for (uint64_t q0 = (uint64_t)blockIdx.x * kSampleThreads + t; q0 < nquads; q0 += 2 * step) {
        f32x4 gv[2], ev[2];
        bool  full[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint64_t q = q0 + (uint64_t)u * step;
            const int64_t j = start_of(q);
            full[u] = q < nquads && j + 4 <= d;
            if (full[u]) {
                gv[u] = load4_grad(grow + j);
                ev[u] = *reinterpret_cast<const f32x4*>(erow + j);
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint64_t q = q0 + (uint64_t)u * step;
            if (full[u]) {
                const f32x4 a = gv[u] + ev[u];
                tally(a.x);
                tally(a.y);
                tally(a.z);
                tally(a.w);
            } else if (q < nquads) {
                for (int64_t jj = start_of(q); jj < d; ++jj) tally(load1_grad(grow + jj) + erow[jj]);
            }
        }
    }
    __syncthreads();
    uint32_t* hrow = hist + (size_t)row * kHistBins;
    for (int b = t; b < kHistBins; b += kSampleThreads) {
        uint32_t c = h[b];
        if (c) atomicAdd(&hrow[b], c);
    }
}

// One workgroup per row:
//   tau_bits[row] = lower edge of the highest bin such that at least m_target
//                   sampled coordinates lie in that bin or above (0 if fewer).
// The histogram is cleared after it is read so the next step starts from zero,
// and the row's per-step counters are reset.
__global__ __launch_bounds__(kRowThreads) void mv_pick_threshold(uint32_t* __restrict__ hist,
                                                                 uint32_t m_target,
                                                                 uint32_t* __restrict__ tau_bits,
                                                                 uint32_t* __restrict__ row_count,
                                                                 uint32_t* __restrict__ slow_flag,
                                                                 uint32_t* __restrict__ cnt_ge,
                                                                 uint32_t* __restrict__ ad_count)
{
    __shared__ uint64_t scan_lds[kRowThreads / kWave + 1];
    __shared__ uint32_t found;
    const uint32_t row = blockIdx.x, t = threadIdx.x;
    if (ad_count && t < 2) ad_count[ad_counter(row, t)] = 0;   // lengths of the row's add / drop candidate lists
    uint32_t* hrow = hist + (size_t)row * kHistBins;
    constexpr int per = kHistBins / kRowThreads;   // bins per thread, descending bin order
    uint32_t c[per];
    uint32_t s = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        const int bin = kHistBins - 1 - ((int)t * per + q);
        c[q] = hrow[bin];
        hrow[bin] = 0;
        s += c[q];
    }
    if (t == 0) {
        found = 0;
        row_count[row * kCounterStride] = 0;
        slow_flag[row] = 0;
    }
    if (t < 256) cnt_ge[(size_t)row * 256 + t] = 0;   // the row's 256 vote-level counters
    uint64_t total;
    const uint64_t excl = block_excl_scan64<kRowThreads>(s, scan_lds, total);
    if (excl < m_target && (uint64_t)m_target <= excl + s) {
        uint64_t acc = excl;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            if (acc < m_target && (uint64_t)m_target <= acc + c[q])
                found = (uint32_t)(kHistBins - 1 - ((int)t * per + q)) << kHistShift;
            acc += c[q];
        }
    }
    __syncthreads();
    if (t == 0) tau_bits[row] = (total >= m_target) ? found : 0u;
}

// ----------------------------------------------------------------------------
// 2. the streaming pass
// ----------------------------------------------------------------------------
// One wavefront = one segment of 1024 consecutive coordinates of one row, read
// as 4 sub-blocks of 256 (lane l holds coordinates base + 256u + 4l .. +3); a
// workgroup of 8 wavefronts covers 8 consecutive segments.
// a = g + e overwrites e.  Coordinates with (bits(a) & 0x7FFFFFFF) >= tau are
// appended to the row's candidate list as (magnitude bits, coordinate), in
// ascending coordinate order inside the wavefront's run; seg[row][s] =
// (start of the run, its length).  Runs land in the list in any order; the
// table makes the order recoverable.  The workgroup reserves list space for
// all its runs with ONE atomic on the row's counter (returning atomics on one
// cache line complete only every few nanoseconds chip-wide, so one per
// wavefront would bound the whole pass when candidates are spread evenly).
// Entries beyond `cap` are dropped, the counter keeps counting (the overflow is
// detected from it).
template <typename GT>
__global__ __launch_bounds__(kStreamThreads) void mv_stream_collect(
    const GT* __restrict__ g, int64_t ld_g, float* __restrict__ e, int64_t ld_e, int64_t d,
    const uint32_t* __restrict__ tau_bits, u32x2* __restrict__ cand, uint32_t cap,
    uint32_t* __restrict__ row_count, u32x2* __restrict__ seg, uint32_t* __restrict__ seg_sel,
    uint32_t nseg)
{
    __shared__ uint32_t wave_total[kSegPerBlock];
    __shared__ uint32_t block_base;
    const uint32_t row = blockIdx.y;
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    const uint32_t s = blockIdx.x * kSegPerBlock + wave;
    const bool live = s < nseg;                  // whole wavefront; dead ones only keep the barriers company
    const int64_t base = (int64_t)s * kSeg;
    const GT* grow = g + (int64_t)row * ld_g;
    float*    erow = e + (int64_t)row * ld_e;
    const uint32_t tau = tau_bits[row];

    uint32_t key[16];
    uint32_t flags = 0;
    if (live && base + kSeg <= d) {
        f32x4 gv[4], ev[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = base + u * 256 + lane * 4;
            gv[u] = load4_grad(grow + j);
            ev[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(erow + j));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = base + u * 256 + lane * 4;
            f32x4 a = gv[u] + ev[u];
            __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(erow + j));
            key[u * 4 + 0] = __float_as_uint(a.x) & kAbsMask;
            key[u * 4 + 1] = __float_as_uint(a.y) & kAbsMask;
            key[u * 4 + 2] = __float_as_uint(a.z) & kAbsMask;
            key[u * 4 + 3] = __float_as_uint(a.w) & kAbsMask;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) flags |= (key[i] >= tau ? 1u : 0u) << i;
    } else if (live) {
        // last segment of the row: element-wise, nothing past d is read or written
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int64_t j = base + u * 256 + lane * 4 + c;
                uint32_t k = 0;
                if (j < d) {
                    float a = load1_grad(grow + j) + erow[j];
                    erow[j] = a;
                    k = __float_as_uint(a) & kAbsMask;
                    flags |= (k >= tau ? 1u : 0u) << (u * 4 + c);
                }
                key[u * 4 + c] = k;
            }
    }

    // rank of each kept coordinate inside the wavefront's run
    uint32_t total = 0;
    uint32_t rank[4] = {0, 0, 0, 0};
    const bool any = __ballot(flags != 0) != 0ull;       // wave-uniform
    if (any) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t c = __popc((flags >> (4 * u)) & 15u);
            const uint32_t incl = wave_incl_scan(c);
            rank[u] = total + incl - c;
            total += __shfl(incl, kWave - 1, kWave);
        }
    }
    // one reservation for the workgroup's 8 runs
    if (lane == 0) wave_total[wave] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t sum = 0;
#pragma unroll
        for (int w = 0; w < kSegPerBlock; ++w) {
            const uint32_t t = wave_total[w];
            wave_total[w] = sum;
            sum += t;
        }
        block_base = sum ? atomicAdd(&row_count[row * kCounterStride], sum) : 0u;
    }
    __syncthreads();
    const uint32_t run_start = block_base + wave_total[wave];
    if (any) {
        u32x2* crow = cand + (size_t)row * cap;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (flags & (1u << (u * 4 + c))) {
                    const uint64_t pos = (uint64_t)run_start + rank[u]++;
                    if (pos < cap) {
                        u32x2 rec;
                        rec.x = key[u * 4 + c];
                        rec.y = (uint32_t)(base + u * 256 + lane * 4 + c);
                        crow[pos] = rec;
                    }
                }
    }
    if (live && lane == 0) {
        u32x2 rec;
        rec.x = run_start;
        rec.y = total;
        seg[(size_t)row * nseg + s] = rec;
        seg_sel[(size_t)row * nseg + s] = 0;     // tallied by mv_row_votes
    }
}

}  // namespace mvk
