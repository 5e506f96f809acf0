// Threshold estimate (sample histogram, pick) and the one streaming pass over g and e.
#pragma once

#include "mv_common.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// One kernel: threshold estimate (sample histogram, pick) and the streaming pass
// ----------------------------------------------------------------------------
// The grid is one-dimensional.  Its first N * spr workgroups sample the rows (spr
// per row); the last of a row's sampling workgroups to finish turns the row's
// histogram into the threshold estimate tau and publishes it.  All other workgroups
// stream: a wavefront owns a segment of 1024 coordinates, loads g and e, stores
// a = g + e, and only then needs tau to pick its candidates -- by which time the
// few sampling workgroups, which were started first, have long finished, except for
// the very first streaming workgroups, which wait a few microseconds.  The estimate
// therefore costs no launch of its own and overlaps the head of the streaming pass.
//
// The streaming pass overwrites e, which the sampling reads: a streaming wavefront
// holds back its stores until all of its row's sampling workgroups have their samples
// in registers (reads_done[row], a counter that only ever grows: spr per step).  That
// happens a few microseconds into the kernel, before the first streaming loads are
// back.  (Were a store to slip in early, the estimate would see a = g + e in place of e
// at that spot: a worse estimate, the same result.)
//
// The wait is bounded: a wavefront that has polled spin_limit times without seeing
// its row's tau marks the row (row_poison[row] = this step's number) and goes on
// without candidates; mv_row_select then reads the row's count as overflowed and
// selects the row exactly from memory, like any row whose estimate failed.  The
// result never depends on the estimate, only the time does.
//
// What crosses between workgroups inside the kernel travels through atomics only
// (the histogram, the counters, the published tau), which are performed in memory;
// ordinary stores of one workgroup are not visible to another before the kernel ends.
//
// Sampling: chunk c of a row is the coordinates [32c, 32c+32); chunk c is sampled
// when c % stride == 0.  bin = (bits(|g+e|)) >> kHistShift.  tau = lower edge of the
// highest bin such that at least m_target sampled coordinates lie in that bin or
// above (0 if fewer).  The picking workgroup also clears the row's histogram and
// resets the per-step counters.
//
// Streaming: one wavefront = one segment of 1024 consecutive coordinates of one row,
// read as 4 sub-blocks of 256 (lane l holds coordinates base + 256u + 4l .. +3); a
// workgroup of 8 wavefronts covers 8 consecutive segments.  Coordinates with
// (bits(a) & 0x7FFFFFFF) >= tau are appended to the row's candidate list as
// (magnitude bits, coordinate), in ascending coordinate order inside the wavefront's
// run; seg[row][s] = (start of the run, its length).  Runs land in the list in any
// order; the table makes the order recoverable.  The workgroup reserves list space
// for all its runs with ONE atomic on the row's counter (returning atomics on one
// cache line complete only every few nanoseconds chip-wide, so one per wavefront
// would bound the whole pass when candidates are spread evenly).  Entries beyond
// `cap` are dropped, the counter keeps counting (the overflow is detected from it).
constexpr int      kSampleQuads = 4;              // quads of samples a sampling thread has in flight
constexpr uint32_t kRowPoison = 0x80000000u;      // set in a marked row's candidate counter by mv_row_select

struct StreamLds {
    uint32_t h[kHistBins];                        // sampling workgroups only
    uint64_t scan[kStreamThreads / kWave + 1];
    uint32_t found, is_last;
    uint32_t wave_total[kSegPerBlock];
    uint32_t block_base;
};

template <typename GT>
__device__ __forceinline__ void sample_and_pick(StreamLds& lds, const GT* __restrict__ g, int64_t ld_g,
                                                const float* __restrict__ e, int64_t ld_e, int64_t d,
                                                uint32_t row, uint32_t part, uint32_t spr, uint32_t stride,
                                                uint32_t n_sampled_chunks, uint32_t m_target,
                                                uint32_t* __restrict__ hist, uint32_t* __restrict__ sample_done,
                                                uint32_t* __restrict__ reads_done,
                                                unsigned long long* __restrict__ tau_pub, uint32_t epoch,
                                                uint32_t* __restrict__ next_row_count, uint32_t* __restrict__ lvl_sets,
                                                uint32_t n_lvl_words, uint32_t n_rows,
                                                uint32_t* __restrict__ ad_count)
{
    const uint32_t t = threadIdx.x;
    for (int b = t; b < kHistBins; b += kStreamThreads) lds.h[b] = 0;
    __syncthreads();
    const GT*    grow = g + (int64_t)row * ld_g;
    const float* erow = e + (int64_t)row * ld_e;
    const uint64_t nquads = (uint64_t)n_sampled_chunks * (kChunk / 4);
    const uint64_t step = (uint64_t)spr * kStreamThreads;
    auto start_of = [stride](uint64_t q) {
        return (int64_t)(q / (kChunk / 4)) * stride * kChunk + (int64_t)(q % (kChunk / 4)) * 4;
    };
    auto tally = [&](float a) { atomicAdd(&lds.h[(__float_as_uint(a) & kAbsMask) >> kHistShift], 1u); };
    // The samples lie far apart in memory and every load pays the full latency: kSampleQuads
    // quads' loads are in flight per thread and the grid is sized for one or two rounds.
    for (uint64_t q0 = (uint64_t)part * kStreamThreads + t; q0 < nquads; q0 += kSampleQuads * step) {
        f32x4 gv[kSampleQuads], ev[kSampleQuads];
        bool  full[kSampleQuads];
#pragma unroll
        for (int u = 0; u < kSampleQuads; ++u) {
            const uint64_t q = q0 + (uint64_t)u * step;
            const int64_t j = start_of(q);
            full[u] = q < nquads && j + 4 <= d;
            if (full[u]) {
                gv[u] = load4_grad(grow + j);
                ev[u] = *reinterpret_cast<const f32x4*>(erow + j);
            }
        }
#pragma unroll
        for (int u = 0; u < kSampleQuads; ++u) {
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
    // every sample of this workgroup has been used, so it has arrived: the row's streaming
    // wavefronts may overwrite e as far as this workgroup is concerned
    if (t == 0) atomicAdd(&reads_done[row * kCounterStride], 1u);
    uint32_t* hrow = hist + (size_t)row * kHistBins;
    for (int b = t; b < kHistBins; b += kStreamThreads) {
        const uint32_t c = lds.h[b];
        if (c) atomicAdd(&hrow[b], c);
    }
    // every atomic of this workgroup has been performed before it is counted as done
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t == 0) lds.is_last = atomicAdd(&sample_done[row * kCounterStride], 1u) == spr - 1u;
    __syncthreads();
    if (!lds.is_last) return;                     // whole workgroup

    // ---- the row's last sampling workgroup: histogram -> tau
    constexpr int per = kHistBins / kStreamThreads;   // bins per thread, descending bin order
    uint32_t c[per];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {               // read from memory, where the others' atomics went
        const int bin = kHistBins - 1 - ((int)t * per + q);
        c[q] = __hip_atomic_load(&hrow[bin], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll
    for (int q = 0; q < per; ++q) sum += c[q];
    if (t == 0) lds.found = 0;
    uint64_t total;
    const uint64_t excl = block_excl_scan64<kStreamThreads>(sum, lds.scan, total);
    if (excl < m_target && (uint64_t)m_target <= excl + sum) {
        uint64_t acc = excl;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            if (acc < m_target && (uint64_t)m_target <= acc + c[q])
                lds.found = (uint32_t)(kHistBins - 1 - ((int)t * per + q)) << kHistShift;
            acc += c[q];
        }
    }
    __syncthreads();
    if (t == 0) {
        const uint32_t tau = (total >= m_target) ? lds.found : 0u;
        __hip_atomic_store(&tau_pub[row * (kCounterStride / 2)], ((unsigned long long)epoch << 32) | tau,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Behind the publication, what the NEXT step's kernel must find at zero (ordinary stores: they
    // are in memory when this kernel has ended): the histogram, the sampling counter, the row's
    // candidate counter of the other parity (this step's streaming workgroups bump row_count; the
    // next step's bump next_row_count), the add / drop list lengths, the vote-level counters.
#pragma unroll
    for (int q = 0; q < per; ++q) hrow[kHistBins - 1 - ((int)t * per + q)] = 0;
    if (t == 0) {
        sample_done[row * kCounterStride] = 0;
        next_row_count[row * kCounterStride] = 0;
    }
    if (ad_count && t < 2) ad_count[ad_counter(row, t)] = 0;
    for (uint32_t i = row * kStreamThreads + t; i < n_lvl_words; i += n_rows * kStreamThreads) lvl_sets[i] = 0;
}

template <typename GT>
__global__ __launch_bounds__(kStreamThreads) void mv_stream_collect(
    const GT* __restrict__ g, int64_t ld_g, float* __restrict__ e, int64_t ld_e, int64_t d, uint32_t n_rows,
    uint32_t spr, uint32_t stride, uint32_t n_sampled_chunks, uint32_t m_target,
    uint32_t* __restrict__ hist, uint32_t* __restrict__ sample_done, uint32_t* __restrict__ reads_done,
    unsigned long long* __restrict__ tau_pub, const uint32_t* __restrict__ step_no, uint32_t spin_limit, uint32_t* __restrict__ row_poison, uint32_t* __restrict__ lvl_sets,
    uint32_t n_lvl_words, uint32_t* __restrict__ ad_count,
    u32x2* __restrict__ cand, uint32_t cap, uint32_t* __restrict__ row_count_sets, uint32_t row_count_set_words,
    u32x2* __restrict__ seg,
    uint32_t* __restrict__ seg_sel, uint32_t nseg, uint32_t wgs_per_row, uint32_t head_wgs,
    uint32_t* __restrict__ zero_votes32, int64_t votes_bytes)
{
    __shared__ StreamLds lds;
    // The step's number lives on the device (the step's last kernel counts it up), so that a
    // captured step can be replayed; the rows' candidate counters exist twice, and this step
    // counts into the set of its parity while it clears the other one for the next step.
    const uint32_t epoch = step_no[0] + 1u;
    uint32_t* row_count = row_count_sets + (epoch & 1u) * row_count_set_words;
    uint32_t* next_row_count = row_count_sets + ((epoch & 1u) ^ 1u) * row_count_set_words;
    if (blockIdx.x < n_rows * spr) {
        sample_and_pick<GT>(lds, g, ld_g, e, ld_e, d, blockIdx.x / spr, blockIdx.x % spr, spr, stride, n_sampled_chunks,
                            m_target, hist, sample_done, reads_done, tau_pub, epoch, next_row_count, lvl_sets, n_lvl_words,
                            n_rows, ad_count);
        return;
    }
    const uint32_t sb = blockIdx.x - n_rows * spr;
    const uint32_t row = sb / wgs_per_row, bx = sb % wgs_per_row;
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    const uint32_t s = bx * kSegPerBlock + wave;
    const bool live = s < nseg;                  // whole wavefront; dead ones only keep the barriers company
    const int64_t base = (int64_t)s * kSeg;
    const GT* grow = g + (int64_t)row * ld_g;
    float*    erow = e + (int64_t)row * ld_e;
    const unsigned long long* tau_at = tau_pub + row * (kCounterStride / 2);
    // a first look at the row's tau together with the data loads: after the kernel's first
    // microseconds it is there, and the wavefront never waits
    unsigned long long tw = __hip_atomic_load(tau_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t* rd_at = reads_done + row * kCounterStride;
    const uint32_t rd_target = spr * epoch;       // the counter grows by spr per step and wraps with this product
    uint32_t rd = __hip_atomic_load(rd_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t spins = 0;
    // (all lanes of a wavefront load the same words, so the waits below are wave-uniform)
    auto samples_are_in = [&]() {
        while ((int32_t)(rd - rd_target) < 0 && spins < spin_limit) {
            __builtin_amdgcn_s_sleep(8);
            rd = __hip_atomic_load(rd_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ++spins;
        }
    };

    // The kernel's first streaming workgroups would compete with the sampling for the memory
    // system and delay the estimate for everybody: they hold back even their loads.
    if (sb < head_wgs) samples_are_in();

    uint32_t key[16];
    uint32_t inside = 0;                          // bit i: key[i] is a coordinate of the row
    if (live && base + kSeg <= d) {
        f32x4 gv[4], ev[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = base + u * 256 + lane * 4;
            gv[u] = load4_grad(grow + j);
            ev[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(erow + j));
        }
        // (the counter's load was issued before the data loads, so looking at it waits for none of them;
        // each sub-block is stored as soon as its own loads are back: stores in one burst run slower)
        samples_are_in();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = base + u * 256 + lane * 4;
            const f32x4 a = gv[u] + ev[u];
            __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(erow + j));
            key[u * 4 + 0] = __float_as_uint(a.x) & kAbsMask;
            key[u * 4 + 1] = __float_as_uint(a.y) & kAbsMask;
            key[u * 4 + 2] = __float_as_uint(a.z) & kAbsMask;
            key[u * 4 + 3] = __float_as_uint(a.w) & kAbsMask;
        }
        inside = 0xFFFFu;
    } else if (live) {
        // last segment of the row: element-wise, nothing past d is read or written
        samples_are_in();
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
                    inside |= 1u << (u * 4 + c);
                }
                key[u * 4 + c] = k;
            }
    }

    // tau: wait for it if need be (bounded), then the candidates' flags
    while ((uint32_t)(tw >> 32) != epoch && spins < spin_limit) {
        __builtin_amdgcn_s_sleep(16);
        tw = __hip_atomic_load(tau_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ++spins;
    }
    uint32_t tau = (uint32_t)tw;
    if ((uint32_t)(tw >> 32) != epoch) {                               // not seen in time: the row goes the exact way
        tau = 0xFFFFFFFFu;                                             // above every key
        if (lane == 0) atomicMax(&row_poison[row], epoch);             // step numbers only grow: never reset
    }
    uint32_t flags = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) flags |= (key[i] >= tau ? 1u : 0u) << i;
    flags &= inside;

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
    if (lane == 0) lds.wave_total[wave] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t sum = 0;
#pragma unroll
        for (int w = 0; w < kSegPerBlock; ++w) {
            const uint32_t t = lds.wave_total[w];
            lds.wave_total[w] = sum;
            sum += t;
        }
        lds.block_base = sum ? atomicAdd(&row_count[row * kCounterStride], sum) : 0u;
    }
    __syncthreads();
    const uint32_t run_start = lds.block_base + lds.wave_total[wave];
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
    // Row 0's wavefronts pass over every coordinate once: they also clear the packed vote bytes
    // (one per coordinate, 16 per lane), which the kernels that follow fill and read.
    if (zero_votes32 && row == 0 && live) {
        const int64_t j = base + (int64_t)lane * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        if (j < votes_bytes) *reinterpret_cast<u32x4*>(zero_votes32 + (j >> 2)) = z;
    }
    if (live && lane == 0) {
        u32x2 rec;
        rec.x = run_start;
        rec.y = total;
        seg[(size_t)row * nseg + s] = rec;
        seg_sel[(size_t)row * nseg + s] = 0;     // tallied when the votes are cast
    }
}

}  // namespace mvk
