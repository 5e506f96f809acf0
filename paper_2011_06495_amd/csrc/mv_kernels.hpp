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

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mvk {

typedef float    f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

constexpr int      kWave           = 64;
constexpr int      kSeg            = 1024;   // coordinates per wavefront segment in the streaming pass
constexpr int      kStreamThreads  = 512;    // 8 segments per workgroup
constexpr int      kSegPerBlock    = kStreamThreads / kWave;
constexpr int      kHistBits       = 13;     // sample histogram: exponent + 5 mantissa bits
constexpr int      kHistBins       = 1 << kHistBits;
constexpr int      kHistShift      = 31 - kHistBits;
constexpr int      kChunk          = 32;     // sampled chunk: 32 coordinates (one 128-byte line of fp32)
constexpr int      kRowThreads     = 1024;   // mv_pick_threshold / mv_row_select: one workgroup per row
constexpr int      kVoteBlock      = 16384;  // coordinates per workgroup in mv_mask_count / mv_mask_emit
constexpr int      kVoteThreads    = 256;
constexpr int      kGatherThreads  = 256;
constexpr int      kMaxScanBlocks  = 2048;   // blocks of 1024 segments in a row of up to 2^31 coordinates
constexpr uint32_t kAbsMask        = 0x7FFFFFFFu;
constexpr int      kFineBins       = 2048;   // mv_row_select: histogram of the candidates' magnitudes above tau
constexpr int      kFineShift      = 12;     // 2048 bins of 4096 bit patterns = one octave above tau

// ----------------------------------------------------------------------------
// small helpers
// ----------------------------------------------------------------------------

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        uint32_t t = __shfl_up(v, o, kWave);
        if (lane >= (uint32_t)o) v += t;
    }
    return v;
}

__device__ __forceinline__ uint64_t wave_incl_scan64(uint64_t v)
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        uint64_t t = __shfl_up((unsigned long long)v, o, kWave);
        if (lane >= (uint32_t)o) v += t;
    }
    return v;
}

// Exclusive scan of one 64-bit value per thread over the whole workgroup
// (thread order).  `lds` holds NT/64 + 1 entries.  Returns the exclusive prefix;
// `total` receives the workgroup sum.  Ends with the LDS scratch free to reuse
// only after the caller's next __syncthreads().
template <int NT>
__device__ __forceinline__ uint64_t block_excl_scan64(uint64_t v, uint64_t* lds, uint64_t& total)
{
    constexpr int NW = NT / kWave;
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    uint64_t incl = wave_incl_scan64(v);
    if (lane == kWave - 1) lds[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        uint64_t w = (lane < (uint32_t)NW) ? lds[lane] : 0;
        uint64_t wi = wave_incl_scan64(w);
        if (lane < (uint32_t)NW) lds[lane] = wi - w;
        if (lane == (uint32_t)NW - 1) lds[NW] = wi;
    }
    __syncthreads();
    total = lds[NW];
    return lds[wave] + incl - v;
}

__device__ __forceinline__ uint64_t pack2(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

// bin of a candidate's magnitude key (>= tau) in the row's fine histogram; order preserving
__device__ __forceinline__ uint32_t fine_bin(uint32_t key, uint32_t tau)
{
    return min((key - tau) >> kFineShift, (uint32_t)(kFineBins - 1));
}

// widen four gradient elements to fp32
__device__ __forceinline__ f32x4 load4_grad(const float* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ f32x4 load4_grad(const uint16_t* p)
{
    u16x4 h = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(p));
    f32x4 r;
    r.x = __uint_as_float((uint32_t)h.x << 16);
    r.y = __uint_as_float((uint32_t)h.y << 16);
    r.z = __uint_as_float((uint32_t)h.z << 16);
    r.w = __uint_as_float((uint32_t)h.w << 16);
    return r;
}
__device__ __forceinline__ float load1_grad(const float* p) { return *p; }
__device__ __forceinline__ float load1_grad(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

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

// List length counters (the rows' candidate lists, the add-drop lists): many workgroups
// bump them with returning atomics, which complete one after the other per cache line,
// so every counter has a 128-byte line of its own.
constexpr uint32_t kCounterStride = 32;
__device__ __forceinline__ uint32_t ad_counter(uint32_t row, uint32_t which)
{
    return (2u * row + which) * kCounterStride;
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

// ----------------------------------------------------------------------------
// 3. per-row exact select
// ----------------------------------------------------------------------------

constexpr int kSelBins = 2048;   // radix-select digit: 11, 10, 10 bits of the 31-bit key
constexpr int kKeyBins = 4096;   // exact magnitudes inside one fine-histogram bin (1 << kFineShift)
constexpr int kKeep    = 32;     // candidate keys a thread of mv_row_select can hold in registers
constexpr int kTieCap  = 8192;   // ties with the K-th magnitude that fit the LDS list
constexpr int kRankCap = 256;    // at most this many entries are ranked by counting (quadratic work)

__device__ __forceinline__ int      sel_shift(int pass) { return pass == 0 ? 20 : pass == 1 ? 10 : 0; }
__device__ __forceinline__ uint32_t sel_dmask(int pass) { return pass == 0 ? 2047u : 1023u; }

// Adds one key's digit to the LDS histogram.  Must be called by all lanes of
// the wavefront together.  Gradient magnitudes share a few exponents, so most
// lanes hit the same digit in the first pass: one lane adds the whole group's
// count, the others add their own.
__device__ __forceinline__ void tally_digit(uint32_t* hist, bool active, uint32_t dg, uint32_t lane)
{
    const uint64_t am = __ballot(active);
    if (am != 0ull) {                                   // wave-uniform
        const int      leader = __ffsll((long long)am) - 1;
        const uint32_t ldg = __shfl(dg, leader, kWave);
        const uint64_t same = __ballot(active && dg == ldg);
        if (lane == (uint32_t)leader) atomicAdd(&hist[ldg], (uint32_t)__popcll(same));
        if (active && dg != ldg) atomicAdd(&hist[dg], 1u);
    }
}

// With a histogram of BINS bins complete (bins ordered like the keys): finds the
// bin that holds the `want`-th largest entry.  `bin` receives it, `want_in_bin`
// the rank inside the bin counted from its top (>= 1), `in_bin` the bin's count.
// Requires 1 <= want <= total count.  All kRowThreads threads must call it.
template <int BINS>
__device__ __forceinline__ void find_rank_bin(const uint32_t* hist, uint64_t* scan_lds, uint32_t* bcast,
                                              uint32_t want, uint32_t& bin, uint32_t& want_in_bin,
                                              uint32_t& in_bin)
{
    constexpr int per = BINS / kRowThreads;       // bins per thread, descending bin order over threads
    uint32_t h[per];
    uint32_t s = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        h[q] = hist[BINS - 1 - ((int)threadIdx.x * per + q)];
        s += h[q];
    }
    uint64_t total;
    const uint64_t ex = block_excl_scan64<kRowThreads>(s, scan_lds, total);
    if (ex < want && (uint64_t)want <= ex + s) {
        uint64_t acc = ex;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            if (acc < want && (uint64_t)want <= acc + h[q]) {
                bcast[0] = (uint32_t)(BINS - 1 - ((int)threadIdx.x * per + q));
                bcast[1] = want - (uint32_t)acc;
                bcast[2] = h[q];
            }
            acc += h[q];
        }
    }
    __syncthreads();
    bin = bcast[0];
    want_in_bin = bcast[1];
    in_bin = bcast[2];
    __syncthreads();
}

// Key sources for the selects below.  each(f) calls f(key, i, valid) the same
// number of times in every lane of the workgroup (so f may use wave-wide
// operations); i is the key's position in the source, valid says whether it
// exists.
struct KeysInRegs {                     // thread t holds key number q * kRowThreads + t in k[q]
    const uint32_t (&k)[kKeep];
    uint32_t count;
    template <typename F>
    __device__ __forceinline__ void each(F f) const
    {
#pragma unroll
        for (int q = 0; q < kKeep; ++q) {
            if ((uint32_t)q * kRowThreads < count) {              // uniform over the workgroup
                const uint32_t i = (uint32_t)q * kRowThreads + threadIdx.x;
                f(k[q], (uint64_t)i, i < count);
            }
        }
    }
};
template <typename KeyAt>
struct KeysInMemory {                   // re-read on every pass
    KeyAt    key_at;
    uint64_t count;
    template <typename F>
    __device__ __forceinline__ void each(F f) const
    {
        for (uint64_t base = 0; base < count; base += (uint64_t)kRowThreads * 8) {
            uint32_t k[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint64_t i = base + (uint64_t)u * kRowThreads + threadIdx.x;
                k[u] = (i < count) ? key_at(i) : 0u;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint64_t i = base + (uint64_t)u * kRowThreads + threadIdx.x;
                f(k[u], i, i < count);
            }
        }
    }
};

// Exact K-th largest of the source's keys by an MSB-first radix select
// (11 + 10 + 10 bits) in one workgroup of kRowThreads threads.  Returns the K-th
// largest key; `take_eq` receives how many keys EQUAL to it belong to the top K
// (>= 1) and `n_eq` how many keys equal it in all.  Requires 1 <= K <= count.
template <typename Keys>
__device__ __forceinline__ uint32_t block_radix_select(const Keys& keys, uint32_t K, uint32_t* hist,
                                                       uint64_t* scan_lds, uint32_t* bcast,
                                                       uint32_t& take_eq, uint32_t& n_eq)
{
    const uint32_t lane = lane_id();
    uint32_t prefix = 0, known = 0, remaining = K, in_digit = 0;
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        for (int b = threadIdx.x; b < kSelBins; b += kRowThreads) hist[b] = 0;
        __syncthreads();
        keys.each([&](uint32_t k, uint64_t, bool valid) {
            tally_digit(hist, valid && ((k & known) == prefix), (k >> sel_shift(pass)) & sel_dmask(pass), lane);
        });
        __syncthreads();
        uint32_t digit;
        find_rank_bin<kSelBins>(hist, scan_lds, bcast, remaining, digit, remaining, in_digit);
        prefix |= digit << sel_shift(pass);
        known |= sel_dmask(pass) << sel_shift(pass);
    }
    take_eq = remaining;
    n_eq = in_digit;
    return prefix;
}

// Adds one vote for coordinate j.  Votes are bytes packed four to a word; N <= 255
// keeps a byte from carrying into its neighbour.  lvl[v] counts coordinates that
// just reached v votes (so that, summed over all workgroups, lvl[v] = number of
// coordinates with at least v votes).
__device__ __forceinline__ void cast_vote(uint32_t* __restrict__ votes32, uint32_t j, uint32_t* lvl)
{
    const uint32_t sh = (j & 3u) * 8u;
    const uint32_t old = atomicAdd(&votes32[j >> 2], 1u << sh);
    atomicAdd(&lvl[((old >> sh) & 255u) + 1u], 1u);
}

// A candidate (magnitude bits, coordinate) is in the row's top K iff its
// magnitude is above the K-th largest, or equals it and its coordinate is not
// beyond the last tie taken (ties go to the lowest coordinates).
__device__ __forceinline__ bool is_taken(u32x2 c, uint32_t kth, uint32_t tie_cut)
{
    return c.x > kth || (c.x == kth && c.y <= tie_cut);
}

// LDS of mv_row_select
struct SelectLds {
    __attribute__((aligned(16))) uint32_t hist[kKeyBins];   // histograms; then magnitudes of a bin's members
    __attribute__((aligned(16))) uint32_t ties[kTieCap];    // coordinates of a bin's members / of the ties
    uint32_t lvl[257];
    uint32_t bcast[3];
    uint32_t n_list;
    uint64_t scan[kRowThreads / kWave + 1];
};

// The take-th SMALLEST of the n distinct coordinates in lds.ties[0..n): ranked by
// counting when few; else narrowed by one histogram and then ranked by counting;
// a radix select on (0x7FFFFFFF - coordinate) if they crowd into one bin.
__device__ __forceinline__ uint32_t smallest_coordinate(SelectLds& lds, uint32_t n, uint32_t take)
{
    if (n <= (uint32_t)kRankCap) {
        if (threadIdx.x < 4) lds.ties[n + threadIdx.x] = 0xFFFFFFFFu;   // pad to a multiple of 4, ranked last
        __syncthreads();
        if (threadIdx.x < n) {
            const uint32_t mine = lds.ties[threadIdx.x];
            const u32x4* tv = reinterpret_cast<const u32x4*>(lds.ties);
            uint32_t below = 0;
#pragma unroll 4
            for (uint32_t j = 0; j < (n + 3) / 4; ++j) {
                const u32x4 o = tv[j];
                below += (o.x < mine) + (o.y < mine) + (o.z < mine) + (o.w < mine);
            }
            if (below == take - 1) lds.bcast[0] = mine;
        }
        __syncthreads();
        const uint32_t r = lds.bcast[0];
        __syncthreads();
        return r;
    }
    // Many ties: their coordinates are spread over the row, so one histogram of the
    // coordinate's leading bits (relative to the ties' own range) isolates a handful
    // around the wanted rank, which are then ranked by counting.
    const uint32_t t = threadIdx.x;
    if (t == 0) {
        lds.bcast[0] = 0u;
        lds.bcast[1] = 0xFFFFFFFFu;
    }
    for (int b = t; b < kSelBins; b += kRowThreads) lds.hist[b] = 0;
    __syncthreads();
    uint32_t mx = 0u, mn = 0xFFFFFFFFu;
    for (uint32_t i = t; i < n; i += kRowThreads) {
        const uint32_t c = lds.ties[i];
        mx = max(mx, c);
        mn = min(mn, c);
    }
    for (int o = 1; o < kWave; o <<= 1) {
        mx = max(mx, (uint32_t)__shfl_xor(mx, o, kWave));
        mn = min(mn, (uint32_t)__shfl_xor(mn, o, kWave));
    }
    if (lane_id() == 0) {
        atomicMax(&lds.bcast[0], mx);
        atomicMin(&lds.bcast[1], mn);
    }
    __syncthreads();
    mx = lds.bcast[0];
    mn = lds.bcast[1];
    const uint32_t span = mx - mn;
    const uint32_t shift = span < (uint32_t)kSelBins ? 0u : (32u - (uint32_t)__clz(span)) - 11u;
    // bins ordered like the select's keys: the smallest coordinates in the highest bin
    for (uint32_t i = t; i < n; i += kRowThreads)
        atomicAdd(&lds.hist[(uint32_t)(kSelBins - 1) - ((lds.ties[i] - mn) >> shift)], 1u);
    __syncthreads();                                  // also: everyone has read bcast
    uint32_t bin, want, in_bin;
    find_rank_bin<kSelBins>(lds.hist, lds.scan, lds.bcast, take, bin, want, in_bin);
    if (in_bin <= (uint32_t)kRowThreads) {            // uniform
        if (t == 0) lds.n_list = 0;
        __syncthreads();
        for (uint32_t i = t; i < n; i += kRowThreads) {
            const uint32_t c = lds.ties[i];
            if ((uint32_t)(kSelBins - 1) - ((c - mn) >> shift) == bin) lds.hist[atomicAdd(&lds.n_list, 1u)] = c;
        }
        if (t < 4) lds.hist[in_bin + t] = 0xFFFFFFFFu;
        __syncthreads();
        if (t < in_bin) {
            const uint32_t mine = lds.hist[t];
            const u32x4* tv = reinterpret_cast<const u32x4*>(lds.hist);
            uint32_t below = 0;
#pragma unroll 4
            for (uint32_t j = 0; j < (in_bin + 3) / 4; ++j) {
                const u32x4 o = tv[j];
                below += (o.x < mine) + (o.y < mine) + (o.z < mine) + (o.w < mine);
            }
            if (below == want - 1) lds.bcast[0] = mine;
        }
        __syncthreads();
        const uint32_t r = lds.bcast[0];
        __syncthreads();
        return r;
    }
    uint32_t t_eq, n_eq;
    const uint32_t* ties = lds.ties;
    auto at = [ties](uint64_t i) { return kAbsMask - ties[i]; };
    const KeysInMemory<decltype(at)> src{at, n};
    return kAbsMask - block_radix_select(src, take, lds.hist, lds.scan, lds.bcast, t_eq, n_eq);
}

// K-th largest magnitude of a row's candidate list and the tie cut.  `keys`
// delivers the candidates' magnitudes (position i = position in the list crow).
// Returns through kth / tie_cut; `path` = 0 when the fine histogram sufficed,
// 2 when the radix select over all candidates had to run.
template <typename Keys>
__device__ __forceinline__ void select_among_candidates(const Keys& keys, const u32x2* __restrict__ crow,
                                                        uint32_t C, uint32_t K, uint32_t tau, SelectLds& lds,
                                                        uint32_t& kth, uint32_t& tie_cut, uint32_t& path)
{
    const uint32_t lane = lane_id(), t = threadIdx.x;
    uint32_t take_eq = 0, n_eq = 0;
    bool have_kth = false;
    path = 0;
    if (t == 0) lds.n_list = 0;                   // ordered by the first barrier below
    if (tau != 0) {
        // All candidates are >= tau and most lie within an octave of it: one
        // histogram of (key - tau) in 2048 bins finds the bin of the K-th largest.
        for (int b = t; b < kFineBins; b += kRowThreads) lds.hist[b] = 0;
        __syncthreads();
        keys.each([&](uint32_t k, uint64_t, bool valid) { tally_digit(lds.hist, valid, fine_bin(k, tau), lane); });
        __syncthreads();
        uint32_t bin, want, in_bin;
        find_rank_bin<kFineBins>(lds.hist, lds.scan, lds.bcast, K, bin, want, in_bin);
        if (in_bin <= (uint32_t)kRankCap) {       // uniform
            // few candidates in that bin: collect them (magnitude in hist[], coordinate
            // in ties[]) and rank them by brute force under (magnitude desc, coordinate
            // asc); the one with exactly want-1 others ahead is the last of the top K
            keys.each([&](uint32_t k, uint64_t i, bool valid) {
                if (valid && fine_bin(k, tau) == bin) {
                    const uint32_t p = atomicAdd(&lds.n_list, 1u);
                    lds.hist[p] = k;
                    lds.ties[p] = crow[i].y;
                }
            });
            if (t < 4) {                          // pad to a multiple of 4 with entries ranked last
                lds.hist[in_bin + t] = 0;
                lds.ties[in_bin + t] = 0xFFFFFFFFu;
            }
            __syncthreads();
            if (t < in_bin) {
                const uint32_t mk = lds.hist[t], mi = lds.ties[t];
                const u32x4* hk = reinterpret_cast<const u32x4*>(lds.hist);
                const u32x4* hi = reinterpret_cast<const u32x4*>(lds.ties);
                uint32_t ahead = 0;
#pragma unroll 4
                for (uint32_t j = 0; j < (in_bin + 3) / 4; ++j) {
                    const u32x4 ok = hk[j], oi = hi[j];
                    ahead += (ok.x > mk) || (ok.x == mk && oi.x < mi);
                    ahead += (ok.y > mk) || (ok.y == mk && oi.y < mi);
                    ahead += (ok.z > mk) || (ok.z == mk && oi.z < mi);
                    ahead += (ok.w > mk) || (ok.w == mk && oi.w < mi);
                }
                if (ahead == want - 1) {
                    lds.bcast[0] = mk;
                    lds.bcast[1] = mi;
                }
            }
            __syncthreads();
            kth = lds.bcast[0];
            tie_cut = lds.bcast[1];
            return;
        }
        if (in_bin <= (uint32_t)kKeyBins) {       // uniform
            // A crowded bin that still fits in LDS.  Values on a lattice put hundreds of
            // EQUAL magnitudes there: if all members share one key, that key is the K-th
            // largest and only the tie cut is left to find, among coordinates already in LDS.
            if (t < 2) lds.bcast[t] = t ? 0xFFFFFFFFu : 0u;          // max, min of the members' keys
            keys.each([&](uint32_t k, uint64_t i, bool valid) {
                if (valid && fine_bin(k, tau) == bin) {
                    const uint32_t p = atomicAdd(&lds.n_list, 1u);
                    lds.hist[p] = k;
                    lds.ties[p] = crow[i].y;
                }
            });
            __syncthreads();
            for (uint32_t i = t; i < in_bin; i += kRowThreads) {
                const uint32_t k = lds.hist[i];
                if (k != lds.hist[0]) {                              // any writer will do: both end up != hist[0]
                    atomicMax(&lds.bcast[0], k);
                    atomicMin(&lds.bcast[1], k);
                }
            }
            __syncthreads();
            const bool one_key = lds.bcast[0] == 0u && lds.bcast[1] == 0xFFFFFFFFu;   // nobody differed from hist[0]
            const uint32_t the_key = lds.hist[0];
            __syncthreads();
            if (one_key) {                                           // uniform
                kth = the_key;
                tie_cut = want < in_bin ? smallest_coordinate(lds, in_bin, want) : 0xFFFFFFFFu;
                return;
            }
            if (t == 0) lds.n_list = 0;                              // distinct keys: go on below
            __syncthreads();
        }
        if (bin < (uint32_t)(kFineBins - 1)) {
            // a crowded bin (many equal magnitudes): it spans exactly 4096 key values,
            // so a second histogram over the exact keys inside it finds the K-th largest
            const uint32_t bin_lo = tau + (bin << kFineShift);
            for (int b = t; b < kKeyBins; b += kRowThreads) lds.hist[b] = 0;
            __syncthreads();
            keys.each([&](uint32_t k, uint64_t, bool valid) {
                tally_digit(lds.hist, valid && fine_bin(k, tau) == bin, (k - bin_lo) & (uint32_t)(kKeyBins - 1), lane);
            });
            __syncthreads();
            uint32_t sub;
            find_rank_bin<kKeyBins>(lds.hist, lds.scan, lds.bcast, want, sub, take_eq, n_eq);
            kth = bin_lo + sub;
            have_kth = true;
        }
    }
    if (!have_kth) {
        path = 2;
        kth = block_radix_select(keys, K, lds.hist, lds.scan, lds.bcast, take_eq, n_eq);
    }
    // ties with the K-th magnitude: all taken, or only the take_eq lowest coordinates
    tie_cut = 0xFFFFFFFFu;
    if (take_eq < n_eq) {                         // uniform
        if (n_eq <= (uint32_t)kTieCap) {
            keys.each([&](uint32_t k, uint64_t i, bool valid) {
                if (valid && k == kth) lds.ties[atomicAdd(&lds.n_list, 1u)] = crow[i].y;
            });
            __syncthreads();
            tie_cut = smallest_coordinate(lds, n_eq, take_eq);
        } else {
            // more ties than the LDS list holds: select over the whole candidate list in
            // memory, entries that are not ties mapped below every tie
            uint32_t t_eq, t_n;
            auto at = [crow, kth](uint64_t i) {
                const u32x2 c = crow[i];
                return c.x == kth ? kAbsMask - c.y : 0u;
            };
            const KeysInMemory<decltype(at)> src{at, C};
            tie_cut = kAbsMask - block_radix_select(src, take_eq, lds.hist, lds.scan, lds.bcast, t_eq, t_n);
        }
    }
}

// One workgroup per row.
// Usual case: an exact select over the row's candidate list gives the K-th
// largest magnitude kth[row] and tie_cut[row], the largest coordinate taken
// among the candidates tied with it (0xFFFFFFFF: all ties taken).
// If the candidate count is < K or overflowed the list (for instance a row of
// equal magnitudes), the row is instead selected exactly from memory (e already
// holds a = g + e), and its vote is emitted and cast here; slow_flag[row] = 1
// tells the later kernels to skip the row.
__global__ __launch_bounds__(kRowThreads) void mv_row_select(
    const float* __restrict__ e, int64_t ld_e, int64_t d, uint32_t K,
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count,
    const uint32_t* __restrict__ tau_bits,
    uint32_t* __restrict__ kth_out, uint32_t* __restrict__ tie_cut_out,
    uint32_t* __restrict__ worker_idx, uint32_t* __restrict__ votes32,
    uint32_t* __restrict__ cnt_ge, uint32_t* __restrict__ slow_flag, int thresholds_only, int slow_rows_only)
{
    __shared__ SelectLds lds;
    const uint32_t row = blockIdx.x, t = threadIdx.x;
    if (slow_rows_only) {                         // the candidate lists are selected by the mv_sel_* kernels
        const uint32_t C0 = row_count[row * kCounterStride];
        if (C0 >= K && C0 <= cap) return;         // whole workgroup
    }
    // The first kKeep * kRowThreads list entries are fetched before the row's
    // candidate count is known (the list's storage holds cap entries; what lies at
    // or beyond the count is ignored later), so the two loads do not queue up.
    const u32x2* crow = cand + (size_t)row * cap;
    uint32_t k[kKeep];
#pragma unroll
    for (int q = 0; q < kKeep; ++q) {
        k[q] = crow[min((uint32_t)q * kRowThreads + t, cap - 1)].x;
        if ((q & 7) == 7) __builtin_amdgcn_sched_barrier(0);   // keep address arithmetic from piling up
    }
    const uint32_t C = row_count[row * kCounterStride];

    if (C >= K && C <= cap) {
        const uint32_t tau = tau_bits[row];
        uint32_t kth, tie_cut, path;
        if (C <= (uint32_t)kKeep * kRowThreads) {
            const KeysInRegs src{k, C};
            select_among_candidates(src, crow, C, K, tau, lds, kth, tie_cut, path);
        } else {
            auto at = [crow](uint64_t i) { return crow[i].x; };
            const KeysInMemory<decltype(at)> src{at, C};
            select_among_candidates(src, crow, C, K, tau, lds, kth, tie_cut, path);
        }
        if (t == 0) {
            kth_out[row] = kth;
            tie_cut_out[row] = tie_cut;
            if (path) slow_flag[row] = path;      // diagnostic only
        }
        return;
    }

    // ---- exact path from memory
    if (t == 0) slow_flag[row] = 1;
    for (int i = t; i < 257; i += kRowThreads) lds.lvl[i] = 0;   // ordered by the select's first barrier
    uint32_t* out = worker_idx ? worker_idx + (size_t)row * K : nullptr;
    const float* arow = e + (int64_t)row * ld_e;
    uint32_t take_eq, n_eq;
    auto at = [arow](uint64_t i) { return __float_as_uint(arow[i]) & kAbsMask; };
    const KeysInMemory<decltype(at)> src{at, (uint64_t)d};
    const uint32_t kth = block_radix_select(src, K, lds.hist, lds.scan, lds.bcast, take_eq, n_eq);
    if (thresholds_only) {
        // add-drop voting only needs the membership test: the tie cut is the take_eq-th
        // smallest coordinate among the row's ties, selected from memory
        uint32_t tie_cut = 0xFFFFFFFFu;
        if (take_eq < n_eq) {
            uint32_t t_eq, t_n;
            auto tie_at = [arow, kth](uint64_t i) {
                return (__float_as_uint(arow[i]) & kAbsMask) == kth ? kAbsMask - (uint32_t)i : 0u;
            };
            const KeysInMemory<decltype(tie_at)> ties_src{tie_at, (uint64_t)d};
            tie_cut = kAbsMask - block_radix_select(ties_src, take_eq, lds.hist, lds.scan, lds.bcast, t_eq, t_n);
        }
        if (t == 0) {
            kth_out[row] = kth;
            tie_cut_out[row] = tie_cut;
        }
        return;
    }
    uint32_t gt_before = 0, eq_before = 0;
    for (int64_t j0 = 0; j0 < d; j0 += (int64_t)kRowThreads * 4) {
        const int64_t j = j0 + (int64_t)t * 4;
        uint32_t k[4];
        uint32_t gt = 0, eq = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool valid = (j + c < d);
            k[c] = valid ? (__float_as_uint(arow[j + c]) & kAbsMask) : 0u;
            gt += (valid && k[c] > kth);
            eq += (valid && k[c] == kth);
        }
        uint64_t total;
        const uint64_t ex = block_excl_scan64<kRowThreads>(pack2(gt, eq), lds.scan, total);
        uint32_t g0 = gt_before + (uint32_t)(ex >> 32), e0 = eq_before + (uint32_t)ex;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (j + c < d) {
                const bool is_gt = k[c] > kth, is_eq = k[c] == kth;
                if (is_gt || (is_eq && e0 < take_eq)) {
                    const uint32_t pos = g0 + min(e0, take_eq);
                    if (out && pos < K) out[pos] = (uint32_t)(j + c);
                    cast_vote(votes32, (uint32_t)(j + c), lds.lvl);
                }
                g0 += is_gt;
                e0 += is_eq;
            }
        }
        gt_before += (uint32_t)(total >> 32);
        eq_before += (uint32_t)total;
        __syncthreads();   // lds.scan is reused by the next round
    }
    __syncthreads();
    for (int i = t; i < 256; i += kRowThreads) {
        const uint32_t c = lds.lvl[i];
        if (c) atomicAdd(&cnt_ge[(size_t)row * 256 + i], c);
    }
}

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
    if (slow_flag[row] == 1u) return;                              // whole workgroup
    const uint32_t C = row_count[row * kCounterStride];
    if ((uint64_t)blockIdx.x * kVoteThreads >= C) return;    // whole workgroup
    for (int i = t; i < 257; i += kVoteThreads) lvl[i] = 0;
    __syncthreads();
    const uint32_t kth = kth_in[row], tie_cut = tie_cut_in[row];
    const u32x2* crow = cand + (size_t)row * cap;
    uint32_t*    ssel = seg_sel ? seg_sel + (size_t)row * nseg : nullptr;
    const uint32_t lane = lane_id();
    for (uint64_t i0 = (uint64_t)blockIdx.x * kVoteThreads; i0 < C; i0 += (uint64_t)gridDim.x * kVoteThreads) {
        const uint64_t i = i0 + t;
        u32x2 c = {0u, 0xFFFFFFFFu};
        bool taken = false;
        if (i < C) {
            c = crow[i];
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
    const uint32_t C = row_count[row * kCounterStride];
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
__global__ __launch_bounds__(kVoteThreads) void mv_ad_compact_count(const uint32_t* __restrict__ ad_bits,
                                                                    uint32_t nwords_pad, uint32_t nblk,
                                                                    u32x2* __restrict__ blk_cnt,
                                                                    const uint32_t* __restrict__ vote_bits,
                                                                    int64_t ld_bits)
{
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    compact_count_block(ad_bits, nwords_pad, nblk, blk_cnt, vote_bits, ld_bits, blockIdx.y, blockIdx.x, scan_lds);
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

// Histogram of the vote levels of msum (one byte per coordinate, values 0..N):
// lvl_cnt[v] = number of coordinates with exactly v votes.
__device__ __forceinline__ void ad_levels_block(const uint32_t* __restrict__ msum32, int64_t d,
                                                uint32_t* __restrict__ lvl_cnt, uint32_t n_sets, uint32_t bx,
                                                uint32_t* h /*256*/)
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
    uint32_t zeros = 0;                           // most coordinates have no vote
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        if (j < d) {
            const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
            if ((ww[0] | ww[1] | ww[2] | ww[3]) == 0u) {
                zeros += (uint32_t)min((int64_t)16, d - j);
            } else {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                    if (j + q < d) {
                        if (v) atomicAdd(&h[v], 1u);
                        else   ++zeros;
                    }
                }
            }
        }
    }
    if (zeros) atomicAdd(&h[0], zeros);
    __syncthreads();
    // the workgroups take turns over the n_sets sets of counters (the sum counts), so that
    // their atomics do not all queue up on one cache line
    const uint32_t c = h[threadIdx.x];
    if (c) atomicAdd(&lvl_cnt[(size_t)(bx % n_sets) * 256 + threadIdx.x], c);
}

// One launch after mv_ad_apply: the first n_count_blocks workgroups count the additions
// and removals marked in the N scratch bitmaps per block, the others take the histogram of msum's levels.
__global__ __launch_bounds__(kVoteThreads) void mv_ad_count_levels(const uint32_t* __restrict__ ad_bits,
                                                                   uint32_t nwords_pad, uint32_t nblk,
                                                                   u32x2* __restrict__ blk_cnt,
                                                                   const uint32_t* __restrict__ vote_bits,
                                                                   int64_t ld_bits, uint32_t n_count_blocks,
                                                                   const uint32_t* __restrict__ msum32, int64_t d,
                                                                   uint32_t* __restrict__ lvl_cnt, uint32_t n_sets)
{
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    __shared__ uint32_t h[256];
    if (blockIdx.x < n_count_blocks)
        compact_count_block(ad_bits, nwords_pad, nblk, blk_cnt, vote_bits, ld_bits, blockIdx.x / nblk,
                            blockIdx.x % nblk, scan_lds);
    else
        ad_levels_block(msum32, d, lvl_cnt, n_sets, blockIdx.x - n_count_blocks, h);
}

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

// ---- exact select over a long list with many workgroups ----------------------
// Three kernels find the `want` largest keys of lists too long for one workgroup
// to read more than once: (1) a histogram of kSelBins bins of (key - base) >> shift
// over the list, (2) every workgroup locates the bin of the want-th largest and
// moves that bin's members to a second list (and, with a bitmap, marks the
// entries of higher bins), (3) one workgroup per list ranks the second list
// exactly.  They serve the random selection (one list, base 0, shift 20: the 11
// leading key bits) and the rows' top-K when K is large (one list per row, base =
// the row's threshold estimate, shift = kFineShift).
constexpr int kListPerThread = 4;
constexpr int kListPerBlock = kRowThreads * kListPerThread;

struct ListSelect {
    const u32x2* list;        // rows of `cap` entries
    uint32_t     cap;
    const uint32_t* count;    // entries per row (clamped to cap), row r at count[r * count_stride]
    uint32_t     count_stride;
    const uint32_t* base;     // per row, or null: 0
    uint32_t     shift;
    uint32_t     want;        // K
    uint32_t*    hist;        // rows of kSelBins counters, zero between steps
    u32x2*       list2;       // rows of `cap` entries: members of the want-th largest's bin
    uint32_t*    count2;      // per row, zero between steps
    uint32_t*    bin_want;    // per row: the bin, and how many of its members are wanted
};

__device__ __forceinline__ uint32_t list_bin(uint32_t key, uint32_t base, uint32_t shift)
{
    return min((key - base) >> shift, (uint32_t)(kSelBins - 1));
}
// a row takes part when its list holds at least `want` entries and did not overflow
__device__ __forceinline__ bool list_row_ok(const ListSelect& a, uint32_t row, uint32_t& n)
{
    n = a.count[row * a.count_stride];
    return n >= a.want && n <= a.cap;
}

__device__ __forceinline__ void list_hist_body(const ListSelect& a, uint32_t row, uint32_t* hist_lds)
{
    const uint32_t t = threadIdx.x;
    uint32_t n;
    if (!list_row_ok(a, row, n)) return;                             // whole workgroup
    const uint32_t i0 = blockIdx.x * (uint32_t)kListPerBlock;
    if (i0 >= n) return;                                             // whole workgroup
    const u32x2* list = a.list + (size_t)row * a.cap;
    const uint32_t base = a.base ? a.base[row] : 0u;
    uint32_t k[kListPerThread];
#pragma unroll
    for (int u = 0; u < kListPerThread; ++u) {
        const uint32_t i = i0 + (uint32_t)u * kRowThreads + t;
        k[u] = (i < n) ? list[i].x : 0xFFFFFFFFu;                   // keys are at most 0x7FFFFFFF
    }
    for (int b = t; b < kSelBins; b += kRowThreads) hist_lds[b] = 0;
    __syncthreads();
    const uint32_t lane = lane_id();
#pragma unroll
    for (int u = 0; u < kListPerThread; ++u) tally_digit(hist_lds, k[u] != 0xFFFFFFFFu, list_bin(k[u], base, a.shift), lane);
    __syncthreads();
    uint32_t* hrow = a.hist + (size_t)row * kSelBins;
    for (int b = t; b < kSelBins; b += kRowThreads) {
        const uint32_t c = hist_lds[b];
        if (c) atomicAdd(&hrow[b], c);
    }
}

struct ListSplitLds {
    uint32_t hist[kSelBins];
    uint64_t scan[kRowThreads / kWave + 1];
    uint32_t bcast[3];
    uint32_t base_sh;
};

__device__ __forceinline__ void list_split_body(const ListSelect& a, uint32_t row, ListSplitLds& lds,
                                                uint32_t* __restrict__ bits)
{
    const uint32_t t = threadIdx.x;
    uint32_t n;
    if (!list_row_ok(a, row, n)) return;                             // whole workgroup
    const uint32_t i0 = blockIdx.x * (uint32_t)kListPerBlock;
    if (i0 >= n && blockIdx.x != 0) return;                          // whole workgroup
    const u32x2* list = a.list + (size_t)row * a.cap;
    const uint32_t base = a.base ? a.base[row] : 0u;
    u32x2 c[kListPerThread];
#pragma unroll
    for (int u = 0; u < kListPerThread; ++u) {
        const uint32_t i = i0 + (uint32_t)u * kRowThreads + t;
        const u32x2 none = {0u, 0xFFFFFFFFu};
        c[u] = (i < n) ? list[i] : none;
    }
    const uint32_t* hrow = a.hist + (size_t)row * kSelBins;
    for (int b = t; b < kSelBins; b += kRowThreads) lds.hist[b] = hrow[b];
    __syncthreads();
    uint32_t bin, want, in_bin;
    find_rank_bin<kSelBins>(lds.hist, lds.scan, lds.bcast, a.want, bin, want, in_bin);
    if (blockIdx.x == 0 && t == 0) {
        a.bin_want[2 * row] = bin;
        a.bin_want[2 * row + 1] = want;
    }
    uint32_t mine = 0;
#pragma unroll
    for (int u = 0; u < kListPerThread; ++u) {
        const bool valid = c[u].y != 0xFFFFFFFFu;
        const uint32_t b = list_bin(c[u].x, base, a.shift);
        if (bits && valid && b > bin) atomicOr(&bits[c[u].y >> 5], 1u << (c[u].y & 31u));
        mine += (valid && b == bin);
    }
    uint64_t total;
    const uint64_t ex = block_excl_scan64<kRowThreads>(mine, lds.scan, total);
    if (total == 0) return;                                          // whole workgroup
    if (t == 0) lds.base_sh = atomicAdd(&a.count2[row], (uint32_t)total);
    __syncthreads();
    uint32_t pos = lds.base_sh + (uint32_t)ex;
    u32x2* list2 = a.list2 + (size_t)row * a.cap;
#pragma unroll
    for (int u = 0; u < kListPerThread; ++u) {
        const bool valid = c[u].y != 0xFFFFFFFFu;
        if (valid && list_bin(c[u].x, base, a.shift) == bin) {
            if (pos < a.cap) list2[pos] = c[u];
            ++pos;
        }
    }
}

// Ranks the second list exactly: kth / tie_cut as for a row's candidate list.
// Leaves the row's histogram and count2 at zero.  Returns false when the row does
// not take part.
__device__ __forceinline__ bool list_rank_body(const ListSelect& a, uint32_t row, SelectLds& lds, uint32_t& kth,
                                               uint32_t& tie_cut, uint32_t& path)
{
    const uint32_t t = threadIdx.x;
    uint32_t n;
    if (!list_row_ok(a, row, n)) return false;                       // whole workgroup
    const uint32_t C = min(a.count2[row], a.cap), bin = a.bin_want[2 * row], want = a.bin_want[2 * row + 1];
    __syncthreads();                                                  // everyone has read the counters
    uint32_t* hrow = a.hist + (size_t)row * kSelBins;
    for (int b = t; b < kSelBins; b += kRowThreads) hrow[b] = 0;
    if (t == 0) a.count2[row] = 0;
    if (C == 0 || want == 0 || want > C) return false;                // cannot happen after the split
    const u32x2* list2 = a.list2 + (size_t)row * a.cap;
    const uint32_t base = (a.base ? a.base[row] : 0u) + (bin << a.shift);
    if (C > 8u * kRowThreads && C <= (uint32_t)kKeep * kRowThreads) {   // short lists: a few loads per pass are cheaper
        uint32_t k[kKeep];
        const uint32_t last = C - 1;
#pragma unroll
        for (int q = 0; q < kKeep; ++q) {
            k[q] = list2[min((uint32_t)q * kRowThreads + t, last)].x;
            if ((q & 7) == 7) __builtin_amdgcn_sched_barrier(0);
        }
        const KeysInRegs src{k, C};
        select_among_candidates(src, list2, C, want, base, lds, kth, tie_cut, path);
    } else {
        auto at = [list2](uint64_t i) { return list2[i].x; };
        const KeysInMemory<decltype(at)> src{at, C};
        select_among_candidates(src, list2, C, want, base, lds, kth, tie_cut, path);
    }
    return true;
}

// ---- the rows' top-K when K is large (grid: blocks of the candidate list x rows)
__global__ __launch_bounds__(kRowThreads) void mv_sel_hist(ListSelect a)
{
    __shared__ uint32_t hist[kSelBins];
    list_hist_body(a, blockIdx.y, hist);
}
__global__ __launch_bounds__(kRowThreads) void mv_sel_split(ListSelect a)
{
    __shared__ ListSplitLds lds;
    list_split_body(a, blockIdx.y, lds, nullptr);
}
__global__ __launch_bounds__(kRowThreads) void mv_sel_rank(ListSelect a, uint32_t* __restrict__ kth_out,
                                                           uint32_t* __restrict__ tie_cut_out,
                                                           uint32_t* __restrict__ slow_flag)
{
    __shared__ SelectLds lds;
    const uint32_t row = blockIdx.x;
    uint32_t kth, tie_cut, path;
    if (!list_rank_body(a, row, lds, kth, tie_cut, path)) return;
    if (threadIdx.x == 0) {
        kth_out[row] = kth;
        tie_cut_out[row] = tie_cut;
        if (path) slow_flag[row] = path;          // diagnostic only
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
