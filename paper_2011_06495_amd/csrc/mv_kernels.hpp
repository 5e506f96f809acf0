// Device kernels of the majority-voting vote step for gfx950 (MI355X).
//
// The step is bound by HBM traffic: the only work that touches all N*d
// coordinates is the error compensation a = g + e (Algorithm 1) and finding
// each worker's K largest |a| (its vote).  Nothing here is a dense
// contraction, so no MFMA; the design goal is ONE streaming pass over g and e.
//
// How the per-worker top-K is found without re-reading the row:
//   1. mv_sample_hist     histogram of the magnitude bit patterns of a strided
//                         sample of each row (cache-line sized chunks)
//   2. mv_pick_threshold  per row, a bin edge tau that about 3K sampled-scaled
//                         coordinates exceed (an ESTIMATE, never trusted)
//   3. mv_stream_collect  the streaming pass: a = g + e is written over e, and
//                         every coordinate with |a| >= tau is appended to the
//                         row's candidate list; each wavefront's 1024-coordinate
//                         segment records where its run of candidates went
//   4. mv_row_finish      per row: EXACT radix select of the K-th largest
//                         magnitude among the candidates (their number is known
//                         exactly; if it is < K or overflowed the list, the row
//                         is selected exactly from memory instead), then the
//                         vote is emitted in ascending coordinate order by
//                         walking the segment table, and counted
//   5. mv_mask_count /    counting-sort selection of the K most voted
//      mv_mask_emit       coordinates, ties to the lowest coordinate
//   6. mv_gather_update   masked gather, sum over workers in order, mean, and
//                         the error update (zero on the mask)
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
constexpr int      kStreamThreads  = 256;    // 4 segments per workgroup
constexpr int      kSegPerBlock    = kStreamThreads / kWave;
constexpr int      kHistBits       = 12;     // sample histogram: exponent + 4 mantissa bits
constexpr int      kHistBins       = 1 << kHistBits;
constexpr int      kHistShift      = 31 - kHistBits;
constexpr int      kChunk          = 32;     // sampled chunk: 32 coordinates (one 128-byte line of fp32)
constexpr int      kRowThreads     = 1024;   // mv_pick_threshold / mv_row_finish: one workgroup per row
constexpr int      kVoteBlock      = 16384;  // coordinates per workgroup in mv_mask_count / mv_mask_emit
constexpr int      kVoteThreads    = 256;
constexpr int      kGatherThreads  = 256;
constexpr uint32_t kAbsMask        = 0x7FFFFFFFu;

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
// 1. sample histogram
// ----------------------------------------------------------------------------
// Chunk c of a row is the coordinates [32c, 32c+32); chunk c is sampled when
// c % stride == 0.  bin = (bits(|g+e|)) >> kHistShift.
template <typename GT>
__global__ __launch_bounds__(256) void mv_sample_hist(const GT* __restrict__ g, int64_t ld_g,
                                                      const float* __restrict__ e, int64_t ld_e,
                                                      int64_t d, uint32_t stride,
                                                      uint32_t n_sampled_chunks,
                                                      uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[kHistBins];
    const uint32_t row = blockIdx.y;
    for (int b = threadIdx.x; b < kHistBins; b += blockDim.x) h[b] = 0;
    __syncthreads();

    const GT*    grow = g + (int64_t)row * ld_g;
    const float* erow = e + (int64_t)row * ld_e;
    const uint64_t nquads = (uint64_t)n_sampled_chunks * (kChunk / 4);
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nquads;
         q += (uint64_t)gridDim.x * blockDim.x) {
        const int64_t j = (int64_t)(q / (kChunk / 4)) * stride * kChunk + (int64_t)(q % (kChunk / 4)) * 4;
        if (j + 4 <= d) {
            f32x4 gv = load4_grad(grow + j);
            f32x4 ev = *reinterpret_cast<const f32x4*>(erow + j);
            f32x4 a = gv + ev;
            atomicAdd(&h[(__float_as_uint(a.x) & kAbsMask) >> kHistShift], 1u);
            atomicAdd(&h[(__float_as_uint(a.y) & kAbsMask) >> kHistShift], 1u);
            atomicAdd(&h[(__float_as_uint(a.z) & kAbsMask) >> kHistShift], 1u);
            atomicAdd(&h[(__float_as_uint(a.w) & kAbsMask) >> kHistShift], 1u);
        } else {
            for (int64_t jj = j; jj < d; ++jj) {
                float a = load1_grad(grow + jj) + erow[jj];
                atomicAdd(&h[(__float_as_uint(a) & kAbsMask) >> kHistShift], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t* hrow = hist + (size_t)row * kHistBins;
    for (int b = threadIdx.x; b < kHistBins; b += blockDim.x) {
        uint32_t c = h[b];
        if (c) atomicAdd(&hrow[b], c);
    }
}

// ----------------------------------------------------------------------------
// 2. threshold pick (one workgroup per row) + per-step reset of the counters
// ----------------------------------------------------------------------------
// tau_bits[row] = lower edge of the highest bin such that at least `m_target`
// sampled coordinates lie in that bin or above; 0 if the sample holds fewer.
// The histogram is cleared after it is read so the next step starts from zero.
__global__ __launch_bounds__(kRowThreads) void mv_pick_threshold(uint32_t* __restrict__ hist,
                                                                 uint32_t m_target,
                                                                 uint32_t* __restrict__ tau_bits,
                                                                 uint32_t* __restrict__ row_count,
                                                                 uint32_t* __restrict__ slow_flag,
                                                                 uint32_t* __restrict__ cnt_ge)
{
    __shared__ uint64_t scan_lds[kRowThreads / kWave + 1];
    __shared__ uint32_t found;
    const uint32_t row = blockIdx.x, t = threadIdx.x;
    uint32_t* hrow = hist + (size_t)row * kHistBins;
    constexpr int per = kHistBins / kRowThreads;   // 4 bins per thread, descending bin order
    uint32_t c[per];
    uint32_t s = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        const int bin = kHistBins - 1 - (t * per + q);
        c[q] = hrow[bin];
        hrow[bin] = 0;
        s += c[q];
    }
    if (t == 0) {
        found = 0;
        row_count[row] = 0;
        slow_flag[row] = 0;
    }
    if (row == 0 && t < 256) cnt_ge[t] = 0;
    uint64_t total;
    const uint64_t excl = block_excl_scan64<kRowThreads>(s, scan_lds, total);
    if (excl < m_target && (uint64_t)m_target <= excl + s) {
        uint64_t acc = excl;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            if (acc < m_target && (uint64_t)m_target <= acc + c[q])
                found = (uint32_t)(kHistBins - 1 - (t * per + q)) << kHistShift;
            acc += c[q];
        }
    }
    __syncthreads();
    if (t == 0) tau_bits[row] = (total >= m_target) ? found : 0u;
}

// ----------------------------------------------------------------------------
// 3. the streaming pass
// ----------------------------------------------------------------------------
// One wavefront = one segment of 1024 consecutive coordinates of one row, read
// as 4 sub-blocks of 256 (lane l holds coordinates base + 256u + 4l .. +3).
// a = g + e overwrites e.  Coordinates with (bits(a) & 0x7FFFFFFF) >= tau are
// appended to the row's candidate list as (magnitude bits, coordinate), in
// ascending coordinate order inside the wavefront's run; seg[row][s] =
// (start of the run, its length).  Runs land in the list in any order; the
// table makes the order recoverable.  Entries beyond `cap` are dropped, the
// counter keeps counting (the overflow is detected from it).
template <typename GT>
__global__ __launch_bounds__(kStreamThreads) void mv_stream_collect(
    const GT* __restrict__ g, int64_t ld_g, float* __restrict__ e, int64_t ld_e, int64_t d,
    const uint32_t* __restrict__ tau_bits, u32x2* __restrict__ cand, uint32_t cap,
    uint32_t* __restrict__ row_count, u32x2* __restrict__ seg, uint32_t nseg)
{
    const uint32_t row = blockIdx.y;
    const uint32_t lane = lane_id();
    const uint32_t s = blockIdx.x * kSegPerBlock + threadIdx.x / kWave;
    if (s >= nseg) return;                       // whole wavefront
    const int64_t base = (int64_t)s * kSeg;
    const GT* grow = g + (int64_t)row * ld_g;
    float*    erow = e + (int64_t)row * ld_e;
    const uint32_t tau = tau_bits[row];

    uint32_t key[16];
    uint32_t flags = 0;
    if (base + kSeg <= d) {
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
    } else {
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

    uint32_t total = 0, run_start = 0;
    if (__ballot(flags != 0) != 0ull) {          // wave-uniform
        uint32_t rank[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t c = __popc((flags >> (4 * u)) & 15u);
            const uint32_t incl = wave_incl_scan(c);
            rank[u] = total + incl - c;
            total += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) run_start = atomicAdd(&row_count[row], total);
        run_start = __shfl(run_start, 0, kWave);
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
    if (lane == 0) {
        u32x2 rec;
        rec.x = run_start;
        rec.y = total;
        seg[(size_t)row * nseg + s] = rec;
    }
}

// ----------------------------------------------------------------------------
// 4. per-row exact select + ordered emission + vote counting
// ----------------------------------------------------------------------------

// Exact K-th largest of `count` keys delivered by `key_at(i)`, by an MSB-first
// 8-bit radix select in one workgroup.  Returns the K-th largest key; `take_eq`
// receives how many keys EQUAL to it belong to the top K (>= 1).
// Requires 1 <= K <= count.  All threads of the workgroup must call it.
template <typename KeyAt>
__device__ __forceinline__ uint32_t block_radix_select(KeyAt key_at, uint64_t count, uint32_t K,
                                                       uint32_t* hist /*256*/, uint32_t* bcast /*2*/,
                                                       uint32_t& take_eq)
{
    uint32_t prefix = 0, known = 0, remaining = K;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        for (uint64_t i = threadIdx.x; i < count; i += blockDim.x) {
            const uint32_t k = key_at(i);
            if ((k & known) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x < kWave) {
            // lane l owns digits 255-4l .. 252-4l (descending)
            const int top = 255 - 4 * (int)threadIdx.x;
            uint32_t h[4];
            uint32_t s = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                h[q] = hist[top - q];
                s += h[q];
            }
            const uint32_t incl = wave_incl_scan(s);
            uint32_t acc = incl - s;
            if (acc < remaining && remaining <= incl) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (acc < remaining && remaining <= acc + h[q]) {
                        bcast[0] = (uint32_t)(top - q);
                        bcast[1] = remaining - acc;
                    }
                    acc += h[q];
                }
            }
        }
        __syncthreads();
        prefix |= bcast[0] << shift;
        known |= 255u << shift;
        remaining = bcast[1];
    }
    take_eq = remaining;
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

__global__ __launch_bounds__(kRowThreads) void mv_row_finish(
    const float* __restrict__ e, int64_t ld_e, int64_t d, uint32_t K,
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count,
    const u32x2* __restrict__ seg, uint32_t nseg,
    uint32_t* __restrict__ worker_idx, uint32_t* __restrict__ votes32,
    uint32_t* __restrict__ cnt_ge, uint32_t* __restrict__ slow_flag)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t lvl[257];
    __shared__ uint32_t bcast[2];
    __shared__ uint64_t scan_lds[kRowThreads / kWave + 1];

    const uint32_t row = blockIdx.x, t = threadIdx.x;
    const uint32_t C = row_count[row];
    uint32_t* out = worker_idx ? worker_idx + (size_t)row * K : nullptr;
    for (int i = t; i < 257; i += kRowThreads) lvl[i] = 0;
    // (the first __syncthreads inside block_radix_select orders this)

    if (C >= K && C <= cap) {
        // ---- the usual path: everything needed is in the candidate list
        const u32x2* crow = cand + (size_t)row * cap;
        uint32_t take_eq;
        const uint32_t kth =
            block_radix_select([&](uint64_t i) { return crow[i].x; }, C, K, hist, bcast, take_eq);

        // thread t owns a contiguous range of segments, hence of coordinates
        const uint32_t per = (nseg + kRowThreads - 1) / kRowThreads;
        const uint32_t s0 = min(t * per, nseg), s1 = min(s0 + per, nseg);
        const u32x2* srow = seg + (size_t)row * nseg;
        uint32_t gt = 0, eq = 0;
        for (uint32_t s = s0; s < s1; ++s) {
            const u32x2 sr = srow[s];
            for (uint32_t i = 0; i < sr.y; ++i) {
                const uint32_t k = crow[sr.x + i].x;
                gt += (k > kth);
                eq += (k == kth);
            }
        }
        uint64_t total;
        const uint64_t ex = block_excl_scan64<kRowThreads>(pack2(gt, eq), scan_lds, total);
        uint32_t gt_before = (uint32_t)(ex >> 32), eq_before = (uint32_t)ex;
        for (uint32_t s = s0; s < s1; ++s) {
            const u32x2 sr = srow[s];
            for (uint32_t i = 0; i < sr.y; ++i) {
                const u32x2 c = crow[sr.x + i];
                const bool is_gt = c.x > kth, is_eq = c.x == kth;
                if (is_gt || (is_eq && eq_before < take_eq)) {
                    const uint32_t pos = gt_before + min(eq_before, take_eq);
                    if (out && pos < K) out[pos] = c.y;
                    cast_vote(votes32, c.y, lvl);
                }
                gt_before += is_gt;
                eq_before += is_eq;
            }
        }
    } else {
        // ---- exact path from memory: e already holds a = g + e for this row.
        // Taken when the estimate kept fewer than K coordinates or more than
        // the list holds (for instance a row of equal magnitudes).
        if (t == 0) slow_flag[row] = 1;
        const float* arow = e + (int64_t)row * ld_e;
        uint32_t take_eq;
        const uint32_t kth = block_radix_select(
            [&](uint64_t i) { return __float_as_uint(arow[i]) & kAbsMask; }, (uint64_t)d, K, hist,
            bcast, take_eq);
        uint32_t gt_before = 0, eq_before = 0;
        for (int64_t j0 = 0; j0 < d; j0 += (int64_t)kRowThreads * 4) {
            const int64_t j = j0 + (int64_t)t * 4;
            uint32_t k[4];
            uint32_t gt = 0, eq = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                k[c] = (j + c < d) ? (__float_as_uint(arow[j + c]) & kAbsMask) : 0u;
                const bool valid = (j + c < d);
                gt += (valid && k[c] > kth);
                eq += (valid && k[c] == kth);
            }
            uint64_t total;
            const uint64_t ex = block_excl_scan64<kRowThreads>(pack2(gt, eq), scan_lds, total);
            uint32_t g0 = gt_before + (uint32_t)(ex >> 32), e0 = eq_before + (uint32_t)ex;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (j + c < d) {
                    const bool is_gt = k[c] > kth, is_eq = k[c] == kth;
                    if (is_gt || (is_eq && e0 < take_eq)) {
                        const uint32_t pos = g0 + min(e0, take_eq);
                        if (out && pos < K) out[pos] = (uint32_t)(j + c);
                        cast_vote(votes32, (uint32_t)(j + c), lvl);
                    }
                    g0 += is_gt;
                    e0 += is_eq;
                }
            }
            gt_before += (uint32_t)(total >> 32);
            eq_before += (uint32_t)total;
            __syncthreads();   // scan_lds is reused by the next round
        }
    }
    __syncthreads();
    for (int i = t; i < 257; i += kRowThreads) {
        const uint32_t c = lvl[i];
        if (c && i < 256) atomicAdd(&cnt_ge[i], c);
    }
}

// ----------------------------------------------------------------------------
// 5. global mask = the K most voted coordinates, ties to the lowest coordinate
// ----------------------------------------------------------------------------
// cnt_ge[v] = number of coordinates with at least v votes (v = 1..N).  The
// threshold v* is the largest v with cnt_ge[v] >= K: all cnt_ge[v*+1]
// coordinates above it are taken, and the first K - cnt_ge[v*+1] coordinates
// (in coordinate order) with exactly v* votes.
__device__ __forceinline__ void vote_threshold(const uint32_t* __restrict__ cnt_ge, uint32_t N,
                                               uint32_t K, uint32_t* lds2, uint32_t& vstar,
                                               uint32_t& take_eq)
{
    if (threadIdx.x == 0) {
        uint32_t v = N;
        while (v > 1 && cnt_ge[v] < K) --v;
        lds2[0] = v;
        lds2[1] = K - ((v < N) ? cnt_ge[v + 1] : 0u);
    }
    __syncthreads();
    vstar = lds2[0];
    take_eq = lds2[1];
}

// counts, per block of kVoteBlock coordinates, how many have votes > v* and == v*;
// optionally copies the vote bytes to the caller's array.
__global__ __launch_bounds__(kVoteThreads) void mv_mask_count(const uint32_t* __restrict__ votes32,
                                                              int64_t d, uint32_t N, uint32_t K,
                                                              const uint32_t* __restrict__ cnt_ge,
                                                              u32x2* __restrict__ block_cnt,
                                                              uint8_t* __restrict__ votes_out)
{
    __shared__ uint32_t lds2[2];
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    uint32_t vstar, take_eq;
    vote_threshold(cnt_ge, N, K, lds2, vstar, take_eq);
    const int64_t base = (int64_t)blockIdx.x * kVoteBlock;
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int it = 0; it < kVoteBlock / (kVoteThreads * 16); ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        if (j < d) {   // the vote buffer is padded to 16 bytes with zeros
            const u32x4 w = *reinterpret_cast<const u32x4*>(votes32 + (j >> 2));
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t v = (ww[q] >> (8 * b)) & 255u;
                    gt += (v > vstar);
                    eq += (v == vstar);
                }
            if (votes_out) {
                if (j + 16 <= d && ((reinterpret_cast<uintptr_t>(votes_out) & 15) == 0)) {
                    *reinterpret_cast<u32x4*>(votes_out + j) = w;
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
    }
}

// emits the mask in ascending order and clears the vote words for the next step
__global__ __launch_bounds__(kVoteThreads) void mv_mask_emit(uint32_t* __restrict__ votes32,
                                                             int64_t d, uint32_t N, uint32_t K,
                                                             const uint32_t* __restrict__ cnt_ge,
                                                             const u32x2* __restrict__ block_cnt,
                                                             uint32_t* __restrict__ mask_idx)
{
    __shared__ uint32_t lds2[2];
    __shared__ uint64_t scan_lds[kVoteThreads / kWave + 1];
    uint32_t vstar, take_eq;
    vote_threshold(cnt_ge, N, K, lds2, vstar, take_eq);

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

    const int64_t base = (int64_t)blockIdx.x * kVoteBlock;
    for (int it = 0; it < kVoteBlock / (kVoteThreads * 16); ++it) {
        const int64_t j = base + ((int64_t)it * kVoteThreads + threadIdx.x) * 16;
        uint32_t ww[4] = {0, 0, 0, 0};
        uint32_t gt = 0, eq = 0;
        if (j < d) {
            u32x4* p = reinterpret_cast<u32x4*>(votes32 + (j >> 2));
            const u32x4 w = *p;
            ww[0] = w.x; ww[1] = w.y; ww[2] = w.z; ww[3] = w.w;
            if ((w.x | w.y | w.z | w.w) != 0u) {
                const u32x4 z = {0u, 0u, 0u, 0u};
                *p = z;
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                gt += (v > vstar);
                eq += (v == vstar);
            }
        }
        uint64_t total;
        const uint64_t ex = block_excl_scan64<kVoteThreads>(pack2(gt, eq), scan_lds, total);
        if (gt | eq) {
            uint32_t g0 = gt_before + (uint32_t)(ex >> 32), e0 = eq_before + (uint32_t)ex;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const uint32_t v = (ww[q >> 2] >> (8 * (q & 3))) & 255u;
                const bool is_gt = v > vstar, is_eq = v == vstar;
                if (is_gt || (is_eq && e0 < take_eq)) {
                    const uint32_t pos = g0 + min(e0, take_eq);
                    if (pos < K) mask_idx[pos] = (uint32_t)(j + q);
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
__global__ __launch_bounds__(kGatherThreads) void mv_gather_update(float* __restrict__ e, int64_t ld_e,
                                                                   int64_t d, uint32_t N, uint32_t K,
                                                                   const uint32_t* __restrict__ mask_idx,
                                                                   float scale, int apply_scale,
                                                                   float* __restrict__ agg)
{
    const uint32_t k = blockIdx.x * kGatherThreads + threadIdx.x;
    if (k >= K) return;
    const uint32_t j = mask_idx[k];
    if ((int64_t)j >= d) return;   // cannot happen for a mask built by mv_mask_emit
    float* p = e + j;
    float s = *p;                  // worker 0
    *p = 0.0f;
    for (uint32_t n = 1; n < N; ++n) {
        p += ld_e;
        s = s + *p;                // workers in order, fp32, no contraction
        *p = 0.0f;
    }
    agg[k] = apply_scale ? s * scale : s;
}

}  // namespace mvk
