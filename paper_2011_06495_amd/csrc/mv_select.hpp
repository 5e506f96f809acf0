// Exact selects: the K-th largest magnitude of a row's candidate list with its tie cut
// (one workgroup per row, or three kernels with many workgroups for long lists).
#pragma once

#include "mv_common.hpp"

namespace mvk {

// ----------------------------------------------------------------------------
// 3. per-row exact select
// ----------------------------------------------------------------------------

constexpr int kSelBins = 2048;   // radix-select digit: 11, 10, 10 bits of the 31-bit key
constexpr int kKeyBins = 4096;   // exact magnitudes inside one fine-histogram bin (1 << kFineShift)
constexpr int kKeep    = 32;     // candidate keys a thread of the generic select can hold in registers
constexpr int kRep     = 8;      // copies of the candidates' fine histogram, one per lane % kRep
constexpr int kTieCap  = 8192;   // ties with the K-th magnitude that fit the LDS list
constexpr int kRankCap = 256;    // at most this many entries are ranked by counting (quadratic work)
constexpr int kKeepShort = 32;   // list entries per thread of the two instances of mv_row_select
constexpr int kKeepLong  = 160;
constexpr int kSpec    = 32;     // list entries per thread that mv_row_select can fetch ahead of the row's count

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
// With REP > 1 the histogram is kept in REP copies, bin b's counters at hist[b * REP .. b * REP + REP).
template <int BINS, int REP = 1>
__device__ __forceinline__ void find_rank_bin(const uint32_t* hist, uint64_t* scan_lds, uint32_t* bcast,
                                              uint32_t want, uint32_t& bin, uint32_t& want_in_bin,
                                              uint32_t& in_bin)
{
    constexpr int per = BINS / kRowThreads;       // bins per thread, descending bin order over threads
    uint32_t h[per];
    uint32_t s = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        const int b = BINS - 1 - ((int)threadIdx.x * per + q);
        h[q] = 0;
#pragma unroll
        for (int r = 0; r < REP; ++r) h[q] += hist[b * REP + r];
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
    static constexpr bool kCheapPasses = true;
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
    static constexpr bool kCheapPasses = false;
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
// keeps a byte from carrying into its neighbour.  lvl[v] (LDS, 257 counters) counts
// coordinates that just reached v votes, so that, summed over all workgroups, lvl[v] =
// number of coordinates with at least v votes: the mask's vote threshold then follows
// from N + 1 numbers, and the passes over the vote bytes do work that does not depend
// on how the votes are spread.
__device__ __forceinline__ void cast_vote(uint32_t* __restrict__ votes32, uint32_t j, uint32_t* lvl)
{
    const uint32_t sh = (j & 3u) * 8u;
    const uint32_t old = atomicAdd(&votes32[j >> 2], 1u << sh);
    atomicAdd(&lvl[((old >> sh) & 255u) + 1u], 1u);
}

// The vote-level counters in memory: kLvlSets sets of 256 that the workgroups take turns
// over, so that their atomics do not queue up on one cache line.
constexpr int kLvlSets = 32;
__device__ __forceinline__ void merge_levels(const uint32_t* lvl, uint32_t* __restrict__ lvl_sets, uint32_t wg)
{
    for (uint32_t v = threadIdx.x; v < 256u; v += blockDim.x) {
        const uint32_t c = lvl[v];
        if (c) atomicAdd(&lvl_sets[(size_t)(wg % kLvlSets) * 256 + v], c);
    }
}

// One slot per lane with `want` set, consecutive within the wavefront: one LDS atomic
// per wavefront instead of one per entry.  All lanes of the wavefront must call it.
__device__ __forceinline__ uint32_t wave_slots(bool want, uint32_t* counter, uint32_t lane)
{
    const uint64_t m = __ballot(want);
    if (m == 0ull) return 0u;                              // wave-uniform
    const int leader = __ffsll((long long)m) - 1;
    uint32_t base = 0;
    if (lane == (uint32_t)leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = __shfl(base, leader, kWave);
    return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
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
    __attribute__((aligned(16))) uint32_t rhist[kFineBins * kRep];   // the candidates' fine histogram, kRep copies
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

// Moves the members of fine-histogram bin `bin` into LDS: magnitude in lds.hist[p],
// coordinate in lds.ties[p], p = 0 .. in_bin-1 in no particular order.  The slots
// first receive the members' list positions; their coordinates are then fetched by
// all lanes together (one round trip, not one per member).  `in_bin` <= kKeyBins.
template <typename Keys>
__device__ __forceinline__ void collect_bin_members(const Keys& keys, const u32x2* __restrict__ crow, uint32_t tau,
                                                    uint32_t bin, uint32_t in_bin, SelectLds& lds)
{
    const uint32_t lane = lane_id(), t = threadIdx.x;
    keys.each([&](uint32_t k, uint64_t i, bool valid) {
        const bool mine = valid && fine_bin(k, tau) == bin;
        const uint32_t p = wave_slots(mine, &lds.n_list, lane);
        if (mine) {
            lds.hist[p] = k;
            lds.ties[p] = (uint32_t)i;
        }
    });
    __syncthreads();
    for (uint32_t p = t; p < in_bin; p += kRowThreads) lds.ties[p] = crow[lds.ties[p]].y;
    __syncthreads();
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
        // Values on a lattice put thousands of candidates on a few dozen keys, and LDS
        // atomics of one instruction that meet on one address are served one after the
        // other: lane l adds to copy l % kRep of the histogram, which divides those queues.
        {
            const u32x4 z = {0u, 0u, 0u, 0u};
            u32x4* rz = reinterpret_cast<u32x4*>(lds.rhist);
            for (int b = t; b < kFineBins * kRep / 4; b += kRowThreads) rz[b] = z;
        }
        __syncthreads();
        keys.each([&](uint32_t k, uint64_t, bool valid) {
            if (valid) atomicAdd(&lds.rhist[fine_bin(k, tau) * kRep + (lane & (kRep - 1))], 1u);
        });
        __syncthreads();
        uint32_t bin, want, in_bin;
        find_rank_bin<kFineBins, kRep>(lds.rhist, lds.scan, lds.bcast, K, bin, want, in_bin);
        if (in_bin <= (uint32_t)kRankCap) {       // uniform
            // few candidates in that bin: rank them by brute force under (magnitude desc,
            // coordinate asc); the one with exactly want-1 others ahead is the last of the top K
            collect_bin_members(keys, crow, tau, bin, in_bin, lds);
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
        if (Keys::kCheapPasses && in_bin <= (uint32_t)kKeyBins) {   // uniform; an extra pass only where passes are cheap
            // A crowded bin that still fits in LDS.  Values on a lattice put hundreds of
            // EQUAL magnitudes there: if all members share one key, that key is the K-th
            // largest and only the tie cut is left to find, among coordinates already in LDS.
            if (t < 2) lds.bcast[t] = t ? 0xFFFFFFFFu : 0u;          // max, min of the members' keys
            collect_bin_members(keys, crow, tau, bin, in_bin, lds);
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
                const bool mine = valid && k == kth;
                const uint32_t p = wave_slots(mine, &lds.n_list, lane);
                if (mine) lds.ties[p] = (uint32_t)i;
            });
            __syncthreads();
            for (uint32_t p = t; p < n_eq; p += kRowThreads) lds.ties[p] = crow[lds.ties[p]].y;
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

// Casts the votes of the list entries i with (i / kRowThreads) % parts == part:
// a taken candidate adds one to its coordinate's vote byte and, when the sorted
// vote lists are wanted (ssel != nullptr), is tallied in its 1024-coordinate
// segment (ssel was zeroed by the streaming pass).  Lanes of a wavefront hold
// consecutive list entries, which mostly share a segment (they are one run): the
// first lane of each group of equal segments adds the group's count.  All threads of
// the workgroup must call it.
template <int NT, bool MERGE>
__device__ __forceinline__ void cast_votes_of_share(const u32x2* __restrict__ crow, uint32_t C, uint32_t kth,
                                                    uint32_t tie_cut, uint32_t part, uint32_t parts,
                                                    uint32_t* __restrict__ votes32, uint32_t* lvl,
                                                    uint32_t* __restrict__ ssel)
{
    constexpr int kU = 8;                         // list entries per thread in flight together
    const uint32_t t = threadIdx.x, lane = lane_id();
    for (uint64_t q0 = part; q0 * NT < C; q0 += (uint64_t)parts * kU) {
        // all the loads, then all the vote atomics, then what depends on their results: a thread's
        // entries wait for memory together, not one after the other
        u32x2 c[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const uint64_t i = (q0 + (uint64_t)u * parts) * NT + t;
            const u32x2 none = {0u, 0xFFFFFFFFu};
            c[u] = (i < C) ? crow[i] : none;
        }
        // MERGE (long lists, where the atomics' rate at the memory side is what the step waits for): lanes
        // hold consecutive list entries, ascending inside a run, and a row votes at most once per
        // coordinate, so neighbouring taken lanes whose coordinates share a vote word (four bytes) cast
        // their votes with ONE atomic, the sum of their byte increments, issued by the first of them;
        // the returned word holds every byte's count before this row's vote.  Where the mask is dense
        // that is up to four votes per atomic (measured at K = d/100: 27 -> 19 us).  Short lists
        // wait for latency, not rate: there every taken lane issues its own.
        uint32_t old[kU];
        uint32_t taken_mask = 0;
        uint32_t ahead[kU];                           // lanes between this lane and the first of its group
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const bool taken = c[u].y != 0xFFFFFFFFu && is_taken(c[u], kth, tie_cut);
            if (taken) taken_mask |= 1u << u;
            const uint32_t inc = taken ? 1u << ((c[u].y & 3u) * 8u) : 0u;
            uint32_t before = 0;                      // lanes of the same group just below this one
            uint32_t sum = inc;
            if (MERGE) {
                const uint32_t key = taken ? (c[u].y >> 2) : (0xFFFFFF00u | lane);   // never equal to a neighbour's
                bool run = true;
#pragma unroll
                for (int k = 1; k < 4; ++k) {
                    const uint32_t below = __shfl_up(key, k, kWave);
                    run = run && lane >= (uint32_t)k && below == key;
                    before += run ? 1u : 0u;
                }
                run = true;
#pragma unroll
                for (int k = 1; k < 4; ++k) {
                    const uint32_t above_key = __shfl_down(key, k, kWave);
                    const uint32_t above_inc = __shfl_down(inc, k, kWave);
                    run = run && lane + (uint32_t)k < (uint32_t)kWave && above_key == key;
                    sum += run ? above_inc : 0u;
                }
            }
            ahead[u] = before;
            old[u] = 0;
            if (taken && before == 0u) old[u] = atomicAdd(&votes32[c[u].y >> 2], sum);
        }
        if (MERGE) {
#pragma unroll
            for (int u = 0; u < kU; ++u) old[u] = __shfl(old[u], lane - ahead[u], kWave);   // the group's returned word
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if ((q0 + (uint64_t)u * parts) * NT >= C) break;        // uniform over the workgroup
            const bool taken = (taken_mask >> u) & 1u;
            if (taken) atomicAdd(&lvl[((old[u] >> ((c[u].y & 3u) * 8u)) & 255u) + 1u], 1u);
            if (ssel) {
                const uint32_t sg = c[u].y / kSeg;
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
    }
}

// ---- the rows' select from registers ------------------------------------------
// A thread keeps, for each of its list entries, only the number of the entry's bin
// in the fine histogram (16 bits, two to a register; 0xFFFF: no entry): that is all
// the histogram pass and the search for the bin's members need, and it lets one
// workgroup hold lists of KEEP * 1024 entries.  The members of the bin that holds
// the K-th largest are then fetched from the list by position, all lanes together.
template <int KEEP>
struct PackedBins {
    uint32_t b[KEEP / 2];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int q = 0; q < KEEP / 2; ++q) b[q] = 0xFFFFFFFFu;
    }
    template <int Q>
    __device__ __forceinline__ void set(uint32_t bin)
    {
        if (Q & 1) b[Q / 2] = (b[Q / 2] & 0x0000FFFFu) | (bin << 16);
        else       b[Q / 2] = (b[Q / 2] & 0xFFFF0000u) | bin;
    }
    // f(bin, list position) for every entry slot below `count`, the same number of
    // times in every lane of the workgroup
    template <typename F>
    __device__ __forceinline__ void each(uint32_t count, F f) const
    {
#pragma unroll
        for (int q = 0; q < KEEP; ++q) {
            if ((uint32_t)q * kRowThreads < count) {              // uniform over the workgroup
                const uint32_t bin = (q & 1) ? (b[q / 2] >> 16) : (b[q / 2] & 0xFFFFu);
                f(bin, (uint32_t)q * kRowThreads + threadIdx.x);
            }
        }
    }
};

// Exact K-th largest magnitude and tie cut of a candidate list whose entries' bins
// are in registers.  Returns false when the bin of the K-th largest holds more
// members than the LDS lists take (the caller then runs the generic select).
// LDS use: rhist holds the histogram, then (words [0, 4096)) the members' magnitudes,
// ([4096, 8192)) their coordinates, ([8192, 12288)) the histogram of their exact keys.
template <int KEEP>
__device__ __forceinline__ bool select_from_bins(const PackedBins<KEEP>& bins, const u32x2* __restrict__ crow,
                                                 uint32_t C, uint32_t K, uint32_t tau, SelectLds& lds,
                                                 uint32_t& kth, uint32_t& tie_cut)
{
    static_assert(kFineBins * kRep >= 3 * kKeyBins, "the members' lists reuse the histogram's storage");
    const uint32_t lane = lane_id(), t = threadIdx.x;
    // (the caller has zeroed lds.rhist and lds.n_list, and a barrier has passed since)
    // Values on a lattice put thousands of candidates on a few dozen keys, and LDS
    // atomics of one instruction that meet on one address are served one after the
    // other: lane l adds to copy l % kRep of the histogram, which divides those queues.
    bins.each(C, [&](uint32_t bin, uint32_t) {
        if (bin != 0xFFFFu) atomicAdd(&lds.rhist[bin * kRep + (lane & (kRep - 1))], 1u);
    });
    __syncthreads();
    uint32_t bin, want, in_bin;
    find_rank_bin<kFineBins, kRep>(lds.rhist, lds.scan, lds.bcast, K, bin, want, in_bin);
    if (in_bin > (uint32_t)kKeyBins) return false;                  // uniform
    // the last bin is open-ended: its members' keys do not fit the exact-key histogram
    if (in_bin > (uint32_t)kRankCap && bin == (uint32_t)(kFineBins - 1)) return false;

    uint32_t* mkey = lds.rhist;                   // find_rank_bin ended with a barrier: the histogram is free
    uint32_t* mpos = lds.rhist + kKeyBins;
    {
        // the members' list positions, in no particular order: count, scan, place
        uint32_t mine = 0;
        bins.each(C, [&](uint32_t b, uint32_t) { mine += (b == bin); });
        uint64_t total;
        uint32_t p = (uint32_t)block_excl_scan64<kRowThreads>(mine, lds.scan, total);
        if (mine) bins.each(C, [&](uint32_t b, uint32_t i) { if (b == bin) mpos[p++] = i; });
    }
    __syncthreads();
    for (uint32_t p = t; p < in_bin; p += kRowThreads) {             // all lanes together: one round trip
        const u32x2 c = crow[mpos[p]];
        mkey[p] = c.x;
        mpos[p] = c.y;                            // from here on: the member's coordinate
    }
    __syncthreads();
    if (in_bin <= (uint32_t)kRankCap) {           // uniform
        // few members: ranked by counting under (magnitude desc, coordinate asc);
        // the one with exactly want-1 others ahead is the last of the top K
        if (t < 4) {                              // pad to a multiple of 4 with entries ranked last
            mkey[in_bin + t] = 0;
            mpos[in_bin + t] = 0xFFFFFFFFu;
        }
        __syncthreads();
        if (t < in_bin) {
            const uint32_t mk = mkey[t], mi = mpos[t];
            const u32x4* hk = reinterpret_cast<const u32x4*>(mkey);
            const u32x4* hi = reinterpret_cast<const u32x4*>(mpos);
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
        __syncthreads();
        return true;
    }
    // Values on a lattice put hundreds of EQUAL magnitudes there: if all members share one
    // key, that key is the K-th largest and only the tie cut is left to find.
    if (t == 0) lds.bcast[2] = 0;
    __syncthreads();
    {
        bool differs = false;
        const uint32_t k0 = mkey[0];
        for (uint32_t p = t; p < in_bin; p += kRowThreads) {
            differs |= mkey[p] != k0;
            lds.ties[p] = mpos[p];                // in_bin <= kKeyBins <= kTieCap
        }
        if (differs) lds.bcast[2] = 1;
    }
    __syncthreads();
    if (lds.bcast[2] == 0) {                      // uniform
        kth = mkey[0];
        __syncthreads();                          // everyone has read bcast and mkey
        tie_cut = want < in_bin ? smallest_coordinate(lds, in_bin, want) : 0xFFFFFFFFu;
        return true;
    }
    // up to 4096 members: the bin spans exactly 4096 key values, so a histogram over the
    // members' exact keys finds the K-th largest, and its ties' coordinates are in LDS
    uint32_t* h2 = lds.rhist + 2 * kKeyBins;
    const uint32_t bin_lo = tau + (bin << kFineShift);
    for (int b = t; b < kKeyBins; b += kRowThreads) h2[b] = 0;
    __syncthreads();
    for (uint32_t p0 = 0; p0 < in_bin; p0 += kRowThreads) {          // wave-wide grouping: many keys are equal
        const uint32_t p = p0 + t;
        tally_digit(h2, p < in_bin, p < in_bin ? (mkey[p] - bin_lo) & (uint32_t)(kKeyBins - 1) : 0u, lane);
    }
    __syncthreads();
    uint32_t sub, take_eq, n_eq;
    find_rank_bin<kKeyBins>(h2, lds.scan, lds.bcast, want, sub, take_eq, n_eq);
    kth = bin_lo + sub;
    tie_cut = 0xFFFFFFFFu;
    if (take_eq < n_eq) {                         // uniform: only the take_eq lowest coordinates of the ties
        if (t == 0) lds.n_list = 0;
        __syncthreads();
        for (uint32_t p0 = 0; p0 < in_bin; p0 += kRowThreads) {
            const uint32_t p = p0 + t;
            const bool mine = p < in_bin && mkey[p] == kth;
            const uint32_t s = wave_slots(mine, &lds.n_list, lane);
            if (mine) lds.ties[s] = mpos[p];
        }
        __syncthreads();
        tie_cut = smallest_coordinate(lds, n_eq, take_eq);
    }
    return true;
}

// parts workgroups per row; the grid is one-dimensional and workgroup ids are laid
// out so that the workgroups of one row have equal id % 8: consecutive ids go to
// different XCDs (each with an L2 of its own), so a row's list is then read from
// memory once and served to the row's other workgroups from that L2.
// Usual case: EVERY workgroup of a row runs the same exact select over the row's
// candidate list (the work is repeated rather than shared so that no workgroup
// waits for another): the K-th largest magnitude kth[row] and tie_cut[row], the
// largest coordinate taken among the candidates tied with it (0xFFFFFFFF: all ties
// taken).  Each workgroup then casts the votes of its share of the list.  With
// thresholds_only (add-drop voting) no vote is cast; with slow_rows_only the
// candidate lists are selected by the mv_sel_* kernels and their votes cast by
// mv_row_votes.
// If the candidate count is < K or overflowed the list (for instance a row of
// equal magnitudes), the row's first workgroup selects it exactly from memory (e
// already holds a = g + e), emits and casts its vote; slow_flag[row] = 1 tells the
// later kernels to skip the row.
// n_spec (<= kSpec): how many of a thread's list entries are fetched before the
// row's count is known (the list's storage holds cap entries; what lies at or
// beyond the count is ignored), so that the two loads do not queue up.
template <int KEEP>
__global__ __launch_bounds__(kRowThreads) void mv_row_select(
    const float* __restrict__ e, int64_t ld_e, int64_t d, uint32_t N, uint32_t K,
    const u32x2* __restrict__ cand, uint32_t cap, const uint32_t* __restrict__ row_count_sets,
    uint32_t row_count_set_words, const uint32_t* __restrict__ step_no,
    const unsigned long long* __restrict__ tau_pub, const uint32_t* __restrict__ row_poison,
    uint32_t* __restrict__ cand_count, uint32_t* __restrict__ tau_bits, uint32_t* __restrict__ kth_out, uint32_t* __restrict__ tie_cut_out,
    uint32_t* __restrict__ worker_idx, uint32_t* __restrict__ votes32,
    uint32_t* __restrict__ seg_sel, uint32_t nseg, uint32_t* __restrict__ lvl_sets,
    uint32_t* __restrict__ slow_flag, uint32_t parts, uint32_t n_spec, int thresholds_only, int slow_rows_only)
{
    __shared__ SelectLds lds;
    const uint32_t t = threadIdx.x;
    const uint32_t within = blockIdx.x % (8u * parts);
    const uint32_t row = (blockIdx.x / (8u * parts)) * 8u + within % 8u, part = within / 8u;
    if (row >= N) return;                         // whole workgroup
    const u32x2* crow = cand + (size_t)row * cap;
    uint32_t raw[kSpec];
#pragma unroll
    for (int q = 0; q < kSpec; ++q) {
        raw[q] = 0;
        if ((uint32_t)q < n_spec) raw[q] = crow[min((uint32_t)q * kRowThreads + t, cap - 1)].x;
        if ((q & 7) == 7) __builtin_amdgcn_sched_barrier(0);   // keep address arithmetic from piling up
    }
    // (the streaming kernel counted into the counter set of this step's parity)
    const uint32_t epoch = step_no[0] + 1u;
    uint32_t C = row_count_sets[(epoch & 1u) * row_count_set_words + row * kCounterStride];
    const uint32_t tau = (uint32_t)tau_pub[row * (kCounterStride / 2)];   // with the count, not after it
    // a row whose streaming wavefronts did not all see tau in time: its list is incomplete
    const bool poisoned = row_poison[row] == epoch;
    // the fine histogram is cleared while those loads are under way
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        u32x4* rz = reinterpret_cast<u32x4*>(lds.rhist);
        for (int b = t; b < kFineBins * kRep / 4; b += kRowThreads) rz[b] = z;
        if (t == 0) lds.n_list = 0;
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    if (poisoned) C = kRowPoison | C;             // reads as overflowed, here and for every later reader
    if (part == 0 && t == 0) {                    // for the kernels that follow, and the row statistics
        cand_count[row] = C;
        tau_bits[row] = tau;
        slow_flag[row] = 0;
    }
    const bool from_list = C >= K && C <= cap;
    if (slow_rows_only && from_list) return;      // whole workgroup
    if (!from_list && part != 0) return;          // whole workgroup

    if (from_list) {
        uint32_t kth = 0, tie_cut = 0, path = 0;
        bool done = false;
        if (tau != 0 && C <= (uint32_t)KEEP * kRowThreads) {
            PackedBins<KEEP> bins;
            bins.clear();
            auto pack = [&](auto qc, uint32_t key) {
                constexpr int Q = decltype(qc)::value;
                const uint32_t i = (uint32_t)Q * kRowThreads + t;
                bins.template set<Q>(i < C ? fine_bin(key, tau) : 0xFFFFu);
            };
            // what was fetched ahead, then the rest of the list
            static_for<0, (KEEP < kSpec ? KEEP : kSpec)>([&](auto qc) {
                constexpr int Q = decltype(qc)::value;
                if ((uint32_t)Q < n_spec && (uint32_t)Q * kRowThreads < C) pack(qc, raw[Q]);
            });
            // (sixteen loads at a time, all issued before the first is used: used one by one, each load
            // would wait for the one before)
            static_for<0, KEEP / 16>([&](auto gc) {
                constexpr int G = decltype(gc)::value;
                if ((uint32_t)(G * 16 + 15) >= n_spec && (uint32_t)(G * 16) * kRowThreads < C) {   // uniform
                    uint32_t more[16];
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        more[q] = 0;
                        if ((uint32_t)(G * 16 + q) >= n_spec && (uint32_t)(G * 16 + q) * kRowThreads < C)   // uniform
                            more[q] = crow[min((uint32_t)(G * 16 + q) * kRowThreads + t, cap - 1)].x;
                    }
                    static_for<0, 16>([&](auto qc) {
                        constexpr int Q = G * 16 + decltype(qc)::value;
                        if ((uint32_t)Q >= n_spec && (uint32_t)Q * kRowThreads < C)
                            pack(std::integral_constant<int, Q>{}, more[decltype(qc)::value]);
                    });
                }
            });
            done = select_from_bins<KEEP>(bins, crow, C, K, tau, lds, kth, tie_cut);
        }
        if (!done) {                              // uniform
            __syncthreads();
            path = 2;
            auto at = [crow](uint64_t i) { return crow[i].x; };
            const KeysInMemory<decltype(at)> src{at, C};
            uint32_t p2;
            select_among_candidates(src, crow, C, K, tau, lds, kth, tie_cut, p2);
        }
        if (part == 0 && t == 0) {
            kth_out[row] = kth;
            tie_cut_out[row] = tie_cut;
            if (path) slow_flag[row] = path;      // diagnostic only
        }
        if (!thresholds_only) {
            for (int i = t; i < 257; i += kRowThreads) lds.lvl[i] = 0;
            __syncthreads();
            cast_votes_of_share<kRowThreads, (KEEP > kKeepShort)>(crow, C, kth, tie_cut, part, parts, votes32, lds.lvl,
                                             seg_sel ? seg_sel + (size_t)row * nseg : nullptr);
            __syncthreads();
            merge_levels(lds.lvl, lvl_sets, blockIdx.x);
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
        uint32_t kk[4];
        uint32_t gt = 0, eq = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool valid = (j + c < d);
            kk[c] = valid ? (__float_as_uint(arow[j + c]) & kAbsMask) : 0u;
            gt += (valid && kk[c] > kth);
            eq += (valid && kk[c] == kth);
        }
        uint64_t total;
        const uint64_t ex = block_excl_scan64<kRowThreads>(pack2(gt, eq), lds.scan, total);
        uint32_t g0 = gt_before + (uint32_t)(ex >> 32), e0 = eq_before + (uint32_t)ex;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (j + c < d) {
                const bool is_gt = kk[c] > kth, is_eq = kk[c] == kth;
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
    merge_levels(lds.lvl, lvl_sets, blockIdx.x);
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
#pragma unroll
    for (int u = 0; u < kListPerThread; ++u)
        if (k[u] != 0xFFFFFFFFu) atomicAdd(&hist_lds[list_bin(k[u], base, a.shift)], 1u);
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
            k[q] = 0;
            if ((uint32_t)q * kRowThreads < C) k[q] = list2[min((uint32_t)q * kRowThreads + t, last)].x;
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

}  // namespace mvk
