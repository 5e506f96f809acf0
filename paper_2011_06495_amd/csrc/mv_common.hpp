// Types, constants and workgroup-wide helpers (scans) shared by the vote step's kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

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

// f(std::integral_constant<int, I>) for I = A .. B-1, unrolled at compile time
template <int A, int B, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (A < B) {
        f(std::integral_constant<int, A>{});
        static_for<A + 1, B>(f);
    }
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

// List length counters (the rows' candidate lists, the add-drop lists): many workgroups
// bump them with returning atomics, which complete one after the other per cache line,
// so every counter has a 128-byte line of its own.
constexpr uint32_t kCounterStride = 32;
__device__ __forceinline__ uint32_t ad_counter(uint32_t row, uint32_t which)
{
    return (2u * row + which) * kCounterStride;
}

}  // namespace mvk
