// Fractional quantisation of the paper's Sec. 4.3.2 on the GPU, for batches of
// rows (for instance the N workers' K masked values).
//
// q bits per value: q-1 bits name one of L = 2^(q-1) geometric intervals of |v|
// between the row's largest and smallest non-zero magnitude, one bit is the sign;
// L means (of the magnitudes that fell into each interval) follow, and the
// receiver reproduces sign * mean.
//
// The interval edges are computed in fp64 from correctly rounded operations only
// (a division, q-1 square roots -- L is a power of two, so that is the L-th root --
// and L-1 divisions), so they are the same numbers on any IEEE machine:
//   alpha = (v_max / v_min)^(1/L),  edge_0 = v_max,  edge_l = edge_{l-1} / alpha,
//   interval of |v| = 1 + #{ j in 1..L-1 : |v| <= edge_j }   (a value on an edge
//   goes to the interval of the smaller magnitudes; zeros go to the last one).
// code = (interval - 1) | sign << (q-1); value k occupies bits [k q, (k+1) q) of the
// row's stream, bit b of a stream being bit b % 32 of word b / 32.
//
// One workgroup per row: the data is tiny (K values), the work is latency.
#include "../../include/mv.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mvq {

constexpr int kThreads = 1024;
constexpr int kMaxL = 128;          // q <= 8
constexpr int kGroup = 32;          // most values per packing group (32 values = q whole words)

// values per packing group: the fewest whose codes fill whole words
__host__ __device__ constexpr int group_size(int q)
{
    int g = 32;
    while (g > 1 && ((g / 2) * q) % 32 == 0) g /= 2;
    return g;
}

__device__ __forceinline__ uint32_t interval_of(double m, const double* edges, int L)
{
    uint32_t l = 0;
    for (int j = 1; j < L; ++j) l += (m <= edges[j]) ? 1u : 0u;
    return l;                       // interval - 1
}

// partial[row][group][l] = sum of the magnitudes of the group's values in interval l, in index order
template <int q>                      // the bit budget is a template parameter: the packing indexes registers
__global__ __launch_bounds__(kThreads) void quant_encode_kernel(
    const float* __restrict__ vals, int64_t ld_vals, int64_t n, uint32_t* __restrict__ streams,
    int64_t ld_words, float* __restrict__ means, double* __restrict__ partial, uint32_t* __restrict__ pcount,
    int64_t n_groups)
{
    __shared__ uint32_t red_max[kThreads / 64], red_min[kThreads / 64];
    __shared__ double edges[kMaxL];
    constexpr int L = 1 << (q - 1);
    const uint32_t row = blockIdx.x, t = threadIdx.x;
    const float* v = vals + (int64_t)row * ld_vals;

    // largest and smallest non-zero magnitude, as bit patterns (same order as the values)
    uint32_t vmax = 0, vmin = 0xFFFFFFFFu;
    for (int64_t k = t; k < n; k += kThreads) {
        const uint32_t m = __float_as_uint(v[k]) & 0x7FFFFFFFu;
        vmax = max(vmax, m);
        if (m) vmin = min(vmin, m);
    }
    for (int o = 32; o >= 1; o >>= 1) {
        vmax = max(vmax, (uint32_t)__shfl_xor(vmax, o, 64));
        vmin = min(vmin, (uint32_t)__shfl_xor(vmin, o, 64));
    }
    if ((t & 63) == 0) {
        red_max[t / 64] = vmax;
        red_min[t / 64] = vmin;
    }
    __syncthreads();
    if (t == 0) {
        for (int w = 1; w < kThreads / 64; ++w) {
            vmax = max(vmax, red_max[w]);
            vmin = min(vmin, red_min[w]);
        }
        if (vmax == 0) {
            for (int l = 0; l < L; ++l) edges[l] = 0.0;
        } else {
            const double hi = (double)__uint_as_float(vmax), lo = (double)__uint_as_float(vmin);
            double alpha = hi / lo;
            for (int r = 0; r < q - 1; ++r) alpha = sqrt(alpha);
            edges[0] = hi;
            for (int l = 1; l < L; ++l) edges[l] = edges[l - 1] / alpha;
        }
    }
    __syncthreads();

    // codes: a thread packs groups of 32 consecutive values into q whole words
    uint32_t* out = streams + (int64_t)row * ld_words;
    double* prow = partial + (int64_t)row * n_groups * L;
    uint32_t* crow = pcount + (int64_t)row * n_groups * L;
    constexpr int G = group_size(q);                 // G values = G q / 32 whole words
    constexpr int gw = G * q / 32;
    for (int64_t g = t; g < n_groups; g += kThreads) {
        // the group's values in registers: codes first, then per-interval sums in index order
        uint32_t words[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        float    mag[kGroup];
        uint8_t  lv[kGroup];
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int64_t k = g * G + i;
            const bool live = k < n;
            const float x = live ? v[k] : 0.0f;
            mag[i] = fabsf(x);
            const uint32_t l = live ? interval_of((double)mag[i], edges, L) : 0xFFu;
            lv[i] = (uint8_t)l;
            if (live) {
                const uint32_t code = l | ((__float_as_uint(x) >> 31) << (q - 1));
                const uint32_t bit = (uint32_t)i * (uint32_t)q;
                words[bit >> 5] |= code << (bit & 31);
                if ((bit & 31) + q > 32) words[(bit >> 5) + 1] |= code >> (32 - (bit & 31));
            }
        }
        for (int l = 0; l < L; ++l) {
            double s = 0.0;
            uint32_t c = 0;
#pragma unroll
            for (int i = 0; i < G; ++i)
                if (lv[i] == (uint8_t)l) {
                    s += (double)mag[i];
                    ++c;
                }
            prow[g * L + l] = s;
            crow[g * L + l] = c;
        }
        const int64_t w0 = g * gw;
        const int64_t n_words = ((int64_t)n * q + 31) / 32;
        for (int w = 0; w < gw; ++w)
            if (w0 + w < n_words) out[w0 + w] = words[w];
    }
    __syncthreads();
    // means: one wavefront per interval; lane j adds the partial sums of groups j, j+64, ...
    // and the lanes are then added in a fixed tree, so the result does not depend on timing
    for (int l = (int)(t / 64); l < L; l += kThreads / 64) {
        double s = 0.0;
        uint32_t c = 0;
        for (int64_t g = t & 63; g < n_groups; g += 64) {
            s += prow[g * L + l];
            c += crow[g * L + l];
        }
        for (int o = 32; o >= 1; o >>= 1) {
            s += __shfl_xor(s, o, 64);
            c += __shfl_xor(c, o, 64);
        }
        if ((t & 63) == 0) means[(int64_t)row * L + l] = c ? (float)(s / (double)c) : 0.0f;
    }
}

__global__ __launch_bounds__(256) void quant_decode_kernel(const uint32_t* __restrict__ streams, int64_t ld_words,
                                                           int64_t n, int32_t q, const float* __restrict__ means,
                                                           float* __restrict__ out, int64_t ld_out)
{
    const uint32_t row = blockIdx.y;
    const int L = 1 << (q - 1);
    const uint32_t* w = streams + (int64_t)row * ld_words;
    const float* mu = means + (int64_t)row * L;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < n; k += (int64_t)gridDim.x * 256) {
        const uint64_t bit = (uint64_t)k * (uint64_t)q;
        uint32_t code = w[bit >> 5] >> (bit & 31);
        if ((bit & 31) + q > 32) code |= w[(bit >> 5) + 1] << (32 - (bit & 31));
        code &= (1u << q) - 1;
        const float m = mu[code & (uint32_t)(L - 1)];
        out[(int64_t)row * ld_out + k] = (code >> (q - 1)) ? -m : m;
    }
}

}  // namespace mvq

extern "C" {

size_t mv_quant_scratch_bytes(int64_t n, int32_t rows, int32_t q)
{
    if (n < 1 || rows < 1 || q < 2 || q > 8) return 0;
    const int64_t groups = (n + mvq::group_size(q) - 1) / mvq::group_size(q);
    return (size_t)rows * (size_t)groups * (size_t)(1 << (q - 1)) * (sizeof(double) + sizeof(uint32_t)) + 256;
}

mv_status mv_quant_encode(const float* vals, int64_t ld_vals, int64_t n, int32_t rows, int32_t q,
                          uint32_t* streams, int64_t ld_words, float* means, void* scratch, size_t scratch_bytes,
                          void* stream)
{
    if (!vals || !streams || !means || !scratch) return MV_ERR_INVALID_ARG;
    if (n < 1 || rows < 1 || rows > 65535 || q < 2 || q > 8 || ld_vals < n) return MV_ERR_INVALID_ARG;
    if (ld_words < (n * q + 31) / 32) return MV_ERR_INVALID_ARG;
    if (scratch_bytes < mv_quant_scratch_bytes(n, rows, q)) return MV_ERR_INVALID_ARG;
    const int64_t groups = (n + mvq::group_size(q) - 1) / mvq::group_size(q);
    const int L = 1 << (q - 1);
    uintptr_t base = (reinterpret_cast<uintptr_t>(scratch) + 255) & ~(uintptr_t)255;
    double* partial = reinterpret_cast<double*>(base);
    uint32_t* pcount = reinterpret_cast<uint32_t*>(base + (size_t)rows * groups * L * sizeof(double));
    hipStream_t st = static_cast<hipStream_t>(stream);
#define MV_QUANT_LAUNCH(Q)                                                                                     \
    case Q:                                                                                                    \
        hipLaunchKernelGGL(mvq::quant_encode_kernel<Q>, dim3((uint32_t)rows), dim3(mvq::kThreads), 0, st, vals, \
                           ld_vals, n, streams, ld_words, means, partial, pcount, groups);                     \
        break;
    switch (q) {
        MV_QUANT_LAUNCH(2) MV_QUANT_LAUNCH(3) MV_QUANT_LAUNCH(4) MV_QUANT_LAUNCH(5)
        MV_QUANT_LAUNCH(6) MV_QUANT_LAUNCH(7) MV_QUANT_LAUNCH(8)
        default: return MV_ERR_INVALID_ARG;
    }
#undef MV_QUANT_LAUNCH
    return hipGetLastError() == hipSuccess ? MV_OK : MV_ERR_DEVICE;
}

mv_status mv_quant_decode(const uint32_t* streams, int64_t ld_words, int64_t n, int32_t rows, int32_t q,
                          const float* means, float* out, int64_t ld_out, void* stream)
{
    if (!streams || !means || !out) return MV_ERR_INVALID_ARG;
    if (n < 1 || rows < 1 || rows > 65535 || q < 2 || q > 8 || ld_out < n) return MV_ERR_INVALID_ARG;
    if (ld_words < (n * q + 31) / 32) return MV_ERR_INVALID_ARG;
    int64_t bx = (n + 255) / 256;
    if (bx > 1024) bx = 1024;
    hipLaunchKernelGGL(mvq::quant_decode_kernel, dim3((uint32_t)bx, (uint32_t)rows), dim3(256), 0,
                       static_cast<hipStream_t>(stream), streams, ld_words, n, q, means, out, ld_out);
    return hipGetLastError() == hipSuccess ? MV_OK : MV_ERR_DEVICE;
}

}  // extern "C"
