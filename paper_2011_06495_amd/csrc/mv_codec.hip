// Sparse position code of the paper's Sec. 4.3.1 on the GPU: encoder and decoder
// for batches of ascending coordinate lists (the workers' votes, the add / drop
// lists, the global mask).
//
// Stream of one list: the vector's d coordinates are cut into blocks of
// block_len = 1/phi; per listed position a 1 bit followed by the position inside
// its block in B = ceil(log2(block_len)) bits, most significant first; a 0 bit
// closes every block.  Bit k of a stream is bit k % 32 of its word k / 32.
// With n positions the stream has n (1 + B) + ceil(d / block_len) bits.
//
// Encoder: position i of the list lies in block b_i = idx[i] / block_len and is
// preceded by i codes and b_i closing bits, so its code starts at bit
// i (1 + B) + b_i -- no prefix sum is needed.  One thread per OUTPUT word finds the
// codes that overlap it by bisection over that increasing function and writes the
// word once: no atomics, no clearing pass, coalesced stores.
//
// Decoder: the receiver's parse is a finite automaton (state = offset bits still
// to skip, 0..B).  Each 64-bit chunk of the stream is run once for every possible
// entry state (exit state, codes begun, blocks closed); composing these maps along
// the stream gives every chunk its true entry state and the number of codes and
// closed blocks before it; a last pass parses each chunk for real and writes
// coordinate = closed blocks * block_len + offset at its place in the list.
#include "../../include/mv.h"

#include <mutex>

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mvc {

constexpr int kThreads = 256;
constexpr int kMaxB = 31;
constexpr int kChunkBits = 64;
constexpr int kWalkThreads = 1024;

__host__ __device__ inline int offset_bits(int64_t block_len)
{
    int b = 0;
    while (((int64_t)1 << b) < block_len) ++b;
    return b;
}

__device__ __forceinline__ uint32_t stream_bit(const uint32_t* __restrict__ w, uint64_t k)
{
    return (w[k >> 5] >> (k & 31u)) & 1u;
}

// first bit of the code of list entry i
__device__ __forceinline__ uint64_t code_start(const uint32_t* __restrict__ idx, uint32_t i, uint32_t code_len,
                                               uint32_t block_len)
{
    return (uint64_t)i * code_len + idx[i] / block_len;
}

__global__ __launch_bounds__(kThreads) void codec_encode_kernel(
    const uint32_t* __restrict__ idx, int64_t ld_idx, const uint32_t* __restrict__ counts, int64_t counts_stride,
    uint32_t n_fixed, int64_t d, uint32_t block_len, uint32_t B, uint32_t* __restrict__ streams, int64_t ld_words,
    unsigned long long* __restrict__ n_bits_out)
{
    const uint32_t row = blockIdx.y;
    // a length read from device memory is wire-side data: never trusted beyond the row's storage
    const uint32_t n = counts ? min(counts[(int64_t)row * counts_stride], n_fixed) : n_fixed;
    const uint32_t code_len = 1 + B;
    const uint64_t n_blocks = ((uint64_t)d + block_len - 1) / block_len;
    const uint64_t total = (uint64_t)n * code_len + n_blocks;
    const uint64_t n_words = (total + 31) / 32;
    const uint32_t* list = idx + (int64_t)row * ld_idx;
    if (blockIdx.x == 0 && threadIdx.x == 0) n_bits_out[row] = total;
    for (uint64_t w = (uint64_t)blockIdx.x * kThreads + threadIdx.x; w < n_words; w += (uint64_t)gridDim.x * kThreads) {
        const uint64_t lo_bit = w * 32, hi_bit = lo_bit + 32;
        // first entry whose code ends beyond the word's first bit
        uint32_t lo = 0, hi = n;
        while (lo < hi) {
            const uint32_t mid = lo + (hi - lo) / 2;
            if (code_start(list, mid, code_len, block_len) + code_len > lo_bit) hi = mid;
            else lo = mid + 1;
        }
        uint32_t word = 0;
        for (uint32_t i = lo; i < n; ++i) {
            const uint64_t s = code_start(list, i, code_len, block_len);
            if (s >= hi_bit) break;
            // the code as it lies in the stream, first bit in bit 0: the flag, then the offset MSB first
            const uint32_t off = list[i] % block_len;
            const uint64_t code = 1ull | ((uint64_t)(B ? (__brev(off) >> (32 - B)) : 0u) << 1);
            word |= (s >= lo_bit) ? (uint32_t)(code << (s - lo_bit)) : (uint32_t)(code >> (lo_bit - s));
        }
        streams[(int64_t)row * ld_words + w] = word;
    }
}

// ---- decoder -----------------------------------------------------------------

struct ChunkMap {                // what a chunk does to the parse, for one entry state
    uint8_t  exit_state;
    uint8_t  codes;              // codes begun in the chunk (at most 64)
    uint8_t  closed;             // blocks closed in the chunk (at most 64)
};

// up to 64 stream bits from bit `first` (a multiple of 64), first bit in bit 0;
// bits at or beyond `total` read as zero
__device__ __forceinline__ uint64_t load_chunk(const uint32_t* __restrict__ words, uint64_t first, uint64_t total)
{
    const uint64_t n_words = (total + 31) / 32, i = first >> 5;
    uint64_t v = (i < n_words) ? words[i] : 0u;
    if (i + 1 < n_words) v |= (uint64_t)words[i + 1] << 32;
    const uint64_t len = total - first;
    return len < 64 ? (v & ((1ull << len) - 1)) : v;
}

// `len` (at most 31) stream bits from bit k, first bit in bit 0; zero beyond `total`
__device__ __forceinline__ uint32_t load_field(const uint32_t* __restrict__ words, uint64_t k, uint32_t len,
                                               uint64_t total)
{
    const uint64_t n_words = (total + 31) / 32, i = k >> 5;
    uint64_t v = (i < n_words) ? words[i] : 0u;
    if (i + 1 < n_words) v |= (uint64_t)words[i + 1] << 32;
    uint32_t f = (uint32_t)(v >> (k & 31u)) & ((1u << len) - 1u);
    if (k + len > total) f &= (k < total) ? ((1u << (uint32_t)(total - k)) - 1u) : 0u;
    return f;
}

// Parse the `len` bits of a chunk held in `w`, entering with `state` offset bits
// still to skip.  Runs of zero flags are taken in one step, so the loop runs once
// per code.
__device__ __forceinline__ ChunkMap run_chunk(uint64_t w, uint32_t len, uint32_t state, uint32_t B)
{
    ChunkMap m = {0, 0, 0};
    uint32_t j = min(state, len);
    state -= j;
    while (j < len) {
        const uint64_t rest = w >> j;
        const uint32_t zeros = rest ? (uint32_t)__builtin_ctzll(rest) : 64u;
        const uint32_t run = min(zeros, len - j);
        m.closed += (uint8_t)run;
        j += run;
        if (j >= len) break;
        ++m.codes;                                   // flag bit, then B offset bits
        const uint32_t end = j + 1 + B;
        state = end > len ? end - len : 0;
        j = min(end, len);
    }
    m.exit_state = (uint8_t)state;
    return m;
}

// Three byte tables per row, each [chunk][state] with B + 1 states per chunk:
// exit state, codes begun, blocks closed.
struct MapTables {
    uint8_t* exit_state;
    uint8_t* codes;
    uint8_t* closed;
};

__device__ __forceinline__ MapTables row_tables(uint8_t* base, uint64_t max_chunks, uint32_t row)
{
    const uint64_t per_table = max_chunks * (kMaxB + 1);
    uint8_t* r = base + (uint64_t)row * 3 * per_table;
    return MapTables{r, r + per_table, r + 2 * per_table};
}

__global__ __launch_bounds__(kThreads) void codec_chunk_maps_kernel(
    const uint32_t* __restrict__ streams, int64_t ld_words, const unsigned long long* __restrict__ n_bits,
    uint64_t max_bits, uint32_t B, uint8_t* __restrict__ maps, uint64_t max_chunks)
{
    const uint32_t row = blockIdx.y;
    // the received length is wire-side data: clamped to what the scratch tables were sized for
    const uint64_t total = min((uint64_t)n_bits[row], max_bits);
    const uint64_t n_chunks = (total + kChunkBits - 1) / kChunkBits;
    const uint32_t* words = streams + (int64_t)row * ld_words;
    const uint32_t n_states = B + 1;
    const MapTables tb = row_tables(maps, max_chunks, row);
    for (uint64_t item = (uint64_t)blockIdx.x * kThreads + threadIdx.x; item < n_chunks * n_states;
         item += (uint64_t)gridDim.x * kThreads) {
        const uint64_t c = item / n_states;
        const uint32_t s = (uint32_t)(item % n_states);
        const uint64_t first = c * kChunkBits, last = min(first + kChunkBits, total);
        const ChunkMap m = run_chunk(load_chunk(words, first, total), (uint32_t)(last - first), s, B);
        tb.exit_state[item] = m.exit_state;      // compact: index = chunk * n_states + state
        tb.codes[item] = m.codes;
        tb.closed[item] = m.closed;
    }
}

struct Entry {                   // the parse at the start of a chunk
    uint32_t state;
    uint32_t codes;              // codes begun before the chunk
    uint32_t closed;             // blocks closed before the chunk
};

constexpr int kExitLds = 24576;  // exit-state bytes staged in LDS when the row's table fits

// One workgroup per row.  Thread t owns a contiguous range of chunks and composes
// the range's exit states for every entry state; 32 threads compose 32 ranges each;
// one thread walks the 32 groups from state 0; the true entry states then flow back
// down the two levels, and every thread walks its range for real, counting the codes
// and closed blocks before each chunk (a workgroup scan joins the ranges).
__global__ __launch_bounds__(kWalkThreads) void codec_walk_kernel(
    const unsigned long long* __restrict__ n_bits, uint64_t max_bits, uint32_t B, uint8_t* __restrict__ maps,
    uint64_t max_chunks, Entry* __restrict__ entries, uint32_t* __restrict__ counts_out)
{
    __shared__ uint8_t  ex_lds[kExitLds];
    __shared__ uint8_t  r_exit[kWalkThreads][kMaxB + 1];
    __shared__ uint8_t  g_exit[32][kMaxB + 1];
    __shared__ uint8_t  r_state[kWalkThreads];
    __shared__ uint8_t  g_state[32];
    __shared__ unsigned long long wave_sum[kWalkThreads / 64 + 1];
    const uint32_t row = blockIdx.x, t = threadIdx.x;
    const uint64_t total = min((uint64_t)n_bits[row], max_bits);
    const uint64_t n_chunks = (total + kChunkBits - 1) / kChunkBits;
    const uint64_t per = (n_chunks + kWalkThreads - 1) / kWalkThreads;
    const uint64_t c0 = min((uint64_t)t * per, n_chunks), c1 = min(c0 + per, n_chunks);
    const MapTables tb = row_tables(maps, max_chunks, row);
    const uint32_t n_states = B + 1;
    const bool staged = n_chunks * n_states <= (uint64_t)kExitLds;
    if (staged)
        for (uint64_t i = t; i < n_chunks * n_states; i += kWalkThreads) ex_lds[i] = tb.exit_state[i];
    __syncthreads();
    const uint8_t* ex = staged ? ex_lds : tb.exit_state;

    for (uint32_t s = 0; s < n_states; ++s) {                 // range maps
        uint32_t st = s;
        for (uint64_t c = c0; c < c1; ++c) st = ex[c * n_states + st];
        r_exit[t][s] = (uint8_t)st;
    }
    __syncthreads();
    if (t < 32)                                               // group maps: 32 ranges each
        for (uint32_t s = 0; s < n_states; ++s) {
            uint32_t st = s;
            for (uint32_t r = t * 32; r < t * 32 + 32; ++r) st = r_exit[r][st];
            g_exit[t][s] = (uint8_t)st;
        }
    __syncthreads();
    if (t == 0) {                                             // true entry state of every group
        uint32_t st = 0;
        for (uint32_t g = 0; g < 32; ++g) {
            g_state[g] = (uint8_t)st;
            st = g_exit[g][st];
        }
    }
    __syncthreads();
    if (t < 32) {                                             // ... of every range
        uint32_t st = g_state[t];
        for (uint32_t r = t * 32; r < t * 32 + 32; ++r) {
            r_state[r] = (uint8_t)st;
            st = r_exit[r][st];
        }
    }
    __syncthreads();
    // codes and closed blocks of the range on its true path, then their prefix over the ranges
    uint32_t st = r_state[t], codes = 0, closed = 0;
    for (uint64_t c = c0; c < c1; ++c) {
        codes += tb.codes[c * n_states + st];
        closed += tb.closed[c * n_states + st];
        st = ex[c * n_states + st];
    }
    unsigned long long v = ((unsigned long long)codes << 32) | closed, incl = v;
    const uint32_t lane = t & 63, wave = t / 64;
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(incl, o, 64);
        if (lane >= (uint32_t)o) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    if (t == 0) {
        unsigned long long run = 0;
        for (int w = 0; w < kWalkThreads / 64; ++w) {
            const unsigned long long x = wave_sum[w];
            wave_sum[w] = run;
            run += x;
        }
        wave_sum[kWalkThreads / 64] = run;
        counts_out[row] = (uint32_t)(run >> 32);
    }
    __syncthreads();
    const unsigned long long before = wave_sum[wave] + incl - v;
    Entry e;
    e.state = r_state[t];
    e.codes = (uint32_t)(before >> 32);
    e.closed = (uint32_t)before;
    for (uint64_t c = c0; c < c1; ++c) {                      // every chunk's entry
        entries[(uint64_t)row * max_chunks + c] = e;
        const uint64_t i = c * n_states + e.state;
        e.codes += tb.codes[i];
        e.closed += tb.closed[i];
        e.state = ex[i];
    }
}

__global__ __launch_bounds__(kThreads) void codec_emit_kernel(
    const uint32_t* __restrict__ streams, int64_t ld_words, const unsigned long long* __restrict__ n_bits,
    uint64_t max_bits, int64_t d, uint32_t block_len, uint32_t B, const Entry* __restrict__ entries,
    uint64_t max_chunks, uint32_t* __restrict__ idx_out, int64_t ld_idx, uint32_t max_n)
{
    const uint32_t row = blockIdx.y;
    const uint64_t total = min((uint64_t)n_bits[row], max_bits);
    const uint64_t n_chunks = (total + kChunkBits - 1) / kChunkBits;
    const uint32_t* words = streams + (int64_t)row * ld_words;
    uint32_t* out = idx_out + (int64_t)row * ld_idx;
    for (uint64_t c = (uint64_t)blockIdx.x * kThreads + threadIdx.x; c < n_chunks; c += (uint64_t)gridDim.x * kThreads) {
        Entry e = entries[(uint64_t)row * max_chunks + c];
        const uint64_t first = c * kChunkBits;
        const uint32_t len = (uint32_t)(min(first + kChunkBits, total) - first);
        const uint64_t w = load_chunk(words, first, total);
        uint32_t j = min(e.state, len);                                // rest of a code begun earlier
        while (j < len) {
            const uint64_t rest = w >> j;
            const uint32_t zeros = rest ? (uint32_t)__builtin_ctzll(rest) : 64u;
            const uint32_t run = min(zeros, len - j);
            e.closed += run;
            j += run;
            if (j >= len) break;
            // the offset lies MSB first in the stream and may run into the next chunk
            const uint32_t field = B ? load_field(words, first + j + 1, B, total) : 0u;
            const uint32_t off = B ? (__brev(field) >> (32 - B)) : 0u;
            const uint64_t pos = (uint64_t)e.closed * block_len + off;
            if (e.codes < max_n && pos < (uint64_t)d) out[e.codes] = (uint32_t)pos;
            ++e.codes;
            j += 1 + B;
        }
    }
}

}  // namespace mvc

extern "C" {

uint64_t mv_codec_stream_bits(int64_t n, int64_t d, int64_t block_len)
{
    if (n < 0 || d < 1 || block_len < 1 || block_len > 0x7FFFFFFFll || d > 0x7FFFFFFFll || n > d) return 0;
    return (uint64_t)n * (uint64_t)(1 + mvc::offset_bits(block_len)) + (uint64_t)((d + block_len - 1) / block_len);
}

size_t mv_codec_scratch_bytes(uint64_t max_bits, int32_t rows)
{
    if (rows < 1) return 0;
    const uint64_t chunks = (max_bits + mvc::kChunkBits - 1) / mvc::kChunkBits;
    return (size_t)rows * chunks * (3 * (mvc::kMaxB + 1) + sizeof(mvc::Entry)) + 512;
}

mv_status mv_codec_encode(const uint32_t* idx, int64_t ld_idx, const uint32_t* counts, int64_t counts_stride,
                          int64_t n, int32_t rows, int64_t d, int64_t block_len, uint32_t* streams,
                          int64_t ld_words, uint64_t* n_bits, void* stream)
{
    if (!idx || !streams || !n_bits || rows < 1 || rows > 65535) return MV_ERR_INVALID_ARG;
    if (d < 1 || d > 0x7FFFFFFFll || block_len < 1 || block_len > d || n < 0 || n > d || ld_idx < n)
        return MV_ERR_INVALID_ARG;
    if (counts && counts_stride < 1) return MV_ERR_INVALID_ARG;
    const uint64_t max_bits = mv_codec_stream_bits(n, d, block_len);
    const uint64_t max_words = (max_bits + 31) / 32;
    if ((uint64_t)ld_words < max_words) return MV_ERR_INVALID_ARG;
    uint64_t bx = (max_words + mvc::kThreads - 1) / mvc::kThreads;
    if (bx > 4096) bx = 4096;
    if (bx < 1) bx = 1;
    hipLaunchKernelGGL(mvc::codec_encode_kernel, dim3((uint32_t)bx, (uint32_t)rows), dim3(mvc::kThreads), 0,
                       static_cast<hipStream_t>(stream), idx, ld_idx, counts, counts_stride, (uint32_t)n, d,
                       (uint32_t)block_len, (uint32_t)mvc::offset_bits(block_len), streams, ld_words,
                       reinterpret_cast<unsigned long long*>(n_bits));
    return hipGetLastError() == hipSuccess ? MV_OK : MV_ERR_DEVICE;
}

// ---- the decoder's scratch for callers that cannot allocate -----------------
// One array per GPU, there from the moment the library's code is loaded on that GPU
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; what kernels and copies are given is the address that call
// returns for the device that is current, kept per device below.
static __device__ __align__(256) unsigned char scratch[MV_CODEC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void*      g_scratch_ptr[kMaxDevices];      // the array's address on each device, once asked for

// The address of `scratch` on the current device; asked for once per device.
mv_status static_scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return MV_ERR_DEVICE;
    if (dev >= kMaxDevices) return MV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MV_ERR_DEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MV_OK;
}
}  // namespace

static mv_status decode_with_scratch(const uint32_t* streams, int64_t ld_words, const uint64_t* n_bits,
                                     uint64_t max_bits, int32_t rows, int64_t d, int64_t block_len,
                                     uint32_t* idx_out, int64_t ld_idx, int64_t max_n, uint32_t* counts_out,
                                     void* scratch, void* stream)
{
    const uint64_t max_chunks = (max_bits + mvc::kChunkBits - 1) / mvc::kChunkBits;
    uintptr_t base = (reinterpret_cast<uintptr_t>(scratch) + 255) & ~(uintptr_t)255;
    uint8_t* maps = reinterpret_cast<uint8_t*>(base);
    const size_t maps_bytes = ((size_t)rows * max_chunks * 3 * (mvc::kMaxB + 1) + 255) & ~(size_t)255;
    mvc::Entry* entries = reinterpret_cast<mvc::Entry*>(base + maps_bytes);
    const uint32_t B = (uint32_t)mvc::offset_bits(block_len);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned long long* nb = reinterpret_cast<const unsigned long long*>(n_bits);
    uint64_t bx = (max_chunks * (B + 1) + mvc::kThreads - 1) / mvc::kThreads;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(mvc::codec_chunk_maps_kernel, dim3((uint32_t)bx, (uint32_t)rows), dim3(mvc::kThreads), 0, st,
                       streams, ld_words, nb, max_bits, B, maps, max_chunks);
    hipLaunchKernelGGL(mvc::codec_walk_kernel, dim3((uint32_t)rows), dim3(mvc::kWalkThreads), 0, st, nb, max_bits, B,
                       maps, max_chunks, entries, counts_out);
    uint64_t bx2 = (max_chunks + mvc::kThreads - 1) / mvc::kThreads;
    if (bx2 > 4096) bx2 = 4096;
    hipLaunchKernelGGL(mvc::codec_emit_kernel, dim3((uint32_t)bx2, (uint32_t)rows), dim3(mvc::kThreads), 0, st,
                       streams, ld_words, nb, max_bits, d, (uint32_t)block_len, B, entries, max_chunks, idx_out,
                       ld_idx, (uint32_t)max_n);
    return hipGetLastError() == hipSuccess ? MV_OK : MV_ERR_DEVICE;
}

static bool decode_args_valid(const uint32_t* streams, int64_t ld_words, const uint64_t* n_bits, uint64_t max_bits,
                              int32_t rows, int64_t d, int64_t block_len, const uint32_t* idx_out, int64_t ld_idx,
                              int64_t max_n, const uint32_t* counts_out)
{
    if (!streams || !n_bits || !idx_out || !counts_out || rows < 1 || rows > 65535) return false;
    if (d < 1 || d > 0x7FFFFFFFll || block_len < 1 || block_len > d || max_n < 0 || ld_idx < max_n ||
        max_n > 0xFFFFFFFFll)
        return false;
    if (ld_words < 0 || (uint64_t)ld_words * 32 < max_bits) return false;
    return max_bits != 0;
}

mv_status mv_codec_decode(const uint32_t* streams, int64_t ld_words, const uint64_t* n_bits, uint64_t max_bits,
                          int32_t rows, int64_t d, int64_t block_len, uint32_t* idx_out, int64_t ld_idx,
                          int64_t max_n, uint32_t* counts_out, void* scratch, size_t scratch_bytes, void* stream)
{
    if (!scratch || !decode_args_valid(streams, ld_words, n_bits, max_bits, rows, d, block_len, idx_out, ld_idx,
                                       max_n, counts_out))
        return MV_ERR_INVALID_ARG;
    if (scratch_bytes < mv_codec_scratch_bytes(max_bits, rows)) return MV_ERR_INVALID_ARG;
    return decode_with_scratch(streams, ld_words, n_bits, max_bits, rows, d, block_len, idx_out, ld_idx, max_n,
                               counts_out, scratch, stream);
}

mv_status mv_codec_decode_static(const uint32_t* streams, int64_t ld_words, const uint64_t* n_bits,
                                 uint64_t max_bits, int32_t rows, int64_t d, int64_t block_len, uint32_t* idx_out,
                                 int64_t ld_idx, int64_t max_n, uint32_t* counts_out, void* stream)
{
    if (!decode_args_valid(streams, ld_words, n_bits, max_bits, rows, d, block_len, idx_out, ld_idx, max_n,
                           counts_out))
        return MV_ERR_INVALID_ARG;
    if (mv_codec_scratch_bytes(max_bits, rows) > (size_t)MV_CODEC_STATIC_SCRATCH_BYTES) return MV_ERR_UNSUPPORTED;
    void* ptr = nullptr;
    const mv_status got = static_scratch_of_current_device(&ptr);
    if (got != MV_OK) return got;
    // the kernels write every scratch entry they later read: nothing of the last call's contents matters
    return decode_with_scratch(streams, ld_words, n_bits, max_bits, rows, d, block_len, idx_out, ld_idx, max_n,
                               counts_out, ptr, stream);
}

}  // extern "C"
