/*
 * mv.h -- C ABI of the majority-voting vote step for AMD MI355X (gfx950).
 *
 * One call of mv_vote_step() is one iteration of sparse SGD with majority
 * voting for N workers whose vectors are held as an N x d matrix on one GPU
 * (paper: Algorithm 1, from the error compensation to the error update):
 *
 *   a[n][j]      = g[n][j] + e[n][j]                      (error compensation)
 *   worker_idx[n] = supp S_top(|a[n]|, K)                 (local mask, the vote)
 *   votes[j]     = #{ n : j in worker_idx[n] }            (vote count, Sec. 2)
 *   mask_idx     = supp S_top(votes, K)                   (global mask, Sec. 2 mask equation)
 *   agg[k]       = (sum_n a[n][mask_idx[k]]) * (1/N)      (masked send + aggregate; mean of Sec. 2)
 *   e[n][j]      = 0 if j in mask_idx else a[n][j]        (error update)
 *
 * S_top(x, K) marks the K entries with the highest values; the paper does not
 * say how ties are broken.  Here ties go to the LOWEST index, both for the
 * magnitudes of a row and for the vote counts.  "Highest absolute value" is the
 * order of the fp32 bit pattern with the sign bit cleared (so -0 == +0,
 * denormals are ordered and never flushed, and an infinity of either sign is
 * above all finite values; equal infinities tie like any equal magnitudes).
 * Infinite values are handled exactly as long as no NaN arises from them
 * (Inf - Inf in g + e or in the sum over workers).  NaN, given or arising, is
 * outside the contract: the values written are then unspecified (a NaN's
 * payload after an addition is the processor's choice); the call still ends,
 * every index written is a coordinate below d, index lists stay ascending and
 * nothing outside the output arrays is touched.
 *
 * All tensor pointers are DEVICE pointers owned by the caller.  The library
 * keeps none of them after a call returns, except cfg.workspace, which must
 * outlive the context.  Nothing throws; every entry point returns a status.
 */
#ifndef MV_H
#define MV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mv_ctx mv_ctx; /* opaque */

typedef enum {
    MV_OK = 0,
    MV_ERR_INVALID_ARG = 1, /* null pointer, size out of range, misalignment, bad struct_size */
    MV_ERR_UNSUPPORTED = 2,
    MV_ERR_ALLOC = 3,       /* device or host allocation failed */
    MV_ERR_DEVICE = 4,      /* a HIP call failed */
    MV_ERR_STATE = 5        /* context already ended, or an earlier step on it failed with MV_ERR_DEVICE */
} mv_status;

typedef enum { MV_F32 = 0, MV_BF16 = 1 } mv_dtype;          /* dtype of g only; e and agg are fp32 */
typedef enum { MV_REDUCE_MEAN = 0, MV_REDUCE_SUM = 1 } mv_reduce;
/* mv_config.flags: the context also carries the scratch of mv_ad_vote_step */
#define MV_FLAG_ADD_DROP 1

typedef struct {
    uint32_t struct_size;   /* = sizeof(mv_config) */
    int32_t  device;        /* HIP device ordinal */
    int32_t  n_workers;     /* N, 1..255 (a vote count fits one byte) */
    int32_t  grad_dtype;    /* mv_dtype */
    int64_t  d;             /* coordinates per worker, 1 .. 2^31-1 */
    int64_t  k;             /* K, 1 .. d */
    int32_t  reduce;        /* mv_reduce; MEAN is Sec. 2's definition, SUM is Algorithm 1's last line */
    int32_t  flags;         /* MV_FLAG_* bits; unknown bits are refused */
    void*    workspace;     /* optional device scratch of >= mv_workspace_bytes(); NULL: the context allocates it */
    size_t   workspace_bytes;
} mv_config;

/*
 * Bytes of device scratch a context for this configuration needs.  Pure host
 * arithmetic, no device call.  Returns 0 if the configuration is invalid.
 */
size_t mv_workspace_bytes(const mv_config* cfg);

/*
 * Creates a context: validates cfg on the host first (no device call is made
 * for an invalid configuration), then allocates and zeroes the scratch.
 * cfg.workspace, when given, must be 256-byte aligned device memory.
 * Errors: MV_ERR_INVALID_ARG (null, struct_size, N, d, k, dtype, reduce,
 * unknown flags, workspace too small or misaligned), MV_ERR_ALLOC, MV_ERR_DEVICE.
 */
mv_status mv_begin(const mv_config* cfg, mv_ctx** out_ctx);

/*
 * One vote step (Algorithm 1, error compensation .. error update), enqueued on
 * `stream`; returns without waiting for the GPU and allocates nothing.
 *
 *   grads      device, N rows of d elements (fp32 or bf16 per cfg), row stride ld_g elements
 *   err        device, N rows of d fp32, row stride ld_e; in: e_t, out: e_{t+1} (in place)
 *   worker_idx device, N x K uint32 out, row n = the coordinates worker n votes for,
 *              ascending; may be NULL
 *   votes      device, d bytes out, votes[j] in 0..N; may be NULL
 *   mask_idx   device, K uint32 out, ascending
 *   agg_vals   device, K fp32 out, agg_vals[k] belongs to coordinate mask_idx[k]
 *   stream     hipStream_t, NULL = the default stream
 *
 * Only the first d elements of each row are read or written.  Row starts must
 * be 16-byte aligned: base pointers 16-byte aligned, ld_g a multiple of 4
 * (fp32) or 8 (bf16), ld_e a multiple of 4; mask_idx, agg_vals and worker_idx
 * 4-byte aligned.  The buffers must not overlap each other.
 *
 * Argument errors are found on the host before anything is enqueued, so err is
 * untouched when the call fails with MV_ERR_INVALID_ARG or MV_ERR_STATE.
 * Calls on one context must not overlap in time (one stream at a time); distinct
 * contexts are independent.  The result does not depend on earlier calls.
 */
mv_status mv_vote_step(mv_ctx* ctx,
                       const void* grads, int64_t ld_g,
                       float* err, int64_t ld_e,
                       uint32_t* worker_idx,
                       uint8_t* votes,
                       uint32_t* mask_idx,
                       float* agg_vals,
                       void* stream);

/*
 * One iteration of majority voting with random selection (paper: Algorithm 1, the
 * line with S_rand-weighted; Sec. 2, paragraph after Algorithm 1; Sec. 4.2),
 * enqueued on `stream` like mv_vote_step and with the same arguments, outputs and
 * error behaviour, except for how the mask is chosen: winners are drawn at random,
 * a coordinate's chance growing in proportion to its votes, until K distinct ones
 * are selected.  The paper names no sampler; here every voted coordinate j gets the
 * time rand_exp[j] / votes[j] (one correctly rounded fp32 division) and the K
 * soonest win, equal times going to the lowest coordinate.  With rand_exp[j]
 * independent Exp(1) variates this is that law (successive sampling without
 * replacement); the random numbers are the caller's, so a step is reproducible.
 *
 *   rand_exp   device, d fp32, non-negative and finite, 4-byte aligned; in.  Only the
 *              entries of voted coordinates are read.  Use fresh numbers every step.
 *   mask_idx   device, K uint32, ascending; out.  Every coordinate in it has a vote.
 *
 * worker_idx and votes (both optional) are those of mv_vote_step.  MV_ERR_INVALID_ARG
 * also for a null or misaligned rand_exp.
 */
mv_status mv_rs_vote_step(mv_ctx* ctx,
                          const void* grads, int64_t ld_g,
                          float* err, int64_t ld_e,
                          const float* rand_exp,
                          uint32_t* worker_idx,
                          uint8_t* votes,
                          uint32_t* mask_idx,
                          float* agg_vals,
                          void* stream);

/*
 * One iteration of majority voting with add-drop (paper: Algorithm 2, Sec. 3),
 * enqueued on `stream` like mv_vote_step.  The context must have been begun with
 * MV_FLAG_ADD_DROP (else MV_ERR_STATE).  Every worker keeps a standing vote
 * M~_n; per step at most k_ad coordinates join it (the k_ad largest |a| among
 * the worker's current top-K that are not in it) and at most k_ad leave it (the
 * k_ad smallest |a| among its members that are not in the current top-K), ties to
 * the lowest coordinate in both; M^sum, the sum of the standing votes, moves
 * with them, and the mask is the K most voted coordinates of M^sum.  The state is
 * the caller's (zero it to start; a first step with k_ad = K then is a plain
 * majority vote):
 *
 *   vote_bits  device, N rows of ld_bits 32-bit words, bit (j % 32) of word j / 32 of
 *              row n = M~_n[j]; in/out.  ld_bits >= ceil(d/32) rounded up to a multiple
 *              of 4, itself a multiple of 4; 16-byte aligned; at most K bits per row
 *   msum       device, d bytes rounded up to a multiple of 16 (the padding stays
 *              zero), 16-byte aligned; in: M^sum_{t-1}, out: M^sum_t
 *   k_ad       1 .. K
 *   add_idx    device, N x k_ad uint32 out: row n = the coordinates added to M~_n,
 *              ascending, counts[2n] of them valid
 *   drop_idx   device, N x k_ad uint32 out: the coordinates removed, counts[2n+1] valid
 *   counts     device, 2N uint32 out
 *   grads, err, mask_idx, agg_vals: as in mv_vote_step (err is updated with the mask
 *              of this step)
 *
 * Errors as mv_vote_step, plus MV_ERR_INVALID_ARG for k_ad, ld_bits, alignment or a
 * null state / output pointer.
 */
mv_status mv_ad_vote_step(mv_ctx* ctx,
                          const void* grads, int64_t ld_g,
                          float* err, int64_t ld_e,
                          int64_t k_ad,
                          uint32_t* vote_bits, int64_t ld_bits,
                          uint8_t* msum,
                          uint32_t* add_idx, uint32_t* drop_idx, uint32_t* counts,
                          uint32_t* mask_idx, float* agg_vals,
                          void* stream);

/*
 * Ends the context: waits for the stream of the context's last step (steps are
 * serialized by the caller, so that is the only one with work of this context
 * still in flight), frees scratch the context allocated
 * (never cfg.workspace).  The handle stays a valid pointer so that a later
 * mv_vote_step / mv_end on it reports MV_ERR_STATE; mv_release frees it.
 */
mv_status mv_end(mv_ctx* ctx);

/* Frees the handle itself (ends the context first if needed). NULL is allowed. */
void mv_release(mv_ctx* ctx);

/* Static string for a status code; never NULL, never freed. */
const char* mv_status_string(mv_status s);

/* ---- measurement hooks (not part of the method) ------------------------- */

/* Number of kernels one vote step launches, and their names (static strings). */
int32_t     mv_kernel_count(void);
const char* mv_kernel_name(int32_t i);

/*
 * level 0: no events (default).  level 1: the step records a pair of HIP
 * events around its dominant kernel (the streaming error-compensation pass).
 * level 2: a pair around every kernel.
 */
mv_status mv_set_profiling(mv_ctx* ctx, int32_t level);

/*
 * Inside the streaming kernel the wavefronts of a row wait for the row's threshold
 * estimate, which other workgroups of the same launch publish; the wait is bounded by
 * `polls` looks at memory (default 2^20, about a second), after which the wavefront
 * gives up and the row is selected exactly from memory instead.  The same bound holds
 * for the one other wait between workgroups: a block of the mask kernel waits for the
 * counts of the blocks before it, and if it gives up the kernel behind it finds the
 * mask from the counts instead.  Results never depend on the bound.  A test hook: 0
 * makes every waiter that does not find what it needs at its first look give up, which
 * forces both alternative paths without any kernel waiting.
 */
mv_status mv_set_spin_limit(mv_ctx* ctx, uint32_t polls);

/*
 * Durations, in milliseconds, of the kernels of the step enqueued `steps_back`
 * steps ago on this context (0 = the last one; the last 64 steps are kept),
 * one per kernel in mv_kernel_name order, -1 for kernels that were not
 * bracketed at the level then in force.  Waits for that step's events.  `ms`
 * is a HOST array of n >= mv_kernel_count() floats.
 */
mv_status mv_step_kernel_ms(mv_ctx* ctx, int32_t steps_back, float* ms, int32_t n);

/*
 * Diagnostics of the LAST step (waits for the stream the step ran on): per
 * worker row, how many candidates the streaming pass kept (cand_count), the
 * magnitude bit pattern it compared against (threshold_bits) and how the row's
 * K-th magnitude was found (slow_path: 0 = from the candidates through their
 * fine histogram, 2 = the generic select over the candidates, 1 = the slow exact
 * path over the whole row in memory).  A cand_count with its top bit set marks a row
 * whose wavefronts did not all see the threshold in time (see mv_set_spin_limit).
 * HOST arrays of N uint32 each; any may be NULL.
 */
mv_status mv_last_step_row_stats(mv_ctx* ctx, uint32_t* cand_count,
                                 uint32_t* threshold_bits, uint32_t* slow_path);

/* ---- sparse position code (paper: Sec. 4.3.1) ------------------------------ */

/*
 * The code of an ascending list of n coordinates of a d-vector: the coordinates
 * are cut into blocks of block_len = 1/phi; per listed coordinate a 1 bit and the
 * position inside its block in B = ceil(log2(block_len)) bits, most significant
 * first; a 0 bit closes every block (also empty ones and the last, shorter one).
 * Bit k of a stream is bit k % 32 of its 32-bit word k / 32; unused bits of the
 * last word are 0.  A stream has n (1 + B) + ceil(d / block_len) bits, i.e.
 * log2(1/phi) + 2 bits per coordinate when n = phi d (Sec. 2.1).
 * Returns that length in bits (host arithmetic), 0 for invalid arguments.
 */
uint64_t mv_codec_stream_bits(int64_t n, int64_t d, int64_t block_len);

/* Bytes of device scratch mv_codec_decode needs for `rows` streams of up to max_bits bits. */
size_t mv_codec_scratch_bytes(uint64_t max_bits, int32_t rows);

/*
 * Encodes `rows` lists at once (for instance the N workers' votes), enqueued on
 * `stream`; allocates nothing.
 *   idx       device, row r = idx + r * ld_idx: ascending coordinates < d
 *   counts    device or NULL: the length of row r is counts[r * counts_stride]
 *             (a value above n is read as n); NULL: every row holds n coordinates
 *   streams   device out, row r = streams + r * ld_words; ld_words >=
 *             ceil(mv_codec_stream_bits(n, d, block_len) / 32); words beyond a
 *             row's stream are left untouched
 *   n_bits    device out, rows entries: the length of each stream in bits
 * Lists that are not ascending or reach beyond d give an unspecified stream (no
 * out-of-bounds access).  Errors: MV_ERR_INVALID_ARG, MV_ERR_DEVICE.
 */
mv_status mv_codec_encode(const uint32_t* idx, int64_t ld_idx, const uint32_t* counts, int64_t counts_stride,
                          int64_t n, int32_t rows, int64_t d, int64_t block_len, uint32_t* streams,
                          int64_t ld_words, uint64_t* n_bits, void* stream);

/*
 * Decodes `rows` streams as the receiver of Sec. 4.3.1 reads them (a 1 bit: the
 * next B bits are a position inside the current block; a 0 bit: next block).
 *   streams, ld_words   device, as written by mv_codec_encode
 *   n_bits    device, rows entries: the length of each stream in bits (a value above
 *             max_bits is read as max_bits)
 *   idx_out   device out, row r = idx_out + r * ld_idx, room for max_n coordinates
 *   counts_out device out, rows entries: coordinates found in each stream (those
 *             beyond max_n are counted but not written)
 *   scratch   device, >= mv_codec_scratch_bytes(max_bits, rows) bytes
 * Malformed streams give unspecified lists (no out-of-bounds access).
 */
mv_status mv_codec_decode(const uint32_t* streams, int64_t ld_words, const uint64_t* n_bits, uint64_t max_bits,
                          int32_t rows, int64_t d, int64_t block_len, uint32_t* idx_out, int64_t ld_idx,
                          int64_t max_n, uint32_t* counts_out, void* scratch, size_t scratch_bytes, void* stream);

/*
 * mv_codec_decode for callers that cannot allocate device memory and have no
 * scratch buffer to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * mv_codec_decode without `scratch` / `scratch_bytes`: the decoder's tables live
 * in an array of MV_CODEC_STATIC_SCRATCH_BYTES bytes that is part of the
 * library's device code (every GPU the library runs on holds its own copy from
 * the first call on it until the process ends).  The call allocates and frees
 * nothing, on the device or through any library.
 *   - mv_codec_scratch_bytes(max_bits, rows) must not exceed
 *     MV_CODEC_STATIC_SCRATCH_BYTES, else MV_ERR_UNSUPPORTED (nothing is enqueued);
 *     MV_ERR_UNSUPPORTED also for a device number of 64 or more.
 *   - The array is shared by every call on a GPU, whatever the stream: two calls
 *     that may overlap in time on one GPU race on it and must be ordered by the
 *     caller (same stream, or an event between them).  mv_codec_decode with
 *     buffers of its own has no such limit.
 *   - Runs on the CURRENT device, enqueued on `stream`.
 */
#define MV_CODEC_STATIC_SCRATCH_BYTES (16u << 20)
mv_status mv_codec_decode_static(const uint32_t* streams, int64_t ld_words, const uint64_t* n_bits,
                                 uint64_t max_bits, int32_t rows, int64_t d, int64_t block_len, uint32_t* idx_out,
                                 int64_t ld_idx, int64_t max_n, uint32_t* counts_out, void* stream);

/* ---- fractional quantisation (paper: Sec. 4.3.2) --------------------------- */

/*
 * q bits per value (2 <= q <= 8): q-1 bits name one of L = 2^(q-1) geometric
 * intervals of |v| between the row's largest and smallest non-zero magnitude,
 * I_l = [v_max / alpha^(l-1), v_max / alpha^l], alpha = (v_max / v_min)^(1/L); one
 * bit is the sign; L means of the magnitudes that fell into the intervals follow
 * and the receiver reproduces sign * mean.  The paper leaves the arithmetic of the
 * edges open; here they are fp64 numbers from correctly rounded operations only
 * (alpha by q-1 square roots of v_max / v_min, edge_l = edge_{l-1} / alpha), a value
 * on an edge goes to the interval of the smaller magnitudes and zeros to the last.
 *   vals      device, `rows` rows of n fp32 values, row stride ld_vals
 *   streams   device out, row stride ld_words >= ceil(n q / 32): value k occupies
 *             bits [k q, (k+1) q) of its row's stream (bit b = bit b % 32 of word
 *             b / 32), code = (interval - 1) | sign << (q - 1)
 *   means     device out, rows x L fp32 (0 for an empty interval)
 *   scratch   device, >= mv_quant_scratch_bytes(n, rows, q)
 * Enqueued on `stream`; allocates nothing.
 */
size_t    mv_quant_scratch_bytes(int64_t n, int32_t rows, int32_t q);
mv_status mv_quant_encode(const float* vals, int64_t ld_vals, int64_t n, int32_t rows, int32_t q,
                          uint32_t* streams, int64_t ld_words, float* means, void* scratch, size_t scratch_bytes,
                          void* stream);
/* out[r][k] = +-means[r][interval of value k], row stride ld_out >= n. */
mv_status mv_quant_decode(const uint32_t* streams, int64_t ld_words, int64_t n, int32_t rows, int32_t q,
                          const float* means, float* out, int64_t ld_out, void* stream);

/*
 * Measurement aid, not part of the method: enqueues a plain streaming copy of
 * `bytes` (a multiple of 16; dst and src 16-byte aligned DEVICE pointers, not
 * overlapping) on `stream` of the current device.  Its achieved bandwidth is
 * the yardstick for the streaming pass, and its known byte count calibrates the
 * profiler's memory counters.
 */
mv_status mv_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MV_H */
