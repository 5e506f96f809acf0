/*
 * mv_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct CPU statement of what one iteration of
 * sparse SGD with majority voting computes between "the worker has its model
 * difference" and "the error buffer is updated" (Algorithm 1 of the paper,
 * the steps from error compensation to the aggregate).  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call this file.  It shares
 * no code, header, table or helper with the HIP library.
 *
 * Precision: the paper fixes 32-bit floating point for every value (Sec. 1.2.1
 * and Sec. 2.1, q = 32), so the arithmetic that decides a mask
 * is done in fp32 here, with round-to-nearest-even, denormals kept, and no
 * fused multiply-add (build with -ffp-contract=off, never -ffast-math).
 *
 * Every selection is the definition written out: build all (value, index)
 * pairs, sort ALL of them with the C library's qsort under the stated total
 * order, keep the first K.  No histograms, no partial selection, no blocking.
 *
 * Readings of the paper where it is silent (each one is also listed in the
 * design notes of the repository):
 *   - S_top ties (Sec. 2, definition of S_top; Sec. 2, vote description):
 *     larger value first, then LOWEST INDEX first; used for the per-worker
 *     selection and for the selection over vote counts.  The paper does not
 *     fix a tie rule: the tie-break is "parity unpinned" by the paper and
 *     pinned only by this build's contract.
 *   - the order by magnitude (Sec. 2, S_top) is the order of the fp32 bit pattern with the
 *     sign bit cleared: -0 == +0, denormals are ordered (not flushed), +Inf is
 *     above every finite value, NaNs above Inf by payload.
 *   - The aggregate is a mean (Sec. 2, definition of G-tilde and the linearity
 *     equation) although Algorithm 1's last step prints a plain sum; the sum is
 *     available through `reduce_mean = 0`.  The sum runs over workers in order
 *     n = 0..N-1 in fp32 and is then multiplied once by fp32 (1/N).
 *   - The error update uses the GLOBAL mask (Algorithm 1, "e = Delta-bar minus
 *     Delta-tilde_n"): the residual is exactly zero (+0.0) on the mask and the
 *     compensated value elsewhere.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* helpers                                                             */
/* ------------------------------------------------------------------ */

static uint32_t f32_bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    return u;
}

/* magnitude key: the fp32 bit pattern with the sign bit cleared */
static uint32_t magnitude_key(float x) { return f32_bits(x) & 0x7FFFFFFFu; }

typedef struct {
    uint32_t value; /* magnitude key, or vote count */
    uint32_t index; /* coordinate j */
} mvo_pair;

/* total order of S_top with this build's tie rule:
 * larger value first; among equal values the lower index first */
static int cmp_value_desc_index_asc(const void* pa, const void* pb)
{
    const mvo_pair* a = (const mvo_pair*)pa;
    const mvo_pair* b = (const mvo_pair*)pb;
    if (a->value != b->value) return (a->value > b->value) ? -1 : 1;
    if (a->index != b->index) return (a->index < b->index) ? -1 : 1;
    return 0;
}

static int cmp_u32_asc(const void* pa, const void* pb)
{
    uint32_t a = *(const uint32_t*)pa, b = *(const uint32_t*)pb;
    return (a > b) - (a < b);
}

/* S_top over an array of non-negative integer "values" of length d:
 * the K coordinates that come first under (value desc, index asc),
 * written in ascending index order.  Returns 0, or -1 on bad arguments
 * or allocation failure. */
static int s_top_indices(const uint32_t* values, int64_t d, int64_t K, uint32_t* idx_out)
{
    if (d <= 0 || K < 0 || K > d) return -1;
    mvo_pair* pairs = (mvo_pair*)malloc((size_t)d * sizeof(mvo_pair));
    if (!pairs) return -1;
    for (int64_t j = 0; j < d; ++j) {
        pairs[j].value = values[j];
        pairs[j].index = (uint32_t)j;
    }
    qsort(pairs, (size_t)d, sizeof(mvo_pair), cmp_value_desc_index_asc);
    for (int64_t k = 0; k < K; ++k) idx_out[k] = pairs[k].index;
    qsort(idx_out, (size_t)K, sizeof(uint32_t), cmp_u32_asc);
    free(pairs);
    return 0;
}

/* ------------------------------------------------------------------ */
/* the steps of Algorithm 1, one function each                          */
/* ------------------------------------------------------------------ */

/* bf16 -> fp32 is exact: the 16 bits are the upper half of the fp32 pattern.
 * (bf16 gradients are an extension of this build's workloads; the paper uses
 * fp32 throughout.) */
void mvo_widen_bf16(const uint16_t* g_bf16, float* g_f32, int64_t d)
{
    for (int64_t j = 0; j < d; ++j) {
        uint32_t u = ((uint32_t)g_bf16[j]) << 16;
        memcpy(&g_f32[j], &u, sizeof u);
    }
}

/* Algorithm 1, error compensation: Delta-bar = Delta + e, one fp32 add. */
void mvo_error_compensate(const float* delta, const float* e, float* delta_bar, int64_t d)
{
    for (int64_t j = 0; j < d; ++j) delta_bar[j] = delta[j] + e[j];
}

/* Algorithm 1, local mask: supp(S_top(|Delta-bar|, K)) for one worker. */
int mvo_row_topk(const float* delta_bar, int64_t d, int64_t K, uint32_t* idx_out)
{
    if (d <= 0) return -1;
    uint32_t* keys = (uint32_t*)malloc((size_t)d * sizeof(uint32_t));
    if (!keys) return -1;
    for (int64_t j = 0; j < d; ++j) keys[j] = magnitude_key(delta_bar[j]);
    int rc = s_top_indices(keys, d, K, idx_out);
    free(keys);
    return rc;
}

/* Sec. 2, the server tallies the supports it receives:
 * votes = sum over workers of the 0/1 local masks. */
int mvo_votes(const uint32_t* worker_idx, int32_t N, int64_t K, int64_t d, uint8_t* votes)
{
    if (N < 1 || N > 255) return -1;
    memset(votes, 0, (size_t)d);
    for (int32_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            uint32_t j = worker_idx[(int64_t)n * K + k];
            if ((int64_t)j >= d) return -1;
            votes[j] += 1;
        }
    return 0;
}

/* Sec. 2, mask equation, outer S_top: the K most voted coordinates. */
int mvo_mask(const uint8_t* votes, int64_t d, int64_t K, uint32_t* mask_idx)
{
    if (d <= 0) return -1;
    uint32_t* v = (uint32_t*)malloc((size_t)d * sizeof(uint32_t));
    if (!v) return -1;
    for (int64_t j = 0; j < d; ++j) v[j] = votes[j];
    int rc = s_top_indices(v, d, K, mask_idx);
    free(v);
    return rc;
}

/* Algorithm 1, "Delta-tilde_n = M (x) Delta-bar_n" then the aggregate over
 * workers; the 1/N is the mean of Sec. 2's G-tilde.  delta_bar is N rows of
 * stride ld. */
void mvo_aggregate(const float* delta_bar, int64_t ld, int32_t N,
                   const uint32_t* mask_idx, int64_t K, int32_t reduce_mean, float* agg)
{
    const float inv_N = 1.0f / (float)N;
    for (int64_t k = 0; k < K; ++k) {
        const uint32_t j = mask_idx[k];
        float s = delta_bar[j]; /* worker 0 */
        for (int32_t n = 1; n < N; ++n) s = s + delta_bar[(int64_t)n * ld + j];
        agg[k] = reduce_mean ? s * inv_N : s;
    }
}

/* Algorithm 1, error update for one worker: e_new = Delta-bar - Delta-tilde_n,
 * which is +0.0 on the mask and Delta-bar elsewhere. */
void mvo_error_update(const float* delta_bar, int64_t d,
                      const uint32_t* mask_idx, int64_t K, float* e_new)
{
    for (int64_t j = 0; j < d; ++j) e_new[j] = delta_bar[j];
    for (int64_t k = 0; k < K; ++k) e_new[mask_idx[k]] = 0.0f;
}

/* ------------------------------------------------------------------ */
/* one whole vote step                                                 */
/* ------------------------------------------------------------------ */

/*
 * grads      : N rows, stride ld_g elements; fp32 (grad_is_bf16 = 0) or bf16
 * err        : N rows, stride ld_e, fp32; in: e_t, out: e_{t+1}
 * worker_idx : N x K out, each row ascending
 * votes      : d out
 * mask_idx   : K out, ascending
 * agg        : K out
 * threads    : >1 runs the row-local steps (compensation, local top-K) with
 *              one OpenMP task per worker row; the arithmetic is unchanged.
 * Returns 0 on success, -1 on bad arguments / allocation failure.
 */
int mvo_rs_mask_keys(const uint8_t* votes, int64_t d, int64_t K, const float* rand_exp, uint32_t* mask_idx);

/* rand_exp == NULL: the mask is the K most voted coordinates (Algorithm 1, the
 * line with S_top); else the randomly selected one (the line with
 * S_rand-weighted), see mvo_rs_mask_keys. */
static int vote_step_impl(const void* grads, int64_t ld_g, int32_t grad_is_bf16,
                          float* err, int64_t ld_e,
                          int32_t N, int64_t d, int64_t K, int32_t reduce_mean, const float* rand_exp,
                          uint32_t* worker_idx, uint8_t* votes, uint32_t* mask_idx, float* agg,
                          int32_t threads)
{
    if (N < 1 || N > 255 || d < 1 || d > 0x7FFFFFFF || K < 1 || K > d) return -1;
    if (ld_g < d || ld_e < d) return -1;
    if (threads < 1) threads = 1;

    float* delta_bar = (float*)malloc((size_t)N * (size_t)d * sizeof(float));
    if (!delta_bar) return -1;
    int failed = 0;

#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
#endif
    for (int32_t n = 0; n < N; ++n) {
        float* row = delta_bar + (int64_t)n * d;
        if (grad_is_bf16) {
            float* wide = (float*)malloc((size_t)d * sizeof(float));
            if (!wide) {
                failed = 1;
                continue;
            }
            mvo_widen_bf16((const uint16_t*)grads + (int64_t)n * ld_g, wide, d);
            mvo_error_compensate(wide, err + (int64_t)n * ld_e, row, d);
            free(wide);
        } else {
            mvo_error_compensate((const float*)grads + (int64_t)n * ld_g,
                                 err + (int64_t)n * ld_e, row, d);
        }
        if (mvo_row_topk(row, d, K, worker_idx + (int64_t)n * K) != 0) failed = 1;
    }
    if (failed) {
        free(delta_bar);
        return -1;
    }

    int mask_rc = mvo_votes(worker_idx, N, K, d, votes);
    if (mask_rc == 0)
        mask_rc = rand_exp ? mvo_rs_mask_keys(votes, d, K, rand_exp, mask_idx) : mvo_mask(votes, d, K, mask_idx);
    if (mask_rc != 0) {
        free(delta_bar);
        return -1;
    }
    mvo_aggregate(delta_bar, d, N, mask_idx, K, reduce_mean, agg);

#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
#endif
    for (int32_t n = 0; n < N; ++n)
        mvo_error_update(delta_bar + (int64_t)n * d, d, mask_idx, K, err + (int64_t)n * ld_e);

    free(delta_bar);
    return 0;
}

int mvo_vote_step(const void* grads, int64_t ld_g, int32_t grad_is_bf16,
                  float* err, int64_t ld_e,
                  int32_t N, int64_t d, int64_t K, int32_t reduce_mean,
                  uint32_t* worker_idx, uint8_t* votes, uint32_t* mask_idx, float* agg,
                  int32_t threads)
{
    return vote_step_impl(grads, ld_g, grad_is_bf16, err, ld_e, N, d, K, reduce_mean, NULL,
                          worker_idx, votes, mask_idx, agg, threads);
}

/* ------------------------------------------------------------------ */
/* majority voting with random selection (Algorithm 1, S_rand-weighted) */
/* ------------------------------------------------------------------ */

/*
 * Sec. 2 (the paragraph after Algorithm 1): winners are drawn at random, a
 * position's chance growing in proportion to its votes; Sec. 4.2: the drawing
 * goes on until K distinct positions are selected.
 *
 * Reading (the paper names no sampler and no random generator): positions are
 * drawn one at a time, each draw independent with P(j) = votes[j] / sum(votes),
 * a position drawn before is drawn again in vain, and the procedure stops at K
 * distinct positions.  mvo_rs_mask_draws is that procedure, fed with uniform
 * numbers from the caller.  Discarding repeats means each NEW position is drawn
 * in proportion to its votes among the positions not yet selected (successive
 * sampling without replacement).
 *
 * mvo_rs_mask_keys states the same distribution in a form that does not depend
 * on the order of the draws: give every voted position j an independent
 * exponential clock of rate votes[j], i.e. the time rand_exp[j] / votes[j] with
 * rand_exp[j] ~ Exp(1) supplied by the caller, and select the K positions
 * whose clocks ring first.  The first clock to ring is j with probability
 * votes[j] / sum(votes), and the clocks are memoryless, so the order of ringing
 * is a successive sample -- the two functions agree in distribution, not draw
 * by draw.  The key is one fp32 division; ties (equal times) go to the lowest
 * position; positions without a vote are never selected.  "Parity unpinned" by
 * the paper beyond the proportionality of the probabilities to the votes.
 */

/* The sequential procedure.  u: n_u numbers in [0, 1).  Writes the K selected
 * positions ascending; returns the number of draws used, or -1 (bad arguments,
 * fewer than K voted positions, or u exhausted). */
int64_t mvo_rs_mask_draws(const uint8_t* votes, int64_t d, int64_t K, const double* u, int64_t n_u,
                          uint32_t* mask_idx)
{
    if (d < 1 || K < 1 || K > d) return -1;
    int64_t* cum = (int64_t*)malloc((size_t)d * sizeof(int64_t));
    uint8_t* chosen = (uint8_t*)calloc((size_t)d, 1);
    if (!cum || !chosen) {
        free(cum);
        free(chosen);
        return -1;
    }
    int64_t total = 0, voted = 0;
    for (int64_t j = 0; j < d; ++j) {
        total += votes[j];
        voted += votes[j] != 0;
        cum[j] = total; /* votes of positions 0..j */
    }
    int64_t used = -1;
    if (voted >= K) {
        int64_t n_chosen = 0, t = 0;
        while (n_chosen < K && t < n_u) {
            int64_t x = (int64_t)(u[t] * (double)total); /* the x-th vote, 0 <= x < total */
            if (x >= total) x = total - 1;
            ++t;
            int64_t lo = 0, hi = d - 1; /* first j with cum[j] > x: the position that holds vote x */
            while (lo < hi) {
                const int64_t mid = lo + (hi - lo) / 2;
                if (cum[mid] > x) hi = mid;
                else lo = mid + 1;
            }
            if (!chosen[lo]) {
                chosen[lo] = 1;
                ++n_chosen;
            }
        }
        if (n_chosen == K) {
            used = t;
            int64_t k = 0;
            for (int64_t j = 0; j < d; ++j)
                if (chosen[j]) mask_idx[k++] = (uint32_t)j;
        }
    }
    free(cum);
    free(chosen);
    return used;
}

typedef struct {
    float    time;
    uint32_t index;
} rs_clock;

static int cmp_time_asc_index_asc(const void* pa, const void* pb)
{
    const rs_clock* a = (const rs_clock*)pa;
    const rs_clock* b = (const rs_clock*)pb;
    if (a->time != b->time) return a->time < b->time ? -1 : 1;
    return a->index < b->index ? -1 : (a->index > b->index ? 1 : 0);
}

/* The exponential-clock form.  rand_exp: d non-negative finite fp32 numbers
 * (only those of voted positions are read).  Returns 0, or -1 (bad arguments or
 * fewer than K voted positions). */
int mvo_rs_mask_keys(const uint8_t* votes, int64_t d, int64_t K, const float* rand_exp, uint32_t* mask_idx)
{
    if (d < 1 || K < 1 || K > d) return -1;
    int64_t voted = 0;
    for (int64_t j = 0; j < d; ++j) voted += votes[j] != 0;
    if (voted < K) return -1;
    rs_clock* c = (rs_clock*)malloc((size_t)voted * sizeof(rs_clock));
    uint32_t* sel = (uint32_t*)malloc((size_t)K * sizeof(uint32_t));
    if (!c || !sel) {
        free(c);
        free(sel);
        return -1;
    }
    int64_t n = 0;
    for (int64_t j = 0; j < d; ++j)
        if (votes[j]) {
            c[n].time = rand_exp[j] / (float)votes[j];
            c[n].index = (uint32_t)j;
            ++n;
        }
    qsort(c, (size_t)voted, sizeof(rs_clock), cmp_time_asc_index_asc);
    for (int64_t k = 0; k < K; ++k) sel[k] = c[k].index;
    qsort(sel, (size_t)K, sizeof(uint32_t), cmp_u32_asc);
    memcpy(mask_idx, sel, (size_t)K * sizeof(uint32_t));
    free(c);
    free(sel);
    return 0;
}

/* Algorithm 1 with the S_rand-weighted line: as mvo_vote_step, the mask being
 * mvo_rs_mask_keys of the step's votes.  rand_exp: d fp32 numbers. */
int mvo_rs_vote_step(const void* grads, int64_t ld_g, int32_t grad_is_bf16,
                     float* err, int64_t ld_e,
                     int32_t N, int64_t d, int64_t K, int32_t reduce_mean, const float* rand_exp,
                     uint32_t* worker_idx, uint8_t* votes, uint32_t* mask_idx, float* agg,
                     int32_t threads)
{
    if (!rand_exp) return -1;
    return vote_step_impl(grads, ld_g, grad_is_bf16, err, ld_e, N, d, K, reduce_mean, rand_exp,
                          worker_idx, votes, mask_idx, agg, threads);
}

/* ------------------------------------------------------------------ */
/* majority voting with add-drop (Algorithm 2)                          */
/* ------------------------------------------------------------------ */

/*
 * Readings of Algorithm 2 and Sec. 3 where they are silent or garbled:
 *   - The add set is taken among A = supp(M_n) \ supp(M~_{n,t-1}), the drop set
 *     among D = supp(M~_{n,t-1}) \ supp(M_n) (Sec. 3, second paragraph).  The
 *     printed formulas apply S_top / S_bot to a vector that is zero outside A
 *     (resp. D); read literally they would pick coordinates outside the set
 *     when the set has fewer than K_ad members.  Sec. 3 bounds the additions
 *     and the removals by K_ad each, so: add = the min(K_ad, |A|) members of A
 *     with the largest |Delta-bar|, drop = the min(K_ad, |D|) members of D with
 *     the smallest |Delta-bar|.
 *   - Ties: add under (magnitude desc, index asc); drop under (magnitude asc,
 *     index asc).  Unpinned by the paper, as for S_top.
 *   - M~_{n,0} and M^sum_0 are not given: the state starts empty (all zero) and
 *     is carried by the caller; a first step with K_ad = K then makes
 *     M~_{n,1} = M_n and M^sum_1 the plain vote count of Algorithm 1.
 *   - The magnitudes that rank the drop candidates are those of the CURRENT
 *     Delta-bar (the formula multiplies by Delta-bar_{n,t}).
 *   - The mask is S_top(M^sum_t, K) with the tie rule of Algorithm 1's mask.
 */

/* S_top restricted to a set: among the coordinates j with member[j] != 0, the
 * first `take` under (key desc, index asc) if largest != 0, else under
 * (key asc, index asc); written ascending.  Returns how many were taken
 * (min(take, set size)), or -1. */
static int64_t pick_in_set(const uint32_t* keys, const uint8_t* member, int64_t d, int64_t take,
                           int largest, uint32_t* idx_out)
{
    int64_t n = 0;
    for (int64_t j = 0; j < d; ++j) n += member[j] ? 1 : 0;
    mvo_pair* pairs = (mvo_pair*)malloc((size_t)(n > 0 ? n : 1) * sizeof(mvo_pair));
    if (!pairs) return -1;
    int64_t m = 0;
    for (int64_t j = 0; j < d; ++j)
        if (member[j]) {
            /* ascending order of keys = descending order of the complemented keys */
            pairs[m].value = largest ? keys[j] : (0x7FFFFFFFu - keys[j]);
            pairs[m].index = (uint32_t)j;
            ++m;
        }
    qsort(pairs, (size_t)n, sizeof(mvo_pair), cmp_value_desc_index_asc);
    const int64_t got = take < n ? take : n;
    for (int64_t k = 0; k < got; ++k) idx_out[k] = pairs[k].index;
    qsort(idx_out, (size_t)got, sizeof(uint32_t), cmp_u32_asc);
    free(pairs);
    return got;
}

/*
 * One iteration of Algorithm 2 for all workers.
 *   vote      : N x d bytes (0/1), in: M~_{n,t-1}, out: M~_{n,t}
 *   msum      : d bytes, in: M^sum_{t-1}, out: M^sum_t
 *   worker_idx: N x K out, supp(M_{n,t}) ascending (the plain top-K, not transmitted)
 *   add_idx, drop_idx : N x K_ad out, ascending, the first n_add[n] / n_drop[n] entries valid
 *   mask_idx, agg, err: as in mvo_vote_step
 * Returns 0, or -1 on bad arguments / allocation failure / inconsistent state.
 */
int mvo_ad_vote_step(const void* grads, int64_t ld_g, int32_t grad_is_bf16,
                     float* err, int64_t ld_e,
                     int32_t N, int64_t d, int64_t K, int64_t K_ad, int32_t reduce_mean,
                     uint8_t* vote, uint8_t* msum,
                     uint32_t* worker_idx, uint32_t* add_idx, uint32_t* drop_idx,
                     int64_t* n_add, int64_t* n_drop,
                     uint32_t* mask_idx, float* agg, int32_t threads)
{
    if (N < 1 || N > 255 || d < 1 || d > 0x7FFFFFFF || K < 1 || K > d || K_ad < 1 || K_ad > K) return -1;
    if (ld_g < d || ld_e < d) return -1;
    if (threads < 1) threads = 1;
    float* delta_bar = (float*)malloc((size_t)N * (size_t)d * sizeof(float));
    if (!delta_bar) return -1;
    int failed = 0;

    /* worker side (Algorithm 2, voting phase): each worker's add and drop lists
     * depend only on its own row and its own previous vote */
#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
#endif
    for (int32_t n = 0; n < N; ++n) {
        float* row = delta_bar + (int64_t)n * d;
        const uint8_t* vt = vote + (int64_t)n * d;
        uint32_t* keys = (uint32_t*)malloc((size_t)d * sizeof(uint32_t));
        uint8_t*  cur = (uint8_t*)calloc((size_t)d, 1);     /* M_{n,t} */
        uint8_t*  setA = (uint8_t*)malloc((size_t)d);
        uint8_t*  setD = (uint8_t*)malloc((size_t)d);
        float*    wide = grad_is_bf16 ? (float*)malloc((size_t)d * sizeof(float)) : NULL;
        if (!keys || !cur || !setA || !setD || (grad_is_bf16 && !wide)) {
            failed = 1;
        } else {
            if (grad_is_bf16) {
                mvo_widen_bf16((const uint16_t*)grads + (int64_t)n * ld_g, wide, d);
                mvo_error_compensate(wide, err + (int64_t)n * ld_e, row, d);
            } else {
                mvo_error_compensate((const float*)grads + (int64_t)n * ld_g, err + (int64_t)n * ld_e, row, d);
            }
            uint32_t* widx = worker_idx + (int64_t)n * K;
            if (mvo_row_topk(row, d, K, widx) != 0) {
                failed = 1;
            } else {
                for (int64_t k = 0; k < K; ++k) cur[widx[k]] = 1;
                for (int64_t j = 0; j < d; ++j) {
                    keys[j] = magnitude_key(row[j]);
                    setA[j] = (uint8_t)(cur[j] && !vt[j]);    /* max(M_n - M~, 0) */
                    setD[j] = (uint8_t)(vt[j] && !cur[j]);    /* max(M~ - M_n, 0) */
                }
                n_add[n] = pick_in_set(keys, setA, d, K_ad, 1, add_idx + (int64_t)n * K_ad);
                n_drop[n] = pick_in_set(keys, setD, d, K_ad, 0, drop_idx + (int64_t)n * K_ad);
                if (n_add[n] < 0 || n_drop[n] < 0) failed = 1;
            }
        }
        free(keys); free(cur); free(setA); free(setD); free(wide);
    }
    if (failed) {
        free(delta_bar);
        return -1;
    }

    /* M~_n = M~_n + M^add_n - M^drop_n ;  PS side: M^sum += sum_n (M^add_n - M^drop_n) */
    for (int32_t n = 0; n < N; ++n) {
        uint8_t* vt = vote + (int64_t)n * d;
        for (int64_t k = 0; k < n_add[n]; ++k) {
            const uint32_t j = add_idx[(int64_t)n * K_ad + k];
            vt[j] = 1;
            if (msum[j] == 255) failed = 1;
            msum[j] += 1;
        }
    }
    for (int32_t n = 0; n < N; ++n) {
        uint8_t* vt = vote + (int64_t)n * d;
        for (int64_t k = 0; k < n_drop[n]; ++k) {
            const uint32_t j = drop_idx[(int64_t)n * K_ad + k];
            vt[j] = 0;
            if (msum[j] == 0) failed = 1;            /* the state was not a sum of votes */
            msum[j] -= 1;
        }
    }
    if (failed || mvo_mask(msum, d, K, mask_idx) != 0) {
        free(delta_bar);
        return -1;
    }
    mvo_aggregate(delta_bar, d, N, mask_idx, K, reduce_mean, agg);
#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
#endif
    for (int32_t n = 0; n < N; ++n)
        mvo_error_update(delta_bar + (int64_t)n * d, d, mask_idx, K, err + (int64_t)n * ld_e);
    free(delta_bar);
    return 0;
}

/* ------------------------------------------------------------------ */
/* sparse position code (Sec. 4.3.1)                                    */
/* ------------------------------------------------------------------ */

/*
 * The vector's d coordinates are cut into blocks of block_len = 1/phi
 * coordinates.  The stream lists, block after block, every non-zero position
 * of the block as a 1 bit followed by the position inside the block in
 * B = ceil(log2(block_len)) bits, and closes the block with a 0 bit.
 *
 * Readings where Sec. 4.3.1 is silent: the in-block position is written most
 * significant bit first; every block, also an empty one and the last (possibly
 * shorter) one, gets its closing 0, so the stream has exactly
 * n * (1 + B) + ceil(d / block_len) bits -- with n = phi * d positions that is
 * log(1/phi) + 2 bits per position, the figure of Sec. 2.1; bit k of the stream
 * is bit (k % 32) of 32-bit word k / 32; unused bits of the last word are 0.
 */
int32_t mvo_codec_offset_bits(int64_t block_len)
{
    int32_t b = 0;
    while (((int64_t)1 << b) < block_len) ++b;
    return b;
}

static void put_bit(uint32_t* words, uint64_t k, uint32_t bit)
{
    if (bit) words[k >> 5] |= (uint32_t)1 << (k & 31);
}

static uint32_t get_bit(const uint32_t* words, uint64_t k) { return (words[k >> 5] >> (k & 31)) & 1u; }

/* Encoder: writes the stream of the ascending positions idx[0..n) and returns its
 * length in bits, or -1 on bad arguments (positions not ascending or >= d, or
 * `words` too short: max_words 32-bit words are available and are zeroed first). */
int64_t mvo_codec_encode(const uint32_t* idx, int64_t n, int64_t d, int64_t block_len,
                         uint32_t* words, int64_t max_words)
{
    if (d < 1 || block_len < 1 || n < 0 || n > d) return -1;
    const int32_t B = mvo_codec_offset_bits(block_len);
    const int64_t n_blocks = (d + block_len - 1) / block_len;
    const uint64_t total = (uint64_t)n * (uint64_t)(1 + B) + (uint64_t)n_blocks;
    if ((int64_t)((total + 31) / 32) > max_words) return -1;
    memset(words, 0, (size_t)max_words * sizeof(uint32_t));
    uint64_t k = 0;
    int64_t i = 0;
    for (int64_t b = 0; b < n_blocks; ++b) {
        const int64_t lo = b * block_len, hi = lo + block_len;
        while (i < n && (int64_t)idx[i] < hi) {
            if ((int64_t)idx[i] < lo || (int64_t)idx[i] >= d) return -1;     /* not ascending / out of range */
            if (i > 0 && idx[i] <= idx[i - 1]) return -1;
            const uint32_t off = (uint32_t)((int64_t)idx[i] - lo);
            put_bit(words, k++, 1);                                           /* a position follows */
            for (int32_t q = B - 1; q >= 0; --q) put_bit(words, k++, (off >> q) & 1u);
            ++i;
        }
        put_bit(words, k++, 0);                                               /* end of block */
    }
    if (i != n || k != total) return -1;
    return (int64_t)total;
}

/* Decoder (the receiving side of the code of Sec. 4.3.1).  It keeps a cursor into
 * the stream and the number of the block it is in, starting at block 0.  A set
 * bit under the cursor announces a position: the B bits behind it are that
 * position's offset inside the current block, so the coordinate is
 * block * block_len + offset.  A clear bit ends the current block and the next
 * one begins.  Decoding stops when the cursor has passed n_bits.  Returns the
 * number of positions written to idx_out, or -1 (more than max_n positions, a
 * position outside its block or the vector, or an offset cut short by the end
 * of the stream). */
int64_t mvo_codec_decode(const uint32_t* words, int64_t n_bits, int64_t d, int64_t block_len,
                         uint32_t* idx_out, int64_t max_n)
{
    if (d < 1 || block_len < 1 || n_bits < 0) return -1;
    const int32_t B = mvo_codec_offset_bits(block_len);
    int64_t block = 0, n = 0;
    uint64_t k = 0;
    while (k < (uint64_t)n_bits) {
        if (get_bit(words, k++)) {
            if (k + (uint64_t)B > (uint64_t)n_bits) return -1;
            uint32_t off = 0;
            for (int32_t q = 0; q < B; ++q) off = (off << 1) | get_bit(words, k++);
            const int64_t pos = block * block_len + (int64_t)off;
            if ((int64_t)off >= block_len || pos >= d || n >= max_n) return -1;
            idx_out[n++] = (uint32_t)pos;
        } else {
            ++block;
        }
    }
    return n;
}

/* ------------------------------------------------------------------ */
/* fractional quantisation (Sec. 4.3.2)                                 */
/* ------------------------------------------------------------------ */

/*
 * q bits per value: q-1 bits name one of L = 2^(q-1) geometric intervals of
 * |v| between v_max and v_min, I_l = [v_max / alpha^(l-1), v_max / alpha^l] with
 * alpha = (v_max / v_min)^(1/L), one bit is the sign; the L means mu_l of the
 * magnitudes that fall into I_l follow the codes, and the receiver reproduces
 * sign * mu_l.
 *
 * Readings where Sec. 4.3.2 is silent or loose (the interval ends overlap as
 * printed, and nothing fixes the arithmetic of the edges):
 *   - v_min is the smallest NON-ZERO magnitude (a zero would make alpha
 *     infinite); zeros go to the last interval.  If all values are zero every
 *     mean is zero.
 *   - Edges in fp64: ratio = v_max / v_min; alpha = ratio under q-1 successive
 *     square roots (L is a power of two, so this is the L-th root, and every step
 *     is a correctly rounded IEEE operation on any machine); edge_0 = v_max,
 *     edge_l = edge_{l-1} / alpha for l = 1..L-1.
 *   - |v| belongs to interval l = 1 + #{ j in 1..L-1 : |v| <= edge_j }: a value on
 *     an edge goes to the interval of the smaller magnitudes.
 *   - code = (l - 1) | (sign << (q-1)), sign = 1 for negative values (and -0);
 *     value k occupies bits [k q, (k+1) q) of the stream, bit b of the stream
 *     being bit b % 32 of word b / 32.
 *   - mu_l = (sum of the magnitudes in I_l, accumulated in fp64 in index order)
 *     / count, rounded to fp32; 0 for an empty interval.
 */
int32_t mvo_quant_edges(const float* v, int64_t n, int32_t q, double* edges /* L entries: edge_0..edge_{L-1} */)
{
    if (n < 1 || q < 2 || q > 9) return -1;
    const int32_t L = 1 << (q - 1);
    double vmax = 0.0, vmin = 0.0;
    for (int64_t k = 0; k < n; ++k) {
        const double m = fabs((double)v[k]);
        if (m > vmax) vmax = m;
        if (m > 0.0 && (vmin == 0.0 || m < vmin)) vmin = m;
    }
    if (vmax == 0.0) {
        for (int32_t l = 0; l < L; ++l) edges[l] = 0.0;
        return 0;
    }
    double alpha = vmax / vmin;
    for (int32_t r = 0; r < q - 1; ++r) alpha = sqrt(alpha);
    edges[0] = vmax;
    for (int32_t l = 1; l < L; ++l) edges[l] = edges[l - 1] / alpha;
    return 0;
}

/* codes: one uint8 per value ((l-1) | sign << (q-1)); means: L floats. */
int32_t mvo_quant_encode(const float* v, int64_t n, int32_t q, uint8_t* codes, float* means)
{
    if (n < 1 || q < 2 || q > 8) return -1;
    const int32_t L = 1 << (q - 1);
    double edges[256];
    if (mvo_quant_edges(v, n, q, edges) != 0) return -1;
    double sum[256];
    int64_t cnt[256];
    for (int32_t l = 0; l < L; ++l) {
        sum[l] = 0.0;
        cnt[l] = 0;
    }
    for (int64_t k = 0; k < n; ++k) {
        const double m = fabs((double)v[k]);
        int32_t l = 0;                                   /* l - 1 */
        for (int32_t j = 1; j < L; ++j) l += (m <= edges[j]) ? 1 : 0;
        const uint32_t sign = (f32_bits(v[k]) >> 31) & 1u;
        codes[k] = (uint8_t)((uint32_t)l | (sign << (q - 1)));
        sum[l] += m;
        cnt[l] += 1;
    }
    for (int32_t l = 0; l < L; ++l) means[l] = cnt[l] ? (float)(sum[l] / (double)cnt[l]) : 0.0f;
    return 0;
}

void mvo_quant_decode(const uint8_t* codes, int64_t n, int32_t q, const float* means, float* out)
{
    const uint32_t lmask = ((uint32_t)1 << (q - 1)) - 1;
    for (int64_t k = 0; k < n; ++k) {
        const float m = means[codes[k] & lmask];
        out[k] = ((codes[k] >> (q - 1)) & 1u) ? -m : m;
    }
}

/* packs / unpacks q-bit codes into the stream layout stated above */
void mvo_quant_pack(const uint8_t* codes, int64_t n, int32_t q, uint32_t* words /* ceil(n q / 32), zeroed here */)
{
    memset(words, 0, (size_t)(((uint64_t)n * (uint64_t)q + 31) / 32) * sizeof(uint32_t));
    for (int64_t k = 0; k < n; ++k)
        for (int32_t b = 0; b < q; ++b)
            put_bit(words, (uint64_t)k * (uint64_t)q + (uint64_t)b, (codes[k] >> b) & 1u);
}

/* ------------------------------------------------------------------ */
/* communication-load arithmetic (Sec. 2.1 and Sec. 4.4), reporting only */
/* ------------------------------------------------------------------ */

/* bits per transmitted position: log2(1/phi) rounded up to whole bits, plus
 * the one-bit "position follows" flag and the amortised end-of-block bit
 * (Sec. 2.1, Q_loc; Sec. 4.3.1).  phi is given as the block length 1/phi. */
int32_t mvo_bits_per_position(double inv_phi)
{
    int32_t b = 0;
    while (ldexp(1.0, b) < inv_phi) ++b; /* smallest b with 2^b >= 1/phi */
    return b + 2;
}

/* Q_val = q * phi * d  (Sec. 2.1) */
double mvo_q_val(double q_bits, double phi, double d) { return q_bits * phi * d; }

/* Q_loc = d * phi * (log(1/phi) + 2)  (Sec. 2.1) */
double mvo_q_loc(double phi, double d) { return d * phi * (double)mvo_bits_per_position(1.0 / phi); }

/* per-parameter budgets q-bar = Q / (d H) and the compression rate
 * 32 / (q-bar_loc + q-bar_val)  (Sec. 4.4, discussion of Table 1) */
double mvo_compression(double qbar_loc, double qbar_val) { return 32.0 / (qbar_loc + qbar_val); }

int32_t mvo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
