/* Drives every entry point of oracle/mv_oracle.c on small problems whose buffers are
 * allocated to the exact size, for a build under -fsanitize=address,undefined: an
 * access one element past any argument, a signed overflow or a misaligned access in
 * the oracle ends the program with a report.  Shapes: ragged sizes, K = d, N = 1,
 * heavy ties, bf16 gradients, the rejected-argument paths.  Prints "ok" at the end. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void mvo_widen_bf16(const uint16_t* g_bf16, float* g_f32, int64_t d);
int mvo_row_topk(const float* delta_bar, int64_t d, int64_t K, uint32_t* idx_out);
int mvo_votes(const uint32_t* worker_idx, int32_t N, int64_t K, int64_t d, uint8_t* votes);
int mvo_mask(const uint8_t* votes, int64_t d, int64_t K, uint32_t* mask_idx);
int mvo_vote_step(const void* grads, int64_t ld_g, int32_t grad_is_bf16, float* err, int64_t ld_e, int32_t N,
                  int64_t d, int64_t K, int32_t reduce_mean, uint32_t* worker_idx, uint8_t* votes,
                  uint32_t* mask_idx, float* agg, int32_t threads);
int mvo_rs_vote_step(const void* grads, int64_t ld_g, int32_t grad_is_bf16, float* err, int64_t ld_e, int32_t N,
                     int64_t d, int64_t K, int32_t reduce_mean, const float* rand_exp, uint32_t* worker_idx,
                     uint8_t* votes, uint32_t* mask_idx, float* agg, int32_t threads);
int64_t mvo_rs_mask_draws(const uint8_t* votes, int64_t d, int64_t K, const double* u, int64_t n_u,
                          uint32_t* mask_idx);
int mvo_ad_vote_step(const void* grads, int64_t ld_g, int32_t grad_is_bf16, float* err, int64_t ld_e, int32_t N,
                     int64_t d, int64_t K, int64_t K_ad, int32_t reduce_mean, uint8_t* vote, uint8_t* msum,
                     uint32_t* worker_idx, uint32_t* add_idx, uint32_t* drop_idx, int64_t* n_add, int64_t* n_drop,
                     uint32_t* mask_idx, float* agg, int32_t threads);
int32_t mvo_codec_offset_bits(int64_t block_len);
int64_t mvo_codec_encode(const uint32_t* idx, int64_t n, int64_t d, int64_t block_len, uint32_t* words,
                         int64_t max_words);
int64_t mvo_codec_decode(const uint32_t* words, int64_t n_bits, int64_t d, int64_t block_len, uint32_t* idx_out,
                         int64_t max_n);
int32_t mvo_quant_encode(const float* v, int64_t n, int32_t q, uint8_t* codes, float* means);
void mvo_quant_decode(const uint8_t* codes, int64_t n, int32_t q, const float* means, float* out);
void mvo_quant_pack(const uint8_t* codes, int64_t n, int32_t q, uint32_t* words);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
static float rnd_value(int lattice)
{
    if (lattice) return (float)((int)(rnd() % 9) - 4) * 0.25f;     /* few distinct magnitudes: heavy ties */
    return ((float)(rnd() % 200001) - 100000.0f) / 777.0f;
}
#define CHECK(c)                                                            \
    do {                                                                    \
        if (!(c)) {                                                         \
            fprintf(stderr, "driver check failed, line %d: %s\n", __LINE__, #c); \
            exit(3);                                                        \
        }                                                                   \
    } while (0)

static void plain_and_random_selection(int32_t N, int64_t d, int64_t K, int bf16, int lattice, int threads)
{
    const size_t gs = bf16 ? 2 : 4;
    void* g = malloc((size_t)N * d * gs);
    float* e = malloc((size_t)N * d * 4);
    float* e2 = malloc((size_t)N * d * 4);
    float* r = malloc((size_t)d * 4);
    uint32_t* widx = malloc((size_t)N * K * 4);
    uint8_t* votes = malloc((size_t)d);
    uint32_t* mask = malloc((size_t)K * 4);
    float* agg = malloc((size_t)K * 4);
    memset(e, 0, (size_t)N * d * 4);
    for (int step = 0; step < 2; ++step) {
        for (int64_t i = 0; i < (int64_t)N * d; ++i) {
            const float v = rnd_value(lattice);
            if (bf16) {
                uint32_t b;
                memcpy(&b, &v, 4);
                ((uint16_t*)g)[i] = (uint16_t)(b >> 16);
            } else {
                ((float*)g)[i] = v;
            }
        }
        for (int64_t j = 0; j < d; ++j) r[j] = (float)(rnd() % 100000 + 1) / 25000.0f;
        memcpy(e2, e, (size_t)N * d * 4);
        CHECK(mvo_vote_step(g, d, bf16, e, d, N, d, K, step, widx, votes, mask, agg, threads) == 0);
        int64_t total = 0;
        for (int64_t j = 0; j < d; ++j) total += votes[j];
        CHECK(total == (int64_t)N * K);
        for (int64_t k = 1; k < K; ++k) CHECK(mask[k] > mask[k - 1]);
        CHECK(mvo_rs_vote_step(g, d, bf16, e2, d, N, d, K, 1, r, widx, votes, mask, agg, threads) == 0);
        for (int64_t k = 0; k < K; ++k) CHECK(mask[k] < (uint64_t)d && votes[mask[k]] >= 1);
    }
    /* the sequential drawing procedure on the last votes */
    {
        const int64_t n_u = 64 * K + 64;
        double* u = malloc((size_t)n_u * 8);
        for (int64_t i = 0; i < n_u; ++i) u[i] = (double)(rnd() % 1000000) / 1000000.0;
        const int64_t used = mvo_rs_mask_draws(votes, d, K, u, n_u, mask);
        CHECK(used >= -1 && used <= n_u);
        free(u);
    }
    /* the steps one by one */
    CHECK(mvo_row_topk(e, d, K, widx) == 0);
    CHECK(mvo_votes(widx, 1, K, d, votes) == 0);
    CHECK(mvo_mask(votes, d, K, mask) == 0);
    /* rejected arguments */
    CHECK(mvo_vote_step(g, d - 1, bf16, e, d, N, d, K, 1, widx, votes, mask, agg, threads) != 0);
    CHECK(mvo_vote_step(g, d, bf16, e, d, N, d, d + 1, 1, widx, votes, mask, agg, threads) != 0);
    CHECK(mvo_vote_step(g, d, bf16, e, d, 0, d, K, 1, widx, votes, mask, agg, threads) != 0);
    free(g); free(e); free(e2); free(r); free(widx); free(votes); free(mask); free(agg);
}

static void add_drop(int32_t N, int64_t d, int64_t K, int64_t K_ad, int lattice, int threads)
{
    float* g = malloc((size_t)N * d * 4);
    float* e = malloc((size_t)N * d * 4);
    uint8_t* vote = malloc((size_t)N * d);
    uint8_t* msum = malloc((size_t)d);
    uint32_t* widx = malloc((size_t)N * K * 4);
    uint32_t* add_full = malloc((size_t)N * K * 4);
    uint32_t* drop_full = malloc((size_t)N * K * 4);
    uint32_t* add = malloc((size_t)N * K_ad * 4);
    uint32_t* drop = malloc((size_t)N * K_ad * 4);
    int64_t* n_add = malloc((size_t)N * 8);
    int64_t* n_drop = malloc((size_t)N * 8);
    uint32_t* mask = malloc((size_t)K * 4);
    float* agg = malloc((size_t)K * 4);
    memset(e, 0, (size_t)N * d * 4);
    memset(vote, 0, (size_t)N * d);
    memset(msum, 0, (size_t)d);
    for (int step = 0; step < 4; ++step) {
        for (int64_t i = 0; i < (int64_t)N * d; ++i) g[i] = rnd_value(lattice);
        const int full = step == 0;                      /* the first vote is a full one: K_ad = K */
        CHECK(mvo_ad_vote_step(g, d, 0, e, d, N, d, K, full ? K : K_ad, 1, vote, msum, widx, full ? add_full : add,
                               full ? drop_full : drop, n_add, n_drop, mask, agg, threads) == 0);
        for (int32_t n = 0; n < N; ++n) {
            CHECK(n_add[n] >= 0 && n_add[n] <= (full ? K : K_ad) && n_drop[n] >= 0 && n_drop[n] <= (full ? K : K_ad));
            int64_t standing = 0;
            for (int64_t j = 0; j < d; ++j) standing += vote[(int64_t)n * d + j];
            CHECK(standing == K);
        }
        for (int64_t j = 0; j < d; ++j) {
            int s = 0;
            for (int32_t n = 0; n < N; ++n) s += vote[(int64_t)n * d + j];
            CHECK(s == msum[j]);
        }
    }
    CHECK(mvo_ad_vote_step(g, d, 0, e, d, N, d, K, K + 1, 1, vote, msum, widx, add, drop, n_add, n_drop, mask, agg,
                           threads) != 0);
    free(g); free(e); free(vote); free(msum); free(widx); free(add_full); free(drop_full); free(add); free(drop);
    free(n_add); free(n_drop); free(mask); free(agg);
}

static void codec(int64_t d, int64_t block_len, int64_t n)
{
    uint32_t* idx = malloc((size_t)(n > 0 ? n : 1) * 4);
    /* n ascending positions: every (d / n)-th coordinate, jittered */
    for (int64_t i = 0; i < n; ++i) idx[i] = (uint32_t)(i * d / n + (int64_t)(rnd() % (uint32_t)(d / n)));
    const int32_t B = mvo_codec_offset_bits(block_len);
    const int64_t bits = n * (1 + B) + (d + block_len - 1) / block_len;
    const int64_t n_words = (bits + 31) / 32;
    uint32_t* words = malloc((size_t)n_words * 4);
    uint32_t* back = malloc((size_t)(n > 0 ? n : 1) * 4);
    CHECK(mvo_codec_encode(idx, n, d, block_len, words, n_words) == bits);
    CHECK(mvo_codec_decode(words, bits, d, block_len, back, n) == n);
    CHECK(memcmp(idx, back, (size_t)n * 4) == 0);
    if (n_words > 1) CHECK(mvo_codec_encode(idx, n, d, block_len, words, n_words - 1) == -1);   /* too short */
    if (n > 1) CHECK(mvo_codec_decode(words, bits, d, block_len, back, n - 1) == -1);           /* too many */
    /* truncated and damaged streams are refused or decoded, never read past their end */
    for (int64_t cut = bits - 1; cut >= 0 && cut > bits - 40; --cut)
        (void)mvo_codec_decode(words, cut, d, block_len, back, n);
    for (int64_t w = 0; w < n_words; ++w) words[w] = rnd();
    (void)mvo_codec_decode(words, bits, d, block_len, back, n);
    for (int64_t w = 0; w < n_words; ++w) words[w] = 0xFFFFFFFFu;
    (void)mvo_codec_decode(words, bits, d, block_len, back, n);
    free(idx); free(words); free(back);
}

static void quantiser(int64_t n, int32_t q, int zeros)
{
    float* v = malloc((size_t)n * 4);
    float* out = malloc((size_t)n * 4);
    uint8_t* codes = malloc((size_t)n);
    float* means = malloc(((size_t)1 << (q - 1)) * 4);
    uint32_t* words = malloc((size_t)(((uint64_t)n * q + 31) / 32) * 4);
    for (int64_t k = 0; k < n; ++k) v[k] = zeros == 2 ? 0.0f : (zeros && k % 3 == 0) ? -0.0f : rnd_value(0);
    CHECK(mvo_quant_encode(v, n, q, codes, means) == 0);
    mvo_quant_decode(codes, n, q, means, out);
    mvo_quant_pack(codes, n, q, words);
    for (int64_t k = 0; k < n; ++k) CHECK(fabsf(out[k]) <= 200.0f);
    CHECK(mvo_quant_encode(v, n, 1, codes, means) != 0);
    free(v); free(out); free(codes); free(means); free(words);
}

int main(void)
{
    static const struct { int32_t N; int64_t d, K; int bf16, lattice, threads; } cases[] = {
        {1, 1, 1, 0, 0, 1},     {3, 2, 1, 0, 1, 2},      {2, 5, 5, 0, 1, 1},      {4, 31, 7, 1, 0, 3},
        {3, 1023, 10, 0, 1, 2}, {2, 1024, 1024, 0, 0, 2}, {5, 4099, 41, 1, 1, 4}, {255, 257, 3, 0, 0, 4},
        {7, 20011, 200, 0, 0, 4},
    };
    for (size_t c = 0; c < sizeof(cases) / sizeof(cases[0]); ++c)
        plain_and_random_selection(cases[c].N, cases[c].d, cases[c].K, cases[c].bf16, cases[c].lattice,
                                   cases[c].threads);
    add_drop(1, 1, 1, 1, 0, 1);
    add_drop(2, 33, 5, 2, 1, 2);
    add_drop(3, 1025, 40, 4, 0, 2);
    add_drop(2, 4099, 4099, 100, 1, 2);
    add_drop(4, 7001, 700, 70, 0, 4);
    codec(1, 1, 1);
    codec(1000, 10, 100);
    codec(1000, 10, 0 + 1);
    codec(1003, 7, 59);
    codec(70001, 100, 700);
    codec(70001, 1000, 70);
    codec(4096, 4096, 4096 / 64);
    quantiser(1, 2, 0);
    quantiser(1000, 4, 0);
    quantiser(1000, 4, 1);
    quantiser(333, 8, 1);
    quantiser(64, 3, 2);
    puts("ok");
    return 0;
}
