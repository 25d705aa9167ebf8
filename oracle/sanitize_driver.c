/*
 * TEST INFRASTRUCTURE ONLY. Runs every exported function of the CPU oracle (qes_oracle.c) on
 * small, ragged shapes in a program built with -fsanitize=address,undefined, so that an
 * out-of-bounds access, a signed overflow or an invalid shift in the oracle aborts the run.
 * Prints one checksum line of everything the calls produced; the test that builds and runs this
 * program (tests/test_oracle_sanitized.py) also builds it with the oracle's ordinary flags and no
 * sanitizer and requires the same checksum: results that depended on undefined behaviour or on the
 * optimisation level would differ. Inputs come from a small LCG.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    void *qweight;
    const uint16_t *scales;
    int32_t out_features, in_features;
    int32_t bits;
    int32_t group_size;
    int32_t qmin, qmax;
    uint32_t tensor_id;
} oracle_tensor;

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
float oracle_ln_u1(uint32_t m);
void oracle_sincos_quarter(float f, float *s_out, float *c_out);
void oracle_noise_words(uint64_t seed, uint32_t tensor_id, uint64_t pair_begin, uint64_t n_pairs, uint32_t *out4);
void oracle_noise_gauss(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems, float *out);
void oracle_noise_delta(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems, float sigma, int8_t *out);
void oracle_noise_from_words(const uint32_t *words4, uint64_t n, float sigma, float *eps2, int8_t *delta2);
int oracle_perturbed_qgemm(const oracle_tensor *w, const uint64_t *seeds, const uint8_t *perturb_mask, int32_t N, float sigma,
                           const uint16_t *x, int32_t T, uint16_t *y, int32_t act_mode, const int32_t *rows, int32_t n_rows,
                           int32_t antithetic);
int oracle_normalize_fitness(const float *reward, int32_t N, float *fit);
int oracle_replay_residual(const oracle_tensor *w, const uint64_t *hist_seeds, const float *hist_fit, int32_t hist_len,
                           int32_t N, float sigma, float alpha, float gamma, float *residual, const int32_t *rows,
                           int32_t n_rows, int32_t antithetic);
int oracle_update(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                  const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha, float gamma, uint64_t *stats,
                  const int32_t *rows, int32_t n_rows, int32_t antithetic);
int oracle_update_full_residual(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                float alpha, float gamma, float *e_state, float *u_out, uint64_t *stats);
int oracle_update_full_residual_f16(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                    float alpha, float gamma, uint16_t *e_state, uint64_t *stats);
int oracle_update_stochastic_rounding(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                      float alpha, uint64_t round_seed, uint64_t *stats, const int32_t *rows, int32_t n_rows);
int oracle_aggregate(const oracle_tensor *w, const uint64_t *seeds, const float *fit, int32_t N, float sigma, float *g_out,
                     int32_t antithetic);
float oracle_f16_to_f32(uint16_t h);
uint16_t oracle_f32_to_f16_sat(float f);

static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static uint32_t lcg(void)
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(lcg_state >> 32);
}

static uint64_t sum = 1469598103934665603ull;          /* FNV-1a over every output byte */
static void mix(const void *p, size_t n)
{
    const unsigned char *b = (const unsigned char *)p;
    for (size_t i = 0; i < n; ++i) { sum ^= b[i]; sum *= 1099511628211ull; }
}

#define CHECK(call) do { if ((call) != 0) { fprintf(stderr, "oracle call failed: %s\n", #call); return 2; } } while (0)

/* every entry point on one tensor; all buffers are heap blocks of exactly the size the call may touch */
static int exercise(int bits, int group, int out_f, int in_f, int N, int T, int K, int qmin, int qmax)
{
    const size_t elems = (size_t)out_f * in_f;
    const size_t wbytes = bits == 4 ? elems / 2 : elems;
    const size_t n_scales = group ? elems / group : (size_t)out_f;
    uint8_t *qw = malloc(wbytes), *qw0 = malloc(wbytes);
    uint16_t *sc = malloc(n_scales * 2);
    uint16_t *x = malloc((size_t)N * T * in_f * 2), *y = malloc((size_t)N * T * out_f * 2);
    uint64_t *seeds = malloc((size_t)(K + 1) * N * 8);
    float *rew = malloc((size_t)N * 4), *fit = malloc((size_t)(K + 1) * N * 4);
    float *res = malloc(elems * 4), *u = malloc(elems * 4);
    uint16_t *res16 = malloc(elems * 2);
    int32_t rows[3] = { 0, out_f / 2, out_f - 1 };   /* distinct rows only: each listed row is updated once */
    const int32_t n_sel = out_f >= 3 ? 3 : 1;
    if (!qw || !qw0 || !sc || !x || !y || !seeds || !rew || !fit || !res || !u || !res16) return 3;
    for (size_t i = 0; i < wbytes; ++i) {
        if (bits == 4) {
            int lo = qmin + (int)(lcg() % (uint32_t)(qmax - qmin + 1)), hi = qmin + (int)(lcg() % (uint32_t)(qmax - qmin + 1));
            qw0[i] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
        } else {
            qw0[i] = (uint8_t)(int8_t)(qmin + (int)(lcg() % (uint32_t)(qmax - qmin + 1)));
        }
    }
    for (size_t i = 0; i < n_scales; ++i) sc[i] = (uint16_t)(0x2000u + lcg() % 0x400u);      /* halves near 0.01 */
    for (size_t i = 0; i < (size_t)N * T * in_f; ++i) x[i] = (uint16_t)((lcg() & 0x8000u) | (0x3E00u + lcg() % 0x200u));
    for (size_t i = 0; i < (size_t)(K + 1) * N; ++i) seeds[i] = ((uint64_t)lcg() << 32) | lcg();
    for (int t = 0; t <= K; ++t) {
        for (int i = 0; i < N; ++i) rew[i] = (float)(int32_t)(lcg() % 2001u) / 250.0f - 4.0f;
        CHECK(oracle_normalize_fitness(rew, N, fit + (size_t)t * N));
    }
    mix(fit, (size_t)(K + 1) * N * 4);
    oracle_tensor w = { qw, sc, out_f, in_f, bits, group, qmin, qmax, 9u };

    memcpy(qw, qw0, wbytes);
    memset(y, 0, (size_t)N * T * out_f * 2);
    CHECK(oracle_perturbed_qgemm(&w, seeds, NULL, N, 1.0f, x, T, y, 0, NULL, 0, 0));
    mix(y, (size_t)N * T * out_f * 2);
    memset(y, 0, (size_t)N * T * out_f * 2);
    CHECK(oracle_perturbed_qgemm(&w, seeds, NULL, N, 1.0f, x, T, y, 0, rows, n_sel, 0));
    mix(y, (size_t)N * T * out_f * 2);
    if ((N & 1) == 0) {
        memset(y, 0, (size_t)N * T * out_f * 2);
        CHECK(oracle_perturbed_qgemm(&w, seeds, NULL, N, 1.5f, x, T, y, 0, NULL, 0, 1));
        mix(y, (size_t)N * T * out_f * 2);
    }
    if (bits == 8 && group == 0) {
        memset(y, 0, (size_t)N * T * out_f * 2);
        CHECK(oracle_perturbed_qgemm(&w, seeds, NULL, N, 1.0f, x, T, y, 1, NULL, 0, 0));
        mix(y, (size_t)N * T * out_f * 2);
    }
    memset(res, 0, elems * 4);
    CHECK(oracle_replay_residual(&w, seeds, fit, K, N, 1.0f, 1.5f, 0.9f, res, NULL, 0, 0));
    mix(res, elems * 4);
    memset(res, 0, elems * 4);
    CHECK(oracle_replay_residual(&w, seeds, fit, K, N, 1.0f, 1.5f, 0.9f, res, rows, n_sel, 0));
    mix(res, elems * 4);
    CHECK(oracle_aggregate(&w, seeds, fit, N, 1.0f, u, 0));
    mix(u, elems * 4);
    uint64_t stats[2] = { 0, 0 };
    CHECK(oracle_update(&w, seeds + (size_t)K * N, fit + (size_t)K * N, seeds, fit, K, N, 1.0f, 1.5f, 0.9f, stats, NULL, 0, 0));
    mix(qw, wbytes);
    memcpy(qw, qw0, wbytes);
    CHECK(oracle_update(&w, seeds + (size_t)K * N, fit + (size_t)K * N, seeds, fit, K, N, 1.0f, 1.5f, 0.9f, stats, rows, n_sel, 0));
    mix(qw, wbytes);
    if ((N & 1) == 0) {
        memcpy(qw, qw0, wbytes);
        /* antithetic: N/2 seeds per generation, read from the front of the same array */
        CHECK(oracle_update(&w, seeds + (size_t)K * (N / 2), fit + (size_t)K * N, seeds, fit, K, N, 1.0f, 1.5f, 0.9f, stats,
                            NULL, 0, 1));
        mix(qw, wbytes);
    }
    memcpy(qw, qw0, wbytes);
    memset(res, 0, elems * 4);
    for (int t = 0; t <= K; ++t)
        CHECK(oracle_update_full_residual(&w, seeds + (size_t)t * N, fit + (size_t)t * N, N, 1.0f, 1.5f, 0.9f, res, u, stats));
    mix(qw, wbytes);
    mix(res, elems * 4);
    mix(u, elems * 4);
    memcpy(qw, qw0, wbytes);
    memset(res16, 0, elems * 2);
    for (int t = 0; t <= K; ++t)
        CHECK(oracle_update_full_residual_f16(&w, seeds + (size_t)t * N, fit + (size_t)t * N, N, 1.0f, 1.5f, 0.9f, res16, stats));
    mix(qw, wbytes);
    mix(res16, elems * 2);
    memcpy(qw, qw0, wbytes);
    CHECK(oracle_update_stochastic_rounding(&w, seeds, fit, N, 1.0f, 3.0f, 0x123456789ull, stats, NULL, 0));
    CHECK(oracle_update_stochastic_rounding(&w, seeds, fit, N, 1.0f, 3.0f, 0x123456789ull, stats, rows, n_sel));
    mix(qw, wbytes);
    mix(stats, sizeof stats);
    free(qw); free(qw0); free(sc); free(x); free(y); free(seeds); free(rew); free(fit); free(res); free(u); free(res16);
    return 0;
}

int main(void)
{
    /* noise probes: windows that start and end inside a pair, 64-bit counters */
    uint32_t words[4 * 5];
    float g[7];
    int8_t d[7];
    float eps2[10];
    int8_t delta2[10];
    oracle_noise_words(0xFEDCBA9876543210ull, 7u, 0xFFFFFFFFull - 1, 5, words);
    oracle_noise_gauss(3u, 7u, 0x1FFFFFFFFull, 7, g);
    oracle_noise_delta(3u, 7u, 0x1FFFFFFFFull, 7, 2.5f, d);
    oracle_noise_from_words(words, 5, 8.0f, eps2, delta2);
    mix(words, sizeof words); mix(g, sizeof g); mix(d, sizeof d); mix(eps2, sizeof eps2); mix(delta2, sizeof delta2);
    const uint32_t edge[4 * 3] = { 0u, 0u, 0u, 0u, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFF00u, 0x40000000u, 0x80000000u, 1u };
    oracle_noise_from_words(edge, 3, 1000.0f, eps2, delta2);
    mix(eps2, 6 * sizeof(float)); mix(delta2, 6);
    float s, c, l;
    l = oracle_ln_u1(1u); mix(&l, 4);
    l = oracle_ln_u1(1u << 24); mix(&l, 4);
    oracle_sincos_quarter(0.0f, &s, &c); mix(&s, 4); mix(&c, 4);
    oracle_sincos_quarter(0x1.fffffep-1f, &s, &c); mix(&s, 4); mix(&c, 4);
    for (uint32_t h = 0; h < 0x10000u; h += 37u) {
        float f = oracle_f16_to_f32((uint16_t)h);
        if (f == f) { uint16_t back = oracle_f32_to_f16_sat(f); mix(&back, 2); }
    }
    const float conv[] = { 0.0f, -0.0f, 65504.0f, 65520.0f, 1e30f, -1e30f, 5.9604645e-8f, 2.9802322e-8f, 1e-30f, 0.33325195f };
    for (size_t i = 0; i < sizeof conv / sizeof conv[0]; ++i) { uint16_t h = oracle_f32_to_f16_sat(conv[i]); mix(&h, 2); }

    int rc;
    if ((rc = exercise(4, 32, 6, 64, 4, 3, 2, -8, 7)) != 0) return rc;
    if ((rc = exercise(4, 0, 5, 34, 3, 1, 0, -7, 7)) != 0) return rc;     /* per-row scale, odd N, no history */
    if ((rc = exercise(8, 0, 7, 70, 6, 2, 3, -127, 127)) != 0) return rc; /* W8A8 path as well */
    if ((rc = exercise(8, 0, 1, 2, 2, 1, 1, -128, 127)) != 0) return rc;  /* the smallest tensor */
    printf("checksum %016llx\n", (unsigned long long)sum);
    return 0;
}
