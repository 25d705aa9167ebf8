/*
 * CPU oracle for the Quantized Evolution Strategies (QES) hot path.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the plain, slow, obviously-correct statement of what the
 * GPU library must compute. Only tests, the smoke check and the benchmark's cpu_baseline leg may
 * load it; the product path never does. It shares no source, header, table or helper with the HIP
 * kernels: both sides implement docs/NOISE_SPEC.md and the paper's algorithms separately.
 *
 * What follows the paper, passage by passage:
 *   - noise draw              : paper §3.2 Eq. 3 (stochastically rounded Gaussian), App. A.1 (4-bit δ)
 *   - evaluation gate          : §3.2 Eq. 4 (out-of-range perturbations are masked)
 *   - perturbed linear layer   : Alg. 1 steps "reconstruct δ_i", "W' = Gate(W_t + δ_i)", inference
 *   - gradient estimate        : §3.2 Eq. 5, ĝ = 1/(Nσ) Σ_i F_i δ_i
 *   - error feedback           : §3.2 Eq. 6-8 and Alg. 1 (u = αĝ + γe; ΔW = Round(u); e = u − ΔW)
 *   - stateless seed replay    : §3.3 and Alg. 2 (rebuild the residual from the last K (seeds,
 *                                fitnesses), gating against the CURRENT weights, then update)
 *
 * Readings taken where the paper is silent or inconsistent (all listed in the design document):
 *   - "RNG(S)" in Alg. 2 regenerates ε and b, hence δ; Agg is Eq. 5 on δ (same as Alg. 1).
 *   - codebook range is data (qmin, qmax): Eq. 4 becomes qmin ≤ W+δ ≤ qmax.
 *   - σ and α are in integer-grid units; scales never enter the update.
 *   - Round = round-half-to-even.
 *   - both algorithms use the gated Δ in W and in the residual (so W + e stays exact at edges).
 *   - u_t = c·g_t + γ·e_entering_step_t with e_0 = 0, c = α/(Nσ); residual arithmetic in fp32.
 *
 * Parity pins (tests/test_oracle_*.py): Philox known answers and inverse rounds; ln/sin/cos against
 * libm within the stated polynomial error; Gaussian moments and KS distance; E[δ|ε] = σε by
 * enumeration; σ=0 GEMM equals a library matmul of the dequantised matrix; brute-force loops on
 * tiny layers; the bit-exact telescoping identity Σ Δ + e_T = c Σ g for dyadic inputs; replayed
 * residual equals stored residual; zero fitness variance gives zero update; gate behaviour at the
 * range edges. Accuracy figures of the paper's experiments need its datasets and are unpinned.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (see oracle/build.py). The flag
 * -ffp-contract=off matters: every fused operation below is an explicit fmaf().
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ----------------------------------------------------------------------------------------------
 * Tensor description (host pointers).
 *   qweight : logical [out_features, in_features], row-major, in_features contiguous.
 *             bits=4: two elements per byte, element 2b in the low nibble of byte b, element 2b+1 in
 *             the high nibble, each a 4-bit two's-complement integer.  bits=8: int8.
 *   scales  : IEEE binary16 bit patterns. group_size>0: [out_features, in_features/group_size];
 *             group_size==0: one scale per row, [out_features].
 * -------------------------------------------------------------------------------------------- */
typedef struct {
    void *qweight;
    const uint16_t *scales;
    int32_t out_features, in_features;
    int32_t bits;
    int32_t group_size;
    int32_t qmin, qmax;
    uint32_t tensor_id;
} oracle_tensor;

enum { ORACLE_OK = 0, ORACLE_ERR_INVALID_ARG = -1 };

/* ---------------------------------------- N1: Philox4x32-10 ---------------------------------- */

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* N2: words for one pair of K-adjacent elements */
static void pair_words(uint64_t seed, uint32_t tensor_id, uint64_t pair, uint32_t w[4])
{
    uint32_t ctr[4] = { (uint32_t)(pair & 0xFFFFFFFFu), (uint32_t)(pair >> 32), tensor_id, 0u };
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    oracle_philox4x32_10(ctr, key, w);
}

static inline uint32_t f2u(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float u2f(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ---------------------------------------- N4: fixed polynomials ------------------------------ */

/* ln(m * 2^-24), m in [1, 2^24] */
float oracle_ln_u1(uint32_t m)
{
    const float LN2 = 0x1.62e430p-1f;
    const float LP0 = -0x1.000060p-1f, LP1 = 0x1.5559f0p-2f, LP2 = -0x1.ff7476p-3f,
                LP3 = 0x1.976dd8p-3f, LP4 = -0x1.6049d0p-3f, LP5 = 0x1.4d64acp-3f,
                LP6 = -0x1.a7d988p-4f;
    float xf = (float)m;
    uint32_t ix = f2u(xf) - 0x3F3504F3u;
    int32_t e = (int32_t)(ix >> 23);
    float t = u2f((ix & 0x007FFFFFu) + 0x3F3504F3u) - 1.0f;
    float p = LP6;
    p = fmaf(p, t, LP5);
    p = fmaf(p, t, LP4);
    p = fmaf(p, t, LP3);
    p = fmaf(p, t, LP2);
    p = fmaf(p, t, LP1);
    p = fmaf(p, t, LP0);
    float l1 = fmaf(t * t, p, t);
    return fmaf((float)(e - 24), LN2, l1);
}

/* sin and cos of (pi/2)*f for f in [0,1) */
void oracle_sincos_quarter(float f, float *s_out, float *c_out)
{
    const float SP0 = 0x1.921fb6p+0f, SP1 = -0x1.4abbc4p-1f, SP2 = 0x1.4668f2p-4f,
                SP3 = -0x1.32535ap-8f, SP4 = 0x1.3e17cap-13f;
    const float CP0 = 0x1.fffffep-1f, CP1 = -0x1.3bd3a6p+0f, CP2 = 0x1.03bd06p-2f,
                CP3 = -0x1.54f61ap-6f, CP4 = 0x1.c1f064p-11f;
    float z = f * f;
    float sp = SP4;
    sp = fmaf(sp, z, SP3);
    sp = fmaf(sp, z, SP2);
    sp = fmaf(sp, z, SP1);
    sp = fmaf(sp, z, SP0);
    float c = CP4;
    c = fmaf(c, z, CP3);
    c = fmaf(c, z, CP2);
    c = fmaf(c, z, CP1);
    c = fmaf(c, z, CP0);
    *s_out = f * sp;
    *c_out = c;
}

/* N3+N4: the two Gaussians of one Philox call */
static void words_to_gauss(const uint32_t w[4], float eps[2])
{
    uint32_t m = (w[0] >> 8) + 1u;
    uint32_t q = w[1] >> 30;
    float f = (float)((w[1] >> 6) & 0xFFFFFFu) * 0x1p-24f;
    float L = oracle_ln_u1(m);
    float r = sqrtf(-2.0f * L);
    float s, c, cr, sr;
    oracle_sincos_quarter(f, &s, &c);
    switch (q) {
    case 0:  cr = c;  sr = s;  break;
    case 1:  cr = -s; sr = c;  break;
    case 2:  cr = -c; sr = -s; break;
    default: cr = s;  sr = -c; break;
    }
    eps[0] = r * cr;
    eps[1] = r * sr;
}

/* N5+N6: one lane's integer perturbation */
static int32_t gauss_to_delta(float eps, uint32_t wround, float sigma)
{
    float ub = (float)(wround >> 8) * 0x1p-24f;
    float t = sigma * eps;
    float fl = floorf(t);
    float fr = t - fl;
    int32_t d = (int32_t)fl + ((ub < fr) ? 1 : 0);
    if (d < -8) d = -8;
    if (d > 7) d = 7;
    return d;
}

/* the two δ of one Philox call: d[0] for element 2·pair, d[1] for element 2·pair+1 */
static void pair_deltas(uint64_t seed, uint32_t tensor_id, uint64_t pair, float sigma, int32_t d[2])
{
    uint32_t w[4];
    float eps[2];
    pair_words(seed, tensor_id, pair, w);
    words_to_gauss(w, eps);
    d[0] = gauss_to_delta(eps[0], w[2], sigma);
    d[1] = gauss_to_delta(eps[1], w[3], sigma);
}

/* δ for element index e (pair = e>>1, lane = e&1) */
static int32_t delta_of_element(uint64_t seed, uint32_t tensor_id, uint64_t e, float sigma)
{
    int32_t d[2];
    pair_deltas(seed, tensor_id, e >> 1, sigma, d);
    return d[e & 1u];
}

/* ---------------------------------------- probes (tests compare these bit for bit) ----------- */

void oracle_noise_words(uint64_t seed, uint32_t tensor_id, uint64_t pair_begin, uint64_t n_pairs,
                        uint32_t *out4)
{
    for (uint64_t i = 0; i < n_pairs; ++i)
        pair_words(seed, tensor_id, pair_begin + i, out4 + 4 * i);
}

void oracle_noise_gauss(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems,
                        float *out)
{
    for (uint64_t i = 0; i < n_elems; ++i) {
        uint64_t e = elem_begin + i;
        uint32_t w[4];
        float eps[2];
        pair_words(seed, tensor_id, e >> 1, w);
        words_to_gauss(w, eps);
        out[i] = eps[e & 1u];
    }
}

void oracle_noise_delta(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems,
                        float sigma, int8_t *out)
{
    for (uint64_t i = 0; i < n_elems; ++i)
        out[i] = (int8_t)delta_of_element(seed, tensor_id, elem_begin + i, sigma);
}

/* N3-N6 on caller-supplied words: Gaussians and perturbations of n word quadruples */
void oracle_noise_from_words(const uint32_t *words4, uint64_t n, float sigma, float *eps2, int8_t *delta2)
{
    for (uint64_t i = 0; i < n; ++i) {
        float eps[2];
        words_to_gauss(words4 + 4 * i, eps);
        if (eps2) { eps2[2 * i] = eps[0]; eps2[2 * i + 1] = eps[1]; }
        if (delta2) {
            delta2[2 * i] = (int8_t)gauss_to_delta(eps[0], words4[4 * i + 2], sigma);
            delta2[2 * i + 1] = (int8_t)gauss_to_delta(eps[1], words4[4 * i + 3], sigma);
        }
    }
}

/* δ for a caller-supplied Gaussian and rounding word: lets a test enumerate the rounding uniform */
int32_t oracle_delta_from_gauss(float eps, uint32_t wround, float sigma)
{
    return gauss_to_delta(eps, wround, sigma);
}

/* ---------------------------------------- formats -------------------------------------------- */

static int32_t load_q(const oracle_tensor *w, int64_t row, int64_t col)
{
    if (w->bits == 4) {
        const uint8_t *p = (const uint8_t *)w->qweight;
        uint8_t byte = p[(row * (int64_t)w->in_features + col) >> 1];
        int32_t nib = (col & 1) ? (byte >> 4) : (byte & 0xF);
        return nib >= 8 ? nib - 16 : nib;
    }
    return ((const int8_t *)w->qweight)[row * (int64_t)w->in_features + col];
}

static void store_q(oracle_tensor *w, int64_t row, int64_t col, int32_t v)
{
    if (w->bits == 4) {
        uint8_t *p = (uint8_t *)w->qweight;
        int64_t b = (row * (int64_t)w->in_features + col) >> 1;
        uint8_t nib = (uint8_t)(v & 0xF);
        if (col & 1) p[b] = (uint8_t)((p[b] & 0x0F) | (nib << 4));
        else         p[b] = (uint8_t)((p[b] & 0xF0) | nib);
    } else {
        ((int8_t *)w->qweight)[row * (int64_t)w->in_features + col] = (int8_t)v;
    }
}

static double half_to_double(uint16_t h)
{
    int sign = h >> 15, ex = (h >> 10) & 0x1F, man = h & 0x3FF;
    double v;
    if (ex == 0)       v = ldexp((double)man, -24);
    else if (ex == 31) v = man ? NAN : INFINITY;
    else               v = ldexp((double)(man | 0x400), ex - 25);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t b) { return (double)u2f((uint32_t)b << 16); }

/* nearest bfloat16 to a double, ties to even */
static uint16_t double_to_bf16(double d)
{
    if (isnan(d)) return 0x7FC0;
    float f = (float)d;
    uint32_t u = f2u(f);
    uint32_t lo = u & 0xFFFF0000u;          /* truncated toward zero */
    if (isinf(f)) return (uint16_t)(u >> 16);
    uint32_t hi = lo + 0x10000u;            /* next bf16 away from zero (may become inf) */
    double dlo = (double)u2f(lo), dhi = (double)u2f(hi);
    double ad = fabs(d), elo = fabs(ad - fabs(dlo)), ehi = fabs(fabs(dhi) - ad);
    uint32_t pick;
    if (elo < ehi) pick = lo;
    else if (ehi < elo) pick = hi;
    else pick = ((lo >> 16) & 1u) ? hi : lo;
    return (uint16_t)(pick >> 16);
}

static uint16_t float_to_bf16(float f) { return double_to_bf16((double)f); }

static int tensor_ok(const oracle_tensor *w)
{
    if (!w || !w->qweight) return 0;
    if (w->out_features <= 0 || w->in_features <= 0 || (w->in_features & 1)) return 0;
    if (w->bits != 4 && w->bits != 8) return 0;
    if (w->group_size < 0) return 0;
    if (w->group_size > 0 && (w->in_features % w->group_size)) return 0;
    if (w->qmin > w->qmax) return 0;
    if (w->bits == 4 && (w->qmin < -8 || w->qmax > 7)) return 0;
    if (w->bits == 8 && (w->qmin < -128 || w->qmax > 127)) return 0;
    return 1;
}

static double scale_of(const oracle_tensor *w, int64_t row, int64_t col)
{
    if (w->group_size > 0) {
        int64_t groups = w->in_features / w->group_size;
        return half_to_double(w->scales[row * groups + col / w->group_size]);
    }
    return half_to_double(w->scales[row]);
}

/* ---------------------------------------- perturbed quantised GEMM --------------------------- */

/*
 * Y[i,t,n] for every member i, token t and every output row n listed in `rows` (all rows when
 * rows == NULL). x: bf16 bits [N,T,in]; y: bf16 bits [N,T,out] (only the selected columns are
 * written). perturb_mask[i]==0 evaluates member i on the unperturbed weights.
 * act_mode 0: bf16 activations, fp64 accumulation of s[n,g]·Σ_k X·W'.
 * act_mode 1 (bits=8, per-row scale): dynamic symmetric per-token int8 activations, exact int32
 * accumulation, Y = bf16(((float)acc·a[t])·(float)s[n]).
 * antithetic != 0 (App. A.1, "antithetic perturbation pairs"): N is even, seeds has N/2 entries,
 * members 2j and 2j+1 share seed j and member 2j+1 uses the negated perturbation -δ_j.
 */
int oracle_perturbed_qgemm(const oracle_tensor *w, const uint64_t *seeds, const uint8_t *perturb_mask,
                           int32_t N, float sigma, const uint16_t *x, int32_t T, uint16_t *y,
                           int32_t act_mode, const int32_t *rows, int32_t n_rows, int32_t antithetic)
{
    if (antithetic && (N & 1)) return ORACLE_ERR_INVALID_ARG;
    if (!tensor_ok(w) || !w->scales || !seeds || !x || !y || N <= 0 || T <= 0) return ORACLE_ERR_INVALID_ARG;
    if (!(sigma >= 0.0f)) return ORACLE_ERR_INVALID_ARG;
    if (act_mode != 0 && act_mode != 1) return ORACLE_ERR_INVALID_ARG;
    if (act_mode == 1 && (w->bits != 8 || w->group_size != 0)) return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features, O = w->out_features;
    const int32_t nsel = rows ? n_rows : (int32_t)O;

    /* per-token activation quantisation for act_mode 1 */
    int8_t *xq = NULL;
    float *ascale = NULL;
    if (act_mode == 1) {
        xq = (int8_t *)malloc((size_t)N * T * K);
        ascale = (float *)malloc((size_t)N * T * sizeof(float));
        if (!xq || !ascale) { free(xq); free(ascale); return ORACLE_ERR_INVALID_ARG; }
#pragma omp parallel for schedule(static)
        for (int64_t it = 0; it < (int64_t)N * T; ++it) {   /* tokens are independent */
            float amax = 0.0f;
            for (int64_t k = 0; k < K; ++k) {
                float v = fabsf(u2f((uint32_t)x[it * K + k] << 16));
                if (v > amax) amax = v;
            }
            float a = amax / 127.0f;
            if (a == 0.0f) a = 1.0f;
            ascale[it] = a;
            for (int64_t k = 0; k < K; ++k) {
                float v = rintf(u2f((uint32_t)x[it * K + k] << 16) / a);
                if (v > 127.0f) v = 127.0f;
                if (v < -127.0f) v = -127.0f;
                xq[it * K + k] = (int8_t)v;
            }
        }
    }

#pragma omp parallel
    {
        int32_t *wp = (int32_t *)malloc((size_t)K * sizeof(int32_t));
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int32_t i = 0; i < N; ++i) {
            for (int32_t r = 0; r < nsel; ++r) {
                const int64_t n = rows ? rows[r] : r;
                /* this member's perturbed, gated row (Eq. 3, Eq. 4) */
                for (int64_t k = 0; k < K; k += 2) {
                    int32_t d[2] = { 0, 0 };
                    if (!perturb_mask || perturb_mask[i]) {
                        pair_deltas(seeds[antithetic ? i / 2 : i], w->tensor_id, (uint64_t)(n * K + k) >> 1, sigma, d);
                        if (antithetic && (i & 1)) { d[0] = -d[0]; d[1] = -d[1]; }
                    }
                    for (int l = 0; l < 2; ++l) {
                        int32_t q = load_q(w, n, k + l);
                        int32_t v = q + d[l];
                        wp[k + l] = (v >= w->qmin && v <= w->qmax) ? v : q;
                    }
                }
                for (int32_t t = 0; t < T; ++t) {
                    const int64_t it = (int64_t)i * T + t;
                    if (act_mode == 1) {
                        int32_t acc = 0;
                        for (int64_t k = 0; k < K; ++k) acc += (int32_t)xq[it * K + k] * wp[k];
                        float sc = (float)half_to_double(w->scales[n]);
                        float v = ((float)acc * ascale[it]) * sc;
                        y[it * O + n] = float_to_bf16(v);
                    } else {
                        double total = 0.0;
                        const int64_t gs = w->group_size > 0 ? w->group_size : K;
                        for (int64_t g0 = 0; g0 < K; g0 += gs) {
                            double part = 0.0;
                            for (int64_t k = g0; k < g0 + gs; ++k)
                                part += bf16_to_double(x[it * K + k]) * (double)wp[k];
                            total += scale_of(w, n, g0) * part;
                        }
                        y[it * O + n] = double_to_bf16(total);
                    }
                }
            }
        }
        free(wp);
    }
    free(xq);
    free(ascale);
    return ORACLE_OK;
}

/* ---------------------------------------- fitness normalisation ------------------------------ */

/* z-score with the population standard deviation; zero variance (or N<2) gives all zeros */
int oracle_normalize_fitness(const float *reward, int32_t N, float *fit)
{
    if (!reward || !fit || N <= 0) return ORACLE_ERR_INVALID_ARG;
    double mu = 0.0;
    for (int32_t i = 0; i < N; ++i) mu += (double)reward[i];
    mu /= (double)N;
    double var = 0.0;
    for (int32_t i = 0; i < N; ++i) { double d = (double)reward[i] - mu; var += d * d; }
    var /= (double)N;
    double sd = sqrt(var);
    for (int32_t i = 0; i < N; ++i)
        fit[i] = (N < 2 || sd == 0.0) ? 0.0f : (float)(((double)reward[i] - mu) / sd);
    return ORACLE_OK;
}

/* ---------------------------------------- error-feedback step -------------------------------- */

static float step_coeff(float alpha, int32_t N, float sigma)
{
    return (float)((double)alpha / ((double)N * (double)sigma));
}

/* Eq. 5: g = Σ_i F_i δ_i for the two elements of one pair, members in index order, fp32 fma chain */
static void aggregate_pair(const uint64_t *seeds, const float *fit, int32_t N, uint32_t tensor_id,
                           uint64_t pair, float sigma, int32_t antithetic, float g[2])
{
    g[0] = 0.0f;
    g[1] = 0.0f;
    for (int32_t i = 0; i < N; ++i) {
        int32_t d[2];
        /* antithetic pairs: members 2j and 2j+1 share seed j; the odd member's δ is negated */
        pair_deltas(seeds[antithetic ? i / 2 : i], tensor_id, pair, sigma, d);
        if (antithetic && (i & 1)) { d[0] = -d[0]; d[1] = -d[1]; }
        g[0] = fmaf(fit[i], (float)d[0], g[0]);
        g[1] = fmaf(fit[i], (float)d[1], g[1]);
    }
}

/* saturating float -> int32 of an already integral value; NaN gives 0 */
static int32_t sat_i32(float v)
{
    if (v != v) return 0;
    if (v >= 2147483648.0f) return INT32_MAX;
    if (v <= -2147483648.0f) return INT32_MIN;
    return (int32_t)v;
}

/*
 * One error-feedback step for one element (Eq. 6-8 with the gate of Alg. 2):
 * u = c·g + γ·e; Δ = Round(u); Δf = Δ if qmin ≤ wq+Δ ≤ qmax else 0. Returns Δf, writes u.
 */
static int32_t ef_step(float c, float g, float gamma, float e, int32_t wq, int32_t qmin, int32_t qmax,
                       float *u_out, int32_t *raw_delta)
{
    float u = fmaf(c, g, gamma * e);
    int32_t d = sat_i32(rintf(u));
    int64_t v = (int64_t)wq + (int64_t)d;
    *u_out = u;
    if (raw_delta) *raw_delta = d;
    return (v >= qmin && v <= qmax) ? d : 0;
}

static int hist_ok(const uint64_t *hs, const float *hf, int32_t hist_len, int32_t N, float sigma)
{
    if (hist_len < 0 || N <= 0) return 0;
    if (hist_len > 0 && (!hs || !hf)) return 0;
    if (!(sigma > 0.0f)) return 0;
    return 1;
}

/* Alg. 2, replay loop: proxy residuals of the two elements of one pair, rebuilt from the
 * history, oldest first, gating every simulated step against the current weights wq[]. */
static void replay_pair(const oracle_tensor *w, const uint64_t *hist_seeds, const float *hist_fit,
                        int32_t hist_len, int32_t N, float sigma, float c, float gamma,
                        uint64_t pair, const int32_t wq[2], int32_t antithetic, float res[2])
{
    const int64_t seeds_per_gen = antithetic ? N / 2 : N;
    res[0] = 0.0f;
    res[1] = 0.0f;
    for (int32_t tau = 0; tau < hist_len; ++tau) {
        float g[2];
        aggregate_pair(hist_seeds + (int64_t)tau * seeds_per_gen, hist_fit + (int64_t)tau * N, N, w->tensor_id,
                       pair, sigma, antithetic, g);
        for (int l = 0; l < 2; ++l) {
            float u;
            int32_t df = ef_step(c, g[l], gamma, res[l], wq[l], w->qmin, w->qmax, &u, NULL);
            res[l] = u - (float)df;
        }
    }
}

/*
 * Alg. 2 (the replay loop only): residual[out,in] fp32 for the rows listed (all when rows == NULL;
 * other rows of `residual` are left untouched).
 */
int oracle_replay_residual(const oracle_tensor *w, const uint64_t *hist_seeds, const float *hist_fit,
                           int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                           float *residual, const int32_t *rows, int32_t n_rows, int32_t antithetic)
{
    if (!tensor_ok(w) || !residual || !hist_ok(hist_seeds, hist_fit, hist_len, N, sigma))
        return ORACLE_ERR_INVALID_ARG;
    if (antithetic && (N & 1)) return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features;
    const int32_t nsel = rows ? n_rows : w->out_features;
    const float c = step_coeff(alpha, N, sigma);
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t r = 0; r < nsel; ++r) {
        const int64_t n = rows ? rows[r] : r;
        for (int64_t k = 0; k < K; k += 2) {
            const int32_t wq[2] = { load_q(w, n, k), load_q(w, n, k + 1) };
            float res[2];
            replay_pair(w, hist_seeds, hist_fit, hist_len, N, sigma, c, gamma,
                        (uint64_t)(n * K + k) >> 1, wq, antithetic, res);
            residual[n * K + k] = res[0];
            residual[n * K + k + 1] = res[1];
        }
    }
    return ORACLE_OK;
}

/*
 * Alg. 2 in full: replay the history, then apply the new population's step to the weights in
 * place (all rows, or the distinct rows listed in `rows`: a row listed twice would be updated twice). stats (may be NULL): stats[0] += number of elements whose weight changed, stats[1] +=
 * number of elements whose non-zero rounded update was masked by the gate (final step only; Eq. 4
 * masks updates, so a zero update is never counted, whatever the stored weight is).
 */
int oracle_update(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t,
                  const uint64_t *hist_seeds, const float *hist_fit, int32_t hist_len, int32_t N,
                  float sigma, float alpha, float gamma, uint64_t *stats,
                  const int32_t *rows, int32_t n_rows, int32_t antithetic)
{
    if (!tensor_ok(w) || !seeds_t || !fit_t || !hist_ok(hist_seeds, hist_fit, hist_len, N, sigma))
        return ORACLE_ERR_INVALID_ARG;
    if (antithetic && (N & 1)) return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features;
    const int32_t nsel = rows ? n_rows : w->out_features;
    const float c = step_coeff(alpha, N, sigma);
    uint64_t changed = 0, gated = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : changed, gated)
    for (int32_t r = 0; r < nsel; ++r) {
        const int64_t n = rows ? rows[r] : r;
        for (int64_t k = 0; k < K; k += 2) {
            const uint64_t pair = (uint64_t)(n * K + k) >> 1;
            const int32_t wq[2] = { load_q(w, n, k), load_q(w, n, k + 1) };
            float res[2], g[2];
            replay_pair(w, hist_seeds, hist_fit, hist_len, N, sigma, c, gamma, pair, wq, antithetic, res);
            aggregate_pair(seeds_t, fit_t, N, w->tensor_id, pair, sigma, antithetic, g);
            for (int l = 0; l < 2; ++l) {
                float u;
                int32_t raw;
                int32_t df = ef_step(c, g[l], gamma, res[l], wq[l], w->qmin, w->qmax, &u, &raw);
                if (df != 0) { store_q(w, n, k + l, wq[l] + df); ++changed; }
                else if (raw != 0) ++gated;
            }
        }
    }
    if (stats) { stats[0] += changed; stats[1] += gated; }
    return ORACLE_OK;
}

/*
 * Alg. 1 (Full-Residual variant): one step with an explicitly stored fp32 residual e[out,in],
 * updated in place together with the weights. u_out (may be NULL) receives the high-precision
 * update u of every element, for the telescoping-identity pin.
 */
int oracle_update_full_residual(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t,
                                int32_t N, float sigma, float alpha, float gamma, float *e_state,
                                float *u_out, uint64_t *stats)
{
    if (!tensor_ok(w) || !seeds_t || !fit_t || !e_state || N <= 0 || !(sigma > 0.0f))
        return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features;
    const float c = step_coeff(alpha, N, sigma);
    uint64_t changed = 0, gated = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : changed, gated)
    for (int32_t n = 0; n < w->out_features; ++n) {
        for (int64_t k = 0; k < K; k += 2) {
            const uint64_t e0 = (uint64_t)((int64_t)n * K + k);
            float g[2];
            aggregate_pair(seeds_t, fit_t, N, w->tensor_id, e0 >> 1, sigma, 0, g);
            for (int l = 0; l < 2; ++l) {
                int32_t wq = load_q(w, n, k + l);
                float u;
                int32_t raw;
                int32_t df = ef_step(c, g[l], gamma, e_state[e0 + l], wq, w->qmin, w->qmax, &u, &raw);
                e_state[e0 + l] = u - (float)df;
                if (u_out) u_out[e0 + l] = u;
                if (df != 0) { store_q(w, n, k + l, wq + df); ++changed; }
                else if (raw != 0) ++gated;
            }
        }
    }
    if (stats) { stats[0] += changed; stats[1] += gated; }
    return ORACLE_OK;
}

/*
 * Stateless baseline of §5 (W ← W + Q(α ĝ) with a stochastic Q; the rule the paper attributes to
 * QuZO-style training): no residual; Δ = ⌊u⌋ + [ub < u − ⌊u⌋] with u = c·g and ub the element's
 * rounding uniform of the step (N8: Philox keyed by round_seed, stream tag 1, words 2 and 3); the
 * range gate is Eq. 4's (masked). Unbiased per step, E[Δ] = u, but the errors do not cancel over
 * steps.
 */
int oracle_update_stochastic_rounding(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t,
                                      int32_t N, float sigma, float alpha, uint64_t round_seed,
                                      uint64_t *stats, const int32_t *rows, int32_t n_rows)
{
    if (!tensor_ok(w) || !seeds_t || !fit_t || N <= 0 || !(sigma > 0.0f)) return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features;
    const int32_t nsel = rows ? n_rows : w->out_features;
    const float c = step_coeff(alpha, N, sigma);
    const uint32_t key[2] = { (uint32_t)(round_seed & 0xFFFFFFFFu), (uint32_t)(round_seed >> 32) };
    uint64_t changed = 0, gated = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : changed, gated)
    for (int32_t r = 0; r < nsel; ++r) {
        const int64_t n = rows ? rows[r] : r;
        for (int64_t k = 0; k < K; k += 2) {
            const uint64_t pair = (uint64_t)(n * K + k) >> 1;
            float g[2];
            aggregate_pair(seeds_t, fit_t, N, w->tensor_id, pair, sigma, 0, g);
            const uint32_t ctr[4] = { (uint32_t)(pair & 0xFFFFFFFFu), (uint32_t)(pair >> 32), w->tensor_id, 1u };
            uint32_t words[4];
            oracle_philox4x32_10(ctr, key, words);
            for (int l = 0; l < 2; ++l) {
                const int32_t wq = load_q(w, n, k + l);
                const float u = c * g[l];
                const float ub = (float)(words[2 + l] >> 8) * 0x1p-24f;
                const float fl = floorf(u);
                const float fr = u - fl;
                const int32_t d = sat_i32(fl) + ((ub < fr) ? 1 : 0);
                const int64_t v = (int64_t)wq + (int64_t)d;
                /* Eq. 4 masks a perturbation that would leave the range; a zero update has nothing
                 * to mask, also when the stored weight itself lies outside [qmin, qmax] */
                if (d == 0) continue;
                if (v >= w->qmin && v <= w->qmax) { store_q(w, n, k + l, (int32_t)v); ++changed; }
                else ++gated;
            }
        }
    }
    if (stats) { stats[0] += changed; stats[1] += gated; }
    return ORACLE_OK;
}

/*
 * IEEE binary16 <-> binary32, written out (Alg. 1 initialises the residuals as FP16, and the
 * Full-Residual variant of the residual ablation in §4 stores them so). Encoding rounds to nearest even after saturating at the largest finite
 * half (±65504), so a stored residual is always finite; NaN does not occur (inputs are finite).
 */
float oracle_f16_to_f32(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const int32_t e = (h >> 10) & 0x1F;
    const uint32_t m = h & 0x3FFu;
    double v;
    if (e == 0) v = ldexp((double)m, -24);                 /* zero and subnormals: m · 2^-24 */
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m | 0x400u), e - 25);          /* (1024+m) · 2^(e-15-10) */
    float f = (float)v;                                    /* exact: 11 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    u |= sign;
    memcpy(&f, &u, 4);
    return f;
}

uint16_t oracle_f32_to_f16_sat(float f)
{
    const double a = fabs((double)f);
    const uint16_t sign = signbit(f) ? 0x8000u : 0u;
    if (a >= 65504.0) return (uint16_t)(sign | 0x7BFFu);
    if (a == 0.0) return sign;
    /* spacing of halves around a: 2^(e-10) with e = floor(log2 a), never below 2^-24 */
    int e;
    (void)frexp(a, &e);                                    /* a = m·2^e, m in [0.5,1) -> floor(log2 a) = e-1 */
    int q = (e - 1) - 10;
    if (q < -24) q = -24;
    const double steps = nearbyint(ldexp(a, -q));          /* ties to even in the default rounding mode */
    const double r = ldexp(steps, q);                      /* the nearest half, as a double; r <= 65504 */
    /* encode r exactly */
    if (r == 0.0) return sign;
    (void)frexp(r, &e);
    const int eb = (e - 1) + 15;                           /* biased exponent */
    if (eb <= 0) return (uint16_t)(sign | (uint16_t)ldexp(r, 24));          /* subnormal: r / 2^-24 */
    const uint32_t mant = (uint32_t)ldexp(r, 10 - (e - 1)) - 1024u;
    return (uint16_t)(sign | ((uint32_t)eb << 10) | mant);
}

/*
 * Alg. 1 with the residual held in binary16: each step reads e as a half, computes in fp32 exactly
 * as oracle_update_full_residual does, and stores e' = half(u - ΔW) (saturating, round to nearest
 * even).
 */
int oracle_update_full_residual_f16(oracle_tensor *w, const uint64_t *seeds_t, const float *fit_t,
                                    int32_t N, float sigma, float alpha, float gamma, uint16_t *e_state,
                                    uint64_t *stats)
{
    if (!tensor_ok(w) || !seeds_t || !fit_t || !e_state || N <= 0 || !(sigma > 0.0f))
        return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features;
    const float c = step_coeff(alpha, N, sigma);
    uint64_t changed = 0, gated = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : changed, gated)
    for (int32_t n = 0; n < w->out_features; ++n) {
        for (int64_t k = 0; k < K; k += 2) {
            const uint64_t e0 = (uint64_t)((int64_t)n * K + k);
            float g[2];
            aggregate_pair(seeds_t, fit_t, N, w->tensor_id, e0 >> 1, sigma, 0, g);
            for (int l = 0; l < 2; ++l) {
                int32_t wq = load_q(w, n, k + l);
                float u;
                int32_t raw;
                int32_t df = ef_step(c, g[l], gamma, oracle_f16_to_f32(e_state[e0 + l]), wq, w->qmin, w->qmax, &u, &raw);
                e_state[e0 + l] = oracle_f32_to_f16_sat(u - (float)df);
                if (df != 0) { store_q(w, n, k + l, wq + df); ++changed; }
                else if (raw != 0) ++gated;
            }
        }
    }
    if (stats) { stats[0] += changed; stats[1] += gated; }
    return ORACLE_OK;
}

/* g = Σ_i F_i δ_i per element (Eq. 5 without the 1/(Nσ) factor), for pins */
int oracle_aggregate(const oracle_tensor *w, const uint64_t *seeds, const float *fit, int32_t N,
                     float sigma, float *g_out, int32_t antithetic)
{
    if (!tensor_ok(w) || !seeds || !fit || !g_out || N <= 0) return ORACLE_ERR_INVALID_ARG;
    if (antithetic && (N & 1)) return ORACLE_ERR_INVALID_ARG;
    const int64_t K = w->in_features;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t n = 0; n < w->out_features; ++n)
        for (int64_t k = 0; k < K; k += 2) {
            float g[2];
            aggregate_pair(seeds, fit, N, w->tensor_id, (uint64_t)((int64_t)n * K + k) >> 1, sigma, antithetic, g);
            g_out[(int64_t)n * K + k] = g[0];
            g_out[(int64_t)n * K + k + 1] = g[1];
        }
    return ORACLE_OK;
}
