// Seeded error-feedback update with stateless seed replay (paper §3.3 Alg. 2; §3.2 Eq. 5-8).
//
// One thread owns PPT consecutive pairs of K-adjacent elements (PPT bytes of packed INT4, or
// 2*PPT bytes of INT8) and walks the generations oldest -> newest, regenerating every member's
// perturbation from its seed. Nothing but the packed weights is read from or written to HBM:
// (seed, fitness) records are wave-uniform and come through the scalar cache. The kernels are
// bound by the vector ALU work of the noise generator, so the layout goal is only that memory
// never appears on the critical path: one coalesced load and (if anything changed) one coalesced
// store per thread.
//
// Arithmetic order is part of the definition (bit-exact integer results):
//   g = fma(F_i, δ_i, g) for i = 0..N-1;  u = fma(c, g, γ*e);  Δ = rne(u);  e = u - Δ_gated.
#include "qes_internal.hpp"
#include "qes_noise.hpp"

namespace qes {

namespace {

constexpr int kBlock = 256;

template <int BITS>
struct Pack;

template <>
struct Pack<4> {
    // one byte = one pair
    __device__ static __forceinline__ void unpack(uint32_t byte, int32_t &a, int32_t &b)
    {
        a = ((int32_t)(byte << 28)) >> 28;
        b = ((int32_t)(byte << 24)) >> 28;
    }
    __device__ static __forceinline__ uint32_t pack(int32_t a, int32_t b)
    {
        return ((uint32_t)a & 0xFu) | (((uint32_t)b & 0xFu) << 4);
    }
    static constexpr int kBytesPerPair = 1;
};

template <>
struct Pack<8> {
    // two bytes = one pair
    __device__ static __forceinline__ void unpack(uint32_t half, int32_t &a, int32_t &b)
    {
        a = ((int32_t)(half << 24)) >> 24;
        b = ((int32_t)(half << 16)) >> 24;
    }
    __device__ static __forceinline__ uint32_t pack(int32_t a, int32_t b)
    {
        return ((uint32_t)a & 0xFFu) | (((uint32_t)b & 0xFFu) << 8);
    }
    static constexpr int kBytesPerPair = 2;
};

// raw bytes of PPT pairs, as 32-bit words where possible
template <int BYTES>
struct Raw {
    static_assert(BYTES == 1 || BYTES == 2 || BYTES % 4 == 0, "unsupported width");
    static constexpr int kWords = BYTES >= 4 ? BYTES / 4 : 1;
    uint32_t w[kWords];

    __device__ __forceinline__ void load(const void *base, size_t byte_off)
    {
        const char *p = (const char *)base + byte_off;
        if (BYTES == 1) w[0] = *(const uint8_t *)p;
        else if (BYTES == 2) w[0] = *(const uint16_t *)p;
        else {
#pragma unroll
            for (int i = 0; i < kWords; ++i) w[i] = ((const uint32_t *)p)[i];
        }
    }
    __device__ __forceinline__ void store(void *base, size_t byte_off) const
    {
        char *p = (char *)base + byte_off;
        if (BYTES == 1) *(uint8_t *)p = (uint8_t)w[0];
        else if (BYTES == 2) *(uint16_t *)p = (uint16_t)w[0];
        else {
#pragma unroll
            for (int i = 0; i < kWords; ++i) ((uint32_t *)p)[i] = w[i];
        }
    }
    // the bits of pair j
    __device__ __forceinline__ uint32_t pair_bits(int j, int bytes_per_pair) const
    {
        const int bit = j * bytes_per_pair * 8;
        return (w[bit >> 5] >> (bit & 31)) & (bytes_per_pair == 1 ? 0xFFu : 0xFFFFu);
    }
    __device__ __forceinline__ void set_pair_bits(int j, int bytes_per_pair, uint32_t v)
    {
        const int bit = j * bytes_per_pair * 8;
        const uint32_t mask = (bytes_per_pair == 1 ? 0xFFu : 0xFFFFu) << (bit & 31);
        w[bit >> 5] = (w[bit >> 5] & ~mask) | (v << (bit & 31));
    }
};

// RMODE 0: Alg. 2 (replay + update in place). 1: replay only, residual written. 2: Alg. 1 step with a
// stored residual (read, advanced one generation, written back together with the weights). 3: the
// same with the residual stored as binary16 (decoded exactly, arithmetic in fp32, encoded with
// round-to-nearest-even after saturating at the largest finite half). 4: the stateless baseline of
// §5, W <- W + Q(c g) with stochastic rounding Q (no residual; rounding uniforms from the Philox
// stream keyed by the step's rounding seed, stream tag 1).
// A thread owns PPT pairs and regenerates the noise of MI members at a time; PPT*MI = 4 independent
// Philox/Box-Muller chains are in flight per thread whatever the split, and the sum of Eq. 5 still
// runs in member order. Small PPT makes waves short, which evens out the last round of a launch.
template <int BITS, int PPT, int MI, int RMODE, bool CLAMP, bool ANTI>
__global__ __launch_bounds__(kBlock, 8) void update_kernel(const UpdateArgs a)
{
    using P = Pack<BITS>;
    constexpr int kBytes = PPT * P::kBytesPerPair;
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t pair0 = t * PPT;
    if (pair0 >= a.n_pairs) return;   // n_pairs is a multiple of PPT (checked on the host)

    Raw<kBytes> raw;
    raw.load(a.qweight, (size_t)t * kBytes);
    int32_t wq[2 * PPT];
#pragma unroll
    for (int j = 0; j < PPT; ++j) P::unpack(raw.pair_bits(j, P::kBytesPerPair), wq[2 * j], wq[2 * j + 1]);

    float res[2 * PPT];
#pragma unroll
    for (int j = 0; j < 2 * PPT; ++j) {
        if (RMODE == 2) res[j] = a.residual[(size_t)pair0 * 2 + j];
        else if (RMODE == 3) res[j] = (float)((const _Float16 *)a.residual)[(size_t)pair0 * 2 + j];
        else res[j] = 0.0f;
    }

    uint32_t changed = 0, gated = 0;
    const Entry *__restrict__ ent = a.entries;
    for (int32_t tau = 0; tau < a.steps; ++tau) {
        float g[2 * PPT];
#pragma unroll
        for (int j = 0; j < 2 * PPT; ++j) g[j] = 0.0f;
        const Entry *__restrict__ gen = ent + (size_t)tau * a.N;
        // one member: its draws for this thread's pairs, added to g
        auto accumulate = [&](const Entry &en, const float (&d)[2 * PPT]) {
            const float fit = __uint_as_float(en.fit_bits);
            const float fit_mirror = __uint_as_float(en.pad);   // antithetic pairs: fitness of the -δ member
#pragma unroll
            for (int j = 0; j < 2 * PPT; ++j) {
                g[j] = __builtin_fmaf(fit, d[j], g[j]);
                // one draw serves members 2i (+δ) and 2i+1 (-δ), summed in member order
                if (ANTI) g[j] = __builtin_fmaf(fit_mirror, -d[j], g[j]);
            }
        };
        auto draw = [&](const Entry &en, float (&d)[2 * PPT]) {
#pragma unroll
            for (int j = 0; j < PPT; ++j)
                delta_pair_f32<CLAMP>(en.seed_lo, en.seed_hi, a.tensor_id, pair0 + j, a.sigma, d[2 * j], d[2 * j + 1]);
        };
        int32_t i = 0;
        for (; i + MI <= a.N; i += MI) {
            Entry en[MI];                                 // wave-uniform: scalar loads
            float d[MI][2 * PPT];
#pragma unroll
            for (int m = 0; m < MI; ++m) en[m] = gen[i + m];
#pragma unroll
            for (int m = 0; m < MI; ++m) draw(en[m], d[m]);
#pragma unroll
            for (int m = 0; m < MI; ++m) accumulate(en[m], d[m]);
        }
        for (; i < a.N; ++i) {                            // N % MI leftover members
            const Entry en = gen[i];
            float d[2 * PPT];
            draw(en, d);
            accumulate(en, d);
        }
        const bool last = (RMODE != 1) && (tau == a.steps - 1);
        uint32_t round_word[2 * PPT];
        if (RMODE == 4) {
#pragma unroll
            for (int j = 0; j < PPT; ++j) {
                const Words rw = philox4x32_10(pair0 + j, 0u, a.tensor_id, 1u, a.round_k0, a.round_k1);
                round_word[2 * j] = rw.w2;
                round_word[2 * j + 1] = rw.w3;
            }
        }
#pragma unroll
        for (int j = 0; j < 2 * PPT; ++j) {
            float u;
            int32_t d;
            if (RMODE == 4) {
                u = a.c * g[j];
                const float fl = __builtin_floorf(u);
                const float ub = (float)(round_word[j] >> 8) * 0x1p-24f;
                d = (int32_t)fl + ((ub < u - fl) ? 1 : 0);
            } else {
                u = __builtin_fmaf(a.c, g[j], a.gamma * res[j]);
                d = (int32_t)__builtin_rintf(u);
            }
            const int32_t nv = gate(wq[j], d, a.qmin, a.qspan);
            const int32_t df = nv - wq[j];
            res[j] = u - (float)df;
            if (last) {
                changed += (df != 0);
                gated += (df == 0 && d != 0);
                wq[j] = nv;
            }
        }
    }

    if (RMODE == 1 || RMODE == 2) {
        float *out = a.residual + (size_t)pair0 * 2;
#pragma unroll
        for (int j = 0; j < 2 * PPT; ++j) out[j] = res[j];
    }
    if (RMODE == 3) {
        _Float16 *out = (_Float16 *)a.residual + (size_t)pair0 * 2;
#pragma unroll
        for (int j = 0; j < 2 * PPT; ++j) out[j] = (_Float16)fminf(fmaxf(res[j], -65504.0f), 65504.0f);
    }
    if (RMODE != 1) {
        if (changed) {
#pragma unroll
            for (int j = 0; j < PPT; ++j) raw.set_pair_bits(j, P::kBytesPerPair, P::pack(wq[2 * j], wq[2 * j + 1]));
            raw.store(a.qweight, (size_t)t * kBytes);
        }
        if (a.stats) {
            // wavefront reduction, then one atomic per wave and counter
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                changed += __shfl_xor(changed, off);
                gated += __shfl_xor(gated, off);
            }
            if ((threadIdx.x & 63) == 0) {
                if (changed) atomicAdd(&a.stats[0], (unsigned long long)changed);
                if (gated) atomicAdd(&a.stats[1], (unsigned long long)gated);
            }
        }
    }
}

template <int BITS, int RMODE, bool CLAMP, bool ANTI>
void launch_ppt(const UpdateArgs &a, int ppt, unsigned blocks, hipStream_t s)
{
    switch (ppt) {
    case 4: update_kernel<BITS, 4, 1, RMODE, CLAMP, ANTI><<<blocks, kBlock, 0, s>>>(a); break;
    case 2: update_kernel<BITS, 2, 2, RMODE, CLAMP, ANTI><<<blocks, kBlock, 0, s>>>(a); break;
    default: update_kernel<BITS, 1, 4, RMODE, CLAMP, ANTI><<<blocks, kBlock, 0, s>>>(a); break;
    }
}

// Relative duration of a launch of `waves` waves whose work is proportional to ppt, on 1024 SIMDs
// holding 8 waves each: whole rounds run at full rate; the waves left over run at the rate a SIMD
// reaches with that few waves (measured with the noise loop: 1 wave 49 %, 2 waves 73 %, 4 waves
// 93 % of the 8-wave rate).
double launch_cost(uint64_t n_pairs, int ppt)
{
    const double x = (double)((n_pairs / ppt + 63) / 64) / (1024.0 * 8.0);
    const double full = (double)(uint64_t)x;
    const double f = x - full;
    double tail = 0.0;
    if (f > 0.0) {
        const double pts[5][2] = {{0.0, 0.255}, {0.125, 0.255}, {0.25, 0.34}, {0.5, 0.54}, {1.0, 1.0}};
        for (int k = 0; k < 4; ++k)
            if (f >= pts[k][0] && f <= pts[k + 1][0])
                tail = pts[k][1] + (pts[k + 1][1] - pts[k][1]) * (f - pts[k][0]) / (pts[k + 1][0] - pts[k][0]);
    }
    return (full + tail) * ppt;
}

template <int BITS, int RMODE>
hipError_t launch_variant(const UpdateArgs &a, bool antithetic, hipStream_t s)
{
    // pairs per thread: the split with the shortest predicted launch (ties go to the wider thread)
    int ppt = 1;
    double best = launch_cost(a.n_pairs, 1);
    for (int cand = 2; cand <= 4; cand *= 2) {
        if (a.n_pairs % cand) break;
        const double c = launch_cost(a.n_pairs, cand);
        if (c <= best) { best = c; ppt = cand; }
    }
    const uint64_t threads = a.n_pairs / ppt;
    const unsigned blocks = (unsigned)((threads + kBlock - 1) / kBlock);
    // |sigma*eps| <= 1.2 * 5.77 < 7: the 4-bit container clamp cannot fire and is compiled out
    const bool clamp = !(a.sigma <= 1.2f);
    if (clamp) {
        if (antithetic) launch_ppt<BITS, RMODE, true, true>(a, ppt, blocks, s);
        else launch_ppt<BITS, RMODE, true, false>(a, ppt, blocks, s);
    } else {
        if (antithetic) launch_ppt<BITS, RMODE, false, true>(a, ppt, blocks, s);
        else launch_ppt<BITS, RMODE, false, false>(a, ppt, blocks, s);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_update(const UpdateArgs &a, int bits, int rmode, bool antithetic, hipStream_t s)
{
    if (a.n_pairs == 0) return hipSuccess;
    if (bits == 4) {
        switch (rmode) {
        case 0: return launch_variant<4, 0>(a, antithetic, s);
        case 1: return launch_variant<4, 1>(a, antithetic, s);
        case 2: return launch_variant<4, 2>(a, antithetic, s);
        case 3: return launch_variant<4, 3>(a, antithetic, s);
        default: return launch_variant<4, 4>(a, antithetic, s);
        }
    }
    switch (rmode) {
    case 0: return launch_variant<8, 0>(a, antithetic, s);
    case 1: return launch_variant<8, 1>(a, antithetic, s);
    case 2: return launch_variant<8, 2>(a, antithetic, s);
    case 3: return launch_variant<8, 3>(a, antithetic, s);
    default: return launch_variant<8, 4>(a, antithetic, s);
    }
}

}  // namespace qes
