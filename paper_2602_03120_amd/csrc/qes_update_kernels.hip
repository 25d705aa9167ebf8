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
#include <type_traits>

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
// A thread owns PPT pairs and regenerates the noise of MI members at a time: PPT*MI independent
// Philox/Box-Muller chains in flight per thread, while the sum of Eq. 5 still runs in member order.
// BATCH: one launch covers several tensors (same seeds, fitnesses and history: the whole model's
// update is one call); a block finds its tensor by bisection over the tensors' first blocks.
template <int BITS, int PPT, int MI, int RMODE, bool CLAMP, bool ANTI, bool BATCH>
__global__ __launch_bounds__(kBlock, 8) void update_kernel(const UpdateArgs args)
{
    using P = Pack<BITS>;
    constexpr int kBytes = PPT * P::kBytesPerPair;
    UpdateArgs a = args;
    uint32_t block = blockIdx.x;
    if (BATCH) {
        int lo = 0, hi = args.n_tensors - 1;   // wave-uniform: scalar loads
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (args.descs[mid].first_block <= block) lo = mid;
            else hi = mid - 1;
        }
        const TensorDesc td = args.descs[lo];
        a.qweight = td.qweight;
        a.n_pairs = td.n_pairs;
        a.qmin = td.qmin;
        a.qspan = td.qspan;
        a.tensor_id = td.tensor_id;
        block -= td.first_block;
    }
    // A wave that lies wholly past the tensor leaves. In the wave that straddles the end, the lanes
    // past it stay alive for the wavefront reduction of the counters: they redo the last thread's
    // work (in bounds), store nothing and count nothing. n_pairs is a multiple of PPT (host-checked).
    const uint32_t wave_first = (block * kBlock + (threadIdx.x & ~63u)) * PPT;
    if (wave_first >= a.n_pairs) return;
    uint32_t t = block * kBlock + threadIdx.x;
    const bool active = t * PPT < a.n_pairs;
    if (!active) t = a.n_pairs / PPT - 1u;
    const uint32_t pair0 = t * PPT;

    Raw<kBytes> raw;
    raw.load(a.qweight, (size_t)t * kBytes);
    int32_t wq[2 * PPT];
#pragma unroll
    for (int j = 0; j < PPT; ++j) P::unpack(raw.pair_bits(j, P::kBytesPerPair), wq[2 * j], wq[2 * j + 1]);

    float res[2 * PPT];
    if constexpr (RMODE == 2 && PPT % 2 == 0) {
        // 16-byte aligned: the residual is, and pair0 is a multiple of PPT
        const float4 *src = (const float4 *)(a.residual + (size_t)pair0 * 2);
#pragma unroll
        for (int q = 0; q < PPT / 2; ++q) {
            const float4 v = src[q];
            res[4 * q] = v.x;
            res[4 * q + 1] = v.y;
            res[4 * q + 2] = v.z;
            res[4 * q + 3] = v.w;
        }
    } else if constexpr (RMODE == 3 && PPT % 4 == 0) {
        typedef __attribute__((ext_vector_type(8))) _Float16 half8;
        const half8 *src = (const half8 *)((const _Float16 *)a.residual + (size_t)pair0 * 2);
#pragma unroll
        for (int q = 0; q < PPT / 4; ++q) {
            const half8 v = src[q];
#pragma unroll
            for (int j = 0; j < 8; ++j) res[8 * q + j] = (float)v[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 2 * PPT; ++j) {
            if (RMODE == 2) res[j] = a.residual[(size_t)pair0 * 2 + j];
            else if (RMODE == 3) res[j] = (float)((const _Float16 *)a.residual)[(size_t)pair0 * 2 + j];
            else res[j] = 0.0f;
        }
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
        // M members at a time: M x PPT independent chains, then the fmas in member order
        auto round = [&](auto m_tag, int32_t first) {
            constexpr int M = decltype(m_tag)::value;
            Entry en[M];                                  // wave-uniform: scalar loads
            float d[M][2 * PPT];
#pragma unroll
            for (int m = 0; m < M; ++m) en[m] = gen[first + m];
#pragma unroll
            for (int m = 0; m < M; ++m) draw(en[m], d[m]);
#pragma unroll
            for (int m = 0; m < M; ++m) accumulate(en[m], d[m]);
        };
        int32_t i = 0;
        for (; i + MI <= a.N; i += MI) round(std::integral_constant<int, MI>{}, i);
        // N % MI leftover members, still as wide as they allow
        if constexpr (MI >= 4) {
            if (i + 2 <= a.N) {
                round(std::integral_constant<int, 2>{}, i);
                i += 2;
            }
        }
        if constexpr (MI >= 2) {
            if (i < a.N) round(std::integral_constant<int, 1>{}, i);
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
                float r = __builtin_rintf(u);
                if (RMODE == 2 || RMODE == 3) {
                    // the stored residual is caller data: saturate like the conversion is defined to
                    // (NaN -> 0); elsewhere the host has bounded |u| below 2^30
                    r = __builtin_fminf(__builtin_fmaxf(r, -2147483648.0f), 2147483520.0f);
                    r = (u != u) ? 0.0f : r;
                }
                d = (int32_t)r;
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

    if (!active) {
        changed = 0;
        gated = 0;
    }
    if (active && (RMODE == 1 || RMODE == 2)) {
        float *out = a.residual + (size_t)pair0 * 2;
        if constexpr (PPT % 2 == 0) {
#pragma unroll
            for (int q = 0; q < PPT / 2; ++q)
                ((float4 *)out)[q] = make_float4(res[4 * q], res[4 * q + 1], res[4 * q + 2], res[4 * q + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < 2 * PPT; ++j) out[j] = res[j];
        }
    }
    if (active && RMODE == 3) {
        _Float16 *out = (_Float16 *)a.residual + (size_t)pair0 * 2;
        if constexpr (PPT % 4 == 0) {
            typedef __attribute__((ext_vector_type(8))) _Float16 half8;
#pragma unroll
            for (int q = 0; q < PPT / 4; ++q) {
                half8 v;
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = (_Float16)fminf(fmaxf(res[8 * q + j], -65504.0f), 65504.0f);
                ((half8 *)out)[q] = v;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2 * PPT; ++j) out[j] = (_Float16)fminf(fmaxf(res[j], -65504.0f), 65504.0f);
        }
    }
    if (RMODE != 1) {
        if (changed) {   // zero in the lanes past the end
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

// One pair per thread, four members at a time. Measured on the tensor shapes of every
// configuration against 2 x 2 and 4 x 1 (pairs x members) and against 5, 6 and 8 members at a time:
// four chains per thread at 8 waves per SIMD already reach the noise ceiling, and the shortest
// waves give the cheapest last round of a launch, so this split is never slower.
constexpr int kPairsPerThread = 1;
constexpr int kMembersAtATime = 4;

// One Alg. 1 step on a stored residual with a small population is the one launch on this path
// where memory traffic is comparable to the noise work (N draws per element against 5 to 9 bytes):
// there a thread owns four pairs (a dword of INT4 or two of INT8, 32 bytes of fp32 or 16 bytes of
// binary16 residual, moved with vector loads and stores) and regenerates one member's draws for
// all four at a time. Same arithmetic per element, same results.
constexpr int kWidePairsPerThread = 4;
constexpr int kWideMaxPopulation = 8;

template <int BITS, int RMODE>
hipError_t launch_wide_variant(const UpdateArgs &a, hipStream_t s)
{
    constexpr int P = kWidePairsPerThread;
    const uint64_t threads = a.n_pairs / P;
    const unsigned blocks = (unsigned)((threads + kBlock - 1) / kBlock);
    if (!(a.sigma <= 1.2f)) update_kernel<BITS, P, 1, RMODE, true, false, false><<<blocks, kBlock, 0, s>>>(a);
    else update_kernel<BITS, P, 1, RMODE, false, false, false><<<blocks, kBlock, 0, s>>>(a);
    return hipGetLastError();
}

template <int BITS, int RMODE>
hipError_t launch_variant(const UpdateArgs &a, bool antithetic, hipStream_t s)
{
    if constexpr (RMODE == 2 || RMODE == 3) {
        if (!antithetic && a.N <= kWideMaxPopulation && a.n_pairs % kWidePairsPerThread == 0)
            return launch_wide_variant<BITS, RMODE>(a, s);
    }
    const uint64_t threads = a.n_pairs / kPairsPerThread;
    const unsigned blocks = (unsigned)((threads + kBlock - 1) / kBlock);
    // |sigma*eps| <= 1.2 * 5.77 < 7: the 4-bit container clamp cannot fire and is compiled out
    const bool clamp = !(a.sigma <= 1.2f);
    constexpr int P = kPairsPerThread, M = kMembersAtATime;
    if (clamp) {
        if (antithetic) update_kernel<BITS, P, M, RMODE, true, true, false><<<blocks, kBlock, 0, s>>>(a);
        else update_kernel<BITS, P, M, RMODE, true, false, false><<<blocks, kBlock, 0, s>>>(a);
    } else {
        if (antithetic) update_kernel<BITS, P, M, RMODE, false, true, false><<<blocks, kBlock, 0, s>>>(a);
        else update_kernel<BITS, P, M, RMODE, false, false, false><<<blocks, kBlock, 0, s>>>(a);
    }
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_batch_variant(const UpdateArgs &a, bool antithetic, uint32_t total_blocks, hipStream_t s)
{
    static_assert(kPairsPerThread == 1, "the host lays out ceil(n_pairs / 256) blocks per tensor");
    const bool clamp = !(a.sigma <= 1.2f);
    constexpr int P = kPairsPerThread, M = kMembersAtATime;
    if (clamp) {
        if (antithetic) update_kernel<BITS, P, M, 0, true, true, true><<<total_blocks, kBlock, 0, s>>>(a);
        else update_kernel<BITS, P, M, 0, true, false, true><<<total_blocks, kBlock, 0, s>>>(a);
    } else {
        if (antithetic) update_kernel<BITS, P, M, 0, false, true, true><<<total_blocks, kBlock, 0, s>>>(a);
        else update_kernel<BITS, P, M, 0, false, false, true><<<total_blocks, kBlock, 0, s>>>(a);
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

hipError_t launch_update_batch(const UpdateArgs &a, int bits, bool antithetic, uint32_t total_blocks, hipStream_t s)
{
    if (total_blocks == 0) return hipSuccess;
    return bits == 4 ? launch_batch_variant<4>(a, antithetic, total_blocks, s)
                     : launch_batch_variant<8>(a, antithetic, total_blocks, s);
}

}  // namespace qes
