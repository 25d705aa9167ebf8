// Noise probes (bit-for-bit test access to the generator of docs/NOISE_SPEC.md) and the ceiling
// microbenchmarks the benchmark reports next to the kernels: Philox words and noise draws per
// second with no memory traffic, matrix instructions per second on register operands, and a plain
// streaming copy.
#include "qes_internal.hpp"
#include "qes_noise.hpp"

namespace qes {

namespace {

constexpr int kBlock = 256;

__global__ __launch_bounds__(kBlock) void noise_words_kernel(uint32_t k0, uint32_t k1, uint32_t tensor_id,
                                                              uint64_t pair_begin, uint64_t n_pairs,
                                                              uint4 *__restrict__ out)
{
    const uint64_t j = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j >= n_pairs) return;
    const uint64_t pair = pair_begin + j;
    const Words w = philox4x32_10((uint32_t)pair, (uint32_t)(pair >> 32), tensor_id, 0u, k0, k1);
    out[j] = make_uint4(w.w0, w.w1, w.w2, w.w3);
}

// MODE 0: Gaussian (float), MODE 1: delta (int8). One thread per pair touching the window.
template <int MODE>
__global__ __launch_bounds__(kBlock) void noise_elems_kernel(uint32_t k0, uint32_t k1, uint32_t tensor_id,
                                                             uint64_t elem_begin, uint64_t n_elems,
                                                             float sigma, void *__restrict__ out)
{
    const uint64_t first_pair = elem_begin >> 1;
    const uint64_t j = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t pair = first_pair + j;
    const uint64_t e0 = pair << 1;
    if (e0 >= elem_begin + n_elems) return;
    const Words w = philox4x32_10((uint32_t)pair, (uint32_t)(pair >> 32), tensor_id, 0u, k0, k1);
    float g0, g1;
    gauss_pair(w.w0, w.w1, g0, g1);
    const float g[2] = {g0, g1};
    const uint32_t wr[2] = {w.w2, w.w3};
#pragma unroll
    for (int l = 0; l < 2; ++l) {
        const uint64_t e = e0 + l;
        if (e < elem_begin || e >= elem_begin + n_elems) continue;
        if (MODE == 0) ((float *)out)[e - elem_begin] = g[l];
        else ((int8_t *)out)[e - elem_begin] = (int8_t)delta_of(g[l], wr[l], sigma);
    }
}

__global__ __launch_bounds__(kBlock) void noise_from_words_kernel(const uint4 *__restrict__ words, uint64_t n, float sigma,
                                                                  float2 *__restrict__ eps2, char2 *__restrict__ delta2)
{
    const uint64_t j = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j >= n) return;
    const uint4 w = words[j];
    float g0, g1;
    gauss_pair(w.x, w.y, g0, g1);
    if (eps2) eps2[j] = make_float2(g0, g1);
    if (delta2) delta2[j] = make_char2((signed char)delta_of(g0, w.z, sigma), (signed char)delta_of(g1, w.w, sigma));
}

// Noise ceiling: what the generator alone sustains, in the shape the tensor kernels run it in: four
// independent chains per thread (four members of one pair at a time, each with its own
// wave-uniform key), eight waves per SIMD, no memory traffic in the loop. MODE 0: Philox words only;
// MODE 1: full pair draws (Philox + Box-Muller + two stochastic roundings, δ kept in fp32).
constexpr int kChains = 4;

template <int MODE>
__global__ __launch_bounds__(kBlock, 8) void bench_noise_kernel(uint64_t n_threads, int iters, float sigma,
                                                                uint32_t *__restrict__ sink)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t >= n_threads) return;
    uint32_t acc = 0;
    float facc = 0.0f;
    const uint32_t pair = (uint32_t)t;
    for (int it = 0; it < iters; it += kChains) {
        uint32_t k0[kChains], k1[kChains];
#pragma unroll
        for (int m = 0; m < kChains; ++m) {
            k0[m] = 0x1234567u + (uint32_t)(it + m) * 0x9E3779B1u;   // wave-uniform, as a member's seed is
            k1[m] = 0x89ABCDEu ^ (uint32_t)(it + m);
        }
        if (MODE == 0) {
            Words w[kChains];
#pragma unroll
            for (int m = 0; m < kChains; ++m) w[m] = philox_tensor(pair, 7u, k0[m], k1[m]);
#pragma unroll
            for (int m = 0; m < kChains; ++m) acc ^= w[m].w0 ^ w[m].w1 ^ w[m].w2 ^ w[m].w3;
        } else {
            float d0[kChains], d1[kChains];
#pragma unroll
            for (int m = 0; m < kChains; ++m) delta_pair_f32<false>(k0[m], k1[m], 7u, pair, sigma, d0[m], d1[m]);
#pragma unroll
            for (int m = 0; m < kChains; ++m) facc += d0[m] * 16.0f + d1[m];
        }
    }
    sink[t] = acc + (uint32_t)(int32_t)facc;
}

// MFMA ceiling: eight independent accumulator tiles per wave, operands in registers, no memory.
// MODE 0: v_mfma_f32_16x16x32_bf16 (16384 flop per wave instruction); MODE 1: v_mfma_i32_16x16x64_i8
// (32768 op). Two waves per SIMD.
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(4))) float probe_f32x4;
typedef __attribute__((ext_vector_type(4))) int probe_i32x4;
constexpr int kMfmaTiles = 8;

template <int MODE>
__global__ __launch_bounds__(kBlock) void bench_mfma_kernel(int iters, uint32_t *__restrict__ sink)
{
    union {
        uint32_t u[4];
        probe_bf16x8 bf;
        probe_i32x4 i8;
    } a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a.u[i] = 0x3F803F80u ^ (threadIdx.x & 0x7Fu);   // finite bf16 pairs near 1 / arbitrary int8 quadruples
        b.u[i] = 0x3F003F00u ^ (uint32_t)i;
    }
    probe_f32x4 cf[kMfmaTiles];
    probe_i32x4 ci[kMfmaTiles];
#pragma unroll
    for (int t = 0; t < kMfmaTiles; ++t) {
        cf[t] = probe_f32x4{0, 0, 0, 0};
        ci[t] = probe_i32x4{0, 0, 0, 0};
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < kMfmaTiles; ++t) {
            if (MODE == 0) cf[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.bf, b.bf, cf[t], 0, 0, 0);
            else ci[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.i8, b.i8, ci[t], 0, 0, 0);
        }
    }
    uint32_t acc = 0;
#pragma unroll
    for (int t = 0; t < kMfmaTiles; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc ^= (MODE == 0) ? __float_as_uint(cf[t][j]) : (uint32_t)ci[t][j];
    sink[(size_t)blockIdx.x * kBlock + threadIdx.x] = acc;
}

// Plain streaming copy, four 16-byte loads in flight per thread before the four stores.
__global__ __launch_bounds__(kBlock) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                      size_t n16)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

inline unsigned blocks_for(uint64_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

}  // namespace

hipError_t launch_noise_words(uint64_t seed, uint32_t tensor_id, uint64_t pair_begin, uint64_t n_pairs,
                              uint32_t *out4, hipStream_t s)
{
    noise_words_kernel<<<blocks_for(n_pairs), kBlock, 0, s>>>((uint32_t)seed, (uint32_t)(seed >> 32), tensor_id,
                                                            pair_begin, n_pairs, (uint4 *)out4);
    return hipGetLastError();
}

hipError_t launch_noise_gauss(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n,
                              float *out, hipStream_t s)
{
    const uint64_t pairs = ((elem_begin + n + 1) >> 1) - (elem_begin >> 1);
    noise_elems_kernel<0><<<blocks_for(pairs), kBlock, 0, s>>>((uint32_t)seed, (uint32_t)(seed >> 32), tensor_id,
                                                             elem_begin, n, 0.0f, out);
    return hipGetLastError();
}

hipError_t launch_noise_delta(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n,
                              float sigma, int8_t *out, hipStream_t s)
{
    const uint64_t pairs = ((elem_begin + n + 1) >> 1) - (elem_begin >> 1);
    noise_elems_kernel<1><<<blocks_for(pairs), kBlock, 0, s>>>((uint32_t)seed, (uint32_t)(seed >> 32), tensor_id,
                                                             elem_begin, n, sigma, out);
    return hipGetLastError();
}

hipError_t launch_noise_from_words(const uint32_t *words4, uint64_t n, float sigma, float *eps2, int8_t *delta2,
                                   hipStream_t s)
{
    noise_from_words_kernel<<<blocks_for(n), kBlock, 0, s>>>((const uint4 *)words4, n, sigma, (float2 *)eps2,
                                                           (char2 *)delta2);
    return hipGetLastError();
}

hipError_t launch_bench_noise(int mode, uint64_t n_threads, int iters, float sigma, uint32_t *sink,
                              hipStream_t s)
{
    if (mode == 0)
        bench_noise_kernel<0><<<blocks_for(n_threads), kBlock, 0, s>>>(n_threads, iters, sigma, sink);
    else
        bench_noise_kernel<1><<<blocks_for(n_threads), kBlock, 0, s>>>(n_threads, iters, sigma, sink);
    return hipGetLastError();
}

hipError_t launch_bench_mfma(int mode, uint32_t n_blocks, int iters, uint32_t *sink, hipStream_t s)
{
    if (n_blocks == 0) return hipSuccess;
    if (mode == 0) bench_mfma_kernel<0><<<n_blocks, kBlock, 0, s>>>(iters, sink);
    else bench_mfma_kernel<1><<<n_blocks, kBlock, 0, s>>>(iters, sink);
    return hipGetLastError();
}

hipError_t launch_bench_copy(const void *src, void *dst, size_t n_bytes, hipStream_t s)
{
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + kBlock - 1) / kBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks == 0) return hipSuccess;
    copy_kernel<<<(unsigned)blocks, kBlock, 0, s>>>((const uint4 *)src, (uint4 *)dst, n16);
    return hipGetLastError();
}

}  // namespace qes
