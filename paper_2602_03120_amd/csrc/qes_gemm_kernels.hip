// Population-batched perturbed quantised GEMM (paper Alg. 1: "reconstruct δ_i", "W' = Gate(W_t+δ_i)",
// inference; §3.2 Eq. 3-4; App. A.1 formats).
//
//   Y[i,t,n] = Σ_g s[n,g] · Σ_{k in g} X[i,t,k] · W'_i[n,k],   W'_i = Gate(W + δ_i)
//
// Work decomposition. The cost is the regeneration of δ (about a hundred vector-ALU issue slots
// per weight element and member) against 2·T MFMA flops, so every (member, n, k) draw is generated
// exactly once: a workgroup owns one member and an n-tile of 16·kWaves output rows and ALL of that
// member's tokens (up to TM per pass), and walks K. Each wave owns 16 output rows; per 32-wide
// k-substep a lane regenerates the 8 K-consecutive elements of its MFMA B fragment in registers
// (4 Philox calls), gates them against the base integers and hands them to the matrix core as
// exact small integers (bf16 or int8). The activation tile is staged once per 128-k stage through
// LDS and shared by all waves. Group scales multiply fp32 partial sums at group boundaries, so
// the integer weights are never rounded.
//
// MFMA shapes (gfx950): v_mfma_f32_16x16x32_bf16 and v_mfma_i32_16x16x64_i8. Operand layout for a
// 64-lane wave: A lane l holds row l%16, k-chunk l/16; B lane l holds column l%16, k-chunk l/16;
// C lane l holds column l%16, rows 4·(l/16)..+3.
#include "qes_internal.hpp"
#include "qes_noise.hpp"

namespace qes {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kTileN = 16 * kWaves;
constexpr int kStageK = 128;   // k extent staged through LDS per barrier pair

union Frag {
    uint32_t u[4];
    bf16x8 bf;
    i32x4 i8;
    uint4 v;
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}

// The 8 gated integers W'[n, k..k+8) of one lane: 4 pairs starting at pair index `pair`.
template <int BITS>
__device__ __forceinline__ void perturbed8(const void *__restrict__ qw, size_t elem, bool perturb,
                                           uint32_t k0, uint32_t k1, uint32_t tensor_id, float sigma,
                                           int32_t qmin, uint32_t qspan, int32_t w[8])
{
    if (BITS == 4) {
        const uint32_t word = *(const uint32_t *)((const char *)qw + (elem >> 1));
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = ((int32_t)(word << (28 - 4 * j))) >> 28;
    } else {
        const uint2 words = *(const uint2 *)((const char *)qw + elem);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            w[j] = ((int32_t)(words.x << (24 - 8 * j))) >> 24;
            w[4 + j] = ((int32_t)(words.y << (24 - 8 * j))) >> 24;
        }
    }
    if (perturb) {
        const uint32_t pair = (uint32_t)(elem >> 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int32_t d0, d1;
            delta_pair(k0, k1, tensor_id, pair + j, sigma, d0, d1);
            w[2 * j] = gate(w[2 * j], d0, qmin, qspan);
            w[2 * j + 1] = gate(w[2 * j + 1], d1, qmin, qspan);
        }
    }
}

// exact bf16 images of 8 small integers, packed for the MFMA B operand
__device__ __forceinline__ void to_bf16_frag(const int32_t w[8], Frag &f)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t lo = __float_as_uint((float)w[2 * j]);
        const uint32_t hi = __float_as_uint((float)w[2 * j + 1]);
        f.u[j] = (lo >> 16) | (hi & 0xFFFF0000u);
    }
}

__device__ __forceinline__ uint32_t pack_i8x4(const int32_t *w)
{
    return ((uint32_t)w[0] & 0xFFu) | (((uint32_t)w[1] & 0xFFu) << 8) | (((uint32_t)w[2] & 0xFFu) << 16) |
           ((uint32_t)w[3] << 24);
}

// XCD-aware block -> (member, n-tile): consecutive work items (same member, neighbouring tiles)
// land on the same XCD (blocks are dealt round-robin over 8 XCDs), so a member's activations stay
// in one L2.
__device__ __forceinline__ bool block_to_work(uint32_t n_tiles, uint32_t n_members, uint32_t &member, uint32_t &tile)
{
    const uint32_t total = n_tiles * n_members;
    const uint32_t per_xcd = (total + 7u) / 8u;
    const uint32_t idx = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || idx >= total) return false;
    member = idx / n_tiles;
    tile = idx - member * n_tiles;
    return true;
}

// ------------------------------------------------------------------------------------------------
// bf16 activations (act_mode 0), INT4 or INT8 weights.
// TM: tokens held in accumulators per pass (multiple of 16).
template <int BITS, int TM>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(const GemmArgs a)
{
    constexpr int kRowBytes = kStageK * 2 + 16;             // padded LDS row: conflict-free b128 reads
    constexpr int kMT = TM / 16;
    __shared__ __attribute__((aligned(16))) char lds[TM * kRowBytes];

    uint32_t member, tile;
    const uint32_t n_tiles = (a.out_features + kTileN - 1) / kTileN;
    if (!block_to_work(n_tiles, (uint32_t)a.N, member, tile)) return;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ln = lane & 15;        // column of B / C within the wave's 16 rows
    const int kc = lane >> 4;        // k-chunk 0..3
    const int n = tile * kTileN + wave * 16 + ln;
    const int n_ld = n < a.out_features ? n : a.out_features - 1;   // clamp loads, skip stores

    const Entry en = a.entries[member];
    const bool perturb = (en.fit_bits != 0u) && (a.sigma != 0.0f);
    const int gs = a.group_size > 0 ? a.group_size : a.in_features;
    const int groups_per_row = a.in_features / gs;
    const uint16_t *__restrict__ scales = (const uint16_t *)a.scales;
    const uint16_t *__restrict__ xg = (const uint16_t *)a.x + (size_t)member * a.T * a.in_features;
    uint16_t *__restrict__ yg = (uint16_t *)a.y + (size_t)member * a.T * a.out_features;

    for (int t0 = 0; t0 < a.T; t0 += TM) {
        f32x4 acc[kMT], part[kMT];
#pragma unroll
        for (int m = 0; m < kMT; ++m) {
            acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
            part[m] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (int ks = 0; ks < a.in_features; ks += kStageK) {
            // ---- stage the activation tile X[member, t0..t0+TM, ks..ks+128) into LDS
            __syncthreads();
            for (int c = threadIdx.x; c < TM * 16; c += kThreads) {
                const int row = c >> 4, ch = c & 15;
                const int t = t0 + row, k = ks + ch * 8;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (t < a.T && k < a.in_features) v = *(const uint4 *)(xg + (size_t)t * a.in_features + k);
                *(uint4 *)(lds + row * kRowBytes + ch * 16) = v;
            }
            __syncthreads();
            const int nsub = (a.in_features - ks) >= kStageK ? 4 : (a.in_features - ks) / 32;
            for (int sub = 0; sub < nsub; ++sub) {
                const int k = ks + sub * 32 + kc * 8;
                int32_t w[8];
                perturbed8<BITS>(a.qweight, (size_t)n_ld * a.in_features + k, perturb, en.seed_lo, en.seed_hi,
                                 a.tensor_id, a.sigma, a.qmin, a.qspan, w);
                Frag b;
                to_bf16_frag(w, b);
#pragma unroll
                for (int m = 0; m < kMT; ++m) {
                    Frag af;
                    af.v = *(const uint4 *)(lds + (m * 16 + ln) * kRowBytes + (sub * 32 + kc * 8) * 2);
                    part[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af.bf, b.bf, part[m], 0, 0, 0);
                }
                const int k_end = ks + sub * 32 + 32;
                if (k_end % gs == 0) {   // group boundary: fold the scaled partial sums
                    const float s = f16_bits_to_f32(scales[(size_t)n_ld * groups_per_row + (k_end / gs - 1)]);
#pragma unroll
                    for (int m = 0; m < kMT; ++m) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[m][j] = __builtin_fmaf(s, part[m][j], acc[m][j]);
                        part[m] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
        if (n < a.out_features) {
#pragma unroll
            for (int m = 0; m < kMT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = t0 + m * 16 + kc * 4 + j;
                    if (t < a.T) yg[(size_t)t * a.out_features + n] = f32_to_bf16_rne(acc[m][j]);
                }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// W8A8 (act_mode 1): int8 activations quantised per token by quantize_kernel, int8 MFMA, exact
// int32 accumulation, Y = bf16(((float)acc · a[t]) · s[n]).
template <int TM>
__global__ __launch_bounds__(kThreads) void gemm_i8_kernel(const GemmArgs a)
{
    constexpr int kRowBytes = kStageK + 16;
    constexpr int kMT = TM / 16;
    __shared__ __attribute__((aligned(16))) char lds[TM * kRowBytes];

    uint32_t member, tile;
    const uint32_t n_tiles = (a.out_features + kTileN - 1) / kTileN;
    if (!block_to_work(n_tiles, (uint32_t)a.N, member, tile)) return;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ln = lane & 15;
    const int kc = lane >> 4;
    const int n = tile * kTileN + wave * 16 + ln;
    const int n_ld = n < a.out_features ? n : a.out_features - 1;

    const Entry en = a.entries[member];
    const bool perturb = (en.fit_bits != 0u) && (a.sigma != 0.0f);
    const int8_t *__restrict__ xg = (const int8_t *)a.x + (size_t)member * a.T * a.in_features;
    const float *__restrict__ xs = a.x_scale + (size_t)member * a.T;
    uint16_t *__restrict__ yg = (uint16_t *)a.y + (size_t)member * a.T * a.out_features;
    const float s_n = f16_bits_to_f32(((const uint16_t *)a.scales)[n_ld]);

    for (int t0 = 0; t0 < a.T; t0 += TM) {
        i32x4 acc[kMT];
#pragma unroll
        for (int m = 0; m < kMT; ++m) acc[m] = i32x4{0, 0, 0, 0};
        for (int ks = 0; ks < a.in_features; ks += kStageK) {
            __syncthreads();
            for (int c = threadIdx.x; c < TM * 8; c += kThreads) {
                const int row = c >> 3, ch = c & 7;
                const int t = t0 + row, k = ks + ch * 16;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (t < a.T && k < a.in_features) v = *(const uint4 *)(xg + (size_t)t * a.in_features + k);
                *(uint4 *)(lds + row * kRowBytes + ch * 16) = v;
            }
            __syncthreads();
            // 64-wide k-substeps; a 32-wide tail (in_features % 64 == 32) runs with zeroed upper halves
            const int kleft = a.in_features - ks;
            const int nsub = kleft >= kStageK ? 2 : (kleft + 63) / 64;
            for (int sub = 0; sub < nsub; ++sub) {
                const int k = ks + sub * 64 + kc * 16;
                // in_features % 32 == 0 and k % 16 == 0: the 16-chunk is wholly inside or wholly outside
                Frag b;
                b.v = make_uint4(0, 0, 0, 0);
                if (k < a.in_features) {
                    int32_t w[16];
                    perturbed8<8>(a.qweight, (size_t)n_ld * a.in_features + k, perturb, en.seed_lo, en.seed_hi,
                                  a.tensor_id, a.sigma, a.qmin, a.qspan, w);
                    perturbed8<8>(a.qweight, (size_t)n_ld * a.in_features + k + 8, perturb, en.seed_lo, en.seed_hi,
                                  a.tensor_id, a.sigma, a.qmin, a.qspan, w + 8);
                    b.u[0] = pack_i8x4(w);
                    b.u[1] = pack_i8x4(w + 4);
                    b.u[2] = pack_i8x4(w + 8);
                    b.u[3] = pack_i8x4(w + 12);
                }
#pragma unroll
                for (int m = 0; m < kMT; ++m) {
                    Frag af;
                    af.v = *(const uint4 *)(lds + (m * 16 + ln) * kRowBytes + sub * 64 + kc * 16);
                    acc[m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af.i8, b.i8, acc[m], 0, 0, 0);
                }
            }
        }
        if (n < a.out_features) {
#pragma unroll
            for (int m = 0; m < kMT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = t0 + m * 16 + kc * 4 + j;
                    if (t < a.T) {
                        const float v = ((float)acc[m][j] * xs[t]) * s_n;
                        yg[(size_t)t * a.out_features + n] = f32_to_bf16_rne(v);
                    }
                }
        }
    }
}

// Per-token symmetric int8 quantisation of bf16 activations: a = max|x|/127 (1 if 0),
// xq = clamp(rne(x / a), -127, 127) with IEEE fp32 division. One wave per token row.
__global__ __launch_bounds__(256) void quantize_kernel(const uint16_t *__restrict__ x, int8_t *__restrict__ xq,
                                                       float *__restrict__ x_scale, int64_t rows, int32_t in_features)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    const uint16_t *xr = x + row * in_features;
    float amax = 0.0f;
    for (int k = lane; k < in_features; k += 64)
        amax = fmaxf(amax, fabsf(__uint_as_float((uint32_t)xr[k] << 16)));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    float sc = amax / 127.0f;
    if (sc == 0.0f) sc = 1.0f;
    if (lane == 0) x_scale[row] = sc;
    for (int k = lane; k < in_features; k += 64) {
        float v = __builtin_rintf(__uint_as_float((uint32_t)xr[k] << 16) / sc);
        v = fminf(fmaxf(v, -127.0f), 127.0f);
        xq[row * in_features + k] = (int8_t)(int32_t)v;
    }
}

template <int BITS>
hipError_t launch_bf16(const GemmArgs &a, unsigned blocks, hipStream_t s)
{
    if (a.T <= 16) gemm_bf16_kernel<BITS, 16><<<blocks, kThreads, 0, s>>>(a);
    else if (a.T <= 32) gemm_bf16_kernel<BITS, 32><<<blocks, kThreads, 0, s>>>(a);
    else if (a.T <= 64) gemm_bf16_kernel<BITS, 64><<<blocks, kThreads, 0, s>>>(a);
    else if (a.T <= 128) gemm_bf16_kernel<BITS, 128><<<blocks, kThreads, 0, s>>>(a);
    else gemm_bf16_kernel<BITS, 256><<<blocks, kThreads, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize_activations(const void *x_bf16, int8_t *xq, float *x_scale, int64_t rows,
                                       int32_t in_features, hipStream_t s)
{
    if (rows == 0) return hipSuccess;
    quantize_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>((const uint16_t *)x_bf16, xq, x_scale, rows,
                                                              in_features);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs &a, int bits, int act_mode, hipStream_t s)
{
    const uint32_t n_tiles = (a.out_features + kTileN - 1) / kTileN;
    const uint32_t total = n_tiles * (uint32_t)a.N;
    const unsigned blocks = ((total + 7u) / 8u) * 8u;
    if (act_mode == 1) {
        if (a.T <= 64) gemm_i8_kernel<64><<<blocks, kThreads, 0, s>>>(a);
        else if (a.T <= 128) gemm_i8_kernel<128><<<blocks, kThreads, 0, s>>>(a);
        else if (a.T <= 256) gemm_i8_kernel<256><<<blocks, kThreads, 0, s>>>(a);
        else gemm_i8_kernel<512><<<blocks, kThreads, 0, s>>>(a);
        return hipGetLastError();
    }
    return bits == 4 ? launch_bf16<4>(a, blocks, s) : launch_bf16<8>(a, blocks, s);
}

}  // namespace qes
