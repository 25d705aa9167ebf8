// Host-side declarations shared by the translation units of libqes (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace qes {

// One (seed, fitness) record as the kernels read it: 16 bytes, one scalar load.
struct Entry {
    uint32_t seed_lo, seed_hi;
    uint32_t fit_bits;   // update/replay: fitness bits. GEMM: 0 = base weights, 1 = +δ, 2 = -δ
    uint32_t pad;        // update/replay with antithetic pairs: fitness bits of the -δ member
};

// One tensor of a batched update launch: its blocks are [first_block, first_block + ceil(n_pairs/256)).
struct TensorDesc {
    void *qweight;
    uint32_t n_pairs;
    uint32_t first_block;
    int32_t qmin;
    uint32_t qspan;
    uint32_t tensor_id;
    uint32_t pad;
};

struct UpdateArgs {
    void *qweight;
    const Entry *entries;        // [steps][N], oldest generation first, current step last
    float *residual;             // replay: written; full-residual step: read and written
    unsigned long long *stats;   // update only, may be null
    uint32_t n_pairs;            // out*in/2
    int32_t steps;               // generations to run (hist_len for replay, hist_len+1 for update)
    int32_t N;                   // records per generation (members, or pairs when antithetic)
    float sigma, c, gamma;
    int32_t qmin;
    uint32_t qspan;              // qmax - qmin
    uint32_t tensor_id;
    uint32_t round_k0, round_k1; // stochastic-rounding baseline: key of the step's rounding stream
    const TensorDesc *descs;     // batched launch: per-tensor fields above come from here
    int32_t n_tensors;
};

struct GemmArgs {
    const void *qweight;
    const void *scales;          // fp16
    const Entry *entries;        // [N]: seed + perturb flag ([N/2] for the paired launch)
    const void *x;               // bf16 [N,T,in] (act_mode 0) or int8 [N,T,in] (act_mode 1)
    const float *x_scale;        // act_mode 1: [N,T]
    void *y;                     // bf16 [N,T,out]
    int32_t out_features, in_features, group_size;
    int32_t N, T;
    float sigma;
    int32_t qmin;
    uint32_t qspan;
    uint32_t tensor_id;
    // batched launch: the kernel argument carries N, T and these three; each tensor's own GemmArgs
    // (all fields above) sits in `batch`. Work is queued per XCD: a tensor with W work items
    // occupies ceil(W/8) consecutive slots of every XCD's queue, starting at its work_begin.
    const GemmArgs *batch;
    int32_t n_batch;
    uint32_t work_begin;         // per tensor: first slot; kernel argument: slots per XCD queue
};

hipError_t launch_noise_words(uint64_t seed, uint32_t tensor_id, uint64_t pair_begin, uint64_t n_pairs,
                              uint32_t *out4, hipStream_t s);
hipError_t launch_noise_gauss(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n,
                              float *out, hipStream_t s);
hipError_t launch_noise_delta(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n,
                              float sigma, int8_t *out, hipStream_t s);
hipError_t launch_noise_from_words(const uint32_t *words4, uint64_t n, float sigma, float *eps2, int8_t *delta2,
                                   hipStream_t s);
hipError_t launch_bench_noise(int mode, uint64_t n_threads, int iters, float sigma, uint32_t *sink,
                              hipStream_t s);
hipError_t launch_bench_mfma(int mode, uint32_t n_blocks, int iters, uint32_t *sink, hipStream_t s);
hipError_t launch_bench_copy(const void *src, void *dst, size_t n_bytes, hipStream_t s);

// bits: 4|8; rmode 0: Alg. 2 in place; 1: replay only, residual written; 2: Alg. 1 step on a stored residual
hipError_t launch_update(const UpdateArgs &a, int bits, int rmode, bool antithetic, hipStream_t s);
// Alg. 2 on several tensors of one width in one launch (a.descs, a.n_tensors; total_blocks = sum of their blocks)
hipError_t launch_update_batch(const UpdateArgs &a, int bits, bool antithetic, uint32_t total_blocks, hipStream_t s);

hipError_t launch_quantize_activations(const void *x_bf16, int8_t *xq, float *x_scale, int64_t rows,
                                       int32_t in_features, hipStream_t s);
// returns hipErrorInvalidValue when no kernel covers the request
// paired: a.entries holds one record per antithetic pair (fit_bits bit 0 / bit 1: even / odd member
// perturbed) and one workgroup evaluates both members from one draw; needs gemm_pairs_supported()
bool gemm_pairs_supported(int32_t T, bool batched);
hipError_t launch_gemm(const GemmArgs &a, int bits, int act_mode, bool paired, hipStream_t s);
// work items (tiles of 64 output rows x members, or x pairs) of one tensor
uint32_t gemm_work_items(int32_t out_features, int32_t N, bool paired);

}  // namespace qes
