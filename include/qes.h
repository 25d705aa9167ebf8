/*
 * libqes: the data-parallel hot path of Quantized Evolution Strategies (QES) on one MI355X.
 *
 * C ABI. Plain pointers and sizes only; every pointer is marked HOST or DEVICE. The library never
 * takes ownership of caller memory. All device work is enqueued on the caller's stream
 * (`stream` is a hipStream_t passed as void*; NULL is the default stream) and the calls return
 * without waiting for it. Small HOST arrays (seeds, fitnesses) are copied before the call
 * returns, so the caller may reuse them immediately.
 *
 * Every entry point returns QES_OK (0) or a negative qes_status; nothing throws. Every check
 * that can refuse a call (arguments, limits, workspace) is made before any device work is enqueued:
 * a call that returns QES_ERR_INVALID_ARG, QES_ERR_UNSUPPORTED, QES_ERR_WORKSPACE or
 * QES_ERR_TOO_LARGE has touched no device memory. QES_ERR_HIP reports a failing runtime call and
 * may leave earlier launches of the same call on the stream.
 *
 * Device memory the library owns. Entry points that take HOST arrays of seeds and fitnesses stage
 * them through a ring of 8 slot pairs (pinned host + device, about 4.6 MB each: room for
 * QES_MAX_HISTORY + 1 generations of QES_MAX_POPULATION records plus QES_MAX_BATCH descriptors).
 * The ring is allocated by the first such call on a device (hipHostMalloc / hipMalloc, once) and
 * kept until the process ends; no later call allocates or frees. A slot is reused once an event
 * recorded behind its last consumer has completed, so with more than 8 calls outstanding the host
 * waits for the oldest (not while holding the library's lock: callers on other streams go on).
 * Because of the first-call allocation and the copy from the pinned slot, these entry points are
 * not for use under stream capture; qes_update_noalloc is.
 *
 * Passages of the paper each operation implements are cited at its declaration:
 *   §3.2 Eq. 3  stochastically rounded integer perturbation δ
 *   §3.2 Eq. 4  boundary gate (out-of-range perturbations are masked, not saturated)
 *   §3.2 Eq. 5  discrete gradient estimate ĝ = 1/(Nσ) Σ_i F_i δ_i
 *   §3.2 Eq. 6-8, Alg. 1  accumulated error feedback
 *   §3.3, Alg. 2  stateless seed replay
 *   App. A.1  weight formats, 4-bit δ container
 * The noise generator (Philox4x32-10 -> Box-Muller -> stochastic rounding) is specified operation
 * by operation in docs/NOISE_SPEC.md.
 */
#ifndef QES_H
#define QES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QES_OK = 0,
    QES_ERR_INVALID_ARG = -1, /* null pointer, bad size, non-finite fitness, sigma out of range ... */
    QES_ERR_UNSUPPORTED = -2, /* a legal request this build has no kernel for (stated per call)   */
    QES_ERR_HIP = -3,         /* a HIP runtime call failed; qes_last_hip_error() has its code      */
    QES_ERR_WORKSPACE = -4,   /* workspace missing or smaller than qes_gemm_workspace_bytes()      */
    QES_ERR_TOO_LARGE = -5    /* qes_update_noalloc: more records than its fixed scratch holds     */
} qes_status;

/* Limits of the small HOST arrays. */
#define QES_MAX_POPULATION 1024 /* N */
#define QES_MAX_HISTORY 256     /* hist_len */
#define QES_MAX_BATCH 4096      /* tensors per qes_update_batch / qes_perturbed_qgemm_batch call */
#define QES_NOALLOC_MAX_RECORDS 16384 /* (hist_len + 1) * N accepted by qes_update_noalloc */

/*
 * One quantised linear weight (App. A.1; INT4 group-scaled and INT8 per-output-channel formats).
 *
 *   qweight  DEVICE. Logical [out_features, in_features], row-major, in_features contiguous.
 *            bits=4: two elements per byte; element 2b in the low nibble of byte b, element 2b+1 in
 *            the high nibble; each nibble a 4-bit two's-complement integer.
 *            bits=8: int8.
 *            Must be 16-byte aligned. Updated IN PLACE by qes_update; read-only elsewhere.
 *   scales   DEVICE, IEEE binary16. group_size>0: [out_features, in_features/group_size];
 *            group_size==0: [out_features]. Read by qes_perturbed_qgemm only (may be NULL for
 *            qes_update / qes_replay_residual: scales never enter the update).
 *   qmin,qmax  the codebook range used by the gate: qmin <= value <= qmax.
 *            bits=4: within [-8,7]; bits=8: within [-128,127].
 *   tensor_id  caller-assigned, distinct per tensor; enters the Philox counter so that two
 *            tensors never share noise.
 * in_features must be even. out_features*in_features must not exceed 2^33 - 4096 (pair and thread
 * indices are kept in 32 bits inside the tensor kernels); larger tensors are QES_ERR_UNSUPPORTED.
 */
typedef struct {
    void *qweight;
    const void *scales;
    int32_t out_features, in_features;
    int32_t bits;       /* 4 or 8 */
    int32_t group_size; /* bits=4: multiple of 32 dividing in_features; 0 = one scale per row */
    int32_t qmin, qmax;
    uint32_t tensor_id;
} qes_tensor;

/* ---- noise probes (docs/NOISE_SPEC.md; §3.2 Eq. 3). For tests and for callers that want δ. ---- */

/*
 * Raw Philox4x32-10 words of pairs [pair_begin, pair_begin+n_pairs): out4[j][0..3] for pair
 * pair_begin+j, key = seed, counter = (pair lo, pair hi, tensor_id, 0).
 * out4: DEVICE uint32 [n_pairs][4]. n_pairs == 0 is a no-op.
 */
int qes_noise_words(uint64_t seed, uint32_t tensor_id, uint64_t pair_begin, uint64_t n_pairs,
                    uint32_t *out4, void *stream);

/*
 * The standard Gaussians ε of elements [elem_begin, elem_begin+n_elems) (element e uses pair e>>1,
 * lane e&1). out: DEVICE float32 [n_elems].
 */
int qes_noise_gauss(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems,
                    float *out, void *stream);

/*
 * The integer perturbations δ (Eq. 3, clamped to the 4-bit container [-8,7]) of elements
 * [elem_begin, elem_begin+n_elems). sigma >= 0 and finite. out: DEVICE int8 [n_elems].
 */
int qes_noise_delta(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems,
                    float sigma, int8_t *out, void *stream);

/*
 * N3-N6 of docs/NOISE_SPEC.md applied to caller-supplied Philox words instead of generated ones:
 * for each of n word quadruples, the two Gaussians (eps2, DEVICE float32 [n][2], may be NULL) and
 * the two perturbations (delta2, DEVICE int8 [n][2], may be NULL). Lets a test sweep the radius
 * and angle inputs exhaustively. words4: DEVICE uint32 [n][4], 16-byte aligned.
 */
int qes_noise_from_words(const uint32_t *words4, uint64_t n, float sigma, float *eps2, int8_t *delta2,
                         void *stream);

/* ---- population evaluation (Alg. 1, steps "reconstruct δ_i", "W' = Gate(W_t+δ_i)", inference) ---- */

/*
 * Y[i,t,n] = Σ_g s[n,g] · Σ_{k in g} X[i,t,k] · W'_i[n,k] for every member i < N, where
 * W'_i = Gate(W + δ_i) (Eq. 3, Eq. 4) is regenerated from seeds[i] inside the kernel and never
 * stored.
 *
 *   seeds         HOST uint64 [N]
 *   perturb_mask  HOST uint8 [N] or NULL (= all ones); 0 evaluates that member on the base weights
 *   sigma         >= 0, finite; 0 evaluates every member on the base weights
 *   x             DEVICE bfloat16 [N, T, in_features], 16-byte aligned
 *   y             DEVICE bfloat16 [N, T, out_features] (written)
 *   act_mode      0: bfloat16 activations; integer weights enter the MFMA as exact bfloat16 values
 *                    and the scale is applied to fp32 partial sums at group boundaries.
 *                 1: W8A8 (bits=8, group_size=0 only): symmetric dynamic per-token int8
 *                    activations (a[t] = max|x|/127, 1 if that is 0), int8 MFMA with exact int32
 *                    accumulation, Y = bf16(((float)acc·a[t])·s[n]).
 *   workspace     DEVICE scratch of at least qes_gemm_workspace_bytes() bytes, 16-byte aligned
 *                 (may be NULL when that is 0). Contents are overwritten.
 *
 * Requires in_features % 32 == 0, 1 <= N <= QES_MAX_POPULATION, T >= 1.
 * QES_ERR_UNSUPPORTED: in_features not a multiple of 32, or group_size not a multiple of 32.
 */
int qes_perturbed_qgemm(const qes_tensor *w, const uint64_t *seeds, const uint8_t *perturb_mask,
                        int32_t N, float sigma, const void *x, int32_t T, void *y, int32_t act_mode,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same with antithetic perturbation pairs (App. A.1: "antithetic perturbation pairs"): N is
 * even, pair_seeds is HOST uint64 [N/2], members 2j and 2j+1 share pair_seeds[j], member 2j is
 * evaluated on Gate(W + δ_j) and member 2j+1 on Gate(W − δ_j). x, y and perturb_mask stay per
 * member. Up to 128 tokens per member (256 in the batched call) one workgroup evaluates both
 * members of a pair from a single draw (half the noise work); longer token counts regenerate δ_j
 * per member. Same results either way.
 */
int qes_perturbed_qgemm_antithetic(const qes_tensor *w, const uint64_t *pair_seeds, const uint8_t *perturb_mask,
                                   int32_t N, float sigma, const void *x, int32_t T, void *y, int32_t act_mode,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of DEVICE workspace qes_perturbed_qgemm needs for these arguments (0 for act_mode 0). */
size_t qes_gemm_workspace_bytes(const qes_tensor *w, int32_t N, int32_t T, int32_t act_mode);

/*
 * qes_perturbed_qgemm for every tensor of a list (the linears of a layer: same members, same token
 * count, each with its own activations and outputs) in one launch per weight width: the workgroups
 * of all tensors fill the chip together instead of each launch ending in a partly filled round.
 * Results are bit-identical to n_tensors single calls.
 *
 *   tensors   HOST array [n_tensors] of descriptors, 1 <= n_tensors <= QES_MAX_BATCH
 *   x, y      HOST arrays [n_tensors] of DEVICE pointers: x[i] bfloat16 [N, T, in_features of tensor i],
 *             y[i] bfloat16 [N, T, out_features of tensor i]. Tensors may share an x (q/k/v, gate/up);
 *             with act_mode 1 a shared x is quantised once.
 *   workspace at least qes_gemm_batch_workspace_bytes() bytes (0 for act_mode 0)
 * Other arguments, requirements and errors as for qes_perturbed_qgemm(_antithetic).
 */
int qes_perturbed_qgemm_batch(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *seeds,
                              const uint8_t *perturb_mask, int32_t N, float sigma, const void *const *x, int32_t T,
                              void *const *y, int32_t act_mode, void *workspace, size_t workspace_bytes, void *stream);

int qes_perturbed_qgemm_batch_antithetic(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *pair_seeds,
                                         const uint8_t *perturb_mask, int32_t N, float sigma, const void *const *x,
                                         int32_t T, void *const *y, int32_t act_mode, void *workspace,
                                         size_t workspace_bytes, void *stream);

size_t qes_gemm_batch_workspace_bytes(const qes_tensor *tensors, int32_t n_tensors, const void *const *x, int32_t N,
                                      int32_t T, int32_t act_mode);

/* ---- the seeded update (Alg. 2 whole; Eq. 5-8) ---- */

/*
 * Stateless QES update with seed replay, per element and in place:
 *   c = α/(Nσ); e~ = 0
 *   for τ = 0 .. hist_len-1 (oldest first):  g = Σ_i hist_fit[τ][i]·δ(hist_seeds[τ][i])
 *        u = c·g + γ·e~;  Δ = Round(u);  Δf = Δ if qmin <= W_t+Δ <= qmax else 0;  e~ = u − Δf
 *   g = Σ_i fit_t[i]·δ(seeds_t[i]);  u = c·g + γ·e~;  Δ = Round(u);  W_{t+1} = W_t+Δ if in range
 * Every simulated step gates against the CURRENT weights W_t. Round is round-half-to-even; all
 * residual arithmetic is fp32 in the fixed order given in docs/NOISE_SPEC.md and the oracle.
 *
 *   seeds_t, fit_t        HOST [N]; fit_t already normalised (see qes_normalize_fitness)
 *   hist_seeds, hist_fit  HOST [hist_len][N], oldest generation first; NULL when hist_len == 0
 *   hist_len              0 .. QES_MAX_HISTORY. 0 is the stateless deterministic-rounding update.
 *   sigma > 0; alpha, gamma finite; every fitness finite.
 *   stats                 DEVICE uint64 [2] or NULL. stats[0] += elements whose weight changed,
 *                         stats[1] += elements whose non-zero Δ was masked by the gate (final
 *                         step only). Accumulated with atomics; the caller zeroes it.
 * The library owns no optimiser state: appending (seeds_t, fit_t) to the history is the caller's.
 */
int qes_update(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
               const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha,
               float gamma, uint64_t *stats, void *stream);

/*
 * qes_update for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. Same arguments, same results. The (seed, fitness) records do not
 * go through the staging ring but into a fixed array in the library's device image (256 KiB per
 * GPU, held until the process ends), written by small kernels that carry the records in their
 * kernel arguments. The call enqueues kernel launches only: no hipMalloc, hipFree, memcpy or
 * memset, no wait; a captured call replays with the records it was captured with. The first call
 * on a device looks up the array's device address (hipGetSymbolAddress): make it outside a capture.
 *   Limit: (hist_len + 1) * N <= QES_NOALLOC_MAX_RECORDS, else QES_ERR_TOO_LARGE (nothing enqueued).
 *   All calls on a GPU share that GPU's array, which keeps the last call's records: calls on one
 *   stream are ordered and safe; calls that overlap on one GPU (different streams without an
 *   ordering between them, or two host threads) race on it.
 */
int qes_update_noalloc(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                       const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha,
                       float gamma, uint64_t *stats, void *stream);

/*
 * The replay loop of Alg. 2 alone: the proxy residual e~ after replaying the history, before the
 * new population's step. residual: DEVICE float32 [out_features, in_features], 16-byte aligned.
 * Weights are read, not written. Arguments as for qes_update.
 */
int qes_replay_residual(const qes_tensor *w, const uint64_t *hist_seeds, const float *hist_fit,
                        int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                        float *residual, void *stream);

/*
 * qes_update (Alg. 2 whole) applied to every tensor of a list: all linears of a model share the
 * generation's seeds, fitnesses and history, so the records are staged once and the tensors are
 * updated by one launch per weight width, which also spares the partly filled last round of
 * workgroups that every single-tensor launch ends with. Results are those of n_tensors qes_update
 * calls (each element's noise depends on its own tensor_id and index only).
 *
 *   tensors    HOST array [n_tensors] of descriptors; 1 <= n_tensors <= QES_MAX_BATCH; their qweight
 *              buffers are DEVICE memory as for qes_update and must not overlap; `scales` is unused
 *   stats      DEVICE uint64 [2] or NULL: counters summed over all tensors
 * Other arguments as for qes_update / qes_update_antithetic.
 */
int qes_update_batch(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *seeds_t, const float *fit_t,
                     const uint64_t *hist_seeds, const float *hist_fit, int32_t hist_len, int32_t N, float sigma,
                     float alpha, float gamma, uint64_t *stats, void *stream);

int qes_update_batch_antithetic(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *pair_seeds_t,
                                const float *fit_t, const uint64_t *hist_pair_seeds, const float *hist_fit,
                                int32_t hist_len, int32_t N, float sigma, float alpha, float gamma, uint64_t *stats,
                                void *stream);

/*
 * qes_update / qes_replay_residual with antithetic perturbation pairs (App. A.1): N is even; every
 * generation has N/2 seeds (pair_seeds_t: HOST [N/2]; hist_pair_seeds: HOST [hist_len][N/2]) and N
 * fitnesses (fit_t: HOST [N]; hist_fit: HOST [hist_len][N]), members 2j and 2j+1 adjacent. Eq. 5 is
 * summed in member order with δ_{2j+1} = −δ_{2j}, c = α/(Nσ) with N the number of members; one
 * draw serves both members of a pair, so the noise work is half that of qes_update at equal N.
 */
int qes_update_antithetic(qes_tensor *w, const uint64_t *pair_seeds_t, const float *fit_t,
                          const uint64_t *hist_pair_seeds, const float *hist_fit, int32_t hist_len, int32_t N,
                          float sigma, float alpha, float gamma, uint64_t *stats, void *stream);

int qes_replay_residual_antithetic(const qes_tensor *w, const uint64_t *hist_pair_seeds, const float *hist_fit,
                                   int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                                   float *residual, void *stream);

/*
 * Alg. 1, the Full-Residual variant (§3.2 Eq. 6-8 with an explicitly stored residual): one step
 *   g = Σ_i fit_t[i]·δ(seeds_t[i]);  u = c·g + γ·e;  Δ = Round(u);  Δf = Δ if in range else 0;
 *   W ← W + Δf;  e ← u − Δf
 * e_state: DEVICE float32 [out_features, in_features], 16-byte aligned, read and written; the
 * caller zeroes it before the first step. Other arguments as for qes_update (no history).
 */
int qes_update_full_residual(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                             float alpha, float gamma, float *e_state, uint64_t *stats, void *stream);

/*
 * The same step with the residual stored as IEEE binary16, the precision Alg. 1 initialises it in
 * (and the Full-Residual variant of the §4 residual ablation stores): e is decoded exactly, the
 * step is computed in fp32 as above, and e ← half(u − Δf), rounded to nearest even after
 * saturating at ±65504, so a stored residual is always finite.
 * e_state_f16: DEVICE binary16 [out_features, in_features], 16-byte aligned, read and written.
 */
int qes_update_full_residual_f16(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                 float alpha, float gamma, uint16_t *e_state_f16, uint64_t *stats, void *stream);

/*
 * Stateless baseline the paper's §5 analyses (W ← W + Q(α ĝ), Eq. 9-10, with a stochastic Q), for
 * comparisons on the same kernels; not part of QES. No residual and no history:
 *   g = Σ_i fit_t[i]·δ(seeds_t[i]);  u = c·g;  Δ = ⌊u⌋ + [ub < u − ⌊u⌋];  W ← W + Δ if in range else W
 * with ub the element's rounding uniform of this step (docs/NOISE_SPEC.md N8: Philox keyed by
 * round_seed, stream tag 1). The deterministic stateless baseline is qes_update with hist_len = 0.
 * Other arguments as for qes_update.
 */
int qes_update_stochastic_rounding(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                   float alpha, uint64_t round_seed, uint64_t *stats, void *stream);

/*
 * Alg. 1 "normalize reward for population": z-score with the population standard deviation,
 * computed in fp64; zero variance or N < 2 gives all zeros. HOST in, HOST out, no GPU work.
 */
int qes_normalize_fitness(const float *reward, int32_t N, float *fit);

/* ---- machine ceilings measured with the library's own noise code (benchmark support) ---- */

/*
 * Noise ceiling. Runs `iters` (a multiple of 4) Philox calls (mode 0) or full pair draws (mode 1:
 * Philox + Box-Muller + two stochastic roundings) per thread on `n_threads` threads, four
 * independent chains at a time and eight waves per SIMD, the shape the update kernel runs the
 * generator in, and folds the results into sink[n_threads] (DEVICE uint32) so the work cannot be
 * elided. No memory traffic in the loop.
 */
int qes_bench_noise(int32_t mode, uint64_t n_threads, int32_t iters, float sigma, uint32_t *sink,
                    void *stream);

/*
 * MFMA ceiling. Every wave of n_blocks workgroups (4 waves each) issues iters x 8 independent
 * matrix instructions on register operands: mode 0 v_mfma_f32_16x16x32_bf16 (16384 flop each),
 * mode 1 v_mfma_i32_16x16x64_i8 (32768 op each). sink: DEVICE uint32 [n_blocks * 256].
 */
int qes_bench_mfma(int32_t mode, uint32_t n_blocks, int32_t iters, uint32_t *sink, void *stream);

/* Plain streaming copy of n_bytes (multiple of 16) from src to dst, both DEVICE, 16-byte aligned. */
int qes_bench_copy(const void *src, void *dst, size_t n_bytes, void *stream);

/* ---- diagnostics ---- */

const char *qes_status_string(int status);
/* hipError_t of the last failing HIP call on this thread (0 if none). */
int qes_last_hip_error(void);
/* Library ABI version; bumped when a signature changes. */
int qes_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QES_H */
