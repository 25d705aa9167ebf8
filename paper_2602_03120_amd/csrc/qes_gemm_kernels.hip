// Population-batched perturbed quantised GEMM (paper Alg. 1: "reconstruct δ_i", "W' = Gate(W_t+δ_i)",
// inference; §3.2 Eq. 3-4; App. A.1 formats).
//
//   Y[i,t,n] = Σ_g s[n,g] · Σ_{k in g} X[i,t,k] · W'_i[n,k],   W'_i = Gate(W + δ_i)
//
// Work decomposition. The cost is the regeneration of δ (about sixty vector-ALU operations per
// weight element and member) against 2·T MFMA flops, so every (member, n, k) draw is generated
// exactly once: a workgroup owns one member, an n-tile of 16·kWaves output rows and ALL of that
// member's tokens (up to TM per pass), and walks K. Each wave owns 16 output rows; per k-substep a
// lane regenerates the K-consecutive elements of its MFMA B fragment in registers, gates them
// against the base integers and hands them to the matrix core as exact small integers (bf16 or
// int8).
//
// Overlap. The noise of substep s+1 is generated while the MFMAs of substep s execute: the B
// fragment is double-buffered in registers and the source interleaves one Philox pair with a
// quarter of the substep's MFMAs and their LDS reads. The activation tile of the next 64-k stage
// is fetched straight into LDS (global_load_lds_dwordx4, no registers) while the current stage is
// consumed; LDS is double-buffered and XOR-swizzled so that the b128 fragment reads are
// conflict-free without padding. One barrier per stage.
//
// Group scales. The accumulators are kept in units of the current group's scale: at a group
// boundary they are multiplied by s_old/s_new (one multiply per accumulator) and the integers
// enter the MFMA unscaled, so the weights are never rounded and no second accumulator set is
// needed. A zero scale contributes nothing and leaves the unit unchanged.
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
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kTileN = 16 * kWaves;
constexpr int kStageK = 64;   // k extent of one LDS stage

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

// Base integers of one lane's fragment slice.
__device__ __forceinline__ void unpack_int4x8(uint32_t word, int32_t w[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = ((int32_t)(word << (28 - 4 * j))) >> 28;
}

__device__ __forceinline__ void unpack_int8x4(uint32_t word, int32_t w[4])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = ((int32_t)(word << (24 - 8 * j))) >> 24;
}

// One pair: draw, gate (Eq. 4) in place.
__device__ __forceinline__ void perturb_pair(int32_t &w0, int32_t &w1, uint32_t k0, uint32_t k1, uint32_t tensor_id,
                                             uint32_t pair, float sigma, int32_t qmin, uint32_t qspan)
{
    int32_t d0, d1;
    delta_pair(k0, k1, tensor_id, pair, sigma, d0, d1);
    w0 = gate(w0, d0, qmin, qspan);
    w1 = gate(w1, d1, qmin, qspan);
}

// exact bf16 images of two small integers in one dword (low half = first element)
__device__ __forceinline__ uint32_t pack_bf16x2(int32_t a, int32_t b)
{
    const uint32_t lo = __float_as_uint((float)a);
    const uint32_t hi = __float_as_uint((float)b);
    return (lo >> 16) | (hi & 0xFFFF0000u);
}

__device__ __forceinline__ uint32_t pack_i8x4(const int32_t *w)
{
    return ((uint32_t)w[0] & 0xFFu) | (((uint32_t)w[1] & 0xFFu) << 8) | (((uint32_t)w[2] & 0xFFu) << 16) |
           ((uint32_t)w[3] << 24);
}

// ------------------------------------------------------------------------------------------------
// Activation tile -> LDS, asynchronously. ROW_BYTES is 128 (64 bf16) or 64 (64 int8). One wave
// instruction moves 64 chunks of 16 bytes = 1 KiB of consecutive LDS. A chunk's position inside
// its row is XOR-swizzled with row bits so that 8 consecutive rows read at the same logical chunk
// hit 8 different bank groups.
template <int ROW_BYTES>
__device__ __forceinline__ int swizzle(int row, int chunk)
{
    return ROW_BYTES == 128 ? (chunk ^ (row & 7)) : (chunk ^ ((row >> 2) & 3));
}

template <int TM, int ROW_BYTES, int ELEM_BYTES>
__device__ __forceinline__ void issue_tile(const char *__restrict__ x_member, int T, int in_features, int t0, int ks,
                                           char *lds_buf, int wave, int lane)
{
    constexpr int kChunksPerRow = ROW_BYTES / 16;
    constexpr int kRowsPerInstr = 64 / kChunksPerRow;
    constexpr int kInstr = TM / kRowsPerInstr;
    constexpr int kElemsPerChunk = 16 / ELEM_BYTES;
#pragma unroll
    for (int j = wave; j < kInstr; j += kWaves) {
        const int row = j * kRowsPerInstr + lane / kChunksPerRow;
        const int pch = lane % kChunksPerRow;
        const int ch = swizzle<ROW_BYTES>(row, pch);
        // rows past T and chunks past in_features are clamped to valid memory; what they deliver is
        // never used (those outputs are not stored, those substeps are not run)
        int t = t0 + row;
        t = t < T ? t : T - 1;
        int k = ks + ch * kElemsPerChunk;
        k = k < in_features ? k : in_features - kElemsPerChunk;
        const char *src = x_member + ((size_t)t * in_features + k) * ELEM_BYTES;
        __builtin_amdgcn_global_load_lds((gbl_void *)src, (lds_void *)(lds_buf + j * 1024), 16, 0, 0);
    }
}

// Slice schedule shared by both GEMM kernels. A substep's MFMA tiles are cut into kSlices slices;
// slice q's A fragments are read from LDS one slice ahead, then one Philox pair of the NEXT
// substep's B fragment is generated, then slice q's MFMAs are issued, so LDS latency and MFMA
// execution both hide behind the noise arithmetic of the same wave. sched_barrier(0) pins that
// order against the compiler's own scheduling.
template <int kMT, int kSlices>
__device__ __forceinline__ constexpr int slice_of(int m)
{
    return kMT >= kSlices ? (m * kSlices) / kMT : kSlices - kMT + m;
}
template <int kMT, int kSlices>
constexpr int kSliceTiles = kMT >= kSlices ? (kMT + kSlices - 1) / kSlices : 1;

#define QES_PIN_ORDER() __builtin_amdgcn_sched_barrier(0)

// ------------------------------------------------------------------------------------------------
// bf16 activations (act_mode 0), INT4 or INT8 weights. TM: tokens per pass (multiple of 16).
template <int BITS, int TM>
struct Bf16Gemm {
    static constexpr int kMT = TM / 16;
    static constexpr int kTileBytes = TM * 128;
    static constexpr int kSlices = 4;
    static constexpr int kST = kSliceTiles<kMT, kSlices>;

    const GemmArgs &a;
    Entry en;
    int lane, wave, ln, kc, n, n_ld, gs, n_sub;
    const uint16_t *scales;
    const char *xg;
    const char *wrow;
    size_t elem_row;
    // running state of one pass
    f32x4 acc[kMT];
    Frag b_cur;
    float s_cur;
    bool zero_b;

    __device__ __forceinline__ void load_base(int s, int32_t w[8]) const
    {
        const int k = s * 32 + kc * 8;
        if (BITS == 4) {
            unpack_int4x8(*(const uint32_t *)(wrow + (k >> 1)), w);
        } else {
            const uint2 two = *(const uint2 *)(wrow + k);
            unpack_int8x4(two.x, w);
            unpack_int8x4(two.y, w + 4);
        }
    }

    // Rows m*16+ln share their low bits with ln, so the swizzled chunk does not depend on m: one
    // per-lane address plus an immediate offset per tile.
    __device__ __forceinline__ void read_slice(const char *lane_base, int q, Frag (&af)[kST]) const
    {
        int i = 0;
#pragma unroll
        for (int m = 0; m < kMT; ++m) {
            if (slice_of<kMT, kSlices>(m) != q) continue;
            af[i++].v = *(const uint4 *)(lane_base + m * 16 * 128);
        }
    }

    __device__ __forceinline__ void mfma_slice(int q, const Frag (&af)[kST])
    {
        int i = 0;
#pragma unroll
        for (int m = 0; m < kMT; ++m) {
            if (slice_of<kMT, kSlices>(m) != q) continue;
            acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i++].bf, b_cur.bf, acc[m], 0, 0, 0);
        }
    }

    // Substep s: MFMAs of B fragment b_cur against LDS buffer `buf`, while the B fragment of substep
    // s+1 is produced (NOISE: with perturbation; otherwise base integers only, if there is a next).
    template <bool NOISE>
    __device__ __forceinline__ void substep(const char *buf, int s, bool has_next)
    {
        const int sub = s & 1;
        int32_t wn[8];
        bool zero_next = zero_b;
        bool rescale = false;
        float ratio = 1.0f;
        if (has_next) {
            load_base(s + 1, wn);
            const int k_next = (s + 1) * 32;
            if ((k_next % gs) == 0) {   // the next substep opens a new group
                const float s_new = f16_bits_to_f32(scales[k_next / gs]);
                zero_next = (s_new == 0.0f);
                if (!zero_next) {
                    ratio = s_cur / s_new;
                    s_cur = s_new;
                    rescale = true;
                }
            }
        }
        const uint32_t pair_next = (uint32_t)((elem_row + (size_t)(s + 1) * 32 + kc * 8) >> 1);

        const char *lane_base = buf + ln * 128 + swizzle<128>(ln, sub * 4 + kc) * 16;
        Frag af[2][kST];
        read_slice(lane_base, 0, af[0]);
#pragma unroll
        for (int q = 0; q < kSlices; ++q) {
            if (q + 1 < kSlices) read_slice(lane_base, q + 1, af[(q + 1) & 1]);
            QES_PIN_ORDER();
            if (NOISE)
                perturb_pair(wn[2 * q], wn[2 * q + 1], en.seed_lo, en.seed_hi, a.tensor_id, pair_next + q, a.sigma,
                             a.qmin, a.qspan);
            QES_PIN_ORDER();
            mfma_slice(q, af[q & 1]);
        }
        QES_PIN_ORDER();
        if (has_next) {
#pragma unroll
            for (int q = 0; q < 4; ++q) b_cur.u[q] = zero_next ? 0u : pack_bf16x2(wn[2 * q], wn[2 * q + 1]);
            zero_b = zero_next;
            if (rescale) {   // new unit for the accumulators before the next group adds to them
#pragma unroll
                for (int m = 0; m < kMT; ++m) acc[m] *= ratio;
            }
        }
    }

    // One 64-k stage: consume `rd`, prefetch the next stage's activations into `wr`.
    template <bool PERTURB>
    __device__ __forceinline__ void stage(const char *rd, char *wr, int st, int n_stage, int t0)
    {
        if (st + 1 < n_stage)
            issue_tile<TM, 128, 2>(xg, a.T, a.in_features, t0, (st + 1) * kStageK, wr, wave, lane);
        const int s = 2 * st;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (s + h >= n_sub) break;
            const bool has_next = (s + h + 1) < n_sub;
            if (PERTURB && has_next) substep<true>(rd, s + h, true);
            else substep<false>(rd, s + h, has_next);
        }
        // the next tile must have landed, and everyone must be done with this one
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
    }

    template <bool PERTURB>
    __device__ __forceinline__ void pass(char *lds0, char *lds1, int t0, uint16_t *yg)
    {
#pragma unroll
        for (int m = 0; m < kMT; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
        // unit of the accumulators: scale of the group being accumulated (1 while that is zero)
        s_cur = f16_bits_to_f32(scales[0]);
        zero_b = (s_cur == 0.0f);
        if (zero_b) s_cur = 1.0f;

        __syncthreads();   // the previous pass has finished reading LDS
        issue_tile<TM, 128, 2>(xg, a.T, a.in_features, t0, 0, lds0, wave, lane);

        // B fragment of substep 0 (nothing to overlap with yet)
        int32_t w[8];
        load_base(0, w);
        if (PERTURB) {
            const uint32_t pair = (uint32_t)((elem_row + kc * 8) >> 1);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                perturb_pair(w[2 * q], w[2 * q + 1], en.seed_lo, en.seed_hi, a.tensor_id, pair + q, a.sigma, a.qmin,
                             a.qspan);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) b_cur.u[q] = zero_b ? 0u : pack_bf16x2(w[2 * q], w[2 * q + 1]);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();

        const int n_stage = (n_sub + 1) / 2;
        for (int st = 0; st < n_stage; st += 2) {
            stage<PERTURB>(lds0, lds1, st, n_stage, t0);
            if (st + 1 < n_stage) stage<PERTURB>(lds1, lds0, st + 1, n_stage, t0);
        }

        if (n < a.out_features) {
#pragma unroll
            for (int m = 0; m < kMT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = t0 + m * 16 + kc * 4 + j;
                    if (t < a.T) yg[(size_t)t * a.out_features + n] = f32_to_bf16_rne(acc[m][j] * s_cur);
                }
        }
    }
};

template <int BITS, int TM>
__global__ __launch_bounds__(kThreads, 2) void gemm_bf16_kernel(const GemmArgs a)
{
    using G = Bf16Gemm<BITS, TM>;
    // two separate arrays (not one array with two halves): the compiler then knows that reads of
    // one never alias the asynchronous loads into the other and does not wait for them
    __shared__ __attribute__((aligned(1024))) char lds0[G::kTileBytes];
    __shared__ __attribute__((aligned(1024))) char lds1[G::kTileBytes];

    uint32_t member, tile;
    const uint32_t n_tiles = (a.out_features + kTileN - 1) / kTileN;
    if (!block_to_work(n_tiles, (uint32_t)a.N, member, tile)) return;

    G g{a};
    g.lane = threadIdx.x & 63;
    g.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    g.ln = g.lane & 15;        // column of B / C within the wave's 16 rows
    g.kc = g.lane >> 4;        // k-chunk 0..3
    g.n = tile * kTileN + g.wave * 16 + g.ln;
    g.n_ld = g.n < a.out_features ? g.n : a.out_features - 1;   // clamp loads, skip stores
    g.en = a.entries[member];
    g.gs = a.group_size > 0 ? a.group_size : a.in_features;
    g.n_sub = a.in_features / 32;
    g.scales = (const uint16_t *)a.scales + (size_t)g.n_ld * (a.in_features / g.gs);
    g.xg = (const char *)a.x + (size_t)member * a.T * a.in_features * 2;
    g.wrow = (const char *)a.qweight + ((size_t)g.n_ld * a.in_features * BITS) / 8;
    g.elem_row = (size_t)g.n_ld * a.in_features;
    uint16_t *yg = (uint16_t *)a.y + (size_t)member * a.T * a.out_features;
    const bool perturb = (g.en.fit_bits != 0u) && (a.sigma != 0.0f);

    for (int t0 = 0; t0 < a.T; t0 += TM) {
        if (perturb) g.template pass<true>(lds0, lds1, t0, yg);
        else g.template pass<false>(lds0, lds1, t0, yg);
    }
}

// ------------------------------------------------------------------------------------------------
// W8A8 (act_mode 1): int8 activations quantised per token by quantize_kernel, int8 MFMA, exact
// int32 accumulation, Y = bf16(((float)acc · a[t]) · s[n]). One 64-k substep per LDS stage.
template <int TM>
struct I8Gemm {
    static constexpr int kMT = TM / 16;
    static constexpr int kTileBytes = TM * 64;
    static constexpr int kSlices = kMT >= 32 ? 16 : 8;   // more, smaller slices keep 512 tokens within 256 VGPRs
    static constexpr int kSlicesPerPair = kSlices / 8;   // 8 Philox pairs per 64-k fragment
    static constexpr int kST = kSliceTiles<kMT, kSlices>;

    const GemmArgs &a;
    Entry en;
    int lane, wave, ln, kc, n, n_ld, n_sub;
    const char *xg;
    const char *wrow;
    size_t elem_row;
    i32x4 acc[kMT];
    Frag b_cur;

    // a lane whose 16-chunk lies past in_features (only when in_features % 64 == 32) feeds zeros
    __device__ __forceinline__ bool lane_in_range(int s) const { return s * 64 + kc * 16 < a.in_features; }
    __device__ __forceinline__ int lane_k(int s) const
    {
        const int k = s * 64 + kc * 16;
        return k < a.in_features ? k : a.in_features - 16;
    }
    __device__ __forceinline__ void load_base(int s, int32_t w[16]) const
    {
        const uint4 four = *(const uint4 *)(wrow + lane_k(s));
        unpack_int8x4(four.x, w);
        unpack_int8x4(four.y, w + 4);
        unpack_int8x4(four.z, w + 8);
        unpack_int8x4(four.w, w + 12);
    }
    __device__ __forceinline__ void pack(const int32_t w[16], bool in_range)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) b_cur.u[q] = in_range ? pack_i8x4(w + 4 * q) : 0u;
    }
    __device__ __forceinline__ void read_slice(const char *lane_base, int q, Frag (&af)[kST]) const
    {
        int i = 0;
#pragma unroll
        for (int m = 0; m < kMT; ++m) {
            if (slice_of<kMT, kSlices>(m) != q) continue;
            af[i++].v = *(const uint4 *)(lane_base + m * 16 * 64);
        }
    }
    __device__ __forceinline__ void mfma_slice(int q, const Frag (&af)[kST])
    {
        int i = 0;
#pragma unroll
        for (int m = 0; m < kMT; ++m) {
            if (slice_of<kMT, kSlices>(m) != q) continue;
            acc[m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[i++].i8, b_cur.i8, acc[m], 0, 0, 0);
        }
    }

    template <bool NOISE>
    __device__ __forceinline__ void substep(const char *buf, int s, bool has_next)
    {
        int32_t wn[16];
        if (has_next) load_base(s + 1, wn);
        const uint32_t pair_next = (uint32_t)((elem_row + lane_k(s + 1)) >> 1);
        const char *lane_base = buf + ln * 64 + swizzle<64>(ln, kc) * 16;
        Frag af[2][kST];
        read_slice(lane_base, 0, af[0]);
#pragma unroll
        for (int q = 0; q < kSlices; ++q) {
            if (q + 1 < kSlices) read_slice(lane_base, q + 1, af[(q + 1) & 1]);
            QES_PIN_ORDER();
            if (NOISE && (q % kSlicesPerPair) == 0) {
                const int pq = q / kSlicesPerPair;
                perturb_pair(wn[2 * pq], wn[2 * pq + 1], en.seed_lo, en.seed_hi, a.tensor_id, pair_next + pq, a.sigma,
                             a.qmin, a.qspan);
            }
            QES_PIN_ORDER();
            mfma_slice(q, af[q & 1]);
        }
        QES_PIN_ORDER();
        if (has_next) pack(wn, lane_in_range(s + 1));
    }

    template <bool PERTURB>
    __device__ __forceinline__ void stage(const char *rd, char *wr, int s, int t0)
    {
        const bool has_next = (s + 1) < n_sub;
        if (has_next) issue_tile<TM, 64, 1>(xg, a.T, a.in_features, t0, (s + 1) * 64, wr, wave, lane);
        if (PERTURB && has_next) substep<true>(rd, s, true);
        else substep<false>(rd, s, has_next);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
    }

    template <bool PERTURB>
    __device__ __forceinline__ void pass(char *lds0, char *lds1, int t0, uint16_t *yg, const float *xs, float s_n)
    {
#pragma unroll
        for (int m = 0; m < kMT; ++m) acc[m] = i32x4{0, 0, 0, 0};
        __syncthreads();
        issue_tile<TM, 64, 1>(xg, a.T, a.in_features, t0, 0, lds0, wave, lane);
        int32_t w[16];
        load_base(0, w);
        if (PERTURB) {
            const uint32_t pair = (uint32_t)((elem_row + lane_k(0)) >> 1);
#pragma unroll
            for (int q = 0; q < 8; ++q)
                perturb_pair(w[2 * q], w[2 * q + 1], en.seed_lo, en.seed_hi, a.tensor_id, pair + q, a.sigma, a.qmin,
                             a.qspan);
        }
        pack(w, lane_in_range(0));
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();

        for (int s = 0; s < n_sub; s += 2) {
            stage<PERTURB>(lds0, lds1, s, t0);
            if (s + 1 < n_sub) stage<PERTURB>(lds1, lds0, s + 1, t0);
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
};

template <int TM>
__global__ __launch_bounds__(kThreads, 2) void gemm_i8_kernel(const GemmArgs a)
{
    using G = I8Gemm<TM>;
    __shared__ __attribute__((aligned(1024))) char lds0[G::kTileBytes];
    __shared__ __attribute__((aligned(1024))) char lds1[G::kTileBytes];

    uint32_t member, tile;
    const uint32_t n_tiles = (a.out_features + kTileN - 1) / kTileN;
    if (!block_to_work(n_tiles, (uint32_t)a.N, member, tile)) return;

    G g{a};
    g.lane = threadIdx.x & 63;
    g.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    g.ln = g.lane & 15;
    g.kc = g.lane >> 4;
    g.n = tile * kTileN + g.wave * 16 + g.ln;
    g.n_ld = g.n < a.out_features ? g.n : a.out_features - 1;
    g.en = a.entries[member];
    g.n_sub = (a.in_features + 63) / 64;
    g.xg = (const char *)a.x + (size_t)member * a.T * a.in_features;
    g.wrow = (const char *)a.qweight + (size_t)g.n_ld * a.in_features;
    g.elem_row = (size_t)g.n_ld * a.in_features;
    const float *xs = a.x_scale + (size_t)member * a.T;
    uint16_t *yg = (uint16_t *)a.y + (size_t)member * a.T * a.out_features;
    const float s_n = f16_bits_to_f32(((const uint16_t *)a.scales)[g.n_ld]);
    const bool perturb = (g.en.fit_bits != 0u) && (a.sigma != 0.0f);

    for (int t0 = 0; t0 < a.T; t0 += TM) {
        if (perturb) g.template pass<true>(lds0, lds1, t0, yg, xs, s_n);
        else g.template pass<false>(lds0, lds1, t0, yg, xs, s_n);
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
