// Population-batched perturbed quantised GEMM (paper Alg. 1: "reconstruct δ_i", "W' = Gate(W_t+δ_i)",
// inference; §3.2 Eq. 3-4; App. A.1 formats).
//
//   Y[i,t,n] = Σ_g s[n,g] · Σ_{k in g} X[i,t,k] · W'_i[n,k],   W'_i = Gate(W + δ_i)
//
// The cost is the regeneration of δ (about sixty vector-ALU operations per weight element and
// member) against 2·T MFMA flops, so the design goal is that every (member, n, k) draw is generated
// exactly once and that the noise arithmetic is spread evenly over all waves, with the MFMAs, the
// LDS traffic and the global loads hidden underneath it.
//
// Decomposition. A workgroup (8 waves, 16 for the 512-token tile) owns one member, 4 groups of 16
// output rows and ALL tokens of that member (TM per pass). Per k-substep (32 k for bf16, 64 k for
// int8 operands) the MFMA B fragment of a row group is 4 dwords per lane; the waves split the four
// fragments evenly (a half or a quarter of one each: one to four Philox pairs per lane: draw, gate
// against the base integers, pack as exact small-integer bf16 or int8), publish them through LDS,
// and after the workgroup barrier wave (wm, wr) reads the fragments of row groups 2 wr and 2 wr + 1
// back (one b128 each) and runs the MFMAs of the token tiles m = wm (mod 4 or 8). So the noise work
// per wave is an equal share of the workgroup's whatever the token count, and short token counts
// still use all waves for noise.
//
// Antithetic pairs (PAIRED). Members 2j and 2j+1 use +δ and -δ of one draw, so a workgroup owns the
// pair: every draw is generated once, gated twice (W+δ for the even member, W-δ for the odd one),
// published as two fragments, and each member's token tiles meet their own fragment. Half the
// noise work per member; accumulators, activation tiles and MFMAs are per member as before.
//
// Pipelining. B fragments are double-buffered in LDS: the dword for substep s+1 is generated while
// the MFMAs of substep s run. The activation tile of substep s+1 goes straight from global memory
// into LDS (global_load_lds_dwordx4, no registers) while substep s is consumed; it is
// double-buffered in two separate LDS arrays (so the compiler knows reads of one never wait for
// loads into the other) and XOR-swizzled so the b128 fragment reads are conflict-free without
// padding. One workgroup barrier per substep. Where registers allow, a substep is one straight-line
// block and scheduling groups spread its matrix instructions over the noise job, so that a wave's
// vector work continues while the matrix pipe runs.
//
// Group scales. The accumulators are kept in units of the current group's scale: at a group
// boundary they are multiplied by s_old/s_new (one multiply per accumulator) and the integers
// enter the MFMA unscaled, so the weights are never rounded and no second accumulator set is
// needed. A zero scale contributes nothing and leaves the unit unchanged.
//
// MFMA shapes (gfx950): v_mfma_f32_16x16x32_bf16 and v_mfma_i32_16x16x64_i8. Operand layout for a
// 64-lane wave: A lane l holds row l%16, k-chunk l/16; B lane l holds column l%16, k-chunk l/16;
// C lane l holds column l%16, rows 4·(l/16)..+3.
#include <type_traits>

#include "qes_internal.hpp"
#include "qes_noise.hpp"

namespace qes {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;
// Kernel arguments and batch descriptors are read through the constant address space: wave-uniform
// reads from it are scalar loads issued where a field is needed, so the fields never occupy
// registers for long (a by-value copy of the 100-byte argument block would).
typedef const __attribute__((address_space(4))) GemmArgs ConstGemmArgs;

constexpr int kRG = 4;          // row groups (of 16 output rows) per workgroup
constexpr int kTileN = 16 * kRG;
// Waves per workgroup: 8, or 16 where 8 waves would hold 64 accumulator registers per lane (the
// 512-token tile; a pair of members at 256 tokens), which spills or leaves two waves per SIMD.
constexpr int waves_for(int tm, bool paired) { return (tm >= 512 || (paired && tm >= 256)) ? 16 : 8; }
constexpr int kWR = 2;          // MFMA blocking: wave (wm, wr) owns row groups 2*wr and 2*wr+1 ...
constexpr int kRowBytes = 64;   // one LDS row of the activation tile: 32 bf16 or 64 int8
constexpr int kFragBytes = kRG * 64 * 16;   // one buffer of B fragments: 16 bytes per lane and row group

enum Mode { kBf16W4 = 0, kBf16W8 = 1, kI8W8 = 2 };

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
__device__ __forceinline__ uint32_t gemm_work_items_device(int32_t out_features, int32_t N, bool paired)
{
    return (uint32_t)((out_features + kTileN - 1) / kTileN) * ((uint32_t)N / (paired ? 2u : 1u));
}

__device__ __forceinline__ bool block_to_index(uint32_t total, uint32_t &idx)
{
    const uint32_t per_xcd = (total + 7u) / 8u;
    idx = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    return (blockIdx.x >> 3) < per_xcd && idx < total;
}

// The noise job works in fp32 throughout: base integers, perturbations and gated results are small
// integers, exact in fp32, so the gate is an add, a median and a select, the 4-bit container clamp
// of δ is compiled out when sigma <= 1.2 (|sigma*eps| <= 1.2 * 5.77 < 7 cannot reach it), and the
// bf16 operand is the upper half of the fp32 bit pattern. No int <-> float conversion of δ.

// One pair of elements for both members of an antithetic pair: one draw; the even member gates
// W + δ, the odd member W - δ (Eq. 4 each). on_even / on_odd are 1 or 0: a member whose
// perturbation is switched off gates W + 0 = W.
template <bool CLAMP>
__device__ __forceinline__ void perturb_pair_both(const float (&w)[2], float (&even)[2], float (&odd)[2], uint32_t k0,
                                                  uint32_t k1, uint32_t tensor_id, uint32_t pair, float sigma, float qmin,
                                                  float qmax, float on_even, float on_odd)
{
    float d[2];
    delta_pair_f32<CLAMP>(k0, k1, tensor_id, pair, sigma, d[0], d[1]);
#pragma unroll
    for (int l = 0; l < 2; ++l) {
        even[l] = gate_f32(w[l], d[l] * on_even, qmin, qmax);
        odd[l] = gate_f32(w[l], -d[l] * on_odd, qmin, qmax);
    }
}

// One pair: draw, gate (Eq. 4) in place. SIGN = -1 is the mirrored member of an antithetic pair.
template <int SIGN, bool CLAMP>
__device__ __forceinline__ void perturb_pair(float &w0, float &w1, uint32_t k0, uint32_t k1, uint32_t tensor_id,
                                             uint32_t pair, float sigma, float qmin, float qmax)
{
    float d0, d1;
    delta_pair_f32<CLAMP>(k0, k1, tensor_id, pair, sigma, d0, d1);
    w0 = gate_f32(w0, SIGN < 0 ? -d0 : d0, qmin, qmax);
    w1 = gate_f32(w1, SIGN < 0 ? -d1 : d1, qmin, qmax);
}

// exact bf16 images of two small integers held in fp32, in one dword (low half = first element):
// the upper halves of the two bit patterns
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    return __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);
}

__device__ __forceinline__ uint32_t pack_i8x4(float a, float b, float c, float d)
{
    return ((uint32_t)(int32_t)a & 0xFFu) | (((uint32_t)(int32_t)b & 0xFFu) << 8) | (((uint32_t)(int32_t)c & 0xFFu) << 16) |
           ((uint32_t)(int32_t)d << 24);
}

// Position of logical 16-byte chunk `chunk` (0..3) inside the 64-byte LDS row `row`: XOR-swizzled
// with row bits 1..2. A b128 read serves eight consecutive lanes (eight rows, one chunk each) per
// pass of the 128-byte-wide LDS; two rows share a 128-byte line, so rows 2i and 2i+1 take the two
// halves and the swizzle gives the four row pairs four different chunks: all 32 banks, once each.
// (SQ_LDS_BANK_CONFLICT of a config-5 layer: 3.3e8 with row bits 2..3, 1.1e8 with bits 1..2, the rest
// being the 8-byte fragment writes at a 16-byte lane stride.)
__device__ __forceinline__ int swizzle(int row, int chunk) { return chunk ^ ((row >> 1) & 3); }

template <int MODE, int TM, bool PAIRED>
struct Gemm {
    static constexpr int kP = PAIRED ? 2 : 1;                  // members per workgroup
    static constexpr bool kI8 = (MODE == kI8W8);
    static constexpr int kSubK = kI8 ? 64 : 32;                // k extent of one substep
    static constexpr int kElemBytes = kI8 ? 1 : 2;             // activation element
    static constexpr int kMT = TM / 16;                        // token tiles per pass
    static constexpr int kWaves = waves_for(TM, PAIRED);
    static constexpr int kWM = kWaves / kWR;                   // ... and the token tiles m = wm (mod kWM)
    static constexpr int kParts = kWaves / kRG;                // waves that share the noise of one row group's fragment
    static constexpr int kPartBytes = 16 / kParts;             // bytes of a lane's fragment one wave generates
    static constexpr int kMy = (kMT + kWM - 1) / kWM;          // token tiles per wave
    static constexpr int kTileBytes = TM * kRowBytes;
    static constexpr int kInstr = TM / 16;                     // wave instructions per activation tile
    static constexpr int kMyInstr = (kInstr + kWaves - 1) / kWaves;
    static constexpr int H = (kI8 ? 16 : 8) / kParts;          // elements in this wave's part of a fragment
    // One straight-line block per substep with the matrix instructions spread over the noise job,
    // except where 32 accumulator registers per lane leave no room for the longer fragment lifetimes
    // (a pair of members at 128 tokens, the 8-wave 256-token tile with int8 operands): those would
    // need more than 128 registers (one workgroup per CU) or spill.
    static constexpr bool kStraight = !(TM == 128 && PAIRED) && !(TM == 256 && !PAIRED && kI8);
    static constexpr int kWBytesPerSub = (MODE == kBf16W4) ? 16 : (MODE == kBf16W8 ? 32 : 64);   // weight bytes per row and substep
    using Acc = typename std::conditional<kI8, i32x4, f32x4>::type;

    ConstGemmArgs &a;
    Entry en;
    int lane, wave, wm, wr, ln, kc, n_sub;
    int jrg, jpart;               // noise job of this wave: part `jpart` of row group `jrg`'s fragment
    bool tail;                    // int8 only: in_features % 64 == 32, the last substep is half empty
    const uint16_t *scales[kWR];  // scale rows of this lane's two MFMA row groups
    const uint16_t *job_scales;   // scale row of this lane's noise job
    const char *xg[kP];           // activations of this workgroup's member(s)
    float keep[2];                // PAIRED: 1 / 0 per member: perturbation on / off
    float qmin_f, qmax_f;         // the gate's range, as fp32
    const char *wrow_lane;        // this lane's packed base integers of substep 0 (noise job)
    uint32_t pair0;               // pair index of this lane's half fragment of substep 0
    uint32_t a_off;               // LDS offset of this lane's A fragment of token tile wm
    uint32_t frag_rd[kWR];        // LDS offsets of this lane's two B fragments inside a fragment buffer
    uint32_t frag_wr;             // LDS offset of this lane's half fragment (noise job)
    char *bfrag;                  // 2 buffers x kP members x kFragBytes
    // per pass
    uint32_t tile_off[kMyInstr];  // global offset of this lane's 16-byte chunk of substep 0, per instruction
    Acc acc[kP][kMy][kWR];
    float s_cur[kWR];
    bool job_zero;
    int subs_per_group, subs_to_group_end;
    int group;
    uint2 raw_next;               // packed base integers of this wave's half fragment of the next substep
    uint16_t job_scale_next;      // scale bits of the group after the current one (noise job row) ...
    uint16_t scale_next[kWR];     // ... and of the two MFMA rows, fetched a whole group ahead

    // ---- activation tile of substep s -> LDS buffer, asynchronously. One wave instruction moves
    // 64 chunks of 16 bytes = 16 rows of 64 bytes = 1 KiB of consecutive LDS. Lane l fills row
    // l/4 of the instruction's 16 rows, physical chunk l%4, with logical chunk swizzle(row, l%4).
    // Rows past T are clamped to the last token (their outputs are never stored).
    __device__ __forceinline__ void prepare_tile_offsets(int t0)
    {
#pragma unroll
        for (int i = 0; i < kMyInstr; ++i) {
            const int j = i * kWaves + wave;
            const int row = j * 16 + (lane >> 2);
            int t = t0 + row;
            t = t < a.T ? t : a.T - 1;
            tile_off[i] = (uint32_t)(((size_t)t * a.in_features) * kElemBytes) + swizzle(row, lane & 3) * 16;
        }
    }

    __device__ __forceinline__ void issue_tile(int s, char *buf) const
    {
#pragma unroll
        for (int h = 0; h < kP; ++h) {
            const char *sbase = xg[h] + (size_t)s * (kSubK * kElemBytes);   // wave-uniform
#pragma unroll
            for (int i = 0; i < kMyInstr; ++i) {
                const int j = i * kWaves + wave;
                if (kInstr % kWaves != 0 && j >= kInstr) break;
                uint32_t off = tile_off[i];
                if (kI8 && tail && s == n_sub - 1) {
                    // chunks 2 and 3 of the half-empty last substep lie past the row: read chunk 0
                    // instead (in bounds); the fragments they meet are zero
                    const int ch = swizzle(j * 16 + (lane >> 2), lane & 3);
                    if (ch >= 2) off -= ch * 16;
                }
                __builtin_amdgcn_global_load_lds((gbl_void *)(sbase + off), (lds_void *)(buf + h * kTileBytes + j * 1024), 16, 0,
                                                 0);
            }
        }
    }

    // the packed base integers of this wave's part of the fragment of substep s (1 to 8 bytes),
    // fetched one substep before they are needed
    __device__ __forceinline__ uint2 load_raw(int s) const
    {
        constexpr int kBytes = (MODE == kBf16W4) ? H / 2 : H;
        const char *p = wrow_lane + (size_t)s * kWBytesPerSub;
        if (kI8 && tail && s == n_sub - 1 && kc >= 2) p -= 32;   // past the row: any valid address, value unused
        if (kBytes == 1) return make_uint2(*(const uint8_t *)p, 0u);
        if (kBytes == 2) return make_uint2(*(const uint16_t *)p, 0u);
        if (kBytes == 4) return make_uint2(*(const uint32_t *)p, 0u);
        return *(const uint2 *)p;
    }

    // this wave's part of a B fragment of substep s: draw, gate (Eq. 4), pack as exact small integers
    struct Halves {
        uint2 d[kP];
    };

    __device__ __forceinline__ uint2 pack_half(const float (&w)[H]) const
    {
        if (kI8) {
            const uint32_t lo = pack_i8x4(w[0], w[1], w[2], w[3]);
            return make_uint2(lo, H > 4 ? pack_i8x4(w[H - 4], w[H - 3], w[H - 2], w[H - 1]) : 0u);
        }
        const uint32_t lo = pack_bf16x2(w[0], w[1]);
        return make_uint2(lo, H > 2 ? pack_bf16x2(w[H - 2], w[H - 1]) : 0u);
    }

    // PERTURB: 0 base weights, 1 +δ, -1 -δ (mirrored member). CLAMP: the 4-bit container clamp of δ.
    template <int PERTURB, bool CLAMP>
    __device__ __forceinline__ Halves make_half(int s, uint2 raw, bool zero) const
    {
        float w[H];
#pragma unroll
        for (int j = 0; j < H; ++j) {
            if (MODE == kBf16W4) w[j] = (float)(((int32_t)(raw.x << (28 - 4 * j))) >> 28);
            else w[j] = (float)(((int32_t)((j < 4 ? raw.x : raw.y) << (24 - 8 * (j & 3)))) >> 24);
        }
        Halves out;
        const uint32_t pair = pair0 + (uint32_t)s * (kSubK / 2);
        if constexpr (PAIRED) {
            float even[H], odd[H];
#pragma unroll
            for (int p = 0; p < H / 2; ++p) {
                const float wp[2] = {w[2 * p], w[2 * p + 1]};
                float e2[2] = {wp[0], wp[1]}, o2[2] = {wp[0], wp[1]};
                if (PERTURB != 0)
                    perturb_pair_both<CLAMP>(wp, e2, o2, en.seed_lo, en.seed_hi, a.tensor_id, pair + p, a.sigma, qmin_f, qmax_f,
                                             keep[0], keep[1]);
                even[2 * p] = e2[0];
                even[2 * p + 1] = e2[1];
                odd[2 * p] = o2[0];
                odd[2 * p + 1] = o2[1];
            }
            out.d[0] = pack_half(even);
            out.d[kP - 1] = pack_half(odd);
        } else {
            if (PERTURB != 0) {
#pragma unroll
                for (int p = 0; p < H / 2; ++p)
                    perturb_pair<PERTURB, CLAMP>(w[2 * p], w[2 * p + 1], en.seed_lo, en.seed_hi, a.tensor_id, pair + p, a.sigma,
                                                 qmin_f, qmax_f);
            }
            out.d[0] = pack_half(w);
        }
        if (zero || (kI8 && tail && s == n_sub - 1 && kc >= 2)) {
#pragma unroll
            for (int h = 0; h < kP; ++h) out.d[h] = make_uint2(0u, 0u);
        }
        return out;
    }

    __device__ __forceinline__ void publish(int buffer, const Halves &hv)
    {
#pragma unroll
        for (int h = 0; h < kP; ++h) {
            char *dst = bfrag + (buffer * kP + h) * kFragBytes + frag_wr;
            if (kPartBytes == 8) *(uint2 *)dst = hv.d[h];
            else *(uint32_t *)dst = hv.d[h].x;
        }
    }

    // scales of group g+1, requested when group g opens so that nothing waits for them
    __device__ __forceinline__ void prefetch_scales(int g)
    {
        if ((g + 1) * subs_per_group < n_sub) {
            job_scale_next = job_scales[g + 1];
#pragma unroll
            for (int r = 0; r < kWR; ++r) scale_next[r] = scales[r][g + 1];
        }
    }

    // ---- one substep: MFMAs of the fragments of substep s on tile buffer `xbuf`, this wave's half
    // fragment of substep s+1 underneath. PAR is the parity of s: it selects the B-fragment buffer
    // at compile time.
    template <int PERTURB, bool CLAMP, int PAR, bool LAST>
    __device__ __forceinline__ void substep(int s, const char *xbuf, char *xbuf_next)
    {
        // kStraight: whether a next substep exists is known at compile time (LAST) and the substep
        // is one straight-line block. Otherwise it is tested at run time (LAST is false throughout).
        const bool has_next = kStraight ? !LAST : (s + 1) < n_sub;
        if (has_next) issue_tile(s + 1, xbuf_next);   // xbuf_next was last read in substep s-1
        const uint2 raw = raw_next;                   // for substep s+1, fetched during substep s-1
        if (kStraight) {
            // for substep s+2; past the end the last substep's bytes are fetched again and never used
            if (has_next) raw_next = load_raw(s + 2 < n_sub ? s + 2 : n_sub - 1);
        } else if (s + 2 < n_sub) {
            raw_next = load_raw(s + 2);
        }

        // Fragments of this wave's (member, token tile) items, member-major (at most 4 items). In
        // the straight-line form all of them are requested here, in the order the matrix
        // instructions use them (the scheduling groups below place the reads); otherwise the B
        // fragments and one batch of A fragments, the next batch after the first one's MFMAs.
        constexpr int kSteps = kP * kMy;
        constexpr int kBatch = kStraight ? kSteps : (kMy < 4 ? kMy : 4);
        Frag b[kP][kWR];
        Frag af[kBatch];
        auto read_b = [&](int h) {
#pragma unroll
            for (int r = 0; r < kWR; ++r) b[h][r].v = *(const uint4 *)(bfrag + (PAR * kP + h) * kFragBytes + frag_rd[r]);
        };
        auto read_batch = [&](int q0) {
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const int h = (q0 + q) / kMy, i = (q0 + q) % kMy;
                if (kStraight && i == 0) read_b(h);
                if (kMT % kWM == 0 || wm + i * kWM < kMT)
                    af[q].v = *(const uint4 *)(xbuf + h * kTileBytes + a_off + i * kWM * 16 * kRowBytes);
            }
        };
        if (!kStraight) {
#pragma unroll
            for (int h = 0; h < kP; ++h) read_b(h);
        }
        read_batch(0);

        // half fragment of the next substep; a new scale group may start there (bf16 modes)
        bool new_group = false;
        if (has_next) {
            if (!kI8) {
                new_group = (--subs_to_group_end == 0);   // wave-uniform selects, no branch
                subs_to_group_end = new_group ? subs_per_group : subs_to_group_end;
                group += new_group ? 1 : 0;
                job_zero = new_group ? ((job_scale_next & 0x7FFFu) == 0) : job_zero;
            }
            publish(1 - PAR, make_half<PERTURB, CLAMP>(s + 1, raw, job_zero));
        }

#pragma unroll
        for (int q0 = 0; q0 < kSteps; q0 += kBatch) {
            if (q0 > 0) read_batch(q0);
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const int h = (q0 + q) / kMy, i = (q0 + q) % kMy;
                if (kMT % kWM != 0 && wm + i * kWM >= kMT) continue;
#pragma unroll
                for (int r = 0; r < kWR; ++r) {
                    if constexpr (kI8)
                        acc[h][i][r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[q].i8, b[h][r].i8, acc[h][i][r], 0, 0, 0);
                    else
                        acc[h][i][r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[q].bf, b[h][r].bf, acc[h][i][r], 0, 0, 0);
                }
            }
        }
        if constexpr (kStraight && !LAST) {
            // Instruction order of the block above: the first part of the noise job, then the LDS
            // reads of the first two items' fragments, then one matrix instruction after every kGap
            // vector instructions of the rest of the noise job, each further item's fragments read
            // two items ahead of their use. So a wave's own vector work runs while the matrix pipe
            // is busy, instead of all MFMAs queueing up behind the noise, and only the fragments of
            // three items are held in registers at a time. Accumulation order per accumulator is
            // unchanged.
            constexpr int kAhead = (kSteps < 2 || TM == 256) ? 1 : 2;   // the 256-token tiles have no registers for two
            constexpr int kMfma = kSteps * kWR;
            constexpr int kNoiseValu = (H / 2) * (PAIRED ? 140 : 115);
            constexpr int kGap = (kNoiseValu - 10) / (kMfma + 1);
            auto reads_of = [](int q) constexpr { return 1 + (q % kMy == 0 ? kWR : 0); };   // A, and B at a member's first item
            __builtin_amdgcn_sched_group_barrier(0x100, reads_of(0) + (kAhead > 1 ? reads_of(1) : 0), 0);
#pragma unroll
            for (int q = 0; q < kSteps; ++q) {
#pragma unroll
                for (int r = 0; r < kWR; ++r) {
                    __builtin_amdgcn_sched_group_barrier(0x002, kGap, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                if (q + kAhead < kSteps) {
                    if ((q + kAhead) % kMy == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1 + kWR, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
        }
        if constexpr (!kI8) {
            if (new_group) {
                // the next substep opens a new group: express the accumulators in its scale (a zero
                // scale keeps the unit; its fragments are zero)
#pragma unroll
                for (int r = 0; r < kWR; ++r) {
                    const float s_new = f16_bits_to_f32(scale_next[r]);
                    if (s_new != 0.0f) {
                        const float ratio = s_cur[r] / s_new;
                        s_cur[r] = s_new;
#pragma unroll
                        for (int h = 0; h < kP; ++h)
#pragma unroll
                            for (int i = 0; i < kMy; ++i) acc[h][i][r] *= ratio;
                    }
                }
                prefetch_scales(group);
            }
        }

        // the next tile has landed, the next fragments are published, everyone is done with these
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
    }

    template <int PERTURB, bool CLAMP>
    __device__ __forceinline__ void pass(int t0, int n0, char *x0, char *x1, uint16_t *const (&yg)[kP],
                                         const float *const (&xs)[kP], const float (&s_row)[kWR])
    {
#pragma unroll
        for (int h = 0; h < kP; ++h)
#pragma unroll
            for (int i = 0; i < kMy; ++i)
#pragma unroll
                for (int r = 0; r < kWR; ++r) acc[h][i][r] = Acc{0, 0, 0, 0};
        group = 0;
        subs_to_group_end = subs_per_group;
        job_zero = false;
        if (!kI8) {
            // unit of the accumulators: scale of the group being accumulated (1 while that is zero)
#pragma unroll
            for (int r = 0; r < kWR; ++r) {
                s_cur[r] = f16_bits_to_f32(scales[r][0]);
                if (s_cur[r] == 0.0f) s_cur[r] = 1.0f;
            }
            job_zero = ((job_scales[0] & 0x7FFFu) == 0);
            prefetch_scales(0);
        }
        prepare_tile_offsets(t0);
        __syncthreads();   // the previous pass has finished reading LDS
        issue_tile(0, x0);
        raw_next = n_sub > 1 ? load_raw(1) : make_uint2(0u, 0u);
        publish(0, make_half<PERTURB, CLAMP>(0, load_raw(0), job_zero));
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();

        if constexpr (kStraight) {
            // every substep but the last generates the next substep's fragments under its MFMAs
            int s = 0;
            for (; s + 2 < n_sub; s += 2) {
                substep<PERTURB, CLAMP, 0, false>(s, x0, x1);
                substep<PERTURB, CLAMP, 1, false>(s + 1, x1, x0);
            }
            if (s + 1 < n_sub) {
                substep<PERTURB, CLAMP, 0, false>(s, x0, x1);
                substep<PERTURB, CLAMP, 1, true>(s + 1, x1, x0);
            } else {
                substep<PERTURB, CLAMP, 0, true>(s, x0, x1);
            }
        } else {
            for (int s = 0; s < n_sub; s += 2) {
                substep<PERTURB, CLAMP, 0, false>(s, x0, x1);
                if (s + 1 < n_sub) substep<PERTURB, CLAMP, 1, false>(s + 1, x1, x0);
            }
        }

#pragma unroll
        for (int h = 0; h < kP; ++h)
#pragma unroll
            for (int r = 0; r < kWR; ++r) {
                const int n = n0 + (wr * kWR + r) * 16 + ln;
                if (n >= a.out_features) continue;
#pragma unroll
                for (int i = 0; i < kMy; ++i) {
                    const int m = wm + i * kWM;
                    if (kMT % kWM != 0 && m >= kMT) continue;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int t = t0 + m * 16 + kc * 4 + j;
                        if (t < a.T) {
                            float v;
                            if constexpr (kI8) v = ((float)acc[h][i][r][j] * xs[h][t]) * s_row[r];
                            else v = acc[h][i][r][j] * s_cur[r];
                            yg[h][(size_t)t * a.out_features + n] = f32_to_bf16_rne(v);
                        }
                    }
                }
            }
    }
};

// BATCH: one launch covers several tensors (a layer's linears: same members, same token count);
// a block finds its tensor by bisection over the tensors' first slots in the per-XCD queues.
// Register budget: two workgroups per CU (4 waves per SIMD) also for the largest accumulator sets;
// three (6 waves per SIMD, 80 registers) for one member at up to 64 tokens, where a few values that
// only the prologue and the epilogue use go to scratch memory (none inside the substep loop).
template <int MODE, int TM, bool PAIRED, bool BATCH>
__global__ __launch_bounds__(waves_for(TM, PAIRED) * 64, ((TM >= 512 || (PAIRED && TM >= 128)) ? 4 : ((TM <= 64 && !PAIRED) ? 6 : 1))) void gemm_kernel(const GemmArgs args)
{
    using G = Gemm<MODE, TM, PAIRED>;
    constexpr int kP = G::kP;
    // separate arrays, not halves of one: reads of one tile buffer must not wait for the
    // asynchronous loads into the other, and the compiler tells them apart per LDS variable
    __shared__ __attribute__((aligned(1024))) char x0[kP * G::kTileBytes];
    __shared__ __attribute__((aligned(1024))) char x1[kP * G::kTileBytes];
    __shared__ __attribute__((aligned(16))) char bfrag[2 * kP * kFragBytes];

    // work item: a member, or an antithetic pair of members (PAIRED; a.entries then holds one record per pair)
    // this kernel's only parameter sits at the start of the kernel-argument segment
    ConstGemmArgs *ap = (ConstGemmArgs *)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t idx = 0;
    if (BATCH) {
        // Blocks are dealt round-robin over the 8 XCDs; XCD x runs slots 0, 1, 2, ... of its own
        // queue. Every tensor puts an eighth of its work items (a contiguous range, so that a
        // member's tiles share an L2) into each queue, one tensor after the other.
        ConstGemmArgs *descs = (ConstGemmArgs *)(uintptr_t)args.batch;   // read-only for the whole launch
        const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
        int lo = 0, hi = args.n_batch - 1;   // wave-uniform
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (descs[mid].work_begin <= slot) lo = mid;
            else hi = mid - 1;
        }
        ap = descs + lo;
        const uint32_t total = gemm_work_items_device(ap->out_features, ap->N, PAIRED);
        const uint32_t per_xcd = (total + 7u) / 8u;
        const uint32_t local = slot - ap->work_begin;
        idx = xcd * per_xcd + local;
        if (local >= per_xcd || idx >= total) return;
    }
    ConstGemmArgs &a = *ap;
    const uint32_t n_tiles = (a.out_features + kTileN - 1) / kTileN;
    if (!BATCH && !block_to_index(n_tiles * ((uint32_t)a.N / kP), idx)) return;
    const uint32_t member = idx / n_tiles;
    const uint32_t tile = idx - member * n_tiles;

    G g{a};
    g.lane = threadIdx.x & 63;
    g.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    g.wm = g.wave % G::kWM;
    g.wr = g.wave / G::kWM;
    g.jrg = g.wave / G::kParts;
    g.jpart = g.wave % G::kParts;
    g.ln = g.lane & 15;        // column of B / C within a row group
    g.kc = g.lane >> 4;        // k-chunk 0..3
    const int n0 = tile * kTileN;
    auto clamp_row = [&](int n) { return n < a.out_features ? n : a.out_features - 1; };   // clamp loads, skip stores
    g.en = a.entries[member];
    const int gs = a.group_size > 0 ? a.group_size : a.in_features;
    const int groups_per_row = a.in_features / gs;
    g.n_sub = (a.in_features + G::kSubK - 1) / G::kSubK;
    g.tail = G::kI8 && (a.in_features % 64) != 0;
    g.subs_per_group = gs / G::kSubK;            // bf16 modes: group_size is a multiple of 32
    float s_row[kWR];
#pragma unroll
    for (int r = 0; r < kWR; ++r) {
        const int n = clamp_row(n0 + (g.wr * kWR + r) * 16 + g.ln);
        g.scales[r] = (const uint16_t *)a.scales + (size_t)n * groups_per_row;
        s_row[r] = G::kI8 ? f16_bits_to_f32(((const uint16_t *)a.scales)[n]) : 1.0f;
        g.frag_rd[r] = (g.wr * kWR + r) * 1024 + g.lane * 16;
    }
    uint16_t *yg[kP];
    const float *xs[kP];
#pragma unroll
    for (int h = 0; h < kP; ++h) {
        const size_t m = (size_t)member * kP + h;
        g.xg[h] = (const char *)a.x + m * a.T * a.in_features * G::kElemBytes;
        yg[h] = (uint16_t *)a.y + m * a.T * a.out_features;
        xs[h] = G::kI8 ? a.x_scale + m * a.T : nullptr;
    }
    // noise job: part `jpart` of row group jrg's fragment: elements k0 .. k0+H-1, k0 = s*kSubK + kc*(kSubK/4) + jpart*H
    const int jn = clamp_row(n0 + g.jrg * 16 + g.ln);
    const int k0 = g.kc * (G::kSubK / 4) + g.jpart * G::H;
    const size_t elem0 = (size_t)jn * a.in_features + k0;
    g.job_scales = (const uint16_t *)a.scales + (size_t)jn * groups_per_row;
    g.wrow_lane = (const char *)a.qweight + (MODE == kBf16W4 ? (elem0 >> 1) : elem0);
    g.pair0 = (uint32_t)(elem0 >> 1);
    g.frag_wr = g.jrg * 1024 + g.lane * 16 + g.jpart * G::kPartBytes;
    g.a_off = (g.wm * 16 + g.ln) * kRowBytes + swizzle(g.ln, g.kc) * 16;
    g.bfrag = bfrag;
    // per member: 0 base weights, 1 +δ, 2 -δ (antithetic mirror); per pair: bit 0 = even member
    // perturbed, bit 1 = odd member perturbed
    const uint32_t mode = (a.sigma != 0.0f) ? g.en.fit_bits : 0u;
    g.keep[0] = (mode & 1u) ? 1.0f : 0.0f;
    g.keep[1] = (mode & 2u) ? 1.0f : 0.0f;
    g.qmin_f = (float)a.qmin;
    g.qmax_f = (float)(a.qmin + (int32_t)a.qspan);
    // |sigma*eps| <= 1.2 * 5.77 < 7: the 4-bit container clamp of δ cannot fire and is compiled out
    const bool clamp = !(a.sigma <= 1.2f);

    for (int t0 = 0; t0 < a.T; t0 += TM) {
        if constexpr (PAIRED) {
            if (mode == 0u) g.template pass<0, false>(t0, n0, x0, x1, yg, xs, s_row);
            else if (clamp) g.template pass<1, true>(t0, n0, x0, x1, yg, xs, s_row);
            else g.template pass<1, false>(t0, n0, x0, x1, yg, xs, s_row);
        } else {
            if (mode == 0u) g.template pass<0, false>(t0, n0, x0, x1, yg, xs, s_row);
            else if (clamp) {
                if (mode == 1u) g.template pass<1, true>(t0, n0, x0, x1, yg, xs, s_row);
                else g.template pass<-1, true>(t0, n0, x0, x1, yg, xs, s_row);
            } else {
                if (mode == 1u) g.template pass<1, false>(t0, n0, x0, x1, yg, xs, s_row);
                else g.template pass<-1, false>(t0, n0, x0, x1, yg, xs, s_row);
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

template <int MODE, int TM, bool PAIRED>
void launch_one(const GemmArgs &a, hipStream_t s)
{
    if (a.batch) {
        const unsigned blocks = a.work_begin * 8u;   // slots per XCD queue x 8 queues
        gemm_kernel<MODE, TM, PAIRED, true><<<blocks, waves_for(TM, PAIRED) * 64, 0, s>>>(a);
    } else {
        const uint32_t total = gemm_work_items(a.out_features, a.N, PAIRED);
        const unsigned blocks = ((total + 7u) / 8u) * 8u;
        gemm_kernel<MODE, TM, PAIRED, false><<<blocks, waves_for(TM, PAIRED) * 64, 0, s>>>(a);
    }
}

template <int MODE, bool PAIRED>
hipError_t launch_mode(const GemmArgs &a, hipStream_t s)
{
    if (a.T <= 16) launch_one<MODE, 16, PAIRED>(a, s);
    else if (a.T <= 32) launch_one<MODE, 32, PAIRED>(a, s);
    else if (a.T <= 64) launch_one<MODE, 64, PAIRED>(a, s);
    else if (a.T <= 128) launch_one<MODE, 128, PAIRED>(a, s);
    else if (a.T <= 256 || PAIRED) launch_one<MODE, 256, PAIRED>(a, s);
    else launch_one<MODE, 512, false>(a, s);
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

// A pair's workgroup holds the accumulators of both members. Up to 128 tokens per member that
// leaves room for two workgroups per CU and the shared draw wins (1.4-1.6x per launch). At 256
// tokens the 64 accumulator registers per lane take the whole CU: a single-tensor launch loses
// more on its small tensors than it gains on the large ones, a launch over a whole layer still
// gains (7 % on the 1.5B-model layer), so only batched launches pair up there. Longer token counts
// regenerate the draw per member.
bool gemm_pairs_supported(int32_t T, bool batched) { return T <= 128 || (batched && T <= 256); }

uint32_t gemm_work_items(int32_t out_features, int32_t N, bool paired)
{
    return (uint32_t)((out_features + kTileN - 1) / kTileN) * ((uint32_t)N / (paired ? 2u : 1u));
}

hipError_t launch_gemm(const GemmArgs &a, int bits, int act_mode, bool paired, hipStream_t s)
{
    if (paired) {
        if (!gemm_pairs_supported(a.T, a.batch != nullptr) || (a.N & 1)) return hipErrorInvalidValue;
        if (act_mode == 1) return launch_mode<kI8W8, true>(a, s);
        return bits == 4 ? launch_mode<kBf16W4, true>(a, s) : launch_mode<kBf16W8, true>(a, s);
    }
    if (act_mode == 1) return launch_mode<kI8W8, false>(a, s);
    return bits == 4 ? launch_mode<kBf16W4, false>(a, s) : launch_mode<kBf16W8, false>(a, s);
}

}  // namespace qes
