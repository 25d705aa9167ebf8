// C ABI of libqes (declared in include/qes.h): argument validation, staging of the small host
// arrays (seeds, fitnesses) into device memory in stream order, kernel launches.
#include <algorithm>
#include <cmath>
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/qes.h"
#include "qes_internal.hpp"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    (void)hipGetLastError();   // clear the sticky error of a failed launch
    return QES_ERR_HIP;
}

#define QES_HIP(expr)                                  \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) return hip_fail(e__);   \
    } while (0)

// ---- staging ring: host arrays -> pinned slot -> device slot, ordered on the caller's stream.
// Every slot is large enough for the largest request the ABI accepts (records of
// QES_MAX_HISTORY + 1 generations of QES_MAX_POPULATION members plus QES_MAX_BATCH descriptors), so
// the ring is allocated once, on the first staging call on a device, and nothing is allocated or
// freed on the call path afterwards. A slot is reused only after the event recorded behind its
// last consumer has completed. The mutex guards slot bookkeeping only: filling a slot, the copy,
// the launches and any wait for a slot's event happen outside it, so callers on different streams
// do not serialise behind each other.
constexpr int kSlots = 8;
constexpr int kMaxDevices = 16;
constexpr size_t kMaxDescBytes = sizeof(qes::GemmArgs) > sizeof(qes::TensorDesc) ? sizeof(qes::GemmArgs) : sizeof(qes::TensorDesc);
constexpr size_t kSlotBytes =
    (((size_t)(QES_MAX_HISTORY + 1) * QES_MAX_POPULATION * sizeof(qes::Entry) + (size_t)QES_MAX_BATCH * kMaxDescBytes) + 4095u) &
    ~(size_t)4095u;

struct Slot {
    void *host = nullptr;
    void *dev = nullptr;
    hipEvent_t ev = nullptr;
    bool in_flight = false;   // an event behind the slot's last consumer has been recorded
    bool held = false;        // a host thread is filling it
};

struct DeviceCtx {
    bool ready = false;
    Slot slots[kSlots];
    int next = 0;
};

std::mutex g_mu;
std::condition_variable g_cv;
DeviceCtx g_ctx[kMaxDevices];

int init_ring(DeviceCtx &c)   // caller holds g_mu; first staging call on this device only
{
    for (int i = 0; i < kSlots; ++i) {
        Slot &s = c.slots[i];
        if (!s.host) QES_HIP(hipHostMalloc(&s.host, kSlotBytes, hipHostMallocDefault));
        if (!s.dev) QES_HIP(hipMalloc(&s.dev, kSlotBytes));
        if (!s.ev) QES_HIP(hipEventCreateWithFlags(&s.ev, hipEventDisableTiming));
    }
    c.ready = true;
    return QES_OK;
}

// A slot the calling thread may fill: taken round-robin among the slots no other thread is
// filling; if its last consumer is still running, waits for it (outside the mutex).
int acquire_slot(size_t bytes, Slot **out)
{
    if (bytes > kSlotBytes) return QES_ERR_INVALID_ARG;   // cannot happen for arguments within the ABI limits
    int dev = 0;
    QES_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return QES_ERR_UNSUPPORTED;
    DeviceCtx &c = g_ctx[dev];
    Slot *s = nullptr;
    {
        std::unique_lock<std::mutex> lock(g_mu);
        if (!c.ready) {
            const int rc = init_ring(c);
            if (rc != QES_OK) return rc;
        }
        for (;;) {
            for (int i = 0; i < kSlots && !s; ++i) {
                Slot &cand = c.slots[(c.next + i) % kSlots];
                if (!cand.held) {
                    s = &cand;
                    c.next = (c.next + i + 1) % kSlots;
                }
            }
            if (s) break;
            g_cv.wait(lock);   // every slot is being filled by another thread
        }
        s->held = true;
    }
    if (s->in_flight) {
        const hipError_t e = hipEventSynchronize(s->ev);
        if (e != hipSuccess) {
            std::lock_guard<std::mutex> lock(g_mu);
            s->held = false;
            g_cv.notify_one();
            return hip_fail(e);
        }
        s->in_flight = false;
    }
    *out = s;
    return QES_OK;
}

// Hands the slot back. `enqueued`: device work that reads the slot was put on `stream`; the slot
// then stays busy until an event recorded now has completed. Returns the event record's status.
hipError_t release_slot(Slot *s, bool enqueued, hipStream_t stream)
{
    hipError_t e = hipSuccess;
    bool in_flight = false;
    if (enqueued) {
        e = hipEventRecord(s->ev, stream);
        if (e == hipSuccess) in_flight = true;
        else (void)hipStreamSynchronize(stream);   // no event to wait for later: drain the consumers now
    }
    std::lock_guard<std::mutex> lock(g_mu);
    s->in_flight = in_flight;
    s->held = false;
    g_cv.notify_one();
    return e;
}

// ---- the entry point that allocates nothing (qes_update_noalloc) keeps its (seed, fitness)
// records in this fixed device array instead of a ring slot. Each GPU holds its own copy at its
// own address; host code only ever uses the address hipGetSymbolAddress returned for the current
// device, never the array's name.
constexpr uint32_t kScratchRecords = QES_NOALLOC_MAX_RECORDS;
constexpr int kStageRecords = 240;   // records per staging launch: 3840 bytes of kernel arguments

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchRecords * sizeof(qes::Entry)];

namespace {

struct StageChunk {
    qes::Entry e[kStageRecords];
};

// Writes `count` records, passed by value in the kernel arguments, to dst[0..count). Host arrays
// reach the device this way without a copy engine, a pinned buffer or a memcpy node.
__global__ __launch_bounds__(256) void stage_records_kernel(const StageChunk chunk, qes::Entry *__restrict__ dst, int count)
{
    const int i = threadIdx.x;
    if (i < count) dst[i] = chunk.e[i];
}

void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int scratch_address(qes::Entry **out)
{
    int dev = 0;
    QES_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return QES_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        QES_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return QES_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = (qes::Entry *)g_scratch_ptr[dev];
    return QES_OK;
}

int tensor_check(const qes_tensor *w)
{
    if (!w || !w->qweight) return QES_ERR_INVALID_ARG;
    if (w->out_features <= 0 || w->in_features <= 0 || (w->in_features & 1)) return QES_ERR_INVALID_ARG;
    if (w->bits != 4 && w->bits != 8) return QES_ERR_INVALID_ARG;
    if (w->group_size < 0) return QES_ERR_INVALID_ARG;
    if (w->group_size > 0 && (w->in_features % w->group_size) != 0) return QES_ERR_INVALID_ARG;
    if (w->qmin > w->qmax) return QES_ERR_INVALID_ARG;
    if (w->bits == 4 && (w->qmin < -8 || w->qmax > 7)) return QES_ERR_INVALID_ARG;
    if (w->bits == 8 && (w->qmin < -128 || w->qmax > 127)) return QES_ERR_INVALID_ARG;
    if (((uintptr_t)w->qweight & 15u) != 0) return QES_ERR_INVALID_ARG;
    // the tensor kernels number threads and pairs in 32 bits: the last, partly filled workgroup of
    // the largest tensor must not wrap
    if ((uint64_t)w->out_features * (uint64_t)w->in_features > (1ull << 33) - 4096u) return QES_ERR_UNSUPPORTED;
    return QES_OK;
}

// Validates the update/replay scalars and fills the entry array (history first, current last).
// One record per member, or per antithetic pair (then `stride` = 2 fitnesses per record: the +δ
// member's in fit_bits, the -δ member's in pad). Also bounds |u| so that the float -> int
// conversion in the kernel can never overflow.
int fill_generation(qes::Entry *dst, const uint64_t *seeds, const float *fit, int32_t records, int stride,
                    double *abs_sum)
{
    for (int32_t i = 0; i < records; ++i) {
        uint32_t fb[2] = {0u, 0u};
        for (int k = 0; k < stride; ++k) {
            const float f = fit[(size_t)i * stride + k];
            if (!std::isfinite(f)) return QES_ERR_INVALID_ARG;
            *abs_sum += std::fabs((double)f);
            std::memcpy(&fb[k], &f, 4);
        }
        dst[i] = qes::Entry{(uint32_t)seeds[i], (uint32_t)(seeds[i] >> 32), fb[0], fb[1]};
    }
    return QES_OK;
}

int fill_entries(qes::Entry *dst, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                 const float *hist_fit, int32_t hist_len, int32_t N, bool antithetic, double c)
{
    const int stride = antithetic ? 2 : 1;
    const int32_t records = N / stride;
    double abs_sum = 0.0;
    for (int32_t tau = 0; tau < hist_len; ++tau) {
        const int rc = fill_generation(dst + (size_t)tau * records, hist_seeds + (size_t)tau * records,
                                       hist_fit + (size_t)tau * N, records, stride, &abs_sum);
        if (rc != QES_OK) return rc;
    }
    if (seeds_t) {
        const int rc = fill_generation(dst + (size_t)hist_len * records, seeds_t, fit_t, records, stride, &abs_sum);
        if (rc != QES_OK) return rc;
    }
    // |δ| <= 8 and 0 <= γ <= 1, so |u| <= |c|·8·Σ|F| over every generation replayed
    if (std::fabs(c) * 8.0 * abs_sum >= 1073741824.0) return QES_ERR_INVALID_ARG;
    return QES_OK;
}

// Argument checks shared by every single-tensor update / replay entry point.
int update_check(const qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                 const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                 const uint64_t *stats, const float *residual, int rmode, bool antithetic)
{
    const int rc = tensor_check(w);
    if (rc != QES_OK) return rc;
    if (N <= 0 || N > QES_MAX_POPULATION || hist_len < 0 || hist_len > QES_MAX_HISTORY) return QES_ERR_INVALID_ARG;
    if (antithetic && (N & 1)) return QES_ERR_INVALID_ARG;
    if (rmode >= 2 && hist_len != 0) return QES_ERR_INVALID_ARG;
    if (hist_len > 0 && (!hist_seeds || !hist_fit)) return QES_ERR_INVALID_ARG;
    if (rmode != 1 && (!seeds_t || !fit_t)) return QES_ERR_INVALID_ARG;
    if (rmode != 0 && rmode != 4 && (!residual || ((uintptr_t)residual & 15u) != 0)) return QES_ERR_INVALID_ARG;
    if (!(sigma > 0.0f) || !std::isfinite(sigma) || !std::isfinite(alpha)) return QES_ERR_INVALID_ARG;
    if (!(gamma >= 0.0f && gamma <= 1.0f)) return QES_ERR_INVALID_ARG;
    if (stats && ((uintptr_t)stats & 7u) != 0) return QES_ERR_INVALID_ARG;
    return QES_OK;
}

// Kernel arguments of a single-tensor update / replay launch (entries are filled in by the caller).
qes::UpdateArgs update_args(const qes_tensor *w, int32_t steps, int32_t records, float sigma, double c64, float gamma,
                            uint64_t *stats, float *residual, uint64_t round_seed)
{
    qes::UpdateArgs a{};
    a.qweight = w->qweight;
    a.entries = nullptr;
    a.residual = residual;
    a.stats = (unsigned long long *)stats;
    a.n_pairs = (uint32_t)(((uint64_t)w->out_features * (uint64_t)w->in_features) >> 1);
    a.steps = steps;
    a.N = records;
    a.sigma = sigma;
    a.c = (float)c64;
    a.gamma = gamma;
    a.qmin = w->qmin;
    a.qspan = (uint32_t)(w->qmax - w->qmin);
    a.tensor_id = w->tensor_id;
    a.round_k0 = (uint32_t)round_seed;
    a.round_k1 = (uint32_t)(round_seed >> 32);
    return a;
}

int update_common(const qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                  const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                  uint64_t *stats, float *residual, int rmode, bool antithetic, void *stream, uint64_t round_seed = 0)
{
    int rc = update_check(w, seeds_t, fit_t, hist_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, stats, residual, rmode,
                          antithetic);
    if (rc != QES_OK) return rc;
    const bool replay_only = (rmode == 1);
    const double c64 = (double)alpha / ((double)N * (double)sigma);
    const int32_t steps = hist_len + (replay_only ? 0 : 1);
    const int32_t records = antithetic ? N / 2 : N;   // one record per member, or per antithetic pair
    const size_t n_entries = (size_t)steps * (size_t)records;
    hipStream_t s = (hipStream_t)stream;
    qes::UpdateArgs a = update_args(w, steps, records, sigma, c64, gamma, stats, residual, round_seed);

    Slot *slot = nullptr;
    if (n_entries > 0) {
        rc = acquire_slot(n_entries * sizeof(qes::Entry), &slot);
        if (rc != QES_OK) return rc;
        rc = fill_entries((qes::Entry *)slot->host, replay_only ? nullptr : seeds_t, fit_t, hist_seeds, hist_fit,
                          hist_len, N, antithetic, c64);
        if (rc != QES_OK) {
            (void)release_slot(slot, false, s);
            return rc;
        }
        hipError_t ec = hipMemcpyAsync(slot->dev, slot->host, n_entries * sizeof(qes::Entry), hipMemcpyHostToDevice, s);
        if (ec != hipSuccess) {
            (void)release_slot(slot, true, s);
            return hip_fail(ec);
        }
        a.entries = (const qes::Entry *)slot->dev;
    }
    hipError_t e = qes::launch_update(a, w->bits, rmode, antithetic, s);
    if (slot) {
        // the slot is busy until everything enqueued so far (copy and kernel) has run
        const hipError_t e2 = release_slot(slot, true, s);
        if (e == hipSuccess) e = e2;
    }
    if (e != hipSuccess) return hip_fail(e);
    return QES_OK;
}

// Alg. 2 on every tensor of a list in one launch per weight width: the records are staged once,
// the tensors' descriptors behind them in the same slot.
int update_batch_common(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *seeds_t, const float *fit_t,
                        const uint64_t *hist_seeds, const float *hist_fit, int32_t hist_len, int32_t N, float sigma,
                        float alpha, float gamma, uint64_t *stats, bool antithetic, void *stream)
{
    if (!tensors || n_tensors <= 0 || n_tensors > QES_MAX_BATCH) return QES_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_tensors; ++i) {
        const int rc = tensor_check(&tensors[i]);
        if (rc != QES_OK) return rc;
    }
    if (N <= 0 || N > QES_MAX_POPULATION || hist_len < 0 || hist_len > QES_MAX_HISTORY) return QES_ERR_INVALID_ARG;
    if (antithetic && (N & 1)) return QES_ERR_INVALID_ARG;
    if (hist_len > 0 && (!hist_seeds || !hist_fit)) return QES_ERR_INVALID_ARG;
    if (!seeds_t || !fit_t) return QES_ERR_INVALID_ARG;
    if (!(sigma > 0.0f) || !std::isfinite(sigma) || !std::isfinite(alpha)) return QES_ERR_INVALID_ARG;
    if (!(gamma >= 0.0f && gamma <= 1.0f)) return QES_ERR_INVALID_ARG;
    if (stats && ((uintptr_t)stats & 7u) != 0) return QES_ERR_INVALID_ARG;

    const double c64 = (double)alpha / ((double)N * (double)sigma);
    const int32_t steps = hist_len + 1;
    const int32_t records = antithetic ? N / 2 : N;
    const size_t entry_bytes = (size_t)steps * (size_t)records * sizeof(qes::Entry);
    const size_t desc_bytes = (size_t)n_tensors * sizeof(qes::TensorDesc);
    hipStream_t s = (hipStream_t)stream;

    // descriptors grouped by weight width: [all INT4 tensors][all INT8 tensors], blocks numbered per group
    uint64_t blocks[2] = {0, 0};
    for (int32_t i = 0; i < n_tensors; ++i) {
        const uint64_t n_pairs = ((uint64_t)tensors[i].out_features * (uint64_t)tensors[i].in_features) >> 1;
        blocks[tensors[i].bits == 4 ? 0 : 1] += (n_pairs + 255u) / 256u;
    }
    if (blocks[0] >= (1ull << 31) || blocks[1] >= (1ull << 31)) return QES_ERR_UNSUPPORTED;

    Slot *slot = nullptr;
    int rc = acquire_slot(entry_bytes + desc_bytes, &slot);
    if (rc != QES_OK) return rc;
    rc = fill_entries((qes::Entry *)slot->host, seeds_t, fit_t, hist_seeds, hist_fit, hist_len, N, antithetic, c64);
    if (rc != QES_OK) {
        (void)release_slot(slot, false, s);
        return rc;
    }
    qes::TensorDesc *descs = (qes::TensorDesc *)((char *)slot->host + entry_bytes);
    int32_t count[2] = {0, 0};
    int32_t at = 0;
    for (int g = 0; g < 2; ++g) {
        const int bits = g == 0 ? 4 : 8;
        uint64_t first_block = 0;
        for (int32_t i = 0; i < n_tensors; ++i) {
            const qes_tensor &w = tensors[i];
            if (w.bits != bits) continue;
            const uint64_t n_pairs = ((uint64_t)w.out_features * (uint64_t)w.in_features) >> 1;
            descs[at++] = qes::TensorDesc{w.qweight, (uint32_t)n_pairs, (uint32_t)first_block, w.qmin,
                                          (uint32_t)(w.qmax - w.qmin), w.tensor_id, 0u};
            first_block += (n_pairs + 255u) / 256u;
            ++count[g];
        }
    }
    hipError_t e = hipMemcpyAsync(slot->dev, slot->host, entry_bytes + desc_bytes, hipMemcpyHostToDevice, s);

    qes::UpdateArgs a{};
    a.entries = (const qes::Entry *)slot->dev;
    a.stats = (unsigned long long *)stats;
    a.steps = steps;
    a.N = records;
    a.sigma = sigma;
    a.c = (float)c64;
    a.gamma = gamma;
    const qes::TensorDesc *dev_descs = (const qes::TensorDesc *)((const char *)slot->dev + entry_bytes);
    for (int g = 0; g < 2 && e == hipSuccess; ++g) {
        if (count[g] == 0) continue;
        a.descs = dev_descs + (g == 0 ? 0 : count[0]);
        a.n_tensors = count[g];
        e = qes::launch_update_batch(a, g == 0 ? 4 : 8, antithetic, (uint32_t)blocks[g], s);
    }
    const hipError_t e2 = release_slot(slot, true, s);
    if (e == hipSuccess) e = e2;
    if (e != hipSuccess) return hip_fail(e);
    return QES_OK;
}

// Alg. 2 on one tensor with the records staged through the fixed device array `scratch` by small
// kernels that carry them in their arguments: only kernel launches are enqueued, nothing is
// allocated, freed, copied by a copy engine or waited for.
int update_noalloc(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                   const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                   uint64_t *stats, void *stream)
{
    int rc = update_check(w, seeds_t, fit_t, hist_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, stats, nullptr, 0, false);
    if (rc != QES_OK) return rc;
    const int32_t steps = hist_len + 1;
    const uint64_t n_records = (uint64_t)steps * (uint64_t)N;
    if (n_records > kScratchRecords) return QES_ERR_TOO_LARGE;
    const double c64 = (double)alpha / ((double)N * (double)sigma);
    // every fitness finite, and |u| <= |c|·8·Σ|F| small enough for the float -> int conversion
    double abs_sum = 0.0;
    for (int32_t tau = 0; tau < steps; ++tau) {
        const float *f = tau < hist_len ? hist_fit + (size_t)tau * N : fit_t;
        for (int32_t i = 0; i < N; ++i) {
            if (!std::isfinite(f[i])) return QES_ERR_INVALID_ARG;
            abs_sum += std::fabs((double)f[i]);
        }
    }
    if (std::fabs(c64) * 8.0 * abs_sum >= 1073741824.0) return QES_ERR_INVALID_ARG;
    qes::Entry *dev_records = nullptr;
    rc = scratch_address(&dev_records);
    if (rc != QES_OK) return rc;

    hipStream_t s = (hipStream_t)stream;
    StageChunk chunk;
    for (uint64_t r0 = 0; r0 < n_records; r0 += kStageRecords) {
        const int count = (int)std::min<uint64_t>(kStageRecords, n_records - r0);
        for (int j = 0; j < count; ++j) {
            const uint64_t r = r0 + (uint64_t)j;
            const int32_t tau = (int32_t)(r / (uint64_t)N), i = (int32_t)(r % (uint64_t)N);
            const uint64_t sd = tau < hist_len ? hist_seeds[(size_t)tau * N + i] : seeds_t[i];
            const float f = tau < hist_len ? hist_fit[(size_t)tau * N + i] : fit_t[i];
            uint32_t fb;
            std::memcpy(&fb, &f, 4);
            chunk.e[j] = qes::Entry{(uint32_t)sd, (uint32_t)(sd >> 32), fb, 0u};
        }
        stage_records_kernel<<<1, 256, 0, s>>>(chunk, dev_records + r0, count);
        QES_HIP(hipGetLastError());
    }
    qes::UpdateArgs a = update_args(w, steps, N, sigma, c64, gamma, stats, nullptr, 0);
    a.entries = dev_records;
    QES_HIP(qes::launch_update(a, w->bits, 0, false, s));
    return QES_OK;
}

}  // namespace

extern "C" {

int qes_abi_version(void) { return 1; }

int qes_last_hip_error(void) { return g_last_hip_error; }

const char *qes_status_string(int status)
{
    switch (status) {
    case QES_OK: return "ok";
    case QES_ERR_INVALID_ARG: return "invalid argument";
    case QES_ERR_UNSUPPORTED: return "unsupported configuration";
    case QES_ERR_HIP: return "HIP runtime error";
    case QES_ERR_WORKSPACE: return "workspace missing or too small";
    case QES_ERR_TOO_LARGE: return "request exceeds the fixed scratch of the entry point that allocates nothing";
    default: return "unknown status";
    }
}

int qes_noise_words(uint64_t seed, uint32_t tensor_id, uint64_t pair_begin, uint64_t n_pairs, uint32_t *out4,
                    void *stream)
{
    if (n_pairs == 0) return QES_OK;
    if (!out4 || ((uintptr_t)out4 & 15u) != 0 || n_pairs > (1ull << 31)) return QES_ERR_INVALID_ARG;
    if (pair_begin + n_pairs < pair_begin) return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_noise_words(seed, tensor_id, pair_begin, n_pairs, out4, (hipStream_t)stream));
    return QES_OK;
}

int qes_noise_gauss(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems, float *out,
                    void *stream)
{
    if (n_elems == 0) return QES_OK;
    if (!out || n_elems > (1ull << 31) || elem_begin + n_elems < elem_begin) return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_noise_gauss(seed, tensor_id, elem_begin, n_elems, out, (hipStream_t)stream));
    return QES_OK;
}

int qes_noise_delta(uint64_t seed, uint32_t tensor_id, uint64_t elem_begin, uint64_t n_elems, float sigma,
                    int8_t *out, void *stream)
{
    if (n_elems == 0) return QES_OK;
    if (!out || n_elems > (1ull << 31) || elem_begin + n_elems < elem_begin) return QES_ERR_INVALID_ARG;
    if (!(sigma >= 0.0f) || !std::isfinite(sigma)) return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_noise_delta(seed, tensor_id, elem_begin, n_elems, sigma, out, (hipStream_t)stream));
    return QES_OK;
}

int qes_noise_from_words(const uint32_t *words4, uint64_t n, float sigma, float *eps2, int8_t *delta2, void *stream)
{
    if (n == 0) return QES_OK;
    if (!words4 || ((uintptr_t)words4 & 15u) != 0 || n > (1ull << 31)) return QES_ERR_INVALID_ARG;
    if ((eps2 && ((uintptr_t)eps2 & 7u) != 0) || (delta2 && ((uintptr_t)delta2 & 1u) != 0)) return QES_ERR_INVALID_ARG;
    if (!(sigma >= 0.0f) || !std::isfinite(sigma)) return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_noise_from_words(words4, n, sigma, eps2, delta2, (hipStream_t)stream));
    return QES_OK;
}

size_t qes_gemm_workspace_bytes(const qes_tensor *w, int32_t N, int32_t T, int32_t act_mode)
{
    if (!w || act_mode != 1 || N <= 0 || T <= 0) return 0;
    const size_t rows = (size_t)N * (size_t)T;
    const size_t xq = (rows * (size_t)w->in_features + 15u) & ~(size_t)15u;
    return xq + rows * sizeof(float);
}

// Validation of one tensor's GEMM arguments and the kernel arguments that follow from them
// (activations and entries are filled in by the caller).
static int gemm_prepare(const qes_tensor *w, const void *x, void *y, int32_t N, int32_t T, float sigma, int32_t act_mode,
                        bool antithetic, qes::GemmArgs *out)
{
    int rc = tensor_check(w);
    if (rc != QES_OK) return rc;
    if (antithetic && (N & 1)) return QES_ERR_INVALID_ARG;
    if (!w->scales || !x || !y || N <= 0 || N > QES_MAX_POPULATION || T <= 0) return QES_ERR_INVALID_ARG;
    if (((uintptr_t)x & 15u) != 0 || ((uintptr_t)y & 1u) != 0 || ((uintptr_t)w->scales & 1u) != 0)
        return QES_ERR_INVALID_ARG;
    if (!(sigma >= 0.0f) || !std::isfinite(sigma)) return QES_ERR_INVALID_ARG;
    if (act_mode != 0 && act_mode != 1) return QES_ERR_INVALID_ARG;
    if (act_mode == 1 && (w->bits != 8 || w->group_size != 0)) return QES_ERR_INVALID_ARG;
    if ((w->in_features % 32) != 0 || (w->group_size % 32) != 0) return QES_ERR_UNSUPPORTED;
    // one member's activations are addressed with 32-bit byte offsets inside the kernel
    if ((uint64_t)T * (uint64_t)w->in_features * 2u >= (1ull << 32)) return QES_ERR_UNSUPPORTED;
    if ((uint64_t)N * (uint64_t)T * (uint64_t)w->in_features >= (1ull << 40)) return QES_ERR_UNSUPPORTED;
    qes::GemmArgs a{};
    a.qweight = w->qweight;
    a.scales = w->scales;
    a.x = x;
    a.x_scale = nullptr;
    a.y = y;
    a.out_features = w->out_features;
    a.in_features = w->in_features;
    a.group_size = w->group_size;
    a.N = N;
    a.T = T;
    a.sigma = sigma;
    a.qmin = w->qmin;
    a.qspan = (uint32_t)(w->qmax - w->qmin);
    a.tensor_id = w->tensor_id;
    *out = a;
    return QES_OK;
}

// bytes of one quantised activation tensor [rows, in_features] int8 + its per-row scales
static size_t quantised_bytes(size_t rows, int32_t in_features)
{
    return ((rows * (size_t)in_features + 15u) & ~(size_t)15u) + ((rows * sizeof(float) + 15u) & ~(size_t)15u);
}

// One record per member, or per antithetic pair when a workgroup serves both members of a pair
// from one draw (then bit 0 / bit 1 of the mode say which member is perturbed); otherwise mode
// 0 = base weights, 1 = +δ, 2 = -δ (mirrored member regenerating its pair's draw).
static int32_t fill_gemm_entries(qes::Entry *ent, const uint64_t *seeds, const uint8_t *perturb_mask, int32_t N,
                                 bool antithetic, bool paired)
{
    const int32_t records = paired ? N / 2 : N;
    auto on = [&](int32_t i) { return !(perturb_mask != nullptr && perturb_mask[i] == 0); };
    for (int32_t i = 0; i < records; ++i) {
        if (paired) {
            const uint64_t sd = seeds[i];
            const uint32_t mode = (on(2 * i) ? 1u : 0u) | (on(2 * i + 1) ? 2u : 0u);
            ent[i] = qes::Entry{(uint32_t)sd, (uint32_t)(sd >> 32), mode, 0u};
        } else {
            const uint64_t sd = antithetic ? seeds[i / 2] : seeds[i];
            const uint32_t mode = !on(i) ? 0u : ((antithetic && (i & 1)) ? 2u : 1u);
            ent[i] = qes::Entry{(uint32_t)sd, (uint32_t)(sd >> 32), mode, 0u};
        }
    }
    return records;
}

static int gemm_common(const qes_tensor *w, const uint64_t *seeds, const uint8_t *perturb_mask, int32_t N,
                       float sigma, const void *x, int32_t T, void *y, int32_t act_mode, void *workspace,
                       size_t workspace_bytes, bool antithetic, void *stream)
{
    if (!seeds) return QES_ERR_INVALID_ARG;
    qes::GemmArgs a{};
    int rc = gemm_prepare(w, x, y, N, T, sigma, act_mode, antithetic, &a);
    if (rc != QES_OK) return rc;
    hipStream_t s = (hipStream_t)stream;

    int8_t *xq = nullptr;
    float *xs = nullptr;
    if (act_mode == 1) {
        const size_t need = qes_gemm_workspace_bytes(w, N, T, act_mode);
        if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u) != 0) return QES_ERR_WORKSPACE;
        const size_t rows = (size_t)N * (size_t)T;
        xq = (int8_t *)workspace;
        xs = (float *)((char *)workspace + ((rows * (size_t)w->in_features + 15u) & ~(size_t)15u));
        a.x = xq;
        a.x_scale = xs;
    }

    Slot *slot = nullptr;
    rc = acquire_slot((size_t)N * sizeof(qes::Entry), &slot);
    if (rc != QES_OK) return rc;
    // antithetic pairs share one draw inside a workgroup when both members' accumulators fit
    // and two workgroups still share a CU; longer token counts regenerate the draw per member
    const bool paired = antithetic && qes::gemm_pairs_supported(T, false);
    const int32_t records = fill_gemm_entries((qes::Entry *)slot->host, seeds, perturb_mask, N, antithetic, paired);
    // every check that can refuse the call lies above: from here on device work is enqueued
    hipError_t e = hipSuccess;
    if (act_mode == 1) e = qes::launch_quantize_activations(x, xq, xs, (int64_t)N * (int64_t)T, w->in_features, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync(slot->dev, slot->host, (size_t)records * sizeof(qes::Entry), hipMemcpyHostToDevice, s);
    a.entries = (const qes::Entry *)slot->dev;
    if (e == hipSuccess) e = qes::launch_gemm(a, w->bits, act_mode, paired, s);
    const hipError_t e2 = release_slot(slot, true, s);
    if (e == hipSuccess) e = e2;
    if (e != hipSuccess) return hip_fail(e);
    return QES_OK;
}

// The distinct activation tensors of a batch (linears of a layer share inputs): index of x[i] in
// the list of distinct (pointer, in_features) pairs, in order of first appearance.
static int32_t distinct_inputs(const qes_tensor *tensors, int32_t n, const void *const *x, int32_t *which)
{
    int32_t n_distinct = 0;
    for (int32_t i = 0; i < n; ++i) {
        int32_t found = -1;
        for (int32_t j = 0; j < i && found < 0; ++j)
            if (x[j] == x[i] && tensors[j].in_features == tensors[i].in_features) found = which[j];
        which[i] = found >= 0 ? found : n_distinct++;
    }
    return n_distinct;
}

size_t qes_gemm_batch_workspace_bytes(const qes_tensor *tensors, int32_t n_tensors, const void *const *x, int32_t N,
                                      int32_t T, int32_t act_mode)
{
    if (!tensors || !x || n_tensors <= 0 || n_tensors > QES_MAX_BATCH || act_mode != 1 || N <= 0 || T <= 0) return 0;
    std::vector<int32_t> which;
    try {
        which.resize((size_t)n_tensors);
    } catch (...) {
        return 0;
    }
    const int32_t n_distinct = distinct_inputs(tensors, n_tensors, x, which.data());
    size_t total = 0;
    for (int32_t d = 0; d < n_distinct; ++d)
        for (int32_t i = 0; i < n_tensors; ++i)
            if (which[i] == d) {
                total += quantised_bytes((size_t)N * (size_t)T, tensors[i].in_features);
                break;
            }
    return total;
}

static int gemm_batch_common(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *seeds,
                             const uint8_t *perturb_mask, int32_t N, float sigma, const void *const *x, int32_t T,
                             void *const *y, int32_t act_mode, void *workspace, size_t workspace_bytes, bool antithetic,
                             void *stream)
{
    if (!tensors || !x || !y || !seeds || n_tensors <= 0 || n_tensors > QES_MAX_BATCH) return QES_ERR_INVALID_ARG;
    std::vector<qes::GemmArgs> args((size_t)n_tensors);
    for (int32_t i = 0; i < n_tensors; ++i) {
        const int rc = gemm_prepare(&tensors[i], x[i], y[i], N, T, sigma, act_mode, antithetic, &args[(size_t)i]);
        if (rc != QES_OK) return rc;
    }
    hipStream_t s = (hipStream_t)stream;
    const size_t rows = (size_t)N * (size_t)T;

    // W8A8: every distinct activation tensor gets one region of the workspace and is quantised once
    struct Quantise {
        const void *x;
        char *region;
        int32_t in_features;
    };
    std::vector<Quantise> quantise;
    if (act_mode == 1) {
        const size_t need = qes_gemm_batch_workspace_bytes(tensors, n_tensors, x, N, T, act_mode);
        if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u) != 0) return QES_ERR_WORKSPACE;
        std::vector<int32_t> which((size_t)n_tensors);
        const int32_t n_distinct = distinct_inputs(tensors, n_tensors, x, which.data());
        std::vector<char *> region((size_t)n_distinct, nullptr);
        char *at = (char *)workspace;
        for (int32_t i = 0; i < n_tensors; ++i) {
            const int32_t in_f = tensors[i].in_features;
            char *&r = region[(size_t)which[i]];
            if (!r) {
                r = at;
                at += quantised_bytes(rows, in_f);
                quantise.push_back(Quantise{x[i], r, in_f});
            }
            args[(size_t)i].x = r;
            args[(size_t)i].x_scale = (const float *)(r + ((rows * (size_t)in_f + 15u) & ~(size_t)15u));
        }
    }

    const bool paired = antithetic && qes::gemm_pairs_supported(T, true);
    const int32_t records = paired ? N / 2 : N;
    const size_t entry_bytes = (size_t)records * sizeof(qes::Entry);
    const size_t desc_bytes = (size_t)n_tensors * sizeof(qes::GemmArgs);

    // Launch order: grouped by weight width; inside a group the tensors with the longest rows first
    // (their workgroups run longest, the short ones then fill the end of the launch). Each tensor
    // takes ceil(W/8) slots in every XCD's queue.
    std::vector<int32_t> order[2];
    uint64_t work[2] = {0, 0};
    for (int g = 0; g < 2; ++g) {
        const int bits = g == 0 ? 4 : 8;
        for (int32_t i = 0; i < n_tensors; ++i)
            if (tensors[i].bits == bits) order[g].push_back(i);
        std::stable_sort(order[g].begin(), order[g].end(),
                         [&](int32_t p, int32_t q) { return tensors[p].in_features > tensors[q].in_features; });
        for (int32_t i : order[g]) work[g] += (qes::gemm_work_items(tensors[i].out_features, N, paired) + 7u) / 8u;
        if (work[g] >= (1ull << 27)) return QES_ERR_UNSUPPORTED;
    }

    Slot *slot = nullptr;
    int rc = acquire_slot(entry_bytes + desc_bytes, &slot);
    if (rc != QES_OK) return rc;
    fill_gemm_entries((qes::Entry *)slot->host, seeds, perturb_mask, N, antithetic, paired);
    qes::GemmArgs *descs = (qes::GemmArgs *)((char *)slot->host + entry_bytes);
    int32_t at = 0;
    for (int g = 0; g < 2; ++g) {
        uint64_t begin = 0;
        for (int32_t i : order[g]) {
            qes::GemmArgs d = args[(size_t)i];
            d.entries = (const qes::Entry *)slot->dev;
            d.work_begin = (uint32_t)begin;
            begin += (qes::gemm_work_items(d.out_features, N, paired) + 7u) / 8u;
            descs[at++] = d;
        }
    }
    // every check that can refuse the call lies above: from here on device work is enqueued
    hipError_t e = hipSuccess;
    for (size_t q = 0; q < quantise.size() && e == hipSuccess; ++q) {
        const Quantise &z = quantise[q];
        float *xs = (float *)(z.region + ((rows * (size_t)z.in_features + 15u) & ~(size_t)15u));
        e = qes::launch_quantize_activations(z.x, (int8_t *)z.region, xs, (int64_t)rows, z.in_features, s);
    }
    if (e == hipSuccess) e = hipMemcpyAsync(slot->dev, slot->host, entry_bytes + desc_bytes, hipMemcpyHostToDevice, s);
    const qes::GemmArgs *dev_descs = (const qes::GemmArgs *)((const char *)slot->dev + entry_bytes);
    for (int g = 0; g < 2 && e == hipSuccess; ++g) {
        if (order[g].empty()) continue;
        qes::GemmArgs a{};
        a.N = N;
        a.T = T;
        a.batch = dev_descs + (g == 0 ? 0 : order[0].size());
        a.n_batch = (int32_t)order[g].size();
        a.work_begin = (uint32_t)work[g];   // slots per XCD queue of this launch
        e = qes::launch_gemm(a, g == 0 ? 4 : 8, act_mode, paired, s);
    }
    const hipError_t e2 = release_slot(slot, true, s);
    if (e == hipSuccess) e = e2;
    if (e != hipSuccess) return hip_fail(e);
    return QES_OK;
}

int qes_perturbed_qgemm(const qes_tensor *w, const uint64_t *seeds, const uint8_t *perturb_mask, int32_t N,
                        float sigma, const void *x, int32_t T, void *y, int32_t act_mode, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    return gemm_common(w, seeds, perturb_mask, N, sigma, x, T, y, act_mode, workspace, workspace_bytes, false, stream);
}

int qes_perturbed_qgemm_antithetic(const qes_tensor *w, const uint64_t *pair_seeds, const uint8_t *perturb_mask,
                                   int32_t N, float sigma, const void *x, int32_t T, void *y, int32_t act_mode,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_common(w, pair_seeds, perturb_mask, N, sigma, x, T, y, act_mode, workspace, workspace_bytes, true,
                       stream);
}

int qes_perturbed_qgemm_batch(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *seeds,
                              const uint8_t *perturb_mask, int32_t N, float sigma, const void *const *x, int32_t T,
                              void *const *y, int32_t act_mode, void *workspace, size_t workspace_bytes, void *stream)
{
    try {
        return gemm_batch_common(tensors, n_tensors, seeds, perturb_mask, N, sigma, x, T, y, act_mode, workspace,
                                 workspace_bytes, false, stream);
    } catch (...) {   // host memory for the launch tables could not be obtained; nothing was enqueued
        return QES_ERR_UNSUPPORTED;
    }
}

int qes_perturbed_qgemm_batch_antithetic(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *pair_seeds,
                                         const uint8_t *perturb_mask, int32_t N, float sigma, const void *const *x,
                                         int32_t T, void *const *y, int32_t act_mode, void *workspace,
                                         size_t workspace_bytes, void *stream)
{
    try {
        return gemm_batch_common(tensors, n_tensors, pair_seeds, perturb_mask, N, sigma, x, T, y, act_mode, workspace,
                                 workspace_bytes, true, stream);
    } catch (...) {
        return QES_ERR_UNSUPPORTED;
    }
}

int qes_update(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
               const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
               uint64_t *stats, void *stream)
{
    return update_common(w, seeds_t, fit_t, hist_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, stats, nullptr,
                         0, false, stream);
}

int qes_update_noalloc(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, const uint64_t *hist_seeds,
                       const float *hist_fit, int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                       uint64_t *stats, void *stream)
{
    return update_noalloc(w, seeds_t, fit_t, hist_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, stats, stream);
}

int qes_update_antithetic(qes_tensor *w, const uint64_t *pair_seeds_t, const float *fit_t,
                          const uint64_t *hist_pair_seeds, const float *hist_fit, int32_t hist_len, int32_t N,
                          float sigma, float alpha, float gamma, uint64_t *stats, void *stream)
{
    return update_common(w, pair_seeds_t, fit_t, hist_pair_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, stats,
                         nullptr, 0, true, stream);
}

int qes_update_batch(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *seeds_t, const float *fit_t,
                     const uint64_t *hist_seeds, const float *hist_fit, int32_t hist_len, int32_t N, float sigma,
                     float alpha, float gamma, uint64_t *stats, void *stream)
{
    return update_batch_common(tensors, n_tensors, seeds_t, fit_t, hist_seeds, hist_fit, hist_len, N, sigma, alpha, gamma,
                               stats, false, stream);
}

int qes_update_batch_antithetic(const qes_tensor *tensors, int32_t n_tensors, const uint64_t *pair_seeds_t,
                                const float *fit_t, const uint64_t *hist_pair_seeds, const float *hist_fit,
                                int32_t hist_len, int32_t N, float sigma, float alpha, float gamma, uint64_t *stats,
                                void *stream)
{
    return update_batch_common(tensors, n_tensors, pair_seeds_t, fit_t, hist_pair_seeds, hist_fit, hist_len, N, sigma,
                               alpha, gamma, stats, true, stream);
}

int qes_replay_residual(const qes_tensor *w, const uint64_t *hist_seeds, const float *hist_fit, int32_t hist_len,
                        int32_t N, float sigma, float alpha, float gamma, float *residual, void *stream)
{
    return update_common(w, nullptr, nullptr, hist_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, nullptr,
                         residual, 1, false, stream);
}

int qes_replay_residual_antithetic(const qes_tensor *w, const uint64_t *hist_pair_seeds, const float *hist_fit,
                                   int32_t hist_len, int32_t N, float sigma, float alpha, float gamma,
                                   float *residual, void *stream)
{
    return update_common(w, nullptr, nullptr, hist_pair_seeds, hist_fit, hist_len, N, sigma, alpha, gamma, nullptr,
                         residual, 1, true, stream);
}

int qes_update_full_residual(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                             float alpha, float gamma, float *e_state, uint64_t *stats, void *stream)
{
    return update_common(w, seeds_t, fit_t, nullptr, nullptr, 0, N, sigma, alpha, gamma, stats, e_state, 2, false,
                         stream);
}

int qes_update_full_residual_f16(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                 float alpha, float gamma, uint16_t *e_state_f16, uint64_t *stats, void *stream)
{
    return update_common(w, seeds_t, fit_t, nullptr, nullptr, 0, N, sigma, alpha, gamma, stats, (float *)e_state_f16, 3,
                         false, stream);
}

int qes_update_stochastic_rounding(qes_tensor *w, const uint64_t *seeds_t, const float *fit_t, int32_t N, float sigma,
                                   float alpha, uint64_t round_seed, uint64_t *stats, void *stream)
{
    return update_common(w, seeds_t, fit_t, nullptr, nullptr, 0, N, sigma, alpha, 0.0f, stats, nullptr, 4, false,
                         stream, round_seed);
}

int qes_normalize_fitness(const float *reward, int32_t N, float *fit)
{
    if (!reward || !fit || N <= 0) return QES_ERR_INVALID_ARG;
    // running mean and sum of squared deviations, updated member by member (Welford), in fp64
    double mean = 0.0, m2 = 0.0;
    for (int32_t i = 0; i < N; ++i) {
        const double r = (double)reward[i];
        const double before = r - mean;
        mean += before / (double)(i + 1);
        m2 += before * (r - mean);
    }
    const double spread = std::sqrt(m2 / (double)N);   // population standard deviation
    const bool flat = N < 2 || !(spread > 0.0);
    for (int32_t i = 0; i < N; ++i) fit[i] = flat ? 0.0f : (float)(((double)reward[i] - mean) / spread);
    return QES_OK;
}

int qes_bench_noise(int32_t mode, uint64_t n_threads, int32_t iters, float sigma, uint32_t *sink, void *stream)
{
    if ((mode != 0 && mode != 1) || !sink || n_threads == 0 || n_threads > (1ull << 31) || iters < 0)
        return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_bench_noise(mode, n_threads, iters, sigma, sink, (hipStream_t)stream));
    return QES_OK;
}

int qes_bench_mfma(int32_t mode, uint32_t n_blocks, int32_t iters, uint32_t *sink, void *stream)
{
    if ((mode != 0 && mode != 1) || !sink || n_blocks == 0 || n_blocks > (1u << 20) || iters < 0) return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_bench_mfma(mode, n_blocks, iters, sink, (hipStream_t)stream));
    return QES_OK;
}

int qes_bench_copy(const void *src, void *dst, size_t n_bytes, void *stream)
{
    if (!src || !dst || (n_bytes & 15u) != 0 || ((uintptr_t)src & 15u) != 0 || ((uintptr_t)dst & 15u) != 0)
        return QES_ERR_INVALID_ARG;
    QES_HIP(qes::launch_bench_copy(src, dst, n_bytes, (hipStream_t)stream));
    return QES_OK;
}

}  // extern "C"
