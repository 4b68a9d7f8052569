// Host side of the ABS-SGD hot-path library: argument checks, the ragged
// layout's chunk table, the double-buffer context, and the C ABI.  The kernels
// and their launch functions live in the launch_*.hip units (abs_host.hpp).
// The C ABI and the arithmetic contract are stated in include/abs_sgd.h.
#include "abs_host.hpp"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <vector>

using namespace absh;
using absk::ADAM;
using absk::Job;
using absk::MAX_JOBS;
using absk::SGD;
using absk::SGD_DC;
using absk::SGD_DCM;

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return ABS_EHIP;
}

#define ABS_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return hip_fail(e_);      \
    } while (0)

inline bool aligned_to(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Do [a, a + an) and [b, b + bn) share a byte?
inline bool overlap(const void *a, int64_t an, const void *b, int64_t bn)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return an > 0 && bn > 0 && a0 < b0 + (uintptr_t)bn && b0 < a0 + (uintptr_t)an;
}

inline int launch_status()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return ABS_OK;
}

// Process-wide defaults; a context may carry settings of its own.  Atomics, so that
// a launch racing with one of the setters reads either the old or the new value.
std::atomic<int> g_blocks_per_cu{0}, g_max_rows{ABS_MAX_ROWS};
std::atomic<int> g_policy_acc{-1}, g_policy_upd{-1};
std::atomic<int64_t> g_slice_bytes{ABS_SLICE_BYTES};

inline Tuning process_tuning()
{
    return Tuning{g_blocks_per_cu.load(std::memory_order_relaxed), g_max_rows.load(std::memory_order_relaxed),
                  g_policy_acc.load(std::memory_order_relaxed), g_policy_upd.load(std::memory_order_relaxed),
                  g_slice_bytes.load(std::memory_order_relaxed)};
}

inline bool tuning_ok(int blocks_per_cu, int max_rows) { return blocks_per_cu >= 0 && blocks_per_cu <= 32 && max_rows >= 0; }
inline bool policy_ok(int a, int u) { return a >= -1 && a <= 1 && u >= -1 && u <= 1; }

// counts -> compacted list of non-empty workers and their total.
struct Combine {
    int idx[ABS_MAX_K];
    int n = 0;
    int64_t M = 0;
};

int plan_combine(const int64_t *counts, int K, Combine &c)
{
    if (!counts || K < 1 || K > ABS_MAX_K) return ABS_EINVAL;
    for (int k = 0; k < K; ++k) {
        if (counts[k] < 0) return ABS_EINVAL;
        if (counts[k] > 0) {
            if (c.M > std::numeric_limits<int64_t>::max() - counts[k]) return ABS_EINVAL;
            c.M += counts[k];
            c.idx[c.n++] = k;
        }
    }
    return c.M == 0 ? ABS_EMPTY : ABS_OK;
}

// Hyper-parameters of the rules in one struct.
Hyper hyper_sgd(float lr, float mu, float wd, float lambda, float lr_prev = 0.f)
{
    Hyper h = {};
    h.lr = lr; h.mu = mu; h.wd = wd; h.lambda = lambda; h.nlr_prev = -lr_prev;
    return h;
}

int hyper_adam(Hyper &h, float lr, float beta1, float beta2, float eps, float wd, int64_t step)
{
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f)) return ABS_EINVAL;
    h = Hyper{};
    h.lr = lr; h.wd = wd; h.beta1 = beta1; h.beta2 = beta2; h.eps = eps;
    h.omb1 = 1.0f - beta1;
    h.omb2 = 1.0f - beta2;
    h.bc1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    h.bc2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    return ABS_OK;
}

int launch_sync_flat(const Tuning &tu, int rule, float *x, float *s1, float *s2, const float *const *ptrs, int n,
                     int64_t P, const Hyper &h, int vec_ok, hipStream_t s)
{
    switch (rule) {
    case SGD: return launch_sync_flat_r<SGD>(tu, x, s1, s2, ptrs, n, P, h, vec_ok, s);
    case SGD_DC: return launch_sync_flat_r<SGD_DC>(tu, x, s1, s2, ptrs, n, P, h, vec_ok, s);
    case ADAM: return launch_sync_flat_r<ADAM>(tu, x, s1, s2, ptrs, n, P, h, vec_ok, s);
    case SGD_DCM: return launch_sync_flat_r<SGD_DCM>(tu, x, s1, s2, ptrs, n, P, h, vec_ok, s);
    default: return ABS_EINVAL;
    }
}

int launch_sync_ragged(const Tuning &tu, int rule, const RaggedView &L, float *const *xt, float *const *s1t,
                       float *const *s2t, const float *const *const *tabs, int n, const Hyper &h, hipStream_t s)
{
    switch (rule) {
    case SGD: return launch_sync_ragged_r<SGD>(tu, L, xt, s1t, s2t, tabs, n, h, s);
    case SGD_DC: return launch_sync_ragged_r<SGD_DC>(tu, L, xt, s1t, s2t, tabs, n, h, s);
    case ADAM: return launch_sync_ragged_r<ADAM>(tu, L, xt, s1t, s2t, tabs, n, h, s);
    case SGD_DCM: return launch_sync_ragged_r<SGD_DCM>(tu, L, xt, s1t, s2t, tabs, n, h, s);
    default: return ABS_EINVAL;
    }
}

}  // namespace

// ---------------------------------------------------------------- ragged types

struct abs_layout {
    std::vector<int64_t> sizes;
    std::vector<Chunk> chunks;
    int64_t total = 0;
    int tile = ROW;                      // elements per chunk, a multiple of ROW
    // Device copies and the LARS scratch (first chunk of every tensor, T + 1 entries;
    // per-chunk sums of squares; per-tensor step factors): made by abs_layout_upload,
    // which creating a tensor set over the layout calls, so no launch ever allocates.
    mutable Chunk *d_chunks = nullptr;
    mutable int64_t *d_sizes = nullptr;
    mutable int32_t *d_chunk_begin = nullptr;
    mutable double *d_partials = nullptr;
    mutable float *d_step = nullptr;
    mutable int device = -1;             // -1: not uploaded
};

struct abs_tensorset {
    const abs_layout *layout = nullptr;
    abs_dtype elem = ABS_F32;
    std::vector<void *> ptrs;
    void **d_tab = nullptr;
};

struct abs_ctx {
    int K = 0;
    int64_t P = 0;                       // flat form
    abs_layout *layout = nullptr;        // ragged form (else null)
    std::vector<float *> acc[2];         // flat: [generation][k]
    std::vector<const abs_tensorset *> set[2];
    std::vector<int64_t> counts[2];
    int cur = 0;
    std::vector<hipStream_t> s_acc;      // worker k accumulates on s_acc[slot[k]]
    hipStream_t s_upd = nullptr;
    std::vector<hipEvent_t> ev_acc;      // one per accumulate stream
    hipEvent_t ev_upd = nullptr;
    bool joins = false;                  // more than one distinct stream in use

    std::vector<int> slot;               // worker k accumulates on s_acc[slot[k]]
    std::vector<int64_t> launches;       // accumulate launches of worker k in the current step
    float lr_applied = 0.f;              // step size of the last abs_ctx_sync_update_dcm* call; 0 after an empty one

    // settings of this context's calls; where not set, the process-wide ones at the time of the call
    bool own_shape = false, own_policy = false;
    int blocks_per_cu = 0, max_rows = ABS_MAX_ROWS, policy_acc = -1, policy_upd = -1;

    hipStream_t stream_of(int k) const { return s_acc[(size_t)slot[(size_t)k]]; }

    Tuning tuning() const
    {
        Tuning t = process_tuning();
        if (own_shape) { t.blocks_per_cu = blocks_per_cu; t.max_rows = max_rows; }
        if (own_policy) { t.policy_acc = policy_acc; t.policy_upd = policy_upd; }
        return t;
    }
};

namespace {

void layout_free_device(const abs_layout *L)
{
    if (L->d_chunks) (void)hipFree(L->d_chunks);
    if (L->d_sizes) (void)hipFree(L->d_sizes);
    if (L->d_chunk_begin) (void)hipFree(L->d_chunk_begin);
    if (L->d_partials) (void)hipFree(L->d_partials);
    if (L->d_step) (void)hipFree(L->d_step);
    L->d_chunks = nullptr;
    L->d_sizes = nullptr;
    L->d_chunk_begin = nullptr;
    L->d_partials = nullptr;
    L->d_step = nullptr;
    L->device = -1;
}

int scratch_on_current_device(LarsScratch &sc);

// Copies the tables to the current device and allocates the LARS scratch.  Blocking;
// called when a tensor set is created (or explicitly), never from a launch.
int layout_upload(const abs_layout *L)
{
    static std::mutex upload_mutex;      // two threads may make their first tensor sets over one layout at once
    std::lock_guard<std::mutex> lock(upload_mutex);
    int dev = 0;
    ABS_HIP(hipGetDevice(&dev));
    if (L->device >= 0) return L->device == dev ? ABS_OK : ABS_EINVAL;
    const size_t T = L->sizes.size(), C = L->chunks.size();
    std::vector<int32_t> begin(T + 1, 0);
    for (const Chunk &c : L->chunks) begin[(size_t)c.tensor + 1] += 1;
    for (size_t t = 0; t < T; ++t) begin[t + 1] += begin[t];
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&L->d_sizes), T * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&L->d_chunk_begin), (T + 1) * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&L->d_step), T * sizeof(float));
    if (e == hipSuccess && C > 0) e = hipMalloc(reinterpret_cast<void **>(&L->d_chunks), C * sizeof(Chunk));
    if (e == hipSuccess && C > 0) e = hipMalloc(reinterpret_cast<void **>(&L->d_partials), 2 * C * sizeof(double));
    if (e == hipSuccess) e = hipMemcpy(L->d_sizes, L->sizes.data(), T * sizeof(int64_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(L->d_chunk_begin, begin.data(), (T + 1) * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess && C > 0) e = hipMemcpy(L->d_chunks, L->chunks.data(), C * sizeof(Chunk), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        layout_free_device(L);
        return hip_fail(e);
    }
    L->device = dev;
    // Set-up time on this device: look the fixed scratch array's address up now, so that the
    // allocation-free entry point has nothing left to ask the runtime for (its first call may
    // then already be inside a graph capture).  A failure here is reported by that call.
    LarsScratch unused;
    (void)scratch_on_current_device(unused);
    return ABS_OK;
}

// The layout's device tables for a launch on the current device.  Never allocates:
// a layout that no tensor set was ever made over cannot reach a launch.
int layout_view(const abs_layout *L, RaggedView &v)
{
    int dev = 0;
    ABS_HIP(hipGetDevice(&dev));
    if (L->device != dev) return ABS_EINVAL;
    v.chunks = L->d_chunks;
    v.sizes = L->d_sizes;
    v.nchunks = (unsigned)L->chunks.size();
    v.ntensors = (int)L->sizes.size();
    v.tile = L->tile;
    v.total = L->total;
    return ABS_OK;
}

bool set_ok(const abs_tensorset *s, const abs_layout *L) { return s && s->layout == L; }

// ------------------------------------------------------------------ flat

// If a HIP error stops a call that needs several launches, *count has advanced by
// the samples of the launches already enqueued.
int accumulate_batch_flat(const Tuning &tu, float *acc, const void *const *grads, abs_dtype grad_dtype, int J,
                          int64_t P, const int64_t *n_samples, int64_t *count, hipStream_t s)
{
    if (!count || !grads || !n_samples || J < 1 || P < 0 || *count < 0) return ABS_EINVAL;
    if (grad_dtype != ABS_F32 && grad_dtype != ABS_BF16) return ABS_EINVAL;
    int64_t total = *count;
    for (int j = 0; j < J; ++j) {
        if (n_samples[j] <= 0 || total > std::numeric_limits<int64_t>::max() - n_samples[j]) return ABS_EINVAL;
        total += n_samples[j];
    }
    if (P == 0) {
        *count = total;
        return ABS_OK;
    }
    if (!acc || !aligned_to(acc, 4)) return ABS_EINVAL;
    const int64_t gsz = grad_dtype == ABS_BF16 ? 2 : 4;
    int vec_ok = aligned_to(acc, 16);
    for (int j = 0; j < J; ++j) {
        if (!grads[j] || !aligned_to(grads[j], (uintptr_t)gsz)) return ABS_EINVAL;
        if (overlap(acc, 4 * P, grads[j], gsz * P)) return ABS_EINVAL;
        vec_ok = vec_ok && aligned_to(grads[j], grad_dtype == ABS_BF16 ? 8 : 16);
    }
    for (int j0 = 0; j0 < J; j0 += ABS_MAX_BATCH) {
        const int jn = J - j0 < ABS_MAX_BATCH ? J - j0 : ABS_MAX_BATCH;
        float nf[ABS_MAX_BATCH];
        int64_t samples = 0;
        for (int j = 0; j < jn; ++j) {
            nf[j] = (float)n_samples[j0 + j];
            samples += n_samples[j0 + j];
        }
        int rc = launch_accumulate_flat(tu, acc, grads + j0, nf, jn, grad_dtype, P, *count == 0 ? 1 : 0, vec_ok, s);
        if (rc != ABS_OK) return rc;
        rc = launch_status();
        if (rc != ABS_OK) return rc;
        *count += samples;
    }
    return ABS_OK;
}

// s1: momentum (SGD rules) or first moment (ADAM); s2: previous iterate (SGD_DC)
// or second moment (ADAM), unused otherwise.
int sync_update_flat(const Tuning &tu, int rule, float *params, float *s1, float *s2, const float *const *acc,
                     const int64_t *counts, int K, int64_t P, Hyper h, hipStream_t s)
{
    if (!acc || P < 0) return ABS_EINVAL;
    const bool has2 = rule == SGD_DC || rule == ADAM;
    Combine c;
    int rc = plan_combine(counts, K, c);
    if (rc != ABS_OK && rc != ABS_EMPTY) return rc;
    const bool empty = rc == ABS_EMPTY;
    if (empty && rule != SGD_DC) return ABS_EMPTY;
    if (P == 0) return empty ? ABS_EMPTY : ABS_OK;
    if (!params || !s1 || !aligned_to(params, 4) || !aligned_to(s1, 4)) return ABS_EINVAL;
    if (has2 && (!s2 || !aligned_to(s2, 4))) return ABS_EINVAL;
    const int64_t nb = 4 * P;
    if (overlap(params, nb, s1, nb)) return ABS_EINVAL;
    if (has2 && (overlap(s2, nb, params, nb) || overlap(s2, nb, s1, nb))) return ABS_EINVAL;
    if (empty) {
        // x_{t+1} = x_t: the previous-iterate buffer must still advance
        rc = launch_copy_flat(tu, s2, params, P, s);
        if (rc != ABS_OK) return rc;
        rc = launch_status();
        return rc == ABS_OK ? ABS_EMPTY : rc;
    }
    const float *ptrs[ABS_MAX_K];
    bool vec = aligned_to(params, 16) && aligned_to(s1, 16) && (!has2 || aligned_to(s2, 16));
    for (int j = 0; j < c.n; ++j) {
        const float *p = acc[c.idx[j]];
        if (!p || !aligned_to(p, 4)) return ABS_EINVAL;
        // what the pass writes must not be what it reads of another vector
        if (overlap(p, nb, params, nb) || overlap(p, nb, s1, nb) || (has2 && overlap(p, nb, s2, nb))) return ABS_EINVAL;
        vec = vec && aligned_to(p, 16);
        ptrs[j] = p;
    }
    h.M = (float)c.M;
    rc = launch_sync_flat(tu, rule, params, s1, has2 ? s2 : nullptr, ptrs, c.n, P, h, vec ? 1 : 0, s);
    if (rc != ABS_OK) return rc;
    return launch_status();
}

// ---------------------------------------------------------------- ragged

int accumulate_batch_mt(const Tuning &tu, const abs_layout *L, const abs_tensorset *acc,
                        const abs_tensorset *const *grads, int J, const int64_t *n_samples, int64_t *count,
                        hipStream_t s)
{
    if (!L || !set_ok(acc, L) || acc->elem != ABS_F32 || !grads || !n_samples || J < 1) return ABS_EINVAL;
    if (!count || *count < 0) return ABS_EINVAL;
    int64_t total = *count;
    for (int j = 0; j < J; ++j) {
        if (!set_ok(grads[j], L) || grads[j]->elem != grads[0]->elem || grads[j] == acc) return ABS_EINVAL;
        if (n_samples[j] <= 0 || total > std::numeric_limits<int64_t>::max() - n_samples[j]) return ABS_EINVAL;
        total += n_samples[j];
    }
    if (L->chunks.empty()) {
        *count = total;
        return ABS_OK;
    }
    RaggedView V;
    int rc = layout_view(L, V);
    if (rc != ABS_OK) return rc;
    float *const *at = reinterpret_cast<float *const *>(acc->d_tab);
    for (int j0 = 0; j0 < J; j0 += ABS_MAX_BATCH) {
        const int jn = J - j0 < ABS_MAX_BATCH ? J - j0 : ABS_MAX_BATCH;
        float nf[ABS_MAX_BATCH];
        const void *const *gt[ABS_MAX_BATCH];
        int64_t samples = 0;
        for (int j = 0; j < jn; ++j) {
            nf[j] = (float)n_samples[j0 + j];
            samples += n_samples[j0 + j];
            gt[j] = reinterpret_cast<const void *const *>(grads[j0 + j]->d_tab);
        }
        rc = launch_accumulate_ragged(tu, V, at, gt, nf, jn, grads[0]->elem, *count == 0 ? 1 : 0, s);
        if (rc != ABS_OK) return rc;
        rc = launch_status();
        if (rc != ABS_OK) return rc;
        *count += samples;
    }
    return ABS_OK;
}

int sync_update_mt(const Tuning &tu, int rule, const abs_layout *L, const abs_tensorset *params,
                   const abs_tensorset *s1, const abs_tensorset *s2, const abs_tensorset *const *acc,
                   const int64_t *counts, int K, Hyper h, hipStream_t s)
{
    if (!L || !acc) return ABS_EINVAL;
    const bool has2 = rule == SGD_DC || rule == ADAM;
    Combine c;
    int rc = plan_combine(counts, K, c);
    if (rc != ABS_OK && rc != ABS_EMPTY) return rc;
    const bool empty = rc == ABS_EMPTY;
    if (empty && rule != SGD_DC) return ABS_EMPTY;
    if (!set_ok(params, L) || !set_ok(s1, L) || params == s1) return ABS_EINVAL;
    if (params->elem != ABS_F32 || s1->elem != ABS_F32) return ABS_EINVAL;
    if (has2 && (!set_ok(s2, L) || s2 == params || s2 == s1 || s2->elem != ABS_F32)) return ABS_EINVAL;
    const float *const *tabs[ABS_MAX_K];
    for (int j = 0; j < c.n; ++j) {
        const abs_tensorset *a = acc[c.idx[j]];
        if (!set_ok(a, L) || a->elem != ABS_F32 || a == params || a == s1 || (has2 && a == s2)) return ABS_EINVAL;
        tabs[j] = reinterpret_cast<const float *const *>(a->d_tab);
    }
    if (L->chunks.empty()) return empty ? ABS_EMPTY : ABS_OK;
    RaggedView V;
    rc = layout_view(L, V);
    if (rc != ABS_OK) return rc;
    float *const *xt = reinterpret_cast<float *const *>(params->d_tab);
    float *const *pt = has2 ? reinterpret_cast<float *const *>(s2->d_tab) : nullptr;
    if (empty) {
        rc = launch_copy_ragged(V, pt, xt, s);
        if (rc == ABS_OK) rc = launch_status();
        return rc == ABS_OK ? ABS_EMPTY : rc;
    }
    h.M = (float)c.M;
    rc = launch_sync_ragged(tu, rule, V, xt, reinterpret_cast<float *const *>(s1->d_tab), pt, tabs, c.n, h, s);
    if (rc != ABS_OK) return rc;
    return launch_status();
}

// LARS with its scratch taken from `sc`; when begin_on_device, the first-chunk table
// is first rebuilt in sc.chunk_begin from the chunk table (one small launch).
int sync_update_lars(const abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                     const abs_tensorset *gbar, const abs_tensorset *const *acc, const int64_t *counts, int K,
                     float lr, float mu, float wd, float eta, const LarsScratch *sc, bool begin_on_device,
                     hipStream_t s)
{
    if (!L || !acc) return ABS_EINVAL;
    Combine c;
    int rc = plan_combine(counts, K, c);
    if (rc != ABS_OK) return rc;
    if (!set_ok(params, L) || !set_ok(momentum, L) || !set_ok(gbar, L)) return ABS_EINVAL;
    if (params == momentum || gbar == params || gbar == momentum) return ABS_EINVAL;
    if (params->elem != ABS_F32 || momentum->elem != ABS_F32 || gbar->elem != ABS_F32) return ABS_EINVAL;
    const float *const *tabs[ABS_MAX_K];
    for (int j = 0; j < c.n; ++j) {
        const abs_tensorset *a = acc[c.idx[j]];
        if (!set_ok(a, L) || a->elem != ABS_F32 || a == gbar || a == params || a == momentum) return ABS_EINVAL;
        tabs[j] = reinterpret_cast<const float *const *>(a->d_tab);
    }
    if (L->chunks.empty()) return ABS_OK;
    RaggedView V;
    rc = layout_view(L, V);
    if (rc != ABS_OK) return rc;
    LarsScratch own{L->d_partials, L->d_step, L->d_chunk_begin};
    if (!sc) sc = &own;
    if (begin_on_device) {
        rc = launch_lars_chunk_begin(V, sc->chunk_begin, s);
        if (rc == ABS_OK) rc = launch_status();
        if (rc != ABS_OK) return rc;
    }
    rc = launch_lars(process_tuning(), V, reinterpret_cast<float *const *>(params->d_tab),
                     reinterpret_cast<float *const *>(momentum->d_tab),
                     reinterpret_cast<float *const *>(gbar->d_tab), tabs, c.n, (float)c.M, lr, mu, wd, eta, *sc, s);
    if (rc != ABS_OK) return rc;
    return launch_status();
}

// ------------------------------------------------- allocation-free scratch
//
// The LARS launches need per-chunk partial sums, per-tensor step factors and the
// first-chunk table.  abs_sync_update_lars_mt keeps them in memory the layout
// allocated; abs_sync_update_lars_mt_noalloc, for callers that may not allocate,
// keeps them in this fixed array instead.  Every GPU the library runs on holds its
// own copy at its own address until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress: the address the kernels
// get is the one that call returns for the current device.
struct StaticScratch {
    double partials[2 * ABS_NOALLOC_MAX_CHUNKS];
    float step[ABS_NOALLOC_MAX_TENSORS];
    int32_t chunk_begin[ABS_NOALLOC_MAX_TENSORS + 1];
};

static __device__ __attribute__((used)) __align__(256) unsigned char scratch[sizeof(StaticScratch)];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on device d; null until asked

// Device address of the scratch array on the current device, looked up once per device.
int scratch_on_current_device(LarsScratch &sc)
{
    int dev = 0;
    ABS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ABS_EINVAL;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            ABS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) return ABS_EINVAL;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    StaticScratch *st = static_cast<StaticScratch *>(ptr);       // device memory: only addresses are formed here
    sc.partials = st->partials;
    sc.step = st->step;
    sc.chunk_begin = st->chunk_begin;
    return ABS_OK;
}

// ------------------------------------------------------------- job lists
//
// One worker's share of a step, in device terms (flat: buffers; ragged: pointer tables).
struct Work {
    void *acc;
    const void *const *g;          // HOST array of J device pointers (flat) or pointer tables (ragged)
    const int64_t *n;
    int J;
    int64_t *count;
};

// Launch r carries, for every job that still has gradients, its next `fold` of them;
// at most MAX_JOBS jobs travel in one launch.  Per job the gradients are applied in
// order with the roundings of single launches, whatever `fold` is.
template <class Launch>
int run_jobs(const Work *w, int nw, int fold, Launch launch)
{
    int maxJ = 0;
    for (int i = 0; i < nw; ++i) maxJ = std::max(maxJ, w[i].J);
    for (int j0 = 0; j0 < maxJ; j0 += fold) {
        int i = 0;
        while (i < nw) {
            JobList list;
            std::memset(&list, 0, sizeof list);
            int64_t samples[MAX_JOBS];
            int owner[MAX_JOBS];
            int nj = 0, jmax = 0;
            for (; i < nw && nj < MAX_JOBS; ++i) {
                const int jn = std::min(fold, w[i].J - j0);
                if (jn <= 0) continue;
                Job &jb = list.job[nj];
                jb.acc = w[i].acc;
                jb.J = jn;
                jb.first = *w[i].count == 0 ? 1 : 0;
                samples[nj] = 0;
                for (int j = 0; j < jn; ++j) {
                    jb.g[j] = w[i].g[j0 + j];
                    jb.n[j] = (float)w[i].n[j0 + j];
                    samples[nj] += w[i].n[j0 + j];
                }
                owner[nj] = i;
                jmax = std::max(jmax, jn);
                ++nj;
            }
            if (nj == 0) continue;
            int rc = launch(list, nj, jmax);
            if (rc != ABS_OK) return rc;
            rc = launch_status();
            if (rc != ABS_OK) return rc;
            for (int q = 0; q < nj; ++q) *w[owner[q]].count += samples[q];
        }
    }
    return ABS_OK;
}

// Checks shared by the flat and ragged job lists; counts may not overflow.
int check_job_counts(int J, const int64_t *n_samples, const int64_t *count)
{
    if (J < 0 || !count || *count < 0 || (J > 0 && !n_samples)) return ABS_EINVAL;
    int64_t total = *count;
    for (int j = 0; j < J; ++j) {
        if (n_samples[j] <= 0 || total > std::numeric_limits<int64_t>::max() - n_samples[j]) return ABS_EINVAL;
        total += n_samples[j];
    }
    return ABS_OK;
}

int accumulate_jobs_flat(const Tuning &tu, const abs_job *jobs, int njobs, abs_dtype grad_dtype, int64_t P,
                         int fold, hipStream_t s)
{
    if (!jobs || njobs < 1 || njobs > ABS_MAX_K || P < 0 || fold < 1 || fold > ABS_MAX_BATCH) return ABS_EINVAL;
    if (grad_dtype != ABS_F32 && grad_dtype != ABS_BF16) return ABS_EINVAL;
    const int64_t gsz = grad_dtype == ABS_BF16 ? 2 : 4;
    Work w[ABS_MAX_K];
    for (int i = 0; i < njobs; ++i) {
        const abs_job &jb = jobs[i];
        int rc = check_job_counts(jb.J, jb.n_samples, jb.count);
        if (rc != ABS_OK) return rc;
        if (jb.J > 0 && !jb.grads) return ABS_EINVAL;
        for (int q = 0; q < i; ++q)
            if (jobs[q].count == jb.count) return ABS_EINVAL;
        if (P > 0 && jb.J > 0) {
            if (!jb.acc || !aligned_to(jb.acc, 4)) return ABS_EINVAL;
            for (int j = 0; j < jb.J; ++j)
                if (!jb.grads[j] || !aligned_to(jb.grads[j], (uintptr_t)gsz)) return ABS_EINVAL;
        }
        w[i] = Work{jb.acc, jb.grads, jb.n_samples, jb.J, jb.count};
    }
    if (P > 0) {
        // every accumulator is written: none may share bytes with another job's or with any gradient
        for (int i = 0; i < njobs; ++i) {
            if (jobs[i].J == 0) continue;
            for (int q = 0; q < njobs; ++q) {
                if (jobs[q].J == 0) continue;
                if (q < i && overlap(jobs[i].acc, 4 * P, jobs[q].acc, 4 * P)) return ABS_EINVAL;
                for (int j = 0; j < jobs[q].J; ++j)
                    if (overlap(jobs[i].acc, 4 * P, jobs[q].grads[j], gsz * P)) return ABS_EINVAL;
            }
        }
    }
    if (P == 0) {
        for (int i = 0; i < njobs; ++i)
            for (int j = 0; j < jobs[i].J; ++j) *jobs[i].count += jobs[i].n_samples[j];
        return ABS_OK;
    }
    return run_jobs(w, njobs, fold, [&](const JobList &list, int nj, int jmax) {
        return launch_accumulate_jobs_flat(tu, list, nj, jmax, grad_dtype, P, s);
    });
}

int accumulate_jobs_mt(const Tuning &tu, const abs_layout *L, const abs_job_mt *jobs, int njobs, int fold,
                       hipStream_t s)
{
    if (!L || !jobs || njobs < 1 || njobs > ABS_MAX_K || fold < 1 || fold > ABS_MAX_BATCH) return ABS_EINVAL;
    Work w[ABS_MAX_K];
    std::vector<const void *> tabs;          // per job, its gradients' device pointer tables
    size_t ngrads = 0;
    for (int i = 0; i < njobs; ++i) ngrads += jobs[i].J > 0 ? (size_t)jobs[i].J : 0;
    tabs.reserve(ngrads);
    int elem = -1;
    for (int i = 0; i < njobs; ++i) {
        const abs_job_mt &jb = jobs[i];
        int rc = check_job_counts(jb.J, jb.n_samples, jb.count);
        if (rc != ABS_OK) return rc;
        if (jb.J > 0 && (!jb.grads || !set_ok(jb.acc, L) || jb.acc->elem != ABS_F32)) return ABS_EINVAL;
        for (int q = 0; q < i; ++q)
            if (jobs[q].count == jb.count || (jb.J > 0 && jobs[q].J > 0 && jobs[q].acc == jb.acc)) return ABS_EINVAL;
        const size_t first_tab = tabs.size();
        for (int j = 0; j < jb.J; ++j) {
            const abs_tensorset *g = jb.grads[j];
            if (!set_ok(g, L)) return ABS_EINVAL;
            if (elem < 0) elem = (int)g->elem;
            if ((int)g->elem != elem) return ABS_EINVAL;
            for (int q = 0; q < njobs; ++q)
                if (jobs[q].J > 0 && jobs[q].acc == g) return ABS_EINVAL;
            tabs.push_back(g->d_tab);
        }
        w[i] = Work{jb.J > 0 ? jb.acc->d_tab : nullptr, tabs.data() + first_tab, jb.n_samples, jb.J, jb.count};
    }
    if (L->chunks.empty() || elem < 0) {
        for (int i = 0; i < njobs; ++i)
            for (int j = 0; j < jobs[i].J; ++j) *jobs[i].count += jobs[i].n_samples[j];
        return ABS_OK;
    }
    RaggedView V;
    int rc = layout_view(L, V);
    if (rc != ABS_OK) return rc;
    return run_jobs(w, njobs, fold, [&](const JobList &list, int nj, int jmax) {
        return launch_accumulate_jobs_ragged(tu, V, list, nj, jmax, (abs_dtype)elem, s);
    });
}

}  // namespace

// =========================================================================
// C ABI
// =========================================================================
extern "C" {

int abs_version(void) { return 200; }

int abs_last_hip_error(void) { return g_last_hip_error; }

const char *abs_error_string(int rc)
{
    switch (rc) {
    case ABS_OK: return "ok";
    case ABS_EMPTY: return "nothing to apply (total sample count is zero)";
    case ABS_EINVAL: return "invalid argument";
    case ABS_EHIP: return "HIP runtime call failed (see abs_last_hip_error)";
    default: return "unknown return code";
    }
}

int64_t abs_row_elems(void) { return ROW; }

int abs_set_launch_tuning(int blocks_per_cu, int max_rows_per_tile)
{
    if (!tuning_ok(blocks_per_cu, max_rows_per_tile)) return ABS_EINVAL;
    g_blocks_per_cu.store(blocks_per_cu, std::memory_order_relaxed);
    g_max_rows.store(max_rows_per_tile, std::memory_order_relaxed);
    return ABS_OK;
}

int abs_set_launch_slice_bytes(int64_t bytes)
{
    if (bytes < 0) return ABS_EINVAL;
    g_slice_bytes.store(bytes, std::memory_order_relaxed);
    return ABS_OK;
}

int64_t abs_launch_count(void) { return t_launches; }

int64_t abs_slice_workgroups(int64_t workgroups, int64_t bytes, int resident_workgroups)
{
    if (workgroups < 0 || bytes < 0 || resident_workgroups < 1) return ABS_EINVAL;
    return slice_wgs(process_tuning(), workgroups, bytes, resident_workgroups);
}

int abs_set_cache_policy(int accumulate_mode, int update_mode)
{
    if (!policy_ok(accumulate_mode, update_mode)) return ABS_EINVAL;
    g_policy_acc.store(accumulate_mode, std::memory_order_relaxed);
    g_policy_upd.store(update_mode, std::memory_order_relaxed);
    return ABS_OK;
}

// ------------------------------------------------------------------ flat

int abs_accumulate_batch(float *acc, const void *const *grads, abs_dtype grad_dtype, int J, int64_t P,
                         const int64_t *n_samples, int64_t *count, void *stream)
{
    return accumulate_batch_flat(process_tuning(), acc, grads, grad_dtype, J, P, n_samples, count,
                                 static_cast<hipStream_t>(stream));
}

int abs_accumulate(float *acc, const void *grad, abs_dtype grad_dtype, int64_t P,
                   int64_t n_samples, int64_t *count, void *stream)
{
    const void *grads[1] = {grad};
    return abs_accumulate_batch(acc, grads, grad_dtype, 1, P, &n_samples, count, stream);
}

int abs_accumulate_jobs(const abs_job *jobs, int njobs, abs_dtype grad_dtype, int64_t P, int fold, void *stream)
{
    return accumulate_jobs_flat(process_tuning(), jobs, njobs, grad_dtype, P, fold, static_cast<hipStream_t>(stream));
}

int abs_sync_update(float *params, float *momentum, const float *const *acc,
                    const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                    void *stream)
{
    return sync_update_flat(process_tuning(), SGD, params, momentum, nullptr, acc, counts, K, P,
                            hyper_sgd(lr, mu, wd, 0.f), static_cast<hipStream_t>(stream));
}

int abs_sync_update_dc(float *params, float *params_prev, float *momentum, const float *const *acc,
                       const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                       float lambda, void *stream)
{
    return sync_update_flat(process_tuning(), SGD_DC, params, momentum, params_prev, acc, counts, K, P,
                            hyper_sgd(lr, mu, wd, lambda), static_cast<hipStream_t>(stream));
}

int abs_sync_update_dcm(float *params, float *momentum, const float *const *acc, const int64_t *counts,
                        int K, int64_t P, float lr, float mu, float wd, float lambda, float lr_prev,
                        void *stream)
{
    return sync_update_flat(process_tuning(), SGD_DCM, params, momentum, nullptr, acc, counts, K, P,
                            hyper_sgd(lr, mu, wd, lambda, lr_prev), static_cast<hipStream_t>(stream));
}

int abs_sync_update_adam(float *params, float *exp_avg, float *exp_avg_sq, const float *const *acc,
                         const int64_t *counts, int K, int64_t P, float lr, float beta1, float beta2,
                         float eps, float wd, int64_t step, void *stream)
{
    Hyper h;
    int rc = hyper_adam(h, lr, beta1, beta2, eps, wd, step);
    if (rc != ABS_OK) return rc;
    return sync_update_flat(process_tuning(), ADAM, params, exp_avg, exp_avg_sq, acc, counts, K, P, h,
                            static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------- ragged

int abs_layout_create(abs_layout **out, int T, const int64_t *sizes)
{
    if (!out || T < 1 || !sizes) return ABS_EINVAL;
    abs_layout *L = new (std::nothrow) abs_layout;
    if (!L) return ABS_EINVAL;
    int64_t rows = 0;
    for (int t = 0; t < T; ++t) {
        if (sizes[t] < 0 || L->total > std::numeric_limits<int64_t>::max() - sizes[t]) {
            delete L;
            return ABS_EINVAL;
        }
        L->total += sizes[t];
        rows += rows_of(sizes[t]);
    }
    // one tile size for the whole layout, from the accumulate kernel's residency
    const Tuning tu = process_tuning();
    const int64_t tile = choose_tile(rows, acc_resident(tu), tu.max_rows);
    int64_t nchunks = 0;
    for (int t = 0; t < T; ++t) nchunks += tiles_for(sizes[t], tile);
    if (tile > kMaxTile || nchunks > kMaxGrid) { delete L; return ABS_EINVAL; }
    L->tile = (int)tile;
    L->sizes.assign(sizes, sizes + T);
    L->chunks.reserve((size_t)nchunks);
    // Tensor order, tile order within a tensor: consecutive workgroups stream
    // consecutive memory of one tensor.
    for (int t = 0; t < T; ++t)
        for (int64_t i = 0, n = tiles_for(sizes[t], tile); i < n; ++i)
            L->chunks.push_back(Chunk{(int32_t)t, (int32_t)i});
    *out = L;
    return ABS_OK;
}

int abs_layout_upload(const abs_layout *L)
{
    if (!L) return ABS_EINVAL;
    return layout_upload(L);
}

int abs_layout_destroy(abs_layout *L)
{
    if (!L) return ABS_EINVAL;
    layout_free_device(L);
    delete L;
    return ABS_OK;
}

int abs_layout_num_tensors(const abs_layout *L) { return L ? (int)L->sizes.size() : ABS_EINVAL; }
int64_t abs_layout_total(const abs_layout *L) { return L ? L->total : ABS_EINVAL; }
int64_t abs_layout_num_chunks(const abs_layout *L) { return L ? (int64_t)L->chunks.size() : ABS_EINVAL; }
int64_t abs_layout_tile(const abs_layout *L) { return L ? L->tile : ABS_EINVAL; }

int abs_layout_chunk(const abs_layout *L, int64_t c, int *tensor, int64_t *offset, int64_t *len)
{
    if (!L || c < 0 || c >= (int64_t)L->chunks.size() || !tensor || !offset || !len) return ABS_EINVAL;
    const Chunk ch = L->chunks[(size_t)c];
    *tensor = ch.tensor;
    *offset = (int64_t)ch.index * L->tile;
    const int64_t rest = L->sizes[(size_t)ch.tensor] - *offset;
    *len = rest < L->tile ? rest : L->tile;
    return ABS_OK;
}

int abs_tensorset_create(abs_tensorset **out, const abs_layout *L, void *const *ptrs, abs_dtype elem)
{
    if (!out || !L || !ptrs) return ABS_EINVAL;
    if (elem != ABS_F32 && elem != ABS_BF16) return ABS_EINVAL;
    const size_t T = L->sizes.size();
    const uintptr_t esz = elem == ABS_BF16 ? 2 : 4;
    for (size_t t = 0; t < T; ++t) {
        if (L->sizes[t] > 0 && (!ptrs[t] || !aligned_to(ptrs[t], esz))) return ABS_EINVAL;
    }
    int rc = layout_upload(L);           // the first set over a layout puts its tables on the device
    if (rc != ABS_OK) return rc;
    abs_tensorset *S = new (std::nothrow) abs_tensorset;
    if (!S) return ABS_EINVAL;
    S->layout = L;
    S->elem = elem;
    S->ptrs.assign(ptrs, ptrs + T);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&S->d_tab), T * sizeof(void *));
    if (e == hipSuccess) e = hipMemcpy(S->d_tab, S->ptrs.data(), T * sizeof(void *), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (S->d_tab) (void)hipFree(S->d_tab);
        delete S;
        return hip_fail(e);
    }
    *out = S;
    return ABS_OK;
}

int abs_tensorset_destroy(abs_tensorset *S)
{
    if (!S) return ABS_EINVAL;
    if (S->d_tab) (void)hipFree(S->d_tab);
    delete S;
    return ABS_OK;
}

int abs_accumulate_batch_mt(abs_layout *L, const abs_tensorset *acc, const abs_tensorset *const *grads,
                            int J, const int64_t *n_samples, int64_t *count, void *stream)
{
    return accumulate_batch_mt(process_tuning(), L, acc, grads, J, n_samples, count, static_cast<hipStream_t>(stream));
}

int abs_accumulate_mt(abs_layout *L, const abs_tensorset *acc, const abs_tensorset *grad,
                      int64_t n_samples, int64_t *count, void *stream)
{
    return abs_accumulate_batch_mt(L, acc, &grad, 1, &n_samples, count, stream);
}

int abs_accumulate_jobs_mt(abs_layout *L, const abs_job_mt *jobs, int njobs, int fold, void *stream)
{
    return accumulate_jobs_mt(process_tuning(), L, jobs, njobs, fold, static_cast<hipStream_t>(stream));
}

int abs_sync_update_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                       const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                       float mu, float wd, void *stream)
{
    return sync_update_mt(process_tuning(), SGD, L, params, momentum, nullptr, acc, counts, K,
                          hyper_sgd(lr, mu, wd, 0.f), static_cast<hipStream_t>(stream));
}

int abs_sync_update_dc_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *params_prev,
                          const abs_tensorset *momentum, const abs_tensorset *const *acc,
                          const int64_t *counts, int K, float lr, float mu, float wd, float lambda,
                          void *stream)
{
    return sync_update_mt(process_tuning(), SGD_DC, L, params, momentum, params_prev, acc, counts, K,
                          hyper_sgd(lr, mu, wd, lambda), static_cast<hipStream_t>(stream));
}

int abs_sync_update_dcm_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                           const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                           float mu, float wd, float lambda, float lr_prev, void *stream)
{
    return sync_update_mt(process_tuning(), SGD_DCM, L, params, momentum, nullptr, acc, counts, K,
                          hyper_sgd(lr, mu, wd, lambda, lr_prev), static_cast<hipStream_t>(stream));
}

int abs_sync_update_adam_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *exp_avg,
                            const abs_tensorset *exp_avg_sq, const abs_tensorset *const *acc,
                            const int64_t *counts, int K, float lr, float beta1, float beta2, float eps,
                            float wd, int64_t step, void *stream)
{
    Hyper h;
    int rc = hyper_adam(h, lr, beta1, beta2, eps, wd, step);
    if (rc != ABS_OK) return rc;
    return sync_update_mt(process_tuning(), ADAM, L, params, exp_avg, exp_avg_sq, acc, counts, K, h,
                          static_cast<hipStream_t>(stream));
}

int abs_sync_update_lars_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                            const abs_tensorset *gbar, const abs_tensorset *const *acc,
                            const int64_t *counts, int K, float lr, float mu, float wd, float eta,
                            void *stream)
{
    return sync_update_lars(L, params, momentum, gbar, acc, counts, K, lr, mu, wd, eta, nullptr, false,
                            static_cast<hipStream_t>(stream));
}

int abs_sync_update_lars_mt_noalloc(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                                    const abs_tensorset *gbar, const abs_tensorset *const *acc,
                                    const int64_t *counts, int K, float lr, float mu, float wd, float eta,
                                    void *stream)
{
    if (!L) return ABS_EINVAL;
    if (L->chunks.size() > (size_t)ABS_NOALLOC_MAX_CHUNKS || L->sizes.size() > (size_t)ABS_NOALLOC_MAX_TENSORS)
        return ABS_EINVAL;                   // beyond what the fixed scratch array holds
    LarsScratch sc;
    int rc = scratch_on_current_device(sc);
    if (rc != ABS_OK) return rc;
    // every entry of the three tables that the kernels read is written earlier in this same call
    // (first-chunk table, then per-chunk sums, then per-tensor factors): nothing needs clearing
    return sync_update_lars(L, params, momentum, gbar, acc, counts, K, lr, mu, wd, eta, &sc, true,
                            static_cast<hipStream_t>(stream));
}

// --------------------------------------------------------- double buffer

// Everything that can fail happens before the context is touched: after an error the
// context still works with the streams it had.
static int ctx_set_streams(abs_ctx *C, const hipStream_t *streams, int n)
{
    bool joins = false;
    for (int i = 0; i < n; ++i) joins = joins || streams[i] != C->s_upd;
    hipEvent_t upd = C->ev_upd;
    std::vector<hipEvent_t> ev;
    if (joins) {
        hipError_t e = hipSuccess;
        if (!upd) e = hipEventCreateWithFlags(&upd, hipEventDisableTiming);
        for (int i = 0; i < n && e == hipSuccess; ++i) {
            hipEvent_t one = nullptr;
            e = hipEventCreateWithFlags(&one, hipEventDisableTiming);
            if (e == hipSuccess) ev.push_back(one);
        }
        if (e != hipSuccess) {
            for (hipEvent_t one : ev) (void)hipEventDestroy(one);
            if (upd && upd != C->ev_upd) (void)hipEventDestroy(upd);
            return hip_fail(e);
        }
    }
    for (hipEvent_t one : C->ev_acc) (void)hipEventDestroy(one);
    C->ev_acc.swap(ev);
    C->ev_upd = upd;
    C->s_acc.assign(streams, streams + n);
    C->slot.resize((size_t)C->K);
    for (int k = 0; k < C->K; ++k) C->slot[(size_t)k] = k % n;
    C->launches.assign((size_t)C->K, 0);
    C->joins = joins;
    return ABS_OK;
}

static int ctx_common(abs_ctx *C, int K, void *stream_acc, void *stream_upd)
{
    C->K = K;
    C->counts[0].assign((size_t)K, 0);
    C->counts[1].assign((size_t)K, 0);
    C->s_upd = static_cast<hipStream_t>(stream_upd);
    hipStream_t sa = static_cast<hipStream_t>(stream_acc);
    return ctx_set_streams(C, &sa, 1);
}

int abs_ctx_create(abs_ctx **out, int K, int64_t P, float *const *acc_A, float *const *acc_B,
                   void *stream_acc, void *stream_upd)
{
    if (!out || K < 1 || K > ABS_MAX_K || P < 0 || !acc_A || !acc_B) return ABS_EINVAL;
    for (int k = 0; k < K; ++k) {
        if (P > 0 && (!acc_A[k] || !acc_B[k])) return ABS_EINVAL;
        if (!aligned_to(acc_A[k], 4) || !aligned_to(acc_B[k], 4)) return ABS_EINVAL;
        // the 2K accumulators are all written: no two may share bytes
        for (int q = 0; q < K; ++q) {
            if (overlap(acc_A[k], 4 * P, acc_B[q], 4 * P)) return ABS_EINVAL;
            if (q < k && (overlap(acc_A[k], 4 * P, acc_A[q], 4 * P) || overlap(acc_B[k], 4 * P, acc_B[q], 4 * P)))
                return ABS_EINVAL;
        }
    }
    abs_ctx *C = new (std::nothrow) abs_ctx;
    if (!C) return ABS_EINVAL;
    C->P = P;
    C->acc[0].assign(acc_A, acc_A + K);
    C->acc[1].assign(acc_B, acc_B + K);
    int rc = ctx_common(C, K, stream_acc, stream_upd);
    if (rc != ABS_OK) { abs_ctx_destroy(C); return rc; }
    *out = C;
    return ABS_OK;
}

int abs_ctx_create_mt(abs_ctx **out, int K, abs_layout *L, const abs_tensorset *const *acc_A,
                      const abs_tensorset *const *acc_B, void *stream_acc, void *stream_upd)
{
    if (!out || K < 1 || K > ABS_MAX_K || !L || !acc_A || !acc_B) return ABS_EINVAL;
    for (int k = 0; k < K; ++k) {
        if (!set_ok(acc_A[k], L) || !set_ok(acc_B[k], L)) return ABS_EINVAL;
        if (acc_A[k]->elem != ABS_F32 || acc_B[k]->elem != ABS_F32) return ABS_EINVAL;
        for (int q = 0; q < K; ++q) {
            if (acc_A[k] == acc_B[q]) return ABS_EINVAL;
            if (q < k && (acc_A[k] == acc_A[q] || acc_B[k] == acc_B[q])) return ABS_EINVAL;
        }
    }
    abs_ctx *C = new (std::nothrow) abs_ctx;
    if (!C) return ABS_EINVAL;
    C->layout = L;
    C->P = L->total;
    C->set[0].assign(acc_A, acc_A + K);
    C->set[1].assign(acc_B, acc_B + K);
    int rc = ctx_common(C, K, stream_acc, stream_upd);
    if (rc != ABS_OK) { abs_ctx_destroy(C); return rc; }
    *out = C;
    return ABS_OK;
}

int abs_ctx_destroy(abs_ctx *C)
{
    if (!C) return ABS_EINVAL;
    for (hipEvent_t e : C->ev_acc) (void)hipEventDestroy(e);
    if (C->ev_upd) (void)hipEventDestroy(C->ev_upd);
    delete C;
    return ABS_OK;
}

int abs_ctx_set_launch_tuning(abs_ctx *C, int blocks_per_cu, int max_rows_per_tile)
{
    if (!C || !tuning_ok(blocks_per_cu, max_rows_per_tile)) return ABS_EINVAL;
    C->own_shape = true;
    C->blocks_per_cu = blocks_per_cu;
    C->max_rows = max_rows_per_tile;
    return ABS_OK;
}

int abs_ctx_set_cache_policy(abs_ctx *C, int accumulate_mode, int update_mode)
{
    if (!C || !policy_ok(accumulate_mode, update_mode)) return ABS_EINVAL;
    C->own_policy = true;
    C->policy_acc = accumulate_mode;
    C->policy_upd = update_mode;
    return ABS_OK;
}

int abs_ctx_accumulate_batch(abs_ctx *C, int k, const void *const *grads, abs_dtype grad_dtype, int J,
                             const int64_t *n_samples)
{
    if (!C || C->layout || k < 0 || k >= C->K) return ABS_EINVAL;
    const int rc = accumulate_batch_flat(C->tuning(), C->acc[C->cur][(size_t)k], grads, grad_dtype, J, C->P,
                                         n_samples, &C->counts[C->cur][(size_t)k], C->stream_of(k));
    if (rc == ABS_OK) C->launches[(size_t)k] += (J + ABS_MAX_BATCH - 1) / ABS_MAX_BATCH;
    return rc;
}

int abs_ctx_accumulate(abs_ctx *C, int k, const void *grad, abs_dtype grad_dtype, int64_t n_samples)
{
    const void *grads[1] = {grad};
    return abs_ctx_accumulate_batch(C, k, grads, grad_dtype, 1, &n_samples);
}

int abs_ctx_accumulate_batch_mt(abs_ctx *C, int k, const abs_tensorset *const *grads, int J,
                                const int64_t *n_samples)
{
    if (!C || !C->layout || k < 0 || k >= C->K) return ABS_EINVAL;
    const int rc = accumulate_batch_mt(C->tuning(), C->layout, C->set[C->cur][(size_t)k], grads, J, n_samples,
                                       &C->counts[C->cur][(size_t)k], C->stream_of(k));
    if (rc == ABS_OK) C->launches[(size_t)k] += (J + ABS_MAX_BATCH - 1) / ABS_MAX_BATCH;
    return rc;
}

int abs_ctx_accumulate_mt(abs_ctx *C, int k, const abs_tensorset *grad, int64_t n_samples)
{
    return abs_ctx_accumulate_batch_mt(C, k, &grad, 1, &n_samples);
}

// Step 2 of all K workers in one call.  grads / n_samples: worker 0's m[0] entries, then
// worker 1's m[1], ...  Runs on the context's first accumulate stream.
static int ctx_step_checks(const abs_ctx *C, const int *m, int64_t &total)
{
    if (!C || !m || C->s_acc.size() != 1) return ABS_EINVAL;
    total = 0;
    for (int k = 0; k < C->K; ++k) {
        if (m[k] < 0) return ABS_EINVAL;
        total += m[k];
    }
    return ABS_OK;
}

int abs_ctx_accumulate_step(abs_ctx *C, const void *const *grads, const int *m, const int64_t *n_samples,
                            abs_dtype grad_dtype, int fold)
{
    int64_t total = 0;
    int rc = ctx_step_checks(C, m, total);
    if (rc != ABS_OK || C->layout || (total > 0 && (!grads || !n_samples))) return ABS_EINVAL;
    abs_job jobs[ABS_MAX_K];
    int64_t at = 0;
    for (int k = 0; k < C->K; ++k) {
        jobs[k] = abs_job{C->acc[C->cur][(size_t)k], grads + at, n_samples + at, m[k],
                          &C->counts[C->cur][(size_t)k]};
        at += m[k];
    }
    return accumulate_jobs_flat(C->tuning(), jobs, C->K, grad_dtype, C->P, fold, C->s_acc[0]);
}

int abs_ctx_accumulate_step_mt(abs_ctx *C, const abs_tensorset *const *grads, const int *m,
                               const int64_t *n_samples, int fold)
{
    int64_t total = 0;
    int rc = ctx_step_checks(C, m, total);
    if (rc != ABS_OK || !C->layout || (total > 0 && (!grads || !n_samples))) return ABS_EINVAL;
    abs_job_mt jobs[ABS_MAX_K];
    int64_t at = 0;
    for (int k = 0; k < C->K; ++k) {
        jobs[k] = abs_job_mt{C->set[C->cur][(size_t)k], grads + at, n_samples + at, m[k],
                             &C->counts[C->cur][(size_t)k]};
        at += m[k];
    }
    return accumulate_jobs_mt(C->tuning(), C->layout, jobs, C->K, fold, C->s_acc[0]);
}

int abs_ctx_set_accumulate_streams(abs_ctx *C, void *const *streams, int n)
{
    if (!C || !streams || n < 1 || n > ABS_MAX_K) return ABS_EINVAL;
    for (const auto &gen : C->counts)
        for (int64_t c : gen)
            if (c != 0) return ABS_EINVAL;   // only between creation and the first accumulate
    std::vector<hipStream_t> s((size_t)n);
    for (int i = 0; i < n; ++i) s[(size_t)i] = static_cast<hipStream_t>(streams[i]);
    return ctx_set_streams(C, s.data(), n);
}

int abs_suggest_accumulate_streams(int64_t P, int K)
{
    const int64_t bytes = 4 * P;
    return (K >= 2 && bytes >= (int64_t(24) << 20) && bytes <= (int64_t(112) << 20)) ? 2 : 1;
}

int abs_ctx_sync_update(abs_ctx *C, float *params, float *momentum, float lr, float mu, float wd)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return sync_update_flat(C->tuning(), SGD, params, momentum, nullptr, C->acc[prev].data(),
                            C->counts[prev].data(), C->K, C->P, hyper_sgd(lr, mu, wd, 0.f), C->s_upd);
}

int abs_ctx_sync_update_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *momentum,
                           float lr, float mu, float wd)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return sync_update_mt(C->tuning(), SGD, C->layout, params, momentum, nullptr, C->set[prev].data(),
                          C->counts[prev].data(), C->K, hyper_sgd(lr, mu, wd, 0.f), C->s_upd);
}

int abs_ctx_sync_update_dc(abs_ctx *C, float *params, float *params_prev, float *momentum, float lr,
                           float mu, float wd, float lambda)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return sync_update_flat(C->tuning(), SGD_DC, params, momentum, params_prev, C->acc[prev].data(),
                            C->counts[prev].data(), C->K, C->P, hyper_sgd(lr, mu, wd, lambda), C->s_upd);
}

int abs_ctx_sync_update_dc_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *params_prev,
                              const abs_tensorset *momentum, float lr, float mu, float wd, float lambda)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return sync_update_mt(C->tuning(), SGD_DC, C->layout, params, momentum, params_prev, C->set[prev].data(),
                          C->counts[prev].data(), C->K, hyper_sgd(lr, mu, wd, lambda), C->s_upd);
}

int abs_ctx_sync_update_dcm(abs_ctx *C, float *params, float *momentum, float lr, float mu, float wd,
                            float lambda)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    const int rc = sync_update_flat(C->tuning(), SGD_DCM, params, momentum, nullptr, C->acc[prev].data(),
                                    C->counts[prev].data(), C->K, C->P,
                                    hyper_sgd(lr, mu, wd, lambda, C->lr_applied), C->s_upd);
    if (rc == ABS_OK) C->lr_applied = lr;
    else if (rc == ABS_EMPTY) C->lr_applied = 0.f;
    return rc;
}

int abs_ctx_sync_update_dcm_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *momentum,
                               float lr, float mu, float wd, float lambda)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    const int rc = sync_update_mt(C->tuning(), SGD_DCM, C->layout, params, momentum, nullptr,
                                  C->set[prev].data(), C->counts[prev].data(), C->K,
                                  hyper_sgd(lr, mu, wd, lambda, C->lr_applied), C->s_upd);
    if (rc == ABS_OK) C->lr_applied = lr;
    else if (rc == ABS_EMPTY) C->lr_applied = 0.f;
    return rc;
}

int abs_ctx_sync_update_adam(abs_ctx *C, float *params, float *exp_avg, float *exp_avg_sq, float lr,
                             float beta1, float beta2, float eps, float wd, int64_t step)
{
    if (!C || C->layout) return ABS_EINVAL;
    Hyper h;
    int rc = hyper_adam(h, lr, beta1, beta2, eps, wd, step);
    if (rc != ABS_OK) return rc;
    const int prev = C->cur ^ 1;
    return sync_update_flat(C->tuning(), ADAM, params, exp_avg, exp_avg_sq, C->acc[prev].data(),
                            C->counts[prev].data(), C->K, C->P, h, C->s_upd);
}

int abs_ctx_sync_update_adam_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *exp_avg,
                                const abs_tensorset *exp_avg_sq, float lr, float beta1, float beta2,
                                float eps, float wd, int64_t step)
{
    if (!C || !C->layout) return ABS_EINVAL;
    Hyper h;
    int rc = hyper_adam(h, lr, beta1, beta2, eps, wd, step);
    if (rc != ABS_OK) return rc;
    const int prev = C->cur ^ 1;
    return sync_update_mt(C->tuning(), ADAM, C->layout, params, exp_avg, exp_avg_sq, C->set[prev].data(),
                          C->counts[prev].data(), C->K, h, C->s_upd);
}

int abs_ctx_sync_update_lars_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *momentum,
                                const abs_tensorset *gbar, float lr, float mu, float wd, float eta)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return sync_update_lars(C->layout, params, momentum, gbar, C->set[prev].data(), C->counts[prev].data(),
                            C->K, lr, mu, wd, eta, nullptr, false, C->s_upd);
}

int abs_swap_buffers(abs_ctx *C)
{
    if (!C) return ABS_EINVAL;
    if (C->joins) {
        // next accumulation overwrites what the sync-update has been reading
        ABS_HIP(hipEventRecord(C->ev_upd, C->s_upd));
        for (size_t i = 0; i < C->s_acc.size(); ++i) {
            if (C->s_acc[i] == C->s_upd) continue;
            // next sync-update reads what accumulation has written so far
            ABS_HIP(hipEventRecord(C->ev_acc[i], C->s_acc[i]));
            ABS_HIP(hipStreamWaitEvent(C->s_upd, C->ev_acc[i], 0));
            ABS_HIP(hipStreamWaitEvent(C->s_acc[i], C->ev_upd, 0));
        }
    }
    // Fewer streams than workers: place the workers for the next step so that the
    // streams carry about equal numbers of launches, taking this step's counts as
    // the forecast (static heterogeneity persists from step to step; under purely
    // dynamic heterogeneity any placement is as good as another).  Longest first,
    // each to the least loaded stream.  Safe at this point only: every stream has
    // just been ordered after everything the others have enqueued.
    const size_t ns = C->s_acc.size();
    if (ns > 1 && ns < (size_t)C->K) {
        std::vector<int> order((size_t)C->K);
        for (int k = 0; k < C->K; ++k) order[(size_t)k] = k;
        std::stable_sort(order.begin(), order.end(),
                         [&](int a, int b) { return C->launches[(size_t)a] > C->launches[(size_t)b]; });
        std::vector<int64_t> load(ns, 0);
        for (int k : order) {
            size_t best = 0;
            for (size_t i = 1; i < ns; ++i)
                if (load[i] < load[best]) best = i;
            C->slot[(size_t)k] = (int)best;
            load[best] += C->launches[(size_t)k] > 0 ? C->launches[(size_t)k] : 1;
        }
    }
    for (auto &l : C->launches) l = 0;
    C->cur ^= 1;
    for (auto &c : C->counts[C->cur]) c = 0;
    return ABS_OK;
}

int abs_ctx_counts(const abs_ctx *C, int which, int64_t *out)
{
    if (!C || !out || (which != 0 && which != 1)) return ABS_EINVAL;
    const auto &c = C->counts[which == 0 ? C->cur : C->cur ^ 1];
    for (int k = 0; k < C->K; ++k) out[k] = c[(size_t)k];
    return ABS_OK;
}

}  // extern "C"
