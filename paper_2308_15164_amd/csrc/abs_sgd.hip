// Host side of the ABS-SGD hot-path library: argument checks, the ragged
// layout's chunk table, the double-buffer context, and kernel launches.
// The C ABI and the arithmetic contract are stated in include/abs_sgd.h.
#include "abs_kernels.hpp"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

#include "abs_sgd.h"

#ifndef ABS_ACC_STREAM_BYTES
#define ABS_ACC_STREAM_BYTES (int64_t(160) << 20)
#endif
#ifndef ABS_MAX_ROWS
#define ABS_MAX_ROWS 4
#endif
#ifndef ABS_UPD_STREAM_BYTES
#define ABS_UPD_STREAM_BYTES (int64_t(256) << 20)
#endif

using namespace absk;

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

inline int launch_status()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return ABS_OK;
}

constexpr int64_t kMaxGrid = 0x7fffffff;
constexpr int64_t kMaxTile = int64_t(1) << 30;   // tile sizes travel as int

// ------------------------------------------------------------ launch shape
//
// A launch should fill the chip in whole rounds: with `resident` workgroups
// able to run at once, the tile is the smallest whole number of rows that
// covers n rows in `rounds` rounds, rounds being the fewest that keep a tile
// within g_max_rows rows (0 = no limit: always one round, every workgroup
// walks one long run of memory).  Measured on MI355X: short tiles (<= 4 rows,
// many rounds) beat long per-workgroup runs by 15-20 % at P >= 1e8, because all
// resident workgroups then sweep one compact window of memory.
int g_blocks_per_cu = 0;                  // 0 = what each kernel's register use allows
int g_max_rows = ABS_MAX_ROWS;

// Compute units of the current device; 256 (MI355X) when no device can be asked,
// e.g. when a layout is built on a host without a GPU.
int cu_count()
{
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            return cus;
        (void)hipGetLastError();
        return 256;
    }();
    return n;
}

inline int64_t rows_of(int64_t P) { return (P + ROW - 1) / ROW; }

int64_t choose_tile(int64_t rows, int resident)
{
    if (rows <= resident) return ROW;
    int64_t rounds = 1;
    if (g_max_rows > 0) rounds = (rows + (int64_t)resident * g_max_rows - 1) / ((int64_t)resident * g_max_rows);
    const int64_t slots = (int64_t)resident * rounds;
    return ((rows + slots - 1) / slots) * ROW;
}

inline int64_t tiles_for(int64_t P, int64_t tile) { return (P + tile - 1) / tile; }

// Workgroups of `kernel` one CU can hold, from the runtime's occupancy calculator.
template <class Kernel>
int occupancy_per_cu(Kernel kernel, int fallback)
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, BLOCK, 0) == hipSuccess && n > 0) return n;
    (void)hipGetLastError();
    return fallback;
}

// Workgroups resident on the whole chip, with the caller's override applied.
inline int resident(int per_cu) { return (g_blocks_per_cu > 0 ? g_blocks_per_cu : per_cu) * cu_count(); }

// The accumulate kernels need few registers: 8 workgroups of 4 wavefronts per CU.
constexpr int kAccBlocksPerCU = 8;
inline int acc_resident() { return resident(kAccBlocksPerCU); }

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

// ------------------------------------------------------------ cache policy
//
// Accumulators, x and v are touched again soon after a kernel ends.  When they
// fit the memory-side cache (256 MiB on this part) keeping them cached pays;
// when they do not, streaming (non-temporal) accesses avoid allocating lines
// that are evicted before their reuse.  -1 = decide from the sizes.
int g_policy_acc = -1, g_policy_upd = -1;
constexpr int64_t kAccStreamBytes = ABS_ACC_STREAM_BYTES;   // accumulator bytes above which accumulate streams
constexpr int64_t kUpdStreamBytes = ABS_UPD_STREAM_BYTES;   // bytes of x + v (+ previous x) above which sync-update streams

inline bool stream_acc(int64_t P) { return g_policy_acc < 0 ? 4 * P > kAccStreamBytes : g_policy_acc != 0; }
inline bool stream_upd(int64_t P, int vectors = 2) { return g_policy_upd < 0 ? 4 * vectors * P > kUpdStreamBytes : g_policy_upd != 0; }

// ------------------------------------------------------------ flat launches

template <bool BF16, int J>
void launch_accumulate_flat_j(float *acc, const void *const *grads, const float *nf, int64_t P, int tile,
                              unsigned nblocks, int first, int vec_ok, bool nta, hipStream_t s)
{
    GradArgs<BF16, J> G;
    for (int j = 0; j < J; ++j) {
        G.g[j] = static_cast<const typename GradT<BF16>::elem *>(grads[j]);
        G.n[j] = nf[j];
    }
    const dim3 grid(nblocks), block(BLOCK);
    if (nta) hipLaunchKernelGGL((accumulate_flat<BF16, true, J>), grid, block, 0, s, acc, G, P, tile, first, vec_ok);
    else hipLaunchKernelGGL((accumulate_flat<BF16, false, J>), grid, block, 0, s, acc, G, P, tile, first, vec_ok);
}

// One launch: J <= ABS_MAX_BATCH gradients into one accumulator.
int launch_accumulate_flat(float *acc, const void *const *grads, const float *nf, int J, abs_dtype dt,
                           int64_t P, int first, int vec_ok, hipStream_t s)
{
    const int64_t tile64 = choose_tile(rows_of(P), acc_resident());
    if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
    const int tile = (int)tile64;
    const unsigned nb = (unsigned)tiles_for(P, tile64);
    const bool bf = dt == ABS_BF16, nta = stream_acc(P);
    switch (J) {
#define ABS_CASE(N)                                                                                     \
    case N:                                                                                             \
        if (bf) launch_accumulate_flat_j<true, N>(acc, grads, nf, P, tile, nb, first, vec_ok, nta, s);  \
        else launch_accumulate_flat_j<false, N>(acc, grads, nf, P, tile, nb, first, vec_ok, nta, s);    \
        break;
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
#undef ABS_CASE
    default: return ABS_EINVAL;
    }
    return ABS_OK;
}

template <int K, int RULE>
int launch_sync_flat_kr(float *x, float *v, float *xp, const float *const *ptrs, int64_t P, const Hyper &h,
                        int vec_ok, hipStream_t s)
{
    static const int per_cu = occupancy_per_cu(sync_update_flat<K, false, RULE>, 4);
    const int64_t tile64 = choose_tile(rows_of(P), resident(per_cu));
    if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
    const int tile = (int)tile64;
    AccPtrs<K> A;
    for (int k = 0; k < K; ++k) A.p[k] = ptrs[k];
    const dim3 grid((unsigned)tiles_for(P, tile64)), block(BLOCK);
    // x and each state vector are re-read one iteration later
    if (stream_upd(P, uses_s2<RULE>() ? 3 : 2))
        hipLaunchKernelGGL((sync_update_flat<K, true, RULE>), grid, block, 0, s, x, v, xp, A, P, tile, h, vec_ok);
    else
        hipLaunchKernelGGL((sync_update_flat<K, false, RULE>), grid, block, 0, s, x, v, xp, A, P, tile, h, vec_ok);
    return ABS_OK;
}

template <int RULE>
int launch_sync_flat_r(float *x, float *v, float *xp, const float *const *ptrs, int n, int64_t P,
                       const Hyper &h, int vec_ok, hipStream_t s)
{
    switch (n) {
#define ABS_CASE(K) case K: return launch_sync_flat_kr<K, RULE>(x, v, xp, ptrs, P, h, vec_ok, s);
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
        ABS_CASE(9) ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15)
        ABS_CASE(16)
#undef ABS_CASE
    default: {
        const int64_t tile64 = choose_tile(rows_of(P), resident(4));
        if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
        AccPtrsAny A;
        std::memset(&A, 0, sizeof A);
        for (int k = 0; k < n; ++k) A.p[k] = ptrs[k];
        hipLaunchKernelGGL(sync_update_flat_any<RULE>, dim3((unsigned)tiles_for(P, tile64)), dim3(BLOCK), 0,
                           s, x, v, xp, A, n, P, (int)tile64, h, vec_ok);
        return ABS_OK;
    }
    }
}

int launch_sync_flat(int rule, float *x, float *v, float *xp, const float *const *ptrs, int n, int64_t P,
                     const Hyper &h, int vec_ok, hipStream_t s)
{
    switch (rule) {
    case SGD: return launch_sync_flat_r<SGD>(x, v, xp, ptrs, n, P, h, vec_ok, s);
    case SGD_DC: return launch_sync_flat_r<SGD_DC>(x, v, xp, ptrs, n, P, h, vec_ok, s);
    case ADAM: return launch_sync_flat_r<ADAM>(x, v, xp, ptrs, n, P, h, vec_ok, s);
    case SGD_DCM: return launch_sync_flat_r<SGD_DCM>(x, v, xp, ptrs, n, P, h, vec_ok, s);
    default: return ABS_EINVAL;
    }
}

int launch_copy_flat(float *dst, const float *src, int64_t P, hipStream_t s)
{
    const int64_t tile64 = choose_tile(rows_of(P), acc_resident());
    if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
    const int vec_ok = aligned_to(dst, 16) && aligned_to(src, 16);
    hipLaunchKernelGGL(copy_flat, dim3((unsigned)tiles_for(P, tile64)), dim3(BLOCK), 0, s, dst, src, P,
                       (int)tile64, vec_ok);
    return ABS_OK;
}

}  // namespace

// ---------------------------------------------------------------- ragged types

struct abs_layout {
    std::vector<int64_t> sizes;
    std::vector<Chunk> chunks;
    int64_t total = 0;
    int tile = ROW;                      // elements per chunk, a multiple of ROW
    // device copies, made on first use
    Chunk *d_chunks = nullptr;
    int64_t *d_sizes = nullptr;
    int device = -1;
    // LARS only, made on its first use: first chunk of every tensor (T + 1 entries),
    // per-chunk sums of squares, per-tensor step factors
    int32_t *d_chunk_begin = nullptr;
    double *d_partials = nullptr;
    float *d_step = nullptr;
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
    std::vector<hipStream_t> s_acc;      // worker k accumulates on s_acc[k % size]
    hipStream_t s_upd = nullptr;
    std::vector<hipEvent_t> ev_acc;      // one per accumulate stream
    hipEvent_t ev_upd = nullptr;
    bool joins = false;                  // more than one distinct stream in use

    std::vector<int> slot;               // worker k accumulates on s_acc[slot[k]]
    std::vector<int64_t> launches;       // accumulate launches of worker k in the current step
    float lr_applied = 0.f;              // step size of the last abs_ctx_sync_update_dcm* call; 0 after an empty one

    hipStream_t stream_of(int k) const { return s_acc[(size_t)slot[(size_t)k]]; }
};

namespace {

int layout_to_device(abs_layout *L)
{
    int dev = 0;
    ABS_HIP(hipGetDevice(&dev));
    if (L->d_chunks) return L->device == dev ? ABS_OK : ABS_EINVAL;
    if (L->chunks.empty()) { L->device = dev; return ABS_OK; }
    Chunk *dc = nullptr;
    int64_t *ds = nullptr;
    ABS_HIP(hipMalloc(&dc, L->chunks.size() * sizeof(Chunk)));
    hipError_t e = hipMalloc(&ds, L->sizes.size() * sizeof(int64_t));
    if (e == hipSuccess) e = hipMemcpy(dc, L->chunks.data(), L->chunks.size() * sizeof(Chunk), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ds, L->sizes.data(), L->sizes.size() * sizeof(int64_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dc);
        if (ds) (void)hipFree(ds);
        return hip_fail(e);
    }
    L->d_chunks = dc;
    L->d_sizes = ds;
    L->device = dev;
    return ABS_OK;
}

int layout_lars_scratch(abs_layout *L)
{
    if (L->d_partials) return ABS_OK;
    std::vector<int32_t> begin(L->sizes.size() + 1, 0);
    for (const Chunk &c : L->chunks) begin[(size_t)c.tensor + 1] += 1;
    for (size_t t = 0; t < L->sizes.size(); ++t) begin[t + 1] += begin[t];
    int32_t *db = nullptr;
    double *dp = nullptr;
    float *ds = nullptr;
    hipError_t e = hipMalloc(&db, begin.size() * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(&dp, 2 * L->chunks.size() * sizeof(double));
    if (e == hipSuccess) e = hipMalloc(&ds, L->sizes.size() * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(db, begin.data(), begin.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (db) (void)hipFree(db);
        if (dp) (void)hipFree(dp);
        if (ds) (void)hipFree(ds);
        return hip_fail(e);
    }
    L->d_chunk_begin = db;
    L->d_partials = dp;
    L->d_step = ds;
    return ABS_OK;
}

template <int K, int RULE>
void launch_sync_ragged_kr(const abs_layout *L, float *const *xt, float *const *vt, float *const *pt,
                           const float *const *const *tabs, const Hyper &h, hipStream_t s)
{
    TabPtrs<K> T;
    for (int k = 0; k < K; ++k) T.t[k] = tabs[k];
    const dim3 grid((unsigned)L->chunks.size()), block(BLOCK);
    if (stream_upd(L->total, uses_s2<RULE>() ? 3 : 2))
        hipLaunchKernelGGL((sync_update_ragged<K, true, RULE>), grid, block, 0, s, L->d_chunks, L->d_sizes, xt, vt, pt, T, L->tile, h);
    else
        hipLaunchKernelGGL((sync_update_ragged<K, false, RULE>), grid, block, 0, s, L->d_chunks, L->d_sizes, xt, vt, pt, T, L->tile, h);
}

template <int RULE>
void launch_sync_ragged_r(const abs_layout *L, float *const *xt, float *const *vt, float *const *pt,
                          const float *const *const *tabs, int n, const Hyper &h, hipStream_t s)
{
    switch (n) {
#define ABS_CASE(K) case K: launch_sync_ragged_kr<K, RULE>(L, xt, vt, pt, tabs, h, s); break;
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
        ABS_CASE(9) ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15)
        ABS_CASE(16)
#undef ABS_CASE
    default: {
        TabPtrsAny T;
        std::memset(&T, 0, sizeof T);
        for (int k = 0; k < n; ++k) T.t[k] = tabs[k];
        hipLaunchKernelGGL(sync_update_ragged_any<RULE>, dim3((unsigned)L->chunks.size()), dim3(BLOCK), 0, s,
                           L->d_chunks, L->d_sizes, xt, vt, pt, T, n, L->tile, h);
    }
    }
}

void launch_sync_ragged(int rule, const abs_layout *L, float *const *xt, float *const *vt, float *const *pt,
                        const float *const *const *tabs, int n, const Hyper &h, hipStream_t s)
{
    switch (rule) {
    case SGD: launch_sync_ragged_r<SGD>(L, xt, vt, pt, tabs, n, h, s); break;
    case SGD_DC: launch_sync_ragged_r<SGD_DC>(L, xt, vt, pt, tabs, n, h, s); break;
    case SGD_DCM: launch_sync_ragged_r<SGD_DCM>(L, xt, vt, pt, tabs, n, h, s); break;
    default: launch_sync_ragged_r<ADAM>(L, xt, vt, pt, tabs, n, h, s); break;
    }
}

template <int J>
void launch_accumulate_ragged_j(const abs_layout *L, float *const *at, const void *const *const *gt,
                                       const float *nf, int first, bool bf, bool nta, hipStream_t s)
{
    GradTabs<J> T;
    for (int j = 0; j < J; ++j) {
        T.t[j] = gt[j];
        T.n[j] = nf[j];
    }
    const dim3 grid((unsigned)L->chunks.size()), block(BLOCK);
    if (bf && nta) hipLaunchKernelGGL((accumulate_ragged<true, true, J>), grid, block, 0, s, L->d_chunks, L->d_sizes, at, T, L->tile, first);
    else if (bf) hipLaunchKernelGGL((accumulate_ragged<true, false, J>), grid, block, 0, s, L->d_chunks, L->d_sizes, at, T, L->tile, first);
    else if (nta) hipLaunchKernelGGL((accumulate_ragged<false, true, J>), grid, block, 0, s, L->d_chunks, L->d_sizes, at, T, L->tile, first);
    else hipLaunchKernelGGL((accumulate_ragged<false, false, J>), grid, block, 0, s, L->d_chunks, L->d_sizes, at, T, L->tile, first);
}

bool set_ok(const abs_tensorset *s, const abs_layout *L) { return s && s->layout == L; }

}  // namespace

// =========================================================================
// C ABI
// =========================================================================
extern "C" {

int abs_version(void) { return 100; }

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
    if (blocks_per_cu < 0 || blocks_per_cu > 32 || max_rows_per_tile < 0) return ABS_EINVAL;
    g_blocks_per_cu = blocks_per_cu;
    g_max_rows = max_rows_per_tile;
    return ABS_OK;
}

int abs_set_cache_policy(int accumulate_mode, int update_mode)
{
    if (accumulate_mode < -1 || accumulate_mode > 1 || update_mode < -1 || update_mode > 1) return ABS_EINVAL;
    g_policy_acc = accumulate_mode;
    g_policy_upd = update_mode;
    return ABS_OK;
}

// ------------------------------------------------------------------ flat

int abs_accumulate_batch(float *acc, const void *const *grads, abs_dtype grad_dtype, int J, int64_t P,
                         const int64_t *n_samples, int64_t *count, void *stream)
{
    if (!count || !grads || !n_samples || J < 1 || P < 0 || *count < 0) return ABS_EINVAL;
    if (grad_dtype != ABS_F32 && grad_dtype != ABS_BF16) return ABS_EINVAL;
    int64_t total = *count;
    for (int j = 0; j < J; ++j) {
        if (n_samples[j] <= 0 || total > std::numeric_limits<int64_t>::max() - n_samples[j]) return ABS_EINVAL;
        total += n_samples[j];
    }
    if (P > 0) {
        if (!acc || !aligned_to(acc, 4)) return ABS_EINVAL;
        const uintptr_t gsz = grad_dtype == ABS_BF16 ? 2 : 4;
        int vec_ok = aligned_to(acc, 16);
        for (int j = 0; j < J; ++j) {
            if (!grads[j] || !aligned_to(grads[j], gsz)) return ABS_EINVAL;
            vec_ok = vec_ok && aligned_to(grads[j], grad_dtype == ABS_BF16 ? 8 : 16);
        }
        hipStream_t s = static_cast<hipStream_t>(stream);
        int first = *count == 0 ? 1 : 0;
        for (int j0 = 0; j0 < J; j0 += ABS_MAX_BATCH) {
            const int jn = J - j0 < ABS_MAX_BATCH ? J - j0 : ABS_MAX_BATCH;
            float nf[ABS_MAX_BATCH];
            for (int j = 0; j < jn; ++j) nf[j] = (float)n_samples[j0 + j];
            int rc = launch_accumulate_flat(acc, grads + j0, nf, jn, grad_dtype, P, first, vec_ok, s);
            if (rc != ABS_OK) return rc;
            rc = launch_status();
            if (rc != ABS_OK) return rc;
            first = 0;
        }
    }
    *count = total;
    return ABS_OK;
}

int abs_accumulate(float *acc, const void *grad, abs_dtype grad_dtype, int64_t P,
                   int64_t n_samples, int64_t *count, void *stream)
{
    const void *grads[1] = {grad};
    return abs_accumulate_batch(acc, grads, grad_dtype, 1, P, &n_samples, count, stream);
}

// Hyper-parameters of the three rules in one struct.
static Hyper hyper_sgd(float lr, float mu, float wd, float lambda, float lr_prev = 0.f)
{
    Hyper h = {};
    h.lr = lr; h.mu = mu; h.wd = wd; h.lambda = lambda; h.nlr_prev = -lr_prev;
    return h;
}

static int hyper_adam(Hyper &h, float lr, float beta1, float beta2, float eps, float wd, int64_t step)
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

// s1: momentum (SGD rules) or first moment (ADAM); s2: previous iterate (SGD_DC)
// or second moment (ADAM), unused for SGD.
static int sync_update_flat_impl(int rule, float *params, float *s1, float *s2, const float *const *acc,
                                 const int64_t *counts, int K, int64_t P, Hyper h, void *stream)
{
    if (!acc || P < 0) return ABS_EINVAL;
    const bool has2 = rule == SGD_DC || rule == ADAM;
    Combine c;
    int rc = plan_combine(counts, K, c);
    if (rc != ABS_OK && rc != ABS_EMPTY) return rc;
    const bool empty = rc == ABS_EMPTY;
    if (empty && rule != SGD_DC) return ABS_EMPTY;
    if (P == 0) return empty ? ABS_EMPTY : ABS_OK;
    if (!params || !s1 || params == s1) return ABS_EINVAL;
    if (!aligned_to(params, 4) || !aligned_to(s1, 4)) return ABS_EINVAL;
    if (has2 && (!s2 || s2 == params || s2 == s1 || !aligned_to(s2, 4))) return ABS_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (empty) {
        // x_{t+1} = x_t: the previous-iterate buffer must still advance
        rc = launch_copy_flat(s2, params, P, s);
        if (rc != ABS_OK) return rc;
        rc = launch_status();
        return rc == ABS_OK ? ABS_EMPTY : rc;
    }
    const float *ptrs[ABS_MAX_K];
    bool vec = aligned_to(params, 16) && aligned_to(s1, 16) && (!has2 || aligned_to(s2, 16));
    for (int j = 0; j < c.n; ++j) {
        const float *p = acc[c.idx[j]];
        if (!p || !aligned_to(p, 4)) return ABS_EINVAL;
        vec = vec && aligned_to(p, 16);
        ptrs[j] = p;
    }
    h.M = (float)c.M;
    rc = launch_sync_flat(rule, params, s1, has2 ? s2 : nullptr, ptrs, c.n, P, h, vec ? 1 : 0, s);
    if (rc != ABS_OK) return rc;
    return launch_status();
}

int abs_sync_update(float *params, float *momentum, const float *const *acc,
                    const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                    void *stream)
{
    return sync_update_flat_impl(SGD, params, momentum, nullptr, acc, counts, K, P, hyper_sgd(lr, mu, wd, 0.f),
                                 stream);
}

int abs_sync_update_dc(float *params, float *params_prev, float *momentum, const float *const *acc,
                       const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                       float lambda, void *stream)
{
    return sync_update_flat_impl(SGD_DC, params, momentum, params_prev, acc, counts, K, P,
                                 hyper_sgd(lr, mu, wd, lambda), stream);
}

int abs_sync_update_dcm(float *params, float *momentum, const float *const *acc, const int64_t *counts,
                        int K, int64_t P, float lr, float mu, float wd, float lambda, float lr_prev,
                        void *stream)
{
    return sync_update_flat_impl(SGD_DCM, params, momentum, nullptr, acc, counts, K, P,
                                 hyper_sgd(lr, mu, wd, lambda, lr_prev), stream);
}

int abs_sync_update_adam(float *params, float *exp_avg, float *exp_avg_sq, const float *const *acc,
                         const int64_t *counts, int K, int64_t P, float lr, float beta1, float beta2,
                         float eps, float wd, int64_t step, void *stream)
{
    Hyper h;
    int rc = hyper_adam(h, lr, beta1, beta2, eps, wd, step);
    if (rc != ABS_OK) return rc;
    return sync_update_flat_impl(ADAM, params, exp_avg, exp_avg_sq, acc, counts, K, P, h, stream);
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
    const int64_t tile = choose_tile(rows, acc_resident());
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

int abs_layout_destroy(abs_layout *L)
{
    if (!L) return ABS_EINVAL;
    if (L->d_chunks) (void)hipFree(L->d_chunks);
    if (L->d_sizes) (void)hipFree(L->d_sizes);
    if (L->d_chunk_begin) (void)hipFree(L->d_chunk_begin);
    if (L->d_partials) (void)hipFree(L->d_partials);
    if (L->d_step) (void)hipFree(L->d_step);
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
    if (!L || !set_ok(acc, L) || acc->elem != ABS_F32 || !grads || !n_samples || J < 1) return ABS_EINVAL;
    if (!count || *count < 0) return ABS_EINVAL;
    int64_t total = *count;
    for (int j = 0; j < J; ++j) {
        if (!set_ok(grads[j], L) || grads[j]->elem != grads[0]->elem) return ABS_EINVAL;
        if (n_samples[j] <= 0 || total > std::numeric_limits<int64_t>::max() - n_samples[j]) return ABS_EINVAL;
        total += n_samples[j];
    }
    if (!L->chunks.empty()) {
        int rc = layout_to_device(L);
        if (rc != ABS_OK) return rc;
        hipStream_t s = static_cast<hipStream_t>(stream);
        float *const *at = reinterpret_cast<float *const *>(acc->d_tab);
        const bool bf = grads[0]->elem == ABS_BF16, nta = stream_acc(L->total);
        int first = *count == 0 ? 1 : 0;
        for (int j0 = 0; j0 < J; j0 += ABS_MAX_BATCH) {
            const int jn = J - j0 < ABS_MAX_BATCH ? J - j0 : ABS_MAX_BATCH;
            float nf[ABS_MAX_BATCH];
            const void *const *gt[ABS_MAX_BATCH];
            for (int j = 0; j < jn; ++j) {
                nf[j] = (float)n_samples[j0 + j];
                gt[j] = reinterpret_cast<const void *const *>(grads[j0 + j]->d_tab);
            }
            switch (jn) {
#define ABS_CASE(N) case N: launch_accumulate_ragged_j<N>(L, at, gt, nf, first, bf, nta, s); break;
                ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
#undef ABS_CASE
            }
            rc = launch_status();
            if (rc != ABS_OK) return rc;
            first = 0;
        }
    }
    *count = total;
    return ABS_OK;
}

int abs_accumulate_mt(abs_layout *L, const abs_tensorset *acc, const abs_tensorset *grad,
                      int64_t n_samples, int64_t *count, void *stream)
{
    return abs_accumulate_batch_mt(L, acc, &grad, 1, &n_samples, count, stream);
}

static int sync_update_mt_impl(int rule, abs_layout *L, const abs_tensorset *params, const abs_tensorset *s1,
                               const abs_tensorset *s2, const abs_tensorset *const *acc,
                               const int64_t *counts, int K, Hyper h, void *stream)
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
        const abs_tensorset *s = acc[c.idx[j]];
        if (!set_ok(s, L) || s->elem != ABS_F32) return ABS_EINVAL;
        tabs[j] = reinterpret_cast<const float *const *>(s->d_tab);
    }
    if (L->chunks.empty()) return empty ? ABS_EMPTY : ABS_OK;
    rc = layout_to_device(L);
    if (rc != ABS_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *const *xt = reinterpret_cast<float *const *>(params->d_tab);
    float *const *pt = has2 ? reinterpret_cast<float *const *>(s2->d_tab) : nullptr;
    if (empty) {
        hipLaunchKernelGGL(copy_ragged, dim3((unsigned)L->chunks.size()), dim3(BLOCK), 0, s, L->d_chunks,
                           L->d_sizes, pt, xt, L->tile);
        rc = launch_status();
        return rc == ABS_OK ? ABS_EMPTY : rc;
    }
    h.M = (float)c.M;
    launch_sync_ragged(rule, L, xt, reinterpret_cast<float *const *>(s1->d_tab), pt, tabs, c.n, h, s);
    return launch_status();
}

int abs_sync_update_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                       const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                       float mu, float wd, void *stream)
{
    return sync_update_mt_impl(SGD, L, params, momentum, nullptr, acc, counts, K, hyper_sgd(lr, mu, wd, 0.f),
                               stream);
}

int abs_sync_update_dc_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *params_prev,
                          const abs_tensorset *momentum, const abs_tensorset *const *acc,
                          const int64_t *counts, int K, float lr, float mu, float wd, float lambda,
                          void *stream)
{
    return sync_update_mt_impl(SGD_DC, L, params, momentum, params_prev, acc, counts, K,
                               hyper_sgd(lr, mu, wd, lambda), stream);
}

int abs_sync_update_dcm_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                           const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                           float mu, float wd, float lambda, float lr_prev, void *stream)
{
    return sync_update_mt_impl(SGD_DCM, L, params, momentum, nullptr, acc, counts, K,
                               hyper_sgd(lr, mu, wd, lambda, lr_prev), stream);
}

int abs_sync_update_adam_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *exp_avg,
                            const abs_tensorset *exp_avg_sq, const abs_tensorset *const *acc,
                            const int64_t *counts, int K, float lr, float beta1, float beta2, float eps,
                            float wd, int64_t step, void *stream)
{
    Hyper h;
    int rc = hyper_adam(h, lr, beta1, beta2, eps, wd, step);
    if (rc != ABS_OK) return rc;
    return sync_update_mt_impl(ADAM, L, params, exp_avg, exp_avg_sq, acc, counts, K, h, stream);
}

int abs_sync_update_lars_mt(abs_layout *L, const abs_tensorset *params, const abs_tensorset *momentum,
                            const abs_tensorset *gbar, const abs_tensorset *const *acc,
                            const int64_t *counts, int K, float lr, float mu, float wd, float eta,
                            void *stream)
{
    if (!L || !acc) return ABS_EINVAL;
    Combine c;
    int rc = plan_combine(counts, K, c);
    if (rc != ABS_OK) return rc;
    if (!set_ok(params, L) || !set_ok(momentum, L) || !set_ok(gbar, L)) return ABS_EINVAL;
    if (params == momentum || gbar == params || gbar == momentum) return ABS_EINVAL;
    if (params->elem != ABS_F32 || momentum->elem != ABS_F32 || gbar->elem != ABS_F32) return ABS_EINVAL;
    TabPtrsAny tabs;
    std::memset(&tabs, 0, sizeof tabs);
    for (int j = 0; j < c.n; ++j) {
        const abs_tensorset *s = acc[c.idx[j]];
        if (!set_ok(s, L) || s->elem != ABS_F32 || s == gbar) return ABS_EINVAL;
        tabs.t[j] = reinterpret_cast<const float *const *>(s->d_tab);
    }
    if (L->chunks.empty()) return ABS_OK;
    rc = layout_to_device(L);
    if (rc == ABS_OK) rc = layout_lars_scratch(L);
    if (rc != ABS_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *const *xt = reinterpret_cast<float *const *>(params->d_tab);
    float *const *vt = reinterpret_cast<float *const *>(momentum->d_tab);
    float *const *gt = reinterpret_cast<float *const *>(gbar->d_tab);
    const dim3 grid((unsigned)L->chunks.size()), block(BLOCK);
    hipLaunchKernelGGL(lars_reduce_ragged, grid, block, 0, s, L->d_chunks, L->d_sizes, xt, gt, tabs, c.n, L->tile,
                       (float)c.M, L->d_partials);
    hipLaunchKernelGGL(lars_rates, dim3((unsigned)L->sizes.size()), dim3(BLOCK), 0, s, L->d_chunk_begin,
                       L->d_partials, L->d_step, (double)lr, (double)wd, (double)eta);
    hipLaunchKernelGGL(lars_update_ragged, grid, block, 0, s, L->d_chunks, L->d_sizes, xt, vt, gt, L->d_step,
                       L->tile, mu, wd);
    return launch_status();
}

// --------------------------------------------------------- double buffer

static int ctx_set_streams(abs_ctx *C, const hipStream_t *streams, int n)
{
    for (hipEvent_t e : C->ev_acc) (void)hipEventDestroy(e);
    C->ev_acc.clear();
    C->s_acc.assign(streams, streams + n);
    C->slot.resize((size_t)C->K);
    for (int k = 0; k < C->K; ++k) C->slot[(size_t)k] = k % n;
    C->launches.assign((size_t)C->K, 0);
    C->joins = false;
    for (hipStream_t s : C->s_acc) C->joins = C->joins || s != C->s_upd;
    if (C->joins) {
        if (!C->ev_upd) ABS_HIP(hipEventCreateWithFlags(&C->ev_upd, hipEventDisableTiming));
        for (int i = 0; i < n; ++i) {
            hipEvent_t e = nullptr;
            ABS_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            C->ev_acc.push_back(e);
        }
    }
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
        if (P > 0 && (!acc_A[k] || !acc_B[k] || acc_A[k] == acc_B[k])) return ABS_EINVAL;
        if (!aligned_to(acc_A[k], 4) || !aligned_to(acc_B[k], 4)) return ABS_EINVAL;
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
        if (!set_ok(acc_A[k], L) || !set_ok(acc_B[k], L) || acc_A[k] == acc_B[k]) return ABS_EINVAL;
        if (acc_A[k]->elem != ABS_F32 || acc_B[k]->elem != ABS_F32) return ABS_EINVAL;
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

int abs_ctx_accumulate(abs_ctx *C, int k, const void *grad, abs_dtype grad_dtype, int64_t n_samples)
{
    if (!C || C->layout || k < 0 || k >= C->K) return ABS_EINVAL;
    C->launches[(size_t)k] += 1;
    return abs_accumulate(C->acc[C->cur][(size_t)k], grad, grad_dtype, C->P, n_samples,
                          &C->counts[C->cur][(size_t)k], C->stream_of(k));
}

int abs_ctx_accumulate_batch(abs_ctx *C, int k, const void *const *grads, abs_dtype grad_dtype, int J,
                             const int64_t *n_samples)
{
    if (!C || C->layout || k < 0 || k >= C->K) return ABS_EINVAL;
    C->launches[(size_t)k] += J > 0 ? (J + ABS_MAX_BATCH - 1) / ABS_MAX_BATCH : 0;
    return abs_accumulate_batch(C->acc[C->cur][(size_t)k], grads, grad_dtype, J, C->P, n_samples,
                                &C->counts[C->cur][(size_t)k], C->stream_of(k));
}

int abs_ctx_accumulate_batch_mt(abs_ctx *C, int k, const abs_tensorset *const *grads, int J,
                                const int64_t *n_samples)
{
    if (!C || !C->layout || k < 0 || k >= C->K) return ABS_EINVAL;
    C->launches[(size_t)k] += J > 0 ? (J + ABS_MAX_BATCH - 1) / ABS_MAX_BATCH : 0;
    return abs_accumulate_batch_mt(C->layout, C->set[C->cur][(size_t)k], grads, J, n_samples,
                                   &C->counts[C->cur][(size_t)k], C->stream_of(k));
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

int abs_ctx_accumulate_mt(abs_ctx *C, int k, const abs_tensorset *grad, int64_t n_samples)
{
    if (!C || !C->layout || k < 0 || k >= C->K) return ABS_EINVAL;
    C->launches[(size_t)k] += 1;
    return abs_accumulate_mt(C->layout, C->set[C->cur][(size_t)k], grad, n_samples,
                             &C->counts[C->cur][(size_t)k], C->stream_of(k));
}

int abs_ctx_sync_update(abs_ctx *C, float *params, float *momentum, float lr, float mu, float wd)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update(params, momentum, C->acc[prev].data(), C->counts[prev].data(), C->K, C->P,
                           lr, mu, wd, C->s_upd);
}

int abs_ctx_sync_update_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *momentum,
                           float lr, float mu, float wd)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update_mt(C->layout, params, momentum, C->set[prev].data(), C->counts[prev].data(),
                              C->K, lr, mu, wd, C->s_upd);
}

int abs_ctx_sync_update_dc(abs_ctx *C, float *params, float *params_prev, float *momentum, float lr,
                           float mu, float wd, float lambda)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update_dc(params, params_prev, momentum, C->acc[prev].data(), C->counts[prev].data(),
                              C->K, C->P, lr, mu, wd, lambda, C->s_upd);
}

int abs_ctx_sync_update_dc_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *params_prev,
                              const abs_tensorset *momentum, float lr, float mu, float wd, float lambda)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update_dc_mt(C->layout, params, params_prev, momentum, C->set[prev].data(),
                                 C->counts[prev].data(), C->K, lr, mu, wd, lambda, C->s_upd);
}

int abs_ctx_sync_update_dcm(abs_ctx *C, float *params, float *momentum, float lr, float mu, float wd,
                            float lambda)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    const int rc = abs_sync_update_dcm(params, momentum, C->acc[prev].data(), C->counts[prev].data(), C->K,
                                       C->P, lr, mu, wd, lambda, C->lr_applied, C->s_upd);
    if (rc == ABS_OK) C->lr_applied = lr;
    else if (rc == ABS_EMPTY) C->lr_applied = 0.f;
    return rc;
}

int abs_ctx_sync_update_dcm_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *momentum,
                               float lr, float mu, float wd, float lambda)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    const int rc = abs_sync_update_dcm_mt(C->layout, params, momentum, C->set[prev].data(),
                                          C->counts[prev].data(), C->K, lr, mu, wd, lambda, C->lr_applied,
                                          C->s_upd);
    if (rc == ABS_OK) C->lr_applied = lr;
    else if (rc == ABS_EMPTY) C->lr_applied = 0.f;
    return rc;
}

int abs_ctx_sync_update_adam(abs_ctx *C, float *params, float *exp_avg, float *exp_avg_sq, float lr,
                             float beta1, float beta2, float eps, float wd, int64_t step)
{
    if (!C || C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update_adam(params, exp_avg, exp_avg_sq, C->acc[prev].data(), C->counts[prev].data(),
                                C->K, C->P, lr, beta1, beta2, eps, wd, step, C->s_upd);
}

int abs_ctx_sync_update_adam_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *exp_avg,
                                const abs_tensorset *exp_avg_sq, float lr, float beta1, float beta2,
                                float eps, float wd, int64_t step)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update_adam_mt(C->layout, params, exp_avg, exp_avg_sq, C->set[prev].data(),
                                   C->counts[prev].data(), C->K, lr, beta1, beta2, eps, wd, step, C->s_upd);
}

int abs_ctx_sync_update_lars_mt(abs_ctx *C, const abs_tensorset *params, const abs_tensorset *momentum,
                                const abs_tensorset *gbar, float lr, float mu, float wd, float eta)
{
    if (!C || !C->layout) return ABS_EINVAL;
    const int prev = C->cur ^ 1;
    return abs_sync_update_lars_mt(C->layout, params, momentum, gbar, C->set[prev].data(),
                                   C->counts[prev].data(), C->K, lr, mu, wd, eta, C->s_upd);
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
