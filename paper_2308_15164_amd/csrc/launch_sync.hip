// Launches of the fused combine + update kernels for ONE update rule: this file
// is compiled once per rule (-DABS_RULE=0..3, the values of absk::Rule), which
// keeps the units small enough to build side by side.
#include "abs_kernels.hpp"

#include "abs_host.hpp"

#include <cstring>

#ifndef ABS_RULE
#error "compile with -DABS_RULE=<value of absk::Rule>"
#endif

using namespace absk;

namespace absh {

namespace {

template <class Kernel>
int occupancy_per_cu(Kernel kernel, int fallback)
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, BLOCK, 0) == hipSuccess && n > 0) return n;
    (void)hipGetLastError();
    return fallback;
}

template <int K, int RULE>
int sync_flat_k(const Tuning &tu, float *x, float *v, float *xp, const float *const *ptrs, int64_t P,
                const Hyper &h, int vec_ok, hipStream_t s)
{
    static const int per_cu = occupancy_per_cu(sync_update_flat<K, false, RULE>, 4);
    const int64_t tile64 = choose_tile(rows_of(P), resident(tu, per_cu), tu.max_rows);
    if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
    const int tile = (int)tile64;
    AccPtrs<K> A;
    for (int k = 0; k < K; ++k) A.p[k] = ptrs[k];
    const dim3 block(BLOCK);
    // x and each state vector are re-read one iteration later
    const bool ntx = stream_upd(tu, P, uses_s2<RULE>() ? 3 : 2);
    const int64_t wgs = tiles_for(P, tile64);
    for_slices(wgs, slice_wgs(tu, wgs, P * (4 * K + (uses_s2<RULE>() ? 24 : 16)), resident(tu, per_cu)), [&](unsigned b0, unsigned n) {
        if (ntx)
            hipLaunchKernelGGL((sync_update_flat<K, true, RULE>), dim3(n), block, 0, s, x, v, xp, A, P, tile, h, vec_ok, b0);
        else
            hipLaunchKernelGGL((sync_update_flat<K, false, RULE>), dim3(n), block, 0, s, x, v, xp, A, P, tile, h, vec_ok, b0);
    });
    return ABS_OK;
}

template <int K, int RULE>
void sync_ragged_k(const Tuning &tu, const RaggedView &L, float *const *xt, float *const *vt, float *const *pt,
                   const float *const *const *tabs, const Hyper &h, hipStream_t s)
{
    TabPtrs<K> T;
    for (int k = 0; k < K; ++k) T.t[k] = tabs[k];
    const dim3 block(BLOCK);
    const bool ntx = stream_upd(tu, L.total, uses_s2<RULE>() ? 3 : 2);
    for_slices(L.nchunks, slice_wgs(tu, L.nchunks, L.total * (4 * K + (uses_s2<RULE>() ? 24 : 16)), resident(tu, 4)), [&](unsigned b0, unsigned n) {
        if (ntx)
            hipLaunchKernelGGL((sync_update_ragged<K, true, RULE>), dim3(n), block, 0, s, L.chunks, L.sizes, xt, vt, pt, T, L.tile, h, b0);
        else
            hipLaunchKernelGGL((sync_update_ragged<K, false, RULE>), dim3(n), block, 0, s, L.chunks, L.sizes, xt, vt, pt, T, L.tile, h, b0);
    });
}

}  // namespace

// Workers up to this many get a kernel of their own (the K-way read fully unrolled);
// beyond it the run-time-K kernels loop over batches of workers.
constexpr int kMaxSpecialisedK = 8;

template <int RULE>
int launch_sync_flat_r(const Tuning &tu, float *x, float *s1, float *s2, const float *const *ptrs, int n,
                       int64_t P, const Hyper &h, int vec_ok, hipStream_t s)
{
    switch (n) {
#define ABS_CASE(K) case K: return sync_flat_k<K, RULE>(tu, x, s1, s2, ptrs, P, h, vec_ok, s);
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
#undef ABS_CASE
    default: {
        static_assert(kMaxSpecialisedK == 8, "the cases above");
        if (n < 1 || n > ABS_MAX_K) return ABS_EINVAL;
        static const int per_cu = occupancy_per_cu(sync_update_flat_any<RULE, false>, 3);
        const int64_t tile64 = choose_tile(rows_of(P), resident(tu, per_cu), tu.max_rows);
        if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
        AccPtrsAny A;
        std::memset(&A, 0, sizeof A);
        for (int k = 0; k < n; ++k) A.p[k] = ptrs[k];
        const dim3 block(BLOCK);
        const bool ntx = stream_upd(tu, P, uses_s2<RULE>() ? 3 : 2);
        const int64_t wgs = tiles_for(P, tile64);
        for_slices(wgs, slice_wgs(tu, wgs, P * (4 * n + (uses_s2<RULE>() ? 24 : 16)), resident(tu, per_cu)), [&](unsigned b0, unsigned nb) {
            if (ntx)
                hipLaunchKernelGGL((sync_update_flat_any<RULE, true>), dim3(nb), block, 0, s, x, s1, s2, A, n, P, (int)tile64, h, vec_ok, b0);
            else
                hipLaunchKernelGGL((sync_update_flat_any<RULE, false>), dim3(nb), block, 0, s, x, s1, s2, A, n, P, (int)tile64, h, vec_ok, b0);
        });
        return ABS_OK;
    }
    }
}

template <int RULE>
int launch_sync_ragged_r(const Tuning &tu, const RaggedView &L, float *const *xt, float *const *s1t,
                         float *const *s2t, const float *const *const *tabs, int n, const Hyper &h,
                         hipStream_t s)
{
    switch (n) {
#define ABS_CASE(K) case K: sync_ragged_k<K, RULE>(tu, L, xt, s1t, s2t, tabs, h, s); return ABS_OK;
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
#undef ABS_CASE
    default: {
        if (n < 1 || n > ABS_MAX_K) return ABS_EINVAL;
        TabPtrsAny T;
        std::memset(&T, 0, sizeof T);
        for (int k = 0; k < n; ++k) T.t[k] = tabs[k];
        const dim3 block(BLOCK);
        const bool ntx = stream_upd(tu, L.total, uses_s2<RULE>() ? 3 : 2);
        for_slices(L.nchunks, slice_wgs(tu, L.nchunks, L.total * (4 * n + (uses_s2<RULE>() ? 24 : 16)), resident(tu, 3)), [&](unsigned b0, unsigned nb) {
            if (ntx)
                hipLaunchKernelGGL((sync_update_ragged_any<RULE, true>), dim3(nb), block, 0, s, L.chunks, L.sizes, xt, s1t, s2t, T, n, L.tile, h, b0);
            else
                hipLaunchKernelGGL((sync_update_ragged_any<RULE, false>), dim3(nb), block, 0, s, L.chunks, L.sizes, xt, s1t, s2t, T, n, L.tile, h, b0);
        });
        return ABS_OK;
    }
    }
}

template int launch_sync_flat_r<ABS_RULE>(const Tuning &, float *, float *, float *, const float *const *, int,
                                          int64_t, const Hyper &, int, hipStream_t);
template int launch_sync_ragged_r<ABS_RULE>(const Tuning &, const RaggedView &, float *const *, float *const *,
                                            float *const *, const float *const *const *, int, const Hyper &,
                                            hipStream_t);

}  // namespace absh
