// Launches of the one-worker accumulate kernels (flat and ragged, J = 1..8
// gradients per launch), of the copy kernels and of the three LARS kernels.
#include "abs_kernels_aux.hpp"

#include "abs_host.hpp"

#include <cstring>

using namespace absk;

namespace absh {

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

namespace {

template <bool BF16, int J>
void accumulate_flat_j(float *acc, const void *const *grads, const float *nf, int64_t P, int tile,
                       unsigned nblocks, int first, int vec_ok, bool nta, int64_t per, hipStream_t s)
{
    GradArgs<BF16, J> G;
    for (int j = 0; j < J; ++j) {
        G.g[j] = static_cast<const typename GradT<BF16>::elem *>(grads[j]);
        G.n[j] = nf[j];
    }
    const dim3 block(BLOCK);
    for_slices(nblocks, per, [&](unsigned b0, unsigned n) {
        if (nta) hipLaunchKernelGGL((accumulate_flat<BF16, true, J>), dim3(n), block, 0, s, acc, G, P, tile, first, vec_ok, b0);
        else hipLaunchKernelGGL((accumulate_flat<BF16, false, J>), dim3(n), block, 0, s, acc, G, P, tile, first, vec_ok, b0);
    });
}

template <int J>
void accumulate_ragged_j(const RaggedView &L, float *const *at, const void *const *const *gt, const float *nf,
                         int first, bool bf, bool nta, int64_t per, hipStream_t s)
{
    GradTabs<J> T;
    for (int j = 0; j < J; ++j) {
        T.t[j] = gt[j];
        T.n[j] = nf[j];
    }
    const dim3 block(BLOCK);
    for_slices(L.nchunks, per, [&](unsigned b0, unsigned n) {
        const dim3 grid(n);
        if (bf && nta) hipLaunchKernelGGL((accumulate_ragged<true, true, J>), grid, block, 0, s, L.chunks, L.sizes, at, T, L.tile, first, b0);
        else if (bf) hipLaunchKernelGGL((accumulate_ragged<true, false, J>), grid, block, 0, s, L.chunks, L.sizes, at, T, L.tile, first, b0);
        else if (nta) hipLaunchKernelGGL((accumulate_ragged<false, true, J>), grid, block, 0, s, L.chunks, L.sizes, at, T, L.tile, first, b0);
        else hipLaunchKernelGGL((accumulate_ragged<false, false, J>), grid, block, 0, s, L.chunks, L.sizes, at, T, L.tile, first, b0);
    });
}

}  // namespace

int launch_accumulate_flat(const Tuning &tu, float *acc, const void *const *grads, const float *nf, int J,
                           abs_dtype dt, int64_t P, int first, int vec_ok, hipStream_t s)
{
    const int64_t tile64 = choose_tile(rows_of(P), acc_resident(tu), tu.max_rows);
    if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
    const int tile = (int)tile64;
    const unsigned nb = (unsigned)tiles_for(P, tile64);
    const bool bf = dt == ABS_BF16, nta = stream_acc(tu, P);
    const int64_t per = slice_wgs(tu, nb, P * (J * (bf ? 2 : 4) + (first ? 4 : 8)), acc_resident(tu));
    switch (J) {
#define ABS_CASE(N)                                                                                   \
    case N:                                                                                           \
        if (bf) accumulate_flat_j<true, N>(acc, grads, nf, P, tile, nb, first, vec_ok, nta, per, s);  \
        else accumulate_flat_j<false, N>(acc, grads, nf, P, tile, nb, first, vec_ok, nta, per, s);    \
        break;
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
#undef ABS_CASE
    default: return ABS_EINVAL;
    }
    return ABS_OK;
}

int launch_accumulate_ragged(const Tuning &tu, const RaggedView &L, float *const *acc_tab,
                             const void *const *const *grad_tabs, const float *nf, int J, abs_dtype dt,
                             int first, hipStream_t s)
{
    const bool bf = dt == ABS_BF16, nta = stream_acc(tu, L.total);
    const int64_t per = slice_wgs(tu, L.nchunks, L.total * (J * (bf ? 2 : 4) + (first ? 4 : 8)), acc_resident(tu));
    switch (J) {
#define ABS_CASE(N) case N: accumulate_ragged_j<N>(L, acc_tab, grad_tabs, nf, first, bf, nta, per, s); break;
        ABS_CASE(1) ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8)
#undef ABS_CASE
    default: return ABS_EINVAL;
    }
    return ABS_OK;
}

int launch_copy_flat(const Tuning &tu, float *dst, const float *src, int64_t P, hipStream_t s)
{
    const int64_t tile64 = choose_tile(rows_of(P), acc_resident(tu), tu.max_rows);
    if (tile64 > kMaxTile || tiles_for(P, tile64) > kMaxGrid) return ABS_EINVAL;
    const int vec_ok = ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) == 0;
    hipLaunchKernelGGL(copy_flat, dim3((unsigned)tiles_for(P, tile64)), dim3(BLOCK), 0, s, dst, src, P,
                       (int)tile64, vec_ok);
    ++t_launches;
    return ABS_OK;
}

int launch_copy_ragged(const RaggedView &L, float *const *dst_tab, float *const *src_tab, hipStream_t s)
{
    hipLaunchKernelGGL(copy_ragged, dim3(L.nchunks), dim3(BLOCK), 0, s, L.chunks, L.sizes, dst_tab, src_tab,
                       L.tile);
    ++t_launches;
    return ABS_OK;
}

int launch_lars_chunk_begin(const RaggedView &L, int32_t *chunk_begin, hipStream_t s)
{
    const unsigned threads = L.nchunks + 1;
    hipLaunchKernelGGL(lars_chunk_begin, dim3((threads + BLOCK - 1) / BLOCK), dim3(BLOCK), 0, s, L.chunks,
                       (int)L.nchunks, L.ntensors, chunk_begin);
    ++t_launches;
    return ABS_OK;
}

int launch_lars(const Tuning &tu, const RaggedView &L, float *const *xt, float *const *vt, float *const *gt,
                const float *const *const *tabs, int n, float M, float lr, float mu, float wd, float eta,
                const LarsScratch &sc, hipStream_t s)
{
    if (n < 1 || n > ABS_MAX_K) return ABS_EINVAL;
    TabPtrsAny T;
    std::memset(&T, 0, sizeof T);
    for (int k = 0; k < n; ++k) T.t[k] = tabs[k];
    const dim3 block(BLOCK);
    // K accumulators and x read, Gbar written; then Gbar, x and v read, x and v written
    for_slices(L.nchunks, slice_wgs(tu, L.nchunks, L.total * (4 * n + 8), resident(tu, 4)), [&](unsigned b0, unsigned nb) {
        hipLaunchKernelGGL(lars_reduce_ragged, dim3(nb), block, 0, s, L.chunks, L.sizes, xt, gt, T, n, L.tile, M,
                           sc.partials, b0);
    });
    hipLaunchKernelGGL(lars_rates, dim3((unsigned)L.ntensors), dim3(BLOCK), 0, s, sc.chunk_begin, sc.partials,
                       sc.step, (double)lr, (double)wd, (double)eta);
    ++t_launches;
    for_slices(L.nchunks, slice_wgs(tu, L.nchunks, L.total * 20, resident(tu, 4)), [&](unsigned b0, unsigned nb) {
        hipLaunchKernelGGL(lars_update_ragged, dim3(nb), block, 0, s, L.chunks, L.sizes, xt, vt, gt, sc.step, L.tile, mu,
                           wd, b0);
    });
    return ABS_OK;
}

}  // namespace absh
