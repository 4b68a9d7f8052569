// Launches of the job-list accumulate kernels: one launch for several workers.
#include "abs_kernels.hpp"

#include "abs_host.hpp"

using namespace absk;

namespace absh {

namespace {

// Workgroups of `kernel` one CU can hold, from the runtime's occupancy calculator.
template <class Kernel>
int occupancy_per_cu(Kernel kernel, int fallback)
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, BLOCK, 0) == hipSuccess && n > 0) return n;
    (void)hipGetLastError();
    return fallback;
}

// The tile is chosen as if the jobs were one vector of njobs * P elements, so that
// the whole launch, not each job, is a whole number of resident rounds.
template <bool BF16, int JMAX>
int jobs_flat(const Tuning &tu, const JobList &jobs, int njobs, int64_t P, hipStream_t s)
{
    int64_t bytes = 0;
    for (int i = 0; i < njobs; ++i) bytes += P * (jobs.job[i].J * (BF16 ? 2 : 4) + (jobs.job[i].first ? 4 : 8));
    static const int per_cu = occupancy_per_cu(accumulate_jobs_flat<BF16, false, JMAX>, 4);
    const int64_t tile64 = choose_tile(rows_of(P) * njobs, resident(tu, per_cu), tu.max_rows);
    const int64_t tiles = tiles_for(P, tile64);
    if (tile64 > kMaxTile || tiles * njobs > kMaxGrid) return ABS_EINVAL;
    // one-dimensional: workgroup b works on tile b % tiles of job b / tiles, the jobs one after the other
    const dim3 block(BLOCK);
    const bool nta = stream_jobs(tu, P, njobs);
    for_slices(tiles * njobs, slice_wgs(tu, tiles * njobs, bytes, resident(tu, per_cu)), [&](unsigned b0, unsigned n) {
        if (nta)
            hipLaunchKernelGGL((accumulate_jobs_flat<BF16, true, JMAX>), dim3(n), block, 0, s, jobs, P, (int)tile64, (unsigned)tiles, b0);
        else
            hipLaunchKernelGGL((accumulate_jobs_flat<BF16, false, JMAX>), dim3(n), block, 0, s, jobs, P, (int)tile64, (unsigned)tiles, b0);
    });
    return ABS_OK;
}

template <bool BF16, int JMAX>
int jobs_ragged(const Tuning &tu, const RaggedView &L, const JobList &jobs, int njobs, hipStream_t s)
{
    if ((int64_t)L.nchunks * njobs > kMaxGrid) return ABS_EINVAL;
    int64_t bytes = 0;
    for (int i = 0; i < njobs; ++i) bytes += L.total * (jobs.job[i].J * (BF16 ? 2 : 4) + (jobs.job[i].first ? 4 : 8));
    const dim3 block(BLOCK);
    const bool nta = stream_jobs(tu, L.total, njobs);
    const int64_t wgs = (int64_t)L.nchunks * njobs;
    for_slices(wgs, slice_wgs(tu, wgs, bytes, acc_resident(tu)), [&](unsigned b0, unsigned n) {
        if (nta)
            hipLaunchKernelGGL((accumulate_jobs_ragged<BF16, true, JMAX>), dim3(n), block, 0, s, L.chunks, L.sizes, jobs, L.tile, L.nchunks, b0);
        else
            hipLaunchKernelGGL((accumulate_jobs_ragged<BF16, false, JMAX>), dim3(n), block, 0, s, L.chunks, L.sizes, jobs, L.tile, L.nchunks, b0);
    });
    return ABS_OK;
}

}  // namespace

int launch_accumulate_jobs_flat(const Tuning &tu, const JobList &jobs, int njobs, int jmax, abs_dtype dt,
                                int64_t P, hipStream_t s)
{
    if (njobs < 1 || njobs > MAX_JOBS || jmax < 1 || jmax > ABS_MAX_BATCH) return ABS_EINVAL;
    const bool bf = dt == ABS_BF16;
    if (jmax == 1) return bf ? jobs_flat<true, 1>(tu, jobs, njobs, P, s) : jobs_flat<false, 1>(tu, jobs, njobs, P, s);
    if (jmax == 2) return bf ? jobs_flat<true, 2>(tu, jobs, njobs, P, s) : jobs_flat<false, 2>(tu, jobs, njobs, P, s);
    if (jmax <= 4) return bf ? jobs_flat<true, 4>(tu, jobs, njobs, P, s) : jobs_flat<false, 4>(tu, jobs, njobs, P, s);
    return bf ? jobs_flat<true, 8>(tu, jobs, njobs, P, s) : jobs_flat<false, 8>(tu, jobs, njobs, P, s);
}

int launch_accumulate_jobs_ragged(const Tuning &tu, const RaggedView &L, const JobList &jobs, int njobs,
                                  int jmax, abs_dtype dt, hipStream_t s)
{
    if (njobs < 1 || njobs > MAX_JOBS || jmax < 1 || jmax > ABS_MAX_BATCH) return ABS_EINVAL;
    const bool bf = dt == ABS_BF16;
    if (jmax == 1) return bf ? jobs_ragged<true, 1>(tu, L, jobs, njobs, s) : jobs_ragged<false, 1>(tu, L, jobs, njobs, s);
    if (jmax == 2) return bf ? jobs_ragged<true, 2>(tu, L, jobs, njobs, s) : jobs_ragged<false, 2>(tu, L, jobs, njobs, s);
    if (jmax <= 4) return bf ? jobs_ragged<true, 4>(tu, L, jobs, njobs, s) : jobs_ragged<false, 4>(tu, L, jobs, njobs, s);
    return bf ? jobs_ragged<true, 8>(tu, L, jobs, njobs, s) : jobs_ragged<false, 8>(tu, L, jobs, njobs, s);
}

}  // namespace absh
