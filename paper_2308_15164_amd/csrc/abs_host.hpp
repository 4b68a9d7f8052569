// Host-side declarations shared by the translation units of the library: the
// settings a call works with, the launch-shape rule, and the launch functions
// (defined next to the kernels they instantiate, one unit per kernel family so
// that the units compile in parallel).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "abs_sgd.h"
#include "abs_types.hpp"

#ifndef ABS_ACC_STREAM_BYTES
#define ABS_ACC_STREAM_BYTES (int64_t(160) << 20)
#endif
#ifndef ABS_JOBS_STREAM_BYTES
#define ABS_JOBS_STREAM_BYTES (int64_t(224) << 20)
#endif
#ifndef ABS_MAX_ROWS
#define ABS_MAX_ROWS 4
#endif
#ifndef ABS_UPD_STREAM_BYTES
#define ABS_UPD_STREAM_BYTES (int64_t(256) << 20)
#endif
#ifndef ABS_SLICE_BYTES
#define ABS_SLICE_BYTES (int64_t(1) << 30)
#endif

namespace absh {

using absk::BLOCK;
using absk::Chunk;
using absk::Hyper;
using absk::JobList;
using absk::ROW;

// The settings one call works with, read once at its start: the process-wide
// defaults, or a context's own.
struct Tuning {
    int blocks_per_cu;   // resident workgroups per CU to plan for; 0 = what the kernel's register use allows
    int max_rows;        // cap on rows per tile; 0 = none
    int policy_acc;      // cache policy of accumulator traffic: -1 from the sizes, 0 cached, 1 streaming
    int policy_upd;      // the same for x and the state vectors
    int64_t slice_bytes; // a call moving n times this many bytes goes in n launches; 0 = never cut
};

constexpr int64_t kMaxGrid = 0x7fffffff;
constexpr int64_t kMaxTile = int64_t(1) << 30;   // tile sizes travel as int

// Compute units of the current device; 256 (MI355X) when no device can be asked,
// e.g. when a layout is built on a host without a GPU.
int cu_count();

inline int64_t rows_of(int64_t P) { return (P + ROW - 1) / ROW; }
inline int64_t tiles_for(int64_t P, int64_t tile) { return (P + tile - 1) / tile; }

// A launch should fill the chip in whole rounds: with `resident` workgroups
// able to run at once, the tile is the smallest whole number of rows that
// covers n rows in `rounds` rounds, rounds being the fewest that keep a tile
// within max_rows rows (0 = no limit: always one round, every workgroup
// walks one long run of memory).  Measured on MI355X: short tiles (<= 4 rows,
// many rounds) beat long per-workgroup runs by 15-20 % at P >= 1e8, because all
// resident workgroups then sweep one compact window of memory.
inline int64_t choose_tile(int64_t rows, int resident, int max_rows)
{
    if (rows <= resident) return ROW;
    int64_t rounds = 1;
    if (max_rows > 0) rounds = (rows + (int64_t)resident * max_rows - 1) / ((int64_t)resident * max_rows);
    const int64_t slots = (int64_t)resident * rounds;
    return ((rows + slots - 1) / slots) * ROW;
}

// Workgroups resident on the whole chip, with the caller's override applied.
inline int resident(const Tuning &tu, int per_cu) { return (tu.blocks_per_cu > 0 ? tu.blocks_per_cu : per_cu) * cu_count(); }

// The one-gradient accumulate kernels need few registers: 8 workgroups of 4 wavefronts per CU.
constexpr int kAccBlocksPerCU = 8;
inline int acc_resident(const Tuning &tu) { return resident(tu, kAccBlocksPerCU); }

// Long launches lose rate on this part.  Measured at P = 1.38e8 with consecutive launches
// over sub-ranges of the same vectors: a launch moving 1-2 GB is as fast as any shorter
// one, but the sync-update over 8 workers (6.6 GB in one launch) gains 4-6 % when cut
// into 4-12 launches, over 16 workers (11 GB) 4-7 % in 6-12, an accumulate over a 2.2 GB
// vector (6.6 GB) 6 % in 4-8 -- and a job list of four 553 MB accumulators in one launch
// is 4-8 % SLOWER than four launches.  So a call is cut into floor(bytes / slice_bytes)
// launches over consecutive workgroup ranges (one launch below twice that), each a whole
// number of resident rounds.  One unit for every kernel, 1 GiB: kernels over few vectors
// (one to four gradients into an accumulator, the sync-update over up to four workers) are
// indifferent between 0.5 and 2 GiB and lose 1-3 % at 256 MiB; kernels over many vectors
// would take another 2-4 % from launches of one or two resident rounds (sync-update over 16
// workers: 5.6 TB/s uncut, 6.0 at 1 GiB, 6.1-6.2 at 48-256 MiB), but a step of the GPT-2-
// sized configuration then needs 270 launches and waits for the host, and launches that
// short lose where the buffers sit in the memory-side cache.
// Returns the workgroups per launch.
inline int64_t slice_wgs(const Tuning &tu, int64_t wgs, int64_t bytes, int resident_wgs)
{
    if (tu.slice_bytes <= 0) return wgs;
    const int64_t slices = bytes / tu.slice_bytes;
    if (slices <= 1 || wgs <= resident_wgs) return wgs;
    const int64_t per = (wgs + slices - 1) / slices;
    return ((per + resident_wgs - 1) / resident_wgs) * resident_wgs;
}

// Kernel launches this thread has enqueued through the library (abs_launch_count).
inline thread_local int64_t t_launches = 0;

// launch(b0, n) for every slice [b0, b0 + n) of `wgs` workgroups, `per` at a time.
template <class Launch>
inline void for_slices(int64_t wgs, int64_t per, Launch launch)
{
    for (int64_t b0 = 0; b0 < wgs; b0 += per) {
        launch((unsigned)b0, (unsigned)(wgs - b0 < per ? wgs - b0 : per));
        ++t_launches;
    }
}

// Accumulators, x and v are touched again soon after a kernel ends.  When they
// fit the memory-side cache (256 MiB on this part) keeping them cached pays;
// when they do not, streaming (non-temporal) accesses avoid allocating lines
// that are evicted before their reuse.
inline bool stream_acc(const Tuning &tu, int64_t P)
{
    return tu.policy_acc < 0 ? 4 * P > ABS_ACC_STREAM_BYTES : tu.policy_acc != 0;
}
// A job-list launch writes njobs accumulators one after the other; they are next read a
// launch (fold < m_k) or a whole iteration later, after everything else the launch moved.
// What decides is whether ALL of them together stay in the memory-side cache: measured,
// 4 x 47 MB (ResNet18-sized, K = 4) gains 2 % cached, 8 x 102 MB (ResNet50-sized, K = 8)
// gains 6 % streaming.
inline bool stream_jobs(const Tuning &tu, int64_t P, int njobs)
{
    return tu.policy_acc < 0 ? 4 * P * njobs > ABS_JOBS_STREAM_BYTES : tu.policy_acc != 0;
}
inline bool stream_upd(const Tuning &tu, int64_t P, int vectors)
{
    return tu.policy_upd < 0 ? 4 * vectors * P > ABS_UPD_STREAM_BYTES : tu.policy_upd != 0;
}

// What a ragged launch needs of a layout: its device-resident tables.
struct RaggedView {
    const Chunk *chunks;      // DEVICE, nchunks entries
    const int64_t *sizes;     // DEVICE, one per tensor
    unsigned nchunks;
    int ntensors;
    int tile;
    int64_t total;
};

// Scratch of the LARS launches (DEVICE): per-chunk sums of squares (2 doubles per
// chunk), per-tensor step factors, first chunk of every tensor (ntensors + 1).
struct LarsScratch {
    double *partials;
    float *step;
    int32_t *chunk_begin;
};

// ---- launches.  Each enqueues on `s` and returns ABS_OK or ABS_EINVAL (a shape the
// grid cannot express); launch errors are read by the caller with hipGetLastError.

// J <= ABS_MAX_BATCH gradients into one accumulator.
int launch_accumulate_flat(const Tuning &tu, float *acc, const void *const *grads, const float *nf, int J,
                           abs_dtype dt, int64_t P, int first, int vec_ok, hipStream_t s);
int launch_accumulate_ragged(const Tuning &tu, const RaggedView &L, float *const *acc_tab,
                             const void *const *const *grad_tabs, const float *nf, int J, abs_dtype dt,
                             int first, hipStream_t s);

// njobs <= MAX_JOBS jobs, every job's J within 1..jmax, jmax <= ABS_MAX_BATCH.
int launch_accumulate_jobs_flat(const Tuning &tu, const JobList &jobs, int njobs, int jmax, abs_dtype dt,
                                int64_t P, hipStream_t s);
int launch_accumulate_jobs_ragged(const Tuning &tu, const RaggedView &L, const JobList &jobs, int njobs,
                                  int jmax, abs_dtype dt, hipStream_t s);

// Fused combine + update over n non-empty workers; one explicit instantiation per rule.
template <int RULE>
int launch_sync_flat_r(const Tuning &tu, float *x, float *s1, float *s2, const float *const *ptrs, int n,
                       int64_t P, const Hyper &h, int vec_ok, hipStream_t s);
template <int RULE>
int launch_sync_ragged_r(const Tuning &tu, const RaggedView &L, float *const *xt, float *const *s1t,
                         float *const *s2t, const float *const *const *tabs, int n, const Hyper &h,
                         hipStream_t s);

int launch_copy_flat(const Tuning &tu, float *dst, const float *src, int64_t P, hipStream_t s);
int launch_copy_ragged(const RaggedView &L, float *const *dst_tab, float *const *src_tab, hipStream_t s);

// First chunk of every tensor, from the chunk table (one small launch).
int launch_lars_chunk_begin(const RaggedView &L, int32_t *chunk_begin, hipStream_t s);
// The three LARS launches; chunk_begin must already be valid in `sc` on the stream.
int launch_lars(const Tuning &tu, const RaggedView &L, float *const *xt, float *const *vt, float *const *gt,
                const float *const *const *tabs, int n, float M, float lr, float mu, float wd, float eta,
                const LarsScratch &sc, hipStream_t s);

}  // namespace absh
