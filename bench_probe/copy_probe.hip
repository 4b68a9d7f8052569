// Plain streaming kernels of known size, separate from the method's library.
// They serve two purposes in the benchmark: (1) calibrating the profiler's
// HBM byte counters against a transfer whose size is known, and (2) measuring
// what the box's memory system gives to plain kernels with the traffic mixes of
// the method's kernels: copy, read, write, triad (a += s*b: two reads and a
// write, the steady accumulate), R vectors read of which two are written in
// place (the fused combine + update over R - 2 workers), and the same R
// vectors only read (what the write stream costs).  Nothing in the method calls them.
//
// One shape for all of them: a workgroup of 256 lanes owns 4 rows of 256
// 128-bit vectors per stream, issues every load of its tile before the first
// use, then stores.  Tiles that lie wholly inside the vector take a path
// without bounds checks (straight-line code: the compiler keeps all loads in
// flight); only the last tile checks.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int BLOCK = 256;
constexpr int VPT = 4;           // rows per workgroup
constexpr int MAXR = 18;

struct Streams { f32x4 *p[MAXR]; };

// R streams read and summed; W output streams: W = 0 none (the sum only feeds a
// never-taken branch), else out[w] = sum * (w + 1) * scale.  INPLACE: the outputs
// are the first W read streams; otherwise they are p[R], p[R + 1].
template <int R, int W, bool INPLACE, bool WHOLE>
__device__ __forceinline__ void tile(const Streams &S, int64_t nvec, float scale, float *sink)
{
    // The tile's base is uniform over the workgroup and the lane's part of the index fits 32 bits:
    // every access is (scalar base) + (32-bit lane offset), which leaves the registers to the data.
    const int64_t tile0 = (int64_t)blockIdx.x * (BLOCK * VPT);
    const int lane = threadIdx.x;
    const int left = (int)(nvec - tile0 < BLOCK * VPT ? nvec - tile0 : BLOCK * VPT);   // vectors of this tile
    f32x4 a[VPT][R > 0 ? R : 1];
    if constexpr (R > 0) {
        // stream by stream: 4 KiB of one stream per wavefront before the next stream is touched
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const f32x4 *p = S.p[r] + tile0;
#pragma unroll
            for (int u = 0; u < VPT; ++u) {
                const int i = lane + u * BLOCK;
                if (WHOLE || i < left) a[u][r] = __builtin_nontemporal_load(p + i);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int i = lane + u * BLOCK;
        if (WHOLE || i < left) {
            f32x4 s = {scale, scale, scale, scale};
            if constexpr (R > 0) {
                s = a[u][0];
#pragma unroll
                for (int r = 1; r < R; ++r) s += a[u][r];
            }
            if constexpr (W == 0) {
                // never true for finite data: keeps the loads alive without a store stream
                if (s.x + s.y + s.z + s.w == 1.2345678e38f) *sink = s.x;
            } else {
#pragma unroll
                for (int w = 0; w < W; ++w)
                    __builtin_nontemporal_store(R > 0 ? s * (scale * (w + 1)) : s, S.p[INPLACE ? w : R + w] + tile0 + i);
            }
        }
    }
}

template <int R, int W, bool INPLACE>
__global__ __launch_bounds__(BLOCK) void probe_kernel(Streams S, int64_t nvec, float scale, float *sink)
{
    if (((int64_t)blockIdx.x + 1) * (BLOCK * VPT) <= nvec) tile<R, W, INPLACE, true>(S, nvec, scale, sink);
    else tile<R, W, INPLACE, false>(S, nvec, scale, sink);
}

inline unsigned grid_for(int64_t nvec) { return (unsigned)((nvec + BLOCK * VPT - 1) / (BLOCK * VPT)); }
inline bool bad(const void *p) { return !p || ((uintptr_t)p & 15); }

template <int R, int W, bool INPLACE>
int launch(void *const *ptrs, int n, int64_t nbytes, float scale, float *sink, void *stream)
{
    if (nbytes <= 0 || (nbytes & 15)) return -1;
    Streams S = {};
    for (int r = 0; r < n; ++r) {
        if (bad(ptrs[r])) return -1;
        S.p[r] = (f32x4 *)ptrs[r];
    }
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL((probe_kernel<R, W, INPLACE>), dim3(grid_for(nvec)), dim3(BLOCK), 0, (hipStream_t)stream, S, nvec,
                       scale, sink);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
}  // namespace

extern "C" {

// All pointers DEVICE, 16-byte aligned; nbytes a multiple of 16 per vector.  Returns 0 or -1.

int probe_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    void *p[2] = {const_cast<void *>(src), dst};
    return launch<1, 1, false>(p, 2, nbytes, 1.0f, nullptr, stream);
}

int probe_read(const void *src, int64_t nbytes, float *sink, void *stream)
{
    void *p[1] = {const_cast<void *>(src)};
    if (!sink) return -1;
    return launch<1, 0, false>(p, 1, nbytes, 1.0f, sink, stream);
}

int probe_write(void *dst, int64_t nbytes, float val, void *stream)
{
    void *p[1] = {dst};
    return launch<0, 1, false>(p, 1, nbytes, val, nullptr, stream);
}

// a (read and written) and b (read): a = (a + b) * s.
int probe_triad(void *a, const void *b, int64_t nbytes, float s, void *stream)
{
    void *p[2] = {a, const_cast<void *>(b)};
    return launch<2, 1, true>(p, 2, nbytes, s, nullptr, stream);
}

// ptrs: HOST array of R DEVICE pointers (R = 6, 10 or 18: the shapes of K = 4, 8, 16
// workers), nbytes each; all are read, the first two are also written.
int probe_mix(void *const *ptrs, int R, int64_t nbytes, void *stream)
{
    if (!ptrs) return -1;
    switch (R) {
    case 6: return launch<6, 2, true>(ptrs, R, nbytes, 0.5f, nullptr, stream);
    case 10: return launch<10, 2, true>(ptrs, R, nbytes, 0.5f, nullptr, stream);
    case 18: return launch<18, 2, true>(ptrs, R, nbytes, 0.5f, nullptr, stream);
    default: return -1;
    }
}

// The same R vectors read and nothing written.
int probe_readk(void *const *ptrs, int R, int64_t nbytes, float *sink, void *stream)
{
    if (!ptrs || !sink) return -1;
    switch (R) {
    case 6: return launch<6, 0, false>(ptrs, R, nbytes, 1.0f, sink, stream);
    case 10: return launch<10, 0, false>(ptrs, R, nbytes, 1.0f, sink, stream);
    case 18: return launch<18, 0, false>(ptrs, R, nbytes, 1.0f, sink, stream);
    default: return -1;
    }
}

}  // extern "C"
