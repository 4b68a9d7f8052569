// Plain streaming kernels of known size, separate from the method's library.
// They serve two purposes in the benchmark: (1) calibrating the profiler's
// HBM byte counters against a transfer whose size is known, and (2) measuring
// the copy / read / write / triad / K-way-mix ceilings of the box the benchmark runs on, to put the
// method's kernels in context.  Nothing in the method calls them.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int BLOCK = 256;
constexpr int VPT = 4;   // 128-bit vectors per lane, all loads issued before the stores

__global__ __launch_bounds__(BLOCK) void probe_copy_kernel(f32x4 *__restrict__ dst,
                                                          const f32x4 *__restrict__ src, int64_t nvec)
{
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * VPT) + threadIdx.x;
    f32x4 r[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) r[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) __builtin_nontemporal_store(r[u], dst + i);
    }
}

__global__ __launch_bounds__(BLOCK) void probe_read_kernel(const f32x4 *__restrict__ src, int64_t nvec,
                                                          float *__restrict__ sink)
{
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * VPT) + threadIdx.x;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) acc += __builtin_nontemporal_load(src + i);
    }
    // never true for finite data: keeps the loads alive without a store stream
    if (acc.x + acc.y + acc.z + acc.w == 1.2345678e38f) *sink = acc.x;
}

__global__ __launch_bounds__(BLOCK) void probe_write_kernel(f32x4 *__restrict__ dst, int64_t nvec, float val)
{
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * VPT) + threadIdx.x;
    const f32x4 r = {val, val, val, val};
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) __builtin_nontemporal_store(r, dst + i);
    }
}

// a = a + s * b in place: two reads and one write per element, the traffic mix
// of a steady gradient accumulation, with no structure beyond one vector per lane.
__global__ __launch_bounds__(BLOCK) void probe_triad_kernel(f32x4 *__restrict__ a, const f32x4 *__restrict__ b,
                                                           int64_t nvec, float s)
{
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * VPT) + threadIdx.x;
    f32x4 ra[VPT], rb[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) {
            ra[u] = __builtin_nontemporal_load(a + i);
            rb[u] = __builtin_nontemporal_load(b + i);
        }
    }
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) __builtin_nontemporal_store(ra[u] + s * rb[u], a + i);
    }
}

// R vectors read, the first two also written in place (p0 = sum, p1 = sum / 2): the
// traffic mix of a fused combine + update over R - 2 workers, one vector per lane
// and stream, VPT rows at a time, nothing else.
template <int R> struct MixPtrs { f32x4 *p[R]; };

template <int R>
__global__ __launch_bounds__(BLOCK) void probe_mix_kernel(MixPtrs<R> P, int64_t nvec)
{
    const int64_t base = (int64_t)blockIdx.x * (BLOCK * VPT) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t i = base + u * BLOCK;
        if (i < nvec) {
            f32x4 s = __builtin_nontemporal_load(P.p[0] + i);
#pragma unroll
            for (int r = 1; r < R; ++r) s += __builtin_nontemporal_load(P.p[r] + i);
            __builtin_nontemporal_store(s, P.p[0] + i);
            __builtin_nontemporal_store(s * 0.5f, P.p[1] + i);
        }
    }
}

template <int R>
int launch_mix(void *const *ptrs, int64_t nvec, hipStream_t stream);

inline unsigned grid_for(int64_t nvec) { return (unsigned)((nvec + BLOCK * VPT - 1) / (BLOCK * VPT)); }
template <int R>
int launch_mix(void *const *ptrs, int64_t nvec, hipStream_t stream)
{
    MixPtrs<R> P;
    for (int r = 0; r < R; ++r) P.p[r] = (f32x4 *)ptrs[r];
    hipLaunchKernelGGL(probe_mix_kernel<R>, dim3(grid_for(nvec)), dim3(BLOCK), 0, stream, P, nvec);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
}  // namespace

extern "C" {

// dst, src: DEVICE, 16-byte aligned, nbytes a multiple of 16.  Returns 0 or -1.
int probe_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (!dst || !src || nbytes <= 0 || (nbytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return -1;
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid_for(nvec)), dim3(BLOCK), 0, (hipStream_t)stream,
                       (f32x4 *)dst, (const f32x4 *)src, nvec);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int probe_read(const void *src, int64_t nbytes, float *sink, void *stream)
{
    if (!src || !sink || nbytes <= 0 || (nbytes & 15) || ((uintptr_t)src & 15)) return -1;
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid_for(nvec)), dim3(BLOCK), 0, (hipStream_t)stream,
                       (const f32x4 *)src, nvec, sink);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int probe_write(void *dst, int64_t nbytes, float val, void *stream)
{
    if (!dst || nbytes <= 0 || (nbytes & 15) || ((uintptr_t)dst & 15)) return -1;
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(probe_write_kernel, dim3(grid_for(nvec)), dim3(BLOCK), 0, (hipStream_t)stream,
                       (f32x4 *)dst, nvec, val);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// a (read and written) and b (read): DEVICE, 16-byte aligned, nbytes each.
int probe_triad(void *a, const void *b, int64_t nbytes, float s, void *stream)
{
    if (!a || !b || nbytes <= 0 || (nbytes & 15) || ((uintptr_t)a & 15) || ((uintptr_t)b & 15)) return -1;
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(probe_triad_kernel, dim3(grid_for(nvec)), dim3(BLOCK), 0, (hipStream_t)stream,
                       (f32x4 *)a, (const f32x4 *)b, nvec, s);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ptrs: HOST array of R DEVICE pointers (R = 6, 10 or 18: the shapes of K = 4, 8, 16
// workers), 16-byte aligned, nbytes each; the first two are read and written.
int probe_mix(void *const *ptrs, int R, int64_t nbytes, void *stream)
{
    if (!ptrs || nbytes <= 0 || (nbytes & 15)) return -1;
    for (int r = 0; r < R && r < 18; ++r)
        if (!ptrs[r] || ((uintptr_t)ptrs[r] & 15)) return -1;
    const int64_t nvec = nbytes / 16;
    switch (R) {
    case 6: return launch_mix<6>(ptrs, nvec, (hipStream_t)stream);
    case 10: return launch_mix<10>(ptrs, nvec, (hipStream_t)stream);
    case 18: return launch_mix<18>(ptrs, nvec, (hipStream_t)stream);
    default: return -1;
    }
}

}  // extern "C"
