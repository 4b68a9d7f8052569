// Device code of the ABS-SGD hot path for gfx950 (CDNA4, 64-wide wavefronts).
//
// Both operations are streaming, element-wise passes with ~0.2 flop/byte, so
// the design goal is bytes in flight, not arithmetic:
//   * every lane moves 128 bits per load/store; a wavefront touches 1 KiB of
//     consecutive memory per instruction;
//   * a workgroup owns one TILE of consecutive elements and issues ALL loads of
//     a pass before the first use, so a CU with 8 resident groups keeps tens
//     of KiB outstanding;
//   * every kernel (accumulate fp32 / bf16, sync-update for any K, flat or
//     ragged) uses the SAME tile size and the same workgroup -> tile order.
//     Workgroups are handed to the 8 XCDs round-robin, so tile c is always
//     served by XCD c % 8: an accumulator tile written by one launch is found
//     in that XCD's L2 by the next launch when the working set is small
//     enough, and never bounces between L2s.
//   * gradients are read once and never again: non-temporal loads keep them
//     from displacing accumulator / parameter lines in L2 and the memory-side
//     cache.
//
// Arithmetic order is fixed (see include/abs_sgd.h) and written with explicit
// fused multiply-adds; the file is compiled with contraction off.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef ABS_BLOCK
#define ABS_BLOCK 256          // threads per workgroup (4 wavefronts)
#endif
#ifndef ABS_TILE
#define ABS_TILE 4096          // elements per workgroup, all kernels
#endif
#ifndef ABS_NT_GRAD
#define ABS_NT_GRAD 1          // non-temporal gradient loads
#endif
#ifndef ABS_NT_ACC_LOAD
#define ABS_NT_ACC_LOAD 0      // accumulator loads in accumulate
#endif
#ifndef ABS_NT_ACC_STORE
#define ABS_NT_ACC_STORE 0     // accumulator stores in accumulate
#endif
#ifndef ABS_NT_SYNC_ACC
#define ABS_NT_SYNC_ACC 1      // accumulator loads in sync-update (dead afterwards)
#endif
#ifndef ABS_NT_SYNC_XV
#define ABS_NT_SYNC_XV 0       // x / v loads and stores in sync-update
#endif
#ifndef ABS_SYNC_INFLIGHT
#define ABS_SYNC_INFLIGHT 24   // target number of 128-bit loads in flight per lane in sync-update
#endif

namespace absk {

constexpr int BLOCK = ABS_BLOCK;
constexpr int TILE = ABS_TILE;
constexpr int VEC = 4;                          // elements per lane per access
constexpr int VPT = TILE / (BLOCK * VEC);       // 128-bit vectors per lane per tile
static_assert(TILE % (BLOCK * VEC) == 0 && VPT >= 1, "tile must be a whole number of block-wide vectors");

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(T *p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// bfloat16 is the high half of a binary32: widening is a shift.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

__device__ __forceinline__ f32x4 widen(u32x2 w)
{
    f32x4 r;
    r.x = bf16_lo(w.x); r.y = bf16_hi(w.x); r.z = bf16_lo(w.y); r.w = bf16_hi(w.y);
    return r;
}

// ---------------------------------------------------------------- accumulate

template <bool FIRST>
__device__ __forceinline__ float acc_one(float nf, float g, float a)
{
    if constexpr (FIRST) return nf * g;
    else return __builtin_fmaf(nf, g, a);
}

template <bool FIRST>
__device__ __forceinline__ f32x4 acc_vec(float nf, f32x4 g, f32x4 a)
{
    f32x4 r;
    r.x = acc_one<FIRST>(nf, g.x, a.x); r.y = acc_one<FIRST>(nf, g.y, a.y);
    r.z = acc_one<FIRST>(nf, g.z, a.z); r.w = acc_one<FIRST>(nf, g.w, a.w);
    return r;
}

template <bool BF16> struct GradT { typedef float elem; typedef f32x4 vec; };
template <> struct GradT<true> { typedef uint16_t elem; typedef u32x2 vec; };

template <bool BF16>
__device__ __forceinline__ f32x4 load_grad_vec(const typename GradT<BF16>::vec *p)
{
    if constexpr (BF16) return widen(ld<ABS_NT_GRAD != 0>(p));
    else return ld<ABS_NT_GRAD != 0>(p);
}

template <bool BF16>
__device__ __forceinline__ float load_grad_one(const typename GradT<BF16>::elem *p)
{
    if constexpr (BF16) return bf16_one(*p);
    else return *p;
}

// One workgroup, one tile: acc[0..len) (+)= nf * grad[0..len), len <= TILE.
template <bool FIRST, bool BF16>
__device__ __forceinline__ void accumulate_tile(float *__restrict__ acc,
                                                const typename GradT<BF16>::elem *__restrict__ grad,
                                                int len, float nf, bool vec_ok)
{
    typedef typename GradT<BF16>::vec gvec;
    const int tid = threadIdx.x;
    if (vec_ok) {
        f32x4 *av = reinterpret_cast<f32x4 *>(acc);
        const gvec *gv = reinterpret_cast<const gvec *>(grad);
        if (len == TILE) {
            f32x4 g[VPT], a[VPT] = {};
#pragma unroll
            for (int u = 0; u < VPT; ++u) g[u] = load_grad_vec<BF16>(gv + u * BLOCK + tid);
            if constexpr (!FIRST) {
#pragma unroll
                for (int u = 0; u < VPT; ++u) a[u] = ld<ABS_NT_ACC_LOAD != 0>(av + u * BLOCK + tid);
            }
#pragma unroll
            for (int u = 0; u < VPT; ++u)
                st<ABS_NT_ACC_STORE != 0>(av + u * BLOCK + tid, acc_vec<FIRST>(nf, g[u], a[u]));
            return;
        }
        const int nvec = len / VEC;
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const int i = u * BLOCK + tid;
            if (i < nvec) {
                f32x4 g = load_grad_vec<BF16>(gv + i);
                f32x4 a = {0.f, 0.f, 0.f, 0.f};
                if constexpr (!FIRST) a = av[i];
                av[i] = acc_vec<FIRST>(nf, g, a);
            }
        }
        const int i = nvec * VEC + tid;          // at most VEC-1 trailing elements
        if (i < len) acc[i] = acc_one<FIRST>(nf, load_grad_one<BF16>(grad + i), FIRST ? 0.f : acc[i]);
        return;
    }
    for (int i = tid; i < len; i += BLOCK)
        acc[i] = acc_one<FIRST>(nf, load_grad_one<BF16>(grad + i), FIRST ? 0.f : acc[i]);
}

// --------------------------------------------------------------- sync-update

struct Hyper { float M, lr, mu, wd; };

__device__ __forceinline__ void update_one(float s, float &x, float &v, const Hyper &h)
{
    const float gbar = s / h.M;
    const float d = __builtin_fmaf(h.wd, x, gbar);
    v = __builtin_fmaf(h.mu, v, d);
    x = __builtin_fmaf(-h.lr, v, x);
}

__device__ __forceinline__ void update_vec(f32x4 s, f32x4 &x, f32x4 &v, const Hyper &h)
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float xs = x[c], vs = v[c];
        update_one(s[c], xs, vs, h);
        x[c] = xs;
        v[c] = vs;
    }
}

template <int K> struct AccPtrs { const float *p[K]; };

// vectors per lane per pass so that about ABS_SYNC_INFLIGHT loads are outstanding
template <int K>
constexpr int sync_unroll()
{
    int u = ABS_SYNC_INFLIGHT / (K + 2);
    if (u < 1) u = 1;
    if (u > VPT) u = VPT;
    while (VPT % u) --u;
    return u;
}

// One workgroup, one tile of the fused combine + update; K compile-time.
template <int K>
__device__ __forceinline__ void sync_tile(float *__restrict__ x, float *__restrict__ v,
                                          const AccPtrs<K> &A, int len, const Hyper &h, bool vec_ok)
{
    const int tid = threadIdx.x;
    if (vec_ok) {
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        f32x4 *vv = reinterpret_cast<f32x4 *>(v);
        if (len == TILE) {
            constexpr int U = sync_unroll<K>();
#pragma unroll 1
            for (int pass = 0; pass < VPT / U; ++pass) {
                f32x4 a[U][K], xr[U], vr[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = (pass * U + u) * BLOCK + tid;
#pragma unroll
                    for (int k = 0; k < K; ++k)
                        a[u][k] = ld<ABS_NT_SYNC_ACC != 0>(reinterpret_cast<const f32x4 *>(A.p[k]) + i);
                    xr[u] = ld<ABS_NT_SYNC_XV != 0>(xv + i);
                    vr[u] = ld<ABS_NT_SYNC_XV != 0>(vv + i);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = (pass * U + u) * BLOCK + tid;
                    f32x4 s = a[u][0];
#pragma unroll
                    for (int k = 1; k < K; ++k) s = s + a[u][k];
                    update_vec(s, xr[u], vr[u], h);
                    st<ABS_NT_SYNC_XV != 0>(vv + i, vr[u]);
                    st<ABS_NT_SYNC_XV != 0>(xv + i, xr[u]);
                }
            }
            return;
        }
        const int nvec = len / VEC;
        for (int i = tid; i < nvec; i += BLOCK) {
            f32x4 s = reinterpret_cast<const f32x4 *>(A.p[0])[i];
#pragma unroll
            for (int k = 1; k < K; ++k) s = s + reinterpret_cast<const f32x4 *>(A.p[k])[i];
            f32x4 xr = xv[i], vr = vv[i];
            update_vec(s, xr, vr, h);
            vv[i] = vr;
            xv[i] = xr;
        }
        const int i = nvec * VEC + tid;
        if (i < len) {
            float s = A.p[0][i];
#pragma unroll
            for (int k = 1; k < K; ++k) s = s + A.p[k][i];
            update_one(s, x[i], v[i], h);
        }
        return;
    }
    for (int i = tid; i < len; i += BLOCK) {
        float s = A.p[0][i];
#pragma unroll
        for (int k = 1; k < K; ++k) s = s + A.p[k][i];
        update_one(s, x[i], v[i], h);
    }
}

// K known only at run time (K above the specialised range).  get(k) yields
// worker k's accumulator pointer for this tile; it is uniform across the
// workgroup, so it costs scalar loads only.
template <class GetPtr>
__device__ __forceinline__ void sync_tile_any(float *__restrict__ x, float *__restrict__ v,
                                              GetPtr get, int K, int len, const Hyper &h,
                                              bool vec_ok)
{
    const int tid = threadIdx.x;
    if (vec_ok) {
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        f32x4 *vv = reinterpret_cast<f32x4 *>(v);
        const int nvec = len / VEC;
        for (int i = tid; i < nvec; i += BLOCK) {
            f32x4 s = ld<ABS_NT_SYNC_ACC != 0>(reinterpret_cast<const f32x4 *>(get(0)) + i);
#pragma unroll 8
            for (int k = 1; k < K; ++k)
                s = s + ld<ABS_NT_SYNC_ACC != 0>(reinterpret_cast<const f32x4 *>(get(k)) + i);
            f32x4 xr = xv[i], vr = vv[i];
            update_vec(s, xr, vr, h);
            vv[i] = vr;
            xv[i] = xr;
        }
        const int i = nvec * VEC + tid;
        if (i < len) {
            float s = get(0)[i];
            for (int k = 1; k < K; ++k) s = s + get(k)[i];
            update_one(s, x[i], v[i], h);
        }
        return;
    }
    for (int i = tid; i < len; i += BLOCK) {
        float s = get(0)[i];
        for (int k = 1; k < K; ++k) s = s + get(k)[i];
        update_one(s, x[i], v[i], h);
    }
}

struct AccPtrsAny { const float *p[64]; };

// -------------------------------------------------------------------- kernels

__device__ __forceinline__ bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
__device__ __forceinline__ bool aligned8(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; }

// Flat vector: workgroup b owns elements [b*TILE, min(P, (b+1)*TILE)).
template <bool FIRST, bool BF16>
__global__ __launch_bounds__(ABS_BLOCK) void accumulate_flat(float *__restrict__ acc,
                                                            const void *__restrict__ grad,
                                                            int64_t P, float nf, int vec_ok)
{
    typedef typename GradT<BF16>::elem gelem;
    const int64_t base = (int64_t)blockIdx.x * TILE;
    const int64_t rest = P - base;
    const int len = rest < TILE ? (int)rest : TILE;
    accumulate_tile<FIRST, BF16>(acc + base, static_cast<const gelem *>(grad) + base, len, nf,
                                 vec_ok != 0);
}

template <int K>
__global__ __launch_bounds__(ABS_BLOCK) void sync_update_flat(float *__restrict__ x,
                                                             float *__restrict__ v, AccPtrs<K> A,
                                                             int64_t P, Hyper h, int vec_ok)
{
    const int64_t base = (int64_t)blockIdx.x * TILE;
    const int64_t rest = P - base;
    const int len = rest < TILE ? (int)rest : TILE;
    AccPtrs<K> B;
#pragma unroll
    for (int k = 0; k < K; ++k) B.p[k] = A.p[k] + base;
    sync_tile<K>(x + base, v + base, B, len, h, vec_ok != 0);
}

__global__ __launch_bounds__(ABS_BLOCK) void sync_update_flat_any(float *__restrict__ x,
                                                                 float *__restrict__ v,
                                                                 AccPtrsAny A, int K, int64_t P,
                                                                 Hyper h, int vec_ok)
{
    const int64_t base = (int64_t)blockIdx.x * TILE;
    const int64_t rest = P - base;
    const int len = rest < TILE ? (int)rest : TILE;
    sync_tile_any(x + base, v + base, [&](int k) { return A.p[k] + base; }, K, len, h,
                  vec_ok != 0);
}

// Ragged layout: workgroup b looks its (tensor, tile index) up in a table; the
// per-tensor base pointers come from device-resident pointer tables.  All of
// these reads are uniform across the workgroup (scalar loads).
struct Chunk { int32_t tensor; int32_t index; };

template <bool FIRST, bool BF16>
__global__ __launch_bounds__(ABS_BLOCK) void accumulate_ragged(const Chunk *__restrict__ chunks,
                                                              const int64_t *__restrict__ sizes,
                                                              float *const *__restrict__ acc_tab,
                                                              const void *const *__restrict__ grad_tab,
                                                              float nf)
{
    typedef typename GradT<BF16>::elem gelem;
    const Chunk c = chunks[blockIdx.x];
    const int64_t base = (int64_t)c.index * TILE;
    const int64_t rest = sizes[c.tensor] - base;
    const int len = rest < TILE ? (int)rest : TILE;
    float *acc = acc_tab[c.tensor] + base;
    const gelem *grad = static_cast<const gelem *>(grad_tab[c.tensor]) + base;
    const bool vec_ok = aligned16(acc) && (BF16 ? aligned8(grad) : aligned16(grad));
    accumulate_tile<FIRST, BF16>(acc, grad, len, nf, vec_ok);
}

template <int K> struct TabPtrs { const float *const *t[K]; };
struct TabPtrsAny { const float *const *t[64]; };

template <int K>
__global__ __launch_bounds__(ABS_BLOCK) void sync_update_ragged(const Chunk *__restrict__ chunks,
                                                               const int64_t *__restrict__ sizes,
                                                               float *const *__restrict__ x_tab,
                                                               float *const *__restrict__ v_tab,
                                                               TabPtrs<K> tabs, Hyper h)
{
    const Chunk c = chunks[blockIdx.x];
    const int64_t base = (int64_t)c.index * TILE;
    const int64_t rest = sizes[c.tensor] - base;
    const int len = rest < TILE ? (int)rest : TILE;
    float *x = x_tab[c.tensor] + base;
    float *v = v_tab[c.tensor] + base;
    bool vec_ok = aligned16(x) && aligned16(v);
    AccPtrs<K> A;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        A.p[k] = tabs.t[k][c.tensor] + base;
        vec_ok = vec_ok && aligned16(A.p[k]);
    }
    sync_tile<K>(x, v, A, len, h, vec_ok);
}

__global__ __launch_bounds__(ABS_BLOCK) void sync_update_ragged_any(const Chunk *__restrict__ chunks,
                                                                   const int64_t *__restrict__ sizes,
                                                                   float *const *__restrict__ x_tab,
                                                                   float *const *__restrict__ v_tab,
                                                                   TabPtrsAny tabs, int K, Hyper h)
{
    const Chunk c = chunks[blockIdx.x];
    const int64_t base = (int64_t)c.index * TILE;
    const int64_t rest = sizes[c.tensor] - base;
    const int len = rest < TILE ? (int)rest : TILE;
    float *x = x_tab[c.tensor] + base;
    float *v = v_tab[c.tensor] + base;
    bool vec_ok = aligned16(x) && aligned16(v);
    for (int k = 0; k < K; ++k) vec_ok = vec_ok && aligned16(tabs.t[k][c.tensor] + base);
    sync_tile_any(x, v, [&](int k) { return tabs.t[k][c.tensor] + base; }, K, len, h, vec_ok);
}

}  // namespace absk
