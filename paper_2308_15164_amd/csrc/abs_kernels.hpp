// Device code of the ABS-SGD hot path for gfx950 (CDNA4, 64-wide wavefronts).
//
// Both operations are streaming, element-wise passes with ~0.2 flop/byte, so
// the design goal is bytes in flight and an even finish, not arithmetic:
//   * every lane moves 128 bits per load/store; a wavefront touches 1 KiB of
//     consecutive memory per instruction; a workgroup "row" is BLOCK such
//     vectors (ROW elements);
//   * a workgroup owns one tile = a run of consecutive rows and walks it in
//     groups of 4 rows, issuing the loads of a group before the first use (the
//     K-way read of sync-update in batches of up to 4 workers);
//   * the host picks the tile size per launch so that the grid is a whole
//     number of resident rounds (256 CUs x resident workgroups per CU): every
//     CU then finishes together instead of idling behind a ragged last round,
//     which matters when a launch lasts only tens of microseconds;
//   * workgroup b owns tile b in every kernel; workgroups go to the 8 XCDs
//     round-robin, so consecutive tiles (consecutive memory) are spread over all
//     XCDs and their L2s at any moment.  No reuse is sought in L2: the byte
//     counters show that nothing survives there from one launch to the next
//     (a steady accumulate launch over 4 MiB buffers still fetches gradient +
//     accumulator in full), so the only cache that spans launches is the
//     memory-side cache, which all XCDs share;
//   * gradients are read once and never again: non-temporal loads keep them
//     from displacing accumulator / parameter lines in L2 and the memory-side
//     cache.  Accumulators, x and v are re-read soon (next micro-batch, next
//     step): whether they should be cached depends on whether the working set
//     fits the memory-side cache, so every kernel exists in a cached and a
//     streaming (non-temporal) flavour chosen per launch by the host.
//
// Arithmetic order is fixed (see include/abs_sgd.h) and written with explicit
// fused multiply-adds; the file is compiled with contraction off.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "abs_types.hpp"

#define ABS_BLOCK 256          // threads per workgroup (4 wavefronts); literal for __launch_bounds__
#ifndef ABS_ACC_UNROLL
#define ABS_ACC_UNROLL 4       // rows per group in accumulate (2 loads per row in flight)
#endif
#ifndef ABS_NT_GRAD
#define ABS_NT_GRAD 1          // non-temporal gradient loads
#endif
#ifndef ABS_NT_SYNC_ACC
#define ABS_NT_SYNC_ACC 1      // accumulator loads in sync-update (dead afterwards)
#endif
#ifndef ABS_SYNC_ROWS
#define ABS_SYNC_ROWS 4        // rows per group in sync-update
#endif
#ifndef ABS_SYNC_INFLIGHT
#define ABS_SYNC_INFLIGHT 24   // 128-bit loads in flight per lane in sync-update (bounds the workers per load batch)
#endif

namespace absk {

static_assert(BLOCK == ABS_BLOCK, "the host plans launches for this workgroup size");
constexpr int VEC = 4;                 // elements per lane per access
static_assert(ROW == BLOCK * VEC, "a workgroup row is one 128-bit vector per lane");

// Vector index of (row u, lane tid) in a group of U rows starting at g0.  Two
// layouts, both covering [g0, g0 + U*BLOCK) exactly once:
//   row-major      : a row is BLOCK consecutive vectors, one per lane;
//   wave-contiguous: each wavefront owns U*64 consecutive vectors (U KiB per
//                    stream), row u being its u-th 64-vector piece.
#ifndef ABS_WAVE_CONTIG
#define ABS_WAVE_CONTIG 1      // 0 disables the wave-contiguous layout everywhere
#endif
#define GIDX(g0, u, tid, U, wc)                                                              \
    (((wc) && ABS_WAVE_CONTIG) ? ((g0) + ((((tid) >> 6) * (U)) + (u)) * 64 + ((tid) & 63))   \
                               : ((g0) + (u) * BLOCK + (tid)))

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Every buffer this library touches is device (global) memory.  Pointers that reach a
// kernel through a table in memory carry no address space the compiler could know of,
// and would be accessed with generic (flat) instructions; the casts say what they are.
#define ABS_GLOBAL __attribute__((address_space(1)))

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *p)
{
    const ABS_GLOBAL T *g = (const ABS_GLOBAL T *)p;
    if constexpr (NT) return __builtin_nontemporal_load(g);
    else return *g;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(T *p, T v)
{
    ABS_GLOBAL T *g = (ABS_GLOBAL T *)p;
    if constexpr (NT) __builtin_nontemporal_store(v, g);
    else *g = v;
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

// first: the accumulator holds nothing yet (its logical value is 0); the
// result is the rounded product and the old contents are never read.
__device__ __forceinline__ float acc_one(bool first, float nf, float g, float a)
{
    return first ? nf * g : __builtin_fmaf(nf, g, a);
}

__device__ __forceinline__ f32x4 acc_vec(bool first, float nf, f32x4 g, f32x4 a)
{
    f32x4 r;
    r.x = acc_one(first, nf, g.x, a.x); r.y = acc_one(first, nf, g.y, a.y);
    r.z = acc_one(first, nf, g.z, a.z); r.w = acc_one(first, nf, g.w, a.w);
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

// J micro-batch gradients of one worker, applied in order in one pass:
//   r = first ? n_0*g_0 : fma(n_0, g_0, acc);  r = fma(n_j, g_j, r) for j = 1..J-1;  acc = r.
// Every intermediate is rounded exactly as J separate launches would round it,
// so batching changes the traffic ((J*g_b + 8) instead of J*(g_b + 8) bytes per
// parameter), never the bits.
template <bool BF16, int J>
struct GradArgs {
    const typename GradT<BF16>::elem *g[J];
    float n[J];
};

// Rows per group and gradients whose loads are issued together.  One gradient per
// launch: 4 rows (8 loads in flight per lane).  Several: 4 rows x 4 gradients at a time
// (up to 20 loads).  Measured at P = 1.4e8 with J distinct gradient vectors, J = 2..8:
// groups of 4 rows move 2-4 % more than groups of 2 rows for both gradient types, and
// whether 2, 4 or 8 gradients are loaded at a time then matters little.
#ifndef ABS_ACCB_BATCH
#define ABS_ACCB_BATCH 4       // gradients per load batch when a launch folds in several
#endif
#ifndef ABS_ACCB_ROWS
#define ABS_ACCB_ROWS 4        // rows per group when a launch folds in several gradients
#endif
template <int J>
constexpr int acc_batch() { return J < ABS_ACCB_BATCH ? J : ABS_ACCB_BATCH; }
template <int J>
constexpr int acc_rows() { return J == 1 ? ABS_ACC_UNROLL : ABS_ACCB_ROWS; }

// r = first ? n_0*g_0 : fma(n_0, g_0, a)   -- only for the first gradient of a chain
// r = fma(n_j, g_j, r)                     -- for the rest
__device__ __forceinline__ f32x4 fma_vec(float n, f32x4 g, f32x4 r)
{
    r.x = __builtin_fmaf(n, g.x, r.x); r.y = __builtin_fmaf(n, g.y, r.y);
    r.z = __builtin_fmaf(n, g.z, r.z); r.w = __builtin_fmaf(n, g.w, r.w);
    return r;
}

template <int J>
__device__ __forceinline__ float acc_chain(bool first, const float (&n)[J], const float (&g)[J], float a)
{
    float r = acc_one(first, n[0], g[0], a);
#pragma unroll
    for (int j = 1; j < J; ++j) r = __builtin_fmaf(n[j], g[j], r);
    return r;
}

// One group of U rows starting at vector g0.  WHOLE: the group lies inside the
// tile and needs no bounds checks (straight-line code: loads, then stores).
template <bool BF16, bool NTA, int J, bool WHOLE>
__device__ __forceinline__ void accumulate_group(f32x4 *__restrict__ av, const GradArgs<BF16, J> &G, int g0,
                                                 int nvec, int tid, bool first)
{
    typedef typename GradT<BF16>::vec gvec;
    constexpr int U = acc_rows<J>();
    constexpr int JC = acc_batch<J>();
    constexpr bool wc = false;     // wave-contiguous: within noise for fp32, -3 to -7 % for bf16 at P = 1.2e7
    f32x4 g[U][JC] = {}, r[U] = {};
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GIDX(g0, u, tid, U, wc);
        if (WHOLE || i < nvec) {
#pragma unroll
            for (int j = 0; j < JC; ++j) g[u][j] = load_grad_vec<BF16>(reinterpret_cast<const gvec *>(G.g[j]) + i);
        }
    }
    if (!first) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = GIDX(g0, u, tid, U, wc);
            if (WHOLE || i < nvec) r[u] = ld<NTA>(av + i);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        r[u] = acc_vec(first, G.n[0], g[u][0], r[u]);
#pragma unroll
        for (int j = 1; j < JC; ++j) r[u] = fma_vec(G.n[j], g[u][j], r[u]);
    }
    // remaining gradients in batches of JC, in order
#pragma unroll
    for (int j0 = JC; j0 < J; j0 += JC) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = GIDX(g0, u, tid, U, wc);
            if (WHOLE || i < nvec) {
#pragma unroll
                for (int j = 0; j < JC; ++j)
                    if (j0 + j < J) g[u][j] = load_grad_vec<BF16>(reinterpret_cast<const gvec *>(G.g[j0 + j]) + i);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < JC; ++j)
                if (j0 + j < J) r[u] = fma_vec(G.n[j0 + j], g[u][j], r[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GIDX(g0, u, tid, U, wc);
        if (WHOLE || i < nvec) st<NTA>(av + i, r[u]);
    }
}

// One workgroup, one tile: acc[0..len) (+)= sum_j n_j * grad_j[0..len), in order.
// `first` is uniform over the launch.  NTA: accumulator traffic is streaming.
template <bool BF16, bool NTA, int J>
__device__ __forceinline__ void accumulate_tile(float *__restrict__ acc, const GradArgs<BF16, J> &G,
                                                int len, bool first, bool vec_ok)
{
    constexpr int U = acc_rows<J>();
    const int tid = threadIdx.x;
    if (!vec_ok) {
        for (int i = tid; i < len; i += BLOCK) {
            float g[J];
#pragma unroll
            for (int j = 0; j < J; ++j) g[j] = load_grad_one<BF16>(G.g[j] + i);
            acc[i] = acc_chain<J>(first, G.n, g, first ? 0.f : acc[i]);
        }
        return;
    }
    f32x4 *av = reinterpret_cast<f32x4 *>(acc);
    const int nvec = len / VEC;
    int g0 = 0;
    for (; g0 + U * BLOCK <= nvec; g0 += U * BLOCK) accumulate_group<BF16, NTA, J, true>(av, G, g0, nvec, tid, first);
    if (g0 < nvec) accumulate_group<BF16, NTA, J, false>(av, G, g0, nvec, tid, first);
    const int i = nvec * VEC + tid;          // at most VEC-1 trailing elements
    if (i < len) {
        float g[J];
#pragma unroll
        for (int j = 0; j < J; ++j) g[j] = load_grad_one<BF16>(G.g[j] + i);
        acc[i] = acc_chain<J>(first, G.n, g, first ? 0.f : acc[i]);
    }
}

// --------------------------------------------------------------- sync-update

// The update rules (enum Rule) and their hyper-parameters (Hyper) are in abs_types.hpp.
//
// One element.  s = sum of the workers' accumulators.  Orders (every operation
// rounded to fp32, fused where written as fma):
//   Gbar = s / M
//   SGD    d = fma(wd, x, Gbar); v = fma(mu, v, d); x = fma(-lr, v, x)
//   SGD_DC q = Gbar*Gbar; c = lambda*q; diff = x - xp; Gt = fma(c, diff, Gbar);
//          d = fma(wd, x, Gt); v = fma(mu, v, d); xp = x; x = fma(-lr, v, x)
//   SGD_DCM as SGD_DC with diff = nlr_prev * v (v before this update), no xp
//   ADAM   g = fma(wd, x, Gbar); m = fma(beta1, m, omb1*g); v = fma(beta2, v, omb2*(g*g));
//          mh = m / bc1; vh = v / bc2; den = sqrt(vh) + eps; x = fma(-lr, mh / den, x)
template <int RULE>
__device__ __forceinline__ void update_one(float s, float &x, float &s1, float &s2, const Hyper &h)
{
    float g = s / h.M;
    if constexpr (RULE == ADAM) {
        g = __builtin_fmaf(h.wd, x, g);
        const float t1 = h.omb1 * g;
        s1 = __builtin_fmaf(h.beta1, s1, t1);
        const float g2 = g * g;
        const float t2 = h.omb2 * g2;
        s2 = __builtin_fmaf(h.beta2, s2, t2);
        const float mh = s1 / h.bc1;
        const float vh = s2 / h.bc2;
        const float den = __builtin_sqrtf(vh) + h.eps;
        const float q = mh / den;
        x = __builtin_fmaf(-h.lr, q, x);
    } else {
        if constexpr (RULE == SGD_DC) {
            const float q = g * g;
            const float c = h.lambda * q;
            const float diff = x - s2;
            g = __builtin_fmaf(c, diff, g);
            s2 = x;
        }
        if constexpr (RULE == SGD_DCM) {
            const float q = g * g;
            const float c = h.lambda * q;
            const float diff = h.nlr_prev * s1;
            g = __builtin_fmaf(c, diff, g);
        }
        const float d = __builtin_fmaf(h.wd, x, g);
        s1 = __builtin_fmaf(h.mu, s1, d);
        x = __builtin_fmaf(-h.lr, s1, x);
    }
}

template <int RULE>
__device__ __forceinline__ void update_vec(f32x4 s, f32x4 &x, f32x4 &s1, f32x4 &s2, const Hyper &h)
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float xs = x[c], a = s1[c], b = s2[c];
        update_one<RULE>(s[c], xs, a, b, h);
        x[c] = xs;
        s1[c] = a;
        s2[c] = b;
    }
}

template <int K> struct AccPtrs { const float *p[K]; };

// Workers whose accumulators are loaded together.  A group always spans
// ABS_SYNC_ROWS rows, so a workgroup reads ABS_SYNC_ROWS x 4 KiB of consecutive
// memory per stream at a time (each wavefront 1 KiB of every row); with many workers the K-way read is cut into batches of KC
// so that about ABS_SYNC_INFLIGHT loads are outstanding per lane.  Measured at
// P = 1.2e8, K = 16: 4 rows x 4 workers at a time reach 5.8 TB/s, 1 row x 16
// workers 5.1 TB/s.  The sum still runs over the workers in ascending order.
template <int K, int RULE>
constexpr int sync_batch()
{
    int kc = ABS_SYNC_INFLIGHT / ABS_SYNC_ROWS - 2 - (uses_s2<RULE>() ? 1 : 0);
    return kc < 1 ? 1 : (kc > K ? K : kc);
}

// One group of ABS_SYNC_ROWS rows starting at vector g0.  WHOLE: the group lies
// inside the tile and needs no bounds checks.
template <int K, bool NTX, int RULE, bool WHOLE>
__device__ __forceinline__ void sync_group(f32x4 *__restrict__ xv, f32x4 *__restrict__ vv,
                                           f32x4 *__restrict__ pv, const AccPtrs<K> &A, int g0, int nvec,
                                           int tid, const Hyper &h)
{
    constexpr bool S2 = uses_s2<RULE>();
    constexpr int U = ABS_SYNC_ROWS;
    constexpr int KC = sync_batch<K, RULE>();
    // wave-contiguous pays when the K workers are read in exactly two batches (K = 5..8:
    // +3 % at P >= 6e7); one batch is indifferent, more lose a quarter of the rate (K = 16)
    constexpr bool WC = K > KC && K <= 2 * KC;
    f32x4 a[U][KC] = {}, sum[U] = {}, xr[U] = {}, vr[U] = {}, pr[U] = {};
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GIDX(g0, u, tid, U, WC);
        if (WHOLE || i < nvec) {
#pragma unroll
            for (int k = 0; k < KC; ++k)
                a[u][k] = ld<ABS_NT_SYNC_ACC != 0>(reinterpret_cast<const f32x4 *>(A.p[k]) + i);
            xr[u] = ld<NTX>(xv + i);
            vr[u] = ld<NTX>(vv + i);
            if constexpr (S2) pr[u] = ld<NTX>(pv + i);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        sum[u] = a[u][0];
#pragma unroll
        for (int k = 1; k < KC; ++k) sum[u] = sum[u] + a[u][k];
    }
    // remaining workers in batches of KC, still in ascending order
#pragma unroll
    for (int k0 = KC; k0 < K; k0 += KC) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = GIDX(g0, u, tid, U, WC);
            if (WHOLE || i < nvec) {
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    if (k0 + k < K) a[u][k] = ld<ABS_NT_SYNC_ACC != 0>(reinterpret_cast<const f32x4 *>(A.p[k0 + k]) + i);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < KC; ++k)
                if (k0 + k < K) sum[u] = sum[u] + a[u][k];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GIDX(g0, u, tid, U, WC);
        if (WHOLE || i < nvec) {
            update_vec<RULE>(sum[u], xr[u], vr[u], pr[u], h);
            st<NTX>(vv + i, vr[u]);
            if constexpr (S2) st<NTX>(pv + i, pr[u]);
            st<NTX>(xv + i, xr[u]);
        }
    }
}

// One workgroup, one tile of the fused combine + update; K compile-time.
// NTX: the traffic of x and the state vectors is streaming.  xp (the rule's
// second state vector) is only touched by rules that have one.
template <int K, bool NTX, int RULE>
__device__ __forceinline__ void sync_tile(float *__restrict__ x, float *__restrict__ v,
                                          float *__restrict__ xp, const AccPtrs<K> &A, int len,
                                          const Hyper &h, bool vec_ok)
{
    constexpr bool S2 = uses_s2<RULE>();
    constexpr int U = ABS_SYNC_ROWS;
    const int tid = threadIdx.x;
    int done = 0;
    if (vec_ok) {
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        f32x4 *vv = reinterpret_cast<f32x4 *>(v);
        f32x4 *pv = reinterpret_cast<f32x4 *>(xp);
        const int nvec = len / VEC;
        int g0 = 0;
        for (; g0 + U * BLOCK <= nvec; g0 += U * BLOCK) sync_group<K, NTX, RULE, true>(xv, vv, pv, A, g0, nvec, tid, h);
        if (g0 < nvec) sync_group<K, NTX, RULE, false>(xv, vv, pv, A, g0, nvec, tid, h);
        done = nvec * VEC;           // at most VEC-1 trailing elements remain
    }
    for (int i = done + tid; i < len; i += BLOCK) {
        float s = A.p[0][i];
#pragma unroll
        for (int k = 1; k < K; ++k) s = s + A.p[k][i];
        float ps = S2 ? xp[i] : 0.f;
        update_one<RULE>(s, x[i], v[i], ps, h);
        if constexpr (S2) xp[i] = ps;
    }
}

// K known only at run time (K above the specialised range).  The workers' base
// pointers for this tile sit in LDS (`ptrs`, filled by the kernel before the call).
// Same shape as the specialised kernels -- groups of ABS_SYNC_ROWS rows, the K-way read
// in batches of ANY_KC workers, ascending order -- but as a LOOP over the batches: the
// registers hold one batch whatever K is, where the unrolled form at K = 14 or 16 leaves
// the compiler so short of registers that it issues the loads one at a time.
#ifndef ABS_ANY_KC
#define ABS_ANY_KC 4           // workers per batch in the run-time-K kernels
#endif
constexpr int ANY_KC = ABS_ANY_KC;

template <int RULE, bool NTX, bool WHOLE>
__device__ __forceinline__ void sync_group_any(f32x4 *__restrict__ xv, f32x4 *__restrict__ vv,
                                               f32x4 *__restrict__ pv, const float *const *ptrs, int K, int g0,
                                               int nvec, int tid, const Hyper &h)
{
    constexpr bool S2 = uses_s2<RULE>();
    constexpr int U = ABS_SYNC_ROWS;
    f32x4 sum[U] = {}, xr[U] = {}, vr[U] = {}, pr[U] = {};
    const f32x4 *p0 = reinterpret_cast<const f32x4 *>(ptrs[0]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GIDX(g0, u, tid, U, false);
        if (WHOLE || i < nvec) {
            sum[u] = ld<ABS_NT_SYNC_ACC != 0>(p0 + i);
            xr[u] = ld<NTX>(xv + i);
            vr[u] = ld<NTX>(vv + i);
            if constexpr (S2) pr[u] = ld<NTX>(pv + i);
        }
    }
    for (int k0 = 1; k0 < K; k0 += ANY_KC) {
        f32x4 a[U][ANY_KC] = {};
#pragma unroll
        for (int kk = 0; kk < ANY_KC; ++kk) {
            if (k0 + kk < K) {
                const f32x4 *pk = reinterpret_cast<const f32x4 *>(ptrs[k0 + kk]);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = GIDX(g0, u, tid, U, false);
                    if (WHOLE || i < nvec) a[u][kk] = ld<ABS_NT_SYNC_ACC != 0>(pk + i);
                }
            }
        }
#pragma unroll
        for (int kk = 0; kk < ANY_KC; ++kk) {
            if (k0 + kk < K) {
#pragma unroll
                for (int u = 0; u < U; ++u) sum[u] = sum[u] + a[u][kk];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GIDX(g0, u, tid, U, false);
        if (WHOLE || i < nvec) {
            update_vec<RULE>(sum[u], xr[u], vr[u], pr[u], h);
            st<NTX>(vv + i, vr[u]);
            if constexpr (S2) st<NTX>(pv + i, pr[u]);
            st<NTX>(xv + i, xr[u]);
        }
    }
}

template <int RULE, bool NTX>
__device__ __forceinline__ void sync_tile_any(float *__restrict__ x, float *__restrict__ v,
                                              float *__restrict__ xp, const float *const *ptrs, int K, int len,
                                              const Hyper &h, bool vec_ok)
{
    constexpr bool S2 = uses_s2<RULE>();
    constexpr int U = ABS_SYNC_ROWS;
    const int tid = threadIdx.x;
    int done = 0;
    if (vec_ok) {
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        f32x4 *vv = reinterpret_cast<f32x4 *>(v);
        f32x4 *pv = reinterpret_cast<f32x4 *>(xp);
        const int nvec = len / VEC;
        int g0 = 0;
        for (; g0 + U * BLOCK <= nvec; g0 += U * BLOCK)
            sync_group_any<RULE, NTX, true>(xv, vv, pv, ptrs, K, g0, nvec, tid, h);
        if (g0 < nvec) sync_group_any<RULE, NTX, false>(xv, vv, pv, ptrs, K, g0, nvec, tid, h);
        done = nvec * VEC;
    }
    for (int i = done + tid; i < len; i += BLOCK) {
        float s = ptrs[0][i];
        for (int k = 1; k < K; ++k) s = s + ptrs[k][i];
        float ps = 0.f;
        if constexpr (S2) ps = xp[i];
        update_one<RULE>(s, x[i], v[i], ps, h);
        if constexpr (S2) xp[i] = ps;
    }
}

struct AccPtrsAny { const float *p[64]; };

// -------------------------------------------------------------------- kernels

__device__ __forceinline__ bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
__device__ __forceinline__ bool aligned8(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; }

__device__ __forceinline__ int tile_len(int64_t total, int64_t base, int tile)
{
    const int64_t rest = total - base;
    return rest < tile ? (int)rest : tile;
}

// Flat vector: workgroup b owns elements [b*tile, min(P, (b+1)*tile)); tile is a
// multiple of ROW chosen by the host.  A call may be cut into several launches
// (abs_host.hpp, slice_wgs): b0 is the index of the launch's first workgroup in the
// call, so b = blockIdx.x + b0 in every kernel below.
template <bool BF16, bool NTA, int J>
__global__ __launch_bounds__(ABS_BLOCK) void accumulate_flat(float *__restrict__ acc,
                                                            GradArgs<BF16, J> G, int64_t P, int tile,
                                                            int first, int vec_ok, unsigned b0)
{
    const int64_t base = (int64_t)(blockIdx.x + b0) * tile;
#pragma unroll
    for (int j = 0; j < J; ++j) G.g[j] += base;
    accumulate_tile<BF16, NTA, J>(acc + base, G, tile_len(P, base, tile), first != 0, vec_ok != 0);
}

template <int K, bool NTX, int RULE>
__global__ __launch_bounds__(ABS_BLOCK) void sync_update_flat(float *__restrict__ x,
                                                             float *__restrict__ v,
                                                             float *__restrict__ xp, AccPtrs<K> A,
                                                             int64_t P, int tile, Hyper h, int vec_ok,
                                                             unsigned b0)
{
    const int64_t base = (int64_t)(blockIdx.x + b0) * tile;
    AccPtrs<K> B;
#pragma unroll
    for (int k = 0; k < K; ++k) B.p[k] = A.p[k] + base;
    sync_tile<K, NTX, RULE>(x + base, v + base, uses_s2<RULE>() ? xp + base : nullptr, B,
                            tile_len(P, base, tile), h, vec_ok != 0);
}

template <int RULE, bool NTX>
__global__ __launch_bounds__(ABS_BLOCK) void sync_update_flat_any(float *__restrict__ x,
                                                                 float *__restrict__ v,
                                                                 float *__restrict__ xp,
                                                                 AccPtrsAny A, int K, int64_t P,
                                                                 int tile, Hyper h, int vec_ok, unsigned b0)
{
    __shared__ const float *ptrs[64];
    const int64_t base = (int64_t)(blockIdx.x + b0) * tile;
    if ((int)threadIdx.x < K) ptrs[threadIdx.x] = A.p[threadIdx.x] + base;
    __syncthreads();
    sync_tile_any<RULE, NTX>(x + base, v + base, uses_s2<RULE>() ? xp + base : nullptr, ptrs, K,
                             tile_len(P, base, tile), h, vec_ok != 0);
}

// Ragged layout: workgroup b looks its (tensor, tile index) up in a table; the
// per-tensor base pointers come from device-resident pointer tables.  All of
// these reads are uniform across the workgroup (scalar loads).

// J gradient pointer tables (one per micro-batch) and their sample counts.
template <int J>
struct GradTabs {
    const void *const *t[J];
    float n[J];
};

template <bool BF16, bool NTA, int J>
__global__ __launch_bounds__(ABS_BLOCK) void accumulate_ragged(const Chunk *__restrict__ chunks,
                                                              const int64_t *__restrict__ sizes,
                                                              float *const *__restrict__ acc_tab,
                                                              GradTabs<J> tabs, int tile, int first,
                                                              unsigned b0)
{
    typedef typename GradT<BF16>::elem gelem;
    const Chunk c = chunks[blockIdx.x + b0];
    const int64_t base = (int64_t)c.index * tile;
    float *acc = acc_tab[c.tensor] + base;
    bool vec_ok = aligned16(acc);
    GradArgs<BF16, J> G;
#pragma unroll
    for (int j = 0; j < J; ++j) {
        G.g[j] = static_cast<const gelem *>(tabs.t[j][c.tensor]) + base;
        G.n[j] = tabs.n[j];
        vec_ok = vec_ok && (BF16 ? aligned8(G.g[j]) : aligned16(G.g[j]));
    }
    accumulate_tile<BF16, NTA, J>(acc, G, tile_len(sizes[c.tensor], base, tile), first != 0, vec_ok);
}

// ---------------------------------------------------------------- job lists
//
// One launch for several workers: job w is one worker's share of the launch, its
// accumulator and the J_w <= 8 gradients folded into it, in order, with the
// roundings of J_w single launches.  The grid is ONE-dimensional: workgroup b owns
// tile b % tiles of job b / tiles, and workgroups start in the order of their index,
// so the jobs stream through the chip one after the other with no ramp-up or drain
// between them, and a launch lasts as long as all of them together.  (A two-
// dimensional grid, job = blockIdx.y, runs the jobs side by side instead: measured
// at P = 1.4e8, lists of 2 and 4 jobs then move 2-8 % less per second than single
// launches, the chip streaming through 2-4 times as many vectors at once.)  The job
// table travels in the kernel arguments and is read with scalar loads (the job index
// is uniform over the workgroup).
// JMAX bounds the J of every job of the launch (the host instantiates 1, 2, 4, 8), so
// that a launch of single gradients does not carry the registers of an 8-gradient one.
//
// A workgroup lives for some microseconds only, so what it waits for before its first
// vector load matters: everything it needs of its job (J, the flag, the accumulator,
// JMAX gradient pointers and sample counts) is read in ONE batch of scalar loads, whether
// or not the job uses all JMAX entries, and only then does the code branch on J.
template <int JMAX>
struct JobView {
    float *acc;
    const void *g[JMAX];
    float n[JMAX];
    int J, first;
};

template <int JMAX>
__device__ __forceinline__ JobView<JMAX> view_job(const Job &jb)
{
    JobView<JMAX> v;
    v.acc = static_cast<float *>(jb.acc);
    v.J = jb.J;
    v.first = jb.first;
#pragma unroll
    for (int j = 0; j < JMAX; ++j) {
        v.g[j] = jb.g[j];
        v.n[j] = jb.n[j];
    }
    return v;
}

template <bool BF16, bool NTA, int JMAX, int J = 1>
__device__ __forceinline__ void accumulate_job_tile(float *__restrict__ acc, const JobView<JMAX> &jb, int64_t base,
                                                    int len)
{
    typedef typename GradT<BF16>::elem gelem;
    if (jb.J == J) {
        GradArgs<BF16, J> G;
        bool vec_ok = aligned16(acc);
#pragma unroll
        for (int j = 0; j < J; ++j) {
            G.g[j] = static_cast<const gelem *>(jb.g[j]) + base;
            G.n[j] = jb.n[j];
            vec_ok = vec_ok && (BF16 ? aligned8(G.g[j]) : aligned16(G.g[j]));
        }
        accumulate_tile<BF16, NTA, J>(acc, G, len, jb.first != 0, vec_ok);
        return;
    }
    if constexpr (J < JMAX) accumulate_job_tile<BF16, NTA, JMAX, J + 1>(acc, jb, base, len);
}

// (job, tile) of workgroup b in a launch of `tiles` tiles per job; at most MAX_JOBS - 1 steps.
__device__ __forceinline__ void job_and_tile(unsigned b, unsigned tiles, unsigned &job, unsigned &tile_index)
{
    job = 0;
    while (b >= tiles) {
        b -= tiles;
        ++job;
    }
    tile_index = b;
}

template <bool BF16, bool NTA, int JMAX>
__global__ __launch_bounds__(ABS_BLOCK) void accumulate_jobs_flat(JobList L, int64_t P, int tile, unsigned tiles,
                                                                 unsigned b0)
{
    unsigned job, t;
    job_and_tile(blockIdx.x + b0, tiles, job, t);
    const JobView<JMAX> jb = view_job<JMAX>(L.job[job]);
    const int64_t base = (int64_t)t * tile;
    accumulate_job_tile<BF16, NTA, JMAX>(jb.acc + base, jb, base, tile_len(P, base, tile));
}

// Ragged: the job's entries are pointer TABLES; the chunk, the tensor's size and the
// tensor's base pointers (accumulator and JMAX gradients, unused entries read from the
// accumulator's table so that every load is valid) follow in a second batch.
template <bool BF16, bool NTA, int JMAX>
__global__ __launch_bounds__(ABS_BLOCK) void accumulate_jobs_ragged(const Chunk *__restrict__ chunks,
                                                                   const int64_t *__restrict__ sizes,
                                                                   JobList L, int tile, unsigned nchunks,
                                                                   unsigned b0)
{
    unsigned job, t;
    job_and_tile(blockIdx.x + b0, nchunks, job, t);
    const JobView<JMAX> tabs = view_job<JMAX>(L.job[job]);
    const Chunk c = chunks[t];
    const int64_t base = (int64_t)c.index * tile;
    JobView<JMAX> jb;
    jb.J = tabs.J;
    jb.first = tabs.first;
    jb.acc = reinterpret_cast<float *const *>(tabs.acc)[c.tensor];
#pragma unroll
    for (int j = 0; j < JMAX; ++j) {
        const void *const *t = j < tabs.J ? static_cast<const void *const *>(tabs.g[j])
                                          : reinterpret_cast<const void *const *>(tabs.acc);
        jb.g[j] = t[c.tensor];
        jb.n[j] = tabs.n[j];
    }
    accumulate_job_tile<BF16, NTA, JMAX>(jb.acc + base, jb, base, tile_len(sizes[c.tensor], base, tile));
}

template <int K> struct TabPtrs { const float *const *t[K]; };
struct TabPtrsAny { const float *const *t[64]; };

template <int K, bool NTX, int RULE>
__global__ __launch_bounds__(ABS_BLOCK) void sync_update_ragged(const Chunk *__restrict__ chunks,
                                                               const int64_t *__restrict__ sizes,
                                                               float *const *__restrict__ x_tab,
                                                               float *const *__restrict__ v_tab,
                                                               float *const *__restrict__ p_tab,
                                                               TabPtrs<K> tabs, int tile, Hyper h, unsigned b0)
{
    const Chunk c = chunks[blockIdx.x + b0];
    const int64_t base = (int64_t)c.index * tile;
    float *x = x_tab[c.tensor] + base;
    float *v = v_tab[c.tensor] + base;
    float *xp = nullptr;
    bool vec_ok = aligned16(x) && aligned16(v);
    if constexpr (uses_s2<RULE>()) {
        xp = p_tab[c.tensor] + base;
        vec_ok = vec_ok && aligned16(xp);
    }
    AccPtrs<K> A;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        A.p[k] = tabs.t[k][c.tensor] + base;
        vec_ok = vec_ok && aligned16(A.p[k]);
    }
    sync_tile<K, NTX, RULE>(x, v, xp, A, tile_len(sizes[c.tensor], base, tile), h, vec_ok);
}

template <int RULE, bool NTX>
__global__ __launch_bounds__(ABS_BLOCK) void sync_update_ragged_any(const Chunk *__restrict__ chunks,
                                                                   const int64_t *__restrict__ sizes,
                                                                   float *const *__restrict__ x_tab,
                                                                   float *const *__restrict__ v_tab,
                                                                   float *const *__restrict__ p_tab,
                                                                   TabPtrsAny tabs, int K, int tile,
                                                                   Hyper h, unsigned b0)
{
    __shared__ const float *ptrs[64];
    __shared__ int all_aligned;
    const Chunk c = chunks[blockIdx.x + b0];
    const int64_t base = (int64_t)c.index * tile;
    if (threadIdx.x == 0) all_aligned = 1;
    __syncthreads();
    if ((int)threadIdx.x < K) {
        const float *p = tabs.t[threadIdx.x][c.tensor] + base;
        ptrs[threadIdx.x] = p;
        if (!aligned16(p)) all_aligned = 0;          // every writer stores the same value
    }
    __syncthreads();
    float *x = x_tab[c.tensor] + base;
    float *v = v_tab[c.tensor] + base;
    float *xp = uses_s2<RULE>() ? p_tab[c.tensor] + base : nullptr;
    const bool vec_ok = aligned16(x) && aligned16(v) && aligned16(xp) && all_aligned != 0;
    sync_tile_any<RULE, NTX>(x, v, xp, ptrs, K, tile_len(sizes[c.tensor], base, tile), h, vec_ok);
}

}  // namespace absk
