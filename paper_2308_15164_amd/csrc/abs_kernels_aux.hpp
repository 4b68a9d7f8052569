// Device code used by one translation unit only (launch_accumulate.hip): the copy
// kernels and the three LARS kernels.  None of them is a template, so they are kept
// out of abs_kernels.hpp, which several units include.
#pragma once

#include "abs_kernels.hpp"

namespace absk {

// dst[0..len) = src[0..len): keeps the previous-iterate buffer current on a step
// that applies nothing.
__device__ __forceinline__ void copy_tile(float *__restrict__ dst, const float *__restrict__ src, int len,
                                          bool vec_ok)
{
    const int tid = threadIdx.x;
    if (vec_ok) {
        const int nvec = len / VEC;
        for (int i = tid; i < nvec; i += BLOCK)
            reinterpret_cast<f32x4 *>(dst)[i] = reinterpret_cast<const f32x4 *>(src)[i];
        const int i = nvec * VEC + tid;
        if (i < len) dst[i] = src[i];
        return;
    }
    for (int i = tid; i < len; i += BLOCK) dst[i] = src[i];
}

__global__ __launch_bounds__(ABS_BLOCK) void copy_flat(float *__restrict__ dst,
                                                      const float *__restrict__ src, int64_t P,
                                                      int tile, int vec_ok)
{
    const int64_t base = (int64_t)blockIdx.x * tile;
    copy_tile(dst + base, src + base, tile_len(P, base, tile), vec_ok != 0);
}

__global__ __launch_bounds__(ABS_BLOCK) void copy_ragged(const Chunk *__restrict__ chunks,
                                                        const int64_t *__restrict__ sizes,
                                                        float *const *__restrict__ dst_tab,
                                                        float *const *__restrict__ src_tab, int tile)
{
    const Chunk c = chunks[blockIdx.x];
    const int64_t base = (int64_t)c.index * tile;
    float *dst = dst_tab[c.tensor] + base;
    const float *src = src_tab[c.tensor] + base;
    copy_tile(dst, src, tile_len(sizes[c.tensor], base, tile), aligned16(dst) && aligned16(src));
}


// ----------------------------------------------------------------------- LARS
//
// Layer-wise adaptive rate scaling needs two Euclidean norms per tensor before
// any element can be updated, so it takes three launches over the ragged layout:
//   1. lars_reduce : Gbar = (sum_k acc_k) / M is formed once, written to a
//                    workspace, and each workgroup leaves the sums of Gbar^2 and
//                    x^2 over its chunk (4K + 8 B/param);
//   2. lars_rates  : one workgroup per tensor adds its chunks' sums and turns
//                    them into the tensor's step factor (negligible traffic);
//   3. lars_update : v = fma(mu, v, step_l * fma(wd, x, Gbar)); x = x - v
//                    (20 B/param, independent of K).
// Sums are carried in double and added in a fixed order (lane, wavefront,
// workgroup, chunk), so results do not depend on timing.

// Sums a and b over the workgroup; the totals are valid in thread 0.
__device__ __forceinline__ void block_sum2(double &a, double &b)
{
    __shared__ double sm[2][BLOCK / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_down(a, off);
        b += __shfl_down(b, off);
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) { sm[0][wave] = a; sm[1][wave] = b; }
    __syncthreads();
    if (threadIdx.x == 0) {
        a = sm[0][0];
        b = sm[1][0];
        for (int w = 1; w < BLOCK / 64; ++w) { a += sm[0][w]; b += sm[1][w]; }
    }
}

__device__ __forceinline__ void add_squares(double &acc, f32x4 q)
{
    acc += (double)q.x * (double)q.x;
    acc += (double)q.y * (double)q.y;
    acc += (double)q.z * (double)q.z;
    acc += (double)q.w * (double)q.w;
}

__global__ __launch_bounds__(ABS_BLOCK) void lars_reduce_ragged(const Chunk *__restrict__ chunks,
                                                               const int64_t *__restrict__ sizes,
                                                               float *const *__restrict__ x_tab,
                                                               float *const *__restrict__ g_tab,
                                                               TabPtrsAny tabs, int K, int tile, float M,
                                                               double *__restrict__ partials, unsigned b0)
{
    constexpr int U = 4, KC = 4;
    const unsigned cb = blockIdx.x + b0;       // chunk of this workgroup (b0: first workgroup of this launch in the call)
    const Chunk c = chunks[cb];
    const int64_t base = (int64_t)c.index * tile;
    const int len = tile_len(sizes[c.tensor], base, tile);
    const float *__restrict__ x = x_tab[c.tensor] + base;
    float *__restrict__ gb = g_tab[c.tensor] + base;
    bool vec_ok = aligned16(x) && aligned16(gb);
    for (int k = 0; k < K; ++k) vec_ok = vec_ok && aligned16(tabs.t[k][c.tensor] + base);
    const int tid = threadIdx.x;
    double sx = 0.0, sg = 0.0;
    int done = 0;
    if (vec_ok) {
        const int nvec = len / VEC;
        const f32x4 *xv = reinterpret_cast<const f32x4 *>(x);
        f32x4 *gv = reinterpret_cast<f32x4 *>(gb);
        for (int g0 = 0; g0 < nvec; g0 += U * BLOCK) {
            f32x4 sum[U] = {}, xr[U] = {};
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = GIDX(g0, u, tid, U, false);
                if (i < nvec) xr[u] = xv[i];
            }
            for (int k0 = 0; k0 < K; k0 += KC) {
                f32x4 a[U][KC] = {};
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
                    if (k0 + kk < K) {
                        const f32x4 *ap = reinterpret_cast<const f32x4 *>(tabs.t[k0 + kk][c.tensor] + base);
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const int i = GIDX(g0, u, tid, U, false);
                            if (i < nvec) a[u][kk] = ld<ABS_NT_SYNC_ACC != 0>(ap + i);
                        }
                    }
                }
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
                    if (k0 + kk < K) {
#pragma unroll
                        for (int u = 0; u < U; ++u) sum[u] = (k0 + kk == 0) ? a[u][kk] : sum[u] + a[u][kk];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = GIDX(g0, u, tid, U, false);
                if (i < nvec) {
                    f32x4 g;
                    g.x = sum[u].x / M; g.y = sum[u].y / M; g.z = sum[u].z / M; g.w = sum[u].w / M;
                    gv[i] = g;
                    add_squares(sg, g);
                    add_squares(sx, xr[u]);
                }
            }
        }
        done = nvec * VEC;
    }
    for (int i = done + tid; i < len; i += BLOCK) {
        float s = tabs.t[0][c.tensor][base + i];
        for (int k = 1; k < K; ++k) s = s + tabs.t[k][c.tensor][base + i];
        const float g = s / M;
        gb[i] = g;
        sg += (double)g * (double)g;
        sx += (double)x[i] * (double)x[i];
    }
    block_sum2(sx, sg);
    if (tid == 0) {
        partials[2 * (int64_t)cb] = sx;
        partials[2 * (int64_t)cb + 1] = sg;
    }
}

// begin[t] = index of tensor t's first chunk, t = 0..T (begin[T] = nchunks), from the
// chunk table alone: chunks are ordered by tensor, a tensor without elements has none.
// One thread per chunk plus one; every entry is written exactly once.
__global__ __launch_bounds__(ABS_BLOCK) void lars_chunk_begin(const Chunk *__restrict__ chunks, int nchunks,
                                                             int T, int32_t *__restrict__ begin)
{
    const int c = blockIdx.x * BLOCK + threadIdx.x;
    if (c > nchunks) return;
    const int lo = c == 0 ? 0 : chunks[c - 1].tensor + 1;          // first tensor not yet begun before chunk c
    const int hi = c == nchunks ? T : chunks[c].tensor;            // tensors lo..hi begin at chunk c
    for (int t = lo; t <= hi; ++t) begin[t] = c;
}

// One workgroup per tensor: chunk_begin[t] .. chunk_begin[t+1] are its chunks
// (thousands for an embedding matrix, so the reads are spread over the workgroup
// and issued several at a time; the order of the additions stays fixed).
//   rate = eta*||x|| / (||g|| + wd*||x||)  (1 if either norm is 0);  step[t] = (float)(lr * rate)
__global__ __launch_bounds__(ABS_BLOCK) void lars_rates(const int32_t *__restrict__ chunk_begin,
                                                       const double *__restrict__ partials,
                                                       float *__restrict__ step, double lr, double wd, double eta)
{
    const int t = blockIdx.x;
    const int begin = chunk_begin[t], end = chunk_begin[t + 1];
    double sx = 0.0, sg = 0.0;
    int c = begin + (int)threadIdx.x;
    for (; c + 3 * BLOCK < end; c += 4 * BLOCK) {
        double px[4], pg[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            px[u] = partials[2 * (int64_t)(c + u * BLOCK)];
            pg[u] = partials[2 * (int64_t)(c + u * BLOCK) + 1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) { sx += px[u]; sg += pg[u]; }
    }
    for (; c < end; c += BLOCK) {
        sx += partials[2 * (int64_t)c];
        sg += partials[2 * (int64_t)c + 1];
    }
    block_sum2(sx, sg);
    if (threadIdx.x == 0) {
        const double xn = sqrt(sx), gn = sqrt(sg);
        const double rate = (xn > 0.0 && gn > 0.0) ? eta * xn / (gn + wd * xn) : 1.0;
        step[t] = (float)(lr * rate);
    }
}

// d = fma(wd, x, Gbar); v = fma(mu, v, step_l * d); x = x - v.
__global__ __launch_bounds__(ABS_BLOCK) void lars_update_ragged(const Chunk *__restrict__ chunks,
                                                               const int64_t *__restrict__ sizes,
                                                               float *const *__restrict__ x_tab,
                                                               float *const *__restrict__ v_tab,
                                                               float *const *__restrict__ g_tab,
                                                               const float *__restrict__ step, int tile,
                                                               float mu, float wd, unsigned b0)
{
    constexpr int U = 4;
    const Chunk c = chunks[blockIdx.x + b0];
    const int64_t base = (int64_t)c.index * tile;
    const int len = tile_len(sizes[c.tensor], base, tile);
    float *__restrict__ x = x_tab[c.tensor] + base;
    float *__restrict__ v = v_tab[c.tensor] + base;
    const float *__restrict__ gb = g_tab[c.tensor] + base;
    const float st_l = step[c.tensor];
    const bool vec_ok = aligned16(x) && aligned16(v) && aligned16(gb);
    const int tid = threadIdx.x;
    int done = 0;
    if (vec_ok) {
        const int nvec = len / VEC;
        f32x4 *xv = reinterpret_cast<f32x4 *>(x);
        f32x4 *vv = reinterpret_cast<f32x4 *>(v);
        const f32x4 *gv = reinterpret_cast<const f32x4 *>(gb);
        for (int g0 = 0; g0 < nvec; g0 += U * BLOCK) {
            f32x4 g[U] = {}, xr[U] = {}, vr[U] = {};
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = GIDX(g0, u, tid, U, false);
                if (i < nvec) { g[u] = ld<true>(gv + i); xr[u] = xv[i]; vr[u] = vv[i]; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = GIDX(g0, u, tid, U, false);
                if (i < nvec) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = __builtin_fmaf(wd, xr[u][e], g[u][e]);
                        const float vn = __builtin_fmaf(mu, vr[u][e], st_l * d);
                        vr[u][e] = vn;
                        xr[u][e] = xr[u][e] - vn;
                    }
                    vv[i] = vr[u];
                    xv[i] = xr[u];
                }
            }
        }
        done = nvec * VEC;
    }
    for (int i = done + tid; i < len; i += BLOCK) {
        const float d = __builtin_fmaf(wd, x[i], gb[i]);
        const float vn = __builtin_fmaf(mu, v[i], st_l * d);
        v[i] = vn;
        x[i] = x[i] - vn;
    }
}

}  // namespace absk
