// Radial-directional averaging (Appendix D.2 of the paper) as the merge, fused with the outer
// Nesterov step, for one flat tensor.  For each group of `group_len` consecutive elements and
// the contributing learners j (normalised weights w_j, outer gradients d_j = Theta - theta_j):
//
//     N_j   = ||d_j||                     norm over the group
//     R     = sum_j w_j N_j               mean norm
//     u     = sum_j (w_j / N_j) d_j       mean unit direction (learners with N_j = 0 left out)
//     Delta = R * u / ||u||               (0 if u = 0)
//
// Two launch shapes.
// (a) Groups of moderate length (a row of a weight matrix) and many of them: ONE kernel, one
//     workgroup per group, which makes the three sweeps below over its own group back to back
//     and keeps the two reductions in LDS.  The second and third sweep find the group in L2 or
//     in the last-level cache, so HBM sees every byte about once, and no workspace is used.
//     Groups of at most 16384 elements whose data fits the register file take a variant that
//     loads the group once into registers and sweeps those: one pass over HBM, like direct
//     averaging.
// (b) Long or few groups (one norm per tensor): three sweeps over the data, each a grid of one
//     workgroup per "chunk" (at most DDL_RDA_CHUNK consecutive elements of one group), with
//     two small per-group kernels in between:
//   sweep 1  partial sums of d_j^2 per chunk        -> reduce: coefficients c_j = w_j / N_j, R
//   sweep 2  partial sums of u^2 per chunk           -> reduce: scale = R / ||u||
//   sweep 3  Delta = scale * u, outer step, write Theta and v
// Partial sums are combined in a fixed order (no atomics): results are reproducible.
// Sweeps 1 and 2 read with ordinary (cached) loads so that the later sweeps of a small group
// find the data in L2 or the last-level cache; sweep 3 streams.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"
#include "ddl_kernel_util.h"

#define DDL_RDA_CHUNK 8192  // elements per workgroup and sweep: 8 groups of four per lane

struct DdlRdaArgs {
    uint64_t theta, v;          // device addresses
    uint64_t learner[DDL_MAXL]; // compacted: contributing learners only
    float w[DDL_MAXL];          // their normalised weights
    uint64_t n, group_len;
    uint32_t chunks_per_group;
    uint32_t vec_ok;            // all bases 16-byte aligned and group_len % 4 == 0
    float lr, mu;
    // workspace (device): floats
    uint64_t partial1;          // [chunks][Mq]  sums of d_j^2
    uint64_t coef;              // [groups][Mq]  w_j / N_j (0 where N_j = 0)
    uint64_t mean_norm;         // [groups]      R
    uint64_t partial2;          // [chunks]      sums of u^2
    uint64_t scale;             // [groups]      R / ||u|| (0 where u = 0)
};

namespace {

// Elements [begin, end) of chunk `c` (empty if the chunk lies past the end of a short last group).
__device__ __forceinline__ void chunk_range(const DdlRdaArgs& a, uint32_t c, uint64_t& begin,
                                            uint64_t& end, uint32_t& group)
{
    group = c / a.chunks_per_group;
    const uint32_t k = c % a.chunks_per_group;
    const uint64_t g0 = (uint64_t)group * a.group_len;
    const uint64_t g1 = a.n - g0 < a.group_len ? a.n : g0 + a.group_len;
    begin = g0 + (uint64_t)k * DDL_RDA_CHUNK;
    end = begin + DDL_RDA_CHUNK < g1 ? begin + DDL_RDA_CHUNK : g1;
    if (begin > end) begin = end;
}

// Sum over the workgroup; the result is valid in thread 0.  Fixed order: lanes by butterfly,
// then the four waves in sequence.
template <int NTH = DDL_BLOCK>
__device__ __forceinline__ float block_sum(float x, float* lds /* NTH / 64 floats */)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    const int wave = threadIdx.x >> 6;
    __syncthreads();  // lds may still be read from a previous call
    if ((threadIdx.x & 63) == 0) lds[wave] = x;
    __syncthreads();
    float s = 0.0f;
    if (threadIdx.x == 0)
        for (int k = 0; k < NTH / 64; ++k) s += lds[k];
    return s;
}

// The same sum, delivered to every thread.
template <int NTH = DDL_BLOCK>
__device__ __forceinline__ float block_sum_all(float x, float* lds /* NTH / 64 + 1 floats */)
{
    const float s = block_sum<NTH>(x, lds);
    if (threadIdx.x == 0) lds[NTH / 64] = s;
    __syncthreads();
    return lds[NTH / 64];
}

// Sum of count floats at p[k * stride], k < count, by the whole workgroup, in double and in a
// fixed order; valid in thread 0.
__device__ __forceinline__ double block_sum_strided(const float* p, uint32_t count, uint32_t stride,
                                                    double* lds /* DDL_BLOCK doubles */)
{
    double s = 0.0;
    for (uint32_t k = threadIdx.x; k < count; k += DDL_BLOCK) s += (double)p[(size_t)k * stride];
    __syncthreads();
    lds[threadIdx.x] = s;
    __syncthreads();
    for (int half = DDL_BLOCK / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) lds[threadIdx.x] += lds[threadIdx.x + half];
        __syncthreads();
    }
    return lds[0];
}

// Walks the chunk: F(d[MQ], theta, v, element index within the chunk, is the first argument
// pack a vector of 4).  VEC path: groups of four per lane; else element-wise.
template <typename L, int MQ, bool NT, typename F4, typename F1>
__device__ __forceinline__ void sweep_chunk(const DdlRdaArgs& a, uint64_t begin, uint64_t end,
                                            bool need_v, F4&& f4, F1&& f1)
{
    typedef typename L::elem elem;
    const uint32_t len = (uint32_t)(end - begin);
    const uint64_t th = a.theta + begin * 4, vv = a.v + begin * 4;
    uint64_t lp[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) lp[j] = a.learner[j] + begin * sizeof(elem);
    uint32_t done = 0;
    if (a.vec_ok) {
        const uint32_t nvec = len / 4;
        for (uint32_t g = threadIdx.x; g < nvec; g += DDL_BLOCK) {
            typename L::raw raw[MQ];
#pragma unroll
            for (int j = 0; j < MQ; ++j) raw[j] = ld<typename L::raw, NT>(lp[j], g);
            const f32x4 T = ld<f32x4, NT>(th, g);
            f32x4 V = {0.0f, 0.0f, 0.0f, 0.0f};
            if (need_v) V = ld<f32x4, NT>(vv, g);
            float x[MQ][4];
#pragma unroll
            for (int j = 0; j < MQ; ++j) L::widen(raw[j], x[j]);
            const float t4[4] = {T.x, T.y, T.z, T.w};
            float d[4][MQ];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < MQ; ++j) d[k][j] = t4[k] - x[j][k];
            f4(d, T, V, g);
        }
        done = nvec * 4;
    }
    for (uint32_t e = done + threadIdx.x; e < len; e += DDL_BLOCK) {
        const float t = *(reinterpret_cast<const DDL_GLOBAL float*>(th) + e);
        float v = 0.0f;
        if (need_v) v = *(reinterpret_cast<const DDL_GLOBAL float*>(vv) + e);
        float d[MQ];
#pragma unroll
        for (int j = 0; j < MQ; ++j)
            d[j] = t - L::widen1(*(reinterpret_cast<const DDL_GLOBAL elem*>(lp[j]) + e));
        f1(d, t, v, e);
    }
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_sumsq_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[DDL_BLOCK / 64];
    uint64_t begin, end;
    uint32_t group;
    chunk_range(a, blockIdx.x, begin, end, group);
    float ss[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) ss[j] = 0.0f;
    sweep_chunk<L, MQ, false>(
        a, begin, end, false,
        [&](const float (&d)[4][MQ], const f32x4&, const f32x4&, uint32_t) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < MQ; ++j) ss[j] = fmaf(d[k][j], d[k][j], ss[j]);
        },
        [&](const float (&d)[MQ], float, float, uint32_t) {
#pragma unroll
            for (int j = 0; j < MQ; ++j) ss[j] = fmaf(d[j], d[j], ss[j]);
        });
    float* out = reinterpret_cast<float*>(a.partial1) + (size_t)blockIdx.x * MQ;
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const float s = block_sum(ss[j], lds);
        if (threadIdx.x == 0) out[j] = s;
    }
}

// One workgroup per group: norms from the chunk partials (in double, fixed order), then the
// direction coefficients w_j / N_j and the mean norm.
__global__ void __launch_bounds__(DDL_BLOCK) rda_norms_kernel(const DdlRdaArgs a, int Mq)
{
    __shared__ double lds[DDL_BLOCK];
    const uint32_t r = blockIdx.x;
    const float* p1 = reinterpret_cast<const float*>(a.partial1) + (size_t)r * a.chunks_per_group * Mq;
    float* coef = reinterpret_cast<float*>(a.coef) + (size_t)r * Mq;
    double R = 0.0;
    for (int j = 0; j < Mq; ++j) {
        const double ss = block_sum_strided(p1 + j, a.chunks_per_group, (uint32_t)Mq, lds);
        const double N = sqrt(ss);
        R += (double)a.w[j] * N;
        if (threadIdx.x == 0) coef[j] = N > 0.0 ? (float)((double)a.w[j] / N) : 0.0f;
    }
    if (threadIdx.x == 0) reinterpret_cast<float*>(a.mean_norm)[r] = (float)R;
}

template <int MQ>
__device__ __forceinline__ float direction(const float (&d)[MQ], const float (&c)[MQ])
{
    float u = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) u = fmaf(c[j], d[j], u);
    return u;
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_dirsq_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[DDL_BLOCK / 64];
    uint64_t begin, end;
    uint32_t group;
    chunk_range(a, blockIdx.x, begin, end, group);
    float c[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) c[j] = reinterpret_cast<const float*>(a.coef)[(size_t)group * MQ + j];
    float ss = 0.0f;
    sweep_chunk<L, MQ, false>(
        a, begin, end, false,
        [&](const float (&d)[4][MQ], const f32x4&, const f32x4&, uint32_t) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float u = direction<MQ>(d[k], c);
                ss = fmaf(u, u, ss);
            }
        },
        [&](const float (&d)[MQ], float, float, uint32_t) {
            const float u = direction<MQ>(d, c);
            ss = fmaf(u, u, ss);
        });
    const float s = block_sum(ss, lds);
    if (threadIdx.x == 0) reinterpret_cast<float*>(a.partial2)[blockIdx.x] = s;
}

__global__ void __launch_bounds__(DDL_BLOCK) rda_scale_kernel(const DdlRdaArgs a)
{
    __shared__ double lds[DDL_BLOCK];
    const uint32_t r = blockIdx.x;
    const float* p2 = reinterpret_cast<const float*>(a.partial2) + (size_t)r * a.chunks_per_group;
    const double U = sqrt(block_sum_strided(p2, a.chunks_per_group, 1, lds));
    const double R = (double)reinterpret_cast<const float*>(a.mean_norm)[r];
    if (threadIdx.x == 0) reinterpret_cast<float*>(a.scale)[r] = U > 0.0 ? (float)(R / U) : 0.0f;
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_apply_kernel(const DdlRdaArgs a)
{
    uint64_t begin, end;
    uint32_t group;
    chunk_range(a, blockIdx.x, begin, end, group);
    float c[MQ];
    const float scale = reinterpret_cast<const float*>(a.scale)[group];
#pragma unroll
    for (int j = 0; j < MQ; ++j)
        c[j] = reinterpret_cast<const float*>(a.coef)[(size_t)group * MQ + j] * scale;
    const float lr = a.lr, mu = a.mu;
    const uint64_t th = a.theta + begin * 4, vv = a.v + begin * 4;
    sweep_chunk<L, MQ, true>(
        a, begin, end, true,
        [&](const float (&d)[4][MQ], const f32x4& T, const f32x4& V, uint32_t g) {
            float t4[4] = {T.x, T.y, T.z, T.w};
            float v4[4] = {V.x, V.y, V.z, V.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float delta = direction<MQ>(d[k], c);
                v4[k] = fmaf(mu, v4[k], delta);
                t4[k] = fmaf(-lr, fmaf(mu, v4[k], delta), t4[k]);
            }
            const f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
            const f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
            st<f32x4>(th, g, tn);
            st<f32x4>(vv, g, vn);
        },
        [&](const float (&d)[MQ], float t, float v, uint32_t e) {
            const float delta = direction<MQ>(d, c);
            const float v_new = fmaf(mu, v, delta);
            *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = fmaf(-lr, fmaf(mu, v_new, delta), t);
            *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v_new;
        });
}

// Launch shape (a): one workgroup makes all three sweeps over its own group.
template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_group_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[DDL_BLOCK / 64 + 1];
    const uint64_t g0 = (uint64_t)blockIdx.x * a.group_len;
    const uint64_t g1 = a.n - g0 < a.group_len ? a.n : g0 + a.group_len;

    // sweep 1: norms of the outer gradients
    float ss[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) ss[j] = 0.0f;
    for (uint64_t begin = g0; begin < g1; begin += DDL_RDA_CHUNK) {
        const uint64_t end = begin + DDL_RDA_CHUNK < g1 ? begin + DDL_RDA_CHUNK : g1;
        sweep_chunk<L, MQ, false>(
            a, begin, end, false,
            [&](const float (&d)[4][MQ], const f32x4&, const f32x4&, uint32_t) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int j = 0; j < MQ; ++j) ss[j] = fmaf(d[k][j], d[k][j], ss[j]);
            },
            [&](const float (&d)[MQ], float, float, uint32_t) {
#pragma unroll
                for (int j = 0; j < MQ; ++j) ss[j] = fmaf(d[j], d[j], ss[j]);
            });
    }
    float c[MQ];
    float R = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const float N = sqrtf(block_sum_all(ss[j], lds));
        R = fmaf(a.w[j], N, R);
        c[j] = N > 0.0f ? a.w[j] / N : 0.0f;
    }

    // sweep 2: norm of the mean direction
    float uu = 0.0f;
    for (uint64_t begin = g0; begin < g1; begin += DDL_RDA_CHUNK) {
        const uint64_t end = begin + DDL_RDA_CHUNK < g1 ? begin + DDL_RDA_CHUNK : g1;
        sweep_chunk<L, MQ, false>(
            a, begin, end, false,
            [&](const float (&d)[4][MQ], const f32x4&, const f32x4&, uint32_t) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float u = direction<MQ>(d[k], c);
                    uu = fmaf(u, u, uu);
                }
            },
            [&](const float (&d)[MQ], float, float, uint32_t) {
                const float u = direction<MQ>(d, c);
                uu = fmaf(u, u, uu);
            });
    }
    const float U = sqrtf(block_sum_all(uu, lds));
    const float scale = U > 0.0f ? R / U : 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) c[j] *= scale;

    // sweep 3: Delta = scale * u, outer step
    const float lr = a.lr, mu = a.mu;
    for (uint64_t begin = g0; begin < g1; begin += DDL_RDA_CHUNK) {
        const uint64_t end = begin + DDL_RDA_CHUNK < g1 ? begin + DDL_RDA_CHUNK : g1;
        const uint64_t th = a.theta + begin * 4, vv = a.v + begin * 4;
        sweep_chunk<L, MQ, false>(
            a, begin, end, true,
            [&](const float (&d)[4][MQ], const f32x4& T, const f32x4& V, uint32_t g) {
                float t4[4] = {T.x, T.y, T.z, T.w};
                float v4[4] = {V.x, V.y, V.z, V.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float delta = direction<MQ>(d[k], c);
                    v4[k] = fmaf(mu, v4[k], delta);
                    t4[k] = fmaf(-lr, fmaf(mu, v4[k], delta), t4[k]);
                }
                const f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
                const f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
                st<f32x4>(th, g, tn);
                st<f32x4>(vv, g, vn);
            },
            [&](const float (&d)[MQ], float t, float v, uint32_t e) {
                const float delta = direction<MQ>(d, c);
                const float v_new = fmaf(mu, v, delta);
                *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = fmaf(-lr, fmaf(mu, v_new, delta), t);
                *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v_new;
            });
    }
}

// Tells the compiler that a register's value may have changed.  Used between the sweeps of
// the row kernel so that only the packed learner values stay live across them, not their
// widened fp32 images and differences (which it would otherwise keep: 2-4x the registers).
__device__ __forceinline__ void launder(u32x2& r) { asm volatile("" : "+v"(r.x), "+v"(r.y)); }
__device__ __forceinline__ void launder(u32x4& r)
{
    asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w));
}

// Launch shape (a'), for groups of at most K * 4 * NTH elements on the aligned path: the
// workgroup loads its whole group ONCE into registers (learner values stay packed as loaded)
// and makes the three sweeps over the registers.  HBM traffic equals that of direct averaging.
template <typename L, int MQ, int K, int NTH>
__global__ void __launch_bounds__(NTH) rda_row_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[NTH / 64 + 1];
    typedef typename L::elem elem;
    const uint64_t g0 = (uint64_t)blockIdx.x * a.group_len;
    const uint64_t g1 = a.n - g0 < a.group_len ? a.n : g0 + a.group_len;
    const uint32_t nvec = (uint32_t)(g1 - g0) / 4;  // the host sends only multiples of four here
    const uint64_t th = a.theta + g0 * 4, vv = a.v + g0 * 4;
    uint64_t lp[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) lp[j] = a.learner[j] + g0 * sizeof(elem);

    typename L::raw raw[K][MQ];
    f32x4 T[K];
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t g = threadIdx.x + u * NTH;
        if (g < nvec) {
#pragma unroll
            for (int j = 0; j < MQ; ++j) raw[u][j] = ld<typename L::raw, true>(lp[j], g);
            T[u] = ld<f32x4, true>(th, g);
        } else {  // lanes past the end of the group hold a zero outer gradient
#pragma unroll
            for (int j = 0; j < MQ; ++j) raw[u][j] = typename L::raw(0);
            T[u] = f32x4(0.0f);
        }
    }

    // outer gradients of group u, element k, recomputed from the packed registers on demand
    auto diffs = [&](int u, float (&d)[4][MQ]) {
        float x[MQ][4];
#pragma unroll
        for (int j = 0; j < MQ; ++j) L::widen(raw[u][j], x[j]);
        const float t4[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < MQ; ++j) d[k][j] = t4[k] - x[j][k];
    };

    float ss[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) ss[j] = 0.0f;
#pragma unroll
    for (int u = 0; u < K; ++u) {
        float d[4][MQ];
        diffs(u, d);
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < MQ; ++j) ss[j] = fmaf(d[k][j], d[k][j], ss[j]);
    }
    float c[MQ];
    float R = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const float N = sqrtf(block_sum_all<NTH>(ss[j], lds));
        R = fmaf(a.w[j], N, R);
        c[j] = N > 0.0f ? a.w[j] / N : 0.0f;
    }

#pragma unroll
    for (int u = 0; u < K; ++u)
#pragma unroll
        for (int j = 0; j < MQ; ++j) launder(raw[u][j]);
    float uu = 0.0f;
#pragma unroll
    for (int u = 0; u < K; ++u) {
        float d[4][MQ];
        diffs(u, d);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float x = direction<MQ>(d[k], c);
            uu = fmaf(x, x, uu);
        }
    }
    const float U = sqrtf(block_sum_all<NTH>(uu, lds));
    const float scale = U > 0.0f ? R / U : 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) c[j] *= scale;

#pragma unroll
    for (int u = 0; u < K; ++u)
#pragma unroll
        for (int j = 0; j < MQ; ++j) launder(raw[u][j]);
    const float lr = a.lr, mu = a.mu;
    f32x4 V[K];
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t g = threadIdx.x + u * NTH;
        V[u] = g < nvec ? ld<f32x4, true>(vv, g) : f32x4(0.0f);
    }
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t g = threadIdx.x + u * NTH;
        float d[4][MQ];
        diffs(u, d);
        float t4[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
        float v4[4] = {V[u].x, V[u].y, V[u].z, V[u].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float delta = direction<MQ>(d[k], c);
            v4[k] = fmaf(mu, v4[k], delta);
            t4[k] = fmaf(-lr, fmaf(mu, v4[k], delta), t4[k]);
        }
        if (g < nvec) {
            const f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
            const f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
            st<f32x4>(th, g, tn);
            st<f32x4>(vv, g, vn);
        }
    }
}

// Registers the row kernel keeps per lane: K groups of (packed learners + Theta + v); a
// 1024-thread workgroup leaves each lane 128 registers, a 256-thread one 512.
template <typename L, int MQ, int K, int NTH>
constexpr bool row_kernel_fits()
{
    return K * ((int)(sizeof(typename L::raw) / 4) * MQ + 8) <= (NTH > 256 ? 80 : 192);
}

typedef void (*rda_fn)(const DdlRdaArgs);

template <typename L, int MQ, int K, int NTH>
rda_fn row_kernel_or_null()
{
    if constexpr (row_kernel_fits<L, MQ, K, NTH>())
        return rda_row_kernel<L, MQ, K, NTH>;
    else
        return nullptr;
}

// The row kernel with the smallest footprint that holds `len` elements, if its registers fit.
template <typename L, int MQ>
rda_fn pick_row(uint64_t len, uint32_t& threads)
{
    threads = 256;
    if (len <= 1 * 1024) return row_kernel_or_null<L, MQ, 1, 256>();
    if (len <= 2 * 1024) return row_kernel_or_null<L, MQ, 2, 256>();
    if (len <= 4 * 1024) return row_kernel_or_null<L, MQ, 4, 256>();
    if (len <= 8 * 1024) return row_kernel_or_null<L, MQ, 8, 256>();
    threads = 1024;
    if (len <= 16 * 1024) return row_kernel_or_null<L, MQ, 4, 1024>();
    return nullptr;
}

template <typename L>
void pick(int Mq, uint64_t group_len, rda_fn& k1, rda_fn& k2, rda_fn& k3, rda_fn& kg, rda_fn& kr,
          uint32_t& kr_threads)
{
    switch (Mq) {
#define DDL_CASE(k)                        \
    case k:                                \
        k1 = rda_sumsq_kernel<L, k>;       \
        k2 = rda_dirsq_kernel<L, k>;       \
        k3 = rda_apply_kernel<L, k>;       \
        kg = rda_group_kernel<L, k>;       \
        kr = pick_row<L, k>(group_len, kr_threads); \
        break;
        DDL_CASE(1) DDL_CASE(2) DDL_CASE(3) DDL_CASE(4) DDL_CASE(5) DDL_CASE(6) DDL_CASE(7)
        DDL_CASE(8) DDL_CASE(9) DDL_CASE(10) DDL_CASE(11) DDL_CASE(12) DDL_CASE(13)
        DDL_CASE(14) DDL_CASE(15) DDL_CASE(16)
#undef DDL_CASE
    }
}

struct Geometry {
    uint64_t groups, chunks_per_group, chunks;
    size_t off_partial1, off_coef, off_mean, off_partial2, off_scale, bytes;
};

// Workspace layout for n elements in groups of group_len with Mq contributing learners
// (sized for Mq = M, the worst case, by the public size query).
bool geometry(size_t n, size_t group_len, int Mq, Geometry& g)
{
    if (n == 0 || group_len == 0 || Mq < 1) return false;
    const uint64_t glen = std::min<uint64_t>(group_len, n);
    g.groups = (n + glen - 1) / glen;
    g.chunks_per_group = (glen + DDL_RDA_CHUNK - 1) / DDL_RDA_CHUNK;
    g.chunks = g.groups * g.chunks_per_group;
    if (g.chunks > 0x7fffffffull || g.chunks_per_group > 0xffffffffull) return false;
    size_t off = 0;
    auto take = [&](uint64_t floats) {
        const size_t at = off;
        off += ((size_t)floats * 4 + 255) & ~(size_t)255;
        return at;
    };
    g.off_partial1 = take(g.chunks * Mq);
    g.off_coef = take(g.groups * Mq);
    g.off_mean = take(g.groups);
    g.off_partial2 = take(g.chunks);
    g.off_scale = take(g.groups);
    g.bytes = off;
    return true;
}

// Launch shape (a) is taken for groups no longer than this, if there are enough of them to
// fill the GPU (one workgroup each).
constexpr uint64_t kGroupKernelMaxLen = 65536;
constexpr uint32_t kGroupKernelMinGroups = 512;

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

extern "C" size_t ddl_rda_workspace_bytes(size_t n, size_t group_len, int M)
{
    Geometry g;
    if (M < 1 || M > DDL_MAX_LEARNERS || !geometry(n, group_len, M, g)) return 0;
    return g.bytes;
}

extern "C" ddl_status ddl_rda_merge_fragment(float* theta, float* v,
                                             const void* const* learner_params,
                                             ddl_dtype learner_dtype, const uint64_t* token_counts,
                                             const uint8_t* quorum_mask, int M, size_t n,
                                             size_t group_len, float lr, float mu, void* workspace,
                                             size_t workspace_bytes, void* hip_stream)
{
    double w[DDL_MAX_LEARNERS];
    ddl_status st = ddl_compute_weights(token_counts, quorum_mask, M, w);
    if (st != DDL_OK) return st;
    if (learner_dtype != DDL_F32 && learner_dtype != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (!std::isfinite(lr) || lr < 0.0f || !std::isfinite(mu) || mu < 0.0f) return DDL_ERR_INVALID_ARG;
    if (group_len == 0) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!theta || !v || !learner_params || !aligned(theta, 4) || !aligned(v, 4))
        return DDL_ERR_INVALID_ARG;

    DdlRdaArgs a;
    std::memset(&a, 0, sizeof a);
    const size_t b = learner_dtype == DDL_BF16 ? 2 : 4;
    int Mq = 0;
    bool vec_ok = aligned(theta, 16) && aligned(v, 16) && std::min(group_len, n) % 4 == 0;
    // Overlap rules as everywhere: Theta, v and the workspace may overlap nothing.
    struct Range { uintptr_t lo, hi; bool out; };
    std::vector<Range> r;
    r.push_back({(uintptr_t)theta, (uintptr_t)theta + 4 * n, true});
    r.push_back({(uintptr_t)v, (uintptr_t)v + 4 * n, true});
    for (int m = 0; m < M; ++m) {
        if (!(w[m] > 0.0)) continue;
        const void* p = learner_params[m];
        if (!p || !aligned(p, b)) return DDL_ERR_INVALID_ARG;
        vec_ok = vec_ok && aligned(p, 16);
        a.learner[Mq] = (uint64_t)(uintptr_t)p;
        a.w[Mq] = (float)w[m];
        r.push_back({(uintptr_t)p, (uintptr_t)p + b * n, false});
        ++Mq;
    }
    Geometry g;
    if (!geometry(n, group_len, Mq, g)) return DDL_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < g.bytes) return DDL_ERR_INVALID_ARG;
    r.push_back({(uintptr_t)workspace, (uintptr_t)workspace + g.bytes, true});
    std::sort(r.begin(), r.end(), [](const Range& x, const Range& y) { return x.lo < y.lo; });
    uintptr_t hi_any = 0, hi_out = 0;
    for (const Range& x : r) {
        if (x.out ? x.lo < hi_any : x.lo < hi_out) return DDL_ERR_ALIAS;
        hi_any = std::max(hi_any, x.hi);
        if (x.out) hi_out = std::max(hi_out, x.hi);
    }

    a.theta = (uint64_t)(uintptr_t)theta;
    a.v = (uint64_t)(uintptr_t)v;
    a.n = n;
    a.group_len = std::min<uint64_t>(group_len, n);
    a.chunks_per_group = (uint32_t)g.chunks_per_group;
    a.vec_ok = vec_ok ? 1u : 0u;
    a.lr = lr;
    a.mu = mu;
    const uint64_t ws = (uint64_t)(uintptr_t)workspace;
    a.partial1 = ws + g.off_partial1;
    a.coef = ws + g.off_coef;
    a.mean_norm = ws + g.off_mean;
    a.partial2 = ws + g.off_partial2;
    a.scale = ws + g.off_scale;

    rda_fn k1 = nullptr, k2 = nullptr, k3 = nullptr, kg = nullptr, kr = nullptr;
    uint32_t kr_threads = DDL_BLOCK;
    if (learner_dtype == DDL_F32)
        pick<LearnerF32>(Mq, a.group_len, k1, k2, k3, kg, kr, kr_threads);
    else
        pick<LearnerBF16>(Mq, a.group_len, k1, k2, k3, kg, kr, kr_threads);
    if (!k1) return DDL_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const dim3 block(DDL_BLOCK);
    const uint32_t groups = (uint32_t)g.groups;
    if (kr && vec_ok && n % 4 == 0 && groups >= kGroupKernelMinGroups) {
        hipLaunchKernelGGL(kr, dim3(groups), dim3(kr_threads), 0, stream, a);
    } else if (a.group_len <= kGroupKernelMaxLen && groups >= kGroupKernelMinGroups) {
        const long cap = ddl_opt_rda_blocks_per_cu;
        uint32_t lds = cap > 0 ? (uint32_t)(DDL_LDS_PER_CU / cap) & ~511u : 0u;
        if (lds > 60 * 1024) lds = 60 * 1024;  // static LDS of the kernel comes on top
        hipLaunchKernelGGL(kg, dim3(groups), block, lds, stream, a);
    } else {
        const dim3 grid((uint32_t)g.chunks), rgrid(groups);
        hipLaunchKernelGGL(k1, grid, block, 0, stream, a);
        hipLaunchKernelGGL(rda_norms_kernel, rgrid, block, 0, stream, a, Mq);
        hipLaunchKernelGGL(k2, grid, block, 0, stream, a);
        hipLaunchKernelGGL(rda_scale_kernel, rgrid, block, 0, stream, a);
        hipLaunchKernelGGL(k3, grid, block, 0, stream, a);
    }
    return hipGetLastError() == hipSuccess ? DDL_OK : DDL_ERR_RUNTIME;
}
