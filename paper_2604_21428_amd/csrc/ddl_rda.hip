// Radial-directional averaging (Appendix D.2 of the paper) as the merge, fused with the outer
// Nesterov step, for one flat tensor.  For each group of `group_len` consecutive elements and
// the contributing learners j (normalised weights w_j, outer gradients d_j = Theta - theta_j):
//
//     N_j   = ||d_j||                     norm over the group
//     R     = sum_j w_j N_j               mean norm
//     u     = sum_j (w_j / N_j) d_j       mean unit direction (learners with N_j = 0 left out)
//     Delta = R * u / ||u||               (0 if u = 0)
//
// The learners' data are their copies theta_j of the tensor (fp32 or bf16), or -- the outer
// gradients having been compressed for the wire (Appendix D.3) -- the d_j themselves as 4-bit
// codes with block scales, d_j = scale * code: every kernel here is instantiated for the three
// kinds (the 4-bit form then reads neither Theta nor v in the sweeps that only reduce, gets a
// group-of-four's sum of squares from one 4-bit dot-product instruction, and folds the block's
// scale into the direction coefficient).
//
// Two launch shapes.
// (a) Groups of moderate length (a row of a weight matrix) and many of them: ONE kernel, one
//     workgroup per group, which makes the three sweeps below over its own group back to back
//     and keeps the two reductions in LDS.  The second and third sweep find the group in L2 or
//     in the last-level cache, so HBM sees every byte about once, and no workspace is used.
//     Groups of at most 16384 elements whose data fits the register file take a variant that
//     loads the group once into registers and sweeps those: one pass over HBM, like direct
//     averaging.
// (b) Long or few groups (one norm per tensor): sweeps over the data as grids of one workgroup
//     per "chunk" (at most DDL_RDA_CHUNK consecutive elements of one group), with small
//     per-group kernels in between.  Everything the method needs from the first look at the
//     data is in the Gram matrix G_jk = <d_j, d_k> of the group: N_j = sqrt(G_jj), and the norm
//     of the mean direction is ||sum_j c_j d_j||^2 = c' G c with c_j = w_j / N_j.  So for up to
//     kGramMaxLearners contributing learners:
//   sweep 1  partial sums of d_j d_k (j <= k) per chunk   -> reduce (fp64, fixed order): c_j, R,
//                                                             c' G c, scale = R / sqrt(c' G c)
//   sweep 2  Delta = scale * sum_j c_j d_j, outer step, write Theta and v (in the merge
//            kernel's shape: one workgroup per tile, i.e. per eighth of a chunk)
//     -- two passes over HBM instead of three.  c' G c cancels when the outer gradients nearly
//     oppose each other; a group whose c' G c is below kGramTrust of sum_jk |c_j c_k G_jk| gets
//     its direction norm summed from the data after all, by the workgroup of the reduce kernel
//     that found it so.  More learners than that take
//   sweep 1  partial sums of d_j^2 per chunk              -> reduce: c_j, R
//   sweep 2  partial sums of u^2 per chunk                -> reduce: scale = R / ||u||
//   sweep 3  apply.
// Partial sums are combined in a fixed order (no atomics): results are reproducible.
// The sweeps before the last read with ordinary (cached) loads so that the later sweeps of a
// small group find the data in L2 or the last-level cache; the last sweep streams.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"
#include "ddl_host_internal.h"
#include "ddl_kernel_util.h"

#ifndef DDL_RDA_V_EARLY
#define DDL_RDA_V_EARLY 0  // 1: the row kernels load v with the first sweep instead of the last
#endif
#ifndef DDL_RDA_Q4_V_EARLY
#define DDL_RDA_Q4_V_EARLY 0  // the same for the row kernels on 4-bit outer gradients only
#endif
#ifndef DDL_RDA_GRAM_LOAD
#define DDL_RDA_GRAM_LOAD 0  // load form of the Gram sweep (see ld<>): 0 cached, so that the apply
                             // sweep of a tensor that fits the last-level cache finds it there
#endif
#ifndef DDL_RDA_CHUNK
#define DDL_RDA_CHUNK 8192  // elements per partial sum: 8 groups of four per lane in the reducing sweeps
#endif

struct DdlRdaArgs {
    uint64_t theta, v;          // device addresses
    uint64_t theta_bf16;        // optional bf16 copy of the new Theta (0: none)
    uint64_t learner[DDL_MAXL]; // compacted: contributing learners only (their copies of the
                                // tensor, or, for 4-bit outer gradients, their codes)
    uint64_t scales[DDL_MAXL];  // 4-bit outer gradients: their block scales
    uint32_t block_len;         // ... and the block length (block_shift: log2 of it, or
    uint32_t block_shift;       // 0xffffffff if it is no power of two)
    float w[DDL_MAXL];          // their normalised weights
    uint64_t n, group_len;
    uint32_t chunks_per_group;
    uint32_t vec_ok;            // all bases 16-byte aligned and group_len % 4 == 0
    float lr, mu;
    uint32_t piece_shift;       // apply sweep: a workgroup takes one of 1 << piece_shift slices of a chunk
    uint32_t pad;
    // workspace (device): floats
    uint64_t partial1;          // [chunks][Mq] sums of d_j^2, or [chunks][Mq (Mq + 1) / 2] of d_j d_k
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

// N sums at once, each delivered to every thread: lanes by butterfly, then the waves'
// partial sums in sequence (a fixed order, the same in every thread).  Two barriers for all N.
template <int NTH, int N>
__device__ __forceinline__ void block_sum_all(float (&x)[N], float* lds /* NTH / 64 * N floats */)
{
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) x[j] += __shfl_xor(x[j], off, 64);
    const int wave = threadIdx.x >> 6;
    __syncthreads();  // lds may still be read from a previous call
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int j = 0; j < N; ++j) lds[wave * N + j] = x[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < N; ++j) {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < NTH / 64; ++k) s += lds[k * N + j];
        x[j] = s;
    }
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

// The new Theta of one group of four as bf16 (round to nearest even), for the broadcast copy.
__device__ __forceinline__ u32x2 pack_bf16(const float (&t4)[4])
{
    const u32x2 p = {bf16_rne(t4[0]) | (bf16_rne(t4[1]) << 16),
                     bf16_rne(t4[2]) | (bf16_rne(t4[3]) << 16)};
    return p;
}

// Byte offset of element e in a learner's array (4-bit codes: two elements per byte, e even).
template <typename L>
__device__ __forceinline__ uint64_t learner_offset(uint64_t e)
{
    return IsQ4<L>::value ? e / 2 : e * sizeof(typename L::elem);
}

// Number of the scale block that holds element e (4-bit outer gradients).
__device__ __forceinline__ uint64_t q4_block_of(uint64_t e, uint32_t block_len, uint32_t block_shift)
{
    return block_shift != 0xffffffffu ? e >> block_shift : e / block_len;
}

// Walks the chunk: F(d[MQ], theta, v, element index within the chunk, is the first argument
// pack a vector of 4).  VEC path: groups of four per lane; else element-wise.  d is the outer
// gradient: Theta - theta_j, or, for 4-bit outer gradients, scale * code (Theta is then loaded
// only where v is: the reducing sweeps of that kind read neither).
template <typename L, int MQ, int NT, typename F4, typename F1>
__device__ __forceinline__ void sweep_chunk(const DdlRdaArgs& a, uint64_t begin, uint64_t end,
                                            bool need_v, F4&& f4, F1&& f1)
{
    typedef typename L::elem elem;
    constexpr bool Q4 = IsQ4<L>::value;
    const bool need_t = !Q4 || need_v;
    const uint32_t len = (uint32_t)(end - begin);
    const uint64_t th = a.theta + begin * 4, vv = a.v + begin * 4;
    uint64_t lp[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) lp[j] = a.learner[j] + learner_offset<L>(begin);
    uint32_t done = 0;
    if (a.vec_ok) {
        const uint32_t nvec = len / 4;
        for (uint32_t g = threadIdx.x; g < nvec; g += DDL_BLOCK) {
            typename L::raw raw[MQ];
#pragma unroll
            for (int j = 0; j < MQ; ++j) raw[j] = ld<typename L::raw, NT>(lp[j], g);
            float scl[MQ];
            if constexpr (Q4) {  // a group of four lies in one block (block_len % 4 == 0)
                const uint64_t blk = q4_block_of(begin + 4ull * g, a.block_len, a.block_shift);
#pragma unroll
                for (int j = 0; j < MQ; ++j)
                    scl[j] = reinterpret_cast<const DDL_GLOBAL float*>(a.scales[j])[blk];
            }
            f32x4 T = {0.0f, 0.0f, 0.0f, 0.0f};
            if (need_t) T = ld<f32x4, NT>(th, g);
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
                for (int j = 0; j < MQ; ++j) {
                    if constexpr (Q4)
                        d[k][j] = scl[j] * x[j][k];
                    else
                        d[k][j] = t4[k] - x[j][k];
                }
            f4(d, T, V, g);
        }
        done = nvec * 4;
    }
    for (uint32_t e = done + threadIdx.x; e < len; e += DDL_BLOCK) {
        float t = 0.0f;
        if (need_t) t = *(reinterpret_cast<const DDL_GLOBAL float*>(th) + e);
        float v = 0.0f;
        if (need_v) v = *(reinterpret_cast<const DDL_GLOBAL float*>(vv) + e);
        float d[MQ];
        if constexpr (Q4) {  // by absolute element number: the chunk may start at an odd one
            const uint64_t i = begin + e;
            const uint64_t blk = q4_block_of(i, a.block_len, a.block_shift);
#pragma unroll
            for (int j = 0; j < MQ; ++j) {
                const uint32_t byte = reinterpret_cast<const DDL_GLOBAL uint8_t*>(a.learner[j])[i >> 1];
                d[j] = reinterpret_cast<const DDL_GLOBAL float*>(a.scales[j])[blk] *
                       LearnerQ4::nibble(byte, (int)(i & 1));
            }
        } else {
#pragma unroll
            for (int j = 0; j < MQ; ++j)
                d[j] = t - L::widen1(*(reinterpret_cast<const DDL_GLOBAL elem*>(lp[j]) + e));
        }
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

template <int MQ>
__device__ __forceinline__ float direction(const float (&d)[MQ], const float (&c)[MQ])
{
    float u = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) u = fmaf(c[j], d[j], u);
    return u;
}

// Contributing learners up to which the first sweep builds the Gram matrix (register budget
// of the accumulators: Mq (Mq + 1) / 2 of them), and the cancellation it is trusted down to.
constexpr int kGramMaxLearners = 11;
constexpr double kGramTrust = 4e-3;
constexpr int gram_size(int mq) { return mq * (mq + 1) / 2; }

// Sums N values over a wavefront so that every total ends up in ONE lane: at each of the six
// steps a lane keeps one half of its values and hands the other half to its partner, which
// costs about 4 N operations in all where a butterfly per value costs 12 N.  Afterwards slot i
// (i < slots) of lane l holds the total of entry index[i] (valid if index[i] < N).
template <int N>
struct WaveScatterSum {
    static constexpr int half(int n) { return (n + 1) / 2; }
    static constexpr int slots = half(half(half(half(half(half(N))))));
    template <int CNT, int OFF>
    static __device__ __forceinline__ void step(float (&x)[N], int (&index)[slots], bool)
    {
        if constexpr (OFF >= 1) {
            constexpr int H = half(CNT);
            const bool up = (threadIdx.x & OFF) != 0;
#pragma unroll
            for (int i = 0; i < H; ++i) {
                const float lo = x[i];
                const float hi = i + H < CNT ? x[i + H] : 0.0f;
                const float got = __shfl_xor(up ? lo : hi, OFF, 64);
                x[i] = (up ? hi : lo) + got;
            }
            step<H, OFF / 2>(x, index, up);
            // entries of the upper half sit H further up in the previous numbering
#pragma unroll
            for (int i = 0; i < slots; ++i)
                if (up) index[i] = index[i] < H && index[i] + H < CNT ? index[i] + H : N;
        }
    }
    static __device__ __forceinline__ void run(float (&x)[N], int (&index)[slots])
    {
#pragma unroll
        for (int i = 0; i < slots; ++i) index[i] = i;
        step<N, 32>(x, index, false);
    }
};

// Sweep 1 of the Gram form: per chunk, the sums of d_j d_k for j <= k, row-major upper triangle.
template <typename L, int MQ>
__device__ __forceinline__ void gram_body(const DdlRdaArgs& a, uint32_t chunk)
{
    constexpr int P = gram_size(MQ);
    typedef WaveScatterSum<P> Sum;
    __shared__ float lds[DDL_BLOCK / 64][P];
    uint64_t begin, end;
    uint32_t group;
    chunk_range(a, chunk, begin, end, group);
    float acc[P];
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p] = 0.0f;
    auto add = [&](const float (&d)[MQ]) {
        int p = 0;
#pragma unroll
        for (int j = 0; j < MQ; ++j)
#pragma unroll
            for (int k = j; k < MQ; ++k, ++p) acc[p] = fmaf(d[j], d[k], acc[p]);
    };
    sweep_chunk<L, MQ, DDL_RDA_GRAM_LOAD>(
        a, begin, end, false,
        [&](const float (&d)[4][MQ], const f32x4&, const f32x4&, uint32_t) {
#pragma unroll
            for (int k = 0; k < 4; ++k) add(d[k]);
        },
        [&](const float (&d)[MQ], float, float, uint32_t) { add(d); });
    int index[Sum::slots];
    Sum::run(acc, index);
#pragma unroll
    for (int i = 0; i < Sum::slots; ++i)
        if (index[i] < P) lds[threadIdx.x >> 6][index[i]] = acc[i];
    __syncthreads();
    float* out = reinterpret_cast<float*>(a.partial1) + (size_t)chunk * P;
    for (int p = threadIdx.x; p < P; p += DDL_BLOCK) {
        float s = 0.0f;
#pragma unroll
        for (int wv = 0; wv < DDL_BLOCK / 64; ++wv) s += lds[wv][p];  // waves in a fixed order
        out[p] = s;
    }
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_gram_kernel(const DdlRdaArgs a)
{
    gram_body<L, MQ>(a, blockIdx.x);
}

// One workgroup per group: the Gram matrix from the chunk partials (each thread sums its own
// chunks in ascending order in double, then lanes by butterfly, then the waves in sequence),
// and from it the coefficients c_j = w_j / N_j, the mean norm R and scale = R / sqrt(c' G c).
// Where c' G c cannot be trusted (the outer gradients nearly cancel) this workgroup walks its
// group once more and sums the squares of the mean direction itself: slow, since it is one
// workgroup for the whole group, but it concerns only such groups and keeps the common case
// at three launches (Gram sweep, this kernel, apply).
template <typename L, int MQ>
__device__ __forceinline__ void gram_reduce_body(const DdlRdaArgs& a, uint32_t r)
{
    constexpr int P = gram_size(MQ);
    __shared__ double lds[DDL_BLOCK / 64][P];
    __shared__ float coef_lds[MQ];
    __shared__ float verdict[2];  // scale (< 0: not trusted), R
    const float* p1 = reinterpret_cast<const float*>(a.partial1) + (size_t)r * a.chunks_per_group * P;
    double g[P];
#pragma unroll
    for (int p = 0; p < P; ++p) g[p] = 0.0;
    for (uint32_t c = threadIdx.x; c < a.chunks_per_group; c += DDL_BLOCK) {
        const float* row = p1 + (size_t)c * P;
#pragma unroll
        for (int p = 0; p < P; ++p) g[p] += (double)row[p];
    }
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) g[p] += __shfl_xor(g[p], off, 64);
        if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6][p] = g[p];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            double s = 0.0;
#pragma unroll
            for (int wv = 0; wv < DDL_BLOCK / 64; ++wv) s += lds[wv][p];
            g[p] = s;
        }
        double c[MQ];
        double R = 0.0;
        {
            int p = 0;
#pragma unroll
            for (int j = 0; j < MQ; ++j) {
                const double N = sqrt(g[p]);  // the diagonal entry G_jj
                R += (double)a.w[j] * N;
                c[j] = N > 0.0 ? (double)a.w[j] / N : 0.0;
                p += MQ - j;
            }
        }
        double q = 0.0, mass = 0.0;  // c' G c and the sum of the magnitudes of its terms
        {
            int p = 0;
#pragma unroll
            for (int j = 0; j < MQ; ++j)
#pragma unroll
                for (int k = j; k < MQ; ++k, ++p) {
                    const double term = (j == k ? 1.0 : 2.0) * c[j] * c[k] * g[p];
                    q += term;
                    mass += fabs(term);
                }
        }
        float* coef = reinterpret_cast<float*>(a.coef) + (size_t)r * MQ;
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            coef[j] = (float)c[j];
            coef_lds[j] = (float)c[j];
        }
        reinterpret_cast<float*>(a.mean_norm)[r] = (float)R;
        float scale = 0.0f;                          // no direction at all: Delta = 0
        if (mass > 0.0) scale = q >= kGramTrust * mass ? (float)(R / sqrt(q)) : -1.0f;
        verdict[0] = scale;
        verdict[1] = (float)R;
        if (!(scale < 0.0f)) reinterpret_cast<float*>(a.scale)[r] = scale;
    }
    __syncthreads();
    if (!(verdict[0] < 0.0f)) return;  // block-uniform

    // The direct form for this group: ||sum_j c_j d_j||^2 summed from the data.
    float c[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) c[j] = coef_lds[j];
    const uint64_t g0 = (uint64_t)r * a.group_len;
    const uint64_t g1 = a.n - g0 < a.group_len ? a.n : g0 + a.group_len;
    double uu = 0.0;  // per thread over the whole group: double keeps long groups exact enough
    for (uint64_t begin = g0; begin < g1; begin += DDL_RDA_CHUNK) {
        const uint64_t end = begin + DDL_RDA_CHUNK < g1 ? begin + DDL_RDA_CHUNK : g1;
        float part = 0.0f;
        sweep_chunk<L, MQ, false>(
            a, begin, end, false,
            [&](const float (&d)[4][MQ], const f32x4&, const f32x4&, uint32_t) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float u = direction<MQ>(d[k], c);
                    part = fmaf(u, u, part);
                }
            },
            [&](const float (&d)[MQ], float, float, uint32_t) {
                const float u = direction<MQ>(d, c);
                part = fmaf(u, u, part);
            });
        uu += (double)part;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) uu += __shfl_xor(uu, off, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6][0] = uu;
    __syncthreads();
    if (threadIdx.x == 0) {
        double U2 = 0.0;
#pragma unroll
        for (int wv = 0; wv < DDL_BLOCK / 64; ++wv) U2 += lds[wv][0];
        const double U = sqrt(U2);
        reinterpret_cast<float*>(a.scale)[r] = U > 0.0 ? (float)((double)verdict[1] / U) : 0.0f;
    }
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_gram_reduce_kernel(const DdlRdaArgs a)
{
    gram_reduce_body<L, MQ>(a, blockIdx.x);
}

// One workgroup per group: norms from the chunk partials (in double, fixed order), then the
// direction coefficients w_j / N_j and the mean norm.
__global__ void __launch_bounds__(DDL_BLOCK) rda_norms_kernel(const DdlRdaArgs a, int Mq)
{
    __shared__ double lds[DDL_BLOCK];
    const uint32_t r = blockIdx.x;
    const float* p1 =
        reinterpret_cast<const float*>(a.partial1) + (size_t)r * a.chunks_per_group * Mq;
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

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_dirsq_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[DDL_BLOCK / 64];
    uint64_t begin, end;
    uint32_t group;
    chunk_range(a, blockIdx.x, begin, end, group);
    float c[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j)
        c[j] = reinterpret_cast<const float*>(a.coef)[(size_t)group * MQ + j];
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

// The apply sweep of the long-group path runs in the merge kernel's shape: one tile per
// workgroup (a chunk in DDL_RDA_CHUNK / DDL_TILE slices), workgroups rotated within groups of 64.
constexpr uint32_t kLongApplyRotate = 64;
constexpr uint32_t kLongApplyPieceShift = 3;
static_assert((DDL_TILE << kLongApplyPieceShift) == DDL_RDA_CHUNK, "a slice is one tile");

// piece, pieces: the workgroup takes only the piece-th of `pieces` equal slices of the chunk.
template <typename L, int MQ>
__device__ __forceinline__ void apply_body(const DdlRdaArgs& a, uint32_t chunk, uint32_t piece = 0,
                                           uint32_t pieces = 1)
{
    uint64_t begin, end;
    uint32_t group;
    chunk_range(a, chunk, begin, end, group);
    if (pieces > 1) {
        const uint32_t len = DDL_RDA_CHUNK / pieces;
        begin += (uint64_t)piece * len;
        if (begin >= end) return;
        if (begin + len < end) end = begin + len;
    }
    float c[MQ];
    const float scale = reinterpret_cast<const float*>(a.scale)[group];
#pragma unroll
    for (int j = 0; j < MQ; ++j)
        c[j] = reinterpret_cast<const float*>(a.coef)[(size_t)group * MQ + j] * scale;
    const float lr = a.lr, mu = a.mu;
    const uint64_t th = a.theta + begin * 4, vv = a.v + begin * 4;
    const uint64_t tb = a.theta_bf16 ? a.theta_bf16 + begin * 2 : 0;
    sweep_chunk<L, MQ, DDL_NT_LOAD>(
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
            if (tb) st<u32x2>(tb, g, pack_bf16(t4));
        },
        [&](const float (&d)[MQ], float t, float v, uint32_t e) {
            const float delta = direction<MQ>(d, c);
            const float v_new = fmaf(mu, v, delta);
            const float t_new = fmaf(-lr, fmaf(mu, v_new, delta), t);
            *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = t_new;
            *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v_new;
            if (tb) *(reinterpret_cast<DDL_GLOBAL uint16_t*>(tb) + e) = (uint16_t)bf16_rne(t_new);
        });
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_apply_kernel(const DdlRdaArgs a)
{
    const uint32_t b = rotate_tile(blockIdx.x, gridDim.x, kLongApplyRotate);
    apply_body<L, MQ>(a, b >> a.piece_shift, b & ((1u << a.piece_shift) - 1), 1u << a.piece_shift);
}

// The long-group path for ALL such tensors of a fragment at once (through a plan): the three
// kernels above with the tensor looked up per workgroup.  What is fixed per tensor sits in a
// device table made when the groups are set (DdlRdaLongRef: descriptor, chunk and group
// numbering within the fragment's launches, where its partial sums live in the workspace);
// what changes per sync travels in the kernel arguments.
struct DdlRdaLongRef {
    uint32_t seg;               // descriptor index in the plan's table
    uint32_t chunk_begin;       // first chunk of this tensor within the sweep launches
    uint32_t group_begin;       // first group of this tensor within the reduce launch
    uint32_t chunks_per_group;
    uint64_t group_len;         // clamped to n
    uint64_t off_partial1, off_coef, off_mean, off_scale;  // bytes into the workspace
    uint32_t vec_all;           // every base 16-byte aligned and group_len a multiple of four
    uint32_t pad;
};

struct DdlRdaLongArgs {
    const DdlSegDesc* segs;
    const DdlRdaLongRef* refs;  // the fragment's entries
    uint32_t num_refs;
    uint32_t by_group;          // 0: workgroups count chunks, 1: groups
    uint32_t base;              // number of this grid's first workgroup (long sweeps go in parts)
    uint32_t piece_shift;       // apply sweep: a workgroup takes one of 1 << piece_shift slices
                                // of a chunk, and the grid's workgroups are rotated like tiles
    uint64_t workspace;
    float lr, mu;
    float w[DDL_MAXL];          // normalised weights of the contributing learners, compacted
    uint8_t idx[DDL_MAXL];      // learner index of compacted entry j
    // 4-bit outer gradients only: the table parallel to segs, and the block length of the scales
    const DdlQ4Desc* q4;
    uint32_t block_len, block_shift;
};

// The tensor that holds chunk (or group) b of the launch, as the arguments the one-tensor
// bodies take; `local` is b's number within that tensor.
template <typename L, int MQ>
__device__ __forceinline__ void long_locate(const DdlRdaLongArgs& m, uint32_t b, DdlRdaArgs& a,
                                            uint32_t& local)
{
    const DDL_CONST DdlRdaLongRef* refs =
        reinterpret_cast<const DDL_CONST DdlRdaLongRef*>(reinterpret_cast<uint64_t>(m.refs));
    uint32_t lo = 0, hi = m.num_refs - 1;  // last entry whose begin <= b
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        const uint32_t begin = m.by_group ? refs[mid].group_begin : refs[mid].chunk_begin;
        if (begin <= b) lo = mid; else hi = mid - 1;
    }
    const DDL_CONST DdlRdaLongRef* ref = refs + lo;
    const DDL_CONST DdlSegDesc* sp =
        reinterpret_cast<const DDL_CONST DdlSegDesc*>(reinterpret_cast<uint64_t>(m.segs)) + ref->seg;
    local = b - (m.by_group ? ref->group_begin : ref->chunk_begin);
    a.theta = uniform(reinterpret_cast<uint64_t>(sp->theta));
    a.v = uniform(reinterpret_cast<uint64_t>(sp->v));
    a.theta_bf16 = uniform(reinterpret_cast<uint64_t>(sp->theta_bf16));
    if constexpr (IsQ4<L>::value) {
        const DDL_CONST DdlQ4Desc* qp =
            reinterpret_cast<const DDL_CONST DdlQ4Desc*>(reinterpret_cast<uint64_t>(m.q4)) +
            ref->seg;
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            a.learner[j] = uniform(reinterpret_cast<uint64_t>(qp->codes[m.idx[j]]));
            a.scales[j] = uniform(reinterpret_cast<uint64_t>(qp->scales[m.idx[j]]));
            a.w[j] = m.w[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            a.learner[j] = uniform(reinterpret_cast<uint64_t>(sp->learner[m.idx[j]]));
            a.w[j] = m.w[j];
        }
    }
    a.block_len = m.block_len;
    a.block_shift = m.block_shift;
    a.n = sp->n;
    a.group_len = ref->group_len;
    a.chunks_per_group = ref->chunks_per_group;
    a.vec_ok = ref->vec_all;
    a.lr = m.lr;
    a.mu = m.mu;
    a.partial1 = m.workspace + ref->off_partial1;
    a.coef = m.workspace + ref->off_coef;
    a.mean_norm = m.workspace + ref->off_mean;
    a.partial2 = 0;
    a.scale = m.workspace + ref->off_scale;
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_long_gram_kernel(const DdlRdaLongArgs m)
{
    DdlRdaArgs a;
    uint32_t chunk;
    long_locate<L, MQ>(m, m.base + blockIdx.x, a, chunk);
    gram_body<L, MQ>(a, chunk);
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_long_reduce_kernel(const DdlRdaLongArgs m)
{
    DdlRdaArgs a;
    uint32_t group;
    long_locate<L, MQ>(m, m.base + blockIdx.x, a, group);
    gram_reduce_body<L, MQ>(a, group);
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_long_apply_kernel(const DdlRdaLongArgs m)
{
    DdlRdaArgs a;
    uint32_t chunk;
    const uint32_t b = m.base + rotate_tile(blockIdx.x, gridDim.x, kLongApplyRotate);
    long_locate<L, MQ>(m, b >> m.piece_shift, a, chunk);
    apply_body<L, MQ>(a, chunk, b & ((1u << m.piece_shift) - 1), 1u << m.piece_shift);
}

// Launch shape (a): one workgroup makes all three sweeps over its own group.
template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) rda_group_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[DDL_BLOCK / 64 * MQ];
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
    block_sum_all<DDL_BLOCK, MQ>(ss, lds);
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const float N = sqrtf(ss[j]);
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
    float usum[1] = {uu};
    block_sum_all<DDL_BLOCK, 1>(usum, lds);
    const float U = sqrtf(usum[0]);
    const float scale = U > 0.0f ? R / U : 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) c[j] *= scale;

    // sweep 3: Delta = scale * u, outer step
    const float lr = a.lr, mu = a.mu;
    for (uint64_t begin = g0; begin < g1; begin += DDL_RDA_CHUNK) {
        const uint64_t end = begin + DDL_RDA_CHUNK < g1 ? begin + DDL_RDA_CHUNK : g1;
        const uint64_t th = a.theta + begin * 4, vv = a.v + begin * 4;
        const uint64_t tb = a.theta_bf16 ? a.theta_bf16 + begin * 2 : 0;
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
                if (tb) st<u32x2>(tb, g, pack_bf16(t4));
            },
            [&](const float (&d)[MQ], float t, float v, uint32_t e) {
                const float delta = direction<MQ>(d, c);
                const float v_new = fmaf(mu, v, delta);
                const float t_new = fmaf(-lr, fmaf(mu, v_new, delta), t);
                *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = t_new;
                *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v_new;
                if (tb)
                    *(reinterpret_cast<DDL_GLOBAL uint16_t*>(tb) + e) = (uint16_t)bf16_rne(t_new);
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
__device__ __forceinline__ void launder(uint32_t& r) { asm volatile("" : "+v"(r)); }

// Whether the row kernels load v with everything else (one memory round trip fewer per row,
// four more registers per group held through the sweeps) or only before the last sweep.
template <typename L>
constexpr bool row_loads_v_early()
{
    return DDL_RDA_V_EARLY || (IsQ4<L>::value && DDL_RDA_Q4_V_EARLY);
}

// What a lane of the row kernel keeps of a learner's four elements: the packed values as
// loaded, or -- 4-bit outer gradients -- the four codes in one register (their block's scale
// sits in a second one).
template <typename L> struct RowRaw { typedef typename L::raw type; };
template <> struct RowRaw<LearnerQ4> { typedef uint32_t type; };

// Where a row's learner data lies beyond lp: 4-bit outer gradients only.
template <int MQ>
struct RowScales {
    uint64_t sc[MQ];       // the tensor's block scales per contributing learner
    uint64_t first;        // element number of the row's first element within the tensor
    uint32_t block_len, block_shift;
};

// Launch shape (a'), for groups of at most K * 4 * NTH elements on the aligned path: the
// workgroup loads its whole group ONCE into registers (learner values stay packed as loaded)
// and makes the three sweeps over the registers.  HBM traffic equals that of direct averaging.
// th, vv, tb, lp: addresses of the group's first element (tb: the optional bf16 copy of the new
// Theta, 0 if none); nvec: its length in groups of four.
template <typename L, int MQ, int K, int NTH>
__device__ __forceinline__ void rda_row_body(uint64_t th, uint64_t vv, uint64_t tb,
                                             const uint64_t (&lp)[MQ], const RowScales<MQ>& rs,
                                             const float (&w)[MQ], uint32_t nvec, float lr,
                                             float mu, float* lds /* NTH / 64 * MQ floats */)
{
    constexpr bool Q4 = IsQ4<L>::value;
    typedef typename RowRaw<L>::type raw_t;
    raw_t raw[K][MQ];
    float scl[Q4 ? K : 1][MQ];  // 4-bit outer gradients: the block scale of each group of four
    f32x4 T[K];
    f32x4 V[K];
    constexpr bool V_EARLY = row_loads_v_early<L>();
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t g = threadIdx.x + u * NTH;
        if constexpr (V_EARLY) V[u] = g < nvec ? ld<f32x4, DDL_NT_LOAD>(vv, g) : f32x4(0.0f);
        if (g < nvec) {
#pragma unroll
            for (int j = 0; j < MQ; ++j) raw[u][j] = ld<typename L::raw, DDL_NT_LOAD>(lp[j], g);
            if constexpr (Q4) {
                const uint64_t blk = q4_block_of(rs.first + 4ull * g, rs.block_len, rs.block_shift);
#pragma unroll
                for (int j = 0; j < MQ; ++j)
                    scl[u][j] = reinterpret_cast<const DDL_GLOBAL float*>(rs.sc[j])[blk];
            }
            T[u] = ld<f32x4, DDL_NT_LOAD>(th, g);
        } else {  // lanes past the end of the group hold a zero outer gradient
#pragma unroll
            for (int j = 0; j < MQ; ++j) raw[u][j] = raw_t(0);
            if constexpr (Q4) {
#pragma unroll
                for (int j = 0; j < MQ; ++j) scl[u][j] = 0.0f;
            }
            T[u] = f32x4(0.0f);
        }
    }
    (void)scl;

    // outer gradients of group u, element k, recomputed from the packed registers on demand
    auto diffs = [&](int u, float (&d)[4][MQ]) {
        if constexpr (Q4) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < MQ; ++j)
                    d[k][j] = scl[u][j] * LearnerQ4::nibble(raw[u][j], k);
        } else {
            float x[MQ][4];
#pragma unroll
            for (int j = 0; j < MQ; ++j) L::widen(raw[u][j], x[j]);
            const float t4[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < MQ; ++j) d[k][j] = t4[k] - x[j][k];
        }
    };

    // Sweep 1: the learners' norms over the group.  (DDL_RDA_DIAG_NO_SWEEPS is a measurement
    // build that leaves both reductions out -- Delta = sum_j w_j d_j, i.e. direct averaging in
    // this kernel's shape -- to show what the row-per-workgroup structure alone costs.)
    float c[MQ];
    float scale = 1.0f;
#ifdef DDL_RDA_DIAG_NO_SWEEPS
#pragma unroll
    for (int j = 0; j < MQ; ++j) c[j] = w[j];
    (void)lds;
#else
    float ss[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) ss[j] = 0.0f;
#pragma unroll
    for (int u = 0; u < K; ++u) {
        if constexpr (Q4) {
            // sum of (scale * code)^2 over the four codes = scale^2 times the sum of the squared
            // codes, which one 4-bit dot-product instruction gives exactly (the upper four
            // nibbles of the register are zero)
#pragma unroll
            for (int j = 0; j < MQ; ++j) {
                const int sq = __builtin_amdgcn_sdot8((int)raw[u][j], (int)raw[u][j], 0, false);
                ss[j] = fmaf(scl[u][j] * scl[u][j], (float)sq, ss[j]);
            }
        } else {
            float d[4][MQ];
            diffs(u, d);
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < MQ; ++j) ss[j] = fmaf(d[k][j], d[k][j], ss[j]);
        }
    }
    float R = 0.0f;
    block_sum_all<NTH, MQ>(ss, lds);
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        const float N = sqrtf(ss[j]);
        R = fmaf(w[j], N, R);
        c[j] = N > 0.0f ? w[j] / N : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < K; ++u)
#pragma unroll
        for (int j = 0; j < MQ; ++j) launder(raw[u][j]);
#endif

    // Sweep 2: the mean direction u = sum_j c_j d_j, kept in registers (the packed learner
    // values are dead from here on, so this costs no extra registers), and its norm.
    f32x4 dir[K];
    float uu = 0.0f;
#pragma unroll
    for (int u = 0; u < K; ++u) {
        float x[4];
        if constexpr (Q4) {  // the block's scale goes into the coefficient, once per group
            float cs[MQ];
#pragma unroll
            for (int j = 0; j < MQ; ++j) cs[j] = c[j] * scl[u][j];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[k] = 0.0f;
#pragma unroll
                for (int j = 0; j < MQ; ++j)
                    x[k] = fmaf(cs[j], LearnerQ4::nibble(raw[u][j], k), x[k]);
            }
        } else {
            float d[4][MQ];
            diffs(u, d);
#pragma unroll
            for (int k = 0; k < 4; ++k) x[k] = direction<MQ>(d[k], c);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) uu = fmaf(x[k], x[k], uu);
        dir[u] = f32x4{x[0], x[1], x[2], x[3]};
    }
#ifndef DDL_RDA_DIAG_NO_SWEEPS
    float usum[1] = {uu};
    block_sum_all<NTH, 1>(usum, lds);
    const float U = sqrtf(usum[0]);
    scale = U > 0.0f ? R / U : 0.0f;
#else
    (void)uu;
#endif

    // Sweep 3: Delta = scale * u, outer step.
    if constexpr (!V_EARLY) {
#pragma unroll
        for (int u = 0; u < K; ++u) {
            const uint32_t g = threadIdx.x + u * NTH;
            V[u] = g < nvec ? ld<f32x4, DDL_NT_LOAD>(vv, g) : f32x4(0.0f);
        }
    }
#pragma unroll
    for (int u = 0; u < K; ++u) {
        const uint32_t g = threadIdx.x + u * NTH;
        float t4[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
        float v4[4] = {V[u].x, V[u].y, V[u].z, V[u].w};
        const float x[4] = {dir[u].x, dir[u].y, dir[u].z, dir[u].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float delta = scale * x[k];
            v4[k] = fmaf(mu, v4[k], delta);
            t4[k] = fmaf(-lr, fmaf(mu, v4[k], delta), t4[k]);
        }
        if (g < nvec) {
            const f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
            const f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
            st<f32x4>(th, g, tn);
            st<f32x4>(vv, g, vn);
            if (tb) st<u32x2>(tb, g, pack_bf16(t4));
        }
    }
}

// One tensor: workgroup b takes group b.
template <typename L, int MQ, int K, int NTH>
__global__ void __launch_bounds__(NTH) rda_row_kernel(const DdlRdaArgs a)
{
    __shared__ float lds[NTH / 64 * MQ];
    const uint64_t g0 = (uint64_t)blockIdx.x * a.group_len;
    const uint64_t g1 = a.n - g0 < a.group_len ? a.n : g0 + a.group_len;
    const uint32_t nvec = (uint32_t)(g1 - g0) / 4;  // the host sends only multiples of four here
    uint64_t lp[MQ];
    float w[MQ];
    RowScales<MQ> rs;
    rs.first = g0;
    rs.block_len = a.block_len;
    rs.block_shift = a.block_shift;
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        lp[j] = a.learner[j] + learner_offset<L>(g0);
        rs.sc[j] = a.scales[j];
        w[j] = a.w[j];
    }
    rda_row_body<L, MQ, K, NTH>(a.theta + g0 * 4, a.v + g0 * 4,
                                a.theta_bf16 ? a.theta_bf16 + g0 * 2 : 0, lp, rs, w, nvec, a.lr,
                                a.mu, lds);
}

// Many tensors of one fragment in one launch: workgroup b takes row b of the concatenation
// of the listed tensors' groups.  The tensor is found through a coarse index (entry i names
// the list entry that holds row i << shift), then the descriptor table gives its addresses;
// all of that is block-uniform and read with scalar loads from constant address space.
struct DdlRdaRowRef {
    uint32_t seg;        // descriptor index in the plan's table
    uint32_t row_begin;  // first row of this tensor within the launch
    uint32_t group_len;  // elements per group: a multiple of four
    uint32_t pad;
};

struct DdlRdaRowsArgs {
    const DdlSegDesc* segs;
    const DdlRdaRowRef* refs;  // first list entry of this launch
    const uint32_t* coarse;    // first coarse entry of this launch
    uint32_t coarse_shift;
    uint32_t row_base;      // first row this grid covers (a long launch goes out in parts)
    float lr, mu;
    float w[DDL_MAXL];      // normalised weights of the contributing learners, compacted
    uint8_t idx[DDL_MAXL];  // learner index of compacted entry j
    // 4-bit outer gradients only: the table parallel to segs, and the block length of the scales
    const DdlQ4Desc* q4;
    uint32_t block_len, block_shift;
};

template <typename L, int MQ, int K, int NTH>
__global__ void __launch_bounds__(NTH) rda_rows_kernel(const DdlRdaRowsArgs a)
{
    __shared__ float lds[NTH / 64 * MQ];
    const uint32_t r = a.row_base + blockIdx.x;
    const DDL_CONST DdlRdaRowRef* refs =
        reinterpret_cast<const DDL_CONST DdlRdaRowRef*>(reinterpret_cast<uint64_t>(a.refs));
    const DDL_CONST uint32_t* coarse =
        reinterpret_cast<const DDL_CONST uint32_t*>(reinterpret_cast<uint64_t>(a.coarse)) +
        (r >> a.coarse_shift);
    uint32_t lo = coarse[0], hi = coarse[1];  // last list entry whose row_begin <= r
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (refs[mid].row_begin <= r) lo = mid; else hi = mid - 1;
    }
    const DDL_CONST DdlRdaRowRef* ref = refs + lo;
    const DDL_CONST DdlSegDesc* sp =
        reinterpret_cast<const DDL_CONST DdlSegDesc*>(reinterpret_cast<uint64_t>(a.segs)) +
        ref->seg;
    const uint64_t glen = ref->group_len;
    const uint64_t n = sp->n;
    const uint64_t g0 = (uint64_t)(r - ref->row_begin) * glen;
    const uint64_t g1 = n - g0 < glen ? n : g0 + glen;
    const uint32_t nvec = uniform((uint32_t)(g1 - g0) / 4);
    const uint64_t th = uniform(reinterpret_cast<uint64_t>(sp->theta) + g0 * 4);
    const uint64_t vv = uniform(reinterpret_cast<uint64_t>(sp->v) + g0 * 4);
    const uint64_t tb0 = reinterpret_cast<uint64_t>(sp->theta_bf16);
    const uint64_t tb = uniform(tb0 ? tb0 + g0 * 2 : 0);
    uint64_t lp[MQ];
    float w[MQ];
    RowScales<MQ> rs;
    rs.first = g0;
    rs.block_len = a.block_len;
    rs.block_shift = a.block_shift;
    if constexpr (IsQ4<L>::value) {
        const DDL_CONST DdlQ4Desc* qp =
            reinterpret_cast<const DDL_CONST DdlQ4Desc*>(reinterpret_cast<uint64_t>(a.q4)) +
            ref->seg;
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            lp[j] = uniform(reinterpret_cast<uint64_t>(qp->codes[a.idx[j]]) + g0 / 2);
            rs.sc[j] = uniform(reinterpret_cast<uint64_t>(qp->scales[a.idx[j]]));
            w[j] = a.w[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            lp[j] = uniform(reinterpret_cast<uint64_t>(sp->learner[a.idx[j]]) +
                            learner_offset<L>(g0));
            rs.sc[j] = 0;
            w[j] = a.w[j];
        }
    }
    rda_row_body<L, MQ, K, NTH>(th, vv, tb, lp, rs, w, nvec, a.lr, a.mu, lds);
}

// Registers the row kernel keeps per lane: K groups of (packed learners + Theta + v), plus
// about six per learner while a sweep runs (the four differences of a group, a sum, a
// coefficient).  A 1024-thread workgroup leaves each lane 128 registers: the learners' packed
// words per group-of-four slot may then take 12 (K = 4), 16 (K = 2) or 24 (K = 1) registers --
// limits found by building (the build fails on any spill); smaller workgroups have 256 and more.
template <typename L, int MQ, int K, int NTH>
constexpr bool row_kernel_fits()
{
    // packed learner words per slot (4-bit outer gradients: the codes and the block's scale)
    const int words = (IsQ4<L>::value ? 2 : (int)(sizeof(typename L::raw) / 4)) * MQ;
    if (NTH > 512) return words <= (K >= 4 ? 12 : K == 2 ? 16 : 24);
    return K * (words + 8) <= (row_loads_v_early<L>() ? 184 : 192);  // v held through the sweeps
}

typedef void (*rda_fn)(const DdlRdaArgs);
typedef void (*rda_rows_fn)(const DdlRdaRowsArgs);
typedef void (*rda_long_fn)(const DdlRdaLongArgs);

// The register-resident shapes, smallest first: X(class, K groups of four per lane, workgroup
// size, K and workgroup size of the second choice); a class holds groups of up to
// K * 4 * threads elements.  The second choice, of the same capacity, is taken when the first
// does not fit the registers for this many learners (it keeps fewer groups per lane).  The
// 192-thread class is there for rows of 1025 .. 1536 elements (an expert matrix of width 1408):
// on 256 threads a third of the lanes would idle through both sweeps (moe: +4 points of HBM
// peak for bf16 learners, +7 for 4-bit outer gradients).
#ifndef DDL_RDA_ROW_CLASSES
#define DDL_RDA_ROW_CLASSES(X) \
    X(0, 1, 256, 1, 256) X(1, 2, 192, 2, 192) X(2, 2, 256, 1, 512) X(3, 4, 256, 2, 512) \
    X(4, 4, 512, 8, 256) X(5, 8, 512, 4, 1024)
#endif
struct RowClass {
    uint32_t max_len;
};
#define DDL_X(c, k, nth, k2, nth2) {k * 4 * nth},
constexpr RowClass kRowClass[] = {DDL_RDA_ROW_CLASSES(DDL_X)};
#undef DDL_X
#define DDL_X(c, k, nth, k2, nth2) static_assert(k * nth == k2 * nth2, "same capacity");
DDL_RDA_ROW_CLASSES(DDL_X)
#undef DDL_X
constexpr int kNumRowClasses = (int)(sizeof(kRowClass) / sizeof(kRowClass[0]));

// Smallest class that holds a group of `len` elements; kNumRowClasses if none does.
int row_class_for(uint64_t len)
{
    for (int c = 0; c < kNumRowClasses; ++c)
        if (len <= kRowClass[c].max_len) return c;
    return kNumRowClasses;
}

template <typename L, int MQ, int K, int NTH, int K2, int NTH2>
void row_kernels_or_null(rda_fn& one, rda_rows_fn& many, uint32_t& threads)
{
    one = nullptr;
    many = nullptr;
    threads = 0;
    if constexpr (row_kernel_fits<L, MQ, K, NTH>()) {
        one = rda_row_kernel<L, MQ, K, NTH>;
        many = rda_rows_kernel<L, MQ, K, NTH>;
        threads = NTH;
    } else if constexpr (row_kernel_fits<L, MQ, K2, NTH2>()) {
        one = rda_row_kernel<L, MQ, K2, NTH2>;
        many = rda_rows_kernel<L, MQ, K2, NTH2>;
        threads = NTH2;
    }
}

// The row kernels of class `cls` (one tensor / many tensors) and their workgroup size, or null
// if neither choice fits the registers for this learner type and count.
template <typename L, int MQ>
void pick_row(int cls, rda_fn& one, rda_rows_fn& many, uint32_t& threads)
{
    one = nullptr;
    many = nullptr;
    threads = 0;
    switch (cls) {
#define DDL_X(c, k, nth, k2, nth2) \
    case c: row_kernels_or_null<L, MQ, k, nth, k2, nth2>(one, many, threads); break;
        DDL_RDA_ROW_CLASSES(DDL_X)
#undef DDL_X
        default: break;
    }
}

struct Kernels {
    rda_fn sumsq = nullptr, dirsq = nullptr, apply = nullptr, group = nullptr, row = nullptr;
    rda_fn gram = nullptr, gram_reduce = nullptr;  // null beyond kGramMaxLearners
    rda_long_fn long_gram = nullptr, long_reduce = nullptr, long_apply = nullptr;  // likewise
    rda_rows_fn rows = nullptr;
    uint32_t row_threads = 0;  // workgroup size of row / rows
};

template <typename L>
void pick(int Mq, int cls, Kernels& k)
{
    switch (Mq) {
#define DDL_CASE(q)                              \
    case q:                                      \
        k.sumsq = rda_sumsq_kernel<L, q>;        \
        k.dirsq = rda_dirsq_kernel<L, q>;        \
        k.apply = rda_apply_kernel<L, q>;        \
        k.group = rda_group_kernel<L, q>;        \
        if constexpr (q <= kGramMaxLearners) {   \
            k.gram = rda_gram_kernel<L, q>;      \
            k.gram_reduce = rda_gram_reduce_kernel<L, q>; \
            k.long_gram = rda_long_gram_kernel<L, q>;     \
            k.long_reduce = rda_long_reduce_kernel<L, q>; \
            k.long_apply = rda_long_apply_kernel<L, q>;   \
        }                                        \
        pick_row<L, q>(cls, k.row, k.rows, k.row_threads); \
        break;
        DDL_CASE(1) DDL_CASE(2) DDL_CASE(3) DDL_CASE(4) DDL_CASE(5) DDL_CASE(6) DDL_CASE(7)
        DDL_CASE(8) DDL_CASE(9) DDL_CASE(10) DDL_CASE(11) DDL_CASE(12) DDL_CASE(13)
        DDL_CASE(14) DDL_CASE(15) DDL_CASE(16)
#undef DDL_CASE
    }
}

// src: what the learners' data is -- 0 fp32, 1 bf16 copies of the tensor (values of ddl_dtype),
// DDL_SRC_Q4: their outer gradients as 4-bit codes with block scales.
void pick(int src, int Mq, int cls, Kernels& k)
{
    if (src == (int)DDL_F32)
        pick<LearnerF32>(Mq, cls, k);
    else if (src == (int)DDL_BF16)
        pick<LearnerBF16>(Mq, cls, k);
    else
        pick<LearnerQ4>(Mq, cls, k);
}

// Bytes per learner element as the launch-shape choices of the merge kernels count them.
int src_elem_bytes(int src) { return src == DDL_SRC_Q4 ? 0 : src == (int)DDL_BF16 ? 2 : 4; }

struct Geometry {
    uint64_t groups, chunks_per_group, chunks;
    size_t off_partial1, off_coef, off_mean, off_partial2, off_scale, bytes;
};

// Floats per chunk that sweep 1 leaves behind, at most, for up to Mq contributing learners.
int partial_width(int Mq)
{
    return Mq <= kGramMaxLearners ? gram_size(Mq) : std::max(Mq, gram_size(kGramMaxLearners));
}

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
    g.off_partial1 = take(g.chunks * (uint64_t)partial_width(Mq));
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

// Unused dynamic LDS that caps the resident workgroups per compute unit (option
// rda_blocks_per_cu; 0: no cap).
uint32_t row_lds_cap()
{
    const long cap = ddl_opt_rda_blocks_per_cu.load(std::memory_order_relaxed);
    uint32_t lds = cap > 0 ? (uint32_t)(DDL_LDS_PER_CU / cap) & ~511u : 0u;
    return lds > 60 * 1024 ? 60 * 1024 : lds;  // static LDS of the kernel comes on top
}

// Enqueues the RDA merge of ONE tensor.  `a` holds the tensor, the compacted learners and
// weights, n, group_len (already clamped to n), vec_ok, lr and mu; the workspace fields are
// filled in here.  g = geometry(n, group_len, Mq).
ddl_status launch_one(int src, int Mq, DdlRdaArgs& a, const Geometry& g, void* workspace,
                      hipStream_t stream)
{
    a.chunks_per_group = (uint32_t)g.chunks_per_group;
    const uint64_t ws = (uint64_t)(uintptr_t)workspace;
    a.partial1 = ws + g.off_partial1;
    a.coef = ws + g.off_coef;
    a.mean_norm = ws + g.off_mean;
    a.partial2 = ws + g.off_partial2;
    a.scale = ws + g.off_scale;

    const int cls = row_class_for(a.group_len);
    Kernels k;
    pick(src, Mq, cls, k);
    if (!k.sumsq) return DDL_ERR_INVALID_ARG;
    const dim3 block(DDL_BLOCK);
    const uint32_t groups = (uint32_t)g.groups;
    if (k.row && a.vec_ok && a.n % 4 == 0 && groups >= kGroupKernelMinGroups) {
        DDL_COUNT_GRID();
        hipLaunchKernelGGL(k.row, dim3(groups), dim3(k.row_threads), row_lds_cap(), stream,
                           a);
    } else if (a.group_len <= kGroupKernelMaxLen && groups >= kGroupKernelMinGroups) {
        DDL_COUNT_GRID();
        hipLaunchKernelGGL(k.group, dim3(groups), block, row_lds_cap(), stream, a);
    } else {
        const dim3 grid((uint32_t)g.chunks), rgrid(groups);
        if (k.gram) {
            DDL_COUNT_GRID();
            hipLaunchKernelGGL(k.gram, grid, block, 0, stream, a);
            DDL_COUNT_GRID();
            hipLaunchKernelGGL(k.gram_reduce, rgrid, block, 0, stream, a);
        } else {
            DDL_COUNT_GRID();
            hipLaunchKernelGGL(k.sumsq, grid, block, 0, stream, a);
            DDL_COUNT_GRID();
            hipLaunchKernelGGL(rda_norms_kernel, rgrid, block, 0, stream, a, Mq);
            DDL_COUNT_GRID();
            hipLaunchKernelGGL(k.dirsq, grid, block, 0, stream, a);
            DDL_COUNT_GRID();
            hipLaunchKernelGGL(rda_scale_kernel, rgrid, block, 0, stream, a);
        }
        // (workgroup numbers are 32-bit: a sweep too long for slices keeps whole chunks)
        a.piece_shift = g.chunks <= (0x7fffffffu >> kLongApplyPieceShift) ? kLongApplyPieceShift : 0;
        DDL_COUNT_GRID();
        hipLaunchKernelGGL(k.apply, dim3((uint32_t)g.chunks << a.piece_shift), block,
                           ddlh::merge_lds_cap_bytes(src_elem_bytes(src), Mq), stream, a);
    }
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? DDL_OK : ddlh::runtime_error(e, "RDA kernel launch");
}

}  // namespace

extern "C" size_t ddl_rda_workspace_bytes(size_t n, size_t group_len, int M)
{
    Geometry g;
    if (M < 1 || M > DDL_MAX_LEARNERS || !geometry(n, group_len, M, g)) return 0;
    return g.bytes;
}

namespace {

ddl_status static_scratch(void** out);  // device address of the library's own scratch array

// Shared by the two one-tensor entry points.  workspace: the caller's scratch, or NULL for the
// library's own array of workspace_bytes bytes, whose address is looked up only once the
// arguments have been found good (argument errors need no device).
ddl_status rda_merge_one(float* theta, float* v, const void* const* learner_params,
                         ddl_dtype learner_dtype, const uint64_t* token_counts,
                         const uint8_t* quorum_mask, int M, size_t n, size_t group_len, float lr,
                         float mu, void* workspace, size_t workspace_bytes, bool library_scratch,
                         const char* who, void* hip_stream)
{
    double w[DDL_MAX_LEARNERS];
    ddl_status st = ddl_compute_weights(token_counts, quorum_mask, M, w);
    if (st != DDL_OK) return st;
    if (learner_dtype != DDL_F32 && learner_dtype != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (!ddlh::finite_nonneg(lr) || !ddlh::finite_nonneg(mu)) return DDL_ERR_INVALID_ARG;
    if (group_len == 0) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!theta || !v || !learner_params || !aligned(theta, 4) || !aligned(v, 4))
        return DDL_ERR_INVALID_ARG;

    DdlRdaArgs a;
    std::memset(&a, 0, sizeof a);
    const size_t b = learner_dtype == DDL_BF16 ? 2 : 4;
    int Mq = 0;
    bool vec_ok = aligned(theta, 16) && aligned(v, 16) && std::min(group_len, n) % 4 == 0;
    // Overlap rules as everywhere: Theta, v and the workspace may overlap nothing.  (A fixed
    // array: this path must not allocate, not even on the host.)
    struct Range { uintptr_t lo, hi; bool out; };
    Range r[DDL_MAX_LEARNERS + 3];
    int nr = 0;
    auto add = [&](const void* p, size_t elem, bool out) {
        size_t bytes = 0;
        uintptr_t hi = 0;
        if (__builtin_mul_overflow(elem, n, &bytes) ||
            __builtin_add_overflow((uintptr_t)p, bytes, &hi))
            return false;
        r[nr++] = {(uintptr_t)p, hi, out};
        return true;
    };
    if (!add(theta, 4, true) || !add(v, 4, true)) return DDL_ERR_INVALID_ARG;
    for (int m = 0; m < M; ++m) {
        if (!(w[m] > 0.0)) continue;
        const void* p = learner_params[m];
        if (!p || !aligned(p, b) || !add(p, b, false)) return DDL_ERR_INVALID_ARG;
        vec_ok = vec_ok && aligned(p, 16);
        a.learner[Mq] = (uint64_t)(uintptr_t)p;
        a.w[Mq] = (float)w[m];
        ++Mq;
    }
    Geometry g;
    if (!geometry(n, group_len, Mq, g)) return DDL_ERR_INVALID_ARG;
    if (!library_scratch && (!workspace || !aligned(workspace, 256))) return DDL_ERR_INVALID_ARG;
    if (workspace_bytes < g.bytes) {
        ddlh::set_error_message((std::string(who) + ": this tensor and grouping need " +
                                 std::to_string(g.bytes) + " bytes of scratch, " +
                                 std::to_string(workspace_bytes) + " are there").c_str());
        return DDL_ERR_INVALID_ARG;
    }
    if (library_scratch) {
        const ddl_status ws = static_scratch(&workspace);
        if (ws != DDL_OK) return ws;
    }
    r[nr++] = {(uintptr_t)workspace, (uintptr_t)workspace + g.bytes, true};
    std::sort(r, r + nr, [](const Range& x, const Range& y) { return x.lo < y.lo; });
    uintptr_t hi_any = 0, hi_out = 0;
    for (int i = 0; i < nr; ++i) {
        const Range& x = r[i];
        if (x.out ? x.lo < hi_any : x.lo < hi_out) return DDL_ERR_ALIAS;
        hi_any = std::max(hi_any, x.hi);
        if (x.out) hi_out = std::max(hi_out, x.hi);
    }

    a.theta = (uint64_t)(uintptr_t)theta;
    a.v = (uint64_t)(uintptr_t)v;
    a.n = n;
    a.group_len = std::min<uint64_t>(group_len, n);
    a.vec_ok = vec_ok ? 1u : 0u;
    a.lr = lr;
    a.mu = mu;
    return launch_one((int)learner_dtype, Mq, a, g, workspace,
                      static_cast<hipStream_t>(hip_stream));
}

}  // namespace

extern "C" ddl_status ddl_rda_merge_fragment(float* theta, float* v,
                                             const void* const* learner_params,
                                             ddl_dtype learner_dtype, const uint64_t* token_counts,
                                             const uint8_t* quorum_mask, int M, size_t n,
                                             size_t group_len, float lr, float mu, void* workspace,
                                             size_t workspace_bytes, void* hip_stream)
{
    return rda_merge_one(theta, v, learner_params, learner_dtype, token_counts, quorum_mask, M, n,
                         group_len, lr, mu, workspace, workspace_bytes, false,
                         "ddl_rda_merge_fragment", hip_stream);
}

namespace {

uint32_t log2_or_none(uint32_t x)  // log2 of a power of two, else 0xffffffff
{
    if (x == 0 || (x & (x - 1))) return 0xffffffffu;
    uint32_t sh = 0;
    while ((1u << sh) < x) ++sh;
    return sh;
}

bool q4_block_len_ok(size_t block_len)
{
    return block_len >= 8 && block_len % 8 == 0 && block_len <= 0x40000000u;
}

}  // namespace

// RDA as the merge of 4-bit outer gradients, one tensor: the kernels above instantiated for
// codes and block scales as the learners' data.
extern "C" ddl_status ddl_q4_rda_merge_fragment(float* theta, float* v,
                                                const uint8_t* const* codes,
                                                const float* const* scales,
                                                const uint64_t* token_counts,
                                                const uint8_t* quorum_mask, int M, size_t n,
                                                size_t block_len, size_t group_len, float lr,
                                                float mu, void* workspace, size_t workspace_bytes,
                                                void* hip_stream)
{
    double w[DDL_MAX_LEARNERS];
    const ddl_status st = ddl_compute_weights(token_counts, quorum_mask, M, w);
    if (st != DDL_OK) return st;
    if (!ddlh::finite_nonneg(lr) || !ddlh::finite_nonneg(mu)) return DDL_ERR_INVALID_ARG;
    if (!q4_block_len_ok(block_len) || group_len == 0) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!theta || !v || !codes || !scales || !aligned(theta, 16) || !aligned(v, 16))
        return DDL_ERR_INVALID_ARG;
    const uint64_t blocks = (n + block_len - 1) / block_len;
    ddlh::Quorum q;
    ddlh::compact(w, M, q);
    DdlRdaArgs a;
    std::memset(&a, 0, sizeof a);
    std::vector<ddlh::Range> r;
    if (!ddlh::add_range(theta, 4, n, true, r) || !ddlh::add_range(v, 4, n, true, r))
        return DDL_ERR_INVALID_ARG;
    for (int j = 0; j < q.Mq; ++j) {
        const uint8_t* c = codes[q.idx[j]];
        const float* sc = scales[q.idx[j]];
        if (!c || !sc || !aligned(c, 4) || !aligned(sc, 4) ||
            !ddlh::add_range(c, 1, (n + 1) / 2, false, r) ||
            !ddlh::add_range(sc, 4, blocks, false, r))
            return DDL_ERR_INVALID_ARG;
        a.learner[j] = (uint64_t)(uintptr_t)c;
        a.scales[j] = (uint64_t)(uintptr_t)sc;
        a.w[j] = q.w[j];
    }
    Geometry g;
    if (!geometry(n, group_len, q.Mq, g)) return DDL_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < g.bytes)
        return DDL_ERR_INVALID_ARG;
    if (!ddlh::add_range(workspace, 1, g.bytes, true, r)) return DDL_ERR_INVALID_ARG;
    if (ddlh::ranges_alias(r)) return DDL_ERR_ALIAS;
    a.theta = (uint64_t)(uintptr_t)theta;
    a.v = (uint64_t)(uintptr_t)v;
    a.n = n;
    a.group_len = std::min<uint64_t>(group_len, n);
    a.vec_ok = a.group_len % 4 == 0 ? 1u : 0u;  // Theta and v are aligned, codes 4-byte aligned
    a.block_len = (uint32_t)block_len;
    a.block_shift = log2_or_none((uint32_t)block_len);
    a.lr = lr;
    a.mu = mu;
    return launch_one(DDL_SRC_Q4, q.Mq, a, g, workspace, static_cast<hipStream_t>(hip_stream));
}

// ------------------------------------------------------------------------------------------
// The same merge for callers that cannot allocate and have no workspace to pass: the scratch
// is a fixed array in the library's device image.  Each GPU holds its own copy at its own
// address, which is looked up once per device; host code only ever uses that looked-up
// address, never the array's name.
// ------------------------------------------------------------------------------------------
#define DDL_RDA_STATIC_SCRATCH_BYTES (4u << 20)
static __device__ __align__(256) unsigned char scratch[DDL_RDA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxScratchDevices = 16;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxScratchDevices] = {};

// Device address of `scratch` on the current device.
ddl_status static_scratch(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return ddlh::runtime_error(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxScratchDevices) {
        ddlh::set_error_message("device index out of range");
        return DDL_ERR_RUNTIME;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return ddlh::runtime_error(e, "hipGetSymbolAddress(scratch)");
        if (!p) {
            ddlh::set_error_message("hipGetSymbolAddress(scratch) returned a null address");
            return DDL_ERR_RUNTIME;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DDL_OK;
}

}  // namespace

extern "C" size_t ddl_rda_static_scratch_bytes(void) { return DDL_RDA_STATIC_SCRATCH_BYTES; }

extern "C" ddl_status ddl_rda_merge_fragment_static(float* theta, float* v,
                                                    const void* const* learner_params,
                                                    ddl_dtype learner_dtype,
                                                    const uint64_t* token_counts,
                                                    const uint8_t* quorum_mask, int M, size_t n,
                                                    size_t group_len, float lr, float mu,
                                                    void* hip_stream)
{
    // Every kernel of the merge writes the part of the scratch it later reads (chunk sums,
    // coefficients, scales), so nothing has to be cleared between calls.
    return rda_merge_one(theta, v, learner_params, learner_dtype, token_counts, quorum_mask, M, n,
                         group_len, lr, mu, nullptr, DDL_RDA_STATIC_SCRATCH_BYTES, true,
                         "ddl_rda_merge_fragment_static", hip_stream);
}

// ------------------------------------------------------------------------------------------
// RDA through a plan: all tensors of a fragment whose groups fit the register-resident row
// kernels go out in one launch per row class; the rest take the one-tensor path above.
// ------------------------------------------------------------------------------------------
struct DdlRdaPlan {
    struct Class {
        uint32_t ref_begin = 0, num_refs = 0, rows = 0, coarse_begin = 0, coarse_shift = 0;
        uint64_t elems = 0;  // elements of all its tensors
    };
    struct Frag {
        Class cls[kNumRowClasses];
        std::vector<uint32_t> other;   // descriptors that always take the one-tensor path
        std::vector<uint32_t> direct;  // descriptors merged by direct averaging instead
        // tensors of long or few groups: all of them in three launches (table entries
        // [long_begin, long_begin + long_count) of long_refs)
        uint32_t long_begin = 0, long_count = 0, long_chunks = 0, long_groups = 0;
    };
    std::vector<uint64_t> group_len;  // per descriptor, clamped to its n
    std::vector<Frag> frags;
    std::vector<DdlRdaRowRef> refs;
    std::vector<uint32_t> coarse;
    std::vector<DdlRdaLongRef> long_refs;
    void* d_image = nullptr;  // refs, then the coarse index, then long_refs (8-byte aligned)
    size_t long_offset = 0;   // of long_refs within the image
    size_t workspace_bytes = 0;
};

void ddl_rda_plan_free(DdlRdaPlan* p)
{
    if (!p) return;
    if (p->d_image) (void)hipFree(p->d_image);
    delete p;
}

namespace {

// Can descriptor d with groups of g elements go through a row kernel, whatever the quorum?
bool row_eligible(const DdlSegDesc& d, int M, uint64_t g)
{
    const uint32_t all = (1u << M) - 1u;
    return g % 4 == 0 && d.n % 4 == 0 && row_class_for(g) < kNumRowClasses && d.base_aligned &&
           (all & ~(uint32_t)d.learner_aligned) == 0;
}

struct RdaWork {
    uint32_t frag;
    ddlh::Quorum q;
    float lr, mu;
};

}  // namespace

extern "C" ddl_status ddl_plan_set_rda_groups(ddl_plan* plan, const size_t* group_len,
                                              size_t num_segments)
{
    if (!plan || num_segments != plan->table.given_segs || (num_segments > 0 && !group_len))
        return DDL_ERR_INVALID_ARG;
    const ddlh::Table& T = plan->table;
    DdlRdaPlan* R = new (std::nothrow) DdlRdaPlan();
    if (!R) return DDL_ERR_RUNTIME;
    R->group_len.resize(T.segs.size());
    R->frags.resize(T.frags.size());
    for (size_t f = 0; f < T.frags.size(); ++f) {
        const ddlh::FragInfo& fi = T.frags[f];
        DdlRdaPlan::Frag& rf = R->frags[f];
        std::vector<uint32_t> members[kNumRowClasses];
        uint64_t long_bytes = 0;  // workspace of the fragment's long-group tensors, side by side
        for (uint32_t d = fi.seg_begin; d < fi.seg_begin + fi.num_segs; ++d) {
            const DdlSegDesc& sd = T.segs[d];
            uint64_t g = group_len[T.origin[d]];
            if (g == (size_t)-1) {  // this tensor takes direct averaging
                R->group_len[d] = 0;
                rf.direct.push_back(d);
                continue;
            }
            if (g == 0 || g > sd.n) g = sd.n;
            R->group_len[d] = g;
            Geometry geo;
            if (!geometry(sd.n, g, fi.M, geo)) {
                delete R;
                return DDL_ERR_INVALID_ARG;
            }
            R->workspace_bytes = std::max(R->workspace_bytes, geo.bytes);
            if (row_eligible(sd, fi.M, g)) {
                members[row_class_for(g)].push_back(d);
            } else if (g <= kGroupKernelMaxLen && geo.groups >= kGroupKernelMinGroups) {
                rf.other.push_back(d);  // many moderate groups: the one-workgroup-per-group kernel
            } else {
                // long or few groups: one entry of the fragment's three launches
                if (rf.long_count == 0) rf.long_begin = (uint32_t)R->long_refs.size();
                DdlRdaLongRef ref;
                std::memset(&ref, 0, sizeof ref);
                ref.seg = d;
                ref.chunk_begin = rf.long_chunks;
                ref.group_begin = rf.long_groups;
                ref.chunks_per_group = (uint32_t)geo.chunks_per_group;
                ref.group_len = g;
                const uint32_t all = (1u << fi.M) - 1u;
                ref.vec_all = sd.base_aligned && g % 4 == 0 &&
                              (all & ~(uint32_t)sd.learner_aligned) == 0;
                auto take = [&](uint64_t floats) {
                    const uint64_t at = long_bytes;
                    long_bytes += (floats * 4 + 255) & ~(uint64_t)255;
                    return at;
                };
                ref.off_partial1 = take(geo.chunks * (uint64_t)partial_width(fi.M));
                ref.off_coef = take(geo.groups * (uint64_t)fi.M);
                ref.off_mean = take(geo.groups);
                ref.off_scale = take(geo.groups);
                if ((uint64_t)rf.long_chunks + geo.chunks > 0x7fffffffull ||
                    (uint64_t)rf.long_groups + geo.groups > 0x7fffffffull) {
                    delete R;
                    return DDL_ERR_INVALID_ARG;
                }
                rf.long_chunks += (uint32_t)geo.chunks;
                rf.long_groups += (uint32_t)geo.groups;
                ++rf.long_count;
                R->long_refs.push_back(ref);
            }
        }
        R->workspace_bytes = std::max<size_t>(R->workspace_bytes, (size_t)long_bytes);
        for (int c = 0; c < kNumRowClasses; ++c) {
            DdlRdaPlan::Class& k = rf.cls[c];
            k.ref_begin = (uint32_t)R->refs.size();
            k.coarse_begin = (uint32_t)R->coarse.size();
            uint64_t rows = 0;
            for (uint32_t d : members[c]) {
                const uint64_t g = R->group_len[d];
                if (rows > 0x7fffffffull) break;
                R->refs.push_back({d, (uint32_t)rows, (uint32_t)g, 0u});
                rows += (T.segs[d].n + g - 1) / g;
                k.elems += T.segs[d].n;
            }
            if (rows > 0x7fffffffull) {
                delete R;
                return DDL_ERR_INVALID_ARG;
            }
            k.num_refs = (uint32_t)members[c].size();
            k.rows = (uint32_t)rows;
            if (k.num_refs == 0) continue;
            // About four coarse entries per tensor, and one past the end so that entry i + 1
            // is readable for every row.
            const uint64_t target = 4ull * k.num_refs;
            while (k.coarse_shift < 31 && (rows >> (k.coarse_shift + 1)) >= target)
                ++k.coarse_shift;
            const uint32_t entries = (k.rows >> k.coarse_shift) + 2;
            const DdlRdaRowRef* refs = R->refs.data() + k.ref_begin;
            uint32_t s = 0;
            for (uint32_t i = 0; i < entries; ++i) {
                const uint64_t row = (uint64_t)i << k.coarse_shift;
                while (s + 1 < k.num_refs && refs[s + 1].row_begin <= row) ++s;
                R->coarse.push_back(row < rows ? s : k.num_refs - 1);
            }
        }
    }
    const size_t ref_bytes = R->refs.size() * sizeof(DdlRdaRowRef);
    const size_t coarse_bytes = R->coarse.size() * sizeof(uint32_t);
    R->long_offset = (ref_bytes + coarse_bytes + 7) & ~(size_t)7;
    const size_t bytes = R->long_offset + R->long_refs.size() * sizeof(DdlRdaLongRef);
    if (bytes > 0) {
        std::vector<char> image(bytes);
        std::memcpy(image.data(), R->refs.data(), ref_bytes);
        std::memcpy(image.data() + ref_bytes, R->coarse.data(), coarse_bytes);
        std::memcpy(image.data() + R->long_offset, R->long_refs.data(),
                    R->long_refs.size() * sizeof(DdlRdaLongRef));
        hipError_t e = hipMalloc(&R->d_image, bytes);
        if (e == hipSuccess) e = hipMemcpy(R->d_image, image.data(), bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            ddl_rda_plan_free(R);
            return ddlh::runtime_error(e, "RDA plan upload");
        }
    }
    if (plan->rda) ddl_rda_plan_free(plan->rda);
    plan->rda = R;
    return DDL_OK;
}

extern "C" size_t ddl_plan_rda_workspace_bytes(const ddl_plan* plan)
{
    return plan && plan->rda ? plan->rda->workspace_bytes : 0;
}

namespace {

// ddl_plan_rda_merge and ddl_plan_q4_rda_merge: the learners' data are their copies of the
// tensors (the plan's descriptors), or -- q4 -- their outer gradients as 4-bit codes with
// block scales (the plan's 4-bit sources).
ddl_status plan_rda_merge(ddl_plan* plan, const ddl_sync* syncs, int count, void* workspace,
                          size_t workspace_bytes, void* hip_stream, bool q4)
{
    if (!plan || !plan->rda || count < 0 || (count > 0 && !syncs)) return DDL_ERR_INVALID_ARG;
    if (q4 && (plan->q4_block_len == 0 || plan->q4_host.size() != plan->table.segs.size()))
        return DDL_ERR_INVALID_ARG;
    if (count == 0) return DDL_OK;
    const ddlh::Table& T = plan->table;
    const DdlRdaPlan& R = *plan->rda;
    const uint32_t block_len = q4 ? plan->q4_block_len : 0;
    const uint32_t block_shift = log2_or_none(block_len);
    const DdlQ4Desc* d_q4 = static_cast<const DdlQ4Desc*>(plan->d_q4);
    if (R.workspace_bytes > 0 &&
        (!workspace || !aligned(workspace, 256) || workspace_bytes < R.workspace_bytes))
        return DDL_ERR_INVALID_ARG;
    const uintptr_t ws_lo = (uintptr_t)workspace, ws_hi = ws_lo + R.workspace_bytes;
    auto hits_workspace = [&](const void* p, uint64_t bytes) {
        const uintptr_t lo = (uintptr_t)p;
        return p && lo < ws_hi && ws_lo < lo + bytes;
    };

    // Everything is validated before anything is enqueued.
    std::vector<RdaWork> work;
    work.reserve((size_t)count);
    std::vector<char> seen(T.frags.size(), 0);
    for (int i = 0; i < count; ++i) {
        const ddl_sync& s = syncs[i];
        if (s.fragment < 0 || (size_t)s.fragment >= T.frags.size()) return DDL_ERR_INVALID_ARG;
        if (seen[(size_t)s.fragment]) return DDL_ERR_ALIAS;
        seen[(size_t)s.fragment] = 1;
        if (!ddlh::finite_nonneg(s.lr) || !ddlh::finite_nonneg(s.mu)) return DDL_ERR_INVALID_ARG;
        const ddlh::FragInfo& f = T.frags[(size_t)s.fragment];
        double w[DDL_MAXL];
        const ddl_status st = ddlh::weights_tokens(s.token_counts, s.quorum_mask, f.M, w);
        if (st != DDL_OK) return st;
        RdaWork wk;
        wk.frag = (uint32_t)s.fragment;
        wk.lr = s.lr;
        wk.mu = s.mu;
        ddlh::compact(w, f.M, wk.q);
        const uint32_t have = q4 ? plan->q4_nonnull_bits[(size_t)s.fragment] : f.nonnull_bits;
        if (f.num_segs > 0 && (wk.q.present_bits & ~have)) return DDL_ERR_INVALID_ARG;
        const size_t b = f.dt == DDL_BF16 ? 2 : 4;
        for (uint32_t d = f.seg_begin; d < f.seg_begin + f.num_segs; ++d) {
            const DdlSegDesc& sd = T.segs[d];
            bool hit = hits_workspace(sd.theta, 4 * sd.n) || hits_workspace(sd.v, 4 * sd.n) ||
                       hits_workspace(sd.theta_bf16, 2 * sd.n);
            for (int j = 0; j < wk.q.Mq; ++j) {
                if (q4) {
                    const DdlQ4Desc& qd = plan->q4_host[d];
                    hit = hit || hits_workspace(qd.codes[wk.q.idx[j]], (sd.n + 1) / 2) ||
                          hits_workspace(qd.scales[wk.q.idx[j]],
                                         4 * ((sd.n + block_len - 1) / block_len));
                } else {
                    hit = hit || hits_workspace(sd.learner[wk.q.idx[j]], b * sd.n);
                }
            }
            if (hit) return DDL_ERR_ALIAS;
        }
        work.push_back(wk);
    }

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const DdlSegDesc* d_segs = static_cast<const DdlSegDesc*>(plan->d_table);
    const DdlRdaRowRef* d_refs = static_cast<const DdlRdaRowRef*>(R.d_image);
    const uint32_t* d_coarse = reinterpret_cast<const uint32_t*>(
        static_cast<const char*>(R.d_image) + R.refs.size() * sizeof(DdlRdaRowRef));

    // One tensor through the one-tensor path.
    auto one_tensor = [&](const ddlh::FragInfo& f, const RdaWork& wk, uint32_t d) -> ddl_status {
        const DdlSegDesc& sd = T.segs[d];
        DdlRdaArgs a;
        std::memset(&a, 0, sizeof a);
        a.theta = (uint64_t)(uintptr_t)sd.theta;
        a.v = (uint64_t)(uintptr_t)sd.v;
        a.theta_bf16 = (uint64_t)(uintptr_t)sd.theta_bf16;
        a.n = sd.n;
        a.group_len = R.group_len[d];
        a.lr = wk.lr;
        a.mu = wk.mu;
        bool vec_ok = aligned(sd.theta, 16) && aligned(sd.v, 16) && aligned(sd.theta_bf16, 8) &&
                      a.group_len % 4 == 0;
        for (int j = 0; j < wk.q.Mq; ++j) {
            if (q4) {  // codes and scales are 4-byte aligned (checked when they were set)
                a.learner[j] = (uint64_t)(uintptr_t)plan->q4_host[d].codes[wk.q.idx[j]];
                a.scales[j] = (uint64_t)(uintptr_t)plan->q4_host[d].scales[wk.q.idx[j]];
            } else {
                const void* p = sd.learner[wk.q.idx[j]];
                vec_ok = vec_ok && aligned(p, 16);
                a.learner[j] = (uint64_t)(uintptr_t)p;
            }
            a.w[j] = wk.q.w[j];
        }
        a.block_len = block_len;
        a.block_shift = block_shift;
        a.vec_ok = vec_ok ? 1u : 0u;
        Geometry g;
        if (!geometry(sd.n, a.group_len, wk.q.Mq, g)) return DDL_ERR_INVALID_ARG;
        return launch_one(q4 ? DDL_SRC_Q4 : (int)f.dt, wk.q.Mq, a, g, workspace, stream);
    };

    for (const RdaWork& wk : work) {
        const ddlh::FragInfo& f = T.frags[wk.frag];
        const DdlRdaPlan::Frag& rf = R.frags[wk.frag];
        const int src = q4 ? DDL_SRC_Q4 : (int)f.dt;
        for (int c = 0; c < kNumRowClasses; ++c) {
            const DdlRdaPlan::Class& k = rf.cls[c];
            if (k.num_refs == 0) continue;
            Kernels fn;
            pick(src, wk.q.Mq, c, fn);
            const int sd_extra_bytes = 0;
            if (fn.rows) {
                DdlRdaRowsArgs a;
                std::memset(&a, 0, sizeof a);
                a.segs = d_segs;
                a.refs = d_refs + k.ref_begin;
                a.coarse = d_coarse + k.coarse_begin;
                a.coarse_shift = k.coarse_shift;
                a.lr = wk.lr;
                a.mu = wk.mu;
                std::memcpy(a.w, wk.q.w, sizeof a.w);
                std::memcpy(a.idx, wk.q.idx, sizeof a.idx);
                a.q4 = d_q4;
                a.block_len = block_len;
                a.block_shift = block_shift;
                // Like the direct-averaging merge, a long launch goes out as several equal
                // grids, which keeps the XCDs aligned: the limit in elements becomes rows.
                const uint64_t max_tiles = ddlh::max_tiles_per_launch(
                    src_elem_bytes(src), wk.q.Mq, sd_extra_bytes);
                uint64_t part = k.rows;
                if (max_tiles != 0 && k.elems > max_tiles * DDL_TILE) {
                    const uint64_t parts = (k.elems + max_tiles * DDL_TILE - 1) / (max_tiles * DDL_TILE);
                    part = (k.rows + parts - 1) / parts;
                }
                for (uint64_t base = 0; base < k.rows; base += part) {
                    a.row_base = (uint32_t)base;
                    const uint32_t rows = (uint32_t)std::min<uint64_t>(part, k.rows - base);
                    DDL_COUNT_GRID();
                    hipLaunchKernelGGL(fn.rows, dim3(rows), dim3(fn.row_threads), row_lds_cap(),
                                       stream, a);
                    const hipError_t e = hipGetLastError();
                    if (e != hipSuccess) return ddlh::runtime_error(e, "RDA rows kernel launch");
                }
            } else {  // this many learners do not fit the registers of this class
                for (uint32_t r = 0; r < k.num_refs; ++r) {
                    const ddl_status st = one_tensor(f, wk, R.refs[k.ref_begin + r].seg);
                    if (st != DDL_OK) return st;
                }
            }
        }
        for (uint32_t d : rf.other) {
            const ddl_status st = one_tensor(f, wk, d);
            if (st != DDL_OK) return st;
        }
        if (rf.long_count > 0) {
            Kernels fn;
            pick(src, wk.q.Mq, kNumRowClasses, fn);
            if (fn.long_gram) {  // all these tensors in three launches
                DdlRdaLongArgs a;
                std::memset(&a, 0, sizeof a);
                a.segs = d_segs;
                a.refs = reinterpret_cast<const DdlRdaLongRef*>(
                             static_cast<const char*>(R.d_image) + R.long_offset) + rf.long_begin;
                a.num_refs = rf.long_count;
                a.workspace = (uint64_t)(uintptr_t)workspace;
                a.lr = wk.lr;
                a.mu = wk.mu;
                std::memcpy(a.w, wk.q.w, sizeof a.w);
                std::memcpy(a.idx, wk.q.idx, sizeof a.idx);
                a.q4 = d_q4;
                a.block_len = block_len;
                a.block_shift = block_shift;
                const dim3 block(DDL_BLOCK);
                // the two sweeps go out in equal parts like the merge (a chunk is 8 tiles)
                const uint64_t max_tiles =
                    ddlh::max_tiles_per_launch(src_elem_bytes(src), wk.q.Mq);
                uint64_t part = rf.long_chunks;
                const uint64_t max_chunks = max_tiles / (DDL_RDA_CHUNK / DDL_TILE);
                if (max_tiles != 0 && max_chunks > 0 && rf.long_chunks > max_chunks) {
                    const uint64_t parts = (rf.long_chunks + max_chunks - 1) / max_chunks;
                    part = (rf.long_chunks + parts - 1) / parts;
                }
                // `scale` workgroups per chunk; parts of whole rotation groups
                auto sweep = [&](rda_long_fn kernel, uint64_t scale, uint32_t lds) {
                    const uint64_t total = rf.long_chunks * scale;
                    const uint64_t unit = kLongApplyRotate;
                    const uint64_t step = (part * scale + unit - 1) / unit * unit;
                    for (uint64_t base = 0; base < total; base += step) {
                        a.base = (uint32_t)base;
                        DDL_COUNT_GRID();
                        hipLaunchKernelGGL(kernel,
                                           dim3((uint32_t)std::min<uint64_t>(step, total - base)),
                                           block, lds, stream, a);
                    }
                };
                a.by_group = 0;
                a.piece_shift = 0;
                sweep(fn.long_gram, 1, 0);
                a.by_group = 1;
                a.base = 0;
                DDL_COUNT_GRID();
                hipLaunchKernelGGL(fn.long_reduce, dim3(rf.long_groups), block, 0, stream, a);
                a.by_group = 0;
                // (workgroup numbers are 32-bit: a sweep too long for slices keeps whole chunks)
                a.piece_shift =
                    rf.long_chunks <= (0x7fffffffu >> kLongApplyPieceShift) ? kLongApplyPieceShift : 0;
                sweep(fn.long_apply, 1u << a.piece_shift,
                      ddlh::merge_lds_cap_bytes(src_elem_bytes(src), wk.q.Mq));
                const hipError_t e = hipGetLastError();
                if (e != hipSuccess) return ddlh::runtime_error(e, "RDA long-group kernel launch");
            } else {  // more learners than the Gram form takes: tensor by tensor
                for (uint32_t r = 0; r < rf.long_count; ++r) {
                    const ddl_status st = one_tensor(f, wk, R.long_refs[rf.long_begin + r].seg);
                    if (st != DDL_OK) return st;
                }
            }
        }
        for (uint32_t d : rf.direct) {
            const ddl_status st =
                q4 ? ddlh::launch_flat(T.segs[d], DDL_SRC_Q4, wk.q, wk.lr, wk.mu, hip_stream,
                                       &plan->q4_host[d], block_len)
                   : ddlh::launch_one_direct(T.segs[d], f.dt, wk.q, wk.lr, wk.mu, hip_stream);
            if (st != DDL_OK) return st;
        }
    }
    return DDL_OK;
}

}  // namespace

extern "C" ddl_status ddl_plan_rda_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                         void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return plan_rda_merge(plan, syncs, count, workspace, workspace_bytes, hip_stream, false);
}

// The same with the plan's 4-bit sources (ddl_plan_set_q4_sources) as the learners' data.
extern "C" ddl_status ddl_plan_q4_rda_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                            void* workspace, size_t workspace_bytes,
                                            void* hip_stream)
{
    return plan_rda_merge(plan, syncs, count, workspace, workspace_bytes, hip_stream, true);
}
