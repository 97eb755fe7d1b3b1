// gfx950 kernels of the synchronizer hot path: weighted merge of the contributing learners'
// copies into the outer gradient, fused with the outer Nesterov-momentum step (Algorithm 2,
// steps "mergeFn" and "OuterOpt"; Appendix D.2, weighted direct averaging).
//
// The work is a streaming reduction with no reuse: per element it reads Mq learner values
// (2 or 4 bytes each) plus Theta and v, and writes Theta and v -- about 0.7 flop per byte --
// so the kernel is organised around HBM, not around the ALUs:
//   * every lane moves 16 bytes per access and the lanes of a wavefront cover consecutive
//     addresses, so each wave-wide load or store is one contiguous run of 1 KiB (Theta / v /
//     fp32 learners / 8-wide bf16) or 512 B (4-wide bf16);
//   * all loads of DDL_UNROLL vector groups are issued before the first use, which keeps
//     (16 Mq + 64) * UNROLL bytes per lane in flight;
//   * weights, learner selection, lr and mu come from the kernel argument block (scalar
//     loads into SGPRs); absent learners do not appear in it and are never addressed;
//   * Delta, the new v and the new Theta stay in registers; Theta and v are read once and
//     written once.
#include <hip/hip_runtime.h>

#include "ddl_device.h"

#ifndef DDL_NT_LOAD
#define DDL_NT_LOAD 1   // learner / Theta / v loads bypass-hinted: every byte is used once
#endif
#ifndef DDL_NT_STORE
#define DDL_NT_STORE 1
#endif
#ifndef DDL_BF16_VEC
#define DDL_BF16_VEC 8  // bf16 elements per lane per group: 8 (16-byte loads) or 4 (8-byte)
#endif

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// All tensor accesses go through explicit global-address-space pointers built from a
// 64-bit base held in scalar registers plus a 32-bit per-lane index, which is the form the
// global_load / global_store "saddr" encoding takes directly.
#define DDL_GLOBAL __attribute__((address_space(1)))

template <typename T>
__device__ __forceinline__ T ld(uint64_t base, uint32_t index)
{
    const DDL_GLOBAL T* p = reinterpret_cast<const DDL_GLOBAL T*>(base) + index;
#if DDL_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

template <typename T>
__device__ __forceinline__ void st(uint64_t base, uint32_t index, T x)
{
    DDL_GLOBAL T* p = reinterpret_cast<DDL_GLOBAL T*>(base) + index;
#if DDL_NT_STORE
    __builtin_nontemporal_store(x, p);
#else
    *p = x;
#endif
}

// Values that are the same for every lane of a workgroup (tile geometry, base addresses) are
// moved to scalar registers explicitly: descriptor fields read from the device table arrive
// in vector registers, and sixteen 64-bit learner addresses held per lane would halve the
// number of resident wavefronts.
__device__ __forceinline__ uint32_t uniform(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint64_t uniform(uint64_t x)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// bf16 is the upper half of an fp32 word, so widening is a shift or a mask.
__device__ __forceinline__ float bf16_even(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_odd(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// Learner element types.  VEC = elements one lane handles per group, RAW = the register
// image of those VEC elements as loaded.
struct LearnerF32 {
    typedef float elem;
    typedef u32x4 raw;
    static constexpr int VEC = 4;  // elements per lane per group
    static __device__ __forceinline__ void widen(const raw& r, float (&x)[4])
    {
        x[0] = __uint_as_float(r.x);
        x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z);
        x[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ float widen1(float e) { return e; }
};

struct LearnerBF16x8 {
    typedef uint16_t elem;
    typedef u32x4 raw;
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void widen(const raw& r, float (&x)[8])
    {
        x[0] = bf16_even(r.x); x[1] = bf16_odd(r.x);
        x[2] = bf16_even(r.y); x[3] = bf16_odd(r.y);
        x[4] = bf16_even(r.z); x[5] = bf16_odd(r.z);
        x[6] = bf16_even(r.w); x[7] = bf16_odd(r.w);
    }
    static __device__ __forceinline__ float widen1(uint16_t e)
    {
        return __uint_as_float((uint32_t)e << 16);
    }
};

struct LearnerBF16x4 {
    typedef uint16_t elem;
    typedef u32x2 raw;
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void widen(const raw& r, float (&x)[4])
    {
        x[0] = bf16_even(r.x); x[1] = bf16_odd(r.x);
        x[2] = bf16_even(r.y); x[3] = bf16_odd(r.y);
    }
    static __device__ __forceinline__ float widen1(uint16_t e)
    {
        return __uint_as_float((uint32_t)e << 16);
    }
};

// How many vector groups a lane keeps in flight, by register budget: a group holds
// 4 Mq (or 2 Mq) learner registers plus 2 VEC for Theta and v.
template <typename L, int MQ>
struct Unroll {
#ifdef DDL_UNROLL
    static constexpr int value = DDL_UNROLL;
#else
    static constexpr int regs = (int)(sizeof(typename L::raw) / 4) * MQ + 2 * L::VEC;
    static constexpr int value = regs <= 24 ? 4 : (regs <= 48 ? 2 : 1);
#endif
};

// One element: Delta = sum_j w_j (Theta - x_j); v' = mu v + Delta;
// Theta' = Theta - lr (Delta + mu v').  The difference form keeps the fp32 rounding of the
// weights (their sum is 1 only to ~1e-7) away from |Theta|.
template <int MQ>
__device__ __forceinline__ void outer_step(float& theta, float& v, const float (&x)[MQ],
                                           const float (&w)[MQ], float lr, float mu)
{
    float delta = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) delta = fmaf(w[j], theta - x[j], delta);
    const float v_new = fmaf(mu, v, delta);
    theta = fmaf(-lr, fmaf(mu, v_new, delta), theta);
    v = v_new;
}

// U vector groups per lane: group u of this lane is `g + u * DDL_BLOCK`.  th / vv / lp are
// the byte addresses of the tile's first element in each array.
template <typename L, int MQ, int U>
__device__ __forceinline__ void merge_groups(uint64_t th, uint64_t vv, const uint64_t (&lp)[MQ],
                                             const float (&w)[MQ], float lr, float mu, uint32_t g)
{
    constexpr int VEC = L::VEC;
    constexpr int Q = VEC / 4;  // float4 per group for Theta and for v
    typename L::raw raw[U][MQ];
    f32x4 T[U][Q], V[U][Q];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t gi = g + u * DDL_BLOCK;
#pragma unroll
        for (int j = 0; j < MQ; ++j) raw[u][j] = ld<typename L::raw>(lp[j], gi);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            T[u][q] = ld<f32x4>(th, gi * Q + q);
            V[u][q] = ld<f32x4>(vv, gi * Q + q);
        }
    }
    // Keep every load above ahead of the arithmetic: the bytes in flight are the point.
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t gi = g + u * DDL_BLOCK;
        float x[MQ][VEC];
#pragma unroll
        for (int j = 0; j < MQ; ++j) L::widen(raw[u][j], x[j]);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float t4[4] = {T[u][q].x, T[u][q].y, T[u][q].z, T[u][q].w};
            float v4[4] = {V[u][q].x, V[u][q].y, V[u][q].z, V[u][q].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float xe[MQ];
#pragma unroll
                for (int j = 0; j < MQ; ++j) xe[j] = x[j][q * 4 + k];
                outer_step<MQ>(t4[k], v4[k], xe, w, lr, mu);
            }
            f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
            f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
            st<f32x4>(th, gi * Q + q, tn);
            st<f32x4>(vv, gi * Q + q, vn);
        }
    }
}

template <typename L, int MQ>
__device__ __forceinline__ void merge_scalar(uint64_t th, uint64_t vv, const uint64_t (&lp)[MQ],
                                             const float (&w)[MQ], float lr, float mu, uint32_t e)
{
    typedef typename L::elem elem;
    float t = *(reinterpret_cast<const DDL_GLOBAL float*>(th) + e);
    float v = *(reinterpret_cast<const DDL_GLOBAL float*>(vv) + e);
    float xe[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j)
        xe[j] = L::widen1(*(reinterpret_cast<const DDL_GLOBAL elem*>(lp[j]) + e));
    outer_step<MQ>(t, v, xe, w, lr, mu);
    *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = t;
    *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v;
}

template <typename L, int MQ, bool FLAT>
__global__ void __launch_bounds__(DDL_BLOCK) ddl_merge_kernel(const DdlLaunchArgs a)
{
    constexpr int VEC = L::VEC;
    constexpr int U = Unroll<L, MQ>::value;
    typedef typename L::elem elem;

    for (uint32_t tile = blockIdx.x; tile < a.total_tiles; tile += gridDim.x) {
        // Which fragment of the launch, then which of its segments, holds this tile.
        int it = 0;
        if (!FLAT) {
            for (int k = 1; k < a.num_items; ++k)
                if (tile >= a.item[k].tile_off) it = k;
        }
        const DdlItem& I = a.item[it];
        const uint32_t t = tile - I.tile_off;
        const DdlSegDesc* sp;
        if (FLAT) {
            sp = &a.flat;
        } else {
            const DdlSegDesc* segs = a.segs + I.seg_begin;
            uint32_t lo = 0, hi = I.num_segs - 1;  // last segment whose tile_begin <= t
            while (lo < hi) {
                const uint32_t mid = (lo + hi + 1) >> 1;
                if (segs[mid].tile_begin <= t) lo = mid; else hi = mid - 1;
            }
            sp = segs + lo;
        }
        const uint64_t off = (uint64_t)(t - sp->tile_begin) * a.tile_elems;  // elements
        const uint64_t rem = sp->n - off;
        const uint32_t cnt = uniform(rem < a.tile_elems ? (uint32_t)rem : a.tile_elems);
        const uint64_t th = uniform(reinterpret_cast<uint64_t>(sp->theta) + off * 4);
        const uint64_t vv = uniform(reinterpret_cast<uint64_t>(sp->v) + off * 4);
        uint64_t lp[MQ];
        float w[MQ];
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            lp[j] = uniform(reinterpret_cast<uint64_t>(sp->learner[I.idx[j]]) + off * sizeof(elem));
            w[j] = I.w[j];
        }
        const float lr = I.lr, mu = I.mu;
        const bool vec_ok = uniform((uint32_t)(
            sp->base_aligned && ((I.present_bits & ~(uint32_t)sp->learner_aligned) == 0))) != 0;

        if (vec_ok) {
            const uint32_t nvec = cnt / VEC;
            uint32_t g = threadIdx.x;
            if (U > 1) {
                for (; g + (U - 1) * DDL_BLOCK < nvec; g += U * DDL_BLOCK)
                    merge_groups<L, MQ, U>(th, vv, lp, w, lr, mu, g);
            }
            for (; g < nvec; g += DDL_BLOCK) merge_groups<L, MQ, 1>(th, vv, lp, w, lr, mu, g);
            const uint32_t e = nvec * VEC + threadIdx.x;  // fewer than VEC leftover elements
            if (e < cnt) merge_scalar<L, MQ>(th, vv, lp, w, lr, mu, e);
        } else {
            for (uint32_t e = threadIdx.x; e < cnt; e += DDL_BLOCK)
                merge_scalar<L, MQ>(th, vv, lp, w, lr, mu, e);
        }
    }
}

#if DDL_BF16_VEC == 8
typedef LearnerBF16x8 LearnerBF16;
#else
typedef LearnerBF16x4 LearnerBF16;
#endif

// Plain streaming copy, 16 bytes per lane, same access pattern and cache hints as the merge
// kernel: the yardstick for what this GPU's HBM sustains and for scaling profiler counters.
__global__ void __launch_bounds__(DDL_BLOCK) ddl_copy_kernel(uint64_t dst, uint64_t src, uint64_t n16)
{
    constexpr uint32_t kPerBlock = DDL_BLOCK * 4;
    for (uint64_t base = (uint64_t)blockIdx.x * kPerBlock; base < n16;
         base += (uint64_t)gridDim.x * kPerBlock) {
        const uint64_t s = src + base * 16, d = dst + base * 16;
        const uint32_t left = n16 - base < kPerBlock ? (uint32_t)(n16 - base) : kPerBlock;
        u32x4 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i = threadIdx.x + u * DDL_BLOCK;
            if (i < left) r[u] = ld<u32x4>(s, i);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i = threadIdx.x + u * DDL_BLOCK;
            if (i < left) st<u32x4>(d, i, r[u]);
        }
    }
}

typedef void (*kernel_fn)(const DdlLaunchArgs);

template <typename L, bool FLAT>
kernel_fn pick_mq(int Mq)
{
    switch (Mq) {
#define DDL_CASE(k) case k: return ddl_merge_kernel<L, k, FLAT>;
        DDL_CASE(1) DDL_CASE(2) DDL_CASE(3) DDL_CASE(4) DDL_CASE(5) DDL_CASE(6) DDL_CASE(7)
        DDL_CASE(8) DDL_CASE(9) DDL_CASE(10) DDL_CASE(11) DDL_CASE(12) DDL_CASE(13)
        DDL_CASE(14) DDL_CASE(15) DDL_CASE(16)
#undef DDL_CASE
    }
    return nullptr;
}

}  // namespace

int ddl_launch_merge(int dtype, int Mq, bool flat, uint32_t grid, void* stream,
                     const DdlLaunchArgs& args)
{
    kernel_fn k = nullptr;
    if (dtype == 0)
        k = flat ? pick_mq<LearnerF32, true>(Mq) : pick_mq<LearnerF32, false>(Mq);
    else if (dtype == 1)
        k = flat ? pick_mq<LearnerBF16, true>(Mq) : pick_mq<LearnerBF16, false>(Mq);
    if (!k || grid == 0) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(k, dim3(grid), dim3(DDL_BLOCK), 0, static_cast<hipStream_t>(stream), args);
    return (int)hipGetLastError();
}

int ddl_launch_copy(void* dst, const void* src, uint64_t n16, uint32_t grid, void* stream)
{
    if (grid == 0) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(ddl_copy_kernel, dim3(grid), dim3(DDL_BLOCK), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<uint64_t>(dst),
                       reinterpret_cast<uint64_t>(src), n16);
    return (int)hipGetLastError();
}
