// Device-side helpers shared by the gfx950 kernels of libddlsync: explicit address-space
// accesses with cache hints, scalar-register broadcast, bf16 widening and rounding, and the
// per-element outer step.  Everything is in an unnamed namespace: each kernel file gets its
// own inlined copy.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Load form of the streaming merge kernels (see ld<> below): 2 = raw buffer load with "nt".
// The buffer form of the same non-temporal load measured faster than the global form on
// MI355X: moe (11 learner streams) +1.7 %, large_dense +0.7 %, a 243 M-parameter block +0.4 %,
// dense_block equal; adding "sc1" or "sc0 sc1" to the loads changes nothing.
#ifndef DDL_NT_LOAD
#define DDL_NT_LOAD 2
#endif
#ifndef DDL_NT_STATE_LOAD
#define DDL_NT_STATE_LOAD DDL_NT_LOAD
#endif

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// All tensor accesses go through explicit global-address-space pointers built from a
// 64-bit base held in scalar registers plus a 32-bit per-lane index.
#define DDL_GLOBAL __attribute__((address_space(1)))
#define DDL_CONST __attribute__((address_space(4)))

__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(uint64_t base)
{
    // stride 0, no range limit below 4 GiB past the base, 32-bit raw data format
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(base), 0, -1, 0x00020000);
}

// POLICY 0: ordinary cached load; 1: non-temporal global load; any other value: raw buffer
// load with that value as its cache-policy bits (bit 0 sc0, bit 1 nt, bit 4 sc1).
template <typename T, int POLICY>
__device__ __forceinline__ T ld(uint64_t base, uint32_t index)
{
    if constexpr (POLICY == 0 || POLICY == 1) {
        const DDL_GLOBAL T* p = reinterpret_cast<const DDL_GLOBAL T*>(base) + index;
        if (POLICY == 1) return __builtin_nontemporal_load(p);
        return *p;
    } else {
        const uint32_t off = index * (uint32_t)sizeof(T);
        if constexpr (sizeof(T) == 16)
            return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b128(raw_buffer(base), off, 0, POLICY));
        else if constexpr (sizeof(T) == 8)
            return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b64(raw_buffer(base), off, 0, POLICY));
        else
            return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b16(raw_buffer(base), off, 0, POLICY));
    }
}

// Streaming stores carry explicit cache-policy bits: "nt" (streamed through L2, first to be
// evicted) and "sc1" (agent scope: written through to memory instead of waiting in this XCD's
// L2 for a later write-back).  Measured on MI355X against the plain non-temporal store:
// +1.2 % on dense_block, +0.9 % on a 243 M-parameter block, +0.3 % on large_dense, moe equal;
// "sc1" or "sc0 sc1" without "nt" lose 1-5 %.  Global stores cannot be given these bits from
// C++, raw buffer stores can: the store goes through a buffer resource made on the spot from
// the (block-uniform) base, with the index as a 32-bit byte offset.  The compiler knows the
// instruction, so wait counts and the store-data hazard stay its business.
#ifndef DDL_STORE_AUX
#define DDL_STORE_AUX 0x12  // bit 1: nt, bit 4: sc1 (bit 0 would be sc0)
#endif
template <typename T>
__device__ __forceinline__ void st(uint64_t base, uint32_t index, T x)
{
    static_assert(sizeof(T) == 16 || sizeof(T) == 8, "vector stores only");
    const uint32_t off = index * (uint32_t)sizeof(T);
    if constexpr (sizeof(T) == 16)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x), raw_buffer(base), off, 0,
                                               DDL_STORE_AUX);
    else
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, x), raw_buffer(base), off, 0,
                                              DDL_STORE_AUX);
}

// Values that are the same for every lane of a workgroup (tile geometry, base addresses) are
// moved to scalar registers explicitly, so that sixteen 64-bit learner addresses do not sit
// in vector registers of every lane.
__device__ __forceinline__ uint32_t uniform(uint32_t x)
{
    return __builtin_amdgcn_readfirstlane(x);
}
__device__ __forceinline__ uint64_t uniform(uint64_t x)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// Which tile (or row) workgroup b of a grid of `total` takes.  Workgroups are handed to the
// eight XCDs round-robin, so with the identity mapping XCD x works on tiles x, x + 8, ... only:
// always the same residues of the address interleave, hence the same memory channels, for
// every array at once when the arrays' bases are aligned alike (tensors of power-of-two sizes
// allocated back to back).  Rotating the index within each group of k consecutive tiles by
// the group's number lets every XCD sweep all residues, while the tiles in flight stay one
// compact window.  k = 0: identity.  A last, partial group keeps the identity.
__device__ __forceinline__ uint32_t rotate_tile(uint32_t b, uint32_t total, uint32_t k)
{
    if (k == 0) return b;
    const uint32_t g = b / k, r = b - g * k;
    return (g + 1) * k <= total ? g * k + (r + g) % k : b;
}

// bf16 is the upper half of an fp32 word, so widening is a shift or a mask.
__device__ __forceinline__ float bf16_even(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_odd(uint32_t pair)
{
    return __uint_as_float(pair & 0xffff0000u);
}

// Learner element types: `raw` is the register image of the four elements a lane loads.
struct LearnerF32 {
    typedef float elem;
    typedef u32x4 raw;
    static __device__ __forceinline__ void widen(const raw& r, float (&x)[4])
    {
        x[0] = __uint_as_float(r.x);
        x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z);
        x[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ float widen1(float e) { return e; }
};

struct LearnerBF16 {
    typedef uint16_t elem;
    typedef u32x2 raw;
    static __device__ __forceinline__ void widen(const raw& r, float (&x)[4])
    {
        x[0] = bf16_even(r.x);
        x[1] = bf16_odd(r.x);
        x[2] = bf16_even(r.y);
        x[3] = bf16_odd(r.y);
    }
    static __device__ __forceinline__ float widen1(uint16_t e)
    {
        return __uint_as_float((uint32_t)e << 16);
    }
};

// 4-bit outer gradients: `raw` holds the four codes of a lane's group of four elements, and
// what is widened is the code itself (-8 .. 7); the block's scale is folded into the weight.
struct LearnerQ4 {
    typedef uint8_t elem;  // two elements per byte
    typedef uint16_t raw;
    // signed value of nibble k (0 .. 3) of a group of codes
    static __device__ __forceinline__ float nibble(uint32_t c, int k)
    {
        return (float)((int32_t)(c << (28 - 4 * k)) >> 28);
    }
    static __device__ __forceinline__ void widen(const raw& r, float (&x)[4])
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = nibble(r, k);
    }
};
template <typename L> struct IsQ4 { static constexpr bool value = false; };
template <> struct IsQ4<LearnerQ4> { static constexpr bool value = true; };

// fp32 -> bf16, round to nearest, ties to even; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// One element: Delta = sum_j w_j (Theta - x_j); v' = mu v + Delta;
// Theta' = Theta - lr (Delta + mu v').  The difference form keeps the fp32 rounding of the
// weights (their sum is 1 only to ~1e-7) away from |Theta|.  GRAD: the x_j are the learners'
// outer gradients themselves (already Theta - theta_j), so Delta = sum_j w_j x_j.
template <int MQ, bool GRAD = false>
__device__ __forceinline__ void outer_step(float& theta, float& v, const float (&x)[MQ],
                                           const float (&w)[MQ], float lr, float mu)
{
    float delta = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) delta = fmaf(w[j], GRAD ? x[j] : theta - x[j], delta);
    const float v_new = fmaf(mu, v, delta);
    theta = fmaf(-lr, fmaf(mu, v_new, delta), theta);
    v = v_new;
}

}  // namespace
