// 4-bit outer gradients (Appendix D.3 of the paper, "Outer gradients compression": the outer
// gradients are compressed from bf16 to int4 before the merge).  The paper fixes only the
// width; the format here is a plain symmetric block-wise integer quantiser:
//
//   * the flat fragment is cut into blocks of `block_len` consecutive elements;
//   * block b of learner m has one fp32 scale s; element i has a signed 4-bit code q in
//     two's complement, two per byte, element 2k in the low nibble of byte k;
//   * the pair stands for the outer gradient value s * q.
//
// Encoder (the learner side of the wire): d = Theta - theta_m in fp32, s = max|d| / 7 over
// the block, q = round-half-even(d / s) clamped to [-7, 7]; IEEE division, so the codes are
// reproducible bit for bit.
// Merge (the syncer side): Delta_i = sum_j w_j s_j q_ji, then the same fused outer Nesterov
// step as the bf16 path.  Per element it reads Mq / 2 bytes of codes instead of 2 Mq bytes of
// bf16 parameters, so the pass approaches the 16 B/param of the read-modify-write of Theta
// and v.  Same tile shape and cache hints as the bf16 merge kernel: 1024 elements per
// workgroup, one group of four per lane, every tensor access non-temporal.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"
#include "ddl_host_internal.h"
#include "ddl_kernel_util.h"

struct DdlQ4Args {
    uint64_t theta, v;          // device addresses, 16-byte aligned
    uint64_t codes[DDL_MAXL];   // contributing learners only, compacted
    uint64_t scales[DDL_MAXL];
    float w[DDL_MAXL];
    uint64_t n;
    uint32_t block_len;         // multiple of 8
    uint32_t block_shift;       // log2(block_len) if it is a power of two, else 0xffffffff
    float lr, mu;
    uint32_t rotate;            // group size of the tile rotation, 0: off
    uint32_t pad;
};

struct DdlQ4EncodeArgs {
    uint64_t theta, learner, codes, scales;
    uint64_t n;
    uint32_t block_len;
    uint32_t num_blocks;
    uint32_t lanes_per_block;  // power of two, 2..64, lanes_per_block * 4 <= block_len
    uint32_t pad;
};

namespace {

// Signed value of nibble k (0..3) of a 16-bit group of four codes.
__device__ __forceinline__ float nibble(uint32_t c, int k)
{
    return (float)((int32_t)(c << (28 - 4 * k)) >> 28);
}

template <int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) q4_merge_kernel(const DdlQ4Args a)
{
    const uint64_t e0 =                                        // first element of the tile
        (uint64_t)rotate_tile(blockIdx.x, gridDim.x, a.rotate) * DDL_TILE;
    const uint64_t left = a.n - e0;                            // > 0 by the grid size
    const uint32_t cnt = left < DDL_TILE ? (uint32_t)left : DDL_TILE;
    const uint32_t i0 = threadIdx.x * 4;                       // this lane's elements in the tile
    if (i0 >= cnt) return;
    const uint64_t th = a.theta + e0 * 4, vv = a.v + e0 * 4;

    // block of the lane's first element; a group of four never straddles a block
    const uint64_t blk0 = e0 / a.block_len;
    const uint32_t off = (uint32_t)(e0 - blk0 * a.block_len) + i0;
    const uint64_t blk =
        blk0 + (a.block_shift != 0xffffffffu ? off >> a.block_shift : off / a.block_len);

    float sw[MQ];  // w_j * s_j for this lane's block
#pragma unroll
    for (int j = 0; j < MQ; ++j)
        sw[j] = a.w[j] * *(reinterpret_cast<const DDL_GLOBAL float*>(a.scales[j]) + blk);
    const float lr = a.lr, mu = a.mu;

    if (i0 + 4 <= cnt) {
        uint32_t c[MQ];
#pragma unroll
        for (int j = 0; j < MQ; ++j) c[j] = ld<uint16_t, true>(a.codes[j] + e0 / 2, threadIdx.x);
        const f32x4 T = ld<f32x4, true>(th, threadIdx.x);
        const f32x4 V = ld<f32x4, true>(vv, threadIdx.x);
        float t4[4] = {T.x, T.y, T.z, T.w};
        float v4[4] = {V.x, V.y, V.z, V.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float delta = 0.0f;
#pragma unroll
            for (int j = 0; j < MQ; ++j) delta = fmaf(sw[j], nibble(c[j], k), delta);
            v4[k] = fmaf(mu, v4[k], delta);
            t4[k] = fmaf(-lr, fmaf(mu, v4[k], delta), t4[k]);
        }
        const f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
        const f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
        st<f32x4>(th, threadIdx.x, tn);
        st<f32x4>(vv, threadIdx.x, vn);
    } else {  // the last one to three elements of the tensor
        for (uint32_t e = i0; e < cnt; ++e) {
            const uint64_t i = e0 + e;
            float delta = 0.0f;
#pragma unroll
            for (int j = 0; j < MQ; ++j) {
                const uint32_t byte =
                    *(reinterpret_cast<const DDL_GLOBAL uint8_t*>(a.codes[j]) + i / 2);
                delta = fmaf(sw[j], nibble(byte, (int)(i & 1)), delta);
            }
            const float t = *(reinterpret_cast<const DDL_GLOBAL float*>(th) + e);
            const float v = *(reinterpret_cast<const DDL_GLOBAL float*>(vv) + e);
            const float v_new = fmaf(mu, v, delta);
            *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = fmaf(-lr, fmaf(mu, v_new, delta), t);
            *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v_new;
        }
    }
}

// Encoder: a group of `lanes_per_block` lanes (a power of two, at most a wavefront) per block;
// a wavefront holds 64 / lanes_per_block blocks side by side.  The lanes of a group walk their
// block in chunks of four elements (one 16-bit word of codes), first for the block's largest
// magnitude (combined by lane shuffles within the group), then again to quantise (the second
// walk finds the block in the cache).
template <typename L>
__global__ void __launch_bounds__(DDL_BLOCK) q4_encode_kernel(const DdlQ4EncodeArgs a)
{
    typedef typename L::elem elem;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lpb = a.lanes_per_block;
    const uint64_t wave = (uint64_t)blockIdx.x * (DDL_BLOCK / 64) + (threadIdx.x >> 6);
    const uint64_t b = wave * (64 / lpb) + lane / lpb;
    const uint32_t gl = lane & (lpb - 1);  // lane within its group
    // Lanes whose block does not exist keep len = 0: they skip both walks but still take part
    // in the shuffles, which every lane of the wavefront reaches.
    const bool active = b < a.num_blocks;
    const uint64_t b0 = active ? b * a.block_len : 0;
    const uint32_t len = !active ? 0u : a.n - b0 < a.block_len ? (uint32_t)(a.n - b0) : a.block_len;
    const uint32_t chunks = (len + 3) / 4;
    const DDL_GLOBAL float* th = reinterpret_cast<const DDL_GLOBAL float*>(a.theta) + b0;
    const DDL_GLOBAL elem* lp = reinterpret_cast<const DDL_GLOBAL elem*>(a.learner) + b0;

    auto diffs = [&](uint32_t c, float (&d)[4]) {  // outer gradients of chunk c, 0 past the end
        const uint32_t e = c * 4;
        if (e + 4 <= len) {
            const f32x4 t = *reinterpret_cast<const DDL_GLOBAL f32x4*>(th + e);
            const typename L::raw r = *reinterpret_cast<const DDL_GLOBAL typename L::raw*>(lp + e);
            float x[4];
            L::widen(r, x);
            d[0] = t.x - x[0];
            d[1] = t.y - x[1];
            d[2] = t.z - x[2];
            d[3] = t.w - x[3];
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                d[k] = e + k < len ? th[e + k] - L::widen1(lp[e + k]) : 0.0f;
        }
    };

    float amax = 0.0f;
    for (uint32_t c = gl; c < chunks; c += lpb) {
        float d[4];
        diffs(c, d);
#pragma unroll
        for (int k = 0; k < 4; ++k) amax = fmaxf(amax, fabsf(d[k]));
    }
    for (uint32_t o = lpb >> 1; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, (int)o, 64));
    const float s = __fdiv_rn(amax, 7.0f);
    if (active && gl == 0) *(reinterpret_cast<DDL_GLOBAL float*>(a.scales) + b) = s;

    for (uint32_t c = gl; c < chunks; c += lpb) {
        float d[4];
        diffs(c, d);
        uint32_t word = 0;
        if (s > 0.0f) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float r = rintf(__fdiv_rn(d[k], s));  // to nearest, ties to even
                r = fminf(fmaxf(r, -7.0f), 7.0f);
                word |= ((uint32_t)(int32_t)r & 0xfu) << (4 * k);
            }
        }
        const uint64_t e = b0 + (uint64_t)c * 4;  // a multiple of four: byte e / 2
        if (c * 4 + 4 <= len) {
            *(reinterpret_cast<DDL_GLOBAL uint16_t*>(a.codes) + e / 4) = (uint16_t)word;
        } else {  // the tensor's last, partial chunk: only the bytes that exist
            const uint32_t bytes = (len - c * 4 + 1) / 2;
            for (uint32_t k = 0; k < bytes; ++k)
                *(reinterpret_cast<DDL_GLOBAL uint8_t*>(a.codes) + e / 2 + k) =
                    (uint8_t)(word >> (8 * k));
        }
    }
}

typedef void (*q4_fn)(const DdlQ4Args);

q4_fn pick_q4(int Mq)
{
    switch (Mq) {
#define DDL_CASE(q) \
    case q: return q4_merge_kernel<q>;
        DDL_CASE(1) DDL_CASE(2) DDL_CASE(3) DDL_CASE(4) DDL_CASE(5) DDL_CASE(6) DDL_CASE(7)
        DDL_CASE(8) DDL_CASE(9) DDL_CASE(10) DDL_CASE(11) DDL_CASE(12) DDL_CASE(13)
        DDL_CASE(14) DDL_CASE(15) DDL_CASE(16)
#undef DDL_CASE
    }
    return nullptr;
}

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

bool block_len_ok(size_t block_len)
{
    return block_len >= 8 && block_len % 8 == 0 && block_len <= 0x40000000u;
}

}  // namespace

extern "C" ddl_status ddl_q4_encode(const float* theta, const void* learner_params,
                                    ddl_dtype learner_dtype, size_t n, size_t block_len,
                                    uint8_t* codes_out, float* scales_out, void* hip_stream)
{
    if (learner_dtype != DDL_F32 && learner_dtype != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (!block_len_ok(block_len)) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!theta || !learner_params || !codes_out || !scales_out || !aligned(theta, 16) ||
        !aligned(learner_params, 16) || !aligned(codes_out, 4) || !aligned(scales_out, 4))
        return DDL_ERR_INVALID_ARG;
    const uint64_t blocks = (n + block_len - 1) / block_len;
    if (blocks > 0x7fffffffull) return DDL_ERR_INVALID_ARG;
    const size_t b = learner_dtype == DDL_BF16 ? 2 : 4;
    // outputs may overlap nothing
    const uintptr_t lo[4] = {(uintptr_t)codes_out, (uintptr_t)scales_out, (uintptr_t)theta,
                             (uintptr_t)learner_params};
    const uintptr_t hi[4] = {lo[0] + (n + 1) / 2, lo[1] + 4 * blocks, lo[2] + 4 * n, lo[3] + b * n};
    for (int o = 0; o < 2; ++o)
        for (int x = 0; x < 4; ++x)
            if (x != o && lo[o] < hi[x] && lo[x] < hi[o]) return DDL_ERR_ALIAS;

    DdlQ4EncodeArgs a;
    std::memset(&a, 0, sizeof a);
    a.theta = (uint64_t)(uintptr_t)theta;
    a.learner = (uint64_t)(uintptr_t)learner_params;
    a.codes = (uint64_t)(uintptr_t)codes_out;
    a.scales = (uint64_t)(uintptr_t)scales_out;
    a.n = n;
    a.block_len = (uint32_t)block_len;
    a.num_blocks = (uint32_t)blocks;
    a.lanes_per_block = 2;  // block_len >= 8
    while (a.lanes_per_block < 64 && (size_t)a.lanes_per_block * 8 <= block_len)
        a.lanes_per_block *= 2;
    const uint64_t per_wave = 64 / a.lanes_per_block;
    const uint64_t waves = (blocks + per_wave - 1) / per_wave;
    const dim3 grid((uint32_t)((waves + DDL_BLOCK / 64 - 1) / (DDL_BLOCK / 64))), block(DDL_BLOCK);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (learner_dtype == DDL_F32)
        hipLaunchKernelGGL(q4_encode_kernel<LearnerF32>, grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL(q4_encode_kernel<LearnerBF16>, grid, block, 0, stream, a);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? DDL_OK : ddlh::runtime_error(e, "q4 encode kernel launch");
}

extern "C" ddl_status ddl_q4_merge_fragment(float* theta, float* v, const uint8_t* const* codes,
                                            const float* const* scales,
                                            const uint64_t* token_counts,
                                            const uint8_t* quorum_mask, int M, size_t n,
                                            size_t block_len, float lr, float mu, void* hip_stream)
{
    double w[DDL_MAXL];
    const ddl_status st = ddlh::weights_tokens(token_counts, quorum_mask, M, w);
    if (st != DDL_OK) return st;
    if (!ddlh::finite_nonneg(lr) || !ddlh::finite_nonneg(mu)) return DDL_ERR_INVALID_ARG;
    if (!block_len_ok(block_len)) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!theta || !v || !codes || !scales || !aligned(theta, 16) || !aligned(v, 16))
        return DDL_ERR_INVALID_ARG;
    const uint64_t tiles = (n + DDL_TILE - 1) / DDL_TILE;
    if (tiles > 0x7fffffffull) return DDL_ERR_INVALID_ARG;
    const uint64_t blocks = (n + block_len - 1) / block_len;

    ddlh::Quorum q;
    ddlh::compact(w, M, q);
    DdlQ4Args a;
    std::memset(&a, 0, sizeof a);
    const uintptr_t out_lo[2] = {(uintptr_t)theta, (uintptr_t)v};
    if (out_lo[0] < out_lo[1] + 4 * n && out_lo[1] < out_lo[0] + 4 * n) return DDL_ERR_ALIAS;
    for (int j = 0; j < q.Mq; ++j) {
        const uint8_t* c = codes[q.idx[j]];
        const float* s = scales[q.idx[j]];
        if (!c || !s || !aligned(c, 4) || !aligned(s, 4)) return DDL_ERR_INVALID_ARG;
        const uintptr_t in_lo[2] = {(uintptr_t)c, (uintptr_t)s};
        const uintptr_t in_hi[2] = {in_lo[0] + (n + 1) / 2, in_lo[1] + 4 * blocks};
        for (int o = 0; o < 2; ++o)
            for (int x = 0; x < 2; ++x)
                if (out_lo[o] < in_hi[x] && in_lo[x] < out_lo[o] + 4 * n) return DDL_ERR_ALIAS;
        a.codes[j] = (uint64_t)in_lo[0];
        a.scales[j] = (uint64_t)in_lo[1];
        a.w[j] = q.w[j];
    }
    a.theta = (uint64_t)out_lo[0];
    a.v = (uint64_t)out_lo[1];
    a.n = n;
    a.block_len = (uint32_t)block_len;
    a.block_shift = 0xffffffffu;
    if ((block_len & (block_len - 1)) == 0) {
        a.block_shift = 0;
        while (((size_t)1 << a.block_shift) < block_len) ++a.block_shift;
    }
    a.lr = lr;
    a.mu = mu;
    a.rotate = ddlh::tile_rotate();
    const q4_fn fn = pick_q4(q.Mq);
    if (!fn) return DDL_ERR_INVALID_ARG;
    hipLaunchKernelGGL(fn, dim3((uint32_t)tiles), dim3(DDL_BLOCK), ddlh::merge_lds_cap_bytes(0, q.Mq),
                       static_cast<hipStream_t>(hip_stream), a);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? DDL_OK : ddlh::runtime_error(e, "q4 merge kernel launch");
}
