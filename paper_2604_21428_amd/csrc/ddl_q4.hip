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
// and v.  The merge is the ordinary merge kernel (ddl_kernels.hip) instantiated for a third
// kind of learner data, so it has the same tile shape, cache hints, tile rotation, split
// launches, descriptor table and optional bf16 copy of the new Theta; this file holds the
// encoder kernel and the host side: one flat fragment per call, or whole fragments of many
// tensors through a plan.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"
#include "ddl_host_internal.h"
#include "ddl_kernel_util.h"

struct DdlQ4EncodeArgs {
    uint64_t theta, learner, codes, scales;
    uint64_t n;
    uint32_t block_len;
    uint32_t num_blocks;
    uint32_t lanes_per_block;  // power of two, 2..64, lanes_per_block * 4 <= block_len
    uint32_t pad;
};

namespace {

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
    DDL_COUNT_GRID();
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
    const uint64_t blocks = (n + block_len - 1) / block_len;

    ddlh::Quorum q;
    ddlh::compact(w, M, q);
    std::vector<ddlh::Range> r;
    if (!ddlh::add_range(theta, 4, n, true, r) || !ddlh::add_range(v, 4, n, true, r))
        return DDL_ERR_INVALID_ARG;
    DdlQ4Desc qd;
    std::memset(&qd, 0, sizeof qd);
    for (int j = 0; j < q.Mq; ++j) {
        const int m = q.idx[j];
        const uint8_t* c = codes[m];
        const float* s = scales[m];
        if (!c || !s || !aligned(c, 4) || !aligned(s, 4) ||
            !ddlh::add_range(c, 1, (n + 1) / 2, false, r) || !ddlh::add_range(s, 4, blocks, false, r))
            return DDL_ERR_INVALID_ARG;
        qd.codes[m] = c;
        qd.scales[m] = s;
    }
    if (ddlh::ranges_alias(r)) return DDL_ERR_ALIAS;
    DdlSegDesc d;
    ddlh::fill_desc(d, theta, v, nullptr, nullptr, M, n, 0);
    return ddlh::launch_flat(d, DDL_SRC_Q4, q, lr, mu, hip_stream, &qd, (uint32_t)block_len);
}

// ------------------------------------------------------------------------------------------
// 4-bit sources through a plan: whole fragments of many tensors per launch
// ------------------------------------------------------------------------------------------
extern "C" ddl_status ddl_plan_set_q4_sources(ddl_plan* plan, const ddl_q4_segment* segs,
                                              size_t num_segments, size_t block_len)
{
    if (!plan || num_segments != plan->table.given_segs || (num_segments > 0 && !segs))
        return DDL_ERR_INVALID_ARG;
    if (!block_len_ok(block_len)) return DDL_ERR_INVALID_ARG;
    const ddlh::Table& T = plan->table;
    std::vector<DdlQ4Desc> table(T.segs.size());
    std::vector<uint32_t> nonnull(T.frags.size());
    std::vector<ddlh::Range> r;
    for (size_t f = 0; f < T.frags.size(); ++f) {
        const ddlh::FragInfo& fi = T.frags[f];
        nonnull[f] = (1u << fi.M) - 1u;
        for (uint32_t d = fi.seg_begin; d < fi.seg_begin + fi.num_segs; ++d) {
            const DdlSegDesc& sd = T.segs[d];
            const ddl_q4_segment& g = segs[T.origin[d]];
            if (!g.codes || !g.scales) return DDL_ERR_INVALID_ARG;
            // the kernel takes Theta and v of such tensors in 128-bit accesses only
            if (!sd.base_aligned) return DDL_ERR_INVALID_ARG;
            const uint64_t blocks = (sd.n + block_len - 1) / block_len;
            if (!ddlh::add_range(sd.theta, 4, sd.n, true, r) ||
                !ddlh::add_range(sd.v, 4, sd.n, true, r) ||
                (sd.theta_bf16 && !ddlh::add_range(sd.theta_bf16, 2, sd.n, true, r)))
                return DDL_ERR_INVALID_ARG;
            DdlQ4Desc& q = table[d];
            std::memset(&q, 0, sizeof q);
            for (int m = 0; m < fi.M; ++m) {
                const uint8_t* c = g.codes[m];
                const float* s = g.scales[m];
                if (!c || !s) {  // a learner without sources here cannot contribute
                    if (c || s) return DDL_ERR_INVALID_ARG;
                    nonnull[f] &= ~(1u << m);
                    continue;
                }
                if (!aligned(c, 4) || !aligned(s, 4) ||
                    !ddlh::add_range(c, 1, (sd.n + 1) / 2, false, r) ||
                    !ddlh::add_range(s, 4, blocks, false, r))
                    return DDL_ERR_INVALID_ARG;
                q.codes[m] = c;
                q.scales[m] = s;
            }
        }
    }
    if (ddlh::ranges_alias(r)) return DDL_ERR_ALIAS;
    void* dev = nullptr;
    if (!table.empty()) {
        const size_t bytes = table.size() * sizeof(DdlQ4Desc);
        hipError_t e = hipMalloc(&dev, bytes);
        if (e == hipSuccess) e = hipMemcpy(dev, table.data(), bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            if (dev) (void)hipFree(dev);
            return ddlh::runtime_error(e, "q4 source table upload");
        }
    }
    if (plan->d_q4) (void)hipFree(plan->d_q4);
    plan->d_q4 = dev;
    plan->q4_host = table;
    plan->q4_block_len = (uint32_t)block_len;
    plan->q4_nonnull_bits = nonnull;
    return DDL_OK;
}

extern "C" ddl_status ddl_plan_q4_merge(ddl_plan* plan, const ddl_sync* syncs, int count,
                                        void* hip_stream)
{
    if (!plan || plan->q4_block_len == 0 || count < 0 || (count > 0 && !syncs))
        return DDL_ERR_INVALID_ARG;
    if (count == 0) return DDL_OK;
    const ddlh::Table& T = plan->table;
    std::vector<ddlh::Work> work;
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
        ddlh::Work wk;
        wk.frag = (uint32_t)s.fragment;
        wk.lr = s.lr;
        wk.mu = s.mu;
        ddlh::compact(w, f.M, wk.q);
        if (f.num_segs > 0 && (wk.q.present_bits & ~plan->q4_nonnull_bits[(size_t)s.fragment]))
            return DDL_ERR_INVALID_ARG;
        work.push_back(wk);
    }
    const ddlh::Q4Source q4 = {static_cast<const DdlQ4Desc*>(plan->d_q4), plan->q4_block_len};
    return ddlh::launch_work(T, plan->d_table, work, hip_stream, &q4);
}
