// ddl_merge_fragment_ex: the sync of one flat fragment that also hands out the merged outer
// gradient Delta = sum_m w_m (Theta - theta_m) (Appendix D.2, weighted direct averaging) it
// applied -- for inspection (norms and cosines of outer gradients, checks of a caller's own
// optimiser) without a second pass over the learners' copies.  Theta and v come out bit for bit
// as from ddl_merge_fragment: the per-element arithmetic below is the same FMA chain in the
// same order.  The kernel has the merge kernel's shape (one group of four per lane, tiles of
// 1024 elements, non-temporal buffer loads, streamed stores, tile rotation, residency cap, long
// fragments cut into equal grids); everything it needs travels in its argument block.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"
#include "ddl_host_internal.h"
#include "ddl_kernel_util.h"

struct DdlDeltaArgs {
    uint64_t theta, v, delta;    // n fp32 each
    uint64_t learner[DDL_MAXL];  // compacted: entry j is contributing learner j's copy
    uint64_t n;
    uint32_t tile_base;  // first tile this grid covers
    uint32_t total_tiles;
    uint32_t rotate;   // tile rotation group (0: off)
    uint32_t aligned;  // every array 16-byte aligned: full tiles take the vector path
    float w[DDL_MAXL];
    float lr, mu;
};

namespace {

// One element; the same operations in the same order as outer_step, plus Delta itself.
template <int MQ>
__device__ __forceinline__ void outer_step_delta(float& theta, float& v, float& delta,
                                                 const float (&x)[MQ], const float (&w)[MQ],
                                                 float lr, float mu)
{
    float d = 0.0f;
#pragma unroll
    for (int j = 0; j < MQ; ++j) d = fmaf(w[j], theta - x[j], d);
    const float v_new = fmaf(mu, v, d);
    theta = fmaf(-lr, fmaf(mu, v_new, d), theta);
    v = v_new;
    delta = d;
}

template <typename L, int MQ>
__global__ void __launch_bounds__(DDL_BLOCK) ddl_merge_delta_kernel(const DdlDeltaArgs a)
{
    typedef typename L::elem elem;
    const uint32_t tile = a.tile_base + rotate_tile(blockIdx.x, gridDim.x, a.rotate);
    const uint64_t first = (uint64_t)tile * DDL_TILE;
    const uint64_t left = a.n - first;  // > 0: the grid covers exactly the tiles that exist
    const uint64_t th = uniform(a.theta + first * 4), vv = uniform(a.v + first * 4);
    const uint64_t dd = uniform(a.delta + first * 4);
    uint64_t lp[MQ];
    float w[MQ];
#pragma unroll
    for (int j = 0; j < MQ; ++j) {
        lp[j] = uniform(a.learner[j] + first * sizeof(elem));
        w[j] = a.w[j];
    }
    const float lr = a.lr, mu = a.mu;
    if (a.aligned && left >= DDL_TILE) {
        const uint32_t g = threadIdx.x;
        typename L::raw raw[MQ];
#pragma unroll
        for (int j = 0; j < MQ; ++j) raw[j] = ld<typename L::raw, DDL_NT_LOAD>(lp[j], g);
        const f32x4 T = ld<f32x4, DDL_NT_LOAD>(th, g);
        const f32x4 V = ld<f32x4, DDL_NT_LOAD>(vv, g);
        float x[MQ][4];
#pragma unroll
        for (int j = 0; j < MQ; ++j) L::widen(raw[j], x[j]);
        float t4[4] = {T.x, T.y, T.z, T.w};
        float v4[4] = {V.x, V.y, V.z, V.w};
        float d4[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float xe[MQ];
#pragma unroll
            for (int j = 0; j < MQ; ++j) xe[j] = x[j][k];
            outer_step_delta<MQ>(t4[k], v4[k], d4[k], xe, w, lr, mu);
        }
        st<f32x4>(th, g, f32x4{t4[0], t4[1], t4[2], t4[3]});
        st<f32x4>(vv, g, f32x4{v4[0], v4[1], v4[2], v4[3]});
        st<f32x4>(dd, g, f32x4{d4[0], d4[1], d4[2], d4[3]});
    } else {  // a ragged last tile, or bases that are not all 16-byte aligned
        const uint32_t cnt = left < DDL_TILE ? (uint32_t)left : DDL_TILE;
        DDL_GLOBAL float* tp = reinterpret_cast<DDL_GLOBAL float*>(th);
        DDL_GLOBAL float* vp = reinterpret_cast<DDL_GLOBAL float*>(vv);
        DDL_GLOBAL float* dp = reinterpret_cast<DDL_GLOBAL float*>(dd);
        for (uint32_t e = threadIdx.x; e < cnt; e += DDL_BLOCK) {
            float xe[MQ];
#pragma unroll
            for (int j = 0; j < MQ; ++j)
                xe[j] = L::widen1(reinterpret_cast<const DDL_GLOBAL elem*>(lp[j])[e]);
            float t = tp[e], v = vp[e], d;
            outer_step_delta<MQ>(t, v, d, xe, w, lr, mu);
            tp[e] = t;
            vp[e] = v;
            dp[e] = d;
        }
    }
}

typedef void (*delta_fn)(const DdlDeltaArgs);

template <typename L>
delta_fn pick_mq(int Mq)
{
    switch (Mq) {
#define DDL_CASE(k) case k: return ddl_merge_delta_kernel<L, k>;
        DDL_CASE(1) DDL_CASE(2) DDL_CASE(3) DDL_CASE(4) DDL_CASE(5) DDL_CASE(6) DDL_CASE(7)
        DDL_CASE(8) DDL_CASE(9) DDL_CASE(10) DDL_CASE(11) DDL_CASE(12) DDL_CASE(13)
        DDL_CASE(14) DDL_CASE(15) DDL_CASE(16)
#undef DDL_CASE
    }
    return nullptr;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

extern "C" ddl_status ddl_merge_fragment_ex(float* theta, float* v, float* delta_out,
                                            const void* const* learner_params,
                                            ddl_dtype learner_dtype, const uint64_t* token_counts,
                                            const uint8_t* quorum_mask, int M, size_t n, float lr,
                                            float mu, void* hip_stream)
{
    using namespace ddlh;
    if (!delta_out)
        return ddl_merge_fragment(theta, v, learner_params, learner_dtype, token_counts,
                                  quorum_mask, M, n, lr, mu, hip_stream);
    double wd[DDL_MAXL];
    const ddl_status ws = weights_tokens(token_counts, quorum_mask, M, wd);
    if (ws != DDL_OK) return ws;
    if (learner_dtype != DDL_F32 && learner_dtype != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (!finite_nonneg(lr) || !finite_nonneg(mu)) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!learner_params || !theta || !v) return DDL_ERR_INVALID_ARG;
    Quorum q;
    compact(wd, M, q);
    const size_t eb = learner_dtype == DDL_BF16 ? 2 : 4;
    if (((uintptr_t)theta | (uintptr_t)v | (uintptr_t)delta_out) & 3) return DDL_ERR_INVALID_ARG;
    std::vector<Range> ranges;
    if (!add_range(theta, 4, n, true, ranges) || !add_range(v, 4, n, true, ranges) ||
        !add_range(delta_out, 4, n, true, ranges))
        return DDL_ERR_INVALID_ARG;
    DdlDeltaArgs a = {};
    bool vec = aligned16(theta) && aligned16(v) && aligned16(delta_out);
    for (int j = 0; j < q.Mq; ++j) {
        const void* p = learner_params[q.idx[j]];
        if (!p || ((uintptr_t)p & (eb - 1)) || !add_range(p, eb, n, false, ranges))
            return DDL_ERR_INVALID_ARG;
        vec = vec && aligned16(p);
        a.learner[j] = reinterpret_cast<uint64_t>(p);
        a.w[j] = q.w[j];
    }
    if (ranges_alias(ranges)) return DDL_ERR_ALIAS;
    const uint64_t tiles = ((uint64_t)n + DDL_TILE - 1) / DDL_TILE;
    if (tiles > 0x7fffffffull) return DDL_ERR_INVALID_ARG;

    a.theta = reinterpret_cast<uint64_t>(theta);
    a.v = reinterpret_cast<uint64_t>(v);
    a.delta = reinterpret_cast<uint64_t>(delta_out);
    a.n = n;
    a.total_tiles = (uint32_t)tiles;
    a.rotate = tile_rotate();
    a.aligned = vec;
    a.lr = lr;
    a.mu = mu;
    const delta_fn k = learner_dtype == DDL_BF16 ? pick_mq<LearnerBF16>(q.Mq)
                                                 : pick_mq<LearnerF32>(q.Mq);
    if (!k) return DDL_ERR_INVALID_ARG;
    // Equal grids of whole rotation groups, as for the merge kernel; Delta adds 4 bytes per
    // element to a part's traffic.
    const uint32_t max_tiles = max_tiles_per_launch((int)eb, q.Mq, 4);
    uint64_t part = tiles;
    if (max_tiles != 0 && tiles > max_tiles) {
        const uint64_t parts = (tiles + max_tiles - 1) / max_tiles;
        const uint64_t unit = a.rotate > 0 ? a.rotate : 1u;
        part = ((tiles + parts - 1) / parts + unit - 1) / unit * unit;
    }
    const uint32_t lds = merge_lds_cap_bytes((int)eb, q.Mq);
    for (uint64_t base = 0; base < tiles; base += part) {
        a.tile_base = (uint32_t)base;
        const uint32_t grid = (uint32_t)std::min<uint64_t>(part, tiles - base);
        DDL_COUNT_GRID();
        hipLaunchKernelGGL(k, dim3(grid), dim3(DDL_BLOCK), lds, static_cast<hipStream_t>(hip_stream),
                           a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return runtime_error(e, "merge (with Delta) kernel launch");
    }
    return DDL_OK;
}
