// gfx950 kernels of the synchronizer hot path: weighted merge of the contributing learners'
// copies into the outer gradient, fused with the outer Nesterov-momentum step (Algorithm 2,
// steps "mergeFn" and "OuterOpt"; Appendix D.2, weighted direct averaging).
//
// The work is a streaming reduction with no reuse: per element it reads Mq learner values
// (2 or 4 bytes each) plus Theta and v, and writes Theta and v -- about 0.7 flop per byte --
// so the kernel is organised around HBM, not around the ALUs:
//   * the unit of work is a tile of DDL_TILE = 1024 consecutive elements, one group of four
//     elements per lane: every wave-wide access is one contiguous run (1 KiB of Theta, v or
//     an fp32 learner, 512 B of a bf16 learner), and the tiles in flight across the chip at
//     any moment form one compact address window per array, which is what keeps DRAM pages
//     open.  Measured on MI355X, this beats wider per-lane groups, deeper unrolling and
//     persistent grids, all of which widen that window;
//   * workgroup b takes tile rotate_tile(b): consecutive workgroups land on different XCDs, and
//     without the rotation each XCD would keep hitting the same memory channels (+6-8 % on
//     tensors of power-of-two sizes);
//   * a workgroup walks `tiles_per_block` consecutive tiles, so the tile -> tensor lookup
//     (scalar loads from the descriptor table, addressed as constant memory) is paid once
//     per run of tiles, not once per tile;
//   * weights, learner selection, lr and mu come from the kernel argument block (scalar
//     loads into SGPRs); absent learners do not appear in it and are never addressed;
//   * every access is non-temporal: each byte is touched once per sync, and mixing cached
//     and streaming accesses to Theta and v costs 10-20 %;
//   * Delta, the new v and the new Theta stay in registers; Theta and v are read once and
//     written once.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "ddl_device.h"

#ifndef DDL_Q4_CODE_LOAD
#define DDL_Q4_CODE_LOAD DDL_NT_LOAD  // load form of the 2-byte groups of 4-bit codes (see ld<>)
#endif
#ifndef DDL_PAIR
#define DDL_PAIR 0  // 1: issue the loads of two consecutive tiles before the first use
#endif

#include "ddl_kernel_util.h"

namespace {

// Where the learners' data of a run of tiles is.  bf16 / fp32 learners: lp[j] is learner j's
// array at the run's first element.  4-bit outer gradients: lp[j] is learner j's codes there
// (half a byte per element; a run starts at a multiple of 1024 elements), sc[j] its scales at
// the block that holds the run's first element, and rem0 that element's position within its
// block; a lane's group of four never straddles a block (block_len is a multiple of 8).
template <int MQ>
struct Src {
    uint64_t lp[MQ];
    uint64_t sc[MQ];
    uint32_t rem0, block_len, block_shift;
};

// Block of the scales (relative to sc[j]) that holds element `e` of the run.
template <int MQ>
__device__ __forceinline__ uint32_t q4_block(const Src<MQ>& src, uint32_t e)
{
    const uint32_t off = src.rem0 + e;
    return src.block_shift != 0xffffffffu ? off >> src.block_shift : off / src.block_len;
}

// NT full tiles starting at element 0 of the given bases: lane handles group `lane` of each.
// All loads are issued before the first use.
template <typename L, int MQ, int NT>
__device__ __forceinline__ void merge_full_tiles(uint64_t th, uint64_t vv, uint64_t tb,
                                                 const Src<MQ>& src, const float (&w)[MQ],
                                                 float lr, float mu)
{
    constexpr bool Q4 = IsQ4<L>::value;
    typename L::raw raw[NT][MQ];
    float scale[NT][Q4 ? MQ : 1];
    f32x4 T[NT], V[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const uint32_t g = threadIdx.x + u * DDL_BLOCK;
#pragma unroll
        for (int j = 0; j < MQ; ++j)
            raw[u][j] = ld<typename L::raw, Q4 ? DDL_Q4_CODE_LOAD : DDL_NT_LOAD>(src.lp[j], g);
        if constexpr (Q4) {  // the scales are re-read by the lanes of a block: cached loads
            const uint32_t blk = q4_block<MQ>(src, g * 4);
#pragma unroll
            for (int j = 0; j < MQ; ++j) scale[u][j] = ld<float, 0>(src.sc[j], blk);
        }
        T[u] = ld<f32x4, DDL_NT_STATE_LOAD>(th, g);
        V[u] = ld<f32x4, DDL_NT_STATE_LOAD>(vv, g);
    }
    if (NT > 1) __builtin_amdgcn_sched_barrier(0);  // keep the loads ahead of the arithmetic
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const uint32_t g = threadIdx.x + u * DDL_BLOCK;
        float x[MQ][4];
#pragma unroll
        for (int j = 0; j < MQ; ++j) L::widen(raw[u][j], x[j]);
        float wl[MQ];  // per lane for 4-bit sources: weight times the block's scale
#pragma unroll
        for (int j = 0; j < MQ; ++j) wl[j] = Q4 ? w[j] * scale[u][Q4 ? j : 0] : w[j];
        float t4[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
        float v4[4] = {V[u].x, V[u].y, V[u].z, V[u].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float xe[MQ];
#pragma unroll
            for (int j = 0; j < MQ; ++j) xe[j] = x[j][k];
            outer_step<MQ, Q4>(t4[k], v4[k], xe, wl, lr, mu);
        }
        const f32x4 tn = {t4[0], t4[1], t4[2], t4[3]};
        const f32x4 vn = {v4[0], v4[1], v4[2], v4[3]};
        st<f32x4>(th, g, tn);
        st<f32x4>(vv, g, vn);
        if (tb) {  // block-uniform: the broadcast copy of the new Theta
            const u32x2 packed = {bf16_rne(t4[0]) | (bf16_rne(t4[1]) << 16),
                                  bf16_rne(t4[2]) | (bf16_rne(t4[3]) << 16)};
            st<u32x2>(tb, g, packed);
        }
    }
}

template <typename L, int MQ>
__device__ __forceinline__ void merge_scalar(uint64_t th, uint64_t vv, uint64_t tb,
                                             const Src<MQ>& src, const float (&w)[MQ],
                                             float lr, float mu, uint32_t e)
{
    constexpr bool Q4 = IsQ4<L>::value;
    typedef typename L::elem elem;
    float t = *(reinterpret_cast<const DDL_GLOBAL float*>(th) + e);
    float v = *(reinterpret_cast<const DDL_GLOBAL float*>(vv) + e);
    float xe[MQ], wl[MQ];
    if constexpr (Q4) {
        const uint32_t blk = q4_block<MQ>(src, e);
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            const uint32_t byte = *(reinterpret_cast<const DDL_GLOBAL uint8_t*>(src.lp[j]) + e / 2);
            xe[j] = LearnerQ4::nibble(byte, (int)(e & 1));
            wl[j] = w[j] * *(reinterpret_cast<const DDL_GLOBAL float*>(src.sc[j]) + blk);
        }
    } else {
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            xe[j] = L::widen1(*(reinterpret_cast<const DDL_GLOBAL elem*>(src.lp[j]) + e));
            wl[j] = w[j];
        }
    }
    outer_step<MQ, Q4>(t, v, xe, wl, lr, mu);
    *(reinterpret_cast<DDL_GLOBAL float*>(th) + e) = t;
    *(reinterpret_cast<DDL_GLOBAL float*>(vv) + e) = v;
    if (tb) *(reinterpret_cast<DDL_GLOBAL uint16_t*>(tb) + e) = (uint16_t)bf16_rne(t);
}

// A ragged tile (the last of a tensor): guarded groups, then fewer than four left-overs.
template <typename L, int MQ>
__device__ __forceinline__ void merge_ragged_tile(uint64_t th, uint64_t vv, uint64_t tb,
                                                  const Src<MQ>& src, const float (&w)[MQ],
                                                  float lr, float mu, uint32_t cnt)
{
    const uint32_t nvec = cnt / 4;
    if (threadIdx.x < nvec) merge_full_tiles<L, MQ, 1>(th, vv, tb, src, w, lr, mu);
    const uint32_t e = nvec * 4 + threadIdx.x;
    if (e < cnt) merge_scalar<L, MQ>(th, vv, tb, src, w, lr, mu, e);
}

template <typename L, int MQ, bool FLAT>
__global__ void __launch_bounds__(DDL_BLOCK) ddl_merge_kernel(const DdlLaunchArgs a)
{
    constexpr bool Q4 = IsQ4<L>::value;
    typedef typename L::elem elem;
    uint32_t tile = a.tile_base +
                    rotate_tile(blockIdx.x, gridDim.x, (uint32_t)a.rotate) * a.tiles_per_block;
#ifdef DDL_TRACE
    // Diagnostic build: when each workgroup started, on which XCD, with which tile.
    if (a.trace && threadIdx.x == 0) {
        const uint32_t xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf;  // HW_REG_XCC_ID
        uint64_t* rec = a.trace + 2 * (uint64_t)(a.tile_base / a.tiles_per_block + blockIdx.x);
        rec[0] = wall_clock64();
        rec[1] = ((uint64_t)xcc << 32) | tile;
    }
#endif
    const uint32_t last = min(tile + a.tiles_per_block, a.total_tiles);

    while (tile < last) {
        // Which fragment of the launch, then which of its tensors, holds this tile.
        int it = 0;
        if (!FLAT) {
            for (int k = 1; k < a.num_items; ++k)
                if (tile >= a.item[k].tile_off) it = k;
        }
        const DdlItem& I = a.item[it];
        const uint32_t t = tile - I.tile_off;
        // The descriptor table is read-only for the whole launch: address it as constant
        // memory, so that these block-uniform lookups are scalar loads through the scalar
        // cache instead of vector loads queueing behind the streaming traffic.
        const DDL_CONST DdlSegDesc* sp;
        const DDL_CONST DdlQ4Desc* qp = nullptr;
        if (FLAT) {
            // The one descriptor sits in the kernel-argument block.  Reach it through the
            // kernarg segment pointer: taking the address of the by-value argument would make
            // the compiler copy it to private memory, which is not constant address space.
            const DDL_CONST DdlLaunchArgs* ka =
                (const DDL_CONST DdlLaunchArgs*)__builtin_amdgcn_kernarg_segment_ptr();
            sp = &ka->flat;
            if (Q4) qp = &ka->flat_q4;
        } else {
            const DDL_CONST DdlSegDesc* segs =
                reinterpret_cast<const DDL_CONST DdlSegDesc*>(reinterpret_cast<uint64_t>(a.segs)) +
                I.seg_begin;
            const DDL_CONST uint32_t* coarse =
                reinterpret_cast<const DDL_CONST uint32_t*>(reinterpret_cast<uint64_t>(a.coarse)) +
                I.coarse_begin + (t >> I.coarse_shift);
            uint32_t lo = coarse[0], hi = coarse[1];  // last tensor whose tile_begin <= t
            while (lo < hi) {
                const uint32_t mid = (lo + hi + 1) >> 1;
                if (segs[mid].tile_begin <= t) lo = mid; else hi = mid - 1;
            }
            sp = segs + lo;
            if (Q4)
                qp = reinterpret_cast<const DDL_CONST DdlQ4Desc*>(reinterpret_cast<uint64_t>(a.q4)) +
                     I.seg_begin + lo;
        }
        const uint64_t n = sp->n;
        const uint32_t seg_tiles = (uint32_t)((n + DDL_TILE - 1) / DDL_TILE);
        const uint32_t first_in_seg = t - sp->tile_begin;
        // tiles of this tensor that this workgroup handles: [first_in_seg, end_in_seg)
        const uint32_t end_in_seg = uniform(min(seg_tiles, first_in_seg + (last - tile)));
        const uint64_t off = (uint64_t)first_in_seg * DDL_TILE;  // elements
        uint64_t th = uniform(reinterpret_cast<uint64_t>(sp->theta) + off * 4);
        uint64_t vv = uniform(reinterpret_cast<uint64_t>(sp->v) + off * 4);
        const uint64_t tb0 = reinterpret_cast<uint64_t>(sp->theta_bf16);
        uint64_t tb = uniform(tb0 ? tb0 + off * 2 : 0);  // 0: no broadcast copy asked for
        Src<MQ> src;
        float w[MQ];
        src.rem0 = 0;
        src.block_len = a.block_len;
        src.block_shift = a.block_shift;
        uint64_t blk0 = 0;  // 4-bit sources: block that holds the run's first element
        if (Q4) {
            blk0 = a.block_shift != 0xffffffffu ? off >> a.block_shift : off / a.block_len;
            src.rem0 = uniform((uint32_t)(off - blk0 * a.block_len));
        }
#pragma unroll
        for (int j = 0; j < MQ; ++j) {
            if (Q4) {
                src.lp[j] = uniform(reinterpret_cast<uint64_t>(qp->codes[I.idx[j]]) + off / 2);
                src.sc[j] = uniform(reinterpret_cast<uint64_t>(qp->scales[I.idx[j]]) + blk0 * 4);
            } else {
                src.lp[j] = uniform(reinterpret_cast<uint64_t>(sp->learner[I.idx[j]]) +
                                    off * sizeof(elem));
                src.sc[j] = 0;
            }
            w[j] = I.w[j];
        }
        const float lr = I.lr, mu = I.mu;
        // 4-bit sources come with aligned Theta and v (the host sees to it)
        const bool vec_ok = uniform((uint32_t)(
            sp->base_aligned &&
            (Q4 || (I.present_bits & ~(uint32_t)sp->learner_aligned) == 0))) != 0;

        uint32_t s = first_in_seg;
        while (s < end_in_seg) {
            const uint64_t rem = n - (uint64_t)s * DDL_TILE;
            uint32_t step = 1;
            if (!vec_ok) {
                const uint32_t cnt = rem < DDL_TILE ? (uint32_t)rem : DDL_TILE;
                for (uint32_t e = threadIdx.x; e < cnt; e += DDL_BLOCK)
                    merge_scalar<L, MQ>(th, vv, tb, src, w, lr, mu, e);
            } else if (DDL_PAIR && s + 2 <= end_in_seg && rem >= 2 * DDL_TILE) {
                merge_full_tiles<L, MQ, 2>(th, vv, tb, src, w, lr, mu);
                step = 2;
            } else if (rem >= DDL_TILE) {
                merge_full_tiles<L, MQ, 1>(th, vv, tb, src, w, lr, mu);
            } else {
                merge_ragged_tile<L, MQ>(th, vv, tb, src, w, lr, mu, (uint32_t)rem);
            }
            s += step;
            th += (uint64_t)step * DDL_TILE * 4;
            vv += (uint64_t)step * DDL_TILE * 4;
            if (tb) tb += (uint64_t)step * DDL_TILE * 2;
            if (Q4) {  // keep rem0 below block_len: move whole blocks into the scale base
                const uint32_t r = src.rem0 + step * DDL_TILE;
                const uint32_t whole =
                    a.block_shift != 0xffffffffu ? r >> a.block_shift : r / a.block_len;
                src.rem0 = r - whole * a.block_len;
#pragma unroll
                for (int j = 0; j < MQ; ++j) {
                    src.lp[j] += (uint64_t)step * DDL_TILE / 2;
                    src.sc[j] += (uint64_t)whole * 4;
                }
            } else {
#pragma unroll
                for (int j = 0; j < MQ; ++j) src.lp[j] += (uint64_t)step * DDL_TILE * sizeof(elem);
            }
        }
        tile += end_in_seg - first_in_seg;
    }
}

// Plain streaming copy, 16 bytes per lane, one group per lane, same cache hints as the merge
// kernel: the yardstick for what this GPU's HBM sustains and for scaling profiler counters.
__global__ void __launch_bounds__(DDL_BLOCK) ddl_copy_kernel(uint64_t dst, uint64_t src,
                                                             uint64_t n16)
{
    const uint64_t base = (uint64_t)blockIdx.x * DDL_BLOCK;
    if (base + threadIdx.x < n16) {
        const u32x4 r = ld<u32x4, DDL_NT_LOAD>(src + base * 16, threadIdx.x);
        st<u32x4>(dst + base * 16, threadIdx.x, r);
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

int ddl_launch_merge(int dtype, int Mq, bool flat, uint32_t grid, uint32_t lds_bytes, void* stream,
                     const DdlLaunchArgs& args)
{
    kernel_fn k = nullptr;
    if (dtype == 0)
        k = flat ? pick_mq<LearnerF32, true>(Mq) : pick_mq<LearnerF32, false>(Mq);
    else if (dtype == 1)
        k = flat ? pick_mq<LearnerBF16, true>(Mq) : pick_mq<LearnerBF16, false>(Mq);
    else if (dtype == DDL_SRC_Q4)
        k = flat ? pick_mq<LearnerQ4, true>(Mq) : pick_mq<LearnerQ4, false>(Mq);
    if (!k || grid == 0) return (int)hipErrorInvalidValue;
    DDL_COUNT_GRID();
    hipLaunchKernelGGL(k, dim3(grid), dim3(DDL_BLOCK), lds_bytes, static_cast<hipStream_t>(stream),
                       args);
    return (int)hipGetLastError();
}

int ddl_launch_merge_parts(int dtype, int Mq, bool flat, uint32_t max_tiles, uint32_t lds_bytes,
                           void* stream, DdlLaunchArgs& args)
{
    const uint32_t tpb = args.tiles_per_block;
    const uint64_t total = args.total_tiles;
    // Equal parts, each a whole number of workgroups (so that they tile the range exactly)
    // and of rotation groups (so that only the last part ends in a partial group).
    uint64_t part = total;
    if (max_tiles != 0 && total > max_tiles) {
        const uint64_t parts = (total + max_tiles - 1) / max_tiles;
        const uint64_t unit = (uint64_t)tpb * (args.rotate > 0 ? (uint32_t)args.rotate : 1u);
        part = (total + parts - 1) / parts;
        part = (part + unit - 1) / unit * unit;
    }
    for (uint64_t base = 0; base < total; base += part) {
        const uint64_t tiles = std::min<uint64_t>(part, total - base);
        args.tile_base = (uint32_t)base;
        const int e = ddl_launch_merge(dtype, Mq, flat, (uint32_t)((tiles + tpb - 1) / tpb),
                                       lds_bytes, stream, args);
        if (e != (int)hipSuccess) return e;
    }
    return (int)hipSuccess;
}

int ddl_launch_copy(void* dst, const void* src, uint64_t n16, uint32_t grid, void* stream)
{
    if (grid == 0) return (int)hipErrorInvalidValue;
    DDL_COUNT_GRID();
    hipLaunchKernelGGL(ddl_copy_kernel, dim3(grid), dim3(DDL_BLOCK), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<uint64_t>(dst),
                       reinterpret_cast<uint64_t>(src), n16);
    return (int)hipGetLastError();
}
