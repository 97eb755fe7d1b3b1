// Host side of libddlsync: the C ABI of include/ddlsync.h.  Validates arguments, computes the
// quorum weights once per merge in fp64 (Algorithm 2, step "Weight"), drops learners that do
// not contribute, lays the fragments' tensors out as tiles, and enqueues the gfx950 kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"
#include "ddl_host_internal.h"

using namespace ddlh;

static_assert(DDL_MAXL == DDL_MAX_LEARNERS, "device and public learner limits differ");

std::atomic<long> ddl_opt_rda_blocks_per_cu{0};
std::atomic<long> ddl_stat_grids{0};

namespace {

thread_local std::string g_err;

}  // namespace

ddl_status ddlh::runtime_error(hipError_t e, const char* what)
{
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return DDL_ERR_RUNTIME;
}

void ddlh::set_error_message(const char* text) { g_err = text ? text : ""; }

namespace {

#define DDL_HIP(call)                                              \
    do {                                                           \
        hipError_t e__ = (call);                                   \
        if (e__ != hipSuccess) return runtime_error(e__, #call);   \
    } while (0)

// ------------------------------------------------------------------------------------------
// options and per-device state
// ------------------------------------------------------------------------------------------
// The launch-shape options are process-wide atomics: a launch reads each one once, so a call
// racing with ddl_set_option sees either the old or the new value, never a torn one.  No
// lock is taken on any launch path; the only lock guards the staging cache of ddl_merge_batch.
std::atomic<long> g_tiles_per_block{-1};    // consecutive tiles a workgroup walks; -1: chosen
                                            // by the kind of learner data
std::atomic<long> g_tile_rotate{64};        // group size of the tile rotation (0: off)
std::atomic<long> g_max_blocks_per_cu{-1};  // -1: by learner type and count; 0: no cap; k: at
                                            // most k resident workgroups per compute unit
#ifdef DDL_TRACE
std::atomic<long> g_trace_buffer{0};  // diagnostic build: device address of the trace records
#endif
std::atomic<long> g_max_tiles_per_launch{-1};  // 0: a launch is one grid; k: grids of at most
                                               // k tiles; -1: k chosen from the bytes per tile
std::atomic<long> g_part_megabytes{2500};      // the byte size -1 aims at
std::mutex g_stage_mu;                      // guards g_dev (the staging cache) only

constexpr int kMaxDevices = 16;
constexpr int kSlots = 64;

// One staged descriptor table.  The pinned host copy doubles as the key of a small cache: a
// later call that builds the very same table (the same fragments, i.e. the same pointers and
// sizes) finds it here and needs no copy at all.
struct Slot {
    void* host = nullptr;  // pinned; holds the image that `dev` holds (first `bytes` bytes)
    void* dev = nullptr;
    size_t cap = 0;
    size_t bytes = 0;      // 0: nothing valid staged
    uint64_t hash = 0;
    hipEvent_t done = nullptr;       // recorded after the last work that read `dev`
    hipStream_t last_stream = nullptr;
    bool pending = false;
};

struct DeviceState {
    Slot slot[kSlots];
    unsigned next = 0;
};
DeviceState g_dev[kMaxDevices];

ddl_status device_state(DeviceState** out)
{
    int dev = 0;
    DDL_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        g_err = "device index out of range";
        return DDL_ERR_RUNTIME;
    }
    *out = &g_dev[dev];
    return DDL_OK;
}

// Tiles per workgroup when left to the library: one, except for 4-bit codes of more than eight
// learners -- their streams are so thin (512 B per learner and tile) that two tiles per
// workgroup pay (moe, 11 learners: 5985 -> 6244 GB/s; with fewer learners, and for bf16 / fp32
// learners of any count, two tiles per workgroup cost 3-8 %).
uint32_t tiles_per_block(int elem_bytes, int Mq)
{
    const long opt = g_tiles_per_block.load(std::memory_order_relaxed);
    if (opt >= 1) return (uint32_t)opt;
    return elem_bytes == 0 && Mq > 8 ? 2u : 1u;
}

// A long launch goes out as several grids, back to back on the stream.  The eight XCDs each
// work through their own share of a grid's workgroups at their own pace, and nothing
// re-aligns them before the grid ends: over some hundred thousand workgroups their positions
// drift apart, the window of DRAM pages in flight widens, and the achieved rate drops by
// 3-6 %.  A grid boundary re-aligns them at the price of one drain (about 3 us).  Measured on
// MI355X, grids of 0.3-0.5 ms (2-3 GB of traffic) are the best trade for every learner count.
// elem_bytes: bytes per learner element (0: 4-bit codes); extra: other bytes per element.
uint32_t part_tiles(int elem_bytes, int Mq, int extra)
{
    const long opt = g_max_tiles_per_launch.load(std::memory_order_relaxed);
    if (opt >= 0) return (uint32_t)opt;
    const uint64_t per_tile =
        (uint64_t)DDL_TILE * (16 + extra + (elem_bytes ? elem_bytes * Mq : (Mq + 1) / 2));
    const uint64_t tiles =
        (uint64_t)g_part_megabytes.load(std::memory_order_relaxed) * 1000000ull / per_tile;
    return (uint32_t)std::max<uint64_t>(tiles, 4096);
}

// Dynamic LDS requested per workgroup purely to cap residency: floor(LDS per CU / k), kept
// within the 64 KiB a kernel may ask for without opting in.
// The cap itself, when left to the library (measured on MI355X; what matters is roughly the
// bytes one compute unit has in flight): few bf16 learners leave room for six workgroups, many
// want four; fp32 learners, twice the bytes per tile, want four and from four learners on
// three; 4-bit codes (half a byte per element) want eight, the most the kernel's registers
// allow anyway (dense_block / large_dense / moe at 4, 5, 6, 8, none: 6020/6013/5504,
// 6033/6011/5492, 6331/6261/5993, 6408/6538/5995, 6434/6544/5989 GB/s).
// elem_bytes: 4 fp32 learners, 2 bf16, 0 the 4-bit codes.
long auto_blocks_per_cu(int elem_bytes, int Mq)
{
    if (elem_bytes == 4) return Mq >= 4 ? 3 : 4;
    if (elem_bytes == 2) return Mq <= 5 ? 6 : 4;
    return 8;
}

uint32_t lds_cap_bytes(int elem_bytes, int Mq)
{
    const long opt = g_max_blocks_per_cu.load(std::memory_order_relaxed);
    const long k = opt < 0 ? auto_blocks_per_cu(elem_bytes, Mq) : opt;
    if (k <= 0) return 0;
    uint32_t b = (uint32_t)(DDL_LDS_PER_CU / k) & ~511u;
    return b > 64 * 1024 ? 64 * 1024 : b;
}

}  // namespace

uint32_t ddlh::merge_lds_cap_bytes(int elem_bytes, int Mq) { return lds_cap_bytes(elem_bytes, Mq); }
uint32_t ddlh::max_tiles_per_launch(int elem_bytes, int Mq, int extra)
{
    return part_tiles(elem_bytes, Mq, extra);
}
uint32_t ddlh::tile_rotate() { return (uint32_t)g_tile_rotate.load(std::memory_order_relaxed); }

// ------------------------------------------------------------------------------------------
// weights
// ------------------------------------------------------------------------------------------
bool ddlh::finite_nonneg(float x) { return std::isfinite(x) && x >= 0.0f; }

ddl_status ddlh::weights_tokens(const uint64_t* t, const uint8_t* q, int M, double* w)
{
    if (!t || !q || !w || M < 1 || M > DDL_MAX_LEARNERS) return DDL_ERR_INVALID_ARG;
    unsigned __int128 S = 0;  // exact: M counters below 2^64
    for (int m = 0; m < M; ++m) {
        if (q[m] > 1) return DDL_ERR_INVALID_ARG;
        if (q[m]) S += t[m];
    }
    if (S == 0) return DDL_ERR_EMPTY_QUORUM;
    const double Sd = (double)S;
    for (int m = 0; m < M; ++m) w[m] = q[m] ? (double)t[m] / Sd : 0.0;
    return DDL_OK;
}

namespace {

ddl_status weights_quality(const uint64_t* t, const uint64_t* s, const uint8_t* q, int M, double* w)
{
    if (!t || !s || !q || !w || M < 1 || M > DDL_MAX_LEARNERS) return DDL_ERR_INVALID_ARG;
    double raw[DDL_MAXL];
    double S = 0.0;
    for (int m = 0; m < M; ++m) {
        raw[m] = 0.0;
        if (q[m] > 1) return DDL_ERR_INVALID_ARG;
        if (!q[m]) continue;
        if (s[m] == 0) {
            if (t[m] != 0) return DDL_ERR_INVALID_ARG;
            continue;
        }
        const double tok = (double)t[m];
        raw[m] = tok * (tok / (double)s[m]);
        S += raw[m];
    }
    if (S == 0.0) return DDL_ERR_EMPTY_QUORUM;
    for (int m = 0; m < M; ++m) w[m] = raw[m] / S;
    return DDL_OK;
}

// Caller-supplied weights: non-negative, finite, positive sum; normalised here.
ddl_status weights_given(const double* in, int M, double* w)
{
    if (!in || M < 1 || M > DDL_MAX_LEARNERS) return DDL_ERR_INVALID_ARG;
    double S = 0.0;
    for (int m = 0; m < M; ++m) {
        if (!std::isfinite(in[m]) || in[m] < 0.0) return DDL_ERR_INVALID_ARG;
        S += in[m];
    }
    if (!(S > 0.0) || !std::isfinite(S)) return DDL_ERR_EMPTY_QUORUM;
    for (int m = 0; m < M; ++m) w[m] = in[m] / S;
    return DDL_OK;
}

}  // namespace

// Drop learners of weight zero; round the rest once to fp32 for the device.
void ddlh::compact(const double* w, int M, Quorum& out)
{
    out.Mq = 0;
    out.present_bits = 0;
    for (int m = 0; m < M; ++m) {
        if (w[m] > 0.0) {
            out.w[out.Mq] = (float)w[m];
            out.idx[out.Mq] = (uint8_t)m;
            out.present_bits |= 1u << m;
            ++out.Mq;
        }
    }
    for (int j = out.Mq; j < DDL_MAXL; ++j) {
        out.w[j] = 0.0f;
        out.idx[j] = 0;
    }
}

namespace {

// ------------------------------------------------------------------------------------------
// overlap check: an output range (Theta, v) may overlap nothing; inputs may overlap inputs
// ------------------------------------------------------------------------------------------
}  // namespace

bool ddlh::ranges_alias(std::vector<Range>& r)
{
    std::sort(r.begin(), r.end(), [](const Range& a, const Range& b) { return a.lo < b.lo; });
    uintptr_t max_hi_any = 0, max_hi_out = 0;
    for (const Range& x : r) {
        if (x.out ? x.lo < max_hi_any : x.lo < max_hi_out) return true;
        max_hi_any = std::max(max_hi_any, x.hi);
        if (x.out) max_hi_out = std::max(max_hi_out, x.hi);
    }
    return false;
}

// Appends [p, p + elem * n); false if the end is not representable (the range would wrap
// around the address space: no such array exists, and a wrapped end would hide an overlap).
bool ddlh::add_range(const void* p, size_t elem, size_t n, bool out, std::vector<Range>& r)
{
    size_t bytes = 0;
    uintptr_t hi = 0;
    if (__builtin_mul_overflow(elem, n, &bytes) ||
        __builtin_add_overflow((uintptr_t)p, bytes, &hi))
        return false;
    r.push_back({(uintptr_t)p, hi, out});
    return true;
}

namespace {

inline size_t elem_size(ddl_dtype d) { return d == DDL_BF16 ? 2 : 4; }

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Appends the ranges of one segment; false if a needed pointer is NULL or misaligned for its
// element type, or a range wraps.  `learner_bits` selects which learners' ranges count.
bool add_segment_ranges(const float* theta, const float* v, const void* theta_bf16,
                        const void* const* learners, uint32_t learner_bits, ddl_dtype dt, size_t n,
                        std::vector<Range>& r)
{
    if (!theta || !v || !aligned(theta, 4) || !aligned(v, 4) || !aligned(theta_bf16, 2))
        return false;
    if (!add_range(theta, 4, n, true, r) || !add_range(v, 4, n, true, r)) return false;
    if (theta_bf16 && !add_range(theta_bf16, 2, n, true, r)) return false;
    const size_t b = elem_size(dt);
    for (int m = 0; m < DDL_MAXL; ++m) {
        if (!(learner_bits >> m & 1)) continue;
        const void* p = learners[m];
        if (!p || !aligned(p, b) || !add_range(p, b, n, false, r)) return false;
    }
    return true;
}

}  // namespace

void ddlh::fill_desc(DdlSegDesc& d, float* theta, float* v, void* theta_bf16,
                     const void* const* learners, int M, size_t n, uint32_t tile_begin)
{
    std::memset(&d, 0, sizeof d);
    d.theta = theta;
    d.v = v;
    d.theta_bf16 = theta_bf16;
    d.n = n;
    d.tile_begin = tile_begin;
    d.base_aligned = aligned(theta, 16) && aligned(v, 16) && aligned(theta_bf16, 8);
    for (int m = 0; m < M; ++m) {
        d.learner[m] = learners ? learners[m] : nullptr;
        if (learners && aligned(learners[m], 16)) d.learner_aligned |= (uint16_t)(1u << m);
    }
}

namespace {

void fill_item(DdlItem& it, const Quorum& q, float lr, float mu, uint32_t seg_begin,
               uint32_t num_segs, uint32_t tile_off, uint32_t coarse_begin = 0,
               uint32_t coarse_shift = 0)
{
    std::memset(&it, 0, sizeof it);
    it.seg_begin = seg_begin;
    it.num_segs = num_segs;
    it.tile_off = tile_off;
    it.present_bits = q.present_bits;
    std::memcpy(it.w, q.w, sizeof it.w);
    std::memcpy(it.idx, q.idx, sizeof it.idx);
    it.lr = lr;
    it.mu = mu;
    it.coarse_begin = coarse_begin;
    it.coarse_shift = coarse_shift;
}

// ------------------------------------------------------------------------------------------
// table of segment descriptors for a set of fragments
// ------------------------------------------------------------------------------------------
// About four coarse entries per descriptor: a tile's two bracketing entries are then almost
// always equal.  One extra entry past the end keeps entry i + 1 readable for every tile.
void build_coarse(Table& T, FragInfo& fi)
{
    fi.coarse_begin = (uint32_t)T.coarse.size();
    fi.coarse_shift = 0;
    if (fi.num_segs == 0) return;
    const uint64_t target = 4ull * fi.num_segs;
    while (fi.coarse_shift < 31 && ((uint64_t)fi.tiles >> (fi.coarse_shift + 1)) >= target)
        ++fi.coarse_shift;
    const uint32_t entries = (fi.tiles >> fi.coarse_shift) + 2;
    const DdlSegDesc* segs = T.segs.data() + fi.seg_begin;
    uint32_t s = 0;
    for (uint32_t i = 0; i < entries; ++i) {
        const uint64_t tile = (uint64_t)i << fi.coarse_shift;
        while (s + 1 < fi.num_segs && segs[s + 1].tile_begin <= tile) ++s;
        T.coarse.push_back(tile < fi.tiles ? s : fi.num_segs - 1);
    }
}

ddl_status check_fragment_shape(const ddl_fragment& f)
{
    if (f.M < 1 || f.M > DDL_MAX_LEARNERS) return DDL_ERR_INVALID_ARG;
    if (f.learner_dtype != DDL_F32 && f.learner_dtype != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (f.num_segs < 0 || (f.num_segs > 0 && !f.segs)) return DDL_ERR_INVALID_ARG;
    for (int s = 0; s < f.num_segs; ++s)
        if (f.segs[s].n > 0 && !f.segs[s].learner_params) return DDL_ERR_INVALID_ARG;
    return DDL_OK;
}

// Builds the descriptors.  learner_bits[i] says which learners of fragment i must be valid
// and take part in the overlap check.
ddl_status build_table(const ddl_fragment* frags, int num_frags, const uint32_t* learner_bits,
                       Table& T)
{
    T.segs.clear();
    T.origin.clear();
    T.given_segs = 0;
    T.coarse.clear();
    T.frags.assign((size_t)num_frags, FragInfo());
    T.elems = 0;
    std::vector<Range> ranges;
    for (int i = 0; i < num_frags; ++i) {
        const ddl_fragment& f = frags[i];
        FragInfo& fi = T.frags[(size_t)i];
        fi.seg_begin = (uint32_t)T.segs.size();
        fi.M = f.M;
        fi.dt = f.learner_dtype;
        fi.nonnull_bits = (1u << f.M) - 1u;
        uint64_t tiles = 0;
        for (int s = 0; s < f.num_segs; ++s) {
            const ddl_segment& g = f.segs[s];
            const uint32_t position = T.given_segs++;
            if (g.n == 0) continue;
            uint32_t bits = learner_bits[i];
            if (bits == 0xffffffffu) {  // plan creation: every non-NULL learner counts
                bits = 0;
                for (int m = 0; m < f.M; ++m)
                    if (g.learner_params[m]) bits |= 1u << m;
            }
            for (int m = 0; m < f.M; ++m)
                if (!g.learner_params[m]) fi.nonnull_bits &= ~(1u << m);
            if (!add_segment_ranges(g.theta, g.v, g.theta_bf16, g.learner_params, bits,
                                    f.learner_dtype, g.n, ranges))
                return DDL_ERR_INVALID_ARG;
            if (tiles > 0xffffffffull) return DDL_ERR_INVALID_ARG;
            DdlSegDesc d;
            fill_desc(d, g.theta, g.v, g.theta_bf16, g.learner_params, f.M, g.n, (uint32_t)tiles);
            T.segs.push_back(d);
            T.origin.push_back(position);
            tiles += (g.n + DDL_TILE - 1) / DDL_TILE;
            fi.elems += g.n;
        }
        if (tiles > 0x7fffffffull) return DDL_ERR_INVALID_ARG;
        fi.tiles = (uint32_t)tiles;
        fi.num_segs = (uint32_t)T.segs.size() - fi.seg_begin;
        build_coarse(T, fi);
        T.elems += fi.elems;
    }
    if (ranges_alias(ranges)) return DDL_ERR_ALIAS;
    return DDL_OK;
}

uint32_t log2_or_none(uint32_t x)  // log2 of a power of two, else 0xffffffff
{
    if (x == 0 || (x & (x - 1))) return 0xffffffffu;
    uint32_t s = 0;
    while ((1u << s) < x) ++s;
    return s;
}

}  // namespace

// Enqueue the fragments in `work`: one launch per group of up to DDL_MAX_ITEMS fragments with
// the same learner dtype and number of contributing learners.
ddl_status ddlh::launch_work(const Table& T, const void* d_table, std::vector<Work>& work,
                             void* stream, const Q4Source* q4)
{
    // source kind and bytes per learner element of a fragment in this call
    auto kind = [&](const FragInfo& f) { return q4 ? DDL_SRC_Q4 : (int)f.dt; };
    auto ebytes = [&](const FragInfo& f) { return q4 ? 0 : (int)elem_size(f.dt); };
    std::stable_sort(work.begin(), work.end(), [&](const Work& a, const Work& b) {
        const FragInfo& fa = T.frags[a.frag];
        const FragInfo& fb = T.frags[b.frag];
        if (kind(fa) != kind(fb)) return kind(fa) < kind(fb);
        return a.q.Mq < b.q.Mq;
    });
    size_t i = 0;
    while (i < work.size()) {
        const FragInfo& f0 = T.frags[work[i].frag];
        DdlLaunchArgs a;
        std::memset(&a, 0, sizeof a);
        a.segs = static_cast<const DdlSegDesc*>(d_table);
        a.coarse = reinterpret_cast<const uint32_t*>(static_cast<const char*>(d_table) +
                                                     T.seg_bytes());
        a.tiles_per_block = tiles_per_block(ebytes(f0), work[i].q.Mq);
        a.rotate = (int32_t)tile_rotate();
        if (q4) {
            a.q4 = q4->d_table;
            a.block_len = q4->block_len;
            a.block_shift = log2_or_none(q4->block_len);
        }
        uint64_t tiles = 0;
        int items = 0;
        size_t j = i;
        for (; j < work.size() && items < DDL_MAX_ITEMS; ++j) {
            const FragInfo& f = T.frags[work[j].frag];
            if (kind(f) != kind(f0) || work[j].q.Mq != work[i].q.Mq) break;
            if (f.tiles == 0) continue;
            if (tiles + f.tiles > 0x7fffffffull) break;
            fill_item(a.item[items], work[j].q, work[j].lr, work[j].mu, f.seg_begin, f.num_segs,
                      (uint32_t)tiles, f.coarse_begin, f.coarse_shift);
            tiles += f.tiles;
            ++items;
        }
        if (items > 0) {
            a.num_items = items;
            a.total_tiles = (uint32_t)tiles;
#ifdef DDL_TRACE
            a.trace = reinterpret_cast<uint64_t*>(g_trace_buffer.load());
#endif
            const int e = ddl_launch_merge_parts(
                kind(f0), work[i].q.Mq, false, max_tiles_per_launch(ebytes(f0), work[i].q.Mq),
                lds_cap_bytes(ebytes(f0), work[i].q.Mq), stream, a);
            if (e != (int)hipSuccess) return runtime_error((hipError_t)e, "merge kernel launch");
        }
        if (j == i) return DDL_ERR_INVALID_ARG;  // cannot happen: a lone fragment always fits
        i = j;
    }
    return DDL_OK;
}

// ONE tensor whose descriptor travels in the kernel-argument block.
ddl_status ddlh::launch_flat(const DdlSegDesc& desc, int src, const Quorum& q, float lr, float mu,
                             void* stream, const DdlQ4Desc* q4d, uint32_t block_len)
{
    const uint64_t tiles = (desc.n + DDL_TILE - 1) / DDL_TILE;
    if (tiles == 0) return DDL_OK;
    if (tiles > 0x7fffffffull) return DDL_ERR_INVALID_ARG;
    DdlLaunchArgs a;
    std::memset(&a, 0, sizeof a);
    const int ebytes = src == DDL_SRC_Q4 ? 0 : src == (int)DDL_BF16 ? 2 : 4;
    a.tiles_per_block = tiles_per_block(ebytes, q.Mq);
    a.rotate = (int32_t)tile_rotate();
    a.total_tiles = (uint32_t)tiles;
    a.num_items = 1;
    a.flat = desc;
    a.flat.tile_begin = 0;
    if (src == DDL_SRC_Q4) {
        if (!q4d) return DDL_ERR_INVALID_ARG;
        a.flat_q4 = *q4d;
        a.block_len = block_len;
        a.block_shift = log2_or_none(block_len);
    }
    fill_item(a.item[0], q, lr, mu, 0, 1, 0);
    const int e = ddl_launch_merge_parts(src, q.Mq, true, max_tiles_per_launch(ebytes, q.Mq),
                                         lds_cap_bytes(ebytes, q.Mq), stream, a);
    if (e != (int)hipSuccess) return runtime_error((hipError_t)e, "merge kernel launch");
    return DDL_OK;
}

namespace {

ddl_status merge_flat(float* theta, float* v, void* theta_bf16, const void* const* learner_params,
                      ddl_dtype dt, const double* w, int M, size_t n, float lr, float mu,
                      void* stream)
{
    if (dt != DDL_F32 && dt != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (!finite_nonneg(lr) || !finite_nonneg(mu)) return DDL_ERR_INVALID_ARG;
    if (n == 0) return DDL_OK;
    if (!learner_params) return DDL_ERR_INVALID_ARG;
    Quorum q;
    compact(w, M, q);
    std::vector<Range> ranges;
    const void* lp[DDL_MAXL] = {};
    for (int m = 0; m < M; ++m) lp[m] = (q.present_bits >> m & 1) ? learner_params[m] : nullptr;
    if (!add_segment_ranges(theta, v, theta_bf16, lp, q.present_bits, dt, n, ranges))
        return DDL_ERR_INVALID_ARG;
    if (ranges_alias(ranges)) return DDL_ERR_ALIAS;

    DdlSegDesc d;
    fill_desc(d, theta, v, theta_bf16, lp, M, n, 0);
    return launch_flat(d, (int)dt, q, lr, mu, stream);
}

}  // namespace

// Direct averaging of ONE tensor whose descriptor already exists (a tensor of a plan): the
// descriptor travels in the kernel-argument block.  Used by the RDA plan call for tensors
// that are to be merged by direct averaging.
ddl_status ddlh::launch_one_direct(const DdlSegDesc& desc, ddl_dtype dt, const Quorum& q, float lr,
                                   float mu, void* stream)
{
    return launch_flat(desc, (int)dt, q, lr, mu, stream);
}

extern "C" {

int ddl_version(void) { return 200; }

#ifndef DDL_BUILD_ID
#define DDL_BUILD_ID "unknown"
#endif
const char* ddl_build_id(void) { return DDL_BUILD_ID; }

#ifndef DDL_BUILD_ID_MERGE
#define DDL_BUILD_ID_MERGE "unknown"
#define DDL_BUILD_ID_RDA "unknown"
#define DDL_BUILD_ID_Q4 "unknown"
#endif
const char* ddl_kernel_build_id(const char* kernel)
{
    if (kernel && !std::strcmp(kernel, "merge")) return DDL_BUILD_ID_MERGE;
    if (kernel && !std::strcmp(kernel, "rda")) return DDL_BUILD_ID_RDA;
    if (kernel && !std::strcmp(kernel, "q4")) return DDL_BUILD_ID_Q4;
    return "";
}

const char* ddl_status_string(ddl_status s)
{
    switch (s) {
        case DDL_OK: return "ok";
        case DDL_ERR_INVALID_ARG: return "invalid argument";
        case DDL_ERR_EMPTY_QUORUM: return "empty quorum";
        case DDL_ERR_ALIAS: return "output range overlaps another range";
        case DDL_ERR_RUNTIME: return "HIP runtime error";
    }
    return "unknown status";
}

const char* ddl_last_error_message(void) { return g_err.c_str(); }

ddl_status ddl_compute_weights(const uint64_t* token_counts, const uint8_t* quorum_mask, int M,
                               double* w_out)
{
    return weights_tokens(token_counts, quorum_mask, M, w_out);
}

ddl_status ddl_compute_weights_quality(const uint64_t* token_counts, const uint64_t* step_counts,
                                       const uint8_t* quorum_mask, int M, double* w_out)
{
    return weights_quality(token_counts, step_counts, quorum_mask, M, w_out);
}

ddl_status ddl_merge_fragment(float* theta, float* v, const void* const* learner_params,
                              ddl_dtype learner_dtype, const uint64_t* token_counts,
                              const uint8_t* quorum_mask, int M, size_t n, float lr, float mu,
                              void* hip_stream)
{
    double w[DDL_MAXL];
    const ddl_status st = weights_tokens(token_counts, quorum_mask, M, w);
    if (st != DDL_OK) return st;
    return merge_flat(theta, v, nullptr, learner_params, learner_dtype, w, M, n, lr, mu,
                      hip_stream);
}

ddl_status ddl_merge_fragment_bcast(float* theta, float* v, void* theta_bf16,
                                    const void* const* learner_params, ddl_dtype learner_dtype,
                                    const uint64_t* token_counts, const uint8_t* quorum_mask,
                                    int M, size_t n, float lr, float mu, void* hip_stream)
{
    double w[DDL_MAXL];
    const ddl_status st = weights_tokens(token_counts, quorum_mask, M, w);
    if (st != DDL_OK) return st;
    if (n > 0 && !theta_bf16) return DDL_ERR_INVALID_ARG;
    return merge_flat(theta, v, theta_bf16, learner_params, learner_dtype, w, M, n, lr, mu,
                      hip_stream);
}

ddl_status ddl_merge_fragment_weighted(float* theta, float* v, const void* const* learner_params,
                                       ddl_dtype learner_dtype, const double* weights, int M,
                                       size_t n, float lr, float mu, void* hip_stream)
{
    double w[DDL_MAXL];
    const ddl_status st = weights_given(weights, M, w);
    if (st != DDL_OK) return st;
    return merge_flat(theta, v, nullptr, learner_params, learner_dtype, w, M, n, lr, mu,
                      hip_stream);
}

ddl_status ddl_merge_batch(const ddl_fragment* frags, int num_frags, void* hip_stream)
{
    if (num_frags < 0 || (num_frags > 0 && !frags)) return DDL_ERR_INVALID_ARG;
    if (num_frags == 0) return DDL_OK;
    std::vector<Work> work;
    std::vector<uint32_t> bits((size_t)num_frags);
    work.reserve((size_t)num_frags);
    for (int i = 0; i < num_frags; ++i) {
        const ddl_fragment& f = frags[i];
        ddl_status st = check_fragment_shape(f);
        if (st != DDL_OK) return st;
        if (!finite_nonneg(f.lr) || !finite_nonneg(f.mu)) return DDL_ERR_INVALID_ARG;
        double w[DDL_MAXL];
        st = weights_tokens(f.token_counts, f.quorum_mask, f.M, w);
        if (st != DDL_OK) return st;
        Work wk;
        wk.frag = (uint32_t)i;
        wk.lr = f.lr;
        wk.mu = f.mu;
        compact(w, f.M, wk.q);
        bits[(size_t)i] = wk.q.present_bits;
        work.push_back(wk);
    }

    // The staging below copies from a reusable pinned buffer and records an event: neither
    // may become a node of a graph under capture (a replay would read a buffer that later
    // calls overwrite, and the event would never be seen as recorded).  A plan is the form
    // for capture.
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    DDL_HIP(hipStreamIsCapturing(stream, &cap));
    if (cap != hipStreamCaptureStatusNone) return DDL_ERR_INVALID_ARG;

    Table T;
    ddl_status st = build_table(frags, num_frags, bits.data(), T);
    if (st != DDL_OK) return st;
    if (T.segs.empty()) return DDL_OK;
    const size_t bytes = T.bytes();
    std::vector<char> image(bytes);
    T.copy_to(image.data());
    uint64_t hash = 1469598103934665603ull;  // FNV-1a
    for (size_t i = 0; i < bytes; ++i) hash = (hash ^ (unsigned char)image[i]) * 1099511628211ull;

    // The descriptors go to the device through a pinned host copy, on the caller's stream --
    // unless an earlier call staged exactly this table, which is then used as it is.  The lock
    // covers the cache bookkeeping and this call's enqueues, never a wait for the GPU: a slot
    // whose last use has not finished is passed over, and if every slot is busy the lock is
    // dropped while waiting for one.
    std::unique_lock<std::mutex> lock(g_stage_mu);
    DeviceState* ds = nullptr;
    st = device_state(&ds);
    if (st != DDL_OK) return st;
    Slot* sl = nullptr;
    for (Slot& c : ds->slot)
        if (c.bytes == bytes && c.hash == hash && std::memcmp(c.host, image.data(), bytes) == 0) {
            sl = &c;
            break;
        }
    if (sl) {
        // Staged on another stream and possibly not there yet: order this stream after it.
        if (sl->pending && sl->last_stream != stream) DDL_HIP(hipStreamWaitEvent(stream, sl->done, 0));
    } else {
        for (;;) {
            for (int tries = 0; tries < kSlots && !sl; ++tries) {
                Slot& c = ds->slot[ds->next];
                ds->next = (ds->next + 1) % kSlots;
                if (c.pending) {
                    const hipError_t q = hipEventQuery(c.done);
                    if (q == hipErrorNotReady) continue;
                    if (q != hipSuccess) return runtime_error(q, "hipEventQuery");
                    c.pending = false;
                }
                sl = &c;
            }
            if (sl) break;
            // Every slot is still in use by enqueued work: wait for the oldest one without
            // holding the lock (events are never destroyed), then look again.
            hipEvent_t oldest = ds->slot[ds->next].done;
            lock.unlock();
            DDL_HIP(hipEventSynchronize(oldest));
            lock.lock();
        }
        sl->bytes = 0;
        if (bytes > sl->cap) {
            if (sl->host) DDL_HIP(hipHostFree(sl->host));
            if (sl->dev) DDL_HIP(hipFree(sl->dev));
            sl->host = sl->dev = nullptr;
            sl->cap = 0;
            const size_t cap_bytes = std::max<size_t>(bytes * 2, 16 * 1024);
            DDL_HIP(hipHostMalloc(&sl->host, cap_bytes, hipHostMallocDefault));
            DDL_HIP(hipMalloc(&sl->dev, cap_bytes));
            sl->cap = cap_bytes;
        }
        if (!sl->done) DDL_HIP(hipEventCreateWithFlags(&sl->done, hipEventDisableTiming));
        std::memcpy(sl->host, image.data(), bytes);
        DDL_HIP(hipMemcpyAsync(sl->dev, sl->host, bytes, hipMemcpyHostToDevice, stream));
        sl->bytes = bytes;
        sl->hash = hash;
    }
    st = launch_work(T, sl->dev, work, hip_stream);
    // Record even after a failed launch: the copy above may still be in flight.
    if (hipEventRecord(sl->done, stream) == hipSuccess) {
        sl->pending = true;
        sl->last_stream = stream;
    }
    return st;
}

ddl_status ddl_plan_create(const ddl_fragment* frags, int num_frags, ddl_plan** plan_out)
{
    if (!plan_out) return DDL_ERR_INVALID_ARG;
    *plan_out = nullptr;
    if (num_frags < 1 || !frags) return DDL_ERR_INVALID_ARG;
    for (int i = 0; i < num_frags; ++i) {
        const ddl_status st = check_fragment_shape(frags[i]);
        if (st != DDL_OK) return st;
    }
    ddl_plan* p = new (std::nothrow) ddl_plan();
    if (!p) return DDL_ERR_RUNTIME;
    std::vector<uint32_t> bits((size_t)num_frags, 0xffffffffu);
    const ddl_status st = build_table(frags, num_frags, bits.data(), p->table);
    if (st != DDL_OK) {
        delete p;
        return st;
    }
    hipError_t e = hipGetDevice(&p->device);
    if (e == hipSuccess && !p->table.segs.empty()) {
        const size_t bytes = p->table.bytes();
        std::vector<char> image(bytes);
        p->table.copy_to(image.data());
        e = hipMalloc(&p->d_table, bytes);
        if (e == hipSuccess) e = hipMemcpy(p->d_table, image.data(), bytes, hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        if (p->d_table) (void)hipFree(p->d_table);
        delete p;
        return runtime_error(e, "plan upload");
    }
    *plan_out = p;
    return DDL_OK;
}

ddl_status ddl_plan_merge(ddl_plan* plan, const ddl_sync* syncs, int count, void* hip_stream)
{
    if (!plan || count < 0 || (count > 0 && !syncs)) return DDL_ERR_INVALID_ARG;
    if (count == 0) return DDL_OK;
    const Table& T = plan->table;
    std::vector<Work> work;
    work.reserve((size_t)count);
    std::vector<char> seen(T.frags.size(), 0);
    for (int i = 0; i < count; ++i) {
        const ddl_sync& s = syncs[i];
        if (s.fragment < 0 || (size_t)s.fragment >= T.frags.size()) return DDL_ERR_INVALID_ARG;
        if (seen[(size_t)s.fragment]) return DDL_ERR_ALIAS;
        seen[(size_t)s.fragment] = 1;
        if (!finite_nonneg(s.lr) || !finite_nonneg(s.mu)) return DDL_ERR_INVALID_ARG;
        const FragInfo& f = T.frags[(size_t)s.fragment];
        double w[DDL_MAXL];
        const ddl_status st = weights_tokens(s.token_counts, s.quorum_mask, f.M, w);
        if (st != DDL_OK) return st;
        Work wk;
        wk.frag = (uint32_t)s.fragment;
        wk.lr = s.lr;
        wk.mu = s.mu;
        compact(w, f.M, wk.q);
        if (f.num_segs > 0 && (wk.q.present_bits & ~f.nonnull_bits)) return DDL_ERR_INVALID_ARG;
        work.push_back(wk);
    }
    return launch_work(T, plan->d_table, work, hip_stream);
}

ddl_status ddl_plan_destroy(ddl_plan* plan)
{
    if (!plan) return DDL_OK;
    ddl_status st = DDL_OK;
    if (plan->rda) ddl_rda_plan_free(plan->rda);
    if (plan->d_q4) (void)hipFree(plan->d_q4);
    if (plan->d_table) {
        const hipError_t e = hipFree(plan->d_table);
        if (e != hipSuccess) st = runtime_error(e, "hipFree");
    }
    delete plan;
    return st;
}

int ddl_plan_num_fragments(const ddl_plan* plan)
{
    return plan ? (int)plan->table.frags.size() : 0;
}

size_t ddl_plan_num_elements(const ddl_plan* plan) { return plan ? (size_t)plan->table.elems : 0; }

ddl_status ddl_copy_probe(void* dst, const void* src, size_t bytes, void* hip_stream)
{
    if (!dst || !src || bytes % 16 || !aligned(dst, 16) || !aligned(src, 16))
        return DDL_ERR_INVALID_ARG;
    if (bytes == 0) return DDL_OK;
    const uintptr_t d = (uintptr_t)dst, s = (uintptr_t)src;
    if (d < s + bytes && s < d + bytes) return DDL_ERR_ALIAS;
    const uint64_t n16 = bytes / 16;
    const uint64_t blocks = (n16 + DDL_BLOCK - 1) / DDL_BLOCK;
    if (blocks > 0x7fffffffull) return DDL_ERR_INVALID_ARG;
    const uint32_t grid = (uint32_t)blocks;
    const int e = ddl_launch_copy(dst, src, n16, grid, hip_stream);
    if (e != (int)hipSuccess) return runtime_error((hipError_t)e, "copy kernel launch");
    return DDL_OK;
}

ddl_status ddl_set_option(const char* name, long value)
{
    if (!name) return DDL_ERR_INVALID_ARG;
    if (!std::strcmp(name, "tiles_per_block")) {
        if (value != -1 && (value < 1 || value > 1024)) return DDL_ERR_INVALID_ARG;
        g_tiles_per_block = value;
        return DDL_OK;
    }
    if (!std::strcmp(name, "max_blocks_per_cu")) {
        if (value != 0 && value != -1 && (value < 3 || value > 64)) return DDL_ERR_INVALID_ARG;
        g_max_blocks_per_cu = value;
        return DDL_OK;
    }
    if (!std::strcmp(name, "tile_rotate")) {
        if (value != 0 && (value < 2 || value > 4096)) return DDL_ERR_INVALID_ARG;
        g_tile_rotate = value;
        return DDL_OK;
    }
#ifdef DDL_TRACE
    if (!std::strcmp(name, "trace_buffer")) {
        g_trace_buffer = value;
        return DDL_OK;
    }
#endif
    if (!std::strcmp(name, "max_tiles_per_launch")) {
        if (value < -1 || value > 0x7fffffffl) return DDL_ERR_INVALID_ARG;
        g_max_tiles_per_launch = value;
        return DDL_OK;
    }
    if (!std::strcmp(name, "part_megabytes")) {
        if (value < 1 || value > 1000000) return DDL_ERR_INVALID_ARG;
        g_part_megabytes = value;
        return DDL_OK;
    }
    if (!std::strcmp(name, "rda_blocks_per_cu")) {
        if (value != 0 && (value < 3 || value > 64)) return DDL_ERR_INVALID_ARG;
        ddl_opt_rda_blocks_per_cu = value;
        return DDL_OK;
    }
    return DDL_ERR_INVALID_ARG;
}

ddl_status ddl_get_option(const char* name, long* value_out)
{
    if (!name || !value_out) return DDL_ERR_INVALID_ARG;
    if (!std::strcmp(name, "tiles_per_block")) {
        *value_out = g_tiles_per_block;
        return DDL_OK;
    }
    if (!std::strcmp(name, "max_blocks_per_cu")) {
        *value_out = g_max_blocks_per_cu;
        return DDL_OK;
    }
    if (!std::strcmp(name, "tile_rotate")) {
        *value_out = g_tile_rotate;
        return DDL_OK;
    }
    if (!std::strcmp(name, "max_tiles_per_launch")) {
        *value_out = g_max_tiles_per_launch;
        return DDL_OK;
    }
    if (!std::strcmp(name, "part_megabytes")) {
        *value_out = g_part_megabytes;
        return DDL_OK;
    }
    if (!std::strcmp(name, "grids_enqueued")) {
        *value_out = ddl_stat_grids;
        return DDL_OK;
    }
    if (!std::strcmp(name, "rda_blocks_per_cu")) {
        *value_out = ddl_opt_rda_blocks_per_cu;
        return DDL_OK;
    }
    return DDL_ERR_INVALID_ARG;
}

}  // extern "C"
