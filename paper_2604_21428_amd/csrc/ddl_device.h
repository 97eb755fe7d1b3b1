// Structures shared by the host side of libddlsync and its gfx950 kernels.
//
// A launch works on "tiles": runs of DDL_TILE consecutive elements of the tensors ("segments")
// of up to DDL_MAX_ITEMS fragments that share learner dtype and number of contributing
// learners.  A workgroup handles `tiles_per_block` consecutive tiles of the launch.
// Segment descriptors live in device memory (or, for the single flat fragment, inside the
// kernel argument block); everything that changes per sync -- weights, which learners
// contribute, lr, mu -- travels in the kernel argument block, i.e. in constant memory that
// the wave reads with scalar loads.
#pragma once
#include <stdint.h>

#include <atomic>

#define DDL_MAXL 16         // learners per fragment, = DDL_MAX_LEARNERS of the public header
#define DDL_MAX_ITEMS 16    // fragments per launch
#define DDL_BLOCK 256       // threads per workgroup: 4 wavefronts of 64
#define DDL_TILE (DDL_BLOCK * 4)  // elements per tile: one group of four per lane
#define DDL_LDS_PER_CU (160 * 1024)  // bytes of LDS per compute unit on gfx950

struct DdlSegDesc {
    float* theta;                   // n fp32, read and written
    float* v;                       // n fp32, read and written
    const void* learner[DDL_MAXL];  // learner m's copy (bf16 or fp32), read if it contributes
    void* theta_bf16;               // optional: receives the new Theta as bf16 (n elements)
    uint64_t n;                     // elements (> 0)
    uint32_t tile_begin;            // first tile of this segment within its fragment
    uint16_t learner_aligned;       // bit m: learner[m] is 16-byte aligned
    uint8_t base_aligned;           // theta, v 16-byte and theta_bf16 (if any) 8-byte aligned
    uint8_t pad;
};
static_assert(sizeof(DdlSegDesc) == 168, "descriptor layout");

// The 4-bit sources of one tensor (codes and per-block scales of every learner), parallel to
// its DdlSegDesc: entry i of the plan's DdlQ4Desc table belongs to descriptor i.
struct DdlQ4Desc {
    const uint8_t* codes[DDL_MAXL];  // two signed 4-bit codes per byte, element 2k in the low nibble
    const float* scales[DDL_MAXL];   // one fp32 scale per block of block_len elements
};
static_assert(sizeof(DdlQ4Desc) == 256, "q4 descriptor layout");

struct DdlItem {
    uint32_t seg_begin;     // first descriptor of the fragment in the table
    uint32_t num_segs;      // its number of (non-empty) segments
    uint32_t tile_off;      // first tile of the fragment within this launch
    uint32_t present_bits;  // bit m: learner m contributes
    float w[DDL_MAXL];      // normalised weights of the contributing learners, compacted
    uint8_t idx[DDL_MAXL];  // learner index of compacted entry j
    float lr, mu;
    uint32_t coarse_begin;  // first entry of the fragment's coarse index in DdlLaunchArgs::coarse
    uint32_t coarse_shift;  // entry i covers tiles [i << shift, (i + 1) << shift)
};
static_assert(sizeof(DdlItem) == 112, "item layout");

struct DdlLaunchArgs {
    const DdlSegDesc* segs;  // device table (unused by the flat variant)
    // Coarse index into the table: entry i of a fragment is the descriptor that holds tile
    // i << shift (clamped to the last descriptor past the end), so a tile's descriptor lies
    // between entries i and i + 1 -- usually the same one, and no search is needed.
    const uint32_t* coarse;
    uint32_t total_tiles;      // tiles of all fragments of the launch
    uint32_t tile_base;        // first tile this grid covers (a long launch goes out in parts)
    uint32_t tiles_per_block;  // >= 1
    int32_t num_items;
    int32_t rotate;  // 0: workgroup b takes tile b; k > 0: tiles rotated within groups of k
#ifdef DDL_TRACE
    uint64_t* trace;  // diagnostic build only: per workgroup {start clock, XCD, tile}
#endif
    // 4-bit sources only: the table parallel to segs (unused by the flat variant), and the
    // block length of the scales (block_shift = log2 of it, or 0xffffffff if no power of two).
    const DdlQ4Desc* q4;
    uint32_t block_len;
    uint32_t block_shift;
    DdlItem item[DDL_MAX_ITEMS];
    DdlSegDesc flat;         // the one segment of the flat variant
    DdlQ4Desc flat_q4;       // ... and its 4-bit sources
};
static_assert(sizeof(DdlLaunchArgs) <= 4096, "kernel argument block limit");

// Launches the merge kernel specialised for (learner dtype, contributing learners, flat or
// table).  dtype: 0 fp32, 1 bf16 (values of ddl_dtype), 2: the learners' outer gradients as
// 4-bit codes with block scales.  Returns a hipError_t as int.
#define DDL_SRC_Q4 2
// lds_bytes of (unused) dynamic LDS per workgroup cap how many workgroups a compute unit holds.
int ddl_launch_merge(int dtype, int Mq, bool flat, uint32_t grid, uint32_t lds_bytes, void* stream,
                     const DdlLaunchArgs& args);

// The same for a launch of args.total_tiles tiles cut into parts of at most max_tiles tiles
// (0: one part), enqueued back to back: sets args.tile_base per part.
int ddl_launch_merge_parts(int dtype, int Mq, bool flat, uint32_t max_tiles, uint32_t lds_bytes,
                           void* stream, DdlLaunchArgs& args);

// Launches the plain 16-byte-per-lane copy of n16 * 16 bytes; grid = ceil(n16 / DDL_BLOCK).
int ddl_launch_copy(void* dst, const void* src, uint64_t n16, uint32_t grid, void* stream);

// Launch-shape knob of the one-kernel RDA shape (set through ddl_set_option): at most this
// many workgroups resident per compute unit (0: no cap), enforced with unused dynamic LDS.
extern std::atomic<long> ddl_opt_rda_blocks_per_cu;

// Statistic read through ddl_get_option("grids_enqueued"): kernel grids this process has
// enqueued so far (one sync of a fragment may be several).  Every launch site counts itself.
extern std::atomic<long> ddl_stat_grids;
#define DDL_COUNT_GRID() ((void)ddl_stat_grids.fetch_add(1, std::memory_order_relaxed))
