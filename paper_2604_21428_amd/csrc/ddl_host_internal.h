// Host-side structures of libddlsync shared between its translation units: the quorum after
// weighting, the descriptor table of a set of fragments, and the plan object.
#pragma once
#include <hip/hip_runtime.h>

#include <cstring>
#include <vector>

#include "../../include/ddlsync.h"
#include "ddl_device.h"

namespace ddlh {

// The learners that contribute to one sync, compacted, with their normalised weights rounded
// once to fp32 for the device.
struct Quorum {
    int Mq = 0;
    float w[DDL_MAXL];
    uint8_t idx[DDL_MAXL];
    uint32_t present_bits = 0;
};

struct FragInfo {
    uint32_t seg_begin = 0, num_segs = 0, tiles = 0;
    uint32_t coarse_begin = 0, coarse_shift = 0;
    int M = 0;
    ddl_dtype dt = DDL_F32;
    uint64_t elems = 0;
    uint32_t nonnull_bits = 0;  // learners whose pointer is non-NULL in every segment
};

struct Table {
    std::vector<DdlSegDesc> segs;  // empty segments are left out
    std::vector<uint32_t> origin;  // per descriptor: its position among ALL segments given
    uint32_t given_segs = 0;       // segments given, empty ones included
    std::vector<FragInfo> frags;
    std::vector<uint32_t> coarse;  // per fragment: descriptor (relative) holding tile i << shift
    uint64_t elems = 0;

    size_t seg_bytes() const { return segs.size() * sizeof(DdlSegDesc); }
    size_t bytes() const { return seg_bytes() + coarse.size() * sizeof(uint32_t); }
    // Device image: the descriptors followed by the coarse index.
    void copy_to(void* dst) const
    {
        std::memcpy(dst, segs.data(), seg_bytes());
        std::memcpy(static_cast<char*>(dst) + seg_bytes(), coarse.data(),
                    coarse.size() * sizeof(uint32_t));
    }
};

// w_m = q_m n_m / sum_k q_k n_k in fp64 (Algorithm 2, "Weight", tokens-only reading).
ddl_status weights_tokens(const uint64_t* t, const uint8_t* q, int M, double* w);
// Drops learners of weight zero; rounds the rest once to fp32.
void compact(const double* w, int M, Quorum& out);
bool finite_nonneg(float x);
// Unused dynamic LDS per workgroup that enforces the max_blocks_per_cu option on the
// streaming merge kernels (0: no cap).  elem_bytes: bytes per learner element (0: 4-bit codes).
uint32_t merge_lds_cap_bytes(int elem_bytes, int Mq);
// Group size of the tile rotation (option tile_rotate; 0: off).
uint32_t tile_rotate();
// Most 1024-element tiles one kernel launch should cover (0: no limit): options
// max_tiles_per_launch / part_megabytes.  elem_bytes: bytes per learner element (0: 4-bit
// codes); extra: bytes per element beyond the learners' and the 16 of Theta and v.
uint32_t max_tiles_per_launch(int elem_bytes, int Mq, int extra = 0);
// One sync of one fragment of a table, ready to launch.
struct Work {
    uint32_t frag;  // index into Table::frags
    Quorum q;
    float lr, mu;
};
// The learners' outer gradients as 4-bit codes: the device table parallel to the descriptors
// (null for the flat variant) and the block length of the scales.
struct Q4Source {
    const DdlQ4Desc* d_table;
    uint32_t block_len;
};
// Enqueues the fragments in `work` (merge + outer step): one launch per group of up to
// DDL_MAX_ITEMS fragments with the same learner type and number of contributing learners, each
// cut into parts if long.  q4: the fragments' learners come as 4-bit codes (else their
// bf16 / fp32 copies in the descriptors).
ddl_status launch_work(const Table& T, const void* d_table, std::vector<Work>& work, void* stream,
                       const Q4Source* q4 = nullptr);
// The same for ONE tensor whose descriptor travels in the kernel-argument block (src: 0 fp32,
// 1 bf16 learners in desc.learner; DDL_SRC_Q4: codes and scales in *q4d, blocks of block_len).
ddl_status launch_flat(const DdlSegDesc& desc, int src, const Quorum& q, float lr, float mu,
                       void* stream, const DdlQ4Desc* q4d = nullptr, uint32_t block_len = 0);
// Enqueues the direct-averaging merge + outer step of one tensor given by its descriptor.
ddl_status launch_one_direct(const DdlSegDesc& desc, ddl_dtype dt, const Quorum& q, float lr,
                             float mu, void* stream);
// Address ranges of a call and the overlap rule: an output range (Theta, v, a bf16 copy) may
// overlap nothing, inputs may overlap inputs.  add_range: false if the range would wrap.
struct Range {
    uintptr_t lo, hi;
    bool out;
};
bool add_range(const void* p, size_t elem, size_t n, bool out, std::vector<Range>& r);
bool ranges_alias(std::vector<Range>& r);
void fill_desc(DdlSegDesc& d, float* theta, float* v, void* theta_bf16,
               const void* const* learners, int M, size_t n, uint32_t tile_begin);
// Records the message for ddl_last_error_message and returns DDL_ERR_RUNTIME.
ddl_status runtime_error(hipError_t e, const char* what);
// Records a message for ddl_last_error_message (for an error that is not a HIP failure).
void set_error_message(const char* text);

}  // namespace ddlh

// Per-plan data of the RDA merge (row classes, their device tables); owned by the plan.
struct DdlRdaPlan;
void ddl_rda_plan_free(DdlRdaPlan* p);

struct ddl_plan {
    int device = 0;
    ddlh::Table table;
    void* d_table = nullptr;  // descriptors followed by the coarse index
    DdlRdaPlan* rda = nullptr;
    // 4-bit sources (ddl_plan_set_q4_sources): DdlQ4Desc per descriptor, on the device
    void* d_q4 = nullptr;
    std::vector<DdlQ4Desc> q4_host;  // the same table on the host
    uint32_t q4_block_len = 0;
    std::vector<uint32_t> q4_nonnull_bits;  // per fragment: learners with codes and scales in
                                            // every tensor
};
