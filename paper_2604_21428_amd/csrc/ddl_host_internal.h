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
// Enqueues the direct-averaging merge + outer step of one tensor given by its descriptor.
ddl_status launch_one_direct(const DdlSegDesc& desc, ddl_dtype dt, const Quorum& q, float lr,
                             float mu, void* stream);
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
};
