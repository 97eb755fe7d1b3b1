// Host-only helpers around the merge: balanced tensor fragmentation (Appendix C of the paper:
// greedy number partitioning of the model's tensors into fragments of nearly equal total
// size) and the placement of a fragment's resident arrays in device memory.
#include <algorithm>
#include <cstdint>
#include <functional>
#include <numeric>
#include <queue>
#include <utility>
#include <vector>

#include "../../include/ddlsync.h"

extern "C" ddl_status ddl_balanced_fragments(const uint64_t* sizes, int num_tensors,
                                             int num_fragments, int* fragment_of)
{
    if (num_tensors < 0 || num_fragments < 1) return DDL_ERR_INVALID_ARG;
    if (num_tensors > 0 && (!sizes || !fragment_of)) return DDL_ERR_INVALID_ARG;
    // Largest first; equal sizes keep their order.
    std::vector<int> order((size_t)num_tensors);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return sizes[a] > sizes[b]; });
    // Min-heap on (load, fragment index): the lightest fragment, lowest index among equals.
    typedef std::pair<unsigned __int128, int> Bin;
    auto heavier = [](const Bin& a, const Bin& b) {
        return a.first != b.first ? a.first > b.first : a.second > b.second;
    };
    std::priority_queue<Bin, std::vector<Bin>, decltype(heavier)> bins(heavier);
    for (int p = 0; p < num_fragments; ++p) bins.push(Bin(0, p));
    for (int i : order) {
        Bin b = bins.top();
        bins.pop();
        fragment_of[i] = b.second;
        b.first += sizes[i];
        bins.push(b);
    }
    return DDL_OK;
}

// Placement of the syncer's resident state.  The merge streams 2 + Mq arrays in lockstep: at
// any moment a workgroup reads the SAME element range of Theta, v and every contributing
// learner.  If those arrays start at addresses that are equal modulo 64 KiB -- which is what
// back-to-back allocations of tensors with power-of-two sizes give -- the simultaneous
// requests of a tile fall on the same memory channels and banks, and the pass loses 10-16 %
// on MI355X.  Staggering the arrays' start addresses by one tile's footprint (4 KiB of fp32,
// 2 KiB of bf16) within the 64 KiB stripe removes that.
namespace {
constexpr size_t kStripe = 65536;

// Smallest offset >= cur whose remainder modulo the stripe is `residue`.
size_t place(size_t cur, size_t residue)
{
    const size_t base = cur / kStripe * kStripe + residue;
    return base >= cur ? base : base + kStripe;
}
}  // namespace

extern "C" ddl_status ddl_arena_layout(const uint64_t* sizes, int num_tensors, int M,
                                       ddl_dtype learner_dtype, int with_theta_bf16,
                                       ddl_arena_slot* slots_out, size_t* arena_bytes_out)
{
    if (num_tensors < 0 || M < 1 || M > DDL_MAX_LEARNERS || !arena_bytes_out)
        return DDL_ERR_INVALID_ARG;
    if (learner_dtype != DDL_F32 && learner_dtype != DDL_BF16) return DDL_ERR_INVALID_ARG;
    if (num_tensors > 0 && (!sizes || !slots_out)) return DDL_ERR_INVALID_ARG;
    const size_t b = learner_dtype == DDL_BF16 ? 2 : 4;
    size_t cur = 0;
    for (int t = 0; t < num_tensors; ++t) {
        const uint64_t n = sizes[t];
        if (n > (uint64_t)1 << 46) return DDL_ERR_INVALID_ARG;
        ddl_arena_slot& s = slots_out[t];
        size_t residue = 0;  // where, within the stripe, the next array of this tensor starts
        auto take = [&](size_t elem_bytes) {
            const size_t at = place(cur, residue % kStripe);
            cur = at + (size_t)n * elem_bytes;
            residue += 1024 * elem_bytes;  // one tile of this array
            return at;
        };
        s.theta = take(4);
        s.v = take(4);
        s.theta_bf16 = with_theta_bf16 ? take(2) : (size_t)-1;
        for (int m = 0; m < DDL_MAX_LEARNERS; ++m) s.learner[m] = m < M ? take(b) : (size_t)-1;
    }
    *arena_bytes_out = (cur + 255) & ~(size_t)255;
    return DDL_OK;
}
