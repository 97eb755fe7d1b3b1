// Balanced tensor fragmentation (Appendix C of the paper): greedy number partitioning of the
// model's tensors into fragments of nearly equal total size.  Host code only.
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
