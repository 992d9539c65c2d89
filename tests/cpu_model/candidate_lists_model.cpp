// Host-side model of the candidate-mode selection of libxbq.so (select_dense, select_merge and
// its exact rescan) over one query's distances, for tests that run without a GPU.  The rule that
// decides how long the list stays and which later rows still matter is the product's own
// (csrc/xbq_cut.h, included here); the data movement around it -- row groups, the survivor list
// with its capacity, the bounded buffer of the rescan that is compacted whenever another
// workgroup's worth of keys might not fit -- is modelled with std::sort in place of the LDS sorts.
// Built by tests/test_candidate_lists_model.py with g++.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "xbq_cut.h"

namespace {

uint64_t key(uint32_t D, uint32_t row) { return (static_cast<uint64_t>(D) << 32) | row; }
uint32_t dist_of(uint64_t k) { return static_cast<uint32_t>(k >> 32); }

struct State {
    std::vector<uint64_t> list;   // kept keys, ascending
    uint32_t thr = 0xffffffffu;
};

int count_within(const std::vector<uint64_t>& sorted, uint32_t bound)
{
    int c = 0;
    while (c < static_cast<int>(sorted.size()) && dist_of(sorted[c]) <= bound) ++c;
    return c;
}

// write_topk of the kernels, candidate mode
void store_head(State& st, std::vector<uint64_t>& sorted, int k, int extra, int keep_max, uint32_t thr_before,
                bool any_order)
{
    const uint32_t bound = dist_of(sorted[k - 1]) + static_cast<uint32_t>(extra);
    const xbq::ListCut cut =
        xbq::candidate_list_cut(sorted.data(), count_within(sorted, bound), keep_max, bound, thr_before, any_order);
    sorted.resize(cut.keep);
    st.list = sorted;
    st.thr = cut.thr;
}

}  // namespace

// D[n]: distances of one query in the order the rows are taken; rows[i] is the number of the row
// at place i (null: the rows come in ascending order, rows[i] = i; otherwise any permutation, and
// the cut uses the rule for rows in any order).  Group 0 = places [0, first) is sorted whole; every
// later group of `group` rows is filtered with the threshold; a group with more than `cap`
// survivors (or every group, if force_rescan) takes the rescan with a buffer of `capacity` keys
// filled `block` rows at a time.  Writes the final list (at most keep_max keys) and returns its
// length; *thr_out is the final threshold.
extern "C" int model_candidate_lists(const uint32_t* D, const uint32_t* rows, int64_t n, int k, int extra, int keep_max,
                                     int first, int group, int cap, int capacity, int block, int force_rescan,
                                     uint64_t* list_out, uint32_t* thr_out)
{
    const bool any_order = rows != nullptr;
    auto row_at = [&](int64_t i) { return rows != nullptr ? rows[i] : static_cast<uint32_t>(i); };
    if (first > n) first = static_cast<int>(n);
    if (k > first || keep_max < k || capacity < keep_max + 2 * block) return -1;
    State st;
    {
        std::vector<uint64_t> buf;
        for (int r = 0; r < first; ++r) buf.push_back(key(D[r], row_at(r)));
        std::sort(buf.begin(), buf.end());
        store_head(st, buf, k, extra, keep_max, 0xffffffffu, any_order);
    }
    for (int64_t g0 = first; g0 < n; g0 += group) {
        const int64_t g1 = g0 + group < n ? g0 + group : n;
        std::vector<uint64_t> survivors;
        for (int64_t r = g0; r < g1; ++r)
            if (D[r] < st.thr) survivors.push_back(key(D[r], row_at(r)));
        if (!force_rescan && static_cast<int>(survivors.size()) <= cap) {
            if (survivors.empty()) continue;
            std::vector<uint64_t> buf = st.list;
            buf.insert(buf.end(), survivors.begin(), survivors.end());
            std::sort(buf.begin(), buf.end());
            store_head(st, buf, k, extra, keep_max, st.thr, any_order);
            continue;
        }
        std::vector<uint64_t> buf = st.list;           // rescan_rows of the kernels
        uint32_t thr = st.thr;
        for (int64_t base = g0; base < g1; base += block) {
            for (int64_t r = base; r < base + block && r < g1; ++r)
                if (D[r] < thr) buf.push_back(key(D[r], row_at(r)));
            if (static_cast<int>(buf.size()) > capacity) return -2;      // the kernel's buffer would overflow
            if (static_cast<int>(buf.size()) > capacity - block) {
                std::sort(buf.begin(), buf.end());
                const uint32_t bound = dist_of(buf[k - 1]) + static_cast<uint32_t>(extra);
                const xbq::ListCut cut =
                    xbq::candidate_list_cut(buf.data(), count_within(buf, bound), keep_max, bound, thr, any_order);
                buf.resize(cut.keep);
                thr = cut.thr;
            }
        }
        std::sort(buf.begin(), buf.end());
        store_head(st, buf, k, extra, keep_max, thr, any_order);
    }
    for (size_t i = 0; i < st.list.size(); ++i) list_out[i] = st.list[i];
    *thr_out = st.thr;
    return static_cast<int>(st.list.size());
}
