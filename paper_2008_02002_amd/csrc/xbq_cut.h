// How long a candidate list may stay, and which later rows can still enter it (candidate mode
// of the selection kernels: Algorithm 1's list "every row with D <= D_K + extra", bounded to
// the keep_max best keys).  Plain C++ so that a host-side model of the kernels can use the very
// same rule (tests/cpu_model).
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define XBQ_HOST_DEVICE __host__ __device__
#else
#define XBQ_HOST_DEVICE
#endif

namespace xbq {

struct ListCut {
    int keep;        // keys of the sorted buffer that stay in the list
    uint32_t thr;    // a row not seen so far matters iff D < thr
};

// `sorted`: ascending keys (D << 32 | row) of every row seen so far that could still be in the
// list; `within` of them have D <= bound, bound = D_K + extra with D_K the K-th smallest D.
// The list is the first keep_max of those.  While it is not full, a later row enters when
// D <= bound.  Once it is full, a later row enters only by beating the last kept key: when rows
// are seen in ascending order its number is higher, so only with a smaller D; seen in any
// order (any_order) an equal D may win the tie, and the threshold is one higher.  The threshold
// never rises: rows refused under an earlier, tighter threshold are not in the buffer, so a
// wider one would admit rows that sort behind rows already dropped.
XBQ_HOST_DEVICE inline ListCut candidate_list_cut(const uint64_t* sorted, int within, int keep_max, uint32_t bound,
                                                  uint32_t thr_before, bool any_order = false)
{
    ListCut c;
    const bool full = within >= keep_max;
    c.keep = full ? keep_max : within;
    const uint32_t now = full ? static_cast<uint32_t>(sorted[keep_max - 1] >> 32) + (any_order ? 1u : 0u) : bound + 1u;
    c.thr = now < thr_before ? now : thr_before;
    return c;
}

}  // namespace xbq
