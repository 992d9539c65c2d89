// Selection kernels: exact top-K per query on 64-bit keys (D << 32 | row), smaller first.
// Smaller D means larger score S = d(2^B-1)^2 - 2D (Eq. 7 of Section 3.3), so ascending
// keys are "score descending, ties to the lower row number".
//
// The paper selects with a histogram of the integer distances (Section 4.1 "Histogram and
// Select"); here the scan already filtered with a per-query threshold, so what is left per
// query is a short list that one workgroup sorts in LDS.
//
//   select_dense  : first group of rows, every distance stored -> top-K keys + threshold
//   select_merge  : current top-K + candidates that beat the threshold -> new top-K; for a
//                   query whose candidate list overflowed it instead re-scores the group's
//                   rows with a running threshold and a bounded LDS buffer (slow, always
//                   exact, and only ever taken when the row order is adversarial)
// Plain top-K selects with a histogram and orders only the keys of the boundary bin
// (select_by_histogram); the candidate lists of Algorithm 1 (extra >= 0) stay sorted and are
// merged with the LDS sorting network.

#include "xbq_cut.h"
#include "xbq_device.h"

namespace xbq {

__device__ __forceinline__ void write_result(const SelectArgs& a, int q, const uint64_t* keys)
{
    const int32_t full = a.d * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) {
        const uint64_t key = keys[t];
        a.idx[static_cast<size_t>(q) * a.k + t] = static_cast<int32_t>(key & 0xffffffffu);
        a.score[static_cast<size_t>(q) * a.k + t] = full - 2 * static_cast<int32_t>(key >> 32);
    }
}

// Number of keys with D <= bound among `have` ascending keys in LDS (a single step in a sorted
// array).  All threads call this; `scratch` is one LDS word; ends with a barrier.
__device__ int count_within(const uint64_t* keys, int have, uint32_t bound, int* scratch)
{
    __syncthreads();
    if (threadIdx.x == 0) *scratch = static_cast<uint32_t>(keys[have - 1] >> 32) <= bound ? have : 0;
    __syncthreads();
    for (int t = threadIdx.x; t + 1 < have; t += blockDim.x)
        if (static_cast<uint32_t>(keys[t] >> 32) <= bound && static_cast<uint32_t>(keys[t + 1] >> 32) > bound)
            *scratch = t + 1;
    __syncthreads();
    const int within = *scratch;
    __syncthreads();
    return within;
}

// Store the head of the sorted keys as the query's new list and derive its threshold.
// Plain top-K: the first k keys; later rows matter only if D < D_k (an equal D loses the tie
// to the rows already held, which all have lower numbers) -- or, when the row groups are spread
// over the database (bundle_mul > 1) and a later row may have a lower number, if D <= D_k.  Candidate mode (extra >= 0):
// every key with D <= D_k + extra, at most keep_max (the best by key); see candidate_list_cut.
// `have` sorted keys are in LDS; all threads call this, with a barrier before it.
// thr_before: the threshold the keys were collected under (0xffffffff for the first group).
__device__ void write_topk(const SelectArgs& a, int q, const uint64_t* keys, int have, int* scratch, uint32_t thr_before)
{
    const uint32_t dk = static_cast<uint32_t>(keys[a.k - 1] >> 32);
    int keep = a.k;
    if (a.extra >= 0) {
        const uint32_t bound = dk + static_cast<uint32_t>(a.extra);
        const int within = count_within(keys, have, bound, scratch);
        const ListCut cut = candidate_list_cut(keys, within, a.keep_max, bound, thr_before, a.bundle_mul > 1);
        keep = cut.keep;
        if (threadIdx.x == 0) {
            a.len[q] = static_cast<uint32_t>(keep);
            a.thr[q] = cut.thr;
            a.cnt[q] = 0;
        }
    } else if (threadIdx.x == 0) {
        const uint32_t now = dk + (a.bundle_mul > 1 ? 1u : 0u);
        a.thr[q] = now < thr_before ? now : thr_before;
        a.cnt[q] = 0;
    }
    for (int t = threadIdx.x; t < keep; t += blockDim.x) a.topk[static_cast<size_t>(q) * a.keep_max + t] = keys[t];
    if (a.final_group && a.extra < 0) write_result(a, q, keys);
}

// ---------------------------------------------------------------------------------------
// Plain top-K without sorting what is thrown away.  The keys of one query (at most kSortCap:
// the K held so far plus the survivors of a group, or the rows of the first group) sit in
// registers, kSelHeld per thread.  A histogram of D >> shift in LDS gives the bin that holds
// the K-th smallest distance (Algorithm 1's boundary, Section 4.1, at bin resolution); only
// the keys of that one bin are ordered to find the K-th smallest key exactly; every key at or
// below it is kept.  The kept keys go back to the query's list unsorted (nothing downstream
// of a non-final group needs them sorted) and only the final group sorts its K keys.
// Returns false, having written nothing, when the boundary bin holds more keys than the tie
// buffer (massive ties): the caller then sorts everything.
// ---------------------------------------------------------------------------------------
constexpr int kSelHeld = kSortCap / kBlock;              // 16 keys per thread
constexpr int kTieBuf = 1024;                            // keys of the boundary bin that are ordered in LDS; >= XBQ_MAX_K

struct SelectLds {
    uint32_t hist[kHistBins];
    uint64_t tie[kTieBuf];
    uint64_t kth;
    uint32_t fill;
    int bin;
    uint32_t below;
};

__device__ __forceinline__ void append_wave_lds(bool pass, uint64_t key, uint64_t* list, uint32_t* counter)
{
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    const int leader = __ffsll(static_cast<long long>(mask)) - 1;
    uint32_t base = 0;
    if (lane_id() == leader) base = atomicAdd(counter, static_cast<uint32_t>(__popcll(mask)));
    base = __shfl(base, leader);
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
    if (pass) list[base + rank] = key;
}

__device__ bool select_by_histogram(const SelectArgs& a, int q, const uint64_t (&r)[kSelHeld], SelectLds& s)
{
    int shift = 0;
    const int64_t dmax = static_cast<int64_t>(a.d) * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    while ((dmax >> shift) >= kHistBins) ++shift;
    for (int t = threadIdx.x; t < kHistBins; t += kBlock) s.hist[t] = 0;
    if (threadIdx.x == 0) s.fill = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kSelHeld; ++u)
        if (r[u] != kPadKey) atomicAdd(&s.hist[static_cast<uint32_t>(r[u] >> 32) >> shift], 1u);
    __syncthreads();
    if (threadIdx.x < kLanes) {
        uint32_t below;
        const int bin = wave_boundary_bin(s.hist, static_cast<uint32_t>(a.k), &below);
        if (threadIdx.x == 0) { s.bin = bin; s.below = below; }
    }
    __syncthreads();
    const uint32_t bin = static_cast<uint32_t>(s.bin);   // >= 0: the caller passes at least k keys
    const int need = a.k - static_cast<int>(s.below);    // 1 .. keys in the boundary bin
    const int ties = static_cast<int>(s.hist[bin]);
    if (ties > kTieBuf) return false;
#pragma unroll
    for (int u = 0; u < kSelHeld; ++u)
        append_wave_lds(r[u] != kPadKey && (static_cast<uint32_t>(r[u] >> 32) >> shift) == bin, r[u], s.tie, &s.fill);
    __syncthreads();
    if (ties <= kBlock) {                                // one key per thread: its rank among the ties
        if (static_cast<int>(threadIdx.x) < ties) {
            const uint64_t key = s.tie[threadIdx.x];
            int rank = 0;
            for (int j = 0; j < ties; ++j) rank += s.tie[j] < key ? 1 : 0;
            if (rank == need - 1) s.kth = key;
        }
    } else {
        const int P = next_pow2(ties);
        for (int t = ties + threadIdx.x; t < P; t += kBlock) s.tie[t] = kPadKey;
        __syncthreads();
        bitonic_sort_lds(s.tie, P);
        if (threadIdx.x == 0) s.kth = s.tie[need - 1];
    }
    __syncthreads();
    const uint64_t kth = s.kth;
    if (threadIdx.x == 0) s.fill = 0;
    __syncthreads();
    if (!a.final_group) {
        uint64_t* list = a.topk + static_cast<size_t>(q) * a.keep_max;
#pragma unroll
        for (int u = 0; u < kSelHeld; ++u) {             // exactly k keys pass
            const bool pass = r[u] <= kth;               // the pad key is larger than every real key
            const uint64_t mask = __ballot(pass);
            if (mask == 0) continue;
            const int leader = __ffsll(static_cast<long long>(mask)) - 1;
            uint32_t base = 0;
            if (lane_id() == leader) base = atomicAdd(&s.fill, static_cast<uint32_t>(__popcll(mask)));
            base = __shfl(base, leader);
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                  __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
            if (pass) list[base + rank] = r[u];
        }
        if (threadIdx.x == 0) {
            // a later row needs a smaller D: an equal one loses the tie, unless rows come in any order
            a.thr[q] = static_cast<uint32_t>(kth >> 32) + (a.bundle_mul > 1 ? 1u : 0u);
            a.cnt[q] = 0;
        }
        return true;
    }
    // final group: the K keys, sorted, are the result
#pragma unroll
    for (int u = 0; u < kSelHeld; ++u) append_wave_lds(r[u] <= kth, r[u], s.tie, &s.fill);
    __syncthreads();
    const int32_t full = a.d * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    if (a.k <= kBlock) {
        if (static_cast<int>(threadIdx.x) < a.k) {
            const uint64_t key = s.tie[threadIdx.x];
            int rank = 0;
            for (int j = 0; j < a.k; ++j) rank += s.tie[j] < key ? 1 : 0;
            a.idx[static_cast<size_t>(q) * a.k + rank] = static_cast<int32_t>(key & 0xffffffffu);
            a.score[static_cast<size_t>(q) * a.k + rank] = full - 2 * static_cast<int32_t>(key >> 32);
        }
    } else {
        const int P = next_pow2(a.k);
        for (int t = a.k + threadIdx.x; t < P; t += kBlock) s.tie[t] = kPadKey;
        __syncthreads();
        bitonic_sort_lds(s.tie, P);
        write_result(a, q, s.tie);
    }
    return true;
}

// Plain top-K of `total` keys (key(t), t < total, in any order) through a bounded LDS buffer:
// the path for massive ties, when one histogram bin holds more keys than can be ranked.  Keys
// enter while they beat the K-th best so far; the buffer is sorted and cut to K whenever another
// round of one key per thread might not fit.  Leaves the K best keys sorted in keys[].
// capacity >= k + 2 * kBlock.
template <typename KeyAt>
__device__ void stream_topk(const SelectArgs& a, int total, KeyAt key_at, uint64_t* keys, int capacity, int* fill)
{
    if (threadIdx.x == 0) *fill = 0;
    __syncthreads();
    uint64_t bar = kPadKey;                              // only keys below it can still be among the K best
    for (int t0 = 0; t0 < total; t0 += kBlock) {
        const int t = t0 + threadIdx.x;
        if (t < total) {
            const uint64_t key = key_at(t);
            if (key < bar) keys[atomicAdd(fill, 1)] = key;
        }
        __syncthreads();
        const int have = *fill;                          // <= capacity: at most capacity - kBlock before this round
        if (have > capacity - kBlock) {
            const int P = next_pow2(have);
            for (int i = have + threadIdx.x; i < P; i += kBlock) keys[i] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(keys, P);
            bar = keys[a.k - 1];                         // have > k here
            __syncthreads();
            if (threadIdx.x == 0) *fill = a.k;
        }
        __syncthreads();
    }
    const int have = *fill;
    const int P = next_pow2(have);
    for (int i = have + threadIdx.x; i < P; i += kBlock) keys[i] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
}

// The sort buffers of select_dense and select_merge are dynamic LDS sized by the host for the
// launch at hand (a power of two of keys, at most kSortCap): most launches need far less than
// kSortCap keys, and the smaller footprint lets more workgroups share a compute unit.
__global__ __launch_bounds__(kBlock) void select_dense(const SelectArgs a, int capacity)
{
    extern __shared__ uint64_t keys[];               // `capacity` keys
    __shared__ int scratch;
    __shared__ SelectLds sel;
    const int q = blockIdx.x;
    const int P = next_pow2(a.rows);
    const uint32_t* src = a.dense + static_cast<size_t>(q) * a.dense_stride;
    // column t of the dense group is step row_begin + t of the scan's order: the key takes the row's own number
    const int64_t full_bundles = a.n / kLanes;
    auto key_at = [&](int t) {
        const int64_t step = a.row_begin + t;
        const int64_t row = spread_bundle(step / kLanes, a.bundle_mul, full_bundles) * kLanes + step % kLanes;
        return make_key(src[t], static_cast<uint32_t>(row));
    };
    if (a.extra < 0) {
        uint64_t r[kSelHeld];
#pragma unroll
        for (int u = 0; u < kSelHeld; ++u) {
            const int t = u * kBlock + threadIdx.x;
            r[u] = t < a.rows ? key_at(t) : kPadKey;
        }
        if (select_by_histogram(a, q, r, sel)) return;   // same outcome in every thread
        stream_topk(a, a.rows, key_at, keys, capacity, &scratch);
        write_topk(a, q, keys, a.k, &scratch, 0xffffffffu);
        return;
    }
    for (int t = threadIdx.x; t < P; t += blockDim.x)
        keys[t] = t < a.rows ? key_at(t) : kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_topk(a, q, keys, a.rows, &scratch, 0xffffffffu);
}

// Exact re-score of rows [row_begin, row_end) for one query, starting from its current
// top-K.  keys[] holds the best K so far plus survivors; it is compacted (sorted, cut to K,
// threshold tightened) whenever another full workgroup of survivors might not fit.
__device__ void rescan_rows(const MergeArgs& r, int q, uint64_t* keys, int capacity, int* fill)
{
    const SelectArgs& a = r.sel;
    const uint32_t* yq = r.q_rows + static_cast<size_t>(q) * a.q_bits * r.W;
    const int held = a.extra >= 0 ? static_cast<int>(a.len[q]) : a.k;
    for (int t = threadIdx.x; t < held; t += blockDim.x) keys[t] = a.topk[static_cast<size_t>(q) * a.keep_max + t];
    if (threadIdx.x == 0) *fill = held;
    __syncthreads();
    uint32_t thr = a.thr[q];
    const int64_t full_bundles = r.n / kLanes;
    for (int64_t base = r.row_begin; base < r.row_end; base += blockDim.x) {
        const int64_t step = base + threadIdx.x;         // place in the scan's order; the row's own number follows
        if (step < r.row_end) {
            const int64_t row = spread_bundle(step / kLanes, a.bundle_mul, full_bundles) * kLanes + step % kLanes;
            const uint32_t D = distance_generic(r.db, row, yq, a.q_bits, a.db_bits, r.W);
            if (D < thr) keys[atomicAdd(fill, 1)] = make_key(D, static_cast<uint32_t>(row));
        }
        __syncthreads();
        const int have = *fill;                      // <= previous fill + blockDim.x <= capacity
        if (have > capacity - static_cast<int>(blockDim.x)) {
            const int P = next_pow2(have);
            for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(keys, P);
            // cut back to what is still of interest; the threshold can only tighten
            const uint32_t dk = static_cast<uint32_t>(keys[a.k - 1] >> 32);
            int keep = a.k;
            if (a.extra >= 0) {
                const uint32_t bound = dk + static_cast<uint32_t>(a.extra);
                const int within = count_within(keys, have, bound, fill);
                const ListCut cut = candidate_list_cut(keys, within, a.keep_max, bound, thr, a.bundle_mul > 1);
                keep = cut.keep;
                thr = cut.thr;
            } else {
                const uint32_t now = dk + (a.bundle_mul > 1 ? 1u : 0u);
                thr = now < thr ? now : thr;
            }
            if (threadIdx.x == 0) *fill = keep;
        }
        __syncthreads();
    }
    const int have = *fill;
    const int P = next_pow2(have);
    for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_topk(a, q, keys, have, fill, thr);
}

__global__ __launch_bounds__(kBlock) void select_merge(const MergeArgs r, int capacity)
{
    extern __shared__ uint64_t keys[];               // `capacity` keys
    __shared__ int fill;
    __shared__ SelectLds sel;
    const SelectArgs& a = r.sel;
    const int q = blockIdx.x;
    const uint32_t c = a.cnt[q];                     // same value in every lane: branches are uniform
    if (c > static_cast<uint32_t>(a.cap)) {          // the list overflowed: nothing of it is used
        rescan_rows(r, q, keys, capacity, &fill);
        return;
    }
    if (c == 0 && !(a.final_group && a.extra < 0)) return;       // nothing new: list and threshold stand
    const int held = a.extra >= 0 ? static_cast<int>(a.len[q]) : a.k;
    const int total = held + static_cast<int>(c);
    const int P = next_pow2(total);
    const uint64_t* best = a.topk + static_cast<size_t>(q) * a.keep_max;
    const uint64_t* cand = a.cand + static_cast<size_t>(q) * a.cap;
    if (a.extra < 0) {                               // plain top-K: the held keys are in no particular order
        uint64_t r[kSelHeld];
#pragma unroll
        for (int u = 0; u < kSelHeld; ++u) {
            const int t = u * kBlock + threadIdx.x;
            r[u] = t < held ? best[t] : (t < total ? cand[t - held] : kPadKey);
        }
        if (select_by_histogram(a, q, r, sel)) return;       // same outcome in every thread
        stream_topk(a, total, [&](int t) { return t < held ? best[t] : cand[t - held]; }, keys, capacity, &fill);
        write_topk(a, q, keys, a.k, &fill, 0xffffffffu);
        return;
    }
    const int PB = next_pow2(static_cast<int>(c));
    if (c != 0 && held + PB <= P) {  // the kept keys and the padded survivors fit side by side
        // The kept keys are already sorted.  Sort only the survivors, descending, at the end of the
        // buffer; kept keys (ascending), padding, survivors (descending, their padding first) then
        // form one bitonic sequence, and a single merge stage finishes the job.
        const int b0 = P - PB;
        for (int t = threadIdx.x; t < P; t += blockDim.x)
            keys[t] = t < held ? best[t] : (t >= b0 && t - b0 < static_cast<int>(c) ? cand[t - b0] : kPadKey);
        __syncthreads();
        bitonic_sort_lds_descending(keys + b0, PB);
        bitonic_merge_lds(keys, P);
    } else {
        for (int t = threadIdx.x; t < P; t += blockDim.x)
            keys[t] = t < held ? best[t] : (t < total ? cand[t - held] : kPadKey);
        __syncthreads();
        if (c != 0) bitonic_sort_lds(keys, P);
    }
    write_topk(a, q, keys, total, &fill, a.thr[q]);
}

// ---------------------------------------------------------------------------------------
// Refine (Algorithm 1, last loop; Section 4.1 "Refine").  One workgroup per query: the query
// vector sits in LDS, each wavefront takes candidates in turn, reads the candidate's fp32 row
// with coalesced loads and reduces the products across its lanes; the similarities are then
// sorted (descending, ties to the lower row) as 64-bit keys.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void refine_topk(const RefineArgs a)
{
    extern __shared__ uint64_t lds64[];
    uint64_t* keys = lds64;                              // kSortCap keys
    float* qv = reinterpret_cast<float*>(lds64 + kSortCap);   // d floats
    const int q = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int have = static_cast<int>(a.len[q]);
    const float* xq = a.X_q + static_cast<size_t>(q) * a.d;
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) qv[c] = xq[c];
    __syncthreads();
    const uint64_t* list = a.topk + static_cast<size_t>(q) * a.keep_max;
    // each wavefront takes four candidates per round so that their row loads overlap
    constexpr int U = 4;
    for (int t0 = wave * U; t0 < have; t0 += 4 * U) {
        uint32_t row[U];
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u < have ? t0 + u : have - 1;         // the tail repeats the last candidate
            row[u] = static_cast<uint32_t>(list[t] & 0xffffffffu);
            s[u] = 0.0f;
        }
        for (int c = lane; c < a.d; c += 64) {
            float xv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) xv[u] = a.X_db[static_cast<size_t>(row[u]) * a.d + c];
            const float qc = qv[c];
#pragma unroll
            for (int u = 0; u < U; ++u) s[u] = fmaf(xv[u], qc, s[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) s[u] += __shfl_xor(s[u], off);
            if (lane == 0 && t0 + u < have) keys[t0 + u] = (static_cast<uint64_t>(descending_bits(s[u])) << 32) | row[u];
        }
    }
    const int P = next_pow2(have);
    for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) {
        const uint64_t key = keys[t];
        a.idx[static_cast<size_t>(q) * a.k + t] = static_cast<int32_t>(key & 0xffffffffu);
        a.sim[static_cast<size_t>(q) * a.k + t] = bits_to_float_descending(static_cast<uint32_t>(key >> 32));
    }
    if (a.count != nullptr && threadIdx.x == 0) a.count[q] = have;
}

// LDS keys of a selection launch.  Plain top-K keeps its keys in registers and needs the buffer
// only for its slow paths (streaming over massive ties, exact rescan): K plus two rounds of one
// key per thread.  Candidate lists are sorted whole: list plus survivors (or the dense rows).
static int select_capacity(const SelectArgs& a, int whole)
{
    const int need = a.extra < 0 ? a.k + 2 * kBlock : (whole > a.keep_max + 2 * kBlock ? whole : a.keep_max + 2 * kBlock);
    int capacity = 1;
    while (capacity < need) capacity <<= 1;
    return capacity;
}

hipError_t launch_select_dense(const SelectArgs& a, hipStream_t s)
{
    if (a.m <= 0) return hipSuccess;
    if (a.rows < a.k || a.rows > kSortCap) return hipErrorInvalidValue;
    const int capacity = a.extra < 0 ? select_capacity(a, 0) : select_capacity(a, a.rows);
    if (capacity > kSortCap) return hipErrorInvalidValue;
    hipLaunchKernelGGL(select_dense, dim3(a.m), dim3(kBlock), capacity * sizeof(uint64_t), s, a, capacity);
    return hipGetLastError();
}

hipError_t launch_refine(const RefineArgs& a, hipStream_t s)
{
    if (a.m <= 0) return hipSuccess;
    if (a.keep_max > kSortCap || a.k > a.keep_max) return hipErrorInvalidValue;
    const size_t lds = kSortCap * sizeof(uint64_t) + static_cast<size_t>(a.d) * sizeof(float);
    hipLaunchKernelGGL(refine_topk, dim3(a.m), dim3(kBlock), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_select_merge(const MergeArgs& r, hipStream_t s)
{
    if (r.sel.m <= 0) return hipSuccess;
    if (r.sel.keep_max + r.sel.cap > kSortCap || r.row_end > r.n || r.row_begin < 0) return hipErrorInvalidValue;
    // candidate lists: room for the kept keys plus a full survivor list; the exact rescan of an
    // overflowed query works in the same buffer and needs the kept keys plus two rounds of one key
    // per thread
    const int capacity = select_capacity(r.sel, r.sel.keep_max + r.sel.cap);
    hipLaunchKernelGGL(select_merge, dim3(r.sel.m), dim3(kBlock), capacity * sizeof(uint64_t), s, r, capacity);
    return hipGetLastError();
}

}  // namespace xbq
