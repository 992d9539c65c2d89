// Selection kernels: exact top-K per query on 64-bit keys (D << 32 | row), smaller first.
// Smaller D means larger score S = d(2^B-1)^2 - 2D (Eq. 2 of Section 3.3), so ascending
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

#include "xbq_internal.h"

namespace xbq {

constexpr uint64_t kPadKey = ~0ull;

__device__ __forceinline__ int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Ascending bitonic sort of P (power of two) keys in LDS by the whole workgroup.
// The caller has already synchronised after filling `keys`.
__device__ void bitonic_sort_lds(uint64_t* keys, int P)
{
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (P >> 1); t += blockDim.x) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const int l = i | j;
                const bool up = (i & k) == 0;
                const uint64_t a = keys[i], b = keys[l];
                if ((a > b) == up) { keys[i] = b; keys[l] = a; }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ void write_result(const SelectArgs& a, int q, const uint64_t* keys)
{
    const int32_t full = a.d * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) {
        const uint64_t key = keys[t];
        a.idx[static_cast<size_t>(q) * a.k + t] = static_cast<int32_t>(key & 0xffffffffu);
        a.score[static_cast<size_t>(q) * a.k + t] = full - 2 * static_cast<int32_t>(key >> 32);
    }
}

__device__ __forceinline__ void write_topk(const SelectArgs& a, int q, const uint64_t* keys)
{
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) a.topk[static_cast<size_t>(q) * a.k + t] = keys[t];
    if (threadIdx.x == 0) {
        a.thr[q] = static_cast<uint32_t>(keys[a.k - 1] >> 32);
        a.cnt[q] = 0;
    }
    if (a.final_group) write_result(a, q, keys);
}

__global__ __launch_bounds__(kBlock) void select_dense(const SelectArgs a)
{
    __shared__ uint64_t keys[kSortCap];
    const int q = blockIdx.x;
    const int P = next_pow2(a.rows);
    const uint32_t* src = a.dense + static_cast<size_t>(q) * a.dense_stride;
    for (int t = threadIdx.x; t < P; t += blockDim.x)
        keys[t] = t < a.rows ? make_key(src[t], static_cast<uint32_t>(a.row_begin + t)) : kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_topk(a, q, keys);
}

// Eq. 6 for one (row, query) with run-time sizes; slow path used only by the rescan.
__device__ uint32_t distance_generic(const uint32_t* db, int64_t row, const uint32_t* yq, int BQ, int BD, int W)
{
    const uint32_t* xb = db + (row / kLanes) * (static_cast<int64_t>(BD) * W * kLanes) + (row % kLanes);
    uint32_t D = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t x[XBQ_MAX_BITS], y[XBQ_MAX_BITS];
        for (int b = 0; b < BD; ++b) x[b] = xb[(b * W + w) * kLanes];
        for (int b = 0; b < BQ; ++b) y[b] = yq[b * W + w];
        for (int i = 0; i < BD; ++i)
            for (int j = 0; j < BQ; ++j) D += static_cast<uint32_t>(__builtin_popcount(x[i] ^ y[j])) << (i + j);
    }
    return D;
}

// Exact re-score of rows [row_begin, row_end) for one query, starting from its current
// top-K.  keys[] holds the best K so far plus survivors; it is compacted (sorted, cut to K,
// threshold tightened) whenever another full workgroup of survivors might not fit.
__device__ void rescan_rows(const MergeArgs& r, int q, uint64_t* keys, int* fill)
{
    const SelectArgs& a = r.sel;
    const uint32_t* yq = r.q_rows + static_cast<size_t>(q) * a.q_bits * r.W;
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) keys[t] = a.topk[static_cast<size_t>(q) * a.k + t];
    if (threadIdx.x == 0) *fill = a.k;
    __syncthreads();
    uint32_t thr = static_cast<uint32_t>(keys[a.k - 1] >> 32);
    for (int64_t base = r.row_begin; base < r.row_end; base += blockDim.x) {
        const int64_t row = base + threadIdx.x;
        if (row < r.row_end) {
            const uint32_t D = distance_generic(r.db, row, yq, a.q_bits, a.db_bits, r.W);
            if (D < thr) keys[atomicAdd(fill, 1)] = make_key(D, static_cast<uint32_t>(row));
        }
        __syncthreads();
        const int have = *fill;                      // <= previous fill + blockDim.x <= kSortCap
        if (have > kSortCap - static_cast<int>(blockDim.x)) {
            const int P = next_pow2(have);
            for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(keys, P);
            thr = static_cast<uint32_t>(keys[a.k - 1] >> 32);
            if (threadIdx.x == 0) *fill = a.k;
        }
        __syncthreads();
    }
    const int have = *fill;
    const int P = next_pow2(have);
    for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_topk(a, q, keys);
}

__global__ __launch_bounds__(kBlock) void select_merge(const MergeArgs r)
{
    __shared__ uint64_t keys[kSortCap];
    __shared__ int fill;
    const SelectArgs& a = r.sel;
    const int q = blockIdx.x;
    const uint32_t c = a.cnt[q];                     // same value in every lane: branches are uniform
    if (c > static_cast<uint32_t>(a.cap)) {          // the list overflowed: nothing of it is used
        rescan_rows(r, q, keys, &fill);
        return;
    }
    if (c == 0 && !a.final_group) return;            // nothing beat the threshold
    const int total = a.k + static_cast<int>(c);
    const int P = next_pow2(total);
    const uint64_t* best = a.topk + static_cast<size_t>(q) * a.k;
    const uint64_t* cand = a.cand + static_cast<size_t>(q) * a.cap;
    for (int t = threadIdx.x; t < P; t += blockDim.x)
        keys[t] = t < a.k ? best[t] : (t < total ? cand[t - a.k] : kPadKey);
    __syncthreads();
    if (c != 0) bitonic_sort_lds(keys, P);
    write_topk(a, q, keys);
}

hipError_t launch_select_dense(const SelectArgs& a, hipStream_t s)
{
    if (a.m <= 0) return hipSuccess;
    if (a.rows < a.k || a.rows > kSortCap) return hipErrorInvalidValue;
    hipLaunchKernelGGL(select_dense, dim3(a.m), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_select_merge(const MergeArgs& r, hipStream_t s)
{
    if (r.sel.m <= 0) return hipSuccess;
    if (r.sel.k + r.sel.cap > kSortCap || r.row_end > r.n || r.row_begin < 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(select_merge, dim3(r.sel.m), dim3(kBlock), 0, s, r);
    return hipGetLastError();
}

}  // namespace xbq
