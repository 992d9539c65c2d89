// Algorithm 1 (K-Select, Section 4) with its candidate list taken whole: every row whose
// distance is within (K-th smallest distance) + extra distance is refined with the exact fp32
// inner product, however many rows that is, up to a bound the caller chooses to size the
// workspace.
//
// A first stage has already run and gives each query its K-th smallest distance D_K: for few
// queries the plain exact search; otherwise the bounded candidate search, which for most
// queries already holds the whole list (then nothing below touches them again).
// Then:
//   kselect_from_*    threshold of the query = D_K + extra + 1, candidate count = 0; or, for a
//                     query whose bounded list is whole and fits, the list is copied and the
//                     threshold is 0
//   (scan kernels)    one pass over all rows in threshold mode appends every row below it and
//                     counts the passing rows per distance level
//   kselect_levels    only for a query whose rows within the bound exceed the list: the level
//                     counts give the largest distance whose rows still fit (whole distance
//                     levels, never below D_K); if the ties at D_K alone do not fit, the list
//                     is the K best rows by (distance, row)
//   (scan kernels)    a second collecting pass for the queries whose bound was lowered; it
//                     returns at once when there is none
//   refine_wide       similarities of the candidates in pieces, a running top-K in LDS;
//                     a query's list may be split over several workgroups
//   refine_merge      merges the pieces' top-K and writes rows, similarities and |L|

#include "xbq_device.h"

namespace xbq {

constexpr int kLevelBins = XBQ_MAX_EXTRA + 2;            // below D_K, then D_K .. D_K + extra
constexpr int kRefineSort = 2048;                        // keys per sort of refine_wide: K best so far + new ones

// First stage was the plain exact search (few queries): every query is collected by the scan.
// One workgroup per query.
__global__ __launch_bounds__(kBlock) void kselect_from_topk(const KSelectArgs a)
{
    const int q = blockIdx.x;
    const int32_t full = a.d * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    for (int t = threadIdx.x; t < a.k; t += kBlock) {
        const size_t at = static_cast<size_t>(q) * a.k + t;
        a.best[at] = make_key(static_cast<uint32_t>((full - a.score1[at]) / 2), static_cast<uint32_t>(a.idx1[at]));
    }
    if (threadIdx.x == 0) {
        const uint32_t dk = static_cast<uint32_t>((full - a.score1[static_cast<size_t>(q) * a.k + a.k - 1]) / 2);
        a.dk[q] = dk;
        a.thr[q] = dk + static_cast<uint32_t>(a.extra) + 1u;
        a.cnt[q] = 0;
        a.flag[0] = 1;
    }
}

// First stage was the bounded candidate search (keys sorted by (D, row), at most keep1 per
// query).  A list shorter than keep1 is every row within the boundary: if it also fits the
// caller's bound the query is done and skips the collecting scans (threshold 0).
__global__ __launch_bounds__(kBlock) void kselect_from_lists(const KSelectArgs a)
{
    const int q = blockIdx.x;
    const uint64_t* src = a.topk1 + static_cast<size_t>(q) * a.keep1;
    const uint32_t len = a.len1[q];
    const uint32_t dk = static_cast<uint32_t>(src[a.k - 1] >> 32);
    const bool whole = len < static_cast<uint32_t>(a.keep1) && len <= static_cast<uint32_t>(a.cap);
    uint64_t* list = a.list + static_cast<size_t>(q) * a.cap;
    if (whole)
        for (uint32_t t = threadIdx.x; t < len; t += kBlock) list[t] = src[t];
    for (int t = threadIdx.x; t < a.k; t += kBlock) a.best[static_cast<size_t>(q) * a.k + t] = src[t];
    if (threadIdx.x == 0) {
        a.dk[q] = dk;
        a.cnt[q] = whole ? len : 0u;
        a.thr[q] = whole ? 0u : dk + static_cast<uint32_t>(a.extra) + 1u;
        if (!whole) a.flag[0] = 1;
    }
}

// Few queries, first stage = histogram search: every distance is already stored (dist[q][n]), so
// the collection reads those instead of scanning the codes again.  grid = m * blocks_per_query
// workgroups of rows_per_block rows; per round of 16 rows per thread the workgroup reserves its
// slots with one atomic, so a query with a very long list does not serialise on its counter.
// `thr`: a row passes when D < thr[q]; thr[q] == 0 means the query needs nothing.  `levels` may
// be nullptr (second collection).
__global__ __launch_bounds__(kBlock) void kselect_collect_stored(const KSelectArgs a, const uint32_t* dist,
                                                                 const uint32_t* thr, uint32_t* levels,
                                                                 int rows_per_block, int blocks_per_query)
{
    __shared__ uint32_t lvl[kLevelBins];
    __shared__ uint32_t wave_tot[kBlock / kLanes];
    __shared__ uint32_t base_s;
    const int q = blockIdx.x / blocks_per_query;
    const int chunk = blockIdx.x - q * blocks_per_query;
    const uint32_t t = thr[q];
    if (t == 0) return;                                  // same value in every lane
    const uint32_t dk = a.dk[q];
    const int bins = a.extra + 2;
    if (levels != nullptr) {
        for (int i = threadIdx.x; i < bins; i += kBlock) lvl[i] = 0;
    }
    __syncthreads();
    const uint32_t* dq = dist + static_cast<size_t>(q) * a.n;
    uint64_t* list = a.list + static_cast<size_t>(q) * a.cap;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r_begin = static_cast<int64_t>(chunk) * rows_per_block;
    const int64_t r_end = r_begin + rows_per_block < a.n ? r_begin + rows_per_block : a.n;
    for (int64_t r0 = r_begin; r0 < r_end; r0 += 16 * kBlock) {
        uint32_t D[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t row = r0 + (static_cast<int64_t>(u) * kBlock + threadIdx.x) * 4;
            if (row + 3 < r_end && (reinterpret_cast<uintptr_t>(dq + row) & 15) == 0) {
                const uint4 v = *reinterpret_cast<const uint4*>(dq + row);
                D[u][0] = v.x; D[u][1] = v.y; D[u][2] = v.z; D[u][3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) D[u][e] = row + e < r_end ? dq[row + e] : 0xffffffffu;
            }
        }
        uint32_t mine = 0;                               // rows of this thread that pass
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) mine += D[u][e] < t ? 1u : 0u;
        uint32_t incl = mine;                            // inclusive scan inside the wavefront
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t total = 0;
            for (int w = 0; w < kBlock / kLanes; ++w) total += wave_tot[w];
            base_s = total ? atomicAdd(&a.cnt[q], total) : 0u;
        }
        __syncthreads();
        uint32_t pos = base_s + incl - mine;
        for (int w = 0; w < wave; ++w) pos += wave_tot[w];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (D[u][e] < t) {
                    const int64_t row = r0 + (static_cast<int64_t>(u) * kBlock + threadIdx.x) * 4 + e;
                    if (pos < static_cast<uint32_t>(a.cap)) list[pos] = make_key(D[u][e], static_cast<uint32_t>(row));
                    ++pos;
                    if (levels != nullptr) atomicAdd(&lvl[D[u][e] < dk ? 0u : D[u][e] - dk + 1u], 1u);
                }
            }
        __syncthreads();                                 // wave_tot and base_s are reused by the next round
    }
    if (levels != nullptr) {
        __syncthreads();
        for (int i = threadIdx.x; i < bins; i += kBlock) {
            const uint32_t v = lvl[i];
            if (v) atomicAdd(&levels[static_cast<size_t>(q) * bins + i], v);
        }
    }
}

// One workgroup per query.  A query whose rows within the bound fit its list is done
// (thr2 = 0).  Otherwise the level counts of the collecting scan give the largest distance
// whose rows still fit (whole levels, never below D_K): the list is emptied and the query
// takes part in a second collecting scan with that distance as its bound.  If the ties at D_K
// alone do not fit, the list becomes the K best rows by (distance, row).
__global__ __launch_bounds__(kBlock) void kselect_levels(const KSelectArgs a)
{
    __shared__ uint32_t hist[kLevelBins];
    __shared__ uint32_t s_level;
    const int q = blockIdx.x;
    if (a.cnt[q] <= static_cast<uint32_t>(a.cap)) {              // same value in every lane
        if (threadIdx.x == 0) a.thr2[q] = 0;
        return;
    }
    const int bins = a.extra + 2;
    const uint32_t* lv = a.levels + static_cast<size_t>(q) * bins;
    for (int t = threadIdx.x; t < bins; t += kBlock) hist[t] = lv[t];
    __syncthreads();
    if (threadIdx.x == 0) {
        // level j (j >= 1) = all rows with D <= D_K + j - 1; the largest one that fits
        uint32_t cum = hist[0], level = 0;
        for (int j = 1; j < bins; ++j) {
            cum += hist[j];
            if (cum > static_cast<uint32_t>(a.cap)) break;
            level = static_cast<uint32_t>(j);
        }
        s_level = level;
    }
    __syncthreads();
    if (s_level == 0) {                                  // the ties at D_K alone do not fit
        uint64_t* list = a.list + static_cast<size_t>(q) * a.cap;
        for (int t = threadIdx.x; t < a.k; t += kBlock) list[t] = a.best[static_cast<size_t>(q) * a.k + t];
        if (threadIdx.x == 0) {
            a.cnt[q] = static_cast<uint32_t>(a.k);
            a.thr2[q] = 0;
        }
        return;
    }
    if (threadIdx.x == 0) {
        a.cnt[q] = 0;
        a.thr2[q] = a.dk[q] + s_level;                   // D < D_K + level  <=>  D <= D_K + level - 1
        a.flag[1] = 1;
    }
}

// Similarities of candidates list[0 .. nc) with the query in LDS, one wavefront per U candidates
// at a time, written as sort keys to keys[0 .. nc).  VEC: rows are read 16 bytes per lane (d a
// multiple of 4, X_db 16-byte aligned), so one load covers 256 coordinates of a row.
template <bool VEC, int U>
__device__ __forceinline__ void similarities(const KSelectArgs& a, const uint64_t* list, int nc, const float* qv,
                                             uint64_t* keys)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t0 = wave * U; t0 < nc; t0 += (kBlock / kLanes) * U) {
        uint32_t row[U];
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u < nc ? t0 + u : nc - 1;                 // the tail repeats the last candidate
            row[u] = static_cast<uint32_t>(list[t] & 0xffffffffu);
            s[u] = 0.0f;
        }
        if (VEC) {
            const int d4 = a.d >> 2;
            const float4* q4 = reinterpret_cast<const float4*>(qv);
            for (int col = lane; col < d4; col += kLanes) {
                float4 xv[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    xv[u] = reinterpret_cast<const float4*>(a.X_db + static_cast<size_t>(row[u]) * a.d)[col];
                const float4 qc = q4[col];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    s[u] = fmaf(xv[u].w, qc.w, fmaf(xv[u].z, qc.z, fmaf(xv[u].y, qc.y, fmaf(xv[u].x, qc.x, s[u]))));
            }
        } else {
            for (int col = lane; col < a.d; col += kLanes) {
                float xv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) xv[u] = a.X_db[static_cast<size_t>(row[u]) * a.d + col];
                const float qc = qv[col];
#pragma unroll
                for (int u = 0; u < U; ++u) s[u] = fmaf(xv[u], qc, s[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) s[u] += __shfl_xor(s[u], off);
            if (lane == 0 && t0 + u < nc) keys[t0 + u] = (static_cast<uint64_t>(descending_bits(s[u])) << 32) | row[u];
        }
    }
}

// grid = m * parts.  Piece `part` of query q's list: running top-K of (similarity descending,
// row ascending) keys, written sorted to part_keys[q][part][0 .. k), padded with kPadKey.
// Each round sorts the K best so far together with as many new candidates as fill kRefineSort.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void refine_wide(const KSelectArgs a)
{
    extern __shared__ uint64_t lds64[];
    uint64_t* keys = lds64;                              // kRefineSort keys
    float* qv = reinterpret_cast<float*>(lds64 + kRefineSort);   // d floats, 16-byte aligned
    const int q = blockIdx.x / a.parts, part = blockIdx.x - q * a.parts;
    const uint32_t c = a.cnt[q];
    const int have = c < static_cast<uint32_t>(a.cap) ? static_cast<int>(c) : a.cap;
    const int per = (have + a.parts - 1) / a.parts;
    const int begin = part * per < have ? part * per : have;
    const int end = begin + per < have ? begin + per : have;
    const float* xq = a.X_q + static_cast<size_t>(q) * a.d;
    for (int t = threadIdx.x; t < a.d; t += kBlock) qv[t] = xq[t];
    __syncthreads();
    const uint64_t* list = a.list + static_cast<size_t>(q) * a.cap;
    int held = 0;
    for (int base = begin; base < end;) {
        const int room = kRefineSort - held;
        const int nc = end - base < room ? end - base : room;
        similarities<VEC, VEC ? 8 : 4>(a, list + base, nc, qv, keys + held);
        const int total = held + nc;
        const int P = next_pow2(total);
        for (int t = total + threadIdx.x; t < P; t += kBlock) keys[t] = kPadKey;
        __syncthreads();
        bitonic_sort_lds(keys, P);
        held = total < a.k ? total : a.k;
        base += nc;
    }
    uint64_t* out = a.part_keys + (static_cast<size_t>(q) * a.parts + part) * a.k;
    for (int t = threadIdx.x; t < a.k; t += kBlock) out[t] = t < held ? keys[t] : kPadKey;
}

__global__ __launch_bounds__(kBlock) void refine_merge(const KSelectArgs a)
{
    __shared__ uint64_t keys[kSortCap];
    const int q = blockIdx.x;
    const int total = a.parts * a.k;
    const int P = next_pow2(total);
    const uint64_t* in = a.part_keys + static_cast<size_t>(q) * total;
    for (int t = threadIdx.x; t < P; t += kBlock) keys[t] = t < total ? in[t] : kPadKey;
    __syncthreads();
    if (a.parts > 1) bitonic_sort_lds(keys, P);
    for (int t = threadIdx.x; t < a.k; t += kBlock) {
        const uint64_t key = keys[t];
        a.idx[static_cast<size_t>(q) * a.k + t] = static_cast<int32_t>(key & 0xffffffffu);
        a.sim[static_cast<size_t>(q) * a.k + t] = bits_to_float_descending(static_cast<uint32_t>(key >> 32));
    }
    if (a.count != nullptr && threadIdx.x == 0) {
        const uint32_t c = a.cnt[q];
        a.count[q] = static_cast<int32_t>(c < static_cast<uint32_t>(a.cap) ? c : static_cast<uint32_t>(a.cap));
    }
}

static bool kselect_args_ok(const KSelectArgs& a)
{
    return a.m >= 1 && a.k >= 1 && a.k <= XBQ_MAX_K && a.cap >= a.k && a.extra >= 0 && a.extra <= XBQ_MAX_EXTRA &&
           a.parts >= 1 && static_cast<int64_t>(a.parts) * a.k <= kSortCap && 2 * a.k <= kRefineSort;
}

hipError_t launch_kselect_first(const KSelectArgs& a, hipStream_t s)
{
    if (!kselect_args_ok(a)) return hipErrorInvalidValue;
    if (a.topk1 != nullptr) {
        if (a.keep1 < a.k) return hipErrorInvalidValue;
        hipLaunchKernelGGL(kselect_from_lists, dim3(a.m), dim3(kBlock), 0, s, a);
    } else {
        hipLaunchKernelGGL(kselect_from_topk, dim3(a.m), dim3(kBlock), 0, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_kselect_collect_stored(const KSelectArgs& a, const uint32_t* dist, bool second, hipStream_t s)
{
    if (!kselect_args_ok(a) || dist == nullptr) return hipErrorInvalidValue;
    const int rows_per_block = 16 * kBlock;              // one round: workgroups are cheap, parallelism is not
    const int64_t bpq = (a.n + rows_per_block - 1) / rows_per_block;
    if (bpq * a.m > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kselect_collect_stored, dim3(static_cast<unsigned>(bpq * a.m)), dim3(kBlock), 0, s, a, dist,
                       second ? a.thr2 : a.thr, second ? nullptr : a.levels, rows_per_block, static_cast<int>(bpq));
    return hipGetLastError();
}

hipError_t launch_kselect_levels(const KSelectArgs& a, hipStream_t s)
{
    if (!kselect_args_ok(a)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kselect_levels, dim3(a.m), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_kselect_refine(const KSelectArgs& a, hipStream_t s)
{
    if (!kselect_args_ok(a)) return hipErrorInvalidValue;
    const size_t lds = kRefineSort * sizeof(uint64_t) + static_cast<size_t>(a.d) * sizeof(float);
    const dim3 grid(static_cast<unsigned>(a.m) * a.parts);
    if (a.d % 4 == 0 && reinterpret_cast<uintptr_t>(a.X_db) % 16 == 0)
        hipLaunchKernelGGL(refine_wide<true>, grid, dim3(kBlock), lds, s, a);
    else
        hipLaunchKernelGGL(refine_wide<false>, grid, dim3(kBlock), lds, s, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(refine_merge, dim3(a.m), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace xbq
