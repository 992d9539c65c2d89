// Histogram selection for a handful of queries (the single-request mode the paper measures,
// Section 5, and its own selector, Section 4.1 "Histogram and Select" / Algorithm 1).
//
// With few queries the scan is bound by the HBM stream of the database codes, not by the
// ALUs, and what matters is the number of kernel launches.  Four launches:
//   clear_u32     zero the histograms and counters (a kernel, so the sequence can be captured)
//   scan_hist     one pass over all rows: D per (query, row) stored as uint32, and a histogram
//                 of D >> shift per query, built in LDS and merged into global memory
//   hist_collect  per query: the prefix sum of the histogram gives the bin b* holding the K-th
//                 smallest distance; every row whose bin is <= b* is a candidate (a superset of
//                 the K best) and is appended to the query's list
//   hist_finish   one workgroup per query sorts the candidates by (D, row) and writes the K
//                 best.  If the candidates cannot fit the sort buffer (massive ties) it instead
//                 streams over the stored distances with a running threshold, which is slower
//                 and always exact.
// (Finishing in the last collecting workgroup would save a launch, but the device-scope fences
// that needs write back whole L2s on this multi-die part and cost far more than a launch.)
// The paper uses one bin per distinct distance and adds an extra distance before the refine
// stage; here bins are 2^shift wide (at most 1024 per query) and the final sort makes the
// result the exact top-K with ties to the lower row.

#include "xbq_device.h"

namespace xbq {

__global__ void clear_u32(uint32_t* p, int64_t count)
{
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < count;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x)
        p[i] = 0;
}

// One wavefront per bundle of 64 rows (grid-stride); queries come from the chunk-major layout
// [m][nchunks][BQ][WC] (for W <= 8 that is the plain row layout with one chunk).
// Workgroups of 16 wavefronts share one LDS histogram, so that few workgroups (one per CU)
// merge into the global one: the merge is atomics on a few hundred hot addresses.
constexpr int kHistBlock = 1024;

// PREFETCH (the whole row fits WC words, one chunk): the rows of the wavefront's next bundle are
// requested before the current one is scored.
template <int BQ, int BD, int WC, bool PREFETCH>
__global__ __launch_bounds__(kHistBlock) void scan_hist(const HistArgs a)
{
    __shared__ uint32_t lh[kHistMaxQueries * kHistBins];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int bins = a.m * kHistBins;
    for (int t = threadIdx.x; t < bins; t += blockDim.x) lh[t] = 0;

    const int64_t nbundles = (a.n + kLanes - 1) / kLanes;
    constexpr int kWaves = kHistBlock / kLanes;
    const int64_t waves = static_cast<int64_t>(gridDim.x) * kWaves;
    const int64_t row_stride = static_cast<int64_t>(BD) * a.W * kLanes;
    int64_t bundle = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    uint32_t xn[BD][WC];
    if (PREFETCH && bundle < nbundles) {
        const uint32_t* xb = a.db + bundle * row_stride + lane;
#pragma unroll
        for (int b = 0; b < BD; ++b)
#pragma unroll
            for (int w = 0; w < WC; ++w) xn[b][w] = __builtin_nontemporal_load(xb + (b * WC + w) * kLanes);
    }
    __syncthreads();

    for (; bundle < nbundles; bundle += waves) {
        const uint32_t* xb = a.db + bundle * row_stride + lane;
        uint32_t acc[kHistMaxQueries];
#pragma unroll
        for (int t = 0; t < kHistMaxQueries; ++t) acc[t] = 0;
        for (int c = 0; c < (PREFETCH ? 1 : a.nchunks); ++c) {
            uint32_t x[BD][WC];
            if (PREFETCH) {
#pragma unroll
                for (int b = 0; b < BD; ++b)
#pragma unroll
                    for (int w = 0; w < WC; ++w) x[b][w] = xn[b][w];
                if (bundle + waves < nbundles) {
                    const uint32_t* xnb = xb + waves * row_stride;
#pragma unroll
                    for (int b = 0; b < BD; ++b)
#pragma unroll
                        for (int w = 0; w < WC; ++w) xn[b][w] = __builtin_nontemporal_load(xnb + (b * WC + w) * kLanes);
                }
            } else {
#pragma unroll
                for (int b = 0; b < BD; ++b)
#pragma unroll
                    for (int w = 0; w < WC; ++w) {
                        const int ww = c * WC + w;
                        x[b][w] = ww < a.W ? xb[(b * a.W + ww) * kLanes] : 0u;
                    }
            }
#pragma unroll
            for (int t = 0; t < kHistMaxQueries; ++t) {
                if (t < a.m) {
                    uniform_ptr yq = (uniform_ptr)(a.q + (static_cast<size_t>(t) * a.nchunks + c) * (BQ * WC));
                    uint32_t y[BQ][WC];
#pragma unroll
                    for (int b = 0; b < BQ; ++b)
#pragma unroll
                        for (int w = 0; w < WC; ++w) y[b][w] = yq[b * WC + w];
                    acc[t] += xor_popcount<BQ, BD, WC>(x, y);
                }
            }
        }
        const int64_t row = bundle * kLanes + lane;
        if (row < a.n) {
#pragma unroll
            for (int t = 0; t < kHistMaxQueries; ++t) {
                if (t < a.m) {
                    a.dist[static_cast<size_t>(t) * a.n + row] = acc[t];
                    atomicAdd(&lh[t * kHistBins + (acc[t] >> a.shift)], 1u);
                }
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < bins; t += blockDim.x) {
        const uint32_t v = lh[t];
        if (v) atomicAdd(&a.hist[t], v);
    }
}

__device__ void write_result_h(const CollectArgs& a, int q, const uint64_t* keys)
{
    const int32_t full = a.d * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) {
        const uint64_t key = keys[t];
        a.idx[static_cast<size_t>(q) * a.k + t] = static_cast<int32_t>(key & 0xffffffffu);
        a.score[static_cast<size_t>(q) * a.k + t] = full - 2 * static_cast<int32_t>(key >> 32);
    }
}

// Exact top-K of one query from its stored distances, rows in ascending order, with a running
// threshold and a bounded buffer: the path for histograms whose boundary bin is too full.
__device__ void stream_select(const CollectArgs& a, int q, uint64_t* keys, int* fill)
{
    const uint32_t* dq = a.dist + static_cast<size_t>(q) * a.n;
    if (threadIdx.x == 0) *fill = 0;
    __syncthreads();
    uint32_t thr = 0xffffffffu;                          // nothing excluded until K rows are held
    for (int64_t base = 0; base < a.n; base += blockDim.x) {
        const int64_t row = base + threadIdx.x;
        if (row < a.n) {
            const uint32_t D = dq[row];
            if (D < thr) keys[atomicAdd(fill, 1)] = make_key(D, static_cast<uint32_t>(row));
        }
        __syncthreads();
        const int have = *fill;
        if (have > kSortCap - static_cast<int>(blockDim.x)) {
            const int P = next_pow2(have);
            for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(keys, P);
            thr = static_cast<uint32_t>(keys[a.k - 1] >> 32);   // have >= K here: K <= 1024 < have
            if (threadIdx.x == 0) *fill = a.k;
        }
        __syncthreads();
    }
    const int have = *fill;
    const int P = next_pow2(have);
    for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_result_h(a, q, keys);
}

// Exact top-K of one query from a list of `total` candidate keys in global memory, in any order
// (every row up to the boundary bin, more than the sort buffer holds: thousands of rows of one
// tight cluster in the boundary bin): a running threshold on the whole key and a bounded buffer.
__device__ void stream_list(const CollectArgs& a, int q, const uint64_t* list, int total, uint64_t* keys, int* fill)
{
    if (threadIdx.x == 0) *fill = 0;
    __syncthreads();
    uint64_t thr = kPadKey;                              // nothing excluded until K keys are held
    for (int base = 0; base < total; base += 4 * blockDim.x) {
        uint64_t k4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = base + u * blockDim.x + threadIdx.x;
            k4[u] = t < total ? list[t] : kPadKey;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k4[u] < thr) keys[atomicAdd(fill, 1)] = k4[u];
        __syncthreads();
        const int have = *fill;                          // at most 4 * blockDim.x more than before
        if (have > kSortCap - 4 * static_cast<int>(blockDim.x)) {
            const int P = next_pow2(have);
            for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(keys, P);
            thr = keys[a.k - 1];                         // have >= K here: K <= 1024 < have
            if (threadIdx.x == 0) *fill = a.k;
        }
        __syncthreads();
    }
    const int have = *fill;
    const int P = next_pow2(have);
    for (int t = have + threadIdx.x; t < P; t += blockDim.x) keys[t] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_result_h(a, q, keys);
}

// Boundary bin of one query: the smallest b whose bins 0..b hold at least k rows (Algorithm
// 1's boundary at bin resolution), and the number of rows in those bins.  All threads of a
// 256-thread workgroup call this; the result is returned to every thread.
__device__ void boundary_bin(const uint32_t* h, int k, uint32_t* wave_sum, int* s_bin, int* s_total, uint32_t& bin,
                             int& total)
{
    constexpr int per = kHistBins / kBlock;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t mine[per];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < per; ++i) { mine[i] = h[threadIdx.x * per + i]; sum += mine[i]; }
    uint32_t incl = sum;                                 // inclusive scan inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t before = incl - sum;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    const uint32_t kk = static_cast<uint32_t>(k);
    if (before < kk && before + sum >= kk) {
#pragma unroll
        for (int i = 0; i < per; ++i) {
            if (before < kk && before + mine[i] >= kk) {
                *s_bin = threadIdx.x * per + i;
                *s_total = static_cast<int>(before + mine[i]);
            }
            before += mine[i];
        }
    }
    __syncthreads();
    bin = static_cast<uint32_t>(*s_bin);
    total = *s_total;
}

// grid = m * blocks_per_query workgroups; each filters rows_per_block stored distances of one
// query and appends the rows whose bin is at or below the boundary bin.
__global__ __launch_bounds__(kBlock) void hist_collect(const CollectArgs a)
{
    __shared__ uint32_t wave_sum[4];
    __shared__ int s_bin, s_total;
    const int q = blockIdx.x / a.blocks_per_query;
    const int chunk = blockIdx.x - q * a.blocks_per_query;
    uint32_t bin;
    int total;
    boundary_bin(a.hist + static_cast<size_t>(q) * kHistBins, a.k, wave_sum, &s_bin, &s_total, bin, total);
    if (total > a.cand_cap) return;                      // too many ties even for the list: hist_finish streams over the rows

    const uint32_t* dq = a.dist + static_cast<size_t>(q) * a.n;
    uint64_t* list = a.cand + static_cast<size_t>(q) * a.cand_cap;
    const int64_t r_begin = static_cast<int64_t>(chunk) * a.rows_per_block;
    const int64_t r_end = r_begin + a.rows_per_block < a.n ? r_begin + a.rows_per_block : a.n;
    // 16 rows per thread per step: the four 16-byte loads are issued before any is looked at
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
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t row = r0 + (static_cast<int64_t>(u) * kBlock + threadIdx.x) * 4 + e;
                const bool pass = row < r_end && (D[u][e] >> a.shift) <= bin;
                append_keys(pass, D[u][e], static_cast<uint32_t>(row), &a.cand_cnt[q], list, static_cast<uint32_t>(a.cand_cap));
            }
        }
    }
}

// grid = m workgroups: sort the candidates of one query by (D, row) and write the K best.
__global__ __launch_bounds__(kBlock) void hist_finish(const CollectArgs a)
{
    __shared__ uint64_t keys[kSortCap];
    __shared__ uint32_t wave_sum[4];
    __shared__ int s_bin, s_total, fill;
    const int q = blockIdx.x;
    uint32_t bin;
    int total;
    boundary_bin(a.hist + static_cast<size_t>(q) * kHistBins, a.k, wave_sum, &s_bin, &s_total, bin, total);
    if (total > a.cand_cap) {
        stream_select(a, q, keys, &fill);
        return;
    }
    const uint64_t* list = a.cand + static_cast<size_t>(q) * a.cand_cap;
    if (total > kSortCap) {
        stream_list(a, q, list, total, keys, &fill);
        return;
    }
    const int P = next_pow2(total);
    for (int t = threadIdx.x; t < P; t += blockDim.x) keys[t] = t < total ? list[t] : kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    write_result_h(a, q, keys);
}

// ---------------------------------------------------------------------------------------
template <int BQ, int BD>
static hipError_t launch_scan_hist_b(const HistArgs& a, dim3 grid, hipStream_t s)
{
    const bool pre = a.nchunks == 1 && a.W == a.wc;      // whole row in registers: prefetch the next bundle
    switch (a.wc) {
    case 1: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 1, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 1, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 2: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 2, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 2, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 3: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 3, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 3, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 4: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 4, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 4, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 5: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 5, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 5, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 6: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 6, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 6, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 7: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 7, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 7, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    case 8: if (pre) hipLaunchKernelGGL((scan_hist<BQ, BD, 8, true>), grid, dim3(kHistBlock), 0, s, a);
            else     hipLaunchKernelGGL((scan_hist<BQ, BD, 8, false>), grid, dim3(kHistBlock), 0, s, a);
            break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_clear(uint32_t* p, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    const int blocks = static_cast<int>((count + 255) / 256 < 1024 ? (count + 255) / 256 : 1024);
    hipLaunchKernelGGL(clear_u32, dim3(blocks), dim3(256), 0, s, p, count);
    return hipGetLastError();
}

hipError_t launch_scan_hist(const HistArgs& a, hipStream_t s)
{
    if (a.m < 1 || a.m > kHistMaxQueries || a.n < 1 || a.wc < 1 || a.wc > 8 || a.nchunks < 1) return hipErrorInvalidValue;
    const int64_t nbundles = (a.n + kLanes - 1) / kLanes;
    int64_t blocks = (nbundles + 15) / 16;
    if (blocks > 256) blocks = 256;                      // one per CU; the rest is grid-stride (measured: 512 is 3-5 % slower,
                                                         // twice the atomics of the final merge; 128 is far slower)
    dim3 grid(static_cast<unsigned>(blocks));
    switch (a.q_bits * 10 + a.db_bits) {
    case 11: return launch_scan_hist_b<1, 1>(a, grid, s);
    case 22: return launch_scan_hist_b<2, 2>(a, grid, s);
    case 33: return launch_scan_hist_b<3, 3>(a, grid, s);
    case 44: return launch_scan_hist_b<4, 4>(a, grid, s);
    case 21: return launch_scan_hist_b<2, 1>(a, grid, s);
    case 32: return launch_scan_hist_b<3, 2>(a, grid, s);
    case 43: return launch_scan_hist_b<4, 3>(a, grid, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_hist_collect(const CollectArgs& a, hipStream_t s)
{
    if (a.m < 1 || a.blocks_per_query < 1 || a.rows_per_block < 1 || a.rows_per_block % (16 * kBlock) != 0 ||
        a.cand_cap < kSortCap || a.cand_cap > kHistCandCap) return hipErrorInvalidValue;
    if (static_cast<int64_t>(a.blocks_per_query) * a.rows_per_block < a.n) return hipErrorInvalidValue;
    hipLaunchKernelGGL(hist_collect, dim3(static_cast<unsigned>(a.m * a.blocks_per_query)), dim3(kBlock), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(hist_finish, dim3(static_cast<unsigned>(a.m)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace xbq
