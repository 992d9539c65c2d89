// Scan kernels: Eq. 10 of Section 3.3 (the POPCNT form), D = sum_i sum_j POPCNT(xhat_i ^ yhat_j) << (i + j),
// for every (query, database row) pair of a row range, on the vector ALUs of gfx950.
//
// Mapping.  One lane owns one database row (two when the code is short): its plane
// words sit in VGPRs.  The query is uniform across the wavefront, so its words are read
// with scalar loads and reach v_xor_b32 as SGPR operands; v_bcnt_u32_b32 adds the
// population count into an accumulator in the same instruction.  One accumulator per
// weight class i + j, combined by shift-adds once per pair.  The loop keeps no selection
// state: a pair either stores its distance (dense mode) or is compared with the query's
// current threshold and, if it beats it, is appended to that query's candidate list
// (threshold mode).  Nothing here uses the matrix cores: the work is bitwise.
//
// Two kernel families:
//   scan_resident  - whole code of the row(s) in registers, all queries stream past it;
//                    the database is read from memory exactly once per query range.
//   scan_chunked   - for long codes: the row is processed in chunks of WC words per
//                    plane against a register tile of kTileQ queries, one running sum per
//                    query and weight class; the database chunk comes from L2.
// In threshold mode a launch can also count the passing rows per distance level and can be
// switched off by a flag in device memory (both used by the whole-list form of Algorithm 1).

#include "xbq_device.h"

namespace xbq {

// ---------------------------------------------------------------------------------------
// Register-resident scan.  One workgroup = 4*R bundles of rows x one query range.
// ---------------------------------------------------------------------------------------
template <int BQ, int BD, int W, int R, bool DENSE>
__global__ __launch_bounds__(kBlock) void scan_resident(const ScanArgs a)
{
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    int row_block, qrange;
    if (!decode_tile(a.row_blocks, a.qranges, row_block, qrange)) return;
    if (!DENSE && a.run_flag != nullptr && ((uniform_ptr)a.run_flag)[0] == 0) return;
    const int64_t bundle0 = a.row_begin / kLanes + (static_cast<int64_t>(row_block) * 4 + wave) * R;
    if (bundle0 * kLanes >= a.row_end) return;
    const int64_t last_bundle = (a.n - 1) / kLanes;
    const int64_t full_bundles = a.n / kLanes;

    uint32_t x[R][BD][W];
    uint32_t row[R];                                 // the row's own number (in the keys)
    uint32_t col[R];                                 // its place in the range, counted from row_begin (dense columns)
    bool ok[R];                                      // inside the range
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t step = bundle0 + r;
        const int64_t bundle = spread_bundle(step <= last_bundle ? step : last_bundle, a.bundle_mul, full_bundles);
        const uint32_t* p = a.db + bundle * (BD * W * kLanes) + lane;   // inside the buffer in any case
#pragma unroll
        for (int b = 0; b < BD; ++b)
#pragma unroll
            for (int w = 0; w < W; ++w) x[r][b][w] = p[(b * W + w) * kLanes];
        row[r] = static_cast<uint32_t>(bundle * kLanes + lane);
        ok[r] = step * kLanes + lane < a.row_end;
        col[r] = static_cast<uint32_t>(step * kLanes + lane - a.row_begin);
    }

    const int q0 = qrange * a.qsplit;
    const int q1 = q0 + a.qsplit < a.m ? q0 + a.qsplit : a.m;
    __builtin_amdgcn_s_waitcnt(0);      // row words have landed: no per-load waits inside the loop
    for (int q = q0; q < q1; ++q) {
        uniform_ptr yq = (uniform_ptr)(a.q + static_cast<size_t>(q) * (BQ * W));
        uint32_t y[BQ][W];
#pragma unroll
        for (int b = 0; b < BQ; ++b)
#pragma unroll
            for (int w = 0; w < W; ++w) y[b][w] = yq[b * W + w];
        uint32_t D[R];
#pragma unroll
        for (int r = 0; r < R; ++r) D[r] = xor_popcount<BQ, BD, W>(x[r], y);

        if (DENSE) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (ok[r]) a.dense[static_cast<size_t>(q) * a.dense_stride + col[r]] = D[r];
        } else {
            const uint32_t t = ((uniform_ptr)a.thr)[q];
            bool any = false;
#pragma unroll
            for (int r = 0; r < R; ++r) any |= D[r] < t;
            if (__builtin_expect(__ballot(any) != 0, 0)) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const bool pass = D[r] < t && ok[r];
                    append_keys(pass, D[r], row[r], &a.cnt[q], a.cand + static_cast<size_t>(q) * a.cap,
                                static_cast<uint32_t>(a.cap));
                    if (a.levels != nullptr) count_level(pass, D[r], q, a);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Word-chunked scan.  Queries come from the chunk-major padded copy [m][nchunks][B][WC],
// so the B*WC words a (query, chunk) step needs are contiguous.  Words past W are zero on
// both sides and add nothing to D.
// ---------------------------------------------------------------------------------------
// EXACT: W is a multiple of WC, so no chunk reaches past the row's words and the loads need no guard.
template <int BQ, int BD, int WC, bool DENSE, bool EXACT>
__global__ __launch_bounds__(kBlock) void scan_chunked(const ScanArgs a)
{
    constexpr int TQ = kTileQ;
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    int row_block, qrange;
    if (!decode_tile(a.row_blocks, a.qranges, row_block, qrange)) return;
    if (!DENSE && a.run_flag != nullptr && ((uniform_ptr)a.run_flag)[0] == 0) return;
    const int64_t step = a.row_begin / kLanes + static_cast<int64_t>(row_block) * 4 + wave;
    if (step * kLanes >= a.row_end) return;
    const int64_t bundle = spread_bundle(step, a.bundle_mul, a.n / kLanes);
    const int W = a.W;
    const uint32_t* xb = a.db + bundle * (static_cast<int64_t>(BD) * W * kLanes) + lane;
    const uint32_t row = static_cast<uint32_t>(bundle * kLanes + lane);              // the row's own number
    const bool valid = step * kLanes + lane < a.row_end;
    const uint32_t col = static_cast<uint32_t>(step * kLanes + lane - a.row_begin);  // its place in the range

    const int q0 = qrange * a.qsplit;
    const int q1 = q0 + a.qsplit < a.m ? q0 + a.qsplit : a.m;
    for (int qt = q0; qt < q1; qt += TQ) {
        constexpr int C = BQ + BD - 1;
        uint32_t cls[TQ][C];                          // one running sum per query and weight class
#pragma unroll
        for (int t = 0; t < TQ; ++t)
#pragma unroll
            for (int c = 0; c < C; ++c) cls[t][c] = 0;
        for (int c = 0; c < a.nchunks; ++c) {
            uint32_t x[BD][WC];
#pragma unroll
            for (int b = 0; b < BD; ++b)
#pragma unroll
                for (int w = 0; w < WC; ++w) {
                    const int ww = c * WC + w;
                    x[b][w] = (EXACT || ww < W) ? xb[(b * W + ww) * kLanes] : 0u;
                }
#pragma unroll
            for (int t = 0; t < TQ; ++t) {
                const int q = qt + t < a.m ? qt + t : a.m - 1;     // clamp: tail tiles reread the last query
                uniform_ptr yq = (uniform_ptr)(a.q + (static_cast<size_t>(q) * a.nchunks + c) * (BQ * WC));
                uint32_t y[BQ][WC];
#pragma unroll
                for (int b = 0; b < BQ; ++b)
#pragma unroll
                    for (int w = 0; w < WC; ++w) y[b][w] = yq[b * WC + w];
                xor_popcount_classes<BQ, BD, WC>(x, y, cls[t]);
            }
        }
        uint32_t acc[TQ];
#pragma unroll
        for (int t = 0; t < TQ; ++t) acc[t] = combine_classes<C>(cls[t]);
#pragma unroll
        for (int t = 0; t < TQ; ++t) {
            const int q = qt + t;
            if (q < q1) {
                if (DENSE) {
                    if (valid) a.dense[static_cast<size_t>(q) * a.dense_stride + col] = acc[t];
                } else {
                    const uint32_t thr = ((uniform_ptr)a.thr)[q];
                    append_keys(acc[t] < thr && valid, acc[t], row, &a.cnt[q], a.cand + static_cast<size_t>(q) * a.cap,
                                static_cast<uint32_t>(a.cap));
                    if (a.levels != nullptr) count_level(acc[t] < thr && valid, acc[t], q, a);
                }
            }
        }
    }
}

// XBQ_ROWS [m][B][W] -> chunk-major padded [m][nchunks][B][WC]; words past W become zero.
__global__ void repack_queries(const uint32_t* __restrict__ src, int m, int B, int W, int wc, int nchunks,
                               uint32_t* __restrict__ dst)
{
    const int64_t per = static_cast<int64_t>(nchunks) * B * wc;
    const int64_t total = static_cast<int64_t>(m) * per;
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t q = i / per;
        int rem = static_cast<int>(i - q * per);
        const int c = rem / (B * wc);
        rem -= c * B * wc;
        const int b = rem / wc;
        const int w = c * wc + (rem - b * wc);
        dst[i] = w < W ? src[(q * B + b) * W + w] : 0u;
    }
}

// ---------------------------------------------------------------------------------------
// Dispatch
// ---------------------------------------------------------------------------------------
bool scan_is_resident(int W) { return W >= 1 && W <= 8; }

int scan_chunk_words(int W)
{
    int best = 8, best_padded = 1 << 30;
    for (int wc = 5; wc <= 8; ++wc) {
        const int padded = (W + wc - 1) / wc * wc;
        if (padded <= best_padded) { best_padded = padded; best = wc; }
    }
    return best;
}

// One-dimensional grid covering row_blocks x qranges tiles, padded to whole XCD rounds.
static bool tile_grid(ScanArgs& a, int64_t bundles, int bundles_per_block, dim3& grid)
{
    const int64_t row_blocks = (bundles + bundles_per_block - 1) / bundles_per_block;
    const int64_t total = (row_blocks + kXcds - 1) / kXcds * kXcds * a.qranges;
    if (row_blocks > 0x7fffffff || total > 0x7fffffff) return false;
    a.row_blocks = static_cast<int>(row_blocks);
    grid = dim3(static_cast<unsigned>(total));
    return true;
}

template <int BQ, int BD, int W, int R>
static hipError_t launch_resident_brw(ScanArgs a, bool dense, int64_t bundles, hipStream_t s)
{
    dim3 grid;
    if (!tile_grid(a, bundles, 4 * R, grid)) return hipErrorInvalidValue;
    if (dense) hipLaunchKernelGGL((scan_resident<BQ, BD, W, R, true>), grid, dim3(kBlock), 0, s, a);
    else       hipLaunchKernelGGL((scan_resident<BQ, BD, W, R, false>), grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

template <int BQ, int BD, int W>
static hipError_t launch_resident_bw(const ScanArgs& a, bool dense, int64_t bundles, hipStream_t s)
{
    if constexpr (BD * W <= 16) {
        if (a.rows_per_lane == 2) return launch_resident_brw<BQ, BD, W, 2>(a, dense, bundles, s);
    }
    return launch_resident_brw<BQ, BD, W, 1>(a, dense, bundles, s);
}

template <int BQ, int BD>
static hipError_t launch_resident_b(const ScanArgs& a, bool dense, int64_t bundles, hipStream_t s)
{
    switch (a.W) {
    case 1: return launch_resident_bw<BQ, BD, 1>(a, dense, bundles, s);
    case 2: return launch_resident_bw<BQ, BD, 2>(a, dense, bundles, s);
    case 3: return launch_resident_bw<BQ, BD, 3>(a, dense, bundles, s);
    case 4: return launch_resident_bw<BQ, BD, 4>(a, dense, bundles, s);
    case 5: return launch_resident_bw<BQ, BD, 5>(a, dense, bundles, s);
    case 6: return launch_resident_bw<BQ, BD, 6>(a, dense, bundles, s);
    case 7: return launch_resident_bw<BQ, BD, 7>(a, dense, bundles, s);
    case 8: return launch_resident_bw<BQ, BD, 8>(a, dense, bundles, s);
    default: return hipErrorInvalidValue;
    }
}

template <int BQ, int BD, int WC>
static hipError_t launch_chunked_bw(ScanArgs a, bool dense, int64_t bundles, hipStream_t s)
{
    dim3 grid;
    if (!tile_grid(a, bundles, 4, grid)) return hipErrorInvalidValue;
    if (dense)               hipLaunchKernelGGL((scan_chunked<BQ, BD, WC, true, false>), grid, dim3(kBlock), 0, s, a);
    else if (a.W % WC == 0)  hipLaunchKernelGGL((scan_chunked<BQ, BD, WC, false, true>), grid, dim3(kBlock), 0, s, a);
    else                     hipLaunchKernelGGL((scan_chunked<BQ, BD, WC, false, false>), grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

template <int BQ, int BD>
static hipError_t launch_chunked_b(const ScanArgs& a, bool dense, int64_t bundles, hipStream_t s)
{
    switch (a.wc) {
    case 5: return launch_chunked_bw<BQ, BD, 5>(a, dense, bundles, s);
    case 6: return launch_chunked_bw<BQ, BD, 6>(a, dense, bundles, s);
    case 7: return launch_chunked_bw<BQ, BD, 7>(a, dense, bundles, s);
    case 8: return launch_chunked_bw<BQ, BD, 8>(a, dense, bundles, s);
    default: return hipErrorInvalidValue;
    }
}

template <int BQ, int BD>
static hipError_t launch_scan_b(const ScanArgs& a, bool dense, int64_t bundles, hipStream_t s)
{
    return a.wc == 0 ? launch_resident_b<BQ, BD>(a, dense, bundles, s) : launch_chunked_b<BQ, BD>(a, dense, bundles, s);
}

bool scan_supports_bits(int q_bits, int db_bits)
{
    return db_bits >= 1 && db_bits <= XBQ_MAX_BITS && (q_bits == db_bits || q_bits == db_bits + 1) &&
           q_bits <= XBQ_MAX_BITS;
}

hipError_t launch_scan(const ScanArgs& args, bool dense, hipStream_t s)
{
    ScanArgs a = args;
    if (a.row_end <= a.row_begin || a.m <= 0) return hipSuccess;
    if (a.row_begin % kLanes != 0 || a.qsplit < 1 || a.row_end > a.n) return hipErrorInvalidValue;
    const int64_t bundles = (a.row_end - a.row_begin + kLanes - 1) / kLanes;
    a.qranges = (a.m + a.qsplit - 1) / a.qsplit;
    switch (a.q_bits * 10 + a.db_bits) {
    case 11: return launch_scan_b<1, 1>(a, dense, bundles, s);
    case 22: return launch_scan_b<2, 2>(a, dense, bundles, s);
    case 33: return launch_scan_b<3, 3>(a, dense, bundles, s);
    case 44: return launch_scan_b<4, 4>(a, dense, bundles, s);
    case 21: return launch_scan_b<2, 1>(a, dense, bundles, s);
    case 32: return launch_scan_b<3, 2>(a, dense, bundles, s);
    case 43: return launch_scan_b<4, 3>(a, dense, bundles, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_repack_queries(const uint32_t* q_rows, int m, int bits, int W, int wc, int nchunks,
                                 uint32_t* q_chunked, hipStream_t s)
{
    if (m <= 0) return hipSuccess;
    const int64_t total = static_cast<int64_t>(m) * nchunks * bits * wc;
    const int blocks = static_cast<int>((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(repack_queries, dim3(blocks), dim3(256), 0, s, q_rows, m, bits, W, wc, nchunks, q_chunked);
    return hipGetLastError();
}

}  // namespace xbq
