// Cross-check scan: the same integer distances from packed 4-bit dot products.
//
// The decoded value of a B-bit code xbar is m / 2^B with m = (2^B - 1) - 2 xbar (Section 3.2),
// an odd integer, so the score of Eq. 7 (Section 3.3) is the plain integer inner product
// S = sum_k m_xk m_yk.  Writing m = 2u + 1 with u = 2^(B-1) - 1 - xbar, a signed value that
// fits 4 bits for every B <= 4,
//     S = 4 sum u v + 2 sum u + 2 sum v + d,      D = (d (2^Bq - 1)(2^Bd - 1) - S) / 2,
// and sum u v over 8 coordinates is one v_dot8_i32_i4.  This kernel exists to check the XOR +
// population-count scan on the device against a different instruction mix and to measure what
// that formulation costs on this chip; it is opt-in (option "kernel" = 1) and is not the
// method of the paper, which replaces multiplies by XOR.  It produces the same D for every
// pair, so everything downstream (threshold filter, candidate lists, selection) is shared.

#include "xbq_device.h"

namespace xbq {

// 8 bits -> the least significant bit of each of 8 nibbles.
__device__ __forceinline__ uint32_t spread8(uint32_t byte)
{
    uint32_t x = byte & 0xffu;
    x = (x | (x << 12)) & 0x000f000fu;
    x = (x | (x << 6)) & 0x03030303u;
    x = (x | (x << 3)) & 0x11111111u;
    return x;
}

// Nibbles u = 2^(B-1) - 1 - xbar (two's complement, 4 bits) of coordinates 8g .. 8g+7 of one
// plane-word group; plane[b] are the B plane words of 32 coordinates, `live` of them real.
template <int B>
__device__ __forceinline__ uint32_t nibbles_of(const uint32_t (&plane)[B], int g, int live)
{
    uint32_t code = 0;
#pragma unroll
    for (int b = 0; b < B; ++b) code |= spread8(plane[b] >> (8 * g)) << b;
    uint32_t u = code ^ (0x11111111u * ((1u << (B - 1)) - 1u));        // xbar ^ (2^(B-1) - 1)
    if (B < 4) {                                                         // sign-extend from bit B-1
        const uint32_t sign = u & (0x11111111u << (B - 1));
#pragma unroll
        for (int e = B; e < 4; ++e) u |= sign << (e - (B - 1));
    }
    const int keep = live - 8 * g;                                       // real coordinates in this dword
    if (keep <= 0) return 0u;
    if (keep < 8) u &= (1u << (4 * keep)) - 1u;                          // padding contributes u = 0
    return u;
}

// Database: XBQ_BUNDLE64 planes [nb][B][W][64] -> nibbles [nb][4W][64].
template <int B>
__global__ void nibbles_from_bundles(const uint32_t* __restrict__ codes, int64_t bundles, int W, int d,
                                     uint32_t* __restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t total = bundles * W;
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x >> 6) + (threadIdx.x >> 6); i < total;
         i += static_cast<int64_t>(gridDim.x) * (blockDim.x >> 6)) {
        const int64_t bundle = i / W;
        const int w = static_cast<int>(i - bundle * W);
        uint32_t plane[B];
#pragma unroll
        for (int b = 0; b < B; ++b) plane[b] = codes[((bundle * B + b) * W + w) * 64 + lane];
        const int live = d - 32 * w;
#pragma unroll
        for (int g = 0; g < 4; ++g) out[((bundle * W + w) * 4 + g) * 64 + lane] = nibbles_of<B>(plane, g, live);
    }
}

// Queries: XBQ_ROWS planes [m][B][W] -> nibbles [m][4W] and the row sums of v.
template <int B>
__global__ void nibbles_from_rows(const uint32_t* __restrict__ codes, int m, int W, int d, uint32_t* __restrict__ out,
                                  int32_t* __restrict__ vsum)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= m) return;
    int32_t sum = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t plane[B];
#pragma unroll
        for (int b = 0; b < B; ++b) plane[b] = codes[(static_cast<size_t>(q) * B + b) * W + w];
        const int live = d - 32 * w;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t u = nibbles_of<B>(plane, g, live);
            out[(static_cast<size_t>(q) * W + w) * 4 + g] = u;
            sum = __builtin_amdgcn_sdot8(static_cast<int>(u), 0x11111111, sum, false);
        }
    }
    vsum[q] = sum;
}

// Same tiling and workgroup order as scan_resident; WD = 4 * W dwords of nibbles per row.
template <int WD, int R, bool DENSE>
__global__ __launch_bounds__(kBlock) void scan_dot8(const DotArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int row_block, qrange;
    if (!decode_tile(a.row_blocks, a.qranges, row_block, qrange)) return;
    const int64_t bundle0 = a.row_begin / kLanes + (static_cast<int64_t>(row_block) * 4 + wave) * R;
    if (bundle0 * kLanes >= a.row_end) return;
    const int64_t last_bundle = (a.n - 1) / kLanes;

    int x[R][WD];
    int rsum[R];
    uint32_t row[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t bundle = bundle0 + r;
        const int64_t ld = bundle <= last_bundle ? bundle : last_bundle;
        const uint32_t* p = a.dbn + ld * (WD * kLanes) + lane;
        rsum[r] = 0;
#pragma unroll
        for (int w = 0; w < WD; ++w) {
            x[r][w] = static_cast<int>(p[w * kLanes]);
            rsum[r] = __builtin_amdgcn_sdot8(x[r][w], 0x11111111, rsum[r], false);
        }
        row[r] = static_cast<uint32_t>(bundle * kLanes + lane);
    }
    const int q0 = qrange * a.qsplit;
    const int q1 = q0 + a.qsplit < a.m ? q0 + a.qsplit : a.m;
    __builtin_amdgcn_s_waitcnt(0);
    for (int q = q0; q < q1; ++q) {
        uniform_ptr yq = (uniform_ptr)(a.qn + static_cast<size_t>(q) * WD);
        int y[WD];
#pragma unroll
        for (int w = 0; w < WD; ++w) y[w] = static_cast<int>(yq[w]);
        const int base = a.half_full_minus_d - ((uniform_iptr)a.qsum)[q];    // (full - d) / 2 - sum v
        uint32_t D[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            int acc0 = 0, acc1 = 0;
#pragma unroll
            for (int w = 0; w < WD; w += 2) {
                acc0 = __builtin_amdgcn_sdot8(x[r][w], y[w], acc0, false);
                if (w + 1 < WD) acc1 = __builtin_amdgcn_sdot8(x[r][w + 1], y[w + 1], acc1, false);
            }
            D[r] = static_cast<uint32_t>(base - rsum[r] - 2 * (acc0 + acc1));
        }
        if (DENSE) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (row[r] < a.row_end)
                    a.dense[static_cast<size_t>(q) * a.dense_stride + (row[r] - a.row_begin)] = D[r];
        } else {
            const uint32_t t = ((uniform_ptr)a.thr)[q];
            bool any = false;
#pragma unroll
            for (int r = 0; r < R; ++r) any |= D[r] < t;
            if (__builtin_expect(__ballot(any) != 0, 0)) {
#pragma unroll
                for (int r = 0; r < R; ++r)
                    append_keys(D[r] < t && row[r] < a.row_end, D[r], row[r], &a.cnt[q], a.cand + static_cast<size_t>(q) * a.cap,
                                static_cast<uint32_t>(a.cap));
            }
        }
    }
}

template <int WD, int R>
static hipError_t launch_dot_wr(const DotArgs& a, bool dense, dim3 grid, hipStream_t s)
{
    if (dense) hipLaunchKernelGGL((scan_dot8<WD, R, true>), grid, dim3(kBlock), 0, s, a);
    else       hipLaunchKernelGGL((scan_dot8<WD, R, false>), grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

template <int WD>
static hipError_t launch_dot_w(DotArgs a, bool dense, int64_t bundles, hipStream_t s)
{
    const int R = (WD <= 16 && a.rows_per_lane == 2) ? 2 : 1;
    const int64_t row_blocks = (bundles + 4 * R - 1) / (4 * R);
    const int64_t total = (row_blocks + 7) / 8 * 8 * a.qranges;
    if (row_blocks > 0x7fffffff || total > 0x7fffffff) return hipErrorInvalidValue;
    a.row_blocks = static_cast<int>(row_blocks);
    dim3 grid(static_cast<unsigned>(total));
    if constexpr (WD <= 16) {
        if (R == 2) return launch_dot_wr<WD, 2>(a, dense, grid, s);
    }
    return launch_dot_wr<WD, 1>(a, dense, grid, s);
}

hipError_t launch_scan_dot(const DotArgs& args, bool dense, hipStream_t s)
{
    DotArgs a = args;
    if (a.row_end <= a.row_begin || a.m <= 0) return hipSuccess;
    if (a.row_begin % kLanes != 0 || a.qsplit < 1 || a.row_end > a.n) return hipErrorInvalidValue;
    const int64_t bundles = (a.row_end - a.row_begin + kLanes - 1) / kLanes;
    a.qranges = (a.m + a.qsplit - 1) / a.qsplit;
    switch (a.WD) {
    case 4: return launch_dot_w<4>(a, dense, bundles, s);
    case 8: return launch_dot_w<8>(a, dense, bundles, s);
    case 12: return launch_dot_w<12>(a, dense, bundles, s);
    case 16: return launch_dot_w<16>(a, dense, bundles, s);
    case 20: return launch_dot_w<20>(a, dense, bundles, s);
    case 24: return launch_dot_w<24>(a, dense, bundles, s);
    case 28: return launch_dot_w<28>(a, dense, bundles, s);
    case 32: return launch_dot_w<32>(a, dense, bundles, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_nibbles_db(const uint32_t* codes, int64_t n, int d, int bits, uint32_t* out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int W = (d + 31) / 32;
    const int64_t bundles = (n + kLanes - 1) / kLanes;
    const int64_t items = bundles * W;
    const int blocks = static_cast<int>((items + 3) / 4 < 8192 ? (items + 3) / 4 : 8192);
    switch (bits) {
    case 1: hipLaunchKernelGGL(nibbles_from_bundles<1>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    case 2: hipLaunchKernelGGL(nibbles_from_bundles<2>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    case 3: hipLaunchKernelGGL(nibbles_from_bundles<3>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    case 4: hipLaunchKernelGGL(nibbles_from_bundles<4>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_nibbles_q(const uint32_t* codes, int m, int d, int bits, uint32_t* out, int32_t* vsum, hipStream_t s)
{
    if (m <= 0) return hipSuccess;
    const int W = (d + 31) / 32;
    const int blocks = (m + 255) / 256;
    switch (bits) {
    case 1: hipLaunchKernelGGL(nibbles_from_rows<1>, dim3(blocks), dim3(256), 0, s, codes, m, W, d, out, vsum); break;
    case 2: hipLaunchKernelGGL(nibbles_from_rows<2>, dim3(blocks), dim3(256), 0, s, codes, m, W, d, out, vsum); break;
    case 3: hipLaunchKernelGGL(nibbles_from_rows<3>, dim3(blocks), dim3(256), 0, s, codes, m, W, d, out, vsum); break;
    case 4: hipLaunchKernelGGL(nibbles_from_rows<4>, dim3(blocks), dim3(256), 0, s, codes, m, W, d, out, vsum); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace xbq
