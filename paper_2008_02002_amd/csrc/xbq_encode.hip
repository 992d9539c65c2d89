// Encode kernels: scaling (Section 3.5), the quantizer f_B (Section 3.2) and the bit-plane
// reconstruction (Section 3.3, Eq. 5), fused in one pass over the fp32 rows.
//
// A wavefront reads 64 consecutive coordinates of one row (256 contiguous bytes), each
// lane quantizes its coordinate, and one ballot per plane turns the 64 per-lane bits into
// the two 32-bit plane words that cover those coordinates.  The paper does this step on
// the CPU with AVX (Section 4.1 "Quantization"); here it is bandwidth-bound GPU work.
//
// Quantizer.  f_B picks digits greedily, most significant first, with sign(0) = +1.  The
// cells that rule produces are [k / 2^(B-1), (k + 1) / 2^(B-1)), the outermost two open
// ended, so the cell index from the bottom is j = clamp(floor(t * 2^(B-1)) + 2^(B-1), 0,
// 2^B - 1) and the stored code (bit 1 = digit -1) is 2^B - 1 - j.  t * 2^(B-1) is exact in
// binary32 and floor is exact, so this equals the greedy comparisons bit for bit.  The
// product t = x * scale is a single rounded binary32 multiply; denormals are kept.

#include "xbq_internal.h"

namespace xbq {

template <int B>
__device__ __forceinline__ uint32_t quantize(float x, float scale)
{
    constexpr float half = static_cast<float>(1 << (B - 1));
    const float t = __fmul_rn(x, scale);                 // one rounding, never contracted
    float u = floorf(t * half);                          // exact
    u = fminf(fmaxf(u, -half), half - 1.0f);             // saturate before the conversion
    const int j = static_cast<int>(u) + (1 << (B - 1));
    return static_cast<uint32_t>(((1 << B) - 1) - j);
}

// Plane words of 64 coordinates of one row: lane l < 2B returns word (plane l>>1, half l&1).
template <int B>
__device__ __forceinline__ uint32_t plane_words(uint32_t code, bool valid, int lane)
{
    uint32_t mine = 0;
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const uint64_t mask = __ballot(valid && ((code >> b) & 1u));
        const uint32_t lo = static_cast<uint32_t>(mask), hi = static_cast<uint32_t>(mask >> 32);
        if ((lane >> 1) == b) mine = (lane & 1) ? hi : lo;
    }
    return mine;
}

// XBQ_ROWS: one wavefront per row.
template <int B>
__global__ __launch_bounds__(kBlock) void encode_rows(const float* __restrict__ X, int64_t n, int d, float scale,
                                                      uint32_t* __restrict__ codes)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const int W = (d + 31) / 32;
    const float* xr = X + row * d;
    uint32_t* out = codes + row * (static_cast<int64_t>(B) * W);
    for (int c0 = 0; c0 < d; c0 += 64) {
        const int c = c0 + lane;
        const bool valid = c < d;
        const uint32_t code = quantize<B>(valid ? xr[c] : 0.0f, scale);
        const uint32_t word = plane_words<B>(code, valid, lane);
        const int w = (c0 >> 5) + (lane & 1);
        if (lane < 2 * B && w < W) out[(lane >> 1) * W + w] = word;
    }
}

// XBQ_BUNDLE64: one workgroup per bundle of 64 rows; the bundle's words are staged in LDS
// as [B][W][64] and written out as one contiguous block.
template <int B>
__global__ __launch_bounds__(kBlock) void encode_bundle(const float* __restrict__ X, int64_t n, int d, float scale,
                                                        uint32_t* __restrict__ codes)
{
    extern __shared__ uint32_t tile[];                   // B * W * 64 words
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int W = (d + 31) / 32;
    const int64_t bundle = blockIdx.x;
    for (int rr = 0; rr < 16; ++rr) {
        const int r = wave * 16 + rr;                    // row inside the bundle
        const int64_t row = bundle * 64 + r;
        const bool live = row < n;
        const float* xr = X + (live ? row : 0) * d;
        for (int c0 = 0; c0 < d; c0 += 64) {
            const int c = c0 + lane;
            const bool valid = live && c < d;
            const uint32_t code = quantize<B>(valid ? xr[c] : 0.0f, scale);
            const uint32_t word = plane_words<B>(code, valid, lane);
            const int w = (c0 >> 5) + (lane & 1);
            if (lane < 2 * B && w < W) tile[((lane >> 1) * W + w) * 64 + r] = word;
        }
    }
    __syncthreads();
    const int words = B * W * 64;
    uint32_t* out = codes + bundle * static_cast<int64_t>(words);
    for (int t = threadIdx.x; t < words; t += blockDim.x) out[t] = tile[t];
}

template <int B>
static hipError_t launch_encode_b(const float* X, int64_t n, int d, float scale, int layout, uint32_t* codes,
                                  hipStream_t s)
{
    const int W = (d + 31) / 32;
    if (layout == XBQ_ROWS) {
        hipLaunchKernelGGL(encode_rows<B>, dim3(static_cast<unsigned>((n + 3) / 4)), dim3(kBlock), 0, s, X, n, d,
                           scale, codes);
    } else {
        const size_t lds = static_cast<size_t>(B) * W * 64 * sizeof(uint32_t);
        hipLaunchKernelGGL(encode_bundle<B>, dim3(static_cast<unsigned>((n + 63) / 64)), dim3(kBlock), lds, s, X, n,
                           d, scale, codes);
    }
    return hipGetLastError();
}

hipError_t launch_encode(const float* X, int64_t n, int d, int bits, float scale, int layout, uint32_t* codes,
                         hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    switch (bits) {
    case 1: return launch_encode_b<1>(X, n, d, scale, layout, codes, s);
    case 2: return launch_encode_b<2>(X, n, d, scale, layout, codes, s);
    case 3: return launch_encode_b<3>(X, n, d, scale, layout, codes, s);
    case 4: return launch_encode_b<4>(X, n, d, scale, layout, codes, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace xbq
