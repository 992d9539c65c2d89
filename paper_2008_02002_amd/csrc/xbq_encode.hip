// Encode kernels: scaling (Section 3.5), the quantizer f_B (Section 3.2) and the bit-plane
// reconstruction (Section 3.3, Eq. 9), fused in one pass over the fp32 rows.
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

// The fp32 input is read once and never again: non-temporal loads keep it from displacing the
// codes in the caches, and they stream measurably faster on this part.
typedef float native_float4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_streaming(const float4* p)
{
    const native_float4 v = __builtin_nontemporal_load(reinterpret_cast<const native_float4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
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
    // 16 rows per wavefront, 64 coordinates per step; loads are issued eight steps ahead of
    // their use so that each wavefront keeps 2 KB in flight.
    const int steps = (d + 63) >> 6;
    const int items = 16 * steps;
    constexpr int U = 8;
    for (int i0 = 0; i0 < items; i0 += U) {
        float v[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u;
            const int rr = i / steps, c = ((i - rr * steps) << 6) + lane;
            const int64_t row = bundle * 64 + wave * 16 + rr;
            ok[u] = i < items && row < n && c < d;
            v[u] = ok[u] ? __builtin_nontemporal_load(X + row * d + c) : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u;
            if (i < items) {
                const int rr = i / steps, st = i - rr * steps;
                const uint32_t word = plane_words<B>(quantize<B>(v[u], scale), ok[u], lane);
                const int w = (st << 1) + (lane & 1);
                if (lane < 2 * B && w < W) tile[((lane >> 1) * W + w) * 64 + wave * 16 + rr] = word;
            }
        }
    }
    __syncthreads();
    const int words = B * W * 64;
    uint32_t* out = codes + bundle * static_cast<int64_t>(words);
    for (int t = threadIdx.x; t < words; t += blockDim.x) out[t] = tile[t];
}

// OR of a value over each aligned group of 8 lanes (every lane of the group gets the result):
// neighbour swap, pair swap, then mirror within the half row.
__device__ __forceinline__ uint32_t or_reduce8(uint32_t v)
{
    v |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    return v;
}

// XBQ_BUNDLE64 for d a multiple of 4: 16 bytes per lane.  Every row is seen as 8*W slots of
// 4 coordinates (slots past d are padding), so an aligned group of 8 lanes always covers
// exactly one plane word.  A lane quantizes its 4 coordinates; per plane it squeezes its 4
// code bits into a nibble (mask, one 24-bit multiply that moves bits 0,4,8,12 to 12..15,
// bit-field extract), shifts it to its place in the word, and a 3-step DPP OR over the 8
// lanes completes the word.  Lane b of each group stores plane b's word into the LDS tile.
template <int B>
__global__ __launch_bounds__(kBlock) void encode_bundle_vec4(const float4* __restrict__ X4, int64_t n, int d,
                                                             float scale, float inv_slots, uint32_t* __restrict__ codes)
{
    extern __shared__ uint32_t tile[];                   // B * W rows of 65 words: the pad word spreads the
                                                         // lanes of a wavefront, which write one column, over the banks
    const int W = (d + 31) >> 5;
    const int slots = 8 * W;                             // float4 slots per row, padding included
    const int f4_per_row = d >> 2;                       // real float4s per row
    const int64_t bundle = blockIdx.x;
    const int64_t row0 = bundle * 64;
    const int live = n - row0 < 64 ? static_cast<int>(n - row0) : 64;
    const int total = live * slots;                      // multiple of 8
    const float4* src = X4 + row0 * f4_per_row;
    const int words = B * W * 64;
    if (live < 64) {                                     // rows past n must come out as zero words
        for (int t = threadIdx.x; t < words + B * W; t += blockDim.x) tile[t] = 0;
        __syncthreads();
    }
    const int sub = threadIdx.x & 7;                     // position inside the group of 8 lanes
    constexpr int U = 8;                                 // 16-byte loads in flight per lane
    for (int i0 = threadIdx.x; i0 < total; i0 += kBlock * U) {
        float4 v[U];
        int r[U], slot[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // i / slots without an integer division or a full 32-bit multiply: (i + 0.5) / slots is
            // at least 0.5 / 512 away from an integer, far more than the rounding of the two float
            // operations on values below 2^16; the 24-bit multiplies below are exact for the same reason
            const int i = i0 + u * kBlock;
            r[u] = static_cast<int>((static_cast<float>(i) + 0.5f) * inv_slots);
            slot[u] = i - static_cast<int>(__umul24(r[u], slots));
            const bool real = i < total && slot[u] < f4_per_row;
            const uint32_t off = __umul24(r[u], f4_per_row) + static_cast<uint32_t>(slot[u]);
            v[u] = real ? load_streaming(src + off) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u * kBlock;               // groups of 8 lanes are all in or all out
            uint32_t packed = quantize<B>(v[u].x, scale) | (quantize<B>(v[u].y, scale) << 4) |
                              (quantize<B>(v[u].z, scale) << 8) | (quantize<B>(v[u].w, scale) << 12);
            if (slot[u] >= f4_per_row) packed = 0;       // padding coordinates store zero bits
            uint32_t mine = 0;
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const uint32_t spread = packed & (0x1111u << b);                    // bits b, b+4, b+8, b+12
                const uint32_t nib = (__umul24(spread, 0x1248u >> b) >> 12) & 0xFu; // -> bits 0..3
                const uint32_t word = or_reduce8(nib << (4 * sub));
                if (sub == b) mine = word;
            }
            if (i < total && sub < B) tile[(sub * W + (slot[u] >> 3)) * 65 + r[u]] = mine;
        }
    }
    __syncthreads();
    uint32_t* out = codes + bundle * static_cast<int64_t>(words);
    for (int t = threadIdx.x; t < words; t += blockDim.x) out[t] = tile[t + (t >> 6)];
}

template <int B>
static hipError_t launch_encode_b(const float* X, int64_t n, int d, float scale, int layout, uint32_t* codes,
                                  hipStream_t s)
{
    const int W = (d + 31) / 32;
    if (layout == XBQ_ROWS) {
        hipLaunchKernelGGL(encode_rows<B>, dim3(static_cast<unsigned>((n + 3) / 4)), dim3(kBlock), 0, s, X, n, d,
                           scale, codes);
    } else if (d % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0) {
        const float inv_slots = 1.0f / static_cast<float>(8 * W);       // slots = 8 * W <= 512 per row
        const size_t lds = static_cast<size_t>(B) * W * 65 * sizeof(uint32_t);
        hipLaunchKernelGGL(encode_bundle_vec4<B>, dim3(static_cast<unsigned>((n + 63) / 64)), dim3(kBlock), lds, s,
                           reinterpret_cast<const float4*>(X), n, d, scale, inv_slots, codes);
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
