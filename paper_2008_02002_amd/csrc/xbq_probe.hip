// Measurement aids: what this chip sustains on the streams the rooflines of the search are
// quoted against.  probe_xor_popcount issues the scan's credited instruction pair (v_xor_b32
// with a scalar operand, v_bcnt_u32_b32 with accumulate; Section 3.3, Eq. 10) from registers
// only; probe_read streams a buffer from memory with 16-byte loads; probe_encode_traffic moves
// the encoder's bytes (fp32 rows in, code words out, same access pattern) without quantizing.
// All write a checkable result so that nothing can be optimised away, and are timed by the caller.

#include "xbq_device.h"

namespace xbq {

constexpr int kProbeBlocks = 256 * 8;      // 8 workgroups of 4 wavefronts per compute unit: 8 wavefronts per SIMD
constexpr int kProbeWords = 16;            // row words held per lane, as in the 4-bit d = 128 scan
constexpr int kProbeUnroll = 4;

// out[thread] = sum over it < iters * kProbeUnroll, j < kProbeWords of POPCNT(x_j ^ (seed + it)),
// x_j = (thread + 1) * 0x9E3779B1 + j * 0x85EBCA77 (mod 2^32), thread = global thread number.
__global__ __launch_bounds__(kBlock) void probe_xor_popcount(uint32_t* out, uint32_t seed, int iters)
{
    const uint32_t thread = blockIdx.x * kBlock + threadIdx.x;
    uint32_t x[kProbeWords];
#pragma unroll
    for (int j = 0; j < kProbeWords; ++j) x[j] = (thread + 1u) * 0x9E3779B1u + static_cast<uint32_t>(j) * 0x85EBCA77u;
    uint32_t acc[4] = {0, 0, 0, 0};
    uint32_t y = seed;                                   // uniform: lives in a scalar register
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
#pragma unroll
            for (int j = 0; j < kProbeWords; ++j) acc[j & 3] = popcount_add(x[j] ^ y, acc[j & 3]);
            ++y;
        }
    }
    out[thread] = acc[0] + acc[1] + acc[2] + acc[3];
}

// out[workgroup] = sum (mod 2^32) of the 32-bit words this workgroup read.  Each workgroup owns one
// contiguous piece of the buffer and reads it with non-temporal 16-byte loads, eight in flight
// per lane: of the access patterns tried this is the one that streams fastest on this part
// (grid-stride temporal loads reach about three quarters of it).
typedef uint32_t native_uint4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kBlock) void probe_read(const native_uint4* __restrict__ p, size_t n16, size_t per_block,
                                                     uint32_t* out)
{
    __shared__ uint32_t total;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    constexpr int U = 8;
    uint32_t s = 0;
    const size_t b0 = static_cast<size_t>(blockIdx.x) * per_block;
    const size_t b1 = b0 + per_block < n16 ? b0 + per_block : n16;
    size_t i = b0 + threadIdx.x;
    for (; i + (U - 1) * kBlock < b1; i += U * kBlock) {
        native_uint4 a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(p + i + u * kBlock);
#pragma unroll
        for (int u = 0; u < U; ++u) s += a[u].x + a[u].y + a[u].z + a[u].w;
    }
    for (; i < b1; i += kBlock) {
        const native_uint4 a = __builtin_nontemporal_load(p + i);
        s += a.x + a.y + a.z + a.w;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off);
    if (lane_id() == 0) atomicAdd(&total, s);
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = total;
}

// The encoder's memory traffic without its arithmetic: one workgroup per bundle of 64 rows reads
// the bundle's fp32 rows (contiguous, 64 * d * 4 bytes) with non-temporal 16-byte loads, eight in
// flight per lane, and writes the bundle's code words (contiguous, 64 * bits * W * 4 bytes), as
// encode_bundle_vec4 does.  Thread t stores the sum (mod 2^32) of the 32-bit words it read into
// every code word t, t + 256, ... of its bundle, so the result can be checked and nothing can be
// optimised away.
__global__ __launch_bounds__(kBlock) void probe_encode_traffic(const native_uint4* __restrict__ X4, int64_t n,
                                                               int f4_per_row, int words, uint32_t* __restrict__ codes)
{
    const int64_t bundle = blockIdx.x;
    const int64_t row0 = bundle * kLanes;
    const int live = n - row0 < kLanes ? static_cast<int>(n - row0) : kLanes;
    const int total = live * f4_per_row;
    const native_uint4* src = X4 + row0 * f4_per_row;
    constexpr int U = 8;
    uint32_t s = 0;
    for (int i0 = threadIdx.x; i0 < total; i0 += kBlock * U) {
        native_uint4 a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u * kBlock;
            if (i < total) a[u] = __builtin_nontemporal_load(src + i);
            else a[u] = native_uint4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) s += a[u].x + a[u].y + a[u].z + a[u].w;
    }
    uint32_t* out = codes + bundle * static_cast<int64_t>(words);
    for (int t = threadIdx.x; t < words; t += kBlock) out[t] = s;
}

size_t probe_out_bytes() { return static_cast<size_t>(kProbeBlocks) * kBlock * sizeof(uint32_t); }

double probe_valu_lane_ops(int iters)
{
    return 2.0 * kProbeWords * kProbeUnroll * static_cast<double>(iters) * kProbeBlocks * kBlock;
}

hipError_t launch_probe_valu(uint32_t* out, uint32_t seed, int iters, hipStream_t s)
{
    hipLaunchKernelGGL(probe_xor_popcount, dim3(kProbeBlocks), dim3(kBlock), 0, s, out, seed, iters);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void* buf, size_t bytes, uint32_t* out, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    const size_t per_block = (n16 + kProbeBlocks - 1) / kProbeBlocks;
    hipLaunchKernelGGL(probe_read, dim3(kProbeBlocks), dim3(kBlock), 0, s, static_cast<const native_uint4*>(buf), n16,
                       per_block, out);
    return hipGetLastError();
}

hipError_t launch_probe_encode_traffic(const float* X, int64_t n, int d, int bits, uint32_t* codes, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (d % 4 != 0 || reinterpret_cast<uintptr_t>(X) % 16 != 0) return hipErrorInvalidValue;
    const int words = bits * words32(d) * kLanes;
    hipLaunchKernelGGL(probe_encode_traffic, dim3(static_cast<unsigned>((n + kLanes - 1) / kLanes)), dim3(kBlock), 0, s,
                       reinterpret_cast<const native_uint4*>(X), n, d / 4, words, codes);
    return hipGetLastError();
}

}  // namespace xbq
