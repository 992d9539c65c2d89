// Second cross-check scan: the integer inner product S = sum_k m_qk m_xk of the decoded codes
// (m = (2^B - 1) - 2 xbar, |m| <= 15; Section 3.2 and Eq. 7 of Section 3.3) as an int8 matrix
// product on the matrix cores, D = (d (2^Bq - 1)(2^Bd - 1) - S) / 2.  Like the packed-dot
// kernel it is opt-in (option "kernel" = 2), serves d <= 256, produces the same D for every
// pair and shares everything downstream of the scan.  It is not the method of the paper (which
// avoids multiplies); it measures what the multiply form costs on this chip.
//
// Tiling.  One wavefront keeps R tiles of 32 database rows as MFMA B operands in registers
// (int8, K = 32 per instruction).  The workgroup stages tiles of 32 queries in LDS (rows padded
// by 16 bytes so the 16-byte operand reads of 32 lanes hit different banks) and every wavefront
// multiplies each query tile with its R row tiles: 32 x 32 scores per v_mfma_i32_32x32x32_i8
// chain.  The threshold test runs on the accumulator registers (16 compares per 1024 pairs).
//
// Survivors.  With 1024 pairs per accumulator tile almost every tile has a survivor, so the
// returning global atomic that reserves a slot in the query's candidate list must not sit in
// the loop.  Each wavefront appends its survivors to a record list of its own in LDS (the
// slot comes from ballot ranks and a wavefront-uniform count: no atomic at all); once per
// query tile it issues one global atomic per record and only stores the keys one iteration
// later, when the slots have long come back.  A record that does not fit the list takes the
// direct path (append_keys).

#include "xbq_device.h"

namespace xbq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Decoded int8 values of 32 coordinates -> 8 dwords.  plane[b]: the B plane words.
template <int B>
__device__ __forceinline__ void decode32(const uint32_t (&plane)[B], int live, uint32_t (&out)[8])
{
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        uint32_t word = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int t = 4 * g + e;
            uint32_t code = 0;
#pragma unroll
            for (int b = 0; b < B; ++b) code |= ((plane[b] >> t) & 1u) << b;
            const int m = t < live ? ((1 << B) - 1) - 2 * static_cast<int>(code) : 0;
            word |= (static_cast<uint32_t>(m) & 0xffu) << (8 * e);
        }
        out[g] = word;
    }
}

// XBQ_BUNDLE64 planes -> int8 rows [bundles * 64][32 W].
template <int B>
__global__ void bytes_from_bundles(const uint32_t* __restrict__ codes, int64_t bundles, int W, int d,
                                   uint32_t* __restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t total = bundles * W;
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x >> 6) + (threadIdx.x >> 6); i < total;
         i += static_cast<int64_t>(gridDim.x) * (blockDim.x >> 6)) {
        const int64_t bundle = i / W;
        const int w = static_cast<int>(i - bundle * W);
        uint32_t plane[B], bytes[8];
#pragma unroll
        for (int b = 0; b < B; ++b) plane[b] = codes[((bundle * B + b) * W + w) * 64 + lane];
        decode32<B>(plane, d - 32 * w, bytes);
        uint32_t* dst = out + ((bundle * 64 + lane) * W + w) * 8;
#pragma unroll
        for (int g = 0; g < 8; ++g) dst[g] = bytes[g];
    }
}

// XBQ_ROWS planes of m queries -> int8 rows [m_pad][32 W], rows m .. m_pad-1 zero.
template <int B>
__global__ void bytes_from_rows(const uint32_t* __restrict__ codes, int m, int m_pad, int W, int d,
                                uint32_t* __restrict__ out)
{
    const int64_t total = static_cast<int64_t>(m_pad) * W;
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t q = i / W;
        const int w = static_cast<int>(i - q * W);
        uint32_t bytes[8];
        if (q < m) {
            uint32_t plane[B];
#pragma unroll
            for (int b = 0; b < B; ++b) plane[b] = codes[(q * B + b) * W + w];
            decode32<B>(plane, d - 32 * w, bytes);
        } else {
#pragma unroll
            for (int g = 0; g < 8; ++g) bytes[g] = 0;
        }
#pragma unroll
        for (int g = 0; g < 8; ++g) out[i * 8 + g] = bytes[g];
    }
}

// KB = K blocks of 32 coordinates (= W), R = row tiles per wavefront.
template <int KB, int R, bool DENSE>
__global__ __launch_bounds__(kBlock) void scan_mfma(const MfmaArgs a)
{
    constexpr int DK = 32 * KB;                          // bytes per int8 row
    constexpr int LROW = DK + 16;                        // LDS row stride: odd multiple of 16 bytes
    __shared__ __attribute__((aligned(16))) uint8_t tile[2][32 * LROW];
    __shared__ __attribute__((aligned(16))) int tau[2][32];
    constexpr int RC = 2 * kLanes;                       // records per wavefront and query tile: two per lane
    __shared__ uint64_t rec_key[4][RC];
    __shared__ uint32_t rec_q[4][RC];
    uint32_t recorded = 0;                               // records of this wavefront in the current query tile
    uint32_t pend_q[2] = {0, 0}, pend_pos[2] = {0xffffffffu, 0xffffffffu};
    uint64_t pend_key[2] = {0, 0};
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int half = lane >> 5, col = lane & 31;
    int row_block, qrange;
    if (!decode_tile(a.row_blocks, a.qranges, row_block, qrange)) return;       // whole workgroup
    const int64_t row0 = a.row_begin + (static_cast<int64_t>(row_block) * 4 + wave) * (R * 32);
    const bool wave_live = row0 < a.row_end;             // wavefronts past the range still take the barriers

    // B operands: this lane's 16 bytes of every K block of its row in each tile
    v4i bop[R][KB];
    uint32_t row[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t rr = row0 + r * 32 + col;
        row[r] = static_cast<uint32_t>(rr);
        if (rr >= a.rows_padded) rr = a.rows_padded - 1;                          // stay inside the buffer
        const uint8_t* p = a.dbb + rr * DK + 16 * half;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) bop[r][kb] = *reinterpret_cast<const v4i*>(p + 32 * kb);
    }

    const int q0 = qrange * a.qsplit;                    // multiple of 32
    const int q1 = q0 + a.qsplit < a.m ? q0 + a.qsplit : a.m;
    // staging: the 32 x DK bytes of a query tile as 16-byte pieces, 2 * KB per row
    constexpr int kPieces = 32 * 2 * KB;
    constexpr int kPerThread = (kPieces + kBlock - 1) / kBlock;
    v4i stage[kPerThread];
    int stage_tau = 0;
    auto fetch = [&](int qt) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int piece = threadIdx.x + i * kBlock;
            if (piece < kPieces) {
                const int qr = piece / (2 * KB), off = (piece - qr * (2 * KB)) * 16;
                stage[i] = *reinterpret_cast<const v4i*>(a.qb + static_cast<int64_t>(qt + qr) * DK + off);
            }
        }
        if (threadIdx.x < 32) {
            const int q = qt + threadIdx.x;
            stage_tau = (!DENSE && q < a.m) ? a.full - 2 * static_cast<int>(a.thr[q]) : 0x7fffffff;
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int piece = threadIdx.x + i * kBlock;
            if (piece < kPieces) {
                const int qr = piece / (2 * KB), off = (piece - qr * (2 * KB)) * 16;
                *reinterpret_cast<v4i*>(&tile[buf][qr * LROW + off]) = stage[i];
            }
        }
        if (threadIdx.x < 32) tau[buf][threadIdx.x] = stage_tau;
    };

    fetch(q0);
    commit(0);
    __syncthreads();
    int cur = 0;
    for (int qt = q0; qt < q1; qt += 32) {
        const bool more = qt + 32 < q1;
        if (more) fetch(qt + 32);
        if (wave_live) {
            v4i aop[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
                aop[kb] = *reinterpret_cast<const v4i*>(&tile[cur][col * LROW + 32 * kb + 16 * half]);
            int tv[16];
            if (!DENSE) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const v4i t4 = *reinterpret_cast<const v4i*>(&tau[cur][8 * g + 4 * half]);
                    tv[4 * g + 0] = t4.x; tv[4 * g + 1] = t4.y; tv[4 * g + 2] = t4.z; tv[4 * g + 3] = t4.w;
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(aop[kb], bop[r][kb], acc, 0, 0, 0);
                // acc[v] = S(query qt + 8 (v / 4) + 4 half + v % 4, row[r])
                const bool row_ok = row[r] < a.row_end;
                if (DENSE) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int q = qt + 8 * (v >> 2) + 4 * half + (v & 3);
                        if (row_ok && q < a.m)
                            a.dense[static_cast<size_t>(q) * a.dense_stride + (row[r] - a.row_begin)] =
                                static_cast<uint32_t>((a.full - acc[v]) >> 1);
                    }
                } else {
                    bool any = false;
#pragma unroll
                    for (int v = 0; v < 16; ++v) any |= acc[v] > tv[v];
                    if (__builtin_expect(__ballot(any) != 0, 0)) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const bool pass = acc[v] > tv[v] && row_ok;          // tau is INT_MAX for q >= m
                            const uint64_t mask = __ballot(pass);
                            if (mask != 0) {
                                const uint32_t q = static_cast<uint32_t>(qt + 8 * (v >> 2) + 4 * half + (v & 3));
                                const uint32_t D = static_cast<uint32_t>((a.full - acc[v]) >> 1);
                                const uint32_t slot = recorded +
                                    __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                    __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
                                recorded += static_cast<uint32_t>(__popcll(mask));
                                const bool fits = slot < static_cast<uint32_t>(RC);
                                if (pass && fits) {
                                    rec_key[wave][slot] = make_key(D, row[r]);
                                    rec_q[wave][slot] = q;
                                }
                                // the rare record that does not fit goes straight to global memory
                                // (per half: the two halves of a register belong to different queries)
                                const bool spill = pass && !fits;
                                if (__ballot(spill) != 0) {
                                    const uint32_t qa = static_cast<uint32_t>(qt + 8 * (v >> 2) + (v & 3));
                                    const uint32_t q0s = qa < static_cast<uint32_t>(a.m) ? qa : 0u;
                                    const uint32_t q1s = qa + 4 < static_cast<uint32_t>(a.m) ? qa + 4 : 0u;
                                    append_keys(spill && half == 0, D, row[r], &a.cnt[q0s],
                                                a.cand + static_cast<size_t>(q0s) * a.cap, static_cast<uint32_t>(a.cap));
                                    append_keys(spill && half == 1, D, row[r], &a.cnt[q1s],
                                                a.cand + static_cast<size_t>(q1s) * a.cap, static_cast<uint32_t>(a.cap));
                                }
                            }
                        }
                    }
                }
            }
        }
        if (more) commit(cur ^ 1);
        __syncthreads();
        cur ^= 1;
        if (!DENSE) {
            // slots reserved one iteration ago have come back: store those keys ...
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if (pend_pos[i] < static_cast<uint32_t>(a.cap))
                    a.cand[static_cast<size_t>(pend_q[i]) * a.cap + pend_pos[i]] = pend_key[i];
                pend_pos[i] = 0xffffffffu;
            }
            // ... and reserve slots for the records this wavefront made in this query tile (its own
            // LDS writes, read back in program order: no barrier involved)
            const uint32_t have = recorded < static_cast<uint32_t>(RC) ? recorded : static_cast<uint32_t>(RC);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t slot = lane + i * kLanes;
                if (slot < have) {
                    pend_q[i] = rec_q[wave][slot];
                    pend_key[i] = rec_key[wave][slot];
                    pend_pos[i] = atomicAdd(&a.cnt[pend_q[i]], 1u);
                }
            }
            recorded = 0;
        }
    }
    if (!DENSE) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (pend_pos[i] < static_cast<uint32_t>(a.cap))
                a.cand[static_cast<size_t>(pend_q[i]) * a.cap + pend_pos[i]] = pend_key[i];
    }
}

template <int KB, int R>
static hipError_t launch_mfma_kr(const MfmaArgs& a, bool dense, dim3 grid, hipStream_t s)
{
    if (dense) hipLaunchKernelGGL((scan_mfma<KB, R, true>), grid, dim3(kBlock), 0, s, a);
    else       hipLaunchKernelGGL((scan_mfma<KB, R, false>), grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

template <int KB>
static hipError_t launch_mfma_k(MfmaArgs a, bool dense, hipStream_t s)
{
    constexpr int R = KB <= 4 ? 4 : 2;                   // 64 operand registers per lane either way
    const int64_t rows = a.row_end - a.row_begin;
    const int64_t row_blocks = (rows + 4 * R * 32 - 1) / (4 * R * 32);
    const int64_t total = (row_blocks + kXcds - 1) / kXcds * kXcds * a.qranges;
    if (row_blocks > 0x7fffffff || total > 0x7fffffff) return hipErrorInvalidValue;
    a.row_blocks = static_cast<int>(row_blocks);
    return launch_mfma_kr<KB, R>(a, dense, dim3(static_cast<unsigned>(total)), s);
}

hipError_t launch_scan_mfma(const MfmaArgs& args, bool dense, hipStream_t s)
{
    MfmaArgs a = args;
    if (a.row_end <= a.row_begin || a.m <= 0) return hipSuccess;
    if (a.row_begin % 32 != 0 || a.qsplit < 32 || a.qsplit % 32 != 0 || a.row_end > a.rows_padded ||
        a.m > a.m_padded || a.m_padded % 32 != 0)
        return hipErrorInvalidValue;
    a.qranges = (a.m + a.qsplit - 1) / a.qsplit;
    switch (a.W) {
    case 1: return launch_mfma_k<1>(a, dense, s);
    case 2: return launch_mfma_k<2>(a, dense, s);
    case 3: return launch_mfma_k<3>(a, dense, s);
    case 4: return launch_mfma_k<4>(a, dense, s);
    case 5: return launch_mfma_k<5>(a, dense, s);
    case 6: return launch_mfma_k<6>(a, dense, s);
    case 7: return launch_mfma_k<7>(a, dense, s);
    case 8: return launch_mfma_k<8>(a, dense, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_bytes_db(const uint32_t* codes, int64_t n, int d, int bits, uint32_t* out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int W = (d + 31) / 32;
    const int64_t bundles = (n + kLanes - 1) / kLanes;
    const int64_t items = bundles * W;
    const int blocks = static_cast<int>((items + 3) / 4 < 8192 ? (items + 3) / 4 : 8192);
    switch (bits) {
    case 1: hipLaunchKernelGGL(bytes_from_bundles<1>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    case 2: hipLaunchKernelGGL(bytes_from_bundles<2>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    case 3: hipLaunchKernelGGL(bytes_from_bundles<3>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    case 4: hipLaunchKernelGGL(bytes_from_bundles<4>, dim3(blocks), dim3(kBlock), 0, s, codes, bundles, W, d, out); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_bytes_q(const uint32_t* codes, int m, int m_pad, int d, int bits, uint32_t* out, hipStream_t s)
{
    if (m <= 0) return hipSuccess;
    const int W = (d + 31) / 32;
    const int64_t total = static_cast<int64_t>(m_pad) * W;
    const int blocks = static_cast<int>((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    switch (bits) {
    case 1: hipLaunchKernelGGL(bytes_from_rows<1>, dim3(blocks), dim3(256), 0, s, codes, m, m_pad, W, d, out); break;
    case 2: hipLaunchKernelGGL(bytes_from_rows<2>, dim3(blocks), dim3(256), 0, s, codes, m, m_pad, W, d, out); break;
    case 3: hipLaunchKernelGGL(bytes_from_rows<3>, dim3(blocks), dim3(256), 0, s, codes, m, m_pad, W, d, out); break;
    case 4: hipLaunchKernelGGL(bytes_from_rows<4>, dim3(blocks), dim3(256), 0, s, codes, m, m_pad, W, d, out); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace xbq
