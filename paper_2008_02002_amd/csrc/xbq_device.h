// Device functions shared by the kernels of libxbq.so (included by the .hip files only).
#pragma once

#include "xbq_internal.h"

namespace xbq {

// Uniform (wavefront-invariant) data is read through the constant address space so that the
// compiler uses scalar loads and the values arrive in SGPRs.
typedef const uint32_t __attribute__((address_space(4))) * uniform_ptr;
typedef const int32_t __attribute__((address_space(4))) * uniform_iptr;

constexpr uint64_t kPadKey = ~0ull;                      // sorts after every real key

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }

__device__ __forceinline__ int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Workgroup barrier for data exchanged through LDS only: orders LDS accesses around the barrier
// and leaves global loads in flight (__syncthreads() also waits for those).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// acc + POPCNT(v) in one instruction.  Written as an instruction so the compiler keeps one
// running sum per weight class; left to itself it re-associates the sums into trees of
// three-input adds, which costs a fifth more vector instructions.
__device__ __forceinline__ uint32_t popcount_add(uint32_t v, uint32_t acc)
{
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(v), "v"(acc));
    return r;
}

// Eq. 10 of Section 3.3 (the POPCNT form) for one row held in x (BD planes) against the uniform query words y
// (BQ planes), WC words per plane: sum_i sum_j POPCNT(x_i ^ y_j) << (i + j), with one running
// sum per weight class i + j and a Horner combination at the end.
template <int BQ, int BD, int WC>
__device__ __forceinline__ uint32_t xor_popcount(const uint32_t (&x)[BD][WC], const uint32_t (&y)[BQ][WC])
{
    constexpr int C = BQ + BD - 1;
    uint32_t acc[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        bool first = true;
#pragma unroll
        for (int i = 0; i < BD; ++i) {
            const int j = c - i;
            if (j < 0 || j >= BQ) continue;
#pragma unroll
            for (int w = 0; w < WC; ++w) {
                const uint32_t v = x[i][w] ^ y[j][w];
                acc[c] = first ? static_cast<uint32_t>(__builtin_popcount(v)) : popcount_add(v, acc[c]);
                first = false;
            }
        }
    }
    uint32_t D = acc[C - 1];
#pragma unroll
    for (int c = C - 2; c >= 0; --c) D = (D << 1) + acc[c];
    return D;
}

// The same sums left apart: acc[c] += sum over i + j = c, w of POPCNT(x_i[w] ^ y_j[w]).  For rows
// that come in several chunks of words the Horner combination is then done once per row, not
// once per chunk.
template <int BQ, int BD, int WC>
__device__ __forceinline__ void xor_popcount_classes(const uint32_t (&x)[BD][WC], const uint32_t (&y)[BQ][WC],
                                                     uint32_t (&acc)[BQ + BD - 1])
{
#pragma unroll
    for (int c = 0; c < BQ + BD - 1; ++c)
#pragma unroll
        for (int i = 0; i < BD; ++i) {
            const int j = c - i;
            if (j < 0 || j >= BQ) continue;
#pragma unroll
            for (int w = 0; w < WC; ++w) acc[c] = popcount_add(x[i][w] ^ y[j][w], acc[c]);
        }
}

template <int C>
__device__ __forceinline__ uint32_t combine_classes(const uint32_t (&acc)[C])
{
    uint32_t D = acc[C - 1];
#pragma unroll
    for (int c = C - 2; c >= 0; --c) D = (D << 1) + acc[c];
    return D;
}

// Append the keys of the lanes with `pass` set to list[0 .. cap): one atomic per wavefront on
// *counter reserves the slots, v_mbcnt ranks the lanes.  Keys past cap are dropped; the
// counter still counts them, which is how an overflow is seen later.
__device__ __forceinline__ void append_keys(bool pass, uint32_t D, uint32_t row, uint32_t* counter, uint64_t* list,
                                            uint32_t cap)
{
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    const int leader = __ffsll(static_cast<long long>(mask)) - 1;
    uint32_t base = 0;
    if (lane_id() == leader) base = atomicAdd(counter, static_cast<uint32_t>(__popcll(mask)));
    base = __shfl(base, leader);
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
    const uint32_t pos = base + rank;
    if (pass && pos < cap) list[pos] = make_key(D, row);
}

// Optional bookkeeping of the threshold mode: one count per passing row in its distance level.
__device__ __forceinline__ void count_level(bool pass, uint32_t D, int q, const ScanArgs& a)
{
    if (!pass) return;
    const uint32_t base = a.level_base[q];
    atomicAdd(&a.levels[static_cast<size_t>(q) * a.level_stride + (D < base ? 0u : D - base + 1u)], 1u);
}

// By one wavefront: the smallest bin b of h[0 .. kHistBins) such that bins 0..b hold at least k
// rows, or -1 if all bins together hold fewer; *before = rows in bins below b.  Every lane gets
// the result.  (Algorithm 1's boundary, Section 4.1 "Histogram and Select", at bin resolution.)
__device__ __forceinline__ int wave_boundary_bin(const uint32_t* h, uint32_t k, uint32_t* before_out)
{
    constexpr int kPer = kHistBins / kLanes;             // 16 consecutive bins per lane
    const int lane = lane_id();
    uint32_t mine[kPer];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) { mine[i] = h[lane * kPer + i]; sum += mine[i]; }
    uint32_t incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    uint32_t before = incl - sum;
    int bin = -1;
    uint32_t below = 0;
    if (before < k && incl >= k) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (bin < 0 && before + mine[i] >= k) { bin = lane * kPer + i; below = before; }
            before += mine[i];
        }
    }
    const uint64_t found = __ballot(bin >= 0);
    if (found == 0) { *before_out = 0; return -1; }
    const int src = __ffsll(static_cast<long long>(found)) - 1;
    *before_out = __shfl(below, src);
    return __shfl(bin, src);
}

// Order in which the threshold schedule takes the bundles of the database.  Its row groups are
// ranges of this order, and thresholds found on one group filter the next: on rows that come
// sorted or cluster by cluster, groups of consecutive rows would see, again and again, whole
// runs of rows better than anything before (survivor lists overflow, queries are re-scored
// exactly: measured ten times slower).  So step n of the order is full bundle (n * mul) mod
// (number of full bundles), mul coprime to that number and near its golden section: every
// range of steps is spread evenly over the database.  The last, partial bundle keeps its
// place.  mul <= 1 is the plain order.  Results do not depend on the order.
__host__ __device__ inline int64_t spread_bundle(int64_t step, int64_t mul, int64_t full_bundles)
{
    return mul > 1 && step < full_bundles
               ? static_cast<int64_t>((static_cast<uint64_t>(step) * static_cast<uint64_t>(mul)) %
                                      static_cast<uint64_t>(full_bundles))
               : step;
}

// Workgroup -> (row block, query range) of the scan kernels.  The grid is one-dimensional.
// Hardware hands consecutive workgroup ids to the 8 XCDs in turn, each XCD with its own L2,
// so the id is split as (id % 8, id / 8): XCD c works through row blocks c, c + 8, c + 16, ...
// and for each of them through all query ranges back to back.  A row block is then fetched
// from HBM by one XCD only and stays in that L2 while its query ranges run; the (small) query
// array is what every XCD shares.  If the hardware assigned ids differently the result would
// be the same, only the locality would be lost.
constexpr int kXcds = 8;
__device__ __forceinline__ bool decode_tile(int row_blocks, int qranges, int& row_block, int& qrange)
{
    const unsigned id = blockIdx.x;
    const unsigned xcd = id % kXcds, j = id / kXcds;
    row_block = static_cast<int>((j / qranges) * kXcds + xcd);
    qrange = static_cast<int>(j % qranges);
    return row_block < row_blocks;
}

// Ascending bitonic sort of P (power of two) 64-bit keys in LDS by the whole workgroup.
// The caller has synchronised after filling `keys`; the routine ends with a barrier.
__device__ inline void bitonic_sort_lds(uint64_t* keys, int P)
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

// Descending variant of the sort above (same contract).
__device__ inline void bitonic_sort_lds_descending(uint64_t* keys, int P)
{
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (P >> 1); t += blockDim.x) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const int l = i | j;
                const bool down = (i & k) == 0;
                const uint64_t a = keys[i], b = keys[l];
                if ((a < b) == down) { keys[i] = b; keys[l] = a; }
            }
            __syncthreads();
        }
    }
}

// Last stage of the ascending sort alone: turns a bitonic sequence of P keys (ascending run
// followed by a descending run) into an ascending one in log2(P) steps.
__device__ inline void bitonic_merge_lds(uint64_t* keys, int P)
{
    for (int j = P >> 1; j > 0; j >>= 1) {
        for (int t = threadIdx.x; t < (P >> 1); t += blockDim.x) {
            const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
            const int l = i | j;
            const uint64_t a = keys[i], b = keys[l];
            if (a > b) { keys[i] = b; keys[l] = a; }
        }
        __syncthreads();
    }
}

// Eq. 10 for one (row, query) with run-time sizes; the slow path of the exact rescans.
__device__ inline uint32_t distance_generic(const uint32_t* db, int64_t row, const uint32_t* yq, int BQ, int BD, int W)
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

// fp32 similarity as the upper half of a 64-bit sort key: ascending keys = descending floats.
__device__ __forceinline__ uint32_t descending_bits(float v)
{
    uint32_t u = __float_as_uint(v);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);     // ascending order of floats as unsigned
    return ~u;                                           // reversed: larger float = smaller key
}

__device__ __forceinline__ float bits_to_float_descending(uint32_t k)
{
    uint32_t u = ~k;
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __uint_as_float(u);
}

}  // namespace xbq
