// Few queries (the single-request mode the paper measures, Section 5), two launches, no
// distance ever stored: the scan selects while it streams.
//
// With one or two queries the scan is bound by the HBM stream of the database codes, so the
// path moves those bytes once and nothing else of size n.  Algorithm 1's selector (Section 4.1
// "Histogram and Select": histogram of the integer distances, boundary at the K-th smallest)
// is applied per workgroup, on the rows that workgroup streams:
//
//   scan_local    Each workgroup owns one contiguous piece of the database.  It keeps, per
//                 query, a histogram of D >> shift of the rows it let through and a list of
//                 their keys, both in LDS.  A row of the global top-K is also in the top-K of
//                 its own piece, so a row may be dropped as soon as K rows of the same piece
//                 lie in lower bins.  Every wavefront's first chunk is scored without a
//                 threshold and only counted; once the first boundary exists, the boundary is
//                 recomputed from the histogram every time the rows handed out have grown by an
//                 eighth and the threshold lowered (by whichever wavefront notices first, no
//                 barrier); for rows in random order about K ln(rows / first rows) rows pass.
//                 A list that reaches its level (rows ordered towards the query, cluster after
//                 cluster) asks for a compaction: all wavefronts finish their chunk, the lists
//                 are cut at the boundary of the moment (exactly, by sorting, when thousands of
//                 distances share the boundary bin) and the stream goes on; lists of 4096 keys
//                 leave room for every row in flight, so no key is lost on the way.
//                 At the end the list (a superset of the piece's K best, typically K plus the
//                 ties of one bin) goes to the workgroup's own slot: no global atomics, nothing
//                 to clear beforehand.
//                 If a list overflows all the same (ties at the K-th distance itself that no list
//                 can hold) the workgroup re-selects its piece exactly for that query: bounded
//                 buffer, sorted and cut to K whenever it fills (slow, always exact).
//                 The list leaves sorted and cut to the piece's K best keys.
//   local_finish  One workgroup per query merges the lists, reading only their heads: histogram
//                 of D >> shift2 (4096 bins), boundary bin, the keys at or below it sorted by
//                 (D, row), first K written.  When a head turns out too short (the result sits in
//                 a few pieces) the rest of those lists is read, but only keys up to the K-th key
//                 of the heads can matter and those are few; massive ties at the boundary are
//                 streamed with a running threshold on the whole key.
//
// Ties go to the lower row: keys are (D << 32) | row and every cut is made on whole keys or
// keeps whole bins.

#include "xbq_device.h"

namespace xbq {

namespace {

constexpr int kLocalBlock = 1024;                     // threads per workgroup
constexpr int kLocalWaves = kLocalBlock / kLanes;
constexpr int kFinishBins = 4096;
constexpr int kLocalMaxCap = 4096;                    // keys in a per-piece list: room for 2048 rows in flight and more
constexpr int kRankSortMax = 512;                     // most keys sorted by ranking instead of the bitonic network
constexpr int kRankAsIs = 128;                        // a final list this short is ranked without a last compaction
                                                      // (ranking costs have^2 / 1024 comparisons per thread)

__device__ __forceinline__ uint32_t load_stream(const uint32_t* p) { return __builtin_nontemporal_load(p); }

// LDS of scan_local, carved from one dynamic allocation.
struct LocalLds {
    uint64_t* buf;        // [m][cap] keys let through
    uint32_t* hist;       // [m][kHistBins]
    uint32_t* cnt;        // [kLocalMaxQueries] keys in buf[t]
    uint32_t* thr;        // [kLocalMaxQueries] a row passes when D < thr[t]
    uint32_t* ovf;        // [kLocalMaxQueries] set when a key did not fit
    uint32_t* level;      // [kLocalMaxQueries] a list that reaches this length asks for a compaction
    uint32_t* next;       // next chunk of the piece to hand out
    uint32_t* mark;       // chunks handed out when the thresholds were last recomputed
    uint32_t* want;       // set when some list asks for a compaction
    uint32_t* done;       // one bit per wavefront that has no chunk left
};

__device__ __forceinline__ LocalLds carve(uint64_t* base, int m, int cap)
{
    LocalLds s;
    s.buf = base;
    s.hist = reinterpret_cast<uint32_t*>(base + static_cast<size_t>(m) * cap);
    s.cnt = s.hist + m * kHistBins;
    s.thr = s.cnt + kLocalMaxQueries;
    s.ovf = s.thr + kLocalMaxQueries;
    s.level = s.ovf + kLocalMaxQueries;
    s.next = s.level + kLocalMaxQueries;
    s.mark = s.next + 1;
    s.want = s.mark + 1;
    s.done = s.want + 1;
    return s;
}

// Append the keys of the passing lanes to an LDS list: one LDS atomic per wavefront reserves
// the slots.  Keys that do not fit raise *ovf.  Passing rows are also counted in hist.  With
// level given, the append that takes the list across *level raises *want.
__device__ __forceinline__ void append_lds(bool pass, uint32_t D, uint32_t row, uint64_t* list, uint32_t* counter,
                                           uint32_t cap, uint32_t* ovf, uint32_t* hist, int shift,
                                           const uint32_t* level = nullptr, uint32_t* want = nullptr)
{
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    const int leader = __ffsll(static_cast<long long>(mask)) - 1;
    uint32_t base = 0;
    if (lane_id() == leader) {
        const uint32_t count = static_cast<uint32_t>(__popcll(mask));
        base = atomicAdd(counter, count);
        if (level != nullptr && base < *level && base + count >= *level) *want = 1u;
    }
    base = __shfl(base, leader);
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
    if (pass) {
        const uint32_t pos = base + rank;
        if (pos < cap) list[pos] = make_key(D, row);
        else *ovf = 1u;
        if (hist != nullptr) atomicAdd(&hist[D >> shift], 1u);
    }
}

// Smallest bin b such that bins 0..b of h[0 .. PER * blockDim) hold at least k rows; the last
// bin if all of them hold fewer.  *within = rows in bins 0..b.  Called by every thread of the
// workgroup (1024 threads); contains barriers.
template <int PER>
__device__ int boundary_of(const uint32_t* h, int k, uint32_t* wave_sum, int* pick, int* within)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t mine[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) { mine[i] = h[threadIdx.x * PER + i]; sum += mine[i]; }
    uint32_t incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wave_sum[wave] = incl;
    if (threadIdx.x == 0) { pick[0] = PER * kLocalBlock - 1; pick[1] = -1; }
    __syncthreads();
    uint32_t before = incl - sum, all = 0;
    for (int w = 0; w < kLocalWaves; ++w) {
        const uint32_t v = wave_sum[w];
        if (w < wave) before += v;
        all += v;
    }
    const uint32_t kk = static_cast<uint32_t>(k);
    if (before < kk && before + sum >= kk) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (before < kk && before + mine[i] >= kk) {
                pick[0] = threadIdx.x * PER + i;
                pick[1] = static_cast<int>(before + mine[i]);
            }
            before += mine[i];
        }
    }
    __syncthreads();
    const int bin = pick[0];
    *within = pick[1] < 0 ? static_cast<int>(all) : pick[1];
    __syncthreads();                                     // pick and wave_sum may be reused at once
    return bin;
}

// Eq. 10 (Section 3.3, the POPCNT form) for one row against query t of the chunk-major query
// layout, run-time sizes: the slow path of the exact re-selection.
__device__ uint32_t distance_chunked(const LocalArgs& a, int64_t row, int t)
{
    const uint32_t* xb = a.db + (row / kLanes) * (static_cast<int64_t>(a.db_bits) * a.W * kLanes) + (row % kLanes);
    const uint32_t* yq = a.q + static_cast<size_t>(t) * a.nchunks * a.q_bits * a.wc;
    uint32_t D = 0;
    for (int w = 0; w < a.W; ++w) {
        const int c = w / a.wc, o = w - c * a.wc;
        uint32_t x[XBQ_MAX_BITS], y[XBQ_MAX_BITS];
        for (int b = 0; b < a.db_bits; ++b) x[b] = xb[(b * a.W + w) * kLanes];
        for (int b = 0; b < a.q_bits; ++b) y[b] = yq[(c * a.q_bits + b) * a.wc + o];
        for (int i = 0; i < a.db_bits; ++i)
            for (int j = 0; j < a.q_bits; ++j) D += static_cast<uint32_t>(__builtin_popcount(x[i] ^ y[j])) << (i + j);
    }
    return D;
}

// Exact K best rows of the piece [row_begin, row_end) for query t into buf (at most cap keys),
// rows in ascending order: a later row gets in only with a smaller D than the K-th best so far.
__device__ void reselect_piece(const LocalArgs& a, const LocalLds& s, int t, int64_t row_begin, int64_t row_end)
{
    uint64_t* buf = s.buf + static_cast<size_t>(t) * a.cap;
    const int chunk = a.cap / 2 < kLocalBlock ? a.cap / 2 : kLocalBlock;     // k <= cap / 8, so k + chunk fits
    if (threadIdx.x == 0) s.cnt[t] = 0;
    __syncthreads();
    uint32_t thr = 0xffffffffu;
    for (int64_t r0 = row_begin; r0 < row_end; r0 += chunk) {
        const int64_t row = r0 + threadIdx.x;
        if (static_cast<int>(threadIdx.x) < chunk && row < row_end) {
            const uint32_t D = distance_chunked(a, row, t);
            if (D < thr) buf[atomicAdd(&s.cnt[t], 1u)] = make_key(D, static_cast<uint32_t>(row));
        }
        __syncthreads();
        const int have = static_cast<int>(s.cnt[t]);     // <= cap: at most cap - chunk before this round
        if (have > a.cap - chunk) {
            const int P = next_pow2(have);
            for (int i = have + threadIdx.x; i < P; i += kLocalBlock) buf[i] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(buf, P);
            if (have > a.k) {
                thr = static_cast<uint32_t>(buf[a.k - 1] >> 32);
                __syncthreads();
                if (threadIdx.x == 0) s.cnt[t] = static_cast<uint32_t>(a.k);
            }
        }
        __syncthreads();
    }
}

// Rank of every one of `have` distinct keys in LDS (have <= kRankSortMax): rank[i] = number of
// keys smaller than keys[i].  The comparisons of one key are split over 1024 / P threads
// (P = have rounded up to a power of two), which add their counts into rank[].  rank[] is an LDS
// array of at least `have` words; all threads of the workgroup call this; ends with a barrier.
__device__ void rank_keys(const uint64_t* keys, int have, uint32_t* rank)
{
    const int P = next_pow2(have);
    const int parts = kLocalBlock / P;                   // >= 2
    const int i = threadIdx.x & (P - 1), part = threadIdx.x / P;
    if (static_cast<int>(threadIdx.x) < have) rank[threadIdx.x] = 0;
    __syncthreads();
    if (i < have) {
        const uint64_t key = keys[i];
        const int per = (have + parts - 1) / parts;
        const int j0 = part * per, j1 = j0 + per < have ? j0 + per : have;
        uint32_t r = 0;
        for (int j = j0; j < j1; ++j) r += keys[j] < key ? 1u : 0u;
        if (r != 0) atomicAdd(&rank[i], r);
    }
    __syncthreads();
}

// New threshold of a query from its piece histogram, by one wavefront: (b + 1) << shift for the
// smallest bin b such that bins 0..b hold at least k rows; no threshold while there are fewer.
__device__ __forceinline__ uint32_t wave_boundary(const uint32_t* h, int k, int shift)
{
    uint32_t below;
    const int bin = wave_boundary_bin(h, static_cast<uint32_t>(k), &below);
    return (static_cast<uint32_t>(bin < 0 ? kHistBins - 1 : bin) + 1u) << shift;
}

// Exact cut of a list of `have` keys (more than k) by the whole workgroup: sorted, only the keys
// up to the K-th distance stay, *cnt becomes their number and *thr at most that distance + 1.
// Kept out of line: it is rare, and inlined its registers crowd the streaming loop.  Its
// pointers say that they point into LDS: across a call that knowledge would be lost otherwise,
// and the sort would go through the generic address path.
using lds_u64 = __attribute__((address_space(3))) uint64_t;
using lds_u32 = __attribute__((address_space(3))) uint32_t;
__device__ __noinline__ void cut_list_exactly(lds_u64* buf, int have, int k, lds_u32* cnt, lds_u32* thr)
{
    const int P = next_pow2(have);
    for (int i = have + threadIdx.x; i < P; i += kLocalBlock) buf[i] = kPadKey;
    __syncthreads();
    for (int kk = 2; kk <= P; kk <<= 1) {                // ascending bitonic network, as bitonic_sort_lds
        for (int j = kk >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (P >> 1); t += kLocalBlock) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const int l = i | j;
                const bool up = (i & kk) == 0;
                const uint64_t x = buf[i], y = buf[l];
                if ((x > y) == up) { buf[i] = y; buf[l] = x; }
            }
            __syncthreads();
        }
    }
    const uint32_t kth = static_cast<uint32_t>(buf[k - 1] >> 32);
    for (int i = threadIdx.x; i < have; i += kLocalBlock) {
        const bool in = static_cast<uint32_t>(buf[i] >> 32) <= kth;
        const bool next_in = i + 1 < have && static_cast<uint32_t>(buf[i + 1] >> 32) <= kth;
        if (in && !next_in) *cnt = static_cast<uint32_t>(i + 1);
    }
    if (threadIdx.x == 0 && kth + 1u < *thr) *thr = kth + 1u;
    __syncthreads();
}

}  // namespace

// One workgroup per piece of a.bundles_per_group bundles; MQ >= a.m is the number of queries the
// register arrays are sized for (1 or kLocalMaxQueries).
//
// The piece is cut into chunks of R bundles which the wavefronts of the workgroup take from an
// LDS counter: the wavefronts share SIMDs and memory paths unevenly, and with a fixed assignment
// the slowest one, several chunks behind after a few dozen steps, kept the other fifteen waiting
// at every threshold update and at the end with nothing left to load.  The first chunk of every
// wavefront is scored without a threshold and only counted (the rows wait in registers until the
// first thresholds exist); from then on the thresholds are lowered without any barrier.  The
// workgroup stops to compact its lists only when one of them is half full (rows that come
// ordered towards the query, cluster after cluster): every wavefront then finishes the chunk it
// is in, and the request comes early enough for all of those rows to fit (lists of 4096 keys,
// at most 2048 rows in flight), so no key is ever lost.
// PREFETCH (whole row in registers, nchunks == 1): the rows of a wavefront's next chunk are
// requested before the current one is scored, so the stream keeps flowing while the workgroup
// sits in the barriers of a threshold update.
template <int BQ, int BD, int WC, int R, bool PREFETCH, int MQ>
__device__ __forceinline__ void scan_local_body(const LocalArgs& a)
{
    extern __shared__ uint64_t local_lds[];
    const LocalLds s = carve(local_lds, a.m, a.cap);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < a.m * kHistBins; i += kLocalBlock) s.hist[i] = 0;
    // A list asks for a compaction when it reaches its level.  Every wavefront then finishes the
    // chunk it is in, which may add R * 64 rows each, plus the rest of the append that crossed
    // the level: a level at most this low leaves room for all of them, so no key is lost.
    const uint32_t safe_level = static_cast<uint32_t>(a.cap) - static_cast<uint32_t>(kLocalWaves * R * kLanes + 2 * kLanes);
    if (threadIdx.x < kLocalMaxQueries) {
        s.cnt[threadIdx.x] = 0;
        s.thr[threadIdx.x] = 0xffffffffu;
        s.ovf[threadIdx.x] = 0;
        s.level[threadIdx.x] = safe_level;
    }
    // the first epoch: one chunk per wavefront, scored without a threshold
    constexpr int warm = kLocalWaves;
    if (threadIdx.x == 0) {
        *s.next = kLocalWaves;                           // chunks 0 .. 15 are handed out by wavefront number
        *s.mark = static_cast<uint32_t>(warm);
        *s.want = 0;
        *s.done = 0;
    }

    const int64_t nbundles = (a.n + kLanes - 1) / kLanes;
    const int64_t b_begin = static_cast<int64_t>(blockIdx.x) * a.bundles_per_group;
    const int64_t b_end = b_begin + a.bundles_per_group < nbundles ? b_begin + a.bundles_per_group : nbundles;
    const int chunks = static_cast<int>((b_end - b_begin + R - 1) / R);
    const int64_t row_stride = static_cast<int64_t>(BD) * a.W * kLanes;
    // Which chunk of the piece the n-th chunk handed out is.  The first 16 (one per wavefront,
    // scored without a threshold) lie evenly spaced over the piece, so that the first thresholds
    // come from a sample of all of it, not from its beginning (rows ordered by cluster); the others
    // follow in the order they lie, the stream staying sequential.
    const int spacing = chunks / warm;                   // >= 2 for this to matter
    const float per_gap = 1.0f / static_cast<float>(spacing > 1 ? spacing - 1 : 1);
    auto place_of = [&](int c) -> int {
        if (spacing < 2 || c >= chunks) return c;
        if (c < warm) return c * spacing;
        const int j = c - warm;                          // j-th of the chunks that are no multiple of the spacing, or lie behind them
        if (j >= warm * (spacing - 1)) return j + warm;
        if (chunks >= (1 << 23)) {                       // beyond what a float counts exactly: divide
            const int gap = j / (spacing - 1);
            return gap * spacing + 1 + (j - gap * (spacing - 1));
        }
        int gap = static_cast<int>(static_cast<float>(j) * per_gap);   // j / (spacing - 1) by multiplication, then set right
        if ((gap + 1) * (spacing - 1) <= j) ++gap;
        if (gap * (spacing - 1) > j) --gap;
        return gap * spacing + 1 + (j - gap * (spacing - 1));
    };

    uint32_t thr[MQ];
#pragma unroll
    for (int t = 0; t < MQ; ++t) thr[t] = 0xffffffffu;

    int cur = wave;                                      // chunk this wavefront works on (same in every lane)
    uint32_t xn[R][BD][WC];                              // PREFETCH: rows of chunk `cur`, on their way
    if (PREFETCH && cur < chunks) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t bundle = b_begin + static_cast<int64_t>(place_of(cur)) * R + r;
            if (bundle < b_end) {
                const uint32_t* xb = a.db + bundle * row_stride + lane;
#pragma unroll
                for (int b = 0; b < BD; ++b)
#pragma unroll
                    for (int w = 0; w < WC; ++w) xn[r][b][w] = load_stream(xb + (b * WC + w) * kLanes);
            }
        }
    }
    lds_barrier();

    // Rounds.  The first is the chunk every wavefront starts with.  In the later ones the
    // wavefronts stream until the chunks run out or a list asks for a compaction, and single
    // wavefronts lower the thresholds whenever the chunks handed out have grown by an eighth (no
    // barrier: a histogram that is being added to can only give a boundary that is too high, never
    // one that drops a row it should keep).  Between rounds the whole workgroup stops.
    uint32_t acc0[R][MQ];                                // the first chunk's rows, held until thresholds exist
    uint32_t row0[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        row0[r] = 0xffffffffu;                           // no row: fails the `< a.n` test below
#pragma unroll
        for (int t = 0; t < MQ; ++t) acc0[r][t] = 0;
    }
    for (bool first = true; ; ) {
        while (cur < chunks && (first ? cur < warm : *static_cast<volatile uint32_t*>(s.want) == 0)) {
            uint32_t acc[R][MQ];
            uint32_t row[R];
            bool live[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int64_t bundle = b_begin + static_cast<int64_t>(place_of(cur)) * R + r;
                live[r] = bundle < b_end;                // same in every lane
                row[r] = static_cast<uint32_t>(bundle * kLanes + lane);
#pragma unroll
                for (int t = 0; t < MQ; ++t) acc[r][t] = 0;
            }
            // the next chunk of this wavefront: one LDS atomic by the first lane
            int nxt = 0;
            if (lane == 0) nxt = static_cast<int>(atomicAdd(s.next, 1u));
            nxt = __builtin_amdgcn_readfirstlane(nxt);
            // lower the thresholds when enough new rows are out (one wavefront wins the job)
            const uint32_t mark = *s.mark;
            if (static_cast<uint32_t>(nxt) >= mark + (mark >> 3) && !first) {
                int won = 0;
                if (lane == 0) won = atomicCAS(s.mark, mark, static_cast<uint32_t>(nxt)) == mark ? 1 : 0;
                if (__builtin_amdgcn_readfirstlane(won)) {
                    for (int t = 0; t < a.m; ++t) {
                        const uint32_t edge = wave_boundary(s.hist + t * kHistBins, a.k, a.shift);
                        if (lane == 0) atomicMin(&s.thr[t], edge);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < MQ; ++t) thr[t] = s.thr[t < a.m ? t : 0];
            if (PREFETCH) {
                uint32_t x[R][BD][WC];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int b = 0; b < BD; ++b)
#pragma unroll
                        for (int w = 0; w < WC; ++w) x[r][b][w] = xn[r][b][w];
                if (nxt < chunks) {
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const int64_t bundle = b_begin + static_cast<int64_t>(place_of(nxt)) * R + r;
                        if (bundle < b_end) {
                            const uint32_t* xb = a.db + bundle * row_stride + lane;
#pragma unroll
                            for (int b = 0; b < BD; ++b)
#pragma unroll
                                for (int w = 0; w < WC; ++w) xn[r][b][w] = load_stream(xb + (b * WC + w) * kLanes);
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < MQ; ++t) {
                    if (t < a.m) {
                        uniform_ptr yq = (uniform_ptr)(a.q + static_cast<size_t>(t) * (BQ * WC));
                        uint32_t y[BQ][WC];
#pragma unroll
                        for (int b = 0; b < BQ; ++b)
#pragma unroll
                            for (int w = 0; w < WC; ++w) y[b][w] = yq[b * WC + w];
#pragma unroll
                        for (int r = 0; r < R; ++r)
                            if (live[r]) acc[r][t] = xor_popcount<BQ, BD, WC>(x[r], y);
                    }
                }
            } else {
                for (int c = 0; c < a.nchunks; ++c) {
                    uint32_t x[R][BD][WC];
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        if (!live[r]) continue;
                        const uint32_t* xb = a.db + (b_begin + static_cast<int64_t>(place_of(cur)) * R + r) * row_stride + lane;
#pragma unroll
                        for (int b = 0; b < BD; ++b)
#pragma unroll
                            for (int w = 0; w < WC; ++w) {
                                const int ww = c * WC + w;
                                x[r][b][w] = ww < a.W ? load_stream(xb + (b * a.W + ww) * kLanes) : 0u;
                            }
                    }
#pragma unroll
                    for (int t = 0; t < MQ; ++t) {
                        if (t < a.m) {
                            uniform_ptr yq = (uniform_ptr)(a.q + (static_cast<size_t>(t) * a.nchunks + c) * (BQ * WC));
                            uint32_t y[BQ][WC];
#pragma unroll
                            for (int b = 0; b < BQ; ++b)
#pragma unroll
                                for (int w = 0; w < WC; ++w) y[b][w] = yq[b * WC + w];
#pragma unroll
                            for (int r = 0; r < R; ++r)
                                if (live[r]) acc[r][t] += xor_popcount<BQ, BD, WC>(x[r], y);
                        }
                    }
                }
            }
            if (first) {                                 // count only; the rows wait in registers
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (!live[r]) continue;
                    row0[r] = row[r];
#pragma unroll
                    for (int t = 0; t < MQ; ++t) {
                        acc0[r][t] = acc[r][t];
                        if (t < a.m && row[r] < a.n) atomicAdd(&s.hist[t * kHistBins + (acc[r][t] >> a.shift)], 1u);
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (!live[r]) continue;
                    const bool valid = row[r] < a.n;
#pragma unroll
                    for (int t = 0; t < MQ; ++t) {
                        if (t < a.m)
                            append_lds(valid && acc[r][t] < thr[t], acc[r][t], row[r], s.buf + static_cast<size_t>(t) * a.cap,
                                       &s.cnt[t], static_cast<uint32_t>(a.cap), &s.ovf[t], s.hist + t * kHistBins, a.shift,
                                       &s.level[t], s.want);
                    }
                }
            }
            cur = nxt;
        }

        if (first) {
            // First thresholds: wavefront t finds the boundary of query t among the rows counted so
            // far, then every wavefront lists those of its held rows that pass (already counted).
            lds_barrier();
            if (wave < a.m) {
                const uint32_t edge = wave_boundary(s.hist + wave * kHistBins, a.k, a.shift);
                if (lane == 0) s.thr[wave] = edge;
            }
            lds_barrier();
#pragma unroll
            for (int t = 0; t < MQ; ++t) {
                if (t < a.m) {
                    thr[t] = s.thr[t];
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        append_lds(row0[r] < a.n && acc0[r][t] < thr[t], acc0[r][t], row0[r],
                                   s.buf + static_cast<size_t>(t) * a.cap, &s.cnt[t], static_cast<uint32_t>(a.cap),
                                   &s.ovf[t], nullptr, 0);
                }
            }
            first = false;
            continue;
        }

        // End of a round: every wavefront has run out of chunks, or a list asked for a compaction
        // (the wavefronts finish the chunk they are in and keep the one they have prefetched).
        // All queries at once: wavefront t finds the new boundary of query t, then the whole
        // workgroup compacts the lists (keys held in registers across the reset).  Only LDS is
        // exchanged, so the barriers leave the prefetched rows in flight.  At the end of the piece
        // lists short enough to be ranked as they are skip the compaction.
        if (cur >= chunks && lane == 0) atomicOr(s.done, 1u << wave);
        lds_barrier();
        const bool last = *s.done == (1u << kLocalWaves) - 1u;      // same in every thread
        if (last) {
            bool is_short = true;
            for (int t = 0; t < a.m; ++t) is_short = is_short && s.cnt[t] <= static_cast<uint32_t>(kRankAsIs);
            if (is_short) break;
        }
        if (wave < a.m) {
            const uint32_t edge = wave_boundary(s.hist + wave * kHistBins, a.k, a.shift);
            if (lane == 0 && edge < s.thr[wave]) s.thr[wave] = edge;
        }
        constexpr int kHeld = kLocalMaxCap / kLocalBlock;
        uint64_t held[MQ][kHeld];
#pragma unroll
        for (int t = 0; t < MQ; ++t) {
            const int have = t < a.m ? static_cast<int>(s.cnt[t] < static_cast<uint32_t>(a.cap) ? s.cnt[t] : a.cap) : 0;
#pragma unroll
            for (int u = 0; u < kHeld; ++u) {
                const int i = u * kLocalBlock + threadIdx.x;
                held[t][u] = i < have ? s.buf[static_cast<size_t>(t) * a.cap + i] : kPadKey;
            }
        }
        lds_barrier();
        if (threadIdx.x < kLocalMaxQueries) s.cnt[threadIdx.x] = 0;
        if (threadIdx.x == 0) {
            *s.mark = *s.next;
            *s.want = 0;
        }
        lds_barrier();
#pragma unroll
        for (int t = 0; t < MQ; ++t) {
            if (t < a.m) {
                thr[t] = s.thr[t];
#pragma unroll
                for (int u = 0; u < kHeld; ++u) {
                    if (u * kLocalBlock < a.cap) {
                        const uint32_t D = static_cast<uint32_t>(held[t][u] >> 32);
                        append_lds(held[t][u] != kPadKey && D < thr[t], D, static_cast<uint32_t>(held[t][u]),
                                   s.buf + static_cast<size_t>(t) * a.cap, &s.cnt[t], static_cast<uint32_t>(a.cap),
                                   &s.ovf[t], nullptr, 0);
                    }
                }
            }
        }
        lds_barrier();
        if (last) break;
        // A list that the boundary bin alone keeps more than a quarter full (rows of one tight cluster:
        // thousands of distances in one bin) is cut exactly: sorted, and only the keys up to the
        // K-th distance stay; the threshold becomes that distance + 1, finer than any bin edge.
        for (int t = 0; t < a.m; ++t) {
            const int have = static_cast<int>(s.cnt[t]);                  // same in every thread
            if (have <= a.cap / 4 || s.ovf[t] != 0) continue;
            cut_list_exactly((lds_u64*)(s.buf + static_cast<size_t>(t) * a.cap), have, a.k, (lds_u32*)&s.cnt[t],
                             (lds_u32*)&s.thr[t]);
        }
        // The next request comes a quarter of the list later, and always while the list still has
        // room for every row the wavefronts may add before they see it.  A list that even the exact
        // cut could not bring that low (ties at the K-th distance itself) asks no more; when it
        // fills up, it is marked for the exact re-selection at the end.
        if (threadIdx.x < static_cast<unsigned>(a.m)) {
            const uint32_t have = s.cnt[threadIdx.x];
            const uint32_t next = have + static_cast<uint32_t>(a.cap) / 4;
            s.level[threadIdx.x] = have >= safe_level ? 0xffffffffu : next < safe_level ? next : safe_level;
        }
        lds_barrier();
    }
    __syncthreads();

    // The piece's list leaves sorted and cut to its K best keys: the merge then needs only the
    // head of each list.  Short lists are ranked (every key counts the keys before it), long
    // ones (after an overflow, or with many ties in the boundary bin) take the LDS sort.
    const int64_t row_begin = b_begin * kLanes;
    const int64_t row_end = b_end * kLanes < a.n ? b_end * kLanes : a.n;
    for (int t = 0; t < a.m; ++t) {
        if (s.ovf[t] != 0) reselect_piece(a, s, t, row_begin, row_end);          // same value in every thread
        __syncthreads();
        const int have = static_cast<int>(s.cnt[t]);
        uint64_t* buf = s.buf + static_cast<size_t>(t) * a.cap;
        uint64_t* out = a.lists + (static_cast<size_t>(t) * a.groups + blockIdx.x) * a.list_stride;
        if (have <= kRankSortMax) {
            uint32_t* rank = s.hist + t * kHistBins;     // the histogram has done its work
            rank_keys(buf, have, rank);
            if (static_cast<int>(threadIdx.x) < have && rank[threadIdx.x] < static_cast<uint32_t>(a.k))
                out[rank[threadIdx.x]] = buf[threadIdx.x];
        } else {
            const int P = next_pow2(have);
            for (int i = have + threadIdx.x; i < P; i += kLocalBlock) buf[i] = kPadKey;
            __syncthreads();
            bitonic_sort_lds(buf, P);
            const int keep = have < a.k ? have : a.k;
            for (int i = threadIdx.x; i < keep; i += kLocalBlock) out[i] = buf[i];
        }
    }
}

template <int BQ, int BD, int WC, int R, bool PREFETCH, int MQ>
__global__ __launch_bounds__(kLocalBlock) void scan_local(const LocalArgs a)
{
    scan_local_body<BQ, BD, WC, R, PREFETCH, MQ>(a);
}

// One workgroup per query: merge of the pieces' lists, see the head of this file.
//
// List g of a query holds the min(k, rows of piece g) best keys of its piece in ascending
// order.  A list contributes about k / groups keys to the result, so only the first a.prefix
// keys of every list are read (one round trip, keys stay in registers): histogram of
// D >> shift2 over them, boundary bin, the keys at or below it sorted, K-th key.  If the last
// key read of some longer list is not beyond that K-th key, unread keys of that list could
// belong to the result: then (and when ties overfill the sort buffer) the whole lists are
// merged instead, slowly.
constexpr int kFinishHeld = 32;                          // prefix slots per thread, at most
constexpr int kFinishBatch = 8;

// Every piece but the last is full; a.len_full and a.len_last are min(k, rows of the piece).
__device__ __forceinline__ int list_length(const LocalArgs& a, int g)
{
    return g == a.groups - 1 ? a.len_last : a.len_full;
}

__device__ __forceinline__ void finish_collect(uint64_t key, uint32_t bin, int shift2, uint64_t* keys, uint32_t* fill)
{
    const bool pass = key != kPadKey && (static_cast<uint32_t>(key >> 32) >> shift2) <= bin;
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    const int leader = __ffsll(static_cast<long long>(mask)) - 1;
    uint32_t base = 0;
    if (lane_id() == leader) base = atomicAdd(fill, static_cast<uint32_t>(__popcll(mask)));
    base = __shfl(base, leader);
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
    if (pass) keys[base + rank] = key;
}

// Ascending sort of `have` distinct keys in LDS; returns where the sorted keys are (keys or
// keys + kSortCap / 2).  Up to kRankSortMax keys are ranked (rank[] is LDS scratch of that many
// words), more take the bitonic network.  The caller has synchronised after filling keys.
__device__ uint64_t* sort_keys(uint64_t* keys, int have, uint32_t* rank)
{
    if (have <= kRankSortMax) {
        uint64_t* sorted = keys + kSortCap / 2;
        rank_keys(keys, have, rank);
        if (static_cast<int>(threadIdx.x) < have) sorted[rank[threadIdx.x]] = keys[threadIdx.x];
        __syncthreads();
        return sorted;
    }
    const int P = next_pow2(have);
    for (int i = have + threadIdx.x; i < P; i += kLocalBlock) keys[i] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    return keys;
}

// Append a key to the sort buffer if it passes; one LDS atomic per wavefront.  Keys past the
// buffer are dropped (the counter still counts them).
__device__ __forceinline__ void collect_if(bool pass, uint64_t key, uint64_t* keys, uint32_t* fill)
{
    const uint64_t m = __ballot(pass);
    if (m == 0) return;
    const int leader = __ffsll(static_cast<long long>(m)) - 1;
    uint32_t base = 0;
    if (lane_id() == leader) base = atomicAdd(fill, static_cast<uint32_t>(__popcll(m)));
    base = __shfl(base, leader);
    const uint32_t r = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32),
                       __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u));
    if (pass && base + r < static_cast<uint32_t>(kSortCap)) keys[base + r] = key;
}

// Merge over the whole lists; leaves the K best keys sorted at the returned address.
__device__ uint64_t* merge_whole_lists(const LocalArgs& a, const uint64_t* lists, uint64_t* keys, uint32_t* hist,
                                       uint32_t* wave_sum, int* pick, uint32_t* fill)
{
    const int sh = 31 - __builtin_clz(static_cast<uint32_t>(next_pow2(a.k)));
    const int64_t nslots = static_cast<int64_t>(a.groups) << sh;
    const int64_t mask = (int64_t(1) << sh) - 1;
    __syncthreads();
    for (int i = threadIdx.x; i < kFinishBins; i += kLocalBlock) hist[i] = 0;
    if (threadIdx.x == 0) *fill = 0;
    __syncthreads();
    for (int64_t s0 = 0; s0 < nslots; s0 += static_cast<int64_t>(kFinishBatch) * kLocalBlock) {
        uint64_t k8[kFinishBatch];
#pragma unroll
        for (int u = 0; u < kFinishBatch; ++u) {
            const int64_t slot = s0 + static_cast<int64_t>(u) * kLocalBlock + threadIdx.x;
            const int g = static_cast<int>(slot >> sh);
            const int i = static_cast<int>(slot & mask);
            k8[u] = slot < nslots && i < list_length(a, g) ? lists[static_cast<size_t>(g) * a.list_stride + i] : kPadKey;
        }
#pragma unroll
        for (int u = 0; u < kFinishBatch; ++u)
            if (k8[u] != kPadKey) atomicAdd(&hist[static_cast<uint32_t>(k8[u] >> 32) >> a.shift2], 1u);
    }
    __syncthreads();
    int within;
    const uint32_t bin = static_cast<uint32_t>(boundary_of<kFinishBins / kLocalBlock>(hist, a.k, wave_sum, pick, &within));
    if (within <= kSortCap) {
        for (int64_t s0 = 0; s0 < nslots; s0 += static_cast<int64_t>(kFinishBatch) * kLocalBlock) {
            uint64_t k8[kFinishBatch];
#pragma unroll
            for (int u = 0; u < kFinishBatch; ++u) {
                const int64_t slot = s0 + static_cast<int64_t>(u) * kLocalBlock + threadIdx.x;
                const int g = static_cast<int>(slot >> sh);
                const int i = static_cast<int>(slot & mask);
                k8[u] = slot < nslots && i < list_length(a, g) ? lists[static_cast<size_t>(g) * a.list_stride + i] : kPadKey;
            }
#pragma unroll
            for (int u = 0; u < kFinishBatch; ++u) finish_collect(k8[u], bin, a.shift2, keys, fill);
        }
        __syncthreads();
        return sort_keys(keys, static_cast<int>(*fill), hist);
    }
    // massive ties at the boundary: every listed key in turn against the K-th best key so far
    uint64_t thr = kPadKey;
    for (int g = 0; g < a.groups; ++g) {
        const int c = list_length(a, g);
        const uint64_t* list = lists + static_cast<size_t>(g) * a.list_stride;
        for (int i0 = 0; i0 < c; i0 += kLocalBlock) {
            const int i = i0 + threadIdx.x;
            if (i < c) {
                const uint64_t key = list[i];
                if (key < thr) keys[atomicAdd(fill, 1u)] = key;
            }
            __syncthreads();
            const int have = static_cast<int>(*fill);
            if (have > kSortCap - kLocalBlock) {
                const int P = next_pow2(have);
                for (int j = have + threadIdx.x; j < P; j += kLocalBlock) keys[j] = kPadKey;
                __syncthreads();
                bitonic_sort_lds(keys, P);
                thr = keys[a.k - 1];                     // have > k here: k <= 1024 < have
                __syncthreads();
                if (threadIdx.x == 0) *fill = static_cast<uint32_t>(a.k);
            }
            __syncthreads();
        }
    }
    const int have = static_cast<int>(*fill);
    const int P = next_pow2(have);
    for (int i = have + threadIdx.x; i < P; i += kLocalBlock) keys[i] = kPadKey;
    __syncthreads();
    bitonic_sort_lds(keys, P);
    return keys;
}

__global__ __launch_bounds__(kLocalBlock) void local_finish(const LocalArgs a)
{
    __shared__ uint64_t keys[kSortCap];
    __shared__ uint32_t hist[kFinishBins];
    __shared__ uint32_t wave_sum[kLocalWaves];
    __shared__ int pick[2];
    __shared__ uint32_t fill, redo;
    __shared__ uint32_t longer[kLocalMaxGroups / 32];    // one bit per list that may hold more of the result than was read
    const int q = blockIdx.x;
    const uint64_t* lists = a.lists + static_cast<size_t>(q) * a.groups * a.list_stride;
    const int sh = 31 - __builtin_clz(static_cast<uint32_t>(a.prefix));
    const int nslots = a.groups << sh;                   // <= kFinishHeld * kLocalBlock (checked by the host)

    // every load is issued before anything waits: slots past the end read key 0 of list 0, and
    // are masked once the histogram is cleared
    const int rounds = (nslots + kLocalBlock - 1) / kLocalBlock;     // <= kFinishHeld
    uint64_t held[kFinishHeld];
#pragma unroll
    for (int u = 0; u < kFinishHeld; ++u) {
        if (u < rounds) {
            const int slot = u * kLocalBlock + static_cast<int>(threadIdx.x);
            const int g = slot >> sh, i = slot & (a.prefix - 1);
            const bool valid = slot < nslots && i < list_length(a, g);
            held[u] = lists[valid ? static_cast<size_t>(g) * a.list_stride + i : 0];
        }
    }
    for (int i = threadIdx.x; i < kFinishBins; i += kLocalBlock) hist[i] = 0;
    if (threadIdx.x == 0) { fill = 0; redo = 0; }
    if (threadIdx.x < kLocalMaxGroups / 32) longer[threadIdx.x] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kFinishHeld; ++u) {
        if (u < rounds) {
            const int slot = u * kLocalBlock + static_cast<int>(threadIdx.x);
            const int g = slot >> sh, i = slot & (a.prefix - 1);
            if (!(slot < nslots && i < list_length(a, g))) held[u] = kPadKey;
            if (held[u] != kPadKey) atomicAdd(&hist[static_cast<uint32_t>(held[u] >> 32) >> a.shift2], 1u);
        }
    }
    __syncthreads();
    int within;
    const uint32_t bin = static_cast<uint32_t>(boundary_of<kFinishBins / kLocalBlock>(hist, a.k, wave_sum, pick, &within));

    const uint64_t* best = nullptr;
    uint64_t bound = kPadKey;                            // K keys at or below it are known to exist
    if (within <= kSortCap) {
#pragma unroll
        for (int u = 0; u < kFinishHeld; ++u)
            if (u < rounds) finish_collect(held[u], bin, a.shift2, keys, &fill);
        __syncthreads();
        best = sort_keys(keys, static_cast<int>(fill), hist);
        // a longer list whose last key read is not beyond the K-th key may hold more of the result
        const uint64_t kth = best[a.k - 1];
        bound = kth;
#pragma unroll
        for (int u = 0; u < kFinishHeld; ++u) {
            if (u < rounds) {
                const int slot = u * kLocalBlock + static_cast<int>(threadIdx.x);
                const int g = slot >> sh, i = slot & (a.prefix - 1);
                if (i == a.prefix - 1 && held[u] < kth && list_length(a, g) > a.prefix) {
                    redo = 1u;
                    atomicOr(&longer[g >> 5], 1u << (g & 31));
                }
            }
        }
    } else if (threadIdx.x == 0) {
        redo = 1u;
    }
    __syncthreads();
    if (redo != 0) {
        // Some lists hold more of the result than their heads (the result sits in a few pieces: rows
        // ordered by cluster).  K keys at or below `bound` exist, so only keys up to it matter:
        // those among the heads, still in registers, and those in the rest of the marked lists,
        // which the wavefronts read list by list.  They are few; sorted, their first K are the result.
        best = nullptr;
        if (bound != kPadKey) {
            if (threadIdx.x == 0) fill = 0;
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kFinishHeld; ++u)
                if (u < rounds) collect_if(held[u] <= bound, held[u], keys, &fill);      // the pad key is above any bound
            const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
            for (int g = wave; g < a.groups; g += kLocalWaves) {
                if ((longer[g >> 5] >> (g & 31) & 1u) == 0) continue;                  // same in every lane
                const int len = list_length(a, g);
                for (int i0 = a.prefix; i0 < len; i0 += kLanes) {
                    const int i = i0 + lane;
                    const uint64_t key = i < len ? lists[static_cast<size_t>(g) * a.list_stride + i] : kPadKey;
                    collect_if(key <= bound, key, keys, &fill);
                }
            }
            __syncthreads();
            if (fill <= static_cast<uint32_t>(kSortCap)) best = sort_keys(keys, static_cast<int>(fill), hist);
        }
        if (best == nullptr) best = merge_whole_lists(a, lists, keys, hist, wave_sum, pick, &fill);
    }

    const int32_t full = a.d * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    for (int i = threadIdx.x; i < a.k; i += kLocalBlock) {
        const uint64_t key = best[i];
        a.idx[static_cast<size_t>(q) * a.k + i] = static_cast<int32_t>(key & 0xffffffffu);
        a.score[static_cast<size_t>(q) * a.k + i] = full - 2 * static_cast<int32_t>(key >> 32);
    }
}

// ---------------------------------------------------------------------------------------
size_t local_lds_bytes(int m, int cap)
{
    return static_cast<size_t>(m) * cap * sizeof(uint64_t) + static_cast<size_t>(m) * kHistBins * sizeof(uint32_t) +
           (4 * kLocalMaxQueries + 4) * sizeof(uint32_t);                 // counters, levels, next, mark, want, done
}

template <int BQ, int BD, int WC, int MQ>
static hipError_t launch_scan_local_w(const LocalArgs& a, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>(a.groups)), block(kLocalBlock);
    const size_t lds = local_lds_bytes(a.m, a.cap);
#define XBQ_LAUNCH_SCAN_LOCAL(R, PREFETCH)                                                                      \
    do {                                                                                                        \
        if (lds > 64 * 1024) {                           /* more than the default limit has to be asked for */   \
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&scan_local<BQ, BD, WC, R, PREFETCH, MQ>), \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)); \
            if (e != hipSuccess) return e;                                                                      \
        }                                                                                                       \
        hipLaunchKernelGGL((scan_local<BQ, BD, WC, R, PREFETCH, MQ>), grid, block, lds, s, a);                   \
    } while (0)
    // whole row in registers (one chunk, exactly W words): next step's rows are prefetched, two
    // bundles per wavefront and step while both sets fit the register file
    if (a.nchunks == 1 && a.W == WC) {
        if constexpr (BD * WC <= 16)      XBQ_LAUNCH_SCAN_LOCAL(2, true);
        else if constexpr (BD * WC <= 24) XBQ_LAUNCH_SCAN_LOCAL(1, true);
        else                              XBQ_LAUNCH_SCAN_LOCAL(1, false);
    } else {
        XBQ_LAUNCH_SCAN_LOCAL(1, false);
    }
    return hipGetLastError();
#undef XBQ_LAUNCH_SCAN_LOCAL
}

template <int BQ, int BD>
static hipError_t launch_scan_local_b(const LocalArgs& a, hipStream_t s)
{
    switch (a.wc) {
    case 1: return a.m == 1 ? launch_scan_local_w<BQ, BD, 1, 1>(a, s) : launch_scan_local_w<BQ, BD, 1, kLocalMaxQueries>(a, s);
    case 2: return a.m == 1 ? launch_scan_local_w<BQ, BD, 2, 1>(a, s) : launch_scan_local_w<BQ, BD, 2, kLocalMaxQueries>(a, s);
    case 3: return a.m == 1 ? launch_scan_local_w<BQ, BD, 3, 1>(a, s) : launch_scan_local_w<BQ, BD, 3, kLocalMaxQueries>(a, s);
    case 4: return a.m == 1 ? launch_scan_local_w<BQ, BD, 4, 1>(a, s) : launch_scan_local_w<BQ, BD, 4, kLocalMaxQueries>(a, s);
    case 5: return a.m == 1 ? launch_scan_local_w<BQ, BD, 5, 1>(a, s) : launch_scan_local_w<BQ, BD, 5, kLocalMaxQueries>(a, s);
    case 6: return a.m == 1 ? launch_scan_local_w<BQ, BD, 6, 1>(a, s) : launch_scan_local_w<BQ, BD, 6, kLocalMaxQueries>(a, s);
    case 7: return a.m == 1 ? launch_scan_local_w<BQ, BD, 7, 1>(a, s) : launch_scan_local_w<BQ, BD, 7, kLocalMaxQueries>(a, s);
    case 8: return a.m == 1 ? launch_scan_local_w<BQ, BD, 8, 1>(a, s) : launch_scan_local_w<BQ, BD, 8, kLocalMaxQueries>(a, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_scan_local(const LocalArgs& a, hipStream_t s)
{
    if (a.m < 1 || a.m > kLocalMaxQueries || a.n < 1 || a.wc < 1 || a.wc > 8 || a.nchunks < 1 ||
        a.nchunks * a.wc < a.W) return hipErrorInvalidValue;
    if (a.k < 1 || a.cap < 8 * a.k || a.cap < 4 * kLocalBlock || a.cap > kLocalMaxCap || (a.cap & (a.cap - 1)) != 0)
        return hipErrorInvalidValue;
    if (local_lds_bytes(a.m, a.cap) > kLocalMaxLds) return hipErrorInvalidValue;
    const int64_t nbundles = (a.n + kLanes - 1) / kLanes;
    if (a.groups > kLocalMaxGroups || a.list_stride < a.k) return hipErrorInvalidValue;
    if (a.groups < 1 || a.bundles_per_group < 1 || a.groups * a.bundles_per_group < nbundles ||
        (a.groups - 1) * a.bundles_per_group >= nbundles) return hipErrorInvalidValue;
    const int64_t dmax = static_cast<int64_t>(a.d) * ((1 << a.q_bits) - 1) * ((1 << a.db_bits) - 1);
    if ((dmax >> a.shift) >= kHistBins || (dmax >> a.shift2) >= kFinishBins) return hipErrorInvalidValue;
    switch (a.q_bits * 10 + a.db_bits) {
    case 11: return launch_scan_local_b<1, 1>(a, s);
    case 22: return launch_scan_local_b<2, 2>(a, s);
    case 33: return launch_scan_local_b<3, 3>(a, s);
    case 44: return launch_scan_local_b<4, 4>(a, s);
    case 21: return launch_scan_local_b<2, 1>(a, s);
    case 32: return launch_scan_local_b<3, 2>(a, s);
    case 43: return launch_scan_local_b<4, 3>(a, s);
    default: return hipErrorInvalidValue;
    }
}

// After launch_scan_local with the same arguments on the same stream.
hipError_t launch_local_finish(const LocalArgs& a, hipStream_t s)
{
    if (a.m < 1 || a.m > kLocalMaxQueries || a.groups < 1 || a.groups > kLocalMaxGroups || a.k < 1 || a.k > kSortCap / 4)
        return hipErrorInvalidValue;
    if (a.prefix < 1 || (a.prefix & (a.prefix - 1)) != 0 || a.list_stride < a.k ||
        static_cast<int64_t>(a.groups) * a.prefix > static_cast<int64_t>(kFinishHeld) * kLocalBlock)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(local_finish, dim3(static_cast<unsigned>(a.m)), dim3(kLocalBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace xbq
