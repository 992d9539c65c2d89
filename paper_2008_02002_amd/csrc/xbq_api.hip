// C ABI of libxbq.so: argument validation, the search schedule, workspace carving and
// kernel launches.  No device memory is allocated here and nothing synchronises.
//
// Search schedule.  The database rows are split into groups of growing size.  The first,
// small group is scored densely and its exact top-K gives every query a threshold (the
// distance of its K-th best row).  Each later group is scanned with that threshold: only
// rows strictly closer than the K-th best so far can enter the top-K (a row with an equal
// distance has a higher row number than everything already seen, so it loses the tie),
// and for rows in random order about K * (group size / rows seen) of them do.  After each
// group one small kernel per query merges the survivors into the top-K and tightens the
// threshold.  A query whose survivor list overflows its buffer is rescanned exactly inside
// that kernel, so the result never depends on the data order.

#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "xbq_internal.h"

namespace {

using namespace xbq;

thread_local int g_last_hip_error = 0;

// The schedule knobs of one call.  Every entry point takes a snapshot when it starts (of the
// caller's xbq_options, or of the process-wide defaults behind xbq_set_option) and passes it
// down: nothing below reads shared mutable state.
struct Options {
    double growth = 4.0;
    int first = 1024;
    int qsplit = 0;
    int selector = 0;                // 0 automatic, 1 threshold filter, 2 histogram (distances stored), 3 local selection
    int hist_max_queries = 16;       // automatic choice: few-query selection up to this many queries
    int kernel = 0;                  // 0 XOR + population count; cross-checks: 1 packed 4-bit dots, 2 int8 MFMA
    double refine_growth = 1.5;      // growth bound of the bounded candidate search
    int kselect_lists_min = 128;     // xbq_k_select: batches of at least this many queries start from bounded lists
    int local_groups = 256;          // local selection: most pieces (workgroups) the rows are split into
    int row_order = 0;               // threshold schedule: 0 = row groups spread over the database, 1 = consecutive rows
};

std::mutex g_opt_mutex;
Options g_opt;                       // process-wide defaults, guarded by g_opt_mutex

Options default_options()
{
    std::lock_guard<std::mutex> lock(g_opt_mutex);
    return g_opt;
}

// Range check of one knob; shared by xbq_set_option and the xbq_options of the _ex calls.
bool set_knob(Options& o, const char* name, double value)
{
    if (!std::strcmp(name, "growth")) { if (!(value >= 1.25 && value <= 64.0)) return false; o.growth = value; return true; }
    if (!std::strcmp(name, "first")) { if (!(value >= 64 && value <= kSortCap)) return false; o.first = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "kernel")) { if (!(value == 0 || value == 1 || value == 2)) return false; o.kernel = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "selector")) { if (!(value == 0 || value == 1 || value == 2 || value == 3)) return false; o.selector = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "hist_max_queries")) { if (!(value >= 0 && value <= (1 << 20))) return false; o.hist_max_queries = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "refine_growth")) { if (!(value >= 1.25 && value <= 64.0)) return false; o.refine_growth = value; return true; }
    if (!std::strcmp(name, "kselect_lists_min")) { if (!(value >= 0 && value <= (1 << 20))) return false; o.kselect_lists_min = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "qsplit")) { if (!(value >= 0 && value <= 65536)) return false; o.qsplit = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "row_order")) { if (!(value == 0 || value == 1)) return false; o.row_order = static_cast<int>(value); return true; }
    if (!std::strcmp(name, "local_groups")) { if (!(value >= 1 && value <= kLocalMaxGroups)) return false; o.local_groups = static_cast<int>(value); return true; }
    return false;
}

// The options of an _ex call: nullptr = the process-wide defaults.  False if a field is out of range.
bool options_from(const xbq_options* in, Options& o)
{
    if (in == nullptr) { o = default_options(); return true; }
    if (in->struct_bytes != sizeof(xbq_options)) return false;
    o = Options();
    return set_knob(o, "growth", in->growth) && set_knob(o, "first", in->first) && set_knob(o, "qsplit", in->qsplit) &&
           set_knob(o, "selector", in->selector) && set_knob(o, "hist_max_queries", in->hist_max_queries) &&
           set_knob(o, "kernel", in->kernel) && set_knob(o, "refine_growth", in->refine_growth) &&
           set_knob(o, "kselect_lists_min", in->kselect_lists_min) && set_knob(o, "local_groups", in->local_groups) &&
           set_knob(o, "row_order", in->row_order);
}

// Scan timing record of xbq_trace_*: one per calling thread.
struct Trace {
    bool on = false;
    std::vector<hipEvent_t> ev;      // pairs: start, stop
    int used = 0;                    // events used
    double pairs = 0;
};
thread_local Trace g_trace;
constexpr int kTraceMaxLaunches = 4096;

// Scratch of xbq_search_static: the workspace a caller of xbq_search would pass, held by the
// library instead.  Each device that loads the library holds its own copy of the array at its
// own address until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress; the address kernels use is looked up once per device (scratch_address).
static __device__ __align__(256) unsigned char scratch[XBQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int fail_hip(hipError_t e)
{
    g_last_hip_error = static_cast<int>(e);
    return XBQ_EHIP;
}

// Device address of `scratch` on the current device; looked up on the first call per device.
hipError_t scratch_address(char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr || reinterpret_cast<uintptr_t>(p) % 256) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char*>(g_scratch_ptr[dev]);
    return hipSuccess;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

bool valid_shape(int d, int bits) { return d >= 1 && d <= XBQ_MAX_DIM && bits >= 1 && bits <= XBQ_MAX_BITS; }

constexpr int64_t kQueryBatch = 16384;

struct Plan {
    int W = 0, wc = 0, nchunks = 0;      // wc == 0: register-resident scan
    int64_t bundle_mul = 1;              // order of the row groups of the threshold schedule, see spread_bundle()
    int first = 0;                       // rows of the dense group
    int cap = 0;                         // candidate slots per query
    int64_t batch = 0;                   // queries per batch
    int keep_max = 0;                    // keys kept per query (k, or the candidate bound when refining)
    size_t off_len = 0;
    size_t off_thr = 0, off_cnt = 0, off_topk = 0, off_cand = 0, off_dense = 0, off_q = 0;
    bool dot = false;                    // cross-check scan: nibble copies of database and queries
    size_t off_dbn = 0, off_qn = 0, off_qsum = 0;
    bool mfma = false;                   // cross-check scan: int8 copies of database and queries
    size_t off_dbb = 0, off_qb = 0;
    // histogram selection (aliases the regions above: one call runs one of the two paths)
    bool hist = false;
    int hist_wc = 0, hist_nchunks = 0, hist_shift = 0, hist_cand_cap = 0;
    size_t hoff_q = 0, hoff_zero = 0, hoff_dist = 0, hoff_cand = 0;
    size_t zero_words = 0;               // hist + cand_cnt, cleared in one go
    // local selection (few queries, nothing stored; aliases the regions above as well)
    bool local = false;
    int local_cap = 0, local_mq = 0, local_groups = 0, local_shift2 = 0, local_stride = 0, local_prefix = 0;
    int64_t local_bpg = 0;               // bundles per piece
    size_t loff_q = 0, loff_lists = 0;
    size_t total = 0;
};

constexpr int64_t kHistMaxDistBytes = int64_t(1) << 30;   // stored distances of one pass
constexpr int kLocalMaxK = 256;      // local selection keeps lists of 8 k keys per query in LDS

constexpr int kRefineKeep = 2048;    // candidate bound of the refine path
constexpr int kRefineCap = 2048;     // survivor list of the refine path (keep + cap <= kSortCap)

// keep_dist: the caller reads the stored distances of the histogram selection afterwards
// (xbq_k_select with few queries), so the few-query path must be the one that stores them.
Plan make_plan(const Options& o, int64_t n, int64_t m, int d, int bits, int k, bool refine = false,
               bool keep_dist = false)
{
    Plan p;
    p.W = words32(d);
    if (!scan_is_resident(p.W)) {
        p.wc = scan_chunk_words(p.W);
        p.nchunks = (p.W + p.wc - 1) / p.wc;
    }
    const int kpad = next_pow2(k);
    int first = o.first > 4 * kpad ? o.first : 4 * kpad;
    if (first > kSortCap) first = kSortCap;
    first = first / kLanes * kLanes;
    p.first = static_cast<int>(n < first ? n : first);
    p.cap = refine ? kRefineCap : (3 * kpad > 2048 ? 3 * kpad : 2048);
    p.keep_max = refine ? kRefineKeep : k;
    const int64_t max_batch = refine ? kQueryBatch / 2 : kQueryBatch;
    p.batch = m < max_batch ? m : max_batch;
    const size_t b = static_cast<size_t>(p.batch);
    size_t off = 0;
    p.off_thr = off;   off = align_up(off + b * sizeof(uint32_t), 256);
    p.off_cnt = off;   off = align_up(off + b * sizeof(uint32_t), 256);
    p.off_len = off;   off = align_up(off + b * sizeof(uint32_t), 256);
    p.off_topk = off;  off = align_up(off + b * p.keep_max * sizeof(uint64_t), 256);
    p.off_cand = off;  off = align_up(off + b * p.cap * sizeof(uint64_t), 256);
    p.off_dense = off; off = align_up(off + b * static_cast<size_t>(p.first) * sizeof(uint32_t), 256);
    p.off_q = off;
    if (p.wc) off = align_up(off + b * p.nchunks * bits * p.wc * sizeof(uint32_t), 256);
    if (o.kernel == 1 && p.wc == 0) {
        p.dot = true;
        const size_t wd = 4u * p.W;
        p.off_qn = off;   off = align_up(off + b * wd * sizeof(uint32_t), 256);
        p.off_qsum = off; off = align_up(off + b * sizeof(int32_t), 256);
        p.off_dbn = off;  off = align_up(off + static_cast<size_t>((n + kLanes - 1) / kLanes) * kLanes * wd * sizeof(uint32_t), 256);
    }
    if (o.kernel == 2 && p.wc == 0) {
        p.mfma = true;
        const size_t row_bytes = 32u * p.W;
        p.off_qb = off;  off = align_up(off + (b + 31) / 32 * 32 * row_bytes, 256);
        p.off_dbb = off; off = align_up(off + static_cast<size_t>((n + kLanes - 1) / kLanes) * kLanes * row_bytes, 256);
    }
    p.total = off;

    // Row groups spread over the database (the cross-check scans keep consecutive rows): a
    // multiplier coprime to the number of full bundles, near its golden section.
    if (o.row_order == 0 && !p.dot && !p.mfma) {
        const int64_t full = n / kLanes;
        for (int64_t mul = static_cast<int64_t>(static_cast<double>(full) * 0.6180339887); mul > 1 && mul < full; ++mul) {
            int64_t x = mul, y = full;
            while (y != 0) { const int64_t t = x % y; x = y; y = t; }
            if (x == 1) { p.bundle_mul = mul; break; }
        }
    }

    // histogram selection: eligible for plain top-K when the stored distances stay moderate
    // the threshold schedule pays per query for sorting O(k) keys in every row group, the histogram
    // path does not: its range grows with k (measured on C2: even at 40 queries for k = 100, beyond
    // 64 for k = 1000)
    const int64_t hist_limit = static_cast<int64_t>(o.hist_max_queries) * (k > 512 ? 3 : k > 128 ? 2 : 1);
    const bool few = o.selector == 0 && m <= hist_limit;
    const int64_t dmax = static_cast<int64_t>(d) * ((1 << bits) - 1) * ((1 << bits) - 1);
    // local selection: the default for few queries; its lists live in LDS, which bounds k
    // automatic: one pass of it (up to kLocalMaxQueries queries); more queries are served faster by the
    // histogram selection over stored distances, which scores eight queries per pass, unless the
    // database is so long that writing and re-reading 8 bytes per (query, row) costs more than
    // streaming short codes once more per four queries (measured at d = 96 and 128, 4 bits, 8 and 16
    // queries: even at 5 M rows, 5 to 15 % for local passes from 7 M rows on)
    constexpr int64_t kLocalPassesFromRows = 6'000'000;
    const bool short_codes = p.wc == 0;
    const bool want_local = (o.selector == 3 || (few && !keep_dist && (m <= kLocalMaxQueries ||
                             (n >= kLocalPassesFromRows && short_codes)))) && k <= kLocalMaxK;
    if (!refine && !p.dot && !p.mfma && want_local && m <= p.batch) {
        p.local = true;
        // Lists of 4096 keys: a list asks for a compaction while it still has room for every row in
        // flight (2048), so bursts of passing rows (rows ordered towards the query, cluster after
        // cluster) lose nothing.  Four queries take 144 KB of the 160 KB of LDS.
        p.local_cap = 4096;
        p.local_mq = kLocalMaxQueries;
        while (p.local_mq > 1 && local_lds_bytes(p.local_mq, p.local_cap) > kLocalMaxLds) --p.local_mq;
        if (m < p.local_mq) p.local_mq = static_cast<int>(m);
        const int64_t nbundles = (n + kLanes - 1) / kLanes;
        int64_t bpg = (nbundles + o.local_groups - 1) / o.local_groups;
        // Multiples of 16 bundles leave a few of 256 pieces unused (C5: 251, C2: 245).  Measured on
        // C5: 224 to 254 pieces take the same time (the HBM stream is the limit, not the compute
        // units), 255 and 256 take 5 % longer.
        bpg = (bpg + 15) / 16 * 16;
        p.local_bpg = bpg;
        p.local_groups = static_cast<int>((nbundles + bpg - 1) / bpg);
        p.hist_wc = p.wc ? p.wc : p.W;
        p.hist_nchunks = p.wc ? p.nchunks : 1;
        while ((dmax >> p.hist_shift) >= kHistBins) ++p.hist_shift;
        while ((dmax >> p.local_shift2) >= 4096) ++p.local_shift2;
        size_t h = 0;
        p.loff_q = h;
        if (p.wc) h = align_up(h + b * p.nchunks * bits * p.wc * sizeof(uint32_t), 256);
        p.local_stride = (k + 15) / 16 * 16;             // lists start on 128-byte boundaries
        // A list contributes about s = k / groups keys to the result, Poisson-like: read 4 s + 4 keys
        // of each, rounded up to a power of two and at least 8, so that a list holding that many
        // of the k best is a one-in-a-million event per list (s = 0.4, 8 keys: 1e-8; s = 2, 16
        // keys: 1e-10; with 4 keys at s = 0.4 every fourth query found one and merged whole lists).
        // The merge proves afterwards that no list needed more, and reads whole lists if one did.
        p.local_prefix = next_pow2((4 * k + p.local_groups - 1) / p.local_groups + 4);
        if (p.local_prefix < 8) p.local_prefix = 8;
        if (p.local_prefix > next_pow2(k) && next_pow2(k) >= 16) p.local_prefix = next_pow2(k);
        p.loff_lists = h;  h = align_up(h + static_cast<size_t>(p.local_mq) * p.local_groups * p.local_stride * sizeof(uint64_t), 256);
        if (h > p.total) p.total = h;
        return p;
    }
    const bool want = o.selector == 2 || (o.selector == 3 && k > kLocalMaxK) || few;
    const int hq = static_cast<int>(m < kHistMaxQueries ? m : kHistMaxQueries);
    if (!refine && !p.dot && !p.mfma && want && m <= p.batch && n * int64_t(4) * hq <= kHistMaxDistBytes) {
        p.hist = true;
        p.hist_wc = p.wc ? p.wc : p.W;
        p.hist_nchunks = p.wc ? p.nchunks : 1;
        while ((dmax >> p.hist_shift) >= kHistBins) ++p.hist_shift;
        size_t h = 0;
        p.hoff_q = h;
        if (p.wc) h = align_up(h + b * p.nchunks * bits * p.wc * sizeof(uint32_t), 256);
        p.hoff_zero = h;
        p.zero_words = static_cast<size_t>(hq) * (kHistBins + 1);
        h = align_up(h + p.zero_words * sizeof(uint32_t), 256);
        p.hist_cand_cap = n >= kHistCandCap ? kHistCandCap : next_pow2(static_cast<int>(n) > kSortCap ? static_cast<int>(n) : kSortCap);
        p.hoff_cand = h;  h = align_up(h + static_cast<size_t>(hq) * p.hist_cand_cap * sizeof(uint64_t), 256);
        p.hoff_dist = h;  h = align_up(h + static_cast<size_t>(hq) * n * sizeof(uint32_t), 256);
        if (h > p.total) p.total = h;
    }
    return p;
}

bool valid_search_sizes(int64_t n, int64_t m, int d, int bits, int k)
{
    if (!valid_shape(d, bits)) return false;
    if (n < 0 || m < 0 || n >= (int64_t(1) << 31) || m >= (int64_t(1) << 31)) return false;
    if (n > 0 && (k < 1 || k > XBQ_MAX_K || k > n)) return false;
    if (n == 0 && k < 1) return false;
    return true;
}

// Queries per workgroup for a group of `bundles` bundles.
int choose_qsplit(const Options& o, int64_t bundles, int rows_per_lane, int m, int tile)
{
    if (o.qsplit > 0) return (o.qsplit + tile - 1) / tile * tile;
    const int64_t waves = (bundles + rows_per_lane - 1) / rows_per_lane;
    int64_t ranges = (32768 + waves - 1) / waves;            // aim for >= 32k wavefronts
    const int64_t min_ranges = (m + 127) / 128;               // at most 128 queries per workgroup
    if (ranges < min_ranges) ranges = min_ranges;
    int qs = static_cast<int>((m + ranges - 1) / ranges);
    if (qs < 8) qs = 8;                                       // measured: 8 beats 16 for 17..64 queries, no loss above
    qs = (qs + tile - 1) / tile * tile;
    return qs;
}

hipError_t traced_scan(const ScanArgs& a, bool dense, hipStream_t s)
{
    const bool rec = g_trace.on && g_trace.used + 2 <= static_cast<int>(g_trace.ev.size());
    if (rec) {
        hipError_t e = hipEventRecord(g_trace.ev[g_trace.used], s);
        if (e != hipSuccess) return e;
    }
    hipError_t e = launch_scan(a, dense, s);
    if (e != hipSuccess) return e;
    if (rec) {
        e = hipEventRecord(g_trace.ev[g_trace.used + 1], s);
        if (e != hipSuccess) return e;
        g_trace.used += 2;
        if (a.run_flag == nullptr) g_trace.pairs += static_cast<double>(a.row_end - a.row_begin) * a.m;   // a flagged launch may do nothing
    }
    return hipSuccess;
}

hipError_t traced_scan_dot(const DotArgs& a, bool dense, hipStream_t s)
{
    const bool rec = g_trace.on && g_trace.used + 2 <= static_cast<int>(g_trace.ev.size());
    hipError_t e;
    if (rec && (e = hipEventRecord(g_trace.ev[g_trace.used], s)) != hipSuccess) return e;
    e = launch_scan_dot(a, dense, s);
    if (e != hipSuccess) return e;
    if (rec) {
        if ((e = hipEventRecord(g_trace.ev[g_trace.used + 1], s)) != hipSuccess) return e;
        g_trace.used += 2;
        g_trace.pairs += static_cast<double>(a.row_end - a.row_begin) * a.m;
    }
    return hipSuccess;
}

hipError_t traced_scan_mfma(const MfmaArgs& a, bool dense, hipStream_t s)
{
    const bool rec = g_trace.on && g_trace.used + 2 <= static_cast<int>(g_trace.ev.size());
    hipError_t e;
    if (rec && (e = hipEventRecord(g_trace.ev[g_trace.used], s)) != hipSuccess) return e;
    e = launch_scan_mfma(a, dense, s);
    if (e != hipSuccess) return e;
    if (rec) {
        if ((e = hipEventRecord(g_trace.ev[g_trace.used + 1], s)) != hipSuccess) return e;
        g_trace.used += 2;
        g_trace.pairs += static_cast<double>(a.row_end - a.row_begin) * a.m;
    }
    return hipSuccess;
}

// What one search call has to do; extra < 0 is the plain exact top-K, extra >= 0 the
// candidate search of Algorithm 1 followed by the fp32 refine.
struct SearchJob {
    const uint32_t* db_codes; int64_t n; int db_bits;
    const uint32_t* q_codes;  int64_t m; int q_bits;
    int d, k, extra;
    int32_t* idx;
    int32_t* score;            // plain mode
    const float* X_db;         // refine mode
    const float* X_q;
    float* similarity;
    int32_t* candidates;
    bool lists_only = false;   // refine mode: stop after the candidate lists are built
};

// Histogram selection: queries in passes of kHistMaxQueries, three launches per pass.
int run_hist_search(const SearchJob& job, const Plan& p, char* ws, hipStream_t s)
{
    const int64_t n = job.n, m = job.m;
    const uint32_t* q_all = job.q_codes;
    if (p.wc) {                                          // long codes: chunk-major padded query copy
        uint32_t* qc = reinterpret_cast<uint32_t*>(ws + p.hoff_q);
        for (int64_t qb = 0; qb < m; qb += p.batch) {    // p.batch >= m here (m is small)
            const int mb = static_cast<int>(m - qb < p.batch ? m - qb : p.batch);
            const hipError_t e = launch_repack_queries(job.q_codes + qb * (static_cast<int64_t>(job.q_bits) * p.W), mb,
                                                       job.q_bits, p.W, p.wc, p.nchunks,
                                                       qc + qb * (static_cast<int64_t>(p.nchunks) * job.q_bits * p.wc), s);
            if (e != hipSuccess) return fail_hip(e);
        }
        q_all = qc;
    }
    const int64_t q_stride = static_cast<int64_t>(p.hist_nchunks) * job.q_bits * p.hist_wc;
    uint32_t* zero = reinterpret_cast<uint32_t*>(ws + p.hoff_zero);
    for (int64_t qb = 0; qb < m; qb += kHistMaxQueries) {
        const int mb = static_cast<int>(m - qb < kHistMaxQueries ? m - qb : kHistMaxQueries);
        hipError_t e = launch_clear(zero, static_cast<int64_t>(p.zero_words), s);
        if (e != hipSuccess) return fail_hip(e);
        HistArgs ha{};
        ha.db = job.db_codes;
        ha.n = n;
        ha.q = q_all + qb * q_stride;
        ha.m = mb;
        ha.q_bits = job.q_bits;
        ha.db_bits = job.db_bits;
        ha.W = p.W;
        ha.wc = p.hist_wc;
        ha.nchunks = p.hist_nchunks;
        ha.dist = reinterpret_cast<uint32_t*>(ws + p.hoff_dist);
        ha.hist = zero;
        ha.shift = p.hist_shift;
        const bool rec = g_trace.on && g_trace.used + 2 <= static_cast<int>(g_trace.ev.size());
        if (rec && (e = hipEventRecord(g_trace.ev[g_trace.used], s)) != hipSuccess) return fail_hip(e);
        e = launch_scan_hist(ha, s);
        if (e != hipSuccess) return fail_hip(e);
        if (rec) {
            if ((e = hipEventRecord(g_trace.ev[g_trace.used + 1], s)) != hipSuccess) return fail_hip(e);
            g_trace.used += 2;
            g_trace.pairs += static_cast<double>(n) * mb;
        }
        CollectArgs ca{};
        ca.dist = ha.dist;
        ca.hist = zero;
        ca.n = n;
        ca.m = mb;
        ca.k = job.k;
        ca.d = job.d;
        ca.q_bits = job.q_bits;
        ca.db_bits = job.db_bits;
        ca.shift = p.hist_shift;
        ca.rows_per_block = 4 * 16 * kBlock;          // 16384 rows per workgroup: four rounds of loads
        ca.blocks_per_query = static_cast<int>((n + ca.rows_per_block - 1) / ca.rows_per_block);
        ca.cand = reinterpret_cast<uint64_t*>(ws + p.hoff_cand);
        ca.cand_cap = p.hist_cand_cap;
        ca.cand_cnt = zero + static_cast<size_t>(kHistMaxQueries < m ? kHistMaxQueries : m) * kHistBins;
        ca.idx = job.idx + qb * job.k;
        ca.score = job.score + qb * job.k;
        e = launch_hist_collect(ca, s);
        if (e != hipSuccess) return fail_hip(e);
    }
    return XBQ_OK;
}

// Local selection: queries in passes of at most p.local_mq, two launches per pass, nothing cleared.
int run_local_search(const SearchJob& job, const Plan& p, char* ws, hipStream_t s)
{
    const int64_t m = job.m;
    const uint32_t* q_all = job.q_codes;
    if (p.wc) {                                          // long codes: chunk-major padded query copy
        uint32_t* qc = reinterpret_cast<uint32_t*>(ws + p.loff_q);
        const hipError_t e = launch_repack_queries(job.q_codes, static_cast<int>(m), job.q_bits, p.W, p.wc, p.nchunks, qc, s);
        if (e != hipSuccess) return fail_hip(e);
        q_all = qc;
    }
    const int64_t q_stride = static_cast<int64_t>(p.hist_nchunks) * job.q_bits * p.hist_wc;
    // passes of nearly equal size (five queries: 3 + 2, not 4 + 1: a pass of one query costs as
    // much HBM time as one of two)
    const int64_t passes = (m + p.local_mq - 1) / p.local_mq;
    const int64_t per_pass = passes > 0 ? (m + passes - 1) / passes : 1;
    for (int64_t qb = 0; qb < m; qb += per_pass) {
        LocalArgs la{};
        la.db = job.db_codes;
        la.n = job.n;
        la.q = q_all + qb * q_stride;
        la.m = static_cast<int>(m - qb < per_pass ? m - qb : per_pass);
        la.q_bits = job.q_bits;
        la.db_bits = job.db_bits;
        la.W = p.W;
        la.wc = p.hist_wc;
        la.nchunks = p.hist_nchunks;
        la.k = job.k;
        la.d = job.d;
        la.shift = p.hist_shift;
        la.shift2 = p.local_shift2;
        la.cap = p.local_cap;
        la.groups = p.local_groups;
        la.bundles_per_group = p.local_bpg;
        la.lists = reinterpret_cast<uint64_t*>(ws + p.loff_lists);
        la.list_stride = p.local_stride;
        la.prefix = p.local_prefix;
        {
            const int64_t piece = p.local_bpg * kLanes;
            const int64_t last = job.n - (p.local_groups - 1) * piece;
            la.len_full = static_cast<int>(piece < job.k ? piece : job.k);
            la.len_last = static_cast<int>(last < job.k ? last : job.k);
        }
        la.idx = job.idx + qb * job.k;
        la.score = job.score + qb * job.k;
        const bool rec = g_trace.on && g_trace.used + 2 <= static_cast<int>(g_trace.ev.size());
        hipError_t e;
        if (rec && (e = hipEventRecord(g_trace.ev[g_trace.used], s)) != hipSuccess) return fail_hip(e);
        e = launch_scan_local(la, s);
        if (e != hipSuccess) return fail_hip(e);
        if (rec) {
            if ((e = hipEventRecord(g_trace.ev[g_trace.used + 1], s)) != hipSuccess) return fail_hip(e);
            g_trace.used += 2;
            g_trace.pairs += static_cast<double>(job.n) * la.m;
        }
        e = launch_local_finish(la, s);
        if (e != hipSuccess) return fail_hip(e);
    }
    return XBQ_OK;
}

int run_search(const Options& o, const SearchJob& job, const Plan& p, char* ws, hipStream_t s)
{
    const uint32_t* db_codes = job.db_codes;
    const uint32_t* q_codes = job.q_codes;
    const int64_t n = job.n, m = job.m;
    const int db_bits = job.db_bits, q_bits = job.q_bits, d = job.d, k = job.k;
    const bool refine = job.extra >= 0;
    const int rpl_max = (p.wc == 0 && db_bits * p.W <= 16) ? 2 : 1;
    const int tile = p.wc ? kTileQ : 1;

    if (p.local && !refine) return run_local_search(job, p, ws, s);
    if (p.hist && !refine) return run_hist_search(job, p, ws, s);
    if (p.dot) {
        const hipError_t e = launch_nibbles_db(db_codes, n, d, db_bits, reinterpret_cast<uint32_t*>(ws + p.off_dbn), s);
        if (e != hipSuccess) return fail_hip(e);
    }
    if (p.mfma) {
        const hipError_t e = launch_bytes_db(db_codes, n, d, db_bits, reinterpret_cast<uint32_t*>(ws + p.off_dbb), s);
        if (e != hipSuccess) return fail_hip(e);
    }

    for (int64_t qb = 0; qb < m; qb += p.batch) {
        const int mb = static_cast<int>(m - qb < p.batch ? m - qb : p.batch);
        const uint32_t* q_rows = q_codes + qb * (static_cast<int64_t>(q_bits) * p.W);

        ScanArgs sa{};
        sa.db = db_codes;
        sa.n = n;
        sa.bundle_mul = p.bundle_mul;
        sa.m = mb;
        sa.q_bits = q_bits;
        sa.db_bits = db_bits;
        sa.W = p.W;
        sa.wc = p.wc;
        sa.nchunks = p.nchunks;
        sa.thr = reinterpret_cast<uint32_t*>(ws + p.off_thr);
        sa.cnt = reinterpret_cast<uint32_t*>(ws + p.off_cnt);
        sa.cand = reinterpret_cast<uint64_t*>(ws + p.off_cand);
        sa.cap = p.cap;
        sa.dense = reinterpret_cast<uint32_t*>(ws + p.off_dense);
        sa.dense_stride = p.first;
        if (p.wc) {
            uint32_t* qc = reinterpret_cast<uint32_t*>(ws + p.off_q);
            const hipError_t e = launch_repack_queries(q_rows, mb, q_bits, p.W, p.wc, p.nchunks, qc, s);
            if (e != hipSuccess) return fail_hip(e);
            sa.q = qc;
        } else {
            sa.q = q_rows;
        }

        DotArgs da{};
        if (p.dot) {
            uint32_t* qn = reinterpret_cast<uint32_t*>(ws + p.off_qn);
            int32_t* qsum = reinterpret_cast<int32_t*>(ws + p.off_qsum);
            const hipError_t e = launch_nibbles_q(q_rows, mb, d, q_bits, qn, qsum, s);
            if (e != hipSuccess) return fail_hip(e);
            da.dbn = reinterpret_cast<const uint32_t*>(ws + p.off_dbn);
            da.n = n;
            da.qn = qn;
            da.qsum = qsum;
            da.m = mb;
            da.WD = 4 * p.W;
            da.half_full_minus_d = (d * ((1 << q_bits) - 1) * ((1 << db_bits) - 1) - d) / 2;
            da.thr = sa.thr;
            da.cnt = sa.cnt;
            da.cand = sa.cand;
            da.cap = sa.cap;
            da.dense = sa.dense;
            da.dense_stride = sa.dense_stride;
        }

        MfmaArgs fa{};
        if (p.mfma) {
            const int mpad = (mb + 31) / 32 * 32;
            uint32_t* qb8 = reinterpret_cast<uint32_t*>(ws + p.off_qb);
            const hipError_t e = launch_bytes_q(q_rows, mb, mpad, d, q_bits, qb8, s);
            if (e != hipSuccess) return fail_hip(e);
            fa.dbb = reinterpret_cast<const uint8_t*>(ws + p.off_dbb);
            fa.rows_padded = (n + kLanes - 1) / kLanes * kLanes;
            fa.qb = reinterpret_cast<const uint8_t*>(qb8);
            fa.m = mb;
            fa.m_padded = mpad;
            fa.W = p.W;
            fa.full = d * ((1 << q_bits) - 1) * ((1 << db_bits) - 1);
            fa.thr = sa.thr;
            fa.cnt = sa.cnt;
            fa.cand = sa.cand;
            fa.cap = sa.cap;
            fa.dense = sa.dense;
            fa.dense_stride = sa.dense_stride;
            fa.qsplit = mb < 1024 ? mpad : 1024;         // long query ranges: the row tiles are loaded once per range
        }

        SelectArgs sel{};
        sel.n = n;
        sel.bundle_mul = p.bundle_mul;
        sel.m = mb;
        sel.k = k;
        sel.d = d;
        sel.q_bits = q_bits;
        sel.db_bits = db_bits;
        sel.topk = reinterpret_cast<uint64_t*>(ws + p.off_topk);
        sel.thr = reinterpret_cast<uint32_t*>(ws + p.off_thr);
        sel.cnt = reinterpret_cast<uint32_t*>(ws + p.off_cnt);
        sel.cand = sa.cand;
        sel.cap = p.cap;
        sel.dense = sa.dense;
        sel.dense_stride = p.first;
        sel.len = reinterpret_cast<uint32_t*>(ws + p.off_len);
        sel.keep_max = p.keep_max;
        sel.extra = job.extra;
        sel.idx = job.idx + qb * k;
        sel.score = refine ? nullptr : job.score + qb * k;

        // group 0: dense
        int64_t seen = p.first;
        {
            sa.row_begin = 0;
            sa.row_end = seen;
            const int64_t bundles = (seen + kLanes - 1) / kLanes;
            sa.rows_per_lane = 1;
            sa.qsplit = choose_qsplit(o, bundles, 1, mb, tile);
            da.row_begin = sa.row_begin; da.row_end = sa.row_end; da.rows_per_lane = 1; da.qsplit = sa.qsplit;
            fa.row_begin = sa.row_begin; fa.row_end = sa.row_end;
            hipError_t e = p.mfma ? traced_scan_mfma(fa, true, s) : p.dot ? traced_scan_dot(da, true, s) : traced_scan(sa, true, s);
            if (e != hipSuccess) return fail_hip(e);
            sel.row_begin = 0;
            sel.rows = p.first;
            sel.final_group = seen >= n;
            e = launch_select_dense(sel, s);
            if (e != hipSuccess) return fail_hip(e);
        }
        // later groups: threshold scan, merge, exact rescan of overflowed queries
        while (seen < n) {
            // expected survivors per query in a group are about k * (growth - 1): keep them
            // at a third of the list capacity at most
            double growth = 1.0 + static_cast<double>(p.cap) / (3.0 * k);
            if (growth > o.growth) growth = o.growth;
            if (refine && growth > o.refine_growth) growth = o.refine_growth;   // the kept list may be as long as the survivor list
            int64_t size = static_cast<int64_t>(std::ceil(static_cast<double>(seen) * (growth - 1.0)));
            size = (size + 511) / 512 * 512;
            int64_t end = seen + size;
            if (end > n || n - end < 512) end = n;
            sa.row_begin = seen;
            sa.row_end = end;
            const int64_t bundles = (end - seen + kLanes - 1) / kLanes;
            sa.rows_per_lane = (rpl_max == 2 && bundles >= 4096) ? 2 : 1;
            sa.qsplit = choose_qsplit(o, bundles, sa.rows_per_lane, mb, tile);
            da.row_begin = seen; da.row_end = end; da.rows_per_lane = sa.rows_per_lane; da.qsplit = sa.qsplit;
            fa.row_begin = seen; fa.row_end = end;
            hipError_t e = p.mfma ? traced_scan_mfma(fa, false, s) : p.dot ? traced_scan_dot(da, false, s) : traced_scan(sa, false, s);
            if (e != hipSuccess) return fail_hip(e);
            sel.row_begin = seen;
            sel.final_group = end >= n;
            MergeArgs ma{};
            ma.db = db_codes;
            ma.n = n;
            ma.row_begin = seen;
            ma.row_end = end;
            ma.q_rows = q_rows;
            ma.W = p.W;
            ma.sel = sel;
            e = launch_select_merge(ma, s);
            if (e != hipSuccess) return fail_hip(e);
            seen = end;
        }
        if (refine && !job.lists_only) {
            RefineArgs ra{};
            ra.X_db = job.X_db;
            ra.X_q = job.X_q + qb * d;
            ra.m = mb;
            ra.k = k;
            ra.d = d;
            ra.topk = sel.topk;
            ra.len = sel.len;
            ra.keep_max = p.keep_max;
            ra.idx = job.idx + qb * k;
            ra.sim = job.similarity + qb * k;
            ra.count = job.candidates ? job.candidates + qb : nullptr;
            const hipError_t e = launch_refine(ra, s);
            if (e != hipSuccess) return fail_hip(e);
        }
    }
    return XBQ_OK;
}

// Algorithm 1 with the whole candidate list.  First stage of a batch of queries: the plain exact
// search when they are few (histogram path), else the bounded candidate search, whose lists are
// already whole for most queries.  Then up to two collecting scans over all rows for the
// queries that need them, then the refine.
struct KPlan {
    int64_t batch = 0;       // queries per batch: the candidate lists of a batch stay near 2 GiB
    int cap = 0, parts = 1;
    size_t inner = 0;        // workspace of the first stage of one batch
    size_t off_idx1 = 0, off_score1 = 0, off_best = 0, off_dk = 0, off_thr = 0, off_cnt = 0, off_q = 0, off_parts = 0,
           off_list = 0;
    size_t off_thr2 = 0, off_flag = 0, off_levels = 0;
    size_t total = 0;
};

// The first stage of a batch of mb queries and its workspace: the plain search (few = true) for
// few queries, where the longer schedule of the bounded candidate search costs more than the
// collecting scan it may save; else the bounded candidate search.
Plan first_stage_plan(const Options& o, int64_t n, int64_t mb, int d, int q_bits, int k, bool& few)
{
    const Plan plain = make_plan(o, n, mb, d, q_bits, k, false, true);
    few = plain.hist || plain.local || mb < o.kselect_lists_min;
    return few ? plain : make_plan(o, n, mb, d, q_bits, k, true);
}

KPlan make_kplan(const Options& o, int64_t n, int64_t m, int d, int q_bits, int k, int64_t max_candidates, int extra)
{
    KPlan kp;
    kp.cap = static_cast<int>(max_candidates < n ? max_candidates : n);
    int64_t batch = (int64_t(1) << 31) / (int64_t(8) * kp.cap);
    if (batch < 1) batch = 1;
    if (batch > 8192) batch = 8192;
    kp.batch = m < batch ? m : batch;
    bool few = false;
    const Plan whole = first_stage_plan(o, n, kp.batch, d, q_bits, k, few);
    kp.inner = whole.total;
    if (m % kp.batch) {                                   // a short last batch may take the few-query path
        const size_t t = first_stage_plan(o, n, m % kp.batch, d, q_bits, k, few).total;
        if (t > kp.inner) kp.inner = t;
    }
    int parts = kp.batch >= 1024 ? 1 : static_cast<int>((1024 + kp.batch - 1) / kp.batch);
    if (parts > kSortCap / k) parts = kSortCap / k;
    const int pieces = (kp.cap + 1023) / 1024;
    if (parts > pieces) parts = pieces;
    kp.parts = parts < 1 ? 1 : parts;
    const size_t b = static_cast<size_t>(kp.batch);
    size_t off = align_up(kp.inner, 256);
    kp.off_idx1 = off;   off = align_up(off + b * k * sizeof(int32_t), 256);
    kp.off_score1 = off; off = align_up(off + b * k * sizeof(int32_t), 256);
    kp.off_best = off;   off = align_up(off + b * k * sizeof(uint64_t), 256);
    kp.off_dk = off;     off = align_up(off + b * sizeof(uint32_t), 256);
    kp.off_thr = off;    off = align_up(off + b * sizeof(uint32_t), 256);
    kp.off_cnt = off;    off = align_up(off + b * sizeof(uint32_t), 256);
    kp.off_thr2 = off;   off = align_up(off + b * sizeof(uint32_t), 256);
    kp.off_flag = off;   off += 256;                      // two flags; cleared together with the levels behind them
    kp.off_levels = off; off = align_up(off + b * (static_cast<size_t>(extra) + 2) * sizeof(uint32_t), 256);
    kp.off_q = off;
    if (whole.wc) off = align_up(off + b * whole.nchunks * q_bits * whole.wc * sizeof(uint32_t), 256);
    kp.off_parts = off;  off = align_up(off + b * kp.parts * k * sizeof(uint64_t), 256);
    kp.off_list = off;   off = align_up(off + b * static_cast<size_t>(kp.cap) * sizeof(uint64_t), 256);
    kp.total = off;
    return kp;
}

int run_k_select(const Options& o, const SearchJob& job, const KPlan& kp, char* ws, hipStream_t s)
{
    const int64_t n = job.n, m = job.m;
    const int d = job.d, k = job.k, W = words32(d);
    for (int64_t qb = 0; qb < m; qb += kp.batch) {
        const int mb = static_cast<int>(m - qb < kp.batch ? m - qb : kp.batch);
        const uint32_t* q_rows = job.q_codes + qb * (static_cast<int64_t>(job.q_bits) * W);
        bool few = false;
        const Plan p = first_stage_plan(o, n, mb, d, job.q_bits, k, few);
        if (p.total > kp.inner) return XBQ_EWORKSPACE;    // cannot happen: make_kplan took the larger of the two

        KSelectArgs ka{};
        SearchJob first = job;
        first.q_codes = q_rows;
        first.m = mb;
        first.X_q = job.X_q + qb * d;
        if (few) {
            first.extra = -1;
            first.idx = reinterpret_cast<int32_t*>(ws + kp.off_idx1);
            first.score = reinterpret_cast<int32_t*>(ws + kp.off_score1);
            ka.idx1 = first.idx;
            ka.score1 = first.score;
        } else {
            first.lists_only = true;                      // candidate lists of at most kRefineKeep keys, no refine
            first.idx = job.idx + qb * k;                 // not written
            ka.topk1 = reinterpret_cast<const uint64_t*>(ws + p.off_topk);
            ka.len1 = reinterpret_cast<const uint32_t*>(ws + p.off_len);
            ka.keep1 = p.keep_max;
        }
        const int rc = run_search(o, first, p, ws, s);
        if (rc != XBQ_OK) return rc;

        ka.db = job.db_codes;
        ka.n = n;
        ka.q_rows = q_rows;
        ka.m = mb;
        ka.k = k;
        ka.d = d;
        ka.W = W;
        ka.q_bits = job.q_bits;
        ka.db_bits = job.db_bits;
        ka.extra = job.extra;
        ka.cap = kp.cap;
        ka.best = reinterpret_cast<uint64_t*>(ws + kp.off_best);
        ka.dk = reinterpret_cast<uint32_t*>(ws + kp.off_dk);
        ka.thr = reinterpret_cast<uint32_t*>(ws + kp.off_thr);
        ka.cnt = reinterpret_cast<uint32_t*>(ws + kp.off_cnt);
        ka.list = reinterpret_cast<uint64_t*>(ws + kp.off_list);
        ka.X_db = job.X_db;
        ka.X_q = job.X_q + qb * d;
        ka.parts = kp.parts;
        ka.part_keys = reinterpret_cast<uint64_t*>(ws + kp.off_parts);
        ka.idx = job.idx + qb * k;
        ka.sim = job.similarity + qb * k;
        ka.count = job.candidates ? job.candidates + qb : nullptr;
        ka.levels = reinterpret_cast<uint32_t*>(ws + kp.off_levels);
        ka.thr2 = reinterpret_cast<uint32_t*>(ws + kp.off_thr2);
        ka.flag = reinterpret_cast<uint32_t*>(ws + kp.off_flag);
        hipError_t e = launch_clear(ka.flag, 64 + static_cast<int64_t>(mb) * (job.extra + 2), s);    // flags + levels
        if (e != hipSuccess) return fail_hip(e);
        e = launch_kselect_first(ka, s);
        if (e != hipSuccess) return fail_hip(e);

        if (p.hist && mb <= kHistMaxQueries) {
            // one histogram pass scored these queries and its stored distances are still in the
            // workspace: collect from them instead of scanning the codes again
            const uint32_t* dist = reinterpret_cast<const uint32_t*>(ws + p.hoff_dist);
            e = launch_kselect_collect_stored(ka, dist, false, s);
            if (e != hipSuccess) return fail_hip(e);
            e = launch_kselect_levels(ka, s);
            if (e != hipSuccess) return fail_hip(e);
            e = launch_kselect_collect_stored(ka, dist, true, s);
            if (e != hipSuccess) return fail_hip(e);
            e = launch_kselect_refine(ka, s);
            if (e != hipSuccess) return fail_hip(e);
            continue;
        }

        ScanArgs sa{};
        sa.db = job.db_codes;
        sa.n = n;
        sa.m = mb;
        sa.q_bits = job.q_bits;
        sa.db_bits = job.db_bits;
        sa.W = W;
        sa.wc = p.wc;
        sa.nchunks = p.nchunks;
        sa.thr = ka.thr;
        sa.cnt = ka.cnt;
        sa.cand = ka.list;
        sa.cap = kp.cap;
        if (p.wc) {
            uint32_t* qc = reinterpret_cast<uint32_t*>(ws + kp.off_q);
            e = launch_repack_queries(q_rows, mb, job.q_bits, W, p.wc, p.nchunks, qc, s);
            if (e != hipSuccess) return fail_hip(e);
            sa.q = qc;
        } else {
            sa.q = q_rows;
        }
        sa.row_begin = 0;
        sa.row_end = n;
        const int64_t bundles = (n + kLanes - 1) / kLanes;
        const int rpl_max = (p.wc == 0 && job.db_bits * W <= 16) ? 2 : 1;
        sa.rows_per_lane = (rpl_max == 2 && bundles >= 4096) ? 2 : 1;
        sa.qsplit = choose_qsplit(o, bundles, sa.rows_per_lane, mb, p.wc ? kTileQ : 1);
        sa.levels = ka.levels;
        sa.level_base = ka.dk;
        sa.level_stride = job.extra + 2;
        sa.run_flag = ka.flag;                            // first collection: queries whose list is not whole yet
        e = traced_scan(sa, false, s);
        if (e != hipSuccess) return fail_hip(e);
        e = launch_kselect_levels(ka, s);
        if (e != hipSuccess) return fail_hip(e);
        sa.thr = ka.thr2;                                 // second collection: lowered bounds only
        sa.levels = nullptr;
        sa.run_flag = ka.flag + 1;
        e = traced_scan(sa, false, s);
        if (e != hipSuccess) return fail_hip(e);
        e = launch_kselect_refine(ka, s);
        if (e != hipSuccess) return fail_hip(e);
    }
    return XBQ_OK;
}

// xbq_search, xbq_search_asym, xbq_search_ex and xbq_search_static after their options are fixed.
int search_with(const Options& o, const uint32_t* db_codes, int64_t n, int db_bits, const uint32_t* q_codes, int64_t m,
                int q_bits, int d, int k, int32_t* idx, int32_t* score, void* workspace, size_t workspace_bytes,
                void* stream)
{
    if (d < 1 || db_bits < 1 || q_bits < 1 || n < 0 || m < 0) return XBQ_EINVAL;
    if (!valid_shape(d, db_bits) || !valid_shape(d, q_bits) || !scan_supports_bits(q_bits, db_bits))
        return XBQ_EUNSUPPORTED;
    if (!valid_search_sizes(n, m, d, q_bits, k)) return XBQ_EINVAL;
    if (n == 0 || m == 0) return XBQ_OK;
    if (!db_codes || !q_codes || !idx || !score || !workspace) return XBQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(db_codes) % 4 || reinterpret_cast<uintptr_t>(q_codes) % 4 ||
        reinterpret_cast<uintptr_t>(idx) % 4 || reinterpret_cast<uintptr_t>(score) % 4 ||
        reinterpret_cast<uintptr_t>(workspace) % 256)
        return XBQ_EINVAL;
    const Plan p = make_plan(o, n, m, d, q_bits, k, false);
    if (workspace_bytes < p.total) return XBQ_EWORKSPACE;
    SearchJob job{};
    job.db_codes = db_codes; job.n = n; job.db_bits = db_bits;
    job.q_codes = q_codes; job.m = m; job.q_bits = q_bits;
    job.d = d; job.k = k; job.extra = -1;
    job.idx = idx; job.score = score;
    return run_search(o, job, p, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" {

int xbq_version(void) { return 100; }

const char* xbq_strerror(int code)
{
    switch (code) {
    case XBQ_OK: return "ok";
    case XBQ_EINVAL: return "invalid argument";
    case XBQ_EUNSUPPORTED: return "unsupported bits, dimension or layout";
    case XBQ_EWORKSPACE: return "workspace too small";
    case XBQ_EHIP: return "HIP runtime error";
    case XBQ_ESTATIC: return "request needs more scratch than the built-in buffer of xbq_search_static holds";
    default: return "unknown error code";
    }
}

int xbq_last_hip_error(void) { return g_last_hip_error; }

size_t xbq_code_bytes(int64_t n, int d, int bits, int layout)
{
    if (!valid_shape(d, bits) || n < 0 || n >= (int64_t(1) << 31)) return 0;
    const size_t per_row = static_cast<size_t>(bits) * words32(d) * sizeof(uint32_t);
    if (layout == XBQ_ROWS) return static_cast<size_t>(n) * per_row;
    if (layout == XBQ_BUNDLE64) return static_cast<size_t>((n + kLanes - 1) / kLanes) * kLanes * per_row;
    return 0;
}

int xbq_encode(const float* X, int64_t n, int d, int bits, float scale, int layout, uint32_t* codes, void* stream)
{
    if (d < 1 || bits < 1 || n < 0 || n >= (int64_t(1) << 31)) return XBQ_EINVAL;
    if (!valid_shape(d, bits) || (layout != XBQ_ROWS && layout != XBQ_BUNDLE64)) return XBQ_EUNSUPPORTED;
    if (!(scale > 0.0f) || !std::isfinite(scale)) return XBQ_EINVAL;
    if (n == 0) return XBQ_OK;
    if (X == nullptr || codes == nullptr) return XBQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(X) % 4 || reinterpret_cast<uintptr_t>(codes) % 4) return XBQ_EINVAL;
    const hipError_t e = launch_encode(X, n, d, bits, scale, layout, codes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XBQ_OK : fail_hip(e);
}

size_t xbq_search_workspace_bytes(int64_t n, int64_t m, int d, int bits, int k)
{
    return xbq_search_workspace_bytes_ex(n, m, d, bits, k, nullptr);
}

size_t xbq_search_workspace_bytes_ex(int64_t n, int64_t m, int d, int q_bits, int k, const xbq_options* options)
{
    Options o;
    if (!options_from(options, o)) return 0;
    if (!valid_search_sizes(n, m, d, q_bits, k)) return 0;
    if (n == 0 || m == 0) return 256;
    return make_plan(o, n, m, d, q_bits, k).total;
}

void xbq_options_default(xbq_options* options)
{
    if (options == nullptr) return;
    const Options o;
    options->struct_bytes = sizeof(xbq_options);
    options->selector = o.selector;
    options->kernel = o.kernel;
    options->first = o.first;
    options->qsplit = o.qsplit;
    options->hist_max_queries = o.hist_max_queries;
    options->kselect_lists_min = o.kselect_lists_min;
    options->local_groups = o.local_groups;
    options->row_order = o.row_order;
    options->reserved = 0;
    options->growth = o.growth;
    options->refine_growth = o.refine_growth;
}

int xbq_search(const uint32_t* db_codes, int64_t n, const uint32_t* q_codes, int64_t m, int d, int bits, int k,
               int32_t* idx, int32_t* score, void* workspace, size_t workspace_bytes, void* stream)
{
    return xbq_search_ex(db_codes, n, bits, q_codes, m, bits, d, k, idx, score, workspace, workspace_bytes, nullptr, stream);
}

int xbq_search_asym(const uint32_t* db_codes, int64_t n, int db_bits, const uint32_t* q_codes, int64_t m, int q_bits,
                    int d, int k, int32_t* idx, int32_t* score, void* workspace, size_t workspace_bytes, void* stream)
{
    return xbq_search_ex(db_codes, n, db_bits, q_codes, m, q_bits, d, k, idx, score, workspace, workspace_bytes, nullptr,
                         stream);
}

int xbq_search_ex(const uint32_t* db_codes, int64_t n, int db_bits, const uint32_t* q_codes, int64_t m, int q_bits,
                  int d, int k, int32_t* idx, int32_t* score, void* workspace, size_t workspace_bytes,
                  const xbq_options* options, void* stream)
{
    Options o;
    if (!options_from(options, o)) return XBQ_EINVAL;
    return search_with(o, db_codes, n, db_bits, q_codes, m, q_bits, d, k, idx, score, workspace, workspace_bytes, stream);
}

int xbq_search_static(const uint32_t* db_codes, int64_t n, const uint32_t* q_codes, int64_t m, int d, int bits, int k,
                      int32_t* idx, int32_t* score, void* stream)
{
    if (d < 1 || bits < 1 || n < 0 || m < 0) return XBQ_EINVAL;
    if (!valid_shape(d, bits)) return XBQ_EUNSUPPORTED;
    if (!valid_search_sizes(n, m, d, bits, k)) return XBQ_EINVAL;
    if (n == 0 || m == 0) return XBQ_OK;
    const Options o = default_options();
    // the size check comes first: a request that cannot fit is refused without any HIP call
    if (make_plan(o, n, m, d, bits, k, false).total > static_cast<size_t>(XBQ_STATIC_SCRATCH_BYTES)) return XBQ_ESTATIC;
    char* ws = nullptr;
    const hipError_t e = scratch_address(&ws);
    if (e != hipSuccess) return fail_hip(e);
    return search_with(o, db_codes, n, bits, q_codes, m, bits, d, k, idx, score, ws, XBQ_STATIC_SCRATCH_BYTES, stream);
}

size_t xbq_search_refine_workspace_bytes(int64_t n, int64_t m, int d, int q_bits, int k)
{
    if (!valid_search_sizes(n, m, d, q_bits, k)) return 0;
    if (n == 0 || m == 0) return 256;
    return make_plan(default_options(), n, m, d, q_bits, k, true).total;
}

int xbq_search_refine(const float* X_db, const uint32_t* db_codes, int64_t n, int db_bits, const float* X_q,
                      const uint32_t* q_codes, int64_t m, int q_bits, int d, int k, int extra_distance, int32_t* idx,
                      float* similarity, int32_t* candidates, void* workspace, size_t workspace_bytes, void* stream)
{
    if (d < 1 || db_bits < 1 || q_bits < 1 || n < 0 || m < 0) return XBQ_EINVAL;
    if (!valid_shape(d, db_bits) || !valid_shape(d, q_bits) || !scan_supports_bits(q_bits, db_bits))
        return XBQ_EUNSUPPORTED;
    if (!valid_search_sizes(n, m, d, q_bits, k)) return XBQ_EINVAL;
    if (extra_distance < 0 || extra_distance > (1 << 30)) return XBQ_EINVAL;
    if (n == 0 || m == 0) return XBQ_OK;
    if (!X_db || !X_q || !db_codes || !q_codes || !idx || !similarity || !workspace) return XBQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(db_codes) % 4 || reinterpret_cast<uintptr_t>(q_codes) % 4 ||
        reinterpret_cast<uintptr_t>(X_db) % 4 || reinterpret_cast<uintptr_t>(X_q) % 4 ||
        reinterpret_cast<uintptr_t>(idx) % 4 || reinterpret_cast<uintptr_t>(similarity) % 4 ||
        reinterpret_cast<uintptr_t>(candidates) % 4 || reinterpret_cast<uintptr_t>(workspace) % 256)
        return XBQ_EINVAL;
    const Options o = default_options();
    const Plan p = make_plan(o, n, m, d, q_bits, k, true);
    if (workspace_bytes < p.total) return XBQ_EWORKSPACE;
    SearchJob job{};
    job.db_codes = db_codes; job.n = n; job.db_bits = db_bits;
    job.q_codes = q_codes; job.m = m; job.q_bits = q_bits;
    job.d = d; job.k = k; job.extra = extra_distance;
    job.idx = idx; job.X_db = X_db; job.X_q = X_q; job.similarity = similarity; job.candidates = candidates;
    return run_search(o, job, p, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

size_t xbq_k_select_workspace_bytes(int64_t n, int64_t m, int d, int q_bits, int k, int extra_distance,
                                    int64_t max_candidates)
{
    if (!valid_search_sizes(n, m, d, q_bits, k)) return 0;
    if (extra_distance < 0 || extra_distance > XBQ_MAX_EXTRA) return 0;
    if (max_candidates < k || max_candidates > XBQ_MAX_CANDIDATES) return 0;
    if (n == 0 || m == 0) return 256;
    return make_kplan(default_options(), n, m, d, q_bits, k, max_candidates, extra_distance).total;
}

int xbq_k_select(const float* X_db, const uint32_t* db_codes, int64_t n, int db_bits, const float* X_q,
                 const uint32_t* q_codes, int64_t m, int q_bits, int d, int k, int extra_distance,
                 int64_t max_candidates, int32_t* idx, float* similarity, int32_t* candidates, void* workspace,
                 size_t workspace_bytes, void* stream)
{
    if (d < 1 || db_bits < 1 || q_bits < 1 || n < 0 || m < 0) return XBQ_EINVAL;
    if (!valid_shape(d, db_bits) || !valid_shape(d, q_bits) || !scan_supports_bits(q_bits, db_bits))
        return XBQ_EUNSUPPORTED;
    if (!valid_search_sizes(n, m, d, q_bits, k)) return XBQ_EINVAL;
    if (extra_distance < 0 || extra_distance > XBQ_MAX_EXTRA) return XBQ_EINVAL;
    if (max_candidates < k || max_candidates > XBQ_MAX_CANDIDATES) return XBQ_EINVAL;
    if (n == 0 || m == 0) return XBQ_OK;
    if (!X_db || !X_q || !db_codes || !q_codes || !idx || !similarity || !workspace) return XBQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(db_codes) % 4 || reinterpret_cast<uintptr_t>(q_codes) % 4 ||
        reinterpret_cast<uintptr_t>(X_db) % 4 || reinterpret_cast<uintptr_t>(X_q) % 4 ||
        reinterpret_cast<uintptr_t>(idx) % 4 || reinterpret_cast<uintptr_t>(similarity) % 4 ||
        reinterpret_cast<uintptr_t>(candidates) % 4 || reinterpret_cast<uintptr_t>(workspace) % 256)
        return XBQ_EINVAL;
    const Options o = default_options();
    const KPlan kp = make_kplan(o, n, m, d, q_bits, k, max_candidates, extra_distance);
    if (workspace_bytes < kp.total) return XBQ_EWORKSPACE;
    SearchJob job{};
    job.db_codes = db_codes; job.n = n; job.db_bits = db_bits;
    job.q_codes = q_codes; job.m = m; job.q_bits = q_bits;
    job.d = d; job.k = k; job.extra = extra_distance;
    job.idx = idx; job.X_db = X_db; job.X_q = X_q; job.similarity = similarity; job.candidates = candidates;
    return run_k_select(o, job, kp, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

int xbq_trace_enable(int on)
{
    if (on && g_trace.ev.empty()) {
        g_trace.ev.resize(2 * kTraceMaxLaunches);
        for (auto& e : g_trace.ev) {
            const hipError_t r = hipEventCreate(&e);
            if (r != hipSuccess) { g_trace.ev.clear(); return fail_hip(r); }
        }
    }
    g_trace.on = on != 0;
    g_trace.used = 0;
    g_trace.pairs = 0;
    return XBQ_OK;
}

int xbq_trace_read(double* scan_ms, int64_t* launches, double* pairs)
{
    if (!scan_ms || !launches || !pairs) return XBQ_EINVAL;
    double ms = 0;
    for (int i = 0; i + 1 < g_trace.used; i += 2) {
        hipError_t e = hipEventSynchronize(g_trace.ev[i + 1]);
        if (e != hipSuccess) return fail_hip(e);
        float t = 0;
        e = hipEventElapsedTime(&t, g_trace.ev[i], g_trace.ev[i + 1]);
        if (e != hipSuccess) return fail_hip(e);
        ms += t;
    }
    *scan_ms = ms;
    *launches = g_trace.used / 2;
    *pairs = g_trace.pairs;
    g_trace.used = 0;
    g_trace.pairs = 0;
    return XBQ_OK;
}

size_t xbq_probe_out_bytes(void) { return probe_out_bytes(); }

int xbq_probe_valu(uint32_t* out, size_t out_bytes, uint32_t seed, int iters, double* lane_ops, void* stream)
{
    if (!out || reinterpret_cast<uintptr_t>(out) % 4 || iters < 1 || iters > (1 << 24)) return XBQ_EINVAL;
    if (out_bytes < probe_out_bytes()) return XBQ_EWORKSPACE;
    if (lane_ops) *lane_ops = probe_valu_lane_ops(iters);
    const hipError_t e = launch_probe_valu(out, seed, iters, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XBQ_OK : fail_hip(e);
}

int xbq_probe_read(const void* buf, size_t bytes, uint32_t* out, size_t out_bytes, void* stream)
{
    if (!buf || !out || reinterpret_cast<uintptr_t>(buf) % 16 || reinterpret_cast<uintptr_t>(out) % 4 || bytes % 16)
        return XBQ_EINVAL;
    if (out_bytes < probe_out_bytes()) return XBQ_EWORKSPACE;
    const hipError_t e = launch_probe_read(buf, bytes, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XBQ_OK : fail_hip(e);
}

int xbq_probe_encode_traffic(const float* X, int64_t n, int d, int bits, uint32_t* codes, void* stream)
{
    if (d < 1 || bits < 1 || n < 0 || n >= (int64_t(1) << 31)) return XBQ_EINVAL;
    if (!valid_shape(d, bits) || d % 4 != 0) return XBQ_EUNSUPPORTED;
    if (n == 0) return XBQ_OK;
    if (!X || !codes || reinterpret_cast<uintptr_t>(X) % 16 || reinterpret_cast<uintptr_t>(codes) % 4) return XBQ_EINVAL;
    const hipError_t e = launch_probe_encode_traffic(X, n, d, bits, codes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XBQ_OK : fail_hip(e);
}

int xbq_set_option(const char* name, double value)
{
    if (!name) return XBQ_EINVAL;
    std::lock_guard<std::mutex> lock(g_opt_mutex);
    Options o = g_opt;
    if (!set_knob(o, name, value)) return XBQ_EINVAL;
    g_opt = o;
    return XBQ_OK;
}

}  // extern "C"
