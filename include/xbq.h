/*
 * xbq -- XOR-friendly binary quantized exhaustive top-K cosine search on MI355X.
 *
 * C ABI of libxbq.so.  The library implements the search path of "Fast top-K
 * Cosine Similarity Search through XOR-Friendly Binary Quantization on GPUs"
 * (arXiv 2008.02002): encode fp32 vectors into B-bit codes stored as bit-planes,
 * score every query against every database row with XOR + population count, and
 * select the K best rows per query.
 *
 * Equation numbers are the paper's own running numbers: Eq. 1 sigma, Eq. 2 the product/XOR
 * identity (Section 3.1); Eq. 5 x_B y_B from xbar (x) ybar (Section 3.2); Eq. 7 X.Y from
 * Xbar (x) Ybar, Eq. 9 the bit-plane reconstruction xhat_b, Eq. 10 the POPCNT form (Section 3.3).
 *
 * Common rules for every entry point
 *   - Every pointer named X, codes, db_codes, q_codes, idx, score or workspace is
 *     a DEVICE pointer owned by the caller.  The library never allocates, frees
 *     or keeps device memory, and never synchronises the stream or the device.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it and the call returns immediately.
 *   - Return value: XBQ_OK (0) or a negative XBQ_E* code; xbq_strerror() names it.
 *     On an argument error nothing is enqueued and no output is written.
 *   - n == 0 or m == 0 is valid and does nothing.
 *   - Inputs must be finite; NaN is outside the contract.  L2 normalisation is the
 *     caller's business (Section 3: cosine = inner product of normalised vectors).
 */
#ifndef XBQ_H
#define XBQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XBQ_OK            0
#define XBQ_EINVAL       (-1)  /* null pointer, bad size, bad k, misaligned pointer      */
#define XBQ_EUNSUPPORTED (-2)  /* bits, d or layout outside what the kernels cover       */
#define XBQ_EWORKSPACE   (-3)  /* workspace smaller than xbq_search_workspace_bytes()    */
#define XBQ_EHIP         (-4)  /* a HIP launch or query failed; see xbq_last_hip_error() */
#define XBQ_ESTATIC      (-5)  /* xbq_search_static: the request needs more scratch than
                                  XBQ_STATIC_SCRATCH_BYTES                                */

/* Code layouts (both hold uint32 plane words, W = ceil(d/32) per plane, plane b =
 * bit b of every coordinate's code, coordinate 32w+t at bit t of word w, pad bits 0;
 * Section 3.3, Eq. 9, the bit-plane reconstruction xhat_b):
 *   XBQ_ROWS     [n][bits][W]                    exchange layout, used for queries
 *   XBQ_BUNDLE64 [ceil(n/64)][bits][W][64]       scan layout, used for the database:
 *                rows are grouped 64 at a time (one per wavefront lane) and stored
 *                word-major so a wavefront reads one word of 64 rows as 256 contiguous
 *                bytes.  Rows past n in the last bundle are written as zero words.
 * (The bundle idea is the one Section 4.1 "Distance Calculation" describes for
 * 32-wide warps, resized for 64-wide wavefronts.) */
#define XBQ_ROWS     0
#define XBQ_BUNDLE64 1

#define XBQ_MAX_BITS 4      /* bits per coordinate: 1..4                              */
#define XBQ_MAX_DIM  2048   /* d: 1..2048                                             */
#define XBQ_MAX_K    1024   /* k: 1..min(n, 1024)  (Section 5 evaluates K up to 1000) */
#define XBQ_MAX_EXTRA 4095  /* extra distance of xbq_k_select                          */
#define XBQ_MAX_CANDIDATES (1 << 22)   /* candidate bound of xbq_k_select              */

int xbq_version(void);
const char* xbq_strerror(int code);
/* hipError_t (as int) of the most recent XBQ_EHIP on this thread, 0 if none. */
int xbq_last_hip_error(void);

/* Bytes of a codes buffer for n rows in the given layout; 0 if arguments are invalid. */
size_t xbq_code_bytes(int64_t n, int d, int bits, int layout);

/*
 * Encode (Section 3.2 quantizer f_B after the scaling of Section 3.5, then the
 * bit-plane reconstruction of Section 3.3 / Eq. 9).
 *   X      [n][d] fp32 row-major, device, read only
 *   scale  finite, > 0; every coordinate is multiplied by it in binary32 (round to
 *          nearest even) before quantizing; 1.0f gives the bare f_B
 *   codes  device, xbq_code_bytes(n, d, bits, layout) bytes, fully overwritten
 * The code of coordinate value t is chosen digit by digit, most significant first,
 * with sign(0) = +1; stored bit 1 means digit -1.  Values at or beyond +-1 land in the
 * outermost cell (no error).  n < 2^31.
 */
int xbq_encode(const float* X, int64_t n, int d, int bits, float scale, int layout,
               uint32_t* codes, void* stream);

/* Bytes of scratch xbq_search needs for these sizes; 0 if arguments are invalid.  Depends on
 * the process-wide options in force (xbq_set_option; xbq_search_workspace_bytes_ex takes them as
 * an argument instead).  With more than a handful of queries it depends on n only through
 * min(n, small constant) and on m only up to an internal query batch (about 0.33 GiB at k = 100,
 * 0.75 GiB at k = 1000); with few
 * queries it holds per-workgroup candidate lists (at most ~25 MB), or for k > 256 four bytes per
 * (query, row) for up to 8 queries, at most 1 GiB; the cross-check kernels add a copy of the
 * database codes. */
size_t xbq_search_workspace_bytes(int64_t n, int64_t m, int d, int bits, int k);

/*
 * Exhaustive top-K (Section 2 problem statement; Section 3.3, Eq. 10, the POPCNT form,
 * for the distance; Eq. 7 for the score).
 *   db_codes  XBQ_BUNDLE64 codes of the n database rows
 *   q_codes   XBQ_ROWS codes of the m queries (same d, bits and scale as the database)
 *   idx       [m][k] int32: database row numbers, best first
 *   score     [m][k] int32: S = d*(2^bits-1)^2 - 2*D, D = sum_i sum_j POPCNT(x_i ^ y_j) << (i+j);
 *             S is the integer inner product of the decoded codes scaled by 4^bits
 *   workspace device scratch, 256-byte aligned, at least xbq_search_workspace_bytes(...);
 *             contents are undefined afterwards; one workspace serves one call at a time
 * Order: S descending, ties by ascending row number; the result is unique.
 * 1 <= k <= min(n, XBQ_MAX_K), n < 2^31, else XBQ_EINVAL.
 */
int xbq_search(const uint32_t* db_codes, int64_t n, const uint32_t* q_codes, int64_t m, int d,
               int bits, int k, int32_t* idx, int32_t* score, void* workspace,
               size_t workspace_bytes, void* stream);

/*
 * Same search with different code widths on the two sides (Section 3.6 and Section 5 use
 * 4-bit queries against 3-bit documents: three quarters of the operations and of the
 * database bytes of 4 x 4).  db_codes hold db_bits planes, q_codes q_bits planes;
 * supported pairs: q_bits == db_bits or q_bits == db_bits + 1, both in 1..4, else
 * XBQ_EUNSUPPORTED.  score = d*(2^q_bits-1)*(2^db_bits-1) - 2*D.  The workspace must be at
 * least xbq_search_workspace_bytes(n, m, d, q_bits, k).  Everything else as xbq_search.
 */
int xbq_search_asym(const uint32_t* db_codes, int64_t n, int db_bits, const uint32_t* q_codes,
                    int64_t m, int q_bits, int d, int k, int32_t* idx, int32_t* score,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same search with its schedule options passed per call instead of taken from the
 * process-wide defaults (xbq_set_option): two callers with different options can coexist, and
 * the workspace a call needs is a function of its arguments alone.  Code widths as for
 * xbq_search_asym.  options == NULL means the process-wide defaults in force when the call
 * starts (every entry point takes one snapshot of them).  A field out of its range, or a
 * struct_bytes that is not sizeof(xbq_options), gives XBQ_EINVAL (workspace query: 0).
 * Fields: see xbq_set_option below; xbq_options_default fills in the built-in defaults.
 */
typedef struct xbq_options {
    uint32_t struct_bytes;       /* sizeof(xbq_options) */
    int32_t selector;
    int32_t kernel;
    int32_t first;
    int32_t qsplit;
    int32_t hist_max_queries;
    int32_t kselect_lists_min;
    int32_t local_groups;
    int32_t row_order;
    int32_t reserved;            /* keeps the doubles aligned; ignored */
    double growth;
    double refine_growth;
} xbq_options;
void xbq_options_default(xbq_options* options);
size_t xbq_search_workspace_bytes_ex(int64_t n, int64_t m, int d, int q_bits, int k, const xbq_options* options);
int xbq_search_ex(const uint32_t* db_codes, int64_t n, int db_bits, const uint32_t* q_codes, int64_t m,
                  int q_bits, int d, int k, int32_t* idx, int32_t* score, void* workspace,
                  size_t workspace_bytes, const xbq_options* options, void* stream);

/*
 * xbq_search for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and order as xbq_search, without the workspace: the scratch memory is a buffer of
 * XBQ_STATIC_SCRATCH_BYTES that is part of the library image (every GPU the library runs on
 * holds one until the process ends).  The call allocates and frees nothing.
 *   - A request whose xbq_search_workspace_bytes(n, m, d, bits, k) exceeds
 *     XBQ_STATIC_SCRATCH_BYTES returns XBQ_ESTATIC before anything is enqueued (32 MiB serves,
 *     e.g., up to 4 queries at k <= 256 whatever n, 8 queries x 900 000 rows, 1 000 queries at
 *     k = 100 or 1 500 at k = 10 whatever n; it uses the process-wide default options).
 *   - All calls on one GPU share that GPU's buffer, which keeps the previous call's contents
 *     (the kernels clear what they need zeroed): two calls that overlap in time on one GPU --
 *     different streams, or different threads -- race.  Serialise them on one stream.
 */
#define XBQ_STATIC_SCRATCH_BYTES (32u << 20)
int xbq_search_static(const uint32_t* db_codes, int64_t n, const uint32_t* q_codes, int64_t m, int d,
                      int bits, int k, int32_t* idx, int32_t* score, void* stream);

/*
 * Search with the extra-distance candidate list and the exact refine of Algorithm 1
 * (Section 3.6 "extra distance"; Section 4.1 "Histogram and Select" and "Refine").
 * Per query: D_K = the K-th smallest distance over all n rows; the candidate list L holds
 * every row with D <= D_K + extra_distance (ties included), in (D, row) order, cut to the
 * first XBQ_REFINE_MAX_CANDIDATES if longer; each candidate's similarity is the fp32 inner
 * product of its original row with the original query (lane-strided fused multiply-adds
 * and a butterfly sum, so within a few ulp of the exact value); the K best by (similarity
 * descending, row ascending) are returned.
 *   X_db [n][d], X_q [m][d]  the fp32 vectors the codes were made from (device)
 *   extra_distance           >= 0, in units of the integer distance D
 *   idx [m][k] int32, similarity [m][k] fp32
 *   candidates               [m] int32 = |L| per query, or NULL
 *   workspace                at least xbq_search_refine_workspace_bytes(n, m, d, q_bits, k)
 * Code widths as for xbq_search_asym (pass the same value twice for symmetric codes).
 */
#define XBQ_REFINE_MAX_CANDIDATES 2048
size_t xbq_search_refine_workspace_bytes(int64_t n, int64_t m, int d, int q_bits, int k);
int xbq_search_refine(const float* X_db, const uint32_t* db_codes, int64_t n, int db_bits,
                      const float* X_q, const uint32_t* q_codes, int64_t m, int q_bits, int d, int k,
                      int extra_distance, int32_t* idx, float* similarity, int32_t* candidates,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Algorithm 1 (K-Select) with its candidate list taken whole.  For each query: D_K = the K-th
 * smallest distance over all rows (the exact search above); L = every row with
 * D <= D_K + extra_distance; the K rows of L with the largest fp32 inner product with the
 * query are returned, sorted by (similarity descending, row ascending) -- the outputs mean what
 * they mean for xbq_search_refine, and candidates[q] = |L|.
 * max_candidates (k .. XBQ_MAX_CANDIDATES) bounds |L| and sizes the workspace (8 bytes per
 * slot per query of a batch; queries are processed in batches so that the lists stay near
 * 2 GiB).  A query with more rows than that within its boundary has the boundary lowered, one
 * distance unit at a time and never below D_K, until the rows within it fit; if the rows with
 * D <= D_K alone do not fit (ties), L is the K best rows by (D, row).
 * 0 <= extra_distance <= XBQ_MAX_EXTRA.  Cost: that of xbq_search_refine while every list of a
 * batch stays below 2048 rows and max_candidates; otherwise one more scan of the database
 * collects the longer lists, and another one if some query had its boundary lowered.
 */
size_t xbq_k_select_workspace_bytes(int64_t n, int64_t m, int d, int q_bits, int k, int extra_distance,
                                    int64_t max_candidates);
int xbq_k_select(const float* X_db, const uint32_t* db_codes, int64_t n, int db_bits,
                 const float* X_q, const uint32_t* q_codes, int64_t m, int q_bits, int d, int k,
                 int extra_distance, int64_t max_candidates, int32_t* idx, float* similarity,
                 int32_t* candidates, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aid.  While tracing is on, xbq_search brackets every launch of the scan
 * kernel (the XOR + population-count loop) with HIP events on the caller's stream.
 * xbq_trace_read waits for those events, returns the summed kernel time, the number of
 * launches and the number of (query, row) pairs they scored, and clears the record.
 * The record belongs to the calling thread: enable, search and read on the same thread; other
 * threads are not traced and not disturbed.  At most 4096 launches are recorded between reads.
 */
int xbq_trace_enable(int on);
int xbq_trace_read(double* scan_ms, int64_t* launches, double* pairs);

/*
 * Measurement aids: the rates this chip sustains on the streams the path is bound by,
 * for quoting a kernel against a measured ceiling beside the published one.  All are
 * asynchronous on `stream` and timed by the caller; `out` (first two) is device memory of at least
 * xbq_probe_out_bytes() bytes (XBQ_EWORKSPACE otherwise) that receives a checkable result.
 *   xbq_probe_valu  the credited instruction pair of the scan (Section 3.3, Eq. 10: XOR with a
 *                   scalar operand, population count with accumulate) from registers only, 8
 *                   wavefronts per SIMD.  Thread t (0 <= t < xbq_probe_out_bytes()/4) holds
 *                   x_j = (t+1)*0x9E3779B1 + j*0x85EBCA77 (mod 2^32), j < 16, and writes
 *                   out[t] = sum over i < 4*iters, j < 16 of POPCNT(x_j ^ (seed + i)).
 *                   *lane_ops (host, may be NULL) receives the XOR + population-count lane
 *                   operations of the launch.  1 <= iters <= 2^24.
 *   xbq_probe_read  reads `bytes` bytes (multiple of 16, 16-byte aligned, device) once with
 *                   16-byte loads; out[w], w < 2048, is the sum (mod 2^32) of the 32-bit words
 *                   read by workgroup w, so the sum of out[] is the sum of all words.
 *   xbq_probe_encode_traffic  the memory traffic of xbq_encode (XBQ_BUNDLE64) without its
 *                   arithmetic: reads X [n][d] once the way the encoder does (one workgroup per
 *                   bundle of 64 rows, 16-byte loads) and overwrites all xbq_code_bytes(n, d, bits,
 *                   XBQ_BUNDLE64) bytes of `codes`: thread t (0 <= t < 256) of bundle b stores the
 *                   sum (mod 2^32) of the 32-bit words of the 16-byte groups t, t + 256, ... of the
 *                   bundle's rows into code words t, t + 256, ... of the bundle.  d a multiple of
 *                   4 and X 16-byte aligned, else XBQ_EUNSUPPORTED / XBQ_EINVAL.  The rate it
 *                   reaches is the ceiling of the encoder's access pattern on this chip.
 */
size_t xbq_probe_out_bytes(void);
int xbq_probe_valu(uint32_t* out, size_t out_bytes, uint32_t seed, int iters, double* lane_ops, void* stream);
int xbq_probe_read(const void* buf, size_t bytes, uint32_t* out, size_t out_bytes, void* stream);
int xbq_probe_encode_traffic(const float* X, int64_t n, int d, int bits, uint32_t* codes, void* stream);

/*
 * Tuning knobs, host side only.  xbq_set_option changes the process-wide defaults (thread
 * safe; a call already running keeps the snapshot it took); xbq_search_ex takes them per call.
 *   "growth"  upper bound on rows-after-a-group / rows-before-it (default 4.0; lowered
 *             automatically for large k so the survivor lists stay short)
 *   "first"   rows scored densely before any threshold exists (default 1024)
 *   "qsplit"  queries per workgroup (0 = automatic)
 *   "selector"          0 = automatic, 1 = threshold filter with growing row groups (many
 *                       queries), 2 = histogram selection over stored distances (Section 4.1),
 *                       3 = the same selection done per workgroup while the rows stream, nothing
 *                       stored (k <= 256, four queries per pass; the automatic choice for up to
 *                       four queries, and for every few-query search over at least 6 million
 *                       rows of codes of at most 256 dimensions; a larger k falls back to 2)
 *   "hist_max_queries"  automatic choice: few-query selection up to this many queries (default
 *                       16), twice as many for k > 128, three times for k > 512
 *   "local_groups"      selector 3: most pieces the rows are split into (1..1024, default 256: one per compute unit)
 *   "row_order"         selector 1: 0 (default) = every row group of the schedule is spread evenly over
 *                       the database (bundle n of the order is bundle n * c mod the number of
 *                       full bundles), so thresholds found on one group hold for the next even when
 *                       the rows lie sorted or cluster by cluster; 1 = groups of consecutive rows.
 *                       Results do not depend on it
 *   "refine_growth"     the same bound for the bounded candidate search of xbq_search_refine and
 *                       xbq_k_select (default 1.5: safe when the lists reach their bound of 2048 rows;
 *                       2.0 is a few percent faster when they stay well below it and up to
 *                       10 % slower when they do not)
 *   "kselect_lists_min" xbq_k_select starts a batch of at least this many queries from the
 *                       bounded candidate search, a smaller one from the plain search
 *                       (default 128, the measured crossover; results do not depend on it)
 *   "kernel"            0 = XOR + population count (the method of the paper, default);
 *                       1 = cross-check scan that gets the same integer distances from packed
 *                       4-bit dot products, 2 = from an int8 matrix product on the matrix
 *                       cores (both: d <= 256, threshold selector only, and a decoded copy of
 *                       the database codes in the workspace: n*ceil(d/32)*16 resp. *32 bytes)
 * Returns XBQ_EINVAL for an unknown name or a value out of range.
 */
int xbq_set_option(const char* name, double value);

#ifdef __cplusplus
}
#endif
#endif /* XBQ_H */
