// Internal declarations shared by the translation units of libxbq.so.
// Nothing here is part of the C ABI (see include/xbq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xbq.h"

namespace xbq {

constexpr int kLanes = 64;        // wavefront width on gfx950
constexpr int kBlock = 256;       // threads per workgroup (4 wavefronts, one per SIMD)
constexpr int kSortCap = 4096;    // most 64-bit keys one workgroup sorts in LDS
constexpr int kTileQ = 16;        // queries per register tile of the word-chunked scan
constexpr int kHistBins = 1024;   // histogram bins per query (histogram selection)
constexpr int kHistCandCap = 65536;   // rows up to the boundary bin that the histogram selection collects per query
constexpr int kHistMaxQueries = 8;  // queries per pass of the histogram selection
constexpr int kLocalMaxQueries = 4; // queries per pass of the local selection (few queries, nothing stored)
constexpr size_t kLocalMaxLds = 152 * 1024;  // LDS one workgroup of the local selection may take (of 160 KB per CU)
constexpr int kLocalMaxGroups = 1024;   // most pieces (workgroups) of the local selection

// A candidate is ordered by the 64-bit key (D << 32) | row: smaller key = better
// (smaller distance D, then lower row number).  D is the distance of Eq. 10 (Section 3.3, the POPCNT form).
__host__ __device__ inline uint64_t make_key(uint32_t D, uint32_t row)
{
    return (static_cast<uint64_t>(D) << 32) | row;
}

inline int words32(int d) { return (d + 31) / 32; }

// One launch of the scan over database rows [row_begin, row_end) for queries [0, m).
struct ScanArgs {
    const uint32_t* db;      // XBQ_BUNDLE64 codes of the whole database
    int64_t n;               // rows in the database
    int64_t row_begin;       // multiple of 64
    int64_t row_end;         // <= n
    int64_t bundle_mul;      // the range counts steps of the order spread_bundle() defines (<= 1: rows as they lie);
                             // keys carry the rows' own numbers, dense columns count from row_begin in steps
    const uint32_t* q;       // XBQ_ROWS codes (register-resident scan) or chunk-major
                             // padded codes [m][nchunks][B][WC] (word-chunked scan)
    int m;                   // queries in this batch
    int q_bits, db_bits;     // bits per coordinate of the query codes and of the database codes
    int qsplit;              // queries per workgroup
    int qranges;             // ceil(m / qsplit)            (filled in by launch_scan)
    int row_blocks;          // row blocks of one workgroup (filled in by launch_scan)
    int W;                   // 32-bit words per plane
    int rows_per_lane;       // 1 or 2 (register-resident scan only)
    int wc;                  // words per chunk, 0 = register-resident scan
    int nchunks;             // ceil(W / wc)
    // threshold mode: a row passes when D < thr[q]; passing keys are appended to cand[q]
    const uint32_t* thr;     // [m]
    uint32_t* cnt;           // [m] number of keys appended (may exceed cap: overflow)
    uint64_t* cand;          // [m][cap]
    int cap;
    // dense mode: every D is stored
    uint32_t* dense;         // [m][dense_stride], column = row - row_begin
    int dense_stride;
    // threshold mode, optional (nullptr = off): count the passing rows of query q by distance
    // level: levels[q][0] for D < level_base[q], levels[q][D - level_base[q] + 1] otherwise.
    // The caller guarantees thr[q] - level_base[q] < level_stride.
    uint32_t* levels;        // [m][level_stride]
    const uint32_t* level_base;   // [m]
    int level_stride;
    // optional (nullptr = off): the launch does nothing when *run_flag == 0
    const uint32_t* run_flag;
};

// True if codes of W words per plane are served by the register-resident scan.
bool scan_is_resident(int W);
// True if the scan kernels are built for this pair of code widths.
bool scan_supports_bits(int q_bits, int db_bits);
// Chunk width the word-chunked scan uses for W words per plane.
int scan_chunk_words(int W);

hipError_t launch_scan(const ScanArgs& a, bool dense, hipStream_t s);

hipError_t launch_repack_queries(const uint32_t* q_rows, int m, int bits, int W, int wc,
                                 int nchunks, uint32_t* q_chunked, hipStream_t s);

hipError_t launch_encode(const float* X, int64_t n, int d, int bits, float scale, int layout,
                         uint32_t* codes, hipStream_t s);

struct SelectArgs {
    int m, k, d;
    int q_bits, db_bits;
    uint64_t* topk;          // [m][keep_max] best keys so far, ascending
    uint32_t* len;           // [m] keys held in topk[q]; unused (always k) when extra < 0
    int keep_max;            // row stride of topk: k for plain top-K, the candidate bound otherwise
    int extra;               // < 0: plain top-K.  >= 0: keep every key with D <= D_k + extra
                             // (Algorithm 1's candidate list), at most keep_max of them
    uint32_t* thr;           // [m] a later row is of interest when its D < thr[q]
    uint32_t* cnt;           // [m] survivors appended by the scan
    const uint64_t* cand;    // [m][cap]
    int cap;
    const uint32_t* dense;   // [m][dense_stride]
    int dense_stride;
    int64_t row_begin;       // first row of the group just scanned
    int rows;                // rows in the dense group
    int64_t n;               // rows in the database
    int64_t bundle_mul;      // as in ScanArgs
    int final_group;         // 1 = last group: plain mode also writes idx / score
    int32_t* idx;            // [m][k]
    int32_t* score;          // [m][k]
};

// Merge of one scanned group [row_begin, row_end) into the top-K; carries what the exact
// rescan of an overflowed query needs.
struct MergeArgs {
    const uint32_t* db;      // XBQ_BUNDLE64 codes
    int64_t n, row_begin, row_end;
    const uint32_t* q_rows;  // XBQ_ROWS codes of this batch
    int W;
    SelectArgs sel;
};

hipError_t launch_select_dense(const SelectArgs& a, hipStream_t s);
hipError_t launch_select_merge(const MergeArgs& a, hipStream_t s);

// Refine stage of Algorithm 1: exact fp32 inner products of the kept candidates with the
// query, sorted by similarity (descending, ties to the lower row); first k are written.
struct RefineArgs {
    const float* X_db;       // [n][d]
    const float* X_q;        // [m][d] (this batch)
    int m, k, d;
    const uint64_t* topk;    // [m][keep_max] candidate keys
    const uint32_t* len;     // [m]
    int keep_max;
    int32_t* idx;            // [m][k]
    float* sim;              // [m][k]
    int32_t* count;          // [m] candidates refined per query, or nullptr
};
hipError_t launch_refine(const RefineArgs& a, hipStream_t s);

// Cross-check scan with packed 4-bit dot products: see xbq_dot.hip.
struct DotArgs {
    const uint32_t* dbn;     // nibbles of the database rows, [bundles][WD][64]
    int64_t n, row_begin, row_end;
    const uint32_t* qn;      // nibbles of the queries, [m][WD]
    const int32_t* qsum;     // [m] sum of the query's nibble values
    int m, qsplit, qranges, row_blocks;
    int WD;                  // dwords of nibbles per row = 4 * W
    int rows_per_lane;
    int half_full_minus_d;   // (d (2^Bq - 1)(2^Bd - 1) - d) / 2
    const uint32_t* thr; uint32_t* cnt; uint64_t* cand; int cap;
    uint32_t* dense; int dense_stride;
};
hipError_t launch_scan_dot(const DotArgs& a, bool dense, hipStream_t s);
hipError_t launch_nibbles_db(const uint32_t* codes, int64_t n, int d, int bits, uint32_t* out, hipStream_t s);
hipError_t launch_nibbles_q(const uint32_t* codes, int m, int d, int bits, uint32_t* out, int32_t* vsum, hipStream_t s);

// Cross-check scan on the matrix cores (int8 MFMA): see xbq_mfma.hip.
struct MfmaArgs {
    const uint8_t* dbb;      // int8 rows of the database, [rows_padded][32 W]
    int64_t rows_padded;     // bundles * 64
    int64_t row_begin, row_end;   // row_begin a multiple of 32
    const uint8_t* qb;       // int8 rows of the queries, [m_padded][32 W]
    int m, m_padded;         // m_padded a multiple of 32
    int qsplit, qranges, row_blocks;   // qsplit a multiple of 32
    int W;
    int full;                // d (2^Bq - 1)(2^Bd - 1)
    const uint32_t* thr; uint32_t* cnt; uint64_t* cand; int cap;
    uint32_t* dense; int dense_stride;
};
hipError_t launch_scan_mfma(const MfmaArgs& a, bool dense, hipStream_t s);
hipError_t launch_bytes_db(const uint32_t* codes, int64_t n, int d, int bits, uint32_t* out, hipStream_t s);
hipError_t launch_bytes_q(const uint32_t* codes, int m, int m_pad, int d, int bits, uint32_t* out, hipStream_t s);

// Histogram selection (few queries): see xbq_hist.hip.
struct HistArgs {
    const uint32_t* db;      // XBQ_BUNDLE64 codes
    int64_t n;
    const uint32_t* q;       // [m][nchunks][q_bits][wc]
    int m;                   // 1..kHistMaxQueries
    int q_bits, db_bits;
    int W, wc, nchunks;
    uint32_t* dist;          // [m][n] distances, written
    uint32_t* hist;          // [m][kHistBins], zero on entry
    int shift;               // bin = D >> shift  (< kHistBins for every possible D)
};

struct CollectArgs {
    const uint32_t* dist;    // [m][n]
    const uint32_t* hist;    // [m][kHistBins]
    int64_t n;
    int m, k, d, q_bits, db_bits, shift;
    int rows_per_block;      // rows of dist one workgroup filters
    int blocks_per_query;    // ceil(n / rows_per_block)
    uint64_t* cand;          // [m][cand_cap]
    int cand_cap;            // kSortCap .. kHistCandCap (no more than the database has rows, rounded up)
    uint32_t* cand_cnt;      // [m], zero on entry
    int32_t* idx;            // [m][k]
    int32_t* score;          // [m][k]
};

hipError_t launch_clear(uint32_t* p, int64_t count, hipStream_t s);
hipError_t launch_scan_hist(const HistArgs& a, hipStream_t s);
hipError_t launch_hist_collect(const CollectArgs& a, hipStream_t s);

// Local selection (few queries, no stored distances): see xbq_local.hip.
struct LocalArgs {
    const uint32_t* db;      // XBQ_BUNDLE64 codes
    int64_t n;
    const uint32_t* q;       // [m][nchunks][q_bits][wc]
    int m;                   // 1..kLocalMaxQueries
    int q_bits, db_bits;
    int W, wc, nchunks;
    int k, d;
    int shift;               // piece histogram: bin = D >> shift  (< kHistBins for every possible D)
    int shift2;              // merge histogram: bin = D >> shift2 (< 4096 for every possible D)
    int cap;                 // keys per (piece, query) list: 4096
    int groups;              // pieces = workgroups of scan_local
    int64_t bundles_per_group;
    uint64_t* lists;         // [m][groups][list_stride]: the min(k, rows of the piece) best keys of every
                             // piece, ascending, written by scan_local
    int list_stride;         // >= k
    int len_full, len_last;  // list lengths: min(k, rows of a full piece), min(k, rows of the last piece)
    int prefix;              // keys of every list local_finish reads first: power of two, groups * prefix <= 32768
    int32_t* idx;            // [m][k]
    int32_t* score;          // [m][k]
};
size_t local_lds_bytes(int m, int cap);
hipError_t launch_scan_local(const LocalArgs& a, hipStream_t s);
hipError_t launch_local_finish(const LocalArgs& a, hipStream_t s);

// Algorithm 1 with the whole candidate list (xbq_kselect.hip), one batch of queries.
struct KSelectArgs {
    const uint32_t* db;      // XBQ_BUNDLE64 codes
    int64_t n;
    const uint32_t* q_rows;  // XBQ_ROWS codes of this batch
    int m, k, d, W;
    int q_bits, db_bits;
    int extra;               // 0 .. XBQ_MAX_EXTRA
    int cap;                 // candidate slots per query (>= k)
    // first stage, one of two forms:
    const int32_t* idx1;     // [m][k] exact top-K of the plain search (few queries), with score1
    const int32_t* score1;   // [m][k]
    const uint64_t* topk1;   // [m][keep1] sorted candidate keys of the bounded candidate search
    const uint32_t* len1;    // [m] keys held in topk1[q]; keep1 means the list may have been cut
    int keep1;
    uint64_t* best;          // [m][k] the K best keys by (D, row), written by the kselect_from_* kernels
    uint32_t* dk;            // [m] K-th smallest distance
    uint32_t* thr;           // [m] threshold of the collecting scan
    uint32_t* cnt;           // [m] rows within the bound (may exceed cap until kselect_levels ran)
    uint64_t* list;          // [m][cap] candidate keys, any order
    uint32_t* levels;        // [m][extra + 2] rows per distance level, counted by the collecting scan
    uint32_t* thr2;          // [m] threshold of the second collecting scan (0: query is done)
    uint32_t* flag;          // [2] set when some query needs the first / the second collecting scan
    const float* X_db;       // [n][d]
    const float* X_q;        // [m][d] (this batch)
    int parts;               // workgroups per query in refine_wide; parts * k <= kSortCap
    uint64_t* part_keys;     // [m][parts][k]
    int32_t* idx;            // [m][k]
    float* sim;              // [m][k]
    int32_t* count;          // [m] or nullptr
};
hipError_t launch_kselect_first(const KSelectArgs& a, hipStream_t s);
hipError_t launch_kselect_levels(const KSelectArgs& a, hipStream_t s);
// Collection from stored distances dist[m][n] (few queries); second = with the lowered bounds.
hipError_t launch_kselect_collect_stored(const KSelectArgs& a, const uint32_t* dist, bool second, hipStream_t s);
hipError_t launch_kselect_refine(const KSelectArgs& a, hipStream_t s);

// xbq_probe.hip: sustained-rate probes (measurement aids)
size_t probe_out_bytes();
double probe_valu_lane_ops(int iters);
hipError_t launch_probe_valu(uint32_t* out, uint32_t seed, int iters, hipStream_t s);
hipError_t launch_probe_read(const void* buf, size_t bytes, uint32_t* out, hipStream_t s);
hipError_t launch_probe_encode_traffic(const float* X, int64_t n, int d, int bits, uint32_t* codes, hipStream_t s);

}  // namespace xbq
