/*
 * Scale-level CPU oracle for XOR-friendly binary quantized top-K search.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain scalar C, one obvious loop per formula, no
 * blocking, no SIMD intrinsics beyond the compiler's 64-bit popcount.  It shares
 * no code, header, table or memory layout with the HIP library and is pinned
 * against the definition-level Python oracle.  It is also the program timed as
 * the CPU baseline, exactly as it stands.
 *
 * Steps and the passages they follow:
 *   quantize : Section 3.2 (f_B by successive approximation, sign(0) = +1),
 *              after the binary32 scaling of Section 3.5
 *   pack     : Section 3.3, Eq. 9 (bit-plane b of a vector as one integer,
 *              coordinate 0 at the least significant bit), stored in 64-bit
 *              words as in Section 4.1 "Quantization"
 *   distance : Section 3.3, Eq. 10 (sum_i sum_j POPCNT(xhat_i ^ yhat_j) << (i+j))
 *   score    : numerator of Section 3.3, Eq. 7:  S = d(2^Bq-1)(2^Bd-1) - 2 D
 *   top-K    : Section 2 problem statement (K most similar, descending), ties
 *              to the lower index, by bounded sorted insertion
 *
 * Layout used here only: planes[n][B][W64] row-major uint64, W64 = ceil(d/64).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int xfbq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Section 3.2: code of one already-scaled value t.  Bit = 1 means digit -1. */
static unsigned quantize_one(float t, int B)
{
    double partial = 0.0;   /* f_i(t): a multiple of 2^-B, exact */
    double step = 0.5;
    unsigned code = 0;
    for (int i = 0; i < B; ++i) {
        if ((double)t >= partial) {          /* digit +1, stored bit 0 */
            code = (code << 1);
            partial += step;
        } else {                             /* digit -1, stored bit 1 */
            code = (code << 1) | 1u;
            partial -= step;
        }
        step *= 0.5;
    }
    return code;
}

/* X[n][d] fp32 -> codes[n][d] uint8.  The scaling is one binary32 multiply. */
void xfbq_oracle_quantize(const float *X, int64_t n, int d, int B, float scale,
                          uint8_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) {
        for (int k = 0; k < d; ++k) {
            volatile float t = X[r * d + k] * scale;   /* rounded to binary32 */
            codes[r * d + k] = (uint8_t)quantize_one(t, B);
        }
    }
}

/* codes[n][d] -> planes[n][B][W64]; pad bits stay zero. */
void xfbq_oracle_pack(const uint8_t *codes, int64_t n, int d, int B, uint64_t *planes)
{
    const int W64 = (d + 63) / 64;
    memset(planes, 0, (size_t)n * B * W64 * sizeof(uint64_t));
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) {
        for (int b = 0; b < B; ++b) {
            for (int k = 0; k < d; ++k) {
                uint64_t bit = (codes[r * d + k] >> b) & 1u;
                planes[(r * B + b) * W64 + k / 64] |= bit << (k % 64);
            }
        }
    }
}

/* Eq. 10 of Section 3.3 (the POPCNT form) for one pair. */
static int64_t distance_pair(const uint64_t *x, int Bx, const uint64_t *y, int By, int W64)
{
    int64_t D = 0;
    for (int i = 0; i < Bx; ++i) {
        for (int j = 0; j < By; ++j) {
            int64_t pc = 0;
            for (int w = 0; w < W64; ++w)
                pc += __builtin_popcountll(x[i * W64 + w] ^ y[j * W64 + w]);
            D += pc << (i + j);
        }
    }
    return D;
}

static int64_t score_pair(const uint64_t *q, int Bq, const uint64_t *x, int Bd, int W64, int d)
{
    const int64_t full = (int64_t)d * ((1 << Bq) - 1) * ((1 << Bd) - 1);
    return full - 2 * distance_pair(q, Bq, x, Bd, W64);
}

/* All scores, S[m][n] int32 (for medium-size tests). */
void xfbq_oracle_scores(const uint64_t *db, int64_t n, int Bd, const uint64_t *q, int64_t m,
                        int Bq, int d, int32_t *S)
{
    const int W64 = (d + 63) / 64;
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < m; ++a)
        for (int64_t r = 0; r < n; ++r)
            S[a * n + r] = (int32_t)score_pair(q + a * Bq * W64, Bq, db + r * Bd * W64, Bd, W64, d);
}

/* Scores of listed pairs: S[t] = score(query qi[t], row ri[t]). */
void xfbq_oracle_scores_at(const uint64_t *db, int Bd, const uint64_t *q, int Bq, int d,
                           const int64_t *qi, const int64_t *ri, int64_t count, int32_t *S)
{
    const int W64 = (d + 63) / 64;
    for (int64_t t = 0; t < count; ++t)
        S[t] = (int32_t)score_pair(q + qi[t] * Bq * W64, Bq, db + ri[t] * Bd * W64, Bd, W64, d);
}

/* 1 if (s1, i1) ranks before (s2, i2): larger score first, then lower index. */
static int ranks_before(int64_t s1, int64_t i1, int64_t s2, int64_t i2)
{
    return s1 > s2 || (s1 == s2 && i1 < i2);
}

/*
 * Top-K of every query over all n rows.  idx[m][K], score[m][K], sorted by
 * (score desc, idx asc).  Returns 0, or -1 on bad arguments.
 */
int xfbq_oracle_search(const uint64_t *db, int64_t n, int Bd, const uint64_t *q, int64_t m,
                       int Bq, int d, int K, int32_t *idx, int32_t *score)
{
    if (K < 1 || K > n || n < 1 || m < 0) return -1;
    const int W64 = (d + 63) / 64;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t a = 0; a < m; ++a) {
        int32_t *bi = idx + a * K;
        int32_t *bs = score + a * K;
        int have = 0;
        for (int64_t r = 0; r < n; ++r) {
            int64_t s = score_pair(q + a * Bq * W64, Bq, db + r * Bd * W64, Bd, W64, d);
            if (have == K && !ranks_before(s, r, bs[K - 1], bi[K - 1])) continue;
            int pos = have < K ? have : K - 1;       /* slot that is free or dropped */
            while (pos > 0 && ranks_before(s, r, bs[pos - 1], bi[pos - 1])) {
                bs[pos] = bs[pos - 1];
                bi[pos] = bi[pos - 1];
                --pos;
            }
            bs[pos] = (int32_t)s;
            bi[pos] = (int32_t)r;
            if (have < K) ++have;
        }
    }
    return 0;
}
