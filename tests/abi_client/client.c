/* A caller of libxbq.so written in plain C: no Python, no PyTorch, device memory straight from
 * the HIP runtime.  Encodes a small database and a few queries, searches, and compares codes
 * and results bit for bit with the plain-C oracle (test infrastructure, linked only here).
 * Build: see tests/test_gpu_c_client.py.  Prints "abi client ok" and exits 0 on success. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "xbq.h"

void xfbq_oracle_quantize(const float *X, int64_t n, int d, int B, float scale, uint8_t *codes);
void xfbq_oracle_pack(const uint8_t *codes, int64_t n, int d, int B, uint64_t *planes);
int xfbq_oracle_search(const uint64_t *db, int64_t n, int Bd, const uint64_t *q, int64_t m, int Bq, int d, int K,
                       int32_t *idx, int32_t *score);

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_XBQ(x) do { int r_ = (x); if (r_ != XBQ_OK) { fprintf(stderr, "xbq error %d (%s) at line %d\n", r_, xbq_strerror(r_), __LINE__); return 3; } } while (0)

static uint32_t lcg_state = 12345u;
static float next_unit(void)                     /* uniform in (-0.5, 0.5), 24 random bits */
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)(lcg_state >> 8) / 16777216.0f - 0.5f;
}

int main(void)
{
    const int64_t n = 5003, m = 37;
    const int d = 96, bits = 4, k = 10;
    const float scale = 1.9f;
    const int W = (d + 31) / 32, W64 = (d + 63) / 64;
    float *X = malloc(sizeof(float) * n * d), *Q = malloc(sizeof(float) * m * d);
    for (int64_t i = 0; i < n * d; ++i) X[i] = next_unit();
    for (int64_t i = 0; i < m * d; ++i) Q[i] = next_unit();

    /* the GPU path through the C ABI */
    const size_t db_bytes = xbq_code_bytes(n, d, bits, XBQ_BUNDLE64), q_bytes = xbq_code_bytes(m, d, bits, XBQ_ROWS);
    const size_t ws_bytes = xbq_search_workspace_bytes(n, m, d, bits, k);
    if (!db_bytes || !q_bytes || !ws_bytes) { fprintf(stderr, "size query failed\n"); return 4; }
    float *dX, *dQ; uint32_t *dDb, *dQc; int32_t *dIdx, *dScore; void *dWs;
    CHECK_HIP(hipMalloc((void **)&dX, sizeof(float) * n * d));
    CHECK_HIP(hipMalloc((void **)&dQ, sizeof(float) * m * d));
    CHECK_HIP(hipMalloc((void **)&dDb, db_bytes));
    CHECK_HIP(hipMalloc((void **)&dQc, q_bytes));
    CHECK_HIP(hipMalloc((void **)&dIdx, sizeof(int32_t) * m * k));
    CHECK_HIP(hipMalloc((void **)&dScore, sizeof(int32_t) * m * k));
    CHECK_HIP(hipMalloc(&dWs, ws_bytes));
    CHECK_HIP(hipMemcpy(dX, X, sizeof(float) * n * d, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dQ, Q, sizeof(float) * m * d, hipMemcpyHostToDevice));
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_XBQ(xbq_encode(dX, n, d, bits, scale, XBQ_BUNDLE64, dDb, stream));
    CHECK_XBQ(xbq_encode(dQ, m, d, bits, scale, XBQ_ROWS, dQc, stream));
    CHECK_XBQ(xbq_search(dDb, n, dQc, m, d, bits, k, dIdx, dScore, dWs, ws_bytes, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    int32_t *idx = malloc(sizeof(int32_t) * m * k), *score = malloc(sizeof(int32_t) * m * k);
    uint32_t *qc = malloc(q_bytes);
    CHECK_HIP(hipMemcpy(idx, dIdx, sizeof(int32_t) * m * k, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(score, dScore, sizeof(int32_t) * m * k, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(qc, dQc, q_bytes, hipMemcpyDeviceToHost));

    /* the oracle */
    uint8_t *cx = malloc((size_t)n * d), *cq = malloc((size_t)m * d);
    uint64_t *px = malloc(sizeof(uint64_t) * n * bits * W64), *pq = malloc(sizeof(uint64_t) * m * bits * W64);
    int32_t *ridx = malloc(sizeof(int32_t) * m * k), *rscore = malloc(sizeof(int32_t) * m * k);
    xfbq_oracle_quantize(X, n, d, bits, scale, cx);
    xfbq_oracle_quantize(Q, m, d, bits, scale, cq);
    xfbq_oracle_pack(cx, n, d, bits, px);
    xfbq_oracle_pack(cq, m, d, bits, pq);
    if (xfbq_oracle_search(px, n, bits, pq, m, bits, d, k, ridx, rscore) != 0) { fprintf(stderr, "oracle failed\n"); return 5; }

    /* query codes: 32-bit word w of plane b is half (w & 1) of the oracle's 64-bit word w / 2 */
    for (int64_t r = 0; r < m; ++r)
        for (int b = 0; b < bits; ++b)
            for (int w = 0; w < W; ++w) {
                const uint64_t w64 = pq[(r * bits + b) * W64 + w / 2];
                const uint32_t want = (uint32_t)(w & 1 ? w64 >> 32 : w64);
                if (qc[(r * bits + b) * W + w] != want) { fprintf(stderr, "code mismatch at query %lld plane %d word %d\n", (long long)r, b, w); return 6; }
            }
    if (memcmp(idx, ridx, sizeof(int32_t) * m * k) != 0) { fprintf(stderr, "row numbers differ from the oracle\n"); return 7; }
    if (memcmp(score, rscore, sizeof(int32_t) * m * k) != 0) { fprintf(stderr, "scores differ from the oracle\n"); return 8; }
    printf("abi client ok: n=%lld d=%d m=%lld bits=%d k=%d, version %d\n", (long long)n, d, (long long)m, bits, k, xbq_version());
    return 0;
}
