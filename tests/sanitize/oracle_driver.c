/*
 * Runs every C function of the oracle under AddressSanitizer + UndefinedBehaviorSanitizer (gcc,
 * CPU only) on small and ragged shapes with exactly sized heap buffers, so that an index past a
 * buffer, a signed overflow or a misaligned access in the oracle aborts the run.  A few results
 * are checked against values worked by hand; the numerical pins live in tests/test_oracle_*.py.
 * Compiled together with oracle/mquant_oracle.c by tests/test_sanitizers.py.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orc_num_threads(void);
void orc_fwht_block_f32(float *v, int32_t B);
void orc_hadamard_rows_f32(float *u, int64_t T, int64_t K, int32_t B);
void orc_msq_quantize(const float *u, int64_t T, int64_t K, int64_t V, float c_vis, float c_txt, int8_t *xq);
void orc_dyn_quantize(const float *u, int64_t T, int64_t K, double sqrt_b, int8_t *xq, float *s_rows);
void orc_dequant_rows_f32(const int32_t *acc, int64_t T, int64_t N, const float *s_rows, const float *w_scale, float *ref);
void orc_dequant_rms_f32(const int32_t *acc, const int8_t *xq, int64_t T, int64_t N, int64_t K, int64_t V, float s_vis,
                         float s_txt, const float *w_scale, const int32_t *split_idx, const int8_t *wsplit,
                         const float *ssplit, int64_t S, float *ref);
void orc_msq_quantize_bits(const float *u, int64_t T, int64_t K, int64_t V, float c_vis, float c_txt, int32_t bits, int8_t *xq);
float orc_absmax_f32(const float *u, int64_t n);
void orc_unpack_w4(const uint8_t *packed, int64_t N, int64_t K, int8_t *wq);
void orc_gemm_i8_i4_i32(const int8_t *xq, const int8_t *wq, int64_t T, int64_t N, int64_t K, int32_t *acc);
void orc_dequant_f32(const int32_t *acc, int64_t T, int64_t N, int64_t V, float s_vis, float s_txt, const float *w_scale, float *ref);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(1); } } while (0)

static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); CHECK(p != NULL); return p; }

int main(void)
{
    CHECK(orc_num_threads() >= 1);
    /* H_4 on (1,2,3,4): (10, -2, -4, 0) */
    {
        float *v = xmalloc(4 * sizeof(float));
        v[0] = 1; v[1] = 2; v[2] = 3; v[3] = 4;
        orc_fwht_block_f32(v, 4);
        CHECK(v[0] == 10 && v[1] == -2 && v[2] == -4 && v[3] == 0);
        free(v);
    }
    const int32_t blocks[] = {1, 2, 8, 64, 512, 1024};
    for (size_t bi = 0; bi < sizeof(blocks) / sizeof(blocks[0]); ++bi) {
        const int32_t B = blocks[bi];
        const int64_t T = 3, K = (int64_t)B * 3;
        float *u = xmalloc((size_t)(T * K) * sizeof(float)), *w = xmalloc((size_t)(T * K) * sizeof(float));
        for (int64_t i = 0; i < T * K; ++i) u[i] = w[i] = (float)((int)(rnd() % 17) - 8);
        orc_hadamard_rows_f32(u, T, K, B);
        orc_hadamard_rows_f32(u, T, K, B);                       /* involution: B * x on small integers */
        for (int64_t i = 0; i < T * K; ++i) CHECK(u[i] == (float)B * w[i]);
        CHECK(orc_absmax_f32(w, T * K) <= 8.0f);
        int8_t *xq = xmalloc((size_t)(T * K)), *xq4 = xmalloc((size_t)(T * K));
        float *s_rows = xmalloc((size_t)T * sizeof(float));
        orc_msq_quantize(w, T, K, 1, 0.5f, 100.0f, xq);          /* second scale saturates */
        orc_msq_quantize_bits(w, T, K, 2, 0.5f, 100.0f, 4, xq4);
        orc_dyn_quantize(w, T, K, 1.0, xq, s_rows);
        for (int64_t i = 0; i < T * K; ++i) CHECK(xq4[i] >= -8 && xq4[i] <= 7);
        free(u); free(w); free(xq); free(xq4); free(s_rows);
    }
    /* integer GEMM, ragged shapes incl. a single row/column and the extreme values */
    const int64_t shapes[][3] = {{1, 1, 2}, {2, 3, 4}, {5, 7, 64}, {3, 33, 130}, {4, 2, 29568}};
    for (size_t si = 0; si < sizeof(shapes) / sizeof(shapes[0]); ++si) {
        const int64_t T = shapes[si][0], N = shapes[si][1], K = shapes[si][2];
        uint8_t *packed = xmalloc((size_t)(N * K / 2));
        int8_t *wq = xmalloc((size_t)(N * K)), *xq = xmalloc((size_t)(T * K));
        int32_t *acc = xmalloc((size_t)(T * N) * sizeof(int32_t));
        float *ws = xmalloc((size_t)N * sizeof(float)), *ref = xmalloc((size_t)(T * N) * sizeof(float));
        float *s_rows = xmalloc((size_t)T * sizeof(float));
        for (int64_t i = 0; i < N * K / 2; ++i) packed[i] = si == 4 ? 0x88 : (uint8_t)rnd();
        for (int64_t i = 0; i < T * K; ++i) xq[i] = si == 4 ? -128 : (int8_t)rnd();
        for (int64_t n = 0; n < N; ++n) ws[n] = 0.01f;
        for (int64_t t = 0; t < T; ++t) s_rows[t] = 0.5f;
        orc_unpack_w4(packed, N, K, wq);
        orc_gemm_i8_i4_i32(xq, wq, T, N, K, acc);
        if (si == 4) CHECK(acc[0] == 29568 * 1024);
        int64_t want = 0;                                        /* one element by a plain loop */
        for (int64_t k = 0; k < K; ++k) want += (int64_t)xq[(T - 1) * K + k] * wq[(N - 1) * K + k];
        CHECK(acc[(T - 1) * N + N - 1] == (int32_t)want);
        orc_dequant_f32(acc, T, N, T / 2, 0.3f, 0.02f, ws, ref);
        orc_dequant_rows_f32(acc, T, N, s_rows, ws, ref);
        const int64_t S = K >= 4 ? 2 : 1;
        int32_t *idx = xmalloc((size_t)S * sizeof(int32_t));
        int8_t *wsplit = xmalloc((size_t)(S * N));
        float *ssplit = xmalloc((size_t)S * sizeof(float));
        for (int64_t j = 0; j < S; ++j) { idx[j] = (int32_t)(j * (K - 1)); ssplit[j] = 0.1f; }
        for (int64_t i = 0; i < S * N; ++i) wsplit[i] = (int8_t)((int)(rnd() % 16) - 8);
        orc_dequant_rms_f32(acc, xq, T, N, K, T / 2, 0.3f, 0.02f, ws, idx, wsplit, ssplit, S, ref);
        orc_dequant_rms_f32(acc, xq, T, N, K, T / 2, 0.3f, 0.02f, ws, idx, wsplit, ssplit, 0, ref);
        free(packed); free(wq); free(xq); free(acc); free(ws); free(ref); free(s_rows); free(idx); free(wsplit); free(ssplit);
    }
    printf("oracle sanitizer run ok\n");
    return 0;
}
