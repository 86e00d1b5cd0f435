/*
 * CPU oracle for the MQuant W4A8 linear hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C.  Nothing here is shared with the HIP
 * library: no common header, table, helper or constant generator.  Only the
 * tests, the smoke check and the cpu_baseline leg of the benchmark may load
 * the shared object built from this file.
 *
 * Every function follows one passage of the MQuant paper (arXiv 2502.00425):
 *   - uniform signed quantizer ...................... Sec. 2.2, Eq. (2)
 *   - modality-specific static scales (MSQ) ......... Sec. 3.1, Eq. (3)
 *   - Walsh-Hadamard matrix H_{2^n} = H_2 (x) H_{2^{n-1}}  Appendix "Weights
 *     Outliers after Online Hadamard Transformation"
 *   - per-token dynamic quantization (baseline) ...... Sec. 2.2, appendix on
 *     quantization granularity
 *   - Rotation Magnitude Suppression, run-time split path .. Sec. 3.2
 *   - W4A8 integer GEMM with per-channel weight scale and per-modality
 *     activation scale ................................ Sec. 4 (Table 3 text,
 *     "Speedup" paragraphs)
 *
 * Floating point: the online Hadamard transform is evaluated in IEEE fp32,
 * one rounding per add/sub, in the fixed stage order h = 1, 2, 4, ..., B/2.
 * The paper is silent on precision and summation order; this ordering is the
 * reading that decides the int8 codes, so any other implementation that wants
 * bit-identical codes has to use the same order.  Build with
 * -ffp-contract=off and without -ffast-math.
 *
 * The only parallelism is an OpenMP "parallel for" over independent rows, so
 * that the oracle can be timed on all host cores.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * In-place unnormalised Walsh-Hadamard transform of one block of B floats
 * (B a power of two): v <- v * H_B with H_B the +-1 Sylvester matrix, i.e. the
 * Kronecker recursion of the appendix without its 1/sqrt(2) factors.  Stage h
 * combines elements whose indices differ in bit h; the lower index receives
 * the sum, the upper the difference.
 */
void orc_fwht_block_f32(float *v, int32_t B)
{
    for (int32_t h = 1; h < B; h <<= 1) {
        for (int32_t j = 0; j < B; ++j) {
            if ((j & h) == 0) {
                float a = v[j];
                float b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

/*
 * Block-diagonal rotation of a row-major [T,K] fp32 matrix, in place:
 * every contiguous block of B channels of every row is transformed on its own
 * (I_{K/B} (x) H_B).  B == 1 leaves the data untouched.
 */
void orc_hadamard_rows_f32(float *u, int64_t T, int64_t K, int32_t B)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        for (int64_t k0 = 0; k0 < K; k0 += B) {
            orc_fwht_block_f32(u + i * K + k0, B);
        }
    }
}

/*
 * Eq. (2) with z = 0 and a static scale, Eq. (3) for the scale choice:
 * rows [0,V) are visual and use multiplier c_vis, rows [V,T) are text and use
 * c_txt, where c = fp32( 1 / (s * sqrt(B)) ) folds the orthonormal 1/sqrt(B)
 * of the rotation into the division by the scale.  One fp32 multiply, round
 * half to even, clamp to the int8 range.
 */
void orc_msq_quantize(const float *u, int64_t T, int64_t K, int64_t V,
                      float c_vis, float c_txt, int8_t *xq)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        const float c = (i < V) ? c_vis : c_txt;
        for (int64_t k = 0; k < K; ++k) {
            float t = u[i * K + k] * c;
            float r = nearbyintf(t);          /* default mode: ties to even */
            if (r < -128.0f) r = -128.0f;
            if (r > 127.0f) r = 127.0f;
            xq[i * K + k] = (int8_t)r;
        }
    }
}

/*
 * Per-token dynamic quantization (Sec. 2.2: the scale of Eq. (2) taken from
 * runtime statistics; appendix on quantization granularity: one scale per
 * token).  The comparison baseline of the speed tables, not MQuant's own path.
 * For every row i of the unnormalised rotation u:
 *     a_i = max_k |u[i,k]|
 *     s_i = fp32( a_i / sqrt(B) / 127 )            Eq. (2): max|x| / (2^{b-1}-1)
 *     c_i = fp32( 1 / (s_i sqrt(B)) )              same folding as the static path
 *     xq[i,k] = clamp(rne(u[i,k] * c_i), -128, 127)
 * both scalars evaluated in double and rounded once.  The paper does not say
 * what an all-zero token gets: here s_i = 1 and every code is 0.
 */
void orc_dyn_quantize(const float *u, int64_t T, int64_t K, double sqrt_b,
                      int8_t *xq, float *s_rows)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        float a = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float v = fabsf(u[i * K + k]);
            if (v > a) a = v;
        }
        float s = 1.0f, c = 1.0f;
        if (a > 0.0f) {
            s = (float)((double)a / sqrt_b / 127.0);
            c = (float)(1.0 / ((double)s * sqrt_b));
        }
        s_rows[i] = s;
        for (int64_t k = 0; k < K; ++k) {
            float t = u[i * K + k] * c;
            float r = nearbyintf(t);
            if (r < -128.0f) r = -128.0f;
            if (r > 127.0f) r = 127.0f;
            xq[i * K + k] = (int8_t)r;
        }
    }
}

/* Dequantisation with one activation scale per token ("per token scale" of the
 * scheme-comparison table): ref[i,n] = (float(acc[i,n]) * s_rows[i]) * w_scale[n]. */
void orc_dequant_rows_f32(const int32_t *acc, int64_t T, int64_t N,
                          const float *s_rows, const float *w_scale, float *ref)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        for (int64_t n = 0; n < N; ++n) {
            float a = (float)acc[i * N + n];
            ref[i * N + n] = (a * s_rows[i]) * w_scale[n];
        }
    }
}

/*
 * Rotation Magnitude Suppression at run time (Sec. 3.2, "Rotation Mitigation
 * Scheme"; figure "overview of RMS"): the flagged input channels c_0..c_{S-1}
 * have their rows zeroed in the main int4 weight, so acc holds the main GEMM
 * only; each flagged row lives on as a separate int4 vector wsplit[j][0..N)
 * with one scale ssplit[j] and is applied as a GEMV on the same int8 codes,
 * its partial output added to the main path before the result is stored:
 *   ref[i,n] = (float(acc[i,n]) s_i) w_scale[n]
 *              + sum_j (float(xq[i,c_j] * wsplit[j][n]) s_i) ssplit[j]
 * accumulated in fp32 in the order j = 0, 1, ..., one rounding per operation.
 * The paper fixes neither the split row's quantization granularity nor the
 * order of the additions; one scale per split row and this order are the
 * reading taken here.
 */
void orc_dequant_rms_f32(const int32_t *acc, const int8_t *xq, int64_t T, int64_t N, int64_t K,
                         int64_t V, float s_vis, float s_txt, const float *w_scale,
                         const int32_t *split_idx, const int8_t *wsplit, const float *ssplit,
                         int64_t S, float *ref)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        const float s = (i < V) ? s_vis : s_txt;
        for (int64_t n = 0; n < N; ++n) {
            float v = ((float)acc[i * N + n] * s) * w_scale[n];
            for (int64_t j = 0; j < S; ++j) {
                int32_t p = (int32_t)xq[i * K + split_idx[j]] * (int32_t)wsplit[j * N + n];
                v = v + ((float)p * s) * ssplit[j];
            }
            ref[i * N + n] = v;
        }
    }
}

/*
 * Eq. (2)/(3) at another activation bit-width b (the W4A4 setting of the
 * accuracy tables: b = 4, codes in [-8, 7]): as orc_msq_quantize with the clamp
 * range [-2^(b-1), 2^(b-1)-1].  The codes still occupy one int8 each.
 */
void orc_msq_quantize_bits(const float *u, int64_t T, int64_t K, int64_t V,
                           float c_vis, float c_txt, int32_t bits, int8_t *xq)
{
    const float hi = (float)((1 << (bits - 1)) - 1), lo = -(float)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        const float c = (i < V) ? c_vis : c_txt;
        for (int64_t k = 0; k < K; ++k) {
            float r = nearbyintf(u[i * K + k] * c);
            if (r < lo) r = lo;
            if (r > hi) r = hi;
            xq[i * K + k] = (int8_t)r;
        }
    }
}

/* max |u| over a [T,K] fp32 matrix (calibration statistic, Eq. (2)'s max|x|). */
float orc_absmax_f32(const float *u, int64_t n)
{
    float m = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(u[i]);
        if (a > m) m = a;
    }
    return m;
}

/*
 * Canonical int4 storage: byte (n*K/2 + k/2) holds channel k of output row n
 * in its low nibble when k is even and in its high nibble when k is odd; a
 * nibble is a 4-bit two's-complement integer in [-8,7].
 */
void orc_unpack_w4(const uint8_t *packed, int64_t N, int64_t K, int8_t *wq)
{
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = packed[n * (K / 2) + k / 2];
            int nib = (k & 1) ? (byte >> 4) : (byte & 0x0F);
            if (nib >= 8) nib -= 16;
            wq[n * K + k] = (int8_t)nib;
        }
    }
}

/* acc[i,n] = sum_k xq[i,k] * wq[n,k], exact in int32. */
void orc_gemm_i8_i4_i32(const int8_t *xq, const int8_t *wq,
                        int64_t T, int64_t N, int64_t K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) {
                s += (int32_t)xq[i * K + k] * (int32_t)wq[n * K + k];
            }
            acc[i * N + n] = s;
        }
    }
}

/*
 * Dequantisation: ref[i,n] = (float(acc) * s_i) * w_scale[n] in fp32 with
 * s_i = s_vis for rows below V and s_txt otherwise (Eq. (3)); the per-channel
 * weight scale is the one Algorithm 1 outputs.
 */
void orc_dequant_f32(const int32_t *acc, int64_t T, int64_t N, int64_t V,
                     float s_vis, float s_txt, const float *w_scale, float *ref)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        const float s = (i < V) ? s_vis : s_txt;
        for (int64_t n = 0; n < N; ++n) {
            float a = (float)acc[i * N + n];
            ref[i * N + n] = (a * s) * w_scale[n];
        }
    }
}
