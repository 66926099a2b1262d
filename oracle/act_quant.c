/*
 * CPU oracle for the multi-LoRA int4 linear layer with int8 activations.  TEST INFRASTRUCTURE
 * ONLY: plain loops, shares no code with the HIP library and is never called by it.
 *
 * Section 3.3 of the paper: activations are quantised to int8 with ONE scale per tensor, weights
 * to int4.  With xq the int8 rows and s_x their scale, the activation is s_x * xq[m][k], and the
 * layer of Section 3.1, Eq. 1-4 on it is
 *
 *   y[m][n] = s_x * (  sum over groups g of  scale[n][g] * sum_{k in g} code[n][k] * xq[m][k]
 *                    + alpha * sum_j B[a(m)][n][j] * sum_k A[a(m)][j][k] * xq[m][k] )
 *
 * The inner sums over integers are taken in int64 (exact); everything else in double.  LoRA
 * tensors are bf16 as in oracle.c (the paper's int16 LoRA is not modelled).
 *
 * The quantiser (an input recipe: the paper fixes scales offline; symmetric, no zero point):
 * s_x = max|x| / 127 computed in float32 (1 if the tensor is all zero), xq = x / s_x rounded to
 * nearest, ties to even, clamped to [-127, 127].
 *
 * Pinned by tests/test_act_quant_oracle.py: equality with oracle.c's linear on s_x * xq when s_x
 * is a power of two (then s_x * xq is exact in bf16), numpy int64 products for unit scales,
 * rounding and range cases of the quantiser.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

double orc_bf16_to_double(uint16_t b);   /* oracle.c: exact widenings */
double orc_f16_to_double(uint16_t h);

static int code_of(const uint8_t *wq, int32_t K, int32_t n, int32_t k)
{
    const uint8_t byte = wq[(size_t)n * (K / 2) + k / 2];
    const unsigned nib = (k % 2 == 0) ? (byte & 0x0Fu) : (byte >> 4);
    return nib < 8 ? (int)nib : (int)nib - 16;          /* two's-complement nibble */
}

void orc_linear_a8(int32_t K, int32_t N, int32_t G,
                   const uint8_t *wq, const uint16_t *scales,
                   int32_t rank, const uint16_t *lora_a, const uint16_t *lora_b, double alpha,
                   const int8_t *xq, double x_scale, const int32_t *row_adapter, int32_t M,
                   double *y)
{
    double *t = (double *)calloc((size_t)M * (rank > 0 ? rank : 1), sizeof(double));
    for (int32_t m = 0; m < M; ++m) {
        const int32_t a = row_adapter ? row_adapter[m] : -1;
        if (a < 0) continue;
        for (int32_t j = 0; j < rank; ++j) {
            const uint16_t *arow = lora_a + ((size_t)a * rank + j) * K;
            double s = 0.0;
            for (int32_t k = 0; k < K; ++k) s += orc_bf16_to_double(arow[k]) * (double)xq[(size_t)m * K + k];
            t[(size_t)m * rank + j] = s;
        }
    }
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n)
        for (int32_t m = 0; m < M; ++m) {
            double base = 0.0;
            for (int32_t g = 0; g < K / G; ++g) {
                int64_t isum = 0;
                for (int32_t k = g * G; k < (g + 1) * G; ++k)
                    isum += (int64_t)code_of(wq, K, n, k) * (int64_t)xq[(size_t)m * K + k];
                base += orc_f16_to_double(scales[(size_t)n * (K / G) + g]) * (double)isum;
            }
            const int32_t a = row_adapter ? row_adapter[m] : -1;
            if (a >= 0) {
                const uint16_t *brow = lora_b + ((size_t)a * N + n) * rank;
                double lora = 0.0;
                for (int32_t j = 0; j < rank; ++j) lora += orc_bf16_to_double(brow[j]) * t[(size_t)m * rank + j];
                base += alpha * lora;
            }
            y[(size_t)m * N + n] = x_scale * base;
        }
    free(t);
}

/* returns the scale; xq gets count int8 values */
float orc_quantise_act(const float *x, size_t count, int8_t *xq)
{
    float top = 0.0f;
    for (size_t i = 0; i < count; ++i) {
        const float v = fabsf(x[i]);
        if (v > top) top = v;
    }
    const float scale = top > 0.0f ? top / 127.0f : 1.0f;
    for (size_t i = 0; i < count; ++i) {
        float q = nearbyintf(x[i] / scale);             /* default rounding mode: ties to even */
        if (q > 127.0f) q = 127.0f;
        if (q < -127.0f) q = -127.0f;
        xq[i] = (int8_t)q;
    }
    return scale;
}
