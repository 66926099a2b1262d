/*
 * CPU oracle for the multi-LoRA int4 linear layer.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain nested loops in fp64, written from the paper's definition; shares no
 * code, header, table or helper with the HIP library and is never called by it.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes (paper Section 3.1, Eq. 1-4, rewritten column-wise; the
 * paper's row-vector form is Y = XW + X(sAB)):
 *
 *   w[n][k] = code[n][k] * scale[n][k / G]                       (Section 3.3, int4 weights)
 *   t[m][j] = sum_k A[a][j][k] * x[m][k]          a = row_adapter[m]
 *   y[m][n] = sum_k w[n][k] * x[m][k] + alpha * sum_j B[a][n][j] * t[m][j]
 *
 * with the LoRA tensors supplied as call arguments of identical shape for all
 * adapters (Section 3.2, approach c; Limitations) and a == -1 meaning "base
 * model only" (the "Base" columns of Tables 1-2).  alpha is the paper's scale
 * factor s: a direct multiplier.
 *
 * Encodings: bf16 / fp16 values arrive as uint16 bit patterns and are widened
 * exactly; packed codes are uint8 [N][K/2], even k in the low nibble, each
 * nibble a two's-complement 4-bit integer in [-8, 7].
 *
 * Every function here is pinned by tests/test_oracle_pins.py (closed forms,
 * integer-exact cases, numpy's float64 matmul on the dequantised matrix,
 * merged-weight brute force, brute-force sorting).  The paper prints no value
 * of any y, so whole-model numbers stay unpinned; nothing here depends on them.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- exact widening of 16-bit floats ------------------------------------------------ */

double orc_bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;   /* bf16 is the top half of an IEEE binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

double orc_f16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (e == 0)        v = ldexp((double)frac, -24);               /* zero / subnormal */
    else if (e == 31)  v = frac ? NAN : INFINITY;
    else               v = ldexp(1.0 + (double)frac / 1024.0, e - 15);
    return sign ? -v : v;
}

/* float32 -> fp16 bits, round to nearest even (used by the reference quantiser only) */
uint16_t orc_f32_to_f16(float f)
{
    if (isnan(f)) return 0x7E00;
    uint16_t sign = signbit(f) ? 0x8000 : 0;
    double a = fabs((double)f);
    if (a >= 65520.0) return sign | 0x7C00;          /* rounds to infinity */
    if (a < ldexp(1.0, -25)) return sign;             /* below half the smallest subnormal */
    int e;
    (void)frexp(a, &e);                               /* a = m * 2^e, m in [0.5,1) */
    int exp = e - 1;                                  /* a = 1.x * 2^exp */
    if (exp < -14) exp = -14;                         /* subnormal range: fixed quantum 2^-24 */
    double q = ldexp(a, 10 - exp);                    /* in units of the fp16 quantum */
    double r = nearbyint(q);                          /* default mode: ties to even */
    /* r in [0, 2048]; r == 2048 carries into the next binade, which the
       addition below handles because the exponent field sits just above. */
    uint32_t bits;
    if (exp == -14 && r < 1024.0) bits = (uint32_t)r;                 /* subnormal */
    else bits = ((uint32_t)(exp + 15) << 10) + ((uint32_t)r - 1024u);
    return sign | (uint16_t)bits;
}

/* ---- int4 codes ---------------------------------------------------------------------- */

static int nibble_to_code(unsigned nib) { return (nib & 8u) ? (int)nib - 16 : (int)nib; }

void orc_unpack_codes(const uint8_t *wq, int32_t N, int32_t K, int8_t *codes)
{
    for (int32_t n = 0; n < N; ++n)
        for (int32_t k = 0; k < K; ++k) {
            uint8_t byte = wq[(size_t)n * (K / 2) + k / 2];
            unsigned nib = (k % 2 == 0) ? (byte & 0x0Fu) : (byte >> 4);
            codes[(size_t)n * K + k] = (int8_t)nibble_to_code(nib);
        }
}

void orc_pack_codes(const int8_t *codes, int32_t N, int32_t K, uint8_t *wq)
{
    for (int32_t n = 0; n < N; ++n)
        for (int32_t k = 0; k < K; k += 2) {
            unsigned lo = (unsigned)codes[(size_t)n * K + k] & 0x0Fu;
            unsigned hi = (unsigned)codes[(size_t)n * K + k + 1] & 0x0Fu;
            wq[(size_t)n * (K / 2) + k / 2] = (uint8_t)(lo | (hi << 4));
        }
}

void orc_dequant(const uint8_t *wq, const uint16_t *scales, int32_t N, int32_t K, int32_t G,
                 double *w)
{
    for (int32_t n = 0; n < N; ++n)
        for (int32_t k = 0; k < K; ++k) {
            uint8_t byte = wq[(size_t)n * (K / 2) + k / 2];
            unsigned nib = (k % 2 == 0) ? (byte & 0x0Fu) : (byte >> 4);
            double s = orc_f16_to_double(scales[(size_t)n * (K / G) + k / G]);
            w[(size_t)n * K + k] = (double)nibble_to_code(nib) * s;
        }
}

/* Reference quantiser that produces the inputs: symmetric, group-wise along K,
 * fp16 scale = max|w|/7 (1.0 if that rounds to zero), code = clamp(rint(w/scale),-8,7),
 * divisions and rounding in float32, ties to even. */
void orc_quantise(const float *w, int32_t N, int32_t K, int32_t G, uint8_t *wq, uint16_t *scales)
{
    for (int32_t n = 0; n < N; ++n)
        for (int32_t g = 0; g < K / G; ++g) {
            float mx = 0.0f;
            for (int32_t i = 0; i < G; ++i) {
                float a = fabsf(w[(size_t)n * K + (size_t)g * G + i]);
                if (a > mx) mx = a;
            }
            float s32 = mx / 7.0f;
            uint16_t sb = orc_f32_to_f16(s32);
            if ((sb & 0x7FFF) == 0) sb = 0x3C00;     /* 1.0 */
            scales[(size_t)n * (K / G) + g] = sb;
            float s = (float)orc_f16_to_double(sb);
            for (int32_t i = 0; i < G; ++i) {
                size_t k = (size_t)g * G + i;
                float q = nearbyintf(w[(size_t)n * K + k] / s);
                int c = q < -8.0f ? -8 : (q > 7.0f ? 7 : (int)q);
                uint8_t *byte = &wq[(size_t)n * (K / 2) + k / 2];
                if (k % 2 == 0) *byte = (uint8_t)((*byte & 0xF0u) | ((unsigned)c & 0x0Fu));
                else            *byte = (uint8_t)((*byte & 0x0Fu) | (((unsigned)c & 0x0Fu) << 4));
            }
        }
}

/* ---- grouping rows by adapter ---------------------------------------------------------- */

/* Stable order of the rows by (adapter, row): perm lists the rows that carry an
 * adapter, adapter ascending then row ascending, followed by the rows with
 * index -1 in ascending row order, so perm is a permutation of 0..M-1.
 * Segment s (s < *n_seg) is adapter seg_adapter[s] owning perm[seg_start[s] ..
 * seg_start[s+1]); seg_start[*n_seg] = number of rows that carry an adapter.
 * Returns 0, or -1 (and *n_seg = -1) if an index lies outside [-1, n_adapters). */
int32_t orc_group_rows(const int32_t *row_adapter, int32_t M, int32_t n_adapters,
                       int32_t *perm, int32_t *seg_adapter, int32_t *seg_start, int32_t *n_seg)
{
    for (int32_t m = 0; m < M; ++m)
        if (row_adapter[m] < -1 || row_adapter[m] >= n_adapters) { *n_seg = -1; return -1; }
    int32_t pos = 0, segs = 0;
    for (int32_t a = 0; a < n_adapters; ++a) {
        int32_t first = pos;
        for (int32_t m = 0; m < M; ++m)
            if (row_adapter[m] == a) perm[pos++] = m;
        if (pos > first) { seg_adapter[segs] = a; seg_start[segs] = first; ++segs; }
    }
    seg_start[segs] = pos;
    for (int32_t m = 0; m < M; ++m)
        if (row_adapter[m] == -1) perm[pos++] = m;
    *n_seg = segs;
    return 0;
}

/* ---- the linear layer -------------------------------------------------------------------- */

void orc_set_threads(int32_t n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int32_t orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* y[M][N] (double).  t_out, if not NULL, receives t[M][rank] (zeros for rows without adapter).
 * Threads (if any) split the output columns; each (m, n) is summed in the same
 * order whatever the thread count, so results do not depend on it. */
void orc_linear(int32_t K, int32_t N, int32_t G,
                const uint8_t *wq, const uint16_t *scales,
                int32_t n_adapters, int32_t rank,
                const uint16_t *lora_a, const uint16_t *lora_b, double alpha,
                const uint16_t *x, const int32_t *row_adapter, int32_t M,
                double *y, double *t_out)
{
    (void)n_adapters;
    double *xd = (double *)malloc(sizeof(double) * (size_t)M * K);
    double *t = (double *)calloc((size_t)M * (rank > 0 ? rank : 1), sizeof(double));
    for (size_t i = 0; i < (size_t)M * K; ++i) xd[i] = orc_bf16_to_double(x[i]);

    /* shrink: t[m][j] = sum_k A[a][j][k] x[m][k] */
    for (int32_t m = 0; m < M; ++m) {
        int32_t a = row_adapter ? row_adapter[m] : -1;
        if (a < 0) continue;
        for (int32_t j = 0; j < rank; ++j) {
            const uint16_t *arow = lora_a + ((size_t)a * rank + j) * K;
            double s = 0.0;
            for (int32_t k = 0; k < K; ++k) s += orc_bf16_to_double(arow[k]) * xd[(size_t)m * K + k];
            t[(size_t)m * rank + j] = s;
        }
    }

    /* base + expand, one output column at a time */
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int32_t n = 0; n < N; ++n) {
            for (int32_t k = 0; k < K; ++k) {
                uint8_t byte = wq[(size_t)n * (K / 2) + k / 2];
                unsigned nib = (k % 2 == 0) ? (byte & 0x0Fu) : (byte >> 4);
                wrow[k] = (double)nibble_to_code(nib)
                          * orc_f16_to_double(scales[(size_t)n * (K / G) + k / G]);
            }
            for (int32_t m = 0; m < M; ++m) {
                double base = 0.0;
                for (int32_t k = 0; k < K; ++k) base += wrow[k] * xd[(size_t)m * K + k];
                int32_t a = row_adapter ? row_adapter[m] : -1;
                double lora = 0.0;
                if (a >= 0) {
                    const uint16_t *brow = lora_b + ((size_t)a * N + n) * rank;
                    for (int32_t j = 0; j < rank; ++j)
                        lora += orc_bf16_to_double(brow[j]) * t[(size_t)m * rank + j];
                    base += alpha * lora;
                }
                y[(size_t)m * N + n] = base;
            }
        }
        free(wrow);
    }
    if (t_out) memcpy(t_out, t, sizeof(double) * (size_t)M * rank);
    free(t);
    free(xd);
}
