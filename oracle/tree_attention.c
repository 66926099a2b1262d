/*
 * CPU oracle for masked tree attention over a segmented KV cache.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain loops in fp64, written from the paper's description; shares no code, header or helper
 * with the HIP library and is never called by it.
 *
 * What it computes.  One decoding step carries S concurrent output streams (Section 3.4) and,
 * per stream, R rows: the last verified token, the draft tokens of the speculative tree and the
 * forecast embeddings attached to each of them (Section 3.5).  Row i of stream s is row
 * m = s * R + i of the call.  For query head hq (kv head hk = hq / (Hq / Hkv)) of row m,
 *
 *     out[m][hq][:] = sum over visible keys of softmax(scale * q[m][hq] . k)[key] * v[key][:]
 *
 * where the keys a row can see are (Appendix A.1 and A.2, the masks described in the captions
 * of the CTG and DS2D mask figures; the figures themselves are not reproduced in the text):
 *
 *   1. the common prefill segment, all Lp positions: every row of every stream sees it;
 *   2. the segment of its own stream, positions [0, len_stream[s]): the tokens that stream has
 *      produced so far; the segments of other streams are invisible (Appendix A.1: the cache is
 *      split into one common part and one isolated part per sentence);
 *   3. the forecast prefix, all Lf positions, if and only if the row is a forecast embedding
 *      (Appendix A.2: the causal mask keeps the forecast prefix away from ordinary tokens, so the
 *      first token of a step is distributed exactly as without the prefix, Section 3.5);
 *   4. among the rows of this very step: the row itself and its ancestors in the stream's tree,
 *      found by following parent[] (index within the stream, -1 at the root).  A draft token's
 *      parent is the token it continues; forecast embedding 1 of a token hangs off that token,
 *      forecast embedding j > 1 off forecast embedding j - 1 of the same token.
 *
 * Everything else contributes exactly nothing (its weight is not computed at all).  bf16 inputs
 * arrive as uint16 bit patterns and are widened exactly; the softmax is the textbook one
 * (subtract the largest score, exponentiate, normalise), all in double.
 *
 * Layouts: k_prefill, v_prefill [Hkv][Lp][D]; k_fprefix, v_fprefix [Hkv][Lf][D];
 * k_stream, v_stream [S][Hkv][cap][D]; k_new, v_new [S*R][Hkv][D]; q [S*R][Hq][D];
 * out [S*R][Hq][D] (double); weights, if not NULL, [S*R][Hq][Lp + Lf + cap + R] in the key
 * order prefill, forecast prefix, own stream segment, rows of this step (0 where invisible).
 *
 * Pinned by tests/test_tree_attention_oracle.py: numpy's float64 softmax on an explicit 0/1
 * mask built by an independent transitive closure, plain causal attention for chain-shaped
 * trees, closed forms for identical keys, isolation of streams, the forecast-prefix rule, and
 * the visible-key counts of the paper's worked example (branch configuration (3, 2)).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_value(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;   /* bf16 is the top half of an IEEE binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double dot_qk(const uint16_t *q, const uint16_t *k, int32_t D)
{
    double s = 0.0;
    for (int32_t d = 0; d < D; ++d) s += bf16_value(q[d]) * bf16_value(k[d]);
    return s;
}

/* returns 0, or -1 if a parent index is not a smaller index of the same stream (or -1) */
int32_t orc_tree_attention(int32_t Hq, int32_t Hkv, int32_t D, int32_t S, int32_t R, double scale,
                           const uint16_t *k_prefill, const uint16_t *v_prefill, int32_t Lp,
                           const uint16_t *k_fprefix, const uint16_t *v_fprefix, int32_t Lf,
                           const uint16_t *k_stream, const uint16_t *v_stream, int32_t cap,
                           const int32_t *len_stream,
                           const uint16_t *k_new, const uint16_t *v_new,
                           const int32_t *parent, const uint8_t *is_forecast,
                           const uint16_t *q, double *out, double *weights)
{
    const int32_t G = Hq / Hkv;
    const int32_t n_keys = Lp + Lf + cap + R;
    for (int32_t m = 0; m < S * R; ++m) {
        const int32_t p = parent[m];
        if (p < -1 || p >= m % R) return -1;
    }
    double *score = (double *)malloc(sizeof(double) * (size_t)n_keys);
    const uint16_t **kptr = (const uint16_t **)malloc(sizeof(void *) * (size_t)n_keys);
    const uint16_t **vptr = (const uint16_t **)malloc(sizeof(void *) * (size_t)n_keys);
    char *visible = (char *)malloc((size_t)n_keys);

    for (int32_t s = 0; s < S; ++s)
        for (int32_t i = 0; i < R; ++i) {
            const int32_t m = s * R + i;
            for (int32_t hq = 0; hq < Hq; ++hq) {
                const int32_t hk = hq / G;
                /* the key list of this row, in the documented order */
                int32_t n = 0;
                for (int32_t t = 0; t < Lp; ++t, ++n) {
                    kptr[n] = k_prefill + ((size_t)hk * Lp + t) * D;
                    vptr[n] = v_prefill + ((size_t)hk * Lp + t) * D;
                    visible[n] = 1;
                }
                for (int32_t t = 0; t < Lf; ++t, ++n) {
                    kptr[n] = k_fprefix + ((size_t)hk * Lf + t) * D;
                    vptr[n] = v_fprefix + ((size_t)hk * Lf + t) * D;
                    visible[n] = is_forecast[m] != 0;
                }
                for (int32_t t = 0; t < cap; ++t, ++n) {
                    kptr[n] = k_stream + (((size_t)s * Hkv + hk) * cap + t) * D;
                    vptr[n] = v_stream + (((size_t)s * Hkv + hk) * cap + t) * D;
                    visible[n] = t < len_stream[s];
                }
                for (int32_t j = 0; j < R; ++j, ++n) {
                    kptr[n] = k_new + ((size_t)(s * R + j) * Hkv + hk) * D;
                    vptr[n] = v_new + ((size_t)(s * R + j) * Hkv + hk) * D;
                    visible[n] = 0;
                }
                for (int32_t a = i; a >= 0; a = parent[s * R + a])   /* the row and its ancestors */
                    visible[Lp + Lf + cap + a] = 1;

                const uint16_t *qv = q + ((size_t)m * Hq + hq) * D;
                double top = -INFINITY;
                for (int32_t t = 0; t < n_keys; ++t)
                    if (visible[t]) {
                        score[t] = scale * dot_qk(qv, kptr[t], D);
                        if (score[t] > top) top = score[t];
                    }
                double denom = 0.0;
                for (int32_t t = 0; t < n_keys; ++t)
                    if (visible[t]) {
                        score[t] = exp(score[t] - top);
                        denom += score[t];
                    }
                double *o = out + ((size_t)m * Hq + hq) * D;
                for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
                for (int32_t t = 0; t < n_keys; ++t) {
                    const double w = visible[t] ? score[t] / denom : 0.0;
                    if (weights) weights[((size_t)m * Hq + hq) * n_keys + t] = w;
                    if (!visible[t]) continue;
                    for (int32_t d = 0; d < D; ++d) o[d] += w * bf16_value(vptr[t][d]);
                }
            }
        }
    free(score);
    free(kptr);
    free(vptr);
    free(visible);
    return 0;
}
