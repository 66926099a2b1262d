/*
 * mlora_tree_attention -- masked tree attention over a segmented KV cache for AMD MI355X
 * (gfx950), C ABI.  Part of the mlora_w4 library.
 *
 * One decoding step of the paper's deployment carries S concurrent output streams
 * (Section 3.4, concurrent token generation) and, per stream, R rows: the last verified
 * token, the draft tokens of the self-speculative tree and the forecast embeddings attached to
 * each of them (Section 3.5).  Row i of stream s is row m = s * R + i of the call.  This call is
 * the attention between the q/k/v projections and the o projection of such a step:
 *
 *     out[m][hq] = sum over the keys row m may see of softmax(scale * q[m][hq] . k)[key] * v[key]
 *
 * with the masks of Appendix A.1 and A.2 (their figures are described in the captions only; the
 * reading taken here):
 *   - the common prefill segment is seen by every row of every stream;
 *   - each stream has a cache segment of its own (the tokens it has produced so far), seen by
 *     that stream's rows only;
 *   - the forecast prefix (the prefix-tuned positions that make the model semi-autoregressive)
 *     is seen by forecast-embedding rows only, so an ordinary token is distributed exactly as
 *     without it;
 *   - among the rows of the step a row sees itself and the rows it continues: parent[m] is the
 *     index, within the stream, of the row that row m continues (-1 at the last verified token);
 *     a draft token continues its parent in the tree, forecast embedding 1 of a token continues
 *     that token, forecast embedding j > 1 continues forecast embedding j - 1 of the same token.
 *     parent[m] must be smaller than m's index within its stream.
 * Query head hq reads kv head hq / (n_q_heads / n_kv_heads).  Position encodings are applied by
 * the caller before this call.
 *
 * Conventions as in mlora_w4.h: every data pointer is DEVICE memory owned by the caller, the
 * descriptor is HOST memory read during the call; no allocation, no synchronisation, work is
 * enqueued on `stream`; bf16 tensors are arrays of 16-bit patterns, dense, row-major in the
 * index order written next to them; errors a host check can see are reported before anything
 * is launched; results are bit-identical from call to call (fixed merge order, no atomics).
 */
#ifndef MLORA_TREE_ATTENTION_H
#define MLORA_TREE_ATTENTION_H

#include "mlora_w4.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t n_q_heads, n_kv_heads;   /* n_q_heads % n_kv_heads == 0, at most 8 query heads per kv head */
    int32_t head_dim;                /* 64 or 128 */
    int32_t n_streams;               /* S */
    int32_t rows_per_stream;         /* R, 1..64; S * R <= MLORA_MAX_ROWS */
    float scale;                     /* multiplies q.k before the softmax (usually head_dim^-1/2) */
    /* common prefill segment: bf16 [n_kv_heads][len_prefill][head_dim] (len 0: pointers may be NULL) */
    const void *k_prefill, *v_prefill;
    int32_t len_prefill;
    /* forecast prefix: bf16 [n_kv_heads][len_fprefix][head_dim] */
    const void *k_fprefix, *v_fprefix;
    int32_t len_fprefix;
    /* per-stream segments: bf16 [S][n_kv_heads][cap_stream][head_dim]; stream s holds
     * len_stream[s] <= cap_stream valid positions (device int32 [S]) */
    const void *k_stream, *v_stream;
    int32_t cap_stream;
    const int32_t *len_stream;
    /* the rows of this step: bf16 [S * R][n_kv_heads][head_dim] (the k and v projections' outputs) */
    const void *k_new, *v_new;
    const int32_t *parent;           /* device int32 [S * R] */
    const uint8_t *is_forecast;      /* device uint8 [S * R]: 1 = forecast-embedding row */
} mlora_tree_attn;

/* Device scratch the call needs (256-byte aligned): per block of keys and query vector the
 * running maximum, sum and unnormalised output, merged by the call's second kernel.  No state
 * survives the call; nothing has to be initialised.  0 if the descriptor is not supported. */
size_t mlora_tree_attention_workspace_bytes(const mlora_tree_attn *t);

/*   q    bf16 [S * R][n_q_heads][head_dim]
 *   out  [S * R][n_q_heads][head_dim], bf16 (out_dtype = MLORA_Y_BF16, round to nearest even) or fp32 */
mlora_status mlora_tree_attention(const mlora_tree_attn *t, const void *q, void *out, int32_t out_dtype,
                                  void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MLORA_TREE_ATTENTION_H */
