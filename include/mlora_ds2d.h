/*
 * mlora_ds2d -- the token side of a dynamic self-speculative decoding (DS2D) step for AMD
 * MI355X (gfx950), C ABI.  Part of the mlora_w4 library.
 *
 * Section 3.5 and Appendix A.2 of the paper: a prefix-tuned model with m forecast embeddings
 * predicts 1 + m tokens per pass.  Per output stream (Section 3.4: S streams run side by side)
 * the rows of a step are the tokens of a tree -- the last verified token as root, then the draft
 * tokens level by level, level i holding b_1 * ... * b_i nodes with the children of one node
 * next to each other (branch configuration (b_1 .. b_d)) -- followed, for every token in the
 * same order, by its m forecast embeddings.  The worked example of the paper: m = 2, branch
 * (3, 2): 1 + 3 + 6 = 10 tokens and 20 forecast embeddings, 30 rows.  The first step of a
 * stream has no drafts (d = 0): 1 + m rows.
 *
 * Given the logits of all rows of a step, mlora_ds2d_step does, per stream, on the device:
 *   1. verification: walk down from the root; the token the model continues a node with is the
 *      arg-max of that node's logits; if a child of the node carries that token it is accepted
 *      and the walk goes on from it, else (or at a leaf) the walk ends;
 *   2. the tokens given out: those of the accepted drafts, then the arg-max at the node where
 *      the walk ended (the next last verified token);
 *   3. drafting: level i of the next tree is filled from the b'_i highest logits of forecast
 *      embedding i of the node where the walk ended, best first, the same b'_i tokens below
 *      every node of level i - 1 (b' = the branch configuration of the next step, which may
 *      differ from this step's: the paper picks it per use case).
 * The paper describes both choices as sampling after a soft-max; this library takes the
 * deterministic reading (highest logit first).  Order of candidates: larger logit first; among
 * equal logits (+0 equals -0) the lower token id; NaN after everything else.
 *
 * Conventions as in mlora_w4.h: data pointers are DEVICE memory owned by the caller unless
 * marked HOST; no allocation, no synchronisation, work is enqueued on `stream`; errors a host
 * check can see are reported before anything is launched; results are deterministic.
 */
#ifndef MLORA_DS2D_H
#define MLORA_DS2D_H

#include "mlora_w4.h"

#ifdef __cplusplus
extern "C" {
#endif

#define MLORA_DS2D_MAX_FORECAST 8     /* m: forecast embeddings per token */
#define MLORA_DS2D_MAX_BRANCH 16      /* b_i */
#define MLORA_DS2D_MAX_ROWS 64        /* rows of one stream in a step (as in mlora_tree_attention) */

/* Tokens and rows of one stream for a branch configuration of `depth` levels (0 <= depth <=
 * n_forecast) and n_forecast forecast embeddings per token: *n_tokens = 1 + b_1 + b_1 b_2 + ...,
 * *n_rows = n_tokens * (1 + n_forecast).  Host only.  MLORA_EINVAL for null pointers,
 * MLORA_ESHAPE if depth, n_forecast or a b_i is out of range or n_rows > MLORA_DS2D_MAX_ROWS. */
mlora_status mlora_ds2d_rows(const int32_t *branch, int32_t depth, int32_t n_forecast,
                             int32_t *n_tokens, int32_t *n_rows);

/* Row tables of one stream, in the form mlora_tree_attention takes them.  HOST arrays of n_rows
 * entries each: parent[r] = the row that row r continues (-1 at the root), is_forecast[r] = 1
 * for forecast embeddings; level (may be NULL): depth of a token in the tree, and for a forecast
 * embedding its number 1 .. n_forecast.  Same errors as mlora_ds2d_rows. */
mlora_status mlora_ds2d_layout(const int32_t *branch, int32_t depth, int32_t n_forecast,
                               int32_t *parent, uint8_t *is_forecast, int32_t *level);

typedef struct mlora_ds2d {
    int32_t n_streams;                          /* S >= 1 */
    int32_t n_forecast;                         /* m, 1 .. MLORA_DS2D_MAX_FORECAST */
    int32_t depth;                              /* levels of THIS step's tree, 0 .. m */
    int32_t branch[MLORA_DS2D_MAX_FORECAST];    /* b_1 .. b_depth of this step */
    int32_t next_depth;                         /* levels of the NEXT step's tree, 0 .. m */
    int32_t next_branch[MLORA_DS2D_MAX_FORECAST];
    int32_t vocab;                              /* V: logits per row, >= every b'_i, < 2^31 - 1 */
    int32_t logits_dtype;                       /* MLORA_Y_BF16 or MLORA_Y_FP32 */
} mlora_ds2d;

/* Device scratch mlora_ds2d_step needs for this descriptor (16-byte aligned pointer); 0 on a bad
 * descriptor.  Contents need no initialisation and carry nothing from call to call. */
size_t mlora_ds2d_workspace_bytes(const mlora_ds2d *d);

/* One step for all streams.  R = rows of this step's tree, T = its tokens, T' = tokens of the
 * next step's tree (mlora_ds2d_rows).
 *   logits      [S * R][V]   in  bf16 or fp32: row s * R + r is row r of stream s
 *   tokens      [S][T]       in  int32: token ids at the token rows (tokens[s][0] = last verified)
 *   n_accepted  [S]          out int32: drafts accepted, 0 .. depth
 *   accepted_rows [S][m + 1] out int32: rows of the accepted path, root first (row 0), -1 beyond
 *   emitted     [S][m + 1]   out int32: tokens given out (accepted drafts, then the next last
 *                                verified token): n_accepted + 1 entries, -1 beyond
 *   next_tokens [S][T']      out int32: token rows of the next step (entry 0 = the next last
 *                                verified token, then the drafts level by level)
 * Token ids in `tokens` are compared as they are; ids outside [0, V) simply never match.
 * Errors: MLORA_EINVAL (null pointer, bad dtype), MLORA_ESHAPE (descriptor out of range),
 * MLORA_EALIGN (logits or workspace not 16-byte aligned), MLORA_EWORKSPACE, MLORA_EHIP. */
mlora_status mlora_ds2d_step(const mlora_ds2d *d, const void *logits, const int32_t *tokens,
                             int32_t *n_accepted, int32_t *accepted_rows, int32_t *emitted,
                             int32_t *next_tokens, void *workspace, size_t workspace_bytes,
                             void *stream);

#ifdef __cplusplus
}
#endif
#endif
