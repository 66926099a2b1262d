/*
 * mlora_w4 -- multi-LoRA int4 linear layer for AMD MI355X (gfx950), C ABI.
 *
 * One call computes, for a block of M rows (concurrent output streams times
 * the tokens of a speculative draft tree; paper Sections 3.4 and 3.5),
 *
 *     y[m] = dequant(Wq, scales) . x[m]  +  alpha * B[a(m)] . ( A[a(m)] . x[m] )
 *
 * which is the paper's LoRA-augmented projection Y = XW + X(sAB) (Section 3.1,
 * Eq. 1-4) with a frozen int4 base weight (Section 3.3), the LoRA tensors
 * passed as runtime arguments of identical shape for every adapter (Section
 * 3.2, approach c; Limitations), and the task selector generalised from "one
 * LoRA per graph execution" to one adapter index per row.
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller; descriptor
 *    structs and the arrays of pointers handed to mlora_w4_layer_step are HOST
 *    memory read during the call.  The library allocates no device memory,
 *    creates no stream and never synchronises: work is enqueued on `stream`
 *    (a hipStream_t, NULL = default stream) and results are valid once the
 *    caller has synchronised with it.
 *  - bf16 / fp16 tensors are arrays of 16-bit patterns.  All tensors are
 *    dense, row-major in the index order written next to them.
 *  - Errors a host check can see are reported before anything is launched.
 *    An adapter index outside [-1, n_adapters) cannot be seen from the host
 *    without a synchronisation: such a row is computed without adapter
 *    (mlora_group_rows reports it through *n_seg = -1).
 *  - Output is a pure function of the inputs: all reductions run in a fixed
 *    order, so repeated calls return bit-identical results.
 */
#ifndef MLORA_W4_H
#define MLORA_W4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MLORA_OK = 0,
    MLORA_EINVAL = -1,       /* null pointer, bad enum value, bad count */
    MLORA_ESHAPE = -2,       /* dimension outside what the kernels support */
    MLORA_EALIGN = -3,       /* pointer not 16-byte aligned */
    MLORA_EWORKSPACE = -4,   /* workspace missing or smaller than mlora_w4_workspace_bytes */
    MLORA_EUNSUPPORTED = -5, /* valid request this build does not implement */
    MLORA_EHIP = -6          /* a HIP runtime call failed */
} mlora_status;

enum { MLORA_Y_BF16 = 0, MLORA_Y_FP32 = 1 };

/* Limits checked on the host (MLORA_ESHAPE otherwise). */
enum {
    MLORA_MAX_ROWS = 4096,      /* M */
    MLORA_MAX_ADAPTERS = 1024,  /* n_adapters */
    MLORA_MAX_RANK = 128,       /* rank; must also be a multiple of 8 */
    MLORA_STATIC_SCRATCH_MIB = 32 /* size of the built-in scratch of mlora_w4_layer_step_static */
};

/* One projection.  K = input features, N = output features.
 *   K % 128 == 0 (the kernels consume inputs four MFMA steps of 32 at a time), group in
 *   {32, 64, 128}, N >= 1.
 *   w_blob   prepacked base weight made by mlora_w4_prepack (opaque, mlora_w4_blob_bytes bytes)
 *   lora_a   bf16 [n_adapters][rank][K]     (the paper's LoRA-A, transposed)
 *   lora_b   bf16 [n_adapters][N][rank]     (the paper's LoRA-B, transposed)
 *   alpha    the paper's scale factor s: multiplies B.(A.x) directly (no division by rank)
 * n_adapters == 0 (lora_a, lora_b may then be NULL) means a plain int4 linear layer. */
typedef struct {
    int32_t K, N;
    int32_t group;
    const void *w_blob;
    int32_t n_adapters, rank;
    const void *lora_a;
    const void *lora_b;
    float alpha;
} mlora_w4_proj;

/* Size in bytes of the prepacked blob for a K x N weight (0 if the shape is not supported). */
size_t mlora_w4_blob_bytes(int32_t K, int32_t N, int32_t group);

/* Canonical int4 weight -> device blob (one-time, weights are frozen; Section 3.2).
 *   wq          uint8 [N][K/2]: code(n, k) sits in byte k/2 of row n, even k in the low
 *               nibble, odd k in the high nibble, each nibble a two's-complement value in [-8, 7]
 *   scales_f16  fp16  [N][K/group]: w(n, k) = code(n, k) * scales(n, k / group)
 *   w_blob      out, mlora_w4_blob_bytes(K, N, group) bytes, 16-byte aligned */
mlora_status mlora_w4_prepack(int32_t K, int32_t N, int32_t group, const uint8_t *wq,
                              const uint16_t *scales_f16, void *w_blob, void *stream);

/* Inverse of prepack, for bit-exact checks: codes int8 [N][K] (may be NULL) and
 * w_f32 float [N][K] = code * scale, exact in fp32 (may be NULL).  Only K, N, group, w_blob
 * of *p are read. */
mlora_status mlora_w4_unpack(const mlora_w4_proj *p, int8_t *codes, float *w_f32, void *stream);

/* Stable grouping of rows by adapter (the selector of Section 3.2 made per-row):
 *   perm[M]        rows that carry an adapter, adapter ascending then row ascending, followed
 *                  by the rows with index -1 in ascending order
 *   seg_adapter[s], seg_start[s] for s < *n_seg: adapter of segment s and its first position in
 *                  perm; seg_start[*n_seg] = number of rows that carry an adapter.  Callers
 *                  size seg_adapter for min(M, n_adapters) and seg_start for one more.
 *   n_seg          number of adapters present, or -1 if an index was outside [-1, n_adapters)
 * All five arrays are device memory; one int32 for n_seg. */
mlora_status mlora_group_rows(const int32_t *row_adapter, int32_t M, int32_t n_adapters,
                              int32_t *perm, int32_t *seg_adapter, int32_t *seg_start,
                              int32_t *n_seg, void *stream);

/* Device scratch a call over these projections and M rows needs (256-byte aligned pointer).
 * It holds what blocks of one launch hand to each other: the inner LoRA factor t[m] = A[a(m)].x[m]
 * of Eq. 1-4, partial base products of projections with more than 2048 inputs, and the
 * completion counters that order them.
 *  - Layout: a 256-byte header whose first uint32 is a status word, the counters growing from
 *    the front, the data placed against the END of the workspace.  The size returned is
 *    256 + 2 * max(counters, data), so that one workspace sized for the largest of several calls
 *    (different projections, different M) serves all of them, one after another: no call's
 *    counters can fall on another call's leftover data.  For that to hold, pass the SAME
 *    workspace_bytes (the size of the allocation) on every call that uses a workspace.
 *  - The counters must be ZERO when a call starts and are zero again when it ends: call
 *    mlora_w4_workspace_init once after allocating a workspace (or hand in zero-filled memory).
 *    Calls that overlap in time need a workspace each.
 *  - Blocks of a launch are dispatched in index order and producers sit before their
 *    consumers, so every wait ends; the waits are bounded all the same.  If one runs out
 *    (only a foreign write to the counters, or a workspace that was not zero, can cause that), the
 *    status word becomes non-zero, the outputs of the waiting block are stored as NaN, and the
 *    workspace has to be initialised again.  mlora_w4_workspace_status reads the word. */
size_t mlora_w4_workspace_bytes(const mlora_w4_proj *projs, int32_t n_proj, int32_t M);

/* How a call over these projections and M rows would be run, for reading profiles; host only,
 * nothing is launched.  info (HOST memory, 5 int32): [0] kernel launches of the call (one per
 * 128 projections; from 17 rows on also a new one where the group size changes),
 * [1] 1 if the first launch runs blocks of four column tiles ("wide_kernel"), 0 if blocks of
 * one column tile ("layer_kernel"), [2] rows per row chunk (16, 32 or 64; a short launch of 17
 * to 32 rows runs as two chunks of 16), [3] and [4] the first launch's grid: blocks per row chunk
 * (grid.x is that times the number of chunks, rounded up to runs of 8 when there are several)
 * and groups of 16 projections along z.
 * MLORA_EINVAL for null pointers or n_proj <= 0, MLORA_ESHAPE for shapes the library refuses. */
mlora_status mlora_w4_layer_step_plan(const mlora_w4_proj *projs, int32_t n_proj, int32_t M, int32_t *info);

/* Zero-fill a workspace (a small kernel on `stream`; no memset node, so it can be captured). */
mlora_status mlora_w4_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Copy the status word of a workspace to *status_word (HOST memory): 0 = every call since the
 * last mlora_w4_workspace_init completed normally.  Unlike the other calls this one waits for
 * `stream` (it has to, to hand a value back); do not call it under stream capture. */
mlora_status mlora_w4_workspace_status(const void *workspace, int32_t *status_word, void *stream);

/* Test hook: number of polls a waiting block makes before it gives up (default 200000;
 * negative = back to the default; 0 = every wait gives up at once, which lets a test see the
 * failure path -- status word, NaN outputs -- with every kernel still running to its end).
 * Process-wide, read when a call is enqueued.  Returns the previous value. */
int32_t mlora_w4_debug_spin_limit(int32_t limit);

/* The layer step with the decoder layer's glue folded into the output stage (Section 3.3: graph
 * optimisations -- constant folding and operator fusion; Table 10's scalar folding).  As
 * mlora_w4_layer_step, for at most 16 projections, each with an epilogue applied to its outputs
 * before they are stored, in this order:
 *   1. v = row_scale[m] * (base product + LoRA term)       row_scale fp32 [M], NULL = 1.
 *      This is RMSNorm in front of the projection with its weight folded away: with W' = W diag(g)
 *      and A' = A diag(g) prepared offline, W (g * x / rms(x)) = (1 / rms(x)) W' x, so the call
 *      takes the un-normalised rows as x and mlora_rms_scale's output as row_scale.
 *   2. a pair operation on columns (c, c + 32) of every tile of 64 output columns (N % 64 == 0):
 *      MLORA_PAIR_ROPE    rotary position encoding for heads of 64 features laid out as tiles:
 *                         v[c]    <- v[c] cos[m][c % 32] - v[c + 32] sin[m][c % 32]
 *                         v[c+32] <- v[c + 32] cos[m][c % 32] + v[c] sin[m][c % 32]
 *                         rope_cos, rope_sin fp32 [M][32]: the angle of row m's position times
 *                         the i-th frequency, prepared by the caller;
 *      MLORA_PAIR_SWIGLU  the output has N / 2 columns: y[m][32 t + i] = silu(v[64 t + i]) *
 *                         v[64 t + 32 + i], silu(z) = z / (1 + exp(-z)).  The projection is the
 *                         gate and up projections of the MLP stored as one weight whose tile t
 *                         holds gate columns 32 t .. 32 t + 31 followed by the up columns of the
 *                         same features (an offline rearrangement of the two weights; their LoRA
 *                         pairs become one of twice the rank).
 *   3. + residual[m][n]                                     bf16 [M][N_out], NULL = none
 * then rounding to y_dtype.  ys[i] is [M][N_out], N_out = N (N / 2 for MLORA_PAIR_SWIGLU).
 * RMSNorm between two projections without a kernel of its own: with sq_out (fp32
 * [M][ceil(N / 64)]) a projection also leaves, per row and column tile, the sum of the squares
 * of the outputs it stored (as rounded to y_dtype); the projection that takes those outputs as
 * its x names that array as sq_in with sq_parts = ceil(N_producer / 64) and sq_eps, instead of
 * row_scale, and scales by 1 / sqrt(sum over parts / K + sq_eps).  Sums run in a fixed order.
 * Errors as mlora_w4_layer_step, plus MLORA_ESHAPE for more than 16 projections or a pair
 * operation with N % 64 != 0, MLORA_EINVAL for an unknown pair operation, missing tables, or
 * sq_in together with row_scale. */
enum { MLORA_PAIR_NONE = 0, MLORA_PAIR_ROPE = 1, MLORA_PAIR_SWIGLU = 2 };
typedef struct mlora_w4_epilogue {
    const float *row_scale;
    int32_t pair_op;
    const float *rope_cos;
    const float *rope_sin;
    const void *residual;
    const float *sq_in;          /* NULL, or partial sums of squares of the rows of x (not with row_scale) */
    int32_t sq_parts;
    float sq_eps;
    float *sq_out;               /* NULL, or where to leave this projection's own partial sums */
} mlora_w4_epilogue;
mlora_status mlora_w4_layer_step_fused(const mlora_w4_proj *projs, const mlora_w4_epilogue *epis, int32_t n_proj,
                                       const void *const *xs, void *const *ys,
                                       const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* scale[m] = 1 / sqrt(mean_k x[m][k]^2 + eps) for bf16 rows x [M][K] (K % 8 == 0): the per-row
 * factor of RMSNorm, computed in fp32 in a fixed order.  x 16-byte aligned, scale fp32 [M]. */
mlora_status mlora_rms_scale(const void *x, int32_t M, int32_t K, float eps, float *scale, void *stream);

/* LoRA tensors stored as 16-bit integers (the appendix on the 1B model names int16 LoRA weights
 * next to the int4 base weights), with one scale per stack:  A[a] = s_a * a_q[a],
 * B[a] = s_b * b_q[a].  This call turns such a pair of stacks into the bf16 tensors and the alpha
 * that mlora_w4_proj takes, without rounding anything: an int16 is 256 * hi + lo with digits that
 * are bf16 numbers, so  b_q (a_q x) = (256 Bh + Bl) (256 (Ah x) + (Al x))  is the product of a
 * LoRA pair of FOUR TIMES the rank,
 *     lora_a  [n_adapters][4 * rank][K]:  rows  j, rank + j, 2 rank + j, 3 rank + j  = Ah, Ah, Al, Al of row j
 *     lora_b  [n_adapters][N][4 * rank]:  columns likewise = 65536 Bh, 256 Bl, 256 Bh, Bl of column j
 * and  *alpha_out = alpha * s_a * s_b  (fp32, written on the HOST before the call returns).  A
 * projection then uses  {rank = 4 * rank, alpha = *alpha_out, lora_a, lora_b}:  the matrix units
 * multiply exact integers, sums are fp32 as for bf16 adapters.  Cost: four times the bytes of the
 * int16 tensors in the layer step; done once, when an adapter set is loaded.
 *   a_q  DEVICE int16 [n_adapters][rank][K],  b_q  DEVICE int16 [n_adapters][N][rank]
 *   lora_a, lora_b  DEVICE, caller-allocated, sizes as above (bf16), all four 16-byte aligned
 *   rank % 8 == 0, 4 * rank <= MLORA_MAX_RANK;  K % 32 == 0;  s_a, s_b finite and > 0
 * Errors (nothing is launched): MLORA_ESHAPE, MLORA_EINVAL, MLORA_EALIGN; MLORA_EHIP if a launch fails. */
mlora_status mlora_lora_int16_expand(const int16_t *a_q, const int16_t *b_q, int32_t n_adapters, int32_t rank,
                                     int32_t K, int32_t N, float alpha, float s_a, float s_b,
                                     void *lora_a, void *lora_b, float *alpha_out, void *stream);

/* The layer step with int8 activations (Section 3.3: activations quantised to int8 with one
 * scale per tensor, weights to int4).  As mlora_w4_layer_step, except that
 *   xs[i]        int8 [M][K]: the quantised rows; the activation they stand for is
 *                x_scales[i] * xs[i][m][k]
 *   x_scales     HOST array of n_proj floats, each finite and > 0 (a per-tensor scale is fixed
 *                offline, by calibration or quantisation-aware training: it is an input here)
 * and the result is that of Eq. 1-4 on those activations:
 *   y[m] = x_scale * ( sum_g scale[n][g] * sum_{k in g} code[n][k] * xq[m][k]
 *                      + alpha * B[a(m)] . (A[a(m)] . xq[m]) ).
 * The inner sums run on the int8 matrix units and are exact in int32; scales are applied in
 * fp32.  LoRA tensors stay bf16 (the paper's int16 LoRA is not built).  The weight blob is the
 * one mlora_w4_prepack writes.  Every row count runs the blocks of four column tiles; size the
 * workspace with mlora_w4a8_workspace_bytes (same layout and rules as mlora_w4_workspace_bytes).
 * Errors as mlora_w4_layer_step, plus MLORA_EINVAL for a null, non-positive or non-finite scale. */
size_t mlora_w4a8_workspace_bytes(const mlora_w4_proj *projs, int32_t n_proj, int32_t M);
mlora_status mlora_w4a8_layer_step(const mlora_w4_proj *projs, int32_t n_proj,
                                   const void *const *xs, const float *x_scales, void *const *ys,
                                   const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* One projection.
 *   x            bf16 [M][K]
 *   row_adapter  int32 [M], -1 = no adapter for that row; NULL = no adapter for any row
 *   y            [M][N], bf16 (y_dtype = MLORA_Y_BF16, round to nearest even) or fp32
 * M == 0 is a no-op.  x, y, the tensors of *p and workspace must not overlap. */
mlora_status mlora_w4_linear(const mlora_w4_proj *p, const void *x, const int32_t *row_adapter,
                             int32_t M, void *y, int32_t y_dtype, void *workspace,
                             size_t workspace_bytes, void *stream);

/* Several independent projections over the same M rows and the same row->adapter index in
 * one launch per 128 projections: the seven projections of a decoder block (Section 3.1), or
 * those of many blocks at once.
 *   xs[i], ys[i]  device pointers of projection i (host arrays of n_proj pointers); inputs may
 *                 be shared (q, k, v read the same rows), outputs may not
 * Ordering against whatever produces the inputs is the caller's business. */
mlora_status mlora_w4_layer_step(const mlora_w4_proj *projs, int32_t n_proj,
                                 const void *const *xs, void *const *ys,
                                 const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* mlora_w4_layer_step for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): no workspace argument.  What
 * the kernels hand to each other lives in a scratch array inside the library's device image
 * (MLORA_STATIC_SCRATCH_MIB MiB per GPU, held until the process ends).  The call allocates and
 * frees nothing; it clears the status word and the counters it will use with a small fill
 * kernel on `stream`, then enqueues the same kernels as mlora_w4_layer_step, so the results are
 * bit-identical to that call's.
 *  - MLORA_EWORKSPACE if the call needs more than the array holds (counters + data + 256 bytes,
 *    without the doubling of mlora_w4_workspace_bytes): 112 projections of a 1B-like model at
 *    32 rows need 14 MiB; a 512-row call over 16 such layers does not fit.
 *  - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *    streams, two threads) race, as two calls on one workspace would.  The array keeps the last
 *    call's contents between calls. */
mlora_status mlora_w4_layer_step_static(const mlora_w4_proj *projs, int32_t n_proj,
                                        const void *const *xs, void *const *ys,
                                        const int32_t *row_adapter, int32_t M, int32_t y_dtype,
                                        void *stream);

const char *mlora_strerror(mlora_status status);

#ifdef __cplusplus
}
#endif
#endif /* MLORA_W4_H */
