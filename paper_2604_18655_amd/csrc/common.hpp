// Shared device-side definitions of the mlora_w4 library: blob layout, kernel
// argument blocks, small bit helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mlora_w4.h"

namespace mlora {

// ---------------------------------------------------------------------------------------------
// Prepacked weight blob.
//
// The weight is cut into tiles of 64 output columns (4 blocks of 16) and k-steps of 32 inputs:
// one 16x16x32 bf16 MFMA consumes a block of 16 columns x 32 inputs as its B operand, lane l
// holding column l%16 and the 8 consecutive inputs 8*(l/16) .. +7.  The blob stores, for
// every (tile, k-step), one 1 KiB chunk laid out exactly as a wavefront reads it with one
// 128-bit load per lane: lane l's uint4 holds, in component j, the 8 codes of column
// 64*tile + 16*j + l%16 at inputs 32*step + 8*(l/16) + 0..7.
//
// Inside a dword the 8 codes are stored as offset-binary u = code + 8 in bit fields placed so
// that  ((w rotr 4q) & 0x00780078) | 0x41804180  is a pair of bf16 numbers 16 + u = code + 24
// for inputs 2q (low half) and 2q+1 (high half): the field of input i sits at bit
// (3 + 4*(i/2) + 16*(i%2)) mod 32.  The constant offset 24 is removed by seeding the MFMA
// accumulator with -24 * sum(x) over the same inputs, which one more MFMA produces.
//
// Scales follow the codes: fp16, index ((tile * K/group + g) * 16 + c) * 4 + j for column
// 64*tile + 16*j + c, so the lane that holds column c of all four blocks reads its four
// scales of a group with one 64-bit load.  Columns beyond N are stored as code 0, scale 0.
// ---------------------------------------------------------------------------------------------
constexpr int TILE_N = 64;
constexpr int KSTEP = 32;
constexpr int SUPER_K = 128;       // k-steps are consumed four at a time

__host__ __device__ inline int tiles_n(int N) { return (N + TILE_N - 1) / TILE_N; }
__host__ __device__ inline size_t blob_code_bytes(int K, int N) {
    return (size_t)tiles_n(N) * (size_t)(K / KSTEP) * 1024u;
}
__host__ __device__ inline size_t blob_scale_bytes(int K, int N, int group) {
    return (size_t)tiles_n(N) * (size_t)(K / group) * 128u;
}
// The kernels request whole batches of super-steps without clamping the last ones, so a wave
// may read (and ignore) up to 3 super-steps of codes and as many groups of scales past the end
// of its tile: the blob ends with slack that keeps those reads inside the allocation.
constexpr size_t BLOB_SLACK_BYTES = 16384;
__host__ __device__ inline int field_pos(int i) { return (3 + 4 * (i >> 1) + 16 * (i & 1)) & 31; }
__host__ __device__ inline uint32_t rotl32(uint32_t v, int s) {
    s &= 31;
    return s ? (v << s) | (v >> (32 - s)) : v;
}
__host__ __device__ inline uint32_t rotr32(uint32_t v, int s) { return rotl32(v, 32 - (s & 31)); }

// ---------------------------------------------------------------------------------------------
// Kernel argument block of one grouped call (passed by value: about 19 KiB; a block reads only
// the launch scalars, the three table rows of its group and the record of its projection).
// The projections of a launch are cut into groups of up to 16; group z owns slice z of the grid
// (blockIdx.z) and the block tables of a group are one vector of 16 each.
// ---------------------------------------------------------------------------------------------
constexpr int GROUP_PROJ = 16;
constexpr int MAX_GROUPS = 8;
constexpr int MAX_PROJ_PER_LAUNCH = GROUP_PROJ * MAX_GROUPS;
constexpr int ROWS_PER_BLOCK16 = 16;
constexpr int MAX_KCHUNKS = 16;    // partial sums of the shrink step the epilogue adds up

struct ProjArgs {
    const uint4 *codes;        // blob, code region
    const uint2 *scales;       // blob, scale region (4 fp16 per entry)
    const uint16_t *x;         // bf16 [M][K]
    void *y;                   // [M][N]
    const uint16_t *lora_a;    // bf16 [n_adapters][rank][K]
    const uint16_t *lora_b;    // bf16 [n_adapters][N][rank]
    float *t_part;             // fp32 [kch][M][r16], written by the shrink blocks
    float *partial;            // fp32 [ksplit-1][tiles][m_pad][64], written by the split-K units
    int K, N;
    int spg;                   // k-steps per scale group (group / 32)
    int n_adapters, rank;
    int r16;                   // rank rounded up to a multiple of 16
    int kch;                   // number of K chunks of the shrink step
    float alpha;
    float x_scale;             // int8 activations: the per-tensor scale of x (1 otherwise)
    int ksplit;                // K units per tile; unit 0 finishes the tile, the others run ahead
    int n_shrink_blocks;       // shrink blocks of this projection (each bumps its counter once)
    int n_finish_blocks;       // finishing blocks of this projection (tiles x row chunks)
    int part_ctr;              // index of this projection's first split-K counter line in ctrl
    // Derived on the host so that no block starts with integer divisions (each one costs some 30
    // cold instructions, and they sat in front of the first memory request of every block):
    int unit_q, unit_r;        // (K / 128) / ksplit and (K / 128) % ksplit: super-steps per K unit
    int spg_shift;             // log2(spg)
    int ctr_copies;            // copies of the shrink counter in use: a power of two, at most
                               // min(CTR_REPL, n_finish_blocks)
    unsigned tiles_inv;        // ceil(2^32 / tiles) for tiles > 1: block index / tiles = umulhi(index,
                               // tiles_inv), exact while index * tiles < 2^32
};

// Counters in the workspace that order the blocks of one launch (all zero between calls).
// Every counter has a 128-byte line of its own, and what many blocks wait for exists in
// CTR_REPL copies, each polled by a share of the waiting blocks: hundreds of blocks polling one
// line queue up behind each other in one memory channel, and since a wave's loads return in
// order that stalls their weight streams too.
//   shrink_ctr(p, r)      + 0: shrink blocks of projection p that have finished (copy r)
//                         + 1: finishing blocks that have used copy r (the last one resets both)
//   part_ctr + (tile * chunks + chunk) * CTR_STRIDE: split-K units of that tile that have finished
constexpr int CTR_REPL = 16;
constexpr int CTR_STRIDE = 32;                 // uint32 per counter line
__host__ __device__ inline int shrink_ctr(int p, int r) { return (p * CTR_REPL + r) * CTR_STRIDE; }
constexpr size_t WS_HEADER_BYTES = 256;        // status word at the front of every workspace
constexpr int SPIN_LIMIT_DEFAULT = 200000;     // x ~0.5 us: far beyond any launch, still finite

// What a fused call does to the outputs of a projection before they are stored (all optional):
//   v = row_scale[m] * (base + LoRA term); a pair operation on columns (c, c + 32) of every
//   64-column tile; + residual[m][n].  The row scale is either handed in or made from sq_in,
//   the per-tile sums of squares that the projection which produced x left in its sq_out: the
//   RMSNorm between two projections then needs no kernel of its own.
// Pair operations: PAIR_ROPE rotates (v[c], v[c+32]) by the angle whose cosine and sine are
// rope_cos/sin[m][c % 32] (heads of 64 features: a tile is a head); PAIR_SWIGLU stores
// silu(v[c]) * v[c+32] at column 32 * tile + c % 32 of an output of N / 2 columns (the weight
// holds 32 gate columns and the 32 up columns of the same features in every tile).
enum { PAIR_NONE = 0, PAIR_ROPE = 1, PAIR_SWIGLU = 2 };
struct EpiArgs {
    const float *row_scale;        // fp32 [M]
    const float *rope_cos;         // fp32 [M][32]
    const float *rope_sin;
    const uint16_t *residual;      // bf16 [M][N_out]
    const float *sq_in;            // fp32 [M][sq_parts]: partial sums of squares of the rows of x (another
                                   // projection's sq_out); row scale = 1 / sqrt(sum / K + sq_eps)
    float *sq_out;                 // fp32 [M][tiles]: sum of squares of the outputs a tile stores, as stored
    int pair_op;
    int sq_parts;
    float sq_eps;
    int pad_;
};

struct LayerArgs {
    // Slice z of the grid holds, in this order, the shrink blocks, the split-K blocks (units 1..)
    // and the finishing blocks (unit 0) of the projections of group z; first block of each
    // projection within its kind (entries past the group's last projection: INT_MAX):
    int shrink_begin[MAX_GROUPS][GROUP_PROJ];
    int pre_begin[MAX_GROUPS][GROUP_PROJ];
    int main_begin[MAX_GROUPS][GROUP_PROJ];
    ProjArgs p[MAX_PROJ_PER_LAUNCH];
    int shrink_blocks[MAX_GROUPS];     // shrink blocks of the group (first in its slice)
    int pre_base_blocks[MAX_GROUPS];   // split-K blocks of the group (after its shrink blocks)
    int group_blocks[MAX_GROUPS];      // all blocks of the group; the slice's other blocks exit at once
    const int *row_adapter;    // may be null
    int n_proj;
    int M;
    int M_plan;                // the row count the launch was laid out for (chunk size, shrink
                               // blocks): M, except that calls with int8 activations always run
                               // wide blocks and are laid out as for at least 17 rows
    int a8;                    // x is int8 with one scale per tensor (ProjArgs::x_scale)
    int fused;                 // outputs go through epi[] (one group of at most 16 projections)
    EpiArgs epi[GROUP_PROJ];
    int y_fp32;
    int m_pad;                 // M rounded up to whole row chunks of the base kernel
    int spin_limit;            // polls a block makes before it gives up waiting (0: gives up at once)
    int wide;                  // the launch runs wide blocks (see below)
    unsigned *ctrl;            // completion counters of this launch
    unsigned *status;          // workspace status word: set non-zero if a wait ran out
    uint32_t code_mask;        // 0x00780078: the two code fields of a bf16 pair
    uint32_t code_bias;        // 0x41804180: sign, exponent and leading mantissa bit of 16.0
};

// ---------------------------------------------------------------------------------------------
// 16-bit float helpers (bit patterns)
// ---------------------------------------------------------------------------------------------
__device__ inline float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ inline uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7FFFu + ((u >> 16) & 1u);                                              // nearest even
    return (uint16_t)(u >> 16);
}

__device__ inline float half_bits_to_float(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// D[16 rows][16 cols] += A[16][32] * B[32][16]; lane l supplies row l%16 of A and column l%16
// of B at inputs 8*(l/16)..+7, and receives D[4*(l/16) + r][l%16] in element r.
__device__ inline f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}

// D[16][16] (int32) += A[16][32] * B[32][16] over int8; lane l supplies 8 bytes of row l%16 of A
// and of column l%16 of B, both for the same 8 inputs (block l/16 of the 32), and receives
// D[4*(l/16) + r][l%16] in element r.  Which byte stands for which input inside a lane's 8 does
// not matter as long as A and B agree.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ inline i32x4 mfma16_i8(long a, long b, i32x4 c) {
    return __builtin_amdgcn_mfma_i32_16x16x32_i8(a, b, c, 0, 0, 0);
}

// The grouped shrink step (more than 16 rows) works on chunks of 64 rows: the rows of a chunk are
// grouped by adapter (one wave, no sort) and every segment is cut into tiles of 16 rows.  Upper
// bound of the tiles of a chunk of `rows` rows (at most 64): a tile per 16 rows plus one per
// segment, at most a tile per row.  A block's four waves work through up to 16 tiles; a chunk
// that can have more is shared out over several blocks.  Calls of 33 to 127 rows have at most two
// chunks and base blocks that are done early: there the finishing blocks wait for t, so a wave
// gets at most one tile (measured: c5 68 -> 60 us; at 128 rows and more the extra, mostly idle
// blocks cost more than they gain).  Host (grid size) and device (block index -> chunk, share)
// use the same figures.
constexpr int SHRINK_CHUNK_ROWS = 64;
__host__ __device__ inline int max_row_tiles(int rows, int n_adapters)
{
    const int segs = n_adapters < rows ? n_adapters : rows;
    const int bound = rows / 16 + segs;
    return bound < rows ? bound : rows;
}
__host__ __device__ inline int shrink_tile_shares(int M, int n_adapters)
{
    const int tiles = max_row_tiles(M < SHRINK_CHUNK_ROWS ? M : SHRINK_CHUNK_ROWS, n_adapters);
    return (M > 32 && M < 2 * SHRINK_CHUNK_ROWS) ? (tiles + 3) / 4 : (tiles + 15) / 16;
}

// host launchers (each file defines its own)
hipError_t launch_prepack(int K, int N, int group, const uint8_t *wq, const uint16_t *scales,
                          void *blob, hipStream_t s);
hipError_t launch_unpack(int K, int N, int group, const void *blob, int8_t *codes, float *w_f32,
                         hipStream_t s);
hipError_t launch_group_rows(const int *row_adapter, int M, int n_adapters, int *perm,
                             int *seg_adapter, int *seg_start, int *n_seg, hipStream_t s);
hipError_t launch_layer(const LayerArgs &a, int grid_x, int groups, hipStream_t s);
hipError_t launch_zero(void *p, size_t bytes, hipStream_t s);
hipError_t launch_rms_scale(const uint16_t *x, int M, int K, float eps, float *scale, hipStream_t s);
hipError_t launch_lora_int16_expand(const int16_t *aq, const int16_t *bq, int n_adapters, int rank, int K, int N,
                                    uint16_t *a4, uint16_t *b4, hipStream_t s);

constexpr int UNIT_SUPER_STEPS = 16;   // a block streams at most 16 super-steps (2048 inputs)
// Two families of base blocks.  "Tile" blocks cover one column tile and their four waves split
// K (many short-lived blocks: what a small launch needs to fill the chip); "wide" blocks cover
// four column tiles, one per wave, and share the rows of x through LDS (a quarter of the x
// traffic and no reduction across waves: what a long weight stream needs).  Up to 16 rows: tile
// blocks.  33 rows and more: wide blocks with chunks of 64 rows.  17 to 32 rows (chunks of 32
// rows): wide blocks if the launch has at least WIDE32_MIN_BLOCKS of them, else tile blocks.
constexpr int WIDE_ALWAYS_ROWS = 33;
constexpr int WIDE32_MIN_ROWS = 17;
constexpr int WIDE32_MIN_BLOCKS = 300;
constexpr int WIDE_TILES_PER_BLOCK = 4;
constexpr int CHUNK16_MAX_BLOCKS = 300;    // tile launches of 17 to 32 rows below this run chunks of 16 rows
__host__ __device__ inline int rows_per_chunk(int M) { return M <= 16 ? 16 : M <= 32 ? 32 : 64; }
// column tiles a base block covers
__host__ __device__ inline int tiles_per_block(bool wide) { return wide ? WIDE_TILES_PER_BLOCK : 1; }

}  // namespace mlora
