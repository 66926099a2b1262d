// DS2D step on the device (Section 3.5 and Appendix A.2 of the paper): from the logits of all
// rows of a step, verify the draft tree greedily and draft the next one.  Two kernels:
//
//   ds2d_best_partial  grid (slices of the vocabulary, rows): the k best logits of one row inside
//                      one slice, k = 1 for token rows (only the arg-max is needed), b'_j for
//                      forecast embedding j, as sortable 64-bit keys.  Reads every logit once:
//                      this is the kernel that is bound by HBM.
//   ds2d_verify_draft  one block per stream: arg-max of every token row from the partial keys,
//                      the walk down the tree, then the b'_i best of the forecast rows of the node
//                      where the walk ended, and the token rows of the next step.
//
// A candidate is a 64-bit key: the logit mapped to an unsigned number that orders like the
// stated rule (larger logit first, +0 = -0, NaN last) in the high half, the complement of the
// token id in the low half (lower id first among equals).  Keys of different tokens differ, so
// "the best key below the one found in the round before" enumerates candidates in order without
// any bookkeeping; 0 marks an empty slot.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/mlora_ds2d.h"

namespace mlora {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int DS_THREADS = 256;
constexpr int DS_ELEMS = 16;                           // logits per thread
constexpr int DS_SLICE = DS_THREADS * DS_ELEMS;        // logits per block
constexpr int DS_KMAX = MLORA_DS2D_MAX_BRANCH;

struct Ds2dArgs {
    const void *logits;
    const int32_t *tokens;
    int32_t *n_accepted, *accepted_rows, *emitted, *next_tokens;
    unsigned long long *partial;      // [S * R][slices][DS_KMAX]
    long long total;                  // S * R * V
    int V, S, R, T, T_next, m, depth, next_depth, slices, fp32;
    int next_branch[MLORA_DS2D_MAX_FORECAST];
    signed char parent[MLORA_DS2D_MAX_ROWS];   // of the token rows
};

__device__ inline unsigned long long key_of(float v, unsigned token)
{
    unsigned b = __float_as_uint(v);
    unsigned hi;
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) hi = 0u;                     // NaN: after everything
    else {
        if (b == 0x80000000u) b = 0u;                                 // -0 counts as +0
        hi = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    }
    return ((unsigned long long)hi << 32) | (unsigned long long)(~token);
}
__device__ inline float bf16_value(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

__device__ inline unsigned long long wave_max(unsigned long long v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const unsigned long long o = __shfl_xor(v, s, 64);
        v = o > v ? o : v;
    }
    return v;
}
// the largest value over the block; `slot` is 2 x 4 words of LDS, alternated by `phase`
__device__ inline unsigned long long block_max(unsigned long long v, unsigned long long *slot, int phase)
{
    v = wave_max(v);
    unsigned long long *s = slot + (phase & 1) * 4;
    if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long r = s[0];
#pragma unroll
    for (int w = 1; w < DS_THREADS / 64; ++w) r = s[w] > r ? s[w] : r;
    return r;
}

// how many candidates a row needs: 1 for a token row, b'_j for forecast embedding j
__device__ inline int wanted(const Ds2dArgs &a, int r)
{
    if (r < a.T) return 1;
    const int j = (r - a.T) % a.m;                     // 0-based number of the embedding
    return j < a.next_depth ? a.next_branch[j] : 0;
}

// 32-bit keys for bf16 logits: a bf16 value orders by 16 bits, which leaves room for the position
// inside the block's slice (4096 logits): (sortable value << 16) | (0xFFFF - position).  Lower
// positions are lower token ids, so these keys order a slice exactly like the 64-bit ones; they
// are widened when the winners are stored.
__device__ inline unsigned key16_of(unsigned h, unsigned pos)
{
    unsigned hi;
    if ((h & 0x7FFFu) > 0x7F80u) hi = 0u;                              // NaN
    else {
        if (h == 0x8000u) h = 0u;                                      // -0 counts as +0
        hi = (h & 0x8000u) ? (~h & 0xFFFFu) : (h | 0x8000u);
    }
    return (hi << 16) | (0xFFFFu - pos);
}
template <int N>
__device__ __forceinline__ unsigned ror_u32(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x120 + N, 0xF, 0xF, false);
}
// the largest value over the block: rows of 16 lanes by DPP rotations, the 16 rows through LDS
// (`slot` is 2 x 16 words, alternated by `phase`)
__device__ inline unsigned block_max(unsigned v, unsigned *slot, int phase)
{
    unsigned o;
    o = ror_u32<8>(v); v = o > v ? o : v;
    o = ror_u32<4>(v); v = o > v ? o : v;
    o = ror_u32<2>(v); v = o > v ? o : v;
    o = ror_u32<1>(v); v = o > v ? o : v;
    unsigned *s = slot + (phase & 1) * 16;
    if ((threadIdx.x & 15) == 0) s[threadIdx.x >> 4] = v;
    __syncthreads();
    const uint4 *q = reinterpret_cast<const uint4 *>(s);
    unsigned r = 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4 t = q[i];
        const unsigned m0 = t.x > t.y ? t.x : t.y, m1 = t.z > t.w ? t.z : t.w;
        const unsigned m = m0 > m1 ? m0 : m1;
        r = m > r ? m : r;
    }
    return r;
}

template <bool FP32>
__global__ __launch_bounds__(DS_THREADS) void ds2d_best_partial(const Ds2dArgs a)
{
    using Key = typename std::conditional<FP32, unsigned long long, unsigned>::type;
    __shared__ __align__(16) Key slot[32];
    const int row = blockIdx.y;
    const int k = wanted(a, row % a.R);
    if (k == 0) return;
    // The row's logits are elements [row * V, row * V + V) of the whole array.  They are read
    // with aligned 16-byte loads counted from the start of the array (rows need no alignment of
    // their own); elements of a vector that belong to a neighbouring row are ignored, and the
    // last, partial vector of the array is read element by element.
    constexpr int EPV = FP32 ? 4 : 8;                                   // elements per vector
    constexpr int VPT = DS_ELEMS / EPV;                                 // vectors per thread
    const long long first = (long long)row * a.V, last = first + a.V;
    const long long vec0 = first / EPV + (long long)blockIdx.x * (DS_THREADS * VPT);
    const long long full_vectors = a.total / EPV;
    const long long slice_first = vec0 * EPV;                           // element at position 0
    // the row's part of this slice, as positions 0 .. DS_SLICE, and the token id at pos_lo
    const int pos_lo = first > slice_first ? (int)(first - slice_first) : 0;
    const int pos_hi = last - slice_first < DS_SLICE ? (last > slice_first ? (int)(last - slice_first) : 0) : DS_SLICE;
    const unsigned token_lo = (unsigned)(slice_first + pos_lo - first);
    Key key[DS_ELEMS];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const long long vi = vec0 + (long long)u * DS_THREADS + threadIdx.x;
        const long long e0 = vi * EPV;
        const unsigned pos0 = (unsigned)(u * DS_THREADS + threadIdx.x) * EPV;
        unsigned bits[EPV];                     // fp32 patterns, or bf16 patterns in the low half
        if (e0 >= last) {
#pragma unroll
            for (int j = 0; j < EPV; ++j) bits[j] = 0u;
        } else if (vi < full_vectors) {
            const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.logits) + vi);
            if constexpr (FP32) {
                bits[0] = q.x; bits[1] = q.y; bits[2] = q.z; bits[3] = q.w;
            } else {
                bits[0] = q.x & 0xFFFFu; bits[1] = q.x >> 16; bits[2] = q.y & 0xFFFFu; bits[3] = q.y >> 16;
                bits[4] = q.z & 0xFFFFu; bits[5] = q.z >> 16; bits[6] = q.w & 0xFFFFu; bits[7] = q.w >> 16;
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                bits[j] = 0u;
                if (e0 + j < a.total) {
                    if constexpr (FP32) bits[j] = reinterpret_cast<const unsigned *>(a.logits)[e0 + j];
                    else bits[j] = reinterpret_cast<const unsigned short *>(a.logits)[e0 + j];
                }
            }
        }
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const int pos = (int)pos0 + j;                  // inside the row iff pos_lo <= pos < pos_hi
            const bool inside = pos >= pos_lo && pos < pos_hi;
            if constexpr (FP32) key[u * EPV + j] = inside ? key_of(__uint_as_float(bits[j]), (unsigned)(pos - pos_lo) + token_lo) : 0ull;
            else key[u * EPV + j] = inside ? key16_of(bits[j], (unsigned)pos) : 0u;
        }
    }
    unsigned long long *out = a.partial + ((size_t)row * a.slices + blockIdx.x) * DS_KMAX;
    Key below = ~(Key)0;
    for (int round = 0; round < k; ++round) {
        Key best = 0;
#pragma unroll
        for (int u = 0; u < DS_ELEMS; ++u) {
            const Key c = key[u] < below ? key[u] : (Key)0;
            best = c > best ? c : best;
        }
        best = block_max(best, slot, round);
        if (threadIdx.x == 0) {
            if constexpr (FP32) out[round] = best;
            else {
                // widen: the value's 16 bits on top, the complement of the token id below
                const unsigned token = (unsigned)(slice_first + (long long)(0xFFFFu - (best & 0xFFFFu)) - first);
                out[round] = best == 0u ? 0ull : ((unsigned long long)(best >> 16) << 48) | (unsigned long long)(~token);
            }
        }
        below = best;
        if (best == 0) {                         // the slice holds fewer than k logits
            for (int r2 = round + 1 + (int)threadIdx.x; r2 < k; r2 += DS_THREADS) out[r2] = 0ull;
            break;
        }
    }
}

__global__ __launch_bounds__(DS_THREADS) void ds2d_verify_draft(const Ds2dArgs a)
{
    __shared__ unsigned long long slot[8];
    __shared__ unsigned long long best_key[MLORA_DS2D_MAX_ROWS];
    __shared__ int tok[MLORA_DS2D_MAX_ROWS];
    __shared__ int walk_end, walk_token;
    __shared__ int cand[MLORA_DS2D_MAX_FORECAST][DS_KMAX];
    const int s = blockIdx.x, tid = threadIdx.x;

    // arg-max of every token row: the best of the first keys of its slices.  All (row, slice)
    // pairs are spread over the block, so the loads are independent of each other.
    if (tid < a.T) {
        best_key[tid] = 0ull;
        tok[tid] = a.tokens[(size_t)s * a.T + tid];
    }
    __syncthreads();
    const unsigned long long *base = a.partial + (size_t)s * a.R * a.slices * DS_KMAX;
    // (loads are issued in batches of eight before any of them is used: a loop that stores each
    // value as it arrives would wait for memory once per element)
    constexpr int BATCH = 8;
    for (int i0 = 0; i0 < a.T * a.slices; i0 += BATCH * DS_THREADS) {
        unsigned long long v[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int i = i0 + u * DS_THREADS + tid;                          // row * slices + slice
            v[u] = i < a.T * a.slices ? base[(size_t)i * DS_KMAX] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int i = i0 + u * DS_THREADS + tid;
            if (i < a.T * a.slices) atomicMax(&best_key[i / a.slices], v[u]);
        }
    }
    __syncthreads();

    // the walk (one thread; the tree has at most 64 tokens and 8 levels; everything is in LDS)
    if (tid == 0) {
        int32_t *rows = a.accepted_rows + (size_t)s * (a.m + 1);
        int32_t *out = a.emitted + (size_t)s * (a.m + 1);
        int cur = 0, n = 0;
        rows[0] = 0;
        while (true) {
            const int target = (int)(~(unsigned)(best_key[cur] & 0xFFFFFFFFull));
            int next = -1;
            if (n < a.depth)
                for (int c = cur + 1; c < a.T; ++c)
                    if (a.parent[c] == cur && tok[c] == target) { next = c; break; }
            if (next < 0) {
                out[n] = target;
                walk_token = target;
                break;
            }
            out[n] = tok[next];
            cur = next;
            rows[++n] = cur;
        }
        for (int i = n + 1; i <= a.m; ++i) rows[i] = out[i] = -1;
        a.n_accepted[s] = n;
        walk_end = cur;
    }
    __syncthreads();
    const int cur = walk_end;
    int32_t *nt = a.next_tokens + (size_t)s * a.T_next;
    if (tid == 0) nt[0] = walk_token;

    // Level i of the next tree: the b'_i best of forecast embedding i of the node `cur`.  A
    // thread keeps its share of a level's candidates in registers (two each: up to 512
    // candidates, e.g. 32 slices x 16; what lies beyond is read again every round), and the loads
    // of all levels are issued before the first round.
    constexpr int OWN = 2;
    unsigned long long own[MLORA_DS2D_MAX_FORECAST][OWN];
#pragma unroll
    for (int i = 0; i < MLORA_DS2D_MAX_FORECAST; ++i) {
        if (i >= a.next_depth) break;
        const int b = a.next_branch[i];
        const unsigned long long *p = base + (size_t)(a.T + cur * a.m + i) * a.slices * DS_KMAX;
#pragma unroll
        for (int u = 0; u < OWN; ++u) {
            const int c = tid + u * DS_THREADS;
            own[i][u] = c < a.slices * b ? p[(size_t)(c / b) * DS_KMAX + (c % b)] : 0ull;
        }
    }
    int phase = 0;
#pragma unroll
    for (int i = 0; i < MLORA_DS2D_MAX_FORECAST; ++i) {
        if (i >= a.next_depth) break;
        const int b = a.next_branch[i];
        const unsigned long long *p = base + (size_t)(a.T + cur * a.m + i) * a.slices * DS_KMAX;
        const int n_cand = a.slices * b;
        unsigned long long below = ~0ull;
        for (int round = 0; round < b; ++round) {
            unsigned long long v = 0ull;
#pragma unroll
            for (int u = 0; u < OWN; ++u) {
                const unsigned long long q = own[i][u] < below ? own[i][u] : 0ull;
                v = q > v ? q : v;
            }
            for (int c = tid + OWN * DS_THREADS; c < n_cand; c += DS_THREADS) {
                unsigned long long q = p[(size_t)(c / b) * DS_KMAX + (c % b)];
                q = q < below ? q : 0ull;
                v = q > v ? q : v;
            }
            v = block_max(v, slot, phase++);
            if (tid == 0) cand[i][round] = (int)(~(unsigned)(v & 0xFFFFFFFFull));
            below = v;
        }
    }
    __syncthreads();
    int offset = 1, width = 1;
    for (int i = 0; i < a.next_depth; ++i) {
        const int b = a.next_branch[i];
        width *= b;
        for (int q = tid; q < width; q += DS_THREADS) nt[offset + q] = cand[i][q % b];
        offset += width;
    }
}

}  // namespace mlora

using namespace mlora;

namespace {

bool tree_sizes(const int32_t *branch, int depth, int m, int &tokens, int &rows)
{
    if (m < 1 || m > MLORA_DS2D_MAX_FORECAST || depth < 0 || depth > m) return false;
    long long t = 1, w = 1;
    for (int i = 0; i < depth; ++i) {
        if (branch[i] < 1 || branch[i] > MLORA_DS2D_MAX_BRANCH) return false;
        w *= branch[i];
        t += w;
        if (t * (1 + m) > MLORA_DS2D_MAX_ROWS) return false;
    }
    if (t * (1 + m) > MLORA_DS2D_MAX_ROWS) return false;
    tokens = (int)t;
    rows = (int)(t * (1 + m));
    return true;
}

// parent of every token row: level by level, the children of one node next to each other
void token_parents(const int32_t *branch, int depth, int *parent)
{
    parent[0] = -1;
    int level_first = 0, level_count = 1, next = 1;
    for (int i = 0; i < depth; ++i) {
        for (int node = level_first; node < level_first + level_count; ++node)
            for (int c = 0; c < branch[i]; ++c) parent[next++] = node;
        level_first += level_count;
        level_count *= branch[i];
    }
}

int slices_of(const mlora_ds2d &d)
{
    const int epv = d.logits_dtype == MLORA_Y_FP32 ? 4 : 8;
    const long long vectors = (long long)d.vocab / epv + 2;             // a row may straddle two more
    const long long per_block = DS_SLICE / epv;
    return (int)((vectors + per_block - 1) / per_block);
}

mlora_status check(const mlora_ds2d *d, int &T, int &R, int &T_next)
{
    if (!d) return MLORA_EINVAL;
    if (d->logits_dtype != MLORA_Y_BF16 && d->logits_dtype != MLORA_Y_FP32) return MLORA_EINVAL;
    int r_next;
    if (d->n_streams < 1 || d->n_streams > 65535) return MLORA_ESHAPE;
    if (!tree_sizes(d->branch, d->depth, d->n_forecast, T, R)) return MLORA_ESHAPE;
    if (!tree_sizes(d->next_branch, d->next_depth, d->n_forecast, T_next, r_next)) return MLORA_ESHAPE;
    if (d->vocab < 1 || d->vocab >= 0x7FFFFFFF) return MLORA_ESHAPE;
    for (int i = 0; i < d->next_depth; ++i)
        if (d->next_branch[i] > d->vocab) return MLORA_ESHAPE;
    if ((long long)d->n_streams * R > 65535) return MLORA_ESHAPE;       // grid y
    return MLORA_OK;
}

}  // namespace

extern "C" {

mlora_status mlora_ds2d_rows(const int32_t *branch, int32_t depth, int32_t n_forecast,
                             int32_t *n_tokens, int32_t *n_rows)
{
    if (!n_tokens || !n_rows || (depth > 0 && !branch)) return MLORA_EINVAL;
    int t, r;
    if (!tree_sizes(branch, depth, n_forecast, t, r)) return MLORA_ESHAPE;
    *n_tokens = t;
    *n_rows = r;
    return MLORA_OK;
}

mlora_status mlora_ds2d_layout(const int32_t *branch, int32_t depth, int32_t n_forecast,
                               int32_t *parent, uint8_t *is_forecast, int32_t *level)
{
    if (!parent || !is_forecast || (depth > 0 && !branch)) return MLORA_EINVAL;
    int T, R;
    if (!tree_sizes(branch, depth, n_forecast, T, R)) return MLORA_ESHAPE;
    int par[MLORA_DS2D_MAX_ROWS];
    token_parents(branch, depth, par);
    for (int r = 0; r < T; ++r) {
        parent[r] = par[r];
        is_forecast[r] = 0;
        if (level) level[r] = r == 0 ? 0 : level[par[r]] + 1;
    }
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < n_forecast; ++j) {
            const int r = T + t * n_forecast + j;
            parent[r] = j == 0 ? t : r - 1;
            is_forecast[r] = 1;
            if (level) level[r] = j + 1;
        }
    return MLORA_OK;
}

size_t mlora_ds2d_workspace_bytes(const mlora_ds2d *d)
{
    int T, R, T_next;
    if (check(d, T, R, T_next) != MLORA_OK) return 0;
    return (size_t)d->n_streams * R * slices_of(*d) * DS_KMAX * sizeof(unsigned long long);
}

mlora_status mlora_ds2d_step(const mlora_ds2d *d, const void *logits, const int32_t *tokens,
                             int32_t *n_accepted, int32_t *accepted_rows, int32_t *emitted,
                             int32_t *next_tokens, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    int T, R, T_next;
    const mlora_status st = check(d, T, R, T_next);
    if (st != MLORA_OK) return st;
    if (!logits || !tokens || !n_accepted || !accepted_rows || !emitted || !next_tokens) return MLORA_EINVAL;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) || (reinterpret_cast<uintptr_t>(workspace) & 15u)) return MLORA_EALIGN;
    if (!workspace || workspace_bytes < mlora_ds2d_workspace_bytes(d)) return MLORA_EWORKSPACE;

    Ds2dArgs a;
    a.logits = logits;
    a.tokens = tokens;
    a.n_accepted = n_accepted;
    a.accepted_rows = accepted_rows;
    a.emitted = emitted;
    a.next_tokens = next_tokens;
    a.partial = reinterpret_cast<unsigned long long *>(workspace);
    a.V = d->vocab;
    a.S = d->n_streams;
    a.R = R;
    a.T = T;
    a.T_next = T_next;
    a.m = d->n_forecast;
    a.depth = d->depth;
    a.next_depth = d->next_depth;
    a.slices = slices_of(*d);
    a.fp32 = d->logits_dtype == MLORA_Y_FP32;
    a.total = (long long)d->n_streams * R * d->vocab;
    for (int i = 0; i < MLORA_DS2D_MAX_FORECAST; ++i) a.next_branch[i] = i < d->next_depth ? d->next_branch[i] : 0;
    int par[MLORA_DS2D_MAX_ROWS];
    token_parents(d->branch, d->depth, par);
    for (int r = 0; r < MLORA_DS2D_MAX_ROWS; ++r) a.parent[r] = r < T ? (signed char)par[r] : (signed char)-1;

    hipStream_t s = (hipStream_t)stream;
    if (a.fp32) hipLaunchKernelGGL(ds2d_best_partial<true>, dim3(a.slices, d->n_streams * R), dim3(DS_THREADS), 0, s, a);
    else hipLaunchKernelGGL(ds2d_best_partial<false>, dim3(a.slices, d->n_streams * R), dim3(DS_THREADS), 0, s, a);
    hipLaunchKernelGGL(ds2d_verify_draft, dim3(d->n_streams), dim3(DS_THREADS), 0, s, a);
    return hipGetLastError() == hipSuccess ? MLORA_OK : MLORA_EHIP;
}

}  // extern "C"
