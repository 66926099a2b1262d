// Masked tree attention over a segmented KV cache (paper Sections 3.4 and 3.5, Appendix A.1
// and A.2): what stands between the q/k/v projections and the o projection of a decoding step
// that carries several output streams and, per stream, a draft tree with forecast embeddings.
//
// Two kernels.  The first cuts every cache segment into chunks of 64 keys and gives a block a
// run of chunks of one segment and one kv head; the block's four waves share the chunk's keys
// and values through LDS and split the query vectors that may see the segment (all rows for
// the common segments, one stream's rows for that stream's segment and for the rows of the
// step itself) into tiles of 16.  Scores and weighted values run on the matrix units
// (16x16x32 bf16, fp32 accumulation; the weights enter as two bf16 halves, so nothing is
// rounded to 8 bits); the softmax is the running one (maximum, sum and output rescaled from
// chunk to chunk).  Every block leaves, per query vector, its maximum, its sum and its
// unnormalised output in the workspace; the second kernel merges the blocks of a query vector in
// a fixed order and normalises.  Nothing is accumulated with atomics: results are reproducible.
#include "common.hpp"

#include "../../include/mlora_tree_attention.h"

namespace mlora {

namespace {

constexpr int KC = 64;                   // keys per chunk
// Query tiles (of 16 vectors) a wave carries, and query vectors per block (more: grid.z slices).
// One tile per wave: a block runs its code once, so what counts is how little code there is (a
// second tile per wave would be a second copy of the whole tile body, fetched cold).
constexpr int qt_per_wave(int) { return 1; }
constexpr int qv_per_slice(int D) { return 16 * 4 * qt_per_wave(D); }
constexpr float NEG_BIG = -1.0e30f;      // "no key seen yet"

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum SegKind { SEG_PREFILL = 0, SEG_FPREFIX = 1, SEG_STREAM = 2, SEG_NEW = 3 };

struct AttnArgs {
    const uint16_t *q;                   // bf16 [M][Hq][D]
    const uint16_t *k_prefill, *v_prefill, *k_fprefix, *v_fprefix, *k_stream, *v_stream, *k_new, *v_new;
    const int *len_stream, *parent;
    const uint8_t *is_forecast;
    float *part_shared;                  // [shared blocks][Hkv][M*G][D + 2]
    float *part_stream;                  // [S][stream blocks + 1][Hkv][R*G][D + 2]
    void *out;
    int Hq, Hkv, G, S, R, M;
    int Lp, Lf, cap;
    int cpb;                             // chunks per block
    int nb_prefill, nb_fprefix, nb_stream;   // blocks per segment (per stream for nb_stream)
    int out_fp32;
    float scale;
};

template <int D>
struct AttnLds {
    static constexpr int KROW = D * 2 + 16;              // bytes of a key row; +16: rows 4 banks apart
    static constexpr int VROW = KC * 2 + 16;             // bytes of a row of the transposed values
    static constexpr int PROW = KC * 2 + 16;             // bytes of a row of weights (bf16)
    alignas(16) unsigned char k[KC * KROW];
    alignas(16) unsigned char vt[D * VROW];
    alignas(16) unsigned char p[4][2][16 * PROW];        // per wave: high and low halves of the weights
    unsigned long long anc[64];                          // rows of the step a row may see (bit j = row j)
};

// Reductions over the 16 lanes that hold the keys of one row of scores: four rotations within
// the row of 16 lanes (DPP row_ror 8, 4, 2, 1), after which every lane holds the result.
template <int N>
__device__ __forceinline__ float row_ror(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave16_max(float v)
{
    v = fmaxf(v, row_ror<8>(v));
    v = fmaxf(v, row_ror<4>(v));
    v = fmaxf(v, row_ror<2>(v));
    v = fmaxf(v, row_ror<1>(v));
    return v;
}
__device__ __forceinline__ float wave16_sum(float v)
{
    v += row_ror<8>(v);
    v += row_ror<4>(v);
    v += row_ror<2>(v);
    v += row_ror<1>(v);
    return v;
}

// blockIdx.x -> (segment kind, stream, first chunk of the block)
__device__ __forceinline__ void decode_item(const AttnArgs &a, int b, int &kind, int &s, int &blk)
{
    if (b < a.nb_prefill) { kind = SEG_PREFILL; s = 0; blk = b; return; }
    b -= a.nb_prefill;
    if (b < a.nb_fprefix) { kind = SEG_FPREFIX; s = 0; blk = b; return; }
    b -= a.nb_fprefix;
    const int per = a.nb_stream + 1;
    s = b / per;
    blk = b % per;
    kind = blk < a.nb_stream ? SEG_STREAM : SEG_NEW;
}

template <int D>
__global__ __launch_bounds__(256) void tree_attn_partial(const AttnArgs a)
{
    constexpr int QT_PER_WAVE = qt_per_wave(D), QV_PER_SLICE = qv_per_slice(D);
    __shared__ AttnLds<D> lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    const int hk = blockIdx.y;
    int kind, s, blk;
    decode_item(a, (int)blockIdx.x, kind, s, blk);
    const bool shared = kind == SEG_PREFILL || kind == SEG_FPREFIX;

    // the segment: keys [0, seg_len), row pitch in elements
    const uint16_t *kbase, *vbase;
    int seg_len, pitch = D;
    if (kind == SEG_PREFILL)      { kbase = a.k_prefill + (size_t)hk * a.Lp * D; vbase = a.v_prefill + (size_t)hk * a.Lp * D; seg_len = a.Lp; }
    else if (kind == SEG_FPREFIX) { kbase = a.k_fprefix + (size_t)hk * a.Lf * D; vbase = a.v_fprefix + (size_t)hk * a.Lf * D; seg_len = a.Lf; }
    else if (kind == SEG_STREAM)  { const size_t o = ((size_t)s * a.Hkv + hk) * a.cap * D; kbase = a.k_stream + o; vbase = a.v_stream + o; seg_len = max(0, min(a.len_stream[s], a.cap)); }
    else                          { const size_t o = ((size_t)s * a.R * a.Hkv + hk) * D; kbase = a.k_new + o; vbase = a.v_new + o; seg_len = a.R; pitch = a.Hkv * D; }
    const int first_chunk = kind == SEG_NEW ? 0 : blk * a.cpb;
    const int n_chunks = min(a.cpb, (seg_len + KC - 1) / KC - first_chunk);   // may be <= 0: nothing to see

    // the query vectors of this block: vector v is (row v / G, head hk * G + v % G)
    const int n_qv = shared ? a.M * a.G : a.R * a.G;
    const int row0 = shared ? 0 : s * a.R;
    const int qv0 = (int)blockIdx.z * QV_PER_SLICE;
    const int n_tiles = (min(n_qv - qv0, QV_PER_SLICE) + 15) / 16;            // of this slice
    if (n_tiles <= 0) return;                              // (a stream's few vectors fill fewer slices than all rows do)
    float *part = shared ? a.part_shared + ((size_t)(kind == SEG_PREFILL ? blk : a.nb_prefill + blk) * a.Hkv + hk) * (size_t)n_qv * (D + 2)
                         : a.part_stream + (((size_t)s * (a.nb_stream + 1) + blk) * a.Hkv + hk) * (size_t)n_qv * (D + 2);

    // rows of the step a row may see: itself and what it continues (parent pointers)
    if (kind == SEG_NEW && tid < 64) {
        unsigned long long m = 0;
        // (a parent must be an earlier row: the walk strictly descends, so it ends and stays in bounds
        // whatever the array holds)
        if (tid < a.R)
            for (int r = tid; r >= 0;) {
                m |= 1ull << r;
                const int up = a.parent[s * a.R + r];
                r = up < r ? up : -1;
            }
        lds.anc[tid] = m;
    }

    // per wave: its tiles' running maximum, sum and output
    float run_m[QT_PER_WAVE][4], run_l[QT_PER_WAVE][4];
    f32x4 o[QT_PER_WAVE][D / 16];
    u32x4 qf[QT_PER_WAVE][D / 32];
    bool row_fc[QT_PER_WAVE][4];         // (forecast prefix) rows that may see it
    int row_loc[QT_PER_WAVE][4];         // (rows of the step) row within the stream
#pragma unroll
    for (int t = 0; t < QT_PER_WAVE; ++t) {
        const int tile = wave + 4 * t;
        // A operand: lane (l16, lq) holds 8 features of query vector tile * 16 + l16
        const int v = min(qv0 + tile * 16 + l16, n_qv - 1);
        const uint16_t *qp = a.q + ((size_t)(row0 + v / a.G) * a.Hq + hk * a.G + v % a.G) * D + 8 * lq;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk)
            qf[t][kk] = tile < n_tiles ? *reinterpret_cast<const u32x4 *>(qp + kk * 32) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            run_m[t][e] = NEG_BIG;
            run_l[t][e] = 0.f;
            // result rows: lane (l16, lq) holds rows 4 * lq + e of the tile
            const int ve = min(qv0 + tile * 16 + 4 * lq + e, n_qv - 1);
            row_loc[t][e] = ve / a.G;
            row_fc[t][e] = kind != SEG_FPREFIX || a.is_forecast[row0 + ve / a.G] != 0;
        }
#pragma unroll
        for (int db = 0; db < D / 16; ++db) o[t][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int c = 0; c < n_chunks; ++c) {
        const int key0 = (first_chunk + c) * KC;
        const int n_keys = min(KC, seg_len - key0);
        __syncthreads();                                   // the previous chunk has been used by every wave
        // keys: rows of D features, as they are; values: transposed, so that the 8 keys a lane
        // needs of one feature lie side by side.  Rows past the segment's end read its last row.
        for (int i = tid; i < KC * (D / 8); i += 256) {
            const int key = i / (D / 8), piece = i % (D / 8);
            const size_t src = (size_t)min(key0 + key, seg_len - 1) * pitch + piece * 8;
            *reinterpret_cast<u32x4 *>(lds.k + key * AttnLds<D>::KROW + piece * 16) = *reinterpret_cast<const u32x4 *>(kbase + src);
            const u32x4 vv = *reinterpret_cast<const u32x4 *>(vbase + src);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                *reinterpret_cast<uint16_t *>(lds.vt + (piece * 8 + 2 * j) * AttnLds<D>::VROW + key * 2) = (uint16_t)(vv[j] & 0xFFFFu);
                *reinterpret_cast<uint16_t *>(lds.vt + (piece * 8 + 2 * j + 1) * AttnLds<D>::VROW + key * 2) = (uint16_t)(vv[j] >> 16);
            }
        }
        __syncthreads();

#pragma unroll
        for (int t = 0; t < QT_PER_WAVE; ++t) {
            if (wave + 4 * t >= n_tiles) continue;         // (uniform per wave)
            // scores of 16 query vectors x 64 keys: lane (l16, lq) gets rows 4 lq + e, key jt * 16 + l16
            f32x4 sc[4];
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) {
                sc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk) {
                    const u32x4 kf = *reinterpret_cast<const u32x4 *>(lds.k + (jt * 16 + l16) * AttnLds<D>::KROW + kk * 64 + lq * 16);
                    sc[jt] = mfma16(__builtin_bit_cast(uint4, qf[t][kk]), __builtin_bit_cast(uint4, kf), sc[jt]);
                }
            }
            // visibility, chunk maximum, weights, chunk sum
            bool vis[4][4];
            float cm[4], p[4][4], cl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                cm[e] = NEG_BIG;
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) {
                    const int key = jt * 16 + l16;
                    bool ok = key < n_keys && row_fc[t][e];
                    if (kind == SEG_NEW) ok = ok && ((lds.anc[row_loc[t][e]] >> key) & 1ull);
                    vis[jt][e] = ok;
                    sc[jt][e] *= a.scale;
                    cm[e] = ok ? fmaxf(cm[e], sc[jt][e]) : cm[e];
                }
                cm[e] = wave16_max(cm[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float new_m = fmaxf(run_m[t][e], cm[e]);
                const float keep = __expf(run_m[t][e] - new_m);       // (1 while nothing has been seen)
                cl[e] = 0.f;
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) {
                    p[jt][e] = vis[jt][e] ? __expf(sc[jt][e] - new_m) : 0.f;
                    cl[e] += p[jt][e];
                }
                cl[e] = wave16_sum(cl[e]);
                run_l[t][e] = run_l[t][e] * keep + cl[e];
                run_m[t][e] = new_m;
#pragma unroll
                for (int db = 0; db < D / 16; ++db) o[t][db][e] *= keep;
            }
            // weights -> LDS as two bf16 halves, laid out as the A operand of the next product
            unsigned char *ph = lds.p[wave][0], *pl = lds.p[wave][1];
#pragma unroll
            for (int jt = 0; jt < 4; ++jt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t hb = __float_as_uint(p[jt][e]) & 0xFFFF0000u;
                    const uint32_t lb = __float_as_uint(p[jt][e] - __uint_as_float(hb));
                    const int at = (4 * lq + e) * AttnLds<D>::PROW + (jt * 16 + l16) * 2;
                    *reinterpret_cast<uint16_t *>(ph + at) = (uint16_t)(hb >> 16);
                    *reinterpret_cast<uint16_t *>(pl + at) = (uint16_t)(lb >> 16);
                }
            // (the wave's own LDS accesses are ordered: no barrier between the writes and the reads)
#pragma unroll
            for (int ks = 0; ks < KC / 32; ++ks) {
                const u32x4 fh = *reinterpret_cast<const u32x4 *>(ph + l16 * AttnLds<D>::PROW + ks * 64 + lq * 16);
                const u32x4 fl = *reinterpret_cast<const u32x4 *>(pl + l16 * AttnLds<D>::PROW + ks * 64 + lq * 16);
#pragma unroll
                for (int db = 0; db < D / 16; ++db) {
                    const u32x4 vf = *reinterpret_cast<const u32x4 *>(lds.vt + (db * 16 + l16) * AttnLds<D>::VROW + ks * 64 + lq * 16);
                    o[t][db] = mfma16(__builtin_bit_cast(uint4, fh), __builtin_bit_cast(uint4, vf), o[t][db]);
                    o[t][db] = mfma16(__builtin_bit_cast(uint4, fl), __builtin_bit_cast(uint4, vf), o[t][db]);
                }
            }
        }
    }

    // what this block saw, per query vector: [maximum, sum, output[D]]
#pragma unroll
    for (int t = 0; t < QT_PER_WAVE; ++t) {
        if (wave + 4 * t >= n_tiles) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int v = qv0 + (wave + 4 * t) * 16 + 4 * lq + e;
            if (v >= n_qv) continue;
            float *dst = part + (size_t)v * (D + 2);
            if (l16 == 0) { dst[0] = run_m[t][e]; dst[1] = run_l[t][e]; }
#pragma unroll
            for (int db = 0; db < D / 16; ++db) dst[2 + db * 16 + l16] = o[t][db][e];
        }
    }
}

// One block per (row, kv head), D threads per query head of the group: merge what the blocks of
// the first kernel saw, in the order prefill, forecast prefix, own stream segment, rows of the step.
template <int D>
__global__ __launch_bounds__(1024) void tree_attn_combine(const AttnArgs a)
{
    const int m = blockIdx.x, hk = blockIdx.y, d = threadIdx.x % D, g = threadIdx.x / D;
    const int hq = hk * a.G + g, s = m / a.R, i = m % a.R;
    const int n_all = a.M * a.G, n_str = a.R * a.G;
    const bool fc = a.is_forecast[m] != 0;
    const int stream_blocks = a.cap > 0 ? min(a.nb_stream, (max(0, min(a.len_stream[s], a.cap)) + KC * a.cpb - 1) / (KC * a.cpb)) : 0;
    const int n_shared = a.nb_prefill + (fc ? a.nb_fprefix : 0);
    const int n_src = n_shared + stream_blocks + 1;
    auto src = [&](int j) -> const float * {
        if (j < n_shared) return a.part_shared + (((size_t)j * a.Hkv + hk) * n_all + (size_t)m * a.G + g) * (D + 2);
        j -= n_shared;
        const int blk = j < stream_blocks ? j : a.nb_stream;          // (the rows of the step sit in the last slot)
        return a.part_stream + ((((size_t)s * (a.nb_stream + 1) + blk) * a.Hkv + hk) * n_str + (size_t)i * a.G + g) * (D + 2);
    };
    // Sources in rounds of 8: every thread requests the round's maxima, sums and its own feature
    // of the outputs all at once (one memory round trip per round; the maxima and sums are the
    // same addresses for all threads of the block), then folds the round into the running result.
    constexpr int RB = 8;
    float num = 0.f, den = 0.f, run_top = NEG_BIG;
    for (int j0 = 0; j0 < n_src; j0 += RB) {
        float pm[RB], pl[RB], pv[RB];
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const float *p = src(min(j0 + u, n_src - 1));
            pm[u] = p[0];
            pl[u] = j0 + u < n_src ? p[1] : 0.f;
            pv[u] = p[2 + d];
        }
        float top = run_top;
#pragma unroll
        for (int u = 0; u < RB; ++u) top = pl[u] > 0.f ? fmaxf(top, pm[u]) : top;
        const float keep = __expf(run_top - top);          // (1 while nothing has been seen)
        num *= keep;
        den *= keep;
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const float w = pl[u] > 0.f ? __expf(pm[u] - top) : 0.f;
            num += w * pv[u];
            den += w * pl[u];
        }
        run_top = top;
    }
    const float r = num / den;                             // (a row always sees itself: den > 0)
    const size_t at = ((size_t)m * a.Hq + hq) * D + d;
    if (a.out_fp32) reinterpret_cast<float *>(a.out)[at] = r;
    else reinterpret_cast<uint16_t *>(a.out)[at] = float_to_bf16_bits(r);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Chunks a block walks through: as many as give about 128 blocks (per slice of query vectors) for
// the longest segment, at most 16.  A block's result (64 vectors x 66 floats) is four times the
// keys and values of a chunk it reads, and every one is read again by the merging kernel: with
// one chunk per block a call of 2048 keys moved far more partial results than keys; two chunks
// measured 5 % faster there, four slower (blocks are short, and what bounds a call of this size
// is the chain of latencies inside a block).
int chunks_per_block(int longest, int n_kv_heads)
{
    const long long chunks = (longest + KC - 1) / KC;
    const long long cpb = (chunks * n_kv_heads + 127) / 128;
    return cpb < 1 ? 1 : cpb > 16 ? 16 : (int)cpb;
}

struct Plan {
    int cpb, nb_prefill, nb_fprefix, nb_stream;
    size_t shared_floats, stream_floats;
};

Plan plan_of(const mlora_tree_attn &t)
{
    Plan p;
    const int G = t.n_q_heads / t.n_kv_heads;
    const int M = t.n_streams * t.rows_per_stream;
    const int longest = t.len_prefill > t.cap_stream ? t.len_prefill : t.cap_stream;
    p.cpb = chunks_per_block(longest > t.len_fprefix ? longest : t.len_fprefix, t.n_kv_heads);
    auto blocks = [&](int len) { return ((len + KC - 1) / KC + p.cpb - 1) / p.cpb; };
    p.nb_prefill = blocks(t.len_prefill);
    p.nb_fprefix = blocks(t.len_fprefix);
    p.nb_stream = blocks(t.cap_stream);
    const size_t D2 = (size_t)t.head_dim + 2;
    p.shared_floats = (size_t)(p.nb_prefill + p.nb_fprefix) * t.n_kv_heads * (size_t)M * G * D2;
    p.stream_floats = (size_t)t.n_streams * (p.nb_stream + 1) * t.n_kv_heads * (size_t)t.rows_per_stream * G * D2;
    return p;
}

mlora_status check(const mlora_tree_attn *t)
{
    if (!t) return MLORA_EINVAL;
    if (t->head_dim != 64 && t->head_dim != 128) return MLORA_ESHAPE;
    if (t->n_kv_heads <= 0 || t->n_q_heads <= 0 || t->n_q_heads % t->n_kv_heads != 0) return MLORA_ESHAPE;
    if (t->n_q_heads / t->n_kv_heads > 8 || t->n_q_heads > 65535 || t->n_kv_heads > 65535) return MLORA_ESHAPE;
    if (t->n_streams <= 0 || t->rows_per_stream <= 0 || t->rows_per_stream > 64) return MLORA_ESHAPE;
    if ((long long)t->n_streams * t->rows_per_stream > MLORA_MAX_ROWS) return MLORA_ESHAPE;
    if (t->len_prefill < 0 || t->len_fprefix < 0 || t->cap_stream < 0) return MLORA_ESHAPE;
    if (t->len_prefill > (1 << 24) || t->len_fprefix > (1 << 24) || t->cap_stream > (1 << 24)) return MLORA_ESHAPE;
    if (!t->k_new || !t->v_new || !t->parent || !t->is_forecast) return MLORA_EINVAL;
    if (t->len_prefill > 0 && (!t->k_prefill || !t->v_prefill)) return MLORA_EINVAL;
    if (t->len_fprefix > 0 && (!t->k_fprefix || !t->v_fprefix)) return MLORA_EINVAL;
    if (t->cap_stream > 0 && (!t->k_stream || !t->v_stream || !t->len_stream)) return MLORA_EINVAL;
    const void *ptrs[] = {t->k_prefill, t->v_prefill, t->k_fprefix, t->v_fprefix, t->k_stream, t->v_stream, t->k_new, t->v_new};
    for (const void *p : ptrs)
        if (p && !aligned16(p)) return MLORA_EALIGN;
    if ((reinterpret_cast<uintptr_t>(t->parent) & 3u) || (t->len_stream && (reinterpret_cast<uintptr_t>(t->len_stream) & 3u)))
        return MLORA_EALIGN;
    return MLORA_OK;
}

}  // namespace
}  // namespace mlora

using namespace mlora;

extern "C" {

size_t mlora_tree_attention_workspace_bytes(const mlora_tree_attn *t)
{
    if (check(t) != MLORA_OK) return 0;
    const Plan p = plan_of(*t);
    return (p.shared_floats + p.stream_floats) * sizeof(float) + 256;
}

mlora_status mlora_tree_attention(const mlora_tree_attn *t, const void *q, void *out, int32_t out_dtype,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    const mlora_status st = check(t);
    if (st != MLORA_OK) return st;
    if (!q || !out) return MLORA_EINVAL;
    if (out_dtype != MLORA_Y_BF16 && out_dtype != MLORA_Y_FP32) return MLORA_EINVAL;
    if (!aligned16(q) || !aligned16(out)) return MLORA_EALIGN;
    const Plan p = plan_of(*t);
    const size_t need = (p.shared_floats + p.stream_floats) * sizeof(float) + 256;
    if (!workspace || workspace_bytes < need) return MLORA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MLORA_EALIGN;

    AttnArgs a;
    a.q = reinterpret_cast<const uint16_t *>(q);
    a.k_prefill = reinterpret_cast<const uint16_t *>(t->k_prefill);
    a.v_prefill = reinterpret_cast<const uint16_t *>(t->v_prefill);
    a.k_fprefix = reinterpret_cast<const uint16_t *>(t->k_fprefix);
    a.v_fprefix = reinterpret_cast<const uint16_t *>(t->v_fprefix);
    a.k_stream = reinterpret_cast<const uint16_t *>(t->k_stream);
    a.v_stream = reinterpret_cast<const uint16_t *>(t->v_stream);
    a.k_new = reinterpret_cast<const uint16_t *>(t->k_new);
    a.v_new = reinterpret_cast<const uint16_t *>(t->v_new);
    a.len_stream = t->len_stream;
    a.parent = t->parent;
    a.is_forecast = t->is_forecast;
    a.part_shared = reinterpret_cast<float *>(workspace);
    a.part_stream = a.part_shared + p.shared_floats;
    a.out = out;
    a.Hq = t->n_q_heads;
    a.Hkv = t->n_kv_heads;
    a.G = t->n_q_heads / t->n_kv_heads;
    a.S = t->n_streams;
    a.R = t->rows_per_stream;
    a.M = a.S * a.R;
    a.Lp = t->len_prefill;
    a.Lf = t->len_fprefix;
    a.cap = t->cap_stream;
    a.cpb = p.cpb;
    a.nb_prefill = p.nb_prefill;
    a.nb_fprefix = p.nb_fprefix;
    a.nb_stream = p.nb_stream;
    a.out_fp32 = out_dtype == MLORA_Y_FP32;
    a.scale = t->scale;

    hipStream_t s = (hipStream_t)stream;
    const int items = p.nb_prefill + p.nb_fprefix + a.S * (p.nb_stream + 1);
    const int per_slice = qv_per_slice(t->head_dim);
    const int slices = (a.M * a.G + per_slice - 1) / per_slice;   // (stream segments need fewer: their extra slices find no tile)
    const dim3 grid1((unsigned)items, (unsigned)a.Hkv, (unsigned)slices);
    const dim3 grid2((unsigned)a.M, (unsigned)a.Hkv);
    if (t->head_dim == 64) {
        tree_attn_partial<64><<<grid1, dim3(256), 0, s>>>(a);
        tree_attn_combine<64><<<grid2, dim3(64 * a.G), 0, s>>>(a);
    } else {
        tree_attn_partial<128><<<grid1, dim3(256), 0, s>>>(a);
        tree_attn_combine<128><<<grid2, dim3(128 * a.G), 0, s>>>(a);
    }
    return hipGetLastError() == hipSuccess ? MLORA_OK : MLORA_EHIP;
}

}  // extern "C"
