// Base int4 GEMV / skinny GEMM with the LoRA expand step in its epilogue.
//
// One block = one (projection, tile of 64 output columns, chunk of 16*MB rows).  Its four
// waves split K; each streams its share of the tile's packed codes straight from HBM into
// registers with one 128-bit load per lane and k-step, turns every dword into four bf16
// pairs with 7 integer ops, and feeds 16x16x32 bf16 MFMAs whose A operand is the block of
// rows of x.  Scales are applied to the fp32 result of each scale group, so codes enter the
// matrix unit exactly.  The four partial tiles are added in LDS in a fixed order, the LoRA
// term alpha * B[a(m)][n] . t[m] is added, and y is stored.
#include "common.hpp"

namespace mlora {

template <int MB>
struct Stage {
    uint4 w[4];
    uint4 xf[MB][4];
    uint2 sc[4];
};

__device__ inline float half_bits_lo(uint32_t v) { return half_bits_to_float((uint16_t)(v & 0xFFFFu)); }
__device__ inline float half_bits_hi(uint32_t v) { return half_bits_to_float((uint16_t)(v >> 16)); }

// 8 packed codes -> 8 bf16 values code + 24 (4 dwords)
__device__ inline uint4 expand_codes(uint32_t w, uint32_t mask, uint32_t bias)
{
    uint4 o;
    o.x = (w & mask) | bias;
    o.y = (__builtin_amdgcn_alignbit(w, w, 4) & mask) | bias;
    o.z = (__builtin_amdgcn_alignbit(w, w, 8) & mask) | bias;
    o.w = (__builtin_amdgcn_alignbit(w, w, 12) & mask) | bias;
    return o;
}

template <int MB, int SPG>
__device__ inline void compute_stage(const Stage<MB> &st, f32x4 (&acc)[MB][4], uint32_t mask,
                                     uint32_t bias)
{
    const uint4 neg24 = make_uint4(0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u);
#pragma unroll
    for (int gi = 0; gi < 4 / SPG; ++gi) {
        // -24 * sum of x over the group's inputs: cancels the offset of the stored codes
        f32x4 corr[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            corr[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < SPG; ++s) corr[mb] = mfma16(st.xf[mb][gi * SPG + s], neg24, corr[mb]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f32x4 d[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) d[mb] = corr[mb];
#pragma unroll
            for (int s = 0; s < SPG; ++s) {
                const uint4 wv = st.w[gi * SPG + s];
                const uint32_t wj = j == 0 ? wv.x : j == 1 ? wv.y : j == 2 ? wv.z : wv.w;
                const uint4 wb = expand_codes(wj, mask, bias);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) d[mb] = mfma16(st.xf[mb][gi * SPG + s], wb, d[mb]);
            }
            const uint2 sv = st.sc[gi];
            const float sj = j == 0 ? half_bits_lo(sv.x) : j == 1 ? half_bits_hi(sv.x)
                           : j == 2 ? half_bits_lo(sv.y) : half_bits_hi(sv.y);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[mb][j][e] = fmaf(d[mb][e], sj, acc[mb][j][e]);
        }
    }
}

template <int MB, int SPG>
__device__ inline void load_stage(Stage<MB> &st, const uint4 *wp, const uint16_t *const (&xp)[MB],
                                  const bool (&row_ok)[MB], const uint2 *sp, int ss)
{
#pragma unroll
    for (int s = 0; s < 4; ++s) st.w[s] = wp[(size_t)(ss * 4 + s) * 64];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int s = 0; s < 4; ++s)
            st.xf[mb][s] = row_ok[mb]
                ? *reinterpret_cast<const uint4 *>(xp[mb] + (size_t)ss * SUPER_K + s * KSTEP)
                : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int gi = 0; gi < 4 / SPG; ++gi) st.sc[gi] = sp[(size_t)(ss * (4 / SPG) + gi) * 16];
}

template <int MB, int SPG>
__device__ inline void stream_k(f32x4 (&acc)[MB][4], const uint4 *wp, const uint16_t *const (&xp)[MB],
                                const bool (&row_ok)[MB], const uint2 *sp, int count)
{
    // keep the two constants of expand_codes in registers so that each field pair costs one
    // and-or instead of an and and an or with 32-bit literals
    uint32_t mask = 0x00780078u, bias = 0x41804180u;
    asm volatile("" : "+v"(mask), "+v"(bias));
    Stage<MB> s0, s1;
    if (count > 0) load_stage<MB, SPG>(s0, wp, xp, row_ok, sp, 0);
    for (int ss = 0; ss < count; ss += 2) {
        if (ss + 1 < count) load_stage<MB, SPG>(s1, wp, xp, row_ok, sp, ss + 1);
        compute_stage<MB, SPG>(s0, acc, mask, bias);
        if (ss + 1 < count) {
            if (ss + 2 < count) load_stage<MB, SPG>(s0, wp, xp, row_ok, sp, ss + 2);
            compute_stage<MB, SPG>(s1, acc, mask, bias);
        }
    }
}

template <int MB>
__global__ __launch_bounds__(256) void base_expand_kernel(const LayerArgs a)
{
    constexpr int ROWS = 16 * MB;
    __shared__ float red[4][MB * 1024];
    __shared__ float t_s[ROWS][MLORA_MAX_RANK + 4];
    __shared__ int adapter_s[ROWS];

    int pi = 0;
    for (int i = 1; i < a.n_proj; ++i)
        if ((int)blockIdx.x >= a.p[i].tile_begin) pi = i;
    const ProjArgs &P = a.p[pi];
    const int tile = (int)blockIdx.x - P.tile_begin;
    const int m0 = (int)blockIdx.y * ROWS;
    const int K = P.K, N = P.N, M = a.M;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;

    // split the K/128 super-steps over the four waves
    const int nss = K / SUPER_K;
    const int q = nss / 4, r = nss % 4;
    const int my_beg = wave * q + min(wave, r), my_cnt = q + (wave < r ? 1 : 0);

    const int ksteps = K / KSTEP;
    const int ngroups = ksteps / P.spg;
    const uint4 *wp = P.codes + ((size_t)tile * ksteps + (size_t)my_beg * 4) * 64 + lane;
    const uint2 *sp = P.scales + ((size_t)tile * ngroups + (size_t)my_beg * (4 / P.spg)) * 16 + l16;
    const uint16_t *xp[MB];
    bool row_ok[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = m0 + mb * 16 + l16;
        row_ok[mb] = row < M;
        xp[mb] = P.x + (size_t)(row_ok[mb] ? row : 0) * K + (size_t)my_beg * SUPER_K + 8 * lq;
    }

    f32x4 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[mb][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (P.spg == 1)      stream_k<MB, 1>(acc, wp, xp, row_ok, sp, my_cnt);
    else if (P.spg == 2) stream_k<MB, 2>(acc, wp, xp, row_ok, sp, my_cnt);
    else                 stream_k<MB, 4>(acc, wp, xp, row_ok, sp, my_cnt);

    // partial tiles -> LDS; element (mb, j, e) of lane l is row 16*mb + 4*(l/16) + e,
    // column 16*j + l%16 of the block's tile
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[wave][((mb * 4 + j) * 4 + e) * 64 + lane] = acc[mb][j][e];

    // t[m] = alpha * sum of the shrink step's K-chunk partials (fixed order)
    const bool lora = (a.row_adapter != nullptr) && (P.n_adapters > 0);
    const int rows_here = min(ROWS, M - m0);
    if (tid < ROWS) {
        int ad = -1;
        if (lora && tid < rows_here) {
            ad = a.row_adapter[m0 + tid];
            if (ad < 0 || ad >= P.n_adapters) ad = -1;
        }
        adapter_s[tid] = ad;
    }
    if (lora) {
        for (int idx = tid; idx < rows_here * P.r16; idx += 256) {
            const int ml = idx / P.r16, jj = idx % P.r16;
            int ad = a.row_adapter[m0 + ml];
            float v = 0.f;
            if (ad >= 0 && ad < P.n_adapters)
                for (int kc = 0; kc < P.kch; ++kc)
                    v += P.t_part[((size_t)kc * M + (m0 + ml)) * P.r16 + jj];
            t_s[ml][jj] = v * P.alpha;
        }
    }
    __syncthreads();

    // thread (wave = e, lane) finishes elements (mb, j, e) for all mb, j
#pragma unroll
    for (int i = 0; i < 4 * MB; ++i) {
        const int mb = i >> 2, j = i & 3, e = wave;
        const int off = ((mb * 4 + j) * 4 + e) * 64 + lane;
        float v = ((red[0][off] + red[1][off]) + red[2][off]) + red[3][off];
        const int ml = mb * 16 + 4 * lq + e;
        const int m = m0 + ml;
        const int n = tile * TILE_N + 16 * j + l16;
        if (m < M && n < N) {
            const int ad = adapter_s[ml];
            if (ad >= 0) {
                const uint16_t *brow = P.lora_b + ((size_t)ad * N + n) * P.rank;
                float l = 0.f;
                for (int jj = 0; jj < P.rank; jj += 8) {
                    const uint4 b8 = *reinterpret_cast<const uint4 *>(brow + jj);
                    const float *t = &t_s[ml][jj];
                    l = fmaf(bf16_bits_to_float(b8.x & 0xFFFFu), t[0], l);
                    l = fmaf(bf16_bits_to_float(b8.x >> 16), t[1], l);
                    l = fmaf(bf16_bits_to_float(b8.y & 0xFFFFu), t[2], l);
                    l = fmaf(bf16_bits_to_float(b8.y >> 16), t[3], l);
                    l = fmaf(bf16_bits_to_float(b8.z & 0xFFFFu), t[4], l);
                    l = fmaf(bf16_bits_to_float(b8.z >> 16), t[5], l);
                    l = fmaf(bf16_bits_to_float(b8.w & 0xFFFFu), t[6], l);
                    l = fmaf(bf16_bits_to_float(b8.w >> 16), t[7], l);
                }
                v += l;
            }
            if (a.y_fp32) reinterpret_cast<float *>(P.y)[(size_t)m * N + n] = v;
            else reinterpret_cast<uint16_t *>(P.y)[(size_t)m * N + n] = float_to_bf16_bits(v);
        }
    }
}

hipError_t launch_base(const LayerArgs &a, int n_tiles, hipStream_t s)
{
    if (a.M <= 16) {
        base_expand_kernel<1><<<dim3((unsigned)n_tiles, 1), dim3(256), 0, s>>>(a);
    } else {
        const unsigned chunks = (unsigned)((a.M + 31) / 32);
        base_expand_kernel<2><<<dim3((unsigned)n_tiles, chunks), dim3(256), 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace mlora
