// Canonical int4 weight <-> prepacked blob (see common.hpp for the layout).
#include "common.hpp"

namespace mlora {

// one thread per uint4 of the code region
__global__ __launch_bounds__(256) void prepack_codes_kernel(int K, int N, const uint8_t *wq,
                                                           uint4 *codes, size_t n_vec)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_vec) return;
    const int ksteps = K / KSTEP;
    const int lane = (int)(idx & 63);
    const int step = (int)((idx >> 6) % (size_t)ksteps);
    const int tile = (int)((idx >> 6) / (size_t)ksteps);
    const int k0 = step * KSTEP + 8 * (lane >> 4);
    uint32_t out[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = tile * TILE_N + 16 * j + (lane & 15);
        uint32_t nibbles = 0;                       // code 0 everywhere beyond N
        if (n < N) nibbles = *reinterpret_cast<const uint32_t *>(wq + (size_t)n * (K / 2) + k0 / 2);
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t u = ((nibbles >> (4 * i)) & 15u) ^ 8u;   // two's complement -> code + 8
            w |= rotl32(u, field_pos(i));
        }
        out[j] = w;
    }
    codes[idx] = make_uint4(out[0], out[1], out[2], out[3]);
}

// one thread per fp16 of the scale region
__global__ __launch_bounds__(256) void prepack_scales_kernel(int K, int N, int group,
                                                            const uint16_t *scales,
                                                            uint16_t *out, size_t n_half)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_half) return;
    const int ngroups = K / group;
    const int j = (int)(idx & 3);
    const int c = (int)((idx >> 2) & 15);
    const int g = (int)((idx >> 6) % (size_t)ngroups);
    const int tile = (int)((idx >> 6) / (size_t)ngroups);
    const int n = tile * TILE_N + 16 * j + c;
    out[idx] = (n < N) ? scales[(size_t)n * ngroups + g] : (uint16_t)0;
}

// one thread per 8 consecutive inputs of one output column
__global__ __launch_bounds__(256) void unpack_kernel(int K, int N, int group, const uint4 *codes,
                                                    const uint16_t *scales, int8_t *out_codes,
                                                    float *out_w, size_t n_oct)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_oct) return;
    const int octs = K / 8;
    const int n = (int)(idx / (size_t)octs);
    const int k0 = (int)(idx % (size_t)octs) * 8;
    const int tile = n / TILE_N, j = (n % TILE_N) / 16, c = n % 16;
    const int step = k0 / KSTEP, lane = ((k0 % KSTEP) / 8) * 16 + c;
    const uint4 v = codes[((size_t)tile * (K / KSTEP) + step) * 64 + lane];
    const uint32_t w = j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w;
    const int ngroups = K / group;
    const uint16_t sb = scales[(((size_t)tile * ngroups + k0 / group) * 16 + c) * 4 + j];
    const float s = half_bits_to_float(sb);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int code = (int)(rotr32(w, field_pos(i)) & 15u) - 8;
        if (out_codes) out_codes[(size_t)n * K + k0 + i] = (int8_t)code;
        if (out_w) out_w[(size_t)n * K + k0 + i] = (float)code * s;   // exact: 4 bits x 11 bits
    }
}

hipError_t launch_prepack(int K, int N, int group, const uint8_t *wq, const uint16_t *scales,
                          void *blob, hipStream_t s)
{
    const size_t n_vec = blob_code_bytes(K, N) / 16;
    const size_t n_half = blob_scale_bytes(K, N, group) / 2;
    uint4 *codes = reinterpret_cast<uint4 *>(blob);
    uint16_t *sc = reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(blob) + blob_code_bytes(K, N));
    prepack_codes_kernel<<<dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, s>>>(K, N, wq, codes, n_vec);
    prepack_scales_kernel<<<dim3((unsigned)((n_half + 255) / 256)), dim3(256), 0, s>>>(K, N, group, scales, sc, n_half);
    return hipGetLastError();
}

hipError_t launch_unpack(int K, int N, int group, const void *blob, int8_t *codes, float *w_f32,
                         hipStream_t s)
{
    const size_t n_oct = (size_t)N * (K / 8);
    const uint4 *c = reinterpret_cast<const uint4 *>(blob);
    const uint16_t *sc = reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(blob) + blob_code_bytes(K, N));
    unpack_kernel<<<dim3((unsigned)((n_oct + 255) / 256)), dim3(256), 0, s>>>(K, N, group, c, sc, codes, w_f32, n_oct);
    return hipGetLastError();
}

}  // namespace mlora
