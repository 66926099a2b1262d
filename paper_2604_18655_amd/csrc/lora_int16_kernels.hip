// LoRA tensors stored as int16 (one scale per stack) turned into the bf16 operands of the layer
// step, exactly: an int16 is 256 * hi + lo with hi in [-128, 127] and lo in [0, 255], both of
// which (and their multiples by powers of two) are bf16 numbers, so
//     Bq (Aq x) = (256 Bh + Bl) (256 (Ah x) + (Al x))
// is the product of a LoRA pair of four times the rank:
//     A'' = [Ah; Ah; Al; Al]                  rows j, r + j, 2r + j, 3r + j from row j of Aq
//     B'' = [65536 Bh | 256 Bl | 256 Bh | Bl]   columns likewise from column j of Bq.
// The matrix units then see integers, and what rounding there is happens in the fp32 sums.
#include "common.hpp"

namespace mlora {

// bf16 bits of an integer of at most 8 significant bits times a power of two (exact: the top half
// of its float32 pattern)
__device__ __forceinline__ uint16_t small_int_to_bf16_bits(float v) { return (uint16_t)(__float_as_uint(v) >> 16); }

// one thread per int16 of Aq [n_ad][r][K] -> four bf16 of A'' [n_ad][4r][K]
__global__ __launch_bounds__(256) void lora_int16_expand_a_kernel(const int16_t *aq, size_t total, int r, int K, uint16_t *a4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const size_t row = i / (size_t)K, k = i % (size_t)K;      // row = adapter * r + j
    const size_t ad = row / (size_t)r, j = row % (size_t)r;
    const int v = aq[i];
    const uint16_t hi = small_int_to_bf16_bits((float)(v >> 8)), lo = small_int_to_bf16_bits((float)(v & 255));
    uint16_t *dst = a4 + (ad * 4 * (size_t)r + j) * (size_t)K + k;
    const size_t step = (size_t)r * (size_t)K;
    dst[0] = hi;
    dst[step] = hi;
    dst[2 * step] = lo;
    dst[3 * step] = lo;
}

// one thread per int16 of Bq [n_ad][N][r] -> four bf16 of B'' [n_ad][N][4r]
__global__ __launch_bounds__(256) void lora_int16_expand_b_kernel(const int16_t *bq, size_t total, int r, uint16_t *b4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const size_t line = i / (size_t)r, j = i % (size_t)r;     // line = adapter * N + n
    const int v = bq[i];
    const float hi = (float)(v >> 8), lo = (float)(v & 255);
    uint16_t *dst = b4 + line * 4 * (size_t)r + j;
    dst[0] = small_int_to_bf16_bits(65536.0f * hi);
    dst[r] = small_int_to_bf16_bits(256.0f * lo);
    dst[2 * r] = small_int_to_bf16_bits(256.0f * hi);
    dst[3 * r] = small_int_to_bf16_bits(lo);
}

hipError_t launch_lora_int16_expand(const int16_t *aq, const int16_t *bq, int n_adapters, int rank, int K, int N,
                                    uint16_t *a4, uint16_t *b4, hipStream_t s)
{
    const size_t na = (size_t)n_adapters * rank * K, nb = (size_t)n_adapters * N * rank;
    lora_int16_expand_a_kernel<<<dim3((unsigned)((na + 255) / 256)), dim3(256), 0, s>>>(aq, na, rank, K, a4);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    lora_int16_expand_b_kernel<<<dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, s>>>(bq, nb, rank, b4);
    return hipGetLastError();
}

}  // namespace mlora
