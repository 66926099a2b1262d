// Small kernels around the fused layer step: the per-row scale of RMSNorm.
#include "common.hpp"

namespace mlora {

// scale[m] = 1 / sqrt(mean_k x[m][k]^2 + eps).  One wavefront per row (four rows per block): every
// lane adds its share of the squares in a fixed order, and the 64 shares are added in a fixed
// butterfly, so the result does not depend on timing; no barrier, one round trip to memory for
// rows of up to 2048 inputs.
__global__ __launch_bounds__(256) void rms_scale_kernel(const uint16_t *x, int M, int K, float eps, float *scale)
{
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;                                    // (whole wavefronts: no lane of a live row leaves)
    const uint4 *row = reinterpret_cast<const uint4 *>(x + (size_t)m * K);
    float s = 0.f;
    for (int i0 = 0; i0 < K / 8; i0 += 4 * 64) {
        uint4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * 64 + lane;
            q[u] = i < K / 8 ? row[i] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t w[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float lo = __uint_as_float(w[j] << 16), hi = __uint_as_float(w[j] & 0xFFFF0000u);
                s = fmaf(lo, lo, s);
                s = fmaf(hi, hi, s);
            }
        }
    }
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) s += __shfl_xor(s, step, 64);
    if (lane == 0) scale[m] = 1.0f / sqrtf(s / (float)K + eps);
}

hipError_t launch_rms_scale(const uint16_t *x, int M, int K, float eps, float *scale, hipStream_t s)
{
    rms_scale_kernel<<<dim3((unsigned)((M + 3) / 4)), dim3(256), 0, s>>>(x, M, K, eps, scale);
    return hipGetLastError();
}

}  // namespace mlora
