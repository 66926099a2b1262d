// Small kernels around the fused layer step: the per-row scale of RMSNorm.
#include "common.hpp"

namespace mlora {

// scale[m] = 1 / sqrt(mean_k x[m][k]^2 + eps).  One block per row; every thread adds its share of
// the squares in a fixed order and the block adds the shares in a fixed tree: the result does
// not depend on timing.
__global__ __launch_bounds__(256) void rms_scale_kernel(const uint16_t *x, int K, float eps, float *scale)
{
    __shared__ float part[256];
    const int m = blockIdx.x, tid = threadIdx.x;
    const uint4 *row = reinterpret_cast<const uint4 *>(x + (size_t)m * K);
    float s = 0.f;
    for (int i = tid; i < K / 8; i += 256) {
        const uint4 q = row[i];
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float lo = __uint_as_float(w[j] << 16), hi = __uint_as_float(w[j] & 0xFFFF0000u);
            s = fmaf(lo, lo, s);
            s = fmaf(hi, hi, s);
        }
    }
    part[tid] = s;
    __syncthreads();
    for (int step = 128; step >= 1; step >>= 1) {
        if (tid < step) part[tid] += part[tid + step];
        __syncthreads();
    }
    if (tid == 0) scale[m] = 1.0f / sqrtf(part[0] / (float)K + eps);
}

hipError_t launch_rms_scale(const uint16_t *x, int M, int K, float eps, float *scale, hipStream_t s)
{
    rms_scale_kernel<<<dim3((unsigned)M), dim3(256), 0, s>>>(x, K, eps, scale);
    return hipGetLastError();
}

}  // namespace mlora
