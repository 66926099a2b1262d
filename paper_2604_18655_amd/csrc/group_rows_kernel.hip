// Row grouping as a call of its own (the layer kernels run the same code as their first step).
#include "group_rows.hpp"

namespace mlora {

__global__ __launch_bounds__(256) void group_rows_kernel(const int *row_adapter, int M,
                                                        int n_adapters, int *perm,
                                                        int *seg_adapter, int *seg_start,
                                                        int *n_seg)
{
    __shared__ GroupLds g;
    group_rows_lds(row_adapter, M, n_adapters, g);
    const int tid = threadIdx.x;
    for (int m = tid; m < M; m += 256) perm[m] = g.perm[m];
    for (int s = tid; s < g.n_seg; s += 256) seg_adapter[s] = g.seg_adapter[s];
    for (int s = tid; s <= g.n_seg; s += 256) seg_start[s] = g.seg_start[s];
    if (tid == 0) *n_seg = g.bad ? -1 : g.n_seg;
}

hipError_t launch_group_rows(const int *row_adapter, int M, int n_adapters, int *perm,
                             int *seg_adapter, int *seg_start, int *n_seg, hipStream_t s)
{
    group_rows_kernel<<<dim3(1), dim3(256), 0, s>>>(row_adapter, M, n_adapters, perm, seg_adapter,
                                                    seg_start, n_seg);
    return hipGetLastError();
}

}  // namespace mlora
