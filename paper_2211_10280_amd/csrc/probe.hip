// A plain device-to-device copy kernel of known traffic (bytes read = bytes written = size).
// It exists for measurement only: its bandwidth is the ceiling a streaming kernel reaches on
// the box at hand, and its hardware-counter readings calibrate the HBM byte counters.
#include "dev_common.h"
#include "kernels.h"

__global__ void __launch_bounds__(BLOCK) k_copy_probe(const float4 *__restrict__ src,
                                                      float4 *__restrict__ dst, size_t n4)
{
    size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * BLOCK;
    for (; i < n4; i += stride) dst[i] = src[i];
}

void tn_launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    size_t n4 = bytes / 16;
    if (n4 == 0) return;
    size_t want = (n4 + BLOCK - 1) / BLOCK;
    int blocks = (int)(want > 256 * 64 ? 256 * 64 : want);
    hipLaunchKernelGGL(k_copy_probe, dim3(blocks), dim3(BLOCK), 0, st, (const float4 *)src,
                       (float4 *)dst, n4);
}
