// Streaming kernels of known traffic.  They exist for measurement only: their bandwidth is the ceiling that a
// streaming kernel with the same mix of reads and writes reaches on the box at hand, and the plain copy's
// hardware-counter readings calibrate the HBM byte counters.
#include "dev_common.h"
#include "kernels.h"

// MODE 1: dst = src around the caches (non-temporal loads and stores; the plain copy through the caches is
// k_copy_probe below); 2: read only (every workgroup leaves one float4 so that the loads cannot be dropped); 3: three reads per
// write, dst = src[0] + src[1] + src[2] with the three blocks of n4 chunks behind one another in src, around
// the caches -- the read share (75 %) of a table update with many gradient blocks.
template <int MODE>
__global__ void __launch_bounds__(BLOCK) k_stream_probe(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n4)
{
    size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * BLOCK;
    if (MODE == 1) {
        for (; i < n4; i += stride) st4s((float *)(dst + i), ld4s((const float *)(src + i)));
    } else if (MODE == 2) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (; i < n4; i += stride) {
            const float4 v = ld4s((const float *)(src + i));
            acc.x += v.x;
            acc.y += v.y;
            acc.z += v.z;
            acc.w += v.w;
        }
        acc.x = wave_sum(acc.x + acc.y + acc.z + acc.w);
        if (threadIdx.x == 0) dst[blockIdx.x] = acc;
    } else {
        for (; i < n4; i += stride) {
            const float4 a = ld4s((const float *)(src + i));
            const float4 b = ld4s((const float *)(src + n4 + i));
            const float4 c = ld4s((const float *)(src + 2 * n4 + i));
            st4s((float *)(dst + i), make_float4(a.x + b.x + c.x, a.y + b.y + c.y, a.z + b.z + c.z, a.w + b.w + c.w));
        }
    }
}

// the name under which the plain copy appears in profiles
__global__ void __launch_bounds__(BLOCK) k_copy_probe(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n4)
{
    size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * BLOCK;
    for (; i < n4; i += stride) dst[i] = src[i];
}

void tn_launch_stream_probe(void *dst, const void *src, size_t bytes, int mode, hipStream_t st)
{
    size_t n4 = bytes / 16;
    if (n4 == 0) return;
    size_t want = (n4 + BLOCK - 1) / BLOCK;
    int blocks = (int)(want > 256 * 64 ? 256 * 64 : want);
    const float4 *s = (const float4 *)src;
    float4 *d = (float4 *)dst;
    switch (mode) {
    case 0: hipLaunchKernelGGL(k_copy_probe, dim3(blocks), dim3(BLOCK), 0, st, s, d, n4); break;
    case 1: hipLaunchKernelGGL(k_stream_probe<1>, dim3(blocks), dim3(BLOCK), 0, st, s, d, n4); break;
    case 2: hipLaunchKernelGGL(k_stream_probe<2>, dim3(blocks), dim3(BLOCK), 0, st, s, d, n4); break;
    default: hipLaunchKernelGGL(k_stream_probe<3>, dim3(blocks), dim3(BLOCK), 0, st, s, d, n4); break;
    }
}

void tn_launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    tn_launch_stream_probe(dst, src, bytes, 0, st);
}
