// Measurement aids: what this device reaches on a plain copy and on a pure f16 matrix-op loop, so that a benchmark
// can quote its kernels against measured peaks beside the published ones.  Neither is part of the layers.
#include "flex_common.hpp"
#include "../../include/flexconv.h"

namespace flex {

// dst[i] = src[i], 16 bytes per thread, one block per 4 KB: reads n16 * 16 bytes and writes as many.  Blocks that
// each move one piece and are dispatched in order keep the accesses of the whole chip in one narrow, advancing
// window of memory: 6.2 TB/s on this part, where a resident grid striding over the buffer reaches 4.8-5.0 TB/s
// (its blocks drift apart) and the runtime's own device-to-device copy 5.0 TB/s.
__global__ __launch_bounds__(256) void calibrate_copy_kernel(const v4f *__restrict__ src, v4f *__restrict__ dst,
                                                             int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// iters x 4 independent chains of v_mfma_f32_16x16x32_f16 per wave, operands in registers: 16 waves per CU keep the
// matrix pipes of all four SIMDs fed.  One matrix op = 2 * 16 * 16 * 32 = 16 384 flop.
__global__ __launch_bounds__(1024) void calibrate_mfma_f16_kernel(int iters, float *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    h8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.001f * (float)((lane + i) & 15));
        b[i] = (_Float16)(0.002f * (float)((lane * 3 + i) & 7));
    }
    v4f c0 = {0.f, 0.f, 0.f, 0.f}, c1 = c0, c2 = c0, c3 = c0;
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c3, 0, 0, 0);
    }
    const v4f s = (c0 + c1) + (c2 + c3);
    if (s[0] + s[1] + s[2] + s[3] == 12345.678f) sink[0] = s[0];      // keeps the loop alive, never true
}

}  // namespace flex

using namespace flex;

extern "C" {

int flex_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return FLEX_ERR_NULL;
    if (bytes == 0 || (bytes & 15) != 0 || (((uintptr_t)src | (uintptr_t)dst) & 15) != 0) return FLEX_ERR_SHAPE;
    const int64_t n16 = (int64_t)(bytes / 16), blocks = (n16 + 255) / 256;
    if (blocks > 0x7fffffff) return FLEX_ERR_SHAPE;
    hipLaunchKernelGGL(calibrate_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const v4f *)src, (v4f *)dst, n16);
    return hipGetLastError() == hipSuccess ? FLEX_OK : FLEX_ERR_HIP;
}

int flex_calibrate_mfma_f16(int iters, float *sink, double *flop_out, void *stream)
{
    if (!sink) return FLEX_ERR_NULL;
    if (iters <= 0 || iters > (1 << 24)) return FLEX_ERR_SHAPE;
    const int grid = device_cu_count();                 // one 16-wave workgroup per CU
    hipLaunchKernelGGL(calibrate_mfma_f16_kernel, dim3(grid), dim3(1024), 0, (hipStream_t)stream, iters, sink);
    if (flop_out) *flop_out = (double)grid * 16.0 * (double)iters * 4.0 * 16384.0;
    return hipGetLastError() == hipSuccess ? FLEX_OK : FLEX_ERR_HIP;
}

}  // extern "C"
