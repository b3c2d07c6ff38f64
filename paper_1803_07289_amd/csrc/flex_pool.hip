// Flex-max-pooling (Sec. 4.1): per-neighbourhood maximum with the winning
// point's index recorded for the backward pass.  Bandwidth-bound: the forward
// pass gathers whole point-major rows (16 bytes per lane), the backward pass
// scatters by the recorded index with fp32 atomic adds.
#include "flex_common.hpp"

namespace flex {

// (value desc, point index asc): the winner among equal values is the lowest index.
__device__ __forceinline__ void take(float v, int n, float &bv, int &bn)
{
    if (v > bv || (v == bv && n < bn)) { bv = v; bn = n; }
}

// Point-major, C % 4 == 0: one thread per (point, 4 channels).
__global__ __launch_bounds__(256) void pool_fwd_bnc4_kernel(const float *__restrict__ feat,
                                                            const int32_t *__restrict__ nbr,
                                                            float *__restrict__ out,
                                                            int32_t *__restrict__ argmax, int B,
                                                            int N, int K, int C4)
{
    const int64_t total = (int64_t)B * N * C4;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int c4 = (int)(i % C4);
        const int64_t gp = i / C4;
        const int b = (int)(gp / N), l = (int)(gp % N);
        const int32_t *nb = nbr + (int64_t)b * K * N + l;
        const v4f *rows = reinterpret_cast<const v4f *>(feat) + (int64_t)b * N * C4 + c4;
        int n = nb[0];
        const v4f first = rows[(int64_t)n * C4];
        float v0 = first.x, v1 = first.y, v2 = first.z, v3 = first.w;
        int b0 = n, b1 = n, b2 = n, b3 = n;
        for (int k = 1; k < K; ++k) {
            n = nb[(int64_t)k * N];
            const v4f v = rows[(int64_t)n * C4];
            take(v.x, n, v0, b0);
            take(v.y, n, v1, b1);
            take(v.z, n, v2, b2);
            take(v.w, n, v3, b3);
        }
        const v4f bv = {v0, v1, v2, v3};
        reinterpret_cast<v4f *>(out)[i] = bv;
        reinterpret_cast<int4 *>(argmax)[i] = make_int4(b0, b1, b2, b3);
    }
}

// Any C, either layout: one thread per output element.
__global__ __launch_bounds__(256) void pool_fwd_generic_kernel(const float *__restrict__ feat,
                                                               const int32_t *__restrict__ nbr,
                                                               float *__restrict__ out,
                                                               int32_t *__restrict__ argmax, int B,
                                                               int N, int K, int C, int bnc)
{
    const int64_t total = (int64_t)B * N * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int b, c, l;
        if (bnc) { c = (int)(i % C); const int64_t gp = i / C; b = (int)(gp / N); l = (int)(gp % N); }
        else     { l = (int)(i % N); const int64_t bc = i / N; b = (int)(bc / C); c = (int)(bc % C); }
        const int32_t *nb = nbr + (int64_t)b * K * N + l;
        int bn = nb[0];
        float bv = bnc ? feat[((int64_t)b * N + bn) * C + c] : feat[((int64_t)b * C + c) * N + bn];
        for (int k = 1; k < K; ++k) {
            const int n = nb[(int64_t)k * N];
            const float v = bnc ? feat[((int64_t)b * N + n) * C + c] : feat[((int64_t)b * C + c) * N + n];
            take(v, n, bv, bn);
        }
        out[i] = bv;
        argmax[i] = bn;
    }
}

hipError_t launch_pool_fwd(const float *feat, const int32_t *nbr, float *out, int32_t *argmax,
                           int B, int N, int K, int C, int bnc, hipStream_t s)
{
    if (bnc && (C % 4 == 0)) {
        const int64_t total = (int64_t)B * N * (C / 4);
        int64_t blocks = (total + 255) / 256;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(pool_fwd_bnc4_kernel, dim3((unsigned)blocks), dim3(256), 0, s, feat, nbr,
                           out, argmax, B, N, K, C / 4);
    } else {
        const int64_t total = (int64_t)B * N * C;
        int64_t blocks = (total + 255) / 256;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(pool_fwd_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, feat, nbr,
                           out, argmax, B, N, K, C, bnc);
    }
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void pool_bwd_kernel(const float *__restrict__ grad_out,
                                                       const int32_t *__restrict__ argmax,
                                                       float *__restrict__ grad_feat, int B, int N,
                                                       int C, int bnc)
{
    const int64_t total = (int64_t)B * N * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int m = argmax[i];
        int64_t dst;
        if (bnc) { const int c = (int)(i % C); const int64_t gp = i / C; const int64_t b = gp / N;
                   dst = (b * N + m) * C + c; }
        else     { const int64_t bc = i / N; dst = bc * N + m; }
        atomicAdd(&grad_feat[dst], grad_out[i]);
    }
}

hipError_t launch_pool_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat, int B,
                           int N, int C, int bnc, hipStream_t s)
{
    hipError_t e = launch_fill_zero(grad_feat, sizeof(float) * (size_t)B * N * C, s);
    if (e != hipSuccess) return e;
    const int64_t total = (int64_t)B * N * C;
    int64_t blocks = (total + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    hipLaunchKernelGGL(pool_bwd_kernel, dim3((unsigned)blocks), dim3(256), 0, s, grad_out, argmax,
                       grad_feat, B, N, C, bnc);
    return hipGetLastError();
}

}  // namespace flex
