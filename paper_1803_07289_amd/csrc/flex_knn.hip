// Exact K nearest neighbours on a uniform grid (the neighbourhoods of Sec. 3; the paper computes
// them beforehand and does not say how).  Result: for every point the K points of its cloud with the
// smallest squared distance, itself included, ordered by (d2, index).  d2 is evaluated in fp32 as
// ((dx*dx + dy*dy) + dz*dz) with every operation rounded on its own, the form the CPU check uses, so
// that the ranking (an integer-valued decision) comes out identical.
//
// Steps per call: bounding box of each cloud -> grid of cubic cells (at most 2^24 cells, about
// eight cells per point) -> counting sort of the points by cell (count, scan, fill of (x,y,z,id)
// records) -> one thread per point walks the shells of cells around its own cell, keeps the K best
// in registers and stops once the K-th distance is inside the block of cells already searched.
#include "flex_common.hpp"

namespace flex {

static constexpr int KNN_MAX_CELLS_LOG2 = 24;

// cells a cloud's grid may have: about eight per point
__host__ __device__ inline int64_t knn_cell_cap(int64_t N)
{
    const int64_t want = 8 * N;
    return want < ((int64_t)1 << KNN_MAX_CELLS_LOG2) ? want : ((int64_t)1 << KNN_MAX_CELLS_LOG2);
}

struct KnnGrid {
    float lo[3];      // bounding box minimum
    float inv_h, h;   // cell edge
    int n[3];         // cells per axis
};

__device__ __forceinline__ unsigned ordered_bits(float x)
{
    const unsigned u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(unsigned u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

// bbox[b][0..2] = min, [3..5] = max, as order-preserving unsigned keys (min starts at ~0, max at 0)
__global__ __launch_bounds__(256) void knn_bbox_init_kernel(unsigned *__restrict__ bbox, int B)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 6 * B) bbox[i] = (i % 6 < 3) ? 0xffffffffu : 0u;
}

__global__ __launch_bounds__(256) void knn_bbox_kernel(const float *__restrict__ pos, unsigned *__restrict__ bbox, int N)
{
    const int b = blockIdx.y;
    const float *p = pos + (int64_t)b * 3 * N;
    unsigned mn[3] = {0xffffffffu, 0xffffffffu, 0xffffffffu}, mx[3] = {0u, 0u, 0u};
    for (int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; l < N; l += (int64_t)gridDim.x * blockDim.x)
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            const unsigned k = ordered_bits(p[(int64_t)d * N + l]);
            mn[d] = min(mn[d], k);
            mx[d] = max(mx[d], k);
        }
#pragma unroll
    for (int d = 0; d < 3; ++d) {
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            mn[d] = min(mn[d], (unsigned)__shfl_xor((int)mn[d], s, 64));
            mx[d] = max(mx[d], (unsigned)__shfl_xor((int)mx[d], s, 64));
        }
    }
    // one pair of atomics per block and coordinate: thousands of atomics on the same six words serialise
    __shared__ unsigned s_mn[4][3], s_mx[4][3];
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0)
#pragma unroll
        for (int d = 0; d < 3; ++d) { s_mn[w][d] = mn[d]; s_mx[w][d] = mx[d]; }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int d = threadIdx.x;
        atomicMin(&bbox[6 * b + d], min(min(s_mn[0][d], s_mn[1][d]), min(s_mn[2][d], s_mn[3][d])));
        atomicMax(&bbox[6 * b + 3 + d], max(max(s_mx[0][d], s_mx[1][d]), max(s_mx[2][d], s_mx[3][d])));
    }
}

// every thread derives the same grid from the bounding box: cubic cells, about eight per point, at
// most 2^24 in total; a flat or degenerate box gets one layer of cells along its thin axes
__device__ __forceinline__ KnnGrid knn_grid(const unsigned *__restrict__ bbox, int b, int N)
{
    KnnGrid g;
    float ext[3];
#pragma unroll
    for (int d = 0; d < 3; ++d) {
        g.lo[d] = from_ordered_bits(bbox[6 * b + d]);
        ext[d] = fmaxf(from_ordered_bits(bbox[6 * b + 3 + d]) - g.lo[d], 0.f);
    }
    const float longest = fmaxf(fmaxf(ext[0], ext[1]), fmaxf(ext[2], 1e-30f));
    const int64_t cap = knn_cell_cap(N);
    float cells = (float)cap;
    float h = longest;                                   // one cell if everything else fails
    // volume / cells with thin axes counted as one cell thick; two refinements settle the estimate
    for (int it = 0; it < 3; ++it) {
        float vol = 1.f;
#pragma unroll
        for (int d = 0; d < 3; ++d) vol *= fmaxf(ext[d], h);
        h = cbrtf(vol / cells);
        h = fmaxf(h, longest * (1.f / 1024.f));          // at most 1024 cells along an axis
    }
    g.h = h;
    g.inv_h = 1.f / h;
    int64_t total = 1;
#pragma unroll
    for (int d = 0; d < 3; ++d) {
        g.n[d] = max(1, min(1024, (int)(ext[d] * g.inv_h) + 1));
        total *= g.n[d];
    }
    // rounding can push the product over the cap: coarsen until it fits
    for (int it = 0; it < 48 && total > cap; ++it) {
        g.h *= 1.26f; g.inv_h = 1.f / g.h;
        total = 1;
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            g.n[d] = max(1, min(1024, (int)(ext[d] * g.inv_h) + 1));
            total *= g.n[d];
        }
    }
    if (!(total <= cap)) { g.n[0] = g.n[1] = g.n[2] = 1; }   // only non-finite input gets here: one cell, exhaustive
    return g;
}

__device__ __forceinline__ void knn_cell_of(const KnnGrid &g, float x, float y, float z, int &cx, int &cy, int &cz)
{
    cx = min(g.n[0] - 1, max(0, (int)((x - g.lo[0]) * g.inv_h)));
    cy = min(g.n[1] - 1, max(0, (int)((y - g.lo[1]) * g.inv_h)));
    cz = min(g.n[2] - 1, max(0, (int)((z - g.lo[2]) * g.inv_h)));
}

// cell[b*N + l] = linear cell of the point; cnt[b*CELLS + cell] += 1
__global__ __launch_bounds__(256) void knn_count_kernel(const float *__restrict__ pos, const unsigned *__restrict__ bbox,
                                                        int32_t *__restrict__ cell, int32_t *__restrict__ cnt, int N,
                                                        int64_t cells_per_cloud)
{
    const int b = blockIdx.y;
    const KnnGrid g = knn_grid(bbox, b, N);
    const float *p = pos + (int64_t)b * 3 * N;
    for (int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; l < N; l += (int64_t)gridDim.x * blockDim.x) {
        int cx, cy, cz;
        knn_cell_of(g, p[l], p[(int64_t)N + l], p[2 * (int64_t)N + l], cx, cy, cz);
        const int c = (cz * g.n[1] + cy) * g.n[0] + cx;
        cell[(int64_t)b * N + l] = c;
        atomicAdd(&cnt[b * cells_per_cloud + c], 1);
    }
}

// rec[off[cell] + slot] = (x, y, z, id); cnt runs down to zero
__global__ __launch_bounds__(256) void knn_fill_kernel(const float *__restrict__ pos, const int32_t *__restrict__ cell,
                                                       const int32_t *__restrict__ off, int32_t *__restrict__ cnt,
                                                       float4 *__restrict__ rec, int N, int64_t cells_per_cloud)
{
    const int b = blockIdx.y;
    const float *p = pos + (int64_t)b * 3 * N;
    for (int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; l < N; l += (int64_t)gridDim.x * blockDim.x) {
        const int64_t c = b * cells_per_cloud + cell[(int64_t)b * N + l];
        const int slot = atomicSub(&cnt[c], 1) - 1;
        rec[off[c] + slot] = make_float4(p[l], p[(int64_t)N + l], p[2 * (int64_t)N + l], __int_as_float((int)l));
    }
}

// (d2, id) ascending
__device__ __forceinline__ bool knn_before(float d, int i, float bd, int bi) { return d < bd || (d == bd && i < bi); }

// One thread per point, in cell order (neighbouring threads search neighbouring cells).
template <int K>
__global__ __launch_bounds__(256) void knn_query_kernel(const float4 *__restrict__ rec, const int32_t *__restrict__ off,
                                                        const unsigned *__restrict__ bbox, int32_t *__restrict__ nbr,
                                                        int N, int64_t cells_per_cloud)
{
    const int b = blockIdx.y;
    const KnnGrid g = knn_grid(bbox, b, N);
    const int32_t *offb = off + b * cells_per_cloud;
    // slack for the rounding of the cell planes lo + c*h and of the cell a point was put in
    const float span = fmaxf(fmaxf(g.n[0], g.n[1]), (float)g.n[2]) * g.h;
    const float far = fmaxf(fmaxf(fabsf(g.lo[0]), fabsf(g.lo[1])), fabsf(g.lo[2])) + span;
    const float eps = 4e-6f * span + 2e-6f * far;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x) {
        const float4 me = rec[(int64_t)b * N + i];
        const int self = __float_as_int(me.w);
        int cx, cy, cz;
        knn_cell_of(g, me.x, me.y, me.z, cx, cy, cz);
        float bd[K];
        int bi[K];
#pragma unroll
        for (int k = 0; k < K; ++k) { bd[k] = __builtin_inff(); bi[k] = 0x7fffffff; }
        const int rmax = max(max(g.n[0], g.n[1]), g.n[2]);
        for (int r = 0; r <= rmax; ++r) {
            const int z0 = max(cz - r, 0), z1 = min(cz + r, g.n[2] - 1);
            const int y0 = max(cy - r, 0), y1 = min(cy + r, g.n[1] - 1);
            const int x0 = max(cx - r, 0), x1 = min(cx + r, g.n[0] - 1);
            for (int z = z0; z <= z1; ++z)
                for (int y = y0; y <= y1; ++y) {
                    const bool face = (abs(z - cz) == r) || (abs(y - cy) == r);
                    // on a face row every x is on the shell; otherwise only the two ends are
                    const int xs = face ? 1 : max(2 * r, 1);
                    for (int x = face ? x0 : cx - r; x <= x1; x += xs) {
                        if (x < x0) continue;
                        const int c = (z * g.n[1] + y) * g.n[0] + x;
                        const int e1 = offb[c + 1];
                        for (int e = offb[c]; e < e1; ++e) {
                            const float4 q = rec[e];
                            const float dx = __fsub_rn(q.x, me.x), dy = __fsub_rn(q.y, me.y), dz = __fsub_rn(q.z, me.z);
                            const float d2 = __fadd_rn(__fadd_rn(__fmul_rn(dx, dx), __fmul_rn(dy, dy)), __fmul_rn(dz, dz));
                            int id = __float_as_int(q.w);
                            if (!knn_before(d2, id, bd[K - 1], bi[K - 1])) continue;
                            float d = d2;
#pragma unroll
                            for (int k = 0; k < K; ++k) {        // sorted insertion: the candidate bubbles down the list
                                const bool first = knn_before(d, id, bd[k], bi[k]);
                                const float td = first ? bd[k] : d;
                                const int ti = first ? bi[k] : id;
                                bd[k] = first ? d : bd[k];
                                bi[k] = first ? id : bi[k];
                                d = td; id = ti;
                            }
                        }
                    }
                }
            // everything outside the block of cells [c-r, c+r] is at least `reach` away
            float reach = __builtin_inff();
            if (cx - r > 0) reach = fminf(reach, me.x - (g.lo[0] + (float)(cx - r) * g.h));
            if (cx + r < g.n[0] - 1) reach = fminf(reach, (g.lo[0] + (float)(cx + r + 1) * g.h) - me.x);
            if (cy - r > 0) reach = fminf(reach, me.y - (g.lo[1] + (float)(cy - r) * g.h));
            if (cy + r < g.n[1] - 1) reach = fminf(reach, (g.lo[1] + (float)(cy + r + 1) * g.h) - me.y);
            if (cz - r > 0) reach = fminf(reach, me.z - (g.lo[2] + (float)(cz - r) * g.h));
            if (cz + r < g.n[2] - 1) reach = fminf(reach, (g.lo[2] + (float)(cz + r + 1) * g.h) - me.z);
            reach -= eps;
            if (reach == __builtin_inff()) break;                       // the block is the whole grid
            if (reach > 0.f && bd[K - 1] < reach * reach * 0.999999f) break;
        }
#pragma unroll
        for (int k = 0; k < K; ++k) nbr[((int64_t)b * K + k) * N + self] = bi[k];
    }
}

size_t knn_ws_bytes(int B, int N)
{
    const int64_t cells = (int64_t)B * knn_cell_cap(N);
    return align256(sizeof(float4) * (size_t)B * N) + align256(sizeof(int32_t) * (size_t)B * N) +
           align256(sizeof(int32_t) * (size_t)(cells + 1)) * 2 + exclusive_scan_ws_bytes(cells) + align256(sizeof(unsigned) * 6 * (size_t)B);
}

hipError_t launch_knn(const float *pos, int32_t *nbr, int B, int N, int K, void *ws, hipStream_t s)
{
    const int64_t cpc = knn_cell_cap(N), cells = (int64_t)B * cpc;
    char *at = (char *)ws;
    float4 *rec = (float4 *)at;       at += align256(sizeof(float4) * (size_t)B * N);
    int32_t *cell = (int32_t *)at;    at += align256(sizeof(int32_t) * (size_t)B * N);
    int32_t *cnt = (int32_t *)at;     at += align256(sizeof(int32_t) * (size_t)(cells + 1));
    int32_t *off = (int32_t *)at;     at += align256(sizeof(int32_t) * (size_t)(cells + 1));
    void *scan_ws = at;               at += exclusive_scan_ws_bytes(cells);
    unsigned *bbox = (unsigned *)at;
    hipLaunchKernelGGL(knn_bbox_init_kernel, dim3((6 * B + 255) / 256), dim3(256), 0, s, bbox, B);
    int nb = (int)((N + 255) / 256);
    if (nb > 2048) nb = 2048;
    hipLaunchKernelGGL(knn_bbox_kernel, dim3(nb < 512 ? nb : 512, B), dim3(256), 0, s, pos, bbox, N);
    hipError_t e = launch_fill_zero(cnt, sizeof(int32_t) * (size_t)cells, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(knn_count_kernel, dim3(nb, B), dim3(256), 0, s, pos, bbox, cell, cnt, N, cpc);
    e = launch_exclusive_scan_i32(cnt, off, cells, scan_ws, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(knn_fill_kernel, dim3(nb, B), dim3(256), 0, s, pos, cell, off, cnt, rec, N, cpc);
    int qb = (int)((N + 255) / 256);
    if (qb > 65535) qb = 65535;
#define FLEX_KNN_CASE(KK) \
    case KK: hipLaunchKernelGGL(knn_query_kernel<KK>, dim3(qb, B), dim3(256), 0, s, rec, off, bbox, nbr, N, cpc); break;
    switch (K) {
        FLEX_KNN_CASE(1) FLEX_KNN_CASE(2) FLEX_KNN_CASE(3) FLEX_KNN_CASE(4) FLEX_KNN_CASE(5) FLEX_KNN_CASE(6)
        FLEX_KNN_CASE(7) FLEX_KNN_CASE(8) FLEX_KNN_CASE(9) FLEX_KNN_CASE(10) FLEX_KNN_CASE(12) FLEX_KNN_CASE(16)
        FLEX_KNN_CASE(24) FLEX_KNN_CASE(32)
    default: return hipErrorInvalidValue;
    }
#undef FLEX_KNN_CASE
    return hipGetLastError();
}

bool knn_k_supported(int K)
{
    return (K >= 1 && K <= 10) || K == 12 || K == 16 || K == 24 || K == 32;
}

}  // namespace flex
