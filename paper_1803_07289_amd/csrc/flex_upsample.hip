// Flex-upsampling (Sec. 4.1): the smaller layer's features are copied to their points in the
// larger layer, every other point counts as zero, and flex-max-pooling runs over the larger
// layer's neighbourhoods.  The zero-filled tensor is never written: an inverse map
// inv[b*Nf + m] = j (or -1) is built in the workspace and the pooling gather reads row
// inv[n] of the smaller layer, or takes 0.  Same tie rule as the pooling layer.
#include "flex_common.hpp"

namespace flex {

// (value desc, point index asc): the winner among equal values is the lowest index.
__device__ __forceinline__ void take_up(float v, int n, float &bv, int &bn)
{
    // as selects (measured faster here than the short-circuit `if`, which compiles to exec-mask code; the plain
    // pooling kernel is the other way round and keeps the `if`)
    const bool better = (v > bv) | ((v == bv) & (n < bn));
    bv = better ? v : bv;
    bn = better ? n : bn;
}

__device__ __forceinline__ int64_t xcd_tile_up(int64_t total_tiles)
{
    const int64_t per_xcd = (total_tiles + 7) >> 3;
    const int64_t slot = blockIdx.x >> 3;
    const int64_t tile = (int64_t)(blockIdx.x & 7) * per_xcd + slot;
    return (slot < per_xcd && tile < total_tiles) ? tile : -1;
}
static inline unsigned xcd_grid_up(int64_t total_tiles) { return (unsigned)(((total_tiles + 7) >> 3) << 3); }

__global__ __launch_bounds__(256) void upsample_inv_fill_kernel(int32_t *__restrict__ inv, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        inv[i] = -1;
}

// inv[b*Nf + sel[b,j]] = j; entries of sel outside [0,Nf) are skipped (flex_validate_selection counts them)
__global__ __launch_bounds__(256) void upsample_inv_scatter_kernel(const int32_t *__restrict__ sel,
                                                                   int32_t *__restrict__ inv, int B, int Ns,
                                                                   int Nf)
{
    const int64_t total = (int64_t)B * Ns;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = i / Ns;
        const int m = sel[i];
        if (m >= 0 && m < Nf) inv[b * Nf + m] = (int)(i - b * Ns);
    }
}

// Point-major, C % 4 == 0: one thread per (larger-layer point, 4 channels); ids, then inverse-map
// entries, then rows of 8 neighbours are requested before anything is compared.
__global__ __launch_bounds__(256) void upsample_fwd_bnc4_kernel(const float *__restrict__ feat_small,
                                                                const int32_t *__restrict__ inv,
                                                                const int32_t *__restrict__ nbr,
                                                                float *__restrict__ out,
                                                                int32_t *__restrict__ argmax, int64_t BN,
                                                                int Ns, int Nf, int K, int C4, int PT,
                                                                int64_t total_tiles)
{
    constexpr int U = 8;
    const int64_t tile = xcd_tile_up(total_tiles);
    if (tile < 0) return;
    for (int i = threadIdx.x; i < PT * C4; i += 256) {
        const int c4 = i % C4;
        const int64_t gp = tile * PT + i / C4;
        if (gp >= BN) break;
        const int b = (int)(gp / Nf), l = (int)(gp % Nf);
        const int32_t *nb = nbr + (int64_t)b * K * Nf + l;
        const int32_t *iv = inv + (int64_t)b * Nf;
        const v4f *rows = reinterpret_cast<const v4f *>(feat_small) + (int64_t)b * Ns * C4 + c4;
        float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
        int b0 = 0, b1 = 0, b2 = 0, b3 = 0;
        for (int k0 = 0; k0 < K; k0 += U) {
            int n[U], j[U];
            v4f v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) n[u] = nb[(int64_t)min(k0 + u, K - 1) * Nf];   // past K: the last slot again
#pragma unroll
            for (int u = 0; u < U; ++u) j[u] = iv[n[u]];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                v[u] = v4f{0.f, 0.f, 0.f, 0.f};                      // a point that was only zero-filled
                if (j[u] >= 0) v[u] = rows[(int64_t)j[u] * C4];
            }
            if (k0 == 0) {
                v0 = v[0].x; v1 = v[0].y; v2 = v[0].z; v3 = v[0].w;
                b0 = b1 = b2 = b3 = n[0];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                take_up(v[u].x, n[u], v0, b0);
                take_up(v[u].y, n[u], v1, b1);
                take_up(v[u].z, n[u], v2, b2);
                take_up(v[u].w, n[u], v3, b3);
            }
        }
        const v4f bv = {v0, v1, v2, v3};
        // streaming stores, as in the pooling kernels
        typedef int i4v __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(bv, &reinterpret_cast<v4f *>(out)[gp * C4 + c4]);
        const i4v bi = {b0, b1, b2, b3};
        __builtin_nontemporal_store(bi, &reinterpret_cast<i4v *>(argmax)[gp * C4 + c4]);
    }
}

// Any C, either layout: one thread per output element.
__global__ __launch_bounds__(256) void upsample_fwd_generic_kernel(const float *__restrict__ feat_small,
                                                                   const int32_t *__restrict__ inv,
                                                                   const int32_t *__restrict__ nbr,
                                                                   float *__restrict__ out,
                                                                   int32_t *__restrict__ argmax, int B, int Ns,
                                                                   int Nf, int K, int C, int bnc)
{
    const int64_t total = (int64_t)B * Nf * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int b, c, l;
        if (bnc) { c = (int)(i % C); const int64_t gp = i / C; b = (int)(gp / Nf); l = (int)(gp % Nf); }
        else     { l = (int)(i % Nf); const int64_t bc = i / Nf; b = (int)(bc / C); c = (int)(bc % C); }
        const int32_t *nb = nbr + (int64_t)b * K * Nf + l;
        const int32_t *iv = inv + (int64_t)b * Nf;
        auto value = [&](int n) {
            const int j = iv[n];
            if (j < 0) return 0.f;
            return bnc ? feat_small[((int64_t)b * Ns + j) * C + c] : feat_small[((int64_t)b * C + c) * Ns + j];
        };
        int bn = nb[0];
        float bv = value(bn);
        for (int k = 1; k < K; ++k) {
            const int n = nb[(int64_t)k * Nf];
            take_up(value(n), n, bv, bn);
        }
        out[i] = bv;
        argmax[i] = bn;
    }
}

// Backward as a gather over the in-edge lists of the larger layer (sorted, repeats adjacent):
//   grad_small[j][c] = sum over centres l that list m = sel[j] of (argmax[l][c] == m ? grad_out[l][c] : 0)
__global__ __launch_bounds__(256) void upsample_bwd_bnc4_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src, float *__restrict__ grad_small,
    int64_t BNs, int Ns, int Nf, int C4, int PT, int64_t total_tiles)
{
    constexpr int U = 4;
    const int64_t tile = xcd_tile_up(total_tiles);
    if (tile < 0) return;
    for (int i = threadIdx.x; i < PT * C4; i += 256) {
        const int c4 = i % C4;
        const int64_t gj = tile * PT + i / C4;
        if (gj >= BNs) break;
        const int64_t b = gj / Ns;
        const int m = sel[gj];
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        if (m >= 0 && m < Nf) {
            const v4f *g4 = reinterpret_cast<const v4f *>(grad_out) + b * Nf * C4 + c4;
            const int4 *a4 = reinterpret_cast<const int4 *>(argmax) + b * Nf * C4 + c4;
            const int64_t gp = b * Nf + m;
            const int e0 = in_off[gp], e1 = in_off[gp + 1];
            int prev = -1;
            for (int e = e0; e < e1; e += U) {
                int l[U];
                int4 a[U];
                v4f g[U];
#pragma unroll
                for (int u = 0; u < U; ++u) l[u] = in_src[min(e + u, e1 - 1)];     // past the end: the last entry again
#pragma unroll
                for (int u = 0; u < U; ++u) { a[u] = a4[(int64_t)l[u] * C4]; g[u] = g4[(int64_t)l[u] * C4]; }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool fresh = l[u] != prev;   // a centre that lists m twice routes one gradient
                    prev = l[u];
                    acc.x += (fresh && a[u].x == m) ? g[u].x : 0.f;
                    acc.y += (fresh && a[u].y == m) ? g[u].y : 0.f;
                    acc.z += (fresh && a[u].z == m) ? g[u].z : 0.f;
                    acc.w += (fresh && a[u].w == m) ? g[u].w : 0.f;
                }
            }
        }
        reinterpret_cast<v4f *>(grad_small)[gj * C4 + c4] = acc;
    }
}

__global__ __launch_bounds__(256) void upsample_bwd_generic_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src, float *__restrict__ grad_small,
    int B, int Ns, int Nf, int C, int bnc)
{
    const int64_t total = (int64_t)B * Ns * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int64_t b; int c, j;
        if (bnc) { c = (int)(i % C); const int64_t gj = i / C; b = gj / Ns; j = (int)(gj % Ns); }
        else     { j = (int)(i % Ns); const int64_t bc = i / Ns; b = bc / C; c = (int)(bc % C); }
        const int m = sel[b * Ns + j];
        float acc = 0.f;
        if (m >= 0 && m < Nf) {
            const int64_t gp = b * Nf + m;
            const int e1 = in_off[gp + 1];
            int prev = -1;
            for (int e = in_off[gp]; e < e1; ++e) {
                const int64_t l = in_src[e];
                if ((int)l == prev) continue;
                prev = (int)l;
                const int64_t at = bnc ? (b * Nf + l) * C + c : (b * C + c) * Nf + l;
                if (argmax[at] == m) acc += grad_out[at];
            }
        }
        grad_small[i] = acc;
    }
}

// number of sel entries outside [0,Nf) plus the number that repeat an earlier entry of their cloud
// (inv must hold the map built from the same sel)
__global__ __launch_bounds__(256) void upsample_check_sel_kernel(const int32_t *__restrict__ sel,
                                                                 const int32_t *__restrict__ inv, int B, int Ns,
                                                                 int Nf, int32_t *__restrict__ bad)
{
    const int64_t total = (int64_t)B * Ns;
    int mine = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = i / Ns;
        const int m = sel[i];
        if (m < 0 || m >= Nf) ++mine;
        else if (inv[b * Nf + m] != (int)(i - b * Ns)) ++mine;   // another entry of the cloud claimed m
    }
    if (mine) atomicAdd(bad, mine);
}

static unsigned capped_blocks(int64_t items, int64_t cap)
{
    int64_t blocks = (items + 255) / 256;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

hipError_t launch_upsample_inv(const int32_t *sel, int32_t *inv, int B, int Ns, int Nf, hipStream_t s)
{
    hipLaunchKernelGGL(upsample_inv_fill_kernel, dim3(capped_blocks((int64_t)B * Nf, 8192)), dim3(256), 0, s, inv,
                       (int64_t)B * Nf);
    hipLaunchKernelGGL(upsample_inv_scatter_kernel, dim3(capped_blocks((int64_t)B * Ns, 8192)), dim3(256), 0, s, sel,
                       inv, B, Ns, Nf);
    return hipGetLastError();
}

hipError_t launch_upsample_fwd(const float *feat_small, const int32_t *inv, const int32_t *nbr, float *out,
                               int32_t *argmax, int B, int Ns, int Nf, int K, int C, int bnc, hipStream_t s)
{
    if (bnc && (C % 4 == 0)) {
        const int C4 = C / 4;
        const int PT = C4 >= 256 ? 1 : 256 / C4;
        const int64_t BN = (int64_t)B * Nf, tiles = (BN + PT - 1) / PT;
        hipLaunchKernelGGL(upsample_fwd_bnc4_kernel, dim3(xcd_grid_up(tiles)), dim3(256), 0, s, feat_small, inv, nbr,
                           out, argmax, BN, Ns, Nf, K, C4, PT, tiles);
    } else {
        hipLaunchKernelGGL(upsample_fwd_generic_kernel, dim3(capped_blocks((int64_t)B * Nf * C, 1 << 20)), dim3(256),
                           0, s, feat_small, inv, nbr, out, argmax, B, Ns, Nf, K, C, bnc);
    }
    return hipGetLastError();
}

hipError_t launch_upsample_bwd(const float *grad_out, const int32_t *argmax, const int32_t *sel,
                               const int32_t *in_off, const int32_t *in_src, float *grad_small, int B, int Ns,
                               int Nf, int C, int bnc, hipStream_t s)
{
    if (bnc && (C % 4 == 0)) {
        const int C4 = C / 4;
        const int PT = C4 >= 256 ? 1 : 256 / C4;
        const int64_t BNs = (int64_t)B * Ns, tiles = (BNs + PT - 1) / PT;
        hipLaunchKernelGGL(upsample_bwd_bnc4_kernel, dim3(xcd_grid_up(tiles)), dim3(256), 0, s, grad_out, argmax, sel,
                           in_off, in_src, grad_small, BNs, Ns, Nf, C4, PT, tiles);
    } else {
        hipLaunchKernelGGL(upsample_bwd_generic_kernel, dim3(capped_blocks((int64_t)B * Ns * C, 1 << 20)), dim3(256),
                           0, s, grad_out, argmax, sel, in_off, in_src, grad_small, B, Ns, Nf, C, bnc);
    }
    return hipGetLastError();
}

hipError_t launch_upsample_check_sel(const int32_t *sel, const int32_t *inv, int B, int Ns, int Nf, int32_t *bad,
                                     hipStream_t s)
{
    hipError_t e = launch_fill_zero(bad, sizeof(int32_t), s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(upsample_check_sel_kernel, dim3(capped_blocks((int64_t)B * Ns, 4096)), dim3(256), 0, s, sel,
                       inv, B, Ns, Nf, bad);
    return hipGetLastError();
}

}  // namespace flex
