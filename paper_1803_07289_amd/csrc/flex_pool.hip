// Flex-max-pooling (Sec. 4.1): per-neighbourhood maximum with the winning
// point's index recorded for the backward pass.  Bandwidth-bound: the forward
// pass gathers whole point-major rows (16 bytes per lane); the backward pass
// has three forms: a scatter by the recorded index with fp32 atomic adds (no
// lists needed), a gather over the transposed neighbour lists (no atomics,
// fixed order), and that gather through a static per-tile plan that fetches
// every listing row once per 32 points.
#include "flex_common.hpp"
#include <type_traits>

namespace flex {

typedef int i4v __attribute__((ext_vector_type(4)));

// (value desc, point index asc): the winner among equal values is the lowest index.
__device__ __forceinline__ void take(float v, int n, float &bv, int &bn)
{
    if (v > bv || (v == bv && n < bn)) { bv = v; bn = n; }
}

// Element at a 32-bit byte offset from a wave-uniform row pointer (scalar base + vector offset addressing);
// rows of the channel-major kernels are shorter than 4 GiB (checked by their launchers).
template <class T>
__device__ __forceinline__ T at_byte(const T *row, unsigned byte_off)
{
    return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(row) + byte_off);
}

// Blocks are dealt to the 8 XCDs round-robin by block id; giving each XCD one
// contiguous eighth of the point tiles keeps a neighbourhood's rows in one L2.
__device__ __forceinline__ int64_t xcd_tile(int64_t total_tiles)
{
    const int64_t per_xcd = (total_tiles + 7) >> 3;
    const int64_t slot = blockIdx.x >> 3;
    const int64_t tile = (int64_t)(blockIdx.x & 7) * per_xcd + slot;
    return (slot < per_xcd && tile < total_tiles) ? tile : -1;
}
static inline unsigned xcd_grid(int64_t total_tiles) { return (unsigned)(((total_tiles + 7) >> 3) << 3); }

// Point-major, C % 4 == 0: one thread per (point, 4 channels); a block owns PT consecutive points.
// The gather is latency-bound, so a thread first requests the ids of 8 neighbours, then their 8
// rows (16 bytes each), and only then compares: 8 rows per lane are in flight instead of one.
// SUB: pooling with subsampling, only the kept centres sel[b,j] are evaluated (BN = B*Ns output rows).
template <bool SUB>
__device__ __forceinline__ void pool_fwd_bnc4_tile(const float *__restrict__ feat, const int32_t *__restrict__ nbr,
                                                   const int32_t *__restrict__ sel, float *__restrict__ out,
                                                   int32_t *__restrict__ argmax, int64_t BN, int N, int Ns, int K,
                                                   int C4, int PT, int64_t tile)
{
    constexpr int U = 8;
    for (int i = threadIdx.x; i < PT * C4; i += 256) {
        const int c4 = i % C4;
        const int64_t gp = tile * PT + i / C4;
        if (gp >= BN) break;
        int b, l;
        if constexpr (SUB) { b = (int)(gp / Ns); l = min(max(sel[gp], 0), N - 1); }
        else { b = (int)(gp / N); l = (int)(gp % N); }
        const int32_t *nb = nbr + (int64_t)b * K * N + l;
        const v4f *rows = reinterpret_cast<const v4f *>(feat) + (int64_t)b * N * C4 + c4;
        float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
        int b0 = 0, b1 = 0, b2 = 0, b3 = 0;
        // slots k0 .. k0+W-1: ids, then rows, then the comparisons
#define FLEX_POOL_SLOTS(W)                                                                                 \
        {                                                                                                  \
            int n[W];                                                                                      \
            v4f v[W];                                                                                      \
            _Pragma("unroll") for (int u = 0; u < W; ++u)                                                  \
                n[u] = nb[(int64_t)min(k0 + u, K - 1) * N]; /* past K: the last slot again */              \
            _Pragma("unroll") for (int u = 0; u < W; ++u) v[u] = rows[(int64_t)n[u] * C4];                 \
            if (k0 == 0) {                                                                                 \
                v0 = v[0].x; v1 = v[0].y; v2 = v[0].z; v3 = v[0].w;                                        \
                b0 = b1 = b2 = b3 = n[0];                                                                  \
            }                                                                                              \
            _Pragma("unroll") for (int u = 0; u < W; ++u) { /* a repeated pair never changes the winner */ \
                take(v[u].x, n[u], v0, b0);                                                                \
                take(v[u].y, n[u], v1, b1);                                                                \
                take(v[u].z, n[u], v2, b2);                                                                \
                take(v[u].w, n[u], v3, b3);                                                                \
            }                                                                                              \
        }
        int k0 = 0;
        for (; k0 + 4 < K; k0 += U) FLEX_POOL_SLOTS(U)
        if (k0 < K) FLEX_POOL_SLOTS(4)      // a tail of up to four slots
#undef FLEX_POOL_SLOTS
        const v4f bv = {v0, v1, v2, v3};
        // streaming stores: the outputs are not read again by this kernel and should not displace gathered rows in L2
        __builtin_nontemporal_store(bv, &reinterpret_cast<v4f *>(out)[gp * C4 + c4]);
        const i4v bi = {b0, b1, b2, b3};
        __builtin_nontemporal_store(bi, &reinterpret_cast<i4v *>(argmax)[gp * C4 + c4]);
    }
}

template <bool SUB>
__global__ __launch_bounds__(256) void pool_fwd_bnc4_kernel(const float *__restrict__ feat,
                                                            const int32_t *__restrict__ nbr,
                                                            const int32_t *__restrict__ sel,
                                                            float *__restrict__ out,
                                                            int32_t *__restrict__ argmax, int64_t BN,
                                                            int N, int Ns, int K, int C4, int PT,
                                                            int64_t total_tiles)
{
    const int64_t tile = xcd_tile(total_tiles);
    if (tile < 0) return;
    pool_fwd_bnc4_tile<SUB>(feat, nbr, sel, out, argmax, BN, N, Ns, K, C4, PT, tile);
}

// value of lane SRC of the caller's 16-lane row (all 16 lanes must be active)
template <int SRC>
__device__ __forceinline__ int row_bcast(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, 0x150 + SRC, 0xf, 0xf, true);   // row_newbcast:SRC
}

// Channel-major ([B,C,N]) forward.  A block owns 64 consecutive centres of one cloud: lane = centre, so
// the ids, the outputs and the winner table move as whole 256-byte rows, and the four waves split the
// channels in chunks of CH.  A thread requests CH x 8 values (4 bytes each, from CH channel rows) before
// it compares; the ids of the first eight slots are read once for all channels.
// sel == nullptr: every point is a centre (L = N); else the centres are sel[b, 0..L).
template <int CH>
__global__ __launch_bounds__(256) void pool_fwd_bcn_kernel(const float *__restrict__ feat,
                                                           const int32_t *__restrict__ nbr,
                                                           const int32_t *__restrict__ sel,
                                                           float *__restrict__ out,
                                                           int32_t *__restrict__ argmax, int N, int L,
                                                           int K, int C, int tiles_per_cloud,
                                                           int64_t total_tiles)
{
    constexpr int U = 8;
    const int64_t tile = xcd_tile(total_tiles);
    if (tile < 0) return;
    const int64_t b = tile / tiles_per_cloud;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: channel rows get scalar base addresses
    const int j = (int)(tile - b * tiles_per_cloud) * 64 + lane;
    const bool on = j < L;
    const int jc = min(j, L - 1);
    const int l = sel ? min(max(sel[b * L + jc], 0), N - 1) : jc;
    const int32_t *nb = nbr + b * K * N + l;
    int n0[U];
#pragma unroll
    for (int u = 0; u < U; ++u) n0[u] = nb[(int64_t)min(u, K - 1) * N];      // past K: the last slot again
    for (int c0 = w * CH; c0 < C; c0 += 4 * CH) {
        const float *row[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) row[ch] = feat + (b * C + min(c0 + ch, C - 1)) * N;
        float bv[CH];
        int bn[CH];
        {
            float v[CH][U];
#pragma unroll
            for (int ch = 0; ch < CH; ++ch)
#pragma unroll
                for (int u = 0; u < U; ++u) v[ch][u] = at_byte(row[ch], 4u * (unsigned)n0[u]);
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) {
                bv[ch] = v[ch][0];
                bn[ch] = n0[0];
#pragma unroll
                for (int u = 1; u < U; ++u) take(v[ch][u], n0[u], bv[ch], bn[ch]);   // a repeated pair never changes the winner
            }
        }
        for (int k0 = U; k0 < K; k0 += U) {
            int n[U];
            float v[CH][U];
#pragma unroll
            for (int u = 0; u < U; ++u) n[u] = nb[(int64_t)min(k0 + u, K - 1) * N];
#pragma unroll
            for (int ch = 0; ch < CH; ++ch)
#pragma unroll
                for (int u = 0; u < U; ++u) v[ch][u] = at_byte(row[ch], 4u * (unsigned)n[u]);
#pragma unroll
            for (int ch = 0; ch < CH; ++ch)
#pragma unroll
                for (int u = 0; u < U; ++u) take(v[ch][u], n[u], bv[ch], bn[ch]);
        }
#pragma unroll
        for (int ch = 0; ch < CH; ++ch)
            if (on && c0 + ch < C) {
                const int64_t at = (b * C + c0 + ch) * L + j;
                __builtin_nontemporal_store(bv[ch], &out[at]);
                __builtin_nontemporal_store(bn[ch], &argmax[at]);
            }
    }
}

// sel == nullptr: every point is a centre (L = N); else the centres are sel[b, 0..L).
__global__ __launch_bounds__(256) void pool_fwd_generic_kernel(const float *__restrict__ feat,
                                                               const int32_t *__restrict__ nbr,
                                                               const int32_t *__restrict__ sel,
                                                               float *__restrict__ out,
                                                               int32_t *__restrict__ argmax, int B,
                                                               int N, int L, int K, int C, int bnc)
{
    const int64_t total = (int64_t)B * L * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int b, c, l;
        if (bnc) { c = (int)(i % C); const int64_t gp = i / C; b = (int)(gp / L); l = (int)(gp % L); }
        else     { l = (int)(i % L); const int64_t bc = i / L; b = (int)(bc / C); c = (int)(bc % C); }
        if (sel) l = min(max(sel[(int64_t)b * L + l], 0), N - 1);
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
        const int C4 = C / 4;
        const int PT = C4 >= 256 ? 1 : 256 / C4;
        const int64_t BN = (int64_t)B * N, tiles = (BN + PT - 1) / PT;
        hipLaunchKernelGGL(pool_fwd_bnc4_kernel<false>, dim3(xcd_grid(tiles)), dim3(256), 0, s, feat, nbr,
                           (const int32_t *)nullptr, out, argmax, BN, N, N, K, C4, PT, tiles);
    } else if (!bnc && N < (1 << 30)) {
        const int tpc = (N + 63) / 64;
        const int64_t tiles = (int64_t)B * tpc;
        hipLaunchKernelGGL(pool_fwd_bcn_kernel<4>, dim3(xcd_grid(tiles)), dim3(256), 0, s, feat, nbr,
                           (const int32_t *)nullptr, out, argmax, N, N, K, C, tpc, tiles);
    } else {
        const int64_t total = (int64_t)B * N * C;
        int64_t blocks = (total + 255) / 256;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(pool_fwd_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, feat, nbr,
                           (const int32_t *)nullptr, out, argmax, B, N, N, K, C, bnc);
    }
    return hipGetLastError();
}

// Pooling with subsampling: out / argmax hold the Ns kept centres sel[b,j] only.
hipError_t launch_pool_sub_fwd(const float *feat, const int32_t *nbr, const int32_t *sel, float *out,
                               int32_t *argmax, int B, int N, int Ns, int K, int C, int bnc, hipStream_t s)
{
    if (bnc && (C % 4 == 0)) {
        const int C4 = C / 4;
        const int PT = C4 >= 256 ? 1 : 256 / C4;
        const int64_t BNs = (int64_t)B * Ns, tiles = (BNs + PT - 1) / PT;
        hipLaunchKernelGGL(pool_fwd_bnc4_kernel<true>, dim3(xcd_grid(tiles)), dim3(256), 0, s, feat, nbr, sel,
                           out, argmax, BNs, N, Ns, K, C4, PT, tiles);
    } else if (!bnc && N < (1 << 30)) {
        const int tpc = (Ns + 63) / 64;
        const int64_t tiles = (int64_t)B * tpc;
        hipLaunchKernelGGL(pool_fwd_bcn_kernel<4>, dim3(xcd_grid(tiles)), dim3(256), 0, s, feat, nbr, sel, out,
                           argmax, N, Ns, K, C, tpc, tiles);
    } else {
        const int64_t total = (int64_t)B * Ns * C;
        int64_t blocks = (total + 255) / 256;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(pool_fwd_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, feat, nbr, sel,
                           out, argmax, B, N, Ns, K, C, bnc);
    }
    return hipGetLastError();
}

// grad_out / argmax have L rows per cloud (L = N, or the kept centres of a subsampled pooling),
// grad_feat has N.
__global__ __launch_bounds__(256) void pool_bwd_kernel(const float *__restrict__ grad_out,
                                                       const int32_t *__restrict__ argmax,
                                                       float *__restrict__ grad_feat, int B, int N, int L,
                                                       int C, int bnc)
{
    const int64_t total = (int64_t)B * L * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int m = argmax[i];
        int64_t dst;
        if (bnc) { const int c = (int)(i % C); const int64_t gp = i / C; const int64_t b = gp / L;
                   dst = (b * N + m) * C + c; }
        else     { const int64_t bc = i / L; dst = bc * N + m; }
        atomicAdd(&grad_feat[dst], grad_out[i]);
    }
}

// Gather form of the backward pass over in-edge lists (sorted, so repeats are adjacent; no
// atomics, fixed summation order):
// grad_feat[m][c] = sum over centres l that list m of (argmax[l][c] == m ? grad_out[l][c] : 0).
// Entries are taken four at a time: their ids first, then the eight rows (winner table and
// gradient), so that a lane has 128 bytes in flight instead of 32 (eight at a time is slower:
// the mean in-degree is K, so most of a second batch would be padding).
template <int U>
__global__ __launch_bounds__(256) void pool_bwd_gather_bnc4_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src,
    float *__restrict__ grad_feat, int64_t BN, int N, int L, int C4, int PT, int64_t total_tiles)
{
    // L = rows of grad_out / argmax per cloud: N, or the kept centres of a subsampled pooling (the lists
    // then hold row numbers among the kept centres).  U = entries per batch: about half the mean list length.
    const int64_t tile = xcd_tile(total_tiles);
    if (tile < 0) return;
    for (int i = threadIdx.x; i < PT * C4; i += 256) {
        const int c4 = i % C4;
        const int64_t gp = tile * PT + i / C4;
        if (gp >= BN) break;
        const int64_t b = gp / N;
        const int m = (int)(gp - b * N);
        const v4f *g4 = reinterpret_cast<const v4f *>(grad_out) + b * L * C4 + c4;
        const int4 *a4 = reinterpret_cast<const int4 *>(argmax) + b * L * C4 + c4;
        v4f acc = {0.f, 0.f, 0.f, 0.f};
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
                // a centre that lists m twice (adjacent entries, also the repeats past the end) routes one gradient
                const bool fresh = l[u] != prev;
                prev = l[u];
                acc.x += (fresh && a[u].x == m) ? g[u].x : 0.f;
                acc.y += (fresh && a[u].y == m) ? g[u].y : 0.f;
                acc.z += (fresh && a[u].z == m) ? g[u].z : 0.f;
                acc.w += (fresh && a[u].w == m) ? g[u].w : 0.f;
            }
        }
        __builtin_nontemporal_store(acc, &reinterpret_cast<v4f *>(grad_feat)[gp * C4 + c4]);
    }
}

// Gather form for C % 64 == 0 (a point's lanes fill whole 16-lane rows).  In the kernel above all 16
// lanes of a point load the same list entries; every memory instruction costs the texture path the same
// however few distinct bytes it fetches, and the backward pass issues many.  Here lane t of a row loads
// list entry t, one instruction for up to 16 entries, and DPP row broadcasts on the vector ALU hand them
// round (the same change does nothing for the forward pass, which is bound by HBM, not by instructions).
// U = entries whose rows are requested together.
template <int U>
__device__ __forceinline__ void pool_bwd_gather_row16_tile(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src,
    float *__restrict__ grad_feat, int64_t BN, int N, int L, int C4, int PT, int64_t tile)
{
    static_assert(U == 2 || U == 4, "batches tile the 16 entries of one load");
    const int t16 = threadIdx.x & 15;
    for (int i = threadIdx.x; i < PT * C4; i += 256) {
        const int c4 = i % C4;
        const int64_t gp = tile * PT + i / C4;
        if (gp >= BN) break;
        const int64_t b = gp / N;
        const int m = (int)(gp - b * N);
        const v4f *g4 = reinterpret_cast<const v4f *>(grad_out) + b * L * C4 + c4;
        const int4 *a4 = reinterpret_cast<const int4 *>(argmax) + b * L * C4 + c4;
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        const int bound = in_off[gp + (t16 & 1)];
        const int e0 = row_bcast<0>(bound), e1 = row_bcast<1>(bound);
        int prev = -1;
        for (int e = e0; e < e1; e += 16) {
            const int mine = in_src[min(e + t16, e1 - 1)];               // past the end: the last entry again
            auto batch = [&](const int (&l)[U]) {
                int4 a[U];
                v4f g[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { a[u] = a4[(int64_t)l[u] * C4]; g[u] = g4[(int64_t)l[u] * C4]; }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    // a centre that lists m twice (adjacent entries, also the repeats past the end) routes one gradient
                    const bool fresh = l[u] != prev;
                    prev = l[u];
                    acc.x += (fresh && a[u].x == m) ? g[u].x : 0.f;
                    acc.y += (fresh && a[u].y == m) ? g[u].y : 0.f;
                    acc.z += (fresh && a[u].z == m) ? g[u].z : 0.f;
                    acc.w += (fresh && a[u].w == m) ? g[u].w : 0.f;
                }
            };
#define FLEX_POOL_BATCH(J)                                                                               \
            if (e + (J) * U < e1) {                                                                          \
                if constexpr (U == 4) {                                                                      \
                    const int l[U] = {row_bcast<((J) * U) & 15>(mine), row_bcast<((J) * U + 1) & 15>(mine),   \
                                      row_bcast<((J) * U + 2) & 15>(mine), row_bcast<((J) * U + 3) & 15>(mine)}; \
                    batch(l);                                                                                \
                } else {                                                                                     \
                    const int l[U] = {row_bcast<((J) * U) & 15>(mine), row_bcast<((J) * U + 1) & 15>(mine)};   \
                    batch(l);                                                                                \
                }                                                                                            \
            }
            FLEX_POOL_BATCH(0) FLEX_POOL_BATCH(1) FLEX_POOL_BATCH(2) FLEX_POOL_BATCH(3)
            if constexpr (U == 2) { FLEX_POOL_BATCH(4) FLEX_POOL_BATCH(5) FLEX_POOL_BATCH(6) FLEX_POOL_BATCH(7) }
#undef FLEX_POOL_BATCH
        }
        __builtin_nontemporal_store(acc, &reinterpret_cast<v4f *>(grad_feat)[gp * C4 + c4]);
    }
}

template <int U>
__global__ __launch_bounds__(256) void pool_bwd_gather_row16_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src,
    float *__restrict__ grad_feat, int64_t BN, int N, int L, int C4, int PT, int64_t total_tiles)
{
    const int64_t tile = xcd_tile(total_tiles);
    if (tile < 0) return;
    pool_bwd_gather_row16_tile<U>(grad_out, argmax, in_off, in_src, grad_feat, BN, N, L, C4, PT, tile);
}

// ---- gather form with a static plan (point-major, 64-channel blocks of the rows) ---------------------------------------------------
// Neighbouring points are listed by mostly the same centres: the 32 consecutive points of a tile have about 256
// list entries but only about 94 distinct source rows, and the kernels above ask the texture path for a row's
// 512 bytes (winner table + gradient) once per entry.  The neighbourhoods are static (Sec. 4.1), so which rows a
// tile needs and where each list entry finds its row can be written down once per cloud: the plan.
//   hdr  int32 [1] (+ padding)   the number of tiles the plan does not cover in full (the two kinds below).  Where
//                                 they are more than an eighth of all tiles (a cloud whose point order has no
//                                 locality: every tile of 32 points is listed by some 250 distinct centres) the
//                                 planned kernel returns at once and the list form runs in its place
//   cnt  int32 [tiles]            distinct source rows of the tile that are listed (at most RMAX - 1), + PLAN_HAS_DIRECT
//                                 if some entry's row is not among them; or -1: a tile with more than EMAX list
//                                 entries, which the kernel serves entry by entry
//   rows int32 [tiles][RMAX]      those rows (unused places: row 0)
//   slot uint16 [entries]         per list entry (the order of in_src): the place of its row in the tile's list;
//                                 PLAN_NULL if the entry repeats the one before it in the same list (it routes
//                                 nothing: the kernel keeps a row that matches no point at that place);
//                                 PLAN_DIRECT if its row is not listed (fetch it by in_src)
//   ctr  int32 [8][64]           scratch of the list-form kernel that runs where the plan does not pay: the next
//                                 tile of each XCD's share, one counter per 256-byte block (cleared at every call)
// A row listed twice (two entries of one tile that lost each other in the hash table) costs bandwidth only.
constexpr int PLAN_T = 32, PLAN_RMAX = 128, PLAN_EMAX = 512, PLAN_HASH = 2048;
constexpr unsigned PLAN_NULL = PLAN_RMAX - 1, PLAN_DIRECT = 0x7fffu;
constexpr int PLAN_HAS_DIRECT = 1 << 30;
constexpr int PLAN_CTR_STRIDE = 64;     // ints between the XCDs' counters: a 256-byte block each
// the plan pays where most tiles are covered in full
__device__ __forceinline__ bool pool_plan_pays(const int32_t *plan_hdr, int total_tiles)
{
    return (int64_t)plan_hdr[0] * 8 <= total_tiles;
}

struct PoolPlanLayout {
    size_t hdr_off, cnt_off, rows_off, slot_off, ctr_off, bytes;
    int tiles_per_cloud;
    int64_t tiles;
};
static PoolPlanLayout pool_plan_layout(int B, int N, int K)
{
    PoolPlanLayout l;
    l.tiles_per_cloud = (N + PLAN_T - 1) / PLAN_T;
    l.tiles = (int64_t)B * l.tiles_per_cloud;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    l.hdr_off = 0;
    l.cnt_off = 256;
    l.rows_off = l.cnt_off + up(sizeof(int32_t) * (size_t)l.tiles);
    l.slot_off = l.rows_off + up(sizeof(int32_t) * (size_t)l.tiles * PLAN_RMAX);
    l.ctr_off = l.slot_off + up(sizeof(unsigned short) * (size_t)B * K * N);
    l.bytes = l.ctr_off + 8 * PLAN_CTR_STRIDE * sizeof(int32_t);   // tile counters of the list-form kernel, one per XCD
    return l;
}
size_t pool_plan_bytes(int B, int N, int K) { return pool_plan_layout(B, N, K).bytes; }

// One block per tile.  Every entry writes its own number into a table slot chosen by a hash of its row, reads back
// which entry kept the slot and follows it if that one names the same row (else it stays its own leader); the
// leaders are numbered by a prefix sum over the block.
// FWD == false: the tile's entries are the in-edge lists of its points (in_off / in_src; the pooling backward pass).
// FWD == true: they are the neighbour lists themselves, entry p * K + k = nbr[b, k, m0 + p] (in_src = nbr, in_off
// unused; the pooling forward pass): K entries per point, no repeats to mark (a maximum does not mind them).
template <bool FWD>
__global__ __launch_bounds__(256) void pool_plan_build_kernel(const int32_t *__restrict__ in_off,
                                                              const int32_t *__restrict__ in_src,
                                                              int32_t *__restrict__ plan_hdr,
                                                              int32_t *__restrict__ plan_cnt,
                                                              int32_t *__restrict__ plan_rows,
                                                              unsigned short *__restrict__ plan_slot, int N, int K,
                                                              int tiles_per_cloud)
{
    constexpr int T = PLAN_T, RMAX = PLAN_RMAX, EMAX = PLAN_EMAX, HASH = PLAN_HASH;
    __shared__ int s_off[T + 1];
    __shared__ int s_l[EMAX];
    __shared__ unsigned short s_rank[EMAX];
    __shared__ unsigned short s_tab[HASH];
    __shared__ unsigned char s_start[EMAX];
    __shared__ int s_cnt[8];
    const int64_t tile = blockIdx.x;
    const int64_t b = tile / tiles_per_cloud;
    const int m0 = (int)(tile - b * tiles_per_cloud) * T;
    const int np = min(T, N - m0);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid <= T) s_off[tid] = FWD ? min(tid, np) * K : in_off[b * N + m0 + min(tid, np)];   // past the cloud: empty lists
    s_start[tid] = 0;
    s_start[tid + 256] = 0;
    __syncthreads();
    // first entry of the tile in the plan's slot array (backward: the lists' own order; forward: point by point)
    const int64_t E0 = FWD ? (b * N + m0) * K : s_off[0];
    const int E = s_off[T] - s_off[0];
    if (E > EMAX) {
        for (int r = tid; r < RMAX; r += 256) plan_rows[tile * RMAX + r] = 0;
        if (tid == 0) {
            plan_cnt[tile] = -1;
            atomicAdd(plan_hdr, 1);
        }
        return;
    }
    if (tid < T && s_off[tid + 1] > s_off[tid]) s_start[s_off[tid] - s_off[0]] = 1;
    int l[2], lead[2], rank[2];
    unsigned h[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + 256 * r;
        if constexpr (FWD) l[r] = i < E ? in_src[(b * K + i % K) * N + m0 + i / K] : -1;
        else l[r] = i < E ? in_src[E0 + i] : -1;
        h[r] = ((unsigned)l[r] * 0x9E3779B1u) >> 21;
        if (i < E) { s_l[i] = l[r]; s_tab[h[r]] = (unsigned short)i; }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + 256 * r;
        bool leader = false;
        lead[r] = i;
        if (i < E) {
            const int j = s_tab[h[r]];
            if (s_l[j] == l[r]) lead[r] = j;
            leader = lead[r] == i;
        }
        const unsigned long long bal = __ballot(leader);
        rank[r] = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) s_cnt[r * 4 + w] = __popcll(bal);
    }
    __syncthreads();
    int R = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int c = s_cnt[q];
        if (q < w) rank[0] += c;
        if (q < 4 + w) rank[1] += c;
        R += c;
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + 256 * r;
        if (i < E && lead[r] == i) {
            s_rank[i] = (unsigned short)rank[r];
            if (rank[r] < RMAX - 1) plan_rows[tile * RMAX + rank[r]] = l[r];
        }
    }
    __syncthreads();
    bool direct = false;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + 256 * r;
        if (i < E) {
            const unsigned place = s_rank[lead[r]];
            const bool repeat = !FWD && i > 0 && !s_start[i] && s_l[i - 1] == l[r];
            const bool listed = place < (unsigned)(RMAX - 1);
            direct |= !repeat && !listed;
            plan_slot[E0 + i] = (unsigned short)(repeat ? PLAN_NULL : listed ? place : PLAN_DIRECT);
        }
    }
    const int any_direct = __syncthreads_or(direct);
    const int listed_rows = min(R, RMAX - 1);
    for (int r = listed_rows + tid; r < RMAX; r += 256) plan_rows[tile * RMAX + r] = 0;
    if (tid == 0) {
        plan_cnt[tile] = listed_rows | (any_direct ? PLAN_HAS_DIRECT : 0);
        if (any_direct) atomicAdd(plan_hdr, 1);
    }
}

hipError_t launch_pool_plan_build(const int32_t *in_off, const int32_t *in_src, void *plan, int B, int N, int K,
                                  hipStream_t s)
{
    const PoolPlanLayout l = pool_plan_layout(B, N, K);
    if (l.tiles > 0x7fffffff) return hipErrorInvalidValue;
    char *base = reinterpret_cast<char *>(plan);
    const hipError_t e = launch_fill_zero(base + l.hdr_off, 256, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(pool_plan_build_kernel<false>, dim3((unsigned)l.tiles), dim3(256), 0, s, in_off, in_src,
                       reinterpret_cast<int32_t *>(base + l.hdr_off), reinterpret_cast<int32_t *>(base + l.cnt_off),
                       reinterpret_cast<int32_t *>(base + l.rows_off),
                       reinterpret_cast<unsigned short *>(base + l.slot_off), N, K, l.tiles_per_cloud);
    return hipGetLastError();
}

// the plan of the forward pass: the same layout, over the neighbour lists themselves
hipError_t launch_pool_fwd_plan_build(const int32_t *nbr, void *plan, int B, int N, int K, hipStream_t s)
{
    const PoolPlanLayout l = pool_plan_layout(B, N, K);
    if (l.tiles > 0x7fffffff) return hipErrorInvalidValue;
    char *base = reinterpret_cast<char *>(plan);
    const hipError_t e = launch_fill_zero(base + l.hdr_off, 256, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(pool_plan_build_kernel<true>, dim3((unsigned)l.tiles), dim3(256), 0, s,
                       (const int32_t *)nullptr, nbr, reinterpret_cast<int32_t *>(base + l.hdr_off),
                       reinterpret_cast<int32_t *>(base + l.cnt_off), reinterpret_cast<int32_t *>(base + l.rows_off),
                       reinterpret_cast<unsigned short *>(base + l.slot_off), N, K, l.tiles_per_cloud);
    return hipGetLastError();
}

// The sums of one point, entry by entry from memory (tiles and entries the plan does not cover).
// One workgroup of 512 threads per (POOL_BWD_PLAN_TPW consecutive tiles, half of the block's 64 channels), dispatched
// in order (block index -> XCD share, position in it, channel half), four workgroups per CU (58 registers, 32 KB of
// LDS).  A staged half row is 8 x 16 bytes of the winner table and 8 x 16 bytes of the gradient, kept as they are in
// memory, in two planes; place PLAN_NULL holds a row that no point wins (index -1).  A workgroup asks for list
// bounds and plan, then for the rows of both its tiles (the second tile's wait in registers while the first is summed);
// 8 lanes stage a row half, 16 lanes own a point (2 channels each).  The sums run in list order with the same
// operations as the kernels above: bit-identical results.
typedef int i2v __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
constexpr int POOL_BWD_PLAN_TPW = 2;
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(8, 8))) void pool_bwd_planned64_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax, const int32_t *__restrict__ in_off,
    const int32_t *__restrict__ in_src, const int32_t *__restrict__ plan_hdr, const int32_t *__restrict__ plan_cnt,
    const int32_t *__restrict__ plan_rows, const unsigned short *__restrict__ plan_slot,
    float *__restrict__ grad_feat, int N, int L, int tiles_per_cloud, int total_tiles, int rc, int chunk0)
{
    constexpr int T = PLAN_T, RMAX = PLAN_RMAX, TRIPS = RMAX / 64, U = POOL_BWD_PLAN_TPW;
    __shared__ i4v s_a[RMAX * 8];       // staged half rows of the winner table: 8 x 16 bytes each
    __shared__ i4v s_g[RMAX * 8];       // ... and of the gradient
    const int tid = threadIdx.x, c8 = tid & 7, pr = tid >> 3;        // staging: 64 row groups of 8 lanes
    const int c2 = tid & 15, t16 = tid & 15, p = tid >> 4;           // sums: 16 lanes (2 channels each) per point
    const int per_xcd = (total_tiles + 7) >> 3;
    const int xbeg = (int)(blockIdx.x & 7) * per_xcd;
    const int xcount = min(per_xcd, total_tiles - xbeg);
    const int wgx = (int)(blockIdx.x >> 3);
    const int half = wgx & 1;
    const int j0 = (wgx >> 1) * U;
    if (j0 >= xcount) return;
    if (!pool_plan_pays(plan_hdr, total_tiles)) return;      // (the same in every thread) the list form runs instead
    if (tid < 8) s_a[PLAN_NULL * 8 + tid] = i4v{-1, -1, -1, -1};
    else if (tid < 16) s_g[PLAN_NULL * 8 + tid - 8] = i4v{0, 0, 0, 0};
    const int ch0 = chunk0 + 8 * half;                       // first 16-byte chunk of this pass's 32 channels
    int tb[U], tm0[U], cnt[U], e0[U], en[U], rid[U][TRIPS];
    unsigned sw[U];
    i4v a[U][TRIPS], g[U][TRIPS];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int tile = xbeg + min(j0 + u, xcount - 1);
        tb[u] = tile / tiles_per_cloud;
        tm0[u] = (tile - tb[u] * tiles_per_cloud) * T;
        const int np = min(T, N - tm0[u]);
        const int32_t *o = in_off + ((int64_t)tb[u] * N + tm0[u]);
        const int lo = o[min(p, np)], hi = o[min(p + 1, np)];
        e0[u] = lo;
        en[u] = hi - lo;
        cnt[u] = plan_cnt[tile];
        const int32_t *rows = plan_rows + (int64_t)tile * RMAX + pr;
#pragma unroll
        for (int q = 0; q < TRIPS; ++q) rid[u][q] = rows[q * 64];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        sw[u] = t16 < en[u] ? plan_slot[(size_t)e0[u] + t16] : PLAN_NULL;      // lanes past the list: the row that matches nothing
        const i4v *gb = reinterpret_cast<const i4v *>(grad_out) + (int64_t)tb[u] * L * rc + ch0 + c8;
        const i4v *ab = reinterpret_cast<const i4v *>(argmax) + (int64_t)tb[u] * L * rc + ch0 + c8;
        const int rows0 = cnt[u] < 0 ? 0 : (cnt[u] & (PLAN_HAS_DIRECT - 1));
#pragma unroll
        for (int q = 0; q < TRIPS; ++q)
            if (q * 64 + pr < rows0) {
                a[u][q] = ab[(int64_t)rid[u][q] * rc];
                g[u][q] = gb[(int64_t)rid[u][q] * rc];
            }
    }
    const int lane_base = c2 * 8;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (j0 + u >= xcount) break;                 // (the same in every thread)
        if (u > 0) __syncthreads();                  // every sum of the tile before is done with its rows
        const int rows0 = cnt[u] < 0 ? 0 : (cnt[u] & (PLAN_HAS_DIRECT - 1));
#pragma unroll
        for (int q = 0; q < TRIPS; ++q) {
            const int r = q * 64 + pr;
            if (r < rows0) {
                s_a[r * 8 + c8] = a[u][q];
                s_g[r * 8 + c8] = g[u][q];
            }
        }
        __syncthreads();
        const int b = tb[u], m0 = tm0[u], np = min(T, N - m0), n_e = en[u], cn = cnt[u];
        const size_t eb = (size_t)e0[u];
        const unsigned swu = sw[u];
        if (p < np) {
            v2f acc = {0.f, 0.f};
            const int m = m0 + p;
            const char *sa = reinterpret_cast<const char *>(s_a) + lane_base;
            const char *sg = reinterpret_cast<const char *>(s_g) + lane_base;
            auto take_staged = [&](unsigned place) __attribute__((always_inline)) {
                const i2v aa = *reinterpret_cast<const i2v *>(sa + place * 128u);
                const v2f gg = *reinterpret_cast<const v2f *>(sg + place * 128u);
                acc.x += aa.x == m ? gg.x : 0.f;
                acc.y += aa.y == m ? gg.y : 0.f;
            };
            if (cn >= 0 && !(cn & PLAN_HAS_DIRECT)) {
#define FLEX_PLAN_BATCH(J)                                                                                      \
                if ((J) < n_e) {                                                                                    \
                    const unsigned w0 = (unsigned)row_bcast<(J)>((int)swu), w1 = (unsigned)row_bcast<(J) + 1>((int)swu),  \
                                   w2 = (unsigned)row_bcast<(J) + 2>((int)swu), w3 = (unsigned)row_bcast<(J) + 3>((int)swu); \
                    const i2v a0 = *reinterpret_cast<const i2v *>(sa + w0 * 128u), a1 = *reinterpret_cast<const i2v *>(sa + w1 * 128u), \
                               a2 = *reinterpret_cast<const i2v *>(sa + w2 * 128u), a3 = *reinterpret_cast<const i2v *>(sa + w3 * 128u); \
                    const v2f g0 = *reinterpret_cast<const v2f *>(sg + w0 * 128u), g1 = *reinterpret_cast<const v2f *>(sg + w1 * 128u), \
                              g2 = *reinterpret_cast<const v2f *>(sg + w2 * 128u), g3 = *reinterpret_cast<const v2f *>(sg + w3 * 128u); \
                    acc.x += a0.x == m ? g0.x : 0.f; acc.y += a0.y == m ? g0.y : 0.f; \
                    acc.x += a1.x == m ? g1.x : 0.f; acc.y += a1.y == m ? g1.y : 0.f; \
                    acc.x += a2.x == m ? g2.x : 0.f; acc.y += a2.y == m ? g2.y : 0.f; \
                    acc.x += a3.x == m ? g3.x : 0.f; acc.y += a3.y == m ? g3.y : 0.f; \
                }
                FLEX_PLAN_BATCH(0) FLEX_PLAN_BATCH(4) FLEX_PLAN_BATCH(8) FLEX_PLAN_BATCH(12)
#undef FLEX_PLAN_BATCH
                for (int j = 16; j < n_e; ++j) take_staged(plan_slot[eb + j]);
            } else {
                const i2v *a2p = reinterpret_cast<const i2v *>(argmax) + ((int64_t)b * L * rc + ch0) * 2 + c2;
                const v2f *g2p = reinterpret_cast<const v2f *>(grad_out) + ((int64_t)b * L * rc + ch0) * 2 + c2;
                int prev = -1;
                for (int j = 0; j < n_e; ++j) {
                    const unsigned place = cn < 0 ? PLAN_DIRECT : plan_slot[eb + j];
                    if (place < (unsigned)RMAX) {
                        take_staged(place);
                    } else {
                        const int l = in_src[eb + j];
                        const i2v aa = a2p[(int64_t)l * rc * 2];
                        const v2f gg = g2p[(int64_t)l * rc * 2];
                        const bool fresh = l != prev;
                        acc.x += (fresh && aa.x == m) ? gg.x : 0.f;
                        acc.y += (fresh && aa.y == m) ? gg.y : 0.f;
                        prev = l;
                    }
                }
            }
            __builtin_nontemporal_store(acc, &reinterpret_cast<v2f *>(grad_feat)[(((int64_t)b * N + m) * rc + ch0) * 2 + c2]);
        }
    }
}

// The list form for the clouds whose plan does not pay: the same sums by the same code as flexpool_bwd's kernel, as a
// grid of resident blocks (a block that has nothing to do costs nothing to launch) which draw the tiles of their
// XCD's share in order, eight at a time, from a counter per XCD in the plan's last 2 KB.
__global__ __launch_bounds__(256) void pool_bwd_gather_row16_unplanned_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax, const int32_t *__restrict__ in_off,
    const int32_t *__restrict__ in_src, const int32_t *__restrict__ plan_hdr, int plan_tiles,
    int *__restrict__ tile_ctr, float *__restrict__ grad_feat, int64_t BN, int N, int C4, int PT, int total_tiles)
{
    constexpr int DRAW = 8;
    if (pool_plan_pays(plan_hdr, plan_tiles)) return;
    __shared__ int s_first;
    const int per_xcd = (total_tiles + 7) >> 3;
    const int xbeg = (int)(blockIdx.x & 7) * per_xcd;
    const int xcount = min(per_xcd, total_tiles - xbeg);
    int *ctr = tile_ctr + (blockIdx.x & 7) * PLAN_CTR_STRIDE + PLAN_CTR_STRIDE / 2;
    for (;;) {
        if (threadIdx.x == 0) s_first = atomicAdd(ctr, DRAW);
        __syncthreads();
        const int j0 = s_first;
        __syncthreads();                 // everyone has read the draw before the next one replaces it
        if (j0 >= xcount) return;
        for (int j = j0; j < min(j0 + DRAW, xcount); ++j)
            pool_bwd_gather_row16_tile<4>(grad_out, argmax, in_off, in_src, grad_feat, BN, N, N, C4, PT, xbeg + j);
    }
}

hipError_t launch_pool_bwd_planned(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                                   const int32_t *in_src, void *plan, float *grad_feat, int B, int N, int K, int C,
                                   hipStream_t s)
{
    // C: 64, 128 or 256 (a multiple of 64 whose row fits one block of the list form); the planned kernel serves one
    // 64-channel block of the rows per launch
    const PoolPlanLayout l = pool_plan_layout(B, N, K);
    if (l.tiles > 0x7fffffff || C % 64 != 0 || C > 256) return hipErrorInvalidValue;
    char *base = reinterpret_cast<char *>(plan);
    const int32_t *hdr = reinterpret_cast<const int32_t *>(base + l.hdr_off);
    const int64_t per_xcd = (l.tiles + 7) >> 3, wgs = 8 * 2 * ((per_xcd + POOL_BWD_PLAN_TPW - 1) / POOL_BWD_PLAN_TPW);
    if (wgs > 0x7fffffff) return hipErrorInvalidValue;
    for (int blk = 0; blk < C / 64; ++blk)
        hipLaunchKernelGGL(pool_bwd_planned64_kernel, dim3((unsigned)wgs), dim3(512), 0, s, grad_out, argmax, in_off,
                           in_src, hdr, reinterpret_cast<const int32_t *>(base + l.cnt_off),
                           reinterpret_cast<const int32_t *>(base + l.rows_off),
                           reinterpret_cast<const unsigned short *>(base + l.slot_off), grad_feat, N, N,
                           l.tiles_per_cloud, (int)l.tiles, C / 4, 16 * blk);
    {
        // the list form's tile counters (the plan's last 2 KB)
        const hipError_t e = launch_fill_zero(base + l.ctr_off, 8 * PLAN_CTR_STRIDE * sizeof(int32_t), s);
        if (e != hipSuccess) return e;
    }
    {
        const int C4 = C / 4, PT = 256 / C4;
        const int64_t BN = (int64_t)B * N, list_tiles = (BN + PT - 1) / PT;
        if (list_tiles > 0x7fffffff - 64) return hipErrorInvalidValue;
        int64_t blocks = 8 * 256;
        if (blocks > ((list_tiles + 7) & ~(int64_t)7)) blocks = (list_tiles + 7) & ~(int64_t)7;
        hipLaunchKernelGGL(pool_bwd_gather_row16_unplanned_kernel, dim3((unsigned)blocks), dim3(256), 0, s, grad_out,
                           argmax, in_off, in_src, hdr, (int)l.tiles, reinterpret_cast<int *>(base + l.ctr_off),
                           grad_feat, BN, N, C4, PT, (int)list_tiles);
    }
    return hipGetLastError();
}

// ---- forward pass through a static plan (point-major, 64-channel blocks of the rows) ---------------------------
// The same idea one pass earlier: the 32 consecutive centres of a tile list 32 K neighbours but only about 94
// distinct ones; the plan (pool_plan_build_kernel<true>) names them and gives every (centre, slot) its place.  The
// kernel stages each distinct feature row once in LDS together with its point index, and every centre takes the
// (value desc, index asc) maximum over its K places: the comparisons of pool_fwd_bnc4_kernel in the same slot order,
// so values and winners are the same bits.
// Like the backward kernel this one is not resident: one workgroup per POOL_FWD_PLAN_TPW consecutive tiles,
// dispatched in order (block index -> XCD share, position in it), four workgroups per CU (64 registers, 33 KB of
// LDS each).  The chain plan -> rows -> LDS is two memory latencies deep and a tile's comparisons are short, so what
// counts is how many tiles a CU has in flight: a workgroup asks for the plan and then the rows of both its tiles up
// front (the second tile's rows wait in registers while the first is compared) and the four workgroups of a CU
// cover each other's waits.  (A resident form with rows of two tiles ahead in registers, two workgroups per CU:
// 1.68 ms at 7M points against 1.18 ms; one tile per workgroup 1.34 ms; three tiles at three workgroups 1.27 ms;
// runs of four tile pairs per workgroup spill and take 2.1 ms.)
// A cloud whose plan does not pay (pool_plan_pays) is served by the same workgroups with the plain kernel's steps,
// a row group per centre; 7% slower there than pool_fwd_bnc4_kernel (2.39 against 2.22 ms in generator order), whose
// workgroups are half as large and end after one tile.  The kernel only reads the plan.
constexpr int POOL_FWD_PLAN_TPW = 2;
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(8, 8))) void pool_fwd_planned64_kernel(
    const float *__restrict__ feat, const int32_t *__restrict__ nbr, const int32_t *__restrict__ plan_hdr,
    const int32_t *__restrict__ plan_cnt, const int32_t *__restrict__ plan_rows,
    const unsigned short *__restrict__ plan_slot, float *__restrict__ out,
    int32_t *__restrict__ argmax, int N, int K, int tiles_per_cloud, int total_tiles, int rc, int chunk0)
{
    constexpr int T = PLAN_T, RMAX = PLAN_RMAX, TRIPS = RMAX / 32, U = POOL_FWD_PLAN_TPW;
    __shared__ v4f s_v[RMAX * 16];
    __shared__ int s_id[U][RMAX];
    const int tid = threadIdx.x, c4 = tid & 15, t16 = tid & 15, p = tid >> 4;
    const int per_xcd = (total_tiles + 7) >> 3;
    const int xbeg = (int)(blockIdx.x & 7) * per_xcd;
    const int xcount = min(per_xcd, total_tiles - xbeg);
    const int j0 = (int)(blockIdx.x >> 3) * U;
    if (j0 >= xcount) return;
    const int uncovered = plan_hdr[0];               // asked for first, looked at once the plan's loads are under way
    int tb[U], tm0[U], cnt[U], rid[U][TRIPS];
    unsigned sw[U];
    i4v v[U][TRIPS];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int tile = xbeg + min(j0 + u, xcount - 1);
        tb[u] = tile / tiles_per_cloud;
        tm0[u] = (tile - tb[u] * tiles_per_cloud) * T;
        cnt[u] = plan_cnt[tile];
        const int32_t *rows = plan_rows + (int64_t)tile * RMAX + p;
#pragma unroll
        for (int q = 0; q < TRIPS; ++q) rid[u][q] = rows[q * 32];     // (every place of the table is allocated: no wait for the count)
        const int m = min(tm0[u] + p, N - 1);
        sw[u] = plan_slot[((int64_t)tb[u] * N + m) * K + (t16 < K ? t16 : 0)];
    }
    if ((int64_t)uncovered * 8 > total_tiles) {          // pool_plan_pays()
        // (the same in every thread) a cloud whose tiles the plan does not cover: the plain kernel's steps for the
        // workgroup's centres, a row group per centre: eight ids, their eight rows, then the comparisons
        for (int u = 0; u < U && j0 + u < xcount; ++u) {
            const int tile = xbeg + j0 + u, b = tile / tiles_per_cloud, m = (tile - b * tiles_per_cloud) * T + p;
            if (m >= N) continue;
            const int32_t *nb = nbr + (int64_t)b * K * N + m;
            const v4f *frow = reinterpret_cast<const v4f *>(feat) + (int64_t)b * N * rc + chunk0 + c4;
            float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
            int b0 = 0, b1 = 0, b2 = 0, b3 = 0;
            for (int k0 = 0; k0 < K; k0 += 8) {
                int n[8];
                v4f x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) n[i] = nb[(int64_t)min(k0 + i, K - 1) * N];     // past K: the last slot again
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] = frow[(int64_t)n[i] * rc];
                if (k0 == 0) {
                    v0 = x[0].x; v1 = x[0].y; v2 = x[0].z; v3 = x[0].w;
                    b0 = b1 = b2 = b3 = n[0];
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {       // a repeated pair never changes the winner
                    take(x[i].x, n[i], v0, b0);
                    take(x[i].y, n[i], v1, b1);
                    take(x[i].z, n[i], v2, b2);
                    take(x[i].w, n[i], v3, b3);
                }
            }
            const int64_t at = ((int64_t)b * N + m) * rc + chunk0 + c4;
            __builtin_nontemporal_store(v4f{v0, v1, v2, v3}, &reinterpret_cast<v4f *>(out)[at]);
            __builtin_nontemporal_store(i4v{b0, b1, b2, b3}, &reinterpret_cast<i4v *>(argmax)[at]);
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int rows0 = cnt[u] < 0 ? 0 : (cnt[u] & (PLAN_HAS_DIRECT - 1));
        const i4v *fb = reinterpret_cast<const i4v *>(feat) + (int64_t)tb[u] * N * rc + chunk0 + c4;
#pragma unroll
        for (int q = 0; q < TRIPS; ++q)
            if (q * 32 + p < rows0) {
                v[u][q] = fb[(int64_t)rid[u][q] * rc];
                if (c4 == 0) s_id[u][q * 32 + p] = rid[u][q];
            }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (j0 + u >= xcount) break;                 // (the same in every thread)
        if (u > 0) __syncthreads();                  // every centre of the tile before is done with its rows
        const int rows0 = cnt[u] < 0 ? 0 : (cnt[u] & (PLAN_HAS_DIRECT - 1));
#pragma unroll
        for (int q = 0; q < TRIPS; ++q) {
            const int r = q * 32 + p;
            if (r < rows0) {
                s_v[r * 16 + c4] = __builtin_bit_cast(v4f, v[u][q]);
            }
        }
        __syncthreads();
        const int b = tb[u], m0 = tm0[u], np = min(T, N - m0), m = m0 + p;
        if (p < np) {
            const v4f *frow = reinterpret_cast<const v4f *>(feat) + (int64_t)b * N * rc + chunk0 + c4;
            const int32_t *nb = nbr + (int64_t)b * K * N + m;
            float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
            int b0 = 0, b1 = 0, b2 = 0, b3 = 0;
            auto sel = [](float x, int n, float &bv, int &bn) __attribute__((always_inline)) {
                const bool better = (x > bv) | ((x == bv) & (n < bn));
                bv = better ? x : bv;
                bn = better ? n : bn;
            };
            auto take_row = [&](const v4f &x, int n, bool first) __attribute__((always_inline)) {
                if (first) {
                    v0 = x.x; v1 = x.y; v2 = x.z; v3 = x.w; b0 = b1 = b2 = b3 = n;
                } else {
                    sel(x.x, n, v0, b0);
                    sel(x.y, n, v1, b1);
                    sel(x.z, n, v2, b2);
                    sel(x.w, n, v3, b3);
                }
            };
            const unsigned swu = sw[u];
            if (cnt[u] >= 0 && !(cnt[u] & PLAN_HAS_DIRECT) && K <= 16) {
#define FLEX_PLAN_FWD_BATCH(J)                                                                                  \
                if ((J) < K) {                                                                                      \
                    const unsigned w0 = (unsigned)row_bcast<(J)>((int)swu), w1 = (unsigned)row_bcast<((J) + 1) & 15>((int)swu), \
                                   w2 = (unsigned)row_bcast<((J) + 2) & 15>((int)swu), w3 = (unsigned)row_bcast<((J) + 3) & 15>((int)swu); \
                    const v4f x0 = s_v[w0 * 16 + c4], x1 = s_v[w1 * 16 + c4], x2 = s_v[w2 * 16 + c4], x3 = s_v[w3 * 16 + c4]; \
                    const int n0 = s_id[u][w0], n1 = s_id[u][w1], n2 = s_id[u][w2], n3 = s_id[u][w3];                          \
                    take_row(x0, n0, (J) == 0);                                                                     \
                    if ((J) + 1 < K) take_row(x1, n1, false);                                                       \
                    if ((J) + 2 < K) take_row(x2, n2, false);                                                       \
                    if ((J) + 3 < K) take_row(x3, n3, false);                                                       \
                }
                FLEX_PLAN_FWD_BATCH(0) FLEX_PLAN_FWD_BATCH(4) FLEX_PLAN_FWD_BATCH(8) FLEX_PLAN_FWD_BATCH(12)
#undef FLEX_PLAN_FWD_BATCH
            } else {
                for (int k = 0; k < K; ++k) {
                    const unsigned place = cnt[u] < 0 ? PLAN_DIRECT : plan_slot[((int64_t)b * N + m) * K + k];
                    if (place < (unsigned)RMAX) {
                        take_row(s_v[place * 16 + c4], s_id[u][place], k == 0);
                    } else {
                        const int n = nb[(int64_t)k * N];
                        take_row(frow[(int64_t)n * rc], n, k == 0);
                    }
                }
            }
            const int64_t at = ((int64_t)b * N + m) * rc + chunk0 + c4;
            __builtin_nontemporal_store(v4f{v0, v1, v2, v3}, &reinterpret_cast<v4f *>(out)[at]);
            __builtin_nontemporal_store(i4v{b0, b1, b2, b3}, &reinterpret_cast<i4v *>(argmax)[at]);
        }
    }
}

hipError_t launch_pool_fwd_planned(const float *feat, const int32_t *nbr, void *plan, float *out, int32_t *argmax,
                                   int B, int N, int K, int C, hipStream_t s)
{
    const PoolPlanLayout l = pool_plan_layout(B, N, K);
    if (l.tiles > 0x7fffffff - 64 || C % 64 != 0 || C > 256) return hipErrorInvalidValue;
    char *base = reinterpret_cast<char *>(plan);
    const int32_t *hdr = reinterpret_cast<const int32_t *>(base + l.hdr_off);
    const int64_t per_xcd = (l.tiles + 7) >> 3, wgs = 8 * ((per_xcd + POOL_FWD_PLAN_TPW - 1) / POOL_FWD_PLAN_TPW);
    for (int blk = 0; blk < C / 64; ++blk)
        hipLaunchKernelGGL(pool_fwd_planned64_kernel, dim3((unsigned)wgs), dim3(512), 0, s, feat, nbr, hdr,
                           reinterpret_cast<const int32_t *>(base + l.cnt_off),
                           reinterpret_cast<const int32_t *>(base + l.rows_off),
                           reinterpret_cast<const unsigned short *>(base + l.slot_off), out, argmax, N, K,
                           l.tiles_per_cloud, (int)l.tiles, C / 4, 16 * blk);
    return hipGetLastError();
}

// Channel-major ([B,C,N]) gather form.  A block owns 64 consecutive points, whose in-edge lists are one
// contiguous range of entries.  The gathers run over that range with lane = entry (a lane per point would
// idle until the longest of 64 lists is done): per chunk of ECH entries the block parks the entries and
// the point each belongs to in LDS, every wave gathers winner-table and gradient values of its CH channels
// for all entries (CH x 4 pairs in flight per lane) and parks what each entry routes, and then, with
// lane = point, adds up each point's own stretch in list order.
template <int ECH>
__global__ __launch_bounds__(256) void pool_bwd_gather_bcn_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src,
    float *__restrict__ grad_feat, int N, int L, int C, int tiles_per_cloud, int64_t total_tiles)
{
    constexpr int CH = 4, U = 4, J = ECH / 64;
    static_assert(ECH % (64 * U) == 0, "a lane takes U entries of a chunk at a time");
    __shared__ int s_off[65];
    __shared__ int s_l[ECH];            // source row of each entry
    __shared__ unsigned char s_t[ECH];  // its point (0..63), +64 unless it repeats the entry before it
    // what the entry routes, per channel of the pass (rows private to a wave); entry i of point p sits at
    // column i + p, so that the points' stretches, which start about K apart, begin in different banks
    __shared__ float s_c[4 * CH][ECH + 64];
    const int64_t tile = xcd_tile(total_tiles);
    if (tile < 0) return;
    const int64_t b = tile / tiles_per_cloud;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: channel rows get scalar base addresses
    const int m0 = (int)(tile - b * tiles_per_cloud) * 64;
    const int np = min(64, N - m0);
    if (threadIdx.x <= 64) s_off[threadIdx.x] = in_off[b * N + m0 + min((int)threadIdx.x, np)];   // past the cloud: empty lists
    __syncthreads();
    const int E0 = s_off[0], E1 = s_off[64];
    const int my0 = s_off[lane], my1 = s_off[lane + 1];
    for (int cg = 0; cg < C; cg += 4 * CH) {
        const int c0 = cg + w * CH;
        const int32_t *arow[CH];
        const float *grow[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            const int64_t at = (b * C + min(c0 + ch, C - 1)) * L;
            arow[ch] = argmax + at;
            grow[ch] = grad_out + at;
        }
        float acc[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch] = 0.f;
        for (int Ec = E0; Ec < E1; Ec += ECH) {         // the same trips for every thread of the block
            const int nEc = min(ECH, E1 - Ec);
            const int lo = max(my0, Ec) - Ec, hi = min(my1, Ec + nEc) - Ec;   // this lane's point, within the chunk
            __syncthreads();                            // every wave is done with the chunk before
            for (int i = threadIdx.x; i < nEc; i += 256) s_l[i] = in_src[Ec + i];
            if (w == 0)
                for (int i = lo; i < hi; ++i) {
                    // a centre that lists the point twice (adjacent entries) routes one gradient
                    const int e = Ec + i;
                    const bool fresh = e == my0 || in_src[e] != in_src[e - 1];
                    s_t[i] = (unsigned char)(lane + (fresh ? 64 : 0));
                }
            __syncthreads();
#pragma unroll
            for (int j0 = 0; j0 < J; j0 += U) {
                if (j0 * 64 < nEc) {
                    int l[U], t[U], a[CH][U];
                    float g[CH][U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int i = (j0 + u) * 64 + lane;
                        l[u] = s_l[i < nEc ? i : 0];
                        t[u] = i < nEc ? s_t[i] : 0;    // past the end: routes nothing
                    }
#pragma unroll
                    for (int ch = 0; ch < CH; ++ch)
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            a[ch][u] = at_byte(arow[ch], 4u * (unsigned)l[u]);
                            g[ch][u] = at_byte(grow[ch], 4u * (unsigned)l[u]);
                        }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int i = (j0 + u) * 64 + lane;
                        const int m = m0 + (t[u] & 63);
#pragma unroll
                        for (int ch = 0; ch < CH; ++ch)
                            if (i < nEc) s_c[w * CH + ch][i + (t[u] & 63)] = ((t[u] & 64) && a[ch][u] == m) ? g[ch][u] : 0.f;
                    }
                }
            }
            // rows w*CH.. of s_c are written and read by this wave only, whose LDS operations keep their order
#pragma unroll 1
            for (int i = lo; i < hi; ++i)
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) acc[ch] += s_c[w * CH + ch][i + lane];
        }
#pragma unroll
        for (int ch = 0; ch < CH; ++ch)
            if (lane < np && c0 + ch < C)
                __builtin_nontemporal_store(acc[ch], &grad_feat[(b * C + c0 + ch) * N + m0 + lane]);
    }
}

__global__ __launch_bounds__(256) void pool_bwd_gather_generic_kernel(
    const float *__restrict__ grad_out, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ in_off, const int32_t *__restrict__ in_src,
    float *__restrict__ grad_feat, int B, int N, int L, int C, int bnc)
{
    const int64_t total = (int64_t)B * N * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int64_t b; int c, m;
        if (bnc) { c = (int)(i % C); const int64_t gp = i / C; b = gp / N; m = (int)(gp % N); }
        else     { m = (int)(i % N); const int64_t bc = i / N; b = bc / C; c = (int)(bc % C); }
        const int64_t gp = b * N + m;
        float acc = 0.f;
        const int e1 = in_off[gp + 1];
        int prev = -1;
        for (int e = in_off[gp]; e < e1; ++e) {
            const int64_t l = in_src[e];
            if ((int)l == prev) continue;
            prev = (int)l;
            const int64_t at = bnc ? (b * L + l) * C + c : (b * C + c) * L + l;
            if (argmax[at] == m) acc += grad_out[at];
        }
        grad_feat[i] = acc;
    }
}

hipError_t launch_pool_bwd_gather(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                                  const int32_t *in_src, float *grad_feat, int B, int N, int C, int bnc,
                                  hipStream_t s)
{
    return launch_pool_sub_bwd_gather(grad_out, argmax, in_off, in_src, grad_feat, B, N, N, C, bnc, s);
}

// L rows of grad_out / argmax per cloud, lists over them for each of the N points
hipError_t launch_pool_sub_bwd_gather(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                                      const int32_t *in_src, float *grad_feat, int B, int N, int L, int C,
                                      int bnc, hipStream_t s)
{
    if (bnc && (C % 4 == 0)) {
        const int C4 = C / 4;
        const int PT = C4 >= 256 ? 1 : 256 / C4;
        const int64_t BN = (int64_t)B * N, tiles = (BN + PT - 1) / PT;
        if (C4 % 16 == 0 && 2 * (int64_t)L <= N)
            hipLaunchKernelGGL(pool_bwd_gather_row16_kernel<2>, dim3(xcd_grid(tiles)), dim3(256), 0, s, grad_out,
                               argmax, in_off, in_src, grad_feat, BN, N, L, C4, PT, tiles);
        else if (C4 % 16 == 0)
            hipLaunchKernelGGL(pool_bwd_gather_row16_kernel<4>, dim3(xcd_grid(tiles)), dim3(256), 0, s, grad_out,
                               argmax, in_off, in_src, grad_feat, BN, N, L, C4, PT, tiles);
        else if (2 * (int64_t)L <= N)     // lists a quarter as long (subsampling keeps a quarter of the centres)
            hipLaunchKernelGGL(pool_bwd_gather_bnc4_kernel<2>, dim3(xcd_grid(tiles)), dim3(256), 0, s, grad_out,
                               argmax, in_off, in_src, grad_feat, BN, N, L, C4, PT, tiles);
        else
            hipLaunchKernelGGL(pool_bwd_gather_bnc4_kernel<4>, dim3(xcd_grid(tiles)), dim3(256), 0, s, grad_out,
                               argmax, in_off, in_src, grad_feat, BN, N, L, C4, PT, tiles);
    } else if (!bnc && L < (1 << 30)) {
        const int tpc = (N + 63) / 64;
        const int64_t tiles = (int64_t)B * tpc;
        hipLaunchKernelGGL(pool_bwd_gather_bcn_kernel<512>, dim3(xcd_grid(tiles)), dim3(256), 0, s, grad_out,
                           argmax, in_off, in_src, grad_feat, N, L, C, tpc, tiles);
    } else {
        const int64_t total = (int64_t)B * N * C;
        int64_t blocks = (total + 255) / 256;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(pool_bwd_gather_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                           grad_out, argmax, in_off, in_src, grad_feat, B, N, L, C, bnc);
    }
    return hipGetLastError();
}

hipError_t launch_pool_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat, int B,
                           int N, int C, int bnc, hipStream_t s)
{
    return launch_pool_sub_bwd(grad_out, argmax, grad_feat, B, N, N, C, bnc, s);
}

// scatter form for L source rows per cloud (atomics)
hipError_t launch_pool_sub_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat, int B,
                               int N, int L, int C, int bnc, hipStream_t s)
{
    hipError_t e = launch_fill_zero(grad_feat, sizeof(float) * (size_t)B * N * C, s);
    if (e != hipSuccess) return e;
    const int64_t total = (int64_t)B * L * C;
    int64_t blocks = (total + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    hipLaunchKernelGGL(pool_bwd_kernel, dim3((unsigned)blocks), dim3(256), 0, s, grad_out, argmax,
                       grad_feat, B, N, L, C, bnc);
    return hipGetLastError();
}

}  // namespace flex
