// One instantiation of the tiled kernels; compiled once per line of
// flex_shapes.def with -DFLEX_DI= -DFLEX_DO= -DFLEX_W= -DFLEX_T= -DFLEX_OCC= -DFLEX_WS=.
#include "flex_tiled.hpp"
#if FLEX_WS
#include "flex_ws.hpp"
#endif

#if !defined(FLEX_DI) || !defined(FLEX_DO) || !defined(FLEX_W) || !defined(FLEX_T) || !defined(FLEX_OCC) || !defined(FLEX_WS)
#error "build with -DFLEX_DI -DFLEX_DO -DFLEX_W -DFLEX_T -DFLEX_OCC -DFLEX_WS"
#endif

#define FLEX_CAT5(a, b, c) a##_##b##_##c
#define FLEX_NAME(a, b, c) FLEX_CAT5(a, b, c)

namespace flex {

using S = TileShape<FLEX_DI, FLEX_DO, FLEX_W, FLEX_T, FLEX_OCC>;
static constexpr int WG_PER_CU = (FLEX_OCC * 4) / FLEX_W > 0 ? (FLEX_OCC * 4) / FLEX_W : 1;

// 1 if this (shape, K, list form) runs the wave-specialised kernel with the split-half
// contraction, i.e. wants the parameters from launch_pack_theta_f16; 0: fp32 ThetaP.
// the lean fixed-K producers take this neighbour tensor: 32-bit byte offsets in a cloud (any K: batches of 8
// slots, the last one of a tile masked past K)
static bool lean_fixed_ok(int N, int K)
{
    return lean_producer_mode() != 0 && (int64_t)K * N * 4 < (1ll << 32) &&
           (int64_t)N * S::DI * 4 < (1ll << 32) && (int64_t)N * 12 < (1ll << 32);
}

int FLEX_NAME(theta_format, FLEX_DI, FLEX_DO)(int N, int K, int csr)
{
#if FLEX_WS
    using W = WsGeom<S>;
    if (!contract_in_fp32() && (csr || (int64_t)W::PW * K <= W::EW || lean_fixed_ok(N, K))) return 1;
#endif
    (void)N; (void)K; (void)csr;
    return 0;
}

// Which kernel family launch_gc picks for (N, K, list form) with the parameters in the format theta_format
// answers: 3 = lean wave-specialised producers, 2 = LDS-staged wave-specialised, 1 = single-role kernels.
// launch_gc dispatches on this same function.
static int gc_route(int N, int K, int csr, int theta_fmt)
{
#if FLEX_WS
    using W = WsGeom<S>;
    if (csr || (int64_t)W::PW * K <= W::EW || (theta_fmt && lean_fixed_ok(N, K))) {
        if (!csr && theta_fmt && lean_fixed_ok(N, K)) return 3;
        if (csr && theta_fmt && lean_producer_mode() != 0 && (int64_t)N * S::DI * 4 < (1ll << 32) &&
            (int64_t)N * 12 < (1ll << 32))
            return 3;
        return 2;
    }
#endif
    (void)N; (void)K; (void)csr; (void)theta_fmt;
    return 1;
}

int FLEX_NAME(route, FLEX_DI, FLEX_DO)(int N, int K, int csr)
{
    return gc_route(N, K, csr, FLEX_NAME(theta_format, FLEX_DI, FLEX_DO)(N, K, csr));
}

hipError_t FLEX_NAME(launch_gc, FLEX_DI, FLEX_DO)(const float *rows, const float *pos,
                                                  const int32_t *nbr, const int32_t *off,
                                                  const int32_t *src, const int32_t *order, const void *thetaP,
                                                  int theta_fmt, float *out, int B, int N, int K,
                                                  int csr, int out_bcn, hipStream_t s)
{
    const int tiles_per_cloud = (N + S::T - 1) / S::T;
    const int64_t total64 = (int64_t)B * tiles_per_cloud;
    if (total64 > 0x7fffffff) return hipErrorInvalidValue;
    const int total = (int)total64;
    const int grid = persistent_grid(total, WG_PER_CU);
#if FLEX_WS
    {
        using W = WsGeom<S>;
        const int route = gc_route(N, K, csr, theta_fmt);
        if (route >= 2) {
            const int tpc = (N + W::T - 1) / W::T;
            const int tot = B * tpc;
            const dim3 g(persistent_grid(tot, W::WG_PER_CU)), blk(W::NT);
            const int exp_off = (int)theta_f16_exp_offset(S::DIP, S::DOP);
#define FLEX_WS_ARGS rows, pos, nbr, off, src, thetaP, exp_off, out, N, K, tpc, tot
#define FLEX_WS_LAUNCH(CSR_, BCN_)                                                                          \
    do {                                                                                                    \
        if (theta_fmt) hipLaunchKernelGGL((gather_contract_ws_kernel<S, CSR_, BCN_, true>), g, blk, 0, s, FLEX_WS_ARGS); \
        else hipLaunchKernelGGL((gather_contract_ws_kernel<S, CSR_, BCN_, false>), g, blk, 0, s, FLEX_WS_ARGS);          \
    } while (0)
            // lean producer: fixed-K tensor, 32-bit byte offsets inside a cloud
            const bool lean = !csr && route == 3;
            if (lean) {
                // 3 producer waves per consumer wave where 16 waves hold them and the items divide evenly
                constexpr bool WIDE_OK = (S::WAVES * 4 <= 16) && (((S::DOP / 16) * (S::T * 3 / 16)) % S::WAVES == 0);
                constexpr int PMX = WIDE_OK ? 3 : 1;
                const bool wide = PMX > 1 && lean_producer_mode() != 1;
                using WL = WsGeom<S, PMX>;
                const int tl = wide ? WL::T : W::T;
                const int tpcl = (N + tl - 1) / tl;
                const int totl = B * tpcl;
                const dim3 gl(persistent_grid(totl, wide ? WL::WG_PER_CU : W::WG_PER_CU)), bl(wide ? WL::NT : W::NT);
#define FLEX_LEAN_ARGS rows, pos, nbr, thetaP, exp_off, out, N, K, tpcl, totl
#define FLEX_LEAN_LAUNCH(BCN_, PM_)                                                                              \
    do {                                                                                                         \
        if (K % 8 == 0) hipLaunchKernelGGL((gather_contract_lean_kernel<S, BCN_, PM_>), gl, bl, 0, s, FLEX_LEAN_ARGS); \
        else hipLaunchKernelGGL((gather_contract_lean_kernel<S, BCN_, PM_, S::DI, S::DO, false, true>), gl, bl, 0, s, FLEX_LEAN_ARGS); \
    } while (0)
                if (wide && !out_bcn) FLEX_LEAN_LAUNCH(false, PMX);
                else if (wide) FLEX_LEAN_LAUNCH(true, PMX);
                else if (!out_bcn) FLEX_LEAN_LAUNCH(false, 1);
                else FLEX_LEAN_LAUNCH(true, 1);
#undef FLEX_LEAN_LAUNCH
#undef FLEX_LEAN_ARGS
                return hipGetLastError();
            }
            // feature gradient: lean in-edge producers under the same conditions
            const bool lean_csr = csr && route == 3;
            if (lean_csr) {
                if (order == nullptr) return hipErrorInvalidValue;
                constexpr bool WIDE_OK = (S::WAVES * 4 <= 16) && (((S::DOP / 16) * (S::T * 3 / 16)) % S::WAVES == 0);
                constexpr int PMX = WIDE_OK ? 3 : 1;
                const bool wide = PMX > 1 && lean_producer_mode() != 1;
                using WL = WsGeom<S, PMX>;
                const int tl = wide ? WL::T : W::T;
                const int tpcl = (N + tl - 1) / tl;
                const int totl = B * tpcl;
                const dim3 gl(persistent_grid(totl, wide ? WL::WG_PER_CU : W::WG_PER_CU)), bl(wide ? WL::NT : W::NT);
#define FLEX_LEAN_ARGS rows, pos, off, src, order, thetaP, exp_off, out, N, tpcl, totl
                if (wide && !out_bcn) hipLaunchKernelGGL((grad_feat_lean_kernel<S, false, PMX>), gl, bl, 0, s, FLEX_LEAN_ARGS);
                else if (wide) hipLaunchKernelGGL((grad_feat_lean_kernel<S, true, PMX>), gl, bl, 0, s, FLEX_LEAN_ARGS);
                else if (!out_bcn) hipLaunchKernelGGL((grad_feat_lean_kernel<S, false, 1>), gl, bl, 0, s, FLEX_LEAN_ARGS);
                else hipLaunchKernelGGL((grad_feat_lean_kernel<S, true, 1>), gl, bl, 0, s, FLEX_LEAN_ARGS);
#undef FLEX_LEAN_ARGS
                return hipGetLastError();
            }
            if (!csr && !out_bcn) FLEX_WS_LAUNCH(false, false);
            else if (!csr && out_bcn) FLEX_WS_LAUNCH(false, true);
            else if (csr && !out_bcn) FLEX_WS_LAUNCH(true, false);
            else FLEX_WS_LAUNCH(true, true);
#undef FLEX_WS_LAUNCH
#undef FLEX_WS_ARGS
            return hipGetLastError();
        }
    }
#endif
    if (theta_fmt) return hipErrorInvalidValue;   // the single-role kernels take fp32 ThetaP only
    const float *thetaF32 = reinterpret_cast<const float *>(thetaP);
#define FLEX_GC_ARGS rows, pos, nbr, off, src, thetaF32, out, N, K, tiles_per_cloud, total
    const dim3 g(grid), blk(S::NT);
    using G = WaveGeom<S>;
    const bool fast = csr || ((int64_t)G::PW * K <= G::EW);
    if (fast) {
        if (!csr && !out_bcn) hipLaunchKernelGGL((gather_contract_fast_kernel<S, false, false>), g, blk, 0, s, FLEX_GC_ARGS);
        else if (!csr && out_bcn) hipLaunchKernelGGL((gather_contract_fast_kernel<S, false, true>), g, blk, 0, s, FLEX_GC_ARGS);
        else if (csr && !out_bcn) hipLaunchKernelGGL((gather_contract_fast_kernel<S, true, false>), g, blk, 0, s, FLEX_GC_ARGS);
        else hipLaunchKernelGGL((gather_contract_fast_kernel<S, true, true>), g, blk, 0, s, FLEX_GC_ARGS);
    } else {
        // neighbourhoods too large for the wave-private staging: chunked kernel
        if (!out_bcn) hipLaunchKernelGGL((gather_contract_kernel<S, false, false>), g, blk, 0, s, FLEX_GC_ARGS);
        else hipLaunchKernelGGL((gather_contract_kernel<S, false, true>), g, blk, 0, s, FLEX_GC_ARGS);
    }
#undef FLEX_GC_ARGS
    return hipGetLastError();
}

// Launches the per-workgroup partial kernel; *n_wg = number of partial blocks written.
hipError_t FLEX_NAME(launch_gt, FLEX_DI, FLEX_DO)(const float *rows, const float *pos,
                                                  const int32_t *nbr, const float *g_rows,
                                                  float *partials, int B, int N, int K, int *n_wg,
                                                  hipStream_t s)
{
    const int tiles_per_cloud = (N + S::T - 1) / S::T;
    const int64_t total64 = (int64_t)B * tiles_per_cloud;
    if (total64 > 0x7fffffff) return hipErrorInvalidValue;
    const int total = (int)total64;
    const int grid = persistent_grid(total, WG_PER_CU);
    *n_wg = grid;
#if FLEX_WS
    if constexpr (S::WAVES == 4 && S::T == 16) {
        // lean producers + bf16 matrix cores: fixed-K tensor, 32-bit offsets in a cloud
        using WL = WsGeom<S, 2, 2>;
        if (!contract_in_fp32() && lean_fixed_ok(N, K)) {
            const int tpc = (N + WL::T - 1) / WL::T;
            const int tot = B * tpc;
            *n_wg = persistent_grid(tot, 1);
            if (K % 8 == 0)
                hipLaunchKernelGGL((grad_theta_lean_kernel<S>), dim3(*n_wg), dim3(WL::NT), 0, s, rows, pos, nbr, g_rows, partials, N, K, tpc, tot);
            else
                hipLaunchKernelGGL((grad_theta_lean_kernel<S, S::DI, S::DO, true>), dim3(*n_wg), dim3(WL::NT), 0, s, rows, pos, nbr, g_rows, partials, N, K, tpc, tot);
            return hipGetLastError();
        }
    }
    {
        using W = WsGeom<S>;
        if ((int64_t)W::PW * K <= W::EW) {
            const int tpc = (N + W::T - 1) / W::T;
            const int tot = B * tpc;
            *n_wg = persistent_grid(tot, W::WG_PER_CU);
            hipLaunchKernelGGL((grad_theta_ws_kernel<S>), dim3(*n_wg), dim3(W::NT), 0, s, rows, pos, nbr, g_rows, partials, N, K, tpc, tot);
            return hipGetLastError();
        }
    }
#endif
    using G = WaveGeom<S>;
    if ((int64_t)G::PW * K <= G::EW)
        hipLaunchKernelGGL((grad_theta_fast_kernel<S>), dim3(grid), dim3(S::NT), 0, s, rows, pos, nbr, g_rows, partials, N, K, tiles_per_cloud, total);
    else
        hipLaunchKernelGGL((grad_theta_kernel<S>), dim3(grid), dim3(S::NT), 0, s, rows, pos, nbr, g_rows, partials, N, K, tiles_per_cloud, total);
    return hipGetLastError();
}

#if FLEX_WS && FLEX_DI == 64 && FLEX_DO == 64
// The 64 -> 64 layer's feature gradient and parameter gradients as one pass over the in-edge lists
// (bwd_fused_lean_kernel), followed by the stand-alone parameter-gradient kernel in its run-if-flagged form.
// Taken when both of those would run their lean kernels anyway (FLEX_FUSED_BWD=0 in the environment keeps the
// two separate kernels, for comparisons).
bool bwd_fused_ok_64_64(int N, int K)
{
    static const bool off = [] { const char *v = getenv("FLEX_FUSED_BWD"); return v != nullptr && v[0] == '0'; }();
    return !off && !contract_in_fp32() && lean_fixed_ok(N, K) && gc_route(N, K, 1, 1) == 3;
}

// The stand-alone parameter-gradient kernel over the same grid, run on the device only if *control == want.
static hipError_t launch_gt_if(const int *control, int want, const float *own_rows, const float *pos,
                               const int32_t *nbr, const float *g_rows, float *partials, int N, int K, int tpc, int tot,
                               int n_wg, hipStream_t s)
{
    using WL = WsGeom<S, 2, 2>;
    if (K % 8 == 0)
        hipLaunchKernelGGL((grad_theta_lean_if_kernel<S, false>), dim3(n_wg), dim3(WL::NT), 0, s, control, want,
                           own_rows, pos, nbr, g_rows, partials, N, K, tpc, tot);
    else
        hipLaunchKernelGGL((grad_theta_lean_if_kernel<S, true>), dim3(n_wg), dim3(WL::NT), 0, s, control, want,
                           own_rows, pos, nbr, g_rows, partials, N, K, tpc, tot);
    return hipGetLastError();
}

// g_rows / own_rows: upstream gradient and features, point-major; partials: *n_wg blocks of [4*64 x 64];
// control: fused_control_bytes() whose flag word the caller has zeroed on the stream.  Leaves the partials of the
// parameter gradients (the one-pass kernel's, or the stand-alone kernel's if a row overflowed) and the workgroups'
// records for the check after the reduction.
hipError_t launch_bwd_fused_64_64(const float *g_rows, const float *own_rows, const float *pos, const int32_t *nbr,
                                  const int32_t *off, const int32_t *src, const int32_t *order, const void *thetaP,
                                  float *grad_feat, float *partials, int *control, int B, int N, int K, int out_bcn,
                                  int *n_wg, hipStream_t s)
{
    using F = FusedGeom<S>;
    using WL = WsGeom<S, 2, 2>;
    static_assert(WL::T == F::G::T, "the fall-back kernel leaves one partial per workgroup of the same grid");
    if (!bwd_fused_ok_64_64(N, K)) return hipErrorInvalidValue;
    const int tpc = (N + F::G::T - 1) / F::G::T;
    const int64_t tot64 = (int64_t)B * tpc;
    if (tot64 > 0x7fffffff) return hipErrorInvalidValue;
    const int tot = (int)tot64;
    *n_wg = persistent_grid(tot, 1);
    if (*n_wg > FUSED_MAX_WG) return hipErrorInvalidValue;
    const int exp_off = (int)theta_f16_exp_offset(S::DIP, S::DOP);
    const dim3 g(*n_wg);
#define FLEX_FUSED_ARGS g_rows, own_rows, pos, off, src, order, thetaP, exp_off, grad_feat, partials, control, N, tpc, tot
    if (out_bcn) hipLaunchKernelGGL((bwd_fused_lean_kernel<S, true>), g, dim3(F::NT), 0, s, FLEX_FUSED_ARGS);
    else hipLaunchKernelGGL((bwd_fused_lean_kernel<S, false>), g, dim3(F::NT), 0, s, FLEX_FUSED_ARGS);
#undef FLEX_FUSED_ARGS
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_gt_if(control, FUSED_OVERFLOW, own_rows, pos, nbr, g_rows, partials, N, K, tpc, tot, *n_wg, s);
}

// The hand-over after the check: the stand-alone kernel again, run only if the check set FUSED_UNRESOLVED.
hipError_t launch_bwd_fused_late_64_64(const float *g_rows, const float *own_rows, const float *pos,
                                       const int32_t *nbr, float *partials, const int *control, int B, int N, int K,
                                       hipStream_t s)
{
    using F = FusedGeom<S>;
    const int tpc = (N + F::G::T - 1) / F::G::T;
    const int tot = B * tpc;
    return launch_gt_if(control, FUSED_UNRESOLVED, own_rows, pos, nbr, g_rows, partials, N, K, tpc, tot,
                        persistent_grid(tot, 1), s);
}
#endif

#if FLEX_WS && FLEX_DI == 64 && FLEX_DO == 128
// 128 -> 128 layers as two passes of this shape's lean kernels: each gathers one 64-channel half of the
// 128-wide rows (row stride 128) and contracts it with its [4*64 x 128] block of the parameters; the second
// pass adds to the first one's output.  Point-major tensors only.
bool split_ok_128_128(int N, int K, int csr)
{
    if (contract_in_fp32() || lean_producer_mode() == 0) return false;
    if ((int64_t)N * 128 * 4 >= (1ll << 32) || (int64_t)N * 12 >= (1ll << 32)) return false;
    return csr || ((K % 8 == 0) && (int64_t)K * N * 4 < (1ll << 32));
}

hipError_t launch_gc_split_128_128(const float *rows_half, const float *pos, const int32_t *nbr, const int32_t *off,
                                   const int32_t *src, const int32_t *order, const void *thetaP, float *out, int B,
                                   int N, int K, int csr, int accumulate, hipStream_t s)
{
    using W = WsGeom<S, 1>;
    const int tpc = (N + W::T - 1) / W::T;
    const int64_t tot64 = (int64_t)B * tpc;
    if (tot64 > 0x7fffffff) return hipErrorInvalidValue;
    const int tot = (int)tot64;
    const dim3 g(persistent_grid(tot, W::WG_PER_CU)), blk(W::NT);
    const int exp_off = (int)theta_f16_exp_offset(S::DIP, S::DOP);
    if (csr && order == nullptr) return hipErrorInvalidValue;
    if (!csr) {
        if (accumulate) hipLaunchKernelGGL((gather_contract_lean_kernel<S, false, 1, 128, 128, true>), g, blk, 0, s, rows_half, pos, nbr, thetaP, exp_off, out, N, K, tpc, tot);
        else hipLaunchKernelGGL((gather_contract_lean_kernel<S, false, 1, 128, 128, false>), g, blk, 0, s, rows_half, pos, nbr, thetaP, exp_off, out, N, K, tpc, tot);
    } else {
        if (accumulate) hipLaunchKernelGGL((grad_feat_lean_kernel<S, false, 1, 128, 128, true>), g, blk, 0, s, rows_half, pos, off, src, order, thetaP, exp_off, out, N, tpc, tot);
        else hipLaunchKernelGGL((grad_feat_lean_kernel<S, false, 1, 128, 128, false>), g, blk, 0, s, rows_half, pos, off, src, order, thetaP, exp_off, out, N, tpc, tot);
    }
    return hipGetLastError();
}
#endif

#if FLEX_WS && FLEX_DI == 64 && FLEX_DO == 128
// Layers whose widths are multiples of 128 (point-major) run as passes of this shape's lean kernels over column
// blocks, all inside one launch: n_out blocks of 128 output channels (rows os floats apart) as independent jobs,
// each walking its tiles once per block of 64 gathered channels (n_in of them, rows rs floats apart) with its
// [4*64 x 128] block of the parameters (thetaP_all, block j * n_in + i).
bool split_wide_ok(int N, int K, int max_width)
{
    if (contract_in_fp32() || lean_producer_mode() == 0) return false;
    return (int64_t)N * max_width * 4 < (1ll << 32) && (int64_t)N * 12 < (1ll << 32) &&
           (int64_t)K * N * 4 < (1ll << 32);
}

hipError_t launch_gc_split_wide(const float *rows, int rs, const float *pos, const int32_t *nbr, const int32_t *off,
                                const int32_t *src, const int32_t *order, const void *thetaP_all, float *out, int os,
                                int n_in, int n_out, int B, int N, int K, int csr, hipStream_t s)
{
    using W = WsGeom<S, 1>;
    const int tpc = (N + W::T - 1) / W::T;
    const int64_t tot64 = (int64_t)B * tpc;
    if (tot64 > 0x7fffffff) return hipErrorInvalidValue;
    const int tot = (int)tot64;
    // workgroups per output block: enough to fill the device when the blocks are few (whole multiples of 8, so
    // that a share's number tells its XCD), one when they are many
    int chunks = persistent_grid(tot, W::WG_PER_CU) / n_out;
    chunks = chunks >= 8 ? chunks / 8 * 8 : (chunks > 1 ? chunks : 1);
    const dim3 g((unsigned)(n_out * chunks)), blk(W::NT);
    const int exp_off = (int)theta_f16_exp_offset(S::DIP, S::DOP), blk_bytes = (int)theta_f16_bytes(S::DIP, S::DOP);
    if (csr && order == nullptr) return hipErrorInvalidValue;
    if (csr)
        hipLaunchKernelGGL((grad_feat_lean_passes_kernel<S, 1>), g, blk, 0, s, rows, pos, off, src, order, thetaP_all,
                           blk_bytes, exp_off, out, N, tpc, tot, rs, os, n_in, chunks);
    else if (K % 8 == 0)
        hipLaunchKernelGGL((gather_contract_lean_passes_kernel<S, 1, false>), g, blk, 0, s, rows, pos, nbr, thetaP_all,
                           blk_bytes, exp_off, out, N, K, tpc, tot, rs, os, n_in, chunks);
    else
        hipLaunchKernelGGL((gather_contract_lean_passes_kernel<S, 1, true>), g, blk, 0, s, rows, pos, nbr, thetaP_all,
                           blk_bytes, exp_off, out, N, K, tpc, tot, rs, os, n_in, chunks);
    return hipGetLastError();
}
#endif

#if FLEX_WS && FLEX_DI == 64 && FLEX_DO == 64
// Workgroups that share one [4*64 x 64] block of a wide layer's parameter gradient: enough to fill the device
// when the blocks are few, one when they are many.
int split_wide_gt_chunks(int B, int N, int blocks)
{
    using WL = WsGeom<S, 2, 2>;
    const int64_t tot = (int64_t)B * ((N + WL::T - 1) / WL::T);
    const int fill = persistent_grid(tot > 0x7fffffff ? 0x7fffffff : (int)tot, 1);
    return fill / blocks > 1 ? fill / blocks : 1;
}

// All n_hi x n_ho blocks of the parameter gradient of a wide layer in one launch (block p = feature channels
// 64 * (p / n_ho).., upstream-gradient channels 64 * (p % n_ho)..); partials[p * chunks + share].
hipError_t launch_gt_split_wide(const float *rows, int rs, const float *pos, const int32_t *nbr, const float *g_rows,
                                int gst, float *partials, int n_hi, int n_ho, int chunks, int B, int N, int K,
                                hipStream_t s)
{
    using WL = WsGeom<S, 2, 2>;
    const int tpc = (N + WL::T - 1) / WL::T;
    const int64_t tot64 = (int64_t)B * tpc, grid = (int64_t)n_hi * n_ho * chunks;
    if (tot64 > 0x7fffffff || grid > 0x7fffffff) return hipErrorInvalidValue;
    const int tot = (int)tot64;
    if (K % 8 == 0)
        hipLaunchKernelGGL((grad_theta_lean_blocks_kernel<S, false>), dim3((unsigned)grid), dim3(WL::NT), 0, s, rows,
                           pos, nbr, g_rows, partials, N, K, tpc, tot, rs, gst, chunks, n_ho);
    else
        hipLaunchKernelGGL((grad_theta_lean_blocks_kernel<S, true>), dim3((unsigned)grid), dim3(WL::NT), 0, s, rows,
                           pos, nbr, g_rows, partials, N, K, tpc, tot, rs, gst, chunks, n_ho);
    return hipGetLastError();
}

// One [4*64 x 64] block of the parameter gradient of a 128 -> 128 layer: the aggregate of a 64-channel half of
// the 128-wide feature rows against a 64-channel half of the 128-wide upstream gradient rows.
hipError_t launch_gt_split_128_128(const float *rows_half, const float *pos, const int32_t *nbr,
                                   const float *g_half, float *partials, int B, int N, int K, int *n_wg,
                                   hipStream_t s)
{
    using WL = WsGeom<S, 2, 2>;
    const int tpc = (N + WL::T - 1) / WL::T;
    const int64_t tot64 = (int64_t)B * tpc;
    if (tot64 > 0x7fffffff) return hipErrorInvalidValue;
    const int tot = (int)tot64;
    *n_wg = persistent_grid(tot, 1);
    hipLaunchKernelGGL((grad_theta_lean_kernel<S, 128, 128>), dim3(*n_wg), dim3(WL::NT), 0, s, rows_half, pos, nbr,
                       g_half, partials, N, K, tpc, tot);
    return hipGetLastError();
}
#endif

// One term of the location gradient; false / hipErrorNotSupported when this shape has no kernel for it.
bool FLEX_NAME(gp_ok, FLEX_DI, FLEX_DO)(int N, int K)
{
#if FLEX_WS
    if constexpr (S::WAVES == 4 && S::T == 16 && PosGeom<S>::FITS)
        return !contract_in_fp32() && lean_fixed_ok(N, K);
#endif
    (void)N; (void)K;
    return false;
}

hipError_t FLEX_NAME(launch_gp, FLEX_DI, FLEX_DO)(const float *rows, const int32_t *nbr, const int32_t *off,
                                                  const int32_t *src, const void *thetaF,
                                                  const float *dot_rows, float *grad_pos, float sign,
                                                  int accumulate, int B, int N, int K, int csr, hipStream_t s)
{
#if FLEX_WS
    if constexpr (S::WAVES == 4 && S::T == 16 && PosGeom<S>::FITS) {
        constexpr bool WIDE_OK = (((S::DOP / 16) * (S::T * 3 / 16)) % S::WAVES == 0);
        constexpr int PMX = WIDE_OK ? 3 : 1;
        using WL = WsGeom<S, PMX>;
        const int tpc = (N + WL::T - 1) / WL::T;
        const int tot = B * tpc;
        const dim3 g(persistent_grid(tot, WL::WG_PER_CU)), blk(WL::NT);
        const int exp_off = (int)theta_pos_exp_offset(PosGeom<S>::KDP, S::DOP);
        if (csr)
            hipLaunchKernelGGL((grad_pos_kernel<S, true, PMX>), g, blk, 0, s, rows, nbr, off, src, thetaF, exp_off,
                               dot_rows, grad_pos, sign, accumulate, N, K, tpc, tot);
        else if (K % 8 == 0)
            hipLaunchKernelGGL((grad_pos_kernel<S, false, PMX>), g, blk, 0, s, rows, nbr, off, src, thetaF, exp_off,
                               dot_rows, grad_pos, sign, accumulate, N, K, tpc, tot);
        else
            hipLaunchKernelGGL((grad_pos_kernel<S, false, PMX, true>), g, blk, 0, s, rows, nbr, off, src, thetaF,
                               exp_off, dot_rows, grad_pos, sign, accumulate, N, K, tpc, tot);
        return hipGetLastError();
    }
#endif
    return hipErrorNotSupported;
}

}  // namespace flex
