// C-ABI entry points of libflexconv: validation, workspace carving, dispatch.
#include "flex_common.hpp"
#include <stdlib.h>
#include <mutex>
#include "../../include/flexconv.h"

namespace flex {

// ---- per-shape launchers generated from flex_shapes.def ------------------------
#define FLEX_SHAPE(DI, DO, W, T, OCC, WS)                                                             \
    hipError_t launch_gc_##DI##_##DO(const float *, const float *, const int32_t *, const int32_t *, \
                                     const int32_t *, const int32_t *, const void *, int, float *, int, int, int, \
                                     int, int, hipStream_t);                                         \
    int theta_format_##DI##_##DO(int, int, int);                                                       \
    int route_##DI##_##DO(int, int, int);                                                              \
    bool gp_ok_##DI##_##DO(int, int);                                                                 \
    hipError_t launch_gp_##DI##_##DO(const float *, const int32_t *, const int32_t *, const int32_t *, \
                                     const void *, const float *, float *, float, int, int, int, int,  \
                                     int, hipStream_t);                                                        \
    hipError_t launch_gt_##DI##_##DO(const float *, const float *, const int32_t *, const float *,   \
                                     float *, int, int, int, int *, hipStream_t);
#include "flex_shapes.def"
#undef FLEX_SHAPE

// 64 -> 64 layers: feature and parameter gradients in one pass over the in-edge lists (flex_tiled_inst.hip, shape 64x64)
bool bwd_fused_ok_64_64(int N, int K);
hipError_t launch_bwd_fused_64_64(const float *g_rows, const float *own_rows, const float *pos, const int32_t *nbr,
                                  const int32_t *off, const int32_t *src, const int32_t *order, const void *thetaP,
                                  float *grad_feat, float *partials, int *control, int B, int N, int K, int out_bcn,
                                  int *n_wg, hipStream_t s);
hipError_t launch_bwd_fused_late_64_64(const float *g_rows, const float *own_rows, const float *pos,
                                       const int32_t *nbr, float *partials, const int *control, int B, int N, int K,
                                       hipStream_t s);

// 128 -> 128 layers as passes over 64-channel blocks (flex_tiled_inst.hip, shapes 64x128 and 64x64)
bool split_ok_128_128(int N, int K, int csr);
hipError_t launch_gc_split_128_128(const float *rows_half, const float *pos, const int32_t *nbr, const int32_t *off,
                                   const int32_t *src, const int32_t *order, const void *thetaP, float *out, int B,
                                   int N, int K, int csr, int accumulate, hipStream_t s);
hipError_t launch_gt_split_128_128(const float *rows_half, const float *pos, const int32_t *nbr,
                                   const float *g_half, float *partials, int B, int N, int K, int *n_wg,
                                   hipStream_t s);

// layers with both widths multiples of 128 as passes over column blocks (same file, same two shapes)
bool split_wide_ok(int N, int K, int max_width);
hipError_t launch_gc_split_wide(const float *rows, int rs, const float *pos, const int32_t *nbr, const int32_t *off,
                                const int32_t *src, const int32_t *order, const void *thetaP_all, float *out, int os,
                                int n_in, int n_out, int B, int N, int K, int csr, hipStream_t s);
hipError_t launch_gt_split_wide(const float *rows, int rs, const float *pos, const int32_t *nbr, const float *g_rows,
                                int gst, float *partials, int n_hi, int n_ho, int chunks, int B, int N, int K,
                                hipStream_t s);
int split_wide_gt_chunks(int B, int N, int blocks);
hipError_t launch_reduce_partials_blocks(const float *partials, int n_wg, int first, int count, int n_ho, int Din,
                                         int Dout, float *grad_theta, float *grad_bias, hipStream_t s);

hipError_t launch_reduce_partials(const float *partials, int n_wg, int DIP, int DOP, int Din,
                                  int Dout, float *grad_theta, float *grad_bias, hipStream_t s);

bool gather_contract_supported(int DI, int DO)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_) return true;
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return false;
}

hipError_t launch_gather_contract(const float *rows, const float *pos, const int32_t *nbr,
                                  const int32_t *off, const int32_t *src, const int32_t *order, const void *thetaP,
                                  int theta_fmt, float *out, int B, int N, int K, int DI, int DO,
                                  int csr, int out_bcn, hipStream_t s)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_)         \
        return launch_gc_##DI_##_##DO_(rows, pos, nbr, off, src, order, thetaP, theta_fmt, out, B, N, K, csr, out_bcn, s);
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return hipErrorNotSupported;
}

int gather_contract_theta_format(int DI, int DO, int N, int K, int csr)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_) return theta_format_##DI_##_##DO_(N, K, csr);
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return 0;
}

int gather_contract_route(int DI, int DO, int N, int K, int csr)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_) return route_##DI_##_##DO_(N, K, csr);
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return 0;
}

bool grad_pos_supported(int DI, int DO, int N, int K)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_) return gp_ok_##DI_##_##DO_(N, K);
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return false;
}

hipError_t launch_grad_pos_term(const float *rows, const int32_t *nbr, const int32_t *off, const int32_t *src,
                                const void *thetaF, const float *dot_rows, float *grad_pos, float sign,
                                int accumulate, int B, int N, int K, int DI, int DO, int csr, hipStream_t s)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS)                                                               \
    if (DI == DI_ && DO == DO_)                                                                           \
        return launch_gp_##DI_##_##DO_(rows, nbr, off, src, thetaF, dot_rows, grad_pos, sign, accumulate, B, N, K, csr, s);
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return hipErrorNotSupported;
}

bool contract_in_fp32()
{
    static const bool f32 = [] {
        const char *v = getenv("FLEX_CONTRACT");
        return v != nullptr && v[0] == 'f' && v[1] == '3' && v[2] == '2' && v[3] == 0;
    }();
    return f32;
}

int lean_producer_mode()
{
    static const int mode = [] {
        const char *v = getenv("FLEX_PRODUCER");
        if (v == nullptr) return 2;
        if (v[0] == 's') return 0;
        if (v[0] == 'l') return 1;
        return 2;
    }();
    return mode;
}

// 128 -> 128 point-major layers run as passes of the 64-wide lean kernels over channel blocks
// (FLEX_SPLIT=0 in the environment keeps them on the single-pass fp32 kernels, for comparisons)
static bool use_split_128(int Din, int Dout, int layout, int N, int K, int csr)
{
    static const bool off = [] { const char *v = getenv("FLEX_SPLIT"); return v != nullptr && v[0] == '0'; }();
    return !off && Din == 128 && Dout == 128 && layout == FLEX_LAYOUT_BNC && split_ok_128_128(N, K, csr);
}

// Forward (transpose == 0: passes over the input-channel halves) or feature gradient (transpose == 1: passes over
// the halves of the upstream gradient's channels) of a 128 -> 128 layer.  scratch: theta_ws_bytes(128, 128).
static hipError_t split_gather_contract_128(const float *rows, const float *pos, const int32_t *nbr,
                                            const int32_t *off, const int32_t *src, const int32_t *order,
                                            const float *theta,
                                            const float *bias, void *scratch, float *out, int B, int N, int K,
                                            int transpose, hipStream_t s)
{
    float *blk_theta = (float *)scratch, *blk_bias = blk_theta + 3 * 64 * 128;
    void *packed = (char *)scratch + sizeof(float) * 4 * 64 * 128;
    for (int h = 0; h < 2; ++h) {
        hipError_t e;
        if (!transpose) {
            e = launch_param_block((float *)theta, (float *)bias, blk_theta, blk_bias, 128, 128, 64 * h, 0, 64, 128, 0, s);
            if (e != hipSuccess) return e;
            e = launch_pack_theta_f16(blk_theta, blk_bias, packed, 64, 128, 64, 128, 0, s);
        } else {
            e = launch_param_block((float *)theta, (float *)bias, blk_theta, blk_bias, 128, 128, 0, 64 * h, 128, 64, 0, s);
            if (e != hipSuccess) return e;
            e = launch_pack_theta_f16(blk_theta, blk_bias, packed, 128, 64, 64, 128, 1, s);
        }
        if (e != hipSuccess) return e;
        e = launch_gc_split_128_128(rows + 64 * h, pos, nbr, off, src, order, packed, out, B, N, K, transpose, h, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Parameter gradients of a 128 -> 128 layer: four [4*64 x 64] blocks.  scratch: room for one block.
static hipError_t split_grad_theta_128(const float *rows, const float *pos, const int32_t *nbr, const float *g_rows,
                                       float *partials, void *scratch, float *grad_theta, float *grad_bias, int B,
                                       int N, int K, hipStream_t s)
{
    float *blk_theta = (float *)scratch, *blk_bias = blk_theta + 3 * 64 * 64;
    for (int hi = 0; hi < 2; ++hi)
        for (int ho = 0; ho < 2; ++ho) {
            int n_wg = 0;
            hipError_t e = launch_gt_split_128_128(rows + 64 * hi, pos, nbr, g_rows + 64 * ho, partials, B, N, K, &n_wg, s);
            if (e != hipSuccess) return e;
            e = launch_reduce_partials(partials, n_wg, 64, 64, 64, 64, blk_theta, blk_bias, s);
            if (e != hipSuccess) return e;
            e = launch_param_block(grad_theta, grad_bias, blk_theta, blk_bias, 128, 128, 64 * hi, 64 * ho, 64, 64, 1, s);
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

// Wide layers (both widths multiples of 128, not 128 -> 128 itself): the paper's network doubles the feature
// length at every resolution stage (Sec. 4.3), so its deeper stages are of this kind.  They run as passes of the
// 64 -> 128 (forward, feature gradient) and 64 -> 64 (parameter gradients) lean kernels over column blocks of the
// point-major tensors.
static bool split_disabled()
{
    static const bool off = [] { const char *v = getenv("FLEX_SPLIT"); return v != nullptr && v[0] == '0'; }();
    return off;
}
static bool wide_shape(int Din, int Dout)
{
    return !split_disabled() && Din % 128 == 0 && Dout % 128 == 0 && (Din > 128 || Dout > 128) &&
           (int64_t)(Din / 64) * (Dout / 64) <= 65535;      // one grid row of the reduction per block
}
// packed parameter blocks of the whole layer (forward / feature gradient)
// channel-major 128 -> 128: transposed copies and the block passes beat the single-pass fp32 kernels that take
// channel-major tensors directly (1M points: forward 1.9 -> 1.2 ms)
static bool wide_route_128(int Din, int Dout, int layout)
{
    return Din == 128 && Dout == 128 && layout == FLEX_LAYOUT_BCN && !split_disabled();
}

static size_t wide_param_scratch_bytes(int Din, int Dout)
{
    const size_t blocks = (size_t)(Din / 64) * (Dout / 64) / 2;     // 64 x 128 each, either way round
    return blocks * theta_f16_bytes(64, 128);
}

// Forward (transpose == 0: rows = features [.., Din], out [.., Dout]) or feature gradient (transpose == 1:
// rows = upstream gradient [.., Dout], out = grad_feat [.., Din]; in-edge lists) of a wide layer: two launches.
static hipError_t wide_gather_contract(const float *rows, const float *pos, const int32_t *nbr, const int32_t *off,
                                       const int32_t *src, const int32_t *order, const float *theta,
                                       const float *bias, void *scratch,
                                       float *out, int B, int N, int K, int Din, int Dout, int transpose,
                                       hipStream_t s)
{
    const int w_in = transpose ? Dout : Din, w_out = transpose ? Din : Dout;   // gathered / written widths
    const int n_in = w_in / 64, n_out = w_out / 128;
    hipError_t e = launch_pack_theta_f16_blocks(theta, bias, scratch, Din, Dout, 64, 128, n_in, n_out, transpose, s);
    if (e != hipSuccess) return e;
    return launch_gc_split_wide(rows, w_in, pos, nbr, off, src, order, scratch, out, w_out, n_in, n_out, B, N, K, transpose, s);
}

// Parameter gradients of a wide layer: (Din/64) x (Dout/64) independent blocks of [4*64 x 64], two launches
// (partial sums per block and workgroup, then their reduction in double).
static size_t wide_partial_bytes(int B, int N, int Din, int Dout)
{
    const int blocks = (Din / 64) * (Dout / 64);
    return align256(sizeof(float) * (size_t)blocks * split_wide_gt_chunks(B, N, blocks) * 4 * 64 * 64);
}

static hipError_t wide_grad_theta(const float *rows, const float *pos, const int32_t *nbr, const float *g_rows,
                                  float *partials, float *grad_theta, float *grad_bias, int B, int N, int K, int Din,
                                  int Dout, hipStream_t s)
{
    const int n_hi = Din / 64, n_ho = Dout / 64, chunks = split_wide_gt_chunks(B, N, n_hi * n_ho);
    hipError_t e = launch_gt_split_wide(rows, Din, pos, nbr, g_rows, Dout, partials, n_hi, n_ho, chunks, B, N, K, s);
    if (e != hipSuccess) return e;
    return launch_reduce_partials_blocks(partials, chunks, 0, n_hi * n_ho, n_ho, Din, Dout, grad_theta, grad_bias, s);
}

// Packs (theta, bias) for launch_gather_contract in the format that kernel wants.
static hipError_t pack_for_contract(const float *theta, const float *bias, void *thetaP, int Din,
                                    int Dout, int transpose, int fmt, hipStream_t s)
{
    const int RP = transpose ? (Dout + 3) / 4 * 4 : (Din + 3) / 4 * 4;
    const int CP = transpose ? (Din + 15) / 16 * 16 : (Dout + 15) / 16 * 16;
    if (fmt) return launch_pack_theta_f16(theta, bias, thetaP, Din, Dout, RP, CP, transpose, s);
    return launch_pack_theta(theta, bias, (float *)thetaP, Din, Dout, RP, CP, transpose, s);
}

// Workspace bytes of the packed parameters in either format (rows padded to 4, columns to 16).
static size_t theta_ws_bytes(int rows, int cols)
{
    const int RP = (rows + 3) / 4 * 4, CP = (cols + 15) / 16 * 16;
    const size_t f32 = align256(sizeof(float) * (size_t)4 * RP * CP);
    const size_t f16 = theta_f16_bytes(RP, CP);
    return f32 > f16 ? f32 : f16;
}

static int shape_tile_points(int DI, int DO)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_) return T;
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return 0;
}

static int shape_wg_per_cu(int DI, int DO)
{
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS) \
    if (DI == DI_ && DO == DO_) return ((OCC * 4) / W > 0) ? (OCC * 4) / W : 1;
#include "flex_shapes.def"
#undef FLEX_SHAPE
    return 0;
}

static inline int pad4(int x) { return (x + 3) / 4 * 4; }
static inline int pad16(int x) { return (x + 15) / 16 * 16; }

size_t grad_theta_partial_bytes(int64_t B, int64_t N, int Din, int Dout)
{
    const int T = shape_tile_points(Din, Dout);
    if (T == 0) return 0;
    const int64_t tiles = B * ((N + T - 1) / T);
    const int grid = persistent_grid(tiles, shape_wg_per_cu(Din, Dout));
    return align256(sizeof(float) * (size_t)grid * 4 * pad4(Din) * pad16(Dout));
}

hipError_t launch_grad_theta(const float *rows, const float *pos, const int32_t *nbr,
                             const float *g_rows, float *partials, float *grad_theta,
                             float *grad_bias, int B, int N, int K, int Din, int Dout, hipStream_t s)
{
    int n_wg = 0;
    hipError_t e = hipErrorNotSupported;
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS)                                                    \
    if (Din == DI_ && Dout == DO_)                                                         \
        e = launch_gt_##DI_##_##DO_(rows, pos, nbr, g_rows, partials, B, N, K, &n_wg, s);
#include "flex_shapes.def"
#undef FLEX_SHAPE
    if (e != hipSuccess) return e;
    return launch_reduce_partials(partials, n_wg, pad4(Din), pad16(Dout), Din, Dout, grad_theta,
                                  grad_bias, s);
}

// ---- workspace plans -----------------------------------------------------------
struct FwdPlan {
    bool tiled, wide;
    size_t thetaP, featT, outT, total;   // byte offsets / total
};
struct BwdPlan {
    bool tiled, wide;
    bool fused;      // feature and parameter gradients, when both are asked for, come from the one-pass kernel
    size_t thetaP, featT, gT, gfT, partials, order, flag, in_off, in_src, inedge_ws, total;
};

// The route (block passes of the wide path / single-pass tiled kernels / direct form) is decided here, once, from
// everything it depends on (sizes, layout, environment switches); the entry points dispatch on the plan's flags
// and never re-decide, so what they write is what the plan reserved.
static FwdPlan plan_fwd(int64_t B, int64_t N, int K, int Din, int Dout, int layout)
{
    FwdPlan p{};
    p.tiled = gather_contract_supported(Din, Dout);
    p.wide = ((!p.tiled && wide_shape(Din, Dout)) || wide_route_128(Din, Dout, layout)) &&
             split_wide_ok((int)N, K, Din > Dout ? Din : Dout);
    size_t at = 0;
    if (p.tiled || p.wide) {
        p.thetaP = at; at += p.wide ? wide_param_scratch_bytes(Din, Dout) : theta_ws_bytes(Din, Dout);
        if (layout == FLEX_LAYOUT_BCN) { p.featT = at; at += align256(sizeof(float) * (size_t)(B * N) * Din); }
        if (layout == FLEX_LAYOUT_BCN && p.wide) { p.outT = at; at += align256(sizeof(float) * (size_t)(B * N) * Dout); }
    }
    p.total = at > 0 ? at : 256;
    return p;
}

static BwdPlan plan_bwd(int64_t B, int64_t N, int K, int Din, int Dout, int layout, bool build)
{
    BwdPlan p{};
    p.tiled = gather_contract_supported(Din, Dout) && gather_contract_supported(Dout, Din);
    p.wide = ((!p.tiled && wide_shape(Din, Dout)) || wide_route_128(Din, Dout, layout)) &&
             split_wide_ok((int)N, K, Din > Dout ? Din : Dout);
    size_t at = 0;
    if (p.tiled || p.wide) {
        p.thetaP = at; at += p.wide ? wide_param_scratch_bytes(Din, Dout) : theta_ws_bytes(Dout, Din);
        if (layout == FLEX_LAYOUT_BCN) {
            p.featT = at; at += align256(sizeof(float) * (size_t)(B * N) * Din);
            p.gT = at;    at += align256(sizeof(float) * (size_t)(B * N) * Dout);
            if (p.wide) { p.gfT = at; at += align256(sizeof(float) * (size_t)(B * N) * Din); }
        }
        p.partials = at;
        at += p.wide ? wide_partial_bytes((int)B, (int)N, Din, Dout) : grad_theta_partial_bytes(B, N, Din, Dout);
        p.order = at; at += inedges_order_bytes(B * N);      // walking order of the feature gradient's gather
        p.fused = p.tiled && !p.wide && Din == 64 && Dout == 64 && bwd_fused_ok_64_64((int)N, K);
        if (p.fused) { p.flag = at; at += align256(fused_control_bytes()); }   // the one-pass kernel's flag and records
        if (build) {
            p.in_off = at;    at += align256(sizeof(int32_t) * (size_t)(B * N + 1));
            p.in_src = at;    at += align256(sizeof(int32_t) * (size_t)(B * N) * K);
            p.inedge_ws = at; at += inedges_ws_bytes(B * N);
        }
    }
    p.total = at > 0 ? at : 256;
    return p;
}

struct PosPlan {
    bool lean, blocked;
    size_t thetaC, thetaN, featT, gT, thB, in_off, in_src, inedge_ws, total;
};
static inline int pad32(int x) { return (x + 31) / 32 * 32; }
static bool pad_disabled()
{
    static const bool off = [] { const char *v = getenv("FLEX_PAD"); return v != nullptr && v[0] == '0'; }();
    return off;
}

static PosPlan plan_pos(int64_t B, int64_t N, int K, int Din, int Dout, int layout, bool build)
{
    PosPlan p{};
    p.lean = grad_pos_supported(Din, Dout, (int)N, K) && grad_pos_supported(Dout, Din, (int)N, K);
    size_t at = 0;
    if (p.lean) {
        p.thetaC = at; at += theta_pos_bytes(pad32(pad4(Din)), pad16(Dout));
        p.thetaN = at; at += theta_pos_bytes(pad32(pad4(Dout)), pad16(Din));
        if (layout == FLEX_LAYOUT_BCN) {
            p.featT = at; at += align256(sizeof(float) * (size_t)(B * N) * Din);
            p.gT = at;    at += align256(sizeof(float) * (size_t)(B * N) * Dout);
        }
        if (build) {
            p.in_off = at;    at += align256(sizeof(int32_t) * (size_t)(B * N + 1));
            p.in_src = at;    at += align256(sizeof(int32_t) * (size_t)(B * N) * K);
            p.inedge_ws = at; at += inedges_ws_bytes(B * N);
        }
    } else if (!pad_disabled() && grad_pos_supported(64, 64, (int)N, K)) {
        // other widths: the sum over 64 x 64 blocks of the parameters of the 64 -> 64 kernel's result on zero-padded
        // point-major 64-channel column blocks of the two tensors (featT / gT hold those blocks, one after the other)
        p.blocked = true;
        const int n_hi = (Din + 63) / 64, n_ho = (Dout + 63) / 64;
        p.thetaC = at; at += theta_pos_bytes(64, 64);
        p.thetaN = at; at += theta_pos_bytes(64, 64);
        p.thB = at;    at += align256(sizeof(float) * 3 * 64 * 64);
        p.featT = at;  at += align256(sizeof(float) * (size_t)(B * N) * 64) * n_hi;
        p.gT = at;     at += align256(sizeof(float) * (size_t)(B * N) * 64) * n_ho;
        if (build) {
            p.in_off = at;    at += align256(sizeof(int32_t) * (size_t)(B * N + 1));
            p.in_src = at;    at += align256(sizeof(int32_t) * (size_t)(B * N) * K);
            p.inedge_ws = at; at += inedges_ws_bytes(B * N);
        }
    }
    p.total = at > 0 ? at : 256;
    return p;
}

// Widths with neither a tiled nor a wide path run on zero-padded copies at the nearest widths that have one
// (FLEX_PAD=0 in the environment keeps them on the direct-form kernels, for comparisons): extra channels of the
// features / upstream gradient and extra rows / columns of the parameters are zero, so they add nothing, and the
// results are the leading channels / the leading block of what the padded layer returns.
static bool padded_shape(int Din, int Dout, int *DIp, int *DOp)
{
    if (pad_disabled() || wide_shape(Din, Dout)) return false;
    if (gather_contract_supported(Din, Dout) && gather_contract_supported(Dout, Din)) return false;
    if (Din <= 128 && Dout <= 128) {
        int64_t best = -1;
#define FLEX_SHAPE(DI_, DO_, W, T, OCC, WS)                                                         \
        if (DI_ >= Din && DO_ >= Dout && gather_contract_supported(DO_, DI_) &&                         \
            (best < 0 || (int64_t)DI_ * DO_ < best)) {                                                  \
            best = (int64_t)DI_ * DO_; *DIp = DI_; *DOp = DO_;                                          \
        }
#include "flex_shapes.def"
#undef FLEX_SHAPE
        return best > 0;
    }
    *DIp = (Din + 127) / 128 * 128;
    *DOp = (Dout + 127) / 128 * 128;
    return wide_shape(*DIp, *DOp);
}

static FwdPlan plan_fwd(int64_t B, int64_t N, int K, int Din, int Dout, int layout);
static BwdPlan plan_bwd(int64_t B, int64_t N, int K, int Din, int Dout, int layout, bool build);

struct PadPlan {
    size_t featP, gP, thetaP, outP, gfP, gtP, sub, sub_bytes, total;   // thetaP / gtP: [3,DIp,DOp] then [DIp,DOp]
};
static PadPlan plan_pad(int64_t B, int64_t N, int K, int DIp, int DOp, bool bwd, bool build)
{
    PadPlan p{};
    size_t at = 0;
    const size_t rows_in = align256(sizeof(float) * (size_t)(B * N) * DIp);
    const size_t rows_out = align256(sizeof(float) * (size_t)(B * N) * DOp);
    const size_t params = align256(sizeof(float) * (size_t)4 * DIp * DOp);
    p.featP = at; at += rows_in;
    p.thetaP = at; at += params;
    if (!bwd) { p.outP = at; at += rows_out; }
    else {
        p.gP = at;  at += rows_out;
        p.gfP = at; at += rows_in;
        p.gtP = at; at += params;
    }
    p.sub = at;
    p.sub_bytes = bwd ? plan_bwd(B, N, K, DIp, DOp, FLEX_LAYOUT_BNC, build).total
                      : plan_fwd(B, N, K, DIp, DOp, FLEX_LAYOUT_BNC).total;
    p.total = at + p.sub_bytes;
    return p;
}

static bool sizes_ok(int64_t B, int64_t N, int64_t K, int64_t Din, int64_t Dout)
{
    if (B <= 0 || N <= 0 || K <= 0 || Din <= 0 || Dout <= 0) return false;
    if (K > N) return false;
    if (B * N >= 0x7fffffffLL) return false;          // global point ids are int32
    if (B * N * K >= 0x7fffffffLL) return false;      // in-edge offsets are int32
    if (Din > 16384 || Dout > 16384) return false;
    return true;
}

// the draw's integer scale needs N <= 2^25 per cloud; one grid row per cloud
static bool idiss_sizes_ok(int64_t B, int64_t N)
{
    return sizes_ok(B, N, 1, 1, 1) && N <= (1 << 25) && B <= 65535;
}

// cell offsets are int32 over all clouds' cells; one grid row per cloud
static bool knn_sizes_ok(int64_t B, int64_t N, int64_t K)
{
    if (!sizes_ok(B, N, K, 1, 1) || B > 65535 || !knn_k_supported((int)K)) return false;
    const int64_t per_cloud = 8 * N < (1ll << 24) ? 8 * N : (1ll << 24);
    return B * per_cloud < 0x7fffffffLL;
}

static bool ws_ok(const void *ws, size_t have, size_t need)
{
    return ws != nullptr && (((uintptr_t)ws) & 255) == 0 && have >= need;
}

#define FLEX_HIP(expr)                                  \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return FLEX_ERR_HIP;      \
    } while (0)

}  // namespace flex

using namespace flex;

extern "C" {

const char *flex_status_string(int status)
{
    switch (status) {
    case FLEX_OK: return "ok";
    case FLEX_ERR_NULL: return "null pointer argument";
    case FLEX_ERR_SHAPE: return "bad size, layout or op";
    case FLEX_ERR_UNSUPPORTED: return "unsupported";
    case FLEX_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FLEX_ERR_HIP: return "HIP launch error";
    case FLEX_ERR_TOO_LARGE: return "call needs more scratch memory than the library's static buffer holds";
    default: return "unknown status";
    }
}

int flexconv_has_fast_path(int Din, int Dout)
{
    int a, b;
    if (gather_contract_supported(Din, Dout) || wide_shape(Din, Dout)) return 1;
    return padded_shape(Din, Dout, &a, &b) ? 2 : 0;
}

int flexconv_kernel_route(int op, int B, int N, int K, int Din, int Dout, int layout)
{
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return -1;
    if (op != FLEX_OP_CONV_FWD && op != FLEX_OP_CONV_BWD) return -1;
    if (!sizes_ok(B, N, K, Din, Dout)) return -1;
    int DIp, DOp;
    if (padded_shape(Din, Dout, &DIp, &DOp)) return FLEX_ROUTE_PADDED;
    if (op == FLEX_OP_CONV_FWD) {
        const FwdPlan p = plan_fwd(B, N, K, Din, Dout, layout);
        if (p.wide) return FLEX_ROUTE_WIDE;
        if (!p.tiled) return FLEX_ROUTE_DIRECT;
        if (use_split_128(Din, Dout, layout, N, K, 0)) return FLEX_ROUTE_SPLIT128;
        return gather_contract_route(Din, Dout, N, K, 0);
    }
    const BwdPlan p = plan_bwd(B, N, K, Din, Dout, layout, false);
    if (p.wide) return FLEX_ROUTE_WIDE;
    if (!p.tiled) return FLEX_ROUTE_DIRECT;
    if (use_split_128(Din, Dout, layout, N, K, 1)) return FLEX_ROUTE_SPLIT128;
    if (p.fused) return FLEX_ROUTE_LEAN_FUSED;
    return gather_contract_route(Dout, Din, N, K, 1);
}

size_t flexconv_workspace_bytes(int op, int B, int N, int K, int Din, int Dout, int layout)
{
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return 0;
    switch (op) {
    case FLEX_OP_CONV_FWD:
    case FLEX_OP_CONV_BWD:
    case FLEX_OP_CONV_BWD_BUILD: {
        if (!sizes_ok(B, N, K, Din, Dout)) return 0;
        int DIp, DOp;
        if (padded_shape(Din, Dout, &DIp, &DOp))
            return plan_pad(B, N, K, DIp, DOp, op != FLEX_OP_CONV_FWD, op == FLEX_OP_CONV_BWD_BUILD).total;
        if (op == FLEX_OP_CONV_FWD) return plan_fwd(B, N, K, Din, Dout, layout).total;
        return plan_bwd(B, N, K, Din, Dout, layout, op == FLEX_OP_CONV_BWD_BUILD).total;
    }
    case FLEX_OP_INEDGES: return sizes_ok(B, N, K, 1, 1) ? inedges_ws_bytes((int64_t)B * N) : 0;
    case FLEX_OP_CONV_BWD_POS: return sizes_ok(B, N, K, Din, Dout) ? plan_pos(B, N, K, Din, Dout, layout, false).total : 0;
    case FLEX_OP_CONV_BWD_POS_BUILD: return sizes_ok(B, N, K, Din, Dout) ? plan_pos(B, N, K, Din, Dout, layout, true).total : 0;
    case FLEX_OP_UPSAMPLE: return sizes_ok(B, N, 1, 1, 1) ? align256(sizeof(int32_t) * (size_t)B * N) : 0;
    case FLEX_OP_IDISS: return idiss_sizes_ok(B, N) ? idiss_ws_bytes(B, N) : 0;
    case FLEX_OP_KNN: return knn_sizes_ok(B, N, K) ? knn_ws_bytes(B, N) : 0;
    default: return 0;
    }
}

int flexconv_fwd(const float *feat, const float *pos, const int32_t *nbr, const float *theta,
                 const float *bias, float *out, int B, int N, int K, int Din, int Dout, int layout,
                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!feat || !pos || !nbr || !theta || !bias || !out) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, Din, Dout)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int bcn = (layout == FLEX_LAYOUT_BCN);
    int DIp, DOp;
    if (padded_shape(Din, Dout, &DIp, &DOp)) {
        const PadPlan pp = plan_pad(B, N, K, DIp, DOp, false, false);
        if (!ws_ok(workspace, workspace_bytes, pp.total)) return FLEX_ERR_WORKSPACE;
        float *featP = (float *)(ws + pp.featP), *thetaP = (float *)(ws + pp.thetaP), *biasP = thetaP + 3 * DIp * DOp;
        float *outP = (float *)(ws + pp.outP);
        FLEX_HIP(launch_copy_rows(feat, featP, B, N, Din, DIp, bcn, 0, s));
        FLEX_HIP(launch_fill_zero(thetaP, sizeof(float) * (size_t)4 * DIp * DOp, s));
        FLEX_HIP(launch_param_block(thetaP, biasP, (float *)theta, (float *)bias, DIp, DOp, 0, 0, Din, Dout, 1, s));
        const int st = flexconv_fwd(featP, pos, nbr, thetaP, biasP, outP, B, N, K, DIp, DOp, FLEX_LAYOUT_BNC,
                                    ws + pp.sub, pp.sub_bytes, stream);
        if (st != FLEX_OK) return st;
        FLEX_HIP(launch_copy_rows(outP, out, B, N, DOp, Dout, 0, bcn, s));
        return FLEX_OK;
    }
    const FwdPlan p = plan_fwd(B, N, K, Din, Dout, layout);
    if (!ws_ok(workspace, workspace_bytes, p.total)) return FLEX_ERR_WORKSPACE;
    if (p.wide) {
        const float *rows = feat;
        float *dst = out;
        if (bcn) {
            FLEX_HIP(launch_bcn_to_bnc(feat, (float *)(ws + p.featT), B, Din, N, s));
            rows = (float *)(ws + p.featT);
            dst = (float *)(ws + p.outT);
        }
        FLEX_HIP(wide_gather_contract(rows, pos, nbr, nullptr, nullptr, nullptr, theta, bias, ws + p.thetaP, dst, B, N, K,
                                      Din, Dout, 0, s));
        if (bcn) FLEX_HIP(launch_bnc_to_bcn(dst, out, B, Dout, N, s));
        return FLEX_OK;
    }
    if (!p.tiled) {
        FLEX_HIP(launch_generic_fwd(feat, pos, nbr, theta, bias, out, B, N, K, Din, Dout, !bcn, s));
        return FLEX_OK;
    }
    void *thetaP = ws + p.thetaP;
    if (use_split_128(Din, Dout, layout, N, K, 0)) {
        FLEX_HIP(split_gather_contract_128(feat, pos, nbr, nullptr, nullptr, nullptr, theta, bias, thetaP, out, B, N, K, 0,
                                           s));
        return FLEX_OK;
    }
    const int fmt = gather_contract_theta_format(Din, Dout, N, K, 0);
    FLEX_HIP(pack_for_contract(theta, bias, thetaP, Din, Dout, 0, fmt, s));
    const float *rows = feat;
    if (bcn) {
        float *featT = (float *)(ws + p.featT);
        FLEX_HIP(launch_bcn_to_bnc(feat, featT, B, Din, N, s));
        rows = featT;
    }
    FLEX_HIP(launch_gather_contract(rows, pos, nbr, nullptr, nullptr, nullptr, thetaP, fmt, out, B, N, K, Din,
                                    Dout, 0, bcn, s));
    return FLEX_OK;
}

}  // extern "C"

// ---- flexconv_fwd_noalloc: the forward pass with the library's own static scratch memory -------------------
// The scratch (packed parameters; for other layouts / widths also the copies the plan asks for) lives in a
// file-scope device array instead of a caller workspace.  In host code the array's name is only a handle: the
// device address is looked up once per device (with that device current) and kept; every later use goes through
// the kept pointer.  Each GPU holds its own copy of the array at its own address.
static __device__ __align__(256) unsigned char scratch[FLEX_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];       // device address of `scratch` on each device, nullptr until looked up
std::mutex g_scratch_mutex;

int static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return FLEX_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FLEX_ERR_HIP;
        if ((reinterpret_cast<uintptr_t>(p) & 255) != 0) return FLEX_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return FLEX_OK;
}
}  // namespace

extern "C" {

int flexconv_fwd_noalloc(const float *feat, const float *pos, const int32_t *nbr, const float *theta,
                         const float *bias, float *out, int B, int N, int K, int Din, int Dout, int layout,
                         void *stream)
{
    if (!feat || !pos || !nbr || !theta || !bias || !out) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, Din, Dout)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    const size_t need = flexconv_workspace_bytes(FLEX_OP_CONV_FWD, B, N, K, Din, Dout, layout);
    if (need == 0) return FLEX_ERR_SHAPE;
    if (need > (size_t)FLEX_NOALLOC_SCRATCH_BYTES) return FLEX_ERR_TOO_LARGE;
    void *ws = nullptr;
    const int st = static_scratch(&ws);
    if (st != FLEX_OK) return st;
    // Every byte of the plan that a kernel reads is written earlier in the same call (packed parameters with their
    // padding, exponent tables, padded copies after an explicit zero fill), so nothing has to be cleared here.
    return flexconv_fwd(feat, pos, nbr, theta, bias, out, B, N, K, Din, Dout, layout, ws, need, stream);
}

int flex_inedges_build(const int32_t *nbr, int B, int N, int K, int32_t *in_off, int32_t *in_src,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (!nbr || !in_off || !in_src) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, 1, 1)) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, inedges_ws_bytes((int64_t)B * N))) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_inedges_build(nbr, B, N, K, in_off, in_src, workspace, (hipStream_t)stream));
    return FLEX_OK;
}

int flexconv_bwd(const float *feat, const float *pos, const int32_t *nbr, const float *theta,
                 const float *bias, const float *grad_out, float *grad_feat, float *grad_theta,
                 float *grad_bias, const int32_t *in_off, const int32_t *in_src, int B, int N, int K,
                 int Din, int Dout, int layout, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!feat || !pos || !nbr || !theta || !bias || !grad_out) return FLEX_ERR_NULL;
    if ((grad_theta == nullptr) != (grad_bias == nullptr)) return FLEX_ERR_NULL;
    if ((in_off == nullptr) != (in_src == nullptr)) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, Din, Dout)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    const bool build = (in_off == nullptr) && (grad_feat != nullptr);
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int bcn = (layout == FLEX_LAYOUT_BCN);
    int DIp, DOp;
    if (padded_shape(Din, Dout, &DIp, &DOp)) {
        const PadPlan pp = plan_pad(B, N, K, DIp, DOp, true, build);
        if (!ws_ok(workspace, workspace_bytes, pp.total)) return FLEX_ERR_WORKSPACE;
        float *featP = (float *)(ws + pp.featP), *gP = (float *)(ws + pp.gP), *gfP = (float *)(ws + pp.gfP);
        float *thetaP = (float *)(ws + pp.thetaP), *biasP = thetaP + 3 * DIp * DOp;
        float *gtP = (float *)(ws + pp.gtP), *gbP = gtP + 3 * DIp * DOp;
        FLEX_HIP(launch_copy_rows(feat, featP, B, N, Din, DIp, bcn, 0, s));
        FLEX_HIP(launch_copy_rows(grad_out, gP, B, N, Dout, DOp, bcn, 0, s));
        FLEX_HIP(launch_fill_zero(thetaP, sizeof(float) * (size_t)4 * DIp * DOp, s));
        FLEX_HIP(launch_param_block(thetaP, biasP, (float *)theta, (float *)bias, DIp, DOp, 0, 0, Din, Dout, 1, s));
        const int st = flexconv_bwd(featP, pos, nbr, thetaP, biasP, gP, grad_feat ? gfP : nullptr,
                                    grad_theta ? gtP : nullptr, grad_theta ? gbP : nullptr, in_off, in_src, B, N, K,
                                    DIp, DOp, FLEX_LAYOUT_BNC, ws + pp.sub, pp.sub_bytes, stream);
        if (st != FLEX_OK) return st;
        if (grad_feat) FLEX_HIP(launch_copy_rows(gfP, grad_feat, B, N, DIp, Din, 0, bcn, s));
        if (grad_theta) FLEX_HIP(launch_param_block(gtP, gbP, grad_theta, grad_bias, DIp, DOp, 0, 0, Din, Dout, 0, s));
        return FLEX_OK;
    }
    const BwdPlan p = plan_bwd(B, N, K, Din, Dout, layout, build);
    if (!ws_ok(workspace, workspace_bytes, p.total)) return FLEX_ERR_WORKSPACE;
    if (p.wide) {
        const float *rows = feat, *g_rows = grad_out;
        if (bcn) {
            FLEX_HIP(launch_bcn_to_bnc(grad_out, (float *)(ws + p.gT), B, Dout, N, s));
            g_rows = (float *)(ws + p.gT);
            if (grad_theta) {
                FLEX_HIP(launch_bcn_to_bnc(feat, (float *)(ws + p.featT), B, Din, N, s));
                rows = (float *)(ws + p.featT);
            }
        }
        if (grad_theta)
            FLEX_HIP(wide_grad_theta(rows, pos, nbr, g_rows, (float *)(ws + p.partials), grad_theta, grad_bias, B, N,
                                     K, Din, Dout, s));
        if (grad_feat) {
            if (build) {
                int32_t *off = (int32_t *)(ws + p.in_off), *src = (int32_t *)(ws + p.in_src);
                FLEX_HIP(launch_inedges_build(nbr, B, N, K, off, src, ws + p.inedge_ws, s));
                in_off = off;
                in_src = src;
            }
            float *dst = bcn ? (float *)(ws + p.gfT) : grad_feat;
            int32_t *order = (int32_t *)(ws + p.order);
            FLEX_HIP(launch_inedges_order(in_off, B, N, order, s));
            FLEX_HIP(wide_gather_contract(g_rows, pos, nullptr, in_off, in_src, order, theta, bias, ws + p.thetaP, dst,
                                          B, N, K, Din, Dout, 1, s));
            if (bcn) FLEX_HIP(launch_bnc_to_bcn(dst, grad_feat, B, Din, N, s));
        }
        return FLEX_OK;
    }
    if (!p.tiled) {
        FLEX_HIP(launch_generic_bwd(feat, pos, nbr, theta, bias, grad_out, grad_feat, grad_theta,
                                    grad_bias, B, N, K, Din, Dout, !bcn, s));
        return FLEX_OK;
    }
    const float *rows = feat, *g_rows = grad_out;
    if (bcn) {
        float *gT = (float *)(ws + p.gT);
        FLEX_HIP(launch_bcn_to_bnc(grad_out, gT, B, Dout, N, s));
        g_rows = gT;
        if (grad_theta) {
            float *featT = (float *)(ws + p.featT);
            FLEX_HIP(launch_bcn_to_bnc(feat, featT, B, Din, N, s));
            rows = featT;
        }
    }
    if (p.fused && grad_theta && grad_feat) {
        if (build) {
            int32_t *off = (int32_t *)(ws + p.in_off), *src = (int32_t *)(ws + p.in_src);
            FLEX_HIP(launch_inedges_build(nbr, B, N, K, off, src, ws + p.inedge_ws, s));
            in_off = off;
            in_src = src;
        }
        void *thetaP = ws + p.thetaP;
        int32_t *order = (int32_t *)(ws + p.order);
        int *flag = (int *)(ws + p.flag);
        float *partials = (float *)(ws + p.partials);
        FLEX_HIP(launch_inedges_order(in_off, B, N, order, s));
        FLEX_HIP(launch_fill_zero(flag, sizeof(int) * FUSED_FLAG_INTS, s));
        FLEX_HIP(pack_for_contract(theta, bias, thetaP, Din, Dout, 1, 1, s));
        int n_wg = 0;
        FLEX_HIP(launch_bwd_fused_64_64(g_rows, rows, pos, nbr, in_off, in_src, order, thetaP, grad_feat, partials,
                                        flag, B, N, K, bcn, &n_wg, s));
        FLEX_HIP(launch_reduce_partials(partials, n_wg, pad4(Din), pad16(Dout), Din, Dout, grad_theta, grad_bias, s));
        // is the result resolved by the f16 halves?  if not (decided on the device), the stand-alone kernel and a
        // second reduction run; both return at once otherwise
        const float *rscale = reinterpret_cast<const float *>(reinterpret_cast<const char *>(thetaP) +
                                                              theta_f16_rscale_offset(pad4(Dout), pad16(Din)));
        FLEX_HIP(launch_fused_bwd_check(flag, n_wg, rscale, grad_theta, grad_bias, s));
        FLEX_HIP(launch_bwd_fused_late_64_64(g_rows, rows, pos, nbr, partials, flag, B, N, K, s));
        FLEX_HIP(launch_reduce_partials_if(flag, FUSED_UNRESOLVED, partials, n_wg, pad4(Din), pad16(Dout), Din, Dout,
                                           grad_theta, grad_bias, s));
        return FLEX_OK;
    }
    if (grad_theta) {
        if (use_split_128(Din, Dout, layout, N, K, 0))
            FLEX_HIP(split_grad_theta_128(rows, pos, nbr, g_rows, (float *)(ws + p.partials), ws + p.thetaP,
                                          grad_theta, grad_bias, B, N, K, s));
        else
            FLEX_HIP(launch_grad_theta(rows, pos, nbr, g_rows, (float *)(ws + p.partials), grad_theta,
                                       grad_bias, B, N, K, Din, Dout, s));
    }
    if (grad_feat) {
        if (build) {
            int32_t *off = (int32_t *)(ws + p.in_off), *src = (int32_t *)(ws + p.in_src);
            FLEX_HIP(launch_inedges_build(nbr, B, N, K, off, src, ws + p.inedge_ws, s));
            in_off = off;
            in_src = src;
        }
        void *thetaP = ws + p.thetaP;
        int32_t *order = (int32_t *)(ws + p.order);
        FLEX_HIP(launch_inedges_order(in_off, B, N, order, s));
        if (use_split_128(Din, Dout, layout, N, K, 1)) {
            FLEX_HIP(split_gather_contract_128(g_rows, pos, nullptr, in_off, in_src, order, theta, bias, thetaP,
                                               grad_feat, B, N, K, 1, s));
            return FLEX_OK;
        }
        const int fmt = gather_contract_theta_format(Dout, Din, N, K, 1);
        FLEX_HIP(pack_for_contract(theta, bias, thetaP, Din, Dout, 1, fmt, s));
        FLEX_HIP(launch_gather_contract(g_rows, pos, nullptr, in_off, in_src, order, thetaP, fmt, grad_feat, B, N,
                                        K, Dout, Din, 1, bcn, s));
    }
    return FLEX_OK;
}

int flexpool_fwd(const float *feat, const int32_t *nbr, float *out, int32_t *argmax, int B, int N,
                 int K, int C, int layout, void *stream)
{
    if (!feat || !nbr || !out || !argmax) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, C, 1)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_pool_fwd(feat, nbr, out, argmax, B, N, K, C, layout == FLEX_LAYOUT_BNC,
                             (hipStream_t)stream));
    return FLEX_OK;
}

int flexpool_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat,
                 const int32_t *in_off, const int32_t *in_src, int B, int N, int K, int C, int layout,
                 void *stream)
{
    if (!grad_out || !argmax || !grad_feat) return FLEX_ERR_NULL;
    if ((in_off == nullptr) != (in_src == nullptr)) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, in_off ? K : 1, C, 1)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    if (in_off)
        FLEX_HIP(launch_pool_bwd_gather(grad_out, argmax, in_off, in_src, grad_feat, B, N, C,
                                        layout == FLEX_LAYOUT_BNC, (hipStream_t)stream));
    else
        FLEX_HIP(launch_pool_bwd(grad_out, argmax, grad_feat, B, N, C, layout == FLEX_LAYOUT_BNC,
                                 (hipStream_t)stream));
    return FLEX_OK;
}

// FLEX_POOL_PLAN=1: the planned kernels wherever they can run (any size, any K); =0: never; unset: where they are faster
static int pool_plan_mode()
{
    static const int mode = [] { const char *e = getenv("FLEX_POOL_PLAN"); return !e ? -1 : e[0] == '0' ? 0 : 1; }();
    return mode;
}

size_t flexpool_plan_bytes(int B, int N, int K)
{
    if (!sizes_ok(B, N, K, 1, 1)) return 0;
    return pool_plan_bytes(B, N, K);
}

int flexpool_plan_build(const int32_t *in_off, const int32_t *in_src, int B, int N, int K, void *plan,
                        size_t plan_bytes, void *stream)
{
    if (!in_off || !in_src || !plan) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, 1, 1)) return FLEX_ERR_SHAPE;
    if (plan_bytes < pool_plan_bytes(B, N, K) || (reinterpret_cast<uintptr_t>(plan) & 255)) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_pool_plan_build(in_off, in_src, plan, B, N, K, (hipStream_t)stream));
    return FLEX_OK;
}

int flexpool_bwd_planned(const float *grad_out, const int32_t *argmax, float *grad_feat, const int32_t *in_off,
                         const int32_t *in_src, void *plan, size_t plan_bytes, int B, int N, int K, int C,
                         int layout, void *stream)
{
    if (!grad_out || !argmax || !grad_feat || !in_off || !in_src || !plan) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, C, 1)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    if (plan_bytes < pool_plan_bytes(B, N, K) || (reinterpret_cast<uintptr_t>(plan) & 255)) return FLEX_ERR_WORKSPACE;
    const int mode = pool_plan_mode();
    const bool can = layout == FLEX_LAYOUT_BNC && (C == 64 || C == 128 || C == 256);
    const bool pays = K <= FLEX_POOL_PLAN_MAX_K && (int64_t)B * N >= FLEX_POOL_PLAN_MIN_POINTS;
    if (can && (mode == 1 || (mode == -1 && pays)))
        FLEX_HIP(launch_pool_bwd_planned(grad_out, argmax, in_off, in_src, plan, grad_feat, B, N, K, C,
                                         (hipStream_t)stream));
    else        // widths and layouts the plan has no kernel for, sizes and list lengths it does not pay for: the list form, same sums
        FLEX_HIP(launch_pool_bwd_gather(grad_out, argmax, in_off, in_src, grad_feat, B, N, C,
                                        layout == FLEX_LAYOUT_BNC, (hipStream_t)stream));
    return FLEX_OK;
}

int flexpool_fwd_plan_build(const int32_t *nbr, int B, int N, int K, void *plan, size_t plan_bytes, void *stream)
{
    if (!nbr || !plan) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, 1, 1)) return FLEX_ERR_SHAPE;
    if (plan_bytes < pool_plan_bytes(B, N, K) || (reinterpret_cast<uintptr_t>(plan) & 255)) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_pool_fwd_plan_build(nbr, plan, B, N, K, (hipStream_t)stream));
    return FLEX_OK;
}

int flexpool_fwd_planned(const float *feat, const int32_t *nbr, float *out, int32_t *argmax, void *plan,
                         size_t plan_bytes, int B, int N, int K, int C, int layout, void *stream)
{
    if (!feat || !nbr || !out || !argmax || !plan) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, C, 1)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    if (plan_bytes < pool_plan_bytes(B, N, K) || (reinterpret_cast<uintptr_t>(plan) & 255)) return FLEX_ERR_WORKSPACE;
    const int mode = pool_plan_mode();
    const bool can = layout == FLEX_LAYOUT_BNC && (C == 64 || C == 128 || C == 256);
    const bool pays = K <= FLEX_POOL_PLAN_MAX_K && (int64_t)B * N >= FLEX_POOL_PLAN_MIN_POINTS;
    if (can && (mode == 1 || (mode == -1 && pays)))
        FLEX_HIP(launch_pool_fwd_planned(feat, nbr, plan, out, argmax, B, N, K, C, (hipStream_t)stream));
    else
        FLEX_HIP(launch_pool_fwd(feat, nbr, out, argmax, B, N, K, C, layout == FLEX_LAYOUT_BNC, (hipStream_t)stream));
    return FLEX_OK;
}

int flexconv_compose_1x1(const float *W, const float *theta, const float *bias, float *theta_c, float *bias_c,
                         int Din0, int Dmid, int Dout, void *stream)
{
    if (!W || !theta || !bias || !theta_c || !bias_c) return FLEX_ERR_NULL;
    if (Din0 <= 0 || Dmid <= 0 || Dout <= 0 || Din0 > 16384 || Dmid > 16384 ||
        Dout > 16384)
        return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_compose_1x1(W, theta, bias, theta_c, bias_c, Din0, Dmid, Dout, (hipStream_t)stream));
    return FLEX_OK;
}

int flexconv_compose_1x1_bwd(const float *W, const float *theta, const float *bias, const float *grad_theta_c,
                             const float *grad_bias_c, float *grad_W, float *grad_theta, float *grad_bias,
                             int Din0, int Dmid, int Dout, void *stream)
{
    if (!W || !theta || !bias || !grad_theta_c || !grad_bias_c || !grad_W || !grad_theta || !grad_bias)
        return FLEX_ERR_NULL;
    if (Din0 <= 0 || Dmid <= 0 || Dout <= 0 || Din0 > 16384 || Dmid > 16384 ||
        Dout > 16384)
        return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_compose_1x1_bwd(W, theta, bias, grad_theta_c, grad_bias_c, grad_W, grad_theta, grad_bias, Din0,
                                    Dmid, Dout, (hipStream_t)stream));
    return FLEX_OK;
}

int flex_idiss_phi(const float *pos, const int32_t *nbr, float *phi, int B, int N, int K, void *stream)
{
    if (!pos || !nbr || !phi) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, 1, 1)) return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_idiss_phi(pos, nbr, phi, B, N, K, (hipStream_t)stream));
    return FLEX_OK;
}

int flex_idiss_sample(const float *phi, const uint32_t *u, int32_t *sel, int B, int N, int Ns,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (!phi || !u || !sel) return FLEX_ERR_NULL;
    if (!idiss_sizes_ok(B, N) || Ns <= 0 || Ns > N) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, idiss_ws_bytes(B, N))) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_idiss_sample(phi, u, sel, B, N, Ns, workspace, (hipStream_t)stream));
    return FLEX_OK;
}

int flex_selection_make_distinct(int32_t *sel, int B, int N, int Ns, void *workspace, size_t workspace_bytes,
                                 void *stream)
{
    if (!sel) return FLEX_ERR_NULL;
    if (!idiss_sizes_ok(B, N) || Ns <= 0 || Ns > N) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, distinct_ws_bytes(B, Ns))) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_selection_make_distinct(sel, B, N, Ns, workspace, (hipStream_t)stream));
    return FLEX_OK;
}

int flex_knn(const float *pos, int32_t *nbr, int B, int N, int K, void *workspace, size_t workspace_bytes,
             void *stream)
{
    if (!pos || !nbr) return FLEX_ERR_NULL;
    if (!knn_sizes_ok(B, N, K)) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, knn_ws_bytes(B, N))) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_knn(pos, nbr, B, N, K, workspace, (hipStream_t)stream));
    return FLEX_OK;
}

int flexpool_sub_fwd(const float *feat, const int32_t *nbr, const int32_t *sel, float *out,
                     int32_t *argmax, int B, int N, int Ns, int K, int C, int layout, void *stream)
{
    if (!feat || !nbr || !sel || !out || !argmax) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, C, 1) || Ns <= 0 || Ns > N) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_pool_sub_fwd(feat, nbr, sel, out, argmax, B, N, Ns, K, C, layout == FLEX_LAYOUT_BNC,
                                 (hipStream_t)stream));
    return FLEX_OK;
}

int flexpool_sub_bwd(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                     const int32_t *in_src, float *grad_feat, int B, int N, int Ns, int K, int C,
                     int layout, void *stream)
{
    if (!grad_out || !argmax || !grad_feat) return FLEX_ERR_NULL;
    if ((in_off == nullptr) != (in_src == nullptr)) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, in_off ? K : 1, C, 1) || Ns <= 0 || Ns > N) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    const int bnc = layout == FLEX_LAYOUT_BNC;
    if (in_off)
        FLEX_HIP(launch_pool_sub_bwd_gather(grad_out, argmax, in_off, in_src, grad_feat, B, N, Ns, C, bnc, s));
    else
        FLEX_HIP(launch_pool_sub_bwd(grad_out, argmax, grad_feat, B, N, Ns, C, bnc, s));
    return FLEX_OK;
}

int flex_inedges_build_sub(const int32_t *nbr, const int32_t *sel, int B, int N, int Ns, int K,
                           int32_t *in_off, int32_t *in_src, void *workspace, size_t workspace_bytes,
                           void *stream)
{
    if (!nbr || !sel || !in_off || !in_src) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, 1, 1) || Ns <= 0 || Ns > N) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, inedges_ws_bytes((int64_t)B * N))) return FLEX_ERR_WORKSPACE;
    FLEX_HIP(launch_inedges_build_sub(nbr, sel, B, N, Ns, K, in_off, in_src, workspace, (hipStream_t)stream));
    return FLEX_OK;
}

int flexconv_bwd_pos(const float *feat, const int32_t *nbr, const float *theta, const float *grad_out,
                     const int32_t *in_off, const int32_t *in_src, float *grad_pos, int B, int N, int K,
                     int Din, int Dout, int layout, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!feat || !nbr || !theta || !grad_out || !grad_pos) return FLEX_ERR_NULL;
    if ((in_off == nullptr) != (in_src == nullptr)) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, Din, Dout)) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    const bool build = in_off == nullptr;
    const PosPlan p = plan_pos(B, N, K, Din, Dout, layout, build);
    if (!ws_ok(workspace, workspace_bytes, p.total)) return FLEX_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int bcn = (layout == FLEX_LAYOUT_BCN);
    if (p.blocked) {
        const int n_hi = (Din + 63) / 64, n_ho = (Dout + 63) / 64;
        const size_t blk_bytes = align256(sizeof(float) * (size_t)B * N * 64);
        for (int hi = 0; hi < n_hi; ++hi)
            FLEX_HIP(launch_copy_rows(feat, (float *)(ws + p.featT + hi * blk_bytes), B, N, Din, 64, bcn, 0, s, 64 * hi));
        for (int ho = 0; ho < n_ho; ++ho)
            FLEX_HIP(launch_copy_rows(grad_out, (float *)(ws + p.gT + ho * blk_bytes), B, N, Dout, 64, bcn, 0, s, 64 * ho));
        if (build) {
            int32_t *off = (int32_t *)(ws + p.in_off), *src = (int32_t *)(ws + p.in_src);
            FLEX_HIP(launch_inedges_build(nbr, B, N, K, off, src, ws + p.inedge_ws, s));
            in_off = off;
            in_src = src;
        }
        void *thC = ws + p.thetaC, *thN = ws + p.thetaN;
        float *thB = (float *)(ws + p.thB);
        for (int hi = 0; hi < n_hi; ++hi)
            for (int ho = 0; ho < n_ho; ++ho) {
                const float *f_blk = (const float *)(ws + p.featT + hi * blk_bytes);
                const float *g_blk = (const float *)(ws + p.gT + ho * blk_bytes);
                FLEX_HIP(launch_theta_block_padded(theta, thB, Din, Dout, 64 * hi, 64 * ho, 64, 64, s));
                FLEX_HIP(launch_pack_theta_pos(thB, thC, 64, 64, 64, 64, 0, s));
                FLEX_HIP(launch_pack_theta_pos(thB, thN, 64, 64, 64, 64, 1, s));
                FLEX_HIP(launch_grad_pos_term(f_blk, nbr, nullptr, nullptr, thC, g_blk, grad_pos, -1.f,
                                              (hi | ho) != 0, B, N, K, 64, 64, 0, s));
                FLEX_HIP(launch_grad_pos_term(g_blk, nullptr, in_off, in_src, thN, f_blk, grad_pos, 1.f, 1, B, N, K, 64,
                                              64, 1, s));
            }
        return FLEX_OK;
    }
    if (!p.lean) {
        FLEX_HIP(launch_generic_bwd_pos(feat, nbr, theta, grad_out, grad_pos, B, N, K, Din, Dout, !bcn, s));
        return FLEX_OK;
    }
    const float *rows = feat, *g_rows = grad_out;
    if (bcn) {
        FLEX_HIP(launch_bcn_to_bnc(feat, (float *)(ws + p.featT), B, Din, N, s));
        FLEX_HIP(launch_bcn_to_bnc(grad_out, (float *)(ws + p.gT), B, Dout, N, s));
        rows = (const float *)(ws + p.featT);
        g_rows = (const float *)(ws + p.gT);
    }
    if (build) {
        int32_t *off = (int32_t *)(ws + p.in_off), *src = (int32_t *)(ws + p.in_src);
        FLEX_HIP(launch_inedges_build(nbr, B, N, K, off, src, ws + p.inedge_ws, s));
        in_off = off;
        in_src = src;
    }
    void *thC = ws + p.thetaC, *thN = ws + p.thetaN;
    FLEX_HIP(launch_pack_theta_pos(theta, thC, Din, Dout, pad32(pad4(Din)), pad16(Dout), 0, s));
    FLEX_HIP(launch_pack_theta_pos(theta, thN, Din, Dout, pad32(pad4(Dout)), pad16(Din), 1, s));
    // centre term: -<(sum_k feat[n_k(x)])^T theta_d, grad_out[x]>, then neighbour term added on top
    FLEX_HIP(launch_grad_pos_term(rows, nbr, nullptr, nullptr, thC, g_rows, grad_pos, -1.f, 0, B, N, K, Din, Dout, 0, s));
    FLEX_HIP(launch_grad_pos_term(g_rows, nullptr, in_off, in_src, thN, rows, grad_pos, 1.f, 1, B, N, K, Dout, Din, 1, s));
    return FLEX_OK;
}

int flexupsample_fwd(const float *feat_small, const int32_t *sel, const int32_t *nbr, float *out,
                     int32_t *argmax, int B, int Ns, int Nf, int K, int C, int layout, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    if (!feat_small || !sel || !nbr || !out || !argmax) return FLEX_ERR_NULL;
    if (!sizes_ok(B, Nf, K, C, 1) || Ns <= 0 || Ns > Nf) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, align256(sizeof(int32_t) * (size_t)B * Nf))) return FLEX_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    int32_t *inv = (int32_t *)workspace;
    FLEX_HIP(launch_upsample_inv(sel, inv, B, Ns, Nf, s));
    FLEX_HIP(launch_upsample_fwd(feat_small, inv, nbr, out, argmax, B, Ns, Nf, K, C, layout == FLEX_LAYOUT_BNC, s));
    return FLEX_OK;
}

int flexupsample_bwd(const float *grad_out, const int32_t *argmax, const int32_t *sel,
                     const int32_t *in_off, const int32_t *in_src, float *grad_small, int B, int Ns,
                     int Nf, int K, int C, int layout, void *stream)
{
    if (!grad_out || !argmax || !sel || !in_off || !in_src || !grad_small) return FLEX_ERR_NULL;
    if (!sizes_ok(B, Nf, K, C, 1) || Ns <= 0 || Ns > Nf) return FLEX_ERR_SHAPE;
    if (layout != FLEX_LAYOUT_BCN && layout != FLEX_LAYOUT_BNC) return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_upsample_bwd(grad_out, argmax, sel, in_off, in_src, grad_small, B, Ns, Nf, C,
                                 layout == FLEX_LAYOUT_BNC, (hipStream_t)stream));
    return FLEX_OK;
}

int flex_validate_selection(const int32_t *sel, int B, int Ns, int Nf, int32_t *bad_count_dev,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (!sel || !bad_count_dev) return FLEX_ERR_NULL;
    if (!sizes_ok(B, Nf, 1, 1, 1) || Ns <= 0 || Ns > Nf) return FLEX_ERR_SHAPE;
    if (!ws_ok(workspace, workspace_bytes, align256(sizeof(int32_t) * (size_t)B * Nf))) return FLEX_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    int32_t *inv = (int32_t *)workspace;
    FLEX_HIP(launch_upsample_inv(sel, inv, B, Ns, Nf, s));
    FLEX_HIP(launch_upsample_check_sel(sel, inv, B, Ns, Nf, bad_count_dev, s));
    return FLEX_OK;
}

int flex_validate_neighbors(const int32_t *nbr, int B, int N, int K, int32_t *bad_count_dev,
                            void *stream)
{
    if (!nbr || !bad_count_dev) return FLEX_ERR_NULL;
    if (!sizes_ok(B, N, K, 1, 1)) return FLEX_ERR_SHAPE;
    FLEX_HIP(launch_count_bad(nbr, (int64_t)B * K * N, N, bad_count_dev, (hipStream_t)stream));
    return FLEX_OK;
}

}  // extern "C"
