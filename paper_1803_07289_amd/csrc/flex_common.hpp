// Shared host/device helpers for libflexconv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace flex {

constexpr int cdiv_c(int a, int b) { return (a + b - 1) / b; }
constexpr int rup_c(int a, int b) { return cdiv_c(a, b) * b; }
constexpr int npow2_c(int x) { int p = 1; while (p < x) p <<= 1; return p; }

static inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Number of compute units of the current device (cached per process).
int device_cu_count();

// Persistent-grid size: a multiple of 8 (one share per XCD), at most
// `wg_per_cu` workgroups per CU, at most one workgroup per tile.
int persistent_grid(int64_t total_tiles, int wg_per_cu);

typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

// ---- launchers implemented in the .hip translation units -------------------

// thetaP[(j*RP + r)*CP + c], j in 0..3 (x,y,z,bias), zero padded.
//   transpose == 0: r = input channel, c = output channel  (forward / grad_theta)
//   transpose == 1: r = output channel, c = input channel  (grad_feat)
hipError_t launch_pack_theta(const float *theta, const float *bias, float *thetaP,
                             int Din, int Dout, int RP, int CP, int transpose, hipStream_t s);

// Split-half (f16 hi/lo) fragment form of the same matrix for the wave-specialised
// kernels; layout documented at pack_theta_f16_kernel.  RP = padded rows per j, CP =
// padded columns (multiple of 16).
hipError_t launch_pack_theta_f16(const float *theta, const float *bias, void *thetaF, int Din,
                                 int Dout, int RP, int CP, int transpose, hipStream_t s);
size_t theta_f16_exp_offset(int RP, int CP);
size_t theta_f16_rscale_offset(int RP, int CP);
size_t theta_f16_bytes(int RP, int CP);

// Control words of the one-pass backward kernel (bwd_fused_lean_kernel) in the workspace: the flag (0: its parameter
// gradients stand; FUSED_OVERFLOW: a feature row overflowed f16 while the kernel ran; FUSED_UNRESOLVED: the check after
// the reduction found the result too small for the f16 halves to resolve; either way the stand-alone kernel
// recomputes them), then one record per workgroup: its last running exponent, its number of terms, its DO channel
// exponents.
constexpr int FUSED_FLAG_INTS = 64, FUSED_RECORD_INTS = 128, FUSED_MAX_WG = 1024;
constexpr int FUSED_OVERFLOW = 1, FUSED_UNRESOLVED = 2;
constexpr size_t fused_control_bytes() { return sizeof(int) * (size_t)(FUSED_FLAG_INTS + FUSED_RECORD_INTS * FUSED_MAX_WG); }
hipError_t launch_fused_bwd_check(int *control, int n_wg, const float *rscale, const float *grad_theta,
                                  const float *grad_bias, hipStream_t s);
hipError_t launch_reduce_partials_if(const int *flag, int want, const float *partials, int n_wg, int DIP, int DOP,
                                     int Din, int Dout, float *grad_theta, float *grad_bias, hipStream_t s);
hipError_t launch_pack_theta_f16_blocks(const float *theta, const float *bias, void *thetaF_all, int Din, int Dout,
                                        int r_blk, int c_blk, int n_i, int n_j, int transpose, hipStream_t s);

// Location gradient (flex_ws.hpp grad_pos_kernel): Theta_d fragments and one term of the gradient.
// launch_grad_pos_term returns hipErrorNotSupported when (DI, DO, N, K) has no lean kernel.
hipError_t launch_pack_theta_pos(const float *theta, void *thetaF, int Din, int Dout, int KDP, int CP,
                                 int transpose, hipStream_t s);
size_t theta_pos_exp_offset(int KDP, int CP);
size_t theta_pos_bytes(int KDP, int CP);
hipError_t launch_grad_pos_term(const float *rows, const int32_t *nbr, const int32_t *off, const int32_t *src,
                                const void *thetaF, const float *dot_rows, float *grad_pos, float sign,
                                int accumulate, int B, int N, int K, int DI, int DO, int csr, hipStream_t s);
bool grad_pos_supported(int DI, int DO, int N, int K);
// direct-form fallback for any shape (fp32 atomics)
hipError_t launch_generic_bwd_pos(const float *feat, const int32_t *nbr, const float *theta,
                                  const float *grad_out, float *grad_pos, int B, int N, int K, int Din,
                                  int Dout, int bnc, hipStream_t s);

// [B,C,N] -> [B,N,C] and back.
hipError_t launch_copy_rows(const float *src, float *dst, int B, int N, int Cs, int Cd, int src_bcn, int dst_bcn,
                            hipStream_t s, int c_off = 0);
hipError_t launch_theta_block_padded(const float *theta, float *blk, int Din, int Dout, int r0, int c0, int nr, int nc,
                                     hipStream_t s);
hipError_t launch_bcn_to_bnc(const float *src, float *dst, int B, int C, int N, hipStream_t s);
hipError_t launch_bnc_to_bcn(const float *src, float *dst, int B, int C, int N, hipStream_t s);

// Tiled matrix-core path.  `rows` is point-major [B*N, DI].  Returns
// hipErrorNotSupported when (DI,DO) has no instantiation.
//   csr == 0: neighbours from nbr [B,K,N], dp = pos[nbr]-pos[centre]
//   csr == 1: in-edge lists (off,src), dp = pos[centre]-pos[src]
//   theta_fmt: what thetaP holds, as answered by gather_contract_theta_format for the same
//   (DI, DO, N, K, csr): 0 = fp32 ThetaP (launch_pack_theta), 1 = split-half fragments
//   (launch_pack_theta_f16).
//   order (csr == 1 only): the walking order from launch_inedges_order for these lists
hipError_t launch_gather_contract(const float *rows, const float *pos, const int32_t *nbr,
                                  const int32_t *off, const int32_t *src, const int32_t *order,
                                  const void *thetaP, int theta_fmt, float *out, int B, int N, int K, int DI,
                                  int DO, int csr, int out_bcn, hipStream_t s);
bool gather_contract_supported(int DI, int DO);
int gather_contract_theta_format(int DI, int DO, int N, int K, int csr);
// true when the environment asks for the fp32 matrix op in the wave-specialised kernels
// (FLEX_CONTRACT=f32; read once).  For A/B measurements; both forms meet the same tolerance.
bool contract_in_fp32();
// Producer choice for the fixed-K forward (FLEX_PRODUCER, read once; for A/B measurements):
// 0 "staged" = LDS-staged producer, 1 "lean" = lean producers, one per consumer wave,
// 2 (default) = lean producers, three per consumer wave where the shape allows.
int lean_producer_mode();

// grad_theta / grad_bias: per-workgroup partial sums into `partials`
// ([n_wg, KD, DOP] floats), then a reduction into the two outputs.
hipError_t launch_grad_theta(const float *rows, const float *pos, const int32_t *nbr,
                             const float *g_rows, float *partials, float *grad_theta,
                             float *grad_bias, int B, int N, int K, int Din, int Dout,
                             hipStream_t s);
size_t grad_theta_partial_bytes(int64_t B, int64_t N, int Din, int Dout);

// Generic (any Din/Dout) direct-form kernels; strides select the layout.
hipError_t launch_generic_fwd(const float *feat, const float *pos, const int32_t *nbr,
                              const float *theta, const float *bias, float *out,
                              int B, int N, int K, int Din, int Dout, int bnc, hipStream_t s);
hipError_t launch_generic_bwd(const float *feat, const float *pos, const int32_t *nbr,
                              const float *theta, const float *bias, const float *grad_out,
                              float *grad_feat, float *grad_theta, float *grad_bias,
                              int B, int N, int K, int Din, int Dout, int bnc, hipStream_t s);

// In-edge lists.
hipError_t launch_inedges_build(const int32_t *nbr, int B, int N, int K, int32_t *in_off,
                                int32_t *in_src, void *ws, hipStream_t s);
hipError_t launch_inedges_build_sub(const int32_t *nbr, const int32_t *sel, int B, int N, int Ns, int K,
                                    int32_t *in_off, int32_t *in_src, void *ws, hipStream_t s);
size_t inedges_ws_bytes(int64_t BN);
// order[b*N + p] = point at position p: the cloud's points sorted by in-edge list length inside windows of nearby
// points (the walking order of the gather kernels over in-edge lists)
size_t inedges_order_bytes(int64_t BN);
hipError_t launch_inedges_order(const int32_t *in_off, int B, int N, int32_t *order, hipStream_t s);
size_t exclusive_scan_ws_bytes(int64_t n);
hipError_t launch_exclusive_scan_i32(const int32_t *cnt, int32_t *off, int64_t n, void *ws, hipStream_t s);
size_t knn_ws_bytes(int B, int N);
bool knn_k_supported(int K);
hipError_t launch_knn(const float *pos, int32_t *nbr, int B, int N, int K, void *ws, hipStream_t s);

// Pooling.
hipError_t launch_pool_fwd(const float *feat, const int32_t *nbr, float *out, int32_t *argmax,
                           int B, int N, int K, int C, int bnc, hipStream_t s);
hipError_t launch_pool_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat,
                           int B, int N, int C, int bnc, hipStream_t s);
hipError_t launch_pool_bwd_gather(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                                  const int32_t *in_src, float *grad_feat, int B, int N, int C, int bnc,
                                  hipStream_t s);

// Flex-upsampling: inverse selection map (inv[b*Nf + sel[b,j]] = j, -1 elsewhere), pooling through it,
// routing back over the larger layer's in-edge lists, and a check of the selection (out of range / repeated).
hipError_t launch_pool_sub_fwd(const float *feat, const int32_t *nbr, const int32_t *sel, float *out,
                               int32_t *argmax, int B, int N, int Ns, int K, int C, int bnc, hipStream_t s);
hipError_t launch_pool_sub_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat, int B,
                               int N, int L, int C, int bnc, hipStream_t s);
// static gather plan of the pooling backward pass (point-major, C = 64, 128 or 256)
size_t pool_plan_bytes(int B, int N, int K);
hipError_t launch_pool_plan_build(const int32_t *in_off, const int32_t *in_src, void *plan, int B, int N, int K,
                                  hipStream_t s);
hipError_t launch_pool_bwd_planned(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                                   const int32_t *in_src, void *plan, float *grad_feat, int B, int N, int K, int C,
                                   hipStream_t s);
hipError_t launch_pool_fwd_plan_build(const int32_t *nbr, void *plan, int B, int N, int K, hipStream_t s);
hipError_t launch_pool_fwd_planned(const float *feat, const int32_t *nbr, void *plan, float *out, int32_t *argmax,
                                   int B, int N, int K, int C, hipStream_t s);
hipError_t launch_pool_sub_bwd_gather(const float *grad_out, const int32_t *argmax, const int32_t *in_off,
                                      const int32_t *in_src, float *grad_feat, int B, int N, int L, int C,
                                      int bnc, hipStream_t s);
hipError_t launch_upsample_inv(const int32_t *sel, int32_t *inv, int B, int Ns, int Nf, hipStream_t s);
hipError_t launch_upsample_fwd(const float *feat_small, const int32_t *inv, const int32_t *nbr, float *out,
                               int32_t *argmax, int B, int Ns, int Nf, int K, int C, int bnc, hipStream_t s);
hipError_t launch_upsample_bwd(const float *grad_out, const int32_t *argmax, const int32_t *sel,
                               const int32_t *in_off, const int32_t *in_src, float *grad_small, int B, int Ns,
                               int Nf, int C, int bnc, hipStream_t s);
hipError_t launch_upsample_check_sel(const int32_t *sel, const int32_t *inv, int B, int Ns, int Nf, int32_t *bad,
                                     hipStream_t s);

hipError_t launch_count_bad(const int32_t *nbr, int64_t count, int N, int32_t *bad, hipStream_t s);
hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t s);
hipError_t launch_param_block(float *theta, float *bias, float *blk_theta, float *blk_bias, int R, int C, int r0,
                              int c0, int nr, int nc, int insert, hipStream_t s);
size_t idiss_ws_bytes(int B, int N);
size_t distinct_ws_bytes(int B, int Ns);
hipError_t launch_selection_make_distinct(int32_t *sel, int B, int N, int Ns, void *ws, hipStream_t s);
hipError_t launch_idiss_phi(const float *pos, const int32_t *nbr, float *phi, int B, int N, int K, hipStream_t s);
hipError_t launch_idiss_sample(const float *phi, const uint32_t *u, int32_t *sel, int B, int N, int Ns, void *ws,
                               hipStream_t s);
hipError_t launch_compose_1x1(const float *W, const float *theta, const float *bias, float *theta_c, float *bias_c,
                              int Din0, int Dmid, int Dout, hipStream_t s);
hipError_t launch_compose_1x1_bwd(const float *W, const float *theta, const float *bias, const float *gtheta_c,
                                  const float *gbias_c, float *gW, float *gtheta, float *gbias, int Din0, int Dmid,
                                  int Dout, hipStream_t s);

}  // namespace flex
