/*
 * libflexconv — flex-convolution and flex-max-pooling for gfx950 (MI355X).
 *
 * C ABI.  Every data pointer is a DEVICE pointer owned by the caller; the
 * library never allocates, frees or synchronises in these calls.  Work is
 * enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 * and the call returns at once.  Outputs are OVERWRITTEN, never accumulated.
 * Return value: FLEX_OK (0) or a flex_status; nothing throws or aborts.
 * Errors that the host can see (null pointers, non-positive sizes, K > N,
 * unknown layout, B*N >= 2^31, workspace too small) are returned before
 * anything is launched.
 *
 * Tensors (fp32 / int32), following the paper's statement of the layer
 * (Sec. 3.1 for the sum and the weight, Sec. 4.1 for the index tensor):
 *   feat      features, [B,Din,N]  (FLEX_LAYOUT_BCN, the paper's channel-major
 *             form) or [B,N,Din] (FLEX_LAYOUT_BNC, point-major: one point's
 *             feature vector is one contiguous row — the library's native
 *             layout, because a neighbour gather then reads whole rows)
 *   pos       point locations, always [B,3,N]
 *   nbr       neighbour indices, always int32 [B,K,N]; values are per-cloud
 *             point indices in [0,N).  Out-of-range values are undefined
 *             behaviour in the hot path; flex_validate_neighbors checks them.
 *   theta     [3,Din,Dout], bias [Din,Dout]: one (theta, bias) per (c,c') pair
 *   out, grad_out, grad_feat, pool out / argmax: same layout flag as feat.
 * The position difference is (neighbour - centre).
 *
 * Workspace: the entry points with a `workspace` argument take a caller
 * buffer of at least flexconv_workspace_bytes(op, ...) bytes, 256-byte aligned.
 * Its contents are scratch; calls sharing one workspace must be stream-ordered.
 */
#ifndef FLEXCONV_H
#define FLEXCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FLEX_OK = 0,
    FLEX_ERR_NULL = 1,        /* a required pointer is NULL */
    FLEX_ERR_SHAPE = 2,       /* non-positive size, K > N, B*N too large, bad layout/op */
    FLEX_ERR_UNSUPPORTED = 3, /* reserved */
    FLEX_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned or too small */
    FLEX_ERR_HIP = 5,         /* a HIP launch reported an error */
    FLEX_ERR_TOO_LARGE = 6    /* flexconv_fwd_noalloc: the call needs more scratch than the static buffer holds */
} flex_status;

typedef enum { FLEX_LAYOUT_BCN = 0, FLEX_LAYOUT_BNC = 1 } flex_layout;

typedef enum {
    FLEX_OP_CONV_FWD = 0,
    FLEX_OP_CONV_BWD = 1,       /* with caller-supplied in-edge lists */
    FLEX_OP_CONV_BWD_BUILD = 2, /* in-edge lists built inside the call */
    FLEX_OP_INEDGES = 3,
    FLEX_OP_UPSAMPLE = 4,       /* flexupsample_fwd / flex_validate_selection; N = points of the larger layer */
    FLEX_OP_CONV_BWD_POS = 5,       /* flexconv_bwd_pos with caller-supplied in-edge lists */
    FLEX_OP_CONV_BWD_POS_BUILD = 6, /* in-edge lists built inside the call */
    FLEX_OP_IDISS = 7,              /* flex_idiss_sample, flex_selection_make_distinct */
    FLEX_OP_KNN = 8                 /* flex_knn */
} flex_op;

/*
 * Flex-convolution forward: Eq.(4) with the weight of Eq.(6),
 *   out[b,o,l] = sum_k sum_c ( <theta[:,c,o], pos[b,:,n]-pos[b,:,l]> + bias[c,o] ) * feat[b,c,n],
 *   n = nbr[b,k,l].
 * Computed in fp32 in the factored form (per-point 4*Din aggregate, then a
 * (4*Din x Dout) contraction on the matrix cores).  Any Din, Dout: see
 * flexconv_has_fast_path for how a pair of widths is run.
 * Accuracy and dynamic range: on the matrix-core routes every fp32 operand of the contraction is
 * carried as two f16 halves (22 bits) after exact power-of-two scalings: the parameters per
 * (component, input channel) row and per output channel, a point's aggregate by the same row
 * scales and by its own largest magnitude.  Result: within 1e-4 of the fp64 value relative to
 * max(|value|, RMS of the same output channel), also when input channels (with the parameters
 * compensating) or output channels differ in scale by up to 2^24 (measured about 1e-6).  Not
 * covered: one input channel whose own values differ by more than 2^24 between the neighbours and
 * points that meet in one aggregate row; inputs with NaN / Inf.  The same holds for grad_feat of
 * flexconv_bwd.  grad_theta / grad_bias from the stand-alone kernel carry their operands exactly
 * (three bf16 pieces) and sum in fp32; on the one-pass route (FLEX_ROUTE_LEAN_FUSED) they are
 * contracted from the same f16 halves, with per-channel and per-point power-of-two scales, and the
 * call checks on the device whether the halves resolved the result (an overflowing feature row, or a
 * result more than 2^16 times closer to the representation error than ordinary data ever comes):
 * if not, the stand-alone kernel recomputes them inside the same call (correct, about 1.7 x the time).
 * flexconv_bwd_pos still scales the parameters by ONE power of two for the whole matrix:
 * channel scales more than about 2^10 apart cost it bits.
 */
int flexconv_fwd(const float *feat, const float *pos, const int32_t *nbr,
                 const float *theta, const float *bias, float *out,
                 int B, int N, int K, int Din, int Dout, int layout,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * flexconv_fwd for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments and result as flexconv_fwd without the
 * workspace pair: the scratch memory (the packed parameters; for channel-major tensors or widths that run
 * zero-padded also the copies flexconv_workspace_bytes(FLEX_OP_CONV_FWD, ...) counts) is a static device array
 * of FLEX_NOALLOC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends.  A call whose
 * plan needs more returns FLEX_ERR_TOO_LARGE before anything is launched (point-major layers of every tiled
 * width and wide layers up to 256 x 256 always fit; channel-major tensors only while the transposed copy does).
 * The call allocates nothing and frees nothing.  The first call on a device looks the array's address up (make
 * that call outside a graph capture).  All calls on one GPU share the array: calls that overlap on one GPU
 * (different streams, or graphs replayed concurrently) race; stream-ordered calls do not.  The array keeps the
 * last call's contents; nothing in it has to start at zero.
 */
#define FLEX_NOALLOC_SCRATCH_BYTES (2u << 20)
int flexconv_fwd_noalloc(const float *feat, const float *pos, const int32_t *nbr,
                         const float *theta, const float *bias, float *out,
                         int B, int N, int K, int Din, int Dout, int layout, void *stream);

/*
 * Flex-convolution backward (gradients of the forward map above, Sec. 3.1
 * asserts differentiability; formulas follow by differentiating the sum):
 *   grad_feat [b,c,m] = sum_{(l,k): nbr[b,k,l]=m} sum_o w(b,l,k,c,o) * grad_out[b,o,l]
 *   grad_theta[d,c,o] = sum_{b,l,k} (pos[b,d,n]-pos[b,d,l]) * feat[b,c,n] * grad_out[b,o,l]
 *   grad_bias [c,o]   = sum_{b,l,k}                          feat[b,c,n] * grad_out[b,o,l]
 * Any of grad_feat / grad_theta / grad_bias may be NULL (skipped; grad_theta
 * and grad_bias are produced together, pass both or neither).
 * grad_feat is evaluated as a gather over each point's IN-edges (the centres
 * that list it as a neighbour), so it uses no floating-point atomics and is
 * bit-reproducible.  in_off [B*N+1] / in_src [B*K*N] are those lists as built
 * by flex_inedges_build for this nbr; pass both NULL to have them built in the
 * workspace on every call (neighbourhoods are static, so building once and
 * reusing is the intended use).
 */
int flexconv_bwd(const float *feat, const float *pos, const int32_t *nbr,
                 const float *theta, const float *bias, const float *grad_out,
                 float *grad_feat, float *grad_theta, float *grad_bias,
                 const int32_t *in_off, const int32_t *in_src,
                 int B, int N, int K, int Din, int Dout, int layout,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Flex-convolution backward with respect to the point locations (Sec. 3.1: the weight is
 * differentiable in all its arguments, so gradients reach the locations too).  Every edge
 * (l,k), n = nbr[b,k,l], carries s_d = sum_{c,o} theta[d,c,o] * feat[b,c,n] * grad_out[b,o,l]
 * to grad_pos[b,d,n] with + and to grad_pos[b,d,l] with -.  grad_pos is [B,3,N] like pos,
 * overwritten.  Evaluated from plain neighbourhood sums (of feat over each point's neighbours, of
 * grad_out over the centres that list it) and one small contraction per point, without
 * floating-point atomics (widths 32 / 64 directly; any other widths as the sum over 64 x 64 parameter
 * blocks of the 64 -> 64 kernel's result on zero-padded 64-channel column blocks of the two tensors,
 * copied into the workspace).  in_off / in_src as for flexconv_bwd (NULL: built in the workspace).
 */
int flexconv_bwd_pos(const float *feat, const int32_t *nbr, const float *theta, const float *grad_out,
                     const int32_t *in_off, const int32_t *in_src, float *grad_pos,
                     int B, int N, int K, int Din, int Dout, int layout,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Transposed neighbour graph (Sec. 4.1: neighbourhoods are computed once and
 * kept fixed, so this is part of that preprocessing).  For global point
 * g = b*N+m, in_src[in_off[g] .. in_off[g+1]) lists the centres l (per-cloud
 * indices, ascending, one entry per occurrence) with nbr[b,k,l] = m.
 * in_off has B*N+1 entries, in_src has B*K*N entries.
 */
int flex_inedges_build(const int32_t *nbr, int B, int N, int K,
                       int32_t *in_off, int32_t *in_src,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Flex-max-pooling forward (Sec. 4.1): out[b,c,l] = max_k feat[b,c,nbr[b,k,l]];
 * argmax[b,c,l] = per-cloud index of the winning point (Table 1: the forward
 * pass stores a same-sized table for the backward pass).  Ties go to the
 * LOWEST POINT INDEX among the maxima; -0 == +0 is a tie; out carries the
 * winner's bits.  NaN inputs are unsupported.
 */
int flexpool_fwd(const float *feat, const int32_t *nbr, float *out, int32_t *argmax,
                 int B, int N, int K, int C, int layout, void *stream);

/*
 * Flex-max-pooling backward: grad_feat[b,c,m] = sum of grad_out[b,c,l] over
 * the centres l with argmax[b,c,l] = m, zero elsewhere (Table 1: the backward
 * pass reads only the upstream gradient and the table stored by the forward
 * pass).  Two forms:
 *   in_off / in_src NULL: scatter by the recorded index with fp32 atomic adds
 *     (summation order, hence the last bit, may vary between runs when several
 *     centres share a winner); K is ignored.
 *   in_off / in_src given (the lists flex_inedges_build made for the nbr tensor
 *     of the forward pass, with the same K): every point sums over the centres
 *     that list it, keeping those whose recorded winner it is.  No atomics,
 *     fixed order, and several times faster on large clouds.
 */
int flexpool_bwd(const float *grad_out, const int32_t *argmax, float *grad_feat,
                 const int32_t *in_off, const int32_t *in_src,
                 int B, int N, int K, int C, int layout, void *stream);

/*
 * Flex-max-pooling backward with a static gather plan (Sec. 4.1: the neighbourhoods are computed once and kept
 * fixed, so which rows of grad_out / argmax a group of neighbouring points needs is fixed too; Table 1: the
 * backward pass reads the upstream gradient and the recorded table).  The plan lists, for every tile of 32
 * consecutive points, the distinct centres that list any of them, and for every entry of in_src the place of its
 * centre in that list; the kernel fetches each listed row once per tile instead of once per entry.
 *   flexpool_plan_bytes   size of the plan for (B, N, K) in bytes (0 for sizes flexconv would reject);
 *   flexpool_plan_build   writes the plan for the lists (in_off, in_src) flex_inedges_build made with the same
 *                         (B, N, K); plan: device memory, 256-byte aligned, owned by the caller, valid as long
 *                         as the lists are; FLEX_ERR_WORKSPACE if plan_bytes is too small;
 *   flexpool_bwd_planned  grad_feat of flexpool_bwd's list form, bit for bit (same sums in the same order);
 *                         point-major C = 64, 128 or 256 with K <= FLEX_POOL_PLAN_MAX_K and at least
 *                         FLEX_POOL_PLAN_MIN_POINTS points in all runs the planned kernel (that is where it is
 *                         the faster one), everything else the list form itself.  grad_out / argmax / grad_feat
 *                         as for flexpool_bwd.
 * The plan's last 2 KB are scratch of the call (tile counters of the list form that runs in the planned kernel's
 * place on clouds without locality, cleared at every call): calls that share a plan must not overlap in time;
 * nothing else of it is written after the build.
 * The plan depends on the lists only, not on the tensors: build it once per cloud.  It is dimensioned for the
 * paper's neighbourhood sizes (K = 8 or 9): a tile's plan holds up to 127 distinct centres and covers up to 512
 * list entries; what exceeds that is fetched entry by entry, correctly but without the saving, and where more
 * than an eighth of the tiles exceed it (point orders without locality) the call runs the list form instead.
 */
#define FLEX_POOL_PLAN_MAX_K 10
#define FLEX_POOL_PLAN_MIN_POINTS (1 << 18)

/*
 * Flex-max-pooling forward with a static gather plan: the same idea for the forward pass (Sec. 4.1; Table 1: it
 * writes the output and the same-sized winner table).  The plan is over the neighbour lists themselves: per tile of
 * 32 consecutive centres the distinct points they list (about three per centre where a centre lists eight), per
 * (centre, slot) the place of its point among them; the kernel fetches each distinct row once per tile.  Same size
 * and layout as the backward plan (flexpool_plan_bytes serves both), different content: a plan serves only the pass
 * whose build call wrote it.
 *   flexpool_fwd_plan_build  writes the plan for nbr [B,K,N] (device; entries in [0,N): flex_validate_neighbors);
 *                            plan: device, 256-byte aligned, plan_bytes >= flexpool_plan_bytes(B,N,K), owned by the
 *                            caller, valid while nbr is unchanged.
 *   flexpool_fwd_planned     out / argmax of flexpool_fwd, bit for bit (the same comparisons in the same slot order);
 *                            arguments as flexpool_fwd, plus the plan.  The planned kernel runs under the conditions
 *                            of flexpool_bwd_planned (point-major, C = 64 / 128 / 256, K <= FLEX_POOL_PLAN_MAX_K,
 *                            B N >= FLEX_POOL_PLAN_MIN_POINTS), else flexpool_fwd's own kernels; on a cloud whose
 *                            tiles the plan does not cover (stored without locality) the planned kernel itself
 *                            takes flexpool_fwd's steps, a few per cent slower than flexpool_fwd would.  The call
 *                            only reads the plan: forward calls that share one may overlap.
 * Errors: FLEX_ERR_NULL, FLEX_ERR_SHAPE as flexpool_fwd; FLEX_ERR_WORKSPACE for a plan that is too small or
 * misaligned; nothing is launched then.
 */
int flexpool_fwd_plan_build(const int32_t *nbr, int B, int N, int K, void *plan, size_t plan_bytes, void *stream);
int flexpool_fwd_planned(const float *feat, const int32_t *nbr, float *out, int32_t *argmax,
                         void *plan, size_t plan_bytes, int B, int N, int K, int C, int layout, void *stream);
size_t flexpool_plan_bytes(int B, int N, int K);
int flexpool_plan_build(const int32_t *in_off, const int32_t *in_src, int B, int N, int K,
                        void *plan, size_t plan_bytes, void *stream);
int flexpool_bwd_planned(const float *grad_out, const int32_t *argmax, float *grad_feat,
                         const int32_t *in_off, const int32_t *in_src, void *plan, size_t plan_bytes,
                         int B, int N, int K, int C, int layout, void *stream);

/*
 * 1x1 convolution composed into a flex-convolution (Sec. 4.3: a ResNet block chains a 1x1
 * convolution and flex-convolutions; the paper names no bias in the 1x1 step and no activation
 * between it and the next step, and this entry point assumes neither).  With mid = W feat,
 * W [Dmid,Din0], the next layer flexconv(theta [3,Dmid,Dout], bias [Dmid,Dout]) over mid equals a
 * flex-convolution over feat itself with
 *   theta_c[d,c0,o] = sum_c W[c,c0] theta[d,c,o],   bias_c[c0,o] = sum_c W[c,c0] bias[c,o],
 * because the weight function is linear in its parameters.  The 1x1 output (a [B,Dmid,N] tensor
 * written and gathered again) is never formed: call flexconv_fwd / flexconv_bwd with
 * (theta_c [3,Din0,Dout], bias_c [Din0,Dout]).  All arrays device fp32, overwritten.
 */
int flexconv_compose_1x1(const float *W, const float *theta, const float *bias,
                         float *theta_c, float *bias_c, int Din0, int Dmid, int Dout, void *stream);

/*
 * Backward through the composition.  flexconv_bwd with the composed parameters returns grad_feat
 * of the block's input directly, and grad_theta_c / grad_bias_c; this call turns those into
 *   grad_W[c,c0]      = sum_{d,o} theta[d,c,o] grad_theta_c[d,c0,o] + sum_o bias[c,o] grad_bias_c[c0,o]
 *   grad_theta[d,c,o] = sum_c0 W[c,c0] grad_theta_c[d,c0,o],  grad_bias[c,o] = sum_c0 W[c,c0] grad_bias_c[c0,o]
 * (grad_W [Dmid,Din0], grad_theta [3,Dmid,Dout], grad_bias [Dmid,Dout], overwritten).
 */
int flexconv_compose_1x1_bwd(const float *W, const float *theta, const float *bias,
                             const float *grad_theta_c, const float *grad_bias_c,
                             float *grad_W, float *grad_theta, float *grad_bias,
                             int Din0, int Dmid, int Dout, void *stream);

/*
 * Flex-max-pooling with subsampling, forward (Sec. 4.1: pooling runs before the subsampling step;
 * Sec. 4.3: the last layer of an encoder stage, which keeps a quarter of the points).  The result
 * is that of flexpool_fwd restricted to the kept centres, and only those are evaluated:
 *   out[b,c,j] = max_k feat[b,c,nbr[b,k,sel[b,j]]],  argmax[b,c,j] = the winning point, an index
 *   into the N points before subsampling (pooling's tie rule).
 * feat [B,C,N] or [B,N,C]; nbr int32 [B,K,N]; sel int32 [B,Ns], indices in [0,N) (an entry
 * outside is clamped into the range); out / argmax [B,C,Ns] or [B,Ns,C].
 */
int flexpool_sub_fwd(const float *feat, const int32_t *nbr, const int32_t *sel, float *out,
                     int32_t *argmax, int B, int N, int Ns, int K, int C, int layout, void *stream);

/*
 * Flex-max-pooling with subsampling, backward: grad_feat[b,c,m] = sum of grad_out[b,c,j] over
 * the kept centres j with argmax[b,c,j] = m, zero elsewhere; grad_feat [B,C,N] or [B,N,C] is
 * overwritten.  Two forms, as for flexpool_bwd:
 *   in_off / in_src NULL: zero fill + fp32 atomic adds (K is ignored);
 *   in_off / in_src given: the lists flex_inedges_build_sub made for (nbr, sel) of the forward
 *     pass (same K): every point sums over the kept centres that list it.  No atomics, fixed
 *     order, several times faster.
 */
int flexpool_sub_bwd(const float *grad_out, const int32_t *argmax,
                     const int32_t *in_off, const int32_t *in_src, float *grad_feat,
                     int B, int N, int Ns, int K, int C, int layout, void *stream);

/*
 * Transposed neighbour lists restricted to kept centres (static per layer, like the neighbour
 * tensor itself, Sec. 4.1): for every point m of the N, the ascending row numbers j in [0,Ns) of
 * the kept centres sel[b,j] whose neighbourhood names m, once per naming slot.
 * in_off int32 [B*N+1], in_src int32 [B*K*Ns]; workspace as for flex_inedges_build
 * (flexconv_workspace_bytes(FLEX_OP_INEDGES, B, N, ...)).
 */
int flex_inedges_build_sub(const int32_t *nbr, const int32_t *sel, int B, int N, int Ns, int K,
                           int32_t *in_off, int32_t *in_src,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * K nearest neighbours (Sec. 3: neighbourhoods are the k nearest points; Sec. 4.1: the index
 * tensors of every resolution are computed ahead of the network.  The paper does not say how;
 * this is an exact search on a uniform grid).  nbr[b,k,l] = the point with the k-th smallest
 * squared distance to point l in cloud b, the point itself included (slot 0 unless an equal
 * point has a lower index), ordered by (d2, index): equal distances go to the LOWER INDEX.
 * d2 is evaluated in fp32 as ((dx*dx + dy*dy) + dz*dz), dx = pos[n] - pos[l], each operation
 * rounded separately; the result is the exact ranking under that d2.
 * Cost: every query scans the cells around it, so M points at one location (or closer together than the
 * cell edge, about the mean spacing) cost M*M distance evaluations; meant for clouds without such piles.
 * pos [B,3,N] finite; nbr int32 [B,K,N] overwritten.  K in 1..10, 12, 16, 24 or 32, K <= N;
 * B <= 65535.  Workspace: flexconv_workspace_bytes(FLEX_OP_KNN, B, N, K, ...).
 */
int flex_knn(const float *pos, int32_t *nbr, int B, int N, int K,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Inverse density importance sub-sampling, step 1 (Sec. 3.2): phi[b,l] = sum over the K
 * neighbours n of ||pos[b,:,l] - pos[b,:,n]||, the paper's approximation of the inverse
 * density.  pos [B,3,N], nbr int32 [B,K,N], phi fp32 [B,N] (overwritten).
 */
int flex_idiss_phi(const float *pos, const int32_t *nbr, float *phi, int B, int N, int K, void *stream);

/*
 * Inverse density importance sub-sampling, step 2: Ns points per cloud drawn with probability
 * proportional to phi in one pass over the points.  The paper asks for proportional sampling
 * in O(n) and fixes no procedure; the one used is stratified sampling on the running sum, in
 * integer arithmetic so that the result does not depend on summation order:
 *   q[l] = floor(phi[l] * (2^bits / max phi)) in fp32, bits = min(28, 51 - ceil(log2 N)); all 1
 *          if the maximum is 0;  C = running sum of q (64 bit);  Q = its total;
 *   stratum j of [0,Q) has Q / Ns units (+1 for the first Q mod Ns), threshold
 *   t_j = start_j + floor(u[b,j] * len_j / 2^32), sel[b,j] = first l with C[l] > t_j.
 * u uint32 [B,Ns] = the caller's random words (any generator; the library draws none).
 * sel int32 [B,Ns], ascending; a point far heavier than a stratum is drawn for each threshold
 * it spans (drawing with replacement), a point with q = 0 never.  phi must be finite and >= 0.
 * N <= 2^25 per cloud, B <= 65535.  Workspace: flexconv_workspace_bytes(FLEX_OP_IDISS, B, N, ...).
 */
int flex_idiss_sample(const float *phi, const uint32_t *u, int32_t *sel, int B, int N, int Ns,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Repeats removed from an ascending selection, in place (for callers that cannot use a point
 * twice: flexupsample_*, flex_inedges_build_sub with the list form of flexpool_sub_bwd).  The
 * draw is kept and every repeated entry moves to the next free index:
 *   sel[j] = max(sel[j], sel[j-1] + 1) for j = 1 .. Ns-1, then sel[j] = min(sel[j], N - Ns + j)
 * (the second step packs the tail against the end of the cloud should the first run past it).
 * sel int32 [B,Ns], ascending per cloud, entries in [0,N).  Workspace: at least
 * flexconv_workspace_bytes(FLEX_OP_IDISS, B, N, ...) (far less is used).
 */
int flex_selection_make_distinct(int32_t *sel, int B, int N, int Ns,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Flex-upsampling forward (Sec. 4.1): the features of the smaller layer's points are copied
 * to their points in the larger layer, every other point of the larger layer starts at zero,
 * and flex-max-pooling runs over the larger layer's neighbourhoods:
 *   dense[b,c,m] = feat_small[b,c,j] if m = sel[b,j], else 0
 *   out[b,c,l]   = max_k dense[b,c,nbr[b,k,l]],  argmax[b,c,l] = the winning larger-layer point
 * (pooling's tie rule: lowest point index among the maxima; a zero-filled point can win).
 * feat_small [B,C,Ns] or [B,Ns,C]; sel int32 [B,Ns], distinct indices in [0,Nf) per cloud
 * (undefined result otherwise; flex_validate_selection checks); nbr int32 [B,K,Nf];
 * out / argmax [B,C,Nf] or [B,Nf,C].  The zero-filled tensor is never materialised; the
 * workspace (flexconv_workspace_bytes(FLEX_OP_UPSAMPLE, B, Nf, ...)) holds an inverse map.
 */
int flexupsample_fwd(const float *feat_small, const int32_t *sel, const int32_t *nbr,
                     float *out, int32_t *argmax, int B, int Ns, int Nf, int K, int C, int layout,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Flex-upsampling backward: the pooling step routes grad_out[b,c,l] to the recorded winner,
 * the copy step hands a selected point's gradient to the smaller layer's point it came
 * from; what a zero-filled point won is dropped:
 *   grad_small[b,c,j] = sum of grad_out[b,c,l] over centres l with argmax[b,c,l] = sel[b,j].
 * Evaluated as a gather over the in-edge lists of the larger layer's nbr (in_off / in_src
 * from flex_inedges_build, required): no atomics, fixed summation order.
 */
int flexupsample_bwd(const float *grad_out, const int32_t *argmax, const int32_t *sel,
                     const int32_t *in_off, const int32_t *in_src, float *grad_small,
                     int B, int Ns, int Nf, int K, int C, int layout, void *stream);

/* Debug aid: *bad_count_dev (device int32) = number of sel entries outside [0,Nf) or repeating
 * another entry of their cloud.  Workspace as for flexupsample_fwd. */
int flex_validate_selection(const int32_t *sel, int B, int Ns, int Nf, int32_t *bad_count_dev,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace needed by op (a flex_op) at these sizes. 0 on bad sizes. */
size_t flexconv_workspace_bytes(int op, int B, int N, int K, int Din, int Dout, int layout);

/* Debug aid: *bad_count_dev (device int32) = number of nbr entries outside [0,N). */
int flex_validate_neighbors(const int32_t *nbr, int B, int N, int K,
                            int32_t *bad_count_dev, void *stream);

/* 1 if flexconv_fwd / flexconv_bwd run (Din,Dout) on the matrix-core kernels: the tiled widths 32->32, 64->64,
 * 128->128, 9->64, 64->9, 32->64, 64->32, 64->128, 128->64, and every pair of multiples of 128 (run as passes over
 * 64- / 128-channel column blocks; the deeper stages of the network of Sec. 4.3, whose feature length doubles from
 * stage to stage).  2: any other widths, which run zero-padded at the nearest widths of that list (padded copies
 * of the tensors live in the workspace, whose size flexconv_workspace_bytes reports).  0: the direct-form kernels
 * (orders of magnitude slower; only with padding or block passes switched off in the environment). */
int flexconv_has_fast_path(int Din, int Dout);

/* Which kernel family a flexconv_fwd (op = FLEX_OP_CONV_FWD) or the feature gradient of a flexconv_bwd
 * (op = FLEX_OP_CONV_BWD) call of these sizes runs on; -1 on bad sizes.  A host-side query (nothing is launched) of
 * the same decision the entry points dispatch on, so that the size limits of every family (32-bit byte offsets
 * inside a cloud for the lean kernels and the block passes) can be checked without running a cloud that large. */
typedef enum {
    FLEX_ROUTE_DIRECT = 0,     /* direct-form kernels (Eq. 6 per neighbour, channel pair) */
    FLEX_ROUTE_SINGLE_ROLE = 1,/* tiled kernels, every wave gathers then contracts (fp32 matrix op) */
    FLEX_ROUTE_STAGED = 2,     /* wave-specialised kernels with LDS-staged producers */
    FLEX_ROUTE_LEAN = 3,       /* wave-specialised kernels with lean producers (the headline path) */
    FLEX_ROUTE_SPLIT128 = 4,   /* 128 -> 128 point-major as two passes of the 64-wide lean kernels */
    FLEX_ROUTE_WIDE = 5,       /* block passes over 64- / 128-channel column blocks */
    FLEX_ROUTE_PADDED = 6,     /* zero-padded to the nearest widths with a matrix-core path */
    FLEX_ROUTE_LEAN_FUSED = 7  /* flexconv_bwd only: lean kernels, and when grad_feat and grad_theta / grad_bias are
                                  all asked for, ONE kernel makes one pass over the in-edge lists for all of them
                                  (64 -> 64 layers); a call for a subset runs the FLEX_ROUTE_LEAN kernels */
} flex_route;
int flexconv_kernel_route(int op, int B, int N, int K, int Din, int Dout, int layout);

/* Measurement aids for benchmarks (not part of the layers): what this device reaches on a plain copy and on a pure
 * f16 matrix-op loop, so that kernel figures can be quoted against measured peaks beside the published ones.
 * flex_calibrate_copy: dst = src, `bytes` (a multiple of 16, both pointers 16-byte aligned) read and written once.
 * flex_calibrate_mfma_f16: every compute unit runs iters x 4 v_mfma_f32_16x16x32_f16 per wave on 16 waves;
 * *flop_out (host, may be NULL) = the flop count of the launch; sink: one device float, never written in practice.
 * Both only enqueue the kernel on `stream`; time them with events. */
int flex_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream);
int flex_calibrate_mfma_f16(int iters, float *sink, double *flop_out, void *stream);

const char *flex_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FLEXCONV_H */
