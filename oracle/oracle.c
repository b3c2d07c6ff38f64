/*
 * CPU oracle for the flex-convolution layer and flex-max-pooling.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code with the HIP path and is
 * called only from tests, the smoke check and the benchmark's CPU-baseline
 * leg.  Nothing in the product path may call it.
 *
 * Everything is evaluated straight from the definitions, in double precision
 * (inputs are the caller's float32 arrays, promoted element by element):
 *
 *   flex-conv forward   Eq.(4) (neighbourhood convolution: a plain sum over
 *                       the K neighbours and the input channels) with the
 *                       weight function of Eq.(6) (scalar product of a
 *                       learnable theta with the position difference, plus a
 *                       learnable bias; one parameter set per (c, c') pair,
 *                       as the filter-bank signature of Eq.(5) implies).
 *   flex-conv backward  the transposes of that bilinear map (the paper
 *                       asserts differentiability in Sec. 3.1 and prints no
 *                       formulas; they are derived here by differentiating
 *                       the forward sum term by term).
 *   flex-max-pool       Sec. 4.1: maximum over each point's neighbourhood,
 *                       no subsampling; the forward pass also records which
 *                       point won (Table 1's pooling memory is output plus a
 *                       same-sized table; Sec. 4.2 notes the prepared
 *                       intermediate), the backward pass routes by it.
 *
 * Readings of points the paper leaves open:
 *   - position difference is (neighbour - centre), the orientation used in
 *     the caption of Fig. 2; Eq.(6) writes (centre - neighbour), which is the
 *     same layer with theta negated;
 *   - no normalisation by K, no output bias, no activation (Eq.(4) has none);
 *   - whether a point is its own neighbour is decided by the index tensor;
 *   - duplicate indices contribute once per occurrence;
 *   - pooling ties: among the neighbours attaining the maximum, the LOWEST
 *     POINT INDEX wins (independent of slot order); -0 == +0 is a tie; the
 *     output value is the winner's float bit pattern; NaN is unsupported;
 *   - gradients overwrite their output arrays.
 *
 * Layouts (paper / channel-major): feat [B,Din,N], pos [B,3,N],
 * nbr int32 [B,K,N] (per-cloud point indices in [0,N)), theta [3,Din,Dout],
 * bias [Din,Dout], out / grad_out [B,Dout,N].
 *
 * Every routine takes a range [l_begin, l_end) of CENTRE points to process;
 * the full result uses [0, N).  Ranged calls exist so a bounded share of a
 * large workload can be timed or checked; each centre's work is independent.
 * Per-centre outputs (flex-conv out, pool out / argmax) are compact: their last
 * axis has L = l_end - l_begin columns, column l - l_begin.  Scattered outputs
 * (grad_feat of either layer) keep N columns and are ACCUMULATED into, so the
 * caller passes them zero-filled (the Python wrapper does).
 *
 * Parity pins: every function here (flex-upsampling included) is pinned by tests/test_oracle_*.py
 * (brute force via dense weight tensors, regular-grid reduction to ordinary
 * correlation incl. Prewitt and box blur, theta = 0, translation invariance,
 * finite differences, adjoint identities, grid max-pool).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX3(a, b, c, nb, nc) ((((int64_t)(a)) * (nb) + (b)) * (int64_t)(nc) + (c))

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Range check of the index tensor: returns the number of entries outside [0,N). */
int64_t oracle_count_bad_neighbors(const int32_t *nbr, int B, int N, int K)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < (int64_t)B * K * N; ++i)
        bad += (nbr[i] < 0 || nbr[i] >= N);
    return bad;
}

/* ---------------------------------------------------------------------------
 * Flex-conv forward, Eq.(4) with Eq.(6):
 *   out[b,o,l] = sum_k sum_c ( <theta[:,c,o], pos[b,:,n] - pos[b,:,l]> + bias[c,o] ) * feat[b,c,n],
 *   n = nbr[b,k,l].
 * out is double [B,Dout,L], L = l_end - l_begin.
 * ------------------------------------------------------------------------- */
int oracle_flexconv_fwd(const float *feat, const float *pos, const int32_t *nbr,
                        const float *theta, const float *bias, double *out,
                        int B, int N, int K, int Din, int Dout, int l_begin, int l_end)
{
    if (!feat || !pos || !nbr || !theta || !bias || !out) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || Din <= 0 || Dout <= 0) return 2;
    if (l_begin < 0 || l_end > N || l_begin > l_end) return 2;
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * Dout);
#pragma omp for collapse(2) schedule(static)
        for (int b = 0; b < B; ++b)
            for (int l = l_begin; l < l_end; ++l) {
                for (int o = 0; o < Dout; ++o) acc[o] = 0.0;
                for (int k = 0; k < K; ++k) {
                    const int n = nbr[IDX3(b, k, l, K, N)];
                    const double dx = (double)pos[IDX3(b, 0, n, 3, N)] - (double)pos[IDX3(b, 0, l, 3, N)];
                    const double dy = (double)pos[IDX3(b, 1, n, 3, N)] - (double)pos[IDX3(b, 1, l, 3, N)];
                    const double dz = (double)pos[IDX3(b, 2, n, 3, N)] - (double)pos[IDX3(b, 2, l, 3, N)];
                    for (int c = 0; c < Din; ++c) {
                        const double f = (double)feat[IDX3(b, c, n, Din, N)];
                        const float *tx = theta + IDX3(0, c, 0, Din, Dout);
                        const float *ty = theta + IDX3(1, c, 0, Din, Dout);
                        const float *tz = theta + IDX3(2, c, 0, Din, Dout);
                        const float *tb = bias + (int64_t)c * Dout;
                        for (int o = 0; o < Dout; ++o) {
                            const double w = (double)tx[o] * dx + (double)ty[o] * dy + (double)tz[o] * dz + (double)tb[o];
                            acc[o] += w * f;
                        }
                    }
                }
                for (int o = 0; o < Dout; ++o) out[IDX3(b, o, l - l_begin, Dout, l_end - l_begin)] = acc[o];
            }
        free(acc);
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Flex-conv backward.  With g = grad_out and w(b,l,k,c,o) the weight above:
 *   grad_feat [b,c,m] = sum over all (l,k) with nbr[b,k,l] = m of  sum_o w(b,l,k,c,o) * g[b,o,l]
 *   grad_theta[d,c,o] = sum_b sum_l sum_k (pos[b,d,n]-pos[b,d,l]) * feat[b,c,n] * g[b,o,l]
 *   grad_bias [c,o]   = sum_b sum_l sum_k                          feat[b,c,n] * g[b,o,l]
 * Any of the three outputs may be NULL (skipped).  Outputs are double.
 * grad_theta / grad_bias are overwritten; grad_feat [B,Din,N] is accumulated
 * into (pass it zero-filled).  Only centres l in [l_begin,l_end) contribute.
 * ------------------------------------------------------------------------- */
int oracle_flexconv_bwd(const float *feat, const float *pos, const int32_t *nbr,
                        const float *theta, const float *bias, const float *grad_out,
                        double *grad_feat, double *grad_theta, double *grad_bias,
                        int B, int N, int K, int Din, int Dout, int l_begin, int l_end)
{
    if (!feat || !pos || !nbr || !theta || !bias || !grad_out) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || Din <= 0 || Dout <= 0) return 2;
    if (l_begin < 0 || l_end > N || l_begin > l_end) return 2;
    const int64_t n_theta = (int64_t)3 * Din * Dout, n_bias = (int64_t)Din * Dout;
    const int want_params = (grad_theta != NULL) || (grad_bias != NULL);
    if (grad_theta) memset(grad_theta, 0, sizeof(double) * (size_t)n_theta);
    if (grad_bias) memset(grad_bias, 0, sizeof(double) * (size_t)n_bias);
#pragma omp parallel
    {
        /* per-thread parameter-gradient accumulators, merged at the end */
        double *gt = (double *)calloc((size_t)n_theta, sizeof(double));
        double *gb = (double *)calloc((size_t)n_bias, sizeof(double));
        double *g = (double *)malloc(sizeof(double) * Dout);
#pragma omp for collapse(2) schedule(static)
        for (int b = 0; b < B; ++b)
            for (int l = l_begin; l < l_end; ++l) {
                for (int o = 0; o < Dout; ++o) g[o] = (double)grad_out[IDX3(b, o, l, Dout, N)];
                for (int k = 0; k < K; ++k) {
                    const int n = nbr[IDX3(b, k, l, K, N)];
                    const double dx = (double)pos[IDX3(b, 0, n, 3, N)] - (double)pos[IDX3(b, 0, l, 3, N)];
                    const double dy = (double)pos[IDX3(b, 1, n, 3, N)] - (double)pos[IDX3(b, 1, l, 3, N)];
                    const double dz = (double)pos[IDX3(b, 2, n, 3, N)] - (double)pos[IDX3(b, 2, l, 3, N)];
                    for (int c = 0; c < Din; ++c) {
                        const double f = (double)feat[IDX3(b, c, n, Din, N)];
                        const float *tx = theta + IDX3(0, c, 0, Din, Dout);
                        const float *ty = theta + IDX3(1, c, 0, Din, Dout);
                        const float *tz = theta + IDX3(2, c, 0, Din, Dout);
                        const float *tb = bias + (int64_t)c * Dout;
                        double *gtx = gt + IDX3(0, c, 0, Din, Dout);
                        double *gty = gt + IDX3(1, c, 0, Din, Dout);
                        double *gtz = gt + IDX3(2, c, 0, Din, Dout);
                        double *gbb = gb + (int64_t)c * Dout;
                        double s = 0.0;
                        if (grad_feat)
                            for (int o = 0; o < Dout; ++o) {
                                const double w = (double)tx[o] * dx + (double)ty[o] * dy + (double)tz[o] * dz + (double)tb[o];
                                s += w * g[o];
                            }
                        if (want_params)
                            for (int o = 0; o < Dout; ++o) {
                                const double fg = f * g[o];
                                gtx[o] += dx * fg;
                                gty[o] += dy * fg;
                                gtz[o] += dz * fg;
                                gbb[o] += fg;
                            }
                        if (grad_feat) {
#pragma omp atomic
                            grad_feat[IDX3(b, c, n, Din, N)] += s;
                        }
                    }
                }
            }
#pragma omp critical
        {
            if (grad_theta) for (int64_t i = 0; i < n_theta; ++i) grad_theta[i] += gt[i];
            if (grad_bias) for (int64_t i = 0; i < n_bias; ++i) grad_bias[i] += gb[i];
        }
        free(gt); free(gb); free(g);
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * grad_feat of flex-conv at selected target points only (for sampled parity
 * at sizes where the full backward is too slow).  targets[i] = b*N + m.
 * out is double [n_targets, Din].  Every edge (l,k) of every centre is
 * scanned; an edge contributes when its neighbour is a listed target.
 * ------------------------------------------------------------------------- */
int oracle_flexconv_grad_feat_at(const float *pos, const int32_t *nbr,
                                 const float *theta, const float *bias, const float *grad_out,
                                 const int64_t *targets, int64_t n_targets, double *out,
                                 int B, int N, int K, int Din, int Dout)
{
    if (!pos || !nbr || !theta || !bias || !grad_out || !targets || !out) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || Din <= 0 || Dout <= 0 || n_targets < 0) return 2;
    /* slot[b*N+m] = row of `out` (or -1) */
    int64_t *slot = (int64_t *)malloc(sizeof(int64_t) * (size_t)B * N);
    if (!slot) return 6;
    for (int64_t i = 0; i < (int64_t)B * N; ++i) slot[i] = -1;
    for (int64_t i = 0; i < n_targets; ++i) {
        if (targets[i] < 0 || targets[i] >= (int64_t)B * N || slot[targets[i]] != -1) { free(slot); return 2; }
        slot[targets[i]] = i;
    }
    memset(out, 0, sizeof(double) * (size_t)n_targets * Din);
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l)
            for (int k = 0; k < K; ++k) {
                const int n = nbr[IDX3(b, k, l, K, N)];
                const int64_t row = slot[(int64_t)b * N + n];
                if (row < 0) continue;
                const double dx = (double)pos[IDX3(b, 0, n, 3, N)] - (double)pos[IDX3(b, 0, l, 3, N)];
                const double dy = (double)pos[IDX3(b, 1, n, 3, N)] - (double)pos[IDX3(b, 1, l, 3, N)];
                const double dz = (double)pos[IDX3(b, 2, n, 3, N)] - (double)pos[IDX3(b, 2, l, 3, N)];
                for (int c = 0; c < Din; ++c) {
                    double s = 0.0;
                    for (int o = 0; o < Dout; ++o) {
                        const double w = (double)theta[IDX3(0, c, o, Din, Dout)] * dx
                                       + (double)theta[IDX3(1, c, o, Din, Dout)] * dy
                                       + (double)theta[IDX3(2, c, o, Din, Dout)] * dz
                                       + (double)bias[(int64_t)c * Dout + o];
                        s += w * (double)grad_out[IDX3(b, o, l, Dout, N)];
                    }
#pragma omp atomic
                    out[row * Din + c] += s;
                }
            }
    free(slot);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Flex-max-pool forward (Sec. 4.1): out[b,c,l] = max_k feat[b,c,nbr[b,k,l]],
 * argmax[b,c,l] = index of the winning point (lowest point index on ties).
 * out is float (a bit copy of the winning input); out / argmax are [B,C,L].
 * ------------------------------------------------------------------------- */
int oracle_flexpool_fwd(const float *feat, const int32_t *nbr, float *out, int32_t *argmax,
                        int B, int N, int K, int C, int l_begin, int l_end)
{
    if (!feat || !nbr || !out || !argmax) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || C <= 0) return 2;
    if (l_begin < 0 || l_end > N || l_begin > l_end) return 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int l = l_begin; l < l_end; ++l)
            for (int c = 0; c < C; ++c) {
                int best = nbr[IDX3(b, 0, l, K, N)];
                float bv = feat[IDX3(b, c, best, C, N)];
                for (int k = 1; k < K; ++k) {
                    const int n = nbr[IDX3(b, k, l, K, N)];
                    const float v = feat[IDX3(b, c, n, C, N)];
                    if (v > bv || (v == bv && n < best)) { bv = v; best = n; }
                }
                out[IDX3(b, c, l - l_begin, C, l_end - l_begin)] = bv;
                argmax[IDX3(b, c, l - l_begin, C, l_end - l_begin)] = best;
            }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Flex-max-pool backward: grad_feat[b,c,m] = sum of grad_out[b,c,l] over the
 * centres l (in [l_begin,l_end)) whose recorded winner is m.  grad_out and
 * argmax are full [B,C,N] tensors; grad_feat is double [B,C,N], accumulated
 * into (pass it zero-filled).
 * ------------------------------------------------------------------------- */
int oracle_flexpool_bwd(const float *grad_out, const int32_t *argmax, double *grad_feat,
                        int B, int N, int C, int l_begin, int l_end)
{
    if (!grad_out || !argmax || !grad_feat) return 1;
    if (B <= 0 || N <= 0 || C <= 0) return 2;
    if (l_begin < 0 || l_end > N || l_begin > l_end) return 2;
    /* one (b,c) row per iteration: rows are independent, so no atomics */
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int l = l_begin; l < l_end; ++l) {
                const int m = argmax[IDX3(b, c, l, C, N)];
                grad_feat[IDX3(b, c, m, C, N)] += (double)grad_out[IDX3(b, c, l, C, N)];
            }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Flex-upsampling forward (Sec. 4.1, last paragraph before the architecture): the
 * features of the selected points are copied into the larger layer, every other
 * point starts at zero, then flex-max-pooling runs over the larger layer's
 * neighbourhoods.  sel[b,j] is the index, in the larger layer, of the smaller
 * layer's point j (distinct within a cloud).  Taken in exactly those steps:
 * a zero-filled [B,C,Nf] array, the copy, then the neighbourhood maximum with the
 * pooling layer's tie rule (lowest point index; -0 == +0 ties).
 * out / argmax are [B,C,L] for the centres [l_begin,l_end) of the larger layer;
 * argmax holds larger-layer point indices.
 * Returns 2 on bad sizes or a sel entry out of range, 3 on a repeated sel entry.
 * ------------------------------------------------------------------------- */
int oracle_flexupsample_fwd(const float *feat_small, const int32_t *sel, const int32_t *nbr,
                            float *out, int32_t *argmax, int B, int Ns, int Nf, int K, int C,
                            int l_begin, int l_end)
{
    if (!feat_small || !sel || !nbr || !out || !argmax) return 1;
    if (B <= 0 || Ns <= 0 || Nf <= 0 || K <= 0 || C <= 0 || Ns > Nf) return 2;
    if (l_begin < 0 || l_end > Nf || l_begin > l_end) return 2;
    float *dense = (float *)calloc((size_t)B * C * Nf, sizeof(float));
    unsigned char *taken = (unsigned char *)calloc((size_t)B * Nf, 1);
    if (!dense || !taken) { free(dense); free(taken); return 6; }
    int rc = 0;
    for (int b = 0; b < B && rc == 0; ++b)
        for (int j = 0; j < Ns; ++j) {
            const int m = sel[(int64_t)b * Ns + j];
            if (m < 0 || m >= Nf) { rc = 2; break; }
            if (taken[(int64_t)b * Nf + m]) { rc = 3; break; }
            taken[(int64_t)b * Nf + m] = 1;
            for (int c = 0; c < C; ++c) dense[IDX3(b, c, m, C, Nf)] = feat_small[IDX3(b, c, j, C, Ns)];
        }
    if (rc == 0) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int b = 0; b < B; ++b)
            for (int l = l_begin; l < l_end; ++l)
                for (int c = 0; c < C; ++c) {
                    int best = nbr[IDX3(b, 0, l, K, Nf)];
                    float bv = dense[IDX3(b, c, best, C, Nf)];
                    for (int k = 1; k < K; ++k) {
                        const int n = nbr[IDX3(b, k, l, K, Nf)];
                        const float v = dense[IDX3(b, c, n, C, Nf)];
                        if (v > bv || (v == bv && n < best)) { bv = v; best = n; }
                    }
                    out[IDX3(b, c, l - l_begin, C, l_end - l_begin)] = bv;
                    argmax[IDX3(b, c, l - l_begin, C, l_end - l_begin)] = best;
                }
    }
    free(dense); free(taken);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Flex-upsampling backward: the pooling step routes grad_out[b,c,l] to the winner
 * recorded in argmax (a larger-layer point); the copy step hands a selected point's
 * gradient to the smaller layer's point it came from, and the gradient of a point
 * that was only zero-filled is dropped.
 *   grad_small[b,c,j] = sum of grad_out[b,c,l] over centres l with argmax[b,c,l] = sel[b,j]
 * grad_small is double [B,C,Ns], overwritten.
 * ------------------------------------------------------------------------- */
int oracle_flexupsample_bwd(const float *grad_out, const int32_t *argmax, const int32_t *sel,
                            double *grad_small, int B, int Ns, int Nf, int C)
{
    if (!grad_out || !argmax || !sel || !grad_small) return 1;
    if (B <= 0 || Ns <= 0 || Nf <= 0 || C <= 0 || Ns > Nf) return 2;
    double *dense = (double *)calloc((size_t)B * C * Nf, sizeof(double));   /* gradient of the larger layer */
    if (!dense) return 6;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int l = 0; l < Nf; ++l) {
                const int m = argmax[IDX3(b, c, l, C, Nf)];
                if (m < 0 || m >= Nf) { free(dense); return 2; }
                dense[IDX3(b, c, m, C, Nf)] += (double)grad_out[IDX3(b, c, l, C, Nf)];
            }
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < Ns; ++j) {
            const int m = sel[(int64_t)b * Ns + j];
            if (m < 0 || m >= Nf) { free(dense); return 2; }
            for (int c = 0; c < C; ++c) grad_small[IDX3(b, c, j, C, Ns)] = dense[IDX3(b, c, m, C, Nf)];
        }
    free(dense);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Flex-max-pooling with subsampling (Sec. 4.1: pooling is applied before the
 * subsampling step; Sec. 4.3: the layer that ends an encoder stage).  Taken in
 * the paper's order: the neighbourhood maximum at EVERY point (pooling's tie
 * rule), then the columns of the kept points sel[b,j] are copied out.
 * out / argmax are [B,C,Ns]; argmax holds indices into the N points.
 * ------------------------------------------------------------------------- */
int oracle_flexpool_sub_fwd(const float *feat, const int32_t *nbr, const int32_t *sel,
                            float *out, int32_t *argmax, int B, int N, int Ns, int K, int C)
{
    if (!feat || !nbr || !sel || !out || !argmax) return 1;
    if (B <= 0 || N <= 0 || Ns <= 0 || K <= 0 || C <= 0 || Ns > N) return 2;
    float *pooled = (float *)malloc(sizeof(float) * (size_t)B * C * N);
    int32_t *winner = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * C * N);
    if (!pooled || !winner) { free(pooled); free(winner); return 6; }
    int rc = 0;
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l)
            for (int c = 0; c < C; ++c) {
                int best = nbr[IDX3(b, 0, l, K, N)];
                float bv = feat[IDX3(b, c, best, C, N)];
                for (int k = 1; k < K; ++k) {
                    const int n = nbr[IDX3(b, k, l, K, N)];
                    const float v = feat[IDX3(b, c, n, C, N)];
                    if (v > bv || (v == bv && n < best)) { bv = v; best = n; }
                }
                pooled[IDX3(b, c, l, C, N)] = bv;
                winner[IDX3(b, c, l, C, N)] = best;
            }
    for (int b = 0; b < B && rc == 0; ++b)
        for (int j = 0; j < Ns; ++j) {
            const int l = sel[(int64_t)b * Ns + j];
            if (l < 0 || l >= N) { rc = 2; break; }
            for (int c = 0; c < C; ++c) {
                out[IDX3(b, c, j, C, Ns)] = pooled[IDX3(b, c, l, C, N)];
                argmax[IDX3(b, c, j, C, Ns)] = winner[IDX3(b, c, l, C, N)];
            }
        }
    free(pooled); free(winner);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Backward of pooling with subsampling, in reverse order of the forward steps:
 * the subsampling step hands grad_out[b,c,j] to column sel[b,j] of the pooled
 * tensor's gradient (a point that was not kept gets zero; a point kept twice gets
 * both), the pooling step routes every column to its recorded winner.  The winner
 * of a kept centre is argmax[b,c,j] (the forward pass stores the table for the kept
 * centres only).  grad_feat is double [B,C,N], overwritten.
 * ------------------------------------------------------------------------- */
int oracle_flexpool_sub_bwd(const float *grad_out, const int32_t *argmax, const int32_t *sel,
                            double *grad_feat, int B, int N, int Ns, int C)
{
    if (!grad_out || !argmax || !sel || !grad_feat) return 1;
    if (B <= 0 || N <= 0 || Ns <= 0 || C <= 0 || Ns > N) return 2;
    double *gpooled = (double *)calloc((size_t)B * C * N, sizeof(double));
    int32_t *winner = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * C * N);
    if (!gpooled || !winner) { free(gpooled); free(winner); return 6; }
    for (int64_t i = 0; i < (int64_t)B * C * N; ++i) winner[i] = -1;
    int rc = 0;
    for (int b = 0; b < B && rc == 0; ++b)
        for (int j = 0; j < Ns; ++j) {
            const int l = sel[(int64_t)b * Ns + j];
            if (l < 0 || l >= N) { rc = 2; break; }
            for (int c = 0; c < C; ++c) {
                gpooled[IDX3(b, c, l, C, N)] += (double)grad_out[IDX3(b, c, j, C, Ns)];
                winner[IDX3(b, c, l, C, N)] = argmax[IDX3(b, c, j, C, Ns)];
            }
        }
    memset(grad_feat, 0, sizeof(double) * (size_t)B * C * N);
    for (int b = 0; b < B && rc == 0; ++b)
        for (int c = 0; c < C && rc == 0; ++c)
            for (int l = 0; l < N; ++l) {
                const int m = winner[IDX3(b, c, l, C, N)];
                if (m == -1) continue;                       /* not kept: no gradient arrives */
                if (m < 0 || m >= N) { rc = 2; break; }
                grad_feat[IDX3(b, c, m, C, N)] += gpooled[IDX3(b, c, l, C, N)];
            }
    free(gpooled); free(winner);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Flex-conv backward with respect to the point locations (Sec. 3.1: the weight
 * function is differentiable in all its arguments, so gradients pass through the
 * locations as well; no formula is printed).  Differentiating
 *   out[b,o,l] = sum_k sum_c ( <theta[:,c,o], pos[b,:,n] - pos[b,:,l]> + bias[c,o] ) * feat[b,c,n]
 * term by term: the edge (l,k) with n = nbr[b,k,l] carries
 *   s_d = sum_{c,o} theta[d,c,o] * feat[b,c,n] * grad_out[b,o,l]
 * to grad_pos[b,d,n] with a plus sign (the neighbour's location enters with +) and to
 * grad_pos[b,d,l] with a minus sign (the centre's with -); a point that lists itself
 * receives both and they cancel.  grad_pos is double [B,3,N], overwritten.
 * ------------------------------------------------------------------------- */
int oracle_flexconv_bwd_pos(const float *feat, const int32_t *nbr, const float *theta,
                            const float *grad_out, double *grad_pos,
                            int B, int N, int K, int Din, int Dout)
{
    if (!feat || !nbr || !theta || !grad_out || !grad_pos) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || Din <= 0 || Dout <= 0) return 2;
    memset(grad_pos, 0, sizeof(double) * (size_t)B * 3 * N);
    /* clouds are independent; inside a cloud the edges are taken one after the other */
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l)
            for (int k = 0; k < K; ++k) {
                const int n = nbr[IDX3(b, k, l, K, N)];
                for (int d = 0; d < 3; ++d) {
                    double s = 0.0;
                    for (int c = 0; c < Din; ++c) {
                        const double f = (double)feat[IDX3(b, c, n, Din, N)];
                        for (int o = 0; o < Dout; ++o)
                            s += (double)theta[IDX3(d, c, o, Din, Dout)] * f * (double)grad_out[IDX3(b, o, l, Dout, N)];
                    }
                    grad_pos[IDX3(b, d, n, 3, N)] += s;
                    grad_pos[IDX3(b, d, l, 3, N)] -= s;
                }
            }
    return 0;
}

/* ---------------------------------------------------------------------------
 * First two operations of the encoder's ResNet block (Sec. 4.3: 1x1-convolution, then
 * flex-convolution).  The paper names no bias for the 1x1 step and no activation between
 * the two, and none is applied here:
 *   mid[b,c,n] = sum_c0 W[c,c0] * feat[b,c0,n]                          (1x1 convolution)
 *   out[b,o,l] = sum_k sum_c ( <theta[:,c,o], pos[b,:,n]-pos[b,:,l]> + bias[c,o] ) * mid[b,c,n],
 *                n = nbr[b,k,l]                                          (Eq.(4) with Eq.(6))
 * taken in exactly these two steps, mid kept in double.  W is [Dmid,Din0]; out double [B,Dout,N].
 * ------------------------------------------------------------------------- */
int oracle_block_fwd(const float *feat, const float *pos, const int32_t *nbr, const float *W,
                     const float *theta, const float *bias, double *out,
                     int B, int N, int K, int Din0, int Dmid, int Dout)
{
    if (!feat || !pos || !nbr || !W || !theta || !bias || !out) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || Din0 <= 0 || Dmid <= 0 || Dout <= 0) return 2;
    double *mid = (double *)malloc(sizeof(double) * (size_t)B * Dmid * N);
    if (!mid) return 6;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < Dmid; ++c)
            for (int n = 0; n < N; ++n) {
                double s = 0.0;
                for (int c0 = 0; c0 < Din0; ++c0)
                    s += (double)W[(int64_t)c * Din0 + c0] * (double)feat[IDX3(b, c0, n, Din0, N)];
                mid[IDX3(b, c, n, Dmid, N)] = s;
            }
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l)
            for (int o = 0; o < Dout; ++o) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) {
                    const int n = nbr[IDX3(b, k, l, K, N)];
                    const double dx = (double)pos[IDX3(b, 0, n, 3, N)] - (double)pos[IDX3(b, 0, l, 3, N)];
                    const double dy = (double)pos[IDX3(b, 1, n, 3, N)] - (double)pos[IDX3(b, 1, l, 3, N)];
                    const double dz = (double)pos[IDX3(b, 2, n, 3, N)] - (double)pos[IDX3(b, 2, l, 3, N)];
                    for (int c = 0; c < Dmid; ++c) {
                        const double w = (double)theta[IDX3(0, c, o, Dmid, Dout)] * dx +
                                         (double)theta[IDX3(1, c, o, Dmid, Dout)] * dy +
                                         (double)theta[IDX3(2, c, o, Dmid, Dout)] * dz +
                                         (double)bias[(int64_t)c * Dout + o];
                        acc += w * mid[IDX3(b, c, n, Dmid, N)];
                    }
                }
                out[IDX3(b, o, l, Dout, N)] = acc;
            }
    free(mid);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Backward of that block, by the chain rule through the two steps (the paper prints no
 * formulas): with g = grad_out and the edge weight w(c,o) as above,
 *   grad_mid[b,c,n]    = sum over edges (l,k) with nbr[b,k,l] = n of sum_o w(c,o) * g[b,o,l]
 *   grad_theta[d,c,o]  = sum over edges of dp_d * mid[b,c,n] * g[b,o,l]
 *   grad_bias[c,o]     = sum over edges of mid[b,c,n] * g[b,o,l]
 *   grad_W[c,c0]       = sum_{b,n} grad_mid[b,c,n] * feat[b,c0,n]
 *   grad_feat[b,c0,n]  = sum_c W[c,c0] * grad_mid[b,c,n]
 * All outputs double, overwritten: grad_feat [B,Din0,N], grad_W [Dmid,Din0],
 * grad_theta [3,Dmid,Dout], grad_bias [Dmid,Dout].
 * ------------------------------------------------------------------------- */
int oracle_block_bwd(const float *feat, const float *pos, const int32_t *nbr, const float *W,
                     const float *theta, const float *bias, const float *grad_out,
                     double *grad_feat, double *grad_W, double *grad_theta, double *grad_bias,
                     int B, int N, int K, int Din0, int Dmid, int Dout)
{
    if (!feat || !pos || !nbr || !W || !theta || !bias || !grad_out) return 1;
    if (!grad_feat || !grad_W || !grad_theta || !grad_bias) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || Din0 <= 0 || Dmid <= 0 || Dout <= 0) return 2;
    double *mid = (double *)malloc(sizeof(double) * (size_t)B * Dmid * N);
    double *gmid = (double *)calloc((size_t)B * Dmid * N, sizeof(double));
    if (!mid || !gmid) { free(mid); free(gmid); return 6; }
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < Dmid; ++c)
            for (int n = 0; n < N; ++n) {
                double s = 0.0;
                for (int c0 = 0; c0 < Din0; ++c0)
                    s += (double)W[(int64_t)c * Din0 + c0] * (double)feat[IDX3(b, c0, n, Din0, N)];
                mid[IDX3(b, c, n, Dmid, N)] = s;
            }
    memset(grad_theta, 0, sizeof(double) * (size_t)3 * Dmid * Dout);
    memset(grad_bias, 0, sizeof(double) * (size_t)Dmid * Dout);
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l)
            for (int k = 0; k < K; ++k) {
                const int n = nbr[IDX3(b, k, l, K, N)];
                const double dp[3] = {(double)pos[IDX3(b, 0, n, 3, N)] - (double)pos[IDX3(b, 0, l, 3, N)],
                                      (double)pos[IDX3(b, 1, n, 3, N)] - (double)pos[IDX3(b, 1, l, 3, N)],
                                      (double)pos[IDX3(b, 2, n, 3, N)] - (double)pos[IDX3(b, 2, l, 3, N)]};
                for (int c = 0; c < Dmid; ++c) {
                    const double m = mid[IDX3(b, c, n, Dmid, N)];
                    double s = 0.0;
                    for (int o = 0; o < Dout; ++o) {
                        const double g = (double)grad_out[IDX3(b, o, l, Dout, N)];
                        const double w = (double)theta[IDX3(0, c, o, Dmid, Dout)] * dp[0] +
                                         (double)theta[IDX3(1, c, o, Dmid, Dout)] * dp[1] +
                                         (double)theta[IDX3(2, c, o, Dmid, Dout)] * dp[2] +
                                         (double)bias[(int64_t)c * Dout + o];
                        s += w * g;
                        for (int d = 0; d < 3; ++d) grad_theta[IDX3(d, c, o, Dmid, Dout)] += dp[d] * m * g;
                        grad_bias[(int64_t)c * Dout + o] += m * g;
                    }
                    gmid[IDX3(b, c, n, Dmid, N)] += s;
                }
            }
    for (int c = 0; c < Dmid; ++c)
        for (int c0 = 0; c0 < Din0; ++c0) {
            double s = 0.0;
            for (int b = 0; b < B; ++b)
                for (int n = 0; n < N; ++n) s += gmid[IDX3(b, c, n, Dmid, N)] * (double)feat[IDX3(b, c0, n, Din0, N)];
            grad_W[(int64_t)c * Din0 + c0] = s;
        }
    for (int b = 0; b < B; ++b)
        for (int c0 = 0; c0 < Din0; ++c0)
            for (int n = 0; n < N; ++n) {
                double s = 0.0;
                for (int c = 0; c < Dmid; ++c) s += (double)W[(int64_t)c * Din0 + c0] * gmid[IDX3(b, c, n, Dmid, N)];
                grad_feat[IDX3(b, c0, n, Din0, N)] = s;
            }
    free(mid); free(gmid);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Inverse density importance sub-sampling (Sec. 3.2).
 * Step 1: phi[b,l] = sum over the neighbourhood of the distances ||pos[l] - pos[n]|| (the
 * paper's approximation of the inverse density).  phi is double [B,N].
 * ------------------------------------------------------------------------- */
int oracle_idiss_phi(const float *pos, const int32_t *nbr, double *phi, int B, int N, int K)
{
    if (!pos || !nbr || !phi) return 1;
    if (B <= 0 || N <= 0 || K <= 0) return 2;
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) {
                const int n = nbr[IDX3(b, k, l, K, N)];
                double d2 = 0.0;
                for (int d = 0; d < 3; ++d) {
                    const double t = (double)pos[IDX3(b, d, n, 3, N)] - (double)pos[IDX3(b, d, l, 3, N)];
                    d2 += t * t;
                }
                s += sqrt(d2);
            }
            phi[(int64_t)b * N + l] = s;
        }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Step 2: draw Ns points of every cloud with probability proportional to phi, in one
 * pass over the points (the paper states proportional sampling in O(n) and fixes no
 * procedure; this is the reading taken: stratified sampling on the running sum).
 * So that every decision is an integer comparison (the same on any machine, in any
 * summation order), phi is first put on an integer scale:
 *   q[l] = floor(phi[l] * (2^bits / max_l phi[l]))   in float arithmetic, one division and
 *          one product, bits = min(28, 51 - ceil(log2 N));  all q = 1 if the maximum is 0
 *   C[l] = q[0] + ... + q[l],  Q = C[N-1]
 * The range [0,Q) is cut into Ns strata, stratum j = [start_j, start_j + len_j) with
 * len_j = Q / Ns (+1 for the first Q mod Ns strata); the caller's random word u[b,j]
 * places one threshold in it, t_j = start_j + floor(u[b,j] * len_j / 2^32), and
 * sel[b,j] = the first point with C[l] > t_j.  sel is ascending; a point whose q spans
 * several thresholds is drawn for each of them (drawing with replacement), a point with
 * q = 0 is never drawn.  Returns 2 when Q < Ns (fewer units than strata).
 * ------------------------------------------------------------------------- */
int oracle_idiss_sample(const float *phi, const uint32_t *u, int32_t *sel, int B, int N, int Ns)
{
    if (!phi || !u || !sel) return 1;
    if (B <= 0 || N <= 0 || Ns <= 0 || Ns > N) return 2;
    int lg = 0;
    while (((int64_t)1 << lg) < N) ++lg;
    const int bits = (51 - lg) < 28 ? (51 - lg) : 28;
    if (bits < 1) return 2;
    uint64_t *C = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)N);
    if (!C) return 6;
    int rc = 0;
    for (int b = 0; b < B && rc == 0; ++b) {
        const float *ph = phi + (int64_t)b * N;
        float mx = 0.f;
        for (int l = 0; l < N; ++l) {
            if (!(ph[l] >= 0.f)) { rc = 2; break; }          /* negative or NaN */
            if (ph[l] > mx) mx = ph[l];
        }
        if (rc) break;
        const float scale = (mx > 0.f) ? (float)((int64_t)1 << bits) / mx : 0.f;
        uint64_t run = 0;
        for (int l = 0; l < N; ++l) {
            const uint32_t q = (mx > 0.f) ? (uint32_t)(ph[l] * scale) : 1u;
            run += q;
            C[l] = run;
        }
        const uint64_t Q = run;
        if (Q < (uint64_t)Ns) { rc = 2; break; }
        const uint64_t width = Q / (uint64_t)Ns, rem = Q % (uint64_t)Ns;
        int l = 0;
        for (int j = 0; j < Ns; ++j) {
            const uint64_t start = (uint64_t)j * width + ((uint64_t)j < rem ? (uint64_t)j : rem);
            const uint64_t len = width + ((uint64_t)j < rem ? 1u : 0u);
            const uint64_t t = start + (uint64_t)(((unsigned __int128)u[(int64_t)b * Ns + j] * len) >> 32);
            while (C[l] <= t) ++l;                            /* thresholds ascend, so the walk never goes back */
            sel[(int64_t)b * Ns + j] = l;
        }
    }
    free(C);
    return rc;
}

/* ---------------------------------------------------------------------------
 * K nearest neighbours by exhaustive search (Sec. 3: neighbourhoods are the k nearest
 * points; the paper computes them beforehand and does not say how).  For every point l the
 * K points of its cloud with the smallest squared distance, the point itself included,
 * ordered by (d2 ascending, index ascending); equal d2 are broken by the LOWER INDEX.
 * d2 is evaluated in float, exactly as ((dx*dx + dy*dy) + dz*dz) with dx = pos[n] - pos[l]
 * and every operation rounded on its own (no fused multiply-add: build with
 * -ffp-contract=off), because the ranking is an integer-valued decision that both this
 * code and the library must take in the same precision.  nbr is int32 [B,K,N].
 * ------------------------------------------------------------------------- */
int oracle_knn(const float *pos, int32_t *nbr, int B, int N, int K)
{
    if (!pos || !nbr) return 1;
    if (B <= 0 || N <= 0 || K <= 0 || K > N) return 2;
    int rc = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 64)
    for (int b = 0; b < B; ++b)
        for (int l = 0; l < N; ++l) {
            const float *px = pos + IDX3(b, 0, 0, 3, N), *py = px + N, *pz = py + N;
            float *bd = (float *)malloc(sizeof(float) * (size_t)K);
            int32_t *bi = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
            if (!bd || !bi) { rc = 6; free(bd); free(bi); continue; }
            int have = 0;
            for (int n = 0; n < N; ++n) {
                const float dx = px[n] - px[l], dy = py[n] - py[l], dz = pz[n] - pz[l];
                const float xx = dx * dx, yy = dy * dy, zz = dz * dz;
                const float xy = xx + yy;
                const float d2 = xy + zz;
                /* n ascends, so among equal d2 the earlier (lower) index already sits in front */
                if (have == K && !(d2 < bd[K - 1])) continue;
                int at = have < K ? have : K - 1;
                while (at > 0 && d2 < bd[at - 1]) { bd[at] = bd[at - 1]; bi[at] = bi[at - 1]; --at; }
                bd[at] = d2; bi[at] = n;
                if (have < K) ++have;
            }
            for (int k = 0; k < K; ++k) nbr[IDX3(b, k, l, K, N)] = bi[k];
            free(bd); free(bi);
        }
    return rc;
}

/* ---------------------------------------------------------------------------
 * Repeats removed from an ascending selection (the stratified draw above returns a point
 * once per threshold it spans; the layers that copy features between resolutions need
 * distinct points).  The paper does not say how its sampling treats repeats; the reading
 * taken keeps the draw and moves every repeated entry to the next free index:
 *   walking j = 1 .. Ns-1:  if sel[j] <= sel[j-1] then sel[j] = sel[j-1] + 1
 * and, should that run past the end of the cloud, the tail is packed against it:
 *   walking j = Ns-1 .. 0:  sel[j] = min(sel[j], N - Ns + j).
 * In place, int32 [B,Ns]; input must be ascending with entries in [0,N).
 * ------------------------------------------------------------------------- */
int oracle_selection_make_distinct(int32_t *sel, int B, int N, int Ns)
{
    if (!sel) return 1;
    if (B <= 0 || N <= 0 || Ns <= 0 || Ns > N) return 2;
    for (int b = 0; b < B; ++b) {
        int32_t *s = sel + (int64_t)b * Ns;
        for (int j = 0; j < Ns; ++j) {
            if (s[j] < 0 || s[j] >= N) return 2;
            if (j > 0 && s[j] < s[j - 1]) return 2;              /* ascending input required */
        }
        for (int j = 1; j < Ns; ++j)
            if (s[j] <= s[j - 1]) s[j] = s[j - 1] + 1;
        for (int j = Ns - 1; j >= 0; --j)
            if (s[j] > N - Ns + j) s[j] = N - Ns + j;
    }
    return 0;
}
