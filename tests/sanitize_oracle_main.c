/* Driver for a sanitizer build of the CPU oracle (tests/test_oracle_sanitizers.py compiles oracle/oracle.c together
 * with this file under -fsanitize=address,undefined and runs it): every oracle function once on a small seeded
 * problem with exactly sized heap buffers, so that an out-of-bounds index or an overflow in the oracle aborts. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_flexconv_fwd(const float *, const float *, const int32_t *, const float *, const float *, double *, int, int, int, int, int, int, int);
int oracle_flexconv_bwd(const float *, const float *, const int32_t *, const float *, const float *, const float *, double *, double *, double *, int, int, int, int, int, int, int);
int oracle_flexpool_fwd(const float *, const int32_t *, float *, int32_t *, int, int, int, int, int, int);
int oracle_flexpool_bwd(const float *, const int32_t *, double *, int, int, int, int, int);
int oracle_flexupsample_fwd(const float *, const int32_t *, const int32_t *, float *, int32_t *, int, int, int, int, int, int, int);
int oracle_flexupsample_bwd(const float *, const int32_t *, const int32_t *, double *, int, int, int, int);
int oracle_flexpool_sub_fwd(const float *, const int32_t *, const int32_t *, float *, int32_t *, int, int, int, int, int);
int oracle_flexpool_sub_bwd(const float *, const int32_t *, const int32_t *, double *, int, int, int, int);
int oracle_flexconv_bwd_pos(const float *, const int32_t *, const float *, const float *, double *, int, int, int, int, int);
int oracle_block_fwd(const float *, const float *, const int32_t *, const float *, const float *, const float *, double *, int, int, int, int, int, int);
int oracle_block_bwd(const float *, const float *, const int32_t *, const float *, const float *, const float *, const float *, double *, double *, double *, double *, int, int, int, int, int, int);
int oracle_idiss_phi(const float *, const int32_t *, double *, int, int, int);
int oracle_idiss_sample(const float *, const uint32_t *, int32_t *, int, int, int);
int oracle_knn(const float *, int32_t *, int, int, int);
int oracle_selection_make_distinct(int32_t *, int, int, int);

static uint32_t state = 12345u;
static uint32_t rnd(void) { state = state * 1664525u + 1013904223u; return state >> 8; }
static float *fl(size_t n) { float *p = malloc(sizeof(float) * n); for (size_t i = 0; i < n; ++i) p[i] = (float)(rnd() % 2001) / 1000.f - 1.f; return p; }
static double *db(size_t n) { return calloc(n, sizeof(double)); }
#define CHECK(x) do { int rc_ = (x); if (rc_) { printf("FAILED %s -> %d\n", #x, rc_); return 1; } } while (0)

int main(void)
{
    enum { B = 2, N = 37, K = 5, Din = 3, Dmid = 4, Dout = 2, Ns = 9 };
    float *feat = fl(B * Din * N), *pos = fl(B * 3 * N), *theta = fl(3 * Din * Dout), *bias = fl(Din * Dout);
    float *g = fl(B * Dout * N), *W = fl(Dmid * Din), *theta2 = fl(3 * Dmid * Dout), *bias2 = fl(Dmid * Dout);
    int32_t *nbr = malloc(sizeof(int32_t) * B * K * N), *nn = malloc(sizeof(int32_t) * B * K * N);
    for (int i = 0; i < B * K * N; ++i) nbr[i] = (int32_t)(rnd() % N);
    double *out = db(B * Dout * N), *gf = db(B * Din * N), *gt = db(3 * Din * Dout), *gb = db(Din * Dout), *gp = db(B * 3 * N);
    CHECK(oracle_flexconv_fwd(feat, pos, nbr, theta, bias, out, B, N, K, Din, Dout, 0, N));
    CHECK(oracle_flexconv_bwd(feat, pos, nbr, theta, bias, g, gf, gt, gb, B, N, K, Din, Dout, 0, N));
    CHECK(oracle_flexconv_bwd_pos(feat, nbr, theta, g, gp, B, N, K, Din, Dout));
    float *po = malloc(sizeof(float) * B * Din * N); int32_t *pa = malloc(sizeof(int32_t) * B * Din * N);
    CHECK(oracle_flexpool_fwd(feat, nbr, po, pa, B, N, K, Din, 0, N));
    float *gpool = fl(B * Din * N);
    CHECK(oracle_flexpool_bwd(gpool, pa, gf, B, N, Din, 0, N));
    int32_t *sel = malloc(sizeof(int32_t) * B * Ns);
    for (int b = 0; b < B; ++b) for (int j = 0; j < Ns; ++j) sel[b * Ns + j] = 4 * j + b;      /* distinct, ascending */
    float *fs = fl(B * Din * Ns), *uo = malloc(sizeof(float) * B * Din * N); int32_t *ua = malloc(sizeof(int32_t) * B * Din * N);
    double *gs = db(B * Din * Ns);
    CHECK(oracle_flexupsample_fwd(fs, sel, nbr, uo, ua, B, Ns, N, K, Din, 0, N));
    CHECK(oracle_flexupsample_bwd(gpool, ua, sel, gs, B, Ns, N, Din));
    float *so = malloc(sizeof(float) * B * Din * Ns); int32_t *sa = malloc(sizeof(int32_t) * B * Din * Ns);
    CHECK(oracle_flexpool_sub_fwd(feat, nbr, sel, so, sa, B, N, Ns, K, Din));
    CHECK(oracle_flexpool_sub_bwd(fs, sa, sel, gf, B, N, Ns, Din));
    double *bo = db(B * Dout * N), *bgf = db(B * Din * N), *bgW = db(Dmid * Din), *bgt = db(3 * Dmid * Dout), *bgb = db(Dmid * Dout);
    CHECK(oracle_block_fwd(feat, pos, nbr, W, theta2, bias2, bo, B, N, K, Din, Dmid, Dout));
    CHECK(oracle_block_bwd(feat, pos, nbr, W, theta2, bias2, g, bgf, bgW, bgt, bgb, B, N, K, Din, Dmid, Dout));
    double *phi = db(B * N);
    CHECK(oracle_idiss_phi(pos, nbr, phi, B, N, K));
    float *phif = malloc(sizeof(float) * B * N); for (int i = 0; i < B * N; ++i) phif[i] = (float)phi[i];
    uint32_t *u = malloc(sizeof(uint32_t) * B * Ns); for (int i = 0; i < B * Ns; ++i) u[i] = rnd() * 256u + (rnd() & 255u);
    CHECK(oracle_idiss_sample(phif, u, sel, B, N, Ns));
    CHECK(oracle_selection_make_distinct(sel, B, N, Ns));
    CHECK(oracle_knn(pos, nn, B, N, K));
    CHECK(oracle_knn(pos, nn, B, N, 1));
    printf("sanitizer run ok\n");
    free(feat); free(pos); free(theta); free(bias); free(g); free(W); free(theta2); free(bias2); free(nbr); free(nn);
    free(out); free(gf); free(gt); free(gb); free(gp); free(po); free(pa); free(gpool); free(sel); free(fs); free(uo);
    free(ua); free(gs); free(so); free(sa); free(bo); free(bgf); free(bgW); free(bgt); free(bgb); free(phi); free(phif); free(u);
    return 0;
}
