// Small support kernels: parameter packing, layout transposes, the partial-sum
// reduction of grad_theta, range check, zero fill, and the generic (any
// Din/Dout) direct-form flex-conv kernels used when no tiled kernel fits.
#include "flex_common.hpp"

namespace flex {

int device_cu_count()
{
    static int cached = 0;
    if (cached == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cached = n;
        else
            cached = 256;   // MI355X; also the answer on a host without a GPU
    }
    return cached;
}

int persistent_grid(int64_t total_tiles, int wg_per_cu)
{
    int64_t g = (int64_t)device_cu_count() * wg_per_cu;
    if (total_tiles < g) g = total_tiles;
    if (g < 8) g = 8;
    return (int)((g + 7) / 8 * 8);
}

// ---- theta packing ----------------------------------------------------------
__global__ void pack_theta_kernel(const float *__restrict__ theta, const float *__restrict__ bias,
                                  float *__restrict__ thetaP, int Din, int Dout, int RP, int CP,
                                  int transpose)
{
    const int total = 4 * RP * CP;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int c = i % CP, r = (i / CP) % RP, j = i / (CP * RP);
        const int ci = transpose ? c : r;   // input channel
        const int co = transpose ? r : c;   // output channel
        float v = 0.f;
        if (ci < Din && co < Dout)
            v = (j < 3) ? theta[((int64_t)j * Din + ci) * Dout + co] : bias[(int64_t)ci * Dout + co];
        thetaP[i] = v;
    }
}

hipError_t launch_pack_theta(const float *theta, const float *bias, float *thetaP, int Din,
                             int Dout, int RP, int CP, int transpose, hipStream_t s)
{
    const int total = 4 * RP * CP;
    const int blocks = (total + 255) / 256;
    hipLaunchKernelGGL(pack_theta_kernel, dim3(blocks > 1024 ? 1024 : blocks), dim3(256), 0, s,
                       theta, bias, thetaP, Din, Dout, RP, CP, transpose);
    return hipGetLastError();
}

// ---- theta packing for the split-half contraction ---------------------------------
// The wave-specialised kernels contract on the f16 matrix cores with every fp32
// operand x carried as two halves of a scaled x:  hi = half(x s), lo = half(x s - hi),
// and the three products hi*hi + hi*lo + lo*hi (error ~2^-22 per product, the level
// of fp32 rounding) -- as long as x s stays within f16's normal range, i.e. within
// about 2^17 of the largest scaled magnitude.  Scaling by powers of two is exact, so the
// packing equilibrates the matrix first, in both directions:
//   row kd (a depth index: component j, gathered channel) gets 2^er[kd] so that its largest
//       magnitude is in [1/2, 1); the aggregate's column kd is multiplied by 2^-er[kd]
//       (rscale[kd], applied by the producers before their split), so a gathered channel of
//       small magnitude whose parameters are large (or the other way round) keeps its bits;
//   column o (an output channel) then gets 2^ec[o] so that its largest magnitude is in
//       [2^14, 2^15); the consumers undo it with the per-point exponent.
//   ThetaS[kd][o] = ThetaP[kd][o] * 2^(er[kd] + ec[o]);  out[l][o] = 2^-(e_l + ec[o]) * sum_kd As[l][kd] ThetaS[kd][o],
//   As[l][kd] = A[l][kd] * 2^-er[kd] * 2^e_l  (e_l: the point's own exponent, store_split_rows).
// What is left inside one row and column after that (entries of the SAME channel pair block far
// below their neighbours) contributes to the output in proportion to its size, as in any
// fp32 product.  er is clamped to +-60 so that no scale leaves fp32's normal range.
// Buffer layout (halves), the operand fragments of v_mfma_f32_16x16x32_f16 in the order
// a wave loads them:
//   thetaF[(((part*NS + slice)*KS + step)*64 + lane)*8 + e]
//       = part( ThetaS[32*step + 8*(lane>>4) + e][16*slice + (lane&15)] )
// with NS = CP/16 slices, KS = KDP/32 depth steps, rows >= 4*RP and padding zero; then, at
// byte offset theta_f16_exp_offset(RP, CP): int32 ec[CP], and at theta_f16_rscale_offset(RP, CP):
// float rscale[KDP] (1 for padding rows).
struct ThetaView {
    const float *theta, *bias;
    int Din, Dout, ci0, co0, transpose, RP;
    // element (kd = j*RP + r, col) of the (possibly transposed) block that starts at (ci0, co0)
    __device__ __forceinline__ float at(int kd, int col) const
    {
        const int j = kd / RP, r = kd - j * RP;
        const int ci = ci0 + (transpose ? col : r), co = co0 + (transpose ? r : col);
        if (ci >= Din || co >= Dout) return 0.f;
        return (j < 3) ? theta[((int64_t)j * Din + ci) * Dout + co] : bias[(int64_t)ci * Dout + co];
    }
};

constexpr int PACK_MAX_KD = 512, PACK_MAX_CP = 128;

// one workgroup of 1024 threads packs one matrix (KD = 4*RP <= PACK_MAX_KD rows, CP <= PACK_MAX_CP columns).
// Every thread keeps its share of the matrix in registers, taken in the order of the fragment buffer it will
// write (element i = tid + 1024 * j), so the parameters are read once; the row / column maxima are maxima of
// non-negative floats taken as integers with LDS atomics.
__device__ __forceinline__ void pack_theta_f16_block(const ThetaView &v, _Float16 *__restrict__ thetaF, int CP,
                                                     int exp_offset_bytes, int rscale_offset_bytes, int *s_er,
                                                     int *s_ec)
{
    constexpr int MAXE = PACK_MAX_KD * PACK_MAX_CP / 1024;      // elements per thread at the largest shape
    const int KD = 4 * v.RP, KDP = (KD + 31) / 32 * 32, KS = KDP / 32, NS = CP / 16;
    const int per_part = NS * KS * 64 * 8;                      // = KDP * CP, a multiple of 512
    const int n_mine = (per_part - (int)threadIdx.x + 1023) / 1024;   // elements tid, tid + 1024, ...
    float x[MAXE];
    for (int i = threadIdx.x; i < KDP; i += 1024) s_er[i] = 0;
    for (int i = threadIdx.x; i < CP; i += 1024) s_ec[i] = 0;
    __syncthreads();
    // fragment element i = ((slice * KS + step) * 64 + lane) * 8 + e holds (kd, col) = (32 step + 8 (lane >> 4) + e,
    // 16 slice + (lane & 15)); i = tid + 1024 j walks (slice, step) two steps at a time from tid >> 9
    const int kd_lo = 8 * (((int)threadIdx.x >> 7) & 3) + ((int)threadIdx.x & 7), col_lo = ((int)threadIdx.x >> 3) & 15;
    struct Walk {
        int step, slice, KS;
        __device__ __forceinline__ void next() { step += 2; while (step >= KS) { step -= KS; ++slice; } }
    };
    auto start = [&]() { Walk w{(int)threadIdx.x >> 9, 0, KS}; while (w.step >= KS) { w.step -= KS; ++w.slice; } return w; };
    {
        Walk w = start();
#pragma unroll
        for (int j = 0; j < MAXE; ++j) {
            if (j >= n_mine) break;
            const int kd = 32 * w.step + kd_lo, col = 16 * w.slice + col_lo;
            x[j] = (kd < KD) ? v.at(kd, col) : 0.f;
            const float a = fabsf(x[j]);
            if (a > 0.f && a < __builtin_inff()) atomicMax(&s_er[kd], __float_as_int(a));
            w.next();
        }
    }
    __syncthreads();
    for (int kd = threadIdx.x; kd < KDP; kd += 1024) {
        const float m = __int_as_float(s_er[kd]);
        int er = 0;
        if (m > 0.f) { (void)frexpf(m, &er); er = -er; }
        er = er < -60 ? -60 : (er > 60 ? 60 : er);
        s_er[kd] = er;
        reinterpret_cast<float *>(reinterpret_cast<char *>(thetaF) + rscale_offset_bytes)[kd] = ldexpf(1.f, -er);
    }
    __syncthreads();
    {
        Walk w = start();
#pragma unroll
        for (int j = 0; j < MAXE; ++j) {
            if (j >= n_mine) break;
            x[j] = ldexpf(x[j], s_er[32 * w.step + kd_lo]);
            const float a = fabsf(x[j]);
            if (a > 0.f && a < __builtin_inff()) atomicMax(&s_ec[16 * w.slice + col_lo], __float_as_int(a));
            w.next();
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < CP; c += 1024) {
        const float m = __int_as_float(s_ec[c]);
        int ec = 0;
        if (m > 0.f) { (void)frexpf(m, &ec); ec = 15 - ec; }
        s_ec[c] = ec;
        reinterpret_cast<int *>(reinterpret_cast<char *>(thetaF) + exp_offset_bytes)[c] = ec;
    }
    __syncthreads();
    {
        Walk w = start();
#pragma unroll
        for (int j = 0; j < MAXE; ++j) {
            if (j >= n_mine) break;
            const float vs = ldexpf(x[j], s_ec[16 * w.slice + col_lo]);
            const _Float16 hi = (_Float16)vs;
            const _Float16 lo = (_Float16)(vs - (float)hi);
            thetaF[threadIdx.x + 1024 * j] = hi;
            thetaF[per_part + threadIdx.x + 1024 * j] = lo;
            w.next();
        }
    }
}

__global__ __launch_bounds__(1024) void pack_theta_f16_kernel(const float *__restrict__ theta,
                                                              const float *__restrict__ bias,
                                                              _Float16 *__restrict__ thetaF, int Din,
                                                              int Dout, int RP, int CP, int transpose,
                                                              int exp_offset_bytes, int rscale_offset_bytes)
{
    __shared__ int s_er[PACK_MAX_KD], s_ec[PACK_MAX_CP];
    const ThetaView v{theta, bias, Din, Dout, 0, 0, transpose, RP};
    pack_theta_f16_block(v, thetaF, CP, exp_offset_bytes, rscale_offset_bytes, s_er, s_ec);
}

// The parameters of a wide layer as a grid of blocks, each packed like a whole layer's (same buffer layout, its own
// exponents), one workgroup per block.  transpose == 0: block (i, j) = input channels r_blk*i.., output channels
// c_blk*j.. (depth = input channel).  transpose == 1: block (i, j) = output channels r_blk*i.., input channels
// c_blk*j.., packed transposed (depth = output channel).  Block (i, j) lands at index j * n_i + i.
__global__ __launch_bounds__(1024) void pack_theta_f16_blocks_kernel(const float *__restrict__ theta,
                                                                     const float *__restrict__ bias,
                                                                     char *__restrict__ thetaF_all, int Din, int Dout,
                                                                     int r_blk, int c_blk, int n_i, int transpose,
                                                                     int block_bytes, int exp_offset_bytes,
                                                                     int rscale_offset_bytes)
{
    __shared__ int s_er[PACK_MAX_KD], s_ec[PACK_MAX_CP];
    const int i_blk = blockIdx.x % n_i, j_blk = blockIdx.x / n_i;
    _Float16 *thetaF = reinterpret_cast<_Float16 *>(thetaF_all + (size_t)blockIdx.x * block_bytes);
    // the block's first input / output channel
    const int ci0 = transpose ? c_blk * j_blk : r_blk * i_blk, co0 = transpose ? r_blk * i_blk : c_blk * j_blk;
    const ThetaView v{theta, bias, Din, Dout, ci0, co0, transpose, r_blk};
    pack_theta_f16_block(v, thetaF, c_blk, exp_offset_bytes, rscale_offset_bytes, s_er, s_ec);
}

hipError_t launch_pack_theta_f16_blocks(const float *theta, const float *bias, void *thetaF_all, int Din, int Dout,
                                        int r_blk, int c_blk, int n_i, int n_j, int transpose, hipStream_t s)
{
    if (4 * r_blk > PACK_MAX_KD || c_blk > PACK_MAX_CP || c_blk % 16 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_theta_f16_blocks_kernel, dim3((unsigned)(n_i * n_j)), dim3(1024), 0, s, theta, bias,
                       (char *)thetaF_all, Din, Dout, r_blk, c_blk, n_i, transpose,
                       (int)theta_f16_bytes(r_blk, c_blk), (int)theta_f16_exp_offset(r_blk, c_blk),
                       (int)theta_f16_rscale_offset(r_blk, c_blk));
    return hipGetLastError();
}

size_t theta_f16_exp_offset(int RP, int CP)
{
    const int KDP = (4 * RP + 31) / 32 * 32;
    return align256(sizeof(_Float16) * (size_t)2 * CP * KDP);
}
size_t theta_f16_rscale_offset(int RP, int CP) { return theta_f16_exp_offset(RP, CP) + align256(sizeof(int) * (size_t)CP); }
size_t theta_f16_bytes(int RP, int CP)
{
    const int KDP = (4 * RP + 31) / 32 * 32;
    return theta_f16_rscale_offset(RP, CP) + align256(sizeof(float) * (size_t)KDP);
}

hipError_t launch_pack_theta_f16(const float *theta, const float *bias, void *thetaF, int Din,
                                 int Dout, int RP, int CP, int transpose, hipStream_t s)
{
    if (4 * RP > PACK_MAX_KD || CP > PACK_MAX_CP || CP % 16 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_theta_f16_kernel, dim3(1), dim3(1024), 0, s, theta, bias,
                       (_Float16 *)thetaF, Din, Dout, RP, CP, transpose, (int)theta_f16_exp_offset(RP, CP),
                       (int)theta_f16_rscale_offset(RP, CP));
    return hipGetLastError();
}

// ---- theta fragments for the location-gradient kernel --------------------------------
// Theta_d = theta[d] (transpose == 0: depth = input channel, columns = output channel) or its
// transpose (transpose == 1), d = x, y, z, split-half with one exponent for all three:
//   thetaF[((((2*d + part)*NS + slice)*KS + step)*64 + lane)*8 + e]
//       = part( Theta_d[32*step + 8*(lane>>4) + e][16*slice + (lane&15)] * 2^e_theta ),
// NS = CP/16, KS = KDP/32, zero outside the matrix; int32 e_theta at theta_pos_exp_offset(KDP, CP).
__global__ __launch_bounds__(1024) void pack_theta_pos_f16_kernel(const float *__restrict__ theta,
                                                                  _Float16 *__restrict__ thetaF, int Din,
                                                                  int Dout, int KDP, int CP, int transpose,
                                                                  int exp_offset_bytes)
{
    __shared__ float s_max[1024];
    const int n_theta = 3 * Din * Dout;
    float m = 0.f;
    for (int i = threadIdx.x; i < n_theta; i += 1024) m = fmaxf(m, fabsf(theta[i]));
    s_max[threadIdx.x] = m;
    __syncthreads();
    for (int d = 512; d > 0; d >>= 1) {
        if ((int)threadIdx.x < d) s_max[threadIdx.x] = fmaxf(s_max[threadIdx.x], s_max[threadIdx.x + d]);
        __syncthreads();
    }
    m = s_max[0];
    int ex = 0;
    if (m > 0.f && m < __builtin_inff()) { (void)frexpf(m, &ex); ex = 15 - ex; }
    if (threadIdx.x == 0) *reinterpret_cast<int *>(reinterpret_cast<char *>(thetaF) + exp_offset_bytes) = ex;

    const int KS = KDP / 32, NS = CP / 16;
    const int per_part = NS * KS * 64 * 8;
    const int depth = transpose ? Dout : Din, cols = transpose ? Din : Dout;
    for (int i = threadIdx.x; i < 3 * per_part; i += 1024) {
        const int d = i / per_part, j = i % per_part;
        const int e = j & 7, lane = (j >> 3) & 63, step = (j >> 9) % KS, slice = (j >> 9) / KS;
        const int kd = 32 * step + 8 * (lane >> 4) + e, col = 16 * slice + (lane & 15);
        float v = 0.f;
        if (kd < depth && col < cols) {
            const int ci = transpose ? col : kd, co = transpose ? kd : col;
            v = theta[((int64_t)d * Din + ci) * Dout + co];
        }
        const float vs = ldexpf(v, ex);
        const _Float16 hi = (_Float16)vs;
        thetaF[(2 * d) * per_part + j] = hi;
        thetaF[(2 * d + 1) * per_part + j] = (_Float16)(vs - (float)hi);
    }
}

size_t theta_pos_exp_offset(int KDP, int CP) { return align256(sizeof(_Float16) * (size_t)6 * CP * KDP); }
size_t theta_pos_bytes(int KDP, int CP) { return theta_pos_exp_offset(KDP, CP) + 256; }

hipError_t launch_pack_theta_pos(const float *theta, void *thetaF, int Din, int Dout, int KDP, int CP,
                                 int transpose, hipStream_t s)
{
    hipLaunchKernelGGL(pack_theta_pos_f16_kernel, dim3(1), dim3(1024), 0, s, theta, (_Float16 *)thetaF, Din,
                       Dout, KDP, CP, transpose, (int)theta_pos_exp_offset(KDP, CP));
    return hipGetLastError();
}

// ---- [B,R,C] -> [B,C,R] transposes (64x64 tiles through LDS) -----------------
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ src,
                                                        float *__restrict__ dst, int R, int C,
                                                        int tiles_r, int tiles_c)
{
    __shared__ float tile[64][65];
    const int64_t t = blockIdx.x;
    const int tc = (int)(t % tiles_c);
    const int tr = (int)((t / tiles_c) % tiles_r);
    const int64_t b = t / ((int64_t)tiles_c * tiles_r);
    const float *s = src + b * (int64_t)R * C;
    float *d = dst + b * (int64_t)R * C;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int r0 = tr * 64, c0 = tc * 64;
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < R && c < C) ? s[(int64_t)r * C + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (r < R && c < C) d[(int64_t)c * R + r] = tile[tx][i];
    }
}

// The same with 16-byte accesses on both sides (R, C multiples of 4, 16-byte aligned tensors): thread
// (ty, tx) moves four consecutive floats of rows ty, ty+16, .. in, and of columns ty, ty+16, .. out.
__global__ __launch_bounds__(256) void transpose_vec4_kernel(const float *__restrict__ src,
                                                             float *__restrict__ dst, int R, int C,
                                                             int tiles_r, int tiles_c)
{
    __shared__ float tile[64][65];
    const int64_t t = blockIdx.x;
    const int tc = (int)(t % tiles_c);
    const int tr = (int)((t / tiles_c) % tiles_r);
    const int64_t b = t / ((int64_t)tiles_c * tiles_r);
    const float *s = src + b * (int64_t)R * C;
    float *d = dst + b * (int64_t)R * C;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int r0 = tr * 64, c0 = tc * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rl = ty + 16 * i, r = r0 + rl, c = c0 + 4 * tx;
        v4f v = {0.f, 0.f, 0.f, 0.f};
        if (r < R && c < C) v = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(s + (int64_t)r * C + c));
        tile[rl][4 * tx + 0] = v.x; tile[rl][4 * tx + 1] = v.y; tile[rl][4 * tx + 2] = v.z; tile[rl][4 * tx + 3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int cl = ty + 16 * i, c = c0 + cl, r = r0 + 4 * tx;
        if (r < R && c < C) {
            const v4f v = {tile[4 * tx + 0][cl], tile[4 * tx + 1][cl], tile[4 * tx + 2][cl], tile[4 * tx + 3][cl]};
            *reinterpret_cast<v4f *>(d + (int64_t)c * R + r) = v;
        }
    }
}

static hipError_t launch_transpose(const float *src, float *dst, int B, int R, int C, hipStream_t s)
{
    const int tiles_r = (R + 63) / 64, tiles_c = (C + 63) / 64;
    const int64_t blocks = (int64_t)B * tiles_r * tiles_c;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (R % 4 == 0 && C % 4 == 0 && ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0) {
        hipLaunchKernelGGL(transpose_vec4_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src, dst, R, C,
                           tiles_r, tiles_c);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src, dst, R, C,
                       tiles_r, tiles_c);
    return hipGetLastError();
}

hipError_t launch_bcn_to_bnc(const float *src, float *dst, int B, int C, int N, hipStream_t s)
{
    return launch_transpose(src, dst, B, C, N, s);
}
hipError_t launch_bnc_to_bcn(const float *src, float *dst, int B, int C, int N, hipStream_t s)
{
    return launch_transpose(src, dst, B, N, C, s);
}

// ---- grad_theta partial reduction --------------------------------------------
// partials [n_wg][KD][DOP] -> grad_theta [3,Din,Dout], grad_bias [Din,Dout];
// the cross-workgroup sum runs in double so its error does not grow with n_wg.
__global__ void reduce_partials_kernel(const float *__restrict__ partials, int n_wg, int DIP,
                                       int DOP, int Din, int Dout, float *__restrict__ grad_theta,
                                       float *__restrict__ grad_bias)
{
    __shared__ double red[4][64];
    const int o = blockIdx.x * 64 + (threadIdx.x & 63);
    const int part = threadIdx.x >> 6;                      // 4 strided shares of the workgroups
    const int kd = blockIdx.y;                              // row of ThetaP: j*DIP + c
    const int j = kd / DIP, c = kd % DIP;
    double sum = 0.0;
    if (o < DOP) {
        const int64_t stride = (int64_t)4 * DIP * DOP;
        const float *p = partials + (int64_t)kd * DOP + o;
        for (int g = part; g < n_wg; g += 4) sum += (double)p[g * stride];
    }
    red[part][threadIdx.x & 63] = sum;
    __syncthreads();
    if (part == 0 && o < Dout && c < Din) {
        const int x = threadIdx.x & 63;
        const float v = (float)(red[0][x] + red[1][x] + red[2][x] + red[3][x]);
        if (j < 3) grad_theta[((int64_t)j * Din + c) * Dout + o] = v;
        else grad_bias[(int64_t)c * Dout + o] = v;
    }
}

// The same for a run of 64 x 64 blocks of a wider layer: block z of the launch (blockIdx.z) is block
// p = first + z of the (Din / 64) x (Dout / 64) grid, its partials start at partials[z * n_wg], and its sums go to
// rows 64 * (p / n_ho).., columns 64 * (p % n_ho).. of grad_theta [3,Din,Dout] / grad_bias [Din,Dout].
__global__ void reduce_partials_blocks_kernel(const float *__restrict__ partials, int n_wg, int first, int n_ho,
                                              int Din, int Dout, float *__restrict__ grad_theta,
                                              float *__restrict__ grad_bias)
{
    __shared__ double red[4][64];
    const int x = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int kd = blockIdx.y;                              // row of the block: j*64 + c
    const int j = kd / 64, c = kd % 64;
    const int p = first + blockIdx.z, hi = p / n_ho, ho = p - hi * n_ho;
    const int64_t stride = (int64_t)4 * 64 * 64;
    const float *src = partials + (int64_t)blockIdx.z * n_wg * stride + (int64_t)kd * 64 + x;
    double sum = 0.0;
    for (int g = part; g < n_wg; g += 4) sum += (double)src[g * stride];
    red[part][x] = sum;
    __syncthreads();
    if (part == 0) {
        const float v = (float)(red[0][x] + red[1][x] + red[2][x] + red[3][x]);
        const int ci = 64 * hi + c, co = 64 * ho + x;
        if (j < 3) grad_theta[((int64_t)j * Din + ci) * Dout + co] = v;
        else grad_bias[(int64_t)ci * Dout + co] = v;
    }
}

hipError_t launch_reduce_partials_blocks(const float *partials, int n_wg, int first, int count, int n_ho, int Din,
                                         int Dout, float *grad_theta, float *grad_bias, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials_blocks_kernel, dim3(1, 4 * 64, (unsigned)count), dim3(256), 0, s, partials,
                       n_wg, first, n_ho, Din, Dout, grad_theta, grad_bias);
    return hipGetLastError();
}

// The same, run only if *flag == want (the second reduction of the one-pass backward after a late hand-over).
__global__ void reduce_partials_if_kernel(const int *__restrict__ flag, int want, const float *__restrict__ partials,
                                          int n_wg, int DIP, int DOP, int Din, int Dout,
                                          float *__restrict__ grad_theta, float *__restrict__ grad_bias)
{
    if (*flag != want) return;
    __shared__ double red[4][64];
    const int o = blockIdx.x * 64 + (threadIdx.x & 63);
    const int part = threadIdx.x >> 6;
    const int kd = blockIdx.y;
    const int j = kd / DIP, c = kd % DIP;
    double sum = 0.0;
    if (o < DOP) {
        const int64_t stride = (int64_t)4 * DIP * DOP;
        const float *p = partials + (int64_t)kd * DOP + o;
        for (int g = part; g < n_wg; g += 4) sum += (double)p[g * stride];
    }
    red[part][threadIdx.x & 63] = sum;
    __syncthreads();
    if (part == 0 && o < Dout && c < Din) {
        const int x = threadIdx.x & 63;
        const float v = (float)(red[0][x] + red[1][x] + red[2][x] + red[3][x]);
        if (j < 3) grad_theta[((int64_t)j * Din + c) * Dout + o] = v;
        else grad_bias[(int64_t)c * Dout + o] = v;
    }
}

hipError_t launch_reduce_partials_if(const int *flag, int want, const float *partials, int n_wg, int DIP, int DOP,
                                     int Din, int Dout, float *grad_theta, float *grad_bias, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials_if_kernel, dim3((DOP + 63) / 64, 4 * DIP), dim3(256), 0, s, flag, want,
                       partials, n_wg, DIP, DOP, Din, Dout, grad_theta, grad_bias);
    return hipGetLastError();
}

// Do the one-pass backward kernel's parameter gradients (64 -> 64: grad_theta [3,64,64], grad_bias [64,64], already
// reduced) stand clear of what its f16 halves can resolve?  A term of its sum over points -- tile entry times own'
// element -- is off by at most 2^-25 (half the smallest f16 step) times the tile entry (< 2^15), i.e. 2^-10 in the
// units of the workgroup's accumulators, which are 2^-(E + cs_c) / rs_(j,o) true units (E: the workgroup's last
// running exponent, the smallest it had; cs_c: its channel exponent; rs: the row scale of the packed parameters).
// Errors of random sign add in quadrature: err^2[(j,c),o] = Q_c / rs_(j,o)^2 with
// Q_c = sum over workgroups of n_wg * 2^(-20 - 2 (E_wg + cs_wg,c)).  Every row (j,c) over o and every column (j,o)
// over c of the result must have a sum of squares at least 2^32 times that of its error bound (RMS 2^16 times: a
// relative error of 1.5e-5, where ordinary data stands some 2^8 clear of the bar); rows and columns that are exactly
// zero -- a dead channel, a channel without gradient -- are exact and exempt.  Else the flag goes to
// FUSED_UNRESOLVED and the stand-alone kernel recomputes the parameter gradients.  Does nothing if the flag is set
// already (those were recomputed before the reduction).  One block, sums in double (the exponents span more than
// fp32 holds).
__global__ __launch_bounds__(1024) void fused_bwd_check_kernel(int *__restrict__ control, int n_wg,
                                                               const float *__restrict__ rscale,
                                                               const float *__restrict__ grad_theta,
                                                               const float *__restrict__ grad_bias)
{
    constexpr int C = 64, PARTS = 1024 / C;
    __shared__ __attribute__((aligned(16))) float s_P[4 * C * C];      // the result, [j][c][o]
    __shared__ double s_Qp[PARTS][C];
    __shared__ double s_Q[C], s_irs2[4 * C];
    __shared__ double s_Qsum;
    if (control[0] != 0) return;
    const int t = threadIdx.x;
    // the result into LDS (grad_theta is [3][C][C], grad_bias [C][C]: together [4][C][C])
    for (int i = t; i < 4 * C * C; i += 1024) s_P[i] = i < 3 * C * C ? grad_theta[i] : grad_bias[i - 3 * C * C];
    {   // Q_c, the workgroups shared out over PARTS thread groups
        const int c = t % C, part = t / C;
        double q = 0.0;
        constexpr int UN = 8;                        // records requested together
        for (int g0 = part; g0 < n_wg; g0 += PARTS * UN) {
            int e[UN], n[UN], ce[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int g = min(g0 + u * PARTS, n_wg - 1);
                const int *rec = control + FUSED_FLAG_INTS + (int64_t)g * FUSED_RECORD_INTS;
                e[u] = rec[0]; n[u] = (g0 + u * PARTS < n_wg) ? rec[1] : 0; ce[u] = rec[2 + c];
            }
#pragma unroll
            for (int u = 0; u < UN; ++u)
                if (n[u] > 0) q += __builtin_ldexp((double)n[u], -20 - 2 * (e[u] + ce[u]));
        }
        s_Qp[part][c] = q;
    }
    if (t < 4 * C) s_irs2[t] = __builtin_ldexp(1.0, -2 * (__builtin_amdgcn_frexp_expf(rscale[t]) - 1));   // rs = 2^k exactly
    __syncthreads();
    if (t < C) {
        double q = 0.0;
        for (int p2 = 0; p2 < PARTS; ++p2) q += s_Qp[p2][t];
        s_Q[t] = q;
    }
    __syncthreads();
    if (t == 0) {
        double a = 0.0;
        for (int c = 0; c < C; ++c) a += s_Q[c];
        s_Qsum = a;
    }
    __syncthreads();
    if (t >= 2 * 4 * C) return;
    const int j = (t % (4 * C)) / C, x = t % C;      // x: the channel c (t < 256) or the output channel o (t >= 256)
    double sq = 0.0, bound = 0.0;
    if (t < 4 * C) {                                 // row (j, c = x) over o, started at o = x to spread the LDS banks
        for (int i = 0; i < C; ++i) {
            const int o = (i + x) % C;
            const double v = (double)s_P[(j * C + x) * C + o];
            sq += v * v;
            bound += s_irs2[j * C + o];
        }
        bound *= s_Q[x];
    } else {                                         // column (j, o = x) over c
        for (int c = 0; c < C; ++c) { const double v = (double)s_P[(j * C + c) * C + x]; sq += v * v; }
        bound = s_irs2[j * C + x] * s_Qsum;
    }
    if (!(sq == 0.0 || sq >= 4294967296.0 * bound)) control[0] = FUSED_UNRESOLVED;
}

hipError_t launch_fused_bwd_check(int *control, int n_wg, const float *rscale, const float *grad_theta,
                                  const float *grad_bias, hipStream_t s)
{
    if (n_wg > FUSED_MAX_WG) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fused_bwd_check_kernel, dim3(1), dim3(1024), 0, s, control, n_wg, rscale, grad_theta, grad_bias);
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const float *partials, int n_wg, int DIP, int DOP, int Din,
                                  int Dout, float *grad_theta, float *grad_bias, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((DOP + 63) / 64, 4 * DIP), dim3(256), 0, s,
                       partials, n_wg, DIP, DOP, Din, Dout, grad_theta, grad_bias);
    return hipGetLastError();
}

// ---- range check and zero fill --------------------------------------------------
__global__ void count_bad_kernel(const int32_t *__restrict__ nbr, int64_t count, int N,
                                 int32_t *__restrict__ bad)
{
    int local = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int v = nbr[i];
        local += (v < 0 || v >= N);
    }
    if (local) atomicAdd(bad, local);
}

hipError_t launch_count_bad(const int32_t *nbr, int64_t count, int N, int32_t *bad, hipStream_t s)
{
    hipError_t e = launch_fill_zero(bad, sizeof(int32_t), s);
    if (e != hipSuccess) return e;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(count_bad_kernel, dim3((unsigned)blocks), dim3(256), 0, s, nbr, count, N, bad);
    return hipGetLastError();
}

__global__ void fill_zero_kernel(uint32_t *__restrict__ p, int64_t words)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

// bytes must be a multiple of 4 and ptr 4-byte aligned.
hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t s)
{
    const int64_t words = (int64_t)(bytes / 4);
    if (words == 0) return hipSuccess;
    int64_t blocks = (words + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint32_t *)ptr, words);
    return hipGetLastError();
}

// ---- generic direct-form kernels ------------------------------------------------
// Element (b, c, l) of a [B,C,N] / [B,N,C] tensor.
__device__ __forceinline__ int64_t at(int bnc, int b, int c, int l, int C, int N)
{
    return bnc ? ((int64_t)b * N + l) * C + c : ((int64_t)b * C + c) * N + l;
}

__global__ void generic_fwd_kernel(const float *__restrict__ feat, const float *__restrict__ pos,
                                   const int32_t *__restrict__ nbr, const float *__restrict__ theta,
                                   const float *__restrict__ bias, float *__restrict__ out, int B,
                                   int N, int K, int Din, int Dout, int bnc)
{
    const int64_t total = (int64_t)B * N * Dout;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int o = (int)(i % Dout);
        const int64_t gp = i / Dout;
        const int b = (int)(gp / N), l = (int)(gp % N);
        const float *px = pos + (int64_t)b * 3 * N, *py = px + N, *pz = py + N;
        float acc = 0.f;
        for (int k = 0; k < K; ++k) {
            const int n = nbr[((int64_t)b * K + k) * N + l];
            const float dx = px[n] - px[l], dy = py[n] - py[l], dz = pz[n] - pz[l];
            for (int c = 0; c < Din; ++c) {
                const float w = theta[((int64_t)0 * Din + c) * Dout + o] * dx +
                                theta[((int64_t)1 * Din + c) * Dout + o] * dy +
                                theta[((int64_t)2 * Din + c) * Dout + o] * dz +
                                bias[(int64_t)c * Dout + o];
                acc = fmaf(w, feat[at(bnc, b, c, n, Din, N)], acc);
            }
        }
        out[at(bnc, b, o, l, Dout, N)] = acc;
    }
}

hipError_t launch_generic_fwd(const float *feat, const float *pos, const int32_t *nbr,
                              const float *theta, const float *bias, float *out, int B, int N,
                              int K, int Din, int Dout, int bnc, hipStream_t s)
{
    const int64_t total = (int64_t)B * N * Dout;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(generic_fwd_kernel, dim3((unsigned)blocks), dim3(256), 0, s, feat, pos, nbr,
                       theta, bias, out, B, N, K, Din, Dout, bnc);
    return hipGetLastError();
}

// grad_feat by scatter: one thread per (centre, slot, input channel).
__global__ void generic_grad_feat_kernel(const float *__restrict__ pos,
                                         const int32_t *__restrict__ nbr,
                                         const float *__restrict__ theta,
                                         const float *__restrict__ bias,
                                         const float *__restrict__ grad_out,
                                         float *__restrict__ grad_feat, int B, int N, int K, int Din,
                                         int Dout, int bnc)
{
    const int64_t total = (int64_t)B * N * K * Din;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % Din);
        const int64_t e = i / Din;
        const int k = (int)(e % K);
        const int64_t gp = e / K;
        const int b = (int)(gp / N), l = (int)(gp % N);
        const float *px = pos + (int64_t)b * 3 * N, *py = px + N, *pz = py + N;
        const int n = nbr[((int64_t)b * K + k) * N + l];
        const float dx = px[n] - px[l], dy = py[n] - py[l], dz = pz[n] - pz[l];
        float sum = 0.f;
        for (int o = 0; o < Dout; ++o) {
            const float w = theta[((int64_t)0 * Din + c) * Dout + o] * dx +
                            theta[((int64_t)1 * Din + c) * Dout + o] * dy +
                            theta[((int64_t)2 * Din + c) * Dout + o] * dz +
                            bias[(int64_t)c * Dout + o];
            sum = fmaf(w, grad_out[at(bnc, b, o, l, Dout, N)], sum);
        }
        atomicAdd(&grad_feat[at(bnc, b, c, n, Din, N)], sum);
    }
}

// grad_theta / grad_bias: block = (input channel c, chunk of centres); threads over o.
__global__ __launch_bounds__(256) void generic_grad_theta_kernel(
    const float *__restrict__ feat, const float *__restrict__ pos, const int32_t *__restrict__ nbr,
    const float *__restrict__ grad_out, float *__restrict__ grad_theta,
    float *__restrict__ grad_bias, int B, int N, int K, int Din, int Dout, int bnc,
    int64_t pts_per_chunk)
{
    const int c = blockIdx.x;
    const int64_t BN = (int64_t)B * N;
    const int64_t g0 = (int64_t)blockIdx.y * pts_per_chunk;
    const int64_t g1 = (g0 + pts_per_chunk < BN) ? g0 + pts_per_chunk : BN;
    for (int o0 = 0; o0 < Dout; o0 += 256) {
        const int o = o0 + threadIdx.x;
        float ax = 0.f, ay = 0.f, az = 0.f, ab = 0.f;
        for (int64_t gp = g0; gp < g1; ++gp) {
            const int b = (int)(gp / N), l = (int)(gp % N);
            const float *px = pos + (int64_t)b * 3 * N, *py = px + N, *pz = py + N;
            float sx = 0.f, sy = 0.f, sz = 0.f, sb = 0.f;
            for (int k = 0; k < K; ++k) {
                const int n = nbr[((int64_t)b * K + k) * N + l];
                const float f = feat[at(bnc, b, c, n, Din, N)];
                sx = fmaf(px[n] - px[l], f, sx);
                sy = fmaf(py[n] - py[l], f, sy);
                sz = fmaf(pz[n] - pz[l], f, sz);
                sb += f;
            }
            if (o < Dout) {
                const float g = grad_out[at(bnc, b, o, l, Dout, N)];
                ax = fmaf(sx, g, ax); ay = fmaf(sy, g, ay); az = fmaf(sz, g, az); ab = fmaf(sb, g, ab);
            }
        }
        if (o < Dout) {
            atomicAdd(&grad_theta[((int64_t)0 * Din + c) * Dout + o], ax);
            atomicAdd(&grad_theta[((int64_t)1 * Din + c) * Dout + o], ay);
            atomicAdd(&grad_theta[((int64_t)2 * Din + c) * Dout + o], az);
            atomicAdd(&grad_bias[(int64_t)c * Dout + o], ab);
        }
    }
}

hipError_t launch_generic_bwd(const float *feat, const float *pos, const int32_t *nbr,
                              const float *theta, const float *bias, const float *grad_out,
                              float *grad_feat, float *grad_theta, float *grad_bias, int B, int N,
                              int K, int Din, int Dout, int bnc, hipStream_t s)
{
    hipError_t e;
    if (grad_feat) {
        e = launch_fill_zero(grad_feat, sizeof(float) * (size_t)B * N * Din, s);
        if (e != hipSuccess) return e;
        const int64_t total = (int64_t)B * N * K * Din;
        int64_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(generic_grad_feat_kernel, dim3((unsigned)blocks), dim3(256), 0, s, pos, nbr,
                           theta, bias, grad_out, grad_feat, B, N, K, Din, Dout, bnc);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (grad_theta && grad_bias) {
        e = launch_fill_zero(grad_theta, sizeof(float) * (size_t)3 * Din * Dout, s);
        if (e != hipSuccess) return e;
        e = launch_fill_zero(grad_bias, sizeof(float) * (size_t)Din * Dout, s);
        if (e != hipSuccess) return e;
        const int64_t BN = (int64_t)B * N;
        int64_t chunks = (BN + 255) / 256;
        if (chunks > 1024) chunks = 1024;
        const int64_t per = (BN + chunks - 1) / chunks;
        chunks = (BN + per - 1) / per;
        hipLaunchKernelGGL(generic_grad_theta_kernel, dim3(Din, (unsigned)chunks), dim3(256), 0, s,
                           feat, pos, nbr, grad_out, grad_theta, grad_bias, B, N, K, Din, Dout, bnc, per);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- location gradient, direct form (any shape) -------------------------------------
// one thread per edge (b, l, k): s_d = sum_{c,o} theta[d,c,o] feat[c,n] g[o,l]; +s_d to n, -s_d to l
__global__ __launch_bounds__(256) void generic_bwd_pos_kernel(const float *__restrict__ feat,
                                                              const int32_t *__restrict__ nbr,
                                                              const float *__restrict__ theta,
                                                              const float *__restrict__ grad_out,
                                                              float *__restrict__ grad_pos, int B, int N, int K,
                                                              int Din, int Dout, int bnc)
{
    const int64_t total = (int64_t)B * K * N;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int l = (int)(i % N);
        const int64_t bk = i / N;
        const int b = (int)(bk / K);
        const int n = nbr[i];
        if (n == l) continue;                       // a self edge adds and subtracts the same value
        float s[3] = {0.f, 0.f, 0.f};
        for (int c = 0; c < Din; ++c) {
            const float f = feat[at(bnc, b, c, n, Din, N)];
            float t0 = 0.f, t1 = 0.f, t2 = 0.f;
            for (int o = 0; o < Dout; ++o) {
                const float g = grad_out[at(bnc, b, o, l, Dout, N)];
                t0 = fmaf(theta[((int64_t)0 * Din + c) * Dout + o], g, t0);
                t1 = fmaf(theta[((int64_t)1 * Din + c) * Dout + o], g, t1);
                t2 = fmaf(theta[((int64_t)2 * Din + c) * Dout + o], g, t2);
            }
            s[0] = fmaf(f, t0, s[0]); s[1] = fmaf(f, t1, s[1]); s[2] = fmaf(f, t2, s[2]);
        }
        for (int d = 0; d < 3; ++d) {
            atomicAdd(&grad_pos[((int64_t)b * 3 + d) * N + n], s[d]);
            atomicAdd(&grad_pos[((int64_t)b * 3 + d) * N + l], -s[d]);
        }
    }
}

hipError_t launch_generic_bwd_pos(const float *feat, const int32_t *nbr, const float *theta,
                                  const float *grad_out, float *grad_pos, int B, int N, int K, int Din,
                                  int Dout, int bnc, hipStream_t s)
{
    hipError_t e = launch_fill_zero(grad_pos, sizeof(float) * (size_t)B * 3 * N, s);
    if (e != hipSuccess) return e;
    const int64_t total = (int64_t)B * K * N;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(generic_bwd_pos_kernel, dim3((unsigned)blocks), dim3(256), 0, s, feat, nbr, theta,
                       grad_out, grad_pos, B, N, K, Din, Dout, bnc);
    return hipGetLastError();
}

// ---- 1x1 convolution composed into the flex-convolution parameters (Sec. 4.3 block) ----------
// P = [theta; bias] as four [D x Dout] slabs j = 0..3.  Parameter-sized work, but cubic in the width (4 * 1024^3
// multiply-adds for a 1024-wide layer), so it runs as small LDS-tiled matrix products: a 256-thread block owns a
// 64 x 64 tile of the result, depth in steps of 16, 4 x 4 results per thread accumulated in double.
__device__ __forceinline__ const float *slab(const float *theta, const float *bias, int j, int D, int Dout)
{
    return j < 3 ? theta + (int64_t)j * D * Dout : bias;
}

// acc[i][jn] += sum_k A(m0 + ty*4 + i, k) * B(k, n0 + tx*4 + jn), A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn];
// elements outside M x K / K x N read as zero.  All 256 threads of the block must call it together.
__device__ __forceinline__ void tile_product(double (&acc)[4][4], const float *__restrict__ A, int64_t sam, int64_t sak,
                                             const float *__restrict__ B, int64_t sbk, int64_t sbn, int M, int N, int K,
                                             int m0, int n0, float (&As)[16][65], float (&Bs)[16][65])
{
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            // the unit-stride index runs fastest over the threads
            const int am = sam == 1 ? idx & 63 : idx >> 4, ak = sam == 1 ? idx >> 6 : idx & 15;
            const int bn = sbn == 1 ? idx & 63 : idx >> 4, bk = sbn == 1 ? idx >> 6 : idx & 15;
            As[ak][am] = (m0 + am < M && k0 + ak < K) ? A[(int64_t)(m0 + am) * sam + (int64_t)(k0 + ak) * sak] : 0.f;
            Bs[bk][bn] = (n0 + bn < N && k0 + bk < K) ? B[(int64_t)(k0 + bk) * sbk + (int64_t)(n0 + bn) * sbn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = (double)As[k][ty * 4 + i]; b[i] = (double)Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jn = 0; jn < 4; ++jn) acc[i][jn] += a[i] * b[jn];
        }
        __syncthreads();
    }
}

__device__ __forceinline__ void tile_store(const double (&acc)[4][4], float *__restrict__ C, int64_t ldc, int M, int N,
                                           int m0, int n0)
{
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + jn;
            if (m < M && n < N) C[(int64_t)m * ldc + n] = (float)acc[i][jn];
        }
}

// Pc[j][c0][o] = sum_c W[c][c0] * P[j][c][o]; grid (tiles over c0, tiles over o, 4 slabs)
__global__ __launch_bounds__(256) void compose_1x1_kernel(const float *__restrict__ W, const float *__restrict__ theta,
                                                          const float *__restrict__ bias, float *__restrict__ theta_c,
                                                          float *__restrict__ bias_c, int Din0, int Dmid, int Dout)
{
    __shared__ float As[16][65], Bs[16][65];
    const int j = blockIdx.z, m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    double acc[4][4] = {};
    tile_product(acc, W, 1, Din0, slab(theta, bias, j, Dmid, Dout), Dout, 1, Din0, Dout, Dmid, m0, n0, As, Bs);
    tile_store(acc, j < 3 ? theta_c + (int64_t)j * Din0 * Dout : bias_c, Dout, Din0, Dout, m0, n0);
}

// blockIdx.z < 4: gP[j][c][o] = sum_c0 W[c][c0] * gPc[j][c0][o], j = blockIdx.z (tiles over c and o);
// blockIdx.z == 4: gW[c][c0] = sum_{j,o} P[j][c][o] * gPc[j][c0][o] (tiles over c and c0).
__global__ __launch_bounds__(256) void compose_1x1_bwd_kernel(const float *__restrict__ W, const float *__restrict__ theta,
                                                              const float *__restrict__ bias,
                                                              const float *__restrict__ gtheta_c,
                                                              const float *__restrict__ gbias_c, float *__restrict__ gW,
                                                              float *__restrict__ gtheta, float *__restrict__ gbias,
                                                              int Din0, int Dmid, int Dout)
{
    __shared__ float As[16][65], Bs[16][65];
    const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    double acc[4][4] = {};
    if (blockIdx.z < 4) {
        const int j = blockIdx.z;
        if (m0 >= Dmid || n0 >= Dout) return;          // the grid covers the larger of the two tilings
        tile_product(acc, W, Din0, 1, slab(gtheta_c, gbias_c, j, Din0, Dout), Dout, 1, Dmid, Dout, Din0, m0, n0, As, Bs);
        tile_store(acc, j < 3 ? gtheta + (int64_t)j * Dmid * Dout : gbias, Dout, Dmid, Dout, m0, n0);
    } else {
        if (m0 >= Dmid || n0 >= Din0) return;
        for (int j = 0; j < 4; ++j)
            tile_product(acc, slab(theta, bias, j, Dmid, Dout), Dout, 1, slab(gtheta_c, gbias_c, j, Din0, Dout), 1, Dout,
                         Dmid, Din0, Dout, m0, n0, As, Bs);
        tile_store(acc, gW, Din0, Dmid, Din0, m0, n0);
    }
}

hipError_t launch_compose_1x1(const float *W, const float *theta, const float *bias, float *theta_c, float *bias_c,
                              int Din0, int Dmid, int Dout, hipStream_t s)
{
    hipLaunchKernelGGL(compose_1x1_kernel, dim3((Din0 + 63) / 64, (Dout + 63) / 64, 4), dim3(256), 0, s, W, theta, bias,
                       theta_c, bias_c, Din0, Dmid, Dout);
    return hipGetLastError();
}

hipError_t launch_compose_1x1_bwd(const float *W, const float *theta, const float *bias, const float *gtheta_c,
                                  const float *gbias_c, float *gW, float *gtheta, float *gbias, int Din0, int Dmid,
                                  int Dout, hipStream_t s)
{
    const int n_max = Dout > Din0 ? Dout : Din0;
    hipLaunchKernelGGL(compose_1x1_bwd_kernel, dim3((Dmid + 63) / 64, (n_max + 63) / 64, 5), dim3(256), 0, s, W, theta,
                       bias, gtheta_c, gbias_c, gW, gtheta, gbias, Din0, Dmid, Dout);
    return hipGetLastError();
}

// ---- blocks of the parameter tensors (layers run as passes over channel blocks) ----------
// extract (insert == 0): blk_theta[j][r][c] = theta[j][r0 + r][c0 + c], blk_bias likewise;
// insert  (insert == 1): the other way round.  theta [3,R,C], bias [R,C]; block [3,nr,nc], [nr,nc].
__global__ __launch_bounds__(256) void param_block_kernel(float *__restrict__ theta, float *__restrict__ bias,
                                                          float *__restrict__ blk_theta, float *__restrict__ blk_bias,
                                                          int R, int C, int r0, int c0, int nr, int nc, int insert)
{
    const int total = 4 * nr * nc;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int c = i % nc, r = (i / nc) % nr, j = i / (nc * nr);
        float *big = (j < 3 ? theta + (int64_t)j * R * C : bias) + (int64_t)(r0 + r) * C + c0 + c;
        float *small = (j < 3 ? blk_theta + (int64_t)j * nr * nc : blk_bias) + (int64_t)r * nc + c;
        if (insert) *big = *small; else *small = *big;
    }
}

hipError_t launch_param_block(float *theta, float *bias, float *blk_theta, float *blk_bias, int R, int C, int r0,
                              int c0, int nr, int nc, int insert, hipStream_t s)
{
    const int total = 4 * nr * nc;
    hipLaunchKernelGGL(param_block_kernel, dim3((total + 255) / 256), dim3(256), 0, s, theta, bias, blk_theta, blk_bias,
                       R, C, r0, c0, nr, nc, insert);
    return hipGetLastError();
}

// Row copy between feature tensors of different widths and layouts: dst[b, n, c] = src[b, n, c_off + c] where that
// channel exists, else 0, for c < Cd (so it pads with zero channels, keeps the leading ones, or cuts a column block
// out).  *_bcn: that tensor is channel-major.
__global__ __launch_bounds__(256) void copy_rows_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                        int64_t total, int N, int Cs, int Cd, int c_off, int src_bcn,
                                                        int dst_bcn)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int64_t b;
        int n, c;
        if (dst_bcn) { n = (int)(i % N); const int64_t bc = i / N; c = (int)(bc % Cd); b = bc / Cd; }
        else         { c = (int)(i % Cd); const int64_t bn = i / Cd; n = (int)(bn % N); b = bn / N; }
        float v = 0.f;
        const int cs = c_off + c;
        if (cs < Cs) v = src_bcn ? src[(b * Cs + cs) * N + n] : src[(b * N + n) * Cs + cs];
        dst[i] = v;
    }
}

hipError_t launch_copy_rows(const float *src, float *dst, int B, int N, int Cs, int Cd, int src_bcn, int dst_bcn,
                            hipStream_t s, int c_off)
{
    const int64_t total = (int64_t)B * N * Cd;
    int64_t blocks = (total + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src, dst, total, N, Cs, Cd, c_off,
                       src_bcn, dst_bcn);
    return hipGetLastError();
}

// blk[d][r][c] = theta[d][r0 + r][c0 + c] where that entry exists, else 0; blk is [3][nr][nc].
__global__ __launch_bounds__(256) void theta_block_padded_kernel(const float *__restrict__ theta, float *__restrict__ blk,
                                                                 int Din, int Dout, int r0, int c0, int nr, int nc)
{
    const int total = 3 * nr * nc;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int c = c0 + i % nc, r = r0 + (i / nc) % nr, d = i / (nc * nr);
        blk[i] = (r < Din && c < Dout) ? theta[((int64_t)d * Din + r) * Dout + c] : 0.f;
    }
}

hipError_t launch_theta_block_padded(const float *theta, float *blk, int Din, int Dout, int r0, int c0, int nr, int nc,
                                     hipStream_t s)
{
    hipLaunchKernelGGL(theta_block_padded_kernel, dim3((3 * nr * nc + 255) / 256), dim3(256), 0, s, theta, blk, Din,
                       Dout, r0, c0, nr, nc);
    return hipGetLastError();
}

}  // namespace flex
