// Inverse density importance sub-sampling (Sec. 3.2): phi = sum of the distances to the K
// neighbours, then Ns points per cloud drawn with probability proportional to phi in one pass
// over the points (stratified sampling on the running sum).  Every decision of the draw is an
// integer comparison: phi is put on an integer scale of `bits` bits relative to the cloud's
// maximum (one float division, one float product per point), the running sums are 64-bit
// integers (exact in any summation order, so the parallel scan here and a sequential loop give
// the same table), the strata and thresholds are integer expressions of the caller's random
// words.
#include "flex_common.hpp"
#include <climits>

namespace flex {

static constexpr int IDISS_ITEMS = 8;                       // points per thread in the scans
static constexpr int IDISS_CHUNK = 256 * IDISS_ITEMS;       // points per block

__global__ __launch_bounds__(256) void idiss_phi_kernel(const float *__restrict__ pos, const int32_t *__restrict__ nbr,
                                                        float *__restrict__ phi, int64_t BN, int N, int K)
{
    for (int64_t gp = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; gp < BN; gp += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = gp / N;
        const int l = (int)(gp - b * N);
        const float *p = pos + b * 3 * N;
        const int32_t *nb = nbr + b * K * N + l;
        const float cx = p[l], cy = p[(int64_t)N + l], cz = p[2 * (int64_t)N + l];
        float s = 0.f;
        for (int k = 0; k < K; ++k) {
            const int n = nb[(int64_t)k * N];
            const float dx = p[n] - cx, dy = p[(int64_t)N + n] - cy, dz = p[2 * (int64_t)N + n] - cz;
            s += sqrtf(dx * dx + dy * dy + dz * dz);
        }
        phi[gp] = s;
    }
}

// per-cloud maximum; phi >= 0, so the float order is the order of the bit patterns
__global__ __launch_bounds__(256) void idiss_max_kernel(const float *__restrict__ phi, unsigned *__restrict__ mx, int N)
{
    const int b = blockIdx.y;
    unsigned m = 0;
    for (int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; l < N; l += (int64_t)gridDim.x * blockDim.x)
        m = max(m, __float_as_uint(phi[(int64_t)b * N + l]));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, d, 64));
    if ((threadIdx.x & 63) == 0 && m) atomicMax(&mx[b], m);
}

__device__ __forceinline__ unsigned idiss_quantum(float x, float mx, int bits)
{
    if (!(mx > 0.f)) return 1u;                                // coincident points: a uniform draw
    const float scale = (float)((int64_t)1 << bits) / mx;      // the same two float operations as the CPU check
    return (unsigned)(x * scale);
}

__device__ __forceinline__ unsigned long long block_exclusive_scan64(unsigned long long v, unsigned long long *s_wave,
                                                                     unsigned long long &block_total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    unsigned long long x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) s_wave[w] = x;
    __syncthreads();
    unsigned long long base = 0;
    for (int i = 0; i < w; ++i) base += s_wave[i];
    block_total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
    __syncthreads();
    return base + x - v;
}

// bsum[b][blk] = sum of the quanta of chunk blk of cloud b
__global__ __launch_bounds__(256) void idiss_chunk_sums_kernel(const float *__restrict__ phi,
                                                               const unsigned *__restrict__ mx,
                                                               unsigned long long *__restrict__ bsum, int N, int nblk,
                                                               int bits)
{
    __shared__ unsigned long long s_wave[4];
    const int b = blockIdx.y;
    const float m = __uint_as_float(mx[b]);
    const int64_t base = (int64_t)blockIdx.x * IDISS_CHUNK + (int64_t)threadIdx.x * IDISS_ITEMS;
    unsigned long long v = 0;
#pragma unroll
    for (int i = 0; i < IDISS_ITEMS; ++i)
        if (base + i < N) v += idiss_quantum(phi[(int64_t)b * N + base + i], m, bits);
    unsigned long long total;
    block_exclusive_scan64(v, s_wave, total);
    if (threadIdx.x == 0) bsum[(int64_t)b * (nblk + 1) + blockIdx.x] = total;
}

// one block per cloud: exclusive scan of its chunk sums in place; entry nblk = the cloud's total Q
__global__ __launch_bounds__(256) void idiss_scan_sums_kernel(unsigned long long *__restrict__ bsum, int nblk)
{
    __shared__ unsigned long long s_wave[4];
    unsigned long long *row = bsum + (int64_t)blockIdx.x * (nblk + 1);
    unsigned long long carry = 0;
    for (int c0 = 0; c0 < nblk; c0 += 256) {
        const int i = c0 + threadIdx.x;
        const unsigned long long v = (i < nblk) ? row[i] : 0;
        unsigned long long total;
        const unsigned long long ex = block_exclusive_scan64(v, s_wave, total);
        if (i < nblk) row[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) row[nblk] = carry;
}

// C[b][l] = inclusive running sum of the quanta
__global__ __launch_bounds__(256) void idiss_running_sum_kernel(const float *__restrict__ phi,
                                                                const unsigned *__restrict__ mx,
                                                                const unsigned long long *__restrict__ bsum,
                                                                unsigned long long *__restrict__ C, int N, int nblk,
                                                                int bits)
{
    __shared__ unsigned long long s_wave[4];
    const int b = blockIdx.y;
    const float m = __uint_as_float(mx[b]);
    const int64_t base = (int64_t)blockIdx.x * IDISS_CHUNK + (int64_t)threadIdx.x * IDISS_ITEMS;
    unsigned q[IDISS_ITEMS];
    unsigned long long sum = 0;
#pragma unroll
    for (int i = 0; i < IDISS_ITEMS; ++i) {
        q[i] = (base + i < N) ? idiss_quantum(phi[(int64_t)b * N + base + i], m, bits) : 0u;
        sum += q[i];
    }
    unsigned long long total;
    unsigned long long run = bsum[(int64_t)b * (nblk + 1) + blockIdx.x] + block_exclusive_scan64(sum, s_wave, total);
#pragma unroll
    for (int i = 0; i < IDISS_ITEMS; ++i) {
        run += q[i];
        if (base + i < N) C[(int64_t)b * N + base + i] = run;
    }
}

// sel[b][j] = first point whose running sum exceeds the threshold of stratum j
__global__ __launch_bounds__(256) void idiss_select_kernel(const unsigned long long *__restrict__ C,
                                                           const unsigned long long *__restrict__ bsum,
                                                           const uint32_t *__restrict__ u, int32_t *__restrict__ sel,
                                                           int N, int Ns, int nblk)
{
    const int b = blockIdx.y;
    const unsigned long long Q = bsum[(int64_t)b * (nblk + 1) + nblk];
    const unsigned long long width = Q / (unsigned long long)Ns, rem = Q % (unsigned long long)Ns;
    const unsigned long long *Cb = C + (int64_t)b * N;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < Ns; j += gridDim.x * blockDim.x) {
        const unsigned long long jj = (unsigned long long)j;
        const unsigned long long start = jj * width + (jj < rem ? jj : rem);
        const unsigned long long len = width + (jj < rem ? 1u : 0u);
        const unsigned long long t = start + __umul64hi((unsigned long long)u[(int64_t)b * Ns + j] << 32, len);
        int lo = 0, hi = N - 1;            // Q > t, so the last point always qualifies
        while (lo < hi) {
            const int mid = lo + ((hi - lo) >> 1);
            if (Cb[mid] > t) hi = mid; else lo = mid + 1;
        }
        sel[(int64_t)b * Ns + j] = lo;
    }
}

// ---- repeats removed from an ascending selection ---------------------------------------------
// Sequential rule: sel[j] = max(sel[j], sel[j-1] + 1), then sel[j] = min(sel[j], N - Ns + j).  The first is
// a running maximum of sel[i] - i (plus j), so it runs as a three-kernel scan; the second is elementwise.
__device__ __forceinline__ int block_inclusive_max(int v, int *s_wave, int &block_max)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x = max(x, y);
    }
    if (lane == 63) s_wave[w] = x;
    __syncthreads();
    int before = INT_MIN;
    for (int i = 0; i < w; ++i) before = max(before, s_wave[i]);
    block_max = max(max(s_wave[0], s_wave[1]), max(s_wave[2], s_wave[3]));
    __syncthreads();
    return max(before, x);
}

__global__ __launch_bounds__(256) void distinct_chunk_max_kernel(const int32_t *__restrict__ sel, int *__restrict__ cm,
                                                                 int Ns, int nblk)
{
    __shared__ int s_wave[4];
    const int b = blockIdx.y;
    const int64_t base = (int64_t)blockIdx.x * IDISS_CHUNK + (int64_t)threadIdx.x * IDISS_ITEMS;
    int v = INT_MIN;
#pragma unroll
    for (int i = 0; i < IDISS_ITEMS; ++i)
        if (base + i < Ns) v = max(v, sel[(int64_t)b * Ns + base + i] - (int)(base + i));
    int total;
    block_inclusive_max(v, s_wave, total);
    if (threadIdx.x == 0) cm[(int64_t)b * nblk + blockIdx.x] = total;
}

// one block per cloud: cm[blk] <- maximum over the chunks before blk (INT_MIN for the first)
__global__ __launch_bounds__(256) void distinct_scan_max_kernel(int *__restrict__ cm, int nblk)
{
    __shared__ int s_wave[4];
    __shared__ int s_inc[256];
    int *row = cm + (int64_t)blockIdx.x * nblk;
    int carry = INT_MIN;
    for (int c0 = 0; c0 < nblk; c0 += 256) {
        const int i = c0 + threadIdx.x;
        const int v = (i < nblk) ? row[i] : INT_MIN;
        int total;
        s_inc[threadIdx.x] = block_inclusive_max(v, s_wave, total);
        __syncthreads();
        const int before = threadIdx.x > 0 ? s_inc[threadIdx.x - 1] : INT_MIN;
        if (i < nblk) row[i] = max(carry, before);
        carry = max(carry, total);
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void distinct_apply_kernel(int32_t *__restrict__ sel, const int *__restrict__ cm, int N,
                                                             int Ns, int nblk)
{
    __shared__ int s_wave[4];
    const int b = blockIdx.y;
    const int64_t base = (int64_t)blockIdx.x * IDISS_CHUNK + (int64_t)threadIdx.x * IDISS_ITEMS;
    int v[IDISS_ITEMS], mine = INT_MIN;
#pragma unroll
    for (int i = 0; i < IDISS_ITEMS; ++i) {
        v[i] = (base + i < Ns) ? sel[(int64_t)b * Ns + base + i] - (int)(base + i) : INT_MIN;
        mine = max(mine, v[i]);
    }
    int total;
    const int inc = block_inclusive_max(mine, s_wave, total);       // includes this thread's items
    // maximum over everything before this thread's first item
    __shared__ int s_inc[256];
    s_inc[threadIdx.x] = inc;
    __syncthreads();
    int run = max(cm[(int64_t)b * nblk + blockIdx.x], threadIdx.x > 0 ? s_inc[threadIdx.x - 1] : INT_MIN);
#pragma unroll
    for (int i = 0; i < IDISS_ITEMS; ++i) {
        run = max(run, v[i]);
        if (base + i < Ns) {
            const int j = (int)(base + i);
            sel[(int64_t)b * Ns + j] = min(run + j, N - Ns + j);
        }
    }
}

size_t distinct_ws_bytes(int B, int Ns) { return align256(sizeof(int) * (size_t)B * cdiv64(Ns, IDISS_CHUNK)); }

hipError_t launch_selection_make_distinct(int32_t *sel, int B, int N, int Ns, void *ws, hipStream_t s)
{
    const int nblk = (int)cdiv64(Ns, IDISS_CHUNK);
    int *cm = (int *)ws;
    hipLaunchKernelGGL(distinct_chunk_max_kernel, dim3(nblk, B), dim3(256), 0, s, sel, cm, Ns, nblk);
    hipLaunchKernelGGL(distinct_scan_max_kernel, dim3(B), dim3(256), 0, s, cm, nblk);
    hipLaunchKernelGGL(distinct_apply_kernel, dim3(nblk, B), dim3(256), 0, s, sel, cm, N, Ns, nblk);
    return hipGetLastError();
}

int idiss_bits(int N)
{
    int lg = 0;
    while (((int64_t)1 << lg) < N) ++lg;
    return (51 - lg) < 28 ? (51 - lg) : 28;
}

static int idiss_nblk(int N) { return (int)cdiv64(N, IDISS_CHUNK); }

size_t idiss_ws_bytes(int B, int N)
{
    return align256(sizeof(unsigned long long) * (size_t)B * N) +
           align256(sizeof(unsigned long long) * (size_t)B * (idiss_nblk(N) + 1)) + align256(sizeof(unsigned) * (size_t)B);
}

hipError_t launch_idiss_phi(const float *pos, const int32_t *nbr, float *phi, int B, int N, int K, hipStream_t s)
{
    const int64_t BN = (int64_t)B * N;
    int64_t blocks = (BN + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    hipLaunchKernelGGL(idiss_phi_kernel, dim3((unsigned)blocks), dim3(256), 0, s, pos, nbr, phi, BN, N, K);
    return hipGetLastError();
}

hipError_t launch_idiss_sample(const float *phi, const uint32_t *u, int32_t *sel, int B, int N, int Ns, void *ws,
                               hipStream_t s)
{
    const int nblk = idiss_nblk(N), bits = idiss_bits(N);
    unsigned long long *C = (unsigned long long *)ws;
    unsigned long long *bsum = (unsigned long long *)((char *)ws + align256(sizeof(unsigned long long) * (size_t)B * N));
    unsigned *mx = (unsigned *)((char *)bsum + align256(sizeof(unsigned long long) * (size_t)B * (nblk + 1)));
    hipError_t e = launch_fill_zero(mx, sizeof(unsigned) * (size_t)B, s);
    if (e != hipSuccess) return e;
    const int mb = nblk < 1024 ? nblk : 1024;
    hipLaunchKernelGGL(idiss_max_kernel, dim3(mb, B), dim3(256), 0, s, phi, mx, N);
    hipLaunchKernelGGL(idiss_chunk_sums_kernel, dim3(nblk, B), dim3(256), 0, s, phi, mx, bsum, N, nblk, bits);
    hipLaunchKernelGGL(idiss_scan_sums_kernel, dim3(B), dim3(256), 0, s, bsum, nblk);
    hipLaunchKernelGGL(idiss_running_sum_kernel, dim3(nblk, B), dim3(256), 0, s, phi, mx, bsum, C, N, nblk, bits);
    int sb = (Ns + 255) / 256;
    if (sb > 4096) sb = 4096;
    hipLaunchKernelGGL(idiss_select_kernel, dim3(sb, B), dim3(256), 0, s, C, bsum, u, sel, N, Ns, nblk);
    return hipGetLastError();
}

}  // namespace flex
