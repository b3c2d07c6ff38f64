// Transposed neighbour graph: for every point, the list of centres that name
// it as a neighbour (CSR: in_off / in_src).  Counting sort by target point:
// count -> exclusive scan -> fill -> sort each list ascending so that the
// result does not depend on the order in which the fill's atomics landed (and
// so that repeated sources sit next to each other).
#include "flex_common.hpp"

namespace flex {

static constexpr int SCAN_ITEMS = 8;                    // per thread
static constexpr int SCAN_CHUNK = 256 * SCAN_ITEMS;     // per block
static constexpr int SORT_LOCAL = 32;                   // lists up to here sort in registers

__global__ __launch_bounds__(256) void inedge_count_kernel(const int32_t *__restrict__ nbr,
                                                           int32_t *__restrict__ cnt, int64_t E,
                                                           int N, int64_t KN)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < E;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = i / KN;
        atomicAdd(&cnt[b * N + nbr[i]], 1);
    }
}

// Lists over a subset of the centres (pooling with subsampling): edge i = (cloud b, slot k, kept
// centre j) names point nbr[b, k, sel[b,j]]; the lists hold j.  Entries of sel outside [0,N) are clamped.
__device__ __forceinline__ int64_t sub_edge_target(const int32_t *__restrict__ nbr, const int32_t *__restrict__ sel,
                                                   int64_t i, int N, int Ns, int K, int &j)
{
    const int64_t KNs = (int64_t)K * Ns;
    const int64_t b = i / KNs, r = i - b * KNs;
    const int k = (int)(r / Ns);
    j = (int)(r - (int64_t)k * Ns);
    const int l = min(max(sel[b * Ns + j], 0), N - 1);
    return b * N + nbr[(b * K + k) * N + l];
}

__global__ __launch_bounds__(256) void inedge_sub_count_kernel(const int32_t *__restrict__ nbr,
                                                               const int32_t *__restrict__ sel,
                                                               int32_t *__restrict__ cnt, int64_t E, int N,
                                                               int Ns, int K)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < E;
         i += (int64_t)gridDim.x * blockDim.x) {
        int j;
        atomicAdd(&cnt[sub_edge_target(nbr, sel, i, N, Ns, K, j)], 1);
    }
}

__global__ __launch_bounds__(256) void inedge_sub_fill_kernel(const int32_t *__restrict__ nbr,
                                                              const int32_t *__restrict__ sel,
                                                              const int32_t *__restrict__ off,
                                                              int32_t *__restrict__ cnt,
                                                              int32_t *__restrict__ src, int64_t E, int N,
                                                              int Ns, int K)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < E;
         i += (int64_t)gridDim.x * blockDim.x) {
        int j;
        const int64_t g = sub_edge_target(nbr, sel, i, N, Ns, K, j);
        const int slot = atomicSub(&cnt[g], 1) - 1;
        src[off[g] + slot] = j;
    }
}

__device__ __forceinline__ int block_exclusive_scan(int v, int *s_wave, int &block_total)
{
    // inclusive scan inside the wave, then across the 4 waves
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) s_wave[w] = x;
    __syncthreads();
    int base = 0;
    for (int i = 0; i < w; ++i) base += s_wave[i];
    block_total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
    __syncthreads();
    return base + x - v;
}

__global__ __launch_bounds__(256) void scan_block_sums_kernel(const int32_t *__restrict__ cnt,
                                                              int32_t *__restrict__ bsum, int64_t n)
{
    __shared__ int s_wave[4];
    const int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + (int64_t)threadIdx.x * SCAN_ITEMS;
    int v = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i)
        if (base + i < n) v += cnt[base + i];
    int total;
    block_exclusive_scan(v, s_wave, total);
    if (threadIdx.x == 0) bsum[blockIdx.x] = total;
}

// single block: exclusive scan of bsum[0..nblk) in place; bsum[nblk] = grand total
__global__ __launch_bounds__(256) void scan_of_sums_kernel(int32_t *__restrict__ bsum, int nblk)
{
    __shared__ int s_wave[4];
    int carry = 0;
    for (int c0 = 0; c0 < nblk; c0 += 256) {
        const int i = c0 + threadIdx.x;
        const int v = (i < nblk) ? bsum[i] : 0;
        int total;
        const int ex = block_exclusive_scan(v, s_wave, total);
        if (i < nblk) bsum[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) bsum[nblk] = carry;
}

__global__ __launch_bounds__(256) void scan_apply_kernel(const int32_t *__restrict__ cnt,
                                                         const int32_t *__restrict__ bsum,
                                                         int32_t *__restrict__ off, int64_t n,
                                                         int nblk)
{
    __shared__ int s_wave[4];
    const int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + (int64_t)threadIdx.x * SCAN_ITEMS;
    int v[SCAN_ITEMS], sum = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        v[i] = (base + i < n) ? cnt[base + i] : 0;
        sum += v[i];
    }
    int total;
    int run = bsum[blockIdx.x] + block_exclusive_scan(sum, s_wave, total);
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        if (base + i < n) off[base + i] = run;
        run += v[i];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) off[n] = bsum[nblk];
}

__global__ __launch_bounds__(256) void inedge_fill_kernel(const int32_t *__restrict__ nbr,
                                                          const int32_t *__restrict__ off,
                                                          int32_t *__restrict__ cnt,
                                                          int32_t *__restrict__ src, int64_t E,
                                                          int N, int64_t KN)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < E;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = i / KN;
        const int l = (int)(i % N);
        const int64_t g = b * N + nbr[i];
        const int slot = atomicSub(&cnt[g], 1) - 1;     // counts run down to zero
        src[off[g] + slot] = l;
    }
}

__global__ __launch_bounds__(256) void inedge_sort_kernel(const int32_t *__restrict__ off,
                                                          int32_t *__restrict__ src, int64_t BN)
{
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < BN;
         g += (int64_t)gridDim.x * blockDim.x) {
        const int beg = off[g], d = off[g + 1] - beg;
        if (d < 2) continue;
        int32_t *p = src + beg;
        if (d <= SORT_LOCAL) {
            int v[SORT_LOCAL];
#pragma unroll
            for (int i = 0; i < SORT_LOCAL; ++i) v[i] = (i < d) ? p[i] : 0x7fffffff;
            // odd-even transposition network: data-independent, stays in registers
#pragma unroll 1
            for (int pass = 0; pass < d; ++pass) {
#pragma unroll
                for (int i = 0; i + 1 < SORT_LOCAL; i += 2) {
                    const int a = v[i], c = v[i + 1];
                    v[i] = min(a, c); v[i + 1] = max(a, c);
                }
#pragma unroll
                for (int i = 1; i + 1 < SORT_LOCAL; i += 2) {
                    const int a = v[i], c = v[i + 1];
                    v[i] = min(a, c); v[i + 1] = max(a, c);
                }
            }
#pragma unroll
            for (int i = 0; i < SORT_LOCAL; ++i)
                if (i < d) p[i] = v[i];
        } else if (d <= 256) {
            for (int i = 1; i < d; ++i) {                 // rare: insertion sort in place
                const int x = p[i];
                int j = i - 1;
                while (j >= 0 && p[j] > x) { p[j + 1] = p[j]; --j; }
                p[j + 1] = x;
            }
        } else {
            // very rare (a point named by hundreds of centres): heapsort in place, O(d log d)
            auto sift = [&](int root, int end) {
                const int x = p[root];
                for (;;) {
                    int child = 2 * root + 1;
                    if (child >= end) break;
                    if (child + 1 < end && p[child + 1] > p[child]) ++child;
                    if (p[child] <= x) break;
                    p[root] = p[child];
                    root = child;
                }
                p[root] = x;
            };
            for (int i = d / 2 - 1; i >= 0; --i) sift(i, d);
            for (int end = d - 1; end > 0; --end) {
                const int x = p[end]; p[end] = p[0]; p[0] = x;
                sift(0, end);
            }
        }
    }
}

// ---- walking order for the gathers over in-edge lists -----------------------------------------
// order[b*N + p] = the point that stands at position p of cloud b: inside every window of ORDER_WINDOW consecutive
// positions the window's points, sorted by the length of their in-edge list (lengths past 31 count as 31), points
// of equal length in index order.  A wave of the gather kernels takes four consecutive positions and a tile a few
// dozen, so their lists have (nearly) one length: no slot of a batch stays empty and no wave waits for a longer
// list at the tile's barrier, while a window is small enough for its gathered rows to stay in the caches.
// One workgroup per window: lengths -> per (length, 64-point chunk) counts by ballots -> running sum in
// (length, chunk) order -> every point's place.
// The window is 13 tiles of 48 points: the persistent kernels deal tiles to workgroups with a stride that is a
// power of two, and a window of a power-of-two number of tiles would hand a workgroup the same place in every
// window, i.e. always the short or always the long lists.
static constexpr int ORDER_WINDOW = 624;
static constexpr int ORDER_CHUNKS = (ORDER_WINDOW + 63) / 64;  // 64-point chunks of a window
static constexpr int ORDER_ROUNDS = (ORDER_CHUNKS + 3) / 4;    // chunks per wave (4 waves)
static constexpr int ORDER_BUCKETS = 32;

__global__ __launch_bounds__(256) void inedge_order_kernel(const int32_t *__restrict__ off, int32_t *__restrict__ order,
                                                           int N, int windows_per_cloud)
{
    __shared__ int s_cnt[ORDER_BUCKETS * ORDER_CHUNKS];        // [length][chunk], then its exclusive running sum
    const int b = blockIdx.x / windows_per_cloud, w = blockIdx.x - b * windows_per_cloud;
    const int p0 = w * ORDER_WINDOW, n = min(ORDER_WINDOW, N - p0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t lt = (1ull << lane) - 1ull;
    int len[ORDER_ROUNDS], rank[ORDER_ROUNDS];
#pragma unroll
    for (int r = 0; r < ORDER_ROUNDS; ++r) {
        const int chunk = r * 4 + wave, i = chunk * 64 + lane;
        len[r] = -1;
        if (i < n) {
            const int64_t g = (int64_t)b * N + p0 + i;
            len[r] = min(off[g + 1] - off[g], ORDER_BUCKETS - 1);
        }
        rank[r] = 0;
    }
    for (int i = threadIdx.x; i < ORDER_BUCKETS * ORDER_CHUNKS; i += 256) s_cnt[i] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ORDER_ROUNDS; ++r) {
        const int chunk = r * 4 + wave;
        // one round per length that occurs in the chunk (about ten of the 32)
        uint64_t todo = __ballot(len[r] >= 0);
        while (todo) {
            const int d = __shfl(len[r], __ffsll((long long)todo) - 1, 64);     // wave-uniform
            const uint64_t m = __ballot(len[r] == d);
            if (len[r] == d) rank[r] = __popcll(m & lt);
            if (lane == 0) s_cnt[d * ORDER_CHUNKS + chunk] = __popcll(m);
            todo &= ~m;
        }
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive running sum of the ORDER_BUCKETS * ORDER_CHUNKS counts: PER consecutive entries per lane
        constexpr int PER = ORDER_BUCKETS * ORDER_CHUNKS / 64;
        int v[PER], sum = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) { v[i] = s_cnt[lane * PER + i]; sum += v[i]; }
        int x = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(x, d, 64);
            if (lane >= d) x += y;
        }
        int run = x - sum;
#pragma unroll
        for (int i = 0; i < PER; ++i) { s_cnt[lane * PER + i] = run; run += v[i]; }
    }
    __syncthreads();
    // every point's place, through LDS so that the window leaves as one contiguous write
    __shared__ int s_ord[ORDER_WINDOW];
#pragma unroll
    for (int r = 0; r < ORDER_ROUNDS; ++r) {
        const int chunk = r * 4 + wave, i = chunk * 64 + lane;
        if (i < n) s_ord[s_cnt[len[r] * ORDER_CHUNKS + chunk] + rank[r]] = p0 + i;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += 256) order[(int64_t)b * N + p0 + i] = s_ord[i];
}

size_t inedges_order_bytes(int64_t BN) { return align256(sizeof(int32_t) * (size_t)BN); }

hipError_t launch_inedges_order(const int32_t *in_off, int B, int N, int32_t *order, hipStream_t s)
{
    static_assert((ORDER_BUCKETS * ORDER_CHUNKS) % 64 == 0, "order kernel: whole entries per lane in the running sum");
    const int wpc = (N + ORDER_WINDOW - 1) / ORDER_WINDOW;
    const int64_t blocks = (int64_t)B * wpc;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(inedge_order_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in_off, order, N, wpc);
    return hipGetLastError();
}

// off[0..n] = exclusive running sum of cnt[0..n) (off[n] = total); ws: exclusive_scan_ws_bytes(n)
size_t exclusive_scan_ws_bytes(int64_t n) { return align256(sizeof(int32_t) * (size_t)(cdiv64(n, SCAN_CHUNK) + 1)); }

hipError_t launch_exclusive_scan_i32(const int32_t *cnt, int32_t *off, int64_t n, void *ws, hipStream_t s)
{
    const int nblk = (int)cdiv64(n, SCAN_CHUNK);
    int32_t *bsum = (int32_t *)ws;
    hipLaunchKernelGGL(scan_block_sums_kernel, dim3(nblk), dim3(256), 0, s, cnt, bsum, n);
    hipLaunchKernelGGL(scan_of_sums_kernel, dim3(1), dim3(256), 0, s, bsum, nblk);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(nblk), dim3(256), 0, s, cnt, bsum, off, n, nblk);
    return hipGetLastError();
}

size_t inedges_ws_bytes(int64_t BN)
{
    const int64_t nblk = cdiv64(BN, SCAN_CHUNK);
    return align256(sizeof(int32_t) * (size_t)BN) + align256(sizeof(int32_t) * (size_t)(nblk + 1));
}

hipError_t launch_inedges_build(const int32_t *nbr, int B, int N, int K, int32_t *in_off,
                                int32_t *in_src, void *ws, hipStream_t s)
{
    return launch_inedges_build_sub(nbr, nullptr, B, N, N, K, in_off, in_src, ws, s);
}

// sel == nullptr: every point is a centre (Ns = N); else the centres are the kept points sel[b, 0..Ns)
// and the lists hold their row numbers j
hipError_t launch_inedges_build_sub(const int32_t *nbr, const int32_t *sel, int B, int N, int Ns, int K,
                                    int32_t *in_off, int32_t *in_src, void *ws, hipStream_t s)
{
    const int64_t BN = (int64_t)B * N, KN = (int64_t)K * N, E = (int64_t)B * K * (sel ? Ns : N);
    const int64_t nblk64 = cdiv64(BN, SCAN_CHUNK);
    const int nblk = (int)nblk64;
    int32_t *cnt = (int32_t *)ws;
    int32_t *bsum = (int32_t *)((char *)ws + align256(sizeof(int32_t) * (size_t)BN));
    hipError_t e = launch_fill_zero(cnt, sizeof(int32_t) * (size_t)BN, s);
    if (e != hipSuccess) return e;
    int64_t eb = (E + 255) / 256;
    if (eb > (1 << 18)) eb = 1 << 18;
    if (sel)
        hipLaunchKernelGGL(inedge_sub_count_kernel, dim3((unsigned)eb), dim3(256), 0, s, nbr, sel, cnt, E, N, Ns, K);
    else
        hipLaunchKernelGGL(inedge_count_kernel, dim3((unsigned)eb), dim3(256), 0, s, nbr, cnt, E, N, KN);
    hipLaunchKernelGGL(scan_block_sums_kernel, dim3(nblk), dim3(256), 0, s, cnt, bsum, BN);
    hipLaunchKernelGGL(scan_of_sums_kernel, dim3(1), dim3(256), 0, s, bsum, nblk);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(nblk), dim3(256), 0, s, cnt, bsum, in_off, BN, nblk);
    if (sel)
        hipLaunchKernelGGL(inedge_sub_fill_kernel, dim3((unsigned)eb), dim3(256), 0, s, nbr, sel, in_off, cnt, in_src,
                           E, N, Ns, K);
    else
        hipLaunchKernelGGL(inedge_fill_kernel, dim3((unsigned)eb), dim3(256), 0, s, nbr, in_off, cnt, in_src, E, N, KN);
    int64_t sb = (BN + 255) / 256;
    if (sb > (1 << 18)) sb = 1 << 18;
    hipLaunchKernelGGL(inedge_sort_kernel, dim3((unsigned)sb), dim3(256), 0, s, in_off, in_src, BN);
    return hipGetLastError();
}

}  // namespace flex
