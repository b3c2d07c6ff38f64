// Tiled matrix-core kernels for the flex-convolution layer (gfx950, wave64).
//
// The weight of Eq.(6) is linear in the position difference, so the neighbour
// sum of Eq.(4) factors per centre point l into
//     A[l][j*DI + c] = sum_k dp_j(l,k) * row[n_k(l)][c]   (j = 0,1,2: x,y,z)
//     A[l][3*DI + c] = sum_k            row[n_k(l)][c]
//     out[l][o]      = sum_{j,c} A[l][j*DI + c] * ThetaP[j*DI + c][o]
// A workgroup owns a tile of T points:
//   stage   neighbour ids and position differences of the tile -> LDS
//   gather  whole point-major rows (LPR lanes x 16 B) and accumulate A in
//           registers, then park the T x KD aggregate in LDS
//   contract on the matrix cores (v_mfma_f32_16x16x4_f32); the ThetaP
//           fragments of this wave's output slice stay in registers for the
//           whole persistent loop.
// The same kernel serves grad_feat: there the "rows" are grad_out rows, the
// neighbour lists are each point's in-edges (variable length, CSR), the
// position difference changes sign and ThetaP is the transposed parameter.
#pragma once
#include "flex_common.hpp"

namespace flex {

template <int DI_, int DO_, int WAVES_, int T_, int OCC_>
struct TileShape {
    static constexpr int DI = DI_, DO = DO_, WAVES = WAVES_, T = T_, OCC = OCC_;
    static constexpr int NT = 64 * WAVES;
    static constexpr int DIP = rup_c(DI, 4);               // gathered width, padded
    static constexpr int KD = 4 * DIP;                     // contraction depth
    static constexpr int DOP = rup_c(DO, 16);              // output width, padded
    static constexpr int VEC = (DI % 4 == 0) ? 4 : 1;      // floats per lane per row
    static constexpr int LPR = npow2_c(cdiv_c(DIP, VEC));  // lanes per gathered row
    static constexpr int PPP = NT / LPR;                   // points per gather pass
    static constexpr int PASSES = cdiv_c(T, PPP);
    static constexpr int ECAP = 512;                       // staged edges per chunk
    static_assert(LPR <= 64, "row wider than one wave");
    static_assert(T % 16 == 0 && ECAP % T == 0, "tile size");
    static_assert(KD % 16 == 0, "depth");
};

// One staged edge: global row id of the gathered point and the position difference.
struct __attribute__((aligned(16))) Edge {
    int row;
    float dx, dy, dz;
};

// XCD-aware persistent tile schedule.  Workgroups are dealt to the 8 XCDs
// round-robin by block id; each XCD gets one contiguous eighth of the tiles so
// that tiles in flight on one XCD (and its private L2) are spatial neighbours.
struct TileSchedule {
    int first, end, step;
    TileSchedule() = default;
    __device__ __forceinline__ TileSchedule(int total_tiles)
    {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int per_xcd = (total_tiles + 7) >> 3;
        first = xcd * per_xcd + slot;
        end = min((xcd + 1) * per_xcd, total_tiles);
        step = gridDim.x >> 3;
    }
    // share `part` of `parts`, for launches whose workgroups are split over several jobs: the same XCD-aware walk
    // when a job's workgroups are a multiple of 8 starting at a multiple of 8 (then part & 7 is the workgroup's
    // XCD), a plain strided one otherwise
    __device__ __forceinline__ TileSchedule(int total_tiles, int part, int parts)
    {
        if ((parts & 7) == 0) {
            const int xcd = part & 7, slot = part >> 3;
            const int per_xcd = (total_tiles + 7) >> 3;
            first = xcd * per_xcd + slot;
            end = min((xcd + 1) * per_xcd, total_tiles);
            step = parts >> 3;
        } else {
            first = part;
            end = total_tiles;
            step = parts;
        }
    }
};

template <class S, int U, bool CSR>
__device__ __forceinline__ void accumulate_edges(float (&acc)[4][S::VEC], const Edge *s_e,
                                                 const float *__restrict__ rows, int first,
                                                 int count, int stride, int t)
{
    // edges first, first+stride, ... (count of them); U rows in flight per step
    for (int e0 = 0; e0 < count; e0 += U) {
        Edge e[U];
        float f[U][S::VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool on = (e0 + u) < count;
            e[u] = s_e[on ? first + (e0 + u) * stride : first];
            if (!on) { e[u].dx = 0.f; e[u].dy = 0.f; e[u].dz = 0.f; }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool on = (e0 + u) < count;
            const float *p = rows + (int64_t)e[u].row * S::DI + S::VEC * t;
            if constexpr (S::VEC == 4) {
                v4f v = {0.f, 0.f, 0.f, 0.f};
                if (on) v = *reinterpret_cast<const v4f *>(p);
                f[u][0] = v.x; f[u][1] = v.y; f[u][2] = v.z; f[u][3] = v.w;
            } else {
                f[u][0] = on ? *p : 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int v = 0; v < S::VEC; ++v) {
                acc[0][v] = fmaf(e[u].dx, f[u][v], acc[0][v]);
                acc[1][v] = fmaf(e[u].dy, f[u][v], acc[1][v]);
                acc[2][v] = fmaf(e[u].dz, f[u][v], acc[2][v]);
                acc[3][v] += f[u][v];
            }
    }
}

// Fills s_A[T][AST] with the aggregate of the tile (rows >= npts are zero) and
// ends with a barrier.  CSR == false: fixed-K neighbour tensor, dp = pos[n]-pos[l].
// CSR == true: in-edge lists, dp = pos[centre]-pos[source].
template <class S, int AST, bool CSR>
__device__ __forceinline__ void build_aggregate(float *s_A, Edge *s_e, int *s_pb,
                                                const float *__restrict__ rows,
                                                const float *__restrict__ pos,
                                                const int32_t *__restrict__ nbr,
                                                const int32_t *__restrict__ off,
                                                const int32_t *__restrict__ src,
                                                int b, int l0, int npts, int N, int K)
{
    const int tid = threadIdx.x;
    const int grp = tid / S::LPR, t = tid % S::LPR;
    const bool lane_on = (S::VEC * t) < S::DI;
    const float *px = pos + (int64_t)b * 3 * N;
    const float *py = px + N;
    const float *pz = py + N;
    const int rowbase = b * N;

    float acc[S::PASSES][4][S::VEC];
#pragma unroll
    for (int p = 0; p < S::PASSES; ++p)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < S::VEC; ++v) acc[p][j][v] = 0.f;

    if constexpr (!CSR) {
        constexpr int KC = S::ECAP / S::T;
        for (int k0 = 0; k0 < K; k0 += KC) {
            const int kc = min(KC, K - k0);
            if (k0 > 0) __syncthreads();   // readers of the previous chunk are done
            for (int idx = tid; idx < kc * S::T; idx += S::NT) {
                const int kk = idx / S::T, j = idx % S::T;
                Edge e = {0, 0.f, 0.f, 0.f};
                if (j < npts) {
                    const int l = l0 + j;
                    const int n = nbr[((int64_t)b * K + (k0 + kk)) * N + l];
                    e.row = rowbase + n;
                    e.dx = px[n] - px[l];
                    e.dy = py[n] - py[l];
                    e.dz = pz[n] - pz[l];
                }
                s_e[idx] = e;
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < S::PASSES; ++p) {
                const int j = p * S::PPP + grp;
                if (j < npts && lane_on)
                    accumulate_edges<S, 8, CSR>(acc[p], s_e, rows, j, kc, S::T, t);
            }
        }
    } else {
        const int64_t gp0 = (int64_t)b * N + l0;
        for (int j = tid; j <= S::T; j += S::NT) s_pb[j] = off[gp0 + min(j, npts)];
        __syncthreads();
        const int ebeg = s_pb[0], eend = s_pb[S::T];
        for (int c0 = ebeg; c0 < eend; c0 += S::ECAP) {
            if (c0 > ebeg) __syncthreads();
            const int ce = min(S::ECAP, eend - c0);
            for (int idx = tid; idx < ce; idx += S::NT) {
                const int e_id = c0 + idx;
                int lo = 0, hi = S::T;   // s_pb[lo] <= e_id < s_pb[hi]
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (s_pb[mid] <= e_id) lo = mid; else hi = mid;
                }
                const int m = l0 + lo;
                const int l = src[e_id];
                Edge e;
                e.row = rowbase + l;
                e.dx = px[m] - px[l];
                e.dy = py[m] - py[l];
                e.dz = pz[m] - pz[l];
                s_e[idx] = e;
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < S::PASSES; ++p) {
                const int j = p * S::PPP + grp;
                if (j < npts && lane_on) {
                    const int lo_e = max(s_pb[j], c0), hi_e = min(s_pb[j + 1], c0 + ce);
                    if (hi_e > lo_e)
                        accumulate_edges<S, 4, CSR>(acc[p], s_e, rows, lo_e - c0, hi_e - lo_e, 1, t);
                }
            }
        }
    }

#pragma unroll
    for (int p = 0; p < S::PASSES; ++p) {
        const int j = p * S::PPP + grp;
        if (j < S::T && (S::VEC * t) < S::DIP) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                float *dst = s_A + j * AST + jj * S::DIP + S::VEC * t;
                if constexpr (S::VEC == 4) {
                    v4f v = {acc[p][jj][0], acc[p][jj][1], acc[p][jj][2], acc[p][jj][3]};
                    *reinterpret_cast<v4f *>(dst) = v;
                } else {
                    dst[0] = acc[p][jj][0];
                }
            }
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// out[l][:] = A[l][:] * ThetaP   (forward, or grad_feat when CSR)
// ---------------------------------------------------------------------------
template <class S, bool CSR, bool OUT_BCN>
__global__ __launch_bounds__(S::NT) __attribute__((amdgpu_waves_per_eu(S::OCC)))
void gather_contract_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                            const int32_t *__restrict__ nbr, const int32_t *__restrict__ off,
                            const int32_t *__restrict__ src, const float *__restrict__ thetaP,
                            float *__restrict__ out, int N, int K, int tiles_per_cloud,
                            int total_tiles)
{
    constexpr int AST = S::KD + 4;   // row stride: 16-byte reads of 16 rows hit distinct banks
    __shared__ __attribute__((aligned(16))) float s_A[S::T * AST];
    __shared__ Edge s_e[S::ECAP];
    __shared__ int s_pb[S::T + 1];

    constexpr int NS = S::DOP / 16;          // 16-wide output slices
    constexpr int NB = S::T / 16;            // 16-point blocks
    constexpr int NITEMS = NS * NB;
    constexpr int TS = (NS > S::WAVES) ? NS / S::WAVES : 1;   // slices whose theta a wave holds
    static_assert((S::WAVES % NS == 0) || (NS % S::WAVES == 0), "slice/wave split");
    constexpr int IPW = cdiv_c(NITEMS, S::WAVES);
    constexpr int KS = S::KD / 16;
    constexpr int NCH = (IPW == 1) ? 2 : 1;  // independent accumulation chains per item

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int q = lane >> 4, r = lane & 15;

    // ThetaP fragments (matrix A operand: rows = output channel, cols = depth).
    // Lane group q of depth step (s,i) covers depth 16*s + 4*q + i, matching the
    // 16-byte LDS reads of the aggregate below.
    float th[TS][S::KD / 4];
#pragma unroll
    for (int si = 0; si < TS; ++si) {
        const int slice = (NS > S::WAVES) ? (w + si * S::WAVES) : (w % NS);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                th[si][4 * s + i] = thetaP[(int64_t)(16 * s + 4 * q + i) * S::DOP + slice * 16 + r];
    }

    const TileSchedule sched(total_tiles);
    for (int tile = sched.first; tile < sched.end; tile += sched.step) {
        const int b = tile / tiles_per_cloud;
        const int l0 = (tile - b * tiles_per_cloud) * S::T;
        const int npts = min(S::T, N - l0);

        build_aggregate<S, AST, CSR>(s_A, s_e, s_pb, rows, pos, nbr, off, src, b, l0, npts, N, K);

        v4f acc[IPW][NCH];
#pragma unroll
        for (int it = 0; it < IPW; ++it)
#pragma unroll
            for (int c = 0; c < NCH; ++c) acc[it][c] = v4f{0.f, 0.f, 0.f, 0.f};

#pragma unroll
        for (int s = 0; s < KS; ++s) {
            v4f bf[IPW];
#pragma unroll
            for (int it = 0; it < IPW; ++it) {
                const int idx = w + it * S::WAVES;
                const int blk = (NS > S::WAVES) ? (it / TS) : (idx / NS);
                bf[it] = v4f{0.f, 0.f, 0.f, 0.f};
                if (idx < NITEMS)
                    bf[it] = *reinterpret_cast<const v4f *>(&s_A[(blk * 16 + r) * AST + 16 * s + 4 * q]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int it = 0; it < IPW; ++it) {
                    const int si = (NS > S::WAVES) ? (it % TS) : 0;
                    acc[it][s % NCH] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                        th[si][4 * s + i], bf[it][i], acc[it][s % NCH], 0, 0, 0);
                }
        }

        // D[m][n]: m = output channel 4*q+i of the slice, n = point r of the block.
#pragma unroll
        for (int it = 0; it < IPW; ++it) {
            const int idx = w + it * S::WAVES;
            if (idx >= NITEMS) continue;
            const int slice = (NS > S::WAVES) ? (w + (it % TS) * S::WAVES) : (w % NS);
            const int blk = (NS > S::WAVES) ? (it / TS) : (idx / NS);
            v4f d = acc[it][0];
            if constexpr (NCH == 2) d += acc[it][1];
            const int pt = blk * 16 + r;
            const int o = slice * 16 + 4 * q;
            if (pt < npts) {
                if constexpr (OUT_BCN) {
                    float *dst = out + ((int64_t)b * S::DO + o) * N + (l0 + pt);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (o + i < S::DO) dst[(int64_t)i * N] = d[i];
                } else {
                    float *dst = out + ((int64_t)b * N + l0 + pt) * S::DO + o;
                    if constexpr (S::DO % 4 == 0) {
                        if (o < S::DO) *reinterpret_cast<v4f *>(dst) = d;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (o + i < S::DO) dst[i] = d[i];
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Per-workgroup partial of  gradTheta[kd][o] = sum_l A[l][kd] * g[l][o].
// ---------------------------------------------------------------------------
template <class S>
__global__ __launch_bounds__(S::NT) __attribute__((amdgpu_waves_per_eu(S::OCC)))
void grad_theta_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                       const int32_t *__restrict__ nbr, const float *__restrict__ g_rows,
                       float *__restrict__ partials, int N, int K, int tiles_per_cloud,
                       int total_tiles)
{
    constexpr int AST = S::KD + 16;   // row stride = 16 mod 32: two 16-lane groups, disjoint banks
    constexpr int GST = S::DOP + 16;
    __shared__ __attribute__((aligned(16))) float s_A[S::T * AST];
    __shared__ __attribute__((aligned(16))) float s_G[S::T * GST];
    __shared__ Edge s_e[S::ECAP];

    constexpr int MB = S::KD / 16, NB2 = S::DOP / 16;
    constexpr int WN = (NB2 < S::WAVES) ? NB2 : S::WAVES;
    static_assert(S::WAVES % WN == 0 && NB2 % WN == 0, "wave grid");
    constexpr int WM = S::WAVES / WN;
    constexpr int NBW = NB2 / WN;
    constexpr int MBW = cdiv_c(MB, WM);

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int q = lane >> 4, r = lane & 15;
    const int wn = w % WN, wm = w / WN;

    v4f acc[MBW][NBW];
#pragma unroll
    for (int c = 0; c < MBW; ++c)
#pragma unroll
        for (int a = 0; a < NBW; ++a) acc[c][a] = v4f{0.f, 0.f, 0.f, 0.f};

    const TileSchedule sched(total_tiles);
    for (int tile = sched.first; tile < sched.end; tile += sched.step) {
        const int b = tile / tiles_per_cloud;
        const int l0 = (tile - b * tiles_per_cloud) * S::T;
        const int npts = min(S::T, N - l0);

        __syncthreads();   // every wave has finished the previous tile's contraction
        for (int idx = threadIdx.x; idx < S::T * S::DOP; idx += S::NT) {
            const int j = idx / S::DOP, o = idx % S::DOP;
            float v = 0.f;
            if (j < npts && o < S::DO) v = g_rows[((int64_t)b * N + l0 + j) * S::DO + o];
            s_G[j * GST + o] = v;
        }
        build_aggregate<S, AST, false>(s_A, s_e, nullptr, rows, pos, nbr, nullptr, nullptr, b, l0,
                                       npts, N, K);

#pragma unroll
        for (int s = 0; s < S::T / 4; ++s) {
            const int row = 4 * s + q;
            float af[MBW], gf[NBW];
#pragma unroll
            for (int c = 0; c < MBW; ++c) {
                const int mb = wm + c * WM;
                af[c] = (mb < MB) ? s_A[row * AST + mb * 16 + r] : 0.f;
            }
#pragma unroll
            for (int a = 0; a < NBW; ++a) gf[a] = s_G[row * GST + (wn + a * WN) * 16 + r];
#pragma unroll
            for (int c = 0; c < MBW; ++c)
#pragma unroll
                for (int a = 0; a < NBW; ++a)
                    acc[c][a] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[c], gf[a], acc[c][a], 0, 0, 0);
        }
    }

    float *dst = partials + (int64_t)blockIdx.x * S::KD * S::DOP;
#pragma unroll
    for (int c = 0; c < MBW; ++c) {
        const int mb = wm + c * WM;
        if (mb >= MB) continue;
#pragma unroll
        for (int a = 0; a < NBW; ++a) {
            const int nb = wn + a * WN;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                dst[(int64_t)(mb * 16 + 4 * q + i) * S::DOP + nb * 16 + r] = acc[c][a][i];
        }
    }
}


// ===========================================================================
// Pipelined kernels.  Same arithmetic as above, restructured so that the only
// memory latency a wave waits for inside a tile is the row gather itself:
//   * each wave owns PW consecutive points of the tile and stages their
//     neighbour entries in a wave-private slice of LDS (no workgroup barrier);
//   * the neighbour ids of the NEXT tile are fetched while the matrix cores
//     work on the current one;
//   * position loads are issued together with the row loads;
//   * the aggregate tile is double-buffered, so one barrier per tile suffices.
// Fixed-K mode needs PW*K <= EW staged entries per wave (the host picks the
// chunked kernel above otherwise); CSR mode walks lists of any length in
// wave-private chunks.
// ===========================================================================
template <class S>
struct WaveGeom {
    static constexpr int PW = S::T / S::WAVES;       // consecutive points per wave
    static constexpr int GPW = 64 / S::LPR;          // row groups per wave
    static constexpr int PASSES = cdiv_c(PW, GPW);
    static constexpr int SLOTS = (PW * 16 <= 64) ? 1 : 2;   // staged entries per lane: K <= 16 always fits
    static constexpr int EW = 64 * SLOTS;            // staged entries per wave
    static constexpr int U = 8;                      // rows in flight per lane
    static_assert(S::T % S::WAVES == 0, "points per wave");
    static_assert(S::LPR % 4 == 0, "4-lane blocks of the 4x4x1 matrix op must stay inside one row");
    static_assert(PW + 1 <= 64, "offsets live in one wave");
};

// Wave-private staging: for each staged entry the gathered row id and (dx,dy,dz,1).
template <class S>
struct WaveStage {
    int row[WaveGeom<S>::EW];
    v4f dp[WaveGeom<S>::EW];
};

// Orders LDS traffic between lanes of one wave (LDS executes a wave's
// instructions in order; this only stops the compiler from reordering).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <class S>
__device__ __forceinline__ void load_row(float (&f)[S::VEC], const float *__restrict__ rows, int row,
                                         int t, bool on)
{
    const float *p = rows + (int64_t)row * S::DI + S::VEC * t;
    if constexpr (S::VEC == 4) {
        v4f v = {0.f, 0.f, 0.f, 0.f};
        if (on) v = *reinterpret_cast<const v4f *>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    } else {
        f[0] = on ? *p : 0.f;
    }
}

// acc[v][j] += d[j] * f[v]  (j = x,y,z,1; acc[v] is the 4-float accumulator of channel v).  With 4-lane blocks that stay inside one
// gathered row this is sixteen 4x4 outer products per wave: one
// v_mfma_f32_4x4x1_16b_f32 per float of the lane (A = the lane's component of
// (dx,dy,dz,1), B = the feature), which runs on the matrix pipe instead of
// sixteen vector FMAs.  `dpc` is that component, already selected for this lane.
template <class S>
__device__ __forceinline__ void fma_row(v4f (&acc)[S::VEC], float dpc, const float (&f)[S::VEC])
{
#pragma unroll
    for (int v = 0; v < S::VEC; ++v)
        acc[v] = __builtin_amdgcn_mfma_f32_4x4x1f32(dpc, f[v], acc[v], 0, 0, 0);
}

// What a wave carries from one tile to the next.
template <class S>
struct Prefetch {
    int ids[WaveGeom<S>::SLOTS];   // fixed-K: neighbour ids; CSR: first chunk of source ids
    int off;                       // CSR: lane j <= PW holds the in-edge offset of wave point j
};

// Aggregate of this wave's PW points -> acc (registers).  s_w: wave-private staging.
template <class S, bool CSR>
__device__ __forceinline__ void wave_aggregate(v4f (&acc)[WaveGeom<S>::PASSES][S::VEC], WaveStage<S> *s_w,
                                               Prefetch<S> &pf, const float *__restrict__ rows,
                                               const float *__restrict__ px, const float *__restrict__ py,
                                               const float *__restrict__ pz,
                                               const int32_t *__restrict__ src, int rowbase, int lw0,
                                               int N, int K)
{
    using G = WaveGeom<S>;
    const int lane = threadIdx.x & 63;
    const int grp = lane / S::LPR, t = lane % S::LPR;
    const bool lane_on = (S::VEC * t) < S::DI;

#pragma unroll
    for (int p = 0; p < G::PASSES; ++p)
#pragma unroll
        for (int v = 0; v < S::VEC; ++v) acc[p][v] = v4f{0.f, 0.f, 0.f, 0.f};

    // CSR: in-edge offsets of the wave's points, wave-uniform (lane j of pf.off holds offset j)
    int offs[G::PW + 1];
#pragma unroll
    for (int j = 0; j <= G::PW; ++j) offs[j] = CSR ? __builtin_amdgcn_readlane(pf.off, j) : 0;

    // chunk loop (exactly one trip in fixed-K mode)
    const int e_begin = CSR ? offs[0] : 0;
    const int e_end = CSR ? offs[G::PW] : G::PW * K;
    for (int c0 = e_begin; c0 < e_end; c0 += G::EW) {
        const int cnt = min(G::EW, e_end - c0);
        if (CSR && c0 > e_begin) {
#pragma unroll
            for (int s = 0; s < G::SLOTS; ++s) {
                const int i = s * 64 + lane;
                pf.ids[s] = (i < cnt) ? src[c0 + i] : 0;
            }
        }
        // 1. publish the gathered rows' ids
#pragma unroll
        for (int s = 0; s < G::SLOTS; ++s) {
            const int i = s * 64 + lane;
            if (i < cnt) s_w->row[i] = rowbase + pf.ids[s];
        }
        wave_lds_sync();

        // 2. entry owners: raw position loads (difference taken after the rows are requested)
        float ax[G::SLOTS], ay[G::SLOTS], az[G::SLOTS], bx[G::SLOTS], by[G::SLOTS], bz[G::SLOTS];
#pragma unroll
        for (int s = 0; s < G::SLOTS; ++s) {
            const int i = s * 64 + lane;
            ax[s] = ay[s] = az[s] = bx[s] = by[s] = bz[s] = 0.f;
            if (i < cnt) {
                int pj;
                if constexpr (CSR) {
                    pj = 0;
#pragma unroll
                    for (int j = 1; j < G::PW; ++j) pj += (offs[j] <= c0 + i) ? 1 : 0;
                } else {
                    pj = i % G::PW;
                }
                const int l = min(lw0 + pj, N - 1);
                const int n = pf.ids[s];
                ax[s] = px[n]; ay[s] = py[n]; az[s] = pz[n];
                bx[s] = px[l]; by[s] = py[l]; bz[s] = pz[l];
            }
        }

        // 3. row groups: per pass, the entries [lo,hi) of the group's point
        int lo[G::PASSES], hi[G::PASSES], stride;
        bool act[G::PASSES];
#pragma unroll
        for (int p = 0; p < G::PASSES; ++p) {
            const int pj = p * G::GPW + grp;
            act[p] = (pj < G::PW) && (lw0 + pj < N);   // the point exists (every lane of its blocks feeds dp)
            if constexpr (CSR) {
                int a = offs[0], b = offs[1];
#pragma unroll
                for (int j = 1; j < G::PW; ++j)
                    if (pj == j) { a = offs[j]; b = offs[j + 1]; }
                lo[p] = max(a, c0) - c0;
                hi[p] = min(b, c0 + cnt) - c0;
            } else {
                lo[p] = pj;                      // entries pj, pj+PW, ... (K of them)
                hi[p] = pj + K * G::PW;
            }
            if (!act[p]) hi[p] = lo[p];
        }
        stride = CSR ? 1 : G::PW;

        const int dsel = lane & 3;   // this lane's row of the 4x4 blocks: dx, dy, dz or 1
        float f[G::U][S::VEC];
        auto load_batch = [&](int i0, int end) {
#pragma unroll
            for (int u = 0; u < G::U; ++u) {
                const int i = i0 + u * stride;
                const bool on = i < end;
                load_row<S>(f[u], rows, on ? s_w->row[i] : 0, t, on && lane_on);
            }
        };
        auto fma_batch = [&](int p, int i0, int end) {
#pragma unroll
            for (int u = 0; u < G::U; ++u) {
                const int i = i0 + u * stride;
                const float dpc = (i < end) ? reinterpret_cast<const float *>(&s_w->dp[i])[dsel] : 0.f;
                fma_row<S>(acc[p], dpc, f[u]);   // inactive: 0 * 0 (the matrix op ignores EXEC)
            }
        };

        load_batch(lo[0], hi[0]);
        // 4. owners publish the position differences
#pragma unroll
        for (int s = 0; s < G::SLOTS; ++s) {
            const int i = s * 64 + lane;
            if (i < cnt) {
                const float sg = CSR ? -1.f : 1.f;   // CSR: centre - source
                s_w->dp[i] = v4f{sg * (ax[s] - bx[s]), sg * (ay[s] - by[s]), sg * (az[s] - bz[s]), 1.f};
            }
        }
        wave_lds_sync();
        fma_batch(0, lo[0], hi[0]);
        for (int i0 = lo[0] + G::U * stride; i0 < hi[0]; i0 += G::U * stride) {
            load_batch(i0, hi[0]);
            fma_batch(0, i0, hi[0]);
        }
#pragma unroll
        for (int p = 1; p < G::PASSES; ++p)
            for (int i0 = lo[p]; i0 < hi[p]; i0 += G::U * stride) {
                load_batch(i0, hi[p]);
                fma_batch(p, i0, hi[p]);
            }
        wave_lds_sync();   // staging is reused by the next chunk
    }
}

// Writes this wave's PW rows of the aggregate tile.
template <class S, int AST>
__device__ __forceinline__ void wave_store_aggregate(float *s_A, const v4f (&acc)[WaveGeom<S>::PASSES][S::VEC])
{
    using G = WaveGeom<S>;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int grp = lane / S::LPR, t = lane % S::LPR;
#pragma unroll
    for (int p = 0; p < G::PASSES; ++p) {
        const int pj = p * G::GPW + grp;
        if (pj < G::PW && (S::VEC * t) < S::DIP) {
            float *row = s_A + (w * G::PW + pj) * AST + S::VEC * t;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if constexpr (S::VEC == 4) {
                    v4f v = {acc[p][0][jj], acc[p][1][jj], acc[p][2][jj], acc[p][3][jj]};
                    *reinterpret_cast<v4f *>(row + jj * S::DIP) = v;
                } else {
                    row[jj * S::DIP] = acc[p][0][jj];
                }
            }
        }
    }
}

// Start fetching what the next tile's aggregate needs first.
//   fixed-K: the neighbour ids (entry i = k*PW + pj of wave point pj)
//   CSR:     stage 0 loads the in-edge offsets, stage 1 (once they are here) the first source ids
template <class S, bool CSR>
__device__ __forceinline__ void prefetch_ids(Prefetch<S> &pf, const int32_t *__restrict__ nbr,
                                             const int32_t *__restrict__ off,
                                             const int32_t *__restrict__ src, int b, int lw0, int N,
                                             int K, int stage)
{
    using G = WaveGeom<S>;
    const int lane = threadIdx.x & 63;
    if constexpr (!CSR) {
        if (stage == 0) {
#pragma unroll
            for (int s = 0; s < G::SLOTS; ++s) {
                const int i = s * 64 + lane;
                int v = 0;
                if (i < G::PW * K) {
                    const int k = i / G::PW, l = lw0 + (i % G::PW);
                    if (l < N) v = nbr[((int64_t)b * K + k) * N + l];
                }
                pf.ids[s] = v;
            }
        }
    } else {
        if (stage == 0) {
            const int npw = max(0, min(G::PW, N - lw0));
            const int64_t g0 = (int64_t)b * N + min(lw0, N);
            pf.off = off[g0 + min(lane, npw)];
        } else {
            const int e0 = __builtin_amdgcn_readlane(pf.off, 0);
            const int e1 = __builtin_amdgcn_readlane(pf.off, G::PW);
#pragma unroll
            for (int s = 0; s < G::SLOTS; ++s) {
                const int e = e0 + s * 64 + lane;
                pf.ids[s] = (e < e1) ? src[e] : 0;
            }
        }
    }
}

template <class S, bool CSR, bool OUT_BCN>
__global__ __launch_bounds__(S::NT) __attribute__((amdgpu_waves_per_eu(S::OCC)))
void gather_contract_fast_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                                 const int32_t *__restrict__ nbr, const int32_t *__restrict__ off,
                                 const int32_t *__restrict__ src, const float *__restrict__ thetaP,
                                 float *__restrict__ out, int N, int K, int tiles_per_cloud,
                                 int total_tiles)
{
    using G = WaveGeom<S>;
    constexpr int AST = S::KD + 4;
    __shared__ __attribute__((aligned(16))) float s_A[2][S::T * AST];
    __shared__ WaveStage<S> s_e[S::WAVES];

    constexpr int NS = S::DOP / 16, NB = S::T / 16, NITEMS = NS * NB;
    constexpr int TS = (NS > S::WAVES) ? NS / S::WAVES : 1;
    static_assert((S::WAVES % NS == 0) || (NS % S::WAVES == 0), "slice/wave split");
    constexpr int IPW = cdiv_c(NITEMS, S::WAVES);
    constexpr int KS = S::KD / 16;
    constexpr int NCH = (IPW == 1) ? 2 : 1;

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int q = lane >> 4, r = lane & 15;

    float th[TS][S::KD / 4];
#pragma unroll
    for (int si = 0; si < TS; ++si) {
        const int slice = (NS > S::WAVES) ? (w + si * S::WAVES) : (w % NS);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                th[si][4 * s + i] = thetaP[(int64_t)(16 * s + 4 * q + i) * S::DOP + slice * 16 + r];
    }

    const TileSchedule sched(total_tiles);
    Prefetch<S> pf;
    pf.off = 0;
#pragma unroll
    for (int s = 0; s < G::SLOTS; ++s) pf.ids[s] = 0;
    if (sched.first < sched.end) {
        const int b = sched.first / tiles_per_cloud;
        const int lw0 = (sched.first - b * tiles_per_cloud) * S::T + w * G::PW;
        prefetch_ids<S, CSR>(pf, nbr, off, src, b, lw0, N, K, 0);
        if (CSR) prefetch_ids<S, CSR>(pf, nbr, off, src, b, lw0, N, K, 1);
    }

    int buf = 0;
    for (int tile = sched.first; tile < sched.end; tile += sched.step, buf ^= 1) {
        const int b = tile / tiles_per_cloud;
        const int l0 = (tile - b * tiles_per_cloud) * S::T;
        const int npts = min(S::T, N - l0);
        const float *px = pos + (int64_t)b * 3 * N, *py = px + N, *pz = py + N;
        float *sA = s_A[buf];

        {
            v4f agg[G::PASSES][S::VEC];
            wave_aggregate<S, CSR>(agg, &s_e[w], pf, rows, px, py, pz, src, b * N, l0 + w * G::PW, N, K);
            wave_store_aggregate<S, AST>(sA, agg);
        }

        // next tile: first stage of the id fetch rides under the contraction
        const int nt = tile + sched.step;
        const bool has_next = nt < sched.end;
        const int nb_ = has_next ? nt / tiles_per_cloud : 0;
        const int nlw0 = has_next ? (nt - nb_ * tiles_per_cloud) * S::T + w * G::PW : 0;
        if (has_next) prefetch_ids<S, CSR>(pf, nbr, off, src, nb_, nlw0, N, K, 0);

        __syncthreads();   // aggregate tile complete (the other buffer is free again)

        v4f acc[IPW][NCH];
#pragma unroll
        for (int it = 0; it < IPW; ++it)
#pragma unroll
            for (int c = 0; c < NCH; ++c) acc[it][c] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            v4f bf[IPW];
#pragma unroll
            for (int it = 0; it < IPW; ++it) {
                const int idx = w + it * S::WAVES;
                const int blk = (NS > S::WAVES) ? (it / TS) : (idx / NS);
                bf[it] = v4f{0.f, 0.f, 0.f, 0.f};
                if (idx < NITEMS)
                    bf[it] = *reinterpret_cast<const v4f *>(&sA[(blk * 16 + r) * AST + 16 * s + 4 * q]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int it = 0; it < IPW; ++it) {
                    const int si = (NS > S::WAVES) ? (it % TS) : 0;
                    acc[it][s % NCH] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                        th[si][4 * s + i], bf[it][i], acc[it][s % NCH], 0, 0, 0);
                }
        }

        if (CSR && has_next) prefetch_ids<S, CSR>(pf, nbr, off, src, nb_, nlw0, N, K, 1);

#pragma unroll
        for (int it = 0; it < IPW; ++it) {
            const int idx = w + it * S::WAVES;
            if (idx >= NITEMS) continue;
            const int slice = (NS > S::WAVES) ? (w + (it % TS) * S::WAVES) : (w % NS);
            const int blk = (NS > S::WAVES) ? (it / TS) : (idx / NS);
            v4f d = acc[it][0];
            if constexpr (NCH == 2) d += acc[it][1];
            const int pt = blk * 16 + r;
            const int o = slice * 16 + 4 * q;
            if (pt < npts) {
                if constexpr (OUT_BCN) {
                    float *dst = out + ((int64_t)b * S::DO + o) * N + (l0 + pt);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (o + i < S::DO) dst[(int64_t)i * N] = d[i];
                } else {
                    float *dst = out + ((int64_t)b * N + l0 + pt) * S::DO + o;
                    if constexpr (S::DO % 4 == 0) {
                        if (o < S::DO) *reinterpret_cast<v4f *>(dst) = d;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (o + i < S::DO) dst[i] = d[i];
                    }
                }
            }
        }
    }
}

// Pipelined grad_theta partials (fixed-K, PW*K <= EW).
template <class S>
__global__ __launch_bounds__(S::NT) __attribute__((amdgpu_waves_per_eu(S::OCC)))
void grad_theta_fast_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                            const int32_t *__restrict__ nbr, const float *__restrict__ g_rows,
                            float *__restrict__ partials, int N, int K, int tiles_per_cloud,
                            int total_tiles)
{
    using G = WaveGeom<S>;
    constexpr int AST = S::KD + 16;
    constexpr int GST = S::DOP + 16;
    __shared__ __attribute__((aligned(16))) float s_A[2][S::T * AST];
    __shared__ __attribute__((aligned(16))) float s_G[2][S::T * GST];
    __shared__ WaveStage<S> s_e[S::WAVES];

    constexpr int MB = S::KD / 16, NB2 = S::DOP / 16;
    constexpr int WN = (NB2 < S::WAVES) ? NB2 : S::WAVES;
    static_assert(S::WAVES % WN == 0 && NB2 % WN == 0, "wave grid");
    constexpr int WM = S::WAVES / WN;
    constexpr int NBW = NB2 / WN;
    constexpr int MBW = cdiv_c(MB, WM);
    constexpr int GPT = cdiv_c(S::T * S::DOP, S::NT);   // grad_out elements per thread

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int q = lane >> 4, r = lane & 15;
    const int wn = w % WN, wm = w / WN;

    v4f acc[MBW][NBW];
#pragma unroll
    for (int c = 0; c < MBW; ++c)
#pragma unroll
        for (int a = 0; a < NBW; ++a) acc[c][a] = v4f{0.f, 0.f, 0.f, 0.f};

    const TileSchedule sched(total_tiles);
    Prefetch<S> pf;
    pf.off = 0;
#pragma unroll
    for (int s = 0; s < G::SLOTS; ++s) pf.ids[s] = 0;
    if (sched.first < sched.end) {
        const int b = sched.first / tiles_per_cloud;
        const int lw0 = (sched.first - b * tiles_per_cloud) * S::T + w * G::PW;
        prefetch_ids<S, false>(pf, nbr, nullptr, nullptr, b, lw0, N, K, 0);
    }

    int buf = 0;
    for (int tile = sched.first; tile < sched.end; tile += sched.step, buf ^= 1) {
        const int b = tile / tiles_per_cloud;
        const int l0 = (tile - b * tiles_per_cloud) * S::T;
        const int npts = min(S::T, N - l0);
        const float *px = pos + (int64_t)b * 3 * N, *py = px + N, *pz = py + N;
        float *sA = s_A[buf], *sG = s_G[buf];

        // grad_out tile: requested now, parked in LDS after the gather
        float gv[GPT];
#pragma unroll
        for (int i = 0; i < GPT; ++i) {
            const int idx = threadIdx.x + i * S::NT;
            const int j = idx / S::DOP, o = idx % S::DOP;
            gv[i] = 0.f;
            if (idx < S::T * S::DOP && j < npts && o < S::DO)
                gv[i] = g_rows[((int64_t)b * N + l0 + j) * S::DO + o];
        }
        {
            v4f agg[G::PASSES][S::VEC];
            wave_aggregate<S, false>(agg, &s_e[w], pf, rows, px, py, pz, nullptr, b * N, l0 + w * G::PW, N, K);
            wave_store_aggregate<S, AST>(sA, agg);
        }
#pragma unroll
        for (int i = 0; i < GPT; ++i) {
            const int idx = threadIdx.x + i * S::NT;
            if (idx < S::T * S::DOP) sG[(idx / S::DOP) * GST + (idx % S::DOP)] = gv[i];
        }
        const int nt = tile + sched.step;
        if (nt < sched.end) {
            const int nb_ = nt / tiles_per_cloud;
            prefetch_ids<S, false>(pf, nbr, nullptr, nullptr, nb_, (nt - nb_ * tiles_per_cloud) * S::T + w * G::PW, N, K, 0);
        }
        __syncthreads();

#pragma unroll
        for (int s = 0; s < S::T / 4; ++s) {
            const int row = 4 * s + q;
            float af[MBW], gf[NBW];
#pragma unroll
            for (int c = 0; c < MBW; ++c) {
                const int mb = wm + c * WM;
                af[c] = (mb < MB) ? sA[row * AST + mb * 16 + r] : 0.f;
            }
#pragma unroll
            for (int a = 0; a < NBW; ++a) gf[a] = sG[row * GST + (wn + a * WN) * 16 + r];
#pragma unroll
            for (int c = 0; c < MBW; ++c)
#pragma unroll
                for (int a = 0; a < NBW; ++a)
                    acc[c][a] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[c], gf[a], acc[c][a], 0, 0, 0);
        }
    }

    float *dst = partials + (int64_t)blockIdx.x * S::KD * S::DOP;
#pragma unroll
    for (int c = 0; c < MBW; ++c) {
        const int mb = wm + c * WM;
        if (mb >= MB) continue;
#pragma unroll
        for (int a = 0; a < NBW; ++a) {
            const int nb = wn + a * WN;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                dst[(int64_t)(mb * 16 + 4 * q + i) * S::DOP + nb * 16 + r] = acc[c][a][i];
        }
    }
}

}  // namespace flex
