// Wave-specialised flex-convolution kernels (gfx950, wave64).
//
// A workgroup is W PRODUCER waves plus W CONSUMER waves (W = S::WAVES; 16 waves
// per CU in total, i.e. 16/(2W) workgroups).  Producers gather neighbour rows
// and build the per-point aggregate A (see flex_tiled.hpp for the factoring),
// consumers contract it with the packed parameters on the matrix cores.  The
// aggregate tile is double-buffered in LDS and the two halves meet at one
// workgroup barrier per tile, so tile k+1 is being gathered while tile k is
// being contracted:
//
//   producers, iteration k:   request rows / positions of tile k+1 and the
//                             neighbour ids of tile k+2;  finish tile k (its
//                             rows were requested one iteration ago) -> A[k%2];
//                             barrier
//   consumers, iteration k:   barrier;  out[tile k] = A[k%2] * ThetaP
//
// Only consumers keep the parameter fragments in registers, producers spend
// theirs on two tiles' worth of loads in flight; both fit 128 VGPRs, i.e. 4
// waves per SIMD.  Every memory latency on the producer side has a full barrier
// interval (one tile contraction) to complete.  With W = 4 two workgroups share
// a CU and drift apart, so one group's barrier / store phase is covered by the
// other group's contraction.
//
// Limits (the host falls back to the kernels of flex_tiled.hpp otherwise):
// one gather pass per producer wave, fixed-K lists with PW*K <= 64 staged
// entries; in-edge lists (CSR) of any length (entries past the first 64 of a
// wave, or past the first 8 of a point, are fetched synchronously).
#pragma once
#include "flex_tiled.hpp"

#ifndef FLEX_LEAN_VALU_AGG
#define FLEX_LEAN_VALU_AGG 1
#endif
// 1: the position differences reach the compute lanes as (dx, dy, dz, w) through a wave-private LDS array (one
// 16-byte read per row); 0: one component per lane by ds_bpermute, then three quad broadcasts per row
#ifndef FLEX_DP_LDS
#define FLEX_DP_LDS 1
#endif

namespace flex {

template <class S, int PM = 1, int CM = 1>
struct WsGeom {
    static constexpr int NP = S::WAVES * PM, NC = S::WAVES * CM;   // producer / consumer waves
    static constexpr int NT = 64 * (NP + NC);
    static constexpr int WG_PER_CU = 16 / (NP + NC);
    static constexpr int T = S::T * PM;                  // points per tile
    static constexpr int PW = T / NP;                    // points per producer wave
    static constexpr int GPW = 64 / S::LPR;              // row groups per wave
    static constexpr int EW = 64;                        // staged entries per producer wave
    static constexpr int U = 8;                          // rows in flight per lane
    static constexpr int AST = S::KD + 4;
    static_assert(T % NP == 0 && GPW >= PW, "one gather pass per producer wave");
    static_assert(PW * 16 <= EW, "K <= 16 always fits the staging");
    static_assert(S::LPR % 4 == 0, "4-lane blocks stay inside one row");
    static constexpr int NS = S::DOP / 16;               // 16-wide output slices
    static constexpr int NB = T / 16;                    // 16-point blocks
    static constexpr int NITEMS = NS * NB;
    static_assert(NITEMS % NC == 0 || NC % NITEMS == 0, "items per consumer wave");
    static constexpr int IPW = cdiv_c(NITEMS, NC);
    static_assert(IPW == 1 || NS % NC == 0 || NC % NS == 0, "slice split");
    // split-half aggregate tile: per point [hi: KDP halves][lo: KDP halves][16 B pad]
    static constexpr int KDP = rup_c(S::KD, 32);         // depth padded to the f16 matrix op
    static constexpr int KS2 = KDP / 32;                 // depth steps of v_mfma_f32_16x16x32_f16
    static constexpr int ARS = 4 * KDP + 16;             // row stride in bytes (= 16 mod 128: 16-byte reads of
                                                         // 8 consecutive rows hit distinct banks)
    static constexpr int ROWB_F32 = 4 * AST;
    static constexpr int ROWB = ARS > ROWB_F32 ? ARS : ROWB_F32;
};

// max over the LPR lanes of a gathered row's lane group (all lanes of the wave take part)
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
template <int LPR>
__device__ __forceinline__ float group_max(float m)
{
    m = fmaxf(m, dpp_move<0xB1>(m));                           // quad_perm [1,0,3,2]
    m = fmaxf(m, dpp_move<0x4E>(m));                           // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) m = fmaxf(m, dpp_move<0x141>(m));  // row_half_mirror
    if constexpr (LPR >= 16) m = fmaxf(m, dpp_move<0x140>(m)); // row_mirror
    if constexpr (LPR >= 32) m = fmaxf(m, __shfl_xor(m, 16));
    return m;
}

// Writes one point's aggregate (this lane: channels VEC*t.., all four j) as split-half rows:
// the row is scaled by 2^e so that its largest magnitude lands in [2^14, 2^15), e goes to sE[pt].
// Every lane of the wave calls this (the row maximum is taken across the lane group).
// max(m, |a|, |b|) for finite inputs, m >= 0 (one v_max3_f32 with |.| source modifiers)
__device__ __forceinline__ float fmax3_abs(float m, float a, float b)
{
    return __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fabsf(a), __builtin_fabsf(b)));
}

// The depth scales of the packed parameters that belong to this lane's aggregate elements (channels VEC*t..,
// all four j): rs[v][j] = rscale[j*DIP + VEC*t + v], see pack_theta_f16_block.  thetaP: the packed buffer.
template <class S>
__device__ __forceinline__ void load_row_scales(float (&rs)[S::VEC][4], const void *thetaP, int theta_exp_off, int t)
{
    const float *rscale = reinterpret_cast<const float *>(reinterpret_cast<const char *>(thetaP) + theta_exp_off +
                                                          rup_c(4 * S::DOP, 256));
#pragma unroll
    for (int v = 0; v < S::VEC; ++v)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int c = S::VEC * t + v;
            rs[v][jj] = c < S::DIP ? rscale[jj * S::DIP + c] : 1.f;
        }
}

// The swizzled form of the split-half tile (SWZ): rows exactly 4*KDP bytes apart and, inside every 128-byte block
// of a row, the 16-byte chunk index XORed with tile_swizzle(row).  Both ways the tile is read are then free of
// bank conflicts: 16-byte fragments of 8 consecutive rows at one column (the contraction with the parameters) and
// 32-byte runs of 4 consecutive rows (the transposing reads of the contraction over the tile's points).
__device__ __forceinline__ int tile_swizzle(int row) { return (2 * (row & 3) + ((row >> 2) & 1)) << 4; }

template <class S, bool SWZ = false>
__device__ __forceinline__ void store_split_rows(const v4f (&acc_in)[S::VEC], const float (&rs)[S::VEC][4], char *sA,
                                                 int *sE, int pt, int t, bool writer)
{
    using G = WsGeom<S>;   // row format only: the same for every producer multiple
    static_assert(!SWZ || (S::VEC == 4 && (2 * S::DIP) % 128 == 0 && G::KDP == S::KD), "swizzle inside 128-byte blocks");
    v4f acc[S::VEC];
    float m = 0.f;
#pragma unroll
    for (int v = 0; v < S::VEC; ++v)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            acc[v][jj] = acc_in[v][jj] * rs[v][jj];      // the parameters' depth scale (a power of two: exact)
            m = __builtin_amdgcn_fmed3f(m, __builtin_fabsf(acc[v][jj]), __builtin_inff());   // max(m, |a|), one op
        }
    m = group_max<S::LPR>(m);
    const int e = 15 - __builtin_amdgcn_frexp_expf(m);
    if (writer) {
        if (t == 0) sE[pt] = e;
        char *row = SWZ ? sA + pt * (4 * G::KDP) + ((2 * S::VEC * t) ^ tile_swizzle(pt)) : sA + pt * G::ARS + 2 * S::VEC * t;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            if constexpr (S::VEC == 4) {
                typedef float f2 __attribute__((ext_vector_type(2)));
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                h2 h[2], l[2];
#pragma unroll
                for (int p2 = 0; p2 < 2; ++p2) {
                    const f2 x = {__builtin_ldexpf(acc[2 * p2][jj], e), __builtin_ldexpf(acc[2 * p2 + 1][jj], e)};
                    h[p2] = __builtin_convertvector(x, h2);
                    const f2 back = __builtin_convertvector(h[p2], f2);
                    l[p2] = __builtin_convertvector(x - back, h2);
                }
                *reinterpret_cast<h4 *>(row + 2 * jj * S::DIP) = h4{h[0][0], h[0][1], h[1][0], h[1][1]};
                *reinterpret_cast<h4 *>(row + 2 * (G::KDP + jj * S::DIP)) = h4{l[0][0], l[0][1], l[1][0], l[1][1]};
            } else {
                const float x = __builtin_ldexpf(acc[0][jj], e);
                const _Float16 h = (_Float16)x;
                *reinterpret_cast<_Float16 *>(row + 2 * jj * S::DIP) = h;
                *reinterpret_cast<_Float16 *>(row + 2 * (G::KDP + jj * S::DIP)) = (_Float16)(x - (float)h);
            }
        }
    }
}

template <class S>
struct WsStage {
    int row[WsGeom<S>::EW];
    v4f dp[WsGeom<S>::EW];
};

struct TileRef {
    bool valid;
    int b, l0;
};

__device__ __forceinline__ TileRef tile_ref(const TileSchedule &sc, int k, int tiles_per_cloud, int T)
{
    TileRef r;
    const int tile = sc.first + k * sc.step;
    r.valid = (tile < sc.end) && (sc.first < sc.end);
    const int tc = r.valid ? tile : 0;
    r.b = tc / tiles_per_cloud;
    r.l0 = (tc - r.b * tiles_per_cloud) * T;
    return r;
}

// Walks a workgroup's tiles (sc.first, sc.first + sc.step, ... below sc.end) and keeps the cloud and the
// tile's index inside its cloud up to date by additions: a wave issues about one instruction per five
// clocks whatever its kind, so a division per tile (some twenty scalar instructions) is not free.
struct TileWalk {
    int tile, end, step, tpc;
    int step_b, step_t;          // the stride in whole clouds and the rest in tiles
    int b, tic;                  // cloud, tile inside the cloud
    __device__ __forceinline__ TileWalk(const TileSchedule &sc, int tiles_per_cloud)
        : tile(sc.first), end(sc.end), step(sc.step), tpc(tiles_per_cloud)
    {
        const int t0 = sc.first < sc.end ? sc.first : 0;
        b = t0 / tpc;
        tic = t0 - b * tpc;
        step_b = step / tpc;
        step_t = step - step_b * tpc;
    }
    __device__ __forceinline__ bool valid() const { return tile < end; }
    __device__ __forceinline__ bool has_next() const { return tile + step < end; }
    // one stride on if go (selects, no branches)
    __device__ __forceinline__ void next_if(bool go)
    {
        tile += go ? step : 0;
        tic += go ? step_t : 0;
        b += go ? step_b : 0;
        const bool wrap = tic >= tpc;
        tic -= wrap ? tpc : 0;
        b += wrap ? 1 : 0;
    }
    __device__ __forceinline__ void next() { next_if(true); }
    // stays on the last tile instead of walking past it
    __device__ __forceinline__ void next_clamped() { next_if(has_next()); }
};

// ---------------------------------------------------------------------------
// Producer side
// ---------------------------------------------------------------------------
template <class S, bool CSR>
struct Producer {
    using G = WsGeom<S>;
    // loop-carried registers
    int id_next;                 // entry `lane` of the tile to be issued next (neighbour / source id)
    int off_use, off_issue, off_pref;   // CSR: lane j <= PW holds in-edge offset j of the wave's points
    float pa[3], pb[3];          // raw positions (entry / centre) of the newest tile in flight
    float f[2][G::U][S::VEC];    // rows in flight, two tiles deep
    int lo[2], hi[2], cnt[2];    // group's entry range and staged count of those tiles
    unsigned onmask[2];          // which of the U rows in flight are real

    const float *rows, *pos;
    const int32_t *nbr, *off, *src;
    int N, K, lane, pw, grp, t, dsel;
    bool lane_on;
    WsStage<S> *st;              // this wave's two staging buffers
    float rs[S::VEC][4];         // depth scales of the packed parameters for this lane's aggregate elements

    __device__ __forceinline__ void init(const float *rows_, const float *pos_, const int32_t *nbr_,
                                         const int32_t *off_, const int32_t *src_, int N_, int K_,
                                         WsStage<S> *st_, int pw_)
    {
        rows = rows_; pos = pos_; nbr = nbr_; off = off_; src = src_; N = N_; K = K_; st = st_; pw = pw_;
        lane = threadIdx.x & 63;
        grp = lane / S::LPR; t = lane % S::LPR; dsel = lane & 3;
        lane_on = (S::VEC * t) < S::DI;
        id_next = 0; off_use = off_issue = off_pref = 0;
        pa[0] = pa[1] = pa[2] = pb[0] = pb[1] = pb[2] = 0.f;
#pragma unroll
        for (int v = 0; v < S::VEC; ++v)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) rs[v][jj] = 1.f;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            lo[p] = hi[p] = cnt[p] = 0; onmask[p] = 0u;
#pragma unroll
            for (int u = 0; u < G::U; ++u)
#pragma unroll
                for (int v = 0; v < S::VEC; ++v) f[p][u][v] = 0.f;
        }
    }

    // first point of this wave in tile r (cloud-local index)
    __device__ __forceinline__ int lw0(const TileRef &r) const { return r.l0 + pw * G::PW; }

    // CSR: request the in-edge offsets of this wave's points in tile r
    __device__ __forceinline__ int load_offsets(const TileRef &r) const
    {
        if (!r.valid) return 0;
        const int l = lw0(r);
        const int npw = max(0, min(G::PW, N - l));
        const int64_t g0 = (int64_t)r.b * N + min(l, N);
        return off[g0 + min(lane, npw)];
    }

    // request entry `lane` of tile r: fixed-K neighbour id, or CSR source id (needs its offsets)
    __device__ __forceinline__ int load_id(const TileRef &r, int offs) const
    {
        int v = 0;
        if (!r.valid) return 0;
        if constexpr (!CSR) {
            if (lane < G::PW * K) {
                const int k = lane / G::PW, l = lw0(r) + (lane % G::PW);
                if (l < N) v = nbr[((int64_t)r.b * K + k) * N + l];
            }
        } else {
            const int e0 = __builtin_amdgcn_readlane(offs, 0), e1 = __builtin_amdgcn_readlane(offs, G::PW);
            if (e0 + lane < e1) v = src[e0 + lane];
        }
        return v;
    }

    __device__ __forceinline__ const float *row_ptr(int rid, bool on, int rowbase) const
    {
        // lanes without a real row read the cloud's row 0 (always mapped); their value is discarded
        return rows + (int64_t)(on ? rid : rowbase) * S::DI + (lane_on ? S::VEC * t : 0);
    }

    template <int P>
    __device__ __forceinline__ void request_rows(int first, int stride, int end, int rowbase)
    {
        int rid[G::U];
        unsigned m = 0u;
#pragma unroll
        for (int u = 0; u < G::U; ++u) {
            const int i = first + u * stride;
            const bool on = i < end;
            rid[u] = st[P].row[on ? i : 0];
            if (on && lane_on) m |= (1u << u);
        }
        onmask[P] = m;
#pragma unroll
        for (int u = 0; u < G::U; ++u) {
            const float *p = row_ptr(rid[u], (m >> u) & 1u, rowbase);
            if constexpr (S::VEC == 4) {
                const v4f v = *reinterpret_cast<const v4f *>(p);
                f[P][u][0] = v.x; f[P][u][1] = v.y; f[P][u][2] = v.z; f[P][u][3] = v.w;
            } else {
                f[P][u][0] = *p;
            }
        }
    }

    template <int P>
    __device__ __forceinline__ void accumulate_rows(v4f (&acc)[S::VEC], int first, int stride, int end)
    {
#pragma unroll
        for (int u = 0; u < G::U; ++u) {
            const int i = first + u * stride;
            const bool on = (onmask[P] >> u) & 1u;
            float fv[S::VEC];
#pragma unroll
            for (int v = 0; v < S::VEC; ++v) fv[v] = on ? f[P][u][v] : 0.f;
            // the matrix op ignores EXEC: lanes without an entry feed 0 * 0
            const float dpc = (i < end) ? reinterpret_cast<const float *>(&st[P].dp[i < end ? i : 0])[dsel] : 0.f;
            fma_row<S>(acc, dpc, fv);
        }
    }

    // group's entry range inside the staged chunk [c0, c0+cnt) of tile r
    __device__ __forceinline__ void group_range(const TileRef &r, int offs, int c0, int cnt_, int &lo_, int &hi_,
                                                int &stride) const
    {
        const bool act = r.valid && (grp < G::PW) && (lw0(r) + grp < N);
        if constexpr (CSR) {
            int a = __builtin_amdgcn_readlane(offs, 0), b = __builtin_amdgcn_readlane(offs, 1);
#pragma unroll
            for (int j = 1; j < G::PW; ++j)
                if (grp == j) { a = __builtin_amdgcn_readlane(offs, j); b = __builtin_amdgcn_readlane(offs, j + 1); }
            lo_ = max(a, c0) - c0;
            hi_ = min(b, c0 + cnt_) - c0;
            stride = 1;
        } else {
            lo_ = grp;
            hi_ = grp + K * G::PW;
            stride = G::PW;
        }
        if (!act || hi_ < lo_) hi_ = lo_;
    }

    // raw positions for the staged entry `lane` of tile r (entry id in `id`), chunk starting at edge c0
    __device__ __forceinline__ void request_positions(const TileRef &r, int offs, int c0, int cnt_, int id,
                                                      float (&pa)[3], float (&pb)[3])
    {
        pa[0] = pa[1] = pa[2] = pb[0] = pb[1] = pb[2] = 0.f;
        if (lane < cnt_) {
            int pj;
            if constexpr (CSR) {
                pj = 0;
#pragma unroll
                for (int j = 1; j < G::PW; ++j) pj += (__builtin_amdgcn_readlane(offs, j) <= c0 + lane) ? 1 : 0;
            } else {
                pj = lane % G::PW;
            }
            const float *px = pos + (int64_t)r.b * 3 * N, *py = px + N, *pz = py + N;
            const int l = min(lw0(r) + pj, N - 1);
            pa[0] = px[id]; pa[1] = py[id]; pa[2] = pz[id];
            pb[0] = px[l]; pb[1] = py[l]; pb[2] = pz[l];
        }
    }

    template <int P>
    __device__ __forceinline__ void publish_dp(int cnt_, const float (&pa)[3], const float (&pb)[3])
    {
        if (lane < cnt_) {
            const float sg = CSR ? -1.f : 1.f;   // CSR: centre - source
            st[P].dp[lane] = v4f{sg * (pa[0] - pb[0]), sg * (pa[1] - pb[1]), sg * (pa[2] - pb[2]), 1.f};
        }
        wave_lds_sync();
    }

    // Start tile r in buffer P: stage its ids, request positions and the first U rows per point.
    // `id` holds entry `lane`, `offs` its offsets (CSR).
    template <int P>
    __device__ __forceinline__ void issue(const TileRef &r, int id, int offs)
    {
        const int rowbase = r.b * N;
        if constexpr (CSR) {
            const int e0 = __builtin_amdgcn_readlane(offs, 0), e1 = __builtin_amdgcn_readlane(offs, G::PW);
            cnt[P] = r.valid ? min(G::EW, e1 - e0) : 0;
        } else {
            cnt[P] = r.valid ? G::PW * K : 0;
        }
        if (lane < cnt[P]) st[P].row[lane] = rowbase + id;
        wave_lds_sync();
        const int c0 = CSR ? __builtin_amdgcn_readlane(offs, 0) : 0;
        request_positions(r, offs, c0, cnt[P], id, pa, pb);
        int stride;
        group_range(r, offs, c0, cnt[P], lo[P], hi[P], stride);
        request_rows<P>(lo[P], stride, hi[P], rowbase);
    }

    // Turn the positions of the tile in buffer P (requested by issue<P>) into staged differences.
    // Must run before the next issue<>() reuses the position registers.
    template <int P>
    __device__ __forceinline__ void stage_dp() { publish_dp<P>(cnt[P], pa, pb); }

    // Finish tile r (buffer P, issued one iteration ago): aggregate -> sA rows of this wave.
    // F16 == false: fp32 rows of AST floats.  F16 == true: split-half rows (WsGeom::ARS bytes)
    // scaled per point by 2^e, e stored in sE[point] (see pack_theta_f16_kernel for the split).
    template <int P, bool F16>
    __device__ __forceinline__ void finish(const TileRef &r, int offs, char *sA, int *sE)
    {
        v4f acc[S::VEC];
#pragma unroll
        for (int v = 0; v < S::VEC; ++v) acc[v] = v4f{0.f, 0.f, 0.f, 0.f};
        const int rowbase = r.b * N;
        const int stride = CSR ? 1 : G::PW;

        accumulate_rows<P>(acc, lo[P], stride, hi[P]);
        // a point with more than U staged entries: the rest synchronously
        for (int i0 = lo[P] + G::U * stride; i0 < hi[P]; i0 += G::U * stride) {
            request_rows<P>(i0, stride, hi[P], rowbase);
            accumulate_rows<P>(acc, i0, stride, hi[P]);
        }
        if constexpr (CSR) {
            // in-edges past the first staged chunk of this wave: whole chunks synchronously
            const int e0 = __builtin_amdgcn_readlane(offs, 0), e1 = __builtin_amdgcn_readlane(offs, G::PW);
            for (int c0 = e0 + G::EW; c0 < e1; c0 += G::EW) {
                wave_lds_sync();
                const int c = min(G::EW, e1 - c0);
                const int id = (lane < c) ? src[c0 + lane] : 0;
                if (lane < c) st[P].row[lane] = rowbase + id;
                wave_lds_sync();
                float qa[3], qb[3];
                request_positions(r, offs, c0, c, id, qa, qb);
                int l2, h2, s2;
                group_range(r, offs, c0, c, l2, h2, s2);
                request_rows<P>(l2, 1, h2, rowbase);
                publish_dp<P>(c, qa, qb);
                accumulate_rows<P>(acc, l2, 1, h2);
                for (int i0 = l2 + G::U; i0 < h2; i0 += G::U) {
                    request_rows<P>(i0, 1, h2, rowbase);
                    accumulate_rows<P>(acc, i0, 1, h2);
                }
            }
        }
        wave_lds_sync();   // this staging buffer is rewritten two issues from now

        const bool writer = grp < G::PW && (S::VEC * t) < S::DIP;
        if constexpr (!F16) {
            if (writer) {
                float *row = reinterpret_cast<float *>(sA) + (pw * G::PW + grp) * G::AST + S::VEC * t;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    if constexpr (S::VEC == 4) {
                        *reinterpret_cast<v4f *>(row + jj * S::DIP) = v4f{acc[0][jj], acc[1][jj], acc[2][jj], acc[3][jj]};
                    } else {
                        row[jj * S::DIP] = acc[0][jj];
                    }
                }
            }
        } else {
            store_split_rows<S>(acc, rs, sA, sE, pw * G::PW + grp, t, writer);
        }
    }
};

// One producer iteration for tile k living in buffer P.
template <int P, bool F16, class S, bool CSR, class Extra>
__device__ __forceinline__ bool producer_step(Producer<S, CSR> &Pr, const TileSchedule &sc, int k,
                                              int tiles_per_cloud, char *s_A, int *s_E, Extra &&extra)
{
    using G = WsGeom<S>;
    const TileRef r = tile_ref(sc, k, tiles_per_cloud, G::T);
    if (!r.valid) return false;
    const TileRef rn = tile_ref(sc, k + 1, tiles_per_cloud, G::T);
    const TileRef rnn = tile_ref(sc, k + 2, tiles_per_cloud, G::T);
    Pr.template stage_dp<P>();          // positions of tile k -> staged differences
    extra(k, r, 1);                     // park extra data of tile k in LDS
    // tile k+1 goes in flight behind tile k
    const int off_k = Pr.off_use;
    const int id_issue = Pr.id_next;
    if constexpr (CSR) {
        Pr.off_use = Pr.off_issue;
        Pr.off_issue = Pr.off_pref;
        Pr.off_pref = Pr.load_offsets(tile_ref(sc, k + 3, tiles_per_cloud, G::T));
    }
    extra(k + 1, rn, 0);                // request extra data of tile k+1
    Pr.template issue<P ^ 1>(rn, id_issue, Pr.off_use);
    Pr.id_next = Pr.load_id(rnn, Pr.off_issue);
    Pr.template finish<P, F16>(r, off_k, s_A + P * (G::T * G::ROWB), s_E + P * G::T);
    __syncthreads();                    // tile k is complete in buffer P
    return true;
}

// Runs the producer role for every tile of this workgroup; `extra(k, r, phase)` lets the
// grad_theta kernel move its grad_out tile (phase 0: request for tile k, phase 1: park in LDS).
template <bool F16, class S, bool CSR, class Extra>
__device__ __forceinline__ void producer_loop(Producer<S, CSR> &Pr, const TileSchedule &sc, int tiles_per_cloud,
                                              char *s_A, int *s_E, Extra &&extra)
{
    using G = WsGeom<S>;
    // prologue: ids of tile 0 and 1, offsets up to tile 2, tile 0 in flight
    const TileRef r0 = tile_ref(sc, 0, tiles_per_cloud, G::T), r1 = tile_ref(sc, 1, tiles_per_cloud, G::T);
    if constexpr (CSR) {
        Pr.off_use = Pr.load_offsets(r0);
        Pr.off_issue = Pr.load_offsets(r1);
        Pr.off_pref = Pr.load_offsets(tile_ref(sc, 2, tiles_per_cloud, G::T));
    }
    const int id0 = Pr.load_id(r0, Pr.off_use);
    Pr.id_next = Pr.load_id(r1, Pr.off_issue);
    extra(0, r0, 0);
    Pr.template issue<0>(r0, id0, Pr.off_use);
    for (int k = 0;; k += 2) {
        if (!producer_step<0, F16>(Pr, sc, k, tiles_per_cloud, s_A, s_E, extra)) break;
        if (!producer_step<1, F16>(Pr, sc, k + 1, tiles_per_cloud, s_A, s_E, extra)) break;
    }
}

// ---------------------------------------------------------------------------
// Lean producer for the fixed-K neighbour tensor (K a multiple of 8, every per-cloud byte
// offset below 2^32).  Nothing is staged in LDS: each lane of a row group loads its
// point's neighbour ids itself (a broadcast read), turns them into 32-bit row offsets,
// and lane i of every 4-lane block loads component i (x, y, z) of the neighbour's
// position directly, so the (dx,dy,dz,1) operand of the 4x4x1 matrix op is formed in
// registers.  Tail points are clamped to the cloud's last point (computed, never stored).
//
// The work of a wave is a stream of batches, one batch = 8 neighbours of the wave's points
// of one tile (K/8 batches per tile).  Eight rows per lane are in flight at all times: as
// soon as row u of batch m has been accumulated, its registers receive row u of batch
// m+1; the ids of batch m+2 are requested at the start of batch m.  Batches past the
// workgroup's last tile repeat that tile (loaded, never used).
// ---------------------------------------------------------------------------
// SUM == true: only the plain neighbour sum (component j = 3 of the aggregate) is formed; no positions
// are read (used by the location-gradient kernels).
// RS = floats between consecutive rows of the gathered tensor (S::DI unless the rows are a column block of a wider
// one); RS == 0: the stride is the run-time value set with set_row_stride() (one multiply per row instead of a shift).
// TAIL: K is not a multiple of 8; the last batch of a tile has slots past K, which are read from slot K-1 and
// weighted 0 (the weight travels as the fourth position component; in the plain-sum mode it is a wave-uniform
// 0 / 1 per slot), and its rows 4..7 are skipped when empty.
template <class S, int PM, bool SUM = false, int RS = S::DI, bool TAIL = false>
struct LeanProducer {
    using G = WsGeom<S, PM>;
    static constexpr int U = 8;
    static constexpr bool FULL = (S::LPR * S::VEC == S::DI);   // every lane of a group reads real channels
    static_assert(G::PW == 4, "entry layout below: 4 points x 8 neighbours per batch");
    // The aggregate runs on the vector ALU: the fp32 4x4x1 matrix op would need fewer issue slots, but
    // it holds both the vector ALU and the f16/bf16 matrix pipe of the SIMD while it executes, so the
    // consumers' matrix ops could never overlap the producers' work.
    static constexpr bool VALU_AGG = FLEX_LEAN_VALU_AGG;

    const float *rows, *pos;
    const int32_t *nbr;
    int N, K, KB, pw;
    unsigned rs_rt = 0;          // row stride in floats when RS == 0
    __device__ __forceinline__ void set_row_stride(int rs) { rs_rt = (unsigned)rs; }
    __device__ __forceinline__ unsigned row_stride() const { if constexpr (RS != 0) return RS; else return rs_rt; }
    int count, tiles_per_cloud;  // tiles of this workgroup
    TileSchedule sched;
    // compute layout: lane = (row group grp, lane t inside the row)
    int grp, t;
    bool lane_on;
    unsigned lane_off;           // byte offset of the lane's channels in a row
    int perm_id, perm_dp;        // ds_bpermute byte addresses of entry (k = 0, g) in the entry layout
    // entry layout: lane = (entry e = lane>>2 of 16, component c = lane&3); register half h holds the
    // entries 16h+e, entry i = (neighbour slot i>>2, point i&3)
    int e_g, e_k;                // point and slot (within half 0) of this lane's entry
    unsigned e_col;              // position component to read: x, y, z (lane 3 reads z, value unused)
    float e_mul, e_fix;          // dp component = (pn - pc)*e_mul + e_fix   (component lane 3: the constant 1)
    float *s_dp = nullptr;       // this wave's LDS array of 32 entries x (dx, dy, dz, w), entry = 4 * slot + point
    int dp_rd = 0;               // float offset of this lane's entry of slot 0 in it
    __device__ __forceinline__ void set_dp_stage(float *p) { s_dp = p; dp_rd = 4 * (grp % G::PW); }

    __device__ __forceinline__ void init(const float *rows_, const float *pos_, const int32_t *nbr_, int N_,
                                         int K_, int pw_, const TileSchedule &sc, int tiles_per_cloud_)
    {
        rows = rows_; pos = pos_; nbr = nbr_; N = N_; K = K_; KB = (K_ + U - 1) / U; pw = pw_;
        const int lane = threadIdx.x & 63;
        grp = lane / S::LPR; t = lane % S::LPR;
        lane_on = (S::VEC * t) < S::DI;
        lane_off = lane_on ? 4u * S::VEC * t : 0u;       // lanes past the row read its start, value unused
        const int g = grp % G::PW, dsel = lane & 3;
        perm_id = 4 * (4 * g);
        perm_dp = 4 * (4 * g + dsel);
        e_g = (lane >> 2) & 3;
        e_k = lane >> 4;
        const int c = lane & 3;
        e_col = c < 3 ? c : 2;
        e_mul = c < 3 ? 1.f : 0.f;
        e_fix = c < 3 ? 0.f : 1.f;
        sched = sc; tiles_per_cloud = tiles_per_cloud_;
        count = (sc.first < sc.end) ? (sc.end - sc.first + sc.step - 1) / sc.step : 0;
    }

    struct Batch {
        int b;          // cloud
        int lw0;        // first point of this wave in the tile
        int k0;         // first neighbour slot
    };
    // Walks the workgroup's batches in order (KB per tile) and stops on the last one.
    struct BatchWalk {
        TileWalk tw;
        int kb;
        __device__ __forceinline__ BatchWalk(const TileSchedule &sc, int tpc) : tw(sc, tpc), kb(0) {}
    };
    __device__ __forceinline__ Batch get(const BatchWalk &c) const
    {
        return Batch{c.tw.b, c.tw.tic * G::T + pw * G::PW, c.kb * U};
    }
    __device__ __forceinline__ void advance(BatchWalk &c) const
    {
        const bool in_tile = c.kb + 1 < KB;
        const bool go = !in_tile && c.tw.has_next();
        c.kb = in_tile ? c.kb + 1 : (go ? 0 : c.kb);
        c.tw.next_if(go);
    }

    // entry layout: neighbour ids of both halves
    __device__ __forceinline__ void load_ids(int (&id)[2], const Batch &x) const
    {
        const char *base = reinterpret_cast<const char *>(nbr + (int64_t)x.b * K * N);
        const unsigned l = (unsigned)min(x.lw0 + e_g, N - 1);
        if constexpr (TAIL) {
            const unsigned s0 = (unsigned)min(x.k0 + e_k, K - 1), s1 = (unsigned)min(x.k0 + e_k + 4, K - 1);
            id[0] = *reinterpret_cast<const int32_t *>(base + 4u * (s0 * (unsigned)N + l));
            id[1] = *reinterpret_cast<const int32_t *>(base + 4u * (s1 * (unsigned)N + l));
        } else {
            const unsigned o = 4u * ((unsigned)(x.k0 + e_k) * (unsigned)N + l);
            id[0] = *reinterpret_cast<const int32_t *>(base + o);
            id[1] = *reinterpret_cast<const int32_t *>(base + (o + 16u * (unsigned)N));
        }
    }
    // entry layout: position component of the neighbours (both halves) and of the centre
    __device__ __forceinline__ void load_pos(float (&pn)[2], float &pc, const int (&id)[2], const Batch &x) const
    {
        const char *pb = reinterpret_cast<const char *>(pos + (int64_t)x.b * 3 * N);
        const unsigned col = e_col * (unsigned)N;
        pn[0] = *reinterpret_cast<const float *>(pb + 4u * (col + (unsigned)id[0]));
        pn[1] = *reinterpret_cast<const float *>(pb + 4u * (col + (unsigned)id[1]));
        pc = *reinterpret_cast<const float *>(pb + 4u * (col + (unsigned)min(x.lw0 + e_g, N - 1)));
    }
    // entry layout -> compute layout: value of entry (slot u, this lane's point), component lane `base`
    __device__ __forceinline__ int spread(const int (&v)[2], int base, int u) const
    {
        return __builtin_amdgcn_ds_bpermute(base + 64 * (u & 3), v[u >> 2]);
    }

    __device__ __forceinline__ void load_row(float (&fr)[S::VEC], int id, const char *rb) const
    {
        const char *p = rb + ((unsigned)id * (4u * row_stride()) + lane_off);
        if constexpr (S::VEC == 4) {
            const v4f v = *reinterpret_cast<const v4f *>(p);
            fr[0] = v.x; fr[1] = v.y; fr[2] = v.z; fr[3] = v.w;
        } else {
            fr[0] = *reinterpret_cast<const float *>(p);
        }
    }

    // the row at byte offset `off` from the cloud's first row
    __device__ __forceinline__ void load_row_at(float (&fr)[S::VEC], unsigned off, const char *rb) const
    {
        const char *p = rb + (off + lane_off);
        if constexpr (S::VEC == 4) {
            const v4f v = *reinterpret_cast<const v4f *>(p);
            fr[0] = v.x; fr[1] = v.y; fr[2] = v.z; fr[3] = v.w;
        } else {
            fr[0] = *reinterpret_cast<const float *>(p);
        }
    }

    // cloud and first point (of this wave) of the workgroup's first tile
    __device__ __forceinline__ void first_coords(int &b, int &lw0) const
    {
        const TileWalk tw(sched, tiles_per_cloud);
        b = tw.b;
        lw0 = tw.tic * G::T + pw * G::PW;
    }

    // The producer role for every tile of this workgroup.  fin(acc, i, nb, nlw0) parks the finished
    // aggregate of the workgroup's tile i (this lane: channels VEC*t.. of point pw*PW+grp, all four j)
    // in LDS; (nb, nlw0) = cloud and this wave's first point of tile i+1 (of tile i again after the last
    // one).  The workgroup barrier that hands the tile to the consumers follows it.
    template <class Fin>
    __device__ __forceinline__ void run(Fin &&fin)
    {
        if (count == 0) return;
        float f[U][S::VEC];      // rows in flight (compute layout)
        int idn[2];              // entry layout: ids of the batch after the one whose rows are in flight
        float pn[2], pc;         // entry layout: positions for the batch whose rows are in flight
        BatchWalk walk(sched, tiles_per_cloud);
        Batch x1;                // batch m+1 at the top of iteration m
        {
            // prologue: rows and positions of batch 0 in flight, ids of batch 1 requested
            int id0[2];
            const Batch x0 = get(walk);
            advance(walk);
            x1 = get(walk);
            load_ids(id0, x0);
            load_ids(idn, x1);
            pn[0] = pn[1] = pc = 0.f;
            if constexpr (!SUM) load_pos(pn, pc, id0, x0);
            // The rows must be the youngest loads in flight when the loop is entered, as they are at the
            // end of every iteration: the wait at the loop top (for positions and ids) is one instruction
            // for both ways in, and a load issued after the rows would turn it into a wait for the rows.
            __builtin_amdgcn_sched_barrier(0);
            const char *rb = reinterpret_cast<const char *>(rows + (int64_t)x0.b * N * row_stride());
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (!TAIL || u < 4 || x0.k0 + 4 < K) load_row(f[u], spread(id0, perm_id, u), rb);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int total = count * KB;
        int kb = 0, tile_i = 0;
        int k0_cur = 0;          // first slot of the batch being accumulated
        v4f acc[S::VEC];
#pragma unroll
        for (int v = 0; v < S::VEC; ++v) acc[v] = v4f{0.f, 0.f, 0.f, 0.f};

        for (int m = 0; m < total; ++m) {
            // position differences of batch m, entry layout -> this lane's component per slot
            int dpe[2];
            dpe[0] = __float_as_int(fmaf(pn[0] - pc, e_mul, e_fix));
            dpe[1] = __float_as_int(fmaf(pn[1] - pc, e_mul, e_fix));
            if constexpr (TAIL) {                    // slots past K weigh nothing
                if (k0_cur + e_k >= K) dpe[0] = 0;
                if (k0_cur + e_k + 4 >= K) dpe[1] = 0;
            }
            const bool cur_upper = !TAIL || k0_cur + 4 < K, next_upper = !TAIL || x1.k0 + 4 < K;
            const int k0_acc = k0_cur;
            k0_cur = x1.k0;
            // ids of batch m+1 are here: their positions and (below) rows go in flight; ids of batch m+2 too
            constexpr bool DP_LDS = FLEX_DP_LDS && VALU_AGG && !SUM;
            // with a full last batch the fourth component of an entry (the constant 1) is not needed as a weight:
            // it carries the byte offset of the NEXT batch's row instead, which saves that batch's id permutes
            constexpr bool ID_LDS = DP_LDS && !TAIL;
            int idc[ID_LDS ? 1 : U];
            if constexpr (ID_LDS) {
                if ((threadIdx.x & 3) == 3) {
                    dpe[0] = (int)((unsigned)idn[0] * (4u * row_stride()));
                    dpe[1] = (int)((unsigned)idn[1] * (4u * row_stride()));
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) idc[u] = spread(idn, perm_id, u);
            }
            if constexpr (!SUM) load_pos(pn, pc, idn, x1);
            advance(walk);
            const Batch x2 = get(walk);
            load_ids(idn, x2);
            const char *rb = reinterpret_cast<const char *>(rows + (int64_t)x1.b * N * row_stride());
            const int nb = x1.b, nlw0 = x1.lw0;
            x1 = x2;
            float dpc[DP_LDS ? 1 : U];
            v4f dpv[DP_LDS ? 3 : 1];
            if constexpr (DP_LDS) {
                // entry (16 h + e), component c sits at float 4 * (16 h + e) + c = 64 h + lane
                const int lane = threadIdx.x & 63;
                s_dp[lane] = __int_as_float(dpe[0]);
                s_dp[64 + lane] = __int_as_float(dpe[1]);
                wave_lds_sync();
                dpv[0] = *reinterpret_cast<const v4f *>(s_dp + dp_rd);          // rows 0 and 1 now, row u + 2 while
                dpv[1] = *reinterpret_cast<const v4f *>(s_dp + 16 + dp_rd);     // row u is accumulated
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) dpc[u] = SUM ? 0.f : __int_as_float(spread(dpe, perm_dp, u));
            }
            const bool first = (kb == 0);            // first batch of a tile: its first row starts the sums

#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (DP_LDS)
                    if (u + 2 < U) dpv[(u + 2) % 3] = *reinterpret_cast<const v4f *>(s_dp + 16 * (u + 2) + dp_rd);
                if (!TAIL || u < 4 || cur_upper) {
                    float fv[S::VEC];
#pragma unroll
                    for (int v = 0; v < S::VEC; ++v) fv[v] = (FULL || lane_on) ? f[u][v] : 0.f;
                    if constexpr (SUM) {
                        const float one = (!TAIL || k0_acc + u < K) ? 1.f : 0.f;   // 0 for a slot past K
                        if (u == 0 && first) {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) acc[v] = v4f{0.f, 0.f, 0.f, TAIL ? one * fv[v] : fv[v]};
                        } else {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) {
                                if constexpr (TAIL) acc[v][3] = fmaf(one, fv[v], acc[v][3]);
                                else acc[v][3] += fv[v];
                            }
                        }
                    } else if constexpr (VALU_AGG) {
                        float dx, dy, dz, one;
                        if constexpr (DP_LDS) {
                            dx = dpv[u % 3][0]; dy = dpv[u % 3][1]; dz = dpv[u % 3][2]; one = dpv[u % 3][3];
                        } else {
                            // the four lanes of a block hold (dx, dy, dz, 1): broadcast inside the quad
                            dx = dpp_move<0x00>(dpc[u]); dy = dpp_move<0x55>(dpc[u]); dz = dpp_move<0xAA>(dpc[u]);
                            one = TAIL ? dpp_move<0xFF>(dpc[u]) : 1.f;             // 0 for a slot past K
                        }
                        if (u == 0 && first) {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v)
                                acc[v] = v4f{dx * fv[v], dy * fv[v], dz * fv[v], TAIL ? one * fv[v] : fv[v]};
                        } else {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) {
                                acc[v][0] = fmaf(dx, fv[v], acc[v][0]);
                                acc[v][1] = fmaf(dy, fv[v], acc[v][1]);
                                acc[v][2] = fmaf(dz, fv[v], acc[v][2]);
                                if constexpr (TAIL) acc[v][3] = fmaf(one, fv[v], acc[v][3]);
                                else acc[v][3] += fv[v];
                            }
                        }
                    } else {
                        if (u == 0 && first) {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) acc[v] = v4f{0.f, 0.f, 0.f, 0.f};
                        }
                        fma_row<S>(acc, dpc[u], fv);
                    }
                }
                // row u of batch m+1 takes the freed registers
                if constexpr (ID_LDS) {
                    load_row_at(f[u], __float_as_uint(dpv[u % 3][3]), rb);
                } else {
                    if (!TAIL || u < 4 || next_upper) load_row(f[u], idc[u], rb);
                }
                __builtin_amdgcn_sched_barrier(0);   // keep this shape: one row consumed, one requested
            }

            if (++kb == KB) {
                kb = 0;
                fin(acc, tile_i, nb, nlw0);
                ++tile_i;
                __syncthreads();        // tile complete in buffer tile_i & 1
            }
        }
    }
};

// ---------------------------------------------------------------------------
// Lean producer over in-edge lists (feature gradient): the rows are grad_out rows of the
// centres that list a point, dp = pos[point] - pos[centre].  Same machinery as LeanProducer
// (entry-layout loads, ds_bpermute spread, rolling 8-row window, vector-ALU aggregate); a
// batch is list slots 8*bi .. 8*bi+7 of each of the wave's 4 points, a tile takes
// max(1, ceil(longest list / 8)) batches, which differs from wave to wave and tile to tile.
// Slots past a list's end gather the point's own row with dp = (0,0,0,0), i.e. add nothing.
// The list bounds of the next tile are requested when a wave's id cursor enters a tile.
// ---------------------------------------------------------------------------
// ORD: the tiles walk the cloud in the order given by `order` (order[b*N + p] = the point at position p, a
// permutation of the cloud's points that puts points of equal list length next to each other inside windows of
// nearby points, see inedge_order_kernel): the four points of a wave then have lists of (nearly) the same length
// and so have the twelve waves of a tile, so hardly any slot of a batch is empty and no wave waits at the tile's
// barrier for one with a longer list.  The points' ids travel with the tile (s_P) to the consumers' stores.
template <class S, int PM, bool SUM = false, int RS = S::DI, bool ORD = false>
struct LeanCsrProducer {
    using G = WsGeom<S, PM>;
    static constexpr int U = 8;
    static constexpr bool FULL = (S::LPR * S::VEC == S::DI);
    static_assert(G::PW == 4, "entry layout: 4 points x 8 list slots per batch");

    const float *rows, *pos;
    const int32_t *off, *src;
    const int32_t *order = nullptr;
    int N, pw;
    unsigned rs_rt = 0;          // row stride in floats when RS == 0
    __device__ __forceinline__ void set_row_stride(int rs) { rs_rt = (unsigned)rs; }
    __device__ __forceinline__ unsigned row_stride() const { if constexpr (RS != 0) return RS; else return rs_rt; }
    int count, tiles_per_cloud;
    TileSchedule sched;
    int grp, t;
    bool lane_on;
    unsigned lane_off;
    int perm_id, perm_dp;
    int e_g, e_k;
    unsigned e_col;
    float e_mul, e_fix;
    float *s_dp = nullptr;       // this wave's LDS array of 32 entries x (dx, dy, dz, w), entry = 4 * slot + point
    int dp_rd = 0;               // float offset of this lane's entry of slot 0 in it
    __device__ __forceinline__ void set_dp_stage(float *p) { s_dp = p; dp_rd = 4 * (grp % G::PW); }

    __device__ __forceinline__ void init(const float *rows_, const float *pos_, const int32_t *off_,
                                         const int32_t *src_, int N_, int pw_, const TileSchedule &sc,
                                         int tiles_per_cloud_)
    {
        rows = rows_; pos = pos_; off = off_; src = src_; N = N_; pw = pw_;
        const int lane = threadIdx.x & 63;
        grp = lane / S::LPR; t = lane % S::LPR;
        lane_on = (S::VEC * t) < S::DI;
        lane_off = lane_on ? 4u * S::VEC * t : 0u;
        const int g = grp % G::PW, dsel = lane & 3;
        perm_id = 4 * (4 * g);
        perm_dp = 4 * (4 * g + dsel);
        e_g = (lane >> 2) & 3;
        e_k = lane >> 4;
        const int c = lane & 3;
        e_col = c < 3 ? c : 2;
        e_mul = c < 3 ? 1.f : 0.f;
        e_fix = c < 3 ? 0.f : 1.f;
        sched = sc; tiles_per_cloud = tiles_per_cloud_;
        count = (sc.first < sc.end) ? (sc.end - sc.first + sc.step - 1) / sc.step : 0;
    }

    // what the later pipeline stages need to know about a batch
    struct Desc {
        int b, lw0;      // cloud, first position of this wave in the tile
        int pid;         // entry layout: this lane's point (its position's point under ORD)
        bool first;      // first batch of its tile: its first row starts the sums
        bool last;       // last batch of its tile: the aggregate is complete after it
        bool real;       // false past the workgroup's last tile (loaded, never used)
        int nrows;       // slots 0 .. nrows-1 of this batch hold an entry of some point of the wave (the rest is skipped)
        int valid0, valid1;   // entry layout: does this lane's entry (half 0 / 1) exist
    };

    // walks the batches in order; entry-layout list bounds of the current and the next tile
    struct Cursor {
        int i, bi, nb;           // tile (index into the workgroup's tiles), batch in tile, batches of the tile
        int b, lw0;
        int dmax;                // longest list among the wave's four points
        int lo, deg;             // this lane's point: start and length of its list
        int pid;                 // this lane's point
        int lo_n, hi_n, pid_n;   // next tile: this lane's point and its list bounds (in flight)
        int pid_nn;              // ORD: this lane's point in the tile after the next (in flight)
        TileWalk tw;             // the tile those bounds belong to (the last tile again past the end)
        TileWalk tw2;            // ORD: the tile pid_nn belongs to
        __device__ __forceinline__ Cursor(const TileSchedule &sc, int tpc) : tw(sc, tpc), tw2(sc, tpc) {}
    };

    __device__ __forceinline__ void first_coords(int &b, int &lw0) const
    {
        const TileWalk tw(sched, tiles_per_cloud);
        b = tw.b;
        lw0 = tw.tic * G::T + pw * G::PW;
    }
    // this lane's point at its position in the walk's tile (positions past the cloud: the last one)
    __device__ __forceinline__ int point_at(const TileWalk &tw) const
    {
        const int p = min(tw.tic * G::T + pw * G::PW + e_g, N - 1);
        if constexpr (ORD) return order[(int64_t)tw.b * N + p];
        else return p;
    }
    // list bounds of this lane's point (c.pid_n) in the walk's tile
    __device__ __forceinline__ void request_bounds(Cursor &c) const
    {
        const int64_t gp = (int64_t)c.tw.b * N + c.pid_n;
        c.lo_n = off[gp];
        c.hi_n = off[gp + 1];
    }
    // the cursor takes the bounds requested for tile i (in lo_n / hi_n, the walk stands on that tile) and
    // requests tile i+1's (and, under ORD, the points of tile i+2)
    __device__ __forceinline__ void enter_tile(Cursor &c, int i) const
    {
        c.i = i; c.bi = 0;
        c.b = c.tw.b;
        c.lw0 = c.tw.tic * G::T + pw * G::PW;
        c.lo = c.lo_n;
        c.pid = c.pid_n;
        c.deg = (c.lw0 + e_g < N) ? c.hi_n - c.lo_n : 0;      // positions past the cloud have no list
        const int d = max(max(__builtin_amdgcn_readlane(c.deg, 0), __builtin_amdgcn_readlane(c.deg, 4)),
                          max(__builtin_amdgcn_readlane(c.deg, 8), __builtin_amdgcn_readlane(c.deg, 12)));
        c.nb = max(1, (d + U - 1) / U);
        c.dmax = d;
        c.tw.next_clamped();
        if constexpr (ORD) {
            c.pid_n = c.pid_nn;
            c.tw2.next_clamped();
            c.pid_nn = point_at(c.tw2);
        } else {
            c.pid_n = point_at(c.tw);
        }
        request_bounds(c);
    }
    // before the first enter_tile: the points of tile 0 (and 1 under ORD) and tile 0's bounds go in flight
    __device__ __forceinline__ void start(Cursor &c) const
    {
        c.pid_n = point_at(c.tw);
        if constexpr (ORD) {
            c.tw2.next_clamped();
            c.pid_nn = point_at(c.tw2);
        }
        request_bounds(c);
    }
    // entry-layout ids of the cursor's batch + its descriptor; then the cursor moves on
    __device__ __forceinline__ void fetch(Cursor &c, int (&id)[2], Desc &d) const
    {
        d.b = c.b; d.lw0 = c.lw0;
        d.pid = c.pid;
        d.real = c.i < count;
        d.first = c.bi == 0;
        d.last = c.bi == c.nb - 1;
        d.nrows = min(U, max(1, c.dmax - U * c.bi));
        const int s0 = U * c.bi + e_k, s1 = s0 + 4;
        d.valid0 = d.real && s0 < c.deg;
        d.valid1 = d.real && s1 < c.deg;
        const int self = c.pid;
        id[0] = self; id[1] = self;
        if (d.valid0) id[0] = src[c.lo + s0];
        if (d.valid1) id[1] = src[c.lo + s1];
        if (++c.bi == c.nb) enter_tile(c, c.i + 1);
    }
    __device__ __forceinline__ void load_pos(float (&pn)[2], float &pc, const int (&id)[2], const Desc &d) const
    {
        const char *pb = reinterpret_cast<const char *>(pos + (int64_t)d.b * 3 * N);
        const unsigned col = e_col * (unsigned)N;
        pn[0] = *reinterpret_cast<const float *>(pb + 4u * (col + (unsigned)id[0]));
        pn[1] = *reinterpret_cast<const float *>(pb + 4u * (col + (unsigned)id[1]));
        pc = *reinterpret_cast<const float *>(pb + 4u * (col + (unsigned)d.pid));
    }
    __device__ __forceinline__ int spread(const int (&v)[2], int base, int u) const
    {
        return __builtin_amdgcn_ds_bpermute(base + 64 * (u & 3), v[u >> 2]);
    }
    __device__ __forceinline__ void load_row(float (&fr)[S::VEC], int id, const char *rb) const
    {
        const char *p = rb + ((unsigned)id * (4u * row_stride()) + lane_off);
        if constexpr (S::VEC == 4) {
            const v4f v = *reinterpret_cast<const v4f *>(p);
            fr[0] = v.x; fr[1] = v.y; fr[2] = v.z; fr[3] = v.w;
        } else {
            fr[0] = *reinterpret_cast<const float *>(p);
        }
    }
    // position difference of this lane's entries (point - centre), zero for missing entries
    __device__ __forceinline__ void dp_entries(int (&dpe)[2], const float (&pn)[2], float pc, const Desc &d) const
    {
        if constexpr (SUM) {     // every component lane carries the entry's weight: 1 if it exists
            dpe[0] = d.valid0 ? __float_as_int(1.f) : 0;
            dpe[1] = d.valid1 ? __float_as_int(1.f) : 0;
        } else {
            dpe[0] = d.valid0 ? __float_as_int(fmaf(pc - pn[0], e_mul, e_fix)) : 0;
            dpe[1] = d.valid1 ? __float_as_int(fmaf(pc - pn[1], e_mul, e_fix)) : 0;
        }
    }

    template <class Fin>
    __device__ __forceinline__ void run(Fin &&fin)
    {
        if (count == 0) return;
        float f[U][S::VEC];      // rows of the batch being accumulated / next batch (compute layout)
        int idn[2];              // entry layout: ids of the batch after the one whose rows are in flight
        float pn[2], pc;         // entry layout: positions for the batch whose rows are in flight
        Desc d0, d1;             // batch whose rows are in flight; batch of idn
        Cursor c(sched, tiles_per_cloud);
        {
            start(c);
            enter_tile(c, 0);
            int id0[2];
            fetch(c, id0, d0);
            fetch(c, idn, d1);
            pn[0] = pn[1] = pc = 0.f;
            if constexpr (!SUM) load_pos(pn, pc, id0, d0);
            __builtin_amdgcn_sched_barrier(0);      // rows youngest, as at the end of every iteration
            const char *rb = reinterpret_cast<const char *>(rows + (int64_t)d0.b * N * row_stride());
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (u < d0.nrows) load_row(f[u], spread(id0, perm_id, u), rb);
            __builtin_amdgcn_sched_barrier(0);
        }
        int tile_i = 0;
        v4f acc[S::VEC];
#pragma unroll
        for (int v = 0; v < S::VEC; ++v) acc[v] = v4f{0.f, 0.f, 0.f, 0.f};

        while (d0.real) {
            int dpe[2];
            dp_entries(dpe, pn, pc, d0);
            const bool first = d0.first, last = d0.last;
            const int cur_rows = d0.nrows, next_rows = d1.nrows;      // slots to accumulate / to request
            const int pid_cur = d0.pid;
            // batch d1: positions and (below) rows go in flight; the cursor's batch: ids
            int idc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) idc[u] = spread(idn, perm_id, u);
            if constexpr (!SUM) load_pos(pn, pc, idn, d1);
            const char *rb = reinterpret_cast<const char *>(rows + (int64_t)d1.b * N * row_stride());
            d0 = d1;
            fetch(c, idn, d1);
            constexpr bool DP_LDS = FLEX_DP_LDS && !SUM;
            float dpc[DP_LDS ? 1 : U];
            v4f dpv[DP_LDS ? 3 : 1];
            if constexpr (DP_LDS) {
                // entry (16 h + e), component c sits at float 4 * (16 h + e) + c = 64 h + lane
                const int lane = threadIdx.x & 63;
                s_dp[lane] = __int_as_float(dpe[0]);
                s_dp[64 + lane] = __int_as_float(dpe[1]);
                wave_lds_sync();
                dpv[0] = *reinterpret_cast<const v4f *>(s_dp + dp_rd);          // rows 0 and 1 now, row u + 2 while
                dpv[1] = *reinterpret_cast<const v4f *>(s_dp + 16 + dp_rd);     // row u is accumulated
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) dpc[u] = __int_as_float(spread(dpe, perm_dp, u));
            }

#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (DP_LDS)
                    if (u + 2 < U) dpv[(u + 2) % 3] = *reinterpret_cast<const v4f *>(s_dp + 16 * (u + 2) + dp_rd);
                if (u < cur_rows) {
                    float fv[S::VEC];
#pragma unroll
                    for (int v = 0; v < S::VEC; ++v) fv[v] = (FULL || lane_on) ? f[u][v] : 0.f;
                    if constexpr (SUM) {
                        if (u == 0 && first) {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) acc[v] = v4f{0.f, 0.f, 0.f, dpc[u] * fv[v]};
                        } else {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) acc[v][3] = fmaf(dpc[u], fv[v], acc[v][3]);
                        }
                    } else {
                        float dx, dy, dz, one;           // one: 1 for a real entry, 0 for a missing one
                        if constexpr (DP_LDS) {
                            dx = dpv[u % 3][0]; dy = dpv[u % 3][1]; dz = dpv[u % 3][2]; one = dpv[u % 3][3];
                        } else {
                            dx = dpp_move<0x00>(dpc[u]); dy = dpp_move<0x55>(dpc[u]); dz = dpp_move<0xAA>(dpc[u]);
                            one = dpp_move<0xFF>(dpc[u]);
                        }
                        if (u == 0 && first) {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v)
                                acc[v] = v4f{dx * fv[v], dy * fv[v], dz * fv[v], one * fv[v]};
                        } else {
#pragma unroll
                            for (int v = 0; v < S::VEC; ++v) {
                                acc[v][0] = fmaf(dx, fv[v], acc[v][0]);
                                acc[v][1] = fmaf(dy, fv[v], acc[v][1]);
                                acc[v][2] = fmaf(dz, fv[v], acc[v][2]);
                                acc[v][3] = fmaf(one, fv[v], acc[v][3]);
                            }
                        }
                    }
                }
                if (u < next_rows) load_row(f[u], idc[u], rb);
                // keep the loop's shape: the scheduler would otherwise collect the eight loads at the end
                // of the iteration and wait for all of them at its start (no row would be in flight
                // while the previous ones are accumulated)
                __builtin_amdgcn_sched_barrier(0);
            }

            if (last) {
                fin(acc, tile_i, d0.b, d0.lw0, pid_cur);      // d0: first batch of the next tile by now
                ++tile_i;
                __syncthreads();        // tile complete in buffer tile_i & 1
            }
        }
    }
};

// One consumer wave of the split-half contraction: out tile = A tile * Theta for every tile of
// the workgroup.  cw = consumer index; G = the workgroup geometry; barriers pair with the producers'.
// OS = floats between consecutive output rows (point-major form; 0: the run-time value os_rt), ACC (or the
// run-time flag acc_rt): add to what out holds.
// ORD: tile slot pt holds the point s_P[pt] (the producers walk the cloud in a given order), not position l0 + pt.
// NBUF: tile buffers the producers cycle through (tile k sits in buffer k % NBUF).
// hook.begin(k, kb, b) runs right after tile k's barrier (kb = its buffer, b = its cloud), hook.end(k) after the
// wave's stores of tile k: extra per-tile work a kernel hangs on its consumer waves.
struct NoTileHook {
    __device__ __forceinline__ void begin(int, int, int) {}
    __device__ __forceinline__ void end(int) {}
};
template <class S, class G, bool OUT_BCN, int OS = S::DO, bool ACC = false, bool ORD = false, int NBUF = 2,
          class Hook = NoTileHook, bool SWZ = false>
__device__ __forceinline__ void consumer_f16(int cw, const void *__restrict__ thetaP, int theta_exp_off,
                                             float *__restrict__ out, int N, const TileSchedule &sc,
                                             int tiles_per_cloud, const char *s_A, const int *s_E, int os_rt = 0,
                                             bool acc_rt = false, const int *s_P = nullptr, Hook hook = Hook())
{
    const int os = OS != 0 ? OS : os_rt;
    const int lane = threadIdx.x & 63, q = lane >> 4, r16 = lane & 15;
    // item = (slice, block); consumer cw owns items cw, cw+NC, ... ; all share one slice
    static_assert(G::NS <= G::NC, "one parameter slice per consumer wave");
    const int slice = cw % G::NS;
    const bool active = cw < G::NITEMS;   // consumers beyond the item count only keep the barriers company

    auto store_item = [&](const TileRef &r, int it, v4f d, const int *sP) {
        const int idx = cw + it * G::NC;
        if (idx >= G::NITEMS) return;
        const int npts = min(G::T, N - r.l0);
        const int pt = (idx / G::NS) * 16 + r16;
        const int o = slice * 16 + 4 * q;
        if (pt < npts) {
            int l = r.l0 + pt;
            if constexpr (ORD) l = sP[pt];
            if constexpr (OUT_BCN) {
                float *dst = out + ((int64_t)r.b * S::DO + o) * N + l;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (o + i < S::DO) dst[(int64_t)i * N] = d[i];
            } else {
                float *dst = out + ((int64_t)r.b * N + l) * os + o;
                if constexpr (S::DO % 4 == 0) {
                    if (o < S::DO) {
                        if (ACC || acc_rt) d += *reinterpret_cast<const v4f *>(dst);
                        *reinterpret_cast<v4f *>(dst) = d;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (o + i < S::DO) dst[i] = d[i];
                }
            }
        }
    };

    constexpr int KS2 = G::KS2;
    // parameter fragments (matrix A operand: row = output channel r16, depth 32*s + 8*q + e)
    h8 thH[KS2], thL[KS2];
    {
        const _Float16 *tf = reinterpret_cast<const _Float16 *>(thetaP);
        constexpr int PER_PART = G::NS * KS2 * 64 * 8;
#pragma unroll
        for (int s = 0; s < KS2; ++s) {
            const int at = ((slice * KS2 + s) * 64 + lane) * 8;
            thH[s] = *reinterpret_cast<const h8 *>(tf + at);
            thL[s] = *reinterpret_cast<const h8 *>(tf + PER_PART + at);
        }
    }
    // column exponents of the packed parameters for this lane's four output channels
    int e_col[4];
    {
        const int *ec = reinterpret_cast<const int *>(reinterpret_cast<const char *>(thetaP) + theta_exp_off);
#pragma unroll
        for (int i = 0; i < 4; ++i) e_col[i] = ec[slice * 16 + 4 * q + i];
    }

    constexpr int RSTR = SWZ ? 4 * G::KDP : G::ARS;                    // bytes between tile rows
    constexpr int BUFB = SWZ ? G::T * 4 * G::KDP : G::T * G::ROWB;     // bytes per tile buffer
    int a_off[G::IPW];                // byte offset of this lane's 16-byte fragment (hi part, step 0)
    int a_odd[G::IPW];                // SWZ: the same for step 1 minus 64 (the XOR reaches into bit 6)
#pragma unroll
    for (int it = 0; it < G::IPW; ++it) {
        const int idx = active ? cw + it * G::NC : 0;
        const int row = (idx / G::NS) * 16 + r16;
        if constexpr (SWZ) {
            a_off[it] = row * RSTR + ((16 * q) ^ tile_swizzle(row));
            a_odd[it] = row * RSTR + ((16 * q + 64) ^ tile_swizzle(row)) - 64;
        } else {
            a_off[it] = row * RSTR + 16 * q;
            a_odd[it] = a_off[it];
        }
    }
    auto frag_off = [&](int it, int st) { return ((SWZ && (st & 1)) ? a_odd[it] : a_off[it]) + 64 * st; };

    TileWalk tw(sc, tiles_per_cloud);
    int kb = 0;                       // k % NBUF
    for (int k = 0; tw.valid(); ++k, tw.next(), kb = (kb + 1 == NBUF) ? 0 : kb + 1) {
        const TileRef r{true, tw.b, tw.tic * G::T};
        __syncthreads();              // tile k is complete in buffer kb
        hook.begin(k, kb, tw.b);
        if (!active) { hook.end(k); continue; }
        const char *sA = s_A + kb * BUFB;
        const int *sE = s_E + kb * G::T;

        // The wave's items advance together, one 32-deep step at a time: the fragments of all items for a step
        // are requested at once (one LDS round trip per step instead of one per item and step) and the next
        // step's are requested as soon as the matrix ops that read the registers have been issued.  Two
        // accumulation chains per item: hi*hi and the two cross terms lo*hi + hi*lo.
        v4f accA[G::IPW], accB[G::IPW];
        h8 bh[G::IPW], bl[G::IPW];
#pragma unroll
        for (int it = 0; it < G::IPW; ++it) {
            accA[it] = v4f{0.f, 0.f, 0.f, 0.f};
            accB[it] = v4f{0.f, 0.f, 0.f, 0.f};
            bh[it] = *reinterpret_cast<const h8 *>(sA + frag_off(it, 0));
            bl[it] = *reinterpret_cast<const h8 *>(sA + frag_off(it, 0) + 2 * G::KDP);
        }
#pragma unroll
        for (int s = 0; s < KS2; ++s) {
#pragma unroll
            for (int it = 0; it < G::IPW; ++it)
                accA[it] = __builtin_amdgcn_mfma_f32_16x16x32_f16(thH[s], bh[it], accA[it], 0, 0, 0);
#pragma unroll
            for (int it = 0; it < G::IPW; ++it)
                accB[it] = __builtin_amdgcn_mfma_f32_16x16x32_f16(thL[s], bh[it], accB[it], 0, 0, 0);
#pragma unroll
            for (int it = 0; it < G::IPW; ++it) {
                if (s + 1 < KS2) bh[it] = *reinterpret_cast<const h8 *>(sA + frag_off(it, s + 1));
                accB[it] = __builtin_amdgcn_mfma_f32_16x16x32_f16(thH[s], bl[it], accB[it], 0, 0, 0);
            }
#pragma unroll
            for (int it = 0; it < G::IPW; ++it)
                if (s + 1 < KS2) bl[it] = *reinterpret_cast<const h8 *>(sA + frag_off(it, s + 1) + 2 * G::KDP);
        }
#pragma unroll
        for (int it = 0; it < G::IPW; ++it) {
            const int idx = active ? cw + it * G::NC : 0;
            const int e_pt = sE[(idx / G::NS) * 16 + r16];
            v4f d = accA[it] + accB[it];
#pragma unroll
            for (int i = 0; i < 4; ++i) d[i] = __builtin_ldexpf(d[i], -(e_pt + e_col[i]));   // undo both scalings
            store_item(r, it, d, ORD ? s_P + kb * G::T : nullptr);
        }
        hook.end(k);
    }
}

// ---------------------------------------------------------------------------
// Forward with the lean producers: NP = PM * S::WAVES producer waves feed S::WAVES consumer
// waves (PM = 3: twelve gathering waves and four contracting ones per 1024-thread
// workgroup, 48-point tiles, one workgroup per CU).  The gather is latency-bound, so what
// counts is how many rows the CU has in flight; the f16 contraction is cheap enough for a
// quarter of the waves.
// ---------------------------------------------------------------------------
template <class S, bool OUT_BCN, int PM, int RS, int OS, bool ACC, bool TAIL>
__device__ __forceinline__ void gather_contract_lean_body(const float *__restrict__ rows, const float *__restrict__ pos,
                                                          const int32_t *__restrict__ nbr,
                                                          const void *__restrict__ thetaP, int theta_exp_off,
                                                          float *__restrict__ out, int N, int K, int tiles_per_cloud,
                                                          const TileSchedule sc, int rs_rt, int os_rt, bool acc_rt)
{
    using G = WsGeom<S, PM>;
    __shared__ __attribute__((aligned(16))) char s_A[2 * G::T * G::ROWB];
    __shared__ int s_E[2 * G::T];
    __shared__ __attribute__((aligned(16))) float s_D[G::NP][128];     // per producer wave: a batch's position differences

    const int w = threadIdx.x >> 6;

    if constexpr (G::KDP > S::KD) {
        // depth padding of both tile buffers: never written again, must read as zero
        constexpr int PADH = G::KDP - S::KD;
        for (int i = threadIdx.x; i < 2 * G::T * 2 * PADH; i += G::NT) {
            const int e = i % PADH, part = (i / PADH) & 1, row = i / (2 * PADH);
            *reinterpret_cast<_Float16 *>(s_A + (row / G::T) * (G::T * G::ROWB) + (row % G::T) * G::ARS +
                                          2 * (part * G::KDP + S::KD + e)) = (_Float16)0.f;
        }
        // ordered before the first consumer read by the barrier every thread passes for tile 0
    }

    if (w < G::NP) {
        LeanProducer<S, PM, false, RS, TAIL> P;
        P.init(rows, pos, nbr, N, K, w, sc, tiles_per_cloud);
        P.set_row_stride(rs_rt);
        P.set_dp_stage(s_D[w]);
        float rsc[S::VEC][4];
        load_row_scales<S>(rsc, thetaP, theta_exp_off, P.t);
        P.run([&](const v4f (&acc)[S::VEC], int i, int, int) {
            const int buf = i & 1;
            store_split_rows<S>(acc, rsc, s_A + buf * (G::T * G::ROWB), s_E + buf * G::T, P.pw * G::PW + P.grp, P.t,
                                P.grp < G::PW && (S::VEC * P.t) < S::DIP);
        });
        return;
    }
    consumer_f16<S, G, OUT_BCN, OS, ACC>(w - G::NP, thetaP, theta_exp_off, out, N, sc, tiles_per_cloud, s_A, s_E,
                                         os_rt, acc_rt);
}

template <class S, bool OUT_BCN, int PM, int RS = S::DI, int OS = S::DO, bool ACC = false, bool TAIL = false>
__global__ __launch_bounds__((WsGeom<S, PM>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void gather_contract_lean_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                                 const int32_t *__restrict__ nbr, const void *__restrict__ thetaP,
                                 int theta_exp_off, float *__restrict__ out, int N, int K,
                                 int tiles_per_cloud, int total_tiles)
{
    static_assert(RS != 0 && OS != 0, "run-time strides go through gather_contract_lean_passes_kernel");
    gather_contract_lean_body<S, OUT_BCN, PM, RS, OS, ACC, TAIL>(rows, pos, nbr, thetaP, theta_exp_off, out, N, K,
                                                                  tiles_per_cloud, TileSchedule(total_tiles), 0, 0,
                                                                  false);
}

// A layer wider than this shape, point-major, in one launch.  The n_out column blocks (S::DO channels) of the
// output are independent jobs, each shared by `chunks` workgroups: workgroup x serves block j = x / chunks as share
// x % chunks of the tiles.  It walks its tiles once per column block i (S::DI channels) of the gathered rows (rs
// floats apart): pass i contracts that block's aggregate with parameter block j * n_in + i of thetaP_all (blocks
// theta_block_bytes apart, each packed like a whole layer's) and writes (i == 0) or adds to (i > 0) its part of
// output block j (rows os floats apart).  A workgroup owns the same tiles in every pass and a consumer lane the
// same output elements, so the adds need no ordering beyond program order; the barrier between passes keeps a
// pass's first tile out of the LDS buffer the consumers may still be reading.
template <class S, int PM, bool TAIL>
__global__ __launch_bounds__((WsGeom<S, PM>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void gather_contract_lean_passes_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                                        const int32_t *__restrict__ nbr, const void *__restrict__ thetaP_all,
                                        int theta_block_bytes, int theta_exp_off, float *__restrict__ out, int N,
                                        int K, int tiles_per_cloud, int total_tiles, int rs, int os, int n_in,
                                        int chunks)
{
    const int j = blockIdx.x / chunks;
    const TileSchedule sc(total_tiles, (int)blockIdx.x - j * chunks, chunks);
    for (int i = 0; i < n_in; ++i) {
        const void *th = reinterpret_cast<const char *>(thetaP_all) + (size_t)(j * n_in + i) * theta_block_bytes;
        gather_contract_lean_body<S, false, PM, 0, 0, false, TAIL>(rows + S::DI * i, pos, nbr, th, theta_exp_off,
                                                                   out + S::DO * j, N, K, tiles_per_cloud, sc, rs, os,
                                                                   i > 0);
        __syncthreads();
    }
}

// Feature gradient with the lean in-edge producers (same consumers as the forward kernel).
template <class S, bool OUT_BCN, int PM, int RS, int OS, bool ACC>
__device__ __forceinline__ void grad_feat_lean_body(const float *__restrict__ rows, const float *__restrict__ pos,
                                                    const int32_t *__restrict__ off, const int32_t *__restrict__ src,
                                                    const int32_t *__restrict__ order,
                                                    const void *__restrict__ thetaP, int theta_exp_off,
                                                    float *__restrict__ out, int N, int tiles_per_cloud,
                                                    const TileSchedule sc, int rs_rt, int os_rt, bool acc_rt)
{
    using G = WsGeom<S, PM>;
    __shared__ __attribute__((aligned(16))) char s_A[2 * G::T * G::ROWB];
    __shared__ int s_E[2 * G::T];
    __shared__ int s_P[2 * G::T];       // the point in every tile slot (the tiles walk the cloud in `order`)
    __shared__ __attribute__((aligned(16))) float s_D[G::NP][128];     // per producer wave: a batch's position differences

    const int w = threadIdx.x >> 6;

    if constexpr (G::KDP > S::KD) {
        constexpr int PADH = G::KDP - S::KD;
        for (int i = threadIdx.x; i < 2 * G::T * 2 * PADH; i += G::NT) {
            const int e = i % PADH, part = (i / PADH) & 1, row = i / (2 * PADH);
            *reinterpret_cast<_Float16 *>(s_A + (row / G::T) * (G::T * G::ROWB) + (row % G::T) * G::ARS +
                                          2 * (part * G::KDP + S::KD + e)) = (_Float16)0.f;
        }
    }

    if (w < G::NP) {
        LeanCsrProducer<S, PM, false, RS, true> P;
        P.init(rows, pos, off, src, N, w, sc, tiles_per_cloud);
        P.order = order;
        P.set_row_stride(rs_rt);
        P.set_dp_stage(s_D[w]);
        float rsc[S::VEC][4];
        load_row_scales<S>(rsc, thetaP, theta_exp_off, P.t);
        const bool id_writer = (threadIdx.x & 0x33) == 0;        // entry lanes (slot 0, component 0) of the four points
        P.run([&](const v4f (&acc)[S::VEC], int i, int, int, int pid) {
            const int buf = i & 1;
            store_split_rows<S>(acc, rsc, s_A + buf * (G::T * G::ROWB), s_E + buf * G::T, P.pw * G::PW + P.grp, P.t,
                                P.grp < G::PW && (S::VEC * P.t) < S::DIP);
            if (id_writer) s_P[buf * G::T + P.pw * G::PW + P.e_g] = pid;
        });
        return;
    }
    consumer_f16<S, G, OUT_BCN, OS, ACC, true>(w - G::NP, thetaP, theta_exp_off, out, N, sc, tiles_per_cloud, s_A, s_E,
                                               os_rt, acc_rt, s_P);
}

template <class S, bool OUT_BCN, int PM, int RS = S::DI, int OS = S::DO, bool ACC = false>
__global__ __launch_bounds__((WsGeom<S, PM>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_feat_lean_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                           const int32_t *__restrict__ off, const int32_t *__restrict__ src,
                           const int32_t *__restrict__ order,
                           const void *__restrict__ thetaP, int theta_exp_off, float *__restrict__ out,
                           int N, int tiles_per_cloud, int total_tiles)
{
    static_assert(RS != 0 && OS != 0, "run-time strides go through grad_feat_lean_passes_kernel");
    grad_feat_lean_body<S, OUT_BCN, PM, RS, OS, ACC>(rows, pos, off, src, order, thetaP, theta_exp_off, out, N,
                                                     tiles_per_cloud, TileSchedule(total_tiles), 0, 0, false);
}

// The feature gradient of a wider layer in one launch (see gather_contract_lean_passes_kernel).
template <class S, int PM>
__global__ __launch_bounds__((WsGeom<S, PM>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_feat_lean_passes_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                                  const int32_t *__restrict__ off, const int32_t *__restrict__ src,
                                  const int32_t *__restrict__ order,
                                  const void *__restrict__ thetaP_all, int theta_block_bytes, int theta_exp_off,
                                  float *__restrict__ out, int N, int tiles_per_cloud, int total_tiles, int rs,
                                  int os, int n_in, int chunks)
{
    const int j = blockIdx.x / chunks;
    const TileSchedule sc(total_tiles, (int)blockIdx.x - j * chunks, chunks);
    for (int i = 0; i < n_in; ++i) {
        const void *th = reinterpret_cast<const char *>(thetaP_all) + (size_t)(j * n_in + i) * theta_block_bytes;
        grad_feat_lean_body<S, false, PM, 0, 0, false>(rows + S::DI * i, pos, off, src, order, th, theta_exp_off,
                                                       out + S::DO * j, N, tiles_per_cloud, sc, rs, os, i > 0);
        __syncthreads();
    }
}

template <class S, bool CSR, bool OUT_BCN, bool F16>
__global__ __launch_bounds__(WsGeom<S>::NT) __attribute__((amdgpu_waves_per_eu(4, 4)))
void gather_contract_ws_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                               const int32_t *__restrict__ nbr, const int32_t *__restrict__ off,
                               const int32_t *__restrict__ src, const void *__restrict__ thetaP,
                               int theta_exp_off, float *__restrict__ out, int N, int K,
                               int tiles_per_cloud, int total_tiles)
{
    using G = WsGeom<S>;
    constexpr int ROWB = F16 ? G::ARS : G::ROWB_F32;
    __shared__ __attribute__((aligned(16))) char s_A[2 * G::T * G::ROWB];
    __shared__ int s_E[2 * G::T];
    __shared__ WsStage<S> s_st[G::NP][2];

    const int w = threadIdx.x >> 6;
    const TileSchedule sc(total_tiles);

    if constexpr (F16 && G::KDP > S::KD) {
        // depth padding of both tile buffers: never written again, must read as zero
        constexpr int PADH = G::KDP - S::KD;
        for (int i = threadIdx.x; i < 2 * G::T * 2 * PADH; i += G::NT) {
            const int e = i % PADH, part = (i / PADH) & 1, row = i / (2 * PADH);
            *reinterpret_cast<_Float16 *>(s_A + (row / G::T) * (G::T * G::ROWB) + (row % G::T) * ROWB +
                                          2 * (part * G::KDP + S::KD + e)) = (_Float16)0.f;
        }
        // ordered before the first consumer read by the barrier every thread passes for tile 0
    }

    if (w < G::NP) {
        Producer<S, CSR> P;
        P.init(rows, pos, nbr, off, src, N, K, s_st[w], w);
        if constexpr (F16) load_row_scales<S>(P.rs, thetaP, theta_exp_off, P.t);
        producer_loop<F16>(P, sc, tiles_per_cloud, s_A, s_E, [](int, const TileRef &, int) {});
        return;
    }

    // ---- consumer ----
    const int cw = w - G::NP;
    const int lane = threadIdx.x & 63, q = lane >> 4, r16 = lane & 15;
    // item = (slice, block); consumer cw owns items cw, cw+NC, ... ; all share one slice
    static_assert(G::NS <= G::NC || G::IPW * G::NC == G::NITEMS, "slices");
    const int slice = cw % G::NS;
    static_assert(G::NS <= G::NC, "one parameter slice per consumer wave");
    // consumers beyond the item count only keep the barriers company
    const bool active = cw < G::NITEMS;

    auto store_item = [&](const TileRef &r, int it, v4f d) {
        const int idx = cw + it * G::NC;
        if (idx >= G::NITEMS) return;
        const int npts = min(G::T, N - r.l0);
        const int pt = (idx / G::NS) * 16 + r16;
        const int o = slice * 16 + 4 * q;
        if (pt < npts) {
            if constexpr (OUT_BCN) {
                float *dst = out + ((int64_t)r.b * S::DO + o) * N + (r.l0 + pt);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (o + i < S::DO) dst[(int64_t)i * N] = d[i];
            } else {
                float *dst = out + ((int64_t)r.b * N + r.l0 + pt) * S::DO + o;
                if constexpr (S::DO % 4 == 0) {
                    if (o < S::DO) *reinterpret_cast<v4f *>(dst) = d;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (o + i < S::DO) dst[i] = d[i];
                }
            }
        }
    };

    if constexpr (F16) {
        consumer_f16<S, G, OUT_BCN>(cw, thetaP, theta_exp_off, out, N, sc, tiles_per_cloud, s_A, s_E);
    } else {
        constexpr int KS = S::KD / 16;
        const float *th_src = reinterpret_cast<const float *>(thetaP);
        float th[S::KD / 4];
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                th[4 * s + i] = th_src[(int64_t)(16 * s + 4 * q + i) * S::DOP + slice * 16 + r16];

        int a_off[G::IPW];                // LDS float offset of this lane's 16-byte fragment, depth step 0
#pragma unroll
        for (int it = 0; it < G::IPW; ++it) {
            const int idx = active ? cw + it * G::NC : 0;
            a_off[it] = ((idx / G::NS) * 16 + r16) * G::AST + 4 * q;
        }

        TileWalk tw(sc, tiles_per_cloud);
        for (int k = 0; tw.valid(); ++k, tw.next()) {
            const TileRef r{true, tw.b, tw.tic * G::T};
            __syncthreads();              // tile k is complete in buffer k&1
            if (!active) continue;
            const float *sA = reinterpret_cast<const float *>(s_A + (k & 1) * (G::T * G::ROWB));

            // four independent accumulation chains per item (one per depth lane i), fragments one step ahead
            v4f acc[G::IPW][4];
            v4f bf[G::IPW];
#pragma unroll
            for (int it = 0; it < G::IPW; ++it) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[it][c] = v4f{0.f, 0.f, 0.f, 0.f};
                bf[it] = *reinterpret_cast<const v4f *>(&sA[a_off[it]]);
            }
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                v4f nx[G::IPW];
#pragma unroll
                for (int it = 0; it < G::IPW; ++it)
                    nx[it] = (s + 1 < KS) ? *reinterpret_cast<const v4f *>(&sA[a_off[it] + 16 * (s + 1)]) : bf[it];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int it = 0; it < G::IPW; ++it)
                        acc[it][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(th[4 * s + i], bf[it][i], acc[it][i], 0, 0, 0);
#pragma unroll
                for (int it = 0; it < G::IPW; ++it) bf[it] = nx[it];
            }
#pragma unroll
            for (int it = 0; it < G::IPW; ++it)
                store_item(r, it, (acc[it][0] + acc[it][1]) + (acc[it][2] + acc[it][3]));
        }
    }
}

// ---------------------------------------------------------------------------
// Per-workgroup partial of  gradTheta[kd][o] = sum_l A[l][kd] * g[l][o]
// ---------------------------------------------------------------------------
template <class S>
__global__ __launch_bounds__(WsGeom<S>::NT) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_theta_ws_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                          const int32_t *__restrict__ nbr, const float *__restrict__ g_rows,
                          float *__restrict__ partials, int N, int K, int tiles_per_cloud, int total_tiles)
{
    using G = WsGeom<S>;
    constexpr int GST = S::DOP + 16;
    __shared__ __attribute__((aligned(16))) char s_A[2 * G::T * G::ROWB];
    __shared__ __attribute__((aligned(16))) float s_G[2][G::T * GST];
    __shared__ WsStage<S> s_st[G::NP][2];

    const int w = threadIdx.x >> 6;
    const TileSchedule sc(total_tiles);

    if (w < G::NP) {
        // producers also move the grad_out tile: T*DOP floats over their 64*NP threads
        constexpr int PT = 64 * G::NP;
        constexpr int GPT = cdiv_c(G::T * S::DOP, PT);
        float gv[GPT];
        const int ptid = threadIdx.x;     // 0..64*NP-1
        Producer<S, false> P;
        P.init(rows, pos, nbr, nullptr, nullptr, N, K, s_st[w], w);
        producer_loop<false>(P, sc, tiles_per_cloud, s_A, nullptr, [&](int k, const TileRef &r, int phase) {
            if (phase == 0) {
#pragma unroll
                for (int i = 0; i < GPT; ++i) {
                    const int idx = ptid + i * PT;
                    const int j = idx / S::DOP, o = idx % S::DOP;
                    gv[i] = 0.f;
                    if (r.valid && idx < G::T * S::DOP && r.l0 + j < N && o < S::DO)
                        gv[i] = g_rows[((int64_t)r.b * N + r.l0 + j) * S::DO + o];
                }
            } else {
                float *sG = s_G[k & 1];
#pragma unroll
                for (int i = 0; i < GPT; ++i) {
                    const int idx = ptid + i * PT;
                    if (idx < G::T * S::DOP) sG[(idx / S::DOP) * GST + (idx % S::DOP)] = gv[i];
                }
            }
        });
        return;
    }

    // ---- consumer: owns MBW x NBW 16x16 blocks of the (KD x DOP) partial ----
    constexpr int MB = S::KD / 16, NB2 = S::DOP / 16;
    constexpr int WN = (NB2 < G::NC) ? NB2 : G::NC;
    static_assert(G::NC % WN == 0 && NB2 % WN == 0, "wave grid");
    constexpr int WM = G::NC / WN;
    constexpr int NBW = NB2 / WN;
    constexpr int MBW = cdiv_c(MB, WM);
    const int cw = w - G::NP;
    const int lane = threadIdx.x & 63, q = lane >> 4, r16 = lane & 15;
    const int wn = cw % WN, wm = cw / WN;

    v4f acc[MBW][NBW];
#pragma unroll
    for (int c = 0; c < MBW; ++c)
#pragma unroll
        for (int a = 0; a < NBW; ++a) acc[c][a] = v4f{0.f, 0.f, 0.f, 0.f};

    TileWalk tw(sc, tiles_per_cloud);
    for (int k = 0; tw.valid(); ++k, tw.next()) {
        __syncthreads();
        const float *sA = reinterpret_cast<const float *>(s_A + (k & 1) * (G::T * G::ROWB)), *sG = s_G[k & 1];
#pragma unroll
        for (int s = 0; s < G::T / 4; ++s) {
            const int row = 4 * s + q;
            float af[MBW], gf[NBW];
#pragma unroll
            for (int c = 0; c < MBW; ++c) {
                const int mb = wm + c * WM;
                af[c] = (mb < MB) ? sA[row * G::AST + mb * 16 + r16] : 0.f;
            }
#pragma unroll
            for (int a = 0; a < NBW; ++a) gf[a] = sG[row * GST + (wn + a * WN) * 16 + r16];
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
                dst[(int64_t)(mb * 16 + 4 * q + i) * S::DOP + nb * 16 + r16] = acc[c][a][i];
        }
    }
}

// ---------------------------------------------------------------------------
// Parameter gradients with the lean producers and the bf16 matrix cores.
//   partial[kd][o] = sum over the workgroup's points of A[pt][kd] * g[pt][o]
// contracts over POINTS, so no per-point scaling can be taken out of the sum; instead every
// fp32 value is carried as three bf16 pieces by truncation (x = h + m + l exactly: 3 x 8
// significand bits, bf16 has fp32's exponent range, nothing to scale) and six products
// h*h, h*m, m*h, h*l, l*h, m*m go through v_mfma_f32_16x16x32_bf16 (dropped terms ~2^-24).
// Both tiles sit point-major in LDS, [pt][h: W][m: W][l: W] bf16; the matrix operands want
// 8 consecutive points per lane, which ds_read_b64_tr_b16 delivers: in a group of 16 lanes,
// lane i supplies the address of 4 consecutive columns of one row and lane j receives
// column j%4 of the rows supplied by lanes j/4, j/4+4, j/4+8, j/4+12.
// Eight producer waves (32-point tiles) feed eight consumer waves that keep a 4x2 split of
// the (4*Din x Dout) partial in accumulators over the whole persistent loop.
// ---------------------------------------------------------------------------
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

// row stride of a three-piece bf16 tile of W columns: = 32 mod 128 bytes, so the four rows one
// 16-lane group reads (32 bytes each) and the rows four lane groups write fall on distinct banks
constexpr int bf3_stride(int W) { return 6 * W + ((32 - (6 * W) % 128) + 128) % 128; }

// x -> (h, m, l) by truncation, two values at a time, packed as bf16 pairs (first value low)
__device__ __forceinline__ void split_bf3(float x0, float x1, unsigned &h, unsigned &m, unsigned &l)
{
    const unsigned b0 = __float_as_uint(x0), b1 = __float_as_uint(x1);
    const float r0 = x0 - __uint_as_float(b0 & 0xffff0000u), r1 = x1 - __uint_as_float(b1 & 0xffff0000u);
    const unsigned c0 = __float_as_uint(r0), c1 = __float_as_uint(r1);
    const float s0 = r0 - __uint_as_float(c0 & 0xffff0000u), s1 = r1 - __uint_as_float(c1 & 0xffff0000u);
    h = (b0 >> 16) | (b1 & 0xffff0000u);
    m = (c0 >> 16) | (c1 & 0xffff0000u);
    l = (__float_as_uint(s0) >> 16) | (__float_as_uint(s1) & 0xffff0000u);
}

// operand fragment: 8 consecutive points (p0..p0+7 given by the lane's group) of column col0 + lane%16
__device__ __forceinline__ bf8 read_tr_frag(const char *tile, int stride, int p0, int byte_col0, int j16)
{
    typedef __attribute__((address_space(3))) v4s *lds_v4s;
    const char *a = tile + (p0 + (j16 >> 2)) * stride + byte_col0 + 8 * (j16 & 3);
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(__attribute__((address_space(3))) char *)a);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(__attribute__((address_space(3))) char *)(a + 4 * stride));
    const v8s v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf8, v);
}

// RS / GST = floats between consecutive rows of the gathered tensor / of the upstream gradient
template <class S, int RS, int GST, bool TAIL>
__device__ __forceinline__ void grad_theta_lean_body(const float *__restrict__ rows, const float *__restrict__ pos,
                                                     const int32_t *__restrict__ nbr,
                                                     const float *__restrict__ g_rows, float *__restrict__ partial,
                                                     int N, int K, int tiles_per_cloud, const TileSchedule sc,
                                                     int rs_rt, int gst_rt)
{
    // partial: where this workgroup's [KD x DOP] sums go; sc: the tiles it takes
    const int gst = GST != 0 ? GST : gst_rt;
    using G = WsGeom<S, 2, 2>;
    static_assert(G::T == 32, "one 32-point depth step of the matrix op per tile");
    constexpr int AS = bf3_stride(S::KD), GS = bf3_stride(S::DOP);
    __shared__ __attribute__((aligned(16))) char s_A[2][G::T * AS];
    __shared__ __attribute__((aligned(16))) char s_G[2][G::T * GS];
    __shared__ __attribute__((aligned(16))) float s_D[G::NP][128];     // per producer wave: a batch's position differences

    const int w = threadIdx.x >> 6;

    if (w < G::NP) {
        LeanProducer<S, 2, false, RS, TAIL> P;
        P.init(rows, pos, nbr, N, K, w, sc, tiles_per_cloud);
        P.set_row_stride(rs_rt);
        P.set_dp_stage(s_D[w]);
        // grad_out tile: T*DOP/4 four-float chunks over the producer threads, one tile ahead in registers
        constexpr int CPR = S::DOP / 4;                      // chunks per point
        constexpr int NCH = cdiv_c(G::T * CPR, 64 * G::NP);  // chunks per thread
        v4f gv[NCH];
        auto load_g = [&](int b, int lw0) {
            const int l0 = lw0 - P.pw * G::PW;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int ch = threadIdx.x + c * 64 * G::NP;
                const int pt = ch / CPR, o = 4 * (ch % CPR);
                gv[c] = v4f{0.f, 0.f, 0.f, 0.f};
                if (ch < G::T * CPR && l0 + pt < N) {        // points past the cloud contribute nothing
                    const float *src = g_rows + ((int64_t)b * N + l0 + pt) * gst + o;
                    if constexpr (S::DO % 4 == 0) {
                        if (o < S::DO) gv[c] = *reinterpret_cast<const v4f *>(src);
                    } else {
#pragma unroll
                        for (int i2 = 0; i2 < 4; ++i2)
                            if (o + i2 < S::DO) gv[c][i2] = src[i2];
                    }
                }
            }
        };
        if (P.count > 0) {
            int b0, lw00;
            P.first_coords(b0, lw00);
            load_g(b0, lw00);
        }
        P.run([&](const v4f (&acc)[S::VEC], int i, int nb, int nlw0) {
            const int buf = i & 1;
            // aggregate rows, three bf16 pieces
            if (P.grp < G::PW && (S::VEC * P.t) < S::DIP) {
                char *row = s_A[buf] + (P.pw * G::PW + P.grp) * AS + 2 * S::VEC * P.t;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    char *d = row + 2 * jj * S::DIP;
                    if constexpr (S::VEC == 4) {
                        unsigned h0, m0, l0, h1, m1, l1;
                        split_bf3(acc[0][jj], acc[1][jj], h0, m0, l0);
                        split_bf3(acc[2][jj], acc[3][jj], h1, m1, l1);
                        *reinterpret_cast<uint2 *>(d) = make_uint2(h0, h1);
                        *reinterpret_cast<uint2 *>(d + 2 * S::KD) = make_uint2(m0, m1);
                        *reinterpret_cast<uint2 *>(d + 4 * S::KD) = make_uint2(l0, l1);
                    } else {
                        unsigned h, m, l;
                        split_bf3(acc[0][jj], 0.f, h, m, l);
                        *reinterpret_cast<unsigned short *>(d) = (unsigned short)h;
                        *reinterpret_cast<unsigned short *>(d + 2 * S::KD) = (unsigned short)m;
                        *reinterpret_cast<unsigned short *>(d + 4 * S::KD) = (unsigned short)l;
                    }
                }
            }
            // grad_out rows of this tile (requested one tile ago), then the next tile's go in flight
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int ch = threadIdx.x + c * 64 * G::NP;
                if (ch < G::T * CPR) {
                    char *d = s_G[buf] + (ch / CPR) * GS + 2 * 4 * (ch % CPR);
                    unsigned h0, m0, l0, h1, m1, l1;
                    split_bf3(gv[c][0], gv[c][1], h0, m0, l0);
                    split_bf3(gv[c][2], gv[c][3], h1, m1, l1);
                    *reinterpret_cast<uint2 *>(d) = make_uint2(h0, h1);
                    *reinterpret_cast<uint2 *>(d + 2 * S::DOP) = make_uint2(m0, m1);
                    *reinterpret_cast<uint2 *>(d + 4 * S::DOP) = make_uint2(l0, l1);
                }
            }
            load_g(nb, nlw0);
        });
        return;
    }

    // ---- consumer: owns MBW x NBW 16x16 blocks of the (KD x DOP) partial ----
    constexpr int MB = S::KD / 16, NB2 = S::DOP / 16;
    constexpr int WN = (NB2 >= 2) ? 2 : 1;
    static_assert(G::NC % WN == 0 && NB2 % WN == 0, "wave grid");
    constexpr int WM = G::NC / WN;
    constexpr int NBW = NB2 / WN;
    constexpr int MBW = cdiv_c(MB, WM);
    const int cw = w - G::NP;
    const int lane = threadIdx.x & 63, q = lane >> 4, r16 = lane & 15;
    const int wn = cw % WN, wm = cw / WN;

    // The matrix op's internal accumulation rounds toward zero, a bias that would grow with the
    // thousands of tiles a workgroup sums; so its accumulators (acc) only ever hold FLUSH tiles and
    // are then added to the running totals (tot) on the vector ALU, which rounds to nearest.
    constexpr int FLUSH = 8;
    v4f acc[MBW][NBW], tot[MBW][NBW];
#pragma unroll
    for (int c = 0; c < MBW; ++c)
#pragma unroll
        for (int a = 0; a < NBW; ++a) { acc[c][a] = v4f{0.f, 0.f, 0.f, 0.f}; tot[c][a] = v4f{0.f, 0.f, 0.f, 0.f}; }

    TileWalk tw(sc, tiles_per_cloud);
    for (int k = 0; tw.valid(); ++k, tw.next()) {
        if (k % FLUSH == 0 && k > 0) {
#pragma unroll
            for (int c = 0; c < MBW; ++c)
#pragma unroll
                for (int a = 0; a < NBW; ++a) { tot[c][a] += acc[c][a]; acc[c][a] = v4f{0.f, 0.f, 0.f, 0.f}; }
        }
        __syncthreads();
        const char *sA = s_A[k & 1], *sG = s_G[k & 1];
        bf8 gH[NBW], gM[NBW], gL[NBW];
#pragma unroll
        for (int a = 0; a < NBW; ++a) {
            const int col = 2 * 16 * (wn + a * WN);
            gH[a] = read_tr_frag(sG, GS, 8 * q, col, r16);
            gM[a] = read_tr_frag(sG, GS, 8 * q, col + 2 * S::DOP, r16);
            gL[a] = read_tr_frag(sG, GS, 8 * q, col + 4 * S::DOP, r16);
        }
#pragma unroll
        for (int c = 0; c < MBW; ++c) {
            const int mb = wm + c * WM;
            if (mb >= MB) continue;
            const int col = 2 * 16 * mb;
            const bf8 aH = read_tr_frag(sA, AS, 8 * q, col, r16);
            const bf8 aM = read_tr_frag(sA, AS, 8 * q, col + 2 * S::KD, r16);
            const bf8 aL = read_tr_frag(sA, AS, 8 * q, col + 4 * S::KD, r16);
#define FLEX_BF_MFMA(X, Y)                                                                         \
    _Pragma("unroll") for (int a = 0; a < NBW; ++a)                                               \
        acc[c][a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(X, Y[a], acc[c][a], 0, 0, 0)
            FLEX_BF_MFMA(aL, gH);   // small terms first
            FLEX_BF_MFMA(aH, gL);
            FLEX_BF_MFMA(aM, gM);
            FLEX_BF_MFMA(aM, gH);
            FLEX_BF_MFMA(aH, gM);
            FLEX_BF_MFMA(aH, gH);
#undef FLEX_BF_MFMA
        }
    }

    float *dst = partial;
#pragma unroll
    for (int c = 0; c < MBW; ++c) {
        const int mb = wm + c * WM;
        if (mb >= MB) continue;
#pragma unroll
        for (int a = 0; a < NBW; ++a) {
            const int nb = wn + a * WN;
            const v4f sum = tot[c][a] + acc[c][a];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                dst[(int64_t)(mb * 16 + 4 * q + i) * S::DOP + nb * 16 + r16] = sum[i];
        }
    }
}

// RS / GST = floats between consecutive rows of the gathered tensor / of the upstream gradient
template <class S, int RS = S::DI, int GST = S::DO, bool TAIL = false>
__global__ __launch_bounds__((WsGeom<S, 2, 2>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_theta_lean_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                            const int32_t *__restrict__ nbr, const float *__restrict__ g_rows,
                            float *__restrict__ partials, int N, int K, int tiles_per_cloud, int total_tiles)
{
    static_assert(RS != 0 && GST != 0, "run-time strides go through grad_theta_lean_blocks_kernel");
    grad_theta_lean_body<S, RS, GST, TAIL>(rows, pos, nbr, g_rows, partials + (int64_t)blockIdx.x * S::KD * S::DOP, N, K,
                                           tiles_per_cloud, TileSchedule(total_tiles), 0, 0);
}

// Parameter gradients of a layer wider than this shape, point-major, in one launch: the (Din / S::DI) x
// (Dout / S::DO) blocks of the result are independent jobs, and each job's tiles are shared by `chunks`
// workgroups (output-stationary: a deep, low-resolution layer has many blocks and few points, so a workgroup
// walks all points for one block instead of all workgroups walking a few tiles each for every block).
// Workgroup x serves block p = x / chunks = (hi, ho) = (p / n_ho, p % n_ho) as share x % chunks: column block hi
// of the feature rows (rs floats apart) against column block ho of the upstream gradient rows (gst floats apart);
// its partial goes to partials[x].
template <class S, bool TAIL>
__global__ __launch_bounds__((WsGeom<S, 2, 2>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_theta_lean_blocks_kernel(const float *__restrict__ rows, const float *__restrict__ pos,
                                   const int32_t *__restrict__ nbr, const float *__restrict__ g_rows,
                                   float *__restrict__ partials, int N, int K, int tiles_per_cloud, int total_tiles,
                                   int rs, int gst, int chunks, int n_ho)
{
    const int p = blockIdx.x / chunks, q = blockIdx.x - p * chunks;
    const int hi = p / n_ho, ho = p - hi * n_ho;
    grad_theta_lean_body<S, 0, 0, TAIL>(rows + S::DI * hi, pos, nbr, g_rows + S::DO * ho,
                                        partials + (int64_t)blockIdx.x * S::KD * S::DOP, N, K, tiles_per_cloud,
                                        TileSchedule(total_tiles, q, chunks), rs, gst);
}

// ---------------------------------------------------------------------------
// Feature gradient and parameter gradients of a layer in ONE pass over the in-edge lists.
// With Bagg[m, (j,o)] = sum over the centres l that list m of dp_j(l,m) * grad_out[l,o] (dp_3 = 1), the aggregate
// the feature gradient contracts with Theta^T, the parameter gradients are
//   grad_theta[j,c,o] (j < 3), grad_bias[c,o] (j = 3)  =  sum_m Bagg[m, (j,o)] * feat[m, c]:
// regrouping the sum over edges (l, k) by the listed point m instead of by the centre l.  feat[m,:] is the
// point's OWN row (no gather), so the second gather pass of a separate parameter-gradient kernel disappears.
//
// Workgroup = 8 in-edge producer waves (32-point tiles, split-half f16 aggregate tile in LDS, exactly as for
// grad_feat_lean_kernel), 4 waves contracting the tile with Theta^T (consumer_f16) and 4 waves ("T waves", wave j
// owns component j) contracting it over the tile's 32 points with the points' own rows, all on
// v_mfma_f32_16x16x32_f16.  The tile rows are scaled per point (2^e_m), which a sum over points cannot factor out,
// so the own rows carry the inverse: own'[m,c] = feat[m,c] * 2^(cs_c + E - e_m), split into f16 halves like the
// tile.  E is the running minimum of e_m over the workgroup's tiles so far (this tile included: the factor
// 2^(E - e_m) is <= 1 and points with small aggregates just contribute small terms); when E drops, the T waves
// rescale their accumulators.  cs_c puts channel c's magnitude near 2^7: it comes from the largest |feat[.,c]| among
// 256 rows sampled across the workgroup's tiles at kernel start.  A row that exceeds the sampled maximum by more than
// 2^8 would overflow f16: the kernel then raises the flag (FUSED_OVERFLOW) and the stand-alone parameter-gradient
// kernel, launched behind it in its run-if-flagged form, recomputes the partials (results stay correct, that call is
// slower).  What the halves cannot RESOLVE -- a result far below the product of the largest aggregate and the largest
// feature -- is judged after the reduction, on the whole result, from the records the workgroups leave
// (fused_bwd_check_kernel).
// Pipeline: producers fill tile k+1 while the Theta^T waves contract tile k and fetch, scale and split the own rows
// of tile k (ids and exponents are known only once the tile is complete) and the T waves contract tile k-1; hence
// three tile buffers and one trailing barrier.  The matrix op accumulates with round-toward-zero, so the T waves add their
// accumulators to the workgroup's partial in global memory (each lane its own elements, so no ordering issue) every
// FLUSH tiles.  Partial layout = that of grad_theta_lean_kernel: [(j, c)][o], one per workgroup.
// S = (gathered width = the layer's Dout, output width = the layer's Din).
// ---------------------------------------------------------------------------
template <class S>
struct FusedGeom {
    using G = WsGeom<S, 2, 1>;
    static constexpr int NTW = 4;                       // T waves
    static constexpr int NT = 64 * (G::NP + G::NC + NTW);
    static constexpr int NBUF = 3;
    static constexpr int FS = 4 * S::DO + 32;           // own' row: [hi: DO halves][lo: DO halves], = 32 mod 128 bytes
    static constexpr int ARS = 4 * G::KDP;              // aggregate tile rows, swizzled form
    static constexpr int RB = S::DI / 16, CB = S::DO / 16;
    static constexpr int FLUSH = 64;
    static constexpr int LPO = S::DO / 4;               // lanes per own row
    static_assert(S::DI == 64 && S::DO == 64 && S::VEC == 4 && S::LPR == 16, "64 -> 64 layers");
    static_assert(G::NP == 8 && G::NC == 4 && G::T == 32 && NT == 1024 && G::KDP == S::KD, "wave roles");
};

typedef int v4i __attribute__((ext_vector_type(4)));
template <int CTRL>
__device__ __forceinline__ int dpp_movi(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}
// minimum over each half of the wave (lanes 0..31 / 32..63), in every lane
__device__ __forceinline__ int wave_min32(int v)
{
    v = min(v, dpp_movi<0xB1>(v));      // quad_perm [1,0,3,2]
    v = min(v, dpp_movi<0x4E>(v));      // quad_perm [2,3,0,1]
    v = min(v, dpp_movi<0x141>(v));     // row_half_mirror
    v = min(v, dpp_movi<0x140>(v));     // row_mirror
    return min(v, __shfl_xor(v, 16));
}

__device__ __forceinline__ h8 read_tr_frag_h(const char *tile, int stride, int p0, int byte_col0, int j16)
{
    return __builtin_bit_cast(h8, read_tr_frag(tile, stride, p0, byte_col0, j16));
}
// the same from a swizzled tile (store_split_rows<S, true>); byte_col0 a multiple of 32
__device__ __forceinline__ h8 read_tr_frag_swz(const char *tile, int stride, int p0, int byte_col0, int j16)
{
    typedef __attribute__((address_space(3))) v4s *lds_v4s;
    const int row = p0 + (j16 >> 2), in_row = byte_col0 + 8 * (j16 & 3);
    const char *a0 = tile + row * stride + (in_row ^ tile_swizzle(row));
    const char *a1 = tile + (row + 4) * stride + (in_row ^ tile_swizzle(row + 4));
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(__attribute__((address_space(3))) char *)a0);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(__attribute__((address_space(3))) char *)a1);
    const v8s v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(h8, v);
}

template <class S, bool OUT_BCN>
__global__ __launch_bounds__((FusedGeom<S>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void bwd_fused_lean_kernel(const float *__restrict__ g_rows, const float *__restrict__ own_rows,
                           const float *__restrict__ pos, const int32_t *__restrict__ off,
                           const int32_t *__restrict__ src, const int32_t *__restrict__ order,
                           const void *__restrict__ thetaP, int theta_exp_off, float *__restrict__ grad_feat,
                           float *__restrict__ partials, int *__restrict__ overflow, int N, int tiles_per_cloud,
                           int total_tiles)
{
    using F = FusedGeom<S>;
    using G = typename F::G;
    __shared__ __attribute__((aligned(128))) char s_A[F::NBUF * G::T * F::ARS];
    __shared__ __attribute__((aligned(16))) char s_F[2 * G::T * F::FS];
    __shared__ int s_E[F::NBUF * G::T];
    __shared__ int s_P[F::NBUF * G::T];
    __shared__ __attribute__((aligned(16))) float s_D[G::NP][128];
    __shared__ __attribute__((aligned(16))) int s_cs[S::DO];

    const TileSchedule sc(total_tiles);
    const int w = threadIdx.x >> 6;
    const bool any = sc.first < sc.end;
    const int count = any ? (sc.end - sc.first + sc.step - 1) / sc.step : 0;

    // ---- channel exponents of the own rows from a sample of the workgroup's region ----
    for (int i = threadIdx.x; i < S::DO; i += F::NT) s_cs[i] = 0;
    __syncthreads();
    if (any) {
        constexpr int RPP = F::NT / F::LPO;               // rows per pass
        const int qw = threadIdx.x / F::LPO, t = threadIdx.x % F::LPO;
        v4f m = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int si = 0; si < 4; ++si) {
            const int idx = 4 * qw + si;
            const int tile = sc.first + sc.step * (int)(((int64_t)idx * count) / (4 * RPP));
            const int b = tile / tiles_per_cloud;
            const int p = min((tile - b * tiles_per_cloud) * G::T + (idx % G::T), N - 1);
            const v4f x = *reinterpret_cast<const v4f *>(own_rows + ((int64_t)b * N + p) * S::DO + 4 * t);
#pragma unroll
            for (int v = 0; v < 4; ++v) m[v] = fmaxf(m[v], __builtin_fabsf(x[v]));
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) atomicMax(&s_cs[4 * t + v], __float_as_int(m[v]));   // non-negative floats order as ints
    }
    __syncthreads();
    int csv = 0;
    if (threadIdx.x < S::DO) {
        const float mx = __int_as_float(s_cs[threadIdx.x]);
        if (mx > 0.f && mx < __builtin_inff()) csv = 7 - __builtin_amdgcn_frexp_expf(mx);
    }
    __syncthreads();
    if (threadIdx.x < S::DO) s_cs[threadIdx.x] = csv;
    __syncthreads();

    if (w < G::NP) {
        LeanCsrProducer<S, 2, false, S::DI, true> P;
        P.init(g_rows, pos, off, src, N, w, sc, tiles_per_cloud);
        P.order = order;
        P.set_dp_stage(s_D[w]);
        float rsc[S::VEC][4];
        load_row_scales<S>(rsc, thetaP, theta_exp_off, P.t);
        const bool id_writer = (threadIdx.x & 0x33) == 0;
        int buf = 0;
        P.run([&](const v4f (&acc)[S::VEC], int, int, int, int pid) {
            store_split_rows<S, true>(acc, rsc, s_A + buf * (G::T * F::ARS), s_E + buf * G::T, P.pw * G::PW + P.grp,
                                      P.t, P.grp < G::PW && (S::VEC * P.t) < S::DIP);
            if (id_writer) s_P[buf * G::T + P.pw * G::PW + P.e_g] = pid;
            buf = (buf + 1 == F::NBUF) ? 0 : buf + 1;
        });
        if (any) __syncthreads();         // the T waves' last contraction
        return;
    }
    if (w < G::NP + G::NC) {
        // These waves also bring in the own rows: wave cw those of tile slots 8 cw .. 8 cw + 7, requested when the tile
        // is complete (ids and exponents known), scaled, split and parked for the T waves after the wave's own items.
        struct OwnRows {
            const float *own_rows; const int *s_P, *s_E, *s_cs; char *s_F; int *overflow;
            int N, cw, lane;
            int E_run = 1 << 20;
            v4f x0, x1;
            int sh0, sh1;
            __device__ __forceinline__ void begin(int, int kb, int b)
            {
                const int slot = 8 * cw + (lane >> 4), r16 = lane & 15;
                const int p0 = s_P[kb * G::T + slot], p1 = s_P[kb * G::T + slot + 4];
                const float *ob = own_rows + (int64_t)b * N * S::DO + 4 * r16;
                x0 = *reinterpret_cast<const v4f *>(ob + (int64_t)p0 * S::DO);
                x1 = *reinterpret_cast<const v4f *>(ob + (int64_t)p1 * S::DO);
                E_run = min(E_run, wave_min32(s_E[kb * G::T + (lane & 31)]));
                sh0 = E_run - s_E[kb * G::T + slot];
                sh1 = E_run - s_E[kb * G::T + slot + 4];
            }
            __device__ __forceinline__ void park(int fb, int slot, v4f x, int sh) const
            {
                const int r16 = lane & 15;
                const v4i ce = *reinterpret_cast<const v4i *>(s_cs + 4 * r16);
                typedef float f2 __attribute__((ext_vector_type(2)));
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                float m = 0.f;
                h2 h[2], l[2];
#pragma unroll
                for (int p2 = 0; p2 < 2; ++p2) {
                    const f2 y = {__builtin_ldexpf(x[2 * p2], ce[2 * p2] + sh),
                                  __builtin_ldexpf(x[2 * p2 + 1], ce[2 * p2 + 1] + sh)};
                    m = fmax3_abs(m, y[0], y[1]);
                    h[p2] = __builtin_convertvector(y, h2);
                    const f2 back = __builtin_convertvector(h[p2], f2);
                    l[p2] = __builtin_convertvector(y - back, h2);
                }
                if (!(m < 65504.f)) *overflow = FUSED_OVERFLOW;      // also a NaN: the stand-alone kernel takes over
                char *row = s_F + (fb * G::T + slot) * F::FS + 8 * r16;
                *reinterpret_cast<h4 *>(row) = h4{h[0][0], h[0][1], h[1][0], h[1][1]};
                *reinterpret_cast<h4 *>(row + 2 * S::DO) = h4{l[0][0], l[0][1], l[1][0], l[1][1]};
            }
            __device__ __forceinline__ void end(int k)
            {
                const int slot = 8 * cw + (lane >> 4);
                park(k & 1, slot, x0, sh0);
                park(k & 1, slot + 4, x1, sh1);
            }
        };
        OwnRows hook;
        hook.own_rows = own_rows; hook.s_P = s_P; hook.s_E = s_E; hook.s_cs = s_cs; hook.s_F = s_F;
        hook.overflow = overflow; hook.N = N; hook.cw = w - G::NP; hook.lane = threadIdx.x & 63;
        consumer_f16<S, G, OUT_BCN, S::DO, false, true, F::NBUF, OwnRows &, true>(w - G::NP, thetaP, theta_exp_off,
                                                                                  grad_feat, N, sc, tiles_per_cloud,
                                                                                  s_A, s_E, 0, false, s_P, hook);
        if (any) __syncthreads();
        return;
    }

    // ---- T waves ----
    const int j = w - G::NP - G::NC;
    const int lane = threadIdx.x & 63, q = lane >> 4, r16 = lane & 15;
    float *partial = partials + (int64_t)blockIdx.x * (4 * S::DO) * S::DI;
    const float *rscale = reinterpret_cast<const float *>(reinterpret_cast<const char *>(thetaP) + theta_exp_off +
                                                          rup_c(4 * S::DOP, 256));
    v4f acc[F::RB][F::CB];
#pragma unroll
    for (int rb = 0; rb < F::RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < F::CB; ++cb) acc[rb][cb] = v4f{0.f, 0.f, 0.f, 0.f};
    int E_run = 1 << 20, E_acc = 0, E_prev = 0, since = 0;
    bool fresh = true, have_prev = false;

    auto flush = [&]() __attribute__((always_inline)) {
        // addresses are formed here, every time: sixteen of them kept across the tile loop would cost registers
        float *pl = partial + (int64_t)(j * S::DO + r16) * S::DI + 4 * q;
        const float *rl = rscale + j * S::DIP + 4 * q;
        asm volatile("" : "+v"(pl), "+v"(rl));
        int re[F::RB][4];                         // rs = 2^k exactly: frexp exponent = k + 1
#pragma unroll
        for (int rb = 0; rb < F::RB; ++rb) {
            const v4f rs = *reinterpret_cast<const v4f *>(rl + 16 * rb);
#pragma unroll
            for (int i = 0; i < 4; ++i) re[rb][i] = __builtin_amdgcn_frexp_expf(rs[i]) - 1;
        }
#pragma unroll
        for (int cb = 0; cb < F::CB; ++cb) {
            const int ce = s_cs[16 * cb + r16];
            // a column block's four reads go out together: one round trip to memory, not four
            v4f old[F::RB];
#pragma unroll
            for (int rb = 0; rb < F::RB; ++rb)
                old[rb] = have_prev ? *reinterpret_cast<const v4f *>(pl + 16 * cb * S::DI + 16 * rb) : v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int rb = 0; rb < F::RB; ++rb) {
                v4f val;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    val[i] = __builtin_ldexpf(acc[rb][cb][i], -(E_acc + ce + re[rb][i])) + old[rb][i];
                *reinterpret_cast<v4f *>(pl + 16 * cb * S::DI + 16 * rb) = val;
                acc[rb][cb] = v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
        have_prev = true; fresh = true; since = 0;
    };
    // contraction of the tile in buffer kbp with the own' rows in buffer fb, which carry the scale 2^E_t
    auto mma_tile = [&](int kbp, int fb, int E_t) __attribute__((always_inline)) {
        if (fresh) { E_acc = E_t; fresh = false; }
        else if (E_t != E_acc) {
            const int d = E_t - E_acc;      // < 0: the running minimum only falls
#pragma unroll
            for (int rb = 0; rb < F::RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < F::CB; ++cb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[rb][cb][i] = __builtin_ldexpf(acc[rb][cb][i], d);
            E_acc = E_t;
        }
        const char *sA = s_A + kbp * (G::T * F::ARS), *sF = s_F + fb * (G::T * F::FS);
        // the fragment addresses (one per row block and half, because of the swizzle) are formed anew for every
        // tile: a few integer ops, where sixteen loop-invariant registers would not fit beside the accumulators
        int lanev = threadIdx.x;
        asm volatile("" : "+v"(lanev));
        const int r16v = lanev & 15, qv = (lanev >> 4) & 3;
        // the next row block's fragments are requested before the current one's matrix ops are issued, so the wave
        // waits for LDS once per tile and not once per row block
        h8 fh[F::CB], fl[F::CB];
#pragma unroll
        for (int cb = 0; cb < F::CB; ++cb) fh[cb] = read_tr_frag_h(sF, F::FS, 8 * qv, 2 * 16 * cb, r16v);
        h8 bl = read_tr_frag_swz(sA, F::ARS, 8 * qv, 2 * (S::DIP * j) + 2 * G::KDP, r16v);
        h8 bh = read_tr_frag_swz(sA, F::ARS, 8 * qv, 2 * (S::DIP * j), r16v);
#pragma unroll
        for (int cb = 0; cb < F::CB; ++cb) fl[cb] = read_tr_frag_h(sF, F::FS, 8 * qv, 2 * S::DO + 2 * 16 * cb, r16v);
#pragma unroll
        for (int rb = 0; rb < F::RB; ++rb) {
            h8 bl_n = bl, bh_n = bh;
            if (rb + 1 < F::RB) {
                const int col = 2 * (S::DIP * j + 16 * (rb + 1));
                bl_n = read_tr_frag_swz(sA, F::ARS, 8 * qv, col + 2 * G::KDP, r16v);
                bh_n = read_tr_frag_swz(sA, F::ARS, 8 * qv, col, r16v);
            }
            __builtin_amdgcn_sched_barrier(0);      // keep the requests ahead of the matrix ops
#pragma unroll
            for (int cb = 0; cb < F::CB; ++cb)     // small terms first
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bl, fh[cb], acc[rb][cb], 0, 0, 0);
#pragma unroll
            for (int cb = 0; cb < F::CB; ++cb)
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bh, fl[cb], acc[rb][cb], 0, 0, 0);
#pragma unroll
            for (int cb = 0; cb < F::CB; ++cb)
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bh, fh[cb], acc[rb][cb], 0, 0, 0);
            bl = bl_n; bh = bh_n;
            __builtin_amdgcn_sched_barrier(0);
        }
        if (++since == F::FLUSH) flush();
    };
    // iteration k: contraction of tile k-1, whose own' rows the other consumer waves parked during iteration k-1 with
    // the scale 2^E (E = the running minimum of the tile exponents through tile k-1, recomputed here the same way)
    int kb = 0, kb_prev = 0;
    for (int k = 0; any && k <= count; ++k) {
        __syncthreads();                  // tile k is complete in buffer kb (k = count: only the own' rows of the last tile)
        if (k > 0) mma_tile(kb_prev, (k - 1) & 1, E_prev);
        if (k < count) {
            E_run = min(E_run, wave_min32(s_E[kb * G::T + (lane & 31)]));
            E_prev = E_run;
            kb_prev = kb;
            kb = (kb + 1 == F::NBUF) ? 0 : kb + 1;
        }
    }
    if (!fresh || !have_prev) flush();    // a workgroup without tiles still writes its (zero) partial

    // ---- what the check after the reduction needs from this workgroup (fused_bwd_check_kernel) ----
    // its last running exponent, its number of terms and its channel exponents: words 0, 1 and 2 .. 2 + DO of its
    // record, FUSED_RECORD_INTS apart, behind the flag
    if (j == 0) {
        int *rec = overflow + FUSED_FLAG_INTS + (int64_t)blockIdx.x * FUSED_RECORD_INTS;
        if (lane == 0) { rec[0] = E_prev; rec[1] = G::T * count; }
        if (lane < S::DO) rec[2 + lane] = s_cs[lane];
    }
}

// The stand-alone parameter-gradient kernel as the fused kernel's fall-back: runs only if *overflow == want.
template <class S, bool TAIL>
__global__ __launch_bounds__((WsGeom<S, 2, 2>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_theta_lean_if_kernel(const int *__restrict__ overflow, int want, const float *__restrict__ rows,
                               const float *__restrict__ pos, const int32_t *__restrict__ nbr,
                               const float *__restrict__ g_rows, float *__restrict__ partials, int N, int K,
                               int tiles_per_cloud, int total_tiles)
{
    if (*overflow != want) return;
    grad_theta_lean_body<S, S::DI, S::DO, TAIL>(rows, pos, nbr, g_rows, partials + (int64_t)blockIdx.x * S::KD * S::DOP,
                                                N, K, tiles_per_cloud, TileSchedule(total_tiles), 0, 0);
}

// ---------------------------------------------------------------------------
// Gradient with respect to the point locations.  With Fsum[x] = sum_k feat[n_k(x)] and
// Gsum[x] = sum over the centres l that list x of grad_out[l] (plain neighbourhood sums),
//   grad_pos[d][x] = <feat[x], theta_d Gsum[x]>  -  <Fsum[x]^T theta_d, grad_out[x]>,   d = x, y, z,
// which follows from differentiating the forward sum edge by edge (the neighbour's location
// enters the weight with +, the centre's with -).  One kernel serves both terms:
//   sums  = lean producers in SUM mode (fixed-K tensor, or in-edge lists when CSR),
//   R_d   = sums x Theta_d on the f16 matrix cores, split-half as in the forward kernel
//           (consumer wave d holds all of Theta_d: every 16-column slice, hi and lo),
//   value = <R_d[x], dot_rows[x]>, reduced inside the wave, times sign, written or added to
//           grad_pos [B,3,N].
// The centre term runs first (rows = feat, Theta_d = theta[d], dot rows = grad_out, sign -, overwrite),
// the neighbour term second (rows = grad_out, Theta_d = theta[d]^T, dot rows = feat, sign +, accumulate).
// thetaF: fragments [d][part][slice][step][lane][8] of Theta_d scaled by 2^e, e at theta_exp_off.
// ---------------------------------------------------------------------------
template <class S>
struct PosGeom {
    static constexpr int KDP = rup_c(S::DIP, 32);      // contraction depth = gathered width, padded
    static constexpr int KS2 = KDP / 32;
    static constexpr int ARS = 4 * KDP + 16;           // row: [hi: KDP halves][lo: KDP halves][pad]
    static constexpr int NS = S::DOP / 16;
    static constexpr bool FITS = NS * KS2 * 8 <= 64 && S::VEC == 4;   // Theta_d fragments of one wave in 64 VGPRs
};

template <class S, bool CSR, int PM, bool TAIL = false>
__global__ __launch_bounds__((WsGeom<S, PM>::NT)) __attribute__((amdgpu_waves_per_eu(4, 4)))
void grad_pos_kernel(const float *__restrict__ rows, const int32_t *__restrict__ nbr,
                     const int32_t *__restrict__ off, const int32_t *__restrict__ src,
                     const void *__restrict__ thetaF, int theta_exp_off, const float *__restrict__ dot_rows,
                     float *__restrict__ grad_pos, float sign, int accumulate, int N, int K,
                     int tiles_per_cloud, int total_tiles)
{
    using G = WsGeom<S, PM>;
    using PG = PosGeom<S>;
    static_assert(PG::FITS, "shape too wide for the location-gradient kernel");
    static_assert(G::NC >= 3, "one consumer wave per coordinate");
    constexpr int YST = S::DOP + 4;   // floats per parked dot row (= 16 bytes mod 128: conflict-free 16-byte reads)
    __shared__ __attribute__((aligned(16))) char s_A[2 * G::T * PG::ARS];
    __shared__ __attribute__((aligned(16))) float s_Y[2 * G::T * YST];
    __shared__ int s_E[2 * G::T];

    const int w = threadIdx.x >> 6;
    const TileSchedule sc(total_tiles);

    if constexpr (PG::KDP > S::DIP) {
        constexpr int PADH = PG::KDP - S::DIP;   // depth padding: never written again, must read as zero
        for (int i = threadIdx.x; i < 2 * G::T * 2 * PADH; i += G::NT) {
            const int e = i % PADH, part = (i / PADH) & 1, row = i / (2 * PADH);
            *reinterpret_cast<_Float16 *>(s_A + row * PG::ARS + 2 * (part * PG::KDP + S::DIP + e)) = (_Float16)0.f;
        }
    }

    if (w < G::NP) {
        auto park = [&](const v4f (&acc)[S::VEC], int i, int pt, int t, bool writer) {
            // the neighbour sum of one point (this lane: channels 4t..4t+3) as a scaled split-half row
            float m = 0.f;
#pragma unroll
            for (int v = 0; v < S::VEC; ++v) m = __builtin_amdgcn_fmed3f(m, __builtin_fabsf(acc[v][3]), __builtin_inff());
            m = group_max<S::LPR>(m);
            const int e = 15 - __builtin_amdgcn_frexp_expf(m);
            if (writer) {
                const int buf = i & 1;
                if (t == 0) s_E[buf * G::T + pt] = e;
                char *row = s_A + (buf * G::T + pt) * PG::ARS + 2 * S::VEC * t;
                _Float16 h[4], l[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = __builtin_ldexpf(acc[v][3], e);
                    h[v] = (_Float16)x;
                    l[v] = (_Float16)(x - (float)h[v]);
                }
                *reinterpret_cast<h4 *>(row) = h4{h[0], h[1], h[2], h[3]};
                *reinterpret_cast<h4 *>(row + 2 * PG::KDP) = h4{l[0], l[1], l[2], l[3]};
            }
        };
        // the tile's dot rows travel with it: requested one tile ahead (registers), parked beside the sums
        constexpr int CPR = S::DOP / 4;                      // four-float chunks per point
        constexpr int NCH = cdiv_c(G::T * CPR, 64 * G::NP);  // chunks per producer thread
        v4f yv[NCH];
        auto load_y = [&](int b, int l0) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int ch = threadIdx.x + c * 64 * G::NP;
                const int pt = ch / CPR, o = 4 * (ch % CPR);
                yv[c] = v4f{0.f, 0.f, 0.f, 0.f};
                if (ch < G::T * CPR && l0 + pt < N) {
                    const float *srcp = dot_rows + ((int64_t)b * N + l0 + pt) * S::DO + o;
                    if constexpr (S::DO % 4 == 0) {
                        if (o < S::DO) yv[c] = *reinterpret_cast<const v4f *>(srcp);
                    } else {
#pragma unroll
                        for (int i2 = 0; i2 < 4; ++i2)
                            if (o + i2 < S::DO) yv[c][i2] = srcp[i2];
                    }
                }
            }
        };
        auto park_y = [&](int i) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int ch = threadIdx.x + c * 64 * G::NP;
                if (ch < G::T * CPR)
                    *reinterpret_cast<v4f *>(&s_Y[((i & 1) * G::T + ch / CPR) * YST + 4 * (ch % CPR)]) = yv[c];
            }
        };
        if constexpr (CSR) {
            LeanCsrProducer<S, PM, true> P;
            P.init(rows, nullptr, off, src, N, w, sc, tiles_per_cloud);
            if (P.count > 0) {
                int b0, lw00;
                P.first_coords(b0, lw00);
                load_y(b0, lw00 - P.pw * G::PW);
            }
            P.run([&](const v4f (&acc)[S::VEC], int i, int nb, int nlw0, int) {
                park(acc, i, P.pw * G::PW + P.grp, P.t, P.grp < G::PW && (S::VEC * P.t) < S::DIP);
                park_y(i);
                load_y(nb, nlw0 - P.pw * G::PW);
            });
        } else {
            LeanProducer<S, PM, true, S::DI, TAIL> P;
            P.init(rows, nullptr, nbr, N, K, w, sc, tiles_per_cloud);
            if (P.count > 0) {
                int b0, lw00;
                P.first_coords(b0, lw00);
                load_y(b0, lw00 - P.pw * G::PW);
            }
            P.run([&](const v4f (&acc)[S::VEC], int i, int nb, int nlw0) {
                park(acc, i, P.pw * G::PW + P.grp, P.t, P.grp < G::PW && (S::VEC * P.t) < S::DIP);
                park_y(i);
                load_y(nb, nlw0 - P.pw * G::PW);
            });
        }
        return;
    }

    // ---- consumer wave d = coordinate; waves beyond the third only keep the barriers company ----
    const int d = w - G::NP;
    const int lane = threadIdx.x & 63, q = lane >> 4, r16 = lane & 15;
    const bool active = d < 3;
    h8 thH[PG::NS][PG::KS2], thL[PG::NS][PG::KS2];
    {
        const _Float16 *tf = reinterpret_cast<const _Float16 *>(thetaF);
        constexpr int PER_PART = PG::NS * PG::KS2 * 64 * 8;
        const int dd = active ? d : 0;
#pragma unroll
        for (int sl = 0; sl < PG::NS; ++sl)
#pragma unroll
            for (int s = 0; s < PG::KS2; ++s) {
                const int at = ((sl * PG::KS2 + s) * 64 + lane) * 8;
                thH[sl][s] = *reinterpret_cast<const h8 *>(tf + (2 * dd) * PER_PART + at);
                thL[sl][s] = *reinterpret_cast<const h8 *>(tf + (2 * dd + 1) * PER_PART + at);
            }
    }
    const int e_theta = *reinterpret_cast<const int *>(reinterpret_cast<const char *>(thetaF) + theta_exp_off);

    TileWalk tw(sc, tiles_per_cloud);
    for (int k = 0; tw.valid(); ++k, tw.next()) {
        const TileRef r{true, tw.b, tw.tic * G::T};
        __syncthreads();              // tile k is complete in buffer k&1
        if (!active) continue;
        const char *sA = s_A + (k & 1) * (G::T * PG::ARS);
        const float *sY = s_Y + (k & 1) * (G::T * YST);
        const int *sE = s_E + (k & 1) * G::T;
#pragma unroll
        for (int blk = 0; blk < G::T / 16; ++blk) {
            const int pt = blk * 16 + r16;
            const int l = r.l0 + pt;
            const bool on = l < N;
            const char *arow = sA + pt * PG::ARS + 16 * q;
            h8 bh[PG::KS2], bl[PG::KS2];
#pragma unroll
            for (int s = 0; s < PG::KS2; ++s) {
                bh[s] = *reinterpret_cast<const h8 *>(arow + 64 * s);
                bl[s] = *reinterpret_cast<const h8 *>(arow + 2 * PG::KDP + 64 * s);
            }
            const float *yrow = sY + pt * YST;      // zero past the row's width and past the cloud
            float part = 0.f;
#pragma unroll
            for (int sl = 0; sl < PG::NS; ++sl) {
                v4f acc[3];
#pragma unroll
                for (int c = 0; c < 3; ++c) acc[c] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < PG::KS2; ++s) {
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(thH[sl][s], bh[s], acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(thL[sl][s], bh[s], acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(thH[sl][s], bl[s], acc[2], 0, 0, 0);
                }
                const v4f rd = acc[0] + (acc[1] + acc[2]);      // R_d[pt][16 sl + 4 q + i], still scaled
                const v4f y = *reinterpret_cast<const v4f *>(yrow + 16 * sl + 4 * q);
                part += (rd[0] * y[0] + rd[1] * y[1]) + (rd[2] * y[2] + rd[3] * y[3]);
            }
            part = __builtin_ldexpf(part, -(sE[pt] + e_theta));   // undo both scalings
            part += __shfl_xor(part, 16, 64);
            part += __shfl_xor(part, 32, 64);
            if (q == 0 && on) {
                float *dst = grad_pos + ((int64_t)r.b * 3 + d) * N + l;
                *dst = accumulate ? *dst + sign * part : sign * part;
            }
        }
    }
}

}  // namespace flex
