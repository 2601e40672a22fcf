// Weights the inverse-CDF search and the mass kernels draw from: softmax of a row, residual max(0, p - q).
#pragma once
#include "kernel_args.h"

namespace svip {

// ---- weights for the inverse CDF ---------------------------------------------------------

template <typename DT>
struct SoftmaxWeights {        // w_i = exp2(z_i c - L)
    typedef typename RawOf<DT>::type Pack;
    const DT *row;
    int V;
    ExpRef ex;
    __device__ __forceinline__ Pack load(int vi) const { return load_raw<DT>(row, vi); }
    __device__ __forceinline__ Pack load_checked(int vi) const { return load_raw_checked(row, vi, V); }
    __device__ __forceinline__ void weights(const Pack &pk, float (&w)[VecOf<DT>::N]) const
    {
        float z[VecOf<DT>::N];
        unpack<DT>(pk, z);
#pragma unroll
        for (int e = 0; e < VecOf<DT>::N; ++e) w[e] = ex(z[e]);
    }
};

template <typename DT>
struct ResidualWeights {       // w_i = max(0, p_i - q_i), normalised p and q
    struct Pack { typename RawOf<DT>::type p, q; };
    const DT *prow, *qrow;
    int V;
    ExpRef exp_p, exp_q;
    __device__ __forceinline__ Pack load(int vi) const
    {
        Pack pk;
        pk.p = load_raw<DT>(prow, vi);
        pk.q = load_raw<DT>(qrow, vi);
        return pk;
    }
    __device__ __forceinline__ Pack load_checked(int vi) const
    {
        Pack pk;
        pk.p = load_raw_checked(prow, vi, V);
        pk.q = load_raw_checked(qrow, vi, V);
        return pk;
    }
    __device__ __forceinline__ void weights(const Pack &pk, float (&w)[VecOf<DT>::N]) const
    {
        float zp[VecOf<DT>::N], zq[VecOf<DT>::N];
        unpack<DT>(pk.p, zp);
        unpack<DT>(pk.q, zq);
#pragma unroll
        for (int e = 0; e < VecOf<DT>::N; ++e) w[e] = fmaxf(exp_p(zp[e]) - exp_q(zq[e]), 0.f);
    }
};

// One batch of NU vectors per thread of the rejected position's rows: the residual mass
// max(0, p - q) (if RESID) and the target mass p of every tile of the batch, into Wt / Pt at tile
// index u0 + u (tiles of a slice are numbered from 0; at most TILE_MASSES of them are kept apart,
// later ones are added to the last entry).
template <typename DT, int NU, bool RESID, bool CHECKED>
__device__ __forceinline__ void mass_batch(const DT *prow, const DT *qrow, int V, int t0, int u0, const ExpRef &ep,
                                           const ExpRef &eq, float (&Wt)[TILE_MASSES], float (&Pt)[TILE_MASSES])
{
    constexpr int N = VecOf<DT>::N;
    const int tid = threadIdx.x;
    typename RawOf<DT>::type rp[NU], rq[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        const int vi = (t0 + u) * WG + tid;
        rp[u] = CHECKED ? load_raw_checked(prow, vi, V) : load_raw<DT>(prow, vi);
        if (RESID) rq[u] = CHECKED ? load_raw_checked(qrow, vi, V) : load_raw<DT>(qrow, vi);
    }
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        float zp[N], pw[N];
        unpack<DT>(rp[u], zp);
#pragma unroll
        for (int e = 0; e < N; ++e) pw[e] = ep(zp[e]);
        const float Pb = tree_sum<N>(pw);
        float Wb = 0.f;
        if (RESID) {
            float zq[N], w[N];
            unpack<DT>(rq[u], zq);
#pragma unroll
            for (int e = 0; e < N; ++e) w[e] = fmaxf(pw[e] - eq(zq[e]), 0.f);
            Wb = tree_sum<N>(w);
        }
        const int slot = min(u0 + u, TILE_MASSES - 1);
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) {
            Pt[v] += (v == slot) ? Pb : 0.f;
            if (RESID) Wt[v] += (v == slot) ? Wb : 0.f;
        }
    }
}

// Per-thread residual and target masses of tiles [tb, te), tile by tile, in batches of up to
// LOCATE_UNROLL vectors (the same grouping of additions as the in-slice search).
template <typename DT, bool RESID>
__device__ __forceinline__ void slice_mass(const DT *prow, const DT *qrow, int V, int tb, int te,
                                           const ExpRef &ep, const ExpRef &eq, float (&Wt)[TILE_MASSES],
                                           float (&Pt)[TILE_MASSES])
{
    constexpr int N = VecOf<DT>::N;
    const int fe = min(te, V / (WG * N));
    int t0 = tb;
    for (; t0 + 4 <= fe; t0 += 4) mass_batch<DT, 4, RESID, false>(prow, qrow, V, t0, t0 - tb, ep, eq, Wt, Pt);
    if (t0 + 2 <= fe) { mass_batch<DT, 2, RESID, false>(prow, qrow, V, t0, t0 - tb, ep, eq, Wt, Pt); t0 += 2; }
    if (t0 + 1 <= fe) { mass_batch<DT, 1, RESID, false>(prow, qrow, V, t0, t0 - tb, ep, eq, Wt, Pt); t0 += 1; }
    if (t0 < te) mass_batch<DT, 1, RESID, true>(prow, qrow, V, t0, t0 - tb, ep, eq, Wt, Pt);
}

// Choice of the slice that contains `target` among per-lane slice masses M (lane order =
// slice order).  Returns (uniform) the slice and the target relative to the slice start.
__device__ __forceinline__ int pick_slice(double M, double target, double incl, double *local_target)
{
    const unsigned long long cross = __ballot(M > 0.0 && incl > target);
    const unsigned long long mass = __ballot(M > 0.0);
    int s;
    if (cross) s = __ffsll((long long)cross) - 1;
    else if (mass) s = 63 - __clzll((long long)mass);
    else s = 0;
    const double excl = read_lane(incl - M, s);
    *local_target = target - excl;
    return s;
}

// Choice of the tile inside a slice from the slice's tile masses G (uniform values): the first tile
// whose inclusive prefix exceeds `target` (relative to the slice start), else the last tile with mass.
// Returns the tile and the target relative to the tile start.
__device__ __forceinline__ int pick_tile(const double (&G)[TILE_MASSES], double target, double *local_target)
{
    int tile = -1, lastpos = 0;
    double before = 0.0, before_last = 0.0, run = 0.0;
#pragma unroll
    for (int v = 0; v < TILE_MASSES; ++v) {
        if (G[v] > 0.0) {
            if (tile < 0 && run + G[v] > target) {
                tile = v;
                before = run;
            }
            lastpos = v;
            before_last = run;
        }
        run += G[v];
    }
    if (tile < 0) {
        tile = lastpos;
        before = before_last;
    }
    *local_target = target - before;
    return tile;
}

}  // namespace svip
