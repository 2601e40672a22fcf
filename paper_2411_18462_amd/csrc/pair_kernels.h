// Kernels of svip_pair_stats (Section 2.2, Appendix B).
#pragma once
#include "kernel_args.h"
#include "verify_kernels.h"

namespace svip {

// ---- per-position diagnostics (Section 2.2, Appendix B) ----------------------------------------

struct PairArgs {
    VerifyArgs v;        // statistics pass: rows j < draft_len of both models (bonus = 0)
    Geo geo2;            // slicing of the second pass
    float c;             // constant of the approximation bound
    double *L;           // [B k][2] logsumexp * log2(e) of target and draft row
    double *sums;        // [B k][ns2][3] slice sums
    float *out;          // [B k][SVIP_PAIR_NSTAT]
};

// One thread per position (b, j < draft_len): logsumexps of its two rows from the slice statistics.
__global__ __launch_bounds__(64) void k_pair_L(PairArgs a)
{
    const long long y = (long long)blockIdx.x * 64 + threadIdx.x;
    if (y >= (long long)a.v.B * a.v.k) return;
    const int b = (int)(y / a.v.k), j = (int)(y - (long long)b * a.v.k);
    const int graw = a.v.draft_len[b];
    const int g = clamp_len(graw, a.v.k);
    if (graw != g && j == 0) atomicOr(a.v.ws.flags, (unsigned)SVIP_FLAG_BAD_DRAFT_LEN);
    if (j >= g) return;
    a.L[2 * y] = row_L(a.v.ws.part, stat_row(a.v, b, a.v.kd + j), a.v.geo.ns);
    a.L[2 * y + 1] = a.v.draft_lse ? a.v.draft_lse[y] * 1.4426950408889634
                                   : row_L(a.v.ws.part, stat_row(a.v, b, j), a.v.geo.ns);
}

// One batch of NU vector pairs per thread: with p = exp2(xp), q = exp2(xq) the normalised
// probabilities, adds  sum min(p, q),  sum q (xq - xp)  and  sum q xq  (log2 units).
template <typename DT, int NU, bool CHECKED>
__device__ __forceinline__ void pair_batch(const DT *prow, const DT *qrow, int V, int t0, const ExpRef &ep,
                                           const ExpRef &eq, float &beta, float &kl, float &hq)
{
    constexpr int N = VecOf<DT>::N;
    const int tid = threadIdx.x;
    typename RawOf<DT>::type rp[NU], rq[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        const int vi = (t0 + u) * WG + tid;
        rp[u] = CHECKED ? load_raw_checked(prow, vi, V) : load_raw<DT>(prow, vi);
        rq[u] = CHECKED ? load_raw_checked(qrow, vi, V) : load_raw<DT>(qrow, vi);
    }
    float bb = 0.f, kb = 0.f, hb = 0.f;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        float zp[N], zq[N], mn[N], dk[N], dh[N];
        unpack<DT>(rp[u], zp);
        unpack<DT>(rq[u], zq);
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const float xp = ep.arg(zp[e]), xq = eq.arg(zq[e]);
            const float pe = exp2_raw(xp), qe = exp2_raw(xq);
            mn[e] = fminf(pe, qe);
            dk[e] = qe * (xq - xp);
            dh[e] = qe * xq;
        }
        bb += tree_sum<N>(mn);
        kb += tree_sum<N>(dk);
        hb += tree_sum<N>(dh);
    }
    beta += bb;
    kl += kb;
    hq += hb;
}

// grid (positions * slices): the three sums over slice s of the rows of position (b, j).
template <typename DT>
__global__ __launch_bounds__(WG) void k_pair_sums(PairArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ double lds[3 * NWAVE];
    const int ns = a.geo2.ns;
    const long long y = blockIdx.x / ns;
    const int s = (int)(blockIdx.x - y * ns), tid = threadIdx.x;
    const int b = (int)(y / a.v.k), j = (int)(y - (long long)b * a.v.k);
    if (j >= clamp_len(a.v.draft_len[b], a.v.k)) return;
    const DT *prow = static_cast<const DT *>(a.v.target) + row_offset(a.v, a.v.seq_t, b, j);
    const DT *qrow = static_cast<const DT *>(a.v.draft) + row_offset(a.v, a.v.seq_d, b, j);
    const ExpRef ep = make_exp_ref(a.v.sc, a.L[2 * y]), eq = make_exp_ref(a.v.sc, a.L[2 * y + 1]);
    const int V = a.geo2.V, tb = s * a.geo2.tps, te = min(tb + a.geo2.tps, a.geo2.ntiles);
    const int fe = min(te, V / (WG * N));
    float beta = 0.f, kl = 0.f, hq = 0.f;
    int t0 = tb;
    for (; t0 + 4 <= fe; t0 += 4) pair_batch<DT, 4, false>(prow, qrow, V, t0, ep, eq, beta, kl, hq);
    if (t0 + 2 <= fe) { pair_batch<DT, 2, false>(prow, qrow, V, t0, ep, eq, beta, kl, hq); t0 += 2; }
    if (t0 + 1 <= fe) { pair_batch<DT, 1, false>(prow, qrow, V, t0, ep, eq, beta, kl, hq); t0 += 1; }
    if (t0 < te) pair_batch<DT, 1, true>(prow, qrow, V, t0, ep, eq, beta, kl, hq);
    const double bd = wave_sum((double)beta), kd = wave_sum((double)kl), hd = wave_sum((double)hq);
    const int wave = tid >> 6, lane = tid & 63;
    if (lane == 0) {
        lds[wave] = bd;
        lds[NWAVE + wave] = kd;
        lds[2 * NWAVE + wave] = hd;
    }
    __syncthreads();
    if (tid == 0) {
        double o[3] = {0.0, 0.0, 0.0};
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) {
            o[0] += lds[w];
            o[1] += lds[NWAVE + w];
            o[2] += lds[2 * NWAVE + w];
        }
        double *dst = a.sums + ((size_t)y * ns + s) * 3;
        dst[0] = o[0];
        dst[1] = o[1];
        dst[2] = o[2];
    }
}

// One thread per position: slice sums added in slice order, then the bounds.
__global__ __launch_bounds__(64) void k_pair_finish(PairArgs a)
{
    const long long y = (long long)blockIdx.x * 64 + threadIdx.x;
    if (y >= (long long)a.v.B * a.v.k) return;
    const int b = (int)(y / a.v.k), j = (int)(y - (long long)b * a.v.k);
    float *o = a.out + y * SVIP_PAIR_NSTAT;
    if (j >= clamp_len(a.v.draft_len[b], a.v.k)) {
#pragma unroll
        for (int i = 0; i < SVIP_PAIR_NSTAT; ++i) o[i] = __int_as_float(0x7FC00000);
        return;
    }
    double beta = 0.0, A = 0.0, Bq = 0.0;
    for (int s = 0; s < a.geo2.ns; ++s) {
        const double *src = a.sums + ((size_t)y * a.geo2.ns + s) * 3;
        beta += src[0];
        A += src[1];
        Bq += src[2];
    }
    constexpr double LN2 = 0.6931471805599453;
    double kl = LN2 * A, hq = -LN2 * Bq;
    kl = kl > 0.0 ? kl : 0.0;             // both are non-negative; rounding can leave a tiny negative sum
    hq = hq > 0.0 ? hq : 0.0;
    beta = beta < 1.0 ? beta : 1.0;
    const double hqp = hq + kl;
    o[0] = (float)beta;
    o[1] = (float)kl;
    o[2] = (float)hqp;
    o[3] = (float)hq;
    o[4] = (float)(1.0 - sqrt(0.5 * kl));
    o[5] = (float)(1.0 - sqrt(1.0 - exp(-kl)));
    o[6] = (float)(1.0 - sqrt((double)a.c * hq));
    o[7] = hq > 0.0 ? (float)(hqp / hq) : __int_as_float(0x7FC00000);
}

}  // namespace svip
