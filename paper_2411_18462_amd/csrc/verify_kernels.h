// Kernels of svip_verify (Algorithm 2 Verify, Algorithm 4 Correct, the bonus sample of Algorithm 1).
#pragma once
#include "kernel_args.h"
#include "sample_weights.h"

namespace svip {

// ---- verify: statistics ------------------------------------------------------------------------

// Statistics rows of sequence b are numbered jj = 0 .. kd + k: first the kd draft rows (only
// when the draft logsumexps are recomputed), then the k + 1 target rows.
__device__ __forceinline__ size_t stat_row(const VerifyArgs &a, int b, int jj)
{
    return (size_t)b * (a.kd + a.k + 1) + jj;
}

// grid (sequences * rows per sequence * slices).  Draft rows are needed for j < draft_len[b],
// target rows for j <= draft_len[b]; workgroups of other rows exit at once.
template <typename DT>
__global__ __launch_bounds__(WG) void k_verify_stats(VerifyArgs a)
{
    __shared__ CombineLds lds;
    const int y = blockIdx.x / a.geo.ns, s = blockIdx.x - y * a.geo.ns;
    const int rps = a.kd + a.k + 1;
    const int b = y / rps, jj = y - b * rps;
    const int g = clamp_len(a.draft_len[b], a.k);
    const DT *row;
    if (jj < a.kd) {
        if (jj >= g) return;
        row = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, jj);
    } else {
        const int j = jj - a.kd;
        if (j >= g + a.bonus) return;
        row = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, j);
    }
    const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    const Partial p = slice_lse<DT>(row, a.geo.V, tb, te, a.sc, lds);
    if (threadIdx.x == 0) a.ws.part[stat_row(a, b, jj) * a.geo.ns + s] = p;
}

// ---- verify: acceptance test and first rejection -------------------------------------------

// logsumexp * log2(e) of statistics row y from its slices' (ref, S) pairs (slice_lse): the sums are
// brought to the largest reference with single-precision exp2 of the (small, exactly formed)
// reference differences and added in fp64.  Slices are fetched eight at a time so that the loads
// of a chunk are in flight together.
__device__ __forceinline__ double row_L(const Partial *part, size_t y, int ns)
{
    float r = neg_inf();
    double S = 0.0;
    for (int s0 = 0; s0 < ns; s0 += 8) {
        float pm[8];
        double pS[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool in = s0 + u < ns;
            const Partial *p = part + y * ns + (in ? s0 + u : 0);
            pm[u] = p->m;
            pS[u] = p->S;
            if (!in || !(pS[u] > 0.0)) {
                pm[u] = neg_inf();
                pS[u] = 0.0;
            }
        }
        float rc = pm[0];
#pragma unroll
        for (int u = 1; u < 8; ++u) rc = vmax(rc, pm[u]);
        if (rc == neg_inf()) continue;
        if (rc > r) {
            if (r != neg_inf()) S *= (double)exp2_raw((float)((double)r - (double)rc));
            r = rc;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (pm[u] != neg_inf()) S += pS[u] * (double)exp2_raw((float)((double)pm[u] - (double)r));
    }
    return (double)r + log2(S);
}

// The acceptance test of sequence b by one wave: lane = position, 64 positions per pass.  Lanes
// j <= draft_len merge the statistics of target row j; lanes j < draft_len run the acceptance
// test; a ballot finds the first rejection.  Returns (uniform over the wave) what the residual
// kernels need; with `publish` lane 0 also writes n_accepted and the record, every tested lane its
// accept probability, and bad device data sets the flags.
template <typename DT>
__device__ __forceinline__ SeqRec accept_sequence(const VerifyArgs &a, int b, int lane, bool publish)
{
    const int graw = a.draft_len[b];
    const int g = clamp_len(graw, a.k);
    if (publish && graw != g && lane == 0) atomicOr(a.ws.flags, (unsigned)SVIP_FLAG_BAD_DRAFT_LEN);
    const DT *tgt = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, 0);
    const DT *drf = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, 0);
    constexpr double LOG2E = 1.4426950408889634;
    float *accept_prob = publish ? a.accept_prob : nullptr;
    int r = -1;                 // first rejection, once known
    double Lp_r = 0.0, Lq_r = 0.0;
    for (int j0 = 0; j0 <= g && (r < 0 || accept_prob); j0 += 64) {
        const int j = j0 + lane;
        bool reject = false;
        double Lp = 0.0, Lq = 0.0;
        if (j <= g) {
            // loads that do not depend on each other: token, uniform, draft logsumexp, slot statistics
            int x = 0;
            double u = 0.0, lse_q = 0.0;
            if (j < g) {
                x = a.tokens[(size_t)b * a.k + j];
                u = (double)a.u_accept[(size_t)b * a.k + j];
                if (a.draft_lse) lse_q = a.draft_lse[(size_t)b * a.k + j];
            }
            Lp = row_L(a.ws.part, stat_row(a, b, a.kd + j), a.geo.ns);
            if (j < g) {
                Lq = a.draft_lse ? lse_q * LOG2E : row_L(a.ws.part, stat_row(a, b, j), a.geo.ns);
                if (x < 0 || x >= a.geo.V) {
                    if (publish) atomicOr(a.ws.flags, (unsigned)SVIP_FLAG_BAD_TOKEN);
                    x = x < 0 ? 0 : a.geo.V - 1;
                }
                const double zp = (double)load_one<DT>(tgt + (long long)j * a.row_stride, x);
                const double zq = (double)load_one<DT>(drf + (long long)j * a.row_stride, x);
                const double p = exp2(zp * a.sc.c - Lp);
                const double q = exp2(zq * a.sc.c - Lq);
                reject = !(u * q < p);
                if (accept_prob) {
                    const double ratio = q > 0.0 ? p / q : (p > 0.0 ? 1.0 : 0.0);
                    accept_prob[(size_t)b * a.k + j] = (float)(ratio < 1.0 ? ratio : 1.0);
                }
            }
        }
        if (r < 0) {
            const unsigned long long rej = __ballot(reject);
            if (rej) {
                const int first = __ffsll((long long)rej) - 1;
                r = j0 + first;
                Lp_r = read_lane(Lp, first);
                Lq_r = read_lane(Lq, first);
            } else if (g - j0 < 64) {      // row g (the bonus row) was merged in this pass
                r = g;
                Lp_r = read_lane(Lp, g - j0);
            }
        }
    }
    SeqRec rec;
    rec.r = r;
    rec.resid = r < g ? 1 : 0;
    rec.Lp = Lp_r;
    rec.Lq = Lq_r;
    if (publish && lane == 0) {
        a.n_accepted[b] = r;
        a.ws.rec[b] = rec;
    }
    return rec;
}

// grid (sequences), one wave.
template <typename DT>
__global__ __launch_bounds__(64) void k_accept(VerifyArgs a)
{
    accept_sequence<DT>(a, blockIdx.x, threadIdx.x, true);
}

// ---- verify: residual / bonus sampling ------------------------------------------------------

// grid (sequences * slices): slice masses of the weights to sample from -- [0] residual
// max(0, p - q) at the rejected position, [1] target p of the row to sample.
// WITH_ACCEPT: no k_accept ran before; the first wave of every workgroup repeats the sequence's
// acceptance test (slice 0 publishes its outputs), which trades one kernel boundary for repeated work.
template <typename DT, bool WITH_ACCEPT>
__global__ __launch_bounds__(WG) void k_resid_mass(VerifyArgs a)
{
    __shared__ double lds[2 * NWAVE];
    __shared__ SeqRec shrec;
    const int b = blockIdx.x / a.geo_s.ns, s = blockIdx.x - b * a.geo_s.ns, tid = threadIdx.x;
    SeqRec rec;
    if constexpr (WITH_ACCEPT) {
        if (tid < 64) {
            const SeqRec mine = accept_sequence<DT>(a, b, tid, s == 0);
            if (tid == 0) shrec = mine;
        }
        __syncthreads();
        rec = shrec;
    } else {
        rec = a.ws.rec[b];
    }
    const DT *prow = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, rec.r);
    const DT *qrow = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, rec.r);
    const ExpRef ep = make_exp_ref(a.sc, rec.Lp), eq = make_exp_ref(a.sc, rec.Lq);
    const int tb = s * a.geo_s.tps, te = min(tb + a.geo_s.tps, a.geo_s.ntiles);
    float Wacc = 0.f, Pacc = 0.f;
    if (rec.resid) slice_mass<DT, true>(prow, qrow, a.geo_s.V, tb, te, ep, eq, Wacc, Pacc);
    else slice_mass<DT, false>(prow, qrow, a.geo_s.V, tb, te, ep, eq, Wacc, Pacc);
    const double Wd = wave_sum((double)Wacc), Pd = wave_sum((double)Pacc);
    const int wave = tid >> 6, lane = tid & 63;
    if (lane == 0) {
        lds[wave] = Wd;
        lds[NWAVE + wave] = Pd;
    }
    __syncthreads();
    if (tid == 0) {
        double W = 0.0, P = 0.0;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) {
            W += lds[w];
            P += lds[NWAVE + w];
        }
        double *out = a.ws.mass + ((size_t)b * MAX_SLICES + s) * 2;
        out[0] = W;
        out[1] = P;
    }
}

// grid (sequences): choice between residual and target weights, slice selection, inverse CDF.
template <typename DT>
__global__ __launch_bounds__(WG) void k_resid_finish(VerifyArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ FinishLds sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    // independent loads first
    const SeqRec rec = a.ws.rec[b];
    const float u = a.u_resample[b];
    double W = 0.0, P = 0.0;
    if (tid < a.geo_s.ns) {
        const double *in = a.ws.mass + ((size_t)b * MAX_SLICES + tid) * 2;
        W = in[0];
        P = in[1];
    }
    if (tid < 64) {
        const double inclW = wave_inclusive_sum(W), inclP = wave_inclusive_sum(P);
        const double totW = read_lane(inclW, 63), totP = read_lane(inclP, 63);
        const bool resid = rec.resid && totW > 0.0;   // no residual mass: draw from the target row
        const double M = resid ? W : P, incl = resid ? inclW : inclP, tot = resid ? totW : totP;
        double local;
        const int s = pick_slice(M, (double)u * tot, incl, &local);
        if (tid == 0) {
            sh.target = local;
            sh.slice = s;
            sh.use_resid = resid ? 1 : 0;
        }
    }
    __syncthreads();
    const DT *prow = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, rec.r);
    const DT *qrow = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, rec.r);
    const int tb = sh.slice * a.geo_s.tps, te = min(tb + a.geo_s.tps, a.geo_s.ntiles);
    float wtok;
    int tok;
    if (sh.use_resid) {
        ResidualWeights<DT> wf{prow, qrow, a.geo_s.V, make_exp_ref(a.sc, rec.Lp), make_exp_ref(a.sc, rec.Lq)};
        tok = locate_in_slice<N>(wf, tb, te, sh.target, sh.loc, &wtok);
    } else {
        SoftmaxWeights<DT> wf{prow, a.geo_s.V, make_exp_ref(a.sc, rec.Lp)};
        tok = locate_in_slice<N>(wf, tb, te, sh.target, sh.loc, &wtok);
    }
    if (tid == 0) a.next_token[b] = tok;
}

}  // namespace svip
