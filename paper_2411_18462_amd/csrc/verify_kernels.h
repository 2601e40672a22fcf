// Kernels of svip_verify (Algorithm 2 Verify, Algorithm 4 Correct, the bonus sample of Algorithm 1).
#pragma once
#include "exchange.h"
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
// target rows for j <= draft_len[b]; workgroups of other rows exit at once.  (Handing the acceptance
// test to the workgroup that finishes a sequence last was measured and dropped here: the wait for the
// acknowledged stores and the ticket adds about 1 us to every workgroup of a kernel whose workgroups
// live about 5 us, and the pass went from 47 us to 63 us; the separate one-wave kernel costs 5 us.)
template <typename DT>
__global__ __launch_bounds__(WG, 8) void k_verify_stats(VerifyArgs a)
{
    __shared__ CombineLds lds;
    const int rps = a.kd + a.k + 1;
    // one item = one slice of one statistics row; a workgroup takes items blockIdx, blockIdx + grid, ...
    // (the grid covers all items unless the launch asks for fewer, longer-lived workgroups)
    for (long long item = blockIdx.x; item < a.stat_items; item += gridDim.x) {
        const int y = (int)(item / a.geo.ns), s = (int)(item - (long long)y * a.geo.ns);
        const int b = y / rps, jj = y - b * rps;
        if (a.skip && a.skip[b]) continue;
        const int g = clamp_len(a.draft_len[b], a.k);
        const DT *row;
        if (jj < a.kd) {
            if (jj >= g) continue;
            row = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, jj);
        } else {
            const int j = jj - a.kd;
            if (j >= g + a.bonus) continue;
            row = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, j);
        }
        const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
        // the LDS block can be reused at once: every wave has read the maxima before the second barrier of
        // slice_lse, and thread 0 has read the sums before its wave reaches the next item's first barrier
        const Partial p = slice_lse<DT>(row, a.geo.V, tb, te, a.sc, lds);
        if (threadIdx.x == 0) a.ws.part[stat_row(a, b, jj) * a.geo.ns + s] = p;
    }
}

// ---- verify: acceptance test and first rejection -------------------------------------------

// logsumexp * log2(e) of statistics row y from its slices' (ref, S) pairs (slice_lse): the sums are
// brought to the largest reference with single-precision exp2 of the (small, exactly formed)
// reference differences and added in fp64.  Slices are fetched four at a time so that the loads
// of a chunk are in flight together.
template <int CH = 4>       // slices fetched together
__device__ __forceinline__ double row_L(const Partial *part, size_t y, int ns)
{
    float r = neg_inf();
    double S = 0.0;
    for (int s0 = 0; s0 < ns; s0 += CH) {
        float pm[CH];
        double pS[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {          // the loads first, all of them ...
            const Partial *p = part + y * ns + (s0 + u < ns ? s0 + u : 0);
            pm[u] = p->m;
            pS[u] = p->S;
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {          // ... then what depends on them (else each load is waited for in turn)
            if (!(s0 + u < ns) || !(pS[u] > 0.0)) {
                pm[u] = neg_inf();
                pS[u] = 0.0;
            }
        }
        float rc = pm[0];
#pragma unroll
        for (int u = 1; u < CH; ++u) rc = vmax(rc, pm[u]);
        if (rc == neg_inf()) continue;
        if (rc > r) {
            if (r != neg_inf()) S *= (double)exp2_raw((float)((double)r - (double)rc));
            r = rc;
        }
#pragma unroll
        for (int u = 0; u < CH; ++u)
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
    // One wave, a chain of trips to memory: the draft length, then tokens / uniforms / logsumexps / slice
    // statistics, then the two gathered logits.  The first pass's loads that need no draft length (everything
    // indexed by position j < k) are requested together with it, and the gathers before the slice statistics
    // are merged, so a sequence takes three trips instead of five.
    int graw = a.draft_len[b];
    int x0 = 0;
    float u0 = 0.f;
    double lse0 = 0.0;
    if (lane < a.k) {
        x0 = a.tokens[(size_t)b * a.k + lane];
        u0 = a.u_accept[(size_t)b * a.k + lane];
        if (a.draft_lse) lse0 = a.draft_lse[(size_t)b * a.k + lane];
    }
    asm volatile("" : "+v"(graw) : : "memory");     // the draft length is first looked at here
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
            int x = x0;
            double u = (double)u0, lse_q = lse0;
            if (j0 > 0 && j < g) {
                x = a.tokens[(size_t)b * a.k + j];
                u = (double)a.u_accept[(size_t)b * a.k + j];
                if (a.draft_lse) lse_q = a.draft_lse[(size_t)b * a.k + j];
            }
            DT zp_stored = DT(), zq_stored = DT();          // requested here, widened after the statistics are merged
            if (j < g) {
                if (x < 0 || x >= a.geo.V) {
                    if (publish) atomicOr(a.ws.flags, (unsigned)SVIP_FLAG_BAD_TOKEN);
                    x = x < 0 ? 0 : a.geo.V - 1;
                }
                zp_stored = (tgt + (long long)j * a.row_stride)[x];
                zq_stored = (drf + (long long)j * a.row_stride)[x];
            }
            Lp = row_L<8>(a.ws.part, stat_row(a, b, a.kd + j), a.geo.ns);
            if (j < g) {
                Lq = a.draft_lse ? lse_q * LOG2E : row_L<8>(a.ws.part, stat_row(a, b, j), a.geo.ns);
                const double zp = (double)widen(not_before_here(zp_stored)), zq = (double)widen(not_before_here(zq_stored));
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
    if (a.skip && a.skip[blockIdx.x]) return;
    accept_sequence<DT>(a, blockIdx.x, threadIdx.x, true);
}

// ---- verify: residual / bonus sampling ------------------------------------------------------

// What a slice's workgroup hands to the sequence's last workgroup: residual and target mass of each
// of its tiles (slices longer than TILE_MASSES tiles fold the rest into the last entry and are
// searched as a whole).
struct ResidSlot {
    double W[TILE_MASSES], P[TILE_MASSES];
};

struct ResidLds {
    double sums[NWAVE][2 * TILE_MASSES];
    FinishLds fin;
    int last;
};

// What the thread that finds the correction or bonus token does with it (see locate_batch's `report`).
struct StoreNextToken {
    static constexpr bool active = true;
    int *next_token;
    int b;
    __device__ __forceinline__ void operator()(int tok, float) const { next_token[b] = tok; }
};

// grid (sequences * slices), the whole residual / bonus draw in one launch.  Every workgroup sums
// the weights of its slice tile by tile -- residual max(0, p - q) at the rejected position, and target p
// of the row to sample -- and publishes them; the workgroup that draws the sequence's final ticket
// chooses between residual and target weights (no residual mass: draw from p), picks the slice and
// the tile that hold u * total and finds the token there by the inverse CDF.  TILES: slices have at
// most TILE_MASSES tiles, so the search reads one tile; otherwise it walks the chosen slice.
template <typename DT, bool TILES>
__global__ __launch_bounds__(WG, 4) void k_resid(VerifyArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ ResidLds sh;
    const int ns = a.geo_s.ns;
    // Workgroups go to the chip's 8 XCDs in turn: all slices of sequence b are kept on XCD b % 8, so the
    // workgroup that finishes the sequence reads the chosen tile again from the L2 that already streamed it
    // (13.2 -> 12.9 us at 64 sequences of 128K logits, 35 -> 33 us at 256).  The grid is ceil(B / 8) * 8 * ns.
    const unsigned xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
    const int b = (int)((slot / (unsigned)ns) * 8u + xcd), s = (int)(slot % (unsigned)ns), tid = threadIdx.x;
    if (b >= a.B) return;
    if (a.skip && a.skip[b]) return;
    const SeqRec rec = a.ws.rec[b];
    const DT *prow = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, rec.r);
    const DT *qrow = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, rec.r);
    const ExpRef ep = make_exp_ref(a.sc, rec.Lp), eq = make_exp_ref(a.sc, rec.Lq);
    ResidSlot *slots = reinterpret_cast<ResidSlot *>(a.ws.mass) + (size_t)b * ns;
    {
        const int tb = s * a.geo_s.tps, te = min(tb + a.geo_s.tps, a.geo_s.ntiles);
        float Wt[TILE_MASSES], Pt[TILE_MASSES];
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) Wt[v] = Pt[v] = 0.f;
        if (rec.resid) slice_mass<DT, true>(prow, qrow, a.geo_s.V, tb, te, ep, eq, Wt, Pt);
        else slice_mass<DT, false>(prow, qrow, a.geo_s.V, tb, te, ep, eq, Wt, Pt);
        const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) {
            const double Wd = wave_sum((double)Wt[v]), Pd = wave_sum((double)Pt[v]);
            if (lane == 0) {
                sh.sums[wave][v] = Wd;
                sh.sums[wave][TILE_MASSES + v] = Pd;
            }
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int v = 0; v < TILE_MASSES; ++v) {
                double W = 0.0, P = 0.0;
#pragma unroll
                for (int w = 0; w < NWAVE; ++w) {
                    W += sh.sums[w][v];
                    P += sh.sums[w][TILE_MASSES + v];
                }
                publish_f64(&slots[s].W[v], W);
                publish_f64(&slots[s].P[v], P);
            }
            stores_done();
            sh.last = take_ticket(ticket(a.ws.tickets, b, TICKET_RESID)) == (unsigned)ns - 1u;
        }
        __syncthreads();
    }
    if (!sh.last) return;

    // ---- the sequence's last workgroup ----
    if (tid < 64) {
        const float u = a.u_resample[b];
        double W[TILE_MASSES], P[TILE_MASSES];
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) W[v] = P[v] = 0.0;
        if (tid < ns) {
            unsigned long long x[2 * TILE_MASSES];
#pragma unroll
            for (int v = 0; v < TILE_MASSES; ++v) {          // all in flight together
                x[v] = fetch_u64(&slots[tid].W[v]);
                x[TILE_MASSES + v] = fetch_u64(&slots[tid].P[v]);
            }
#pragma unroll
            for (int v = 0; v < TILE_MASSES; ++v) {
                W[v] = __longlong_as_double((long long)x[v]);
                P[v] = __longlong_as_double((long long)x[TILE_MASSES + v]);
            }
        }
        if (tid == 0) reset_tickets(ticket(a.ws.tickets, b, TICKET_RESID));
        double Ws = 0.0, Ps = 0.0;
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) {
            Ws += W[v];
            Ps += P[v];
        }
        const double inclW = wave_inclusive_sum(Ws), inclP = wave_inclusive_sum(Ps);
        const double totW = read_lane(inclW, 63), totP = read_lane(inclP, 63);
        const bool resid = rec.resid && totW > 0.0;   // no residual mass: draw from the target row
        const double M = resid ? Ws : Ps, incl = resid ? inclW : inclP, tot = resid ? totW : totP;
        double local;
        const int sl = pick_slice(M, (double)u * tot, incl, &local);
        int tile = 0;
        if (TILES) {
            double Gs[TILE_MASSES];
#pragma unroll
            for (int v = 0; v < TILE_MASSES; ++v) Gs[v] = read_lane(resid ? W[v] : P[v], sl);
            double in_tile;
            tile = pick_tile(Gs, local, &in_tile);
            local = in_tile;
        }
        if (tid == 0) {
            sh.fin.target = local;
            sh.fin.slice = sl;
            sh.fin.tile = tile;
            sh.fin.use_resid = resid ? 1 : 0;
        }
    }
    __syncthreads();
    int tb = sh.fin.slice * a.geo_s.tps, te = min(tb + a.geo_s.tps, a.geo_s.ntiles);
    if (TILES) {
        tb += sh.fin.tile;
        te = tb + 1;
    }
    constexpr int LU = TILES ? 1 : 2;
    // the thread that finds the token stores it; nothing else in this kernel has used sh.fin.loc
    const StoreNextToken store{a.next_token, b};
    float wtok;
    if (sh.fin.use_resid) {
        ResidualWeights<DT> wf{prow, qrow, a.geo_s.V, ep, eq};
        locate_in_slice<N, LU>(wf, tb, te, sh.fin.target, sh.fin.loc, &wtok, NoHook(), true, store);
    } else {
        SoftmaxWeights<DT> wf{prow, a.geo_s.V, ep};
        locate_in_slice<N, LU>(wf, tb, te, sh.fin.target, sh.fin.loc, &wtok, NoHook(), true, store);
    }
}

}  // namespace svip
