// Kernels of svip_draft_step and svip_draft_step_greedy.
#pragma once
#include "exchange.h"
#include "kernel_args.h"
#include "stage_clock.h"
#include "sample_weights.h"

namespace svip {

// ---- draft step -------------------------------------------------------------------------------

__device__ __forceinline__ long long draft_row_offset(const DraftArgs &a, int b)
{
    return (long long)b * a.row_stride + (a.pos ? (long long)(a.pos[b] + a.step_j) * a.pos_stride : 0ll);
}
__device__ __forceinline__ bool at_cap(const DraftArgs &a, int b)
{
    const int cap = a.cap ? min(a.cap[b], a.k_max) : a.k_max;
    return a.step_j + 1 >= cap;
}

// What a slice's workgroup hands to the row's last workgroup: the slice statistics and, for slices of
// at most TILE_MASSES tiles, the mass of every tile (relative to the slice maximum).  Seven 64-bit words.
struct DraftSlot {
    Partial p;
    double G[TILE_MASSES];
};
template <bool TILES>
__device__ __forceinline__ void publish_slot(DraftSlot *slot, const Partial &p, const double (&G)[TILE_MASSES])
{
    unsigned long long *w = reinterpret_cast<unsigned long long *>(slot);
    publish_u64(w + 0, (unsigned long long)__float_as_uint(p.m) | ((unsigned long long)(unsigned)p.idx << 32));
    publish_u64(w + 1, (unsigned long long)__double_as_longlong(p.S));
    publish_u64(w + 2, (unsigned long long)__double_as_longlong(p.t));
    if (TILES) {
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) publish_u64(w + 3 + v, (unsigned long long)__double_as_longlong(G[v]));
    }
}
template <bool TILES>
__device__ __forceinline__ void fetch_slot(const DraftSlot *slot, Partial &p, double (&G)[TILE_MASSES])
{
    const unsigned long long *w = reinterpret_cast<const unsigned long long *>(slot);
    unsigned long long x[3 + TILE_MASSES];
#pragma unroll
    for (int v = 0; v < (TILES ? 3 + TILE_MASSES : 3); ++v) x[v] = fetch_u64(w + v);      // all in flight together
    p.m = __uint_as_float((unsigned)x[0]);
    p.idx = (int)(unsigned)(x[0] >> 32);
    p.S = __longlong_as_double((long long)x[1]);
    p.t = __longlong_as_double((long long)x[2]);
    if (TILES) {
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) G[v] = __longlong_as_double((long long)x[3 + v]);
    }
}

struct FinishLds {
    LocateLds loc;
    double target, L, S, tt;
    float m;
    int slice, tile;
    int use_resid;
};

struct DraftLds {
    CombineLds comb;
    FinishLds fin;
    DraftSlot own;     // the only slice's record when a row is not cut
    int last;          // this workgroup drew the row's final ticket
};

// Entropy of weights e_i = exp2(x_i) with sum S and tt = sum e_i x_i:  H = ln S - ln2 tt / S, then the
// stop test and the row's outputs that do not depend on the token (Section 2.2, Eq. stop_condition).
__device__ __forceinline__ void write_row_outputs(const DraftArgs &a, int b, long long o, float m, double S, double tt)
{
    const double lnS = log(S);
    double H = lnS - 0.6931471805599453 * tt / S;
    H = H > 0.0 ? H : 0.0;
    if (a.entropy) a.entropy[o] = (float)H;
    a.lse[o] = (double)m * a.sc.inv_T + lnS;
    const bool stop = (sqrt(H) > (double)a.h) || at_cap(a, b);
    a.stop[b] = stop ? 1 : 0;
    if (a.draft_len) a.draft_len[b] = a.step_j + 1;
}

// The whole draft step in one launch, grid (rows * slices).  Every workgroup streams one slice of
// one row and publishes its statistics; the workgroup that draws the row's final ticket merges the
// slices, writes entropy, logsumexp and stop flag, and finds the token: by the inverse CDF in the one
// tile (TILES: slices of at most TILE_MASSES tiles, whose tile masses are published too) or the one
// slice that holds u * S, re-read from cache; or, with ARG (greedy drafting), as the first maximum
// the statistics already carry.  A stopped row's workgroups leave at once; its slice 0 writes the
// token -1 and keeps the flag.
// PHASE 0 is that single launch.  PHASES 1 and 2 are the same work as two launches ordered by the stream:
// 1 = the slices' statistics only, grid (rows * slices), stored plainly; 2 = the rows' last step only,
// grid (rows).  A kernel boundary costs about 2 us; the hand-over inside one launch costs every slice's
// workgroup about 1 us of waiting for acknowledged stores and its ticket, which a grid of more than one
// round of workgroups pays again and again, so large batches take the two launches.
template <typename DT, bool ARG, bool TILES, int PHASE>
__global__ __launch_bounds__(WG, 5) void k_draft_step(DraftArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ DraftLds sh;
    const int ns = a.geo.ns;
    const int b = PHASE == 2 ? blockIdx.x : blockIdx.x / ns, s = PHASE == 2 ? 0 : blockIdx.x - b * ns, tid = threadIdx.x;
    const long long o = (long long)b * a.io_stride;
    STAGE(0);
    STAGE_WHERE();
    // A stopped row leaves at once -- except in the single launch, which is bound by round trips to memory,
    // not by bandwidth: there the flag is only looked at once the slice has been read, so that its load and
    // the logits' loads travel together (the logits of a stopped row are read and ignored).
    const bool stopped = a.stop_in && a.stop_in[b];
    if (PHASE != 0 && stopped) {
        if (s == 0 && tid == 0) {
            a.token[o] = -1;
            a.stop[b] = 1;
        }
        return;
    }
    const DT *row = static_cast<const DT *>(a.logits) + draft_row_offset(a, b);
    DraftSlot *slots = static_cast<DraftSlot *>(a.part) + (size_t)b * ns;
    if (PHASE != 2) {
        const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
        STAGE(1);
        double G[TILE_MASSES];
        const Partial p = slice_stats<DT, ARG, TILES && !ARG>(row, a.geo.V, tb, te, a.sc, sh.comb, G);
        STAGE(2);
        if (PHASE == 0 && stopped) {
            if (s == 0 && tid == 0) {
                a.token[o] = -1;
                a.stop[b] = 1;
            }
            return;
        }
        if (PHASE == 1) {
            if (tid == 0) {
                slots[s].p = p;
                if (TILES && !ARG) {
#pragma unroll
                    for (int v = 0; v < TILE_MASSES; ++v) slots[s].G[v] = G[v];
                }
            }
            return;
        }
        if (tid == 0) {
            if (ns == 1) {
                sh.own.p = p;
#pragma unroll
                for (int v = 0; v < TILE_MASSES; ++v) sh.own.G[v] = G[v];
                sh.last = 1;
            } else {
                publish_slot<TILES && !ARG>(slots + s, p, G);
                stores_done();
                STAGE(3);
                sh.last = take_ticket(ticket(a.tickets, b, TICKET_DRAFT)) == (unsigned)ns - 1u;
            }
        }
        __syncthreads();
        STAGE(4);
        if (!sh.last) return;
    }

    // ---- the row's last workgroup ----
    if (tid < 64) {
        Partial p;
        p.m = neg_inf();
        p.idx = -1;
        p.S = 0.0;
        p.t = 0.0;
        double G[TILE_MASSES];
#pragma unroll
        for (int v = 0; v < TILE_MASSES; ++v) G[v] = 0.0;
        if (PHASE == 2) {
            if (tid < ns) {         // written by the launch before: plain loads
                p = slots[tid].p;
                if (TILES && !ARG) {
#pragma unroll
                    for (int v = 0; v < TILE_MASSES; ++v) G[v] = slots[tid].G[v];
                }
            }
        } else if (ns == 1) {
            if (tid == 0) {
                p = sh.own.p;
#pragma unroll
                for (int v = 0; v < TILE_MASSES; ++v) G[v] = sh.own.G[v];
            }
        } else if (tid < ns) {
            fetch_slot<TILES && !ARG>(slots + tid, p, G);
        }
        float u = 0.f;
        if (!ARG) u = a.u[o];
        if (PHASE == 0 && tid == 0 && ns > 1) reset_tickets(ticket(a.tickets, b, TICKET_DRAFT));
        // everything relative to the row maximum: this lane's slice by the factor f
        const float mrow = wave_max(p.m);
        double f = 0.0, xd = 0.0;
        if (p.m != neg_inf() && p.S > 0.0) {
            xd = ((double)p.m - (double)mrow) * a.sc.c;
            f = exp2(xd);
        }
        const double M = f * p.S;
        const double S = wave_sum(M);
        const double tt = wave_sum(f * (p.t + xd * p.S));
        STAGE(5);
        if (ARG) {
            // slices are in index order: the first slice that reaches the row maximum holds its first index
            const unsigned long long at_max = __ballot(p.m == mrow && p.idx >= 0);
            const int tok = at_max ? read_lane(p.idx, __ffsll((long long)at_max) - 1) : -1;
            if (tid == 0) {
                a.token[o] = tok;
                if (a.q_tok) a.q_tok[o] = (float)(1.0 / S);           // the maximum has weight exp2(0) = 1
                write_row_outputs(a, b, o, mrow, S, tt);
            }
        } else {
            // the draw: slices by the masses the search itself will meet (the tile sums where there are any)
            double Mp = M;
            if (TILES) {
                Mp = 0.0;
#pragma unroll
                for (int v = 0; v < TILE_MASSES; ++v) {
                    G[v] *= f;
                    Mp += G[v];
                }
            }
            const double incl = wave_inclusive_sum(Mp);
            double local;
            const int sl = pick_slice(Mp, (double)u * read_lane(incl, 63), incl, &local);
            int tile = 0;
            if (TILES) {
                double Gs[TILE_MASSES];
#pragma unroll
                for (int v = 0; v < TILE_MASSES; ++v) Gs[v] = read_lane(G[v], sl);
                double in_tile;
                tile = pick_tile(Gs, local, &in_tile);
                local = in_tile;
            }
            if (tid == 0) {
                sh.fin.target = local;
                sh.fin.L = (double)mrow * a.sc.c;
                sh.fin.S = S;
                sh.fin.tt = tt;
                sh.fin.m = mrow;
                sh.fin.slice = sl;
                sh.fin.tile = tile;
            }
        }
    }
    if (ARG) return;
    __syncthreads();
    STAGE(6);
    SoftmaxWeights<DT> wf{row, a.geo.V, make_exp_ref(a.sc, sh.fin.L)};
    // entropy, logsumexp and the stop test do not depend on the token: one thread of the last wave
    // computes and stores them while the logits are on their way
    auto row_outputs = [&]() {
        if (tid == WG - 1) write_row_outputs(a, b, o, sh.fin.m, sh.fin.S, sh.fin.tt);
    };
    float wtok;
    int tok;
    if (TILES) {
        const int tb = sh.fin.slice * a.geo.tps + sh.fin.tile;
        tok = locate_in_slice<N, 1>(wf, tb, tb + 1, sh.fin.target, sh.fin.loc, &wtok, row_outputs);
    } else {
        const int tb = sh.fin.slice * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
        tok = locate_in_slice<N, LOCATE_UNROLL>(wf, tb, te, sh.fin.target, sh.fin.loc, &wtok, row_outputs);
    }
    if (tid == 0) {
        a.token[o] = tok;
        if (a.q_tok) a.q_tok[o] = (float)((double)wtok / sh.fin.S);
    }
    STAGE(7);
}

}  // namespace svip
