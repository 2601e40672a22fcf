// Kernels of svip_draft_step and svip_draft_step_greedy.
#pragma once
#include "kernel_args.h"
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

struct FinishLds {
    LocateLds loc;
    double target, L, S, tt;
    float m;
    int slice, tile;
    int use_resid;
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

// The draft step is two launches ordered by the stream.
//
// k_draft_stats: the statistics of a row as one record per WAVE.  Record r of a row covers tiles
// [r * tps, (r + 1) * tps), and a wave reads a tile (256 consecutive vectors) as four loads of 64
// consecutive vectors.  Nothing is shared between the waves of a workgroup -- no LDS, no barrier, so
// no wave waits for data that another wave's loads are still bringing in.
// k_draft_finish: one workgroup per row; one wave merges the row's records (a record per lane), writes
// entropy, logsumexp and stop flag, and picks the record that holds u * S -- for rows of up to 64 tiles
// a single tile, which is all the inverse-CDF search has to read again; with greedy drafting (ARG) the
// token is the first maximum the records already carry and nothing is read again.
//
// A single launch in which the row's last workgroup does the second part (hand-over through
// write-through stores and a ticket, as the residual pass of verification does) measured the same at 64
// rows of 128K logits and slower beyond, and was dropped for this simpler form.

// A row's stop flag, requested without looking at it: with no flag array the load goes to the start of the
// records (any valid address) and the value is ignored.  flag_after_loads() is where the value is first looked
// at: no access to memory moves across it, and the flag cannot be consumed earlier.  Together they keep the flag
// and the loads issued between them in flight at the same time; written as `stop_in && stop_in[b]` followed by
// an early return, the compiler waits for the flag first and only then issues the other loads (it sinks them
// below the return, or moves the flag to a scalar register at once), one more trip to memory per kernel.
__device__ __forceinline__ unsigned request_stop_flag(const DraftArgs &a, int b)
{
    const unsigned char *p = a.stop_in ? a.stop_in + b : reinterpret_cast<const unsigned char *>(a.part);
    return *p;
}
__device__ __forceinline__ bool flag_after_loads(const DraftArgs &a, unsigned flag)
{
    asm volatile("" : "+v"(flag) : : "memory");
    return a.stop_in && flag;
}

// One batch of a wave: chunks [c0, c0 + NU) of 64 vectors each; CHECKED for the row's last, partial tile.
template <typename DT, int NU, bool CHECKED>
__device__ __forceinline__ void wave_load(const DT *row, int V, int c0, typename RawOf<DT>::type (&raw)[NU])
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < NU; ++u)
        raw[u] = CHECKED ? load_raw_checked<DT>(row, (c0 + u) * 64 + lane, V) : load_raw<DT>(row, (c0 + u) * 64 + lane);
}
template <typename DT, int NU, bool ARG>
__device__ __forceinline__ void wave_accumulate(const typename RawOf<DT>::type (&raw)[NU], int c0, float &m, float &ones,
                                                float &S, float &t, int &idx, const Scale &sc)
{
    constexpr int N = VecOf<DT>::N;
    float z[NU][N];
#pragma unroll
    for (int u = 0; u < NU; ++u) unpack<DT>(raw[u], z[u]);
    accumulate<N, NU, ARG>(z, m, ones, S, t, sc, idx, c0);
}

// grid (ceil(rows * records / 4)), one wave per record.  TWO: the launch's records hold two tiles; a record of
// two whole tiles then requests both before it works on the first (the arithmetic of the first runs while the
// second is still on its way: 0.2 us of an 11.2 us step at 64 rows of 128K logits, 0.55 of 21 us at 256), which
// takes 65 registers; with one tile per record that form is 0.2 us slower, so those launches keep the other.
template <typename DT, bool ARG, bool TWO>
__global__ __launch_bounds__(WG, TWO ? 6 : 8) void k_draft_stats(DraftArgs a)
{
    constexpr int N = VecOf<DT>::N, CPT = WG / 64;       // chunks of 64 vectors per tile
    const int lane = threadIdx.x & 63, nrec = a.geo.ns;
    // Which record this wave takes is the same in all its lanes: worked out in scalar registers, with the one
    // division done by a multiplication the host prepared, so that none of it takes vector-ALU slots (a wave of one
    // tile has about 500 vector instructions in all, and they are what bounds this kernel).
    const unsigned wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int b, r;
    if (a.rows_by_xcd) {
        // Workgroups go to the chip's 8 XCDs in turn, and so do the rows' workgroups of k_draft_finish: keeping
        // row b on XCD b % 8 lets that kernel find the row's records and the tile it reads again in the L2 of
        // its own XCD.  The grid is ceil(B / 8) * 8 * ceil(nrec / 4) workgroups; those of rows past B exit.
        const unsigned xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;           // div = workgroups per row
        const unsigned q = a.div == 1u ? slot : __umulhi(slot, a.div_magic);
        b = (int)(q * 8u + xcd);
        r = (int)((slot - q * a.div) * NWAVE + wv);
        if (b >= a.B || r >= nrec) return;
    } else {
        const unsigned gw = blockIdx.x * NWAVE + wv;                            // div = records per row
        if (gw >= (unsigned)a.B * (unsigned)nrec) return;
        b = (int)(a.div == 1u ? gw : __umulhi(gw, a.div_magic));
        r = (int)(gw - (unsigned)b * (unsigned)nrec);
    }
    const DT *row = static_cast<const DT *>(a.logits) + draft_row_offset(a, b);
    const int tb = r * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    const int fe = min(te, a.geo.V / (WG * N));           // end of the tiles wholly inside the row
    float m = neg_inf(), ones = 0.f, S = 0.f, t = 0.f;
    int idx = -1;
    // The record's first tile is requested before the row's stop flag is looked at, so that the two travel
    // together (a step is bound by round trips to memory); a stopped row costs those loads and nothing else.
    const unsigned flag = request_stop_flag(a, b);
    typename RawOf<DT>::type raw[CPT];
    if (TWO && te - tb == 2 && te <= fe) {
        typename RawOf<DT>::type raw2[CPT];
        wave_load<DT, CPT, false>(row, a.geo.V, tb * CPT, raw);
        wave_load<DT, CPT, false>(row, a.geo.V, (tb + 1) * CPT, raw2);
        if (flag_after_loads(a, flag)) return;
        wave_accumulate<DT, CPT, ARG>(raw, tb * CPT, m, ones, S, t, idx, a.sc);
        wave_accumulate<DT, CPT, ARG>(raw2, (tb + 1) * CPT, m, ones, S, t, idx, a.sc);
    } else {
        if (tb < fe) wave_load<DT, CPT, false>(row, a.geo.V, tb * CPT, raw);
        else wave_load<DT, CPT, true>(row, a.geo.V, tb * CPT, raw);
        if (flag_after_loads(a, flag)) return;
        wave_accumulate<DT, CPT, ARG>(raw, tb * CPT, m, ones, S, t, idx, a.sc);
        for (int t0 = tb + 1; t0 < te; ++t0) {
            if (t0 < fe) wave_load<DT, CPT, false>(row, a.geo.V, t0 * CPT, raw);
            else wave_load<DT, CPT, true>(row, a.geo.V, t0 * CPT, raw);
            wave_accumulate<DT, CPT, ARG>(raw, t0 * CPT, m, ones, S, t, idx, a.sc);
        }
    }
    // the wave's lanes to one record: maximum first, then sums rescaled to it in fp64
    const float mw = wave_max(m);
    double Sd = 0.0, td = 0.0;
    if (m != neg_inf()) {
        const float xd = scaled_diff(m, mw, a.sc);
        const double all = (double)ones + (double)S, f = (double)exp2_raw(xd);
        Sd = f * all;
        td = f * ((double)t + (double)xd * all);
    }
    Sd = wave_sum(Sd);
    td = wave_sum(td);
    int first = -1;
    if (ARG) {      // smallest index among the lanes that hold the wave maximum
        const int cand = (m == mw && idx >= 0) ? idx : 0x7FFFFFFF;
        const int wmin = -wave_reduce(-cand, OpMax{});
        first = wmin == 0x7FFFFFFF ? -1 : wmin;
    }
    if (lane == 0) {
        Partial p;
        p.m = mw;
        p.idx = first;
        p.S = Sd;
        p.t = td;
        a.part[(size_t)b * nrec + r] = p;
    }
}

// What the thread that finds the draft token does with it (see locate_batch's `report`).
struct StoreDraftToken {
    static constexpr bool active = true;
    const DraftArgs &a;
    long long o;
    double S;
    __device__ __forceinline__ void operator()(int tok, float w) const
    {
        a.token[o] = tok;
        if (a.q_tok) a.q_tok[o] = (float)((double)w / S);
    }
};

// grid (rows): the rows' last step over the records of k_draft_stats.  Sampling: WG + 64 threads, greedy: 64.
// Waves 0 .. 3 search for the token; the extra wave writes entropy, logsumexp and stop flag and ends, so that
// work (an fp64 logarithm and a square root, 0.3 us) neither sits in front of the search nor holds up its barriers.
constexpr int FINISH_THREADS = WG + 64;
template <typename DT, bool ARG>
__global__ __launch_bounds__(FINISH_THREADS, 4) void k_draft_finish(DraftArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ LocateLds loc;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, nrec = a.geo.ns;
    const long long o = (long long)b * a.io_stride;
    // independent loads first: the row's flag, its uniform and its records travel together.  Every wave loads and
    // merges the records for itself (a record per lane): the waves then agree on the record to search without
    // passing anything through LDS or waiting for one another.
    const unsigned flag = request_stop_flag(a, b);
    Partial p;
    p.m = neg_inf();
    p.idx = -1;
    p.S = 0.0;
    p.t = 0.0;
    float u = 0.f;
    if (lane < nrec) p = a.part[(size_t)b * nrec + lane];
    if (!ARG) u = a.u[o];
    if (flag_after_loads(a, flag)) {
        if (tid == 0) {
            a.token[o] = -1;
            a.stop[b] = 1;
        }
        return;
    }
    const DT *row = static_cast<const DT *>(a.logits) + draft_row_offset(a, b);
    // everything relative to the row maximum: this lane's record by the factor f
    const float mrow = wave_max(p.m);
    double f = 0.0, xd = 0.0;
    if (p.m != neg_inf() && p.S > 0.0) {
        xd = ((double)p.m - (double)mrow) * a.sc.c;
        f = exp2(xd);
    }
    const double M = f * p.S;
    const double incl = wave_inclusive_sum(M);
    const double S = read_lane(incl, 63);
    const double tt = wave_sum(f * (p.t + xd * p.S));
    if (ARG) {
        // records are in index order: the first that reaches the row maximum holds its first index
        const unsigned long long at_max = __ballot(p.m == mrow && p.idx >= 0);
        const int tok = at_max ? read_lane(p.idx, __ffsll((long long)at_max) - 1) : -1;
        if (tid == 0) {
            a.token[o] = tok;
            if (a.q_tok) a.q_tok[o] = (float)(1.0 / S);           // the maximum has weight exp2(0) = 1
            write_row_outputs(a, b, o, mrow, S, tt);
        }
        return;
    }
    // the extra wave: the outputs that do not depend on the token.  The test is on a scalar register, so the wave
    // branches to the end of the program and is gone before the other waves' first barrier.
    if (__builtin_amdgcn_readfirstlane(tid >> 6) == NWAVE) {
        if (lane == 0) write_row_outputs(a, b, o, mrow, S, tt);
        return;
    }
    double target;
    const int rec = pick_slice(M, (double)u * S, incl, &target);
    SoftmaxWeights<DT> wf{row, a.geo.V, make_exp_ref(a.sc, (double)mrow * a.sc.c)};
    // the thread that finds the token stores it; nothing else in this kernel has used the search's LDS
    const StoreDraftToken store{a, o, S};
    float wtok;
    const int tb = rec * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    // a record of one tile is searched as one batch of one tile, longer records two tiles at a time
    if (a.geo.tps == 1) locate_in_slice<N, 1>(wf, tb, te, target, loc, &wtok, NoHook(), true, store);
    else locate_in_slice<N, 2>(wf, tb, te, target, loc, &wtok, NoHook(), true, store);
}

}  // namespace svip
