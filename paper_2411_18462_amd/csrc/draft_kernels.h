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

// grid (rows * slices): statistics of slice s of row b.  ARG (greedy drafting) also records
// the smallest index that holds the slice maximum.
template <typename DT, bool ARG>
__global__ __launch_bounds__(WG) void k_draft_stats(DraftArgs a)
{
    __shared__ CombineLds lds;
    const int b = blockIdx.x / a.geo.ns, s = blockIdx.x - b * a.geo.ns;
    if (a.stop_in && a.stop_in[b]) return;
    const DT *row = static_cast<const DT *>(a.logits) + draft_row_offset(a, b);
    const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    const Partial p = slice_stats<DT, ARG>(row, a.geo.V, tb, te, a.sc, lds);
    if (threadIdx.x == 0) a.part[(size_t)b * a.geo.ns + s] = p;
}

struct FinishLds {
    LocateLds loc;
    double target, L, S, tt;
    float m;
    int slice;
    int use_resid;
};

// grid (rows): merge of the row's slices, entropy and stop test, inverse CDF.
template <typename DT>
__global__ __launch_bounds__(WG) void k_draft_finish(DraftArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ FinishLds sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    const long long o = (long long)b * a.io_stride;
    // independent loads first: the row's flag, its uniform and its slice statistics
    const unsigned char stopped = a.stop_in ? a.stop_in[b] : (unsigned char)0;
    const float u = a.u[o];
    Partial p;
    p.m = neg_inf();
    p.S = 0.0;
    p.t = 0.0;
    if (tid < a.geo.ns) p = a.part[(size_t)b * a.geo.ns + tid];
    if (stopped) {
        if (tid == 0) {
            a.token[o] = -1;
            a.stop[b] = 1;
        }
        return;
    }
    const DT *row = static_cast<const DT *>(a.logits) + draft_row_offset(a, b);
    if (tid < 64) {
        const Merged mg = merge_lane(tid < a.geo.ns ? p.m : neg_inf(), p.S, p.t, a.sc);
        const double incl = wave_inclusive_sum(mg.M);
        const double S = read_lane(incl, 63);
        const double tt = wave_sum(mg.tt);
        double local;
        const int s = pick_slice(mg.M, (double)u * S, incl, &local);
        if (tid == 0) {
            sh.target = local;
            sh.L = (double)mg.m * a.sc.c;
            sh.S = S;
            sh.tt = tt;
            sh.m = mg.m;
            sh.slice = s;
        }
    }
    __syncthreads();
    SoftmaxWeights<DT> wf{row, a.geo.V, make_exp_ref(a.sc, sh.L)};
    const int tb = sh.slice * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    // entropy, logsumexp and the stop test do not depend on the token: thread 0 computes and stores
    // them while the slice's logits are on their way
    auto row_outputs = [&]() {
        if (tid == 0) {
            // H = ln S - (sum e x ln2) / S  for weights e = exp2(x): the entropy of e / S
            const double S = sh.S, lnS = log(S);
            double H = lnS - 0.6931471805599453 * sh.tt / S;
            H = H > 0.0 ? H : 0.0;
            if (a.entropy) a.entropy[o] = (float)H;
            a.lse[o] = (double)sh.m * a.sc.inv_T + lnS;
            const bool stop = (sqrt(H) > (double)a.h) || at_cap(a, b);
            a.stop[b] = stop ? 1 : 0;
            if (a.draft_len) a.draft_len[b] = a.step_j + 1;
        }
    };
    float wtok;
    const int tok = locate_in_slice<N>(wf, tb, te, sh.target, sh.loc, &wtok, row_outputs);
    if (tid == 0) {
        a.token[o] = tok;
        if (a.q_tok) a.q_tok[o] = (float)((double)wtok / sh.S);
    }
}

// grid (rows), one wave: greedy drafting.  Merge of the row's slices, entropy and stop test;
// the token is the first maximum of the row (Algorithm 1 with argmax in place of the draw).
__global__ __launch_bounds__(64) void k_draft_finish_greedy(DraftArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const long long o = (long long)b * a.io_stride;
    const unsigned char stopped = a.stop_in ? a.stop_in[b] : (unsigned char)0;
    Partial p;
    p.m = neg_inf();
    p.idx = -1;
    p.S = 0.0;
    p.t = 0.0;
    if (lane < a.geo.ns) p = a.part[(size_t)b * a.geo.ns + lane];
    if (stopped) {
        if (lane == 0) {
            a.token[o] = -1;
            a.stop[b] = 1;
        }
        return;
    }
    const Merged mg = merge_lane(lane < a.geo.ns ? p.m : neg_inf(), p.S, p.t, a.sc);
    const double S = wave_sum(mg.M);
    const double tt = wave_sum(mg.tt);
    // slices are in index order: the first slice that reaches the row maximum holds its first index
    const unsigned long long at_max = __ballot(lane < a.geo.ns && p.m == mg.m && p.idx >= 0);
    const int tok = at_max ? read_lane(p.idx, __ffsll((long long)at_max) - 1) : -1;
    if (lane == 0) {
        const double lnS = log(S);
        double H = lnS - 0.6931471805599453 * tt / S;
        H = H > 0.0 ? H : 0.0;
        a.token[o] = tok;
        if (a.entropy) a.entropy[o] = (float)H;
        if (a.q_tok) a.q_tok[o] = (float)(1.0 / S);           // the maximum has weight exp2(0) = 1
        a.lse[o] = (double)mg.m * a.sc.inv_T + lnS;
        const bool stop = (sqrt(H) > (double)a.h) || at_cap(a, b);
        a.stop[b] = stop ? 1 : 0;
        if (a.draft_len) a.draft_len[b] = a.step_j + 1;
    }
}

}  // namespace svip
