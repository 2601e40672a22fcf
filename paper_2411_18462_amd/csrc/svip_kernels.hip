// SVIP hot path for MI355X (gfx950): kernels and the C ABI declared in include/svip.h.
//
// svip_draft_step  =  k_draft_stats    grid (slices, rows)       per-slice (m, S, t) of every active row
//                     k_draft_finish   grid (rows)               merge, entropy, stop test, inverse CDF
//   (greedy)          k_draft_stats<ARG> + k_draft_finish_greedy     token = first maximum, no search
// svip_verify      =  k_verify_stats   grid (slices, stat rows)  per-slice (m, S) of every needed row
//                     k_accept         grid (sequences), 1 wave  p/q test, ballot scan for the first rejection
//                     k_resid_mass     grid (slices, sequences)  slice masses of the residual / bonus row
//                     k_resid_finish   grid (sequences)          inverse CDF of the residual / bonus row
// svip_verify_greedy = k_argmax        grid (slices, target rows) first maximum per slice, no exponentials
//                     k_accept_greedy  grid (sequences), 1 wave  argmax p == x test, ballot, correction = argmax p
//
// svip_pair_stats  =  k_verify_stats   (rows j < draft_len of both models), k_pair_L (logsumexps),
//                     k_pair_sums      grid (slices, positions)  sum min(p,q), sum q log(q/p), sum q log q
//                     k_pair_finish    one thread per position   beta, KL, cross entropy, the bounds
//
// The passes are bound by HBM reads of the logits; there is no dense contraction, hence no MFMA.
// Kernels of one call are ordered by the stream only (no spinning, no device-side waits), and
// each small kernel issues all of its independent loads before the first dependent one, because
// at small batches a step is bound by round trips to memory rather than by bandwidth.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/svip.h"
#include "row_math.h"
#include "svip_internal.h"

namespace svip {

// ---- workspace layout ----------------------------------------------------------------

struct SeqRec {          // what k_accept hands to the residual kernels, one per sequence
    double Lp;           // logsumexp(target row r) * log2(e)
    double Lq;           // logsumexp(draft row r) * log2(e) (residual mode only)
    int r;               // target row to sample from (first rejection, or draft_len for a bonus)
    int resid;           // 1: residual of row r, 0: bonus from row r
};

struct Workspace {
    unsigned *flags;     // sticky device-data flags
    SeqRec *rec;         // [B]
    double *mass;        // [B][MAX_SLICES][2] residual mass, target mass per slice
    Partial *part;       // [stat rows][ns] slice statistics
};

constexpr int MAX_BATCH = 1 << 20;               // sequences per call (grids are one-dimensional)
constexpr size_t HEADER_BYTES = 256;
__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static size_t ws_rec_bytes(int B) { return align256((size_t)B * sizeof(SeqRec)); }
static size_t ws_mass_bytes(int B) { return align256((size_t)B * MAX_SLICES * 2 * sizeof(double)); }

static Workspace carve(void *ws, int B)
{
    char *p = static_cast<char *>(ws);
    Workspace w;
    w.flags = reinterpret_cast<unsigned *>(p);
    p += HEADER_BYTES;
    w.rec = reinterpret_cast<SeqRec *>(p);
    p += ws_rec_bytes(B);
    w.mass = reinterpret_cast<double *>(p);
    p += ws_mass_bytes(B);
    w.part = reinterpret_cast<Partial *>(p);
    return w;
}

// ---- kernel arguments ------------------------------------------------------------------

struct DraftArgs {
    const void *logits;
    long long row_stride;   // between the rows of consecutive sequences
    const int *pos;         // optional [B]: sequence b reads trace row pos[b] + step_j of its own trace
    long long pos_stride;   // elements between consecutive trace rows (used with pos)
    const int *cap;         // optional [B]: per-sequence limit on the draft length (at most k_max)
    int B;
    Geo geo;
    Scale sc;
    float h;
    int step_j, k_max;
    const float *u;
    const unsigned char *stop_in;
    int *token;
    float *entropy;
    float *q_tok;
    double *lse;
    unsigned char *stop;
    int *draft_len;
    long long io_stride;
    Partial *part;
};

struct VerifyArgs {
    const void *target;
    const void *draft;
    long long seq_t, seq_d, row_stride;
    const int *pos;   // optional [B]: row j of sequence b is trace row pos[b] + j
    int B, k;
    int kd;        // draft rows per sequence in the statistics pass: k if the draft logsumexps are recomputed, else 0
    int bonus;     // 1: the statistics pass also covers target row draft_len (verification), 0: rows j < draft_len only
    Geo geo;       // slicing of the statistics pass
    Geo geo_s;     // slicing of the sampling pass (slices of at most LOCATE_UNROLL tiles when possible)
    Scale sc;
    const int *tokens;
    const int *draft_len;
    const double *draft_lse;
    const float *u_accept;
    const float *u_resample;
    int *n_accepted;
    int *next_token;
    float *accept_prob;
    Workspace ws;
};

__device__ __forceinline__ int clamp_len(int g, int k) { return g < 0 ? 0 : (g > k ? k : g); }

// Element offset of row j of sequence b (seq_stride between sequences, optional trace position).
template <typename A>
__device__ __forceinline__ long long row_offset(const A &a, long long seq_stride, int b, int j)
{
    return (long long)b * seq_stride + (long long)(j + (a.pos ? a.pos[b] : 0)) * a.row_stride;
}

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
        unpack(pk, z);
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
        unpack(pk.p, zp);
        unpack(pk.q, zq);
#pragma unroll
        for (int e = 0; e < VecOf<DT>::N; ++e) w[e] = fmaxf(exp_p(zp[e]) - exp_q(zq[e]), 0.f);
    }
};

// One batch of NU vectors per thread of the rejected position's rows: adds the residual
// mass max(0, p - q) (if RESID) and the target mass p of the batch.
template <typename DT, int NU, bool RESID, bool CHECKED>
__device__ __forceinline__ void mass_batch(const DT *prow, const DT *qrow, int V, int t0, const ExpRef &ep,
                                           const ExpRef &eq, float &Wacc, float &Pacc)
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
    float Wb = 0.f, Pb = 0.f;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        float zp[N], pw[N];
        unpack(rp[u], zp);
#pragma unroll
        for (int e = 0; e < N; ++e) pw[e] = ep(zp[e]);
        Pb += tree_sum<N>(pw);
        if (RESID) {
            float zq[N], w[N];
            unpack(rq[u], zq);
#pragma unroll
            for (int e = 0; e < N; ++e) w[e] = fmaxf(pw[e] - eq(zq[e]), 0.f);
            Wb += tree_sum<N>(w);
        }
    }
    Wacc += Wb;
    Pacc += Pb;
}

// Per-thread residual and target masses of tiles [tb, te) in batches of LOCATE_UNROLL vectors
// (the same grouping of additions as the in-register path of k_resid).
template <typename DT, bool RESID>
__device__ __forceinline__ void slice_mass(const DT *prow, const DT *qrow, int V, int tb, int te,
                                           const ExpRef &ep, const ExpRef &eq, float &Wacc, float &Pacc)
{
    constexpr int N = VecOf<DT>::N;
    const int fe = min(te, V / (WG * N));
    int t0 = tb;
    for (; t0 + 4 <= fe; t0 += 4) mass_batch<DT, 4, RESID, false>(prow, qrow, V, t0, ep, eq, Wacc, Pacc);
    if (t0 + 2 <= fe) { mass_batch<DT, 2, RESID, false>(prow, qrow, V, t0, ep, eq, Wacc, Pacc); t0 += 2; }
    if (t0 + 1 <= fe) { mass_batch<DT, 1, RESID, false>(prow, qrow, V, t0, ep, eq, Wacc, Pacc); t0 += 1; }
    if (t0 < te) mass_batch<DT, 1, RESID, true>(prow, qrow, V, t0, ep, eq, Wacc, Pacc);
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
    __shared__ double lds[2 * NWAVE];
    const int b = blockIdx.x / a.geo.ns, s = blockIdx.x - b * a.geo.ns;
    if (a.stop_in && a.stop_in[b]) return;
    const DT *row = static_cast<const DT *>(a.logits) + draft_row_offset(a, b);
    const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    const Partial p = slice_stats<DT, true, ARG>(row, a.geo.V, tb, te, a.sc, lds);
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
    float wtok;
    const int tok = locate_in_slice<N>(wf, tb, te, sh.target, sh.loc, &wtok);
    if (tid == 0) {
        // H = ln S - (sum e x ln2) / S  for weights e = exp2(x): the entropy of e / S
        const double S = sh.S, lnS = log(S);
        double H = lnS - 0.6931471805599453 * sh.tt / S;
        H = H > 0.0 ? H : 0.0;
        a.token[o] = tok;
        if (a.entropy) a.entropy[o] = (float)H;
        if (a.q_tok) a.q_tok[o] = (float)((double)wtok / S);
        a.lse[o] = (double)sh.m * a.sc.inv_T + lnS;
        const bool stop = (sqrt(H) > (double)a.h) || at_cap(a, b);
        a.stop[b] = stop ? 1 : 0;
        if (a.draft_len) a.draft_len[b] = a.step_j + 1;
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

// ---- greedy verification (Algorithms 3 and 5) ------------------------------------------------

struct GreedyArgs {
    const void *target;
    long long seq_t, row_stride;
    const int *pos;   // optional [B]: row j of sequence b is trace row pos[b] + j
    int B, k;
    Geo geo;
    const int *tokens;
    const int *draft_len;
    int *n_accepted;
    int *next_token;
    unsigned long long *keys;    // [B (k+1)][ns] first-maximum keys
    unsigned *flags;
};

// grid (sequences * (k+1) * slices): first maximum of slice s of target row (b, j), j <= draft_len[b].
template <typename DT>
__global__ __launch_bounds__(WG) void k_argmax(GreedyArgs a)
{
    __shared__ unsigned long long lds[NWAVE];
    const int y = blockIdx.x / a.geo.ns, s = blockIdx.x - y * a.geo.ns;
    const int b = y / (a.k + 1), j = y - b * (a.k + 1);
    const int g = clamp_len(a.draft_len[b], a.k);
    if (j > g) return;
    const DT *row = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, j);
    const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    const unsigned long long key = slice_argmax<DT>(row, a.geo.V, tb, te, lds);
    if (threadIdx.x == 0) a.keys[(size_t)y * a.geo.ns + s] = key;
}

// grid (sequences), one wave: lane = position.  argmax of target row j from its slice keys;
// position j < draft_len is accepted iff that argmax is the draft token; a ballot finds the first
// failure r, and the correction (or, if none failed, the bonus token) is the argmax of row r.
__global__ __launch_bounds__(64) void k_accept_greedy(GreedyArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int graw = a.draft_len[b];
    const int g = clamp_len(graw, a.k);
    if (graw != g && lane == 0) atomicOr(a.flags, (unsigned)SVIP_FLAG_BAD_DRAFT_LEN);
    int r = -1, next = -1;
    for (int j0 = 0; j0 <= g && r < 0; j0 += 64) {
        const int j = j0 + lane;
        int am = -1;
        bool reject = false;
        if (j <= g) {
            const unsigned long long *kr = a.keys + ((size_t)b * (a.k + 1) + j) * a.geo.ns;
            unsigned long long best = 0ull;
            for (int s = 0; s < a.geo.ns; ++s) best = kr[s] > best ? kr[s] : best;
            am = argmax_index(best);
            if (j < g) {
                const int x = a.tokens[(size_t)b * a.k + j];
                if (x < 0 || x >= a.geo.V) atomicOr(a.flags, (unsigned)SVIP_FLAG_BAD_TOKEN);
                reject = am != x;
            }
        }
        const unsigned long long rej = __ballot(reject);
        if (rej) {
            const int first = __ffsll((long long)rej) - 1;
            r = j0 + first;
            next = read_lane(am, first);
        } else if (g - j0 < 64) {
            r = g;
            next = read_lane(am, g - j0);
        }
    }
    if (lane == 0) {
        a.n_accepted[b] = r;
        a.next_token[b] = next;
    }
}

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
    __shared__ double lds[2 * NWAVE];
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

// grid (sequences), one wave: lane = position, 64 positions per pass.  Lanes j <= draft_len merge
// the statistics of target row j; lanes j < draft_len run the acceptance test; a ballot finds
// the first rejection.
template <typename DT>
__global__ __launch_bounds__(64) void k_accept(VerifyArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int graw = a.draft_len[b];
    const int g = clamp_len(graw, a.k);
    if (graw != g && lane == 0) atomicOr(a.ws.flags, (unsigned)SVIP_FLAG_BAD_DRAFT_LEN);
    const DT *tgt = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, 0);
    const DT *drf = static_cast<const DT *>(a.draft) + row_offset(a, a.seq_d, b, 0);
    constexpr double LOG2E = 1.4426950408889634;
    int r = -1;                 // first rejection, once known
    double Lp_r = 0.0, Lq_r = 0.0;
    for (int j0 = 0; j0 <= g && (r < 0 || a.accept_prob); j0 += 64) {
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
                    atomicOr(a.ws.flags, (unsigned)SVIP_FLAG_BAD_TOKEN);
                    x = x < 0 ? 0 : a.geo.V - 1;
                }
                const double zp = (double)load_one<DT>(tgt + (long long)j * a.row_stride, x);
                const double zq = (double)load_one<DT>(drf + (long long)j * a.row_stride, x);
                const double p = exp2(zp * a.sc.c - Lp);
                const double q = exp2(zq * a.sc.c - Lq);
                reject = !(u * q < p);
                if (a.accept_prob) {
                    const double ratio = q > 0.0 ? p / q : (p > 0.0 ? 1.0 : 0.0);
                    a.accept_prob[(size_t)b * a.k + j] = (float)(ratio < 1.0 ? ratio : 1.0);
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
    if (lane == 0) {
        a.n_accepted[b] = r;
        SeqRec rec;
        rec.r = r;
        rec.resid = r < g ? 1 : 0;
        rec.Lp = Lp_r;
        rec.Lq = Lq_r;
        a.ws.rec[b] = rec;
    }
}

// ---- verify: residual / bonus sampling ------------------------------------------------------

// grid (sequences * slices): slice masses of the weights to sample from -- [0] residual
// max(0, p - q) at the rejected position, [1] target p of the row to sample.
template <typename DT>
__global__ __launch_bounds__(WG) void k_resid_mass(VerifyArgs a)
{
    __shared__ double lds[2 * NWAVE];
    const int b = blockIdx.x / a.geo_s.ns, s = blockIdx.x - b * a.geo_s.ns, tid = threadIdx.x;
    const SeqRec rec = a.ws.rec[b];
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
        unpack(rp[u], zp);
        unpack(rq[u], zq);
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

__global__ void k_zero(unsigned *p) { *p = 0u; }

// ---- host side -------------------------------------------------------------------------------

static int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return v && *v ? atoi(v) : dflt;
}

// Slices per row: enough workgroups to fill 256 CUs several times over, at most MAX_SLICES,
// and (want_one_batch) slices of at most LOCATE_UNROLL tiles so the sampler scans one batch.
static Geo make_geo(int V, int vec, long long rows, bool want_one_batch, int forced_ns)
{
    Geo g;
    g.V = V;
    const int nvec = (V + vec - 1) / vec;
    g.ntiles = (nvec + WG - 1) / WG;
    long long ns;
    if (want_one_batch) {
        ns = (2048 + rows - 1) / rows;                // aim at >= 2048 workgroups ...
        if (ns * 4 > g.ntiles) ns = g.ntiles / 4;     // ... of at least 4 tiles each
        const long long need = (g.ntiles + LOCATE_UNROLL - 1) / LOCATE_UNROLL;
        if (ns < need) ns = need;
        // large batches are bound by bandwidth, not by latency: longer slices of an odd number of
        // tiles (7) stream better than one-batch slices of 4, at the price of a two-batch search
        if (rows >= 512 && g.ntiles >= 14) ns = (g.ntiles + 6) / 7;
    } else {
        ns = (8192 + rows - 1) / rows;                // streaming passes: about 8192 workgroups ...
        if (ns * 8 > g.ntiles) ns = g.ntiles / 8;     // ... of at least 8 tiles each
    }
    if (forced_ns > 0) ns = forced_ns;
    if (ns > MAX_SLICES) ns = MAX_SLICES;
    if (ns > g.ntiles) ns = g.ntiles;
    if (ns < 1) ns = 1;
    g.tps = (g.ntiles + (int)ns - 1) / (int)ns;
    // an odd number of tiles per slice staggers the slices' start addresses over the memory
    // channels; slices that start a power of two apart measured up to 15 % slower
    if (!want_one_batch && g.tps > 1 && (g.tps & 1) == 0 && env_int("SVIP_EVEN_TPS", 0) == 0) g.tps += 1;
    g.ns = (g.ntiles + g.tps - 1) / g.tps;
    return g;
}

static Scale make_scale(float temperature)
{
    Scale s;
    s.inv_T = 1.0 / (double)temperature;
    s.c = 1.4426950408889634 * s.inv_T;
    s.c_hi = (float)s.c;
    s.c_lo = (float)(s.c - (double)s.c_hi);
    s.c_dn = s.c_hi;
    while ((double)s.c_dn >= s.c) s.c_dn = nextafterf(s.c_dn, 0.f);      // strictly below c: the remainder is > 0
    s.c_up = (float)(s.c - (double)s.c_dn);
    return s;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static svip_status check_launch()
{
    return hipGetLastError() == hipSuccess ? SVIP_OK : SVIP_ERR_HIP;
}

// benchmark timing hook (see svip_profile_begin)
struct Profile {
    hipEvent_t *ev = nullptr;   // pairs: start, stop
    int cap = 0, used = 0;
};
static Profile g_prof;

// ---- the calls behind the entry points ---------------------------------------------------------

svip_status draft_step_call(const DraftCall &c)
{
    if (!c.logits || (!c.greedy && !c.u_sample) || !c.token_out || !c.lse_out || !c.stop_out) return SVIP_ERR_NULL;
    if (c.dtype != SVIP_F32 && c.dtype != SVIP_BF16) return SVIP_ERR_DTYPE;
    if (c.B <= 0 || c.B > MAX_BATCH || c.V <= 0 || c.k_max < 1 || c.k_max > SVIP_MAX_K || c.step_j < 0 ||
        c.step_j >= c.k_max || c.io_stride < 1 || c.row_stride < c.V || (c.pos && c.pos_stride < c.V))
        return SVIP_ERR_SHAPE;
    const int vec = c.dtype == SVIP_BF16 ? 8 : 4;
    if (!aligned16(c.logits) || c.row_stride % vec != 0 || (c.pos && c.pos_stride % vec != 0)) return SVIP_ERR_ALIGN;
    if (!(c.temperature > 0.f) || !isfinite(c.temperature) || !(c.h >= 0.f)) return SVIP_ERR_PARAM;

    DraftArgs a;
    a.geo = make_geo(c.V, vec, c.B, true, env_int("SVIP_DRAFT_SLICES", 0));
    const size_t need = HEADER_BYTES + ws_rec_bytes(c.B) + ws_mass_bytes(c.B) +
                        (size_t)c.B * a.geo.ns * sizeof(Partial);
    if (!c.workspace || (reinterpret_cast<uintptr_t>(c.workspace) & 255u) || c.workspace_bytes < need)
        return SVIP_ERR_WORKSPACE;
    const Workspace w = carve(c.workspace, c.B);
    a.logits = c.logits;
    a.row_stride = c.row_stride;
    a.pos = c.pos;
    a.pos_stride = c.pos_stride;
    a.cap = c.cap;
    a.B = c.B;
    a.sc = make_scale(c.temperature);
    a.h = c.h;
    a.step_j = c.step_j;
    a.k_max = c.k_max;
    a.u = c.u_sample;
    a.stop_in = c.stop_in;
    a.token = c.token_out;
    a.entropy = c.entropy_out;
    a.q_tok = c.q_tok_out;
    a.lse = c.lse_out;
    a.stop = c.stop_out;
    a.draft_len = c.draft_len_out;
    a.io_stride = c.io_stride;
    a.part = w.part;
    hipStream_t st = static_cast<hipStream_t>(c.stream);
    const dim3 grid((unsigned)a.geo.ns * (unsigned)c.B);
    if (c.greedy) {
        if (c.dtype == SVIP_BF16) hipLaunchKernelGGL((k_draft_stats<bf16, true>), grid, dim3(WG), 0, st, a);
        else hipLaunchKernelGGL((k_draft_stats<float, true>), grid, dim3(WG), 0, st, a);
        hipLaunchKernelGGL(k_draft_finish_greedy, dim3(c.B), dim3(64), 0, st, a);
    } else if (c.dtype == SVIP_BF16) {
        hipLaunchKernelGGL((k_draft_stats<bf16, false>), grid, dim3(WG), 0, st, a);
        hipLaunchKernelGGL(k_draft_finish<bf16>, dim3(c.B), dim3(WG), 0, st, a);
    } else {
        hipLaunchKernelGGL((k_draft_stats<float, false>), grid, dim3(WG), 0, st, a);
        hipLaunchKernelGGL(k_draft_finish<float>, dim3(c.B), dim3(WG), 0, st, a);
    }
    return check_launch();
}

static svip_status verify_greedy_call(const VerifyCall &c)
{
    if (!c.target || !c.draft_tokens || !c.draft_len || !c.n_accepted_out || !c.next_token_out) return SVIP_ERR_NULL;
    if (c.dtype != SVIP_F32 && c.dtype != SVIP_BF16) return SVIP_ERR_DTYPE;
    if (c.B <= 0 || c.B > MAX_BATCH || c.V <= 0 || c.k_max < 1 || c.k_max > SVIP_MAX_K || c.row_stride < c.V ||
        c.seq_stride_t < (long long)c.k_max * c.row_stride + c.V)
        return SVIP_ERR_SHAPE;
    const long long rows = (long long)c.B * (c.k_max + 1);
    if (rows * MAX_SLICES > 0x7FFFFFFFLL) return SVIP_ERR_SHAPE;
    const int vec = c.dtype == SVIP_BF16 ? 8 : 4;
    if (!aligned16(c.target) || c.row_stride % vec != 0 || c.seq_stride_t % vec != 0) return SVIP_ERR_ALIGN;
    GreedyArgs a;
    a.geo = make_geo(c.V, vec, rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    const size_t need = HEADER_BYTES + ws_rec_bytes(c.B) + ws_mass_bytes(c.B) +
                        (size_t)rows * a.geo.ns * sizeof(unsigned long long);
    if (!c.workspace || (reinterpret_cast<uintptr_t>(c.workspace) & 255u) || c.workspace_bytes < need)
        return SVIP_ERR_WORKSPACE;
    const Workspace w = carve(c.workspace, c.B);
    a.target = c.target;
    a.seq_t = c.seq_stride_t;
    a.row_stride = c.row_stride;
    a.pos = c.pos;
    a.B = c.B;
    a.k = c.k_max;
    a.tokens = c.draft_tokens;
    a.draft_len = c.draft_len;
    a.n_accepted = c.n_accepted_out;
    a.next_token = c.next_token_out;
    a.keys = reinterpret_cast<unsigned long long *>(w.part);
    a.flags = w.flags;
    hipStream_t st = static_cast<hipStream_t>(c.stream);
    const dim3 grid((unsigned)(rows * a.geo.ns));
    if (c.dtype == SVIP_BF16) hipLaunchKernelGGL(k_argmax<bf16>, grid, dim3(WG), 0, st, a);
    else hipLaunchKernelGGL(k_argmax<float>, grid, dim3(WG), 0, st, a);
    hipLaunchKernelGGL(k_accept_greedy, dim3(c.B), dim3(64), 0, st, a);
    return check_launch();
}

svip_status verify_call(const VerifyCall &c)
{
    if (c.greedy) return verify_greedy_call(c);
    if (!c.target || !c.draft || !c.draft_tokens || !c.draft_len || !c.u_accept || !c.u_resample ||
        !c.n_accepted_out || !c.next_token_out)
        return SVIP_ERR_NULL;
    if (c.dtype != SVIP_F32 && c.dtype != SVIP_BF16) return SVIP_ERR_DTYPE;
    if (c.B <= 0 || c.B > MAX_BATCH || c.V <= 0 || c.k_max < 1 || c.k_max > SVIP_MAX_K || c.row_stride < c.V ||
        c.seq_stride_t < (long long)c.k_max * c.row_stride + c.V ||
        c.seq_stride_d < (long long)(c.k_max - 1) * c.row_stride + c.V)
        return SVIP_ERR_SHAPE;
    const int kd = c.draft_lse ? 0 : c.k_max;
    const long long stat_rows = (long long)c.B * (kd + c.k_max + 1);
    if (stat_rows * MAX_SLICES > 0x7FFFFFFFLL) return SVIP_ERR_SHAPE;          // workgroups of the statistics pass
    const int vec = c.dtype == SVIP_BF16 ? 8 : 4;
    if (!aligned16(c.target) || !aligned16(c.draft) || c.row_stride % vec != 0 || c.seq_stride_t % vec != 0 ||
        c.seq_stride_d % vec != 0)
        return SVIP_ERR_ALIGN;
    if (!(c.temperature > 0.f) || !isfinite(c.temperature)) return SVIP_ERR_PARAM;

    VerifyArgs a;
    a.geo = make_geo(c.V, vec, stat_rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    a.geo_s = make_geo(c.V, vec, c.B, true, env_int("SVIP_SAMPLE_SLICES", 0));
    const size_t need = HEADER_BYTES + ws_rec_bytes(c.B) + ws_mass_bytes(c.B) +
                        (size_t)stat_rows * a.geo.ns * sizeof(Partial);
    if (!c.workspace || (reinterpret_cast<uintptr_t>(c.workspace) & 255u) || c.workspace_bytes < need)
        return SVIP_ERR_WORKSPACE;
    a.target = c.target;
    a.draft = c.draft;
    a.seq_t = c.seq_stride_t;
    a.seq_d = c.seq_stride_d;
    a.row_stride = c.row_stride;
    a.pos = c.pos;
    a.B = c.B;
    a.k = c.k_max;
    a.kd = kd;
    a.bonus = 1;
    a.sc = make_scale(c.temperature);
    a.tokens = c.draft_tokens;
    a.draft_len = c.draft_len;
    a.draft_lse = c.draft_lse;
    a.u_accept = c.u_accept;
    a.u_resample = c.u_resample;
    a.n_accepted = c.n_accepted_out;
    a.next_token = c.next_token_out;
    a.accept_prob = c.accept_prob_out;
    a.ws = carve(c.workspace, c.B);
    hipStream_t st = static_cast<hipStream_t>(c.stream);
    const dim3 g_stats((unsigned)(stat_rows * a.geo.ns)), g_mass((unsigned)a.geo_s.ns * (unsigned)c.B);
    const bool timed = g_prof.ev && g_prof.used < g_prof.cap;
    if (timed) (void)hipEventRecord(g_prof.ev[2 * g_prof.used], st);
    if (c.dtype == SVIP_BF16) hipLaunchKernelGGL(k_verify_stats<bf16>, g_stats, dim3(WG), 0, st, a);
    else hipLaunchKernelGGL(k_verify_stats<float>, g_stats, dim3(WG), 0, st, a);
    if (timed) {
        (void)hipEventRecord(g_prof.ev[2 * g_prof.used + 1], st);
        ++g_prof.used;
    }
    if (c.dtype == SVIP_BF16) {
        hipLaunchKernelGGL(k_accept<bf16>, dim3(c.B), dim3(64), 0, st, a);
        hipLaunchKernelGGL(k_resid_mass<bf16>, g_mass, dim3(WG), 0, st, a);
        hipLaunchKernelGGL(k_resid_finish<bf16>, dim3(c.B), dim3(WG), 0, st, a);
    } else {
        hipLaunchKernelGGL(k_accept<float>, dim3(c.B), dim3(64), 0, st, a);
        hipLaunchKernelGGL(k_resid_mass<float>, g_mass, dim3(WG), 0, st, a);
        hipLaunchKernelGGL(k_resid_finish<float>, dim3(c.B), dim3(WG), 0, st, a);
    }
    return check_launch();
}

}  // namespace svip

using namespace svip;

extern "C" {

const char *svip_status_string(int status)
{
    switch (status) {
        case SVIP_OK: return "SVIP_OK";
        case SVIP_ERR_NULL: return "SVIP_ERR_NULL: a required pointer is NULL";
        case SVIP_ERR_SHAPE: return "SVIP_ERR_SHAPE: size, position or stride out of range";
        case SVIP_ERR_DTYPE: return "SVIP_ERR_DTYPE: unknown logits dtype";
        case SVIP_ERR_ALIGN: return "SVIP_ERR_ALIGN: pointer or stride not 16-byte aligned";
        case SVIP_ERR_WORKSPACE: return "SVIP_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case SVIP_ERR_PARAM: return "SVIP_ERR_PARAM: temperature, threshold or constant out of range";
        case SVIP_ERR_HIP: return "SVIP_ERR_HIP: HIP runtime error";
        default: return "SVIP: unknown status";
    }
}

size_t svip_workspace_bytes(int B, int k_max, int V)
{
    if (B <= 0 || B > MAX_BATCH || k_max < 1 || k_max > SVIP_MAX_K || V <= 0) return 0;
    // slice statistics: the draft step slices its B rows finely (at most MAX_SLICES each); the
    // streaming passes (statistics of verify, argmax, diagnostics) have up to B (2 k + 1) rows, of
    // which make_geo cuts at most ceil(8192 / rows) slices each: rows + 8192 slices at most
    const size_t vrows = (size_t)B * (2 * (size_t)k_max + 1);
    size_t parts = (size_t)B * MAX_SLICES;
    if (vrows + 8192 > parts) parts = vrows + 8192;
    // diagnostics: two logsumexps per position and three sums per slice of its second pass
    const size_t pos = (size_t)B * (size_t)k_max;
    return HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B) + align256(parts * sizeof(Partial)) +
           align256(pos * 2 * sizeof(double)) + align256((pos + 8192) * 3 * sizeof(double));
}

svip_status svip_workspace_reset(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace || workspace_bytes < HEADER_BYTES || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return SVIP_ERR_WORKSPACE;
    hipLaunchKernelGGL(k_zero, dim3(1), dim3(1), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<unsigned *>(workspace));
    return check_launch();
}

svip_status svip_workspace_flags(const void *workspace, void *hip_stream, unsigned *flags_host)
{
    if (!workspace) return SVIP_ERR_WORKSPACE;
    if (!flags_host) return SVIP_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(flags_host, workspace, sizeof(unsigned), hipMemcpyDeviceToHost, st) != hipSuccess)
        return SVIP_ERR_HIP;
    return hipStreamSynchronize(st) == hipSuccess ? SVIP_OK : SVIP_ERR_HIP;
}

svip_status svip_draft_step(const void *draft_logits, svip_dtype dtype, int B, int V, long long row_stride,
                            float temperature, float h, int step_j, int k_max, const float *u_sample,
                            const unsigned char *stop_in, int *token_out, float *entropy_out,
                            float *q_tok_out, double *lse_out, unsigned char *stop_out,
                            int *draft_len_out, long long io_stride, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    const DraftCall c{false, draft_logits, dtype, B, V, row_stride, nullptr, 0, nullptr, temperature, h, step_j,
                      k_max, u_sample, stop_in, token_out, entropy_out, q_tok_out, lse_out, stop_out,
                      draft_len_out, io_stride, workspace, workspace_bytes, hip_stream};
    return draft_step_call(c);
}

svip_status svip_draft_step_greedy(const void *draft_logits, svip_dtype dtype, int B, int V, long long row_stride,
                                   float temperature, float h, int step_j, int k_max,
                                   const unsigned char *stop_in, int *token_out, float *entropy_out,
                                   float *q_tok_out, double *lse_out, unsigned char *stop_out,
                                   int *draft_len_out, long long io_stride, void *workspace,
                                   size_t workspace_bytes, void *hip_stream)
{
    const DraftCall c{true, draft_logits, dtype, B, V, row_stride, nullptr, 0, nullptr, temperature, h, step_j,
                      k_max, nullptr, stop_in, token_out, entropy_out, q_tok_out, lse_out, stop_out,
                      draft_len_out, io_stride, workspace, workspace_bytes, hip_stream};
    return draft_step_call(c);
}

svip_status svip_verify_greedy(const void *target_logits, svip_dtype dtype, int B, int k_max, int V,
                               long long seq_stride_t, long long row_stride, const int *draft_tokens,
                               const int *draft_len, int *n_accepted_out, int *next_token_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const VerifyCall c{true, target_logits, nullptr, dtype, B, k_max, V, seq_stride_t, 0, row_stride, nullptr, 1.f,
                       draft_tokens, draft_len, nullptr, nullptr, nullptr, n_accepted_out, next_token_out,
                       nullptr, workspace, workspace_bytes, hip_stream};
    return verify_call(c);
}

svip_status svip_verify(const void *target_logits, const void *draft_logits, svip_dtype dtype, int B,
                        int k_max, int V, long long seq_stride_t, long long seq_stride_d,
                        long long row_stride, float temperature, const int *draft_tokens,
                        const int *draft_len, const double *draft_lse, const float *u_accept,
                        const float *u_resample, int *n_accepted_out, int *next_token_out,
                        float *accept_prob_out, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    const VerifyCall c{false, target_logits, draft_logits, dtype, B, k_max, V, seq_stride_t, seq_stride_d,
                       row_stride, nullptr, temperature, draft_tokens, draft_len, draft_lse, u_accept,
                       u_resample, n_accepted_out, next_token_out, accept_prob_out, workspace,
                       workspace_bytes, hip_stream};
    return verify_call(c);
}

svip_status svip_pair_stats(const void *target_logits, const void *draft_logits, svip_dtype dtype, int B,
                            int k_max, int V, long long seq_stride_t, long long seq_stride_d,
                            long long row_stride, float temperature, const int *draft_len,
                            const double *draft_lse, float c, float *stats_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    if (!target_logits || !draft_logits || !draft_len || !stats_out) return SVIP_ERR_NULL;
    if (dtype != SVIP_F32 && dtype != SVIP_BF16) return SVIP_ERR_DTYPE;
    if (B <= 0 || B > MAX_BATCH || V <= 0 || k_max < 1 || k_max > SVIP_MAX_K || row_stride < V ||
        seq_stride_t < (long long)(k_max - 1) * row_stride + V || seq_stride_d < (long long)(k_max - 1) * row_stride + V)
        return SVIP_ERR_SHAPE;
    const int kd = draft_lse ? 0 : k_max;
    const long long stat_rows = (long long)B * (kd + k_max + 1), pos = (long long)B * k_max;
    if (stat_rows * MAX_SLICES > 0x7FFFFFFFLL) return SVIP_ERR_SHAPE;
    const int vec = dtype == SVIP_BF16 ? 8 : 4;
    if (!aligned16(target_logits) || !aligned16(draft_logits) || row_stride % vec != 0 ||
        seq_stride_t % vec != 0 || seq_stride_d % vec != 0)
        return SVIP_ERR_ALIGN;
    if (!(temperature > 0.f) || !isfinite(temperature) || !(c >= 0.f) || !isfinite(c)) return SVIP_ERR_PARAM;

    PairArgs a;
    a.v.geo = make_geo(V, vec, stat_rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    a.v.geo_s = a.v.geo;
    a.geo2 = make_geo(V, vec, pos, false, env_int("SVIP_PAIR_SLICES", 0));
    const size_t part_bytes = align256((size_t)stat_rows * a.v.geo.ns * sizeof(Partial));
    const size_t L_bytes = align256((size_t)pos * 2 * sizeof(double));
    const size_t need = HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B) + part_bytes + L_bytes +
                        (size_t)pos * a.geo2.ns * 3 * sizeof(double);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
        return SVIP_ERR_WORKSPACE;
    a.v.target = target_logits;
    a.v.draft = draft_logits;
    a.v.seq_t = seq_stride_t;
    a.v.seq_d = seq_stride_d;
    a.v.row_stride = row_stride;
    a.v.pos = nullptr;
    a.v.B = B;
    a.v.k = k_max;
    a.v.kd = kd;
    a.v.bonus = 0;
    a.v.sc = make_scale(temperature);
    a.v.tokens = nullptr;
    a.v.draft_len = draft_len;
    a.v.draft_lse = draft_lse;
    a.v.u_accept = nullptr;
    a.v.u_resample = nullptr;
    a.v.n_accepted = nullptr;
    a.v.next_token = nullptr;
    a.v.accept_prob = nullptr;
    a.v.ws = carve(workspace, B);
    char *after = reinterpret_cast<char *>(a.v.ws.part) + part_bytes;
    a.L = reinterpret_cast<double *>(after);
    a.sums = reinterpret_cast<double *>(after + L_bytes);
    a.c = c;
    a.out = stats_out;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 g_stats((unsigned)(stat_rows * a.v.geo.ns)), g_pos((unsigned)((pos + 63) / 64)),
        g_sums((unsigned)(pos * a.geo2.ns));
    if (dtype == SVIP_BF16) hipLaunchKernelGGL(k_verify_stats<bf16>, g_stats, dim3(WG), 0, st, a.v);
    else hipLaunchKernelGGL(k_verify_stats<float>, g_stats, dim3(WG), 0, st, a.v);
    hipLaunchKernelGGL(k_pair_L, g_pos, dim3(64), 0, st, a);
    if (dtype == SVIP_BF16) hipLaunchKernelGGL(k_pair_sums<bf16>, g_sums, dim3(WG), 0, st, a);
    else hipLaunchKernelGGL(k_pair_sums<float>, g_sums, dim3(WG), 0, st, a);
    hipLaunchKernelGGL(k_pair_finish, g_pos, dim3(64), 0, st, a);
    return check_launch();
}

svip_status svip_profile_begin(int max_samples)
{
    if (max_samples < 1 || g_prof.ev) return SVIP_ERR_PARAM;
    g_prof.ev = static_cast<hipEvent_t *>(malloc(sizeof(hipEvent_t) * 2 * (size_t)max_samples));
    if (!g_prof.ev) return SVIP_ERR_HIP;
    for (int i = 0; i < 2 * max_samples; ++i) {
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
            free(g_prof.ev);
            g_prof = Profile();
            return SVIP_ERR_HIP;
        }
    }
    g_prof.cap = max_samples;
    g_prof.used = 0;
    return SVIP_OK;
}

svip_status svip_profile_end(double *total_ms_host, int *samples_host)
{
    if (!total_ms_host || !samples_host) return SVIP_ERR_NULL;
    if (!g_prof.ev) return SVIP_ERR_PARAM;
    double total = 0.0;
    svip_status rc = SVIP_OK;
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess)
            rc = SVIP_ERR_HIP;
        total += ms;
    }
    *total_ms_host = total;
    *samples_host = g_prof.used;
    for (int i = 0; i < 2 * g_prof.cap; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    free(g_prof.ev);
    g_prof = Profile();
    return rc;
}

}  // extern "C"
