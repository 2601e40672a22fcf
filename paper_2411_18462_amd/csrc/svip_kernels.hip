// SVIP hot path for MI355X (gfx950): launch code and the C ABI declared in include/svip.h; the kernels
// live in draft_kernels.h, verify_kernels.h, greedy_kernels.h and pair_kernels.h.
//
// svip_draft_step  =  k_draft_stats    grid (slices, rows)       per-slice (m, S, t) of every active row
//                     k_draft_finish   grid (rows)               merge, entropy, stop test, inverse CDF
//   (greedy)          k_draft_stats<ARG> + k_draft_finish_greedy     token = first maximum, no search
// svip_verify      =  k_verify_stats   grid (slices, stat rows)  per-slice (reference, sum) of every needed row
//                     k_accept         grid (sequences), 1 wave  p/q test, ballot scan for the first rejection
//                                      (up to 16 sequences: done by the first wave of every k_resid_mass workgroup)
//                     k_resid_mass     grid (slices, sequences)  slice masses of the residual / bonus row
//                     k_resid_finish   grid (sequences)          inverse CDF of the residual / bonus row
// svip_verify_greedy = k_argmax        grid (slices, target rows) first maximum per slice, no exponentials
//                     k_accept_greedy  grid (sequences), 1 wave  argmax p == x test, ballot, correction = argmax p
//
// svip_pair_stats  =  k_verify_stats   (rows j < draft_len of both models), k_pair_L (logsumexps),
//                     k_pair_sums      grid (slices, positions)  sum min(p,q), sum q log(q/p), sum q log q
//                     k_pair_finish    one thread per position   beta, KL, cross entropy, the bounds
//
// svip_warp_logits =  k_warp           grid (rows), 1024 threads  top-k / top-p thresholds by radix select, masked copy
//
// The passes are bound by HBM reads of the logits; there is no dense contraction, hence no MFMA.
// Kernels of one call are ordered by the stream only (no spinning, no device-side waits), and
// each small kernel issues all of its independent loads before the first dependent one, because
// at small batches a step is bound by round trips to memory rather than by bandwidth.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/svip.h"
#include "row_math.h"
#include "svip_internal.h"

#include "kernel_args.h"
#include "sample_weights.h"
#include "draft_kernels.h"
#include "greedy_kernels.h"
#include "verify_kernels.h"
#include "pair_kernels.h"
#include "warp_kernels.h"

namespace svip {

__global__ void k_zero(unsigned *p) { *p = 0u; }

// ---- host side -------------------------------------------------------------------------------

static int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return v && *v ? atoi(v) : dflt;
}

// Slices per row: enough workgroups to fill 256 CUs several times over, at most MAX_SLICES,
// and (want_one_batch) slices of at most LOCATE_UNROLL tiles so the sampler scans one batch.
static Geo make_geo(int V, int vec, long long rows, bool want_one_batch, int forced_ns, int min_tiles = 4)
{
    Geo g;
    g.V = V;
    const int nvec = (V + vec - 1) / vec;
    g.ntiles = (nvec + WG - 1) / WG;
    long long ns;
    if (want_one_batch) {
        // aim at 2048 workgroups of at least min_tiles tiles each; where that leaves fewer than about
        // 900 workgroups (few rows, or short rows) shorter slices win, down to a single tile (one row
        // of 128K bf16 logits: 6.5 us a step against 7.5 us; 64 rows of 32000: 8.5 against 10.2)
        const long long want = (2048 + rows - 1) / rows;
        const long long floor_wg = env_int("SVIP_MIN_WORKGROUPS", 900);
        for (;;) {
            long long cap = g.ntiles / min_tiles;
            if (cap < 1) cap = 1;
            ns = want < cap ? want : cap;
            if (ns * rows >= floor_wg || min_tiles == 1) break;
            min_tiles /= 2;
        }
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

static bool dtype_ok(svip_dtype d) { return d == SVIP_F32 || d == SVIP_BF16 || d == SVIP_F16; }
static int vec_of(svip_dtype d) { return d == SVIP_F32 ? 4 : 8; }       // logits per 16-byte vector

// Calls f with a value of the storage type that d names (f is a generic lambda).
template <typename F>
static void by_dtype(svip_dtype d, F f)
{
    if (d == SVIP_BF16) f(bf16{});
    else if (d == SVIP_F16) f(f16{});
    else f(float{});
}

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

// ---- workspace each call needs (its own geometry; svip_workspace_bytes bounds them all) -------

static size_t need_draft(int B, int V, int vec)
{
    const Geo g = make_geo(V, vec, B, true, env_int("SVIP_DRAFT_SLICES", 0));
    return HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B) + (size_t)B * g.ns * sizeof(Partial);
}
static size_t need_verify_greedy(int B, int k, int V, int vec)
{
    const long long rows = (long long)B * (k + 1);
    const Geo g = make_geo(V, vec, rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    return HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B) + (size_t)rows * g.ns * sizeof(unsigned long long);
}
static size_t need_verify(int B, int k, int V, int vec, bool recompute_lse)
{
    const long long stat_rows = (long long)B * ((recompute_lse ? k : 0) + k + 1);
    const Geo g = make_geo(V, vec, stat_rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    return HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B) + (size_t)stat_rows * g.ns * sizeof(Partial);
}
static size_t need_pair(int B, int k, int V, int vec, bool recompute_lse, size_t *part_bytes, size_t *L_bytes)
{
    const long long stat_rows = (long long)B * ((recompute_lse ? k : 0) + k + 1), pos = (long long)B * k;
    const Geo g = make_geo(V, vec, stat_rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    const Geo g2 = make_geo(V, vec, pos, false, env_int("SVIP_PAIR_SLICES", 0));
    const size_t pb = align256((size_t)stat_rows * g.ns * sizeof(Partial));
    const size_t lb = align256((size_t)pos * 2 * sizeof(double));
    if (part_bytes) *part_bytes = pb;
    if (L_bytes) *L_bytes = lb;
    return HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B) + pb + lb + (size_t)pos * g2.ns * 3 * sizeof(double);
}

// ---- the calls behind the entry points ---------------------------------------------------------

svip_status draft_step_call(const DraftCall &c)
{
    if (!c.logits || (!c.greedy && !c.u_sample) || !c.token_out || !c.lse_out || !c.stop_out) return SVIP_ERR_NULL;
    if (!dtype_ok(c.dtype)) return SVIP_ERR_DTYPE;
    if (c.B <= 0 || c.B > MAX_BATCH || c.V <= 0 || c.k_max < 1 || c.k_max > SVIP_MAX_K || c.step_j < 0 ||
        c.step_j >= c.k_max || c.io_stride < 1 || c.row_stride < c.V || (c.pos && c.pos_stride < c.V))
        return SVIP_ERR_SHAPE;
    const int vec = vec_of(c.dtype);
    if (!aligned16(c.logits) || c.row_stride % vec != 0 || (c.pos && c.pos_stride % vec != 0)) return SVIP_ERR_ALIGN;
    if (!(c.temperature > 0.f) || !isfinite(c.temperature) || !(c.h >= 0.f)) return SVIP_ERR_PARAM;

    DraftArgs a;
    a.geo = make_geo(c.V, vec, c.B, true, env_int("SVIP_DRAFT_SLICES", 0));
    const size_t need = need_draft(c.B, c.V, vec);
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
    by_dtype(c.dtype, [&](auto tag) {
        using DT = decltype(tag);
        if (c.greedy) {
            hipLaunchKernelGGL((k_draft_stats<DT, true>), grid, dim3(WG), 0, st, a);
            hipLaunchKernelGGL(k_draft_finish_greedy, dim3(c.B), dim3(64), 0, st, a);
        } else {
            hipLaunchKernelGGL((k_draft_stats<DT, false>), grid, dim3(WG), 0, st, a);
            hipLaunchKernelGGL(k_draft_finish<DT>, dim3(c.B), dim3(WG), 0, st, a);
        }
    });
    return check_launch();
}

static svip_status verify_greedy_call(const VerifyCall &c)
{
    if (!c.target || !c.draft_tokens || !c.draft_len || !c.n_accepted_out || !c.next_token_out) return SVIP_ERR_NULL;
    if (!dtype_ok(c.dtype)) return SVIP_ERR_DTYPE;
    if (c.B <= 0 || c.B > MAX_BATCH || c.V <= 0 || c.k_max < 1 || c.k_max > SVIP_MAX_K || c.row_stride < c.V ||
        c.seq_stride_t < (long long)c.k_max * c.row_stride + c.V)
        return SVIP_ERR_SHAPE;
    const long long rows = (long long)c.B * (c.k_max + 1);
    if (rows * MAX_SLICES > 0x7FFFFFFFLL) return SVIP_ERR_SHAPE;
    const int vec = vec_of(c.dtype);
    if (!aligned16(c.target) || c.row_stride % vec != 0 || c.seq_stride_t % vec != 0) return SVIP_ERR_ALIGN;
    GreedyArgs a;
    a.geo = make_geo(c.V, vec, rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    const size_t need = need_verify_greedy(c.B, c.k_max, c.V, vec);
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
    by_dtype(c.dtype, [&](auto tag) { hipLaunchKernelGGL(k_argmax<decltype(tag)>, grid, dim3(WG), 0, st, a); });
    hipLaunchKernelGGL(k_accept_greedy, dim3(c.B), dim3(64), 0, st, a);
    return check_launch();
}

svip_status verify_call(const VerifyCall &c)
{
    if (c.greedy) return verify_greedy_call(c);
    if (!c.target || !c.draft || !c.draft_tokens || !c.draft_len || !c.u_accept || !c.u_resample ||
        !c.n_accepted_out || !c.next_token_out)
        return SVIP_ERR_NULL;
    if (!dtype_ok(c.dtype)) return SVIP_ERR_DTYPE;
    if (c.B <= 0 || c.B > MAX_BATCH || c.V <= 0 || c.k_max < 1 || c.k_max > SVIP_MAX_K || c.row_stride < c.V ||
        c.seq_stride_t < (long long)c.k_max * c.row_stride + c.V ||
        c.seq_stride_d < (long long)(c.k_max - 1) * c.row_stride + c.V)
        return SVIP_ERR_SHAPE;
    const int kd = c.draft_lse ? 0 : c.k_max;
    const long long stat_rows = (long long)c.B * (kd + c.k_max + 1);
    if (stat_rows * MAX_SLICES > 0x7FFFFFFFLL) return SVIP_ERR_SHAPE;          // workgroups of the statistics pass
    const int vec = vec_of(c.dtype);
    if (!aligned16(c.target) || !aligned16(c.draft) || c.row_stride % vec != 0 || c.seq_stride_t % vec != 0 ||
        c.seq_stride_d % vec != 0)
        return SVIP_ERR_ALIGN;
    if (!(c.temperature > 0.f) || !isfinite(c.temperature)) return SVIP_ERR_PARAM;

    VerifyArgs a;
    a.geo = make_geo(c.V, vec, stat_rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    // the residual pass reads two rows per slice: half as many tiles per slice as the draft step
    a.geo_s = make_geo(c.V, vec, c.B, true, env_int("SVIP_SAMPLE_SLICES", 0), 2);
    const size_t need = need_verify(c.B, c.k_max, c.V, vec, kd != 0);
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
    if (timed) {        // the launch itself carries the two events: they take the kernel's own start and end
        hipEvent_t e0 = g_prof.ev[2 * g_prof.used], e1 = g_prof.ev[2 * g_prof.used + 1];
        by_dtype(c.dtype, [&](auto tag) {
            hipExtLaunchKernelGGL(k_verify_stats<decltype(tag)>, g_stats, dim3(WG), 0, st, e0, e1, 0, a);
        });
        ++g_prof.used;
    } else {
        by_dtype(c.dtype, [&](auto tag) { hipLaunchKernelGGL(k_verify_stats<decltype(tag)>, g_stats, dim3(WG), 0, st, a); });
    }
    by_dtype(c.dtype, [&](auto tag) {
        using DT = decltype(tag);
        // few sequences: every workgroup of the mass pass repeats the acceptance test instead of waiting for a
        // kernel of its own (about 1 us less per call up to 16 sequences, 2 us more at 64)
        const int in_mass = env_int("SVIP_ACCEPT_IN_MASS", -1);
        if (in_mass < 0 ? c.B <= 16 : in_mass != 0) {
            hipLaunchKernelGGL((k_resid_mass<DT, true>), g_mass, dim3(WG), 0, st, a);
        } else {
            hipLaunchKernelGGL(k_accept<DT>, dim3(c.B), dim3(64), 0, st, a);
            hipLaunchKernelGGL((k_resid_mass<DT, false>), g_mass, dim3(WG), 0, st, a);
        }
        hipLaunchKernelGGL(k_resid_finish<DT>, dim3(c.B), dim3(WG), 0, st, a);
    });
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

size_t svip_workspace_needed(int call, svip_dtype dtype, int B, int k_max, int V)
{
    if (!dtype_ok(dtype) || B <= 0 || B > MAX_BATCH || k_max < 1 || k_max > SVIP_MAX_K || V <= 0) return 0;
    const int vec = vec_of(dtype);
    switch (call) {
        case SVIP_CALL_DRAFT_STEP: return need_draft(B, V, vec);
        case SVIP_CALL_VERIFY: return need_verify(B, k_max, V, vec, false);
        case SVIP_CALL_VERIFY_RECOMPUTE: return need_verify(B, k_max, V, vec, true);
        case SVIP_CALL_VERIFY_GREEDY: return need_verify_greedy(B, k_max, V, vec);
        case SVIP_CALL_PAIR_STATS: return need_pair(B, k_max, V, vec, false, nullptr, nullptr);
        case SVIP_CALL_PAIR_STATS_RECOMPUTE: return need_pair(B, k_max, V, vec, true, nullptr, nullptr);
        default: return 0;
    }
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

svip_status svip_warp_logits(const void *logits_in, void *logits_out, svip_dtype dtype, int B, int k_max, int V,
                             long long seq_stride, long long row_stride, float temperature, int top_k,
                             double top_p, int *kept_out, void *hip_stream)
{
    if (!logits_in || !logits_out) return SVIP_ERR_NULL;
    if (!dtype_ok(dtype)) return SVIP_ERR_DTYPE;
    if (B <= 0 || B > MAX_BATCH || V <= 0 || k_max < 1 || (long long)B * k_max > 0x7FFFFFFFLL || row_stride < V ||
        seq_stride < (long long)(k_max - 1) * row_stride + V)
        return SVIP_ERR_SHAPE;
    const int vec = vec_of(dtype);
    if (!aligned16(logits_in) || !aligned16(logits_out) || row_stride % vec != 0 || seq_stride % vec != 0)
        return SVIP_ERR_ALIGN;
    if (!(temperature > 0.f) || !isfinite(temperature) || top_k < 0 || !(top_p > 0.0)) return SVIP_ERR_PARAM;

    WarpArgs a;
    a.in = logits_in;
    a.out = logits_out;
    a.seq_stride = seq_stride;
    a.row_stride = row_stride;
    a.k = k_max;
    a.V = V;
    a.sc = make_scale(temperature);
    a.top_k = top_k;
    a.top_p = top_p;
    // weights <= 1 in units of 2^-shift: V of them must stay below 2^62
    int lg = 0;
    while ((1ll << lg) < (long long)V) ++lg;
    const int shift = 62 - lg < 44 ? 62 - lg : 44;
    a.fix_scale = ldexpf(1.f, shift);
    a.kept = kept_out;
    a.no_shortcut = env_int("SVIP_WARP_NO_SHORTCUT", 0);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)((long long)B * k_max));
    by_dtype(dtype, [&](auto tag) { hipLaunchKernelGGL(k_warp<decltype(tag)>, grid, dim3(WARP_WG), 0, st, a); });
    return check_launch();
}

svip_status svip_pair_stats(const void *target_logits, const void *draft_logits, svip_dtype dtype, int B,
                            int k_max, int V, long long seq_stride_t, long long seq_stride_d,
                            long long row_stride, float temperature, const int *draft_len,
                            const double *draft_lse, float c, float *stats_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    if (!target_logits || !draft_logits || !draft_len || !stats_out) return SVIP_ERR_NULL;
    if (!dtype_ok(dtype)) return SVIP_ERR_DTYPE;
    if (B <= 0 || B > MAX_BATCH || V <= 0 || k_max < 1 || k_max > SVIP_MAX_K || row_stride < V ||
        seq_stride_t < (long long)(k_max - 1) * row_stride + V || seq_stride_d < (long long)(k_max - 1) * row_stride + V)
        return SVIP_ERR_SHAPE;
    const int kd = draft_lse ? 0 : k_max;
    const long long stat_rows = (long long)B * (kd + k_max + 1), pos = (long long)B * k_max;
    if (stat_rows * MAX_SLICES > 0x7FFFFFFFLL) return SVIP_ERR_SHAPE;
    const int vec = vec_of(dtype);
    if (!aligned16(target_logits) || !aligned16(draft_logits) || row_stride % vec != 0 ||
        seq_stride_t % vec != 0 || seq_stride_d % vec != 0)
        return SVIP_ERR_ALIGN;
    if (!(temperature > 0.f) || !isfinite(temperature) || !(c >= 0.f) || !isfinite(c)) return SVIP_ERR_PARAM;

    PairArgs a;
    a.v.geo = make_geo(V, vec, stat_rows, false, env_int("SVIP_VERIFY_SLICES", 0));
    a.v.geo_s = a.v.geo;
    a.geo2 = make_geo(V, vec, pos, false, env_int("SVIP_PAIR_SLICES", 0));
    size_t part_bytes, L_bytes;
    const size_t need = need_pair(B, k_max, V, vec, kd != 0, &part_bytes, &L_bytes);
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
    by_dtype(dtype, [&](auto tag) { hipLaunchKernelGGL(k_verify_stats<decltype(tag)>, g_stats, dim3(WG), 0, st, a.v); });
    hipLaunchKernelGGL(k_pair_L, g_pos, dim3(64), 0, st, a);
    by_dtype(dtype, [&](auto tag) { hipLaunchKernelGGL(k_pair_sums<decltype(tag)>, g_sums, dim3(WG), 0, st, a); });
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
