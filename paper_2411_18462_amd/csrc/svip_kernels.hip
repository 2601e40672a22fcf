// SVIP hot path for MI355X (gfx950): launch code and the C ABI declared in include/svip.h; the kernels
// live in draft_kernels.h, verify_kernels.h, greedy_kernels.h, pair_kernels.h and warp_kernels.h.
//
// svip_draft_step  =  k_draft_stats    grid (rows * records / 4) one wave per record: (m, S, t) of a tile of a row
//                     k_draft_finish   grid (rows)               merge of the records: entropy, stop test, inverse
//                                      CDF inside the one record that holds the draw (greedy: the first maximum)
// svip_verify      =  k_verify_stats   grid (stat rows * slices) per-slice (reference, sum) of every needed row
//                     k_accept         grid (sequences), 1 wave  p/q tests, ballot scan for the first rejection
//                     k_resid          grid (sequences * slices) slice masses of the residual / bonus row; the
//                                      workgroup that finishes a sequence last draws the token
// svip_verify_greedy = k_argmax        grid (target rows * slices) first maximum per slice, no exponentials
//                     k_accept_greedy  grid (sequences), 1 wave  argmax p == x test, ballot, correction = argmax p
//
// svip_pair_stats  =  k_verify_stats   (rows j < draft_len of both models), k_pair_L (logsumexps),
//                     k_pair_sums      grid (slices, positions)  sum min(p,q), sum q log(q/p), sum q log q
//                     k_pair_finish    one thread per position   beta, KL, cross entropy, the bounds
//
// svip_warp_logits =  k_warp           grid (rows), 1024 threads  top-k / top-p thresholds by radix select, masked copy
//
// The passes are bound by HBM reads of the logits; there is no dense contraction, hence no MFMA.
// Nothing spins or waits on the device: kernels of one call are ordered by the stream; inside the
// residual pass the "last workgroup" hand-over of exchange.h lets a sequence's draw follow its slices
// without a second launch.  Each finishing step issues all of its independent loads before the first
// dependent one, because at small batches a step is bound by round trips to memory, not by bandwidth.
// Workgroups are handed to the chip's 8 XCDs in turn and each XCD has its own L2: k_draft_stats and k_resid
// map workgroups to (row, records) so that everything of row b runs on XCD b % 8, where the workgroup that
// finishes the row reads records and a tile again.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/svip.h"
#include "../../include/svip_bench.h"
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

// svip_workspace_reset: the flag word and the ticket counters at the end of the workspace.
struct ZeroArgs {
    unsigned *flags;
    uint4 *tail;
    size_t n16;
};
__global__ void k_zero(ZeroArgs z)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *z.flags = 0u;
    const uint4 zero = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < z.n16; i += (size_t)gridDim.x * blockDim.x)
        z.tail[i] = zero;
}

// Reference kernels of the benchmark hooks: an empty launch, and a read-only stream with the access
// pattern of the statistics passes (256-thread workgroups, NV 16-byte non-temporal loads per thread, a
// wave reads 1 KiB contiguous per load) that only folds what it read into one word per wave.
__global__ __launch_bounds__(64) void k_empty(int) {}

struct StreamArgs {
    const u32x4 *buf;
    size_t nvec;
    unsigned *sink;
};
template <int NV>
__global__ __launch_bounds__(WG) void k_stream_read(StreamArgs a)
{
    const size_t base = (size_t)blockIdx.x * (WG * NV) + threadIdx.x;
    u32x4 v[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const size_t i = base + (size_t)u * WG;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        v[u] = i < a.nvec ? __builtin_nontemporal_load(a.buf + i) : zero;
    }
    unsigned x = 0u;
#pragma unroll
    for (int u = 0; u < NV; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    x = (unsigned)wave_reduce((int)x, OpMax{});
    if ((threadIdx.x & 63) == 0) a.sink[(size_t)blockIdx.x * NWAVE + (threadIdx.x >> 6)] = x;
}

// Scratch of svip_draft_step_static: the workspace of a draft step for callers that cannot allocate one.
// One copy per GPU the library runs on, held until the process ends.  Host code never uses this name as an
// address: static_scratch() asks the runtime for the array's device address, once per device.
static __device__ __align__(256) unsigned char scratch[SVIP_STATIC_SCRATCH_BYTES];

// ---- host side -------------------------------------------------------------------------------

// Launch-shape overrides for experiments (svip_bench_set_tuning; all zero = the library's own choice).
// Workspace sizes are always computed for the library's own choice; a forced shape that needs more than
// the workspace holds is rejected by the call.
static svip_bench_tuning g_tune = {0, 0, 0, 0, 0, 0, 0};

// Slices per row of the passes that give a slice to a workgroup: enough workgroups to fill 256 CUs several
// times over, at most MAX_SLICES; want_one_batch (the residual pass): slices of min_tiles tiles, which the
// sampler scans as one batch and whose tiles each get a mass of their own.
static Geo make_geo(int V, int vec, long long rows, bool want_one_batch, int forced_ns, int min_tiles = 4)
{
    Geo g;
    g.V = V;
    const int nvec = (V + vec - 1) / vec;
    g.ntiles = (nvec + WG - 1) / WG;
    long long ns;
    if (want_one_batch) {
        // slices of min_tiles tiles (4: 32 logits per thread, and few enough tiles for tile masses)
        long long cap = g.ntiles / min_tiles;
        if (cap < 1) cap = 1;
        ns = cap;
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
    if (!want_one_batch && g.tps > 1 && (g.tps & 1) == 0 && !g_tune.even_tiles_per_slice) g.tps += 1;
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

static bool dtype_ok(int d) { return d == SVIP_F32 || d == SVIP_BF16 || d == SVIP_F16; }
static int vec_of(int d) { return d == SVIP_F32 ? 4 : 8; }       // logits per 16-byte vector

// Calls f with a value of the storage type that d names (f is a generic lambda).
template <typename F>
static void by_dtype(int d, F f)
{
    if (d == SVIP_BF16) f(bf16{});
    else if (d == SVIP_F16) f(f16{});
    else f(float{});
}

// Benchmark timing hook (svip_bench_time_kernels): caller-owned HIP events, attached pair by pair to
// the launches of one kernel class.
struct KernelTimer {
    void *const *start = nullptr, *const *stop = nullptr;
    int n = 0, used = 0;
};
static KernelTimer g_timer[SVIP_BENCH_KERNEL_CLASSES];

// One kernel launch on the stream; the launch's own status is returned (an error some earlier,
// unrelated HIP call left behind is neither consumed nor reported).  `cls` names the kernel class for
// the timing hook.
template <typename A>
static bool launch(void (*kernel)(A), unsigned grid, unsigned block, hipStream_t st, const A &args, int cls = -1)
{
    A copy = args;
    void *argv[] = {&copy};
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (cls >= 0 && g_timer[cls].used < g_timer[cls].n) {
        e0 = static_cast<hipEvent_t>(g_timer[cls].start[g_timer[cls].used]);
        e1 = static_cast<hipEvent_t>(g_timer[cls].stop[g_timer[cls].used]);
        ++g_timer[cls].used;
    }
    if (!e0)        // the plain launch is the one stream capture records
        return hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(grid), dim3(block), argv, 0, st) == hipSuccess;
    return hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(grid), dim3(block), argv, 0, st, e0, e1, 0) ==
           hipSuccess;
}

// ---- workspace each call needs (its own geometry; svip_workspace_bytes bounds them all) -------

// flag word + records + ticket counters + slice masses of the residual pass (mass_slices per sequence)
static size_t ws_fixed_bytes(int B, int mass_slices)
{
    return HEADER_BYTES + ws_rec_bytes(B) + ws_mass_bytes(B, mass_slices) + ws_ticket_bytes(B);
}

static size_t need_draft(int B, const Geo &g) { return ws_fixed_bytes(B, 0) + align256((size_t)B * g.ns * sizeof(Partial)); }
static size_t need_verify_greedy(int B, int k, const Geo &g)
{
    return ws_fixed_bytes(B, 0) + align256((size_t)B * (k + 1) * g.ns * sizeof(unsigned long long));
}
static size_t need_verify(int B, int k, bool recompute_lse, const Geo &g, const Geo &gs)
{
    const size_t stat_rows = (size_t)B * ((recompute_lse ? k : 0) + k + 1);
    return ws_fixed_bytes(B, gs.ns) + align256(stat_rows * g.ns * sizeof(Partial));
}
static size_t need_pair(int B, int k, bool recompute_lse, const Geo &g, const Geo &g2, size_t *part_bytes,
                        size_t *L_bytes)
{
    const size_t stat_rows = (size_t)B * ((recompute_lse ? k : 0) + k + 1), pos = (size_t)B * k;
    const size_t pb = align256(stat_rows * g.ns * sizeof(Partial));
    const size_t lb = align256(pos * 2 * sizeof(double));
    if (part_bytes) *part_bytes = pb;
    if (L_bytes) *L_bytes = lb;
    return ws_fixed_bytes(B, 0) + pb + lb + align256(pos * g2.ns * 3 * sizeof(double));
}

// The slicing each pass uses (forced = an experiment's override, 0 = the library's choice).
// The draft step: one record (= one wave of the statistics launch) per tile of 32 logits per thread, so the
// search reads a single tile again; rows of more than MAX_SLICES tiles put more tiles into a record, and so do
// batches that would otherwise launch more than 8100 waves (eight per SIMD): about a quarter of a one-tile
// wave's instructions are per-record overhead, which then outweighs the finer grain and the shorter search
// (rows of 128K logits, us per step with 63 and with 32 records, rows placed by XCD in both: 48 rows 9.5 / 10.0,
// 64 rows 10.2 / 10.5, 80 rows 11.0 / 11.9, 96 rows 11.7 / 12.1, 112 rows 12.3 / 13.2, 128 rows 13.2 / 13.6,
// 144 rows 14.95 / 14.6).
static Geo geo_draft(int B, int V, int vec, int forced)
{
    Geo g;
    g.V = V;
    const int nvec = (V + vec - 1) / vec;
    g.ntiles = (nvec + WG - 1) / WG;
    int ns = g.ntiles < MAX_SLICES ? g.ntiles : MAX_SLICES;
    if ((long long)B * ns > 8100 && ns == g.ntiles && ns > 1) ns = (ns + 1) / 2;
    if (forced > 0) ns = forced < MAX_SLICES ? forced : MAX_SLICES;
    if (ns > g.ntiles) ns = g.ntiles;
    if (ns < 1) ns = 1;
    g.tps = (g.ntiles + ns - 1) / ns;
    g.ns = (g.ntiles + g.tps - 1) / g.tps;
    return g;
}
static Geo geo_stats(long long stat_rows, int V, int vec, int forced) { return make_geo(V, vec, stat_rows, false, forced); }
// the residual pass: slices of four tiles like the draft step (at 64 sequences of 128K logits, 16 slices of
// 4 tiles take 13 us, 32 slices of 2 tiles 16 us, 8 slices 20 us, one tile per slice 26 us)
static Geo geo_resid(int B, int V, int vec, int forced) { return make_geo(V, vec, B, true, forced, 4); }

// ---- the calls behind the entry points ---------------------------------------------------------

static bool workspace_ok(const void *ws, size_t have, size_t need)
{
    return ws && (reinterpret_cast<uintptr_t>(ws) & 255u) == 0 && (have & ~(size_t)255) >= need;
}

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
    a.geo = geo_draft(c.B, c.V, vec, g_tune.draft_slices);
    if (!workspace_ok(c.workspace, c.workspace_bytes, need_draft(c.B, a.geo))) return SVIP_ERR_WORKSPACE;
    const Workspace w = carve(c.workspace, c.workspace_bytes, c.B, 0);
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
    const unsigned waves = (unsigned)a.geo.ns * (unsigned)c.B, rows = (unsigned)c.B;
    // Rows pinned to XCDs (see k_draft_stats) while the launch has at most 8100 waves: measured, rows of 128K bf16
    // logits, us per step without / with: 16 rows 8.15 / 8.07, 32 rows 9.2 / 8.9, 64 rows 11.2 / 10.8, 72 rows
    // (4536 one-tile waves) 11.5 / 10.85, 88 rows 12.3 / 11.5, 192 rows (6144 two-tile waves) 16.8 / 16.4; 64 and
    // 256 rows of 32000 logits 8.4 / 8.0 and 13.0 / 12.6; but 256 rows of 128K (8192 two-tile waves) 20.65 / 20.8.
    // Rows of fewer than four records would leave most of a workgroup's waves without one.
    a.rows_by_xcd = waves <= 8100u && a.geo.ns >= NWAVE;
    const unsigned grid = a.rows_by_xcd ? ((rows + 7u) / 8u) * 8u * (((unsigned)a.geo.ns + NWAVE - 1) / NWAVE)
                                        : (waves + NWAVE - 1) / NWAVE;
    // the kernel's division: floor(n / d) = umulhi(n, floor(2^32 / d) + 1) while n * d < 2^32 (n < 2^26 waves, d <= 64)
    a.div = a.rows_by_xcd ? ((unsigned)a.geo.ns + NWAVE - 1) / NWAVE : (unsigned)a.geo.ns;
    a.div_magic = a.div > 1u ? (unsigned)(0x100000000ull / a.div) + 1u : 0u;
    bool ok = false;
    by_dtype(c.dtype, [&](auto tag) {
        using DT = decltype(tag);
        const bool two = a.geo.tps == 2;
        if (c.greedy)
            ok = launch(two ? k_draft_stats<DT, true, true> : k_draft_stats<DT, true, false>, grid, WG, st, a,
                        SVIP_BENCH_K_DRAFT_STATS) &&
                 launch(k_draft_finish<DT, true>, rows, 64, st, a, SVIP_BENCH_K_DRAFT_FINISH);
        else
            ok = launch(two ? k_draft_stats<DT, false, true> : k_draft_stats<DT, false, false>, grid, WG, st, a,
                        SVIP_BENCH_K_DRAFT_STATS) &&
                 launch(k_draft_finish<DT, false>, rows, FINISH_THREADS, st, a, SVIP_BENCH_K_DRAFT_FINISH);
    });
    return ok ? SVIP_OK : SVIP_ERR_HIP;
}

// Device address of `scratch` on the current device, or nullptr.  The first call on a device looks the
// symbol up (hipGetSymbolAddress with that device current); every GPU holds its own copy of the array at
// its own address.  Nothing in it has to start at zero: a draft step writes every record before it reads it.
static void *static_scratch()
{
    constexpr int MAX_DEVICES = 64;
    static void *ptr[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        ptr[dev] = p;
    }
    return ptr[dev];
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
    a.geo = geo_stats(rows, c.V, vec, g_tune.stats_slices);
    if (!workspace_ok(c.workspace, c.workspace_bytes, need_verify_greedy(c.B, c.k_max, a.geo))) return SVIP_ERR_WORKSPACE;
    const Workspace w = carve(c.workspace, c.workspace_bytes, c.B, 0);
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
    a.skip = c.skip;
    a.keys = reinterpret_cast<unsigned long long *>(w.part);
    a.flags = w.flags;
    hipStream_t st = static_cast<hipStream_t>(c.stream);
    bool ok = false;
    by_dtype(c.dtype, [&](auto tag) {
        ok = launch(k_argmax<decltype(tag)>, (unsigned)(rows * a.geo.ns), WG, st, a, SVIP_BENCH_K_VERIFY_STATS);
    });
    ok = ok && launch(k_accept_greedy, (unsigned)c.B, 64, st, a, SVIP_BENCH_K_ACCEPT);
    return ok ? SVIP_OK : SVIP_ERR_HIP;
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
    a.geo = geo_stats(stat_rows, c.V, vec, g_tune.stats_slices);
    a.geo_s = geo_resid(c.B, c.V, vec, g_tune.resid_slices);
    if (!workspace_ok(c.workspace, c.workspace_bytes, need_verify(c.B, c.k_max, kd != 0, a.geo, a.geo_s)))
        return SVIP_ERR_WORKSPACE;
    a.target = c.target;
    a.draft = c.draft;
    a.seq_t = c.seq_stride_t;
    a.seq_d = c.seq_stride_d;
    a.row_stride = c.row_stride;
    a.pos = c.pos;
    a.skip = c.skip;
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
    a.ws = carve(c.workspace, c.workspace_bytes, c.B, a.geo_s.ns);
    hipStream_t st = static_cast<hipStream_t>(c.stream);
    a.stat_items = stat_rows * a.geo.ns;
    unsigned g_stats = (unsigned)a.stat_items;
    if (g_tune.stats_workgroups > 0 && (unsigned)g_tune.stats_workgroups < g_stats) g_stats = (unsigned)g_tune.stats_workgroups;
    const unsigned g_resid = (unsigned)a.geo_s.ns * (((unsigned)c.B + 7u) / 8u) * 8u;   // sequences by XCD, see k_resid
    bool ok = false;
    by_dtype(c.dtype, [&](auto tag) {
        using DT = decltype(tag);
        ok = launch(k_verify_stats<DT>, g_stats, WG, st, a, SVIP_BENCH_K_VERIFY_STATS) &&
             launch(k_accept<DT>, (unsigned)c.B, 64, st, a, SVIP_BENCH_K_ACCEPT) &&
             (a.geo_s.tps <= TILE_MASSES ? launch(k_resid<DT, true>, g_resid, WG, st, a, SVIP_BENCH_K_RESID)
                                         : launch(k_resid<DT, false>, g_resid, WG, st, a, SVIP_BENCH_K_RESID));
    });
    return ok ? SVIP_OK : SVIP_ERR_HIP;
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
    // a row has at most `tiles` slices (fp32 rows have the most vectors)
    const size_t tiles = ((size_t)V + 4 * WG - 1) / (4 * WG);
    const size_t ns_max = tiles < MAX_SLICES ? tiles : MAX_SLICES;
    size_t part_bytes = (size_t)B * ns_max * sizeof(Partial);
    if ((vrows + 8192) * sizeof(Partial) > part_bytes) part_bytes = (vrows + 8192) * sizeof(Partial);
    // diagnostics: two logsumexps per position and three sums per slice of its second pass
    const size_t pos = (size_t)B * (size_t)k_max;
    return ws_fixed_bytes(B, (int)ns_max) + align256(part_bytes) + align256(pos * 2 * sizeof(double)) +
           align256((pos + 8192) * 3 * sizeof(double));
}

size_t svip_workspace_needed(int call, int dtype, int B, int k_max, int V)
{
    if (!dtype_ok(dtype) || B <= 0 || B > MAX_BATCH || k_max < 1 || k_max > SVIP_MAX_K || V <= 0) return 0;
    const int vec = vec_of(dtype);
    const long long rows_t = (long long)B * (k_max + 1), rows_all = (long long)B * (2 * k_max + 1);
    switch (call) {
        case SVIP_CALL_DRAFT_STEP: return need_draft(B, geo_draft(B, V, vec, 0));
        case SVIP_CALL_VERIFY: return need_verify(B, k_max, false, geo_stats(rows_t, V, vec, 0), geo_resid(B, V, vec, 0));
        case SVIP_CALL_VERIFY_RECOMPUTE:
            return need_verify(B, k_max, true, geo_stats(rows_all, V, vec, 0), geo_resid(B, V, vec, 0));
        case SVIP_CALL_VERIFY_GREEDY: return need_verify_greedy(B, k_max, geo_stats(rows_t, V, vec, 0));
        case SVIP_CALL_PAIR_STATS:
            return need_pair(B, k_max, false, geo_stats(rows_t, V, vec, 0), geo_stats((long long)B * k_max, V, vec, 0),
                             nullptr, nullptr);
        case SVIP_CALL_PAIR_STATS_RECOMPUTE:
            return need_pair(B, k_max, true, geo_stats(rows_all, V, vec, 0), geo_stats((long long)B * k_max, V, vec, 0),
                             nullptr, nullptr);
        default: return 0;
    }
}

svip_status svip_workspace_reset(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace || workspace_bytes < 2 * HEADER_BYTES || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return SVIP_ERR_WORKSPACE;
    // the flag word, and the ticket counters at the end of the workspace (for any batch size up to MAX_BATCH
    // that this workspace may later be used with): a fill kernel, so that the call can be captured in a graph
    const size_t end = workspace_bytes & ~(size_t)255;
    size_t tail = ws_ticket_bytes(MAX_BATCH);
    if (tail > end - HEADER_BYTES) tail = end - HEADER_BYTES;
    ZeroArgs z;
    z.flags = static_cast<unsigned *>(workspace);
    z.tail = reinterpret_cast<uint4 *>(static_cast<char *>(workspace) + end - tail);
    z.n16 = tail / 16;
    const unsigned grid = (unsigned)((z.n16 + 255) / 256 < 1024 ? (z.n16 + 255) / 256 : 1024);
    return launch(k_zero, grid ? grid : 1u, 256, static_cast<hipStream_t>(hip_stream), z) ? SVIP_OK : SVIP_ERR_HIP;
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

svip_status svip_draft_step(const void *draft_logits, int dtype, int B, int V, long long row_stride,
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

svip_status svip_draft_step_static(const void *draft_logits, int dtype, int B, int V, long long row_stride,
                                   float temperature, float h, int step_j, int k_max, const float *u_sample,
                                   const unsigned char *stop_in, int *token_out, float *entropy_out,
                                   float *q_tok_out, double *lse_out, unsigned char *stop_out,
                                   int *draft_len_out, long long io_stride, void *hip_stream)
{
    // sizes first: a batch whose slice records do not fit the fixed scratch is refused before anything else
    if (!dtype_ok(dtype)) return SVIP_ERR_DTYPE;
    if (B <= 0 || B > MAX_BATCH || V <= 0) return SVIP_ERR_SHAPE;
    if (need_draft(B, geo_draft(B, V, vec_of(dtype), g_tune.draft_slices)) > (size_t)SVIP_STATIC_SCRATCH_BYTES)
        return SVIP_ERR_WORKSPACE;
    void *ws = static_scratch();
    if (!ws) return SVIP_ERR_HIP;
    const DraftCall c{false, draft_logits, dtype, B, V, row_stride, nullptr, 0, nullptr, temperature, h, step_j,
                      k_max, u_sample, stop_in, token_out, entropy_out, q_tok_out, lse_out, stop_out,
                      draft_len_out, io_stride, ws, (size_t)SVIP_STATIC_SCRATCH_BYTES, hip_stream};
    return draft_step_call(c);
}

svip_status svip_draft_step_greedy(const void *draft_logits, int dtype, int B, int V, long long row_stride,
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

svip_status svip_verify_greedy(const void *target_logits, int dtype, int B, int k_max, int V,
                               long long seq_stride_t, long long row_stride, const int *draft_tokens,
                               const int *draft_len, int *n_accepted_out, int *next_token_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const VerifyCall c{true, target_logits, nullptr, dtype, B, k_max, V, seq_stride_t, 0, row_stride, nullptr, nullptr, 1.f,
                       draft_tokens, draft_len, nullptr, nullptr, nullptr, n_accepted_out, next_token_out,
                       nullptr, workspace, workspace_bytes, hip_stream};
    return verify_call(c);
}

svip_status svip_verify(const void *target_logits, const void *draft_logits, int dtype, int B,
                        int k_max, int V, long long seq_stride_t, long long seq_stride_d,
                        long long row_stride, float temperature, const int *draft_tokens,
                        const int *draft_len, const double *draft_lse, const float *u_accept,
                        const float *u_resample, int *n_accepted_out, int *next_token_out,
                        float *accept_prob_out, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    const VerifyCall c{false, target_logits, draft_logits, dtype, B, k_max, V, seq_stride_t, seq_stride_d,
                       row_stride, nullptr, nullptr, temperature, draft_tokens, draft_len, draft_lse, u_accept,
                       u_resample, n_accepted_out, next_token_out, accept_prob_out, workspace,
                       workspace_bytes, hip_stream};
    return verify_call(c);
}

svip_status svip_warp_logits(const void *logits_in, void *logits_out, int dtype, int B, int k_max, int V,
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
    a.no_shortcut = g_tune.warp_no_shortcut;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    bool ok = false;
    by_dtype(dtype, [&](auto tag) {
        ok = launch(k_warp<decltype(tag)>, (unsigned)((long long)B * k_max), WARP_WG, st, a);
    });
    return ok ? SVIP_OK : SVIP_ERR_HIP;
}

svip_status svip_pair_stats(const void *target_logits, const void *draft_logits, int dtype, int B,
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
    a.v.geo = geo_stats(stat_rows, V, vec, g_tune.stats_slices);
    a.v.geo_s = a.v.geo;
    a.geo2 = geo_stats(pos, V, vec, g_tune.pair_slices);
    size_t part_bytes, L_bytes;
    const size_t need = need_pair(B, k_max, kd != 0, a.v.geo, a.geo2, &part_bytes, &L_bytes);
    if (!workspace_ok(workspace, workspace_bytes, need)) return SVIP_ERR_WORKSPACE;
    a.v.target = target_logits;
    a.v.draft = draft_logits;
    a.v.seq_t = seq_stride_t;
    a.v.seq_d = seq_stride_d;
    a.v.row_stride = row_stride;
    a.v.pos = nullptr;
    a.v.skip = nullptr;
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
    a.v.ws = carve(workspace, workspace_bytes, B, 0);
    char *after = reinterpret_cast<char *>(a.v.ws.part) + part_bytes;
    a.L = reinterpret_cast<double *>(after);
    a.sums = reinterpret_cast<double *>(after + L_bytes);
    a.c = c;
    a.out = stats_out;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    a.v.stat_items = stat_rows * a.v.geo.ns;
    const unsigned g_stats = (unsigned)a.v.stat_items, g_pos = (unsigned)((pos + 63) / 64),
                   g_sums = (unsigned)(pos * a.geo2.ns);
    bool ok = false;
    by_dtype(dtype, [&](auto tag) { ok = launch(k_verify_stats<decltype(tag)>, g_stats, WG, st, a.v); });
    ok = ok && launch(k_pair_L, g_pos, 64, st, a);
    if (ok) by_dtype(dtype, [&](auto tag) { ok = launch(k_pair_sums<decltype(tag)>, g_sums, WG, st, a); });
    ok = ok && launch(k_pair_finish, g_pos, 64, st, a);
    return ok ? SVIP_OK : SVIP_ERR_HIP;
}

// ---- benchmark and experiment hooks (include/svip_bench.h) -------------------------------------------

svip_status svip_bench_time_kernels(int kernel_class, void *const *start_events, void *const *stop_events, int n_pairs)
{
    if (kernel_class < 0 || kernel_class >= SVIP_BENCH_KERNEL_CLASSES || n_pairs < 0) return SVIP_ERR_PARAM;
    if (n_pairs > 0 && (!start_events || !stop_events)) return SVIP_ERR_NULL;
    KernelTimer &t = g_timer[kernel_class];
    t.start = n_pairs ? start_events : nullptr;
    t.stop = n_pairs ? stop_events : nullptr;
    t.n = n_pairs;
    t.used = 0;
    return SVIP_OK;
}

int svip_bench_events_used(int kernel_class)
{
    return kernel_class >= 0 && kernel_class < SVIP_BENCH_KERNEL_CLASSES ? g_timer[kernel_class].used : -1;
}

svip_status svip_bench_empty_kernel(void *hip_stream)
{
    return launch(k_empty, 1u, 64u, static_cast<hipStream_t>(hip_stream), 0) ? SVIP_OK : SVIP_ERR_HIP;
}

size_t svip_bench_stream_sink_words(size_t bytes, int vectors_per_thread)
{
    if (vectors_per_thread != 4 && vectors_per_thread != 8 && vectors_per_thread != 16) return 0;
    const size_t nvec = bytes / 16, per_wg = (size_t)WG * vectors_per_thread;
    return ((nvec + per_wg - 1) / per_wg) * NWAVE;
}

svip_status svip_bench_stream_read(const void *buf, size_t bytes, int vectors_per_thread, unsigned *sink,
                                   void *hip_stream)
{
    if (!buf || !sink) return SVIP_ERR_NULL;
    if (!aligned16(buf)) return SVIP_ERR_ALIGN;
    const size_t words = svip_bench_stream_sink_words(bytes, vectors_per_thread);
    if (words == 0 || words / NWAVE > 0x7FFFFFFFull) return SVIP_ERR_SHAPE;
    StreamArgs a;
    a.buf = static_cast<const u32x4 *>(buf);
    a.nvec = bytes / 16;
    a.sink = sink;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const unsigned grid = (unsigned)(words / NWAVE);
    bool ok;
    if (vectors_per_thread == 4) ok = launch(k_stream_read<4>, grid, WG, st, a);
    else if (vectors_per_thread == 8) ok = launch(k_stream_read<8>, grid, WG, st, a);
    else ok = launch(k_stream_read<16>, grid, WG, st, a);
    return ok ? SVIP_OK : SVIP_ERR_HIP;
}

svip_status svip_bench_set_tuning(const svip_bench_tuning *tuning)
{
    const svip_bench_tuning zero = {0, 0, 0, 0, 0, 0, 0};
    const svip_bench_tuning t = tuning ? *tuning : zero;
    if (t.draft_slices < 0 || t.stats_slices < 0 || t.resid_slices < 0 || t.pair_slices < 0 ||
        t.stats_workgroups < 0)
        return SVIP_ERR_PARAM;
    g_tune = t;
    return SVIP_OK;
}

}  // extern "C"
