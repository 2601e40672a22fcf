// Decoding loop over logit traces (Algorithm 1 and Algorithm 6) with the draft-length rules of
// the paper's baselines (Section 3: Constant, Heuristic), built on the draft and verify calls.
//
// Per round:  k_round_begin  -> per-sequence trace position, length limit and stop flag of the round
//             draft steps    -> svip_draft_step kernels reading trace row pos[b] + j, flags chained on the
//                               device; every `check_every` steps the host reads one counter and ends
//                               the drafting phase once every sequence has stopped
//             verify         -> svip_verify kernels on trace rows pos[b] .. pos[b] + draft_len[b]
//             k_round_end    -> appends the produced tokens, advances positions, applies the length
//                               rule, updates the counters and counts the sequences still running
// The host synchronises once per round (to read that count) and never per draft step unless asked to.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/svip.h"
#include "svip_internal.h"

namespace svip {

constexpr int LOOP_WG = 256;

struct RoundBuffers {          // carved from the loop workspace after the kernels' own workspace
    int *tokens;               // [B, gamma_max]
    double *lse;               // [B, gamma_max]
    unsigned char *stop;       // [B]
    unsigned char *done;       // [B] 1: the sequence has finished, verification skips it
    int *draft_len;            // [B]
    int *n_accepted;           // [B]
    int *next_token;           // [B]
    int *pos;                  // [B] trace position of the round (0 for finished sequences)
    int *cap;                  // [B] length limit of the round
    int *counter;              // [2]: sequences still running after the round, sequences still drafting
};

struct LoopArgs {
    int *state;                // [B, SVIP_LOOP_NSTATE]
    int B, L, gamma_max, inc, dec, max_new, round;
    RoundBuffers rb;
    int *out_tokens;
    long long out_stride;
    int *round_log;            // [rounds, B, 4] or nullptr
};

static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

static size_t round_buffer_bytes(int B, int k)
{
    const size_t n = (size_t)B, nk = n * (size_t)k;
    return up256(nk * 4) + up256(nk * 8) + 2 * up256(n) + 6 * up256(n * 4) + 256;
}

static RoundBuffers carve_round(char *p, int B, int k)
{
    const size_t n = (size_t)B, nk = n * (size_t)k;
    RoundBuffers r;
    r.tokens = reinterpret_cast<int *>(p); p += up256(nk * 4);
    r.lse = reinterpret_cast<double *>(p); p += up256(nk * 8);
    r.stop = reinterpret_cast<unsigned char *>(p); p += up256(n);
    r.done = reinterpret_cast<unsigned char *>(p); p += up256(n);
    r.draft_len = reinterpret_cast<int *>(p); p += up256(n * 4);
    r.n_accepted = reinterpret_cast<int *>(p); p += up256(n * 4);
    r.next_token = reinterpret_cast<int *>(p); p += up256(n * 4);
    r.pos = reinterpret_cast<int *>(p); p += up256(n * 4);
    r.cap = reinterpret_cast<int *>(p); p += up256(n * 4);
    r.counter = reinterpret_cast<int *>(p);
    return r;
}

// A sequence starts another round while it has produced fewer than max_new tokens and the trace
// still holds cap + 1 rows from its position on (Algorithm 1's loop condition, plus the end of
// the synthetic trace).
__device__ __forceinline__ bool finished(int pos, int n0, int cap, int L, int max_new)
{
    return pos - n0 >= max_new || pos + cap + 1 > L;
}

__device__ __forceinline__ int block_count(int mine, int *lds)
{
    // one workgroup: sum of `mine` over its threads, valid in thread 0
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_down(mine, o, 64);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = mine;
    __syncthreads();
    int total = 0;
    if (threadIdx.x == 0)
        for (int w = 0; w < LOOP_WG / 64; ++w) total += lds[w];
    return total;
}

// one workgroup
__global__ __launch_bounds__(LOOP_WG) void k_loop_init(int *state, int B, int n0, int gamma0, int L, int max_new,
                                                       int *counter)
{
    __shared__ int lds[LOOP_WG / 64];
    int running = 0;
    for (int b = threadIdx.x; b < B; b += LOOP_WG) {
        int *st = state + (size_t)b * SVIP_LOOP_NSTATE;
        const int done = finished(n0, n0, gamma0, L, max_new) ? 1 : 0;
        st[0] = n0;
        st[1] = gamma0;
        st[2] = done;
        st[3] = st[4] = st[5] = st[6] = 0;
        st[7] = n0;
        running += !done;
    }
    const int total = block_count(running, lds);
    if (threadIdx.x == 0) {
        counter[0] = total;
        counter[1] = 0;
    }
}

// one workgroup: what the round's kernels read
__global__ __launch_bounds__(LOOP_WG) void k_round_begin(LoopArgs a)
{
    for (int b = threadIdx.x; b < a.B; b += LOOP_WG) {
        const int *st = a.state + (size_t)b * SVIP_LOOP_NSTATE;
        const int done = st[2];
        a.rb.pos[b] = done ? 0 : st[0];
        a.rb.cap[b] = done ? 1 : st[1];
        a.rb.stop[b] = done ? 1 : 0;
        a.rb.done[b] = done ? 1 : 0;
        a.rb.draft_len[b] = 0;
    }
}

// one workgroup: number of sequences that are still drafting
__global__ __launch_bounds__(LOOP_WG) void k_count_drafting(const unsigned char *stop, int B, int *counter)
{
    __shared__ int lds[LOOP_WG / 64];
    int n = 0;
    for (int b = threadIdx.x; b < B; b += LOOP_WG) n += stop[b] ? 0 : 1;
    const int total = block_count(n, lds);
    if (threadIdx.x == 0) counter[1] = total;
}

// one workgroup: bookkeeping of the round for every running sequence
__global__ __launch_bounds__(LOOP_WG) void k_round_end(LoopArgs a)
{
    __shared__ int lds[LOOP_WG / 64];
    int running = 0;
    for (int b = threadIdx.x; b < a.B; b += LOOP_WG) {
        int *st = a.state + (size_t)b * SVIP_LOOP_NSTATE;
        int *lg = a.round_log ? a.round_log + ((size_t)a.round * a.B + b) * 4 : nullptr;
        if (st[2]) {
            if (lg) lg[0] = lg[1] = lg[2] = lg[3] = -1;
            continue;
        }
        const int pos = st[0], cap = st[1];
        const int g = a.rb.draft_len[b], na = a.rb.n_accepted[b];
        int *o = a.out_tokens + (size_t)b * a.out_stride + st[6];
        for (int j = 0; j < na; ++j) o[j] = a.rb.tokens[(size_t)b * a.gamma_max + j];
        o[na] = a.rb.next_token[b];
        if (lg) {
            lg[0] = pos;
            lg[1] = cap;
            lg[2] = g;
            lg[3] = na;
        }
        int ncap = cap + (na == g ? a.inc : -a.dec);          // every drafted token accepted: longer next time
        ncap = ncap < 1 ? 1 : (ncap > a.gamma_max ? a.gamma_max : ncap);
        const int npos = pos + na + 1;
        const int done = finished(npos, st[7], ncap, a.L, a.max_new) ? 1 : 0;
        st[0] = npos;
        st[1] = ncap;
        st[2] = done;
        st[3] += 1;
        st[4] += g;
        st[5] += na;
        st[6] += na + 1;
        running += !done;
    }
    const int total = block_count(running, lds);
    if (threadIdx.x == 0) a.rb.counter[0] = total;
}

static svip_status read_counter(const int *dev, int *host, hipStream_t st)
{
    if (hipMemcpyAsync(host, dev, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return SVIP_ERR_HIP;
    return hipStreamSynchronize(st) == hipSuccess ? SVIP_OK : SVIP_ERR_HIP;
}

static svip_status check_config(const svip_loop_config *c)
{
    if (!c) return SVIP_ERR_NULL;
    if (!c->target_trace || !c->draft_trace || !c->state || !c->out_tokens) return SVIP_ERR_NULL;
    if (!c->greedy && (!c->u_sample || !c->u_accept || !c->u_resample)) return SVIP_ERR_NULL;
    if (c->B <= 0 || c->V <= 0 || c->gamma_max < 1 || c->gamma_max > SVIP_MAX_K || c->gamma0 < 1 ||
        c->gamma0 > c->gamma_max || c->L < c->gamma_max + 1 || c->n0 < 0 || c->n0 >= c->L || c->max_new < 0 ||
        c->row_stride < c->V || c->seq_stride < (long long)c->L * c->row_stride - (c->row_stride - c->V) ||
        c->out_stride < (long long)c->max_new + c->gamma_max || c->rounds < 1)
        return SVIP_ERR_SHAPE;
    if (c->gamma_inc < 0 || c->gamma_dec < 0 || c->check_every < 0) return SVIP_ERR_PARAM;
    const size_t need = svip_loop_workspace_bytes(c->B, c->gamma_max, c->V);
    if (!c->workspace || (reinterpret_cast<uintptr_t>(c->workspace) & 255u) || need == 0 || c->workspace_bytes < need)
        return SVIP_ERR_WORKSPACE;
    return SVIP_OK;
}

}  // namespace svip

using namespace svip;

extern "C" {

size_t svip_loop_workspace_bytes(int B, int gamma_max, int V)
{
    const size_t base = svip_workspace_bytes(B, gamma_max, V);
    if (base == 0) return 0;
    return up256(base) + round_buffer_bytes(B, gamma_max);
}

svip_status svip_loop_init(const svip_loop_config *c)
{
    const svip_status s = check_config(c);
    if (s != SVIP_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(c->hip_stream);
    const size_t base = up256(svip_workspace_bytes(c->B, c->gamma_max, c->V));
    const RoundBuffers rb = carve_round(static_cast<char *>(c->workspace) + base, c->B, c->gamma_max);
    const svip_status r = svip_workspace_reset(c->workspace, base, c->hip_stream);
    if (r != SVIP_OK) return r;
    hipLaunchKernelGGL(k_loop_init, dim3(1), dim3(LOOP_WG), 0, st, c->state, c->B, c->n0, c->gamma0, c->L,
                       c->max_new, rb.counter);
    return hipPeekAtLastError() == hipSuccess ? SVIP_OK : SVIP_ERR_HIP;
}

svip_status svip_loop_run(const svip_loop_config *c, int first_round, int max_rounds, int *rounds_run_host,
                          int *running_host)
{
    const svip_status s = check_config(c);
    if (s != SVIP_OK) return s;
    if (first_round < 0 || max_rounds < 0 || (long long)first_round + max_rounds > c->rounds) return SVIP_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(c->hip_stream);
    const size_t base = up256(svip_workspace_bytes(c->B, c->gamma_max, c->V));
    const RoundBuffers rb = carve_round(static_cast<char *>(c->workspace) + base, c->B, c->gamma_max);
    const int B = c->B, k = c->gamma_max;

    int running = 0, done_rounds = 0;
    svip_status r = read_counter(rb.counter, &running, st);
    if (r != SVIP_OK) return r;
    for (int i = 0; i < max_rounds && running > 0; ++i) {
        const int round = first_round + i;
        LoopArgs a;
        a.state = c->state;
        a.B = B;
        a.L = c->L;
        a.gamma_max = k;
        a.inc = c->gamma_inc;
        a.dec = c->gamma_dec;
        a.max_new = c->max_new;
        a.round = round;
        a.rb = rb;
        a.out_tokens = c->out_tokens;
        a.out_stride = c->out_stride;
        a.round_log = c->round_log;
        hipLaunchKernelGGL(k_round_begin, dim3(1), dim3(LOOP_WG), 0, st, a);

        const size_t uoff = (size_t)round * B * k;
        for (int j = 0; j < k; ++j) {
            DraftCall d;
            d.greedy = c->greedy != 0;
            d.logits = c->draft_trace;
            d.dtype = c->dtype;
            d.B = B;
            d.V = c->V;
            d.row_stride = c->seq_stride;
            d.pos = rb.pos;
            d.pos_stride = c->row_stride;
            d.cap = rb.cap;
            d.temperature = c->temperature;
            d.h = c->h;
            d.step_j = j;
            d.k_max = k;
            d.u_sample = c->greedy ? nullptr : c->u_sample + uoff + j;
            d.stop_in = rb.stop;
            d.token_out = rb.tokens + j;
            d.entropy_out = nullptr;
            d.q_tok_out = nullptr;
            d.lse_out = rb.lse + j;
            d.stop_out = rb.stop;
            d.draft_len_out = rb.draft_len;
            d.io_stride = k;
            d.workspace = c->workspace;
            d.workspace_bytes = base;             // the kernels' own part of the loop workspace
            d.stream = c->hip_stream;
            r = draft_step_call(d);
            if (r != SVIP_OK) return r;
            if (c->check_every > 0 && (j + 1) % c->check_every == 0 && j + 1 < k) {
                hipLaunchKernelGGL(k_count_drafting, dim3(1), dim3(LOOP_WG), 0, st, rb.stop, B, rb.counter);
                int drafting = 0;
                r = read_counter(rb.counter + 1, &drafting, st);
                if (r != SVIP_OK) return r;
                if (drafting == 0) break;
            }
        }

        VerifyCall v;
        v.greedy = c->greedy != 0;
        v.target = c->target_trace;
        v.draft = c->draft_trace;
        v.dtype = c->dtype;
        v.B = B;
        v.k_max = k;
        v.V = c->V;
        v.seq_stride_t = c->seq_stride;
        v.seq_stride_d = c->seq_stride;
        v.row_stride = c->row_stride;
        v.pos = rb.pos;
        v.temperature = c->temperature;
        v.draft_tokens = rb.tokens;
        v.draft_len = rb.draft_len;
        v.draft_lse = rb.lse;
        v.u_accept = c->greedy ? nullptr : c->u_accept + uoff;
        v.u_resample = c->greedy ? nullptr : c->u_resample + (size_t)round * B;
        v.n_accepted_out = rb.n_accepted;
        v.next_token_out = rb.next_token;
        v.accept_prob_out = nullptr;
        v.skip = rb.done;
        v.workspace = c->workspace;
        v.workspace_bytes = base;
        v.stream = c->hip_stream;
        r = verify_call(v);
        if (r != SVIP_OK) return r;

        hipLaunchKernelGGL(k_round_end, dim3(1), dim3(LOOP_WG), 0, st, a);
        if (hipPeekAtLastError() != hipSuccess) return SVIP_ERR_HIP;
        r = read_counter(rb.counter, &running, st);
        if (r != SVIP_OK) return r;
        ++done_rounds;
    }
    if (rounds_run_host) *rounds_run_host = done_rounds;
    if (running_host) *running_host = running;
    return SVIP_OK;
}

}  // extern "C"
