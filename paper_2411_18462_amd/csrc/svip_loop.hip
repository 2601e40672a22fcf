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
// The two counts reach the host as messages: the counting kernel stores (ticket, count) as one 8-byte word
// into pinned host memory and the host reads that word until the ticket shows.  No copy is enqueued and the
// stream is never synchronised inside the loop; the host launches one round ahead of the count it waits for,
// so the GPU always has the next round queued (a round launched after the last sequence finished finds
// every sequence marked done and changes nothing).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <chrono>

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
    unsigned long long *mail;  // k_round_end: where the count of running sequences goes (pinned host memory)
    unsigned ticket;           // and the ticket it goes with
};

// ---- messages from the device to the host ----------------------------------------------------
//
// A host thread's mailbox: MAIL_SLOTS words of pinned host memory, allocated by the thread's first
// svip_loop_run and kept until the process ends.  A message is (ticket << 32 | value), stored by one
// thread of a kernel with a single system-scope store; tickets count up per host thread and never repeat
// within 2^32 messages, message t uses word t % MAIL_SLOTS, and the loop never has more than three
// messages outstanding, so a word is not reused before it has been read.
constexpr unsigned MAIL_SLOTS = 64;
struct Mailbox {
    unsigned long long *host, *dev;
    unsigned next;
};
static thread_local Mailbox g_mail = {nullptr, nullptr, 0};

struct Ticket {
    unsigned id;
    unsigned long long *dev;            // what the kernel gets
    const unsigned long long *host;     // what the host reads
};

static bool mailbox_ready()
{
    if (g_mail.host) return true;
    void *h = nullptr, *d = nullptr;
    // coherent (fine-grained) memory: a word stored by a running kernel is seen by the host without waiting for
    // the kernel to end; without the flag the other two would make the allocation non-coherent
    if (hipHostMalloc(&h, MAIL_SLOTS * sizeof(unsigned long long),
                      hipHostMallocCoherent | hipHostMallocPortable | hipHostMallocMapped) != hipSuccess)
        return false;
    memset(h, 0, MAIL_SLOTS * sizeof(unsigned long long));
    if (hipHostGetDevicePointer(&d, h, 0) != hipSuccess) {
        (void)hipHostFree(h);
        return false;
    }
    g_mail.host = static_cast<unsigned long long *>(h);
    g_mail.dev = static_cast<unsigned long long *>(d);
    g_mail.next = 0;
    return true;
}

static Ticket new_ticket()
{
    Ticket t;
    t.id = ++g_mail.next;
    if (t.id == 0) t.id = ++g_mail.next;       // 0 is what an unused word holds
    t.dev = g_mail.dev + t.id % MAIL_SLOTS;
    t.host = g_mail.host + t.id % MAIL_SLOTS;
    return t;
}

__device__ __forceinline__ void post(unsigned long long *word, unsigned ticket, int value)
{
    __hip_atomic_store(word, ((unsigned long long)ticket << 32) | (unsigned)value, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
}

// Waits until the message of ticket t is there.  The kernel that posts it is already in the stream, so the
// wait ends when the GPU gets there; if nothing shows for a while the stream is asked: one that has drained
// without the message has failed.
static svip_status await(const Ticket &t, int *value, hipStream_t st)
{
    typedef std::chrono::steady_clock clock;
    clock::time_point t0 = clock::now();
    for (unsigned spins = 1;; ++spins) {
        unsigned long long v = __atomic_load_n(t.host, __ATOMIC_ACQUIRE);
        if ((unsigned)(v >> 32) == t.id) {
            *value = (int)(unsigned)v;
            return SVIP_OK;
        }
        if ((spins & 4095u) == 0 && clock::now() - t0 > std::chrono::milliseconds(200)) {
            const hipError_t q = hipStreamQuery(st);
            if (q == hipErrorNotReady) {
                (void)hipGetLastError();        // "not ready" is no error of the loop's: do not leave it behind
                t0 = clock::now();
                continue;
            }
            v = __atomic_load_n(t.host, __ATOMIC_ACQUIRE);
            if (q == hipSuccess && (unsigned)(v >> 32) == t.id) {
                *value = (int)(unsigned)v;
                return SVIP_OK;
            }
            return SVIP_ERR_HIP;
        }
    }
}

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
__global__ __launch_bounds__(LOOP_WG) void k_count_drafting(const unsigned char *stop, int B, int *counter,
                                                            unsigned long long *mail, unsigned ticket)
{
    __shared__ int lds[LOOP_WG / 64];
    int n = 0;
    for (int b = threadIdx.x; b < B; b += LOOP_WG) n += stop[b] ? 0 : 1;
    const int total = block_count(n, lds);
    if (threadIdx.x == 0) {
        counter[1] = total;
        post(mail, ticket, total);
    }
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
    if (threadIdx.x == 0) {
        a.rb.counter[0] = total;
        post(a.mail, a.ticket, total);
    }
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
    if (running > 0 && max_rounds > 0 && !mailbox_ready()) return SVIP_ERR_HIP;
    // `running` is the count after the last round whose message has been read; `before` is the ticket of the
    // round launched since, whose message has not been read yet.  Round i is launched on the strength of
    // the count after round i - 2; if the count after round i - 1 then turns out to be zero, round i has
    // run (or is being dropped) with every sequence marked done and is not counted.
    Ticket before = {0, nullptr, nullptr};
    bool have_before = false;
    for (int i = 0; i < max_rounds && running > 0; ++i) {
        const int round = first_round + i;
        const Ticket mine = new_ticket();
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
        a.mail = mine.dev;
        a.ticket = mine.id;
        hipLaunchKernelGGL(k_round_begin, dim3(1), dim3(LOOP_WG), 0, st, a);

        const size_t uoff = (size_t)round * B * k;
        bool idle = false;        // the round before this one finished the last sequence
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
                const Ticket poll = new_ticket();
                hipLaunchKernelGGL(k_count_drafting, dim3(1), dim3(LOOP_WG), 0, st, rb.stop, B, rb.counter, poll.dev,
                                   poll.id);
                if (hipPeekAtLastError() != hipSuccess) return SVIP_ERR_HIP;
                int drafting = 0;
                r = await(poll, &drafting, st);
                if (r != SVIP_OK) return r;
                if (have_before) {                // the GPU is inside this round: the one before has posted
                    r = await(before, &running, st);
                    if (r != SVIP_OK) return r;
                    have_before = false;
                    if (running == 0) {
                        idle = true;
                        break;
                    }
                }
                if (drafting == 0) break;
            }
        }
        if (idle) break;

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
        if (have_before) {        // with this round queued behind it, wait for the count of the round before
            r = await(before, &running, st);
            if (r != SVIP_OK) return r;
            have_before = false;
            if (running == 0) break;              // this round was idle
        }
        before = mine;
        have_before = true;
        ++done_rounds;
    }
    if (have_before) {
        r = await(before, &running, st);
        if (r != SVIP_OK) return r;
    }
    if (hipStreamSynchronize(st) != hipSuccess) return SVIP_ERR_HIP;
    if (rounds_run_host) *rounds_run_host = done_rounds;
    if (running_host) *running_host = running;
    return SVIP_OK;
}

}  // extern "C"
