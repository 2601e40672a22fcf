/*
 * svip.h -- C ABI of the MI355X (gfx950) hot path of SVIP, the entropy-driven draft-length
 * policy for speculative decoding of arXiv 2411.18462.
 *
 * Two calls cover the per-step vocabulary-wide work of one speculative round:
 *
 *   svip_draft_step   one draft position for every sequence still drafting: softmax of the
 *                     draft logits, Shannon entropy, one sampled token, and the stop test
 *                     sqrt(H_q) > h                     (Algorithm 1, drafting loop;
 *                                                        Section 2.2, Eq. stop_condition)
 *   svip_verify       the whole verification of a round: acceptance test r < p(x)/q(x) at
 *                     every drafted position, first rejection, and either the correction
 *                     drawn from the normalised residual max(0, p - q) or, if nothing was
 *                     rejected, the bonus token drawn from the next target row
 *                                                       (Algorithm 1, verification loop;
 *                                                        Algorithm 2 Verify, Algorithm 4 Correct)
 *   svip_loop_init, svip_loop_run   the decoding loop over logit traces with the draft-length
 *                    policies the paper compares (Algorithm 1, Algorithm 6, Section 3)
 *   svip_pair_stats  acceptance diagnostics per drafted position (Section 2.2, Appendix B)
 *   svip_warp_logits top-k / top-p filtering of logits rows ahead of those calls (not in the paper)
 *   svip_draft_step_greedy, svip_verify_greedy    the same two steps under greedy decoding
 *                                                       (Algorithm 3 Verify, Algorithm 5 Correct)
 *
 * General rules
 *   - Every pointer marked "device" is GPU memory of the current HIP device; "host" is CPU
 *     memory.  The caller owns every buffer; the library allocates nothing, frees nothing
 *     and keeps no pointer after a call returns.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising.  Outputs are valid once the stream
 *     has reached that point.
 *   - Logits are row-major rows of V values, fp32, bf16 or fp16.  Base pointers must be 16-byte
 *     aligned and every stride (in elements) a multiple of 16 bytes' worth of elements
 *     (8 for bf16 and fp16, 4 for fp32).  V itself may be any positive number.
 *   - Arithmetic: fp32 per element with fp64 combination of partial results; entropies are
 *     in nats; logits are divided by `temperature` before the softmax and H is the entropy
 *     of that tempered distribution.  -inf logits carry no mass; a row with no finite logit
 *     or with NaN has undefined results.
 *   - "Sample from weights w with one uniform u" means: the smallest token index i whose
 *     inclusive prefix sum w_0 + ... + w_i exceeds u * sum(w) (strict), in ascending index
 *     order.  Uniforms are caller-supplied floats in [0, 1).
 *   - Host-checkable argument errors return a status before anything is enqueued.  Errors in
 *     device data (token id outside [0, V), draft length outside [0, k_max]) are clamped and
 *     recorded in a sticky flag word inside the workspace (svip_workspace_flags).
 *   - `workspace` is device scratch of at least svip_workspace_bytes(B, k_max, V) bytes,
 *     256-byte aligned, that svip_workspace_reset has cleared once after allocation.  Besides
 *     partial results it holds, at its end, the counters with which the workgroups of svip_verify's
 *     residual pass hand a sequence's draw to whichever of them finishes last; every call leaves
 *     them at zero again.  Pass the same `workspace_bytes` with a workspace on every call.  Calls
 *     that run concurrently must use different workspaces.
 *   - Same inputs give bit-identical outputs (no floating-point atomics, fixed combine order).
 */
#ifndef SVIP_H
#define SVIP_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SVIP_OK = 0,
    SVIP_ERR_NULL = 1,       /* a required pointer is NULL */
    SVIP_ERR_SHAPE = 2,      /* B, V, k_max, step_j or a stride out of range */
    SVIP_ERR_DTYPE = 3,      /* dtype is not one of svip_dtype */
    SVIP_ERR_ALIGN = 4,      /* base pointer or stride not 16-byte aligned */
    SVIP_ERR_WORKSPACE = 5,  /* workspace NULL, misaligned or too small */
    SVIP_ERR_PARAM = 6,      /* temperature <= 0 or not finite, h negative or NaN */
    SVIP_ERR_HIP = 7         /* a HIP runtime call failed */
} svip_status;

/* Storage type of the logits; every value is widened exactly to fp32 on load.  The calls take it as a
 * plain int (`dtype`), so that a value outside this list is an error the library reports
 * (SVIP_ERR_DTYPE), not an invalid enumeration value. */
typedef enum { SVIP_F32 = 0, SVIP_BF16 = 1, SVIP_F16 = 2 } svip_dtype;

/* Bits of the sticky device-data flag word. */
enum { SVIP_FLAG_BAD_TOKEN = 1, SVIP_FLAG_BAD_DRAFT_LEN = 2 };

/* Largest k_max (draft positions per round) the library accepts. */
#define SVIP_MAX_K 1024

/* Human-readable name of a status; static storage, never freed. */
const char *svip_status_string(int status);

/* Bytes of device workspace that both calls need for batches of up to B sequences with up
 * to k_max draft positions over a vocabulary of V.  Pure host function; 0 on bad arguments. */
size_t svip_workspace_bytes(int B, int k_max, int V);

/* Bytes of workspace one particular call uses for these sizes (pure host function; 0 on bad
 * arguments).  svip_workspace_bytes(B, k_max, V) is never smaller than any of them; the calls
 * themselves check against these figures. */
typedef enum {
    SVIP_CALL_DRAFT_STEP = 0,            /* svip_draft_step, svip_draft_step_greedy */
    SVIP_CALL_VERIFY = 1,                /* svip_verify with draft_lse given */
    SVIP_CALL_VERIFY_RECOMPUTE = 2,      /* svip_verify with draft_lse == NULL */
    SVIP_CALL_VERIFY_GREEDY = 3,         /* svip_verify_greedy */
    SVIP_CALL_PAIR_STATS = 4,            /* svip_pair_stats with draft_lse given */
    SVIP_CALL_PAIR_STATS_RECOMPUTE = 5   /* svip_pair_stats with draft_lse == NULL */
} svip_call;
size_t svip_workspace_needed(int call, int dtype, int B, int k_max, int V);

/* Zero the sticky flag word and the hand-over counters at the end of the workspace (enqueued on
 * the stream as a fill kernel).  Call once after allocating a workspace, with the size that the
 * other calls will be given; the calls below only ever set flag bits and leave the counters zero. */
svip_status svip_workspace_reset(void *workspace, size_t workspace_bytes, void *hip_stream);

/* Copy the flag word to *flags_host (host).  Synchronises the stream. */
svip_status svip_workspace_flags(const void *workspace, void *hip_stream, unsigned *flags_host);

/*
 * One draft position for every sequence that is still drafting.
 *
 * For each row b in [0, B) with stop_in == NULL or stop_in[b] == 0:
 *   q = softmax(draft_logits[b, :] / temperature)
 *   H = -sum q ln q                                            (Section 2.2, H_q)
 *   token ~ q with the uniform u_sample[b * io_stride]         (Algorithm 1, "Sample x ~ q")
 *   stop = sqrt(H) > h  or  step_j + 1 >= k_max                (Eq. stop_condition; the cap
 *                                                               is the paper's draft-length limit)
 * and writes, at index b * io_stride of each per-row output array,
 *   token_out, entropy_out = H, q_tok_out = q[token], lse_out = logsumexp(logits / temperature),
 * plus stop_out[b] and, if draft_len_out != NULL, draft_len_out[b] = step_j + 1.
 * Rows with stop_in[b] != 0 get token_out = -1 and stop_out[b] = 1 and nothing else is written
 * for them.  Their logits do not enter any result but may still be read (the flag and the first
 * loads of the logits are requested together: a step is bound by memory round trips, and waiting
 * for the flag first costs 0.16 us of an 11.4 us step at 64 rows and 0.3 us of 8.1 us at 8), so draft_logits must be
 * readable for every row.
 *
 * io_stride lets the per-row arrays be columns of [B, k_max] buffers (pass the address of
 * column step_j and io_stride = k_max), which is the layout svip_verify consumes; likewise
 * draft_logits may point at position step_j of a [B, k_max, V] buffer with
 * row_stride = k_max * V.  stop_out may alias stop_in (in-place update of one flag array
 * across the steps of a round).  entropy_out and q_tok_out may be NULL.
 */
svip_status svip_draft_step(
    const void *draft_logits,        /* device, row b at element offset b * row_stride */
    int dtype, int B, int V, long long row_stride,
    float temperature, float h,
    int step_j, int k_max,           /* 0 <= step_j < k_max <= SVIP_MAX_K */
    const float *u_sample,           /* device, uniforms in [0,1), row b at b * io_stride */
    const unsigned char *stop_in,    /* device [B] or NULL */
    int *token_out,                  /* device, b * io_stride */
    float *entropy_out,              /* device, b * io_stride, or NULL */
    float *q_tok_out,                /* device, b * io_stride, or NULL */
    double *lse_out,                 /* device, b * io_stride */
    unsigned char *stop_out,         /* device [B] */
    int *draft_len_out,              /* device [B] or NULL */
    long long io_stride,             /* >= 1 */
    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * svip_draft_step for callers that cannot allocate device memory or hand a workspace through: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as svip_draft_step (bit for bit), without the workspace: the rows' statistics records
 * live in a fixed array of SVIP_STATIC_SCRATCH_BYTES inside the library's device code, one copy per
 * GPU, held until the process ends.  The call allocates nothing and frees nothing.
 *   - Sizes whose records do not fit that array (svip_workspace_needed(SVIP_CALL_DRAFT_STEP, ...) >
 *     SVIP_STATIC_SCRATCH_BYTES; about 1200 rows of a 128K vocabulary) return SVIP_ERR_WORKSPACE.
 *   - All calls on one GPU share the array: calls that overlap on one GPU (different streams, or
 *     threads) race and must be serialised by the caller.  Device-data flags are not reported.
 *   - The first call on a GPU asks the runtime for the array's address on that GPU (no allocation,
 *     nothing enqueued); nothing in the array has to be cleared.
 */
#define SVIP_STATIC_SCRATCH_BYTES (1 << 20)
svip_status svip_draft_step_static(
    const void *draft_logits, int dtype, int B, int V, long long row_stride,
    float temperature, float h, int step_j, int k_max, const float *u_sample,
    const unsigned char *stop_in, int *token_out, float *entropy_out, float *q_tok_out,
    double *lse_out, unsigned char *stop_out, int *draft_len_out, long long io_stride,
    void *hip_stream);

/*
 * Verification of one round for every sequence.
 *
 * For each sequence b with g = draft_len[b] drafted tokens x_0..x_{g-1} (0 <= g <= k_max):
 *   for j < g:  p_j = softmax(target_logits[b, j, :] / temperature),
 *               q_j = softmax(draft_logits[b, j, :] / temperature),
 *               accept_j = u_accept[b, j] * q_j(x_j) < p_j(x_j)         (Algorithm 2)
 *               accept_prob_out[b, j] = min(1, p_j(x_j) / q_j(x_j))
 *   r = first j with accept_j false, or g if there is none;  n_accepted_out[b] = r
 *   if r < g:  next_token_out[b] ~ max(0, p_r - q_r) (normalised)       (Algorithm 4)
 *              (if that residual has no mass: ~ p_r)
 *   else:      next_token_out[b] ~ p_g, the target row after the drafts (Algorithm 1, bonus token)
 *   both drawn with u_resample[b].
 * Entries of accept_prob_out at j >= g are left untouched.
 *
 * draft_lse[b, j] = logsumexp(draft_logits[b, j, :] / temperature) as written by
 * svip_draft_step; if NULL the library recomputes it, reading every drafted draft row.
 * With draft_lse given, only the draft row at the rejected position is read.
 */
svip_status svip_verify(
    const void *target_logits,       /* device, row (b, j) at b * seq_stride_t + j * row_stride, j <= k_max */
    const void *draft_logits,        /* device, row (b, j) at b * seq_stride_d + j * row_stride, j <  k_max */
    int dtype, int B, int k_max, int V,
    long long seq_stride_t, long long seq_stride_d, long long row_stride,
    float temperature,
    const int *draft_tokens,         /* device [B, k_max] */
    const int *draft_len,            /* device [B] */
    const double *draft_lse,         /* device [B, k_max] or NULL */
    const float *u_accept,           /* device [B, k_max], uniforms in [0,1) */
    const float *u_resample,         /* device [B], uniforms in [0,1) */
    int *n_accepted_out,             /* device [B] */
    int *next_token_out,             /* device [B] */
    float *accept_prob_out,          /* device [B, k_max] or NULL */
    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Greedy decoding (Appendix A, Algorithms 3 and 5; the paper's reasoning-model and greedy
 * long-form runs).
 *
 * svip_draft_step_greedy is svip_draft_step with the draw replaced by the first maximum:
 * token = argmax of the row (the smallest index among equal maxima), q_tok_out = its
 * probability; entropy (of softmax(logits / temperature)), logsumexp, stop test, cap, skipping
 * of stopped rows and the output layout are identical.  No uniforms are needed.
 */
svip_status svip_draft_step_greedy(
    const void *draft_logits, int dtype, int B, int V, long long row_stride,
    float temperature, float h, int step_j, int k_max,
    const unsigned char *stop_in, int *token_out, float *entropy_out, float *q_tok_out,
    double *lse_out, unsigned char *stop_out, int *draft_len_out, long long io_stride,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Greedy verification of one round.  For each sequence b with g = draft_len[b]:
 *   accept_j = (argmax target_logits[b, j, :] == draft_tokens[b, j])  for j < g   (Algorithm 3)
 *   r = first j with accept_j false, or g;  n_accepted_out[b] = r
 *   next_token_out[b] = argmax target_logits[b, r, :]   (Algorithm 5 correction, or the bonus token)
 * argmax takes the smallest index among equal maxima.  Only the target rows j <= g are read; the
 * draft logits are not needed.  Results are exact (comparisons only), for any dtype.
 */
svip_status svip_verify_greedy(
    const void *target_logits,       /* device, row (b, j) at b * seq_stride_t + j * row_stride, j <= k_max */
    int dtype, int B, int k_max, int V,
    long long seq_stride_t, long long row_stride,
    const int *draft_tokens,         /* device [B, k_max] */
    const int *draft_len,            /* device [B] */
    int *n_accepted_out,             /* device [B] */
    int *next_token_out,             /* device [B] */
    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Per-position diagnostics of the acceptance analysis (Section 2.2, Eq. beta, Eq. tvd,
 * Eq. pinsker, Eq. beta-bound, Eq. appro_bound; Appendix B).  For each sequence b and each
 * drafted position j < draft_len[b], with p = softmax(target_logits[b, j] / T) and
 * q = softmax(draft_logits[b, j] / T), stats_out[b, j, :] receives
 *   [0] beta = sum_x min(p(x), q(x))          expected acceptance probability (= 1 - TVD)
 *   [1] KL(q || p)                            nats
 *   [2] H_{q,p} = -sum_x q(x) ln p(x)         cross entropy, nats (= [3] + [1])
 *   [3] H_q                                   nats
 *   [4] 1 - sqrt(KL / 2)                      the oracle bound
 *   [5] 1 - sqrt(1 - exp(-KL))                the Bretagnolle-Huber bound
 *   [6] 1 - sqrt(c H_q)                       the approximation bound with constant c
 *   [7] H_{q,p} / H_q                         the ratio the paper calls gamma (NaN if H_q = 0)
 * and NaN in all SVIP_PAIR_NSTAT entries of positions j >= draft_len[b].  Target row draft_len[b]
 * (the bonus row) is not read.  draft_lse as in svip_verify (NULL: recomputed here).  Two passes
 * over both rows of every drafted position: 4 V elements of traffic per position (3 V when
 * draft_lse is given).  A logit of -inf counts as probability 2^-200 in the sums, so a token
 * the target masks but the draft can emit gives a large finite KL rather than +inf.
 */
#define SVIP_PAIR_NSTAT 8
svip_status svip_pair_stats(
    const void *target_logits,       /* device, row (b, j) at b * seq_stride_t + j * row_stride, j < k_max */
    const void *draft_logits,        /* device, row (b, j) at b * seq_stride_d + j * row_stride, j < k_max */
    int dtype, int B, int k_max, int V,
    long long seq_stride_t, long long seq_stride_d, long long row_stride,
    float temperature,
    const int *draft_len,            /* device [B] */
    const double *draft_lse,         /* device [B, k_max] natural-log logsumexp of draft rows, or NULL */
    float c,                         /* >= 0 */
    float *stats_out,                /* device [B, k_max, SVIP_PAIR_NSTAT] */
    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Decoding loop over logit traces: Algorithm 1 (stop drafting when sqrt(H_q) > h) and Algorithm 6
 * (a fixed draft length) are one loop with different stopping rules, and the Heuristic baseline of
 * Section 3 is a rule for the length limit between rounds:
 *   SVIP:      h finite,   gamma0 = gamma_max = the length limit, gamma_inc = gamma_dec = 0
 *   Constant:  h = +inf,   gamma0 = gamma_max = the draft length,  gamma_inc = gamma_dec = 0
 *   Heuristic: h = +inf,   gamma0 = the first length, gamma_inc = 2, gamma_dec = 1; lengths stay in
 *              [1, gamma_max]
 * The models are stood in for by traces: row n of sequence b's trace holds the logits for the token
 * at absolute position n (independent of the tokens chosen before).  A sequence starts a new round
 * while it has produced fewer than max_new tokens and its trace holds limit + 1 more rows; a round
 * produces the accepted draft tokens followed by the correction or bonus token.  Everything per
 * round stays on the device; the host learns one counter per round (and, if check_every > 0, one
 * more every check_every draft steps to end the drafting phase early).  The counters come as
 * messages the counting kernels store into pinned host memory -- no copy is enqueued and the stream
 * is not synchronised between rounds -- and the host launches one round ahead of the counter it
 * waits for: a round launched after the last sequence finished changes nothing (its sequences are
 * all marked done) except that, with a log, it may fill its round_log entries with -1.  The first
 * svip_loop_run of a host thread allocates 512 bytes of pinned host memory for those messages and
 * keeps them until the process ends.
 *
 * state[b, :] (int32): 0 position, 1 length limit of the next round, 2 finished, 3 rounds,
 * 4 drafted tokens, 5 accepted tokens, 6 produced tokens, 7 start position.
 * round_log[r, b, :] (optional): position, limit, drafted, accepted of round r (-1 when finished).
 * Round r draws with u_sample[r, b, j], u_accept[r, b, j], u_resample[r, b].
 */
#define SVIP_LOOP_NSTATE 8
typedef struct svip_loop_config {
    const void *target_trace;   /* device [B, L, V]: row (b, n) at b * seq_stride + n * row_stride */
    const void *draft_trace;    /* device, same layout */
    int dtype;
    int B, L, V;
    long long seq_stride, row_stride;   /* elements; multiples of 16 bytes */
    float temperature;
    int greedy;                 /* 0: Algorithms 2 and 4 with the uniforms below; 1: Algorithms 3 and 5 */
    float h;                    /* entropy threshold; +inf disables the test */
    int gamma0, gamma_max, gamma_inc, gamma_dec;
    int n0;                     /* first position to generate */
    int max_new;                /* tokens to produce per sequence (a round may overshoot by gamma_max) */
    int rounds;                 /* rounds the uniform arrays and the log hold */
    const float *u_sample;      /* device [rounds, B, gamma_max] (unused when greedy) */
    const float *u_accept;      /* device [rounds, B, gamma_max] */
    const float *u_resample;    /* device [rounds, B] */
    int *state;                 /* device [B, SVIP_LOOP_NSTATE] */
    int *out_tokens;            /* device [B, out_stride], out_stride >= max_new + gamma_max */
    long long out_stride;
    int *round_log;             /* device [rounds, B, 4] or NULL */
    int check_every;            /* 0: never ask the device during drafting */
    void *workspace;            /* device, svip_loop_workspace_bytes(B, gamma_max, V), 256-byte aligned */
    size_t workspace_bytes;
    void *hip_stream;
} svip_loop_config;

/* Bytes of device workspace the loop needs (kernel workspace plus the buffers of one round). */
size_t svip_loop_workspace_bytes(int B, int gamma_max, int V);

/* Set every sequence to position n0 with limit gamma0 and clear the counters and flags (enqueued). */
svip_status svip_loop_init(const svip_loop_config *config /* host */);

/* Run rounds first_round .. first_round + max_rounds - 1 (or until every sequence has finished).
 * Synchronises the stream before it returns.  *rounds_run_host and *running_host (host, optional)
 * receive the rounds executed (a round launched ahead that found every sequence finished is not
 * counted) and the sequences still running. */
svip_status svip_loop_run(const svip_loop_config *config /* host */, int first_round, int max_rounds,
                          int *rounds_run_host, int *running_host);

/*
 * Top-k followed by top-p (nucleus) filtering of logits rows, for callers that sample from a
 * truncated distribution.  The paper's algorithms draw from the full softmax (Algorithms 1, 2
 * and 4); this call is a variant of their sampling rows that the paper does not cover: it writes
 * a copy of the rows in which every filtered-out logit is -inf, and svip_draft_step,
 * svip_verify and svip_pair_stats treat -inf logits as tokens of probability zero, so the
 * filtered rows can be handed to them unchanged (filter draft and target rows alike and the
 * accept / residual rule of Algorithms 2 and 4 stays exact for the truncated distributions).
 *
 * With q = softmax(z / temperature) of a row, both filters are thresholds on the logit VALUE
 * (equal logits are kept or dropped together):
 *   top_k  (0 < top_k < V): keep z >= the top_k-th largest logit of the row;
 *   top_p  (0 < top_p < 1): among the survivors, with Z their total probability, go down the
 *          distinct logit values and keep everything down to the first value at which the
 *          cumulative probability reaches top_p * Z.
 * top_k == 0 or >= V, and top_p >= 1, switch the respective filter off.  Probabilities are
 * fp32 exponentials summed exactly as 64-bit fixed-point numbers (2^-44 units for V <= 2^18);
 * a top-p decision closer than about 1e-6 * Z to its threshold may differ from an exact
 * evaluation.  Top-k decisions are exact.  Results do not depend on thread scheduling.
 *
 * logits_in, logits_out: device, B sequences of n_rows rows (any n_rows >= 1 with B * n_rows < 2^31: a
 * round's rows or a whole trace for the loop), row (b, j) at element offset
 * b * seq_stride + j * row_stride in both; they may be the same buffer (in place), and must
 * not overlap otherwise.  kept_out: device [B * n_rows], survivors per row, or NULL.
 * No workspace.  Enqueues on hip_stream and returns; errors as for the other calls
 * (SVIP_ERR_PARAM: temperature, top_k < 0, top_p <= 0 or NaN).
 */
svip_status svip_warp_logits(const void *logits_in, void *logits_out, int dtype, int B, int n_rows,
                             int V, long long seq_stride, long long row_stride, float temperature,
                             int top_k, double top_p, int *kept_out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SVIP_H */
