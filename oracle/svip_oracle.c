/*
 * SVIP hot-path oracle -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what the per-step vocabulary-wide work of
 * SVIP (arXiv 2411.18462) computes: the draft-side pass (softmax, Shannon entropy,
 * one categorical draw, entropy stop test) and the target-side verification pass
 * (acceptance test per draft position, first rejection, correction or bonus draw).
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 * It shares no code, header, table or constant with the HIP path.
 *
 * Everything is written row by row, in the order and notation of the paper:
 *   - draft token x ~ q(.|prefix)                          Algorithm 1, "Sample" step
 *   - stop iff sqrt(H_q) > h                               Section 2.2, Eq. (stop_condition)
 *   - accept iff r < p(x)/q(x), r ~ U[0,1)                 Algorithm 2 (Verify, sampling)
 *   - walk j = 1..gamma until the first failed Verify      Algorithm 1, verification loop
 *   - correction x^ ~ norm(max(0, p - q))                  Algorithm 4 (Correct, sampling);
 *     the listing prints q - p, which cannot preserve the target law the paper
 *     claims in Section 1 -- the p - q direction is the one that does
 *   - bonus token x ~ p(.|all drafts) if nothing rejected  Algorithm 1, last "Sample" step
 *   - greedy decoding: accept iff argmax p = x, correct with argmax p   Algorithms 3 and 5
 * plus the diagnostics of Section 2.2 and Appendix B: beta = sum min(p,q) (Eq. beta), KL(q||p),
 * the cross entropy H_{q,p} (Eq. pinsker / beta-bound), the oracle, Bretagnolle-Huber and
 * approximation bounds (oracle_diagnostics), and the whole decoding loop over logit traces with
 * the SVIP, Constant and Heuristic draft-length rules (oracle_generate: Algorithm 1, Algorithm 6,
 * Section 3).  oracle_warp_row states a truncation the paper does not have (top-k, then top-p, as
 * thresholds on the logit value); it is pinned by a worked example and a sort-based cross-check.
 *
 * Conventions (stated where the paper is silent):
 *   - entropy in nats; logits are divided by the temperature T before the softmax
 *     and H is the entropy of that tempered distribution;
 *   - "sample from weights w with one uniform u": the smallest index i whose
 *     inclusive prefix sum C_i = w_0 + ... + w_i satisfies C_i > u * sum(w)
 *     (ascending token index, strict inequality); if rounding leaves no such i,
 *     the largest i with w_i > 0;
 *   - the acceptance test is evaluated as r * q(x) < p(x) (no division), so q(x) = 0
 *     with p(x) > 0 accepts and p(x) = 0 rejects;
 *   - all uniforms for a round are drawn up front; positions after the first
 *     rejection are evaluated but ignored.
 *
 * Every decision also reports its margin (distance of the compared quantities from
 * the decision boundary) so that a finite-precision implementation can be compared
 * exactly wherever the margin is not within rounding.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---- one row ------------------------------------------------------------------ */

/* prob[i] = softmax(z/T)[i]; returns logsumexp(z/T).  exp(-inf) contributes 0. */
double oracle_softmax_row(const double *z, long V, double T, double *prob)
{
    double m = -INFINITY;
    for (long i = 0; i < V; ++i) {
        double zi = z[i] / T;
        if (zi > m) m = zi;
    }
    double S = 0.0;
    for (long i = 0; i < V; ++i) {
        double e = exp(z[i] / T - m);
        prob[i] = e;
        S += e;
    }
    for (long i = 0; i < V; ++i) prob[i] /= S;
    return m + log(S);
}

/* Shannon entropy -sum p ln p over p > 0, in nats (Section 2.2, H_q). */
double oracle_entropy_row(const double *prob, long V)
{
    double H = 0.0;
    for (long i = 0; i < V; ++i)
        if (prob[i] > 0.0) H -= prob[i] * log(prob[i]);
    return H > 0.0 ? H : 0.0;
}

/* One categorical draw from non-negative weights w with the uniform u in [0,1).
 * *margin = distance of u*W from the nearer edge of the chosen cell, divided by W.
 * Returns -1 if the total weight is not positive. */
long oracle_inverse_cdf(const double *w, long V, double u, double *margin)
{
    double W = 0.0;
    for (long i = 0; i < V; ++i) W += w[i];
    if (margin) *margin = 0.0;
    if (!(W > 0.0)) return -1;
    double target = u * W;
    double C = 0.0;
    long last_pos = -1;
    for (long i = 0; i < V; ++i) {
        double Cprev = C;
        C += w[i];
        if (w[i] > 0.0) last_pos = i;
        if (C > target) {
            if (margin) {
                double lo = target - Cprev, hi = C - target;
                *margin = (lo < hi ? lo : hi) / W;
            }
            return i;
        }
    }
    return last_pos; /* only reachable through rounding; margin stays 0 */
}

/* ---- draft step (Algorithm 1, drafting loop body; Eq. stop_condition) ---------- */

/*
 * For every row b with stop_in[b] == 0 (or stop_in == NULL):
 *   q = softmax(z_b / T); H = entropy(q); token ~ q via u[b];
 *   stop = sqrt(H) > h, or the row has reached the draft-length cap
 *   (step_j + 1 >= k_max; Section 3 limits the draft length).
 * Rows with stop_in[b] != 0 are skipped: token -1, stop 1, other outputs 0.
 * margin_h = |sqrt(H) - h|, margin_s = sampler margin.
 */
void oracle_draft_step(const double *z, long B, long V, long row_stride,
                       double T, double h, long step_j, long k_max,
                       const double *u, const unsigned char *stop_in,
                       long *token, double *entropy, double *q_tok, double *lse,
                       unsigned char *stop, double *margin_h, double *margin_s)
{
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    for (long b = 0; b < B; ++b) {
        if (stop_in && stop_in[b]) {
            token[b] = -1; entropy[b] = 0; q_tok[b] = 0; lse[b] = 0; stop[b] = 1;
            margin_h[b] = INFINITY; margin_s[b] = INFINITY;
            continue;
        }
        const double *zb = z + b * row_stride;
        lse[b] = oracle_softmax_row(zb, V, T, q);
        double H = oracle_entropy_row(q, V);
        entropy[b] = H;
        long x = oracle_inverse_cdf(q, V, u[b], &margin_s[b]);
        token[b] = x;
        q_tok[b] = x >= 0 ? q[x] : 0.0;
        int by_entropy = sqrt(H) > h;
        int by_cap = (step_j + 1 >= k_max);
        stop[b] = (unsigned char)(by_entropy || by_cap);
        margin_h[b] = by_cap ? INFINITY : fabs(sqrt(H) - h);
    }
    free(q);
}

/* ---- verification (Algorithm 1 verification loop; Algorithms 2 and 4) ---------- */

/*
 * zp: [B][k_max+1][V] target logits, zq: [B][k_max][V] draft logits (both dense),
 * tok: [B][k_max] draft tokens, gamma[b] in 0..k_max, ua: [B][k_max], ur: [B].
 * Outputs per sequence: n_accepted, next_token (correction or bonus),
 * accept_prob[b][j] = min(1, p/q) for j < gamma[b] (others untouched),
 * margin_a[b][j] = |ua - p/q| of the acceptance test at position j < gamma[b] (others untouched),
 * margin_accept[b] = smallest margin_a among the tests that shaped n_accepted: every position
 *   up to and including the first rejection (INFINITY when gamma[b] = 0),
 * margin_sample[b] = sampler margin of the correction / bonus draw (0 when the residual has no
 *   mass and the draw falls back to p),
 * margin[b] = the smaller of the two,
 * resid_mass[b] = sum max(0, p - q) at the rejected position (0 for a bonus draw).
 */
void oracle_verify(const double *zp, const double *zq, long B, long k_max, long V,
                   double T, const long *tok, const long *gamma,
                   const double *ua, const double *ur,
                   long *n_accepted, long *next_token, double *accept_prob,
                   double *margin, double *resid_mass,
                   double *margin_a, double *margin_accept, double *margin_sample)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    for (long b = 0; b < B; ++b) {
        const double *zpb = zp + b * (k_max + 1) * V;
        const double *zqb = zq + b * k_max * V;
        long g = gamma[b];
        long r = g;              /* 0-based index of the first rejection; g = none */
        double mar = INFINITY;
        /* evaluate every drafted position; the first failure ends the walk */
        for (long j = 0; j < g; ++j) {
            oracle_softmax_row(zpb + j * V, V, T, p);
            oracle_softmax_row(zqb + j * V, V, T, q);
            long x = tok[b * k_max + j];
            double px = p[x], qx = q[x];
            double ratio = qx > 0.0 ? px / qx : (px > 0.0 ? INFINITY : 0.0);
            accept_prob[b * k_max + j] = ratio < 1.0 ? ratio : 1.0;
            int acc = ua[b * k_max + j] * qx < px;
            double d = fabs(ua[b * k_max + j] - ratio);
            if (margin_a) margin_a[b * k_max + j] = d;
            if (r == g) {        /* no rejection so far: this decision shapes the output */
                if (d < mar) mar = d;
                if (!acc) r = j;
            }
        }
        n_accepted[b] = r;
        double ms = 0.0;
        resid_mass[b] = 0.0;
        if (r < g) {
            /* Correct: residual of target over draft at the rejected position */
            oracle_softmax_row(zpb + r * V, V, T, p);
            oracle_softmax_row(zqb + r * V, V, T, q);
            double W = 0.0;
            for (long i = 0; i < V; ++i) {
                double d = p[i] - q[i];
                w[i] = d > 0.0 ? d : 0.0;
                W += w[i];
            }
            resid_mass[b] = W;
            if (W > 0.0) {
                next_token[b] = oracle_inverse_cdf(w, V, ur[b], &ms);
            } else {          /* p <= q everywhere: no residual, draw from p */
                next_token[b] = oracle_inverse_cdf(p, V, ur[b], &ms);
                ms = 0.0;
            }
        } else {
            /* every draft accepted: bonus token from the target row after the drafts */
            oracle_softmax_row(zpb + g * V, V, T, p);
            next_token[b] = oracle_inverse_cdf(p, V, ur[b], &ms);
        }
        margin[b] = ms < mar ? ms : mar;
        if (margin_accept) margin_accept[b] = mar;
        if (margin_sample) margin_sample[b] = ms;
    }
    free(p); free(q); free(w);
}

/* ---- greedy decoding (Algorithm 3 Verify, Algorithm 5 Correct) ---------------------- */

/* Index of the largest logit; among equal maxima the smallest index. */
long oracle_argmax_row(const double *z, long V)
{
    long best = 0;
    for (long i = 1; i < V; ++i)
        if (z[i] > z[best]) best = i;
    return best;
}

/*
 * Draft step under greedy decoding: the draft token is argmax q instead of a draw; the
 * entropy of softmax(z / T) still drives the stop test (Section 2.2) and the cap applies.
 */
void oracle_draft_step_greedy(const double *z, long B, long V, long row_stride,
                              double T, double h, long step_j, long k_max,
                              const unsigned char *stop_in,
                              long *token, double *entropy, double *q_tok, double *lse,
                              unsigned char *stop, double *margin_h)
{
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    for (long b = 0; b < B; ++b) {
        if (stop_in && stop_in[b]) {
            token[b] = -1; entropy[b] = 0; q_tok[b] = 0; lse[b] = 0; stop[b] = 1;
            margin_h[b] = INFINITY;
            continue;
        }
        const double *zb = z + b * row_stride;
        lse[b] = oracle_softmax_row(zb, V, T, q);
        double H = oracle_entropy_row(q, V);
        entropy[b] = H;
        long x = oracle_argmax_row(zb, V);
        token[b] = x;
        q_tok[b] = q[x];
        int by_entropy = sqrt(H) > h;
        int by_cap = (step_j + 1 >= k_max);
        stop[b] = (unsigned char)(by_entropy || by_cap);
        margin_h[b] = by_cap ? INFINITY : fabs(sqrt(H) - h);
    }
    free(q);
}

/*
 * Verification under greedy decoding: position j is accepted iff argmax p_j equals the draft
 * token (Algorithm 3); at the first failure the correction is argmax p_j (Algorithm 5); if
 * every draft is accepted the bonus token is argmax of the next target row.
 * zp: [B][k_max+1][V], tok: [B][k_max], gamma[b] in 0..k_max.
 */
void oracle_verify_greedy(const double *zp, long B, long k_max, long V,
                          const long *tok, const long *gamma,
                          long *n_accepted, long *next_token)
{
    for (long b = 0; b < B; ++b) {
        const double *zpb = zp + b * (k_max + 1) * V;
        long g = gamma[b], r = g;
        for (long j = 0; j < g; ++j) {
            if (oracle_argmax_row(zpb + j * V, V) != tok[b * k_max + j]) { r = j; break; }
        }
        n_accepted[b] = r;
        next_token[b] = oracle_argmax_row(zpb + r * V, V);
    }
}

/* ---- diagnostics of Section 2.2 ------------------------------------------------ */

/* out[0] = beta = sum min(p,q)   (Eq. beta)
 * out[1] = KL(q||p)              (Eq. pinsker)
 * out[2] = H_{q,p} = -sum q ln p (Eq. beta-bound)
 * out[3] = H_q
 * out[4] = TVD(p,q) = 0.5 sum |p-q|  (Eq. tvd) */
void oracle_pair_stats(const double *zp_row, const double *zq_row, long V, double T,
                       double *out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    oracle_softmax_row(zp_row, V, T, p);
    oracle_softmax_row(zq_row, V, T, q);
    double beta = 0, kl = 0, hqp = 0, tvd = 0;
    for (long i = 0; i < V; ++i) {
        beta += p[i] < q[i] ? p[i] : q[i];
        tvd += 0.5 * fabs(p[i] - q[i]);
        if (q[i] > 0.0) {
            kl += q[i] * (log(q[i]) - log(p[i]));
            hqp -= q[i] * log(p[i]);
        }
    }
    out[0] = beta; out[1] = kl; out[2] = hqp; out[3] = oracle_entropy_row(q, V); out[4] = tvd;
    free(p); free(q);
}

/*
 * Per-position diagnostics of Section 2.2 and Appendix B for one round.
 * zp [B][k+1][V] target logits, zq [B][k][V] draft logits, gamma[b] drafted positions.
 * out [B][k][8]; entries of positions j >= gamma[b] are NaN.
 *   0 beta                       Eq. beta
 *   1 KL(q||p)                   Eq. pinsker
 *   2 H_{q,p}                    Eq. beta-bound
 *   3 H_q
 *   4 oracle bound        1 - sqrt(KL / 2)            Eq. pinsker / Eq. beta-bound
 *   5 Bretagnolle-Huber   1 - sqrt(1 - exp(-KL))      Appendix B
 *   6 approximation bound 1 - sqrt(c H_q)             Eq. appro_bound, c the constant standing in
 *                                                     for (gamma - 1) / 2
 *   7 ratio H_{q,p} / H_q        the paper's gamma (NaN when H_q = 0)
 */
void oracle_diagnostics(const double *zp, const double *zq, long B, long k, long V, double T,
                        const long *gamma, double c, double *out)
{
    for (long b = 0; b < B; ++b)
        for (long j = 0; j < k; ++j) {
            double *o = out + (b * k + j) * 8;
            if (j >= gamma[b]) {
                for (int i = 0; i < 8; ++i) o[i] = NAN;
                continue;
            }
            double st[5];
            oracle_pair_stats(zp + (b * (k + 1) + j) * V, zq + (b * k + j) * V, V, T, st);
            const double beta = st[0], kl = st[1], hqp = st[2], hq = st[3];
            o[0] = beta;
            o[1] = kl;
            o[2] = hqp;
            o[3] = hq;
            o[4] = 1.0 - sqrt(0.5 * kl);
            o[5] = 1.0 - sqrt(1.0 - exp(-kl));
            o[6] = 1.0 - sqrt(c * hq);
            o[7] = hq > 0.0 ? hqp / hq : NAN;
        }
}

/* ---- the decoding loop (Algorithm 1, Algorithm 6) ------------------------------------- */

/*
 * One sequence decoded over logit traces.  Algorithm 1 (stop drafting when sqrt(H_q) > h) and
 * Algorithm 6 (a fixed draft length) are the same loop with different stopping rules, so one
 * function covers both, and the Heuristic baseline of Section 3 (next draft length + inc if every
 * drafted token was accepted, else - dec) is a rule for the cap between rounds:
 *   SVIP:      h finite, gamma0 = gamma_max = the length limit, inc = dec = 0
 *   Constant:  h = INFINITY, gamma0 = the draft length, inc = dec = 0
 *   Heuristic: h = INFINITY, gamma0 the first length, inc = 2, dec = 1, lengths kept in [1, gamma_max]
 *
 * zq[L][V], zp[L][V]: logits of the draft / target model for the token at absolute position n
 * (in this synthetic setting they do not depend on the tokens chosen before).  Generation
 * starts at position n0 and a new round begins while fewer than max_new tokens were produced
 * and the trace still holds cap + 1 rows from n on.  Round r draws with us[r*kw + j] (draft
 * token j), ua[r*kw + j] (its acceptance test) and ur[r] (correction or bonus token); kw is the
 * row width of those arrays (>= gamma_max).  greedy != 0 uses Algorithms 3 and 5 and no uniforms.
 *
 * out_tok receives the produced tokens in order (accepted draft tokens, then the correction or
 * bonus token, per round); log[r][5] = {n at the start of round r, cap, drafted, accepted, last
 * token of the round}.  Returns the number of rounds; *n_out = tokens produced; *min_margin = the
 * smallest decision margin met (stop tests, draws, acceptance tests).
 */
long oracle_generate(const double *zp, const double *zq, long L, long V, double T,
                     long n0, long max_new, double h, long gamma0, long gamma_max, long inc, long dec,
                     const double *us, const double *ua, const double *ur, long kw, int greedy,
                     long max_rounds, long *out_tok, long *n_out, long *log, double *min_margin)
{
    long n = n0, gamma = gamma0, rounds = 0, produced = 0;
    double mm = INFINITY;
    long *tok = (long *)malloc(sizeof(long) * (size_t)(gamma_max > gamma0 ? gamma_max : gamma0));
    double *ap = (double *)malloc(sizeof(double) * (size_t)(gamma_max > gamma0 ? gamma_max : gamma0));
    while (n - n0 < max_new && n + gamma + 1 <= L && rounds < max_rounds) {
        const long cap = gamma;
        /* drafting: one token per step until the stop test or the cap says stop */
        long drafted = 0;
        unsigned char stop = 0;
        while (!stop) {
            long x; double H, qx, lse, mh, ms = INFINITY;
            if (greedy)
                oracle_draft_step_greedy(zq + (n + drafted) * V, 1, V, V, T, h, drafted, cap, NULL,
                                         &x, &H, &qx, &lse, &stop, &mh);
            else
                oracle_draft_step(zq + (n + drafted) * V, 1, V, V, T, h, drafted, cap,
                                  us + rounds * kw + drafted, NULL, &x, &H, &qx, &lse, &stop, &mh, &ms);
            tok[drafted] = x;
            if (mh < mm) mm = mh;
            if (ms < mm) mm = ms;
            ++drafted;
        }
        /* verification of the drafted tokens against target rows n .. n + drafted */
        long nacc, next;
        if (greedy) {
            oracle_verify_greedy(zp + n * V, 1, cap, V, tok, &drafted, &nacc, &next);
        } else {
            double mv, rm;
            oracle_verify(zp + n * V, zq + n * V, 1, cap, V, T, tok, &drafted, ua + rounds * kw, ur + rounds,
                          &nacc, &next, ap, &mv, &rm, NULL, NULL, NULL);
            if (mv < mm) mm = mv;
        }
        for (long j = 0; j < nacc; ++j) out_tok[produced++] = tok[j];
        out_tok[produced++] = next;
        log[rounds * 5 + 0] = n;
        log[rounds * 5 + 1] = cap;
        log[rounds * 5 + 2] = drafted;
        log[rounds * 5 + 3] = nacc;
        log[rounds * 5 + 4] = next;
        n += nacc + 1;
        gamma += (nacc == drafted) ? inc : -dec;
        if (gamma < 1) gamma = 1;
        if (gamma > gamma_max) gamma = gamma_max;
        ++rounds;
    }
    *n_out = produced;
    *min_margin = mm;
    free(tok); free(ap);
    return rounds;
}

/* ---- top-k / top-p filtering of a row (not in the paper; a variant of the same scan) ---- */

/*
 * Which tokens survive top-k followed by top-p filtering of q = softmax(z / T)?  Both filters
 * are thresholds on the logit VALUE, so equal logits are kept or dropped together:
 *   top-k  (0 < top_k < V): tau_k = the top_k-th largest logit (with multiplicity); keep z >= tau_k.
 *   top-p  (0 < top_p < 1): among the tokens kept so far, with Z their total probability, walk the
 *          distinct logit values downwards and stop at the first value v whose cumulative
 *          probability  sum_{z >= v} q  reaches top_p * Z; keep z >= v.
 * top_k <= 0 or >= V and top_p >= 1 switch the respective filter off.  keep[i] = 1 for survivors.
 * Returns the number kept; *margin = distance of the top-p decision from its threshold, as a
 * fraction of Z (INFINITY when top-p is off).
 */
typedef struct { double z; long i; } oracle_zi;
static int oracle_cmp_desc(const void *a, const void *b)
{
    const oracle_zi *x = (const oracle_zi *)a, *y = (const oracle_zi *)b;
    if (x->z > y->z) return -1;
    if (x->z < y->z) return 1;
    return x->i < y->i ? -1 : (x->i > y->i ? 1 : 0);
}
long oracle_warp_row(const double *z, long V, double T, long top_k, double top_p,
                     unsigned char *keep, double *margin)
{
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    oracle_zi *s = (oracle_zi *)malloc(sizeof(oracle_zi) * (size_t)V);
    oracle_softmax_row(z, V, T, q);
    for (long i = 0; i < V; ++i) { s[i].z = z[i]; s[i].i = i; }
    qsort(s, (size_t)V, sizeof(oracle_zi), oracle_cmp_desc);
    long n = V;                                   /* survivors are s[0 .. n) */
    if (top_k > 0 && top_k < V) {
        const double tau = s[top_k - 1].z;
        n = top_k;
        while (n < V && s[n].z == tau) ++n;       /* the whole tie group of the k-th value */
    }
    double mar = INFINITY;
    if (top_p < 1.0) {
        double Z = 0.0;
        for (long r = 0; r < n; ++r) Z += q[s[r].i];
        const double target = top_p * Z;
        double cum = 0.0;
        long r = 0, cut = n;
        while (r < n) {
            long e = r;
            double grp = 0.0;
            while (e < n && s[e].z == s[r].z) { grp += q[s[e].i]; ++e; }
            const double before = cum;
            cum += grp;
            if (cum >= target) {
                double lo = (target - before) / Z, hi = (cum - target) / Z;
                mar = lo < hi ? lo : hi;
                cut = e;
                break;
            }
            r = e;
        }
        n = cut;
    }
    for (long i = 0; i < V; ++i) keep[i] = 0;
    for (long r = 0; r < n; ++r) keep[s[r].i] = 1;
    if (margin) *margin = mar;
    free(q); free(s);
    return n;
}

/* ---- brute-force law of one speculative position (Algorithms 2 + 4) ------------ */

/*
 * N independent trials on fixed distributions p, q (already normalised, length V):
 *   x ~ q with a fresh uniform; Verify with a fresh uniform; on failure Correct
 *   with a fresh uniform.  hist[i] counts the emitted token, *n_acc the accepts.
 * Uniforms come from a 64-bit SplitMix generator seeded by `seed`, 53 bits each.
 * resid_sign = +1 uses max(0, p - q); -1 uses the printed max(0, q - p) so that a
 * test can show that direction breaks the target law.
 */
static unsigned long long splitmix(unsigned long long *s)
{
    unsigned long long z = (*s += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
static double unif(unsigned long long *s) { return (double)(splitmix(s) >> 11) * 0x1.0p-53; }

void oracle_sd_position_trials(const double *p, const double *q, long V, long N,
                               unsigned long long seed, int resid_sign,
                               long *hist, long *n_acc)
{
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    for (long i = 0; i < V; ++i) {
        double d = resid_sign >= 0 ? p[i] - q[i] : q[i] - p[i];
        w[i] = d > 0.0 ? d : 0.0;
        hist[i] = 0;
    }
    *n_acc = 0;
    unsigned long long s = seed;
    for (long n = 0; n < N; ++n) {
        long x = oracle_inverse_cdf(q, V, unif(&s), NULL);
        double r = unif(&s);
        if (r * q[x] < p[x]) {
            ++*n_acc;
        } else {
            long y = oracle_inverse_cdf(w, V, unif(&s), NULL);
            x = y >= 0 ? y : oracle_inverse_cdf(p, V, unif(&s), NULL);
        }
        ++hist[x];
    }
    free(w);
}
