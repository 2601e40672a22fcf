"""Shared pieces of the GPU parity tests: run a round through the C ABI, run the same round
through the oracle, compare to the stated bar.

Bar (from the benchmark spec): token ids, stop flags, accepted counts and corrected /
bonus tokens must be identical to the fp64 oracle wherever the oracle's decision margin is at
least MARGIN; entropies and probabilities must agree to REL.  Inside the margin the GPU's
choice must still be a valid neighbour (its cell touches the threshold within 2 * MARGIN).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle

MARGIN = 1e-6
REL = 1e-4


class Round:
    """Device buffers of one speculative round in the layout the C ABI chains through."""

    def __init__(self, svip, draft, target, u_sample, u_accept, u_resample, T, h):
        self.svip = svip
        self.draft = draft.cuda()
        self.target = target.cuda()
        self.B, self.k, self.V = self.draft.shape
        self.T, self.h = T, h
        dev = self.draft.device
        B, k = self.B, self.k
        self.u_sample = u_sample.cuda().contiguous()
        self.u_accept = u_accept.cuda().contiguous()
        self.u_resample = u_resample.cuda().contiguous()
        self.tokens = torch.full((B, k), -7, dtype=torch.int32, device=dev)
        self.entropy = torch.full((B, k), float("nan"), dtype=torch.float32, device=dev)
        self.q_tok = torch.full((B, k), float("nan"), dtype=torch.float32, device=dev)
        self.lse = torch.full((B, k), float("nan"), dtype=torch.float64, device=dev)
        self.stop = torch.zeros(B, dtype=torch.uint8, device=dev)
        self.stop_hist = torch.zeros(k, B, dtype=torch.uint8, device=dev)
        self.draft_len = torch.zeros(B, dtype=torch.int32, device=dev)
        self.n_accepted = torch.full((B,), -7, dtype=torch.int32, device=dev)
        self.next_token = torch.full((B,), -7, dtype=torch.int32, device=dev)
        self.accept_prob = torch.full((B, k), float("nan"), dtype=torch.float32, device=dev)
        self.ws = svip.new_workspace(B, k, self.V)

    def draft_all(self, chain=True, greedy=False):
        """k draft steps; chain=True threads the stop flags like Algorithm 1's drafting loop,
        chain=False evaluates every position of every row; greedy=True takes the first maximum."""
        for j in range(self.k):
            self.svip.draft_step(
                self.draft[:, j], temperature=self.T, h=self.h, step_j=j, k_max=self.k, greedy=greedy,
                u_sample=self.u_sample[:, j], stop_in=self.stop if chain else None,
                token_out=self.tokens[:, j], entropy_out=self.entropy[:, j],
                q_tok_out=self.q_tok[:, j], lse_out=self.lse[:, j],
                stop_out=self.stop if chain else self.stop_hist[j],
                draft_len_out=self.draft_len if chain else None, workspace=self.ws)
            if chain:
                self.stop_hist[j].copy_(self.stop)
        torch.cuda.synchronize()

    def verify(self, tokens=None, draft_len=None, lse="given"):
        tok = self.tokens if tokens is None else tokens
        dl = self.draft_len if draft_len is None else draft_len
        self.svip.verify(
            self.target, self.draft, temperature=self.T, draft_tokens=tok, draft_len=dl,
            draft_lse=None if lse is None else (self.lse if isinstance(lse, str) else lse),
            u_accept=self.u_accept, u_resample=self.u_resample,
            n_accepted_out=self.n_accepted, next_token_out=self.next_token,
            accept_prob_out=self.accept_prob, workspace=self.ws)
        torch.cuda.synchronize()


def f32(x):
    """The value the C ABI receives for a float argument, as a Python float."""
    return float(np.float32(x))


def cell_is_valid(prob, tok, u, tol):
    """True if token `tok` is a legitimate draw for uniform u up to `tol` of cumulative mass."""
    if tok < 0 or tok >= prob.size or not prob[tok] > 0:
        return False
    c = np.cumsum(prob)
    lo = c[tok - 1] if tok > 0 else 0.0
    t = u * c[-1]
    return lo - tol * c[-1] <= t <= c[tok] + tol * c[-1]


def check_draft_rows(draft_cpu, T, h, k_max, u_sample, gpu, rows=None, steps=None, stats=None):
    """Compare unchained draft-step outputs of `gpu` (a Round after draft_all(chain=False))
    with the oracle for rows x steps.  Returns a dict of counts."""
    B, k, V = draft_cpu.shape
    T, h = f32(T), f32(h)
    rows = range(B) if rows is None else rows
    steps = range(k) if steps is None else steps
    tok = gpu.tokens.cpu().numpy()
    ent = gpu.entropy.cpu().numpy()
    qt = gpu.q_tok.cpu().numpy()
    lse = gpu.lse.cpu().numpy()
    stop = gpu.stop_hist.cpu().numpy()
    st = dict(rows=0, tok_excluded=0, tok_excluded_diff=0, stop_excluded=0,
              max_rel_H=0.0, max_rel_q=0.0, max_abs_lse=0.0) if stats is None else stats
    for j in steps:
        idx = list(rows)
        z = draft_cpu[idx, j].double().numpy()
        o = oracle.draft_step(z, T, h, j, k_max, u_sample[idx, j].double().numpy())
        for n, b in enumerate(idx):
            st["rows"] += 1
            where = f"row {b} step {j}"
            if o.margin_s[n] >= MARGIN:
                assert tok[b, j] == o.token[n], f"{where}: token {tok[b, j]} != oracle {o.token[n]} (margin {o.margin_s[n]:.3g})"
            else:
                st["tok_excluded"] += 1
                if tok[b, j] != o.token[n]:
                    st["tok_excluded_diff"] += 1
                    p, _ = oracle.softmax_row(z[n], T)
                    assert cell_is_valid(p, int(tok[b, j]), float(u_sample[b, j]), 2 * MARGIN), where
            if o.margin_h[n] >= MARGIN:
                assert stop[j, b] == o.stop[n], f"{where}: stop {stop[j, b]} != oracle {o.stop[n]}"
            else:
                st["stop_excluded"] += 1
            H = o.entropy[n]
            relH = abs(ent[b, j] - H) / max(H, 1e-30) if H > 0 else abs(ent[b, j])
            assert relH <= REL or abs(ent[b, j] - H) <= 1e-9, f"{where}: H {ent[b, j]} vs {H}"
            st["max_rel_H"] = max(st["max_rel_H"], relH if H > 1e-9 else 0.0)
            st["max_abs_lse"] = max(st["max_abs_lse"], abs(lse[b, j] - o.lse[n]))
            assert abs(lse[b, j] - o.lse[n]) <= 1e-5 * max(1.0, abs(o.lse[n])), f"{where}: lse"
            if tok[b, j] == o.token[n]:
                relq = abs(qt[b, j] - o.q_tok[n]) / max(o.q_tok[n], 1e-300)
                assert relq <= REL or abs(qt[b, j] - o.q_tok[n]) <= 1e-37, f"{where}: q_tok {qt[b, j]} vs {o.q_tok[n]}"
                st["max_rel_q"] = max(st["max_rel_q"], relq if o.q_tok[n] > 1e-37 else 0.0)
    return st


def oracle_chain(draft_cpu, T, h, u_sample):
    """Algorithm 1's drafting loop through the oracle.  Returns tokens [B, k] (-1 where not
    drafted), draft_len [B], lse [B, k], and per (row, step) the stop-test margin and the
    sampler margin (inf where the row was no longer drafting)."""
    B, k, V = draft_cpu.shape
    T, h = f32(T), f32(h)
    tokens = np.full((B, k), -1, np.int64)
    lse = np.zeros((B, k))
    dl = np.zeros(B, np.int64)
    mh = np.full((B, k), np.inf)
    ms = np.full((B, k), np.inf)
    stop = np.zeros(B, np.uint8)
    for j in range(k):
        o = oracle.draft_step(draft_cpu[:, j].double().numpy(), T, h, j, k, u_sample[:, j].double().numpy(),
                              stop_in=stop)
        act = stop == 0
        tokens[act, j] = o.token[act]
        lse[act, j] = o.lse[act]
        dl[act] = j + 1
        mh[act, j] = o.margin_h[act]
        ms[act, j] = o.margin_s[act]
        stop = o.stop.copy()
    return tokens, dl, lse, mh, ms


def check_chain(gpu_tokens, gpu_len, tokens, dl, mh, ms, rows=None, draft_cpu=None, T=None, u_sample=None):
    """Chained draft outputs against oracle_chain, decision by decision: a row's draft length is
    compared when every stop test it went through was outside the margin, each token when its
    own draw (and the stop tests before it) were.  A token whose draw lies inside the margin must
    still be a cell that touches the threshold within 2 * MARGIN (checked when the logits are
    handed in: draft_cpu [len(rows), k, V], T, u_sample [len(rows), k]).  Returns counts."""
    B, k = tokens.shape
    rows = range(B) if rows is None else rows
    st = dict(rows=0, len_checked=0, tok_checked=0, tok_excluded=0, tok_excluded_diff=0)
    for n, b in enumerate(rows):
        st["rows"] += 1
        g = int(dl[n])
        stops_ok = np.concatenate([[True], np.cumprod(mh[n, :g] >= MARGIN).astype(bool)])   # [j]: tests before j
        if stops_ok[g]:
            st["len_checked"] += 1
            assert gpu_len[b] == g, f"row {b}: draft_len {gpu_len[b]} != {g}"
            assert (gpu_tokens[b, g:] == -1).all(), f"row {b}: steps after the stop must hold -1"
        for j in range(g):
            if not stops_ok[j]:
                break
            if ms[n, j] >= MARGIN:
                st["tok_checked"] += 1
                assert gpu_tokens[b, j] == tokens[n, j], f"row {b} step {j}: token {gpu_tokens[b, j]} != {tokens[n, j]}"
            else:
                st["tok_excluded"] += 1
                if gpu_tokens[b, j] != tokens[n, j]:
                    st["tok_excluded_diff"] += 1
                    if draft_cpu is not None:
                        q, _ = oracle.softmax_row(draft_cpu[n, j].double().numpy(), f32(T))
                        assert cell_is_valid(q, int(gpu_tokens[b, j]), float(u_sample[n, j]), 2 * MARGIN), \
                            f"row {b} step {j}: token {gpu_tokens[b, j]} is no neighbour of the oracle's {tokens[n, j]}"
    return st


def verify_weights(zp, zq, T, r, g):
    """The weights the correction or bonus token is drawn from when the first rejection is r:
    max(0, p_r - q_r) for r < g (Algorithm 4; p_r itself if that has no mass), p_g for r == g
    (the bonus step of Algorithm 1).  zp [k+1, V], zq [k, V] fp64.  Returns (weights, residual mass)."""
    p, _ = oracle.softmax_row(zp[r], T)
    if r < g:
        q, _ = oracle.softmax_row(zq[r], T)
        w = np.maximum(p - q, 0.0)
        W = float(w.sum())
        if W > 0.0:
            return w, W
    return p, 1.0


def check_verify(draft_cpu, target_cpu, T, tokens, draft_len, u_accept, u_resample, gpu, rows=None,
                 stats=None):
    """Compare verify outputs of `gpu` with the oracle for sequences `rows`.

    The accepted count is compared exactly whenever every acceptance test that shapes it (positions
    up to and including the first rejection) is at least MARGIN away from its threshold; inside
    that margin the GPU's count must be explained by flipping borderline tests only.  The
    corrected / bonus token is compared exactly when the counts agree and the draw is outside the
    margin; otherwise it must be a valid cell (within 2 * MARGIN) of the weights that belong to the
    GPU's own first rejection, and identical to the oracle's draw from those weights when that draw
    is outside the margin."""
    B, k, V = draft_cpu.shape
    T = f32(T)
    rows = list(range(B)) if rows is None else list(rows)
    nacc = gpu.n_accepted.cpu().numpy()
    nxt = gpu.next_token.cpu().numpy()
    ap = gpu.accept_prob.cpu().numpy()
    st = dict(seqs=0, excluded=0, excluded_diff=0, max_rel_a=0.0) if stats is None else stats
    for key in ("acc_excluded", "acc_excluded_diff", "tok_excluded", "tok_excluded_diff"):
        st.setdefault(key, 0)
    for b in rows:
        zp, zq = target_cpu[b].double().numpy(), draft_cpu[b].double().numpy()
        ua = u_accept[b:b + 1].double().numpy()
        o = oracle.verify(zp[None], zq[None], T, np.clip(tokens[b:b + 1], 0, V - 1), draft_len[b:b + 1],
                          ua, u_resample[b:b + 1].double().numpy())
        g = int(draft_len[b])
        st["seqs"] += 1
        where = f"sequence {b}"
        a_ref = o.accept_prob[0, :g]
        a_gpu = ap[b, :g].astype(np.float64)
        rel = np.abs(a_gpu - a_ref) / np.maximum(a_ref, 1e-300)
        ok = (rel <= REL) | (np.abs(a_gpu - a_ref) <= 1e-37)
        assert ok.all(), f"{where}: accept_prob {a_gpu} vs {a_ref}"
        if g:
            st["max_rel_a"] = max(st["max_rel_a"], float(np.where(a_ref > 1e-37, rel, 0).max()))
        assert np.isnan(ap[b, g:]).all(), f"{where}: accept_prob written beyond draft_len"
        assert 0 <= nacc[b] <= g and 0 <= nxt[b] < V, where
        r_o, r_g = int(o.n_accepted[0]), int(nacc[b])
        u_r = float(u_resample[b])
        if o.margin_accept[0] >= MARGIN:
            assert r_g == r_o, f"{where}: n_accepted {r_g} != {r_o} (margin {o.margin_accept[0]:.3g})"
        else:
            st["acc_excluded"] += 1
            if r_g != r_o:
                st["acc_excluded_diff"] += 1
                # only tests within 2 * MARGIN of their threshold may have gone the other way
                acc_o = (ua[0, :g] < a_ref) | (a_ref >= 1.0)
                near = o.margin_a[0, :g] < 2 * MARGIN
                assert (acc_o[:r_g] | near[:r_g]).all(), f"{where}: n_accepted {r_g} skips a clear rejection (oracle {r_o})"
                assert r_g == g or (not acc_o[r_g]) or near[r_g], f"{where}: n_accepted {r_g} stops at a clear accept"
        if r_g == r_o and o.margin_sample[0] >= MARGIN:
            assert nxt[b] == o.next_token[0], f"{where}: next_token {nxt[b]} != {o.next_token[0]} (margin {o.margin_sample[0]:.3g})"
        else:
            st["tok_excluded"] += 1
            w, W = verify_weights(zp, zq, T, r_g, g)
            ref_tok, ref_margin = (int(o.next_token[0]), float(o.margin_sample[0])) if r_g == r_o else oracle.inverse_cdf(w, u_r)
            if nxt[b] != ref_tok:
                st["tok_excluded_diff"] += 1
                assert ref_margin < MARGIN, f"{where}: next_token {nxt[b]} != {ref_tok} for first rejection {r_g}"
                # a residual with little mass magnifies the fp32 rounding of p and q (about 1e-7 each)
                tol = 2 * MARGIN + 4e-7 / W
                valid = cell_is_valid(w, int(nxt[b]), u_r, tol)
                if not valid and r_g < g and W < 1e-5:      # a residual this small may round to nothing: draw from p
                    p, _ = oracle.softmax_row(zp[r_g], T)
                    valid = cell_is_valid(p, int(nxt[b]), u_r, 2 * MARGIN)
                assert valid, f"{where}: next_token {nxt[b]} is no neighbour of {ref_tok}"
        if o.margin[0] < MARGIN:
            st["excluded"] += 1
            st["excluded_diff"] += int(r_g != r_o or nxt[b] != o.next_token[0])
    return st
