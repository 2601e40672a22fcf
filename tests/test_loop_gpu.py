"""GPU parity of the decoding loop (svip_loop_init / svip_loop_run) against the oracle's loop.

Every round the GPU logs (position, limit, drafted, accepted).  The integer bookkeeping between
rounds (positions, the length rule, counters, produced tokens) must be exact.  Each round is also
replayed through the oracle from the GPU's own round state ("teacher forced"), and its decisions must
agree wherever the oracle's smallest margin in that round is at least MARGIN (with vocabularies of
32K and more a round often holds a draw within 1e-6 of a cell edge; those rounds are counted and may
differ); sequences all of whose rounds agreed must match the oracle's free-running loop token for
token.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import svip_inputs as si
from helpers import MARGIN, cell_is_valid, f32

pytestmark = pytest.mark.gpu

POLICIES = {
    # name: (h, gamma0, gamma_max, inc, dec)
    "svip": (3.0, 12, 12, 0, 0),
    "constant": (math.inf, 5, 5, 0, 0),
    "heuristic": (math.inf, 5, 12, 2, 1),
}


def _say(*a):
    print(*a, flush=True)


def _run(svip, tr, w, policy, max_new, greedy=False, check_every=4, chunks=None, n0=0):
    h, g0, gmax, inc, dec = policy
    R = tr["u_sample"].shape[0]
    loop = svip.Loop(tr["target"].cuda(), tr["draft"].cuda(), temperature=w.T, h=h, gamma0=g0, gamma_max=gmax,
                     gamma_inc=inc, gamma_dec=dec, n0=n0, max_new=max_new, rounds=R, greedy=greedy,
                     u_sample=tr["u_sample"][:, :, :gmax].contiguous().cuda(),
                     u_accept=tr["u_accept"][:, :, :gmax].contiguous().cuda(),
                     u_resample=tr["u_resample"].cuda(), check_every=check_every)
    if chunks:
        running = 1
        while running and loop.next_round < R:
            _, running = loop.run(chunks)
    else:
        _, running = loop.run()
    assert running == 0 and loop.flags() == 0
    # a sequence takes part in every round until it has finished, so the longest-running one saw all of them: the
    # round the loop launches ahead of the last count (and finds nothing to do in) must not be counted
    assert loop.next_round == int(loop.state[:, 3].max())
    return dict(state=loop.state.cpu().numpy(), out=loop.out_tokens.cpu().numpy(),
                log=loop.round_log.cpu().numpy()[:loop.next_round], rounds=loop.next_round)


def _check(res, tr, w, policy, max_new, greedy=False, n0=0):
    h, g0, gmax, inc, dec = policy
    B, L, V = tr["draft"].shape
    T, hh = f32(w.T), f32(h)
    log, out, state = res["log"], res["out"], res["state"]
    st = dict(rounds=0, in_margin=0, in_margin_diff=0, free_checked=0)
    for b in range(B):
        zq, zp = tr["draft"][b].double().numpy(), tr["target"][b].double().numpy()
        us = tr["u_sample"][:, b, :gmax].double().numpy()
        ua = tr["u_accept"][:, b, :gmax].double().numpy()
        ur = tr["u_resample"][:, b].double().numpy()
        pos, cap, produced, drafted, accepted, rounds = n0, g0, 0, 0, 0, 0
        clean = True
        for r in range(res["rounds"]):
            if pos - n0 >= max_new or pos + cap + 1 > L:
                assert (log[r:, b] == -1).all(), f"seq {b}: rounds after the end must be idle"
                break
            lp, lc, g, na = log[r, b]
            assert (lp, lc) == (pos, cap), f"seq {b} round {r}: state {(lp, lc)} != {(pos, cap)}"
            assert 1 <= g <= cap and 0 <= na <= g
            o = oracle.generate(zp, zq, T, pos, 1, hh, cap, cap, 0, 0, us[r:r + 1], ua[r:r + 1], ur[r:r + 1],
                                greedy=greedy, max_rounds=1)
            seg = out[b, produced:produced + na + 1]
            st["rounds"] += 1
            same = (g, na) == tuple(o.log[0, 2:4]) and seg.tolist() == o.tokens.tolist()
            if o.min_margin >= MARGIN:
                assert same, f"seq {b} round {r}: {(g, na, seg.tolist())} != {(tuple(o.log[0, 2:4]), o.tokens.tolist())}"
            else:               # some decision of this round sits on a threshold: either side is legitimate
                st["in_margin"] += 1
                if not same:
                    st["in_margin_diff"] += 1
                    clean = False
                    assert ((seg >= 0) & (seg < V)).all()
                    # whatever side a borderline decision fell on, every accepted draft token must still be a
                    # legitimate draw of its own row for its own uniform (a cell within 2 * MARGIN of u)
                    if not greedy:
                        for j in range(int(na)):
                            q, _ = oracle.softmax_row(zq[pos + j], T)
                            assert cell_is_valid(q, int(seg[j]), float(us[r, j]), 2 * MARGIN), \
                                f"seq {b} round {r}: accepted token {seg[j]} at step {j} is no valid draw"
            produced += na + 1
            drafted += g
            accepted += na
            rounds += 1
            pos += na + 1
            cap = min(max(cap + (inc if na == g else -dec), 1), gmax)
        assert state[b].tolist() == [pos, cap, 1, rounds, drafted, accepted, produced, n0], f"seq {b}: state"
        assert (out[b, produced:] == -1).all()
        if clean:       # every round agreed: the free-running oracle loop must give the same sequence
            o = oracle.generate(zp, zq, T, n0, max_new, hh, g0, gmax, inc, dec, us, ua, ur, greedy=greedy)
            assert o.tokens.tolist() == out[b, :produced].tolist()
            assert o.log[:, :4].tolist() == log[:rounds, b].tolist()
            st["free_checked"] += 1
    return st


def _metrics(state):
    rounds, drafted, accepted, produced = (state[:, i].sum() for i in (3, 4, 5, 6))
    return dict(mean_draft_len=drafted / rounds, accept_rate=accepted / max(drafted, 1), tokens_per_round=produced / rounds)


@pytest.mark.parametrize("policy", ["svip", "constant", "heuristic"])
@pytest.mark.parametrize("name,rows,L,max_new", [("cfg2", [0, 1, 2, 3, 4, 5], 72, 48), ("cfg4", [0, 1, 2], 60, 40)])
def test_loop_matches_oracle(svip, name, rows, L, max_new, policy):
    w = si.workload(name, noise=0.7)
    tr = si.gen_trace(w, L, rounds=max_new, gamma_max=12, seed=4, rows=rows)
    _say(f"loop parity {name} rows={rows} policy={policy}")
    res = _run(svip, tr, w, POLICIES[policy], max_new)
    st = _check(res, tr, w, POLICIES[policy], max_new)
    _say(f"  {st} {_metrics(res['state'])}")
    assert st["free_checked"] >= 1 and st["in_margin_diff"] <= 0.05 * st["rounds"]


def test_loop_greedy_matches_oracle(svip):
    w = si.workload("cfg2", noise=0.3)
    tr = si.gen_trace(w, 64, rounds=40, gamma_max=12, seed=6, rows=[0, 1, 2, 3])
    for policy in ("svip", "heuristic"):
        _say(f"greedy loop parity policy={policy}")
        res = _run(svip, tr, w, POLICIES[policy], 40, greedy=True)
        st = _check(res, tr, w, POLICIES[policy], 40, greedy=True)
        _say(f"  {st} {_metrics(res['state'])}")
        assert st["free_checked"] >= 2


def test_loop_is_independent_of_how_it_is_driven(svip):
    """Rounds run one call at a time, or with the drafting phase never / always polled, give the same
    tokens, log and state bit for bit."""
    w = si.workload("cfg2", noise=0.7)
    tr = si.gen_trace(w, 72, rounds=48, gamma_max=12, seed=9, rows=[3, 4, 5])
    ref = _run(svip, tr, w, POLICIES["svip"], 48, check_every=4)
    for kw in (dict(check_every=0), dict(check_every=1), dict(chunks=1), dict(chunks=5)):
        res = _run(svip, tr, w, POLICIES["svip"], 48, **kw)
        assert res["rounds"] == ref["rounds"]
        for key in ("state", "out", "log"):
            assert (res[key] == ref[key]).all(), (kw, key)


def test_loop_edges(svip):
    w = si.workload("cfg1")
    tr = si.gen_trace(w, 20, rounds=8, gamma_max=5, seed=1)
    # nothing to produce: no round runs
    res = _run(svip, tr, w, (math.inf, 5, 5, 0, 0), 0)
    assert res["rounds"] == 0 and res["state"][0].tolist() == [0, 5, 1, 0, 0, 0, 0, 0]
    # a start position from which the trace cannot hold one more round
    res = _run(svip, tr, w, (math.inf, 5, 5, 0, 0), 8, n0=15)
    assert res["rounds"] == 0 and res["state"][0, 2] == 1
    # the last round may not start past L - limit - 1: positions 3, 9 run, 15 does not
    res = _run(svip, tr, w, (math.inf, 5, 5, 0, 0), 100 if False else 8, n0=3)
    _check(res, tr, w, (math.inf, 5, 5, 0, 0), 8, n0=3)
    # host-side argument checks
    with pytest.raises(svip.SvipError, match="SHAPE"):
        svip.Loop(tr["target"].cuda(), tr["draft"].cuda(), temperature=1.0, h=1.0, gamma0=6, gamma_max=5,
                  max_new=4, rounds=8, u_sample=tr["u_sample"].cuda(), u_accept=tr["u_accept"].cuda(),
                  u_resample=tr["u_resample"].cuda())
    with pytest.raises(svip.SvipError, match="PARAM"):
        svip.Loop(tr["target"].cuda(), tr["draft"].cuda(), temperature=1.0, h=1.0, gamma0=5, gamma_max=5,
                  gamma_dec=-1, max_new=4, rounds=8, u_sample=tr["u_sample"].cuda(),
                  u_accept=tr["u_accept"].cuda(), u_resample=tr["u_resample"].cuda())


def test_loop_full_size_as_benchmarked(svip):
    """The benchmark's loop configuration (cfg4_loop traces: B = 8, V = 151936, bf16, limit 40, 96 new
    tokens): the whole batch runs on the GPU, every round of two sampled sequences is replayed through
    the oracle, and the bookkeeping of all sequences is checked."""
    w = si.workload("cfg4_loop")
    max_new, gmax = 96, 40
    tr = si.gen_trace(w, max_new + gmax + 1, rounds=max_new, gamma_max=gmax, seed=0)
    policy = (w.h, gmax, gmax, 0, 0)
    _say("loop full size cfg4_loop")
    res = _run(svip, tr, w, policy, max_new)
    st = res["state"]
    assert (st[:, 2] == 1).all() and (st[:, 6] >= max_new).all() and (st[:, 6] < max_new + gmax + 1).all()
    assert (st[:, 0] == st[:, 7] + st[:, 6]).all() and (st[:, 5] + st[:, 3] == st[:, 6]).all()
    rows = [1, 6]
    sub = dict(draft=tr["draft"][rows], target=tr["target"][rows], u_sample=tr["u_sample"][:, rows],
               u_accept=tr["u_accept"][:, rows], u_resample=tr["u_resample"][:, rows])
    sub_res = dict(state=st[rows], out=res["out"][rows], log=res["log"][:, rows], rounds=res["rounds"])
    chk = _check(sub_res, sub, w, policy, max_new)
    _say(f"  {chk} {_metrics(st)}")
    assert chk["in_margin_diff"] <= 0.05 * chk["rounds"]
