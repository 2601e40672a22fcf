"""GPU parity of the acceptance diagnostics (svip_pair_stats) against the fp64 oracle.

Tolerances: beta, H_q and H_{q,p} to REL; KL to REL * H_{q,p} absolute (it is the difference of two
entropies, each held to REL); the bounds to the same error carried through their square roots
(|sqrt a - sqrt b| <= min(sqrt|a - b|, |a - b| / (2 sqrt b))), and exactly consistent with the
GPU's own KL and H_q.  Quantities that are exactly 0 (identical rows, a one-token vocabulary) come out
within FLOOR of 0.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import svip_inputs as si
from helpers import REL, f32

pytestmark = pytest.mark.gpu

FLOOR = 3e-7     # nats: the logsumexps behind every term are resolved to about one fp32 ulp of a sum near 1


def _say(*a):
    print(*a, flush=True)


def _padded(x, mult=8):
    V = x.shape[-1]
    Vp = (V + mult - 1) // mult * mult
    buf = torch.full(x.shape[:-1] + (Vp,), 3.0e4, dtype=x.dtype)
    buf[..., :V] = x
    return buf.cuda()[..., :V]


def _run(svip, zp_dev, zq_dev, T, glen, c, lse=None):
    B, k, V = zq_dev.shape
    out = torch.full((B, k, svip.PAIR_NSTAT), -5.0, dtype=torch.float32, device=zq_dev.device)
    ws = svip.new_workspace(B, k, V)
    svip.pair_stats(zp_dev, zq_dev, temperature=T, draft_len=torch.as_tensor(glen, dtype=torch.int32).cuda(),
                    c=c, stats_out=out, workspace=ws, draft_lse=lse)
    torch.cuda.synchronize()
    assert svip.workspace_flags(ws) == 0
    return out.cpu().numpy().astype(np.float64)


def _sqrt_tol(delta, base):
    return min(math.sqrt(delta), delta / (2 * math.sqrt(base)) if base > 0 else math.inf)


def _check(g, zp, zq, T, glen, c, stats=None):
    B, k, V = zq.shape
    o = oracle.diagnostics(zp.double().numpy(), zq.double().numpy(), f32(T), glen, f32(c))
    st = dict(n=0, rel_beta=0.0, rel_hq=0.0, rel_hqp=0.0, abs_kl=0.0, abs_bound=0.0) if stats is None else stats
    cc = f32(c)
    for b in range(B):
        assert np.isnan(g[b, glen[b]:]).all(), f"seq {b}: entries past draft_len must be NaN"
        for j in range(int(glen[b])):
            beta, kl, hqp, hq, bo, bh, ba, ratio = o[b, j]
            gb, gk, ghqp, ghq, gbo, gbh, gba, gr = g[b, j]
            where = f"seq {b} pos {j}"
            st["n"] += 1
            assert abs(gb - beta) <= REL * beta + FLOOR, f"{where}: beta {gb} vs {beta}"
            assert abs(ghq - hq) <= REL * hq + FLOOR, f"{where}: H_q {ghq} vs {hq}"
            assert abs(ghqp - hqp) <= REL * hqp + FLOOR, f"{where}: H_qp {ghqp} vs {hqp}"
            d = REL * hqp + FLOOR
            assert abs(gk - kl) <= d, f"{where}: KL {gk} vs {kl}"
            assert abs(gbo - bo) <= _sqrt_tol(d / 2, kl / 2) + 1e-6, f"{where}: oracle bound {gbo} vs {bo}"
            assert abs(gbh - bh) <= _sqrt_tol(d, 1 - math.exp(-kl)) + 1e-6, f"{where}: BH bound {gbh} vs {bh}"
            assert abs(gba - ba) <= _sqrt_tol(cc * (REL * hq + FLOOR), cc * hq) + 1e-6, f"{where}: approx bound"
            if hq > 1e-6:
                assert abs(gr - ratio) <= 3 * REL * ratio + 1e-6, f"{where}: ratio {gr} vs {ratio}"
            # consistent with its own KL and H_q (fp32 outputs of fp64 arithmetic)
            assert abs(gbo - (1 - math.sqrt(gk / 2))) <= 1e-6 + 2e-7 / max(math.sqrt(gk), 1e-3)
            assert abs(gba - (1 - math.sqrt(cc * ghq))) <= 1e-6 + 2e-7 / max(math.sqrt(ghq), 1e-3)
            assert abs(ghqp - (ghq + gk)) <= 1e-6 * max(1.0, ghqp)
            assert 0.0 <= gb <= 1.0 and gk >= 0.0 and gbh > -1e-7
            st["rel_beta"] = max(st["rel_beta"], abs(gb - beta) / beta)
            st["rel_hq"] = max(st["rel_hq"], abs(ghq - hq) / max(hq, 1e-30))
            st["rel_hqp"] = max(st["rel_hqp"], abs(ghqp - hqp) / max(hqp, 1e-30))
            st["abs_kl"] = max(st["abs_kl"], abs(gk - kl))
            st["abs_bound"] = max(st["abs_bound"], abs(gbo - bo), abs(gbh - bh))
    return st


@pytest.mark.parametrize("name,rows,over", [
    ("cfg1", None, {}),
    ("cfg2", None, {}),
    ("cfg2", None, {"T": 0.7}),
    ("cfg3", [0, 1, 2, 3, 4], {}),
    ("cfg3", [5, 6, 7], {"noise": 0.2}),
    ("cfg4", [0, 1], {}),
])
@pytest.mark.parametrize("lse_mode", ["recompute", "given"])
def test_pair_stats_match_oracle(svip, name, rows, over, lse_mode):
    w = si.workload(name, **over)
    d = si.gen_batch(w, seed=2, rows=rows)
    B, k, V = d["draft"].shape
    glen = np.array([(7 * b + 3) % (k + 1) for b in range(B)], np.int64)
    glen[0] = k
    _say(f"pair stats parity {name} rows={rows} {over} lse={lse_mode}")
    zq_dev, zp_dev = d["draft"].cuda(), d["target"].cuda()
    lse = None
    if lse_mode == "given":     # the draft step's own logsumexps, as in a real round
        lse = torch.zeros(B, k, dtype=torch.float64, device=zq_dev.device)
        tok = torch.zeros(B, k, dtype=torch.int32, device=zq_dev.device)
        stop = torch.zeros(B, dtype=torch.uint8, device=zq_dev.device)
        ws = svip.new_workspace(B, k, V)
        for j in range(k):
            svip.draft_step(zq_dev[:, j], greedy=True, temperature=w.T, h=99.0, step_j=j, k_max=k,
                            token_out=tok[:, j], lse_out=lse[:, j], stop_out=stop, workspace=ws)
    g = _run(svip, zp_dev, zq_dev, w.T, glen, 0.15, lse)
    st = _check(g, d["target"], d["draft"], w.T, glen, 0.15)
    _say(f"  {st}")
    assert st["n"] == int(glen.sum())


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("V", [1, 2, 9, 1023, 2049, 4097, 40003, 262147])
def test_pair_stats_ragged_vocab(svip, V, dtype):
    gen = torch.Generator().manual_seed(300 + V)
    B, k = 3, 4
    zq = (torch.randn(B, k, V, generator=gen) * 2.0).to(dtype)
    zp = (zq.float() + torch.randn(B, k, V, generator=gen)).to(dtype)     # no bonus row: [B, k, V] is enough
    zp[1, 2] = zq[1, 2]                                                    # identical pair: beta 1, KL 0
    if V > 8:
        zq[2, 0, ::3] = float("-inf")                                      # masked in both models
        zp[2, 0, ::3] = float("-inf")
    glen = np.array([k, k, 2], np.int64)
    _say(f"pair stats ragged V={V} {dtype}")
    g = _run(svip, _padded(zp), _padded(zq), 0.9, glen, 0.3)
    zp_o = torch.cat([zp, zp[:, :1]], 1)                                   # the oracle's layout has a bonus row
    _check(g, zp_o, zq, 0.9, glen, 0.3)
    assert g[1, 2, 0] > 1 - 1e-6 and g[1, 2, 1] < 1e-6 and (abs(g[1, 2, 7] - 1) < 1e-5 or g[1, 2, 3] < 0.1) or V == 1
    if V == 1:
        assert abs(g[0, 0, 0] - 1.0) < FLOOR and g[0, 0, 3] < FLOOR and g[0, 0, 1] < FLOOR     # a one-token vocabulary


def test_pair_stats_host_errors(svip):
    dev = torch.device("cuda:0")
    z = torch.zeros(2, 3, 64, device=dev)
    out = torch.zeros(2, 3, svip.PAIR_NSTAT, device=dev)
    dl = torch.zeros(2, dtype=torch.int32, device=dev)
    ws = svip.new_workspace(2, 3, 64)
    with pytest.raises(svip.SvipError, match="PARAM"):
        svip.pair_stats(z, z, temperature=1.0, draft_len=dl, c=-1.0, stats_out=out, workspace=ws)
    with pytest.raises(svip.SvipError, match="PARAM"):
        svip.pair_stats(z, z, temperature=0.0, draft_len=dl, c=0.1, stats_out=out, workspace=ws)
    with pytest.raises(svip.SvipError, match="WORKSPACE"):
        svip.pair_stats(z, z, temperature=1.0, draft_len=dl, c=0.1, stats_out=out, workspace=ws[:512])
    svip.pair_stats(z, z, temperature=1.0, draft_len=dl, c=0.1, stats_out=out, workspace=ws)
    torch.cuda.synchronize()
    assert torch.isnan(out).all()                                          # draft_len 0 everywhere


def test_pair_stats_full_size(svip):
    """The benchmark's configuration, every position of the batch on the GPU, sampled sequences
    against the oracle."""
    w = si.workload("cfg3")
    d = si.gen_batch(w, seed=0)
    B, k, V = d["draft"].shape
    glen = np.full(B, k, np.int64)
    _say("pair stats full size cfg3")
    g = _run(svip, d["target"].cuda(), d["draft"].cuda(), w.T, glen, 0.15)
    assert np.isfinite(g).all()
    rows = [0, 17, 42, 63]
    st = _check(g[rows], d["target"][rows], d["draft"][rows], w.T, glen[rows], 0.15)
    _say(f"  {st}")
    # properties that hold for every position: both lower bounds stay below beta
    assert (g[..., 0] >= g[..., 4] - 1e-4).all() and (g[..., 0] >= g[..., 5] - 1e-4).all()


def test_pair_stats_and_greedy_are_bitwise_deterministic(svip):
    """Same inputs, different workspaces and a busy device in between: identical bits (no floating-point
    atomics, fixed combine order)."""
    w = si.workload("cfg2")
    d = si.gen_batch(w, seed=8)
    B, k, V = d["draft"].shape
    zq, zp = d["draft"].cuda(), d["target"].cuda()
    glen = torch.full((B,), k, dtype=torch.int32).cuda()
    outs = []
    for rep in range(3):
        stats = torch.empty(B, k, svip.PAIR_NSTAT, device="cuda")
        svip.pair_stats(zp, zq, temperature=0.9, draft_len=glen, c=0.2, stats_out=stats, workspace=svip.new_workspace(B, k, V))
        tok = torch.zeros(B, dtype=torch.int32, device="cuda")
        ent = torch.zeros(B, device="cuda")
        lse = torch.zeros(B, dtype=torch.float64, device="cuda")
        stop = torch.zeros(B, dtype=torch.uint8, device="cuda")
        svip.draft_step(zq[:, 3], greedy=True, temperature=0.9, h=1.0, step_j=3, k_max=k, token_out=tok,
                        entropy_out=ent, lse_out=lse, stop_out=stop, workspace=svip.new_workspace(B, k, V))
        na = torch.zeros(B, dtype=torch.int32, device="cuda")
        nx = torch.zeros(B, dtype=torch.int32, device="cuda")
        svip.verify_greedy(zp, draft_tokens=torch.zeros(B, k, dtype=torch.int32, device="cuda"), draft_len=glen,
                           n_accepted_out=na, next_token_out=nx, workspace=svip.new_workspace(B, k, V))
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (stats, tok, ent, lse, stop, na, nx)])
        torch.randn(1 << 22, device="cuda").sum().item()
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
