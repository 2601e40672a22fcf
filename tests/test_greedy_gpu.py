"""GPU parity of greedy decoding (Algorithms 3 and 5, greedy drafting) against the fp64 oracle.

Token ids, accepted counts and corrected / bonus tokens come from comparisons only, so they
must be identical for every row, ties included (the first maximum wins on both sides); the
stop flag is compared outside the oracle's margin, entropies and probabilities to REL.
"""
import numpy as np
import pytest
import torch

import oracle
import svip_inputs as si
from helpers import MARGIN, REL, f32

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _padded(x, mult=8):
    """Copy of x[..., V] inside a buffer whose row stride is a multiple of `mult` elements."""
    V = x.shape[-1]
    Vp = (V + mult - 1) // mult * mult
    buf = torch.full(x.shape[:-1] + (Vp,), 3.0e4, dtype=x.dtype)    # huge finite padding: must never be read
    buf[..., :V] = x
    return buf.cuda()[..., :V]


def _greedy_draft(svip, z_dev, T, h, j, k, stop_in=None):
    B = z_dev.shape[0]
    dev = z_dev.device
    out = dict(token=torch.full((B,), -7, dtype=torch.int32, device=dev),
               entropy=torch.full((B,), float("nan"), dtype=torch.float32, device=dev),
               q_tok=torch.full((B,), float("nan"), dtype=torch.float32, device=dev),
               lse=torch.full((B,), float("nan"), dtype=torch.float64, device=dev),
               stop=torch.zeros(B, dtype=torch.uint8, device=dev),
               draft_len=torch.zeros(B, dtype=torch.int32, device=dev))
    ws = svip.new_workspace(B, k, z_dev.shape[1])
    svip.draft_step(z_dev, greedy=True, temperature=T, h=h, step_j=j, k_max=k, stop_in=stop_in,
                    token_out=out["token"], entropy_out=out["entropy"], q_tok_out=out["q_tok"],
                    lse_out=out["lse"], stop_out=out["stop"], draft_len_out=out["draft_len"], workspace=ws)
    torch.cuda.synchronize()
    assert svip.workspace_flags(ws) == 0
    return {n: t.cpu().numpy() for n, t in out.items()}


def _check_draft(g, z_cpu, T, h, j, k, stop_in=None):
    o = oracle.draft_step_greedy(z_cpu.double().numpy(), f32(T), f32(h), j, k, stop_in=stop_in)
    B = z_cpu.shape[0]
    act = np.ones(B, bool) if stop_in is None else (np.asarray(stop_in) == 0)
    assert (g["token"][act] == o.token[act]).all(), (g["token"], o.token)
    assert (g["token"][~act] == -1).all() and (g["stop"][~act] == 1).all()
    sure = act & (o.margin_h >= MARGIN)
    assert (g["stop"][sure] == o.stop[sure]).all()
    for b in np.flatnonzero(act):
        H = o.entropy[b]
        assert abs(g["entropy"][b] - H) <= REL * H + 1e-9, (b, g["entropy"][b], H)
        assert abs(g["q_tok"][b] - o.q_tok[b]) <= REL * o.q_tok[b], (b, g["q_tok"][b], o.q_tok[b])
        assert abs(g["lse"][b] - o.lse[b]) <= 1e-5 * max(1.0, abs(o.lse[b]))
        assert g["draft_len"][b] == j + 1
    return int(sure.sum())


def _plant_ties(z, gen):
    """Give every row several copies of a value above its maximum, at seeded places that include
    vector, tile and slice boundaries; returns nothing (z is edited in place)."""
    V = z.shape[-1]
    flat = z.reshape(-1, V)
    for r in range(flat.shape[0]):
        top = float(flat[r].float().max()) + 1.0
        n = int(torch.randint(2, 6, (1,), generator=gen))
        pos = torch.randint(0, V, (n,), generator=gen)
        if r % 3 == 0:
            pos[0] = V - 1
        if r % 3 == 1 and V > 2048:
            pos[0] = 2047
            pos[1] = 2048
        flat[r, pos] = top


@pytest.mark.parametrize("name,rows", [("cfg1", None), ("cfg2", None), ("cfg3", [0, 1, 2, 3, 4, 5, 6, 7]),
                                       ("cfg4", [0, 1, 2])])
def test_greedy_draft_step_matches_oracle(svip, name, rows):
    w = si.workload(name)
    d = si.gen_batch(w, seed=3, rows=rows)
    _say(f"greedy draft parity {name} rows={rows}")
    sure = 0
    for j in (0, w.k // 2, w.k - 1):
        z = d["draft"][:, j].contiguous()
        for h in (w.h, 0.3):
            g = _greedy_draft(svip, z.cuda(), w.T, h, j, w.k)
            sure += _check_draft(g, z, w.T, h, j, w.k)
    assert sure > 0


@pytest.mark.parametrize("V,dtype", [(1, torch.float32), (5, torch.bfloat16), (2047, torch.bfloat16),
                                     (2049, torch.bfloat16), (4100, torch.float32), (32003, torch.float32),
                                     (50257, torch.bfloat16), (262147, torch.bfloat16), (4100, torch.float16),
                                     (50257, torch.float16)])
def test_greedy_ties_and_ragged_vocab(svip, V, dtype):
    """Equal maxima anywhere in the row (bf16 rows have many): the smallest index wins, in the
    draft step and in verification; ragged V exercises the checked last tile."""
    gen = torch.Generator().manual_seed(1000 + V)
    B, k = 5, 3
    zq = (torch.randn(B, k, V, generator=gen) * 2.0).to(dtype)
    zp = (torch.randn(B, k + 1, V, generator=gen) * 2.0).to(dtype)
    _plant_ties(zq, gen)
    _plant_ties(zp, gen)
    zp[0, 1] = zq[0, 1]                                  # a position whose argmax agrees
    _say(f"greedy ties V={V} {dtype}")
    zq_dev, zp_dev = _padded(zq), _padded(zp)
    for j in range(k):
        g = _greedy_draft(svip, zq_dev[:, j], 0.8, 1.5, j, k)
        _check_draft(g, zq[:, j], 0.8, 1.5, j, k)
    # verification: tokens = the target's own argmax for some positions, the draft's for others
    tok = np.zeros((B, k), np.int64)
    for b in range(B):
        for j in range(k):
            src = zp if (b + j) % 2 == 0 else zq
            tok[b, j] = oracle.argmax_row(src[b, j].double().numpy())
    glen = np.array([k, k, 2, 1, 0], np.int64)[:B]
    nacc, nxt = _verify(svip, zp_dev, tok, glen)
    o_acc, o_next = oracle.verify_greedy(zp.double().numpy(), tok, glen)
    assert (nacc == o_acc).all() and (nxt == o_next).all(), (nacc, o_acc, nxt, o_next)


def _verify(svip, zp_dev, tok, glen, expect_flags=0):
    B, kp1, V = zp_dev.shape
    dev = zp_dev.device
    nacc = torch.full((B,), -7, dtype=torch.int32, device=dev)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=dev)
    ws = svip.new_workspace(B, kp1 - 1, V)
    svip.verify_greedy(zp_dev, draft_tokens=torch.as_tensor(tok, dtype=torch.int32).cuda().contiguous(),
                       draft_len=torch.as_tensor(glen, dtype=torch.int32).cuda(),
                       n_accepted_out=nacc, next_token_out=nxt, workspace=ws)
    torch.cuda.synchronize()
    assert svip.workspace_flags(ws) == expect_flags
    return nacc.cpu().numpy(), nxt.cpu().numpy()


@pytest.mark.parametrize("name,rows", [("cfg2", None), ("cfg3", [0, 1, 2, 3, 4, 5]), ("cfg4", [0, 1])])
def test_greedy_round_matches_oracle(svip, name, rows):
    """Chained greedy drafting (Algorithm 1 with argmax) then greedy verification, each fed by the
    GPU's own outputs; the synthetic target is the draft plus noise, so accepted prefixes of every
    length occur."""
    w = si.workload(name, noise=0.5)
    d = si.gen_batch(w, seed=5, rows=rows)
    B, k, V = d["draft"].shape
    _say(f"greedy round parity {name} rows={rows}")
    zq_dev, zp_dev = d["draft"].cuda(), d["target"].cuda()
    dev = zq_dev.device
    tokens = torch.full((B, k), -7, dtype=torch.int32, device=dev)
    lse = torch.zeros(B, k, dtype=torch.float64, device=dev)
    stop = torch.zeros(B, dtype=torch.uint8, device=dev)
    dl = torch.zeros(B, dtype=torch.int32, device=dev)
    ws = svip.new_workspace(B, k, V)
    for j in range(k):
        svip.draft_step(zq_dev[:, j], greedy=True, temperature=w.T, h=w.h, step_j=j, k_max=k, stop_in=stop,
                        token_out=tokens[:, j], lse_out=lse[:, j], stop_out=stop, draft_len_out=dl, workspace=ws)
    torch.cuda.synchronize()
    g_tok, g_dl = tokens.cpu().numpy().astype(np.int64), dl.cpu().numpy().astype(np.int64)
    # oracle chain
    o_stop = np.zeros(B, np.uint8)
    o_dl = np.zeros(B, np.int64)
    ok = np.ones(B, bool)              # every stop test so far was outside the margin
    for j in range(k):
        o = oracle.draft_step_greedy(d["draft"][:, j].double().numpy(), f32(w.T), f32(w.h), j, k, stop_in=o_stop)
        act = o_stop == 0
        chk = act & ok
        assert (g_tok[chk, j] == o.token[chk]).all(), f"step {j}"
        o_dl[act] = j + 1
        ok &= ~act | (o.margin_h >= MARGIN)
        o_stop = o.stop.copy()
    assert (g_dl[ok] == o_dl[ok]).all() and ok.sum() >= B // 2
    _say(f"  draft_len {g_dl.tolist()} checked {int(ok.sum())}/{B}")
    nacc, nxt = _verify(svip, zp_dev, np.where(g_tok < 0, 0, g_tok), g_dl)
    o_acc, o_next = oracle.verify_greedy(d["target"].double().numpy(), np.where(g_tok < 0, 0, g_tok), g_dl)
    assert (nacc == o_acc).all() and (nxt == o_next).all(), (nacc, o_acc, nxt, o_next)
    _say(f"  n_accepted {nacc.tolist()}")


def test_greedy_verify_edge_cases(svip):
    """k above one wave with everything accepted past position 64; draft_len 0; a rejection at the
    first and at the last position; -inf masked logits; out-of-range inputs set flags."""
    gen = torch.Generator().manual_seed(77)
    B, k, V = 6, 100, 3001
    zp = (torch.randn(B, k + 1, V, generator=gen) * 3.0).to(torch.bfloat16)
    zp[2, :, ::2] = float("-inf")                      # half the vocabulary masked
    zp[3, 5, :] = float("-inf")
    zp[3, 5, 17] = -5.0                                # a single live logit
    am = np.array([[oracle.argmax_row(zp[b, j].double().numpy()) for j in range(k + 1)] for b in range(B)])
    tok = am[:, :k].copy()
    glen = np.array([k, 0, k, k, 70, k], np.int64)
    tok[4, 69] = (tok[4, 69] + 1) % V                  # rejected at the last drafted position
    tok[5, 0] = (tok[5, 0] + 1) % V                    # rejected at once
    _say("greedy verify edges")
    zp_dev = _padded(zp)
    nacc, nxt = _verify(svip, zp_dev, tok, glen)
    o_acc, o_next = oracle.verify_greedy(zp.double().numpy(), tok, glen)
    assert (nacc == o_acc).all() and (nxt == o_next).all(), (nacc, o_acc, nxt, o_next)
    assert nacc.tolist() == [k, 0, k, k, 69, 0]
    assert nxt[3] == am[3, k] and nxt[1] == am[1, 0]
    # flags: a token outside the vocabulary is a rejection and is reported; so is a bad draft_len
    bad = tok.copy()
    bad[0, 3] = V + 5
    nacc, _ = _verify(svip, zp_dev, bad, glen, expect_flags=svip.FLAG_BAD_TOKEN)
    assert nacc[0] == 3
    gl2 = glen.copy()
    gl2[1] = k + 9
    nacc, _ = _verify(svip, zp_dev, tok, gl2, expect_flags=svip.FLAG_BAD_DRAFT_LEN)
    assert nacc[1] == k                                # clamped to k_max


def test_greedy_stopped_rows_are_skipped(svip):
    gen = torch.Generator().manual_seed(5)
    z = torch.randn(7, 4099, generator=gen)
    stop_in = np.array([0, 1, 0, 0, 1, 1, 0], np.uint8)
    g = _greedy_draft(svip, _padded(z), 1.0, 2.0, 1, 4, stop_in=torch.as_tensor(stop_in).cuda())
    _check_draft(g, z, 1.0, 2.0, 1, 4, stop_in=stop_in)


def test_greedy_full_size_round(svip):
    """The benchmark's configuration (cfg3: B = 64, V = 128256, bf16, k = 16): greedy verification
    of the whole batch against the oracle, and greedy drafting on sampled rows."""
    w = si.workload("cfg3")
    d = si.gen_batch(w, seed=0)
    B, k, V = d["draft"].shape
    _say("greedy full size cfg3")
    zp_dev = d["target"].cuda()
    tok = np.zeros((B, k), np.int64)
    zq = d["draft"]
    for b in range(B):
        src = d["target"] if b % 2 == 0 else zq        # even rows agree everywhere, odd rows follow the draft
        tok[b] = src[b, :k].float().argmax(dim=-1).numpy()
    glen = np.array([(5 * b) % (k + 1) for b in range(B)], np.int64)
    nacc, nxt = _verify(svip, zp_dev, tok, glen)
    o_acc, o_next = oracle.verify_greedy(d["target"].double().numpy(), tok, glen)
    assert (nacc == o_acc).all() and (nxt == o_next).all()
    _say(f"  n_accepted {nacc.tolist()}")
    for j in (0, 9):
        z = zq[:, j].contiguous()
        g = _greedy_draft(svip, z.cuda(), w.T, 4.0, j, k)
        _check_draft(g, z, w.T, 4.0, j, k)
