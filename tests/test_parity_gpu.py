"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import svip_inputs as si
from helpers import MARGIN, Round, check_draft_rows, check_verify, oracle_chain

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _batch(name, rows=None, **over):
    w = si.workload(name, **over)
    return w, si.gen_batch(w, seed=0, rows=rows)


@pytest.mark.parametrize("name,rows,over", [
    ("cfg1", None, {}),
    ("cfg2", None, {}),
    ("cfg2", None, {"T": 0.7}),
    ("cfg3", [0, 1, 2, 3, 4, 5], {}),
    ("cfg3", [6, 7, 8], {"T": 0.7}),
    ("cfg4", [0, 1], {}),
])
def test_draft_step_every_position(svip, name, rows, over):
    """Every (row, position) of the workload, no stop chaining, also at the paper's h grid."""
    w, d = _batch(name, rows, **over)
    _say(f"draft parity {name} rows={rows} {over}")
    for h in (w.h, 0.3):
        r = Round(svip, d["draft"], d["target"], d["u_sample"], d["u_accept"], d["u_resample"], w.T, h)
        r.draft_all(chain=False)
        st = check_draft_rows(d["draft"], w.T, h, w.k, d["u_sample"], r)
        _say(f"  h={h}: {st}")
        assert st["tok_excluded"] <= 0.5 * st["rows"]


@pytest.mark.parametrize("name,rows,over", [
    ("cfg1", None, {}),
    ("cfg2", None, {}),
    ("cfg3", [10, 11, 12, 13], {}),
    ("cfg4", [2, 3, 4], {}),
    ("cfg2", None, {"T": 0.7, "h": 2.0}),
])
def test_round_chained_draft_then_verify(svip, name, rows, over):
    """Algorithm 1 round: chained draft steps, then verify fed by the GPU's own draft outputs."""
    w, d = _batch(name, rows, **over)
    _say(f"round parity {name} rows={rows} {over}")
    r = Round(svip, d["draft"], d["target"], d["u_sample"], d["u_accept"], d["u_resample"], w.T, w.h)
    r.draft_all(chain=True)
    tokens, dl, lse, margin = oracle_chain(d["draft"], w.T, w.h, d["u_sample"])
    g_tok = r.tokens.cpu().numpy()
    g_dl = r.draft_len.cpu().numpy()
    sure = margin >= MARGIN
    for b in np.nonzero(sure)[0]:
        assert g_dl[b] == dl[b], f"row {b}: draft_len {g_dl[b]} != {dl[b]}"
        assert (g_tok[b, :dl[b]] == tokens[b, :dl[b]]).all(), f"row {b}: tokens"
        assert (g_tok[b, dl[b]:] == -1).all(), f"row {b}: steps after the stop must hold -1"
    assert (r.stop.cpu().numpy() == 1).all()          # the cap stops everyone by step k-1
    _say(f"  draft_len {g_dl.tolist()} excluded rows {int((~sure).sum())}")
    # verify, fed by the GPU's own tokens / lengths / lse, for rows whose drafts matched
    r.verify(lse="given")
    st = check_verify(d["draft"], d["target"], w.T, g_tok.astype(np.int64), g_dl.astype(np.int64),
                      d["u_accept"], d["u_resample"], r, rows=np.nonzero(sure)[0])
    _say(f"  verify {st}")


@pytest.mark.parametrize("name,rows,over,glen", [
    ("cfg1", None, {}, "full"),
    ("cfg2", None, {}, "full"),
    ("cfg2", None, {"T": 0.7}, "ragged"),
    ("cfg3", [20, 21, 22, 23], {}, "full"),
    ("cfg3", [24, 25, 26], {"T": 0.7}, "ragged"),
    ("cfg4", [5, 6], {}, "full"),
])
@pytest.mark.parametrize("lse_mode", ["given", "recompute"])
def test_verify_all_positions(svip, name, rows, over, glen, lse_mode):
    """Verify with oracle-made draft tokens over every position (draft_len = k or ragged)."""
    w, d = _batch(name, rows, **over)
    _say(f"verify parity {name} rows={rows} {over} {glen} lse={lse_mode}")
    B, k, V = d["draft"].shape
    # drafts: oracle draft tokens at every position (stop test ignored)
    import oracle
    tokens = np.zeros((B, k), np.int64)
    lse = np.zeros((B, k))
    for j in range(k):
        o = oracle.draft_step(d["draft"][:, j].double().numpy(), w.T, 99.0, j, k + 1, d["u_sample"][:, j].double().numpy())
        tokens[:, j], lse[:, j] = o.token, o.lse
    if glen == "full":
        dl = np.full(B, k, np.int64)
    else:
        dl = np.array([(3 * b + 1) % (k + 1) for b in range(B)], np.int64)
        dl[0] = 0
    r = Round(svip, d["draft"], d["target"], d["u_sample"], d["u_accept"], d["u_resample"], w.T, w.h)
    tok_dev = torch.from_numpy(tokens).int().cuda()
    dl_dev = torch.from_numpy(dl).int().cuda()
    r.verify(tokens=tok_dev, draft_len=dl_dev,
             lse=torch.from_numpy(lse).cuda() if lse_mode == "given" else None)
    st = check_verify(d["draft"], d["target"], w.T, tokens, dl, d["u_accept"], d["u_resample"], r)
    _say(f"  {st} n_accepted={r.n_accepted.cpu().tolist()}")
    assert st["excluded"] <= 0.5 * st["seqs"] + 1


def test_bitwise_determinism(svip):
    w, d = _batch("cfg2")
    outs = []
    for _ in range(2):
        r = Round(svip, d["draft"], d["target"], d["u_sample"], d["u_accept"], d["u_resample"], w.T, w.h)
        r.draft_all(chain=True)
        r.verify()
        outs.append([t.clone() for t in (r.tokens, r.entropy, r.q_tok, r.lse, r.draft_len,
                                          r.n_accepted, r.next_token, r.accept_prob)])
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
