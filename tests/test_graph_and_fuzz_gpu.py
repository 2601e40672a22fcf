"""HIP-graph replays of the path and a seeded sweep over shapes, against eager runs and the oracle."""
import numpy as np
import pytest
import torch

import oracle
import svip_inputs as si
from helpers import MARGIN, REL, Round, check_chain, check_draft_rows, check_verify, f32, oracle_chain

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def test_graph_replays_match_eager_runs(svip):
    """A whole round (chained draft steps + verify) captured once and replayed on new inputs copied
    into the captured buffers: every replay must equal the eager run on the same inputs bit for bit
    (the library enqueues only kernels: no allocation, no memset nodes)."""
    w = si.workload("cfg2")
    batches = [si.gen_batch(w, seed=s) for s in (11, 12, 13)]
    d0 = batches[0]
    r = Round(svip, d0["draft"], d0["target"], d0["u_sample"], d0["u_accept"], d0["u_resample"], w.T, w.h)

    def enqueue():
        r.stop.zero_()
        for j in range(r.k):
            svip.draft_step(r.draft[:, j], temperature=w.T, h=w.h, step_j=j, k_max=r.k, u_sample=r.u_sample[:, j],
                            stop_in=r.stop, token_out=r.tokens[:, j], entropy_out=r.entropy[:, j],
                            q_tok_out=r.q_tok[:, j], lse_out=r.lse[:, j], stop_out=r.stop,
                            draft_len_out=r.draft_len, workspace=r.ws)
        svip.verify(r.target, r.draft, temperature=w.T, draft_tokens=r.tokens, draft_len=r.draft_len,
                    draft_lse=r.lse, u_accept=r.u_accept, u_resample=r.u_resample, n_accepted_out=r.n_accepted,
                    next_token_out=r.next_token, accept_prob_out=r.accept_prob, workspace=r.ws)

    def load(d):
        r.draft.copy_(d["draft"])
        r.target.copy_(d["target"])
        r.u_sample.copy_(d["u_sample"])
        r.u_accept.copy_(d["u_accept"])
        r.u_resample.copy_(d["u_resample"])
        r.tokens.fill_(-7)                      # entries of positions that are not drafted are left untouched:
        for t in (r.entropy, r.q_tok, r.lse, r.accept_prob):     # start every run from the same contents
            t.fill_(float("nan"))
        r.draft_len.zero_()

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (r.tokens, r.draft_len, r.entropy, r.lse, r.n_accepted, r.next_token, r.accept_prob)]

    eager = []
    for d in batches:
        load(d)
        enqueue()
        eager.append(snapshot())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()                              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enqueue()
    for rep in range(2):
        for i, d in enumerate(batches):
            load(d)
            g.replay()
            got = snapshot()
            for a, b in zip(got, eager[i]):
                assert torch.equal(a, b) or (a.is_floating_point() and torch.equal(a.isnan(), b.isnan())
                                             and torch.equal(a.nan_to_num(), b.nan_to_num())), f"replay {rep} batch {i}"
            torch.zeros(1 << 20, device="cuda").sum().item()      # unrelated eager work and a sync between replays
    assert svip.workspace_flags(r.ws) == 0


def _case(rng):
    dtype = [torch.bfloat16, torch.float32, torch.float16][int(rng.integers(0, 3))]
    B = int(rng.integers(1, 9))
    k = int(rng.integers(1, 7))
    V = int(rng.choice([3, 17, 255, 1000, 2048, 2049, 6007, 12288, 33000]))
    T = float(rng.choice([1.0, 0.7, 1.3]))
    h = float(rng.choice([0.3, 1.5, 2.5, 3.0]))
    return dtype, B, k, V, T, h


@pytest.mark.parametrize("seed", range(24))
def test_seeded_shapes_round(svip, seed):
    """Small random shapes, storage types, temperatures and thresholds: unchained draft outputs,
    the chained round and verification against the oracle, with row strides padded to 16 bytes."""
    rng = np.random.default_rng(9000 + seed)
    dtype, B, k, V, T, h = _case(rng)
    g = torch.Generator().manual_seed(500 + seed)
    scale = float(rng.choice([0.5, 2.0, 4.0]))
    draft = (scale * torch.randn(B, k, V, generator=g)).to(dtype)
    if rng.random() < 0.5 and V > 8:
        draft[:, :, int(rng.integers(0, V))] += 9.0
    target = torch.cat([draft.float(), scale * torch.randn(B, 1, V, generator=g)], 1)
    target = (target + float(rng.choice([0.3, 1.0])) * torch.randn(B, k + 1, V, generator=g)).to(dtype)
    if rng.random() < 0.3 and V > 8:
        mask = torch.rand(V, generator=g) < 0.3
        mask[0] = False
        draft[:, :, mask] = float("-inf")
        target[:, :, mask] = float("-inf")
    us, ua = torch.rand(B, k, generator=g), torch.rand(B, k, generator=g)
    ur = torch.rand(B, generator=g)
    mult = 4 if dtype == torch.float32 else 8
    Vp = (V + mult - 1) // mult * mult

    def padded(x):
        buf = torch.full((*x.shape[:-1], Vp), 55.0, dtype=dtype)
        buf[..., :V] = x
        return buf.cuda()[..., :V]

    _say(f"seeded case {seed}: {dtype} B={B} k={k} V={V} T={T} h={h}")
    r = Round(svip, padded(draft), padded(target), us, ua, ur, T, h)
    r.draft_all(chain=False)
    check_draft_rows(draft, T, h, k, us, r)
    r2 = Round(svip, padded(draft), padded(target), us, ua, ur, T, h)
    r2.draft_all(chain=True)
    tokens, dl, lse, mh, ms = oracle_chain(draft, T, h, us)
    g_tok, g_dl = r2.tokens.cpu().numpy(), r2.draft_len.cpu().numpy()
    check_chain(g_tok, g_dl, tokens, dl, mh, ms, draft_cpu=draft, T=T, u_sample=us)
    for mode in ("given", None):
        r2.verify(lse=mode)
        check_verify(draft, target, T, np.where(g_tok < 0, 0, g_tok).astype(np.int64), g_dl.astype(np.int64), ua, ur, r2)
    assert svip.workspace_flags(r2.ws) == 0


def test_c_abi_example_program_matches_the_binding(svip, tmp_path):
    """The example program uses nothing but hipMalloc and the C ABI; on the same problem it must print
    exactly what the Python binding computes (and that has been checked against the oracle above)."""
    import json
    import os
    import struct
    import subprocess
    from paper_2411_18462_amd import build as svip_build
    exe = svip_build.EXAMPLE_BIN
    if not os.path.exists(exe):            # normally built together with the library
        svip_build.build_example()
    B, k, V, T, h = 3, 5, 5000, 0.9, 2.0
    g = torch.Generator().manual_seed(77)
    draft = 2.0 * torch.randn(B, k, V, generator=g)
    draft[:, :, 123] += 7.0
    target = torch.cat([draft, 2.0 * torch.randn(B, 1, V, generator=g)], 1) + 0.8 * torch.randn(B, k + 1, V, generator=g)
    us, ua, ur = torch.rand(B, k, generator=g), torch.rand(B, k, generator=g), torch.rand(B, generator=g)
    path = tmp_path / "problem.bin"
    with open(path, "wb") as f:
        f.write(struct.pack("<iiiff", B, k, V, T, h))
        for t in (draft, target, us, ua, ur):
            f.write(t.contiguous().numpy().astype("<f4").tobytes())
    p = subprocess.run([exe, str(path)], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0, p.stderr
    got = json.loads(p.stdout)
    r = Round(svip, draft, target, us, ua, ur, T, h)
    r.tokens.fill_(-1)
    r.draft_all(chain=True)
    r.verify(lse="given")
    assert got["flags"] == 0
    assert got["draft_len"] == r.draft_len.cpu().tolist()
    assert got["n_accepted"] == r.n_accepted.cpu().tolist()
    assert got["next_token"] == r.next_token.cpu().tolist()
    assert got["tokens"] == r.tokens.cpu().flatten().tolist()
    tokens, dl, lse, mh, ms = oracle_chain(draft, T, h, us)
    check_chain(np.array(got["tokens"]).reshape(B, k), np.array(got["draft_len"]), tokens, dl, mh, ms,
                draft_cpu=draft, T=T, u_sample=us)
