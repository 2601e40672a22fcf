"""Parity of svip_warp_logits (top-k then top-p filtering) with the oracle, through the C ABI.

Top-k decisions are integer work and must match exactly; a top-p decision is compared where the oracle's
margin to the threshold is at least MARGIN of the kept mass, and must be an upward-closed set otherwise.
Kept logits keep their bits, dropped ones read -inf, padding between rows is neither read nor written.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import svip_inputs as si
from helpers import MARGIN, REL

pytestmark = pytest.mark.gpu

PAD = 3.0e4


def _say(*a):
    print(*a, flush=True)


def _padded_buf(x, mult=8):
    """x[..., V] inside a device buffer whose row stride is a multiple of `mult`; (buffer, view)."""
    V = x.shape[-1]
    Vp = (V + mult - 1) // mult * mult + mult
    buf = torch.full(x.shape[:-1] + (Vp,), PAD, dtype=x.dtype)
    buf[..., :V] = x
    buf = buf.cuda()
    return buf, buf[..., :V]


def _rows(V, n, dtype, seed, ties=False, masked=False):
    rng = np.random.default_rng(seed)
    z = rng.normal(-2.0, 3.0, (2, n, V)).astype(np.float32)
    z[:, ::2] *= 0.4                                      # flatter rows: larger nuclei
    if ties:
        z = np.round(z * 2) / 2
    if masked:
        z[rng.random(z.shape) < 0.4] = -np.inf
        z[..., 0] = 0.5
    return torch.from_numpy(z).to(dtype)


def _check(svip, x_cpu, T, top_k, top_p, inplace=False):
    B, n, V = x_cpu.shape
    buf, src = _padded_buf(x_cpu)
    kept = torch.full((B * n,), -1, dtype=torch.int32, device="cuda")
    if inplace:
        obuf, out = buf, svip.warp_logits(src, temperature=T, top_k=top_k, top_p=top_p, kept_out=kept)
        assert out.data_ptr() == src.data_ptr()
    else:
        obuf, out = _padded_buf(torch.full_like(x_cpu, float("nan")))
        svip.warp_logits(src, temperature=T, top_k=top_k, top_p=top_p, out=out, kept_out=kept)
        assert torch.equal(src.cpu(), x_cpu)              # the input is untouched
    torch.cuda.synchronize()
    assert (obuf[..., V:] == PAD).all()                   # padding is not written
    g = out.cpu().double().numpy()
    z = x_cpu.double().numpy()
    kept = kept.cpu().numpy()
    n_margin = 0
    for b in range(B):
        for j in range(n):
            keep, margin = oracle.warp_row(z[b, j], T, top_k, top_p)
            gk = ~np.isneginf(g[b, j])                    # survivors with a finite logit
            assert np.array_equal(g[b, j][gk], z[b, j][gk])
            finite = ~np.isneginf(z[b, j])
            if margin >= MARGIN:
                assert np.array_equal(gk, keep & finite), (b, j, int(gk.sum()), int(keep.sum()), margin)
                assert int(kept[b * n + j]) == int(keep.sum())
            else:
                # a cut this close to the threshold may fall one tie group to either side: the kept set
                # must be the top of the row, reach top_p within 2 * MARGIN, and not overshoot by a group
                n_margin += 1
                vals = z[b, j][gk]
                assert vals.size and (z[b, j][finite & ~gk] < vals.min()).all()
                q = scipy.special.softmax(z[b, j] / T)
                Z = q[oracle.warp_row(z[b, j], T, top_k, 1.0)[0]].sum()
                assert q[gk].sum() >= (top_p - 2 * MARGIN) * Z
                assert q[gk & (z[b, j] > vals.min())].sum() < (top_p + 2 * MARGIN) * Z
    return n_margin


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("V", [1, 7, 1000, 4099, 32000])
def test_top_k_is_exact(svip, dtype, V):
    _say(f"warp top-k {dtype} V={V}")
    x = _rows(V, 3, dtype, seed=V, ties=(V % 2 == 1))
    for k in sorted({1, 2, min(50, V), max(V - 1, 1), V, V + 5}):
        assert _check(svip, x, 1.0, k, 1.0) == 0


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("V,T", [(5, 1.0), (1000, 0.7), (4099, 1.0), (32000, 1.3), (128256, 1.0)])
def test_top_p_matches_the_oracle_outside_the_margin(svip, dtype, V, T):
    _say(f"warp top-p {dtype} V={V} T={T}")
    x = _rows(V, 2, dtype, seed=100 + V)
    in_margin = 0
    for p in (0.05, 0.5, 0.9, 0.99, 0.9999):
        in_margin += _check(svip, x, T, 0, p)
    _say(f"  cuts inside the margin: {in_margin} of {5 * x.shape[0] * x.shape[1]}")
    # a cut among tokens of probability below 2 * MARGIN is inside the margin by construction (large V,
    # large top_p): those rows get the neighbour check; most of the rest must compare exactly
    assert in_margin <= 3 * x.shape[0] * x.shape[1]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_top_k_then_top_p_with_ties_and_masks(svip, dtype):
    _say(f"warp k+p {dtype}")
    x = _rows(4099, 3, dtype, seed=7, ties=True, masked=True)
    assert _check(svip, x, 0.8, 40, 0.9) <= 1
    assert _check(svip, x, 0.8, 40, 0.9, inplace=True) <= 1
    assert _check(svip, x, 1.0, 3000, 0.3, inplace=True) <= 1     # top-k reaches into the -inf tail
    assert _check(svip, x, 1.0, 3000, 1.0) == 0
    assert _check(svip, x, 1.0, 0, 1.0) == 0                       # both filters off: a copy


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_crowded_bin_is_refined_by_row_sweeps(svip, dtype):
    """More keys in one first-digit bin than the candidate list holds: the thresholds inside the crowd
    (values that differ only in their low bits) come from sweeps over the row."""
    _say(f"warp crowded {dtype}")
    rng = np.random.default_rng(17)
    V = 40000
    z = rng.normal(0.0, 2.0, (1, 3, V)).astype(np.float32)
    crowd = rng.permutation(V)[:20000]
    step = 2.0 ** -20 if dtype == torch.float32 else 2.0 ** -7
    z[0, :, crowd] = (1.0 + step * rng.integers(0, 8, (20000, 1))).astype(np.float32)
    x = torch.from_numpy(z).to(dtype)
    for top_k, top_p in ((15000, 1.0), (0, 0.7), (15000, 0.8), (30, 0.99), (25000, 0.999), (0, 0.97)):
        _check(svip, x, 1.0, top_k, top_p)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_small_k_shortcut_equals_the_histogram_path(svip, dtype):
    """For a small top_k the thresholds come from a sampled pivot and a candidate list; the result must be
    bit for bit that of the histogram path (same integer arithmetic), also where the sample misleads."""
    _say(f"warp shortcut {dtype}")
    rng = np.random.default_rng(23)
    V = 50000
    z = rng.normal(-1.0, 2.5, (2, 4, V)).astype(np.float32)
    z[0, 0] = np.sort(z[0, 0])                      # largest logits at the end: an evenly spaced sample still sees them
    z[0, 1, :200] += 30.0                           # the top of the row is a cluster the sample can miss
    z[0, 2] = np.round(z[0, 2])                     # heavy ties
    z[1, 0, ::3] = -np.inf
    x = torch.from_numpy(z).to(dtype)
    buf, src = _padded_buf(x)
    for top_k, top_p in ((1, 1.0), (50, 1.0), (50, 0.9), (300, 0.5), (2000, 0.99), (2048, 1.0), (5, 0.999),
                         (0, 0.9), (0, 0.3), (0, 0.999), (0, 0.05)):
        svip.bench_set_tuning()
        k1 = torch.zeros(8, dtype=torch.int32, device="cuda")
        a = svip.warp_logits(src, temperature=0.9, top_k=top_k, top_p=top_p, out=_padded_buf(torch.zeros_like(x))[1], kept_out=k1)
        svip.bench_set_tuning(warp_no_shortcut=1)
        k2 = torch.zeros(8, dtype=torch.int32, device="cuda")
        b = svip.warp_logits(src, temperature=0.9, top_k=top_k, top_p=top_p, out=_padded_buf(torch.zeros_like(x))[1], kept_out=k2)
        torch.cuda.synchronize()
        bits = torch.int32 if dtype == torch.float32 else torch.int16
        assert torch.equal(a.contiguous().view(bits), b.contiguous().view(bits)), (top_k, top_p)
        assert torch.equal(k1, k2)
        svip.bench_set_tuning()       # in place: the shortcut without the early write
        k3 = torch.zeros(8, dtype=torch.int32, device="cuda")
        c = svip.warp_logits(_padded_buf(x)[1], temperature=0.9, top_k=top_k, top_p=top_p, kept_out=k3)
        torch.cuda.synchronize()
        assert torch.equal(a.contiguous().view(bits), c.contiguous().view(bits)), (top_k, top_p, "in place")
        assert torch.equal(k1, k3)
    svip.bench_set_tuning()
    _check(svip, x, 0.9, 50, 0.9)
    _check(svip, x, 0.9, 300, 1.0)
    _check(svip, x, 0.9, 0, 0.9)
    _check(svip, x, 0.9, 0, 0.9, inplace=True)


@pytest.mark.parametrize("seed", range(24))
def test_seeded_shapes_and_settings(svip, seed):
    """Random vocabulary sizes (ragged tails), storage types, temperatures, filters, row kinds, in place or not."""
    rng = np.random.default_rng(1000 + seed)
    dtype = [torch.float32, torch.bfloat16, torch.float16][seed % 3]
    V = int(rng.choice([3, 17, 255, 1025, 4097, 8191, 20011, 65537, 131075]))
    n = 2 if V > 50000 else 3
    z = rng.normal(rng.uniform(-4, 2), rng.uniform(0.3, 6.0), (1, n, V)).astype(np.float32)
    kind = seed % 4
    if kind == 1:
        z = np.round(z)                                        # ties
    elif kind == 2:
        z[rng.random(z.shape) < 0.5] = -np.inf                 # masked vocabulary
        z[..., int(rng.integers(0, V))] = 1.0
    elif kind == 3:
        z[0, :, : max(1, V // 100)] += 15.0                    # a cluster at the front of the row
    x = torch.from_numpy(z).to(dtype)
    top_k = int(rng.choice([0, 1, 5, 50, 700, 3000, V, V + 1]))
    top_p = float(rng.choice([1.0, 0.999, 0.95, 0.9, 0.5, 0.1]))
    T = float(rng.choice([0.6, 1.0, 1.7]))
    _say(f"warp seeded {seed}: {dtype} V={V} kind={kind} top_k={top_k} top_p={top_p} T={T}")
    _check(svip, x, T, top_k, top_p, inplace=bool(seed & 1))


def test_filter_replays_from_a_hip_graph(svip):
    """The call allocates nothing and launches one kernel: captured with a draft step behind it and replayed
    over changing inputs, every replay equals the eager result."""
    B, k, V = 4, 1, 20011
    g = torch.Generator().manual_seed(3)
    src = torch.empty(B, k, 20016, device="cuda", dtype=torch.bfloat16)[..., :V]
    out = torch.empty(B, k, 20016, device="cuda", dtype=torch.bfloat16)[..., :V]
    ws = svip.new_workspace(B, 1, V)
    u = torch.rand(B, generator=g).cuda()
    o = {n: torch.zeros(B, dtype=t, device="cuda") for n, t in
         (("tok", torch.int32), ("ent", torch.float32), ("lse", torch.float64), ("stop", torch.uint8))}

    def step():
        svip.warp_logits(src, temperature=0.8, top_k=64, top_p=0.92, out=out)
        svip.draft_step(out[:, 0], temperature=0.8, h=0.5, step_j=0, k_max=1, u_sample=u, token_out=o["tok"],
                        entropy_out=o["ent"], lse_out=o["lse"], stop_out=o["stop"], workspace=ws)

    src.copy_((2.5 * torch.randn(B, k, V, generator=g)).bfloat16())
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        src.copy_((2.5 * torch.randn(B, k, V, generator=g)).bfloat16())
        step()
        torch.cuda.synchronize()
        eager = (out.clone(), {n: t.clone() for n, t in o.items()})
        out.fill_(float("nan"))
        for t in o.values():
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager[0].view(torch.int16)), rep
        for n, t in o.items():
            assert torch.equal(t, eager[1][n]), (rep, n)
        assert int((~torch.isinf(out)).sum(-1).max()) <= 64 + 8


def test_filtered_rows_feed_the_draft_step(svip):
    """A draft step on rows filtered on the GPU equals the oracle's draft step on rows the oracle filtered."""
    w = si.workload("cfg1")
    d = si.gen_batch(w, seed=5)
    draft = d["draft"]
    B, k, V = draft.shape
    T, top_k, top_p = w.T, 64, 0.95
    z = draft.double().numpy()
    zf = z.copy()
    ok = np.ones((B, k), bool)
    for b in range(B):
        for j in range(k):
            keep, margin = oracle.warp_row(z[b, j], T, top_k, top_p)
            zf[b, j][~keep] = -np.inf
            ok[b, j] = margin >= MARGIN
    _, dev = _padded_buf(draft)
    svip.warp_logits(dev, temperature=T, top_k=top_k, top_p=top_p)
    ws = svip.new_workspace(B, k, V)
    tok = torch.zeros(B, k, dtype=torch.int32, device="cuda")
    ent = torch.zeros(B, k, dtype=torch.float32, device="cuda")
    lse = torch.zeros(B, k, dtype=torch.float64, device="cuda")
    stop = torch.zeros(B, dtype=torch.uint8, device="cuda")
    u = d["u_sample"].cuda().contiguous()
    for j in range(k):
        svip.draft_step(dev[:, j], temperature=T, h=1e9, step_j=j, k_max=k, u_sample=u[:, j], token_out=tok[:, j],
                        entropy_out=ent[:, j], lse_out=lse[:, j], stop_out=stop, workspace=ws)
    torch.cuda.synchronize()
    checked = 0
    for j in range(k):
        r = oracle.draft_step(zf[:, j], T, 1e9, j, k, d["u_sample"][:, j].double().numpy())
        for b in range(B):
            if not ok[b, j]:
                continue
            if r.margin_s[b] >= MARGIN:
                assert int(tok[b, j]) == int(r.token[b])
                checked += 1
            assert math.isclose(float(ent[b, j]), float(r.entropy[b]), rel_tol=REL, abs_tol=1e-6)
    assert checked >= B * k // 2


def test_loop_over_filtered_traces(svip):
    """Traces filtered on the GPU (top-k: exact) drive the decoding loop; the oracle's loop runs on the same
    filtered traces after the rows it reads were checked against the oracle's own filter."""
    from test_loop_gpu import POLICIES, _check as check_loop, _run as run_loop
    w = si.workload("cfg2", noise=0.7)
    L, used = 1100, 64                    # a trace longer than any round; the loop below reads rows < used
    tr = dict(si.gen_trace(w, L, rounds=40, gamma_max=12, seed=12, rows=[0, 1, 2]))
    for name in ("draft", "target"):
        x = tr[name]
        got = svip.warp_logits(x.cuda(), temperature=w.T, top_k=40).cpu()
        for b in range(x.shape[0]):
            for j in list(range(used)) + list(range(used, L, 131)) + [L - 1]:
                keep, _ = oracle.warp_row(x[b, j].double().numpy(), w.T, 40, 1.0)
                assert np.array_equal(~torch.isinf(got[b, j]).numpy(), keep), (name, b, j)
                assert torch.equal(got[b, j][torch.from_numpy(keep)], x[b, j][torch.from_numpy(keep)])
        tr[name] = got[:, :used].contiguous()
    res = run_loop(svip, tr, w, POLICIES["svip"], 40)
    st = check_loop(res, tr, w, POLICIES["svip"], 40)
    _say(f"  filtered loop {st}")
    assert st["rounds"] >= 5
