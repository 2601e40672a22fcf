"""Seeded synthetic inputs for the SVIP hot path (shared by tests, oracle runs and bench).

This module holds NONE of the method's arithmetic: it only draws logits and uniforms.
The paper's workloads (MT-Bench, MATH, AIME, GPQA with Qwen2.5 / QwQ / Vicuna model
pairs, Section 3) need datasets and trained weights; the synthetic rows below stand in
for them with the same shapes (vocabulary sizes of those model families), storage types
and a low/high-entropy structure mirroring the accepted-versus-rejected entropy split the
paper reports (Section 2.1, Table 1).

Every sequence b of a workload is generated from its own seed, so a test can rebuild a
few sampled sequences of a large batch without materialising the whole batch.

Recipe per workload (values are rounded once to the storage dtype; the oracle and the GPU
read the same bits):
  draft row types
    "spike"  : N(0, sigma^2) background with `spike` added at one seeded index
    "low"    : N(0, 1) background, the logit at one seeded index SET to 12.0
    "high"   : N(0, 0.5^2)
  target row = stored draft row (widened to fp32) + N(0, noise^2), rounded to the dtype
  (workloads with noise_high use that std on "high" rows, so that acceptance falls where the
  draft entropy is high);
  the extra target row after the last draft position is a fresh row of a drawn type + noise.
  row types: "mixture" draws low w.p. 0.7 independently per row; "markov" follows a
  two-state chain per sequence (stay-probabilities 0.9 in low, 0.7 in high, start low).
  uniforms: float32 in [0, 1) from the same per-sequence generator.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    V: int
    dtype: str          # "f32" | "bf16"
    k: int              # k_max, draft positions per round
    T: float            # sampling temperature
    h: float            # entropy threshold used with these rows
    rows: str           # "spike" | "mixture" | "markov"
    noise: float        # std of the target perturbation
    sigma: float = 3.0  # background std for "spike" rows
    spike: float = 8.0  # spike height for "spike" rows
    uid: int = 0        # enters the seed
    noise_high: float | None = None   # std of the target perturbation on "high" rows (None: same as noise)


# h = 3.0 separates the synthetic low rows (sqrt(H) <= 2.85) from the high rows
# (sqrt(H) >= 3.18) at every V used here; the paper's h = 0.3 stops every such row at once.
WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 32000, "f32", 8, 1.0, 3.0, "spike", 1.0, uid=1),
    "cfg2": Workload("cfg2", 16, 32000, "f32", 16, 1.0, 3.0, "mixture", 1.0, uid=2),
    "cfg3": Workload("cfg3", 64, 128256, "bf16", 16, 1.0, 3.0, "mixture", 1.5, uid=3),
    "cfg4": Workload("cfg4", 8, 151936, "bf16", 64, 1.0, 3.0, "markov", 1.5, uid=4),
    # traces for the decoding loop: the models agree where the draft is confident (low rows, expected
    # acceptance about 0.9) and disagree where it is not (high rows, about 0.45), the split of Section 2.1
    "cfg4_loop": Workload("cfg4_loop", 8, 151936, "bf16", 64, 1.0, 3.0, "markov", 0.3, uid=5, noise_high=1.5),
}


def workload(name: str, **overrides) -> Workload:
    return replace(WORKLOADS[name], **overrides)


def torch_dtype(w: Workload):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[w.dtype]


def _gen(w: Workload, b: int, seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed((seed * 1_000_003 + w.uid * 10_007 + b) & 0x7FFFFFFFFFFFFFFF)
    return g


def _row_types(w: Workload, n: int, g: torch.Generator) -> list[str]:
    r = torch.rand(n, generator=g).tolist()
    if w.rows == "spike":
        return ["spike"] * n
    if w.rows == "mixture":
        return ["low" if x < 0.7 else "high" for x in r]
    if w.rows == "markov":
        out, state = [], "low"
        for x in r:
            out.append(state)
            stay = 0.9 if state == "low" else 0.7
            if x >= stay:
                state = "high" if state == "low" else "low"
        return out
    raise ValueError(w.rows)


def _rows(w: Workload, types: list[str], g: torch.Generator) -> torch.Tensor:
    n = len(types)
    z = torch.randn(n, w.V, generator=g, dtype=torch.float32)
    idx = torch.randint(0, w.V, (n,), generator=g)
    for i, t in enumerate(types):
        if t == "spike":
            z[i] *= w.sigma
            z[i, idx[i]] += w.spike
        elif t == "low":
            z[i, idx[i]] = 12.0
        elif t == "high":
            z[i] *= 0.5
        else:
            raise ValueError(t)
    return z


def gen_sequence(w: Workload, b: int, seed: int = 0) -> dict:
    """One sequence of workload w: draft [k, V], target [k+1, V] in the storage dtype,
    u_sample [k], u_accept [k], u_resample [] (float32), row types of the k+1 positions."""
    g = _gen(w, b, seed)
    dt = torch_dtype(w)
    types = _row_types(w, w.k + 1, g)
    base = _rows(w, types, g)                     # fp32, k+1 rows; last one has no draft row
    draft = base[: w.k].to(dt)
    stored = torch.cat([draft.float(), base[w.k:].to(dt).float()], 0)
    scale = torch.tensor([w.noise_high if (t == "high" and w.noise_high is not None) else w.noise for t in types])
    target = (stored + scale[:, None] * torch.randn(w.k + 1, w.V, generator=g)).to(dt)
    u = torch.rand(2 * w.k + 1, generator=g, dtype=torch.float32)
    return dict(draft=draft, target=target, u_sample=u[: w.k].clone(),
                u_accept=u[w.k: 2 * w.k].clone(), u_resample=u[2 * w.k].clone(), types=types)


def gen_batch(w: Workload, seed: int = 0, rows=None) -> dict:
    """Stack sequences `rows` (default: all B) of workload w:
    draft [B, k, V], target [B, k+1, V], u_sample [B, k], u_accept [B, k], u_resample [B]."""
    rows = list(range(w.B)) if rows is None else list(rows)
    seqs = [gen_sequence(w, b, seed) for b in rows]
    out = {key: torch.stack([s[key] for s in seqs]) for key in
           ("draft", "target", "u_sample", "u_accept", "u_resample")}
    out["types"] = [s["types"] for s in seqs]
    return out


def gen_trace(w: Workload, L: int, rounds: int, gamma_max: int, seed: int = 0, rows=None) -> dict:
    """Logit traces for the decoding loop: sequence b's workload rows continued to L positions.
    draft [B, L, V], target [B, L, V] (target row n = stored draft row n + noise), and the loop's
    uniforms u_sample / u_accept [rounds, B, gamma_max], u_resample [rounds, B] (float32)."""
    rows = list(range(w.B)) if rows is None else list(rows)
    ww = replace(w, k=L)
    seqs = [gen_sequence(ww, b, seed) for b in rows]
    draft = torch.stack([s["draft"] for s in seqs])
    target = torch.stack([s["target"][:L] for s in seqs])
    g = torch.Generator(device="cpu")
    g.manual_seed((seed * 7_919 + w.uid * 104_729 + 17) & 0x7FFFFFFFFFFFFFFF)
    n = len(rows)
    u = torch.rand(2, rounds, n, gamma_max, generator=g, dtype=torch.float32)
    ur = torch.rand(rounds, n, generator=g, dtype=torch.float32)
    return dict(draft=draft, target=target, u_sample=u[0].contiguous(), u_accept=u[1].contiguous(),
                u_resample=ur, types=[s["types"][:L] for s in seqs])
