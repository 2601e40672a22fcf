"""The seeded synthetic workloads: shapes, determinism and the structure the recipe promises."""
import math

import numpy as np
import torch

import oracle
import svip_inputs as si


def test_shapes_dtypes_and_determinism():
    for name, w in si.WORKLOADS.items():
        s = si.gen_sequence(w, 0, seed=0)
        assert s["draft"].shape == (w.k, w.V) and s["target"].shape == (w.k + 1, w.V)
        assert s["draft"].dtype == si.torch_dtype(w) == s["target"].dtype
        assert s["u_sample"].shape == (w.k,) and s["u_accept"].shape == (w.k,)
        for u in (s["u_sample"], s["u_accept"], s["u_resample"].reshape(1)):
            assert u.dtype == torch.float32 and (u >= 0).all() and (u < 1).all()
        s2 = si.gen_sequence(w, 0, seed=0)
        assert torch.equal(s["draft"], s2["draft"]) and torch.equal(s["target"], s2["target"])
        s3 = si.gen_sequence(w, 0, seed=1)
        assert not torch.equal(s["draft"], s3["draft"])
    w = si.workload("cfg2")
    b = si.gen_batch(w, rows=[3, 7])
    assert b["draft"].shape == (2, w.k, w.V)
    assert torch.equal(b["draft"][1], si.gen_sequence(w, 7)["draft"])


def test_mixture_and_markov_row_types():
    w = si.workload("cfg3", V=64)
    types = [t for b in range(64) for t in si.gen_sequence(w, b)["types"]]
    frac_low = types.count("low") / len(types)
    assert abs(frac_low - 0.7) < 0.05
    w4 = si.workload("cfg4", V=64)
    stay_low = stay_high = n_low = n_high = 0
    for b in range(40):
        t = si.gen_sequence(w4, b)["types"]
        assert t[0] == "low"
        for a, c in zip(t[:-1], t[1:]):
            if a == "low":
                n_low += 1
                stay_low += c == "low"
            else:
                n_high += 1
                stay_high += c == "high"
    assert abs(stay_low / n_low - 0.9) < 0.03 and abs(stay_high / n_high - 0.7) < 0.06


def test_entropy_bands_are_separated_by_h():
    """Low rows stay below, high rows above, the threshold the synthetic workloads use."""
    for name in ("cfg2", "cfg3"):
        w = si.workload(name)
        s = si.gen_sequence(w, 1)
        for j in range(6):
            p, _ = oracle.softmax_row(s["draft"][j], w.T)
            rootH = math.sqrt(oracle.entropy_row(p))
            if s["types"][j] == "low":
                assert rootH < w.h - 0.1
            else:
                assert rootH > w.h + 0.1


def test_target_is_perturbed_draft():
    w = si.workload("cfg3", V=4096)
    s = si.gen_sequence(w, 5)
    d = (s["target"][: w.k].float() - s["draft"].float()).numpy()
    assert abs(d.std() - w.noise) < 0.05 and abs(d.mean()) < 0.02
    assert np.isfinite(s["target"].float().numpy()).all()


def test_traces_for_the_decoding_loop():
    """gen_trace: shapes, determinism, per-sequence seeds, and the acceptance split of the loop
    workload (the models agree on low-entropy rows, disagree on high-entropy ones)."""
    w = si.workload("cfg4_loop", V=4096)
    tr = si.gen_trace(w, 40, rounds=7, gamma_max=5, seed=2, rows=[0, 3])
    assert tr["draft"].shape == (2, 40, 4096) == tr["target"].shape and tr["draft"].dtype == torch.bfloat16
    assert tr["u_sample"].shape == (7, 2, 5) == tr["u_accept"].shape and tr["u_resample"].shape == (7, 2)
    for u in (tr["u_sample"], tr["u_accept"], tr["u_resample"]):
        assert u.dtype == torch.float32 and (u >= 0).all() and (u < 1).all()
    again = si.gen_trace(w, 40, rounds=7, gamma_max=5, seed=2, rows=[3])
    assert torch.equal(again["draft"][0], tr["draft"][1]) and torch.equal(again["target"][0], tr["target"][1])
    assert not torch.equal(tr["draft"][0], tr["draft"][1])
    tr = si.gen_trace(w, 40, rounds=1, gamma_max=5, seed=2, rows=list(range(6)))
    beta = {"low": [], "high": []}
    for b in range(6):
        for n in range(40):
            st = oracle.pair_stats(tr["target"][b, n].double().numpy(), tr["draft"][b, n].double().numpy(), w.T)
            beta[tr["types"][b][n]].append(st["beta"])
    assert len(beta["low"]) > 20 and len(beta["high"]) > 10
    assert np.mean(beta["low"]) > np.mean(beta["high"]) + 0.2
