"""fp64 CPU oracle of the SVIP hot path -- TEST INFRASTRUCTURE, not the product.

Thin ctypes loader around ``svip_oracle.c`` (plain C, gcc -O2).  Only ``tests/``, the
smoke check and the benchmark's CPU-baseline leg may import this package; it shares
nothing with the HIP library and never imports it.

All array arguments are converted to contiguous float64 / int64 numpy arrays; logits in
bf16 or fp32 are widened exactly before they get here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "svip_oracle.c")
_LIB = os.path.join(_HERE, "libsvip_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_D = ctypes.POINTER(ctypes.c_double)
_L = ctypes.POINTER(ctypes.c_long)
_U8 = ctypes.POINTER(ctypes.c_ubyte)


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(ctypes.CDLL(build()))
    return _lib


def _bind(lib):
    """Declare the C signatures of svip_oracle.c on a loaded library (also used by the test that
    compiles copies of the oracle with planted mistakes)."""
    if True:
        lib.oracle_softmax_row.restype = ctypes.c_double
        lib.oracle_softmax_row.argtypes = [_D, ctypes.c_long, ctypes.c_double, _D]
        lib.oracle_entropy_row.restype = ctypes.c_double
        lib.oracle_entropy_row.argtypes = [_D, ctypes.c_long]
        lib.oracle_inverse_cdf.restype = ctypes.c_long
        lib.oracle_inverse_cdf.argtypes = [_D, ctypes.c_long, ctypes.c_double, _D]
        lib.oracle_draft_step.restype = None
        lib.oracle_draft_step.argtypes = [
            _D, ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double, ctypes.c_double,
            ctypes.c_long, ctypes.c_long, _D, _U8, _L, _D, _D, _D, _U8, _D, _D]
        lib.oracle_verify.restype = None
        lib.oracle_verify.argtypes = [
            _D, _D, ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double,
            _L, _L, _D, _D, _L, _L, _D, _D, _D, _D, _D, _D]
        lib.oracle_argmax_row.restype = ctypes.c_long
        lib.oracle_argmax_row.argtypes = [_D, ctypes.c_long]
        lib.oracle_draft_step_greedy.restype = None
        lib.oracle_draft_step_greedy.argtypes = [
            _D, ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double, ctypes.c_double,
            ctypes.c_long, ctypes.c_long, _U8, _L, _D, _D, _D, _U8, _D]
        lib.oracle_verify_greedy.restype = None
        lib.oracle_verify_greedy.argtypes = [_D, ctypes.c_long, ctypes.c_long, ctypes.c_long, _L, _L, _L, _L]
        lib.oracle_pair_stats.restype = None
        lib.oracle_pair_stats.argtypes = [_D, _D, ctypes.c_long, ctypes.c_double, _D]
        lib.oracle_diagnostics.restype = None
        lib.oracle_diagnostics.argtypes = [_D, _D, ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double,
                                           _L, ctypes.c_double, _D]
        lib.oracle_generate.restype = ctypes.c_long
        lib.oracle_generate.argtypes = [
            _D, _D, ctypes.c_long, ctypes.c_long, ctypes.c_double, ctypes.c_long, ctypes.c_long, ctypes.c_double,
            ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_long, _D, _D, _D, ctypes.c_long, ctypes.c_int,
            ctypes.c_long, _L, _L, _L, _D]
        lib.oracle_warp_row.restype = ctypes.c_long
        lib.oracle_warp_row.argtypes = [_D, ctypes.c_long, ctypes.c_double, ctypes.c_long, ctypes.c_double, _U8, _D]
        lib.oracle_sd_position_trials.restype = None
        lib.oracle_sd_position_trials.argtypes = [
            _D, _D, ctypes.c_long, ctypes.c_long, ctypes.c_ulonglong, ctypes.c_int, _L, _L]
    return lib


def _f64(a) -> np.ndarray:
    if hasattr(a, "detach"):  # torch tensor (any float dtype, CPU)
        a = a.detach().to("cpu").double().numpy()
    return np.ascontiguousarray(a, dtype=np.float64)


def _i64(a) -> np.ndarray:
    if hasattr(a, "detach"):
        a = a.detach().to("cpu").long().numpy()
    return np.ascontiguousarray(a, dtype=np.int64)


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(t)


def softmax_row(z, T: float = 1.0):
    """(prob[V], logsumexp) of one row of logits at temperature T."""
    z = _f64(z).ravel()
    prob = np.empty_like(z)
    lse = _load().oracle_softmax_row(_p(z, _D), z.size, float(T), _p(prob, _D))
    return prob, lse


def entropy_row(prob) -> float:
    prob = _f64(prob).ravel()
    return _load().oracle_entropy_row(_p(prob, _D), prob.size)


def inverse_cdf(w, u: float):
    """(index, margin) of one categorical draw from weights w with uniform u."""
    w = _f64(w).ravel()
    m = ctypes.c_double(0.0)
    i = _load().oracle_inverse_cdf(_p(w, _D), w.size, float(u), ctypes.byref(m))
    return int(i), m.value


@dataclass
class DraftStepResult:
    token: np.ndarray      # int64 [B], -1 for skipped rows
    entropy: np.ndarray    # float64 [B], nats
    q_tok: np.ndarray      # float64 [B]
    lse: np.ndarray        # float64 [B]
    stop: np.ndarray       # uint8 [B]
    margin_h: np.ndarray   # float64 [B], |sqrt(H) - h| (inf when the cap decides)
    margin_s: np.ndarray   # float64 [B], sampler margin (fraction of total mass)


def draft_step(z, T, h, step_j, k_max, u, stop_in=None) -> DraftStepResult:
    """Draft-side pass over z[B, V]; see oracle_draft_step in svip_oracle.c."""
    z = _f64(z)
    assert z.ndim == 2
    B, V = z.shape
    u = _f64(u).ravel()
    assert u.size == B
    si = None
    if stop_in is not None:
        si = np.ascontiguousarray(_i64(stop_in).ravel() != 0, dtype=np.uint8)
        assert si.size == B
    out = DraftStepResult(
        np.empty(B, np.int64), np.empty(B), np.empty(B), np.empty(B),
        np.empty(B, np.uint8), np.empty(B), np.empty(B))
    _load().oracle_draft_step(
        _p(z, _D), B, V, V, float(T), float(h), int(step_j), int(k_max), _p(u, _D),
        _p(si, _U8) if si is not None else None,
        _p(out.token, _L), _p(out.entropy, _D), _p(out.q_tok, _D), _p(out.lse, _D),
        _p(out.stop, _U8), _p(out.margin_h, _D), _p(out.margin_s, _D))
    return out


@dataclass
class VerifyResult:
    n_accepted: np.ndarray   # int64 [B]
    next_token: np.ndarray   # int64 [B]
    accept_prob: np.ndarray  # float64 [B, k_max]; NaN where j >= gamma[b]
    margin: np.ndarray       # float64 [B], smallest decision margin of the sequence
    resid_mass: np.ndarray   # float64 [B], sum max(0, p - q) at the rejection (0 if none)
    margin_a: np.ndarray     # float64 [B, k_max], |ua - p/q| per tested position; NaN where j >= gamma[b]
    margin_accept: np.ndarray  # float64 [B], smallest margin_a up to and including the first rejection
    margin_sample: np.ndarray  # float64 [B], sampler margin of the correction / bonus draw


def verify(zp, zq, T, tok, gamma, ua, ur) -> VerifyResult:
    """Target-side pass; zp[B, k+1, V], zq[B, k, V]; see oracle_verify in svip_oracle.c."""
    zp = _f64(zp)
    zq = _f64(zq)
    B, kp1, V = zp.shape
    k = kp1 - 1
    assert zq.shape == (B, k, V)
    tok = _i64(tok).reshape(B, k)
    gamma = _i64(gamma).ravel()
    ua = _f64(ua).reshape(B, k)
    ur = _f64(ur).ravel()
    assert gamma.size == B and ur.size == B
    assert (gamma >= 0).all() and (gamma <= k).all()
    for b in range(B):
        g = int(gamma[b])
        assert ((tok[b, :g] >= 0) & (tok[b, :g] < V)).all()
    out = VerifyResult(
        np.empty(B, np.int64), np.empty(B, np.int64), np.full((B, k), np.nan),
        np.empty(B), np.empty(B), np.full((B, k), np.nan), np.empty(B), np.empty(B))
    _load().oracle_verify(
        _p(zp, _D), _p(zq, _D), B, k, V, float(T), _p(tok, _L), _p(gamma, _L),
        _p(ua, _D), _p(ur, _D), _p(out.n_accepted, _L), _p(out.next_token, _L),
        _p(out.accept_prob, _D), _p(out.margin, _D), _p(out.resid_mass, _D),
        _p(out.margin_a, _D), _p(out.margin_accept, _D), _p(out.margin_sample, _D))
    return out


def argmax_row(z) -> int:
    z = _f64(z).ravel()
    return int(_load().oracle_argmax_row(_p(z, _D), z.size))


def draft_step_greedy(z, T, h, step_j, k_max, stop_in=None) -> DraftStepResult:
    """Greedy draft-side pass over z[B, V]: token = argmax; margin_s is inf (no draw)."""
    z = _f64(z)
    assert z.ndim == 2
    B, V = z.shape
    si = None
    if stop_in is not None:
        si = np.ascontiguousarray(_i64(stop_in).ravel() != 0, dtype=np.uint8)
        assert si.size == B
    out = DraftStepResult(
        np.empty(B, np.int64), np.empty(B), np.empty(B), np.empty(B),
        np.empty(B, np.uint8), np.empty(B), np.full(B, np.inf))
    _load().oracle_draft_step_greedy(
        _p(z, _D), B, V, V, float(T), float(h), int(step_j), int(k_max),
        _p(si, _U8) if si is not None else None,
        _p(out.token, _L), _p(out.entropy, _D), _p(out.q_tok, _D), _p(out.lse, _D),
        _p(out.stop, _U8), _p(out.margin_h, _D))
    return out


def verify_greedy(zp, tok, gamma):
    """(n_accepted[B], next_token[B]) of greedy verification; zp[B, k+1, V]."""
    zp = _f64(zp)
    B, kp1, V = zp.shape
    k = kp1 - 1
    tok = _i64(tok).reshape(B, k)
    gamma = _i64(gamma).ravel()
    assert gamma.size == B and (gamma >= 0).all() and (gamma <= k).all()
    nacc, nxt = np.empty(B, np.int64), np.empty(B, np.int64)
    _load().oracle_verify_greedy(_p(zp, _D), B, k, V, _p(tok, _L), _p(gamma, _L), _p(nacc, _L), _p(nxt, _L))
    return nacc, nxt


def pair_stats(zp_row, zq_row, T: float = 1.0) -> dict:
    """beta, KL(q||p), H_{q,p}, H_q and TVD of one (target, draft) row pair."""
    zp_row = _f64(zp_row).ravel()
    zq_row = _f64(zq_row).ravel()
    assert zp_row.size == zq_row.size
    out = np.empty(5)
    _load().oracle_pair_stats(_p(zp_row, _D), _p(zq_row, _D), zp_row.size, float(T), _p(out, _D))
    return dict(beta=out[0], kl=out[1], hqp=out[2], hq=out[3], tvd=out[4])


DIAG_FIELDS = ("beta", "kl", "hqp", "hq", "bound_oracle", "bound_bh", "bound_approx", "ratio")


def diagnostics(zp, zq, T, gamma, c) -> np.ndarray:
    """[B, k, 8] per-position diagnostics (DIAG_FIELDS order), NaN where j >= gamma[b];
    zp[B, k+1, V], zq[B, k, V]; see oracle_diagnostics in svip_oracle.c."""
    zp = _f64(zp)
    zq = _f64(zq)
    B, kp1, V = zp.shape
    k = kp1 - 1
    assert zq.shape == (B, k, V)
    gamma = _i64(gamma).ravel()
    assert gamma.size == B and (gamma >= 0).all() and (gamma <= k).all()
    out = np.empty((B, k, 8))
    _load().oracle_diagnostics(_p(zp, _D), _p(zq, _D), B, k, V, float(T), _p(gamma, _L), float(c), _p(out, _D))
    return out


@dataclass
class GenerateResult:
    tokens: np.ndarray      # int64 [n_out] produced tokens in order
    log: np.ndarray         # int64 [rounds, 5]: n at round start, cap, drafted, accepted, last token
    min_margin: float       # smallest decision margin met on the way


def generate(zp, zq, T, n0, max_new, h, gamma0, gamma_max, inc, dec, us=None, ua=None, ur=None,
             greedy=False, max_rounds=None) -> GenerateResult:
    """One sequence through the decoding loop over traces zp[L, V], zq[L, V]; see oracle_generate
    in svip_oracle.c.  us, ua: [rounds, kw] uniforms, ur: [rounds]."""
    zp = _f64(zp)
    zq = _f64(zq)
    L, V = zq.shape
    assert zp.shape == (L, V) and 1 <= gamma0 <= gamma_max
    R = int(max_rounds) if max_rounds is not None else int(max_new)
    if greedy:
        us = ua = np.zeros((R, gamma_max))
        ur = np.zeros(R)
    us, ua, ur = _f64(us), _f64(ua), _f64(ur).ravel()
    assert us.ndim == 2 and us.shape == ua.shape and us.shape[1] >= gamma_max
    R = min(R, us.shape[0], ur.size)
    out = np.empty(R * (gamma_max + 1), np.int64)
    log = np.empty((R, 5), np.int64)
    n_out = ctypes.c_long(0)
    mm = ctypes.c_double(0.0)
    rounds = _load().oracle_generate(
        _p(zp, _D), _p(zq, _D), L, V, float(T), int(n0), int(max_new), float(h), int(gamma0), int(gamma_max),
        int(inc), int(dec), _p(us, _D), _p(ua, _D), _p(ur, _D), us.shape[1], int(bool(greedy)), R,
        _p(out, _L), ctypes.byref(n_out), _p(log, _L), ctypes.byref(mm))
    return GenerateResult(out[:n_out.value].copy(), log[:rounds].copy(), mm.value)


def warp_row(z, T: float = 1.0, top_k: int = 0, top_p: float = 1.0):
    """(keep[V] bool, margin) of top-k followed by top-p filtering of one row; see oracle_warp_row."""
    z = _f64(z).ravel()
    keep = np.zeros(z.size, np.uint8)
    m = ctypes.c_double(0.0)
    n = _load().oracle_warp_row(_p(z, _D), z.size, float(T), int(top_k), float(top_p), _p(keep, _U8), ctypes.byref(m))
    assert n == int(keep.sum())
    return keep.astype(bool), m.value


def sd_position_trials(p, q, N: int, seed: int, resid_sign: int = +1):
    """(histogram[V], n_accepted) of N brute-force draft/verify/correct trials."""
    p = _f64(p).ravel()
    q = _f64(q).ravel()
    hist = np.zeros(p.size, np.int64)
    nacc = ctypes.c_long(0)
    _load().oracle_sd_position_trials(
        _p(p, _D), _p(q, _D), p.size, int(N), int(seed), int(resid_sign),
        _p(hist, _L), ctypes.byref(nacc))
    return hist, nacc.value
