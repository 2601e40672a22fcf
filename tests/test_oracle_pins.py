"""Pins for the fp64 oracle: closed forms, library routines, invariants and brute force.

None of these re-type the oracle's own formulas: each compares it with a value fixed by
mathematics (closed forms), with an independent library routine (scipy / numpy), with an
invariant stated in the paper (Section 2.2: Eq. beta, tvd, pinsker, beta-bound; Appendix B)
or with brute-force counting on a tiny vocabulary.
"""
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CHI2_7DOF_999 = 24.32   # 99.9 % quantile of chi-square with 7 degrees of freedom


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- softmax / entropy

@pytest.mark.parametrize("V", [32000, 128256, 151936])
def test_uniform_logits_entropy_is_log_V(V):
    golden = dict(line.split() for line in open(os.path.join(GOLDEN, "log_vocab.txt"))
                  if line.strip() and not line.startswith("#"))
    for const in (0.0, -7.25, 3.5):
        p, lse = oracle.softmax_row(np.full(V, const), T=1.0)
        H = oracle.entropy_row(p)
        assert abs(H - math.log(V)) < 1e-9
        assert abs(H - float(golden[str(V)])) < 5e-5       # 4-decimal values in the fixture
        assert abs(lse - (const + math.log(V))) < 1e-9
    # any h of the paper's grid stops on a uniform row
    u = 0.50001                     # away from a cell edge: token = floor(u V)
    r = oracle.draft_step(np.zeros((1, V)), 1.0, 0.5, 0, 40, [u])
    assert r.stop[0] == 1 and r.token[0] == int(u * V)


def test_one_hot_entropy_zero_and_no_stop():
    V = 1000
    z = np.full((2, V), -np.inf)
    z[0, 17] = 3.0
    z[1, :] = 0.0
    z[1, 999] = 1.0e4          # spike so large every other term underflows to 0
    r = oracle.draft_step(z, 1.0, 0.2, 0, 40, [0.0, 0.999999])
    assert list(r.token) == [17, 999]
    assert np.all(r.entropy == 0.0) and np.all(r.stop == 0)
    assert np.allclose(r.q_tok, 1.0) and np.allclose(r.lse, [3.0, 1.0e4])


@pytest.mark.parametrize("V,d", [(8, 1.0), (32000, 12.0), (128256, 12.0), (50, -3.0)])
def test_spike_over_flat_closed_form(V, d):
    z = np.zeros(V)
    z[V // 3] = d
    ps = math.exp(d) / (math.exp(d) + V - 1)
    H_exact = -ps * math.log(ps) - (1 - ps) * math.log((1 - ps) / (V - 1))
    p, lse = oracle.softmax_row(z)
    assert abs(p[V // 3] - ps) < 1e-12
    assert abs(oracle.entropy_row(p) - H_exact) < 1e-10
    assert abs(lse - math.log(math.exp(d) + V - 1)) < 1e-10


def test_two_point_entropy_log1p_form():
    for d in (0.0, 0.5, 4.0, 30.0):
        p, _ = oracle.softmax_row([0.0, d])
        # H = log(1+e^-d) + d * e^-d / (1+e^-d) for logits (0, d)
        H = math.log1p(math.exp(-d)) + d * math.exp(-d) / (1 + math.exp(-d))
        assert abs(oracle.entropy_row(p) - H) < 1e-13


def test_softmax_entropy_match_scipy_and_invariances():
    rng = _rng(1)
    for V, T in ((8, 1.0), (1000, 0.7), (32000, 1.0), (4099, 2.5)):
        z = rng.normal(0, 3, V)
        p, lse = oracle.softmax_row(z, T)
        assert np.allclose(p, scipy.special.softmax(z / T), rtol=1e-12, atol=0)
        assert abs(lse - scipy.special.logsumexp(z / T)) < 1e-11
        H = oracle.entropy_row(p)
        assert abs(H - scipy.stats.entropy(scipy.special.softmax(z / T))) < 1e-11
        # shift invariance and the temperature identity H_T(z) = H_1(z/T)
        p2, lse2 = oracle.softmax_row(z + 5.0, T)
        assert abs(oracle.entropy_row(p2) - H) < 1e-11 and abs(lse2 - lse - 5.0 / T) < 1e-11
        p3, _ = oracle.softmax_row(z / T, 1.0)
        assert abs(oracle.entropy_row(p3) - H) < 1e-11


def test_minus_inf_logits_carry_no_mass():
    z = np.array([0.0, -np.inf, 1.0, -np.inf])
    p, lse = oracle.softmax_row(z)
    assert p[1] == 0 and p[3] == 0 and abs(p.sum() - 1) < 1e-15
    assert abs(oracle.entropy_row(p) - scipy.stats.entropy([1, math.e])) < 1e-14
    # a zero-mass token is never drawn, whatever u
    for u in (0.0, 0.2689, 0.27, 0.999999):
        i, _ = oracle.inverse_cdf(p, u)
        assert i in (0, 2)


# ---------------------------------------------------------------- stop test (Eq. stop_condition)

def test_stop_rule_two_formulations_agree():
    """1 - sqrt(c H) < h_hat  <=>  sqrt(H) > (1 - h_hat)/sqrt(c)   (Section 2.2)."""
    rng = _rng(2)
    V = 64
    n = 0
    for _ in range(300):
        c, h_hat = rng.uniform(0.05, 3.0), rng.uniform(0.0, 0.95)
        z = rng.normal(0, rng.uniform(0.1, 6.0), (1, V))
        h = (1 - h_hat) / math.sqrt(c)
        r = oracle.draft_step(z, 1.0, h, 0, 40, [0.3])
        if r.margin_h[0] < 1e-9:
            continue
        bound = 1 - math.sqrt(c * r.entropy[0])
        assert bool(r.stop[0]) == (bound < h_hat)
        n += 1
    assert n > 250


def test_stop_is_strict_and_cap_forces_stop():
    V = 16
    z = np.zeros((1, V))
    H = math.log(V)
    h_eq = math.sqrt(oracle.draft_step(z, 1.0, 9.0, 0, 40, [0.1]).entropy[0])
    assert abs(h_eq - math.sqrt(H)) < 1e-12
    assert oracle.draft_step(z, 1.0, h_eq, 0, 40, [0.1]).stop[0] == 0          # equality continues
    assert oracle.draft_step(z, 1.0, np.nextafter(h_eq, 0), 0, 40, [0.1]).stop[0] == 1
    assert oracle.draft_step(z, 1.0, 9.0, 38, 40, [0.1]).stop[0] == 0
    r = oracle.draft_step(z, 1.0, 9.0, 39, 40, [0.1])                            # reached the cap
    assert r.stop[0] == 1 and math.isinf(r.margin_h[0])


def test_skipped_rows():
    z = _rng(3).normal(0, 1, (3, 10))
    r = oracle.draft_step(z, 1.0, 0.3, 0, 8, [0.1, 0.2, 0.3], stop_in=[0, 1, 0])
    assert r.token[1] == -1 and r.stop[1] == 1
    full = oracle.draft_step(z, 1.0, 0.3, 0, 8, [0.1, 0.2, 0.3])
    assert r.token[0] == full.token[0] and r.token[2] == full.token[2]


# ---------------------------------------------------------------- sampler

def test_inverse_cdf_matches_searchsorted_on_fine_grid():
    rng = _rng(4)
    for V in (2, 8, 33):
        q = rng.dirichlet(np.ones(V))
        cdf = np.cumsum(q)
        us = np.concatenate([np.linspace(0, 1, 4001, endpoint=False), rng.random(2000)])
        for u in us:
            i, margin = oracle.inverse_cdf(q, u)
            # keep away from cell edges where cumsum rounding order could differ
            if margin < 1e-12:
                continue
            assert i == int(np.searchsorted(cdf, u * cdf[-1], side="right"))


def test_inverse_cdf_edges():
    q = np.array([0.0, 0.25, 0.0, 0.5, 0.25, 0.0])
    assert oracle.inverse_cdf(q, 0.0)[0] == 1           # first cell with mass
    assert oracle.inverse_cdf(q, 0.25)[0] == 3          # strict: C_1 = 0.25 is not > 0.25
    assert oracle.inverse_cdf(q, np.nextafter(0.25, 0))[0] == 1
    assert oracle.inverse_cdf(q, np.nextafter(1.0, 0))[0] == 4   # never the trailing zero cell
    assert oracle.inverse_cdf(np.zeros(4), 0.3)[0] == -1
    # unnormalised weights give the same draw
    assert oracle.inverse_cdf(7.0 * q, 0.6)[0] == oracle.inverse_cdf(q, 0.6)[0] == 3


def test_draft_sampler_frequencies_chi_square():
    rng = _rng(5)
    V, N = 8, 1_000_000
    z = rng.normal(0, 1.5, V)
    q = scipy.special.softmax(z)
    u = rng.random(N).astype(np.float32)
    zz = np.broadcast_to(z, (N, V))
    r = oracle.draft_step(zz, 1.0, 0.3, 0, 40, u)
    counts = np.bincount(r.token, minlength=V)
    chi2 = ((counts - N * q) ** 2 / (N * q)).sum()
    assert chi2 < CHI2_7DOF_999
    assert np.allclose(r.q_tok, q[r.token], rtol=1e-12)


# ---------------------------------------------------------------- acceptance test (Alg. 2), Eq. beta / tvd / pinsker

def test_identical_models_accept_everything_and_bonus_from_last_row():
    rng = _rng(6)
    B, k, V = 5, 6, 50
    zq = rng.normal(0, 2, (B, k, V))
    zp = np.concatenate([zq, rng.normal(0, 2, (B, 1, V))], 1)
    tok = rng.integers(0, V, (B, k))
    gamma = np.array([6, 3, 1, 0, 5])
    ua = np.concatenate([rng.random((B, k - 1)), np.full((B, 1), np.nextafter(1.0, 0))], 1)
    ur = rng.random(B)
    r = oracle.verify(zp, zq, 1.0, tok, gamma, ua, ur)
    assert np.array_equal(r.n_accepted, gamma)
    for b in range(B):
        g = gamma[b]
        assert np.all(r.accept_prob[b, :g] == 1.0) and np.all(np.isnan(r.accept_prob[b, g:]))
        p = scipy.special.softmax(zp[b, g])
        assert r.next_token[b] == int(np.searchsorted(np.cumsum(p), ur[b] * np.cumsum(p)[-1], side="right"))
        assert r.resid_mass[b] == 0.0


def test_disjoint_supports_reject_at_first_position():
    V, k = 10, 3
    zq = np.full((1, k, V), -np.inf)
    zp = np.full((1, k + 1, V), -np.inf)
    zq[:, :, :5] = 0.0
    zp[:, :, 5:] = np.arange(5)
    r = oracle.verify(zp, zq, 1.0, [[2, 3, 4]], [3], [[0.0, 0.5, 0.5]], [0.37])
    assert r.n_accepted[0] == 0 and r.accept_prob[0, 0] == 0.0
    assert abs(r.resid_mass[0] - 1.0) < 1e-15
    p = scipy.special.softmax(zp[0, 0])
    assert r.next_token[0] == int(np.searchsorted(np.cumsum(p), 0.37, side="right"))


def test_zero_draft_probability_accepts():
    # q(x) = 0 < p(x): the test r*q < p holds for every r
    zq = np.array([[[0.0, -np.inf, 0.0]]])
    zp = np.array([[[0.0, 0.0, 0.0], [0.0, 0.0, 0.0]]])
    r = oracle.verify(zp, zq, 1.0, [[1]], [1], [[0.999]], [0.5])
    assert r.n_accepted[0] == 1 and r.accept_prob[0, 0] == 1.0


def test_accept_probability_is_min_1_ratio_and_frequency_is_beta():
    rng = _rng(7)
    V = 8
    zq, zp = rng.normal(0, 1.5, V), rng.normal(0, 1.5, V)
    q, p = scipy.special.softmax(zq), scipy.special.softmax(zp)
    st = oracle.pair_stats(zp, zq)
    assert abs(st["beta"] - np.minimum(p, q).sum()) < 1e-14
    assert abs(st["beta"] - (1 - st["tvd"])) < 1e-14                        # Eq. tvd
    N = 400_000
    us = rng.random(N)
    d = oracle.draft_step(np.broadcast_to(zq, (N, V)), 1.0, 0.3, 0, 40, us)
    ua = rng.random((N, 1))
    zpp = np.broadcast_to(np.stack([zp, zp]), (N, 2, V))
    r = oracle.verify(zpp, np.broadcast_to(zq, (N, 1, V)), 1.0, d.token[:, None],
                      np.ones(N, np.int64), ua, rng.random(N))
    assert np.allclose(r.accept_prob[:, 0], np.minimum(1.0, p[d.token] / q[d.token]), rtol=1e-12)
    freq = r.n_accepted.mean()
    sigma = math.sqrt(st["beta"] * (1 - st["beta"]) / N)
    assert abs(freq - st["beta"]) < 4.5 * sigma                             # Eq. beta
    # per-token acceptance frequency = min(1, p/q)   (Appendix A, closing remark)
    for x in range(V):
        sel = d.token == x
        a = min(1.0, p[x] / q[x])
        s = math.sqrt(max(a * (1 - a), 1e-12) / sel.sum())
        assert abs(r.n_accepted[sel].mean() - a) < 4.5 * s + 1e-9


def test_kl_direction_and_bounds():
    rng = _rng(8)
    for _ in range(200):
        V = int(rng.integers(2, 40))
        zq, zp = rng.normal(0, rng.uniform(0.1, 4), V), rng.normal(0, rng.uniform(0.1, 4), V)
        q, p = scipy.special.softmax(zq), scipy.special.softmax(zp)
        st = oracle.pair_stats(zp, zq)
        assert abs(st["kl"] - scipy.stats.entropy(q, p)) < 1e-10           # KL(q||p), not KL(p||q)
        assert abs(st["kl"] - (st["hqp"] - st["hq"])) < 1e-10              # Eq. beta-bound
        assert st["beta"] >= 1 - math.sqrt(0.5 * st["kl"]) - 1e-12         # Eq. pinsker
        assert st["beta"] >= 1 - math.sqrt(1 - math.exp(-st["kl"])) - 1e-12  # Appendix B


# ---------------------------------------------------------------- first rejection (Alg. 1 verification loop)

def test_first_rejection_all_patterns():
    k, V = 8, 4
    rng = _rng(9)
    zq = np.zeros((1, k, V))
    zq[:, :, 0] = math.log(2.0)            # q = (.4, .2, .2, .2)
    zp = np.zeros((1, k + 1, V))           # p = uniform: p/q = .625 at token 0
    tok = np.zeros((1, k), np.int64)
    for g in (0, 1, 5, 8):
        for pattern in range(1 << g):
            bits = [(pattern >> j) & 1 for j in range(k)]
            ua = np.array([[0.3 if bits[j] else 0.9 for j in range(k)]])
            r = oracle.verify(zp, zq, 1.0, tok, [g], ua, [rng.random()])
            first = next((j for j in range(g) if not bits[j]), g)
            assert r.n_accepted[0] == first
            assert np.allclose(r.accept_prob[0, :g], 0.625)
            if first < g:
                assert r.next_token[0] != 0 and abs(r.resid_mass[0] - 0.15) < 1e-15
            if g:
                dec = [abs(ua[0, j] - 0.625) for j in range(min(first + 1, g))]
                assert r.margin[0] <= min(dec) + 1e-12


# ---------------------------------------------------------------- decision margins (hand-worked)
#
# The parity tests compare a decision exactly only where the oracle reports a margin of at least
# 1e-6, so a margin that came out too small would silently move decisions out of the comparison
# and one that came out too large would demand more than the bar.  Each margin is pinned to
# values worked by hand on distributions with unequal distances to the two sides.

def test_sampler_margin_hand_worked():
    """Cells of w = (1/4, 1/2, 1/4): [0, 1/4), [1/4, 3/4), [3/4, 1).  The margin is the distance of
    u to the NEARER edge of the chosen cell, as a fraction of the total weight."""
    w = np.array([0.25, 0.5, 0.25])
    for u, tok, m in [(0.3, 1, 0.05), (0.7, 1, 0.05), (0.5, 1, 0.25), (0.74, 1, 0.01), (0.26, 1, 0.01),
                      (0.1, 0, 0.1), (0.2, 0, 0.05), (0.9, 2, 0.1), (0.76, 2, 0.01), (0.0, 0, 0.0)]:
        for scale in (1.0, 8.0, 1e-3):                       # unnormalised weights: same fraction
            i, mar = oracle.inverse_cdf(scale * w, u)
            assert i == tok and abs(mar - m) < 1e-12, (u, scale, i, mar)
    # cells without weight do not shorten the distance: (0, 1/4, 0, 1/2, 1/4, 0), u = 0.3 lies 0.05 into token 3
    i, mar = oracle.inverse_cdf([0.0, 0.25, 0.0, 0.5, 0.25, 0.0], 0.3)
    assert i == 3 and abs(mar - 0.05) < 1e-12
    # the draft step reports the same margin for the same distribution (logits ln 1, ln 2, ln 1)
    z = np.log(np.array([[1.0, 2.0, 1.0]]))
    r = oracle.draft_step(z, 1.0, 9.0, 0, 40, [0.3])
    assert r.token[0] == 1 and abs(r.margin_s[0] - 0.05) < 1e-12
    r = oracle.draft_step(np.repeat(z, 3, 0), 1.0, 9.0, 0, 40, [0.74, 0.1, 0.9])      # per row, not shared
    assert np.allclose(r.margin_s, [0.01, 0.1, 0.1], atol=1e-12)


def test_stop_margin_hand_worked():
    """Uniform logits over 4 tokens: sqrt(H) = sqrt(ln 4) = 1.17741002251547...; margin_h = |sqrt(H) - h|."""
    z = np.zeros((1, 4))
    root = 1.1774100225154747
    for h, stop in [(1.0, 1), (1.5, 0), (1.17, 1), (1.18, 0), (0.3, 1)]:
        r = oracle.draft_step(z, 1.0, h, 0, 40, [0.2])
        assert r.stop[0] == stop and abs(r.margin_h[0] - abs(root - h)) < 1e-12, (h, r.margin_h[0])
    # two-point distribution (1/2, 1/2) at T = 0.5 of logits (0, 0): still uniform, H = ln 2
    r = oracle.draft_step(np.zeros((1, 2)), 0.5, 1.0, 0, 40, [0.2])
    assert abs(r.margin_h[0] - (1.0 - math.sqrt(math.log(2.0)))) < 1e-12
    # at the cap the stop does not depend on the entropy: no margin
    assert math.isinf(oracle.draft_step(z, 1.0, 1.0, 39, 40, [0.2]).margin_h[0])


def test_verify_margins_hand_worked():
    """q = (.4, .2, .2, .2), p uniform: p/q = .625 at token 0, residual max(0, p - q) = (0, .05, .05, .05)."""
    k, V = 4, 4
    zq = np.zeros((1, k, V))
    zq[:, :, 0] = math.log(2.0)
    zp = np.zeros((1, k + 1, V))
    tok = np.zeros((1, k), np.int64)

    def run(ua, ur, g=k):
        return oracle.verify(zp, zq, 1.0, tok, [g], [ua], [ur])

    # accepted, accepted (close), rejected, then a test that would be the closest of all but comes after the rejection
    r = run([0.3, 0.6, 0.9, 0.62], 0.5)
    assert r.n_accepted[0] == 2
    assert np.allclose(r.margin_a[0], [0.325, 0.025, 0.275, 0.005], atol=1e-12)
    assert abs(r.margin_accept[0] - 0.025) < 1e-12            # minimum over positions 0..2 only
    # the correction: u * W = .075 lies in token 2's cell [.05, .10): .025 to either edge, W = .15
    assert r.next_token[0] == 2 and abs(r.margin_sample[0] - 1.0 / 6.0) < 1e-12
    assert abs(r.margin[0] - 0.025) < 1e-12                   # the smaller of the two
    # the rejecting test itself counts
    r = run([0.3, 0.3, 0.63, 0.1], 0.5)
    assert r.n_accepted[0] == 2 and abs(r.margin_accept[0] - 0.005) < 1e-12 and abs(r.margin[0] - 0.005) < 1e-12
    # a draw close to a cell edge: u * W = .0495 -> token 1, .0005 / .15 from the edge at .05
    r = run([0.9, 0.1, 0.1, 0.1], 0.33)
    assert r.n_accepted[0] == 0 and r.next_token[0] == 1
    assert abs(r.margin_accept[0] - 0.275) < 1e-12 and abs(r.margin_sample[0] - 0.0005 / 0.15) < 1e-9
    assert abs(r.margin[0] - 0.0005 / 0.15) < 1e-9
    # everything accepted: the bonus draw from uniform p, u = .3 is .05 into token 1's cell [.25, .5)
    r = run([0.3, 0.1, 0.6, 0.2], 0.3)
    assert r.n_accepted[0] == 4 and r.next_token[0] == 1
    assert abs(r.margin_accept[0] - 0.025) < 1e-12 and abs(r.margin_sample[0] - 0.05) < 1e-12
    # shorter draft: positions at or beyond draft_len are not tested and carry no margin
    r = run([0.3, 0.1, 0.6249, 0.6251], 0.3, g=2)
    assert r.n_accepted[0] == 2 and abs(r.margin_accept[0] - 0.325) < 1e-12 and np.isnan(r.margin_a[0, 2:]).all()
    # nothing drafted: only the bonus draw decides
    r = run([0.3, 0.1, 0.6, 0.2], 0.9, g=0)
    assert r.n_accepted[0] == 0 and r.next_token[0] == 3 and math.isinf(r.margin_accept[0])
    assert abs(r.margin_sample[0] - 0.1) < 1e-12 and abs(r.margin[0] - 0.1) < 1e-12


# ---------------------------------------------------------------- residual direction and the output law

@pytest.mark.parametrize("seed", [11, 12, 13])
def test_output_law_equals_target_brute_force(seed):
    """V = 8, 10^6 draft/verify/correct trials: emitted token ~ p (chi-square, 7 dof, 99.9 %).
    The printed q - p residual (Algorithm 4 as typeset) fails the same test."""
    rng = _rng(seed)
    V, N = 8, 1_000_000
    p, q = rng.dirichlet(np.ones(V)), rng.dirichlet(np.ones(V))
    hist, nacc = oracle.sd_position_trials(p, q, N, seed, +1)
    assert hist.sum() == N
    assert ((hist - N * p) ** 2 / (N * p)).sum() < CHI2_7DOF_999
    beta = np.minimum(p, q).sum()
    assert abs(nacc / N - beta) < 4.5 * math.sqrt(beta * (1 - beta) / N)
    bad, _ = oracle.sd_position_trials(p, q, N, seed, -1)
    assert ((bad - N * p) ** 2 / (N * p)).sum() > 100 * CHI2_7DOF_999


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_output_law_through_the_entry_points(seed):
    """Same law, but through draft_step + verify themselves (k = 1, one sequence per trial)."""
    rng = _rng(seed)
    V, N = 8, 1_000_000
    zq, zp, zb = rng.normal(0, 1.2, V), rng.normal(0, 1.2, V), rng.normal(0, 1.2, V)
    p, pb = scipy.special.softmax(zp), scipy.special.softmax(zb)
    d = oracle.draft_step(np.broadcast_to(zq, (N, V)), 1.0, 0.3, 0, 40, rng.random(N))
    r = oracle.verify(np.broadcast_to(np.stack([zp, zb]), (N, 2, V)),
                      np.broadcast_to(zq, (N, 1, V)), 1.0, d.token[:, None],
                      np.ones(N, np.int64), rng.random((N, 1)), rng.random(N))
    acc = r.n_accepted == 1
    emitted = np.where(acc, d.token, r.next_token)
    hist = np.bincount(emitted, minlength=V)
    assert ((hist - N * p) ** 2 / (N * p)).sum() < CHI2_7DOF_999
    # bonus tokens (drawn when the draft was accepted) follow the next target row
    nb = acc.sum()
    hb = np.bincount(r.next_token[acc], minlength=V)
    assert ((hb - nb * pb) ** 2 / (nb * pb)).sum() < CHI2_7DOF_999
    # corrections never return a token with p <= q
    q = scipy.special.softmax(zq)
    assert np.all((p > q)[r.next_token[~acc]])


def test_exact_output_law_enumeration():
    """P(out = i) = min(p_i, q_i) + (1 - beta) w_i / W must equal p_i, with w from oracle_verify's
    own residual (read back through resid_mass and forced corrections on a u grid)."""
    rng = _rng(31)
    V = 8
    zq, zp = rng.normal(0, 1.5, V), rng.normal(0, 1.5, V)
    q, p = scipy.special.softmax(zq), scipy.special.softmax(zp)
    # force a rejection at position 0 (ua just below 1 with a token where p < q) and sweep ur
    x = int(np.argmax(q - p))
    grid = (np.arange(200_000) + 0.5) / 200_000
    N = grid.size
    r = oracle.verify(np.broadcast_to(np.stack([zp, zp]), (N, 2, V)), np.broadcast_to(zq, (N, 1, V)),
                      1.0, np.full((N, 1), x), np.ones(N, np.int64),
                      np.full((N, 1), np.nextafter(1.0, 0)), grid)
    assert np.all(r.n_accepted == 0)
    w_hat = np.bincount(r.next_token, minlength=V) / N        # law of the correction
    beta = np.minimum(p, q).sum()
    assert abs(r.resid_mass[0] - (1 - beta)) < 1e-14
    out_law = np.minimum(p, q) + (1 - beta) * w_hat
    assert np.allclose(out_law, p, atol=2.0 / N)


def test_zero_residual_falls_back_to_target():
    # p == q exactly, rejection cannot happen for u < 1; force the branch with gamma rows equal
    # and an acceptance uniform of exactly 1.0 (outside [0,1), used only to reach the branch)
    z = np.log(np.array([[0.1, 0.2, 0.3, 0.4]]))
    r = oracle.verify(np.stack([z[0], z[0]])[None], z[None], 1.0, [[2]], [1], [[1.0]], [0.45])
    assert r.n_accepted[0] == 0 and r.resid_mass[0] == 0.0
    assert r.next_token[0] == 2 and r.margin[0] == 0.0


# ---------------------------------------------------------------- greedy decoding (Algorithms 3 and 5)

def test_argmax_first_maximum_and_numpy():
    rng = _rng(41)
    for V in (1, 2, 7, 1000):
        z = rng.normal(0, 2, V)
        assert oracle.argmax_row(z) == int(np.argmax(z))
    z = np.array([0.5, 3.0, -1.0, 3.0, 3.0, 2.0])
    assert oracle.argmax_row(z) == 1                       # smallest index among equal maxima
    assert oracle.argmax_row(np.array([-np.inf, -np.inf, -5.0])) == 2
    zq = np.round(rng.normal(0, 1, (4, 50)) * 4) / 4       # coarse values: ties are common
    r = oracle.draft_step_greedy(zq, 1.0, 0.3, 0, 40)
    assert np.array_equal(r.token, np.argmax(zq, axis=1))
    s = oracle.draft_step(zq, 1.0, 0.3, 0, 40, rng.random(4))
    assert np.allclose(r.entropy, s.entropy) and np.allclose(r.lse, s.lse) and np.array_equal(r.stop, s.stop)
    p = scipy.special.softmax(zq, axis=1)
    assert np.allclose(r.q_tok, p[np.arange(4), r.token], rtol=1e-12)


def test_greedy_verify_all_prefix_lengths():
    rng = _rng(42)
    B, k, V = 9, 8, 30
    zp = rng.normal(0, 2, (B, k + 1, V))
    am = np.argmax(zp, axis=2)
    tok = am[:, :k].copy()
    gamma = np.array([8, 8, 5, 0, 1, 8, 3, 8, 8])
    first_bad = [8, 0, 2, 0, 0, 7, 3, 4, 8]                # where the draft departs from argmax p
    for b, j in enumerate(first_bad):
        if j < k:
            tok[b, j] = (am[b, j] + 1) % V
    nacc, nxt = oracle.verify_greedy(zp, tok, gamma)
    for b in range(B):
        r = min(first_bad[b], gamma[b])
        assert nacc[b] == r and nxt[b] == am[b, r]


def test_greedy_is_the_zero_temperature_limit_of_sampling():
    """At a tiny temperature the softmax of a tie-free row is one-hot at its argmax, so the
    sampling oracle (already pinned) must reproduce the greedy one."""
    rng = _rng(43)
    B, k, V = 6, 5, 40
    zq = rng.normal(0, 3, (B, k, V))
    zp = np.concatenate([zq, rng.normal(0, 3, (B, 1, V))], 1) + rng.normal(0, 2.0, (B, k + 1, V))
    T = 1e-3
    tok = np.zeros((B, k), np.int64)
    for j in range(k):
        g = oracle.draft_step_greedy(zq[:, j], 1.0, 9.0, j, k + 1)
        s = oracle.draft_step(zq[:, j], T, 9e9, j, k + 1, rng.random(B))
        assert np.array_equal(g.token, s.token)
        tok[:, j] = g.token
    gamma = np.full(B, k)
    nacc, nxt = oracle.verify_greedy(zp, tok, gamma)
    s = oracle.verify(zp, zq, T, tok, gamma, rng.random((B, k)), rng.random(B))
    assert np.array_equal(nacc, s.n_accepted) and np.array_equal(nxt, s.next_token)
    assert (nacc < k).any()          # the perturbed target does reject somewhere


def test_greedy_identical_models_accept_everything():
    rng = _rng(44)
    B, k, V = 4, 6, 25
    z = rng.normal(0, 1, (B, k + 1, V))
    tok = np.argmax(z[:, :k], axis=2)
    nacc, nxt = oracle.verify_greedy(z, tok, np.array([6, 4, 0, 1]))
    assert np.array_equal(nacc, [6, 4, 0, 1])
    assert np.array_equal(nxt, [np.argmax(z[b, g]) for b, g in enumerate([6, 4, 0, 1])])


# ---------------------------------------------------------------- diagnostics (Section 2.2, Appendix B)

def test_diagnostics_two_point_closed_form():
    """p = (a, 1-a), q = (b, 1-b): every quantity has an elementary closed form."""
    a, b, c = 0.5, 0.25, 0.2
    zp = np.log(np.array([[[a, 1 - a], [a, 1 - a]]]))          # [1, k+1 = 2, V = 2]
    zq = np.log(np.array([[[b, 1 - b]]]))                      # [1, k = 1, 2]
    d = oracle.diagnostics(zp, zq, 1.0, [1], c)[0, 0]
    beta = 1 - abs(a - b)                                       # min(a,b) + min(1-a,1-b)
    hq = -(b * math.log(b) + (1 - b) * math.log(1 - b))
    hqp = -(b * math.log(a) + (1 - b) * math.log(1 - a))
    kl = b * math.log(b / a) + (1 - b) * math.log((1 - b) / (1 - a))
    want = [beta, kl, hqp, hq, 1 - math.sqrt(kl / 2), 1 - math.sqrt(1 - math.exp(-kl)),
            1 - math.sqrt(c * hq), hqp / hq]
    assert np.allclose(d, want, rtol=0, atol=1e-14)
    # digits worked by hand for this pair: beta = 3/4, KL = 0.75 ln 1.5 - 0.25 ln 2
    assert abs(d[0] - 0.75) < 1e-15 and abs(d[1] - 0.13081203594113694) < 1e-15
    assert abs(d[4] - 0.7442538) < 1e-6 and abs(d[5] - 0.6498333) < 1e-6


def test_diagnostics_identities_and_signs():
    rng = _rng(21)
    B, k = 3, 4
    for trial in range(30):
        V = int(rng.integers(2, 50))
        zq = rng.normal(0, rng.uniform(0.2, 5), (B, k, V))
        zp = rng.normal(0, rng.uniform(0.2, 5), (B, k + 1, V))
        c = float(rng.uniform(0.05, 1.0))
        g = rng.integers(0, k + 1, B)
        d = oracle.diagnostics(zp, zq, 1.0, g, c)
        for b in range(B):
            assert np.isnan(d[b, g[b]:]).all() and np.isfinite(d[b, :g[b]]).all()
            for j in range(g[b]):
                beta, kl, hqp, hq, bo, bh, ba, ratio = d[b, j]
                assert beta >= bo - 1e-12 and beta >= bh - 1e-12          # both are lower bounds
                assert bh > 0.0                                            # Appendix B: always positive
                # the bound written with gamma = H_{q,p}/H_q is the oracle bound again
                assert abs(bo - (1 - math.sqrt(0.5 * (ratio - 1) * hq))) < 1e-9
                # the approximation is conservative exactly when c >= (gamma - 1) / 2
                assert (ba <= bo + 1e-12) == (c >= 0.5 * (ratio - 1) - 1e-12)
    # a far-apart pair: KL > 2 makes the Pinsker form negative while Bretagnolle-Huber stays positive
    zp = np.array([[[8.0, 0.0], [0.0, 0.0]]])
    zq = np.array([[[0.0, 8.0]]])
    d = oracle.diagnostics(zp, zq, 1.0, [1], 0.3)[0, 0]
    assert d[1] > 2 and d[4] < 0 < d[5] <= d[0]


def test_diagnostics_uniform_and_temperature():
    V, k = 64, 2
    z = np.zeros((1, k + 1, V))
    d = oracle.diagnostics(z, z[:, :k], 1.0, [k], 0.1)
    lnV = math.log(V)
    assert np.allclose(d[0, :, :6], [1.0, 0.0, lnV, lnV, 1.0, 1.0], atol=1e-12)
    assert np.allclose(d[0, :, 6], 1 - math.sqrt(0.1 * lnV)) and np.allclose(d[0, :, 7], 1.0)
    rng = _rng(22)
    zp, zq = rng.normal(0, 3, (2, k + 1, V)), rng.normal(0, 3, (2, k, V))
    assert np.allclose(oracle.diagnostics(zp, zq, 2.0, [k, 1], 0.2), oracle.diagnostics(zp / 2, zq / 2, 1.0, [k, 1], 0.2),
                       rtol=1e-12, equal_nan=True)


# ---------------------------------------------------------------- the decoding loop (Algorithms 1 and 6)

def _cdf_draw(z, u):
    """Inverse-CDF draw from softmax(z) written with library routines."""
    c = np.cumsum(scipy.special.softmax(z))
    return int(np.searchsorted(c, u * c[-1], side="right"))


def test_loop_constant_length_identical_models():
    """p = q: every drafted token is accepted, a round of gamma draft tokens yields gamma + 1
    (Algorithm 6); the tokens are the draws themselves."""
    rng = _rng(31)
    L, V, gam, new = 80, 12, 5, 40
    z = rng.normal(0, 2, (L, V))
    R = 20
    us, ua, ur = rng.random((R, gam)), rng.random((R, gam)), rng.random(R)
    r = oracle.generate(z, z, 1.0, 3, new, np.inf, gam, gam, 0, 0, us, ua, ur)
    rounds = -(-new // (gam + 1))
    assert r.log.shape[0] == rounds and r.tokens.size == rounds * (gam + 1)     # overshoots max_new within a round
    for i in range(rounds):
        n = 3 + i * (gam + 1)
        assert r.log[i].tolist()[:4] == [n, gam, gam, gam]
        want = [_cdf_draw(z[n + j], us[i, j]) for j in range(gam)] + [_cdf_draw(z[n + gam], ur[i])]
        assert r.tokens[i * (gam + 1):(i + 1) * (gam + 1)].tolist() == want
        assert r.log[i, 4] == want[-1]


def test_loop_heuristic_length_rule():
    """Next length + 2 after a fully accepted round, - 1 otherwise, kept inside [1, limit]."""
    rng = _rng(32)
    L, V = 400, 6
    z = rng.normal(0, 1, (L, V))
    R = 12
    u = rng.random((R, 12))
    r = oracle.generate(z, z, 1.0, 0, 10 ** 6, np.inf, 5, 12, 2, 1, u, u, rng.random(R), max_rounds=R)
    assert r.log[:, 1].tolist() == [5, 7, 9, 11, 12, 12, 12, 12, 12, 12, 12, 12]
    assert (r.log[:, 2] == r.log[:, 1]).all() and (r.log[:, 3] == r.log[:, 1]).all()
    # disjoint supports: the first drafted token always fails and the correction is the target's token
    zp = np.full((L, V), -np.inf)
    zp[:, 0] = 0.0
    zq = np.full((L, V), -np.inf)
    zq[:, 1] = 0.0
    r = oracle.generate(zp, zq, 1.0, 0, 9, np.inf, 5, 12, 2, 1, u, u, rng.random(R))
    assert r.log[:, 1].tolist() == [5, 4, 3, 2, 1, 1, 1, 1, 1]
    assert (r.log[:, 3] == 0).all() and (r.tokens == 0).all() and r.tokens.size == 9
    assert r.log[:, 0].tolist() == list(range(9))                      # one token per round


def test_loop_entropy_threshold_draft_lengths():
    """Algorithm 1 on a trace whose flat rows (sqrt(H) = sqrt(ln V) > h) sit at known positions:
    drafting runs up to and including the first flat row, the round adds one bonus token."""
    L, V, h, cap = 64, 50, 1.0, 6
    flat = {2, 3, 11, 12, 13, 30, 31, 40, 47, 55}
    z = np.zeros((L, V))
    for n in range(L):
        if n not in flat:
            z[n, (7 * n) % V] = 40.0                                     # H ~ 0
    rng = _rng(33)
    R = 30
    us, ua, ur = rng.random((R, cap)), rng.random((R, cap)), rng.random(R)
    r = oracle.generate(z, z, 1.0, 0, 40, h, cap, cap, 0, 0, us, ua, ur)
    n, want = 0, []
    while n < 40 and n + cap + 1 <= L:
        d = next((f - n + 1 for f in sorted(flat) if f >= n and f - n + 1 <= cap), cap)
        want.append([n, cap, d, d])
        n += d + 1
    assert r.log[:, :4].tolist() == want
    # sharp rows yield their spike
    pos = np.concatenate([np.arange(a, a + d + 1) for a, _, d, _ in want])
    sharp = np.array([p not in flat for p in pos])
    assert (r.tokens[sharp] == (7 * pos[sharp]) % V).all()


def test_loop_tokens_per_round_matches_geometric_law():
    """Same (p, q) at every position: each drafted token is accepted with probability beta, so a
    round of gamma drafts produces (1 - beta^(gamma+1)) / (1 - beta) tokens on average, and the
    produced tokens follow p."""
    rng = _rng(34)
    V, gam, R = 5, 4, 6000
    zq, zp = rng.normal(0, 1, V), rng.normal(0, 1, V)
    L = R * (gam + 1) + gam + 2
    beta = oracle.pair_stats(zp, zq)["beta"]
    r = oracle.generate(np.broadcast_to(zp, (L, V)), np.broadcast_to(zq, (L, V)), 1.0, 0, 10 ** 9, np.inf,
                        gam, gam, 0, 0, rng.random((R, gam)), rng.random((R, gam)), rng.random(R))
    assert r.log.shape[0] == R
    per_round = r.log[:, 3] + 1
    mean = (1 - beta ** (gam + 1)) / (1 - beta)
    assert abs(per_round.mean() - mean) < 4.5 * per_round.std() / math.sqrt(R)
    p = scipy.special.softmax(zp)
    cnt = np.bincount(r.tokens, minlength=V)
    chi2 = ((cnt - r.tokens.size * p) ** 2 / (r.tokens.size * p)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, V - 1)


def test_loop_greedy_and_limits():
    rng = _rng(35)
    L, V = 50, 9
    zq = rng.normal(0, 1, (L, V))
    zp = zq.copy()
    zp[7] = -zq[7]                                                        # argmax differs at position 7
    r = oracle.generate(zp, zq, 1.0, 0, 20, np.inf, 4, 4, 0, 0, greedy=True)
    am_q, am_p = zq.argmax(1), zp.argmax(1)
    assert r.log[:, :4].tolist()[:3] == [[0, 4, 4, 4], [5, 4, 4, 2], [8, 4, 4, 4]]
    assert r.tokens[:5].tolist() == am_q[:5].tolist() and r.tokens[5:8].tolist() == [am_q[5], am_q[6], am_p[7]]
    # the trace must hold cap + 1 rows from n on: no round starts past L - cap - 1
    r = oracle.generate(zq, zq, 1.0, 40, 100, np.inf, 4, 4, 0, 0, greedy=True)
    assert r.log[:, 0].tolist() == [40, 45] and r.tokens.size == 10
    # max_new is tested at the start of a round only
    r = oracle.generate(zq, zq, 1.0, 0, 6, np.inf, 4, 4, 0, 0, greedy=True)
    assert r.log.shape[0] == 2 and r.tokens.size == 10


# ---------------------------------------------------------------- top-k / top-p filtering (a variant, not in the paper)

def test_warp_hand_worked_and_switches():
    z = np.log(np.array([0.1, 0.5, 0.2, 0.2]))
    keep, m = oracle.warp_row(z)                               # both filters off
    assert keep.all() and m == math.inf
    assert oracle.warp_row(z, top_k=4)[0].all() and oracle.warp_row(z, top_k=9)[0].all()
    assert oracle.warp_row(z, top_k=1)[0].tolist() == [False, True, False, False]
    assert oracle.warp_row(z, top_k=2)[0].tolist() == [False, True, True, True]      # the tie at 0.2 stays together
    assert oracle.warp_row(z, top_k=3)[0].tolist() == [False, True, True, True]
    keep, m = oracle.warp_row(z, top_p=0.6)                    # 0.5 < 0.6 <= 0.9
    assert keep.tolist() == [False, True, True, True] and abs(m - 0.1) < 1e-12
    keep, m = oracle.warp_row(z, top_p=0.45)
    assert keep.tolist() == [False, True, False, False] and abs(m - 0.05) < 1e-12
    keep, m = oracle.warp_row(z, top_p=0.95)
    assert keep.all() and abs(m - 0.05) < 1e-12
    # top-k first, then top-p on the renormalised survivors: {0.5, 0.2, 0.2} / 0.9, target 0.5 -> {0.5} has 0.556
    keep, m = oracle.warp_row(z, top_k=2, top_p=0.5)
    assert keep.tolist() == [False, True, False, False] and abs(m - (0.5 / 0.9 - 0.5)) < 1e-12
    # the nucleus is measured against the mass top-k left (0.9), not against 1: 0.5 / 0.9 = 0.556 >= 0.55
    keep, m = oracle.warp_row(z, top_k=2, top_p=0.55)
    assert keep.tolist() == [False, True, False, False] and abs(m - (0.5 / 0.9 - 0.55)) < 1e-12
    assert oracle.warp_row(z, top_p=0.55)[0].sum() == 3
    # temperature changes the nucleus, not the top-k set
    assert oracle.warp_row(z, T=3.0, top_k=1)[0].tolist() == [False, True, False, False]
    assert oracle.warp_row(z, T=5.0, top_p=0.6)[0].sum() == 3 and oracle.warp_row(z, T=0.2, top_p=0.6)[0].sum() == 1


def test_warp_against_sorting_with_library_routines():
    rng = _rng(41)
    for trial in range(300):
        V = int(rng.integers(1, 60))
        z = np.round(rng.normal(0, 2, V), int(rng.integers(0, 3)))          # coarse rounding makes ties
        if rng.random() < 0.3:
            z[rng.random(V) < 0.3] = -np.inf
            z[int(rng.integers(0, V))] = 0.0
        T = float(rng.choice([0.5, 1.0, 2.0]))
        k = int(rng.integers(0, V + 3))
        p_ = float(rng.choice([1.0, 0.9, 0.5, 0.1]))
        keep, margin = oracle.warp_row(z, T, k, p_)
        q = scipy.special.softmax(z / T)
        kept = np.ones(V, bool)
        if 0 < k < V:
            kept = z >= np.sort(z)[::-1][k - 1]
        if p_ < 1.0:
            Zk = q[kept].sum()
            vals = np.unique(z[kept])[::-1]
            for v in vals:
                if q[kept & (z >= v)].sum() >= p_ * Zk - 1e-15:
                    break
            if margin > 1e-12:
                assert (keep == (kept & (z >= v))).all()
                # minimal: without its lowest value the set falls short of top_p
                higher = kept & (z > v)
                assert q[higher].sum() < p_ * Zk
                assert q[keep].sum() >= p_ * Zk - 1e-15
        else:
            assert (keep == kept).all() and margin == math.inf
        # survivors are the largest logits: nothing dropped exceeds anything kept
        if keep.any() and (~keep).any():
            assert z[~keep].max() < z[keep].min()
