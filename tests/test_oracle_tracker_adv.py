"""Pins of the oracle's tracker and advantage routines against what the paper
and the mathematics fix (no GPU, no HIP code involved)."""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats as sps


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split()
            out[k] = float(v)
    return out


G = _golden()


# ------------------------------------------------------------------ tracker
def test_discount_one_gives_beta_posterior_counts(oracle):
    # Beta is the conjugate prior of the Bernoulli: with no forgetting the
    # parameters are prior + number of successes / failures, exactly.
    rng = np.random.default_rng(0)
    N = 7
    a = np.full(N, 0.5)
    b = np.full(N, 0.5)
    succ = np.zeros(N)
    fail = np.zeros(N)
    for step in range(40):
        idx = rng.permutation(N)[:4].astype(np.int32)
        r = rng.integers(0, 2, 4).astype(np.float64)
        a, b, _, rho = oracle.tracker_update(a, b, idx, r, np.zeros(4), 0.25, 1.0, 1.0)
        assert np.all(rho == 1.0)
        np.add.at(succ, idx, r)
        np.add.at(fail, idx, 1 - r)
    assert np.array_equal(a, 0.5 + succ)
    assert np.array_equal(b, 0.5 + fail)


def test_half_life_and_clamp(oracle):
    # D = D_half halves the memory; D = 0 keeps it; both clamps saturate.
    assert oracle.discount(0.25, 0.25, 0.0, 1.0) == 0.5
    assert oracle.discount(0.5, 0.25, 0.0, 1.0) == 0.25
    assert oracle.discount(0.0, 0.25, 0.0, 1.0) == 1.0
    assert oracle.discount(0.0, 0.25, G["rho_min"], G["rho_max"]) == G["rho_max"]
    assert oracle.discount(10.0, 0.25, G["rho_min"], G["rho_max"]) == G["rho_min"]
    mid = oracle.discount(0.03, 0.25, G["rho_min"], G["rho_max"])
    assert mid == pytest.approx(2.0 ** (-0.12), rel=1e-15)
    assert G["rho_min"] < mid < G["rho_max"]
    # negative divergence is read as zero
    assert oracle.discount(-1.0, 0.25, 0.0, 1.0) == 1.0


def test_hand_worked_updates(oracle):
    # Three updates of one prompt worked by hand in exact rationals.
    a, b = Fraction(1, 2), Fraction(1, 2)
    steps = [  # (reward, kl, expected clamped rho)
        (1, 0.25, Fraction(7, 8)),      # 2^-1 = 0.5 -> clamped up to 0.875
        (0, 0.0, Fraction(24, 25)),     # 2^0 = 1   -> clamped down to 0.96
        (1, 10.0, Fraction(7, 8)),
    ]
    oa, ob = np.array([0.5]), np.array([0.5])
    for r, kl, rho in steps:
        v_before = a / (a + b)
        oa, ob, vprev, orho = oracle.tracker_update(oa, ob, [0], [float(r)], [kl], 0.25,
                                                    0.875, 0.96)
        a, b = rho * a + r, rho * b + (1 - r)
        assert orho[0] == pytest.approx(float(rho), abs=1e-16)
        assert vprev[0] == pytest.approx(float(v_before), rel=1e-15)
        assert oa[0] == pytest.approx(float(a), rel=1e-15)
        assert ob[0] == pytest.approx(float(b), rel=1e-15)
    # a success must raise alpha, not beta (catches swapped r / 1-r)
    a1, b1, _, _ = oracle.tracker_update([2.0], [3.0], [0], [1.0], [0.0], 0.25, 1.0, 1.0)
    assert (a1[0], b1[0]) == (3.0, 3.0)
    a0, b0, _, _ = oracle.tracker_update([2.0], [3.0], [0], [0.0], [0.0], 0.25, 1.0, 1.0)
    assert (a0[0], b0[0]) == (2.0, 4.0)


def test_ema_identity(oracle):
    # The update is an EMA on the posterior mean with step 1/(rho*(alpha+beta)+1)
    # taken on the PRE-update parameters.
    rng = np.random.default_rng(1)
    N = 64
    a = rng.uniform(0.5, 50, N)
    b = rng.uniform(0.5, 50, N)
    idx = np.arange(N, dtype=np.int32)
    r = rng.integers(0, 2, N).astype(np.float64)
    kl = rng.exponential(0.02, N)
    a2, b2, vprev, rho = oracle.tracker_update(a, b, idx, r, kl, 0.25, 0.875, 0.96)
    eta = 1.0 / (rho * (a + b) + 1.0)
    v_ema = vprev + eta * (r - vprev)
    np.testing.assert_allclose(a2 / (a2 + b2), v_ema, rtol=1e-13)
    np.testing.assert_allclose(vprev, a / (a + b), rtol=1e-15)


def test_effective_sample_size_fixed_point(oracle):
    # alpha+beta obeys n <- rho*n + 1 whose fixed point is 1/(1-rho):
    # exactly 8 at rho_min = 0.875 (0.875*8+1 = 8) and 25 at rho_max = 0.96.
    a, b = np.array([3.0]), np.array([5.0])
    for r in [1, 0, 0, 1, 1, 0]:
        a, b, _, _ = oracle.tracker_update(a, b, [0], [float(r)], [100.0], 0.25,
                                           G["rho_min"], G["rho_max"])
        assert a[0] + b[0] == G["window_min"]
    a, b = np.array([0.5]), np.array([0.5])
    for i in range(2000):
        a, b, _, _ = oracle.tracker_update(a, b, [0], [float(i % 2)], [0.0], 0.25,
                                           G["rho_min"], G["rho_max"])
    assert a[0] + b[0] == pytest.approx(G["window_max"], rel=1e-12)


def test_duplicates_are_sequential(oracle):
    a, b, vprev, _ = oracle.tracker_update([1.0, 1.0], [1.0, 1.0], [1, 1, 0], [1.0, 1.0, 0.0],
                                           [0.25, 0.25, 0.0], 0.25, 0.0, 1.0)
    # prompt 1: (1,1) -> (1.5, 0.5) -> (1.75, 0.25); prompt 0: (1,1) -> (1,2)
    assert (a[1], b[1]) == (1.75, 0.25)
    assert (a[0], b[0]) == (1.0, 2.0)
    assert list(vprev) == [0.5, 0.75, 0.5]


def test_initialisation(oracle):
    v0 = np.array([0.0, 0.125, 0.5, 1.0])
    a0, b0 = oracle.tracker_init(v0, G["rho_min"])
    assert np.array_equal(a0 + b0, np.full(4, G["window_min"]))   # N0 = 1/(1-0.875) = 8
    assert np.array_equal(a0, 8 * v0)
    # mean of n0 = 8 binary outcomes is reproduced exactly
    outcomes = np.array([1, 0, 0, 1, 1, 0, 1, 1.0])
    a0, b0 = oracle.tracker_init([outcomes.mean()], G["rho_min"])
    assert a0[0] == outcomes.sum() and b0[0] == G["n0"] - outcomes.sum()


# --------------------------------------------------------------- advantages
def _case(seed=0, N=50, B=24):
    rng = np.random.default_rng(seed)
    a = rng.uniform(0.5, 20, N)
    b = rng.uniform(0.5, 20, N)
    idx = rng.permutation(N)[:B].astype(np.int32)
    r = rng.integers(0, 2, B).astype(np.float64)
    return a, b, idx, r


def test_advantages_zero_mean_unit_std_and_zscore(oracle):
    a, b, idx, r = _case()
    raw, nrm, (mu, sigma) = oracle.advantages(a, b, idx, r)
    v = a[idx] / (a[idx] + b[idx])
    np.testing.assert_allclose(raw, r - v, rtol=1e-15)
    assert abs(nrm.mean()) < 1e-14
    assert nrm.std() == pytest.approx(1.0, rel=1e-13)
    np.testing.assert_allclose(nrm, sps.zscore(r - v), rtol=1e-12)          # library routine
    assert mu == pytest.approx(np.mean(r - v), rel=1e-13)
    assert sigma == pytest.approx(np.std(r - v), rel=1e-13)
    # sample standard deviation when ddof = 1
    _, nrm1, (_, s1) = oracle.advantages(a, b, idx, r, ddof=1)
    np.testing.assert_allclose(nrm1, sps.zscore(r - v, ddof=1), rtol=1e-12)
    assert s1 == pytest.approx(np.std(r - v, ddof=1), rel=1e-13)


def test_advantages_sign_and_affine_invariance(oracle):
    a, b, idx, _ = _case(1)
    r = np.zeros(idx.shape[0])
    r[:5] = 1.0
    raw, nrm, _ = oracle.advantages(a, b, idx, r)
    # a success above its baseline is a positive raw advantage
    assert np.all(raw[:5] > 0) and np.all(raw[5:] < 0)
    # normalised advantages do not change when every reward is mapped r -> c r + d
    # with the baseline switched off (then A = r)
    _, n0, _ = oracle.advantages(a, b, idx, r, use_baseline=False)
    _, n1, _ = oracle.advantages(a, b, idx, 3.0 * r + 2.0, use_baseline=False)
    np.testing.assert_allclose(n0, n1, rtol=1e-12)
    np.testing.assert_allclose(n0, sps.zscore(r), rtol=1e-12)


def test_advantages_two_samples_and_degenerate(oracle):
    raw, nrm, _ = oracle.advantages([1.0, 3.0], [1.0, 1.0], [0, 1], [1.0, 0.0])
    assert list(raw) == [0.5, -0.75]
    assert list(nrm) == [1.0, -1.0]
    # all advantages equal -> sigma = 0 -> zeros, not NaN
    _, nrm, (mu, sigma) = oracle.advantages([1.0, 1.0, 1.0], [1.0, 1.0, 1.0], [0, 1, 2],
                                            [1.0, 1.0, 1.0])
    assert sigma == 0.0 and mu == 0.5 and np.array_equal(nrm, np.zeros(3))
    # eps_norm enters the denominator
    _, nrm, (_, s) = oracle.advantages([1.0, 3.0], [1.0, 1.0], [0, 1], [1.0, 0.0], eps_norm=0.375)
    assert s == 0.625 and list(nrm) == [0.625, -0.625]


def test_advantage_uses_pre_update_baseline(oracle):
    a, b, idx, r = _case(2)
    kl = np.full(idx.shape[0], 0.02)
    raw_pre, _, _ = oracle.advantages(a, b, idx, r)
    a2, b2, vprev, _ = oracle.tracker_update(a, b, idx, r, kl, 0.25, 0.875, 0.96)
    raw_post, _, _ = oracle.advantages(a2, b2, idx, r)
    np.testing.assert_allclose(raw_pre, r - vprev, rtol=1e-15)
    # the update pulls the baseline towards the reward: |A| strictly shrinks
    assert np.all(np.abs(raw_post) < np.abs(raw_pre))


def test_dynamic_sampling_cost_constant():
    # off-path doc test of a closed form the paper prints
    p = G["dyn_sampling_p"]
    assert round(1.0 / (p * (1 - p)) - 1.0, 2) == G["dyn_sampling_cost"]


def test_advantage_diagnostics_match_numpy(oracle):
    rng = np.random.default_rng(3)
    a = rng.normal(0, 0.3, 500)
    a[:40] = rng.uniform(-1e-4, 1e-4, 40)      # inside the tight tolerance
    a[40:120] = rng.uniform(0.001, 0.02, 80)   # inside the loose one only
    r = rng.integers(0, 2, 500).astype(float)
    d = oracle.advantage_diagnostics(a, r, 1e-4, 0.02)
    assert d[0] == np.mean(np.abs(a) <= 1e-4) and d[0] >= 40 / 500
    assert d[1] == np.mean(np.abs(a) <= 0.02) and d[1] >= 120 / 500
    assert d[2] == pytest.approx(np.var(a), rel=1e-13)
    assert d[3] == pytest.approx(np.var(r), rel=1e-13)
    # a perfect baseline halves nothing and removes everything: A = r - p has variance p(1-p),
    # the raw reward of a prompt mix has variance >= that (law of total variance)
    p = rng.uniform(0, 1, 20000)
    r = (rng.random(20000) < p).astype(float)
    d = oracle.advantage_diagnostics(r - p, r)
    assert d[2] < d[3]
    assert d[2] == pytest.approx(np.mean(p * (1 - p)), rel=0.05)


def test_general_rewards_follow_the_same_ema(oracle):
    # non-binary rewards in [0, 1]: the same update keeps v = alpha/(alpha+beta) on the EMA
    rng = np.random.default_rng(4)
    N = 32
    a, b = rng.uniform(0.5, 20, N), rng.uniform(0.5, 20, N)
    r = rng.uniform(0, 1, N)
    kl = rng.exponential(0.02, N)
    a2, b2, vprev, rho = oracle.tracker_update(a, b, np.arange(N, dtype=np.int32), r, kl, 0.25, 0.875, 0.96)
    np.testing.assert_allclose(a2 / (a2 + b2), vprev + (r - vprev) / (rho * (a + b) + 1.0), rtol=1e-13)
    np.testing.assert_allclose(a2 + b2, rho * (a + b) + 1.0, rtol=1e-14)


def test_ema_form_is_a_discounted_weighted_mean(oracle):
    # Closed form: with constant discount rho the moving-average form is the
    # weighted mean (rho^k n0 v0 + sum_j rho^(k-1-j) r_j) / (rho^k n0 + sum_j rho^(k-1-j)),
    # in exact rationals, for rewards that are neither binary nor inside [0, 1].
    rho = Fraction(7, 8)
    v0, n0 = Fraction(1, 4), Fraction(8)
    rs = [Fraction(5, 2), Fraction(-3), Fraction(0), Fraction(7, 3), Fraction(1, 10)]
    v, n = np.array([float(v0)]), np.array([float(n0)])
    num, den = n0 * v0, n0
    for r in rs:
        v, n, vprev = oracle.tracker_update_ema(v, n, [0], [float(r)], [10.0], 0.25, float(rho), 0.96)
        assert vprev[0] == pytest.approx(float(num / den), rel=1e-14)
        num, den = rho * num + r, rho * den + 1
        assert v[0] == pytest.approx(float(num / den), rel=1e-14)
        assert n[0] == pytest.approx(float(den), rel=1e-15)
    # rho = 1: the plain running mean with the prior counted n0 times
    v, n, _ = oracle.tracker_update_ema([0.5] * 1, [2.0], [0, 0, 0], [4.0, -1.0, 9.0], [0.0] * 3, 0.25, 1.0, 1.0)
    assert v[0] == pytest.approx((2.0 * 0.5 + 12.0) / 5.0, rel=1e-15) and n[0] == 5.0


def test_ema_form_agrees_with_the_beta_form(oracle):
    # v = alpha/(alpha+beta), n = alpha+beta: both forms track the same estimate,
    # also through repeated ids and both clamps of the discount.
    rng = np.random.default_rng(8)
    N, B = 16, 200
    a, b = rng.uniform(0.5, 20, N), rng.uniform(0.5, 20, N)
    idx = rng.integers(0, N, B).astype(np.int32)
    r = rng.integers(0, 2, B).astype(np.float64)
    kl = rng.exponential(0.03, B)
    a2, b2, vp_beta, _ = oracle.tracker_update(a, b, idx, r, kl, 0.25, 0.875, 0.96)
    v2, n2, vp_ema = oracle.tracker_update_ema(a / (a + b), a + b, idx, r, kl, 0.25, 0.875, 0.96)
    np.testing.assert_allclose(v2, a2 / (a2 + b2), rtol=1e-12)
    np.testing.assert_allclose(n2, a2 + b2, rtol=1e-12)
    np.testing.assert_allclose(vp_ema, vp_beta, rtol=1e-12)


def test_advantages_accept_the_estimate_itself(oracle):
    rng = np.random.default_rng(9)
    a, b = rng.uniform(0.5, 20, 32), rng.uniform(0.5, 20, 32)
    idx = rng.permutation(32)[:12].astype(np.int32)
    r = rng.uniform(-2, 2, 12)
    raw1, nrm1, st1 = oracle.advantages(a, b, idx, r)
    raw2, nrm2, st2 = oracle.advantages(a / (a + b), None, idx, r)
    np.testing.assert_allclose(raw2, raw1, rtol=1e-13)
    np.testing.assert_allclose(nrm2, nrm1, rtol=1e-12)
    np.testing.assert_allclose(raw2, r - (a / (a + b))[idx], rtol=1e-15)
