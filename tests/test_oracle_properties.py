"""Randomised invariants of the oracle (no GPU): properties that the paper's
definitions imply at any size, checked on shapes and values drawn by hypothesis."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

SET = settings(max_examples=25, deadline=None, derandomize=True)


def _state(rng, n):
    return rng.uniform(0.05, 30.0, n), rng.uniform(0.05, 30.0, n)


@SET
@given(st.integers(1, 40), st.integers(1, 60), st.integers(0, 2 ** 31 - 1))
def test_tracker_effective_size_and_range(oracle, n, b, seed):
    # alpha + beta follows rho * (alpha + beta) + 1 whatever the reward, the mean stays in
    # [0, 1] for rewards in [0, 1], and untouched prompts keep their state
    rng = np.random.default_rng(seed)
    a, bb = _state(rng, n)
    idx = rng.integers(0, n, b).astype(np.int32)
    r = rng.uniform(0, 1, b)
    kl = rng.exponential(0.05, b)
    a2, b2, vprev, rho = oracle.tracker_update(a, bb, idx, r, kl, 0.25, 0.875, 0.96)
    assert ((rho >= 0.875) & (rho <= 0.96)).all()
    size = a + bb
    for k in range(b):
        size[idx[k]] = rho[k] * size[idx[k]] + 1.0
    np.testing.assert_allclose(a2 + b2, size, rtol=1e-12)
    v = a2 / (a2 + b2)
    assert ((v >= 0) & (v <= 1)).all() and ((vprev >= 0) & (vprev <= 1)).all()
    untouched = np.setdiff1d(np.arange(n), idx)
    assert np.array_equal(a2[untouched], a[untouched]) and np.array_equal(b2[untouched], bb[untouched])


@SET
@given(st.integers(2, 50), st.integers(0, 2 ** 31 - 1))
def test_tracker_update_of_distinct_prompts_commutes(oracle, b, seed):
    rng = np.random.default_rng(seed)
    n = b + 5
    a, bb = _state(rng, n)
    idx = rng.permutation(n)[:b].astype(np.int32)
    r = rng.integers(0, 2, b).astype(np.float64)
    kl = rng.exponential(0.05, b)
    p = rng.permutation(b)
    a1, b1, _, _ = oracle.tracker_update(a, bb, idx, r, kl, 0.25, 0.875, 0.96)
    a2, b2, _, _ = oracle.tracker_update(a, bb, idx[p], r[p], kl[p], 0.25, 0.875, 0.96)
    assert np.array_equal(a1, a2) and np.array_equal(b1, b2)


@SET
@given(st.integers(2, 64), st.floats(-5, 5), st.floats(0.1, 10), st.integers(0, 2 ** 31 - 1))
def test_advantages_are_equivariant_and_scale_free(oracle, b, shift, scale, seed):
    # permuting the batch permutes the result; without a baseline an affine map of the rewards
    # with positive slope changes nothing after normalisation
    rng = np.random.default_rng(seed)
    n = b + 3
    a, bb = _state(rng, n)
    idx = rng.permutation(n)[:b].astype(np.int32)
    r = rng.normal(size=b)
    raw, nrm, (mu, sg) = oracle.advantages(a, bb, idx, r)
    p = rng.permutation(b)
    raw_p, nrm_p, _ = oracle.advantages(a, bb, idx[p], r[p])
    np.testing.assert_allclose(raw_p, raw[p], rtol=0, atol=0)
    np.testing.assert_allclose(nrm_p, nrm[p], rtol=1e-10, atol=1e-12)
    assert abs(nrm.mean()) < 1e-10 and (sg == 0 or abs(nrm.std() - 1) < 1e-10)
    _, n0, _ = oracle.advantages(a, bb, idx, r, use_baseline=False)
    _, n1, _ = oracle.advantages(a, bb, idx, scale * r + shift, use_baseline=False)
    np.testing.assert_allclose(n1, n0, rtol=1e-8, atol=1e-9)


@SET
@given(st.integers(2, 200), st.integers(1, 64), st.integers(0, 2 ** 20), st.integers(0, 1000))
def test_sampling_without_replacement_is_a_stable_distinct_prefix(oracle, n, b, seed, it):
    b = min(b, n)
    rng = np.random.default_rng(seed)
    a, bb = _state(rng, n)
    a, bb = a.astype(np.float32), bb.astype(np.float32)
    idx = oracle.sample_prompts(a, bb, b, 0.05, seed, it, False)
    assert len(set(idx.tolist())) == b and idx.min() >= 0 and idx.max() < n
    shorter = oracle.sample_prompts(a, bb, max(1, b // 2), 0.05, seed, it, False)
    assert np.array_equal(shorter, idx[:len(shorter)])
    # slot 0 never needs a second attempt, so it equals the first draw with replacement
    assert oracle.sample_prompts(a, bb, 1, 0.05, seed, it, True)[0] == idx[0]


@SET
@given(st.integers(1, 12), st.integers(2, 40), st.integers(0, 2 ** 31 - 1))
def test_loss_is_invariant_to_logit_shifts_and_vocabulary_order(oracle, t, v, seed):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 2, (t, v))
    tgt = rng.integers(0, v, t).astype(np.int32)
    old = rng.normal(-np.log(v), 0.3, t)
    adv = rng.normal(size=2)
    cut = int(rng.integers(0, t + 1))
    cu = np.array([0, cut, t], np.int32)
    mask = (rng.uniform(size=t) < 0.8).astype(np.uint8)
    ref = oracle.pg_loss_fwd(None, None, tgt, old, mask, adv, cu, 0.2, 0.28, logits=z)
    shifted = oracle.pg_loss_fwd(None, None, tgt, old, mask, adv, cu, 0.2, 0.28, logits=z + rng.normal(0, 50, (t, 1)))
    assert shifted["loss"] == pytest.approx(ref["loss"], rel=1e-9, abs=1e-12)
    np.testing.assert_allclose(shifted["logp"], ref["logp"], atol=1e-10)
    perm = rng.permutation(v)
    inv = np.empty(v, np.int64)
    inv[perm] = np.arange(v)
    moved = oracle.pg_loss_fwd(None, None, inv[tgt].astype(np.int32), old, mask, adv, cu, 0.2, 0.28, logits=z[:, perm])
    assert moved["loss"] == pytest.approx(ref["loss"], rel=1e-9, abs=1e-12)
    # every log-probability is at most 0 and the probabilities of a row sum to 1
    assert (ref["logp"] <= 1e-12).all()
    np.testing.assert_allclose(np.exp(z - ref["lse"][:, None]).sum(axis=1), 1.0, rtol=1e-10)


@SET
@given(st.integers(1, 8), st.integers(2, 24), st.integers(1, 6), st.floats(0.1, 4), st.integers(0, 2 ** 31 - 1))
def test_gradient_is_linear_in_the_upstream_gradient_and_sums_to_zero(oracle, t, v, h, c, seed):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(t, h))
    w = rng.normal(0, 0.5, (v, h))
    tgt = rng.integers(0, v, t).astype(np.int32)
    adv = rng.normal(size=1)
    cu = np.array([0, t], np.int32)
    f = oracle.pg_loss_fwd(x, w, tgt, np.zeros(t), None, adv, cu, 0.2, 0.28)
    old = f["logp"] + rng.normal(0, 0.15, t)
    g1 = oracle.pg_loss_bwd(x, w, tgt, old, None, adv, cu, 0.2, 0.28, grad_loss=1.0)
    gc = oracle.pg_loss_bwd(x, w, tgt, old, None, adv, cu, 0.2, 0.28, grad_loss=c)
    np.testing.assert_allclose(gc["d_hidden"], c * g1["d_hidden"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(gc["d_W"], c * g1["d_W"], rtol=1e-12, atol=1e-15)
    # softmax rows sum to one and so does the one-hot: the logit gradient sums to zero over the
    # vocabulary, hence d_W sums to zero over its vocabulary rows
    np.testing.assert_allclose(g1["d_W"].sum(axis=0), 0.0, atol=1e-12)
