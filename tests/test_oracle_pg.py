"""Pins of the oracle's token-level clipped policy-gradient loss (no GPU)."""
import numpy as np
import pytest
import torch
from scipy import special as spc


def _case(seed=0, T=12, H=8, V=16, B=3, w_std=0.5, noise=0.3, masked=True):
    rng = np.random.default_rng(seed)
    cuts = np.sort(rng.choice(np.arange(1, T), B - 1, replace=False))
    cu = np.concatenate([[0], cuts, [T]]).astype(np.int32)
    c = dict(
        hidden=rng.standard_normal((T, H)),
        W=rng.standard_normal((V, H)) * w_std,
        target=rng.integers(0, V, T).astype(np.int32),
        mask=(rng.random(T) > 0.25).astype(np.uint8) if masked else None,
        adv_norm=rng.standard_normal(B),
        cu_seqlens=cu,
    )
    z = c["hidden"] @ c["W"].T
    logp = spc.log_softmax(z, axis=1)[np.arange(T), c["target"]]
    c["old_logp"] = logp + rng.standard_normal(T) * noise
    c["z"], c["logp_ref"] = z, logp
    return c


def _args(c):
    return (c["hidden"], c["W"], c["target"], c["old_logp"], c["mask"], c["adv_norm"],
            c["cu_seqlens"])


def test_logp_and_lse_match_scipy(oracle):
    c = _case(1, T=20, H=16, V=50)
    out = oracle.pg_loss_fwd(*_args(c))
    np.testing.assert_allclose(out["lse"], spc.logsumexp(c["z"], axis=1), rtol=1e-13)
    np.testing.assert_allclose(out["logp"], c["logp_ref"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["ratio"], np.exp(c["logp_ref"] - c["old_logp"]), rtol=1e-12)
    # logits-in variant sees the same numbers
    out2 = oracle.pg_loss_fwd(None, None, *_args(c)[2:], logits=c["z"])
    for k in ("lse", "logp", "ratio", "obj"):
        np.testing.assert_allclose(out2[k], out[k], rtol=1e-12, atol=1e-13)
    assert out2["loss"] == pytest.approx(out["loss"], rel=1e-12)
    # huge logits do not overflow
    big = c["z"] + 5000.0
    out3 = oracle.pg_loss_fwd(None, None, *_args(c)[2:], logits=big)
    np.testing.assert_allclose(out3["logp"], out["logp"], rtol=1e-9, atol=1e-9)


def test_single_vocabulary_entry(oracle):
    c = _case(2, V=1)
    out = oracle.pg_loss_fwd(*_args(c))
    assert np.array_equal(out["logp"], np.zeros_like(out["logp"]))


def test_shift_invariance(oracle):
    # adding one vector to every vocabulary row shifts all logits of a token
    # equally: log-probs, loss and the hidden-state gradient do not move
    c = _case(3)
    base_f = oracle.pg_loss_fwd(*_args(c))
    base_b = oracle.pg_loss_bwd(*_args(c))
    c2 = dict(c)
    c2["W"] = c["W"] + np.random.default_rng(0).standard_normal(c["W"].shape[1])[None, :]
    sh_f = oracle.pg_loss_fwd(*_args(c2))
    sh_b = oracle.pg_loss_bwd(*_args(c2))
    np.testing.assert_allclose(sh_f["logp"], base_f["logp"], rtol=1e-11, atol=1e-12)
    assert sh_f["loss"] == pytest.approx(base_f["loss"], rel=1e-11)
    np.testing.assert_allclose(sh_b["d_hidden"], base_b["d_hidden"], rtol=1e-9, atol=1e-13)


def test_ratio_one_is_mean_cross_entropy(oracle):
    # ratio = 1, advantage = 1, no mask: the objective is 1 per token (loss = -1)
    # and its gradient is the gradient of the mean token cross-entropy.
    c = _case(4, masked=False)
    c["old_logp"] = c["logp_ref"].copy()
    c["adv_norm"] = np.ones_like(c["adv_norm"])
    f = oracle.pg_loss_fwd(*_args(c))
    assert f["loss"] == pytest.approx(-1.0, rel=1e-12)
    assert np.all(f["active"] == 1)
    b = oracle.pg_loss_bwd(*_args(c))
    h = torch.tensor(c["hidden"], requires_grad=True)
    w = torch.tensor(c["W"], requires_grad=True)
    ce = torch.nn.functional.cross_entropy(h @ w.T, torch.tensor(c["target"], dtype=torch.long))
    ce.backward()
    np.testing.assert_allclose(b["d_hidden"], h.grad.numpy(), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(b["d_W"], w.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_logit_gradient_is_minus_adv_softmax_minus_onehot(oracle):
    # at ratio 1 with the clip inactive the gradient of the OBJECTIVE w.r.t. the
    # logits is adv * (onehot - softmax); the loss is minus the objective / M
    c = _case(5, masked=False)
    c["old_logp"] = c["logp_ref"].copy()
    T, V = c["z"].shape
    b = oracle.pg_loss_bwd(None, None, *_args(c)[2:], logits=c["z"])
    p = spc.softmax(c["z"], axis=1)
    onehot = np.eye(V)[c["target"]]
    seq = np.searchsorted(c["cu_seqlens"], np.arange(T), side="right") - 1
    adv_t = c["adv_norm"][seq]
    np.testing.assert_allclose(b["d_logits"], adv_t[:, None] * (p - onehot) / T, rtol=1e-11,
                               atol=1e-15)
    np.testing.assert_allclose(b["d_logits"].sum(axis=1), 0, atol=1e-15)


def _torch_loss(c, eps_low, eps_high):
    """The objective typed in torch only to let autograd derive the gradients."""
    h = torch.tensor(c["hidden"], requires_grad=True)
    w = torch.tensor(c["W"], requires_grad=True)
    T = h.shape[0]
    lp = torch.log_softmax(h @ w.T, dim=1)[torch.arange(T), torch.tensor(c["target"], dtype=torch.long)]
    ratio = torch.exp(lp - torch.tensor(c["old_logp"]))
    seq = np.searchsorted(c["cu_seqlens"], np.arange(T), side="right") - 1
    adv = torch.tensor(c["adv_norm"][seq])
    obj = torch.minimum(ratio * adv, torch.clamp(ratio, 1 - eps_low, 1 + eps_high) * adv)
    m = torch.ones(T, dtype=torch.float64) if c["mask"] is None else torch.tensor(c["mask"], dtype=torch.float64)
    loss = -(m * obj).sum() / m.sum()
    loss.backward()
    return loss.item(), h.grad.numpy(), w.grad.numpy()


@pytest.mark.parametrize("seed", [6, 7, 8])
def test_gradients_match_autograd_and_finite_differences(oracle, seed):
    c = _case(seed, T=10, H=6, V=12, noise=0.35)
    el, eh = 0.2, 0.28
    f = oracle.pg_loss_fwd(*_args(c), eps_low=el, eps_high=eh)
    b = oracle.pg_loss_bwd(*_args(c), eps_low=el, eps_high=eh)
    # the case exercises both branches of the min
    assert 0 < f["active"].sum() < len(f["active"])
    loss_t, dh_t, dw_t = _torch_loss(c, el, eh)
    assert f["loss"] == pytest.approx(loss_t, rel=1e-12)
    np.testing.assert_allclose(b["d_hidden"], dh_t, rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(b["d_W"], dw_t, rtol=1e-9, atol=1e-14)
    # central differences of the oracle's own forward, away from the clip kinks
    margin = np.minimum(np.abs(f["ratio"] - (1 - el)), np.abs(f["ratio"] - (1 + eh)))
    assert margin.min() > 1e-4
    rng = np.random.default_rng(seed)
    h = 1e-6
    for _ in range(12):
        for name, grad in (("hidden", b["d_hidden"]), ("W", b["d_W"])):
            i = rng.integers(0, c[name].shape[0])
            j = rng.integers(0, c[name].shape[1])
            cp, cm = dict(c), dict(c)
            cp[name] = c[name].copy(); cp[name][i, j] += h
            cm[name] = c[name].copy(); cm[name][i, j] -= h
            fd = (oracle.pg_loss_fwd(*_args(cp), eps_low=el, eps_high=eh)["loss"]
                  - oracle.pg_loss_fwd(*_args(cm), eps_low=el, eps_high=eh)["loss"]) / (2 * h)
            assert grad[i, j] == pytest.approx(fd, rel=2e-6, abs=1e-9)
    # grad_loss scales linearly
    b2 = oracle.pg_loss_bwd(*_args(c), eps_low=el, eps_high=eh, grad_loss=-2.5)
    np.testing.assert_allclose(b2["d_W"], -2.5 * b["d_W"], rtol=1e-12, atol=1e-16)


def test_clipped_tokens_have_clipped_value_and_zero_gradient(oracle):
    c = _case(9, T=8, B=2, masked=False)
    c["adv_norm"] = np.array([1.0, -1.0])
    half = int(c["cu_seqlens"][1])
    # ratio 2 everywhere: clipped for positive advantage, active for negative
    c["old_logp"] = c["logp_ref"] - np.log(2.0)
    f = oracle.pg_loss_fwd(*_args(c), eps_low=0.2, eps_high=0.28)
    np.testing.assert_allclose(f["ratio"], 2.0, rtol=1e-12)
    np.testing.assert_allclose(f["obj"][:half], 1.28, rtol=1e-12)
    np.testing.assert_allclose(f["obj"][half:], -2.0, rtol=1e-12)
    assert not f["active"][:half].any() and f["active"][half:].all()
    b = oracle.pg_loss_bwd(*_args(c), eps_low=0.2, eps_high=0.28)
    assert np.array_equal(b["d_hidden"][:half], np.zeros_like(b["d_hidden"][:half]))
    assert np.abs(b["d_hidden"][half:]).min() > 0
    # ratio 1/2: the roles swap, the lower bound 1 - eps_low is the one that binds
    c["old_logp"] = c["logp_ref"] + np.log(2.0)
    f = oracle.pg_loss_fwd(*_args(c), eps_low=0.2, eps_high=0.28)
    np.testing.assert_allclose(f["obj"][:half], 0.5, rtol=1e-12)
    np.testing.assert_allclose(f["obj"][half:], -0.8, rtol=1e-12)
    assert f["active"][:half].all() and not f["active"][half:].any()


def test_ratio_one_loss_is_minus_masked_mean_advantage(oracle):
    c = _case(10)
    c["old_logp"] = c["logp_ref"].copy()
    f = oracle.pg_loss_fwd(*_args(c))
    T = len(c["target"])
    seq = np.searchsorted(c["cu_seqlens"], np.arange(T), side="right") - 1
    m = c["mask"].astype(float)
    assert f["loss"] == pytest.approx(-(m * c["adv_norm"][seq]).sum() / m.sum(), rel=1e-11)
    assert f["M"] == m.sum()


def test_mask_equals_token_removal_and_chunks_add_up(oracle):
    c = _case(11, T=16, B=4)
    f = oracle.pg_loss_fwd(*_args(c))
    b = oracle.pg_loss_bwd(*_args(c))
    keep = np.flatnonzero(c["mask"])
    T = len(c["target"])
    seq = np.searchsorted(c["cu_seqlens"], np.arange(T), side="right") - 1
    cc = dict(c)
    for k in ("hidden", "target", "old_logp"):
        cc[k] = c[k][keep]
    cc["mask"] = None
    cc["cu_seqlens"] = np.concatenate([[0], np.cumsum(np.bincount(seq[keep], minlength=4))]).astype(np.int32)
    f2 = oracle.pg_loss_fwd(*_args(cc))
    b2 = oracle.pg_loss_bwd(*_args(cc))
    assert f2["loss"] == pytest.approx(f["loss"], rel=1e-12)
    np.testing.assert_allclose(b2["d_W"], b["d_W"], rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(b2["d_hidden"], b["d_hidden"][keep], rtol=1e-10, atol=1e-15)
    assert np.array_equal(b["d_hidden"][c["mask"] == 0], np.zeros((T - len(keep), 8)))
    # (sum of mask*obj, sum of mask) is additive over any split of the tokens
    m = c["mask"].astype(float)
    s = -(f["loss"] * f["M"])
    assert s == pytest.approx((m[:7] * f["obj"][:7]).sum() + (m[7:] * f["obj"][7:]).sum(), rel=1e-12)
    # all tokens masked: zero loss, zero gradients
    c0 = dict(c)
    c0["mask"] = np.zeros(T, np.uint8)
    assert oracle.pg_loss_fwd(*_args(c0))["loss"] == 0.0
    assert not oracle.pg_loss_bwd(*_args(c0))["d_W"].any()


def test_row_subsets_and_structure_of_the_gradients(oracle):
    c = _case(12, T=14, H=8, V=20, B=3)
    f = oracle.pg_loss_fwd(*_args(c))
    b = oracle.pg_loss_bwd(*_args(c))
    rows = np.array([13, 2, 7])
    fr = oracle.pg_loss_fwd(*_args(c), rows=rows)
    for k in ("lse", "logp", "ratio", "obj"):
        assert np.array_equal(fr[k], f[k][rows])
    br = oracle.pg_loss_bwd(*_args(c), rows=rows, want_dw=False)
    assert np.array_equal(br["d_hidden"], b["d_hidden"][rows])
    vs = np.array([19, 0, 5])
    bv = oracle.pg_loss_bwd(*_args(c), vsel=vs, want_dx=False)
    assert np.array_equal(bv["d_W"], b["d_W"][vs])
    # softmax rows sum to one -> the head gradient sums to zero over the vocabulary
    np.testing.assert_allclose(b["d_W"].sum(axis=0), 0, atol=1e-14)
    # a token's hidden gradient depends on that token only
    c2 = dict(c)
    c2["hidden"] = c["hidden"].copy()
    c2["hidden"][4] += 1.0
    c2["old_logp"] = c["old_logp"].copy()
    b2 = oracle.pg_loss_bwd(*_args(c2))
    others = np.arange(14) != 4
    np.testing.assert_allclose(b2["d_hidden"][others], b["d_hidden"][others], rtol=1e-12, atol=1e-16)
    # the advantage of response b reaches exactly the tokens of response b
    c3 = dict(c)
    c3["adv_norm"] = c["adv_norm"].copy()
    c3["adv_norm"][1] *= 3.0
    f3 = oracle.pg_loss_fwd(*_args(c3))
    lo, hi = c["cu_seqlens"][1], c["cu_seqlens"][2]
    changed = f3["obj"] != f["obj"]
    assert changed[lo:hi].all() and not changed[:lo].any() and not changed[hi:].any()
