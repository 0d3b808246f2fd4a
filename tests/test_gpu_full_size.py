"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot evaluate 10^5..10^6 tokens over 151936 vocabulary entries, so:
  * lse, logp and dHidden rows are compared on sampled tokens (each evaluated by
    the oracle over the full vocabulary);
  * dW is compared on sampled vocabulary rows in a second run whose loss mask
    keeps only a few hundred tokens: the kernels still sweep every token, but the
    gradient is then fully determined by tokens the oracle can evaluate;
  * properties that hold at any size: the scalar loss equals an fp64 reduction of
    the kernel's own per-token values, dW sums to zero over the vocabulary, rows of
    masked tokens are zero, and sampled rows of the dense run's dW equal the fp64
    sum over ALL tokens of g_t (onehot - exp(h_t.w_v - lse_t)) h_t formed from the
    kernel's own lse and logp (which the sampled-token comparison checks against the
    oracle): the contraction over 131072 tokens per launch and the accumulation across
    launches are exercised exactly as the benchmark runs them;
  * a dense run on a contiguous slice of whole responses (about 1200 tokens) at the
    full hidden and vocabulary size, where the oracle evaluates every token itself:
    loss, lse, logp, dW on sampled vocabulary rows, dHidden rows and their softmax
    part alone, with the benchmark's flat logits and with a peaked softmax (head
    weights scaled by 8).
"""
import numpy as np
import pytest
import torch

from paper_2509_13232_amd import workloads as wl
from pg_cases import f64, rel_l2, say

pytestmark = pytest.mark.gpu
GRAD_TOL = 1e-2


@pytest.fixture(scope="module")
def spo():
    from paper_2509_13232_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _sub_problem(tb, W64, rows, adv, seq, old):
    """Oracle inputs in which every sampled token is a response of its own."""
    n = len(rows)
    h = tb.hidden[torch.as_tensor(rows, device=tb.hidden.device)].double().cpu().numpy()
    return (h, W64, tb.target[rows], old[rows].astype(np.float64), None, adv[seq[rows]].astype(np.float64),
            np.arange(n + 1, dtype=np.int32))


def _dw_rows_fp64(tb, vsel, g, lse, chunk=1 << 15):
    """sum_t g_t (onehot(y_t)[v] - exp(h_t . w_v - lse_t)) h_t for the vocabulary rows in vsel, in fp64
    (torch matmuls on the device the inputs live on; none of the library's kernels)."""
    dev = tb.hidden.device
    Wsel = tb.W[torch.as_tensor(vsel, device=dev)].double()                  # [nv, H]
    out = torch.zeros_like(Wsel)
    vs = torch.as_tensor(vsel, device=dev)
    for s0 in range(0, tb.T, chunk):
        e = min(tb.T, s0 + chunk)
        h = tb.hidden[s0:e].double()
        gt = torch.as_tensor(g[s0:e], device=dev)
        z = h @ Wsel.t()                                                     # [n, nv]
        dz = -torch.exp(z - torch.as_tensor(lse[s0:e], device=dev)[:, None])
        dz += (torch.as_tensor(tb.target[s0:e], device=dev).long()[:, None] == vs[None, :]).double()
        out += (dz * gt[:, None]).t() @ h
    return out.cpu().numpy()


def _run_full(spo, oracle, name, n_rows, n_dw_tokens, n_vsel):
    cfg = wl.CONFIGS[name]
    say(f"full-size {name}: generating inputs")
    tb = wl.token_batch(cfg, device="cuda")
    T, H, V, B = tb.T, cfg.H, cfg.V, cfg.B
    rng = np.random.default_rng([wl.MASTER_SEED, 7])
    adv = rng.standard_normal(B)
    adv = ((adv - adv.mean()) / adv.std()).astype(np.float32)
    seq = np.searchsorted(tb.cu_seqlens, np.arange(T), side="right") - 1
    old_t = wl.behaviour_logp_standin(tb.hidden, tb.W, tb.target, cfg.w_std, tb.noise)
    old = old_t.cpu().numpy()
    dev = lambda x, dt: torch.as_tensor(x).to("cuda", dt).contiguous()
    target, cu, advg = dev(tb.target, torch.int32), dev(tb.cu_seqlens, torch.int32), dev(adv, torch.float32)
    mask = None if tb.mask is None else dev(tb.mask, torch.uint8)
    M = T if tb.mask is None else int(tb.mask.sum())
    W64 = tb.W.double().cpu().numpy()

    # ---------------------------------------------------------------- run 1: the benchmark configuration
    say(f"full-size {name}: T={T} H={H} V={V} forward+backward")
    desc = spo.make_desc(tb.hidden, tb.W, target, old_t, mask, advg, cu, cfg.eps_low, cfg.eps_high)
    special = [0, 255, 256, T - 1, T - 2, (T // 256) * 256 - 1, min(T - 1, (T // 256) * 256)]
    rows = np.unique(np.concatenate([rng.choice(T, n_rows, replace=False), special])).astype(np.int64)
    say(f"full-size {name}: oracle on {len(rows)} sampled tokens")
    sub = _sub_problem(tb, W64, rows, adv, seq, old)
    ref = oracle.pg_loss_fwd(*sub, cfg.eps_low, cfg.eps_high)
    rg = torch.as_tensor(rows, device="cuda")
    # gradient rows: the sub-problem normalises by its own token count, the kernel by M
    rb = oracle.pg_loss_bwd(*sub, cfg.eps_low, cfg.eps_high, grad_loss=len(rows) / M, want_dw=False)
    lo, hi = 1 - cfg.eps_low, 1 + cfg.eps_high
    vs0 = np.unique(np.concatenate([rng.choice(V, 96, replace=False), tb.target[rows[:16]],
                                    [0, 255, 256, V - 1, (V // 256) * 256]])).astype(np.int64)
    # the same checks for both ways to the gradients: forward then backward (logits formed twice),
    # and the one call that keeps a piece's logits (the configuration the benchmark times)
    for path in ("fwd_then_bwd", "one_call"):
        say(f"full-size {name}: T={T} H={H} V={V} {path}")
        if path == "one_call":
            loss, logp, lse, stats, dx, dw = spo.spo_pg_loss_fwd_bwd(desc, 1.0)
        else:
            loss, logp, lse, stats = spo.spo_pg_loss_fwd(desc)
            dx, dw = spo.spo_pg_loss_bwd(desc, logp, lse, 1.0)
        torch.cuda.synchronize()
        np.testing.assert_allclose(f64(lse[rg]), ref["lse"], atol=2e-4, rtol=0)
        np.testing.assert_allclose(f64(logp[rg]), ref["logp"], atol=2e-4, rtol=0)
        keep = np.ones(len(rows), bool)
        keep &= ~((np.abs(ref["ratio"] - lo) < 2e-3 * lo) | (np.abs(ref["ratio"] - hi) < 2e-3 * hi))
        unmasked = np.ones(len(rows), bool) if tb.mask is None else tb.mask[rows].astype(bool)
        got = f64(dx[rg])
        want = rb["d_hidden"] * unmasked[:, None]
        assert keep.sum() > 0.9 * len(rows)
        assert rel_l2(got[keep], want[keep]) < GRAD_TOL
        assert np.abs(got[keep & ~unmasked]).max(initial=0.0) == 0.0
        per_row = np.linalg.norm(got[keep & unmasked] - want[keep & unmasked], axis=1)
        scale = np.linalg.norm(want[keep & unmasked], axis=1)
        active = scale > 0
        assert (per_row[active] <= 2 * GRAD_TOL * scale[active]).all()          # no single bad row hides in the norm
        assert (per_row[~active] == 0).all()                                     # clipped tokens: exactly zero rows
        # loss: equals the fp64 reduction of the kernel's own per-token log-probs
        lp = f64(logp)
        ratio = np.exp(lp - old.astype(np.float64))
        a = adv.astype(np.float64)[seq]
        obj = np.minimum(ratio * a, np.clip(ratio, lo, hi) * a)
        m = np.ones(T) if tb.mask is None else tb.mask.astype(np.float64)
        want_loss = -(m * obj).sum() / m.sum()
        assert abs(loss.item() - want_loss) <= 2e-3 * abs(want_loss) + 1e-7
        assert stats[0].item() == M
        # softmax rows sum to one: dW sums to zero over the vocabulary (per hidden unit)
        col = dw.sum(dim=0).abs().max().item()
        assert col <= 1e-2 * dw.abs().sum(dim=0).max().item()
        # dense dW, every token: sampled vocabulary rows against an fp64 sum over all T tokens formed
        # from the kernel's own lse and logp (a consistency property, not an oracle value).  Rows that a
        # token within rounding of a clip bound points at are left out: fp32 and fp64 may disagree on
        # whether that token carries a gradient.
        say(f"full-size {name}: dense dW rows against an fp64 reduction over all {T} tokens ({path})")
        g_all = -(m / m.sum()) * a * ratio * (ratio * a <= np.clip(ratio, lo, hi) * a)
        edge = (np.abs(ratio - lo) < 1e-5 * lo) | (np.abs(ratio - hi) < 1e-5 * hi)
        vs1 = np.setdiff1d(vs0, tb.target[edge])
        want_rows = _dw_rows_fp64(tb, vs1, g_all, f64(lse))
        got_rows = f64(dw[torch.as_tensor(vs1, device="cuda")])
        assert rel_l2(got_rows, want_rows) < GRAD_TOL
        hit1 = np.isin(vs1, tb.target[g_all != 0])
        if (~hit1).any():      # rows no token sampled: the softmax part alone
            assert rel_l2(got_rows[~hit1], want_rows[~hit1]) < 2 * GRAD_TOL
        per_v = np.linalg.norm(got_rows - want_rows, axis=1)
        assert (per_v <= 3 * GRAD_TOL * np.linalg.norm(want_rows, axis=1) + 1e-3 * np.abs(want_rows).max()).all()
        del dx, dw

    # ---------------------------------------------------------------- run 2: sparse mask, dW on sampled rows
    say(f"full-size {name}: sparse-mask run for dW ({n_dw_tokens} live tokens, {n_vsel} vocabulary rows)")
    live = np.unique(np.concatenate([rng.choice(T, n_dw_tokens, replace=False), [0, T - 1]])).astype(np.int64)
    # tokens whose ratio sits on a clip bound (fp32 and fp64 may take different branches) stay masked
    cand = oracle.pg_loss_fwd(*_sub_problem(tb, W64, live, adv, seq, old), cfg.eps_low, cfg.eps_high)["ratio"]
    live = live[~((np.abs(cand - lo) < 2e-3 * lo) | (np.abs(cand - hi) < 2e-3 * hi))]
    m2 = np.zeros(T, np.uint8)
    m2[live] = 1
    desc2 = spo.make_desc(tb.hidden, tb.W, target, old_t, dev(m2, torch.uint8), advg, cu, cfg.eps_low, cfg.eps_high)
    loss2, logp2, lse2, _ = spo.spo_pg_loss_fwd(desc2)
    _, dw2 = spo.spo_pg_loss_bwd(desc2, logp2, lse2, 1.0, want_d_hidden=False)
    loss3, _, _, _, _, dw3 = spo.spo_pg_loss_fwd_bwd(desc2, 1.0, want_d_hidden=False)
    torch.cuda.synchronize()
    sub2 = _sub_problem(tb, W64, live, adv, seq, old)
    vsel = np.unique(np.concatenate([rng.choice(V, n_vsel, replace=False), tb.target[live[:8]],
                                     [0, V - 1, (V // 256) * 256, 255, 256]])).astype(np.int64)
    rb2 = oracle.pg_loss_bwd(*sub2, cfg.eps_low, cfg.eps_high, vsel=vsel, want_dx=False)
    rf2 = oracle.pg_loss_fwd(*sub2, cfg.eps_low, cfg.eps_high)
    near = (np.abs(rf2["ratio"] - lo) < 2e-3 * lo) | (np.abs(rf2["ratio"] - hi) < 2e-3 * hi)
    assert not near.any(), "a live token sits on a clip bound; change the seed of the live set"
    hit = np.isin(vsel, tb.target[live])          # rows that carry a target term vs pure softmax rows
    assert hit.any() and (~hit).any()
    for loss_k, dw_k in ((loss2, dw2), (loss3, dw3)):
        assert abs(loss_k.item() - rf2["loss"]) <= 2e-3 * abs(rf2["loss"]) + 1e-7
        got2 = f64(dw_k[torch.as_tensor(vsel, device="cuda")])
        assert rel_l2(got2, rb2["d_W"]) < GRAD_TOL
        assert rel_l2(got2[~hit], rb2["d_W"][~hit]) < 2 * GRAD_TOL


@pytest.mark.timeout(600)
def test_small_model_shape_c2(spo, oracle):
    _run_full(spo, oracle, "C2", n_rows=256, n_dw_tokens=160, n_vsel=64)


@pytest.mark.timeout(900)
def test_qwen3_8b_head_shape_c3(spo, oracle):
    _run_full(spo, oracle, "C3", n_rows=1024, n_dw_tokens=256, n_vsel=64)


@pytest.mark.timeout(900)
def test_long_horizon_masked_shape_c4(spo, oracle):
    _run_full(spo, oracle, "C4", n_rows=256, n_dw_tokens=128, n_vsel=64)


def _short_window(cu, lo=1000, hi=1600):
    """Two or more consecutive responses [b0, b1) whose token total is the smallest one within [lo, hi]."""
    best = None
    B = len(cu) - 1
    for b0 in range(B):
        for b1 in range(b0 + 2, B + 1):
            n = int(cu[b1] - cu[b0])
            if n > hi:
                break
            if n >= lo and (best is None or n < best[0]):
                best = (n, b0, b1)
    assert best is not None
    return best[1], best[2]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("w_scale,chunk", [(1.0, 0), (8.0, 512)])
def test_dense_slice_at_full_head_size(spo, oracle, w_scale, chunk):
    # A contiguous slice of whole responses of the Qwen3-8B-shaped workload, nothing masked, at the
    # full H and V: small enough for the oracle to evaluate every token over the whole vocabulary,
    # so every quantity it needs (lse, ratios, gradient scales) is its own.
    cfg = wl.CONFIGS["C3"]
    tb = wl.token_batch(cfg, device="cuda", w_scale=w_scale)
    b0, b1 = _short_window(tb.cu_seqlens)
    t0, t1 = int(tb.cu_seqlens[b0]), int(tb.cu_seqlens[b1])
    n, H, V = t1 - t0, cfg.H, cfg.V
    say(f"dense slice of C3: responses {b0}..{b1 - 1}, {n} tokens, H={H} V={V} w_scale={w_scale} chunk={chunk}")
    hidden = tb.hidden[t0:t1].contiguous()
    h64, W64 = hidden.double().cpu().numpy(), tb.W.double().cpu().numpy()
    tg = tb.target[t0:t1]
    cu = (tb.cu_seqlens[b0:b1 + 1] - tb.cu_seqlens[b0]).astype(np.int32)
    rng = np.random.default_rng([wl.MASTER_SEED, 11])
    adv = np.where(np.arange(b1 - b0) % 2 == 0, 1.0, -1.0) * (1.0 + 0.25 * rng.random(b1 - b0))
    lo, hi = 1 - cfg.eps_low, 1 + cfg.eps_high
    logp0 = oracle.pg_loss_fwd(h64, W64, tg, np.zeros(n), None, adv, cu, cfg.eps_low, cfg.eps_high)["logp"]
    old = (logp0 + tb.noise[t0:t1]).astype(np.float32)
    for _ in range(4):      # keep ratios off the clip bounds: fp32 and fp64 must take the same branch
        r = np.exp(logp0 - old.astype(np.float64))
        near = (np.abs(r - lo) < 2e-3 * lo) | (np.abs(r - hi) < 2e-3 * hi)
        if not near.any():
            break
        old[near] += np.float32(0.01)
    args = (h64, W64, tg, old.astype(np.float64), None, adv, cu, cfg.eps_low, cfg.eps_high)
    ref = oracle.pg_loss_fwd(*args)
    dev = lambda x, dt: torch.as_tensor(x).to("cuda", dt).contiguous()
    desc = spo.make_desc(hidden, tb.W, dev(tg, torch.int32), dev(old, torch.float32), None,
                         dev(adv, torch.float32), dev(cu, torch.int32), cfg.eps_low, cfg.eps_high)
    # oracle references first; then both ways to the gradients are held against them
    vsel = np.unique(np.concatenate([rng.choice(V, 96, replace=False), tg[:12],
                                     [0, 255, 256, V - 1, (V // 256) * 256]])).astype(np.int64)
    rb = oracle.pg_loss_bwd(*args, vsel=vsel, want_dx=False)
    rows = np.unique(np.concatenate([rng.choice(n, 160, replace=False), [0, 255, 256, n - 1, int(cu[1]) - 1,
                                                                          int(cu[1])]])).astype(np.int64)
    rx = oracle.pg_loss_bwd(*args, rows=rows, want_dw=False)
    assert 0.5 * n < ref["active"].sum() < n                       # both branches of the min occur
    for path in ("fwd_then_bwd", "one_call"):
        say(f"dense slice of C3: {path}")
        if path == "one_call":
            loss, logp, lse, stats, dx, dw = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_hidden_dtype=torch.float32,
                                                                     chunk_tokens=chunk)
        else:
            loss, logp, lse, stats = spo.spo_pg_loss_fwd(desc)
            dx, dw = spo.spo_pg_loss_bwd(desc, logp, lse, 1.0, d_hidden_dtype=torch.float32, chunk_tokens=chunk)
        torch.cuda.synchronize()
        np.testing.assert_allclose(f64(lse), ref["lse"], atol=2e-4, rtol=0)
        np.testing.assert_allclose(f64(logp), ref["logp"], atol=2e-4, rtol=0)
        assert abs(loss.item() - ref["loss"]) <= 2e-3 * abs(ref["loss"]) + 1e-7
        assert abs(stats[1].item() - (1 - ref["active"].mean())) < 1e-6
        # dW: sampled vocabulary rows, all tokens of the slice
        got = f64(dw[torch.as_tensor(vsel, device="cuda")])
        assert rel_l2(got, rb["d_W"]) < GRAD_TOL
        hit = np.isin(vsel, tg[rb["g"] != 0])
        assert hit.any() and (~hit).any()
        assert rel_l2(got[~hit], rb["d_W"][~hit]) < 2 * GRAD_TOL        # rows no token sampled: softmax part alone
        scale = np.abs(rb["d_W"]).max()
        per_v = np.linalg.norm(got - rb["d_W"], axis=1)
        assert (per_v <= 3 * GRAD_TOL * np.linalg.norm(rb["d_W"], axis=1) + 1e-3 * scale).all()
        # dHidden: sampled tokens (first, last, tile edges and random ones), total and softmax part
        gx = f64(dx[torch.as_tensor(rows, device="cuda")])
        assert rel_l2(gx, rx["d_hidden"]) < GRAD_TOL
        onehot = rx["g"][:, None] * W64[tg[rows]]
        soft_ref, soft_gpu = rx["d_hidden"] - onehot, gx - onehot
        bound = GRAD_TOL * np.linalg.norm(soft_ref) + 1.1 * 2.0 ** -9 * np.linalg.norm(onehot)
        assert np.linalg.norm(soft_gpu - soft_ref) <= bound
        if w_scale > 1.0:   # peaked softmax: the softmax part is comparable to the target part
            assert np.linalg.norm(soft_ref) > 0.2 * np.linalg.norm(onehot)
            assert rel_l2(soft_gpu, soft_ref) < 2 * GRAD_TOL
        assert not dx[torch.as_tensor(np.flatnonzero(ref["active"] == 0), device="cuda")].any()
