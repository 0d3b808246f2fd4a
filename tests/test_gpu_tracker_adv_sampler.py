"""GPU parity of the tracker update, the advantages and the prioritized sampler
against the fp64 oracle, through the C ABI.  Indices and counts bit-exact,
fp32 values within 1e-5 relative."""
import sys

import numpy as np
import pytest
import torch

from paper_2509_13232_amd import workloads as wl

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def say(msg):
    print("[case]", msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def spo():
    from paper_2509_13232_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def dev(x, dtype=None):
    t = torch.as_tensor(np.asarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


def _update_case(cfg, n, seed, unique=True):
    a, b = wl.tracker_state(cfg, seed)
    if unique:
        idx = wl.distinct_indices(cfg, n, seed)
    else:
        idx = np.random.default_rng(seed).integers(0, min(cfg.N, max(2, n // 4)), n).astype(np.int32)
    r = wl.rewards(cfg, idx, seed)
    kl = wl.kl_divergences(cfg, n, seed)
    return a, b, idx, r, kl


@pytest.mark.parametrize("name,n", [("C1", 8), ("C2", 64), ("C5", 4096)])
def test_tracker_update_matches_oracle(spo, oracle, name, n):
    cfg = wl.CONFIGS[name]
    say(f"tracker_update {name} n={n}")
    a, b, idx, r, kl = _update_case(cfg, n, 11)
    ea, eb, ev, _ = oracle.tracker_update(a, b, idx, r, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
    ga, gb = dev(a), dev(b)
    nobs = torch.zeros(cfg.N, dtype=torch.int32, device="cuda")
    gv = spo.spo_tracker_update(ga, gb, dev(idx), dev(r), dev(kl), cfg.d_half, cfg.rho_min, cfg.rho_max,
                                ids_unique=True, n_obs=nobs, want_v_prev=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(ga.cpu().numpy(), ea, rtol=RTOL)
    np.testing.assert_allclose(gb.cpu().numpy(), eb, rtol=RTOL)
    np.testing.assert_allclose(gv.cpu().numpy(), ev, rtol=RTOL)
    # untouched entries keep their bits, visit counters are exact
    untouched = np.ones(cfg.N, bool)
    untouched[idx] = False
    assert np.array_equal(ga.cpu().numpy()[untouched], a[untouched])
    assert np.array_equal(nobs.cpu().numpy(), np.bincount(idx, minlength=cfg.N))


def test_tracker_counts_are_exact_without_discount(spo, oracle):
    # discount 1: Beta posterior counts, bit for bit, over several iterations
    cfg = wl.CONFIGS["C2"]
    say("tracker_update discount=1 counts")
    a = np.full(cfg.N, 0.5, np.float32)
    b = np.full(cfg.N, 0.5, np.float32)
    ga, gb = dev(a), dev(b)
    ea, eb = a.astype(np.float64), b.astype(np.float64)
    for it in range(6):
        idx = wl.distinct_indices(cfg, 64, 100 + it)
        r = wl.rewards(cfg, idx, 100 + it)
        kl = wl.kl_divergences(cfg, 64, 100 + it)
        ea, eb, _, _ = oracle.tracker_update(ea, eb, idx, r, kl, cfg.d_half, 1.0, 1.0)
        spo.spo_tracker_update(ga, gb, dev(idx), dev(r), dev(kl), cfg.d_half, 1.0, 1.0)
    torch.cuda.synchronize()
    assert np.array_equal(ga.cpu().numpy().astype(np.float64), ea)
    assert np.array_equal(gb.cpu().numpy().astype(np.float64), eb)


def test_tracker_update_with_repeated_ids_is_sequential(spo, oracle):
    cfg = wl.CONFIGS["C2"]
    say("tracker_update repeated ids")
    a, b, idx, r, kl = _update_case(cfg, 300, 5, unique=False)
    assert len(set(idx.tolist())) < 300
    ea, eb, ev, _ = oracle.tracker_update(a, b, idx, r, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
    ga, gb = dev(a), dev(b)
    nobs = torch.zeros(cfg.N, dtype=torch.int32, device="cuda")
    gv = spo.spo_tracker_update(ga, gb, dev(idx), dev(r), dev(kl), cfg.d_half, cfg.rho_min, cfg.rho_max,
                                ids_unique=False, n_obs=nobs, want_v_prev=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(ga.cpu().numpy(), ea, rtol=RTOL)
    np.testing.assert_allclose(gb.cpu().numpy(), eb, rtol=RTOL)
    np.testing.assert_allclose(gv.cpu().numpy(), ev, rtol=RTOL)
    assert np.array_equal(nobs.cpu().numpy(), np.bincount(idx, minlength=cfg.N))


@pytest.mark.parametrize("B,G,N", [(16384, 8, 1 << 20), (40000, 3, 20000), (512, 512, 64)])
def test_tracker_update_of_batches_that_repeat_every_prompt(spo, oracle, B, G, N):
    # batch extensions that sample every prompt G times (Appendix "Batch Extensions"): B observations,
    # each id G times in shuffled order; also a batch beyond one window of the kernel (40000) and one
    # id repeated 512 times (as many rounds as observations).  Values 1e-5, visit counters exact, and
    # the slot table the kernel borrows is handed back clean (a second call gives the same answer).
    say(f"tracker_update B={B}, every id {G} times, N={N}")
    rng = np.random.default_rng([B, G])
    B = B // G * G
    ids = rng.choice(N, B // G, replace=False).astype(np.int32)
    idx = rng.permutation(np.repeat(ids, G)).astype(np.int32)
    a = rng.uniform(0.5, 50, N).astype(np.float32)
    b = rng.uniform(0.5, 50, N).astype(np.float32)
    r = (rng.random(B) < 0.4).astype(np.float32)
    kl = rng.exponential(0.02, B).astype(np.float32)
    ea, eb, ev, _ = oracle.tracker_update(a, b, idx, r, kl, 0.25, 0.875, 0.96)
    ws = torch.empty(spo.lib().spo_tracker_update_workspace_bytes(N), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        ga, gb = dev(a), dev(b)
        nobs = torch.zeros(N, dtype=torch.int32, device="cuda")
        info = torch.full((1,), 7, dtype=torch.int32, device="cuda")
        gv = spo.spo_tracker_update(ga, gb, dev(idx), dev(r), dev(kl), 0.25, 0.875, 0.96, ids_unique=False,
                                    n_obs=nobs, want_v_prev=True, info=info, workspace=ws)
        torch.cuda.synchronize()
        np.testing.assert_allclose(ga.cpu().numpy(), ea, rtol=RTOL)
        np.testing.assert_allclose(gb.cpu().numpy(), eb, rtol=RTOL)
        np.testing.assert_allclose(gv.cpu().numpy(), ev, rtol=RTOL)
        assert np.array_equal(nobs.cpu().numpy(), np.bincount(idx, minlength=N))
        assert info.item() == 0


def test_ids_out_of_range_or_repeated_are_flagged_not_followed(spo, oracle):
    say("tracker_update / advantages: ids outside the table, repeats under ids_unique")
    N, B = 1000, 64
    rng = np.random.default_rng(3)
    a = rng.uniform(0.5, 50, N).astype(np.float32)
    b = rng.uniform(0.5, 50, N).astype(np.float32)
    idx = rng.choice(N, B, replace=False).astype(np.int32)
    r = (rng.random(B) < 0.5).astype(np.float32)
    kl = rng.uniform(0, 0.05, B).astype(np.float32)
    bad = idx.copy()
    bad[[3, 40]] = [N, -1]
    good = np.ones(B, bool)
    good[[3, 40]] = False
    ea, eb, ev, _ = oracle.tracker_update(a, b, idx[good], r[good], kl[good], 0.25, 0.875, 0.96)
    for unique in (True, False):
        ga, gb = dev(a), dev(b)
        info = torch.zeros(1, dtype=torch.int32, device="cuda")
        gv = spo.spo_tracker_update(ga, gb, dev(bad), dev(r), dev(kl), 0.25, 0.875, 0.96, ids_unique=unique,
                                    want_v_prev=True, info=info)
        torch.cuda.synchronize()
        assert info.item() == 1                                            # out of range, nothing else
        np.testing.assert_allclose(ga.cpu().numpy(), ea, rtol=RTOL)       # the other observations are applied
        np.testing.assert_allclose(gb.cpu().numpy(), eb, rtol=RTOL)
        v = gv.cpu().numpy()
        assert np.isnan(v[~good]).all()
        np.testing.assert_allclose(v[good], ev, rtol=RTOL)
    # advantages: the flag, NaN for the response, no read outside the table
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    raw, nrm, _ = spo.spo_advantages(dev(a), dev(b), dev(bad), dev(r), info=info)
    torch.cuda.synchronize()
    assert info.item() == 1 and np.isnan(raw.cpu().numpy()[~good]).all() and np.isfinite(raw.cpu().numpy()[good]).all()
    assert torch.isnan(nrm).all()                                          # the batch statistics are NaN: nothing is normalised
    raw, nrm, _ = spo.spo_advantages(dev(a), dev(b), dev(idx), dev(r), info=info)
    torch.cuda.synchronize()
    assert info.item() == 0 and np.isfinite(nrm.cpu().numpy()).all()
    # a repeated id under ids_unique = 1 is found when the table is there to look
    rep = idx.copy()
    rep[10] = rep[50]
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    spo.spo_tracker_update(dev(a), dev(b), dev(rep), dev(r), dev(kl), 0.25, 0.875, 0.96, info=info, check_repeats=True)
    torch.cuda.synchronize()
    assert info.item() == 2
    spo.spo_tracker_update(dev(a), dev(b), dev(idx), dev(r), dev(kl), 0.25, 0.875, 0.96, info=info, check_repeats=True)
    torch.cuda.synchronize()
    assert info.item() == 0


def test_tracker_init(spo, oracle):
    say("tracker_init")
    v0 = (np.random.default_rng(0).integers(0, 9, 1000) / 8.0).astype(np.float32)
    ea, eb = oracle.tracker_init(v0, 0.875)
    ga, gb = spo.spo_tracker_init(dev(v0), 0.875)
    torch.cuda.synchronize()
    assert np.array_equal(ga.cpu().numpy().astype(np.float64), ea)
    assert np.array_equal(gb.cpu().numpy().astype(np.float64), eb)


@pytest.mark.parametrize("name,n", [("C1", 8), ("C2", 64), ("C3", 128), ("C5", 4096)])
@pytest.mark.parametrize("ddof,eps_norm,baseline", [(0, 0.0, True), (1, 1e-6, True), (0, 0.0, False)])
def test_advantages_match_oracle(spo, oracle, name, n, ddof, eps_norm, baseline):
    cfg = wl.CONFIGS[name]
    say(f"advantages {name} n={n} ddof={ddof} eps={eps_norm} baseline={baseline}")
    a, b, idx, r, _ = _update_case(cfg, n, 21)
    eraw, enrm, (mu, sigma) = oracle.advantages(a, b, idx, r, ddof, float(np.float32(eps_norm)), baseline)
    raw, nrm, st = spo.spo_advantages(dev(a), dev(b), dev(idx), dev(r), ddof, eps_norm, baseline)
    torch.cuda.synchronize()
    np.testing.assert_allclose(raw.cpu().numpy(), eraw, rtol=RTOL, atol=1e-7)
    np.testing.assert_allclose(nrm.cpu().numpy(), enrm, rtol=RTOL, atol=1e-6)
    np.testing.assert_allclose(st.cpu().numpy(), [mu, sigma], rtol=RTOL, atol=1e-7)
    # run-to-run bitwise reproducible
    _, nrm2, _ = spo.spo_advantages(dev(a), dev(b), dev(idx), dev(r), ddof, eps_norm, baseline)
    assert torch.equal(nrm, nrm2)


@pytest.mark.parametrize("B", [16384, 100003, 1 << 20])
@pytest.mark.parametrize("ddof,eps_norm,baseline", [(0, 0.0, True), (1, 1e-6, False)])
def test_advantages_of_large_batches_over_many_workgroups(spo, oracle, B, ddof, eps_norm, baseline):
    # with a workspace, batches of 16384 responses or more are spread over the chip: partial sums of
    # 4096 responses, added in a fixed order (a ragged last part at B = 100003); ids repeat
    cfg = wl.CONFIGS["C5"]
    say(f"advantages, wide path, B={B} ddof={ddof} baseline={baseline}")
    a, b = wl.tracker_state(cfg, 5)
    rng = np.random.default_rng([wl.MASTER_SEED, B])
    idx = rng.integers(0, cfg.N, B).astype(np.int32)
    r = (rng.random(B) < 0.4).astype(np.float32)
    eraw, enrm, (mu, sigma) = oracle.advantages(a, b, idx, r, ddof, float(np.float32(eps_norm)), baseline)
    ws = torch.empty(spo.lib().spo_advantages_workspace_bytes(B), dtype=torch.uint8, device="cuda")
    ga, gb, gi, gr = dev(a), dev(b), dev(idx), dev(r)
    info = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    raw, nrm, st = spo.spo_advantages(ga, gb, gi, gr, ddof, eps_norm, baseline, info=info, workspace=ws)
    torch.cuda.synchronize()
    assert info.item() == 0
    np.testing.assert_allclose(raw.cpu().numpy(), eraw, rtol=RTOL, atol=1e-7)
    np.testing.assert_allclose(nrm.cpu().numpy(), enrm, rtol=RTOL, atol=1e-6)
    np.testing.assert_allclose(st.cpu().numpy(), [mu, sigma], rtol=RTOL, atol=1e-7)
    _, nrm2, st2 = spo.spo_advantages(ga, gb, gi, gr, ddof, eps_norm, baseline, workspace=ws)
    assert torch.equal(nrm, nrm2) and torch.equal(st, st2)                  # bitwise reproducible
    _, nrm1, st1 = spo.spo_advantages(ga, gb, gi, gr, ddof, eps_norm, baseline)   # one workgroup: same to fp64 rounding
    torch.cuda.synchronize()
    np.testing.assert_allclose(nrm1.cpu().numpy(), nrm.cpu().numpy(), rtol=1e-6, atol=1e-7)
    if baseline:    # an id out of range is flagged, not followed, here too
        bad = idx.copy()
        bad[B // 2] = cfg.N
        info.zero_()
        raw, nrm, _ = spo.spo_advantages(ga, gb, dev(bad), gr, ddof, eps_norm, baseline, info=info, workspace=ws)
        torch.cuda.synchronize()
        assert info.item() == 1 and torch.isnan(raw[B // 2]) and torch.isnan(nrm).all()


def test_advantages_degenerate_batch(spo):
    say("advantages all-equal")
    a = dev(np.ones(4, np.float32))
    raw, nrm, st = spo.spo_advantages(a, a, dev(np.arange(4, dtype=np.int32)), dev(np.ones(4, np.float32)))
    torch.cuda.synchronize()
    assert nrm.cpu().tolist() == [0.0] * 4 and st.cpu().tolist() == [0.5, 0.0]


@pytest.mark.parametrize("name,B,seed,replace", [
    ("C1", 8, 0, False), ("C1", 16, 3, False), ("C1", 8, 0, True),
    ("C2", 64, 1, False), ("C3", 128, 2, False),
    ("C5", 4096, 7, False), ("C5", 4096, 7, True), ("C5", 16384, 9, False)])
def test_sampler_indices_are_bit_exact(spo, oracle, name, B, seed, replace):
    cfg = wl.CONFIGS[name]
    say(f"sample_prompts {name} B={B} seed={seed} replace={replace}")
    a, b = wl.tracker_state(cfg, 31)
    for it in (0, 5):
        eidx, eatt = oracle.sample_prompts(a, b, B, cfg.eps_explore, seed, it, replace, return_attempts=True)
        gidx, info = spo.spo_sample_prompts(dev(a), dev(b), B, cfg.eps_explore, seed, it, replace,
                                            return_info=True)
        torch.cuda.synchronize()
        assert np.array_equal(gidx.cpu().numpy(), eidx)
        assert info.cpu().tolist() == [0, int(eatt.max())]
        if not replace:
            assert len(set(eidx.tolist())) == B


def test_sampler_reports_exhausted_attempts(spo, oracle):
    # one prompt holds nearly all the weight: later slots cannot find a free id in 2 attempts
    say("sample_prompts exhausted attempts")
    a = np.full(64, 1e-12, np.float32)
    b = np.full(64, 1.0, np.float32)
    a[3] = 1.0
    with pytest.raises(RuntimeError):
        oracle.sample_prompts(a, b, 8, 0.0, 0, 0, False, max_attempts=2)
    first = oracle.sample_prompts(a, b, 1, 0.0, 0, 0, False)
    gidx, info = spo.spo_sample_prompts(dev(a), dev(b), 8, 0.0, 0, 0, False, max_attempts=2, return_info=True)
    torch.cuda.synchronize()
    out = gidx.cpu().numpy()
    assert info.cpu().numpy()[0] == 1 and (out == -1).any() and out[0] == first[0]
    alive = out[out >= 0]
    assert len(set(alive.tolist())) == len(alive)


@pytest.mark.parametrize("replace", [True, False])
def test_sampler_with_all_weights_zero(spo, oracle, replace):
    # no exploration bonus and every estimate at 0 or 1: every weight is zero
    say(f"sample_prompts total weight zero, replace={replace}")
    a = np.array([0.0, 3.0, 0.0, 1.0], np.float32)
    b = np.array([2.0, 0.0, 5.0, 0.0], np.float32)
    with pytest.raises(RuntimeError):
        oracle.sample_prompts(a, b, 3, 0.0, 1, 2, replace)
    gidx, info = spo.spo_sample_prompts(dev(a), dev(b), 3, 0.0, 1, 2, replace, return_info=True)
    torch.cuda.synchronize()
    assert (gidx.cpu().numpy() == -1).all() and info.cpu().numpy()[0] == 1


def test_sampler_after_update_sees_new_state(spo, oracle):
    # the order of the training loop: sample -> advantages (pre-update) -> update
    cfg = wl.CONFIGS["C2"]
    say("loop order C2")
    a, b = wl.tracker_state(cfg, 41)
    ga, gb = dev(a), dev(b)
    idx = spo.spo_sample_prompts(ga, gb, 64, cfg.eps_explore, 0, 0)
    eidx = oracle.sample_prompts(a, b, 64, cfg.eps_explore, 0, 0)
    r = wl.rewards(cfg, eidx, 41)
    kl = wl.kl_divergences(cfg, 64, 41)
    raw, nrm, _ = spo.spo_advantages(ga, gb, idx, dev(r))
    spo.spo_tracker_update(ga, gb, idx, dev(r), dev(kl), cfg.d_half, cfg.rho_min, cfg.rho_max)
    raw_after, _, _ = spo.spo_advantages(ga, gb, idx, dev(r))
    torch.cuda.synchronize()
    eraw, enrm, _ = oracle.advantages(a, b, eidx, r)
    assert np.array_equal(idx.cpu().numpy(), eidx)
    np.testing.assert_allclose(raw.cpu().numpy(), eraw, rtol=RTOL, atol=1e-7)
    np.testing.assert_allclose(nrm.cpu().numpy(), enrm, rtol=RTOL, atol=1e-6)
    assert (raw_after.abs() < raw.abs()).all()
    ea, eb, _, _ = oracle.tracker_update(a, b, eidx, r, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
    idx2 = spo.spo_sample_prompts(ga, gb, 64, cfg.eps_explore, 0, 1)
    torch.cuda.synchronize()
    # the oracle's fp64 state rounded to fp32 is what the next draw must see
    assert np.array_equal(idx2.cpu().numpy(),
                          oracle.sample_prompts(ga.cpu().numpy(), gb.cpu().numpy(), 64, cfg.eps_explore, 0, 1))
    np.testing.assert_allclose(ga.cpu().numpy(), ea, rtol=RTOL)


def test_advantage_diagnostics_match_oracle(spo, oracle):
    cfg = wl.CONFIGS["C5"]
    say("advantage_diagnostics C5 n=4096")
    a, b, idx, r, _ = _update_case(cfg, 4096, 51)
    raw, _, _ = spo.spo_advantages(dev(a), dev(b), dev(idx), dev(r))
    diag = spo.spo_advantage_diagnostics(raw, dev(r), 1e-4, 0.02)
    torch.cuda.synchronize()
    rawc = raw.cpu().numpy()
    want = oracle.advantage_diagnostics(rawc, r, float(np.float32(1e-4)), float(np.float32(0.02)))
    got = diag.cpu().numpy()
    assert got[0] == np.float32(want[0]) and got[1] == np.float32(want[1])     # counts are exact
    np.testing.assert_allclose(got[2:], want[2:], rtol=RTOL)


def test_tracker_update_with_general_rewards(spo, oracle):
    cfg = wl.CONFIGS["C2"]
    say("tracker_update non-binary rewards")
    a, b, idx, _, kl = _update_case(cfg, 64, 61)
    r = np.random.default_rng(61).uniform(0, 1, 64).astype(np.float32)
    ea, eb, ev, _ = oracle.tracker_update(a, b, idx, r, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
    ga, gb = dev(a), dev(b)
    gv = spo.spo_tracker_update(ga, gb, dev(idx), dev(r), dev(kl), cfg.d_half, cfg.rho_min, cfg.rho_max,
                                want_v_prev=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(ga.cpu().numpy(), ea, rtol=RTOL)
    np.testing.assert_allclose(gb.cpu().numpy(), eb, rtol=RTOL)
    np.testing.assert_allclose(gv.cpu().numpy(), ev, rtol=RTOL)


@pytest.mark.parametrize("unique", [True, False])
def test_tracker_update_ema_matches_oracle(spo, oracle, unique):
    # moving-average form of the tracker, rewards outside [0, 1]
    cfg = wl.CONFIGS["C5"]
    say(f"tracker_update_ema unique={unique}")
    rng = np.random.default_rng(71)
    N, B = 4096, 1500
    v = rng.uniform(-1, 3, N).astype(np.float32)
    n = rng.uniform(1, 25, N).astype(np.float32)
    idx = (rng.permutation(N)[:B] if unique else rng.integers(0, 64, B)).astype(np.int32)
    r = rng.normal(1.0, 2.0, B).astype(np.float32)
    kl = rng.exponential(0.02, B).astype(np.float32)
    ev, en, evp = oracle.tracker_update_ema(v, n, idx, r, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
    gv, gn = dev(v), dev(n)
    cnt = torch.zeros(N, dtype=torch.int32, device="cuda")
    gvp = spo.spo_tracker_update_ema(gv, gn, dev(idx), dev(r), dev(kl), cfg.d_half, cfg.rho_min, cfg.rho_max,
                                     ids_unique=unique, n_obs=cnt, want_v_prev=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(gv.cpu().numpy(), ev, rtol=RTOL, atol=1e-6)
    np.testing.assert_allclose(gn.cpu().numpy(), en, rtol=RTOL)
    np.testing.assert_allclose(gvp.cpu().numpy(), evp, rtol=RTOL, atol=1e-6)
    assert np.array_equal(cnt.cpu().numpy(), np.bincount(idx, minlength=N))


def test_advantages_from_the_estimate_itself(spo, oracle):
    say("advantages with beta=None")
    rng = np.random.default_rng(72)
    N, B = 512, 200
    v = rng.uniform(-1, 3, N).astype(np.float32)
    idx = rng.permutation(N)[:B].astype(np.int32)
    r = rng.normal(1.0, 2.0, B).astype(np.float32)
    eraw, enrm, est = oracle.advantages(v, None, idx, r)
    raw, nrm, st = spo.spo_advantages(dev(v), None, dev(idx), dev(r))
    torch.cuda.synchronize()
    np.testing.assert_allclose(raw.cpu().numpy(), eraw, rtol=RTOL, atol=1e-6)
    np.testing.assert_allclose(nrm.cpu().numpy(), enrm, rtol=RTOL, atol=1e-6)
    np.testing.assert_allclose(st.cpu().numpy(), est, rtol=RTOL)
