"""The whole step (sampling -> advantages -> tracker update -> loss and gradients in one call) is a
fixed sequence of launches on the caller's stream that allocates nothing and never waits for the
device, so a caller can capture it into a HIP graph once and replay it.  Replays are held against
the same steps run eagerly, bit for bit, with the program's own eager work and synchronisations
between the replays."""
import numpy as np
import pytest
import torch

from paper_2509_13232_amd import workloads as wl
from pg_cases import Case, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spo():
    from paper_2509_13232_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


@pytest.mark.parametrize("mask_frac", [None, 0.25], ids=["no_mask", "masked"])
def test_step_replays_from_a_captured_graph(spo, mask_frac):
    # both forms of the one call: without a mask the sweep stores scaled probabilities, with one logits
    cfg = wl.scaled(wl.CONFIGS["C2"], name="graph", H=256, V=3000)
    lengths = [37, 300, 1, 255, 120, 64, 200, 90]
    case = Case(cfg, lengths, mask_frac=mask_frac)
    B, d = len(lengths), "cuda"
    say(f"graph capture of the step: T={case.T} H=256 V=3000 B={B} N={cfg.N}")
    a0, b0 = wl.tracker_state(cfg)
    rng = np.random.default_rng([wl.MASTER_SEED, 31])
    alpha, beta = torch.as_tensor(a0).to(d), torch.as_tensor(b0).to(d)
    reward = torch.as_tensor((rng.random(B) < 0.5).astype(np.float32)).to(d)
    kl = torch.as_tensor(rng.uniform(0, 0.05, B).astype(np.float32)).to(d)
    hidden, W = case.hidden.to(d), case.W.to(d)
    target = torch.as_tensor(case.target).to(d)
    old = torch.as_tensor((-np.log(cfg.V) + case.noise).astype(np.float32)).to(d)
    mask = None if case.mask is None else torch.as_tensor(case.mask).to(d)
    cu = torch.as_tensor(case.cu).to(d)
    adv_holder = torch.zeros(B, dtype=torch.float32, device=d)
    desc = spo.make_desc(hidden, W, target, old, mask, adv_holder, cu, cfg.eps_low, cfg.eps_high)
    ws_s = torch.empty(spo.lib().spo_sample_prompts_workspace_bytes(cfg.N, B), dtype=torch.uint8, device=d)
    ws_t = torch.empty(spo.lib().spo_tracker_update_workspace_bytes(cfg.N), dtype=torch.uint8, device=d)
    ws_l = torch.empty(spo.spo_pg_loss_fwd_bwd_workspace_bytes(desc, 256), dtype=torch.uint8, device=d)
    d_W = torch.zeros((cfg.V, cfg.H), dtype=torch.float32, device=d)

    def step():
        idx = spo.spo_sample_prompts(alpha, beta, B, cfg.eps_explore, cfg.sample_seed, 3, workspace=ws_s)
        _, adv, _ = spo.spo_advantages(alpha, beta, idx, reward)
        spo.spo_tracker_update(alpha, beta, idx, reward, kl, cfg.d_half, cfg.rho_min, cfg.rho_max, ids_unique=False,
                               workspace=ws_t)
        adv_holder.copy_(adv)
        loss, logp, _, _, dx, _ = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_W=d_W, accumulate_dW=True, chunk_tokens=256,
                                                           workspace=ws_l)
        return idx, loss, logp, dx

    def snapshot(out):
        return [t.clone() for t in out] + [alpha.clone(), beta.clone(), d_W.clone()]

    # the steps run eagerly: the tracker moves on and d_W accumulates from step to step
    eager = []
    for _ in range(3):
        eager.append(snapshot(step()))
    torch.cuda.synchronize()
    assert not torch.equal(eager[0][4], eager[1][4]) and not torch.equal(eager[0][6], eager[1][6])

    def reset():
        alpha.copy_(torch.as_tensor(a0))
        beta.copy_(torch.as_tensor(b0))
        d_W.zero_()

    reset()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the side stream, as capture wants it
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = step()
    reset()
    torch.cuda.synchronize()
    scratch = torch.randn(1 << 20, device=d)
    for k in range(3):
        graph.replay()
        got = snapshot(out)
        torch.cuda.synchronize()
        scratch = (scratch * 1.0001).sin()       # eager work and a synchronisation between the replays
        torch.cuda.synchronize()
        for name, g, e in zip(("idx", "loss", "logp", "d_hidden", "alpha", "beta", "d_W"), got, eager[k]):
            assert torch.equal(g, e), f"replay {k}: {name} differs from the eager step"
