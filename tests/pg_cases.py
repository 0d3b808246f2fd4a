"""Helpers of the GPU parity tests of the policy-gradient loss: build a seeded
case, run the oracle on it, keep tokens away from the clip boundary, compare."""
import sys

import numpy as np
import torch

from paper_2509_13232_amd import workloads as wl


def say(msg):
    print("[case]", msg, flush=True)
    sys.stdout.flush()


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def rel_l2(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


class Case:
    """Token-side inputs on the CPU (torch, in the workload dtype) plus numpy side arrays."""

    def __init__(self, cfg, lengths=None, seed=wl.MASTER_SEED, w_scale=1.0, mask_frac=None, adv=None):
        tb = wl.token_batch(cfg if mask_frac is None else wl.scaled(cfg, mask_frac=mask_frac),
                            "cpu", seed, lengths, w_scale)
        self.cfg = cfg
        self.hidden, self.W = tb.hidden, tb.W
        self.target, self.noise, self.mask, self.cu, self.T = tb.target, tb.noise, tb.mask, tb.cu_seqlens, tb.T
        B = self.cu.shape[0] - 1
        rng = np.random.default_rng([seed, 99])
        if adv is None:
            a = rng.standard_normal(B)
            a = (a - a.mean()) / a.std() if B > 1 else np.ones(B)
            adv = a
        self.adv = np.asarray(adv, np.float32)
        self.eps = (cfg.eps_low, cfg.eps_high)
        self.old = None

    def oracle_inputs(self):
        return (f64(self.hidden), f64(self.W), self.target, None if self.old is None else self.old.astype(np.float64),
                self.mask, self.adv.astype(np.float64), self.cu)

    def set_old_from_oracle(self, oracle, margin=2e-3):
        """old log-prob = current (oracle) + seeded noise, with tokens whose ratio falls
        within `margin` (relative) of a clip bound nudged away from it, so that the
        fp32 kernel and the fp64 oracle take the same branch of the min."""
        h, w, tg, _, mk, ad, cu = self.oracle_inputs()
        zero = np.zeros(self.T)
        logp = oracle.pg_loss_fwd(h, w, tg, zero, mk, ad, cu, *self.eps)["logp"]
        old = (logp + self.noise).astype(np.float32)
        for _ in range(4):
            ratio = np.exp(logp - old.astype(np.float64))
            lo, hi = 1.0 - self.eps[0], 1.0 + self.eps[1]
            near = (np.abs(ratio - lo) < margin * lo) | (np.abs(ratio - hi) < margin * hi)
            if not near.any():
                break
            old[near] += np.float32(0.01)
        self.old = old
        self.n_nudged = int(near.sum())
        return logp

    def to_gpu(self, binding, w_layout=0, logits=None):
        d = "cuda"
        W = self.W.to(d)
        if w_layout == 1:
            W = W.t().contiguous()
        t = lambda x, dt: None if x is None else torch.as_tensor(x).to(d, dt).contiguous()
        return binding.make_desc(
            None if logits is not None else self.hidden.to(d), None if logits is not None else W,
            t(self.target, torch.int32), t(self.old, torch.float32), t(self.mask, torch.uint8),
            t(self.adv, torch.float32), t(self.cu, torch.int32), self.eps[0], self.eps[1], w_layout,
            logits=logits)


def check_forward(case, oracle, out_gpu, ref=None, atol_logp=2e-4, rtol_loss=2e-3):
    loss, logp, lse, stats = out_gpu
    if ref is None:
        ref = oracle.pg_loss_fwd(*case.oracle_inputs(), *case.eps)
    np.testing.assert_allclose(f64(lse), ref["lse"], atol=atol_logp, rtol=0)
    np.testing.assert_allclose(f64(logp), ref["logp"], atol=atol_logp, rtol=0)
    gl = float(loss.item())
    assert abs(gl - ref["loss"]) <= rtol_loss * abs(ref["loss"]) + 1e-7, (gl, ref["loss"])
    if stats is not None:
        st = f64(stats)
        m = np.ones(case.T, bool) if case.mask is None else case.mask.astype(bool)
        assert st[0] == ref["M"]
        if ref["M"] > 0:
            assert abs(st[1] - (1 - ref["active"][m].mean())) < 1e-6
            assert abs(st[2] - ref["ratio"][m].mean()) < 1e-4 * max(1.0, ref["ratio"][m].mean())
    return ref
