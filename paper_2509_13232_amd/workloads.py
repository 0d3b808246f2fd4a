"""Seeded synthetic workloads for the SPO hot path.

This module only DRAWS inputs: shapes, value distributions, length mixes and
mask structure of the five benchmark configurations.  It holds none of the
method's arithmetic (no tracker update, advantage, sampling weight, softmax or
surrogate) and is the one module that both the GPU tests and the CPU oracle
tests feed from.  Every tensor comes from its own generator seeded by
(master seed, stream number), so any tensor can be regenerated alone.

The synthetic tensors stand in for the paper's training data and model: they
take Qwen3-8B's LM-head shape (H=4096, V=151936) and the paper's response
length regime (Appendix "Training and Evaluation Details": at most 16384
tokens in training, 32768 in evaluation), nothing else.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass
class Config:
    name: str
    N: int                  # tracked prompts
    B: int                  # responses in the batch
    H: int
    V: int
    dtype: str              # "fp32" | "bf16" | "" (no token part)
    lengths: str            # "fixed:<n>" | "uniform:<lo>:<hi>" | "loguniform:<lo>:<hi>" | ""
    w_std: float = 0.02
    noise_std: float = 0.1  # std of (old log-prob - current log-prob)
    eps_low: float = 0.2
    eps_high: float = 0.28  # Clip-Higher values of the paper's runs
    reward: str = "bernoulli:0.4"   # "bernoulli:<p>" | "per_prompt"
    kl: str = "uniform:0.05"        # "uniform:<hi>" | "exp:<mean>"
    tracker: str = "const:0.5"      # "const:<a>" | "uniform:<lo>:<hi>" | "beta11"
    mask_frac: float = 0.0          # share of tokens zeroed in tool-output spans
    mask_span: tuple = (32, 512)
    sample_seed: int = 0
    d_half: float = 0.25            # the paper names D_half but gives no value
    rho_min: float = 0.875
    rho_max: float = 0.96
    eps_explore: float = 0.05
    extra: dict = field(default_factory=dict)


CONFIGS = {
    # tiny SPO step, fp32
    "C1": Config("C1", N=16, B=8, H=128, V=1000, dtype="fp32", lengths="fixed:64",
                 noise_std=0.05, eps_low=0.2, eps_high=0.2, reward="bernoulli:0.4",
                 kl="uniform:0.1", tracker="const:0.5", sample_seed=0),
    # small-model shape
    "C2": Config("C2", N=512, B=64, H=1024, V=151936, dtype="bf16", lengths="fixed:128",
                 noise_std=0.1, reward="per_prompt", kl="uniform:0.05", tracker="beta11"),
    # Qwen3-8B head shape, variable-length packed
    "C3": Config("C3", N=4096, B=128, H=4096, V=151936, dtype="bf16",
                 lengths="uniform:256:4096", noise_std=0.1, reward="per_prompt",
                 kl="uniform:0.05", tracker="beta11"),
    # long-horizon tool-integrated shape with masked tool-output spans
    "C4": Config("C4", N=4096, B=32, H=4096, V=151936, dtype="bf16",
                 lengths="loguniform:16384:32768", noise_std=0.2, reward="bernoulli:0.3",
                 kl="uniform:0.05", tracker="beta11", mask_frac=0.2),
    # tracker / advantage / sampling at scale, no tokens
    "C5": Config("C5", N=1 << 20, B=4096, H=0, V=0, dtype="", lengths="",
                 reward="per_prompt", kl="exp:0.02", tracker="uniform:0.5:50",
                 sample_seed=7),
}

MASTER_SEED = 20250913


def _rng(stream: int, seed: int = MASTER_SEED) -> np.random.Generator:
    return np.random.default_rng([seed, stream])


def _tgen(stream: int, device, seed: int = MASTER_SEED) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + stream) & 0x7FFFFFFFFFFFFFFF)
    return g


# ----------------------------------------------------------------- tracker side
def tracker_state(cfg: Config, seed: int = MASTER_SEED):
    """alpha[N], beta[N] as float32 numpy arrays."""
    r = _rng(1, seed)
    kind = cfg.tracker.split(":")
    if kind[0] == "const":
        a = np.full(cfg.N, float(kind[1]), np.float32)
        b = np.full(cfg.N, float(kind[1]), np.float32)
    elif kind[0] == "uniform":
        lo, hi = float(kind[1]), float(kind[2])
        a = r.uniform(lo, hi, cfg.N).astype(np.float32)
        b = r.uniform(lo, hi, cfg.N).astype(np.float32)
    elif kind[0] == "beta11":
        # eight pseudo-observations of a prompt whose success rate is Beta(1,1)
        p = r.beta(1.0, 1.0, cfg.N)
        a = (8.0 * p).astype(np.float32) + np.float32(0.5)
        b = (8.0 * (1.0 - p)).astype(np.float32) + np.float32(0.5)
    else:
        raise ValueError(cfg.tracker)
    return a, b


def prompt_success_rate(cfg: Config, seed: int = MASTER_SEED):
    """Hidden per-prompt success probability p_prompt ~ Beta(1,1)."""
    return _rng(2, seed).beta(1.0, 1.0, cfg.N)


def rewards(cfg: Config, idx: np.ndarray, seed: int = MASTER_SEED) -> np.ndarray:
    r = _rng(3, seed)
    u = r.random(idx.shape[0])
    if cfg.reward.startswith("bernoulli:"):
        p = np.full(idx.shape[0], float(cfg.reward.split(":")[1]))
    else:
        p = prompt_success_rate(cfg, seed)[idx]
    return (u < p).astype(np.float32)


def kl_divergences(cfg: Config, n: int, seed: int = MASTER_SEED) -> np.ndarray:
    r = _rng(4, seed)
    kind, val = cfg.kl.split(":")
    if kind == "uniform":
        return r.uniform(0.0, float(val), n).astype(np.float32)
    if kind == "exp":
        return r.exponential(float(val), n).astype(np.float32)
    raise ValueError(cfg.kl)


def distinct_indices(cfg: Config, n: int, seed: int = MASTER_SEED) -> np.ndarray:
    """n distinct prompt ids drawn uniformly (an update batch that does not
    depend on any sampler)."""
    return _rng(5, seed).choice(cfg.N, size=n, replace=False).astype(np.int32)


# ------------------------------------------------------------------- token side
def response_lengths(cfg: Config, seed: int = MASTER_SEED, B: int | None = None) -> np.ndarray:
    B = cfg.B if B is None else B
    r = _rng(6, seed)
    kind = cfg.lengths.split(":")
    if kind[0] == "fixed":
        return np.full(B, int(kind[1]), np.int64)
    lo, hi = int(kind[1]), int(kind[2])
    if kind[0] == "uniform":
        return r.integers(lo, hi + 1, B).astype(np.int64)
    if kind[0] == "loguniform":
        return np.floor(np.exp(r.uniform(math.log(lo), math.log(hi), B))).astype(np.int64)
    raise ValueError(cfg.lengths)


def cu_seqlens(lengths: np.ndarray) -> np.ndarray:
    cu = np.zeros(lengths.shape[0] + 1, np.int32)
    cu[1:] = np.cumsum(lengths)
    return cu


def loss_mask(cfg: Config, T: int, seed: int = MASTER_SEED):
    """None (all ones) or uint8[T] with tool-output spans of random length zeroed
    until the configured share of tokens is masked."""
    if cfg.mask_frac <= 0.0:
        return None
    r = _rng(7, seed)
    m = np.ones(T, np.uint8)
    want = int(cfg.mask_frac * T)
    lo, hi = cfg.mask_span
    while T - int(m.sum()) < want:
        n = int(r.integers(lo, hi + 1))
        s = int(r.integers(0, max(1, T - n)))
        m[s:s + n] = 0
    return m


def _torch_dtype(name: str):
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def hidden_states(T: int, H: int, dtype: str, device="cpu", seed: int = MASTER_SEED,
                  chunk: int = 1 << 15) -> torch.Tensor:
    """[T, H] ~ N(0, 1), drawn in fp32 and rounded to dtype."""
    g = _tgen(10, device, seed)
    out = torch.empty((T, H), dtype=_torch_dtype(dtype), device=device)
    for s in range(0, T, chunk):
        e = min(T, s + chunk)
        out[s:e] = torch.randn((e - s, H), generator=g, device=device,
                               dtype=torch.float32).to(out.dtype)
    return out


def lm_head(V: int, H: int, dtype: str, std: float = 0.02, device="cpu",
            seed: int = MASTER_SEED, chunk: int = 1 << 14) -> torch.Tensor:
    """LM-head weight, one row per vocabulary entry: [V, H] ~ N(0, std^2)."""
    g = _tgen(11, device, seed)
    out = torch.empty((V, H), dtype=_torch_dtype(dtype), device=device)
    for s in range(0, V, chunk):
        e = min(V, s + chunk)
        out[s:e] = (torch.randn((e - s, H), generator=g, device=device,
                                dtype=torch.float32) * std).to(out.dtype)
    return out


def target_tokens(T: int, V: int, seed: int = MASTER_SEED) -> np.ndarray:
    return _rng(12, seed).integers(0, V, T).astype(np.int32)


def logp_noise(T: int, std: float, seed: int = MASTER_SEED) -> np.ndarray:
    """N(0, std^2): the difference old log-prob minus current log-prob."""
    return (_rng(13, seed).standard_normal(T) * std).astype(np.float32)


def behaviour_logp_standin(hidden: torch.Tensor, W: torch.Tensor, target, w_std: float,
                           noise: np.ndarray, chunk: int = 1 << 14) -> torch.Tensor:
    """Synthetic log-probs of the behaviour policy for workloads too large for the
    CPU oracle to produce them.

    With i.i.d. N(0, w_std^2) head weights the logits of a token are i.i.d.
    N(0, s^2), s^2 = w_std^2 |h|^2, so log-sum-exp over V entries concentrates at
    log V + s^2/2 (mean of a log-normal).  The stand-in is that constant plus the
    token's own logit plus the seeded noise.  It is an INPUT recipe: it only has
    to put most importance ratios near one so that the clip is hit about as often
    as with `current + noise`; nothing is checked against it.
    """
    T, H = hidden.shape
    V = W.shape[0]
    tgt = torch.as_tensor(np.asarray(target), device=hidden.device, dtype=torch.long)
    nz = torch.as_tensor(noise, device=hidden.device, dtype=torch.float32)
    out = torch.empty(T, dtype=torch.float32, device=hidden.device)
    for s in range(0, T, chunk):
        e = min(T, s + chunk)
        h = hidden[s:e].float()
        wy = W[tgt[s:e]].float()
        zy = (h * wy).sum(dim=1)
        s2 = (w_std ** 2) * (h * h).sum(dim=1)
        out[s:e] = zy - (math.log(V) + 0.5 * s2) + nz[s:e]
    return out


@dataclass
class TokenBatch:
    hidden: torch.Tensor      # [T, H]
    W: torch.Tensor           # [V, H]
    target: np.ndarray        # int32 [T]
    noise: np.ndarray         # float32 [T]
    mask: np.ndarray | None   # uint8 [T] or None
    cu_seqlens: np.ndarray    # int32 [B+1]
    T: int


def token_batch(cfg: Config, device="cpu", seed: int = MASTER_SEED, lengths=None,
                w_scale: float = 1.0) -> TokenBatch:
    """The token-side tensors of a configuration.  w_scale > 1 gives the "peaked"
    variant (logit std grows, the softmax concentrates)."""
    L = response_lengths(cfg, seed) if lengths is None else np.asarray(lengths, np.int64)
    cu = cu_seqlens(L)
    T = int(cu[-1])
    return TokenBatch(
        hidden=hidden_states(T, cfg.H, cfg.dtype, device, seed),
        W=lm_head(cfg.V, cfg.H, cfg.dtype, cfg.w_std * w_scale, device, seed),
        target=target_tokens(T, cfg.V, seed),
        noise=logp_noise(T, cfg.noise_std, seed),
        mask=loss_mask(cfg, T, seed),
        cu_seqlens=cu,
        T=T,
    )


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a configuration with some sizes replaced (test-sized variants)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return Config(**d)
