"""ctypes binding of ``libspo_hip.so``: the same entry points as ``include/spo.h``.

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the path runs in the library's kernels.  There is no
fallback: a missing library or a non-zero status raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspo_hip.so")

SPO_FP32, SPO_BF16 = 0, 1
SPO_W_VH, SPO_W_HV = 0, 1
SPO_SAMPLE_STATIC_MAX_N = 1 << 20

EXPORTS = (
    "spo_status_string", "spo_sample_prompts_workspace_bytes", "spo_sample_prompts",
    "spo_sample_prompts_static",
    "spo_advantages_workspace_bytes", "spo_advantages", "spo_advantage_diagnostics", "spo_tracker_update_workspace_bytes", "spo_tracker_update",
    "spo_tracker_update_ema",
    "spo_tracker_init",
    "spo_pg_loss_fwd_workspace_bytes", "spo_pg_loss_fwd",
    "spo_pg_loss_bwd_workspace_bytes", "spo_pg_loss_bwd",
    "spo_pg_loss_fwd_bwd_workspace_bytes", "spo_pg_loss_fwd_bwd",
    "spo_kernel_timing_enable", "spo_kernel_timing_read",
)
TIMING_CLASSES = ("fwd_sweep", "bwd_recompute", "bwd_dhidden", "bwd_dw", "logits_fwd", "logits_bwd", "logits_to_dz")


class SpoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class PgDesc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_size_t), ("dtype", C.c_int), ("w_layout", C.c_int),
        ("T", C.c_int64), ("H", C.c_int64), ("V", C.c_int64), ("B", C.c_int32),
        ("hidden", C.c_void_p), ("W", C.c_void_p), ("logits", C.c_void_p),
        ("target", C.c_void_p), ("old_logp", C.c_void_p), ("mask", C.c_void_p),
        ("adv_norm", C.c_void_p), ("cu_seqlens", C.c_void_p),
        ("eps_low", C.c_float), ("eps_high", C.c_float),
    ]


_lib = None


def lib():
    """The loaded library; loading fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2509_13232_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, u64, u32, f32, f64, sz = (C.c_void_p, C.c_int64, C.c_int32, C.c_uint64,
                                                 C.c_uint32, C.c_float, C.c_double, C.c_size_t)
        L.spo_status_string.restype = C.c_char_p
        L.spo_status_string.argtypes = [C.c_int]
        L.spo_sample_prompts_workspace_bytes.restype = sz
        L.spo_sample_prompts_workspace_bytes.argtypes = [i64, i32]
        L.spo_sample_prompts.restype = C.c_int
        L.spo_sample_prompts.argtypes = [vp, vp, i64, i32, f64, u64, u64, C.c_int, u32, vp, vp, vp, sz, vp]
        L.spo_sample_prompts_static.restype = C.c_int
        L.spo_sample_prompts_static.argtypes = [vp, vp, i64, i32, f64, u64, u64, C.c_int, u32, vp, vp, vp]
        L.spo_advantages.restype = C.c_int
        L.spo_advantages.argtypes = [vp, vp, i64, vp, vp, i32, C.c_int, f32, C.c_int, vp, vp, vp, vp, vp, sz, vp]
        L.spo_advantages_workspace_bytes.restype = sz
        L.spo_advantages_workspace_bytes.argtypes = [i32]
        L.spo_advantage_diagnostics.restype = C.c_int
        L.spo_advantage_diagnostics.argtypes = [vp, vp, i32, f32, f32, vp, vp]
        L.spo_tracker_update.restype = C.c_int
        L.spo_tracker_update_workspace_bytes.restype = sz
        L.spo_tracker_update_workspace_bytes.argtypes = [i64]
        L.spo_tracker_update.argtypes = [vp, vp, i64, vp, vp, vp, i32, f32, f32, f32, C.c_int, vp, vp, vp, vp, sz, vp]
        L.spo_tracker_update_ema.restype = C.c_int
        L.spo_tracker_update_ema.argtypes = L.spo_tracker_update.argtypes
        L.spo_tracker_init.restype = C.c_int
        L.spo_tracker_init.argtypes = [vp, i64, f32, vp, vp, vp]
        L.spo_pg_loss_fwd_workspace_bytes.restype = sz
        L.spo_pg_loss_fwd_workspace_bytes.argtypes = [C.POINTER(PgDesc)]
        L.spo_pg_loss_fwd.restype = C.c_int
        L.spo_pg_loss_fwd.argtypes = [C.POINTER(PgDesc), vp, vp, vp, vp, vp, sz, vp]
        L.spo_pg_loss_bwd_workspace_bytes.restype = sz
        L.spo_pg_loss_bwd_workspace_bytes.argtypes = [C.POINTER(PgDesc), i64]
        L.spo_pg_loss_bwd.restype = C.c_int
        L.spo_pg_loss_bwd.argtypes = [C.POINTER(PgDesc), vp, vp, f32, vp, C.c_int, vp, C.c_int, C.c_int,
                                      vp, i64, vp, sz, vp]
        L.spo_pg_loss_fwd_bwd_workspace_bytes.restype = sz
        L.spo_pg_loss_fwd_bwd_workspace_bytes.argtypes = [C.POINTER(PgDesc), i64]
        L.spo_pg_loss_fwd_bwd.restype = C.c_int
        L.spo_pg_loss_fwd_bwd.argtypes = [C.POINTER(PgDesc), f32, vp, vp, vp, vp, vp, C.c_int, vp, C.c_int, C.c_int,
                                          i64, vp, sz, vp]
        L.spo_kernel_timing_enable.restype = C.c_int
        L.spo_kernel_timing_enable.argtypes = [C.c_int]
        L.spo_kernel_timing_read.restype = C.c_int
        L.spo_kernel_timing_read.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().spo_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise SpoError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _want(t, dtype, name, n=None):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of {dtype}")
    if n is not None and t.numel() != n:
        raise ValueError(f"{name}: expected {n} elements, got {t.numel()}")


def _workspace(nbytes: int, device, given=None):
    if given is not None:
        if given.dtype != torch.uint8 or given.numel() < nbytes or given.data_ptr() % 256:
            raise ValueError("workspace must be a 256-byte aligned uint8 tensor of sufficient size")
        return given
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _dt(t):
    return {torch.float32: SPO_FP32, torch.bfloat16: SPO_BF16}[t]


def spo_kernel_timing_enable(enable: bool):
    _check(lib().spo_kernel_timing_enable(int(bool(enable))), "spo_kernel_timing_enable")


def spo_kernel_timing_read():
    """{class name: (milliseconds, launches)} since the last read."""
    n = len(TIMING_CLASSES)
    ms = (C.c_float * n)()
    cnt = (C.c_int32 * n)()
    _check(lib().spo_kernel_timing_read(ms, cnt), "spo_kernel_timing_read")
    return {TIMING_CLASSES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


# ------------------------------------------------------------------ sampler
def spo_sample_prompts(alpha, beta, B, eps_explore=0.05, seed=0, iteration=0, replace=False,
                       max_attempts=0, workspace=None, return_info=False):
    N = alpha.numel()
    _want(alpha, torch.float32, "alpha")
    _want(beta, torch.float32, "beta", N)
    idx = torch.empty(B, dtype=torch.int32, device=alpha.device)
    info = torch.zeros(2, dtype=torch.int32, device=alpha.device)
    nbytes = lib().spo_sample_prompts_workspace_bytes(N, B)
    ws = _workspace(nbytes, alpha.device, workspace)
    _check(lib().spo_sample_prompts(_ptr(alpha), _ptr(beta), N, B, float(eps_explore), int(seed),
                                    int(iteration), int(bool(replace)), int(max_attempts), _ptr(idx),
                                    _ptr(info), _ptr(ws), ws.numel(), _stream()), "spo_sample_prompts")
    return (idx, info) if return_info else idx


def spo_sample_prompts_static(alpha, beta, B, eps_explore=0.05, seed=0, iteration=0, replace=False,
                              max_attempts=0, idx_out=None, info_out=None):
    """spo_sample_prompts without a workspace (the library's own fixed scratch array).  With
    idx_out / info_out given, the call touches no allocator at all."""
    N = alpha.numel()
    _want(alpha, torch.float32, "alpha")
    _want(beta, torch.float32, "beta", N)
    idx = torch.empty(B, dtype=torch.int32, device=alpha.device) if idx_out is None else idx_out
    info = torch.zeros(2, dtype=torch.int32, device=alpha.device) if info_out is None else info_out
    _want(idx, torch.int32, "idx_out", B)
    _want(info, torch.int32, "info_out", 2)
    _check(lib().spo_sample_prompts_static(_ptr(alpha), _ptr(beta), N, B, float(eps_explore), int(seed),
                                           int(iteration), int(bool(replace)), int(max_attempts), _ptr(idx),
                                           _ptr(info), _stream()), "spo_sample_prompts_static")
    return idx, info


# --------------------------------------------------------------- advantages
def spo_advantages(alpha, beta, idx, reward, ddof=0, eps_norm=0.0, use_baseline=True, info=None, workspace=None):
    """Returns (adv_raw, adv_norm, stats).  info: optional int32[1] tensor that receives the range flag."""
    B = reward.numel()
    _want(info, torch.int32, "info", 1)
    _want(reward, torch.float32, "reward")
    if use_baseline:
        _want(alpha, torch.float32, "alpha")
        _want(beta, torch.float32, "beta", alpha.numel())  # None: alpha holds v_hat itself
        _want(idx, torch.int32, "idx", B)
    N = alpha.numel() if alpha is not None else 0
    raw = torch.empty(B, dtype=torch.float32, device=reward.device)
    nrm = torch.empty(B, dtype=torch.float32, device=reward.device)
    st = torch.empty(2, dtype=torch.float32, device=reward.device)
    _check(lib().spo_advantages(_ptr(alpha), _ptr(beta), N, _ptr(idx), _ptr(reward), B, int(ddof),
                                float(eps_norm), int(bool(use_baseline)), _ptr(raw), _ptr(nrm), _ptr(st),
                                _ptr(info), _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                _stream()), "spo_advantages")
    return raw, nrm, st


def spo_advantage_diagnostics(adv_raw, reward, tau_tight=1e-4, tau_loose=0.02):
    """fp32[4]: share |A|<=tau_tight, share |A|<=tau_loose, var(A), var(reward)."""
    B = adv_raw.numel()
    _want(adv_raw, torch.float32, "adv_raw")
    _want(reward, torch.float32, "reward", B)
    diag = torch.empty(4, dtype=torch.float32, device=adv_raw.device)
    _check(lib().spo_advantage_diagnostics(_ptr(adv_raw), _ptr(reward), B, float(tau_tight), float(tau_loose),
                                           _ptr(diag), _stream()), "spo_advantage_diagnostics")
    return diag


# ------------------------------------------------------------------ tracker
def _tracker_update(fn, name, a, b, idx, reward, kl, d_half, rho_min, rho_max, ids_unique, n_obs, want_v_prev,
                    info, workspace, check_repeats):
    N, B = a.numel(), idx.numel()
    _want(a, torch.float32, "state[0]")
    _want(b, torch.float32, "state[1]", N)
    _want(idx, torch.int32, "idx")
    _want(reward, torch.float32, "reward", B)
    _want(kl, torch.float32, "kl", B)
    _want(n_obs, torch.int32, "n_obs", N)
    _want(info, torch.int32, "info", 1)
    vprev = torch.empty(B, dtype=torch.float32, device=a.device) if want_v_prev else None
    ws = workspace
    if ws is None and (not ids_unique or check_repeats):   # the table of one int32 per prompt
        ws = _workspace(lib().spo_tracker_update_workspace_bytes(N), a.device)
    _check(fn(_ptr(a), _ptr(b), N, _ptr(idx), _ptr(reward), _ptr(kl), B, float(d_half), float(rho_min),
              float(rho_max), int(bool(ids_unique)), _ptr(n_obs), _ptr(vprev), _ptr(info), _ptr(ws),
              0 if ws is None else ws.numel(), _stream()), name)
    return vprev


def spo_tracker_update(alpha, beta, idx, reward, kl, d_half, rho_min, rho_max, ids_unique=True,
                       n_obs=None, want_v_prev=False, info=None, workspace=None, check_repeats=False):
    """Updates alpha and beta IN PLACE; returns v_prev[B] when asked.  info: optional int32[1] tensor
    (bit 1: id out of range, bit 2: repeated id with ids_unique, looked for when check_repeats)."""
    return _tracker_update(lib().spo_tracker_update, "spo_tracker_update", alpha, beta, idx, reward, kl, d_half,
                           rho_min, rho_max, ids_unique, n_obs, want_v_prev, info, workspace, check_repeats)


def spo_tracker_update_ema(v_hat, n_eff, idx, reward, kl, d_half, rho_min, rho_max, ids_unique=True,
                           n_obs=None, want_v_prev=False, info=None, workspace=None, check_repeats=False):
    """Moving-average form: updates v_hat and n_eff IN PLACE; returns v_prev[B] when asked."""
    return _tracker_update(lib().spo_tracker_update_ema, "spo_tracker_update_ema", v_hat, n_eff, idx, reward, kl,
                           d_half, rho_min, rho_max, ids_unique, n_obs, want_v_prev, info, workspace, check_repeats)


def spo_tracker_init(v0, rho_min):
    _want(v0, torch.float32, "v0")
    a = torch.empty_like(v0)
    b = torch.empty_like(v0)
    _check(lib().spo_tracker_init(_ptr(v0), v0.numel(), float(rho_min), _ptr(a), _ptr(b), _stream()),
           "spo_tracker_init")
    return a, b


# --------------------------------------------------------------------- loss
def make_desc(hidden, W, target, old_logp, mask, adv_norm, cu_seqlens, eps_low, eps_high,
              w_layout=SPO_W_VH, logits=None):
    """Builds the C descriptor; returns (desc, keepalive tuple)."""
    d = PgDesc()
    d.struct_size = C.sizeof(PgDesc)
    if logits is not None:
        _want(logits, logits.dtype, "logits")
        T, V = logits.shape
        H = 0
        d.dtype = _dt(logits.dtype)
    else:
        _want(hidden, hidden.dtype, "hidden")
        _want(W, hidden.dtype, "W")
        T, H = hidden.shape
        if w_layout == SPO_W_VH:
            V = W.shape[0]
            assert W.shape[1] == H, "SPO_W_VH expects W of shape [V, H]"
        else:
            V = W.shape[1]
            assert W.shape[0] == H, "SPO_W_HV expects W of shape [H, V]"
        d.dtype = _dt(hidden.dtype)
    B = adv_norm.numel()
    _want(target, torch.int32, "target", T)
    _want(old_logp, torch.float32, "old_logp", T)
    _want(mask, torch.uint8, "mask", T)
    _want(adv_norm, torch.float32, "adv_norm")
    _want(cu_seqlens, torch.int32, "cu_seqlens", B + 1)
    d.w_layout = w_layout
    d.T, d.H, d.V, d.B = T, H, V, B
    d.hidden = None if hidden is None else hidden.data_ptr()
    d.W = None if W is None else W.data_ptr()
    d.logits = None if logits is None else logits.data_ptr()
    d.target = target.data_ptr()
    d.old_logp = old_logp.data_ptr()
    d.mask = None if mask is None else mask.data_ptr()
    d.adv_norm = adv_norm.data_ptr()
    d.cu_seqlens = cu_seqlens.data_ptr()
    d.eps_low, d.eps_high = float(eps_low), float(eps_high)
    return d, (hidden, W, logits, target, old_logp, mask, adv_norm, cu_seqlens)


def spo_pg_loss_fwd(desc, workspace=None, want_stats=True):
    """Returns (loss[1], logp[T], lse[T], stats[4] or None)."""
    d, keep = desc
    dev = keep[3].device
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    logp = torch.empty(max(d.T, 1), dtype=torch.float32, device=dev)[:d.T]
    lse = torch.empty(max(d.T, 1), dtype=torch.float32, device=dev)[:d.T]
    stats = torch.empty(4, dtype=torch.float32, device=dev) if want_stats else None
    nbytes = lib().spo_pg_loss_fwd_workspace_bytes(C.byref(d))
    ws = _workspace(nbytes, dev, workspace)
    _check(lib().spo_pg_loss_fwd(C.byref(d), _ptr(loss), _ptr(logp), _ptr(lse), _ptr(stats), _ptr(ws),
                                 ws.numel(), _stream()), "spo_pg_loss_fwd")
    return loss, logp, lse, stats


def spo_pg_loss_bwd_workspace_bytes(desc, chunk_tokens=0) -> int:
    return int(lib().spo_pg_loss_bwd_workspace_bytes(C.byref(desc[0]), int(chunk_tokens)))


def spo_pg_loss_bwd(desc, logp, lse, grad_loss=1.0, d_hidden_dtype=None, d_W_dtype=torch.float32,
                    d_W=None, accumulate_dW=False, want_d_hidden=True, want_d_W=True, chunk_tokens=0,
                    workspace=None):
    """Fused form: returns (d_hidden[T,H] or None, d_W in W's layout or None).
    Logits-in form: returns d_logits[T,V]."""
    d, keep = desc
    dev = keep[3].device
    _want(logp, torch.float32, "logp", d.T)
    _want(lse, torch.float32, "lse", d.T)
    nbytes = lib().spo_pg_loss_bwd_workspace_bytes(C.byref(d), int(chunk_tokens))
    ws = _workspace(nbytes, dev, workspace)
    if d.logits:
        dl = torch.empty((d.T, d.V), dtype=keep[2].dtype, device=dev)
        _check(lib().spo_pg_loss_bwd(C.byref(d), _ptr(logp), _ptr(lse), float(grad_loss), None, 0, None, 0,
                                     0, _ptr(dl), int(chunk_tokens), _ptr(ws), ws.numel(), _stream()),
               "spo_pg_loss_bwd")
        return dl
    hidden, W = keep[0], keep[1]
    dx = None
    if want_d_hidden:
        dx = torch.empty((d.T, d.H), dtype=d_hidden_dtype or hidden.dtype, device=dev)
    if want_d_W and d_W is None:
        if accumulate_dW:
            raise ValueError("accumulate_dW needs an existing d_W")
        d_W = torch.empty(W.shape, dtype=d_W_dtype, device=dev)
    if not want_d_W:
        d_W = None
    _check(lib().spo_pg_loss_bwd(C.byref(d), _ptr(logp), _ptr(lse), float(grad_loss), _ptr(dx),
                                 _dt(dx.dtype) if dx is not None else 0, _ptr(d_W),
                                 _dt(d_W.dtype) if d_W is not None else 0, int(bool(accumulate_dW)), None,
                                 int(chunk_tokens), _ptr(ws), ws.numel(), _stream()), "spo_pg_loss_bwd")
    return dx, d_W


def spo_pg_loss_fwd_bwd_workspace_bytes(desc, chunk_tokens=0) -> int:
    return int(lib().spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(desc[0]), int(chunk_tokens)))


def spo_pg_loss_fwd_bwd(desc, grad_loss=1.0, d_hidden_dtype=None, d_W_dtype=torch.float32, d_W=None,
                        accumulate_dW=False, want_d_hidden=True, want_d_W=True, chunk_tokens=0, workspace=None,
                        want_stats=True):
    """Fused form only.  Returns (loss[1], logp[T], lse[T], stats[4] or None, d_hidden or None, d_W or None)."""
    d, keep = desc
    dev = keep[3].device
    hidden, W = keep[0], keep[1]
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    logp = torch.empty(max(d.T, 1), dtype=torch.float32, device=dev)[:d.T]
    lse = torch.empty(max(d.T, 1), dtype=torch.float32, device=dev)[:d.T]
    stats = torch.empty(4, dtype=torch.float32, device=dev) if want_stats else None
    nbytes = lib().spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(d), int(chunk_tokens))
    ws = _workspace(nbytes, dev, workspace)
    dx = None
    if want_d_hidden:
        dx = torch.empty((d.T, d.H), dtype=d_hidden_dtype or hidden.dtype, device=dev)
    if want_d_W and d_W is None:
        if accumulate_dW:
            raise ValueError("accumulate_dW needs an existing d_W")
        d_W = torch.empty(W.shape, dtype=d_W_dtype, device=dev)
    if not want_d_W:
        d_W = None
    _check(lib().spo_pg_loss_fwd_bwd(C.byref(d), float(grad_loss), _ptr(loss), _ptr(logp), _ptr(lse), _ptr(stats),
                                     _ptr(dx), _dt(dx.dtype) if dx is not None else 0, _ptr(d_W),
                                     _dt(d_W.dtype) if d_W is not None else 0, int(bool(accumulate_dW)),
                                     int(chunk_tokens), _ptr(ws), ws.numel(), _stream()), "spo_pg_loss_fwd_bwd")
    return loss, logp, lse, stats, dx, d_W
