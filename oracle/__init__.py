"""fp64 CPU oracle for the SPO hot path: ctypes front end of ``spo_oracle.c``.

TEST INFRASTRUCTURE ONLY.  It is imported by ``tests/``, by the smoke check and
by the CPU-baseline leg of the benchmark, never by the product package, and it
imports nothing from the product package.  Each function marshals numpy arrays
into the C routine of the same name; all arithmetic lives in the C file, which
states the passage of the paper every routine follows.

Every function is pinned by ``tests/test_oracle_*.py`` (``philox4x32_10`` by
the generator's published known-answer vectors).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spo_oracle.c")
_LIB = os.path.join(_HERE, "libspo_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_d = C.POINTER(C.c_double)
_f = C.POINTER(C.c_float)
_i32 = C.POINTER(C.c_int32)
_i64 = C.POINTER(C.c_int64)
_u8 = C.POINTER(C.c_uint8)
_u32 = C.POINTER(C.c_uint32)
_u64 = C.POINTER(C.c_uint64)


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = C.CDLL(build())
            lib.spo_oracle_discount.restype = C.c_double
            lib.spo_oracle_discount.argtypes = [C.c_double] * 4
            lib.spo_oracle_tracker_update.restype = None
            lib.spo_oracle_tracker_update.argtypes = [
                _d, _d, C.c_int64, _i32, _d, _d, C.c_int32, C.c_double, C.c_double,
                C.c_double, _d, _d]
            lib.spo_oracle_tracker_update_ema.restype = None
            lib.spo_oracle_tracker_update_ema.argtypes = [
                _d, _d, C.c_int64, _i32, _d, _d, C.c_int32, C.c_double, C.c_double, C.c_double, _d]
            lib.spo_oracle_tracker_init.restype = None
            lib.spo_oracle_tracker_init.argtypes = [_d, C.c_int64, C.c_double, _d, _d]
            lib.spo_oracle_advantages.restype = None
            lib.spo_oracle_advantages.argtypes = [
                _d, _d, C.c_int64, _i32, _d, C.c_int32, C.c_int, C.c_double, C.c_int,
                _d, _d, _d]
            lib.spo_oracle_advantage_diagnostics.restype = None
            lib.spo_oracle_advantage_diagnostics.argtypes = [_d, _d, C.c_int32, C.c_double, C.c_double, _d]
            lib.spo_oracle_weights.restype = None
            lib.spo_oracle_weights.argtypes = [_f, _f, C.c_int64, C.c_double, _d]
            lib.spo_oracle_weight_code.restype = C.c_uint64
            lib.spo_oracle_weight_code.argtypes = [C.c_double]
            lib.spo_oracle_weight_cdf.restype = None
            lib.spo_oracle_weight_cdf.argtypes = [_f, _f, C.c_int64, C.c_double, _u64]
            lib.spo_oracle_philox4x32_10.restype = None
            lib.spo_oracle_philox4x32_10.argtypes = [_u32, _u32, _u32]
            lib.spo_oracle_sample.restype = C.c_int
            lib.spo_oracle_sample.argtypes = [
                _f, _f, C.c_int64, C.c_int32, C.c_double, C.c_uint64, C.c_uint64,
                C.c_int, C.c_uint32, _i32, _u32]
            lib.spo_oracle_pg_fwd.restype = None
            lib.spo_oracle_pg_fwd.argtypes = [
                _d, _d, _d, C.c_int64, C.c_int64, C.c_int64, _i32, _d, _u8, _d, _i32,
                C.c_int32, C.c_double, C.c_double, _i64, C.c_int64, _d, _d, _d, _d,
                _u8, _d]
            lib.spo_oracle_pg_bwd.restype = None
            lib.spo_oracle_pg_bwd.argtypes = [
                _d, _d, _d, C.c_int64, C.c_int64, C.c_int64, _i32, _d, _u8, _d, _i32,
                C.c_int32, C.c_double, C.c_double, C.c_double, _i64, C.c_int64, _i64,
                C.c_int64, _d, _d, _d, _d]
            _lib = lib
    return _lib


def _arr(x, dtype):
    return np.ascontiguousarray(np.asarray(x), dtype=dtype)


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(typ)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use (its default team size)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return os.cpu_count() or 1


def set_num_threads(n: int) -> None:
    """Team size of the oracle's OpenMP loops from now on (the OpenMP runtime's own setter,
    reached through the oracle library, which links it)."""
    f = _load().omp_set_num_threads
    f.restype = None
    f.argtypes = [C.c_int]
    f(int(n))
    os.environ["OMP_NUM_THREADS"] = str(int(n))   # num_threads() reports this


# --------------------------------------------------------------------- tracker
def discount(kl, d_half, rho_min, rho_max) -> float:
    return float(_load().spo_oracle_discount(kl, d_half, rho_min, rho_max))


def tracker_update(alpha, beta, idx, reward, kl, d_half, rho_min, rho_max):
    """Returns (alpha', beta', v_prev[B], rho[B]); inputs are not modified."""
    a = _arr(alpha, np.float64).copy()
    b = _arr(beta, np.float64).copy()
    idx = _arr(idx, np.int32)
    r = _arr(reward, np.float64)
    k = _arr(kl, np.float64)
    B = idx.shape[0]
    assert r.shape[0] == B and k.shape[0] == B
    assert B == 0 or (idx.min() >= 0 and idx.max() < a.shape[0])
    vprev = np.empty(B, np.float64)
    rho = np.empty(B, np.float64)
    _load().spo_oracle_tracker_update(_p(a, _d), _p(b, _d), a.shape[0], _p(idx, _i32),
                                      _p(r, _d), _p(k, _d), B, d_half, rho_min, rho_max,
                                      _p(vprev, _d), _p(rho, _d))
    return a, b, vprev, rho


def tracker_update_ema(v_hat, n_eff, idx, reward, kl, d_half, rho_min, rho_max):
    """Moving-average form. Returns (v', n_eff', v_prev[B]); inputs are not modified."""
    v = _arr(v_hat, np.float64).copy()
    n = _arr(n_eff, np.float64).copy()
    idx = _arr(idx, np.int32)
    r = _arr(reward, np.float64)
    k = _arr(kl, np.float64)
    B = idx.shape[0]
    assert r.shape[0] == B and k.shape[0] == B and v.shape == n.shape
    assert B == 0 or (idx.min() >= 0 and idx.max() < v.shape[0])
    vprev = np.empty(B, np.float64)
    _load().spo_oracle_tracker_update_ema(_p(v, _d), _p(n, _d), v.shape[0], _p(idx, _i32),
                                          _p(r, _d), _p(k, _d), B, d_half, rho_min, rho_max,
                                          _p(vprev, _d))
    return v, n, vprev


def tracker_init(v0, rho_min):
    v = _arr(v0, np.float64)
    a = np.empty_like(v)
    b = np.empty_like(v)
    _load().spo_oracle_tracker_init(_p(v, _d), v.shape[0], rho_min, _p(a, _d), _p(b, _d))
    return a, b


# ------------------------------------------------------------------ advantages
def advantages(alpha, beta, idx, reward, ddof=0, eps_norm=0.0, use_baseline=True):
    """Returns (adv_raw[B], adv_norm[B], (mu, sigma)).  ``beta=None``: ``alpha``
    holds the value estimate itself (moving-average form of the tracker)."""
    a = _arr(alpha, np.float64)
    b = None if beta is None else _arr(beta, np.float64)
    idx = _arr(idx, np.int32)
    r = _arr(reward, np.float64)
    B = idx.shape[0]
    assert B == 0 or (idx.min() >= 0 and idx.max() < a.shape[0])
    raw = np.empty(B, np.float64)
    nrm = np.empty(B, np.float64)
    st = np.zeros(2, np.float64)
    _load().spo_oracle_advantages(_p(a, _d), None if b is None else _p(b, _d), a.shape[0], _p(idx, _i32),
                                  _p(r, _d), B, int(ddof), float(eps_norm),
                                  int(bool(use_baseline)), _p(raw, _d), _p(nrm, _d),
                                  _p(st, _d))
    return raw, nrm, (float(st[0]), float(st[1]))


def advantage_diagnostics(adv_raw, reward, tau_tight=1e-4, tau_loose=0.02):
    """Returns [share |A|<=tau_tight, share |A|<=tau_loose, var(A), var(r)]."""
    a = _arr(adv_raw, np.float64)
    r = _arr(reward, np.float64)
    assert a.shape == r.shape and a.shape[0] > 0
    out = np.empty(4, np.float64)
    _load().spo_oracle_advantage_diagnostics(_p(a, _d), _p(r, _d), a.shape[0], float(tau_tight),
                                             float(tau_loose), _p(out, _d))
    return out


# --------------------------------------------------------------------- sampler
def weights(alpha, beta, eps=0.05):
    a = _arr(alpha, np.float32)
    b = _arr(beta, np.float32)
    w = np.empty(a.shape[0], np.float64)
    _load().spo_oracle_weights(_p(a, _f), _p(b, _f), a.shape[0], float(eps), _p(w, _d))
    return w


def weight_code(w: float) -> int:
    return int(_load().spo_oracle_weight_code(float(w)))


def weight_cdf(alpha, beta, eps=0.05):
    a = _arr(alpha, np.float32)
    b = _arr(beta, np.float32)
    c = np.empty(a.shape[0], np.uint64)
    _load().spo_oracle_weight_cdf(_p(a, _f), _p(b, _f), a.shape[0], float(eps), _p(c, _u64))
    return c


def philox4x32_10(ctr, key):
    c = _arr(ctr, np.uint32)
    k = _arr(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, np.uint32)
    _load().spo_oracle_philox4x32_10(_p(c, _u32), _p(k, _u32), _p(out, _u32))
    return out


def sample_prompts(alpha, beta, B, eps=0.05, seed=0, iteration=0, replace=False,
                   max_attempts=1 << 20, return_attempts=False):
    a = _arr(alpha, np.float32)
    b = _arr(beta, np.float32)
    N = a.shape[0]
    if not replace and B > N:
        raise ValueError("sampling without replacement needs B <= N")
    idx = np.empty(B, np.int32)
    att = np.zeros(B, np.uint32)
    rc = _load().spo_oracle_sample(_p(a, _f), _p(b, _f), N, B, float(eps), int(seed),
                                   int(iteration), int(bool(replace)), int(max_attempts),
                                   _p(idx, _i32), _p(att, _u32))
    if rc != 0:
        raise RuntimeError("sampler exceeded max_attempts")
    return (idx, att) if return_attempts else idx


# ------------------------------------------------------------------------ loss
def _pg_common(hidden, W, logits, target, old_logp, mask, adv_norm, cu_seqlens):
    if logits is not None:
        lg = _arr(logits, np.float64)
        T, V = lg.shape
        H = 0
        hd = w = None
    else:
        lg = None
        hd = _arr(hidden, np.float64)
        w = _arr(W, np.float64)
        T, H = hd.shape
        V = w.shape[0]
        assert w.shape[1] == H, "W is [V, H]"
    tg = _arr(target, np.int32)
    ol = _arr(old_logp, np.float64)
    mk = None if mask is None else _arr(mask, np.uint8)
    ad = _arr(adv_norm, np.float64)
    cu = _arr(cu_seqlens, np.int32)
    B = cu.shape[0] - 1
    assert tg.shape[0] == T and ol.shape[0] == T and ad.shape[0] == B
    assert cu[0] == 0 and cu[-1] == T and np.all(np.diff(cu) >= 0)
    assert T == 0 or (tg.min() >= 0 and tg.max() < V)
    assert mk is None or mk.shape[0] == T
    return hd, w, lg, T, H, V, tg, ol, mk, ad, cu, B


def pg_loss_fwd(hidden, W, target, old_logp, mask, adv_norm, cu_seqlens,
                eps_low=0.2, eps_high=0.28, rows=None, logits=None):
    """Returns a dict with per-token lse, logp, ratio, obj, active and, when
    rows is None, the scalar loss (= minus the masked mean objective) and M."""
    hd, w, lg, T, H, V, tg, ol, mk, ad, cu, B = _pg_common(
        hidden, W, logits, target, old_logp, mask, adv_norm, cu_seqlens)
    rw = None if rows is None else _arr(rows, np.int64)
    n = T if rw is None else rw.shape[0]
    assert rw is None or n == 0 or (rw.min() >= 0 and rw.max() < T)
    out = {k: np.empty(n, np.float64) for k in ("lse", "logp", "ratio", "obj")}
    act = np.empty(n, np.uint8)
    loss = np.zeros(2, np.float64)
    _load().spo_oracle_pg_fwd(_p(hd, _d), _p(w, _d), _p(lg, _d), T, H, V, _p(tg, _i32),
                              _p(ol, _d), _p(mk, _u8), _p(ad, _d), _p(cu, _i32), B,
                              float(eps_low), float(eps_high), _p(rw, _i64), n,
                              _p(out["lse"], _d), _p(out["logp"], _d),
                              _p(out["ratio"], _d), _p(out["obj"], _d), _p(act, _u8),
                              _p(loss, _d))
    out["active"] = act
    if rw is None:
        out["loss"] = float(loss[0])
        out["M"] = float(loss[1])
    return out


def pg_loss_bwd(hidden, W, target, old_logp, mask, adv_norm, cu_seqlens,
                eps_low=0.2, eps_high=0.28, grad_loss=1.0, rows=None, vsel=None,
                want_dx=True, want_dw=True, logits=None):
    """Returns a dict with g[n] and, as asked, d_hidden[n,H], d_W[nv,H] (W's own
    [V,H] layout) or d_logits[n,V] for the logits-in variant."""
    hd, w, lg, T, H, V, tg, ol, mk, ad, cu, B = _pg_common(
        hidden, W, logits, target, old_logp, mask, adv_norm, cu_seqlens)
    rw = None if rows is None else _arr(rows, np.int64)
    vs = None if vsel is None else _arr(vsel, np.int64)
    n = T if rw is None else rw.shape[0]
    nv = V if vs is None else vs.shape[0]
    assert rw is None or n == 0 or (rw.min() >= 0 and rw.max() < T)
    assert vs is None or nv == 0 or (vs.min() >= 0 and vs.max() < V)
    g = np.empty(n, np.float64)
    dx = dw = dl = None
    if lg is not None:
        dl = np.empty((n, V), np.float64)
    else:
        if want_dx:
            dx = np.empty((n, H), np.float64)
        if want_dw:
            dw = np.empty((nv, H), np.float64)
    _load().spo_oracle_pg_bwd(_p(hd, _d), _p(w, _d), _p(lg, _d), T, H, V, _p(tg, _i32),
                              _p(ol, _d), _p(mk, _u8), _p(ad, _d), _p(cu, _i32), B,
                              float(eps_low), float(eps_high), float(grad_loss),
                              _p(rw, _i64), n, _p(vs, _i64), nv, _p(dx, _d), _p(dw, _d),
                              _p(dl, _d), _p(g, _d))
    return {"g": g, "d_hidden": dx, "d_W": dw, "d_logits": dl}
