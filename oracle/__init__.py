"""Python face of the CPU oracle (test infrastructure, not product code).

The arithmetic lives in ``impact_oracle.c`` (plain C, fp64); this file only
compiles it with gcc, loads it through ctypes and converts arrays.  The circular
buffer's integer bookkeeping oracle is in ``oracle.buffer`` (plain Python).

Nothing in here imports or calls the GPU library.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "impact_oracle.c")
# ORACLE_LIB_OVERRIDE: load this library instead (the tests that plant mistakes in a copy of the C source
# and check that the pins notice them set it; nothing else does)
_LIB = os.environ.get("ORACLE_LIB_OVERRIDE") or os.path.join(_HERE, "liboracle.so")

CATEGORICAL = 0
GAUSSIAN = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a few hundred ms)."""
    if os.environ.get("ORACLE_LIB_OVERRIDE"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in
                ("gamma", "lam", "rho_bar", "c_bar", "rho_clip", "eps", "vf_coeff", "ent_coeff", "kl_coeff")] + \
               [("ratio_mode", ctypes.c_int)]


RATIO_TARGET_CLIP, RATIO_WORKER = 0, 1      # Section 4.1: R_3 (R_1 when rho_clip = inf) / R_2


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        L.oracle_cat_logsumexp.restype = ctypes.c_double
        L.oracle_cat_logsumexp.argtypes = [dp, ctypes.c_int]
        L.oracle_cat_logp.restype = ctypes.c_double
        L.oracle_cat_logp.argtypes = [dp, ctypes.c_int, ctypes.c_int]
        L.oracle_cat_entropy.restype = ctypes.c_double
        L.oracle_cat_entropy.argtypes = [dp, ctypes.c_int]
        L.oracle_cat_kl.restype = ctypes.c_double
        L.oracle_cat_kl.argtypes = [dp, dp, ctypes.c_int]
        L.oracle_gauss_logp.restype = ctypes.c_double
        L.oracle_gauss_logp.argtypes = [dp, ctypes.c_int, dp]
        L.oracle_gauss_entropy.restype = ctypes.c_double
        L.oracle_gauss_entropy.argtypes = [dp, ctypes.c_int]
        L.oracle_gauss_kl.restype = ctypes.c_double
        L.oracle_gauss_kl.argtypes = [dp, dp, ctypes.c_int]
        for name in ("oracle_ratio", "oracle_ratio_twin"):
            f = getattr(L, name)
            f.restype = ctypes.c_double
            f.argtypes = [ctypes.c_double] * 4
        L.oracle_ratio_worker.restype = ctypes.c_double
        L.oracle_ratio_worker.argtypes = [ctypes.c_double] * 2
        L.oracle_surrogate.restype = ctypes.c_double
        L.oracle_surrogate.argtypes = [ctypes.c_double] * 3
        L.oracle_surrogate_active.restype = ctypes.c_int
        L.oracle_surrogate_active.argtypes = [ctypes.c_double] * 3
        L.oracle_bf16_bits.restype = ctypes.c_uint16
        L.oracle_bf16_bits.argtypes = [ctypes.c_float]
        L.oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def make_config(gamma=0.99, lam=1.0, rho_bar=1.0, c_bar=1.0, rho_clip=2.0, eps=0.2,
                vf_coeff=1.0, ent_coeff=0.01, kl_coeff=0.0, ratio_mode=RATIO_TARGET_CLIP) -> _Cfg:
    return _Cfg(gamma, lam, rho_bar, c_bar, rho_clip, eps, vf_coeff, ent_coeff, kl_coeff, int(ratio_mode))


def config_from_hyper(h) -> _Cfg:
    return make_config(h.gamma, h.lam, h.rho_bar, h.c_bar, h.rho_clip, h.eps,
                       h.vf_coeff, h.ent_coeff, h.kl_coeff, getattr(h, "ratio_mode", RATIO_TARGET_CLIP))


# --- small per-step functions (used by the pin tests) -------------------------

def cat_logsumexp(z) -> float:
    z = _f64(z)
    return lib().oracle_cat_logsumexp(z.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), z.size)


def cat_logp(z, a: int) -> float:
    z = _f64(z)
    return lib().oracle_cat_logp(z.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), z.size, int(a))


def cat_entropy(z) -> float:
    z = _f64(z)
    return lib().oracle_cat_entropy(z.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), z.size)


def cat_kl(z_target, z_theta) -> float:
    zt, zl = _f64(z_target), _f64(z_theta)
    dp = ctypes.POINTER(ctypes.c_double)
    return lib().oracle_cat_kl(zt.ctypes.data_as(dp), zl.ctypes.data_as(dp), zt.size)


def gauss_logp(params, act) -> float:
    p, a = _f64(params), _f64(act)
    dp = ctypes.POINTER(ctypes.c_double)
    return lib().oracle_gauss_logp(p.ctypes.data_as(dp), a.size, a.ctypes.data_as(dp))


def gauss_entropy(params) -> float:
    p = _f64(params)
    return lib().oracle_gauss_entropy(p.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), p.size // 2)


def gauss_kl(p_target, p_theta) -> float:
    pt, pl = _f64(p_target), _f64(p_theta)
    dp = ctypes.POINTER(ctypes.c_double)
    return lib().oracle_gauss_kl(pt.ctypes.data_as(dp), pl.ctypes.data_as(dp), pt.size // 2)


def ratio(lp_theta, lp_target, lp_worker, rho_clip) -> float:
    return lib().oracle_ratio(lp_theta, lp_target, lp_worker, rho_clip)


def ratio_worker(lp_theta, lp_worker) -> float:
    return lib().oracle_ratio_worker(lp_theta, lp_worker)


def ratio_twin(lp_theta, lp_target, lp_worker, rho_clip) -> float:
    return lib().oracle_ratio_twin(lp_theta, lp_target, lp_worker, rho_clip)


def surrogate(R, adv, eps) -> float:
    return lib().oracle_surrogate(R, adv, eps)


def surrogate_active(R, adv, eps) -> int:
    return lib().oracle_surrogate_active(R, adv, eps)


def vtrace_trajectory(logp_target, logp_worker, rewards, dones, values, bootstrap, cfg: _Cfg,
                      twin: bool = False):
    """vs, adv for one trajectory from per-step log-probs (recurrence, or the O(T^2) sums)."""
    lpt, lpw, r, v = _f64(logp_target), _f64(logp_worker), _f64(rewards), _f64(values)
    dn = np.ascontiguousarray(np.asarray(dones, dtype=np.uint8))
    T = lpt.size
    vs, adv = np.empty(T), np.empty(T)
    f = lib().oracle_vtrace_sum if twin else lib().oracle_vtrace_scan
    f.restype = None
    f(ctypes.c_int(T), _ptr(lpt), _ptr(lpw), _ptr(r), _ptr(dn), _ptr(v), ctypes.c_double(bootstrap),
      ctypes.byref(cfg), _ptr(vs), _ptr(adv))
    return vs, adv


# --- batch-level entry points ---------------------------------------------------

def _dist_code(dist) -> int:
    if dist in (CATEGORICAL, "categorical"):
        return CATEGORICAL
    if dist in (GAUSSIAN, "gaussian"):
        return GAUSSIAN
    raise ValueError(dist)


def _actions(dist_code: int, actions) -> np.ndarray:
    if dist_code == CATEGORICAL:
        return np.ascontiguousarray(np.asarray(actions, dtype=np.int32))
    return _f64(actions)


def _opt64(x):
    return None if x is None else _f64(x)


def vtrace_targets(dist, target, worker, actions, rewards, dones, values, bootstrap, cfg: _Cfg,
                   twin: bool = False, n_threads: int = 1, cached_logp=None):
    """cached_logp: [T][B][2] = (log pi_worker(a), log pi_target(a)); target and worker are then not read
    (pass None, with the action dimension A as `actions`' last axis or via the cached array's shape)."""
    d = _dist_code(dist)
    target, worker, cached = _opt64(target), _opt64(worker), _opt64(cached_logp)
    act = _actions(d, actions)
    if cached is not None:
        T, B = cached.shape[:2]
        A = 1 if d == CATEGORICAL else act.shape[-1]
    else:
        T, B, W = target.shape
        A = W if d == CATEGORICAL else W // 2
    r, v, bs = _f64(rewards), _f64(values), _f64(bootstrap)
    dn = np.ascontiguousarray(np.asarray(dones, dtype=np.uint8))
    vs, adv = np.empty((T, B)), np.empty((T, B))
    f = lib().oracle_vtrace_targets
    f.restype = ctypes.c_int
    rc = f(ctypes.c_int(d), ctypes.c_int(T), ctypes.c_int(B), ctypes.c_int(A), _ptr(target), _ptr(worker),
           _ptr(cached), _ptr(act), _ptr(r), _ptr(dn), _ptr(v), _ptr(bs), ctypes.byref(cfg),
           ctypes.c_int(int(twin)), ctypes.c_int(n_threads), _ptr(vs), _ptr(adv))
    if rc:
        raise RuntimeError(f"oracle_vtrace_targets failed: {rc}")
    return vs, adv


def loss_given_targets(dist, learner, target, worker, actions, values, vs, adv, cfg: _Cfg,
                       want_grads: bool = True, n_threads: int = 1, cached_logp=None) -> Dict[str, np.ndarray]:
    d = _dist_code(dist)
    learner, target, worker, cached = _f64(learner), _opt64(target), _opt64(worker), _opt64(cached_logp)
    T, B, W = learner.shape
    A = W if d == CATEGORICAL else W // 2
    act = _actions(d, actions)
    v, vs, adv = _f64(values), _f64(vs), _f64(adv)
    gd = np.empty((T, B, W)) if want_grads else None
    gv = np.empty((T, B)) if want_grads else None
    loss5, R, lp3 = np.empty(5), np.empty((T, B)), np.empty((T, B, 3))
    f = lib().oracle_loss_given_targets
    f.restype = ctypes.c_int
    rc = f(ctypes.c_int(d), ctypes.c_int(T), ctypes.c_int(B), ctypes.c_int(A), _ptr(learner), _ptr(target),
           _ptr(worker), _ptr(cached), _ptr(act), _ptr(v), _ptr(vs), _ptr(adv), ctypes.byref(cfg), ctypes.c_int(n_threads),
           _ptr(gd), _ptr(gv), _ptr(loss5), _ptr(R), _ptr(lp3))
    if rc:
        raise RuntimeError(f"oracle_loss_given_targets failed: {rc}")
    return dict(grad_dist=gd, grad_values=gv, loss5=loss5, ratio=R, logp3=lp3)


def behaviour_logp(dist, target, worker, actions) -> np.ndarray:
    """[T][B][2] fp64: (log pi_worker(a), log pi_target(a)) -- what a caching buffer keeps per step."""
    d = _dist_code(dist)
    target, worker = _f64(target), _f64(worker)
    T, B, W = target.shape
    A = W if d == CATEGORICAL else W // 2
    act = _actions(d, actions)
    out = np.empty((T, B, 2))
    f = lib().oracle_behaviour_logp
    f.restype = ctypes.c_int
    rc = f(ctypes.c_int(d), ctypes.c_int(T), ctypes.c_int(B), ctypes.c_int(A), _ptr(target), _ptr(worker), _ptr(act),
           _ptr(out))
    if rc:
        raise RuntimeError(f"oracle_behaviour_logp failed: {rc}")
    return out


def impact_loss(dist, learner, target, worker, actions, rewards, dones, values, bootstrap, cfg: _Cfg,
                n_threads: int = 1, cached_logp=None) -> Dict[str, np.ndarray]:
    """The whole step on fp64 copies of the inputs.  Returns grads, vs, adv, loss5, ratio, logp3.
    With cached_logp ([T][B][2]) the worker's distribution is not read (None allowed) and the target's
    only for the KL term (None allowed when kl_coeff = 0)."""
    d = _dist_code(dist)
    learner, target, worker, cached = _f64(learner), _opt64(target), _opt64(worker), _opt64(cached_logp)
    T, B, W = learner.shape
    A = W if d == CATEGORICAL else W // 2
    act = _actions(d, actions)
    r, v, bs = _f64(rewards), _f64(values), _f64(bootstrap)
    dn = np.ascontiguousarray(np.asarray(dones, dtype=np.uint8))
    gd, gv = np.empty((T, B, W)), np.empty((T, B))
    vs, adv = np.empty((T, B)), np.empty((T, B))
    loss5, R, lp3 = np.empty(5), np.empty((T, B)), np.empty((T, B, 3))
    f = lib().oracle_impact_loss
    f.restype = ctypes.c_int
    rc = f(ctypes.c_int(d), ctypes.c_int(T), ctypes.c_int(B), ctypes.c_int(A), _ptr(learner), _ptr(target),
           _ptr(worker), _ptr(cached), _ptr(act), _ptr(r), _ptr(dn), _ptr(v), _ptr(bs), ctypes.byref(cfg),
           ctypes.c_int(n_threads), _ptr(gd), _ptr(gv), _ptr(vs), _ptr(adv), _ptr(loss5), _ptr(R), _ptr(lp3))
    if rc:
        raise RuntimeError(f"oracle_impact_loss failed: {rc}")
    out = dict(grad_dist=gd, grad_values=gv, vs=vs, adv=adv, loss5=loss5, ratio=R, logp3=lp3)
    for k, a in out.items():
        if not np.all(np.isfinite(a)):
            raise FloatingPointError(f"oracle produced a non-finite {k}")
    return out


# --- bfloat16 storage -------------------------------------------------------------

def quantize_bf16(x):
    """Round fp32 values to bfloat16 (nearest, ties to even).  Returns (uint16 bits, fp32 values)."""
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    bits = np.empty(x.shape, dtype=np.uint16)
    vals = np.empty(x.shape, dtype=np.float32)
    f = lib().oracle_quantize_bf16
    f.restype = None
    f(_ptr(x), ctypes.c_size_t(x.size), _ptr(bits), _ptr(vals))
    return bits, vals


def max_threads() -> int:
    return lib().oracle_max_threads()
