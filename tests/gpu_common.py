"""Helpers shared by the GPU parity tests: run the HIP path through the binding, run the
oracle on the same arrays, compare with the stated tolerance."""
from __future__ import annotations

import math
import os
import sys
from dataclasses import replace

import numpy as np

import oracle
import workloads
from oracle.buffer import bf16_bits_to_f32

ATOL, RTOL = 1e-6, 1e-5       # fp32 results against the fp64 oracle: |x - y| <= ATOL + RTOL |y|


def say(msg: str) -> None:
    """Name the case before its GPU step: on stdout, and (if IMPACT_TEST_PROGRESS_LOG names a file) in a
    file that survives output capture."""
    print(msg, flush=True)
    sys.stdout.flush()
    path = os.environ.get("IMPACT_TEST_PROGRESS_LOG")
    if path:
        try:
            with open(path, "a") as f:
                f.write(msg + "\n")
        except OSError:
            pass


def to_device(x, torch, device="cuda"):
    return {k: torch.from_numpy(np.ascontiguousarray(v)).to(device) for k, v in x.items()}


def shape_workload(base: workloads.Workload, **kw) -> workloads.Workload:
    return replace(base, **kw)


def oracle_inputs(x, storage: str):
    """What the oracle consumes: the same arrays, the buffer-resident float fields first rounded
    to the storage dtype (by the oracle's own rounding) and then widened exactly."""
    if storage == "f32":
        return x
    y = dict(x)
    for k in ("worker", "target", "rewards"):
        y[k] = oracle.quantize_bf16(x[k])[1]
    if x["actions"].dtype != np.int32:
        y["actions"] = oracle.quantize_bf16(x["actions"])[1]
    return y


def as_passed_to_c(h):
    """The hyper-parameters as the C ABI receives them: fp32 values.  The oracle is given exactly
    these (widened), so that both sides start from the same numbers."""
    f = lambda v: float(np.float32(v))
    return replace(h, gamma=f(h.gamma), lam=f(h.lam), rho_bar=f(h.rho_bar), c_bar=f(h.c_bar), rho_clip=f(h.rho_clip),
                   eps=f(h.eps), vf_coeff=f(h.vf_coeff), ent_coeff=f(h.ent_coeff), kl_coeff=f(h.kl_coeff))


def cached_oracle_inputs(x, xi, wl, cached):
    """What a buffer that caches log-probabilities holds: log pi_worker(a), log pi_target(a) from the fp32
    distributions as handed over and the action as stored; no worker distribution; the target's (rounded
    to the storage dtype) only if it is kept for the KL term.  cached: None, "with_target" or "no_target"."""
    if cached is None:
        return xi
    y = dict(xi)
    y["logp"] = oracle.behaviour_logp(wl.dist, x["target"], x["worker"], xi["actions"])
    y["worker"] = None
    if cached == "no_target":
        y["target"] = None
    return y


def run_oracle(wl, x, hyper=None, n_threads=8, cached=None):
    h = as_passed_to_c(wl.hyper if hyper is None else hyper)
    cfg = oracle.config_from_hyper(h)
    xi = cached_oracle_inputs(x, oracle_inputs(x, wl.storage), wl, cached)
    return oracle.impact_loss(wl.dist, xi["learner"], xi["target"], xi["worker"], xi["actions"], xi["rewards"],
                              xi["dones"], xi["values"], xi["bootstrap"], cfg, n_threads=n_threads,
                              cached_logp=xi.get("logp")), xi, cfg


def max_violation(got, want, scale=1.0):
    got = np.asarray(got, np.float64) * scale
    want = np.asarray(want, np.float64) * scale
    err = np.abs(got - want)
    return float(np.max(err / (ATOL + RTOL * np.abs(want)))) if err.size else 0.0


def check_against_oracle(wl, x, got, hyper=None, label="", cached=None):
    """got: dict of numpy arrays from the GPU (grad_dist, grad_values, vs, adv, loss5)."""
    h = as_passed_to_c(wl.hyper if hyper is None else hyper)
    want, xi, cfg = run_oracle(wl, x, h, cached=cached)
    M = wl.T * x["learner"].shape[1]
    report = {}
    for k in ("vs", "adv"):
        if k in got:
            report[k] = max_violation(got[k], want[k])
    report["loss5"] = max_violation(got["loss5"], want["loss5"])
    # gradients carry a 1/(T*B) factor: compare them rescaled, so that the absolute term stays meaningful
    report["grad_values"] = max_violation(got["grad_values"], want["grad_values"], M)

    gd_got, gd_want = got["grad_dist"].astype(np.float64) * M, want["grad_dist"] * M
    viol = np.abs(gd_got - gd_want) / (ATOL + RTOL * np.abs(gd_want))
    # The min/clip of the surrogate makes the policy gradient discontinuous where R = 1 +- eps.
    # A step whose fp64 ratio lies within rounding distance of such a kink may legitimately fall on
    # either side in fp32: there the GPU value must match one of the two branches.
    if math.isfinite(h.eps):
        R = want["ratio"]
        near = (np.abs(R - (1 + h.eps)) <= 2e-5 * (1 + h.eps)) | (np.abs(R - (1 - h.eps)) <= 2e-5)
        if near.any():
            kw = dict(dist=wl.dist, learner=xi["learner"], target=xi["target"], worker=xi["worker"],
                      actions=xi["actions"], values=xi["values"], vs=want["vs"], cached_logp=xi.get("logp"))
            open_cfg = oracle.make_config(h.gamma, h.lam, h.rho_bar, h.c_bar, h.rho_clip, math.inf, h.vf_coeff,
                                          h.ent_coeff, h.kl_coeff, getattr(h, "ratio_mode", 0))
            g_on = oracle.loss_given_targets(adv=want["adv"], cfg=open_cfg, **kw)["grad_dist"] * M
            g_off = oracle.loss_given_targets(adv=np.zeros_like(want["adv"]), cfg=cfg, **kw)["grad_dist"] * M
            for g_alt in (g_on, g_off):
                alt = np.abs(gd_got - g_alt) / (ATOL + RTOL * np.abs(g_alt))
                viol[near] = np.minimum(viol[near], alt[near])
            report["near_kink_steps"] = int(near.sum())
    report["grad_dist"] = float(viol.max())
    if "fractions" in got:
        # shares of clipped steps (Appendix E's min/clip: no policy gradient) and of truncated importance weights
        # (Section 2.2), counted from the oracle's ratio, advantages and log-probabilities; a step whose ratio or
        # weight lies within rounding of its threshold may be counted either way
        R, adv, lp = np.asarray(want["ratio"]), np.asarray(want["adv"]), np.asarray(want["logp3"])
        w = np.exp(lp[..., 1] - lp[..., 2])
        if math.isfinite(h.eps):
            clipped = ((adv > 0) & (R > 1 + h.eps)) | ((adv < 0) & (R < 1 - h.eps))
            unsure_c = int(((np.abs(R - (1 + h.eps)) <= 2e-5 * (1 + h.eps)) | (np.abs(R - (1 - h.eps)) <= 2e-5) | (np.abs(adv) <= 1e-12)).sum())
        else:
            clipped, unsure_c = np.zeros_like(R, bool), 0
        truncated = w > h.rho_bar
        unsure_t = int((np.abs(w - h.rho_bar) <= 1e-6 * max(h.rho_bar, 1e-30)).sum())
        for name, count, unsure, value in (("clipped", int(clipped.sum()), unsure_c, float(got["fractions"][0])),
                                           ("truncated", int(truncated.sum()), unsure_t, float(got["fractions"][1]))):
            lo, hi = (count - unsure) / M, (count + unsure) / M
            report[name] = value
            assert lo * (1 - 1e-6) - 1e-9 <= value <= hi * (1 + 1e-6) + 1e-9, f"{label}: fraction {name} = {value}, oracle counts {count} +- {unsure} of {M}"
    say(f"    parity {label}: " + ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}"
                                              for k, v in report.items()))
    for k in ("vs", "adv", "loss5", "grad_values", "grad_dist"):
        if k in report:
            assert report[k] <= 1.0, f"{label}: {k} exceeds tolerance by factor {report[k]:.3g}"
    for k in ("grad_dist", "grad_values", "loss5"):
        assert np.all(np.isfinite(got[k])), f"{label}: non-finite {k}"
    return want


def gpu_loss(torch, binding, wl, x, hyper=None, flags=0, want_targets=True):
    """Time-major fp32 batch through impact_loss_fwd_bwd; returns numpy outputs."""
    h = wl.hyper if hyper is None else hyper
    d = to_device(x, torch)
    T, Bn, W = x["learner"].shape
    out = binding.alloc_loss_out(T, Bn, W, want_targets=want_targets)
    cfg = binding.config_from_hyper(h, flags)
    binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg, out=out)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def wide_range_inputs(wl, x, seed):
    """The batch with peaked and nearly flat policies: categorical logits scaled to a magnitude of up to 40;
    Gaussian standard deviations from about e^-4 to e^1.5, one offset per step and dimension moving the three
    policies' log-sigma together and scaling the distances between their means with it (so that they stay as
    close, in standard deviations, as the workload made them), actions out to four standard deviations."""
    x = dict(x)
    rng = np.random.default_rng(seed)
    if wl.dist == "categorical":
        for k, scale in (("learner", 10.0), ("target", 10.0), ("worker", 8.0)):
            x[k] = (x[k] * scale).astype(np.float32)
        return x
    D = wl.A
    u = rng.uniform(-2.5, 1.0, size=x["learner"][..., D:].shape)
    centre = x["learner"][..., :D].astype(np.float64) * 3.0
    for k in ("target", "worker", "learner"):
        p = x[k].astype(np.float64)
        p[..., :D] = centre + (p[..., :D] - x["learner"][..., :D]) * np.exp(u)
        p[..., D:] += u
        x[k] = p.astype(np.float32)
    mu, sigma = x["worker"][..., :D].astype(np.float64), np.exp(x["worker"][..., D:].astype(np.float64))
    x["actions"] = (mu + sigma * rng.uniform(-4.0, 4.0, size=mu.shape)).astype(np.float32)
    return x
