"""Pins for the oracle's cached-log-probability path: the V-trace weights and the surrogate's denominator
depend on the buffer's data alone (Sections 3.1 and 3.2), so log pi_worker(a) and log pi_target(a) can be
stored per step instead of the worker's distribution."""
import math
from dataclasses import replace as shape_workload

import numpy as np
import pytest
from scipy.special import log_softmax
from scipy.stats import norm

import oracle
import workloads


def _small(wl, n, **kw):
    wl = shape_workload(wl, B=n, num_slots=n, **kw)
    return wl, workloads.make_trajectories(wl, n, stream=31)


def test_behaviour_logp_against_library_routines():
    wl, x = _small(workloads.C2, 5, T=6)
    got = oracle.behaviour_logp(wl.dist, x["target"], x["worker"], x["actions"])
    a = x["actions"][..., None].astype(np.int64)
    want_w = np.take_along_axis(log_softmax(x["worker"].astype(np.float64), axis=-1), a, -1)[..., 0]
    want_t = np.take_along_axis(log_softmax(x["target"].astype(np.float64), axis=-1), a, -1)[..., 0]
    np.testing.assert_allclose(got[..., 0], want_w, rtol=0, atol=1e-13)      # column 0: the worker
    np.testing.assert_allclose(got[..., 1], want_t, rtol=0, atol=1e-13)      # column 1: the target
    wl, x = _small(workloads.C3, 4, T=5)
    D = wl.A
    got = oracle.behaviour_logp(wl.dist, x["target"], x["worker"], x["actions"])
    for col, p in ((0, x["worker"]), (1, x["target"])):
        p = p.astype(np.float64)
        want = norm.logpdf(x["actions"].astype(np.float64), loc=p[..., :D], scale=np.exp(p[..., D:])).sum(-1)
        np.testing.assert_allclose(got[..., col], want, rtol=1e-13, atol=1e-12)


@pytest.mark.parametrize("name", ["C2", "C3"])
@pytest.mark.parametrize("ratio_mode", [0, 1])
def test_cached_log_probabilities_reproduce_the_full_computation(name, ratio_mode):
    wl, x = _small(workloads.WORKLOADS[name], 7, T=11)
    h = wl.hyper
    cfg = oracle.make_config(h.gamma, h.lam, h.rho_bar, h.c_bar, h.rho_clip, h.eps, h.vf_coeff, h.ent_coeff, 0.7,
                             ratio_mode=ratio_mode)
    args = (x["actions"], x["rewards"], x["dones"], x["values"], x["bootstrap"], cfg)
    full = oracle.impact_loss(wl.dist, x["learner"], x["target"], x["worker"], *args)
    lp = oracle.behaviour_logp(wl.dist, x["target"], x["worker"], x["actions"])
    cached = oracle.impact_loss(wl.dist, x["learner"], x["target"], None, *args, cached_logp=lp)
    for k in ("grad_dist", "grad_values", "vs", "adv", "loss5", "ratio"):
        np.testing.assert_allclose(cached[k], full[k], rtol=1e-13, atol=1e-15, err_msg=k)
    # without the target's distribution: the same with the KL term switched off, and KL reported as 0
    cfg0 = oracle.make_config(h.gamma, h.lam, h.rho_bar, h.c_bar, h.rho_clip, h.eps, h.vf_coeff, h.ent_coeff, 0.0,
                              ratio_mode=ratio_mode)
    args0 = args[:-1] + (cfg0,)
    full0 = oracle.impact_loss(wl.dist, x["learner"], x["target"], x["worker"], *args0)
    bare = oracle.impact_loss(wl.dist, x["learner"], None, None, *args0, cached_logp=lp)
    for k in ("grad_dist", "grad_values", "vs", "adv", "ratio"):
        np.testing.assert_allclose(bare[k], full0[k], rtol=1e-13, atol=1e-15, err_msg=k)
    np.testing.assert_allclose(bare["loss5"][:4], full0["loss5"][:4], rtol=1e-13)
    assert bare["loss5"][4] == 0.0
    with pytest.raises(RuntimeError):
        oracle.impact_loss(wl.dist, x["learner"], None, None, *args, cached_logp=lp)     # KL wanted, no target


def test_which_column_is_which():
    """One step, closed form: adv = min(rho_bar, pi_t/pi_w) (r + gamma boot - V) and
    R = pi_theta / max(pi_t, pi_w / rho_clip), with the worker in column 0 and the target in column 1."""
    learner = np.log(np.array([[[0.5, 0.3, 0.2]]]))
    lw, lt = math.log(0.4), math.log(0.1)             # target four times less likely: w = 1/4
    cached = np.array([[[lw, lt]]])
    cfg = oracle.make_config(gamma=0.9, rho_bar=1.0, c_bar=1.0, rho_clip=2.0, eps=math.inf, vf_coeff=1.0,
                             ent_coeff=0.0, kl_coeff=0.0)
    out = oracle.impact_loss("categorical", learner, None, None, np.array([[0]], np.int32), np.array([[1.0]]),
                             np.array([[0]], np.uint8), np.array([[0.5]]), np.array([2.0]), cfg, cached_logp=cached)
    assert out["adv"][0, 0] == pytest.approx(0.25 * (1.0 + 0.9 * 2.0 - 0.5), rel=1e-14)
    assert out["ratio"][0, 0] == pytest.approx(0.5 / max(0.1, 0.4 / 2.0), rel=1e-14)
    swapped = oracle.impact_loss("categorical", learner, None, None, np.array([[0]], np.int32), np.array([[1.0]]),
                                 np.array([[0]], np.uint8), np.array([[0.5]]), np.array([2.0]), cfg,
                                 cached_logp=cached[..., ::-1].copy())
    assert swapped["adv"][0, 0] == pytest.approx(1.0 * (1.0 + 0.9 * 2.0 - 0.5), rel=1e-14)   # w = 4, truncated at 1
