"""Pins for the oracle's analytic gradients (Algorithm 1) and their invariants."""
import math

import numpy as np
import pytest
from scipy import special

import oracle
import workloads


def _tiny(dist, seed, T=4, B=2, A=4):
    base = workloads.C1 if dist == "categorical" else workloads.C3
    wl = workloads.Workload(**{**base.__dict__, "T": T, "B": B, "A": A})
    x = workloads.make_batch(wl, stream=seed)
    return {k: v.astype(np.float64) if v.dtype == np.float32 else v for k, v in x.items()}


def _away_from_kinks(out, eps):
    R = out["ratio"]
    return np.all(np.abs(R - (1 + eps)) > 1e-3) and np.all(np.abs(R - (1 - eps)) > 1e-3)


CFGS = [
    dict(gamma=0.99, lam=1.0, rho_bar=1.0, c_bar=1.0, rho_clip=2.0, eps=0.2, vf_coeff=1.0, ent_coeff=0.01, kl_coeff=0.0),
    dict(gamma=0.95, lam=0.9, rho_bar=1.3, c_bar=0.8, rho_clip=math.inf, eps=0.4, vf_coeff=0.5, ent_coeff=0.05, kl_coeff=1.0),
    dict(gamma=0.9, lam=0.995, rho_bar=1.0, c_bar=1.0, rho_clip=1.5, eps=math.inf, vf_coeff=2.0, ent_coeff=0.0, kl_coeff=0.3),
    # the ablation's ratio pi_theta / pi_worker
    dict(gamma=0.99, lam=1.0, rho_bar=1.0, c_bar=1.0, rho_clip=2.0, eps=0.3, vf_coeff=1.0, ent_coeff=0.01, kl_coeff=0.5, ratio_mode=1),
]


def test_worker_ratio_mode_equals_the_method_when_target_is_the_worker():
    """With pi_target = pi_worker the target-clipped ratio is pi_theta / pi_worker for every rho_clip >= 1
    and all importance weights are 1: the two modes must give the same step, output by output."""
    for dist in ("categorical", "gaussian"):
        x = _tiny(dist, 5)
        outs = []
        for mode, rho in ((0, 2.0), (0, 1.0), (1, 2.0)):
            cfg = oracle.make_config(gamma=0.97, lam=0.9, rho_clip=rho, eps=0.25, kl_coeff=0.4, ratio_mode=mode)
            outs.append(oracle.impact_loss(dist, x["learner"], x["worker"], x["worker"], x["actions"], x["rewards"],
                                           x["dones"], x["values"], x["bootstrap"], cfg))
        for o in outs[1:]:
            for k in ("loss5", "grad_dist", "grad_values", "vs", "adv", "ratio"):
                np.testing.assert_allclose(o[k], outs[0][k], rtol=1e-13, atol=1e-15, err_msg=f"{dist} {k}")


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
@pytest.mark.parametrize("ci", range(len(CFGS)))
def test_central_differences_on_learner_parameters(dist, ci):
    cfg = oracle.make_config(**CFGS[ci])
    eps = CFGS[ci]["eps"]
    checked = 0
    for seed in range(40):
        x = _tiny(dist, seed)
        args = lambda learner: (dist, learner, x["target"], x["worker"], x["actions"], x["rewards"], x["dones"],
                                x["values"], x["bootstrap"], cfg)
        out = oracle.impact_loss(*args(x["learner"]))
        if math.isfinite(eps) and not _away_from_kinks(out, eps):
            continue
        h = 1e-6
        g = out["grad_dist"]
        fd = np.zeros_like(g)
        for idx in np.ndindex(*g.shape):
            lp, lm = x["learner"].copy(), x["learner"].copy()
            lp[idx] += h; lm[idx] -= h
            fd[idx] = (oracle.impact_loss(*args(lp))["loss5"][0] - oracle.impact_loss(*args(lm))["loss5"][0]) / (2 * h)
        np.testing.assert_allclose(g, fd, rtol=2e-6, atol=2e-8)
        checked += 1
        if checked >= 4:
            break
    assert checked >= 3


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
def test_central_differences_on_values_with_frozen_targets(dist):
    # Algorithm 1 differentiates V_w only: targets and advantages are constants
    cfg = oracle.make_config(**CFGS[1])
    x = _tiny(dist, 7)
    out = oracle.impact_loss(dist, x["learner"], x["target"], x["worker"], x["actions"], x["rewards"], x["dones"],
                             x["values"], x["bootstrap"], cfg)
    f = lambda v: oracle.loss_given_targets(dist, x["learner"], x["target"], x["worker"], x["actions"], v,
                                            out["vs"], out["adv"], cfg, want_grads=False)["loss5"][0]
    h = 1e-6
    for idx in np.ndindex(*x["values"].shape):
        vp, vm = x["values"].copy(), x["values"].copy()
        vp[idx] += h; vm[idx] -= h
        assert out["grad_values"][idx] == pytest.approx((f(vp) - f(vm)) / (2 * h), rel=1e-6, abs=1e-9)
    # the frozen-target loss at the unperturbed point is the full loss
    np.testing.assert_allclose(oracle.loss_given_targets(dist, x["learner"], x["target"], x["worker"], x["actions"],
                                                         x["values"], out["vs"], out["adv"], cfg)["loss5"],
                               out["loss5"], rtol=1e-14)


def test_logit_gradients_sum_to_zero_and_value_gradient_sum():
    wl = workloads.C2.with_batch(16)
    x = workloads.make_batch(wl, stream=1)
    for kw in (dict(ent_coeff=0.0, kl_coeff=0.0), dict(ent_coeff=0.3, kl_coeff=0.0),
               dict(ent_coeff=0.0, kl_coeff=0.7), dict(ent_coeff=0.01, kl_coeff=0.5)):
        cfg = oracle.make_config(gamma=0.99, eps=0.3, vf_coeff=0.5, **kw)
        out = oracle.impact_loss("categorical", x["learner"], x["target"], x["worker"], x["actions"], x["rewards"],
                                 x["dones"], x["values"], x["bootstrap"], cfg)
        M = wl.T * 16
        np.testing.assert_allclose(out["grad_dist"].sum(axis=2) * M, 0.0, atol=1e-13)
        want = 0.5 * np.mean(x["values"].astype(np.float64) - out["vs"])
        assert out["grad_values"].sum() == pytest.approx(want, rel=1e-12)


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
def test_clipped_steps_have_exactly_zero_policy_gradient(dist):
    wl = (workloads.C4 if dist == "categorical" else workloads.C5).with_batch(24)
    x = workloads.make_batch(wl, stream=2)
    eps = 0.3
    cfg = oracle.make_config(gamma=0.99, eps=eps, ent_coeff=0.0, kl_coeff=0.0)
    out = oracle.impact_loss(dist, x["learner"], x["target"], x["worker"], x["actions"], x["rewards"], x["dones"],
                             x["values"], x["bootstrap"], cfg)
    R, A = out["ratio"], out["adv"]
    clipped = ((A > 0) & (R > 1 + eps)) | ((A < 0) & (R < 1 - eps))
    assert clipped.sum() > 10 and (~clipped).sum() > 50      # both branches exercised
    g = out["grad_dist"]
    assert np.all(g[clipped] == 0.0)
    live = ~clipped & (A != 0)
    assert np.all(np.abs(g[live]).max(axis=1) > 0)


def test_learner_equal_target_is_vanilla_policy_gradient():
    # pi_theta == pi_target and beta = 0: R == 1, nothing clips, grad = -A (1[k=a] - p_k) / M
    wl = workloads.C2.with_batch(8)
    x = workloads.make_batch(wl, stream=4)
    cfg = oracle.make_config(gamma=0.99, rho_clip=math.inf, eps=0.3, ent_coeff=0.0, kl_coeff=0.0)
    out = oracle.impact_loss("categorical", x["target"], x["target"], x["worker"], x["actions"], x["rewards"],
                             x["dones"], x["values"], x["bootstrap"], cfg)
    np.testing.assert_allclose(out["ratio"], 1.0, rtol=1e-14)
    p = special.softmax(x["target"].astype(np.float64), axis=2)
    onehot = np.eye(wl.A)[x["actions"]]
    want = -out["adv"][:, :, None] * (onehot - p) / (wl.T * 8)
    np.testing.assert_allclose(out["grad_dist"], want, rtol=1e-11, atol=1e-16)
    assert out["loss5"][4] == pytest.approx(0.0, abs=1e-15)      # KL(target || learner) = 0


def test_eps_infinite_gives_the_unclipped_gradient_of_algorithm_1():
    # grad wrt logp_theta(a) is -A * pi_theta / max(pi_target, beta pi_worker) / M for every step
    wl = workloads.C3.with_batch(6)
    x = workloads.make_batch(wl, stream=5)
    cfg = oracle.make_config(gamma=0.995, rho_clip=2.0, eps=math.inf, ent_coeff=0.0, kl_coeff=0.0)
    out = oracle.impact_loss("gaussian", x["learner"], x["target"], x["worker"], x["actions"], x["rewards"],
                             x["dones"], x["values"], x["bootstrap"], cfg)
    D = wl.A
    mu, sig = x["learner"][:, :, :D].astype(np.float64), np.exp(x["learner"][:, :, D:].astype(np.float64))
    act = x["actions"].astype(np.float64)
    g = -out["adv"] * out["ratio"] / (wl.T * 6)
    np.testing.assert_allclose(out["grad_dist"][:, :, :D], g[:, :, None] * (act - mu) / sig ** 2, rtol=1e-11)
    np.testing.assert_allclose(out["grad_dist"][:, :, D:], g[:, :, None] * (((act - mu) / sig) ** 2 - 1), rtol=1e-11,
                               atol=1e-16)
    assert out["loss5"][1] == pytest.approx(-np.mean(out["ratio"] * out["adv"]), rel=1e-12)


def test_threads_do_not_change_results():
    wl = workloads.C3.with_batch(33)
    x = workloads.make_batch(wl, stream=6)
    cfg = oracle.config_from_hyper(wl.hyper)
    a = oracle.impact_loss("gaussian", x["learner"], x["target"], x["worker"], x["actions"], x["rewards"], x["dones"],
                           x["values"], x["bootstrap"], cfg, n_threads=1)
    b = oracle.impact_loss("gaussian", x["learner"], x["target"], x["worker"], x["actions"], x["rewards"], x["dones"],
                           x["values"], x["bootstrap"], cfg, n_threads=4)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
