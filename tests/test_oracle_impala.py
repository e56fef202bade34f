"""IMPALA's objective (Section 2.3: V-trace with learner-over-worker weights; Appendix "IMPALA in Continuous
Environments": an importance-sampled policy gradient) as a special case of the same computation: the learner's
own distribution, held constant, in the target's place, no ratio clipping."""
import math
from dataclasses import replace

import numpy as np
import pytest

import oracle
import workloads


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_learner_as_target_gives_the_importance_sampled_policy_gradient(name):
    wl = replace(workloads.WORKLOADS[name], B=6, num_slots=6, T=9)
    x = workloads.make_trajectories(wl, 6, stream=51)
    gamma, rho_bar = 0.97, 1.3
    cfg = oracle.make_config(gamma=gamma, lam=1.0, rho_bar=rho_bar, c_bar=rho_bar, rho_clip=math.inf, eps=math.inf,
                             vf_coeff=0.5, ent_coeff=0.0, kl_coeff=0.0)
    out = oracle.impact_loss(wl.dist, x["learner"], x["learner"], x["worker"], x["actions"], x["rewards"], x["dones"],
                             x["values"], x["bootstrap"], cfg)
    T, B = wl.T, 6
    M = T * B
    lp = out["logp3"]                                     # learner, target (= learner), worker
    np.testing.assert_allclose(out["ratio"], 1.0, rtol=0, atol=1e-13)      # pi_theta / pi_theta
    # V-trace's own identity for equal truncation levels: the advantage of the policy gradient is
    # rho_t (r_t + gamma_t v_{t+1} - V_t) with v the V-trace target and rho_t = min(rho_bar, pi_theta / pi_worker)
    rho = np.minimum(rho_bar, np.exp(lp[..., 0] - lp[..., 2]))
    V = x["values"].astype(np.float64)
    v_next = np.concatenate([out["vs"][1:], x["bootstrap"].astype(np.float64)[None]], axis=0)
    g_t = gamma * (1.0 - x["dones"].astype(np.float64))
    want_adv = rho * (x["rewards"].astype(np.float64) + g_t * v_next - V)
    np.testing.assert_allclose(out["adv"], want_adv, rtol=1e-12, atol=1e-13)
    # ... and the gradient with respect to the distribution's parameters is -adv / M times that of log pi(a):
    # checked through a finite difference of log pi_theta(a) in one coordinate per step
    cfg_lp = oracle.make_config(gamma=gamma, rho_bar=rho_bar, c_bar=rho_bar, rho_clip=math.inf, eps=math.inf,
                                vf_coeff=0.0, ent_coeff=0.0, kl_coeff=0.0)
    h = 1e-6
    rng = np.random.default_rng(3)
    for _ in range(12):
        t, b, k = rng.integers(T), rng.integers(B), rng.integers(wl.W)
        lo, hi = x["learner"].astype(np.float64).copy(), x["learner"].astype(np.float64).copy()
        lo[t, b, k] -= h
        hi[t, b, k] += h
        args = (x["learner"], x["worker"], x["actions"], x["rewards"], x["dones"], x["values"], x["bootstrap"], cfg_lp)
        dlogp = (oracle.impact_loss(wl.dist, hi, *args)["logp3"][t, b, 0]
                 - oracle.impact_loss(wl.dist, lo, *args)["logp3"][t, b, 0]) / (2 * h)
        assert out["grad_dist"][t, b, k] == pytest.approx(-want_adv[t, b] * dlogp / M, rel=2e-6, abs=1e-9)
