"""PPO with generalised advantage estimation (Section 2.1's clipped surrogate; the on-policy baseline of the
evaluation) as a special case of the same computation: the worker's distribution in the target's place makes
every importance weight of the scan one, so the advantages are GAE(lambda)'s, and the ratio pi_theta / pi_worker."""
from dataclasses import replace

import numpy as np
import pytest

import oracle
import workloads


def gae_by_definition(r, V, boot, dones, gamma, lam):
    """A_t = sum_l (prod_{i<l} gamma_i lam) delta_{t+l} with delta_t = r_t + gamma_t V_{t+1} - V_t and gamma_t = 0 at
    an episode's end: the double sum, written out."""
    T, B = r.shape
    g = gamma * (1.0 - dones)
    Vn = np.concatenate([V[1:], boot[None]], axis=0)
    delta = r + g * Vn - V
    A = np.zeros((T, B))
    for t in range(T):
        w = np.ones(B)
        for l in range(t, T):
            A[t] += w * delta[l]
            w = w * g[l] * lam
    return A


@pytest.mark.parametrize("name", ["C2", "C3"])
@pytest.mark.parametrize("lam", [1.0, 0.95])
def test_worker_as_target_gives_ppo_with_gae(name, lam):
    wl = replace(workloads.WORKLOADS[name], B=5, num_slots=5, T=11)
    x = workloads.make_trajectories(wl, 5, stream=77)
    x["dones"][4, 1] = 1
    x["dones"][10, 3] = 1
    gamma, eps, vf_coeff = 0.98, 0.25, 0.5
    cfg = oracle.make_config(gamma=gamma, lam=lam, rho_bar=1.0, c_bar=1.0, rho_clip=2.0, eps=eps,
                             vf_coeff=vf_coeff, ent_coeff=0.0, kl_coeff=0.0)
    out = oracle.impact_loss(wl.dist, x["learner"], x["worker"], x["worker"], x["actions"], x["rewards"], x["dones"],
                             x["values"], x["bootstrap"], cfg)
    f64 = lambda k: x[k].astype(np.float64)
    A = gae_by_definition(f64("rewards"), f64("values"), f64("bootstrap"), f64("dones"), gamma, lam)
    np.testing.assert_allclose(out["adv"], A, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["vs"], f64("values") + A, rtol=1e-12, atol=1e-12)     # the lambda-return
    lp = out["logp3"]
    r = np.exp(lp[..., 0] - lp[..., 2])                                                  # pi_theta / pi_worker
    np.testing.assert_allclose(out["ratio"], r, rtol=1e-12)
    s = np.minimum(r * A, np.clip(r, 1.0 - eps, 1.0 + eps) * A)
    assert out["loss5"][1] == pytest.approx(-s.mean(), rel=1e-12, abs=1e-14)
    assert out["loss5"][2] == pytest.approx(0.5 * (A ** 2).mean(), rel=1e-12)             # (V - (V + A))^2 / 2
    assert out["loss5"][0] == pytest.approx(-s.mean() + vf_coeff * 0.5 * (A ** 2).mean(), rel=1e-12, abs=1e-14)
    np.testing.assert_allclose(out["grad_values"], vf_coeff * (-A) / A.size, rtol=1e-10, atol=1e-15)
