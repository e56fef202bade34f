"""Pins for the oracle's V-trace / V-GAE scan (Section 2.2, Section 3.1)."""
import math

import numpy as np
import pytest

import oracle


def _rand_traj(rng, T, p_done=0.2):
    lpt = rng.normal(size=T) - 1.0
    lpw = rng.normal(size=T) - 1.0
    r = rng.normal(size=T)
    d = (rng.random(T) < p_done).astype(np.uint8)
    v = rng.normal(size=T)
    bs = float(rng.normal())
    return lpt, lpw, r, d, v, bs


@pytest.mark.parametrize("lam", [1.0, 0.995, 0.9])
def test_recurrence_equals_explicit_sums(lam):
    rng = np.random.default_rng(10)
    for T in range(1, 9):
        for trial in range(20):
            lpt, lpw, r, d, v, bs = _rand_traj(rng, T)
            cfg = oracle.make_config(gamma=0.97, lam=lam, rho_bar=rng.uniform(0.5, 2), c_bar=rng.uniform(0.5, 2))
            vs1, adv1 = oracle.vtrace_trajectory(lpt, lpw, r, d, v, bs, cfg)
            vs2, adv2 = oracle.vtrace_trajectory(lpt, lpw, r, d, v, bs, cfg, twin=True)
            np.testing.assert_allclose(vs1, vs2, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(adv1, adv2, rtol=1e-12, atol=1e-13)


def test_on_policy_is_n_step_return():
    # behaviour == target and rho_bar, c_bar >= 1, lambda = 1: the sum telescopes to the discounted return
    rng = np.random.default_rng(11)
    T, gamma = 12, 0.9
    lp = rng.normal(size=T)
    r, v, bs = rng.normal(size=T), rng.normal(size=T), 0.7
    d = np.zeros(T, np.uint8)
    cfg = oracle.make_config(gamma=gamma, lam=1.0, rho_bar=1.0, c_bar=1.5)
    vs, adv = oracle.vtrace_trajectory(lp, lp, r, d, v, bs, cfg)
    for t in range(T):
        want = sum(gamma ** (i - t) * r[i] for i in range(t, T)) + gamma ** (T - t) * bs
        assert vs[t] == pytest.approx(want, rel=1e-12)
        assert adv[t] == pytest.approx(want - v[t], rel=1e-11, abs=1e-13)


def test_constant_reward_geometric_closed_form():
    T, gamma = 30, 0.99
    z = np.zeros(T)
    cfg = oracle.make_config(gamma=gamma, lam=1.0, rho_bar=1.0, c_bar=1.0)
    vs, _ = oracle.vtrace_trajectory(z, z, np.ones(T), np.zeros(T, np.uint8), z, 0.0, cfg)
    for t in range(T):
        assert vs[t] == pytest.approx((1 - gamma ** (T - t)) / (1 - gamma), rel=1e-12)


def test_on_policy_lambda_is_textbook_gae():
    # GAE(lambda): A_t = sum_l (gamma lambda)^l delta_{t+l}, delta = r + gamma V' - V  (Schulman et al.)
    rng = np.random.default_rng(12)
    T, gamma, lam = 9, 0.95, 0.8
    lp = rng.normal(size=T)
    r, v, bs = rng.normal(size=T), rng.normal(size=T), -0.3
    vn = np.append(v[1:], bs)
    delta = r + gamma * vn - v
    cfg = oracle.make_config(gamma=gamma, lam=lam, rho_bar=1.0, c_bar=1.0)
    _, adv = oracle.vtrace_trajectory(lp, lp, r, np.zeros(T, np.uint8), v, bs, cfg)
    for t in range(T):
        want = sum((gamma * lam) ** l * delta[t + l] for l in range(T - t))
        assert adv[t] == pytest.approx(want, rel=1e-12, abs=1e-14)


def test_weights_are_target_over_worker_and_truncated():
    # one step: w = pi_target / pi_worker = 1/2 -> rho = 1/2; the swapped ratio would give min(1, 2) = 1
    cfg = oracle.make_config(gamma=0.5, lam=1.0, rho_bar=1.0, c_bar=1.0)
    vs, adv = oracle.vtrace_trajectory([math.log(0.25)], [math.log(0.5)], [1.0], [0], [2.0], 4.0, cfg)
    assert adv[0] == pytest.approx(0.5 * (1.0 + 0.5 * 4.0 - 2.0), rel=1e-14)
    # w = 3 truncated at rho_bar = 1.25
    cfg = oracle.make_config(gamma=0.5, lam=1.0, rho_bar=1.25, c_bar=1.0)
    vs, adv = oracle.vtrace_trajectory([math.log(0.75)], [math.log(0.25)], [1.0], [0], [2.0], 4.0, cfg)
    assert adv[0] == pytest.approx(1.25 * 1.0, rel=1e-14)
    assert vs[0] == pytest.approx(3.25, rel=1e-14)


def test_c_bar_zero_is_one_step_and_rho_bar_zero_is_identity():
    rng = np.random.default_rng(13)
    T = 7
    lpt, lpw, r, d, v, bs = _rand_traj(rng, T, p_done=0.0)
    cfg = oracle.make_config(gamma=0.9, lam=1.0, rho_bar=1.0, c_bar=0.0)
    vs, adv = oracle.vtrace_trajectory(lpt, lpw, r, d, v, bs, cfg)
    vn = np.append(v[1:], bs)
    rho = np.minimum(1.0, np.exp(lpt - lpw))
    np.testing.assert_allclose(adv, rho * (r + 0.9 * vn - v), rtol=1e-13)
    cfg = oracle.make_config(gamma=0.9, lam=1.0, rho_bar=0.0, c_bar=1.0)
    vs, adv = oracle.vtrace_trajectory(lpt, lpw, r, d, v, bs, cfg)
    np.testing.assert_array_equal(adv, np.zeros(T))
    np.testing.assert_array_equal(vs, v)


def test_c_and_rho_truncations_are_separate():
    # two steps, w = 4 everywhere: rho_bar = 2 scales the TD errors, c_bar = 3 scales the carried trace
    cfg = oracle.make_config(gamma=1.0, lam=1.0, rho_bar=2.0, c_bar=3.0)
    lw = math.log(4.0)
    vs, adv = oracle.vtrace_trajectory([lw, lw], [0.0, 0.0], [1.0, 1.0], [0, 0], [0.0, 0.0], 0.0, cfg)
    assert adv[1] == pytest.approx(2.0)               # rho * (1 + 0 - 0)
    assert adv[0] == pytest.approx(2.0 + 3.0 * 2.0)   # delta_0 + c_0 * adv_1


def test_done_cuts_everything_after_it():
    rng = np.random.default_rng(14)
    T = 10
    lpt, lpw, r, d, v, bs = _rand_traj(rng, T, p_done=0.0)
    d[4] = 1
    cfg = oracle.make_config(gamma=0.97, lam=0.95, rho_bar=1.0, c_bar=1.0)
    vs_a, adv_a = oracle.vtrace_trajectory(lpt, lpw, r, d, v, bs, cfg)
    # change everything after the terminal transition, including V at step 5 and the bootstrap
    lpt2, lpw2, r2, v2 = lpt.copy(), lpw.copy(), r.copy(), v.copy()
    lpt2[5:] += 1.0; lpw2[5:] -= 0.5; r2[5:] += 3.0; v2[5:] -= 2.0
    vs_b, adv_b = oracle.vtrace_trajectory(lpt2, lpw2, r2, d, v2, bs + 5.0, cfg)
    np.testing.assert_array_equal(vs_a[:5], vs_b[:5])
    np.testing.assert_array_equal(adv_a[:5], adv_b[:5])
    # at the terminal step the TD error has no bootstrap
    rho4 = min(1.0, math.exp(lpt[4] - lpw[4]))
    assert adv_a[4] == pytest.approx(rho4 * (r[4] - v[4]), rel=1e-13)


def test_batch_wrapper_matches_per_trajectory_calls():
    import workloads
    wl = workloads.C1.with_batch(5)
    x = workloads.make_batch(wl, stream=3)
    cfg = oracle.config_from_hyper(wl.hyper)
    vs, adv = oracle.vtrace_targets("categorical", x["target"], x["worker"], x["actions"], x["rewards"],
                                    x["dones"], x["values"], x["bootstrap"], cfg, n_threads=2)
    vs2, adv2 = oracle.vtrace_targets("categorical", x["target"], x["worker"], x["actions"], x["rewards"],
                                      x["dones"], x["values"], x["bootstrap"], cfg, twin=True)
    np.testing.assert_allclose(vs, vs2, rtol=1e-12, atol=1e-13)
    for b in range(5):
        lpt = [oracle.cat_logp(x["target"][t, b], x["actions"][t, b]) for t in range(wl.T)]
        lpw = [oracle.cat_logp(x["worker"][t, b], x["actions"][t, b]) for t in range(wl.T)]
        v1, a1 = oracle.vtrace_trajectory(lpt, lpw, x["rewards"][:, b], x["dones"][:, b], x["values"][:, b],
                                          float(x["bootstrap"][b]), cfg)
        np.testing.assert_array_equal(vs[:, b], v1)
        np.testing.assert_array_equal(adv[:, b], a1)
