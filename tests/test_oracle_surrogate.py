"""Pins for the surrogate ratio (Section 3.1) and the epsilon-clip (Section 2.1, Appendix E)."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_two_forms_of_the_clipped_ratio_agree():
    # min(pi_w/pi_t, rho) * pi_theta/pi_w  ==  pi_theta / max(pi_t, pi_w/rho)
    rng = np.random.default_rng(20)
    for _ in range(500):
        a, b, c = rng.normal(size=3) * 2
        rho = rng.uniform(1.0, 4.0)
        assert oracle.ratio(a, b, c, rho) == pytest.approx(oracle.ratio_twin(a, b, c, rho), rel=1e-12)


def test_ratio_bounds_and_limits():
    rng = np.random.default_rng(21)
    for _ in range(300):
        a, b, c = rng.normal(size=3) * 2
        rho = rng.uniform(1.0, 4.0)
        R3 = oracle.ratio(a, b, c, rho)
        R1 = math.exp(a - b)          # pi_theta / pi_target
        R2 = math.exp(a - c)          # pi_theta / pi_worker
        assert R3 <= R1 * (1 + 1e-14)
        assert R3 <= rho * R2 * (1 + 1e-14)
        assert oracle.ratio(a, b, c, math.inf) == pytest.approx(R1, rel=1e-14)
        assert oracle.ratio(a, b, c, 1e300) == pytest.approx(R1, rel=1e-14)
    # exact branch values
    assert oracle.ratio(math.log(0.75), math.log(0.25), math.log(0.75), 2.0) == pytest.approx(2.0, rel=1e-14)
    assert oracle.ratio(math.log(0.75), math.log(0.75), math.log(0.5), 2.0) == pytest.approx(1.0, rel=1e-14)


def test_worker_ratio_of_the_ablation():
    """R_2 = pi_theta / pi_worker (Section 4.1): 1 when learner = worker; equal to the target-clipped
    ratio for every rho_clip >= 1 when target = worker; R_2 = R_1 * pi_target / pi_worker in general."""
    rng = np.random.default_rng(3)
    for _ in range(50):
        lp_l, lp_t, lp_w = rng.normal(size=3) * 2
        assert oracle.ratio_worker(lp_w, lp_w) == 1.0
        for rho in (1.0, 2.0, math.inf):
            assert math.isclose(oracle.ratio_worker(lp_l, lp_w), oracle.ratio(lp_l, lp_w, lp_w, rho), rel_tol=1e-15)
        assert math.isclose(oracle.ratio_worker(lp_l, lp_w), oracle.ratio(lp_l, lp_t, lp_w, math.inf) * math.exp(lp_t - lp_w),
                            rel_tol=1e-13)


def test_ppo_clip_cases():
    eps = 0.2
    assert oracle.surrogate(1.5, 1.0, eps) == pytest.approx(1.2)     # positive advantage, capped
    assert oracle.surrogate(1.5, -1.0, eps) == pytest.approx(-1.5)   # negative advantage, not capped above
    assert oracle.surrogate(0.5, 1.0, eps) == pytest.approx(0.5)
    assert oracle.surrogate(0.5, -1.0, eps) == pytest.approx(-0.8)
    assert oracle.surrogate(1.1, 2.0, eps) == pytest.approx(2.2)
    assert oracle.surrogate(7.0, -3.0, math.inf) == pytest.approx(-21.0)
    assert oracle.surrogate_active(1.5, 1.0, eps) == 0
    assert oracle.surrogate_active(1.5, -1.0, eps) == 1
    assert oracle.surrogate_active(0.5, 1.0, eps) == 1
    assert oracle.surrogate_active(0.5, -1.0, eps) == 0
    assert oracle.surrogate_active(1.1, 1.0, eps) == 1
    assert oracle.surrogate_active(100.0, 1.0, math.inf) == 1
    # the surrogate never exceeds the unclipped objective (pessimistic bound)
    rng = np.random.default_rng(22)
    for _ in range(200):
        R, A = rng.uniform(0, 3), rng.normal()
        assert oracle.surrogate(R, A, eps) <= R * A + 1e-15


def _frac(s):
    return float(Fraction(s))


def test_hand_worked_two_step_example():
    with open(os.path.join(GOLDEN, "worked_example_T2.json")) as f:
        g = json.load(f)
    cfg = oracle.make_config(g["gamma"], g["lambda"], g["rho_bar"], g["c_bar"], g["rho_clip"], g["eps"],
                             g["vf_coeff"], g["ent_coeff"], g["kl_coeff"])
    logit = lambda p: np.log(np.asarray(p, dtype=np.float64))[:, None, :]     # [T, 1, A]
    col = lambda x, dt=np.float64: np.asarray(x, dtype=dt)[:, None]
    out = oracle.impact_loss("categorical", logit(g["learner_probs"]), logit(g["target_probs"]),
                             logit(g["worker_probs"]), col(g["actions"], np.int32), col(g["rewards"]),
                             col(g["dones"], np.uint8), col(g["values"]), np.asarray([g["bootstrap"]]), cfg)
    e = g["expected"]
    np.testing.assert_allclose(out["adv"][:, 0], [_frac(x) for x in e["adv"]], rtol=1e-13)
    np.testing.assert_allclose(out["vs"][:, 0], [_frac(x) for x in e["vs"]], rtol=1e-13)
    np.testing.assert_allclose(out["ratio"][:, 0], [_frac(x) for x in e["ratio"]], rtol=1e-13)
    want_g = np.array([[_frac(x) for x in row] for row in e["grad_logits"]])
    np.testing.assert_allclose(out["grad_dist"][:, 0, :], want_g, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(out["grad_values"][:, 0], [_frac(x) for x in e["grad_values"]], rtol=1e-13)
    assert out["loss5"][1] == pytest.approx(_frac(e["loss_pg"]), rel=1e-13)
    assert out["loss5"][2] == pytest.approx(_frac(e["loss_vf"]), rel=1e-13)
    assert out["loss5"][0] == pytest.approx(_frac(e["loss_total"]), rel=1e-13)
    assert out["loss5"][4] == pytest.approx(math.log(3) / 4, rel=1e-13)


def test_paper_hyperparameters_are_the_workload_defaults():
    import workloads
    with open(os.path.join(GOLDEN, "appendix_b_hyperparameters.json")) as f:
        g = json.load(f)
    for wl, tab in ((workloads.C2, g["discrete"]), (workloads.C4, g["discrete"]),
                    (workloads.C3, g["continuous"]), (workloads.C5, g["continuous"])):
        h = wl.hyper
        assert h.eps == tab["clip_parameter"]
        assert h.ent_coeff == tab["entropy_coeff"]
        assert h.gamma == tab["discount_gamma"]
        assert h.kl_coeff == tab["kl_coeff"]
        assert h.vf_coeff == tab["value_function_coeff"]
        assert h.rho_clip == tab["target_worker_clipping_rho"]
    assert workloads.C2.T == g["discrete"]["sample_batch_size"]
