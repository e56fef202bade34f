"""Pins for the oracle's per-step policy functions (log-prob, entropy, KL)."""
import math

import numpy as np
import pytest
from scipy import integrate, special, stats

import oracle


def test_uniform_logits_closed_form():
    for A in (2, 6, 18):
        z = np.full(A, 0.37)
        assert oracle.cat_logp(z, A - 1) == pytest.approx(-math.log(A), abs=1e-14)
        assert oracle.cat_entropy(z) == pytest.approx(math.log(A), abs=1e-14)


def test_shift_invariance_and_large_logits():
    rng = np.random.default_rng(1)
    z = rng.normal(size=18) * 3
    for c in (-700.0, 5.0, 900.0):   # naive exp would overflow / underflow
        assert oracle.cat_logp(z + c, 3) == pytest.approx(oracle.cat_logp(z, 3), abs=1e-10)
        assert oracle.cat_entropy(z + c) == pytest.approx(oracle.cat_entropy(z), abs=1e-10)


def test_categorical_against_scipy():
    rng = np.random.default_rng(2)
    for A in (2, 6, 18, 33):
        z, zt = rng.normal(size=A) * 2, rng.normal(size=A) * 2
        assert oracle.cat_logsumexp(z) == pytest.approx(special.logsumexp(z), rel=1e-14)
        lsm = special.log_softmax(z)
        for a in range(A):
            assert oracle.cat_logp(z, a) == pytest.approx(lsm[a], abs=1e-13)
        p, pt = special.softmax(z), special.softmax(zt)
        assert oracle.cat_entropy(z) == pytest.approx(stats.entropy(p), rel=1e-12)
        # scipy.stats.entropy(pk, qk) = KL(pk || qk): the target comes first
        assert oracle.cat_kl(zt, z) == pytest.approx(stats.entropy(pt, p), rel=1e-11)
        assert oracle.cat_kl(z, z) == pytest.approx(0.0, abs=1e-15)


def test_gaussian_against_scipy():
    rng = np.random.default_rng(3)
    for D in (1, 6, 17):
        mu, ls = rng.normal(size=D), rng.uniform(-2, 0.5, size=D)
        act = rng.normal(size=D)
        want = stats.norm.logpdf(act, loc=mu, scale=np.exp(ls)).sum()
        assert oracle.gauss_logp(np.concatenate([mu, ls]), act) == pytest.approx(want, rel=1e-13)
        want_h = stats.norm.entropy(loc=mu, scale=np.exp(ls)).sum()
        assert oracle.gauss_entropy(np.concatenate([mu, ls])) == pytest.approx(want_h, rel=1e-13)


def test_gaussian_kl_direction_by_quadrature():
    # KL(p_target || p_theta) = int p_target (log p_target - log p_theta), one dimension, asymmetric case
    mt, st, ml, sl = 0.3, 0.5, -0.4, 1.3
    f = lambda x: stats.norm.pdf(x, mt, st) * (stats.norm.logpdf(x, mt, st) - stats.norm.logpdf(x, ml, sl))
    want, _ = integrate.quad(f, -12, 12, epsabs=1e-13, epsrel=1e-13)
    got = oracle.gauss_kl([mt, math.log(st)], [ml, math.log(sl)])
    assert got == pytest.approx(want, rel=1e-9)
    rev = oracle.gauss_kl([ml, math.log(sl)], [mt, math.log(st)])
    assert abs(rev - want) > 0.1      # the other direction is a different number
    p = [0.2, -1.0, 0.4, 0.1]
    assert oracle.gauss_kl(p, p) == pytest.approx(0.0, abs=1e-15)
    # additivity over dimensions
    a = oracle.gauss_kl([mt, math.log(st)], [ml, math.log(sl)])
    b = oracle.gauss_kl([1.0, 0.2], [0.5, -0.3])
    both = oracle.gauss_kl([mt, 1.0, math.log(st), 0.2], [ml, 0.5, math.log(sl), -0.3])
    assert both == pytest.approx(a + b, rel=1e-13)
