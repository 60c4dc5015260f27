"""The paper's latency model: pins of the numpy oracle against the closed forms the paper gives,
and parity (within Monte-Carlo error) of the product's C++ simulator against oracle and formulas."""
import math

import numpy as np
import pytest

import paper_2506_10911_amd as nl
from oracle import latency as ol


# ------------------------------- oracle pins --------------------------------

@pytest.mark.parametrize("mu,sigma", [(0.0, 0.25), (1.0, 0.5), (-0.5, 1.0)])
def test_oracle_pair_time_matches_closed_form(mu, sigma):
    rng = np.random.default_rng(1)
    t = ol.pair_times(rng, mu, sigma, 400_000)
    want = 2 * ol.expected_max_of_two(mu, sigma)              # appendix: E(t_local) = (1 + erf(sigma/2)) exp(mu + sigma^2/2)
    assert abs(t.mean() - want) < 5 * t.std() / math.sqrt(t.size)


def test_closed_form_against_numerical_integration():
    """E max(t1, t2) = integral of 2 x f(x) F(x) dx, by quadrature over the normal variable."""
    mu, sigma = 0.3, 0.8
    z = np.linspace(-10, 10, 400_001)
    pdf = np.exp(-z * z / 2) / math.sqrt(2 * math.pi)
    cdf = 0.5 * (1 + np.vectorize(math.erf)(z / math.sqrt(2)))
    integral = np.trapezoid(2 * np.exp(mu + sigma * z) * pdf * cdf, z)
    assert ol.expected_max_of_two(mu, sigma) == pytest.approx(integral, rel=1e-9)


@pytest.mark.parametrize("W", [2, 4, 32, 1024])
def test_oracle_constant_latency_gives_log2(W):
    rng = np.random.default_rng(2)
    t = ol.tree_allreduce_times(rng, W, math.log(1.5), 0.0, 3)
    np.testing.assert_allclose(t, 2 * 1.5 * math.log2(W), rtol=1e-12)       # t_all = 2 t_c log2(n)
    np.testing.assert_allclose(ol.pair_times(rng, math.log(1.5), 0.0, 3), 3.0, rtol=1e-12)


def test_oracle_tree_of_two_workers_has_a_closed_form():
    """W = 2: one reduce hop (max of two messages) and one broadcast hop (max of two more)."""
    rng = np.random.default_rng(3)
    t = ol.tree_allreduce_times(rng, 2, 0.2, 0.6, 400_000)
    want = 2 * ol.expected_max_of_two(0.2, 0.6)
    assert abs(t.mean() - want) < 5 * t.std() / math.sqrt(t.size)


def test_oracle_barrier_special_cases():
    rng = np.random.default_rng(4)
    a, b = ol.barrier_penalty(rng, 2, 2, 10, 50, 1.0, 0.7)        # one pair IS the whole world
    assert a == pytest.approx(b, rel=1e-12)
    a, b = ol.barrier_penalty(rng, 16, 16, 10, 50, 1.0, 0.7)      # subgroup = everybody: a global barrier
    assert a == pytest.approx(b, rel=1e-12)
    a, b = ol.barrier_penalty(rng, 64, 2, 10, 50, 1.0, 0.0)       # no variance: nobody waits
    assert a == pytest.approx(b, rel=1e-12) and a == pytest.approx(50 * 10 * math.e, rel=1e-12)
    a, b = ol.barrier_penalty(rng, 64, 1, 20, 40, 1.0, 0.7)       # no sync at all: the slowest worker's own sum
    assert b < a


def test_oracle_reproduces_the_papers_barrier_figure():
    """Paper: with LogNormal(1, 0.5) inner steps and 100 inner steps per outer step the global barrier
    costs about 20 % at 1024 workers; the penalty grows with the world size."""
    rng = np.random.default_rng(5)
    ratios = []
    for W in (16, 128, 1024):
        a, b = ol.barrier_penalty(rng, W, 2, 100, 250, 1.0, math.sqrt(0.5))
        ratios.append(a / b)
    assert ratios[0] < ratios[1] < ratios[2]
    assert 1.12 < ratios[2] < 1.28


# ------------------------- product against oracle ---------------------------

@pytest.mark.parametrize("W,mu,sigma", [(4, 0.0, 0.5), (32, 1.0, 0.25), (256, 0.0, 1.0), (1024, -1.0, 0.7)])
def test_product_tree_vs_pair(W, mu, sigma):
    trials = 20_000 if W <= 256 else 6_000
    got = nl.sim_tree_vs_pair(7, W, mu, sigma, trials)
    rng = np.random.default_rng(70 + W)
    ref = ol.tree_allreduce_times(rng, W, mu, sigma, trials)
    se = math.hypot(got["tree_se"], ref.std() / math.sqrt(trials))
    assert abs(got["tree"] - ref.mean()) < 5 * se
    assert got["tree_se"] == pytest.approx(ref.std() / math.sqrt(trials), rel=0.15)
    assert abs(got["pair"] - 2 * ol.expected_max_of_two(mu, sigma)) < 5 * got["pair_se"]
    # the advantage over the constant-latency ratio log2(W) grows with the variance (paper's figure)
    assert got["tree"] / got["pair"] > math.log2(W) * 0.999


def test_product_constant_latency_and_errors():
    got = nl.sim_tree_vs_pair(0, 32, math.log(2.0), 0.0, 5)
    assert got["tree"] == pytest.approx(2 * 2.0 * 5, rel=1e-12) and got["pair"] == pytest.approx(4.0, rel=1e-12)
    assert got["tree"] / got["pair"] == pytest.approx(math.log2(32), rel=1e-12)          # the paper's log2(32) = 5
    for args, status in [((0, 3, 0.0, 0.1, 10), 2), ((0, 1, 0.0, 0.1, 10), 2), ((0, 4, 0.0, -0.1, 10), 2),
                         ((0, 4, 0.0, 0.1, 0), 2)]:
        with pytest.raises(nl.NolocoError) as e:
            nl.sim_tree_vs_pair(*args)
        assert e.value.status == status
    with pytest.raises(nl.NolocoError) as e:
        nl.sim_barrier_penalty(0, 8, 3, 10, 10, 1.0, 0.5)
    assert e.value.status == 3


def test_product_barrier_penalty():
    sig = math.sqrt(0.5)
    a, b = nl.sim_barrier_penalty(3, 2, 2, 10, 50, 1.0, sig)
    assert a == pytest.approx(b, rel=1e-12)
    a, b = nl.sim_barrier_penalty(3, 16, 16, 10, 50, 1.0, sig)
    assert a == pytest.approx(b, rel=1e-12)
    a, b = nl.sim_barrier_penalty(3, 64, 2, 10, 50, 1.0, 0.0)
    assert a == pytest.approx(b, rel=1e-12) and a == pytest.approx(500 * math.e, rel=1e-12)
    assert nl.sim_barrier_penalty(3, 64, 2, 10, 50, 1.0, sig) == nl.sim_barrier_penalty(3, 64, 2, 10, 50, 1.0, sig)
    # against the oracle on the paper's setting: both estimate the same ratio (run-to-run spread of
    # one 250-round simulation at these sizes is below 1 %)
    rng = np.random.default_rng(9)
    for W in (64, 1024):
        a, b = nl.sim_barrier_penalty(11, W, 2, 100, 250, 1.0, sig)
        ra, rb = ol.barrier_penalty(rng, W, 2, 100, 250, 1.0, sig)
        assert a / b == pytest.approx(ra / rb, rel=0.02)
        assert a == pytest.approx(ra, rel=0.01) and b == pytest.approx(rb, rel=0.01)
    assert 1.12 < a / b < 1.28                                   # the paper's "about 20 % at 1024 accelerators"
