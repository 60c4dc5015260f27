"""Pins of the oracle's replica-spread statistic (the paper's results section: standard deviation
of the model weights across the data-parallel replicas). The statistic has a plain definition,
so the pins are library routines, closed forms and invariances."""
import numpy as np
import pytest
import torch

import oracle


def test_matches_numpy_population_variance():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal((12, 700)) * 0.02).astype(np.float32)
    segs = [(0, 100), (100, 1), (130, 333), (500, 200)]
    got = oracle.replica_spread(x, segs)
    x64 = x.astype(np.float64)
    for i, (o, n) in enumerate(segs):
        want = np.sqrt(np.var(x64[:, o:o + n], axis=0).mean())          # ddof = 0
        assert got[i] == pytest.approx(want, rel=1e-13)
    inside = np.concatenate([np.arange(o, o + n) for o, n in segs])
    assert got[-1] == pytest.approx(np.sqrt(np.var(x64[:, inside], axis=0).mean()), rel=1e-13)
    # torch's routine as a second library
    t = torch.from_numpy(x64[:, inside])
    assert got[-1] == pytest.approx(float(torch.var(t, dim=0, unbiased=False).mean().sqrt()), rel=1e-13)


def test_closed_forms():
    W, P = 8, 50
    base = np.linspace(-1, 1, P, dtype=np.float32)
    # identical replicas: no spread
    assert oracle.replica_spread(np.tile(base, (W, 1)))[-1] == 0.0
    # two replicas a, b: deviation |a - b| / 2 at every element (dyadic values: exact)
    two = np.stack([np.full(P, 0.75, np.float32), np.full(P, 0.25, np.float32)])
    assert oracle.replica_spread(two)[-1] == 0.25
    # replicas in arithmetic progression x_w = c + w d: variance d^2 (W^2 - 1) / 12
    d = 0.125
    prog = np.stack([base + w * d for w in range(W)]).astype(np.float32)
    assert oracle.replica_spread(prog)[-1] == pytest.approx(d * np.sqrt((W * W - 1) / 12.0), rel=1e-6)
    # one worker alone
    assert oracle.replica_spread(base.reshape(1, -1).copy())[-1] == 0.0


def test_invariances():
    rng = np.random.default_rng(1)
    x = rng.integers(-512, 512, (6, 40)).astype(np.float32) / 64      # dyadic: scaling and shifting are exact
    s0 = oracle.replica_spread(x)[-1]
    assert oracle.replica_spread(x * np.float32(4))[-1] == pytest.approx(4 * s0, rel=1e-14)
    assert oracle.replica_spread(x + np.float32(16))[-1] == pytest.approx(s0, rel=1e-14)
    assert oracle.replica_spread(np.ascontiguousarray(x[::-1]))[-1] == pytest.approx(s0, rel=1e-14)
    assert oracle.replica_spread(-x)[-1] == pytest.approx(s0, rel=1e-14)


def test_binary32_per_element_tracks_the_definition():
    rng = np.random.default_rng(2)
    x = (0.02 * rng.standard_normal((16, 5000)) + 1e-3 * rng.standard_normal((16, 5000))).astype(np.float32)
    a = oracle.replica_spread(x, [(0, 2500), (2500, 2500)])
    b = oracle.replica_spread(x, [(0, 2500), (2500, 2500)], binary32=True)
    np.testing.assert_allclose(b, a, rtol=2e-6)


def test_bf16_input_is_widened_exactly():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((4, 300)) * 0.02).astype(np.float32)
    h = torch.from_numpy(x).to(torch.bfloat16)
    bits = h.view(torch.int16).numpy().view(np.uint16).copy()
    wide = h.to(torch.float32).numpy()
    np.testing.assert_array_equal(oracle.replica_spread(bits), oracle.replica_spread(wide))


def test_full_averaging_step_removes_the_spread():
    """Ties the statistic to the method: one outer step with a single group of all workers,
    alpha = 0 and gamma = 1 puts every replica on the group mean (Eq. 2-3), so the spread is zero."""
    rng = np.random.default_rng(4)
    W, P = 8, 64
    phi = rng.integers(-256, 256, (W, P)).astype(np.float32) / 32
    theta = phi.copy()
    delta = np.zeros_like(phi)
    assert oracle.replica_spread(phi)[-1] > 1.0
    oracle.outer_step_f32(phi, delta, theta, (0.0, 0.7, 1.0), np.arange(W, dtype=np.int32),
                          np.array([0, W], dtype=np.int32))
    assert oracle.replica_spread(phi)[-1] == 0.0
