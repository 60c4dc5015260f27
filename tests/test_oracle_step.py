"""Pins of the CPU oracle's outer step against what the paper and the mathematics fix.

Everything here runs without a GPU and touches only oracle/ and workloads/.
References: arxiv 2506.10911, Eq. 1-3 (outer step), the paragraph after Eq. 3 (DiLoCo
reduction when the subgroup is everybody), the convergence appendix (restart of the
fast weights from the slow ones; zero initial momentum; common initial point; Lemma 1).
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from conftest import read_hand_examples


def one_group(n):
    return np.arange(n, dtype=np.int32), np.array([0, n], dtype=np.int32)


def col(v, dtype):
    return np.ascontiguousarray(np.array(v, dtype=dtype).reshape(-1, 1))


# ---------------------------------------------------------------------------
# Hand-worked examples of Eq. 1-3 (tests/golden/eq123_hand_examples.txt)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("case", read_hand_examples(), ids=lambda c: c["name"])
@pytest.mark.parametrize("mode", ["f64", "f32", "bf16"])
def test_hand_examples(case, mode):
    n = len(case["phi"])
    m, o = one_group(n)
    hp = (case["alpha"], case["beta"], case["gamma"])
    tol = case["tol"]
    if mode == "f64":
        phi, delta, theta = (col(case[k], np.float64) for k in ("phi", "delta", "theta"))
        oracle.outer_step_f64(phi, delta, theta, hp, m, o)
        got_theta = theta
        tol = min(tol, 1e-14)
    else:
        phi, delta = col(case["phi"], np.float32), col(case["delta"], np.float32)
        theta = col(case["theta"], np.float32)
        if mode == "bf16":
            theta = oracle.bf16_narrow(theta)       # the inputs are exact in bf16
            assert np.array_equal(oracle.bf16_widen(theta).ravel(), np.float32(case["theta"]))
        oracle.outer_step_f32(phi, delta, theta, hp, m, o)
        got_theta = oracle.bf16_widen(theta) if mode == "bf16" else theta
    np.testing.assert_allclose(delta.ravel(), case["expect_delta"], rtol=0, atol=tol)
    np.testing.assert_allclose(phi.ravel(), case["expect_phi"], rtol=0, atol=tol)
    # restart: the fast weights leave the step equal to the new slow weights
    # (for bf16, equal to their nearest bf16; the dyadic cases are exact)
    if mode == "bf16" and tol == 0:
        np.testing.assert_array_equal(got_theta.ravel(), np.float32(case["expect_phi"]))
    elif mode != "bf16":
        np.testing.assert_array_equal(got_theta, phi)


# ---------------------------------------------------------------------------
# Literal per-worker evaluation, every partition of a tiny worker set
# ---------------------------------------------------------------------------

def all_partitions(workers, n):
    """Every way of splitting `workers` into unordered groups of n."""
    if not workers:
        yield []
        return
    first, rest = workers[0], workers[1:]
    for others in itertools.combinations(rest, n - 1):
        left = [w for w in rest if w not in others]
        for tail in all_partitions(left, n):
            yield [[first, *others]] + tail


def literal_step(phi, delta, theta, hp, groups):
    """Eq. 1-3 evaluated worker by worker in exact rational arithmetic: each worker i looks up
    its own group and recomputes both sums for itself, as the equations are written."""
    alpha, beta, gamma = (Fraction(x) for x in hp)
    W, P = len(phi), len(phi[0])
    group_of = {i: g for g in groups for i in g}
    new_phi = [[None] * P for _ in range(W)]
    new_delta = [[None] * P for _ in range(W)]
    for i in range(W):
        for k in range(P):
            if i not in group_of:
                new_phi[i][k], new_delta[i][k] = phi[i][k], delta[i][k]
                continue
            G = group_of[i]
            n = len(G)
            sum_Delta = sum(phi[j][k] - theta[j][k] for j in G)          # Eq. 1 inside Eq. 2
            sum_phi = sum(phi[j][k] for j in G)
            d = alpha * delta[i][k] - beta / n * sum_Delta - gamma * (phi[i][k] - sum_phi / n)
            new_delta[i][k] = d
            new_phi[i][k] = phi[i][k] + d                                 # Eq. 3
    return new_phi, new_delta


@pytest.mark.parametrize("W,n", [(2, 1), (2, 2), (4, 2), (4, 4), (6, 2), (6, 3), (6, 6)])
def test_brute_force_all_partitions(W, n):
    rng = np.random.default_rng(100 * W + n)
    P = 3
    hp = (0.625, 0.75, 0.875)
    count = 0
    for groups in all_partitions(list(range(W)), n):
        phi = rng.integers(-64, 64, (W, P)) / 16.0
        theta = rng.integers(-64, 64, (W, P)) / 16.0
        delta = rng.integers(-64, 64, (W, P)) / 16.0
        exp_phi, exp_delta = literal_step(
            [[Fraction(x) for x in r] for r in phi], [[Fraction(x) for x in r] for r in delta],
            [[Fraction(x) for x in r] for r in theta], hp, groups)
        # shuffle members inside groups and the groups themselves: the result may not care
        shuffled = [list(rng.permutation(g)) for g in groups]
        shuffled = [shuffled[i] for i in rng.permutation(len(shuffled))]
        members = np.array([w for g in shuffled for w in g], dtype=np.int32)
        offsets = np.cumsum([0] + [len(g) for g in shuffled]).astype(np.int32)
        p64, d64, t64 = phi.copy(), delta.copy(), theta.copy()
        oracle.outer_step_f64(p64, d64, t64, hp, members, offsets)
        np.testing.assert_allclose(p64, np.array(exp_phi, dtype=np.float64), rtol=0, atol=1e-13)
        np.testing.assert_allclose(d64, np.array(exp_delta, dtype=np.float64), rtol=0, atol=1e-13)
        np.testing.assert_array_equal(t64, p64)
        p32, d32, t32 = (a.astype(np.float32) for a in (phi, delta, theta))
        oracle.outer_step_f32(p32, d32, t32, hp, members, offsets)
        np.testing.assert_allclose(p32, np.array(exp_phi, dtype=np.float64), rtol=0, atol=2e-6)
        np.testing.assert_allclose(d32, np.array(exp_delta, dtype=np.float64), rtol=0, atol=2e-6)
        count += 1
    expected_count = {(2, 1): 1, (2, 2): 1, (4, 2): 3, (4, 4): 1, (6, 2): 15, (6, 3): 10, (6, 6): 1}
    assert count == expected_count[(W, n)]


def test_partial_grouping_leaves_other_workers_alone():
    """Workers listed in no group are not touched (a dropped peer), unequal group sizes are fine."""
    rng = np.random.default_rng(5)
    W, P = 7, 5
    phi, delta, theta = (rng.standard_normal((W, P)) for _ in range(3))
    groups = [[4, 1, 6], [0, 3]]                       # workers 2 and 5 sit out
    members = np.array([4, 1, 6, 0, 3], dtype=np.int32)
    offsets = np.array([0, 3, 5], dtype=np.int32)
    F = lambda a: [[Fraction(float(x)) for x in r] for r in a]
    exp_phi, exp_delta = literal_step(F(phi), F(delta), F(theta), (0.5, 0.7, 0.9), groups)
    p, d, t = phi.copy(), delta.copy(), theta.copy()
    oracle.outer_step_f64(p, d, t, (0.5, 0.7, 0.9), members, offsets)
    np.testing.assert_allclose(p, np.array(exp_phi, dtype=np.float64), rtol=0, atol=1e-13)
    np.testing.assert_allclose(d, np.array(exp_delta, dtype=np.float64), rtol=0, atol=1e-13)
    for w in (2, 5):
        np.testing.assert_array_equal(p[w], phi[w])
        np.testing.assert_array_equal(d[w], delta[w])
        np.testing.assert_array_equal(t[w], theta[w])


def test_bad_groups_are_refused():
    a = np.zeros((4, 2))
    for members, offsets in [([0, 0], [0, 2]), ([0, 4], [0, 2]), ([-1, 1], [0, 2]), ([0, 1], [1, 2])]:
        with pytest.raises(ValueError):
            oracle.outer_step_f64(a.copy(), a.copy(), a.copy(), (0.5, 0.5, 0.5), members, offsets)


# ---------------------------------------------------------------------------
# DiLoCo reduction (paragraph after Eq. 3): subgroup = all workers
# ---------------------------------------------------------------------------

def test_diloco_reduction_against_textbook_momentum():
    """With n = N and a common start, the pull term is zero and every worker follows
    delta = alpha delta - beta mean_j(Delta_j), phi += delta: one global momentum descent."""
    rng = np.random.default_rng(7)
    W, P, steps = 8, 257, 12
    alpha, beta = 0.9, 0.7
    phi0 = rng.standard_normal(P) * 0.02
    phi = np.tile(phi0, (W, 1))
    delta = np.zeros((W, P))
    phi32, delta32 = phi.astype(np.float32), delta.astype(np.float32)
    m, o = one_group(W)
    g_phi, g_mom = phi0.copy(), np.zeros(P)          # the textbook loop: one global copy
    for t in range(steps):
        theta = phi + rng.standard_normal((W, P)) * 1e-3
        outer_grad = g_phi[None, :] - theta           # what every worker would send to the all-reduce
        g_mom = alpha * g_mom - beta * outer_grad.mean(axis=0)
        g_phi = g_phi + g_mom
        theta32 = theta.astype(np.float32)
        for gamma in (1.0,):                          # gamma must not matter; checked again below
            oracle.outer_step_f64(phi, delta, theta, (alpha, beta, gamma), m, o)
        oracle.outer_step_f32(phi32, delta32, theta32, (alpha, beta, 1.0), m, o)
        for w in range(W):
            np.testing.assert_allclose(phi[w], g_phi, rtol=0, atol=1e-14)
            np.testing.assert_allclose(delta[w], g_mom, rtol=0, atol=1e-14)
            # binary32: workers that start identical stay bit-identical (n is a power of two,
            # so the mean of n equal values is that value and the pull term is exactly 0)
            np.testing.assert_array_equal(phi32[w], phi32[0])
        np.testing.assert_allclose(phi32[0], g_phi, rtol=0, atol=5e-7)


def test_diloco_reduction_gamma_irrelevant():
    rng = np.random.default_rng(8)
    W, P = 4, 33
    phi = np.tile(rng.standard_normal(P), (W, 1))
    delta = np.tile(rng.standard_normal(P), (W, 1))
    theta = rng.standard_normal((W, P))
    m, o = one_group(W)
    outs = []
    for gamma in (0.0, 0.5, 1.7):
        p, d, t = phi.copy(), delta.copy(), theta.copy()
        oracle.outer_step_f64(p, d, t, (0.5, 0.7, gamma), m, o)
        outs.append((p, d))
    for p, d in outs[1:]:
        np.testing.assert_array_equal(p, outs[0][0])
        np.testing.assert_array_equal(d, outs[0][1])


def test_n1_is_momentum_sgd():
    rng = np.random.default_rng(9)
    W, P = 3, 17
    phi, delta, theta = (rng.standard_normal((W, P)) for _ in range(3))
    members = np.arange(W, dtype=np.int32)
    offsets = np.arange(W + 1, dtype=np.int32)
    exp_delta = 0.9 * delta - 0.7 * (phi - theta)
    exp_phi = phi + exp_delta
    oracle.outer_step_f64(phi, delta, theta, (0.9, 0.7, 1.3), members, offsets)
    np.testing.assert_allclose(delta, exp_delta, rtol=0, atol=1e-15)
    np.testing.assert_allclose(phi, exp_phi, rtol=0, atol=1e-15)


# ---------------------------------------------------------------------------
# Identities that follow from Eq. 2-3 for any partition
# ---------------------------------------------------------------------------

def random_state(rng, W, P):
    phi = rng.standard_normal((W, P)) * 0.02
    delta = rng.standard_normal((W, P)) * 1e-3
    theta = phi + rng.standard_normal((W, P)) * 1e-3
    return phi, delta, theta


@pytest.mark.parametrize("n", [2, 4, 8])
def test_group_mean_law_and_spread_law(n):
    """Averaging Eq. 2 over a group kills the pull term (it sums to zero inside a group), so
    mean_G phi' = mean_G phi + alpha mean_G delta - beta mean_G Delta whatever gamma is; and for
    two members i, k of one group phi'_i - phi'_k = (1 - gamma)(phi_i - phi_k) + alpha (delta_i - delta_k)."""
    rng = np.random.default_rng(20 + n)
    W, P = 16, 41
    alpha, beta, gamma = 0.9, 0.7, 1.1
    phi, delta, theta = random_state(rng, W, P)
    members, offsets = oracle.plan_groups(3, 5, W, n)
    p, d, t = phi.copy(), delta.copy(), theta.copy()
    oracle.outer_step_f64(p, d, t, (alpha, beta, gamma), members, offsets)
    for g in range(W // n):
        G = members[offsets[g]:offsets[g + 1]]
        lhs = p[G].mean(axis=0)
        rhs = phi[G].mean(axis=0) + alpha * delta[G].mean(axis=0) - beta * (phi[G] - theta[G]).mean(axis=0)
        np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-15)
        i, k = G[0], G[-1]
        np.testing.assert_allclose(p[i] - p[k],
                                   (1 - gamma) * (phi[i] - phi[k]) + alpha * (delta[i] - delta[k]),
                                   rtol=0, atol=1e-15)


def test_global_mean_follows_diloco_trajectory():
    """Summing the group-mean law over the groups: the average over all workers obeys
    delta_bar' = alpha delta_bar - beta Delta_bar, phi_bar' = phi_bar + delta_bar' for ANY
    partition and any gamma."""
    rng = np.random.default_rng(31)
    W, P, steps = 12, 19, 100
    alpha, beta, gamma = 0.5, 0.7, 1.0
    phi = np.tile(rng.standard_normal(P) * 0.02, (W, 1))
    delta = np.zeros((W, P))
    bar_phi, bar_delta = phi.mean(axis=0), np.zeros(P)
    for t in range(steps):
        n = (2, 3, 4, 6)[t % 4]
        theta = phi + rng.standard_normal((W, P)) * 1e-3 - 0.05 * phi      # noisy pull to 0
        bar_Delta = (phi - theta).mean(axis=0)
        bar_delta = alpha * bar_delta - beta * bar_Delta
        bar_phi = bar_phi + bar_delta
        members, offsets = oracle.plan_groups(17, t, W, n)
        oracle.outer_step_f64(phi, delta, theta, (alpha, beta, gamma), members, offsets)
        np.testing.assert_allclose(phi.mean(axis=0), bar_phi, rtol=0, atol=1e-13)
        np.testing.assert_allclose(delta.mean(axis=0), bar_delta, rtol=0, atol=1e-13)


def test_pure_gossip_contracts_to_global_mean():
    """theta = phi (no inner progress), alpha = 0, gamma = 1: every group collapses onto its own
    mean; the global sum is preserved and random re-pairing drives all workers to the global mean."""
    rng = np.random.default_rng(32)
    W, P = 8, 9
    phi = rng.standard_normal((W, P))
    delta = np.zeros((W, P))
    total = phi.sum(axis=0)
    spread = np.ptp(phi, axis=0).max()
    for t in range(60):
        theta = phi.copy()
        members, offsets = oracle.plan_groups(1, t, W, 2)
        oracle.outer_step_f64(phi, delta, theta, (0.0, 0.37, 1.0), members, offsets)
        np.testing.assert_allclose(phi.sum(axis=0), total, rtol=0, atol=1e-12)
        for g in range(W // 2):
            a, b = members[offsets[g]:offsets[g + 1]]
            np.testing.assert_allclose(phi[a], phi[b], rtol=0, atol=1e-15)
        new_spread = np.ptp(phi, axis=0).max()
        assert new_spread <= spread + 1e-15
        spread = new_spread
    assert spread < 1e-3
    np.testing.assert_allclose(phi, np.tile(total / W, (W, 1)), rtol=0, atol=1e-3)


def test_first_step_from_common_start_is_identical_inside_a_group():
    """phi_0 common, delta_0 = 0: after one step members of a group hold the same phi_1 (their
    delta_1 is the same group mean), bit for bit in binary32."""
    rng = np.random.default_rng(33)
    W, P = 8, 65
    phi = np.tile((rng.standard_normal(P) * 0.02).astype(np.float32), (W, 1))
    delta = np.zeros((W, P), dtype=np.float32)
    theta = (phi + rng.standard_normal((W, P)).astype(np.float32) * np.float32(1e-3)).astype(np.float32)
    members, offsets = oracle.plan_groups(2, 0, W, 2)
    oracle.outer_step_f32(phi, delta, theta, (0.9, 0.7, 1.0), members, offsets)
    for g in range(W // 2):
        a, b = members[offsets[g]:offsets[g + 1]]
        np.testing.assert_array_equal(phi[a], phi[b])
        np.testing.assert_array_equal(delta[a], delta[b])


def run_noisy_quadratic(omega, steps=400, W=16, P=64, m=20, a=1.0, seed=0, hp=(0.5, 0.7, 1.0)):
    """The setting of the paper's convergence theorem: loss 1/2 a (theta - c)^2 with c ~ N(0, 1) redrawn
    every inner step, m inner SGD steps of rate omega from the slow weights, then one outer step over
    random pairs. Returns the slow weights over the last half of the run, [steps/2, W, P]."""
    rng = np.random.default_rng(seed)
    phi = np.full((W, P), 3.0)                                   # common start, far from the optimum 0
    delta = np.zeros((W, P))
    tail = []
    for t in range(steps):
        theta = phi.copy()
        for _ in range(m):
            theta -= omega * a * (theta - rng.standard_normal((W, P)))
        members, offsets = oracle.plan_groups(seed, t, W, 2)
        oracle.outer_step_f64(phi, delta, theta, hp, members, offsets)
        if t >= steps // 2:
            tail.append(phi.copy())
    return np.array(tail)


def test_convergence_theorem_on_a_noisy_quadratic():
    """Theorem of the paper: E(phi) -> 0 and V(phi) shrinks with the inner learning rate omega (the
    theorem's leading-order statement is omega^2; at a finite number of inner steps the stationary
    variance of this model lies between the omega and the omega^2 law) for hyper-parameters inside
    the stability window (alpha = 0.5, beta = 0.7 > alpha, gamma = 1 lies in
    sqrt(n/(2(n-1))) alpha = 0.5 < gamma < 1.5 for n = 2). A wrong sign in Eq. 1 would diverge here."""
    big = run_noisy_quadratic(0.02)
    small = run_noisy_quadratic(0.01)
    for tail, omega in ((big, 0.02), (small, 0.01)):
        assert np.isfinite(tail).all()
        assert abs(tail.mean()) < 0.02                               # started at 3.0
    ratio = big.var() / small.var()
    assert 1.8 < ratio < 4.5, ratio                                  # omega halves -> variance falls 2x .. 4x
    # replicas stay together: the spread across workers is of the order of the noise, not of the start
    assert big.std(axis=1).mean() < 0.2


# ---------------------------------------------------------------------------
# binary32 instantiation: order invariance, agreement with binary64, segments
# ---------------------------------------------------------------------------

def test_order_invariance_bit_exact():
    rng = np.random.default_rng(40)
    W, P = 8, 301
    phi, delta, theta = (a.astype(np.float32) for a in random_state(rng, W, P))
    groups = [[0, 5, 2, 7], [6, 1], [3], [4]]
    ref = None
    for trial in range(6):
        gs = [list(rng.permutation(g)) for g in groups]
        gs = [gs[i] for i in rng.permutation(len(gs))]
        members = np.array([w for g in gs for w in g], dtype=np.int32)
        offsets = np.cumsum([0] + [len(g) for g in gs]).astype(np.int32)
        p, d, t = phi.copy(), delta.copy(), theta.copy()
        oracle.outer_step_f32(p, d, t, (0.9, 0.7, 1.0), members, offsets)
        if ref is None:
            ref = (p, d, t)
        else:
            for x, y in zip(ref, (p, d, t)):
                np.testing.assert_array_equal(x, y)


@pytest.mark.parametrize("n", [2, 3, 8])
def test_f32_tracks_f64(n):
    """One step from identical inputs: the binary32 result is within a few binary32 roundings
    of the binary64 one (|values| <= ~0.1, so 1e-7 absolute is ~10 ulp of the largest term)."""
    rng = np.random.default_rng(50 + n)
    W, P = 24, 1000
    phi, delta, theta = (a.astype(np.float32) for a in random_state(rng, W, P))
    members, offsets = oracle.plan_groups(9, 1, W, n)
    p64, d64, t64 = (a.astype(np.float64) for a in (phi, delta, theta))
    oracle.outer_step_f64(p64, d64, t64, (0.9, 0.7, 1.0), members, offsets)
    oracle.outer_step_f32(phi, delta, theta, (0.9, 0.7, 1.0), members, offsets)
    np.testing.assert_allclose(phi, p64, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(delta, d64, rtol=1e-6, atol=1e-7)
    np.testing.assert_array_equal(theta, phi)


def test_segments_and_gaps_untouched():
    rng = np.random.default_rng(60)
    W, stride = 4, 64
    segs = [(3, 5), (9, 1), (17, 30), (50, 13)]
    phi, delta, theta = (a.astype(np.float32) for a in random_state(rng, W, stride))
    inside = np.zeros(stride, dtype=bool)
    for o, n in segs:
        inside[o:o + n] = True
    for a in (phi, delta, theta):
        a[:, ~inside] = np.nan                          # canaries
    members, offsets = oracle.plan_groups(0, 0, W, 2)
    full = [a.copy() for a in (phi, delta, theta)]
    oracle.outer_step_f32(phi, delta, theta, (0.9, 0.7, 1.0), members, offsets, segments=segs)
    for a in (phi, delta, theta):
        assert np.isnan(a[:, ~inside]).all()
        assert np.isfinite(a[:, inside]).all()
    # the same columns computed as one dense arena give the same bits
    dense = [np.ascontiguousarray(a[:, inside]) for a in full]
    oracle.outer_step_f32(*dense, (0.9, 0.7, 1.0), members, offsets)
    for a, b in zip((phi, delta, theta), dense):
        np.testing.assert_array_equal(a[:, inside], b)


# ---------------------------------------------------------------------------
# bf16 storage of the fast weights
# ---------------------------------------------------------------------------

def test_bf16_narrow_matches_library_cast_and_ties_to_even():
    rng = np.random.default_rng(70)
    x = np.concatenate([
        rng.standard_normal(200_000).astype(np.float32) * np.float32(0.02),
        rng.standard_normal(1000).astype(np.float32) * np.float32(1e-40),    # subnormals
        np.array([0.0, -0.0, np.inf, -np.inf, 3.4028235e38, -3.4028235e38, 3.3895314e38,
                  1.0, 1.00390625, 1.01171875, 1.0039063, 1.0039062], dtype=np.float32),
        rng.integers(0, 2**32, 200_000, dtype=np.uint64).astype(np.uint32).view(np.float32),
    ])
    got = oracle.bf16_narrow(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    np.testing.assert_array_equal(got[~nan], want[~nan])
    assert (((got[nan] & 0x7F80) == 0x7F80) & ((got[nan] & 0x007F) != 0)).all()      # NaN stays NaN
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even mantissa (1.0);
    #       1 + 3*2^-8 is halfway between 1 + 2^-7 and 1 + 2^-6 -> even mantissa (1 + 2^-6)
    t = oracle.bf16_narrow(np.array([1.00390625, 1.01171875], dtype=np.float32))
    assert list(t) == [0x3F80, 0x3F82]
    # widening is exact and inverts narrowing of representable values
    h = np.arange(0, 65536, dtype=np.uint16)
    w = oracle.bf16_widen(h)
    ok = ~np.isnan(w)
    np.testing.assert_array_equal(oracle.bf16_narrow(w[ok]), h[ok])


def test_bf16_theta_step():
    """bf16 fast weights: Delta uses the exactly widened theta; theta' is the nearest bf16 of phi'."""
    rng = np.random.default_rng(71)
    W, P = 8, 500
    phi, delta, theta = (a.astype(np.float32) for a in random_state(rng, W, P))
    th16 = torch.from_numpy(theta).to(torch.bfloat16)
    theta_wide = th16.to(torch.float32).numpy()
    theta_bits = th16.view(torch.int16).numpy().view(np.uint16).copy()
    members, offsets = oracle.plan_groups(4, 2, W, 2)
    p_ref, d_ref, t_ref = phi.copy(), delta.copy(), theta_wide.copy()
    oracle.outer_step_f32(p_ref, d_ref, t_ref, (0.9, 0.7, 1.0), members, offsets)
    oracle.outer_step_f32(phi, delta, theta_bits, (0.9, 0.7, 1.0), members, offsets)
    np.testing.assert_array_equal(phi, p_ref)
    np.testing.assert_array_equal(delta, d_ref)
    want = torch.from_numpy(phi).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(theta_bits, want)
