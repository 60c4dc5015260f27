"""Pins of the oracle's pipeline-routing plan (paper: section "Inner optimizer step via dynamic
pipeline routing" and the appendix algorithm "Random pipeline routing"). What the paper fixes:
per step groups come from random permutations; a worker may receive from any replica of the
previous stage and send to any replica of the next; re-randomising every step balances load;
gradients flow back along the path of the forward pass."""
import itertools
from collections import Counter

import numpy as np
import pytest

import oracle


@pytest.mark.parametrize("stages,W", [(2, 1), (2, 2), (2, 8), (4, 16), (3, 5), (7, 64), (2, 1000)])
def test_every_boundary_is_a_permutation_with_its_inverse(stages, W):
    for seed, step, mb in [(0, 0, 0), (9, 123, 7), (2**63 + 1, 2**40, 2**33)]:
        send_to, recv_from = oracle.plan_routes(seed, step, mb, stages, W)
        assert send_to.shape == recv_from.shape == (stages - 1, W)
        for b in range(stages - 1):
            assert sorted(send_to[b].tolist()) == list(range(W))      # each replica receives from exactly one
            for r in range(W):
                assert recv_from[b, send_to[b, r]] == r              # the backward pass retraces the path


def test_paths_cover_every_replica_of_every_stage_once():
    stages, W = 4, 16
    send_to, recv_from = oracle.plan_routes(3, 5, 1, stages, W)
    paths = []
    for r0 in range(W):
        path, r = [r0], r0
        for b in range(stages - 1):
            r = int(send_to[b, r])
            path.append(r)
        paths.append(path)
        back = path[-1]                                              # gradients flow back along the same path
        for b in reversed(range(stages - 1)):
            back = int(recv_from[b, back])
        assert back == r0
    for s in range(stages):
        assert sorted(p[s] for p in paths) == list(range(W))


def test_one_stage_routes_nothing_and_bad_sizes_are_refused():
    send_to, recv_from = oracle.plan_routes(0, 0, 0, 1, 8)
    assert send_to.shape == (0, 8)
    for stages, W in [(0, 4), (2, 0), (-1, 3)]:
        with pytest.raises(ValueError):
            oracle.plan_routes(0, 0, 0, stages, W)


def test_plan_is_pure_and_rerandomised_by_step_microbatch_and_seed():
    base = oracle.plan_routes(4, 10, 2, 3, 32)[0]
    assert np.array_equal(base, oracle.plan_routes(4, 10, 2, 3, 32)[0])
    for other in [(5, 10, 2), (4, 11, 2), (4, 10, 3)]:
        assert not np.array_equal(base, oracle.plan_routes(*other, 3, 32)[0])
    assert not np.array_equal(base[0], base[1])                        # boundaries draw independently


@pytest.mark.parametrize("W,limit", [(3, 20.5), (4, 49.7)])
def test_permutations_are_uniform(W, limit):
    """Chi-square over all W! permutations, 60 000 (seed, step, microbatch) triples; limits are the
    99.9 % quantiles for 5 and 23 degrees of freedom."""
    trials = 60_000
    hits = Counter()
    for i in range(trials):
        send_to, _ = oracle.plan_routes(i % 50, (i // 50) % 60, i // 3000, 2, W)
        hits[tuple(send_to[0].tolist())] += 1
    perms = list(itertools.permutations(range(W)))
    assert set(hits) == set(perms)
    expect = trials / len(perms)
    chi2 = sum((hits[p] - expect) ** 2 / expect for p in perms)
    assert chi2 < limit, chi2


def test_boundaries_are_independent():
    """Joint distribution of the permutations of two consecutive boundaries, W = 3: uniform over all 36
    pairs (99.9 % quantile of chi-square with 35 degrees of freedom: 66.6)."""
    trials = 72_000
    hits = Counter()
    for i in range(trials):
        send_to, _ = oracle.plan_routes(i % 40, i // 40, 0, 3, 3)
        hits[(tuple(send_to[0].tolist()), tuple(send_to[1].tolist()))] += 1
    assert len(hits) == 36
    expect = trials / 36
    chi2 = sum((v - expect) ** 2 / expect for v in hits.values())
    assert chi2 < 66.6, chi2


def test_load_is_balanced_over_time():
    """Every replica of the next stage is reached from a given replica equally often (1/W each)."""
    W, steps = 8, 40_000
    hits = np.zeros((W, W))
    for t in range(steps):
        send_to, _ = oracle.plan_routes(11, t, 0, 2, W)
        hits[np.arange(W), send_to[0]] += 1
    expect = steps / W
    chi2 = ((hits - expect) ** 2 / expect).sum()
    assert chi2 < 90.0, chi2                                          # 49 dof: 99.9 % quantile 85.4
