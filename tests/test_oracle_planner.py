"""Pins of the oracle's subgroup planner.

The paper (arxiv 2506.10911, section "Outer optimizer step ...": a randomly chosen subgroup
of n instances, re-sampled every iteration; section "Inner optimizer step ...": groups are
assigned via random permutations) fixes WHAT the planner must deliver: a partition of the
workers into groups of n, uniformly distributed, fresh each step. The generator is this
build's choice; its core is pinned by the published SplitMix64 known-answer vector.
"""
import itertools
import os
from collections import Counter

import numpy as np
import pytest

import oracle
from conftest import GOLDEN

M64 = (1 << 64) - 1
GOLDEN_GAMMA = 0x9E3779B97F4A7C15


def test_splitmix64_known_answers():
    state, outs = None, []
    for line in open(os.path.join(GOLDEN, "splitmix64_kat.txt")):
        line = line.strip()
        if line.startswith("state0"):
            state = int(line.split()[1])
        elif line.startswith("out"):
            outs.append(int(line.split()[1]))
    assert len(outs) == 5
    for k, want in enumerate(outs):
        assert oracle.mix64((state + (k + 1) * GOLDEN_GAMMA) & M64) == want


def test_draw_stream_is_splitmix_from_a_per_step_base():
    """Draw k of (seed, step) is the (k+1)-th SplitMix64 output from a base state that depends on
    seed and step only through mix64: checked with the KAT-pinned mix64 as the only primitive."""
    for seed, step in [(0, 0), (1, 0), (0, 1), (2**63 + 5, 2**40 + 3), (M64, M64)]:
        base = oracle.mix64(seed ^ oracle.mix64((step + GOLDEN_GAMMA) & M64))
        for k in (0, 1, 2, 63, 1000):
            assert oracle.draw(seed, step, k) == oracle.mix64((base + (k + 1) * GOLDEN_GAMMA) & M64)


def test_bounded_draw_rule_is_exactly_uniform_on_a_16_bit_word():
    """Exhaustive: over all 2^16 words, the accepted ones hit every residue equally often, and
    as few words as possible are rejected (2^16 mod m of them)."""
    rs = range(1 << 16)
    for m in list(range(1, 70)) + [100, 255, 256, 257, 1000, 4097, 30000, 32768, 32769, 65535]:
        hits = Counter(oracle.bounded16(r, m) for r in rs)
        rejected = hits.pop(-1, 0)
        assert rejected == (1 << 16) % m
        assert sorted(hits) == list(range(m))
        assert set(hits.values()) == {(1 << 16) // m}


@pytest.mark.parametrize("W", [1, 2, 3, 4, 6, 8, 12, 16, 30, 64, 96, 1000])
def test_every_plan_is_a_partition_into_sorted_groups(W):
    for n in [d for d in range(1, W + 1) if W % d == 0]:
        for seed, step in [(0, 0), (4, 99), (12345678901234567, 3)]:
            members, offsets = oracle.plan_groups(seed, step, W, n)
            assert members.dtype == np.int32 and offsets.dtype == np.int32
            assert sorted(members.tolist()) == list(range(W))
            assert offsets.tolist() == list(range(0, W + 1, n))
            for g in range(W // n):
                grp = members[offsets[g]:offsets[g + 1]]
                assert (np.diff(grp) > 0).all()


def test_bad_sizes_are_refused():
    for W, n in [(8, 3), (8, 0), (8, 16), (0, 1), (7, 2)]:
        with pytest.raises(ValueError):
            oracle.plan_groups(0, 0, W, n)


def test_plan_is_a_pure_function_of_seed_and_step():
    a = [oracle.plan_groups(7, t, 16, 2)[0].tolist() for t in range(50)]
    b = [oracle.plan_groups(7, t, 16, 2)[0].tolist() for t in reversed(range(50))][::-1]
    assert a == b                                          # no hidden state: resume is exact
    assert len({tuple(x) for x in a}) > 45                 # re-sampled every outer step
    c = [oracle.plan_groups(8, t, 16, 2)[0].tolist() for t in range(50)]
    assert sum(x == y for x, y in zip(a, c)) < 3           # the seed matters


def canonical(members, offsets):
    return tuple(sorted(tuple(members[offsets[g]:offsets[g + 1]].tolist()) for g in range(len(offsets) - 1)))


@pytest.mark.parametrize("W,n,count", [(4, 2, 3), (6, 2, 15), (6, 3, 10), (8, 4, 35)])
def test_partitions_are_uniform(W, n, count):
    """Chi-square over all set partitions into groups of n, 10^5 (seed, step) pairs. 99.9 % quantiles
    of chi2 with count-1 degrees of freedom: 13.8 (2), 36.1 (14), 27.9 (9), 65.2 (34)."""
    trials = 100_000
    hits = Counter()
    for i in range(trials):
        seed, step = i // 500, i % 500
        hits[canonical(*oracle.plan_groups(seed, step, W, n))] += 1
    assert len(hits) == count
    expect = trials / count
    chi2 = sum((v - expect) ** 2 / expect for v in hits.values())
    limit = {3: 13.8, 15: 36.1, 10: 27.9, 35: 65.2}[count]
    assert chi2 < limit, (chi2, limit)


def test_each_worker_meets_every_peer_equally_often():
    """n = 2, W = 16: over many steps every unordered pair of workers is matched with probability 1/15."""
    W, steps = 16, 30_000
    pair_hits = Counter()
    for t in range(steps):
        members, offsets = oracle.plan_groups(42, t, W, 2)
        for g in range(W // 2):
            pair_hits[tuple(members[2 * g:2 * g + 2].tolist())] += 1
    assert len(pair_hits) == W * (W - 1) // 2
    expect = steps * (W // 2) / (W * (W - 1) // 2)
    chi2 = sum((v - expect) ** 2 / expect for v in pair_hits.values())
    assert chi2 < 180.0, chi2                               # 99.9 % quantile for 119 dof is 173.6... margin
