"""Oracle of the paper's latency model (TEST INFRASTRUCTURE; numpy, written from the paper).

arxiv 2506.10911, section "Latency results" (theoretical and simulated speed-up) and appendix
"Latency analysis": messages and inner steps take LogNormal(mu, sigma^2) times.
  * tree all-reduce over W = 2^L workers: a parent has its children's result when the later of
    the two messages has arrived, t_local = max(t1, t2); the reduced value is then sent back down
    the tree; with constant message time t_c the total is 2 t_c log2(W);
  * local averaging in pairs: 2 max(t1, t2) in expectation, E max(t1, t2) =
    (1 + erf(sigma / 2)) exp(mu + sigma^2 / 2)  (the appendix' closed form);
  * barrier penalty: with a global barrier each outer round lasts as long as its slowest worker's
    inner phase; without it a worker only waits for its subgroup partners.
Only tests/ import this module; the product's simulator (C++) shares nothing with it.
"""
import math

import numpy as np


def expected_max_of_two(mu: float, sigma: float) -> float:
    """Closed form of E max(t1, t2) for i.i.d. LogNormal(mu, sigma^2)."""
    return (1.0 + math.erf(sigma / 2.0)) * math.exp(mu + sigma * sigma / 2.0)


def tree_allreduce_times(rng, W: int, mu: float, sigma: float, trials: int) -> np.ndarray:
    """`trials` samples of the completion time of one tree all-reduce (level by level, vectorised)."""
    levels = int(round(math.log2(W)))
    assert 2 ** levels == W and W >= 2
    ready = np.zeros((trials, W))
    width = W
    for _ in range(levels):                                   # reduce: pair up neighbours
        t = rng.lognormal(mu, sigma, size=(trials, width))
        arrive = ready + t
        ready = np.maximum(arrive[:, 0::2], arrive[:, 1::2])
        width //= 2
    down = ready                                              # [trials, 1]: the root has the sum
    for _ in range(levels):                                   # broadcast: every node tells its two children
        down = np.repeat(down, 2, axis=1)
        down = down + rng.lognormal(mu, sigma, size=down.shape)
    return down.max(axis=1)


def pair_times(rng, mu: float, sigma: float, trials: int) -> np.ndarray:
    t = rng.lognormal(mu, sigma, size=(trials, 4))
    return np.maximum(t[:, 0], t[:, 1]) + np.maximum(t[:, 2], t[:, 3])


def barrier_penalty(rng, W: int, n: int, inner_steps: int, outer_steps: int, mu: float, sigma: float):
    """(finishing time with a global barrier every round, finishing time with subgroup sync only)."""
    assert W % n == 0
    clock = np.zeros(W)
    barrier = 0.0
    for _ in range(outer_steps):
        phase = rng.lognormal(mu, sigma, size=(W, inner_steps)).sum(axis=1)
        barrier += phase.max()
        clock += phase
        groups = rng.permutation(W).reshape(W // n, n)        # fresh random subgroups every round
        clock[groups] = clock[groups].max(axis=1, keepdims=True)
    return barrier, clock.max()
