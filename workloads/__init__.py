"""Seeded synthetic workloads for the NoLoCo outer step: arena shapes and input values.

This module serves both the CPU oracle and the HIP library (through tests/ and bench.py)
and holds none of the method's arithmetic: no planner, no Eq. 1-3, no bf16 rounding of
its own (casts are torch's). It imports neither side.

Shapes follow the model table of arxiv 2506.10911 (appendix "Additional experiment
details": hidden size / layers / FFN width of 768/12/3072, 2048/24/8192, 4096/32/16384),
its data-parallel world sizes (8 and 16) and its subgroup sizes (2; 2/4/8 in the ablation
on n), laid out as GPT-style blocks. Values stand in for the paper's training runs, which
need its datasets: a common start phi_0 ~ N(0, 0.02^2) for every worker, zero momentum,
and before each outer step a fake inner phase theta_i = cast(phi_i + sigma * z).
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

ALIGN_ELEMS = 64  # worker_stride is rounded up to this many elements


@dataclass
class Workload:
    name: str
    tensors: List[Tuple[str, int]]            # (name, numel), in arena order
    segments: List[Tuple[int, int]]           # (offset, numel) inside one worker's row
    W: int
    theta_dtype: str                          # "f32" | "bf16"
    n_schedule: Tuple[int, ...]               # subgroup size at outer step t is n_schedule[t % len]
    sigma: float                              # std-dev of the fake inner-phase drift
    steps: int
    seed: int
    alpha: float = 0.9                        # outer momentum
    beta: float = 0.7                         # outer learning rate
    gamma: float = 1.0                        # pull towards the subgroup mean
    init_std: float = 0.02
    P: int = field(init=False)                # real elements per worker
    stride: int = field(init=False)           # elements between consecutive workers' rows

    def __post_init__(self):
        self.P = sum(n for _, n in self.segments)
        end = max(o + n for o, n in self.segments)
        self.stride = -(-end // ALIGN_ELEMS) * ALIGN_ELEMS

    def n_at(self, step: int) -> int:
        return self.n_schedule[step % len(self.n_schedule)]

    @property
    def theta_bytes(self) -> int:
        return 2 if self.theta_dtype == "bf16" else 4

    @property
    def bytes_per_update(self) -> int:
        """Algorithmic HBM bytes per worker-parameter: phi, delta, theta each read and written once."""
        return 2 * (4 + 4 + self.theta_bytes)


def gpt_block(d: int, f: int, prefix: str) -> List[Tuple[str, int]]:
    """The 12 tensors of one GPT-style transformer block (2-matrix FFN), 12 d^2 + 9 d + f elements."""
    return [
        (prefix + "ln1.w", d), (prefix + "ln1.b", d),
        (prefix + "attn.qkv.w", d * 3 * d), (prefix + "attn.qkv.b", 3 * d),
        (prefix + "attn.out.w", d * d), (prefix + "attn.out.b", d),
        (prefix + "ln2.w", d), (prefix + "ln2.b", d),
        (prefix + "mlp.fc.w", d * f), (prefix + "mlp.fc.b", f),
        (prefix + "mlp.proj.w", f * d), (prefix + "mlp.proj.b", d),
    ]


def _tight(tensors):
    segs, off = [], 0
    for _, n in tensors:
        segs.append((off, n))
        off += n
    return segs


def _gapped(tensors, seed):
    """Every tensor is followed by 1..7 elements that belong to nobody."""
    rng = np.random.default_rng([seed, 0x6170])
    gaps = rng.integers(1, 8, size=len(tensors))
    segs, off = [], 0
    for (_, n), g in zip(tensors, gaps):
        segs.append((off, n))
        off += n + int(g)
    return segs


def ragged_tensors(count: int, total: int, seed: int, lo_exp: float = 6.0, hi_exp: float = 20.0):
    """`count` odd sizes, log-uniform between 2^lo_exp and 2^hi_exp, rescaled to about `total` elements."""
    rng = np.random.default_rng([seed, 0x7261])
    s = np.floor(2.0 ** rng.uniform(lo_exp, hi_exp, size=count))
    s = np.maximum(np.floor(s * (total / s.sum())), 64).astype(np.int64) | 1
    return [(f"t{i}", int(n)) for i, n in enumerate(s)]


def make(name: str) -> Workload:
    """The five benchmark configurations, plus small variants used by the tests."""
    if name == "tiny":
        t = [("flat", 1 << 20)]
        return Workload(name, t, _tight(t), W=4, theta_dtype="f32", n_schedule=(2,),
                        sigma=1e-3, steps=10, seed=0)
    if name == "gpt125m":
        d, f = 768, 3072
        t = [("wte", 50257 * d), ("wpe", 1024 * d)]
        for l in range(12):
            t += gpt_block(d, f, f"h{l}.")
        t += [("ln_f.w", d), ("ln_f.b", d)]
        return Workload(name, t, _tight(t), W=8, theta_dtype="f32", n_schedule=(2,),
                        sigma=1e-3, steps=50, seed=1)
    if name == "stage1p3b":
        d, f = 2048, 8192
        t = []
        for l in range(6):
            t += gpt_block(d, f, f"h{l}.")
        return Workload(name, t, _tight(t), W=8, theta_dtype="f32", n_schedule=(2,),
                        sigma=5e-4, steps=20, seed=2)
    if name == "stage6p8b":
        d, f = 4096, 16384
        t = []
        for l in range(8):
            t += gpt_block(d, f, f"h{l}.")
        return Workload(name, t, _tight(t), W=16, theta_dtype="bf16", n_schedule=(2,),
                        sigma=5e-4, steps=10, seed=3)
    if name in ("ragged_tight", "ragged_gapped"):
        t = ragged_tensors(4096, 124_439_808, seed=4)
        segs = _tight(t) if name == "ragged_tight" else _gapped(t, seed=4)
        return Workload(name, t, segs, W=64, theta_dtype="f32", n_schedule=(2, 4, 8),
                        sigma=1e-3, steps=100, seed=4)
    raise KeyError(name)


def make_small(theta_dtype="f32", W=8, n_schedule=(2,), layout="gapped", count=24, total=200_000,
               seed=11, steps=4, sigma=1e-3) -> Workload:
    """A ragged arena small enough for the oracle to run in full, still spanning many tiles."""
    t = ragged_tensors(count, total, seed=seed, lo_exp=3.0, hi_exp=16.0)
    t = [(nm, max(n // 2 | 1, 1)) for nm, n in t]
    t[0] = (t[0][0], 1)            # a one-element tensor
    t[1] = (t[1][0], 7)
    segs = _tight(t) if layout == "tight" else _gapped(t, seed)
    return Workload(f"small_{layout}_{theta_dtype}_W{W}", t, segs, W=W, theta_dtype=theta_dtype,
                    n_schedule=tuple(n_schedule), sigma=sigma, steps=steps, seed=seed)


# ---------------------------------------------------------------------------
# Values, CPU side (numpy; used for everything the oracle consumes)
# ---------------------------------------------------------------------------

def phi0_cpu(count: int, seed: int, std: float = 0.02) -> np.ndarray:
    """Common initial slow weights of every worker, float32 [count]."""
    rng = np.random.default_rng([seed, 0x7068])
    return (rng.standard_normal(count, dtype=np.float32) * np.float32(std)).astype(np.float32)


def drift_cpu(shape, seed: int, step: int, sigma: float) -> np.ndarray:
    """sigma * z, z ~ N(0,1) i.i.d., float32; one independent draw per (seed, step)."""
    rng = np.random.default_rng([seed, 0x6472, step])
    return rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)


def fake_inner_phase_cpu(phi: np.ndarray, seed: int, step: int, sigma: float, theta_dtype: str):
    """theta = cast(phi + sigma z). Returns float32, or bf16 bit patterns as uint16 (torch's rounding)."""
    th = (phi + drift_cpu(phi.shape, seed, step, sigma)).astype(np.float32)
    if theta_dtype == "bf16":
        import torch
        return torch.from_numpy(th).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    return th


# ---------------------------------------------------------------------------
# Values, device side (torch; fills arenas too large to build on the host)
# ---------------------------------------------------------------------------

def fill_phi0_device(phi, seed: int, std: float = 0.02, chunk: int = 1 << 27):
    """phi: torch float32 [W, stride] on the GPU. Row 0 gets N(0, std^2) over the whole row (gaps and
    padding included; they belong to nobody), the other rows copy it: the common start phi_0."""
    import torch
    g = torch.Generator(device=phi.device)
    g.manual_seed(seed * (1 << 32) + 0x7068)
    stride = phi.shape[1]
    for a in range(0, stride, chunk):
        b = min(a + chunk, stride)
        phi[0, a:b].normal_(0.0, std, generator=g)
    for w in range(1, phi.shape[0]):
        phi[w].copy_(phi[0])


def fake_inner_phase_device(theta, phi, seed: int, step: int, sigma: float, chunk: int = 1 << 27):
    """theta[w] = cast(phi[w] + sigma z) over whole rows, chunked so the temporaries stay small."""
    import torch
    g = torch.Generator(device=phi.device)
    g.manual_seed(seed * (1 << 32) + 0x6472 + step * 7919)
    stride = phi.shape[1]
    buf = torch.empty(min(chunk, stride), dtype=torch.float32, device=phi.device)
    for w in range(phi.shape[0]):
        for a in range(0, stride, chunk):
            b = min(a + chunk, stride)
            z = buf[: b - a]
            z.normal_(0.0, sigma, generator=g)
            z.add_(phi[w, a:b])
            theta[w, a:b].copy_(z)


# ---------------------------------------------------------------------------
# Column samples (columns of the arena are independent, so an oracle run on a
# sample of them is exact for those columns)
# ---------------------------------------------------------------------------

def column_sample(wl: Workload, strided: int, edge: int = 64) -> np.ndarray:
    """Sorted unique row offsets: the first and last `edge` elements of every segment plus about
    `strided` elements taken at a constant stride over the real elements."""
    cols = []
    for off, n in wl.segments:
        e = min(edge, n)
        cols.append(np.arange(off, off + e, dtype=np.int64))
        cols.append(np.arange(off + n - e, off + n, dtype=np.int64))
    if strided > 0:
        offs = np.array([o for o, _ in wl.segments], dtype=np.int64)
        lens = np.array([n for _, n in wl.segments], dtype=np.int64)
        cum = np.concatenate([[0], np.cumsum(lens)])
        step = max(wl.P // strided, 1)
        if step % 2 == 0:
            step += 1                      # odd stride: visits every lane position of a vector
        flat = np.arange(0, wl.P, step, dtype=np.int64)
        seg = np.searchsorted(cum, flat, side="right") - 1
        cols.append(offs[seg] + (flat - cum[seg]))
    return np.unique(np.concatenate(cols))
