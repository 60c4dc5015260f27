"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Columns of the arena are independent, so the oracle runs on a sample of columns (the first and
last 64 elements of every tensor plus a strided sweep, all W rows) and is exact for those. The
oracle keeps its own phi/delta across steps; before every step its fast weights for the sampled
columns (drawn on the CPU from its own state) are written into the device arena, so both sides
see bit-identical inputs there, while the rest of the arena gets device-drawn drift of the same
distribution. Gaps of the gapped layout carry NaN canaries.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from harness import assert_state_equal, theta_to_device, to_bits

pytestmark = pytest.mark.gpu

import paper_2506_10911_amd as nl

nl.library_path()          # loads libnoloco.so now; a missing library is an error, not a skip

CASES = [
    # workload, W (0 = its own), subgroup size (0 = its schedule), steps compared, strided sample size,
    # vectors per thread (-1 = the library's choice), elements sampled at each end of every tensor.
    # The first six are the benchmark configurations with their own step counts.
    ("tiny", 0, 0, 10, 1 << 20, -1, 64),          # the whole arena
    ("gpt125m", 0, 0, 50, 1 << 18, -1, 64),
    ("stage1p3b", 0, 0, 20, 1 << 18, -1, 64),
    ("stage6p8b", 0, 0, 10, 1 << 18, -1, 64),
    ("ragged_tight", 0, 0, 100, 1 << 16, -1, 16),   # n cycles 2, 4, 8
    ("ragged_gapped", 0, 0, 100, 1 << 16, -1, 16),
    ("ragged_gapped", 0, 0, 6, 1 << 16, -1, 64),    # the same with a wide sample at every tensor edge
    # Larger subgroups, up to all workers in one group (the paragraph after Eq. 3: the update then is
    # DiLoCo's), in the shapes the measurements quote: registers (4, 16), phi-resident (32, 64),
    # two-pass (3, 12).
    ("stage6p8b", 0, 4, 3, 1 << 18, -1, 64),
    ("stage6p8b", 0, 16, 3, 1 << 18, -1, 64),
    ("ragged_tight", 0, 32, 3, 1 << 16, -1, 64),
    ("ragged_tight", 0, 64, 3, 1 << 16, -1, 64),
    ("stage1p3b", 48, 3, 3, 1 << 17, -1, 64),
    ("stage1p3b", 48, 12, 3, 1 << 17, -1, 64),
    # 16 groups of one worker with 1024-column tiles: 25.2 M workgroups, more than one grid may hold,
    # so the call goes out as two launches over tile ranges.
    ("stage6p8b", 0, 1, 2, 1 << 18, 1, 64),
]


def case_id(c):
    return c[0] + (f"-W{c[1]}" if c[1] else "") + (f"-n{c[2]}" if c[2] else "") + (f"-vpt{c[5]}" if c[5] > 0 else "") + \
        (f"-{c[3]}steps" if c[0] == "ragged_gapped" else "")


def gap_columns(wl):
    inside = np.zeros(wl.stride, dtype=bool)
    for o, n in wl.segments:
        inside[o:o + n] = True
    return np.flatnonzero(~inside)


@pytest.mark.parametrize("name,workers,subgroup,steps,strided,vpt,edge", CASES, ids=[case_id(c) for c in CASES])
def test_full_size_sampled_parity(name, workers, subgroup, steps, strided, vpt, edge):
    wl = workloads.make(name)
    if workers:
        wl.W = workers
    W, S = wl.W, wl.stride
    torch.cuda.empty_cache()
    need = W * S * (8 + wl.theta_bytes) + (2 << 30)
    free, _ = torch.cuda.mem_get_info()
    # every configuration fits an MI355X by design (the largest takes 257.8 of 288 GiB): no skip
    assert need <= free, f"{name}: needs {need / 1e9:.0f} GB, only {free / 1e9:.0f} GB free"
    print(f"[case] {name}: W={W} n={subgroup or wl.n_schedule} P={wl.P} tensors={len(wl.tensors)} "
          f"theta={wl.theta_dtype} steps={steps}", flush=True)
    dev = torch.device("cuda")
    tdt = torch.float32 if wl.theta_dtype == "f32" else torch.bfloat16
    phi = torch.empty((W, S), dtype=torch.float32, device=dev)
    delta = torch.zeros((W, S), dtype=torch.float32, device=dev)
    theta = torch.empty((W, S), dtype=tdt, device=dev)
    workloads.fill_phi0_device(phi, wl.seed, wl.init_std)

    cols = workloads.column_sample(wl, strided, edge)
    cols_t = torch.from_numpy(cols).to(dev)
    gaps = gap_columns(wl)
    gaps_t = torch.from_numpy(gaps).to(dev)
    if len(gaps):
        phi[:, gaps_t] = float("nan")
        delta[:, gaps_t] = float("nan")

    # oracle state on the sampled columns, as one dense arena
    o_phi = phi[:, cols_t].cpu().numpy()
    o_delta = np.zeros_like(o_phi)
    plan = nl.LaunchPlan(phi, delta, theta, S, W, nl.F32 if wl.theta_dtype == "f32" else nl.BF16, wl.segments)
    plan.tune(vectors_per_thread=vpt)
    info = plan.info()
    assert info["elements_per_worker"] == wl.P
    assert info["num_runs"] == (1 if name != "ragged_gapped" else len(wl.tensors))
    hp = (wl.alpha, wl.beta, wl.gamma)

    for t in range(steps):
        workloads.fake_inner_phase_device(theta, phi, wl.seed, t, wl.sigma)
        o_theta = workloads.fake_inner_phase_cpu(o_phi, wl.seed, t, wl.sigma, wl.theta_dtype)
        theta[:, cols_t] = theta_to_device(np.ascontiguousarray(o_theta), dev)
        if len(gaps):
            theta[:, gaps_t] = float("nan")
        n = subgroup or wl.n_at(t)
        members, offsets = nl.plan_groups(wl.seed, t, W, n)
        om, oo = oracle.plan_groups(wl.seed, t, W, n)
        assert members.tolist() == om.tolist() and offsets.tolist() == oo.tolist()
        nl.outer_step(plan, phi, delta, theta, hp, members, offsets)
        oracle.outer_step_f32(o_phi, o_delta, o_theta, hp, om, oo)
        torch.cuda.synchronize()
        got = {"phi": phi[:, cols_t].cpu().numpy(), "delta": delta[:, cols_t].cpu().numpy(),
               "theta": to_bits(theta[:, cols_t].cpu())}
        want = {"phi": o_phi, "delta": o_delta, "theta": o_theta}
        assert_state_equal(got, want, f"{name} step {t} (n={n})", wl.theta_dtype)
        if len(gaps):
            assert bool(torch.isnan(phi[:, gaps_t]).all()) and bool(torch.isnan(delta[:, gaps_t]).all())
            assert bool(torch.isnan(theta[:, gaps_t].float()).all())
        # properties that hold at any size, checked on the whole arena: the restart makes the fast
        # weights equal the (rounded) slow weights everywhere, and nothing overflowed
        if t == steps - 1:
            for w in range(0, W, max(1, W // 4)):
                row_phi = phi[w]
                if len(gaps):
                    row_phi = torch.nan_to_num(row_phi, nan=0.0)
                    assert torch.equal(torch.nan_to_num(theta[w].float(), nan=0.0), row_phi.to(tdt).float())
                else:
                    assert torch.equal(theta[w], row_phi.to(tdt))
                assert bool(torch.isfinite(row_phi).all())
    print(f"[done] {name}: {steps} steps, {len(cols)} sampled columns x {W} workers bit-identical", flush=True)
    plan.destroy()
    del phi, delta, theta
    torch.cuda.empty_cache()
