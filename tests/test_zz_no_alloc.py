"""noloco_replica_spread_noalloc (partial sums staged in the library's static per-GPU array) against
noloco_replica_spread (staged in the plan's own buffer): same kernels, so the outputs must agree
bit for bit. Two calls in a row, the second on a smaller arena, so that the second call finds the
first call's leftovers in the shared array; then the documented size limit."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu

import paper_2506_10911_amd as nl

nl.library_path()          # loads libnoloco.so now; a missing library is an error, not a skip


def make_case(W, total, theta_dtype, seed):
    wl = workloads.make_small(theta_dtype=theta_dtype, W=W, layout="gapped", total=total, seed=seed)
    S = wl.stride
    x = (np.tile(workloads.phi0_cpu(S, seed), (W, 1)) + workloads.drift_cpu((W, S), seed, W, 1e-3)).astype(np.float32)
    x_dev = torch.from_numpy(x).cuda()
    dt = nl.F32
    if theta_dtype == "bf16":
        x_dev, dt = x_dev.to(torch.bfloat16), nl.BF16
    segs = list(wl.segments) + [(3, 0)]                          # one empty segment
    plan = nl.LaunchPlan(x_dev, x_dev, x_dev, S, W, dt, segs)
    return plan, x_dev, dt, len(segs)


def both(plan, x_dev, dt, num_segments):
    out_a = torch.full((num_segments + 1,), -1.0, dtype=torch.float64, device="cuda")
    out_b = torch.full((num_segments + 1,), -2.0, dtype=torch.float64, device="cuda")
    nl.replica_spread(plan, x_dev, dt, out_a)
    nl.replica_spread_noalloc(plan, x_dev, dt, out_b)
    torch.cuda.synchronize()
    return out_a.cpu().numpy(), out_b.cpu().numpy()


def test_two_calls_in_a_row_match_the_allocating_entry_point():
    big = make_case(W=16, total=600_000, theta_dtype="f32", seed=21)      # several hundred tiles
    small = make_case(W=5, total=40_000, theta_dtype="bf16", seed=22)     # fewer tiles, other kernel path
    for plan, x_dev, dt, k in (big, small):
        want, got = both(plan, x_dev, dt, k)
        assert np.isfinite(got).all() and (got[:-2] > 0).all() and got[k - 1] == 0.0
        assert np.array_equal(want.view(np.uint64), got.view(np.uint64))
    # and once more in the opposite order, alone: the result does not depend on what ran before
    for plan, x_dev, dt, k in (small, big):
        out = torch.zeros(k + 1, dtype=torch.float64, device="cuda")
        nl.replica_spread_noalloc(plan, x_dev, dt, out)
        ref = torch.zeros(k + 1, dtype=torch.float64, device="cuda")
        nl.replica_spread(plan, x_dev, dt, ref)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
    for plan, *_ in (big, small):
        plan.destroy()


def test_replays_from_a_hip_graph():
    """The callers this entry point is for include code under HIP graph capture: the call is captured
    once and replayed three times, with eager work and synchronisation between the replays and the
    input changed in between; every replay must equal the allocating entry point run eagerly."""
    plan, x_dev, dt, k = make_case(W=16, total=300_000, theta_dtype="f32", seed=23)
    out = torch.zeros(k + 1, dtype=torch.float64, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        nl.replica_spread_noalloc(plan, x_dev, dt, out)
    torch.cuda.synchronize()
    for replay in range(3):
        x_dev.mul_(1.0 + 0.25 * replay)                              # eager work that changes the input
        ref = torch.zeros(k + 1, dtype=torch.float64, device="cuda")
        nl.replica_spread(plan, x_dev, dt, ref)
        torch.cuda.synchronize()
        out.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), replay
        assert float(torch.randn(1 << 14, device="cuda").square().mean()) > 0.5   # more eager work
    plan.destroy()


def test_size_limit_and_argument_errors():
    x = torch.zeros((4, 64), device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    # A layout whose tile count exceeds the static array: 16 rows of 2^31 + 1024 elements is 2^21 + 1
    # tiles of 1024. Plans only describe a layout, and the entry point refuses before any launch, so
    # no memory of that size is ever touched.
    stride = (1 << 31) + 1024
    huge = nl.LaunchPlan(x, x, x, stride, 16, nl.F32, [(0, stride)])
    with pytest.raises(nl.NolocoError) as e:
        nl.replica_spread_noalloc(huge, x, nl.F32, out)
    assert e.value.status == 7                                   # NOLOCO_ERR_UNSUPPORTED
    huge.destroy()
    plan = nl.LaunchPlan(x, x, x, 64, 4, nl.F32, [(0, 64)])
    for fn, status in [(lambda: nl.replica_spread_noalloc(plan, 0, nl.F32, out), 1),
                       (lambda: nl.replica_spread_noalloc(plan, x, nl.F32, 0), 1),
                       (lambda: nl.replica_spread_noalloc(plan, x, 5, out), 2),
                       (lambda: nl.replica_spread_noalloc(plan, x.data_ptr() + 64, nl.F32, out), 5)]:
        with pytest.raises(nl.NolocoError) as e:
            fn()
        assert e.value.status == status
    nl.replica_spread_noalloc(plan, x, nl.F32, out)              # identical rows: zero spread
    torch.cuda.synchronize()
    assert float(out[0]) == 0.0 and float(out[1]) == 0.0
    plan.destroy()
