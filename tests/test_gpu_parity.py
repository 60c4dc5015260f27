"""GPU parity: the HIP library, called through the C ABI, against the CPU oracle, element by
element on whole small arenas (ragged, gapped, many tiles, every kernel variant)."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import workloads
from harness import SmallCase, assert_state_equal, to_bits

pytestmark = pytest.mark.gpu

import paper_2506_10911_amd as nl

nl.library_path()          # loads libnoloco.so now; a missing library is an error, not a skip


def groups_from_lists(lists):
    members = np.array([w for g in lists for w in g], dtype=np.int32)
    offsets = np.cumsum([0] + [len(g) for g in lists]).astype(np.int32)
    return members, offsets


@pytest.mark.parametrize("theta_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["tight", "gapped"])
@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 3, 6, 48])
def test_small_arena_multi_step(theta_dtype, layout, n):
    """4 outer steps, fresh random groups each step, W = 48 workers; everything compared after
    every step, gaps and padding hold NaN canaries that must survive bit for bit."""
    W = 48
    wl = workloads.make_small(theta_dtype=theta_dtype, W=W, n_schedule=(n,), layout=layout)
    case = SmallCase(wl, nl)
    assert case.plan.info()["elements_per_worker"] == wl.P
    for t in range(wl.steps):
        case.inner_phase(t)
        members, offsets = nl.plan_groups(wl.seed, t, W, n)
        om, oo = oracle.plan_groups(wl.seed, t, W, n)
        assert members.tolist() == om.tolist() and offsets.tolist() == oo.tolist()
        case.step(t, members, offsets)
        case.check(f"{wl.name} n={n} step {t}")


@pytest.mark.parametrize("theta_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["tight", "gapped"])
@pytest.mark.parametrize("n", [32, 64, 128, 5, 256])
def test_large_subgroups(theta_dtype, layout, n):
    """Subgroups of 32 and 64 (phi kept in registers), 128 and 5 (two passes), 256 (the largest
    a call accepts), over W = 640 workers (768 for n = 256)."""
    W = 768 if n == 256 else 640
    wl = workloads.make_small(theta_dtype=theta_dtype, W=W, n_schedule=(n,), layout=layout, count=8,
                              total=20_000, steps=2)
    case = SmallCase(wl, nl)
    for t in range(wl.steps):
        case.inner_phase(t)
        members, offsets = nl.plan_groups(wl.seed, t, W, n)
        case.step(t, members, offsets)
        case.check(f"{wl.name} n={n} step {t}")


@pytest.mark.parametrize("theta_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("vpt", [1, 2, 4])
@pytest.mark.parametrize("nontemporal", [0, 1])
@pytest.mark.parametrize("group_major,xcd_map", [(0, 0), (1, 0), (0, 1), (1, 1), (1, 2), (0, 5), (1, 64), (1, 4096)])
def test_launch_shapes_do_not_change_results(theta_dtype, vpt, nontemporal, group_major, xcd_map):
    wl = workloads.make_small(theta_dtype=theta_dtype, W=16, n_schedule=(2, 4, 8, 1), layout="gapped",
                              total=400_000)
    case = SmallCase(wl, nl)
    case.plan.tune(vectors_per_thread=vpt, nontemporal=nontemporal, group_major=group_major,
                   xcd_map=xcd_map)
    assert case.plan.info()["tile_elems"] == 1024 * vpt
    for t in range(4):
        case.inner_phase(t)
        members, offsets = nl.plan_groups(wl.seed, t, wl.W, wl.n_at(t))
        case.step(t, members, offsets)
        case.check(f"vpt={vpt} nt={nontemporal} gm={group_major} xm={xcd_map} step {t}")


@pytest.mark.parametrize("theta_dtype", ["f32", "bf16"])
def test_unequal_groups_and_absent_workers(theta_dtype):
    """One call with groups of 1, 2, 3, 4, 5 and 8 members given in scrambled order; three workers
    sit out and must keep every bit."""
    wl = workloads.make_small(theta_dtype=theta_dtype, W=26, layout="gapped")
    case = SmallCase(wl, nl)
    rng = np.random.default_rng(3)
    perm = rng.permutation(26).tolist()
    sizes, lists, at = [3, 1, 8, 2, 5, 4], [], 0
    for s in sizes:
        lists.append(perm[at:at + s])
        at += s
    absent = perm[at:]
    assert len(absent) == 3
    members, offsets = groups_from_lists(lists)
    case.inner_phase(0)
    case.delta[:, case.inside] = workloads.drift_cpu((26, int(case.inside.sum())), 5, 0, 1e-3)
    case.d_delta.copy_(torch.from_numpy(case.delta))
    before = case.gpu_state()
    case.step(0, members, offsets)
    case.check("unequal groups")
    after = case.gpu_state()
    for w in absent:
        for k in ("phi", "delta", "theta"):
            assert np.array_equal(before[k][w].view(np.uint8), after[k][w].view(np.uint8))
    # the order of members and of groups is irrelevant, bit for bit
    lists2 = [list(reversed(g)) for g in reversed(lists)]
    case2 = SmallCase(wl, nl)
    case2.inner_phase(0)
    case2.delta[:] = 0
    case2.delta[:, case2.inside] = workloads.drift_cpu((26, int(case.inside.sum())), 5, 0, 1e-3)
    case2.delta[:, ~case2.inside] = np.nan
    case2.d_delta.copy_(torch.from_numpy(case2.delta))
    m2, o2 = groups_from_lists(lists2)
    case2.nl.outer_step(case2.plan, case2.d_phi, case2.d_delta, case2.d_theta,
                        (wl.alpha, wl.beta, wl.gamma), m2, o2)
    torch.cuda.synchronize()
    assert_state_equal(case2.gpu_state(), after, "member order", theta_dtype)


def test_diloco_mode_all_workers_one_group():
    """n = W = 64 (two-pass kernel): from a common start the workers stay bit-identical."""
    wl = workloads.make_small(theta_dtype="f32", W=64, n_schedule=(64,), layout="tight")
    case = SmallCase(wl, nl, canary=False)
    for t in range(3):
        case.inner_phase(t)
        members, offsets = nl.plan_groups(wl.seed, t, 64, 64)
        case.step(t, members, offsets)
        case.check(f"diloco step {t}")
        g = case.gpu_state()
        assert (g["phi"] == g["phi"][0]).all()


def test_special_values_propagate():
    """Inf, NaN, signed zeros and subnormals go through the same binary32 operations on both sides."""
    wl = workloads.make_small(theta_dtype="bf16", W=4, layout="tight", count=6, total=5000)
    case = SmallCase(wl, nl, canary=False)
    specials = np.array([np.inf, -np.inf, np.nan, 0.0, -0.0, 1e-40, -1e-40, 3e38, -3e38, 1.0],
                        dtype=np.float32)
    rng = np.random.default_rng(9)
    for arr in (case.phi, case.delta):
        idx = rng.integers(0, wl.P, 400)
        arr[rng.integers(0, 4, 400), idx] = specials[rng.integers(0, len(specials), 400)]
    case.d_phi.copy_(torch.from_numpy(case.phi))
    case.d_delta.copy_(torch.from_numpy(case.delta))
    case.inner_phase(0)
    members, offsets = nl.plan_groups(1, 0, 4, 2)
    case.step(0, members, offsets)
    got, want = case.gpu_state(), case.oracle_state()
    for k in ("phi", "delta"):
        nan = np.isnan(want[k])
        assert np.array_equal(np.isnan(got[k]), nan)
        assert np.array_equal(got[k][~nan].view(np.uint32), want[k][~nan].view(np.uint32))
    tn = (want["theta"] & 0x7FFF) > 0x7F80
    assert np.array_equal((got["theta"] & 0x7FFF) > 0x7F80, tn)
    assert np.array_equal(got["theta"][~tn], want["theta"][~tn])


def test_empty_inputs():
    wl = workloads.make_small(W=4, layout="tight", count=4, total=3000)
    case = SmallCase(wl, nl, canary=False)
    case.inner_phase(0)
    before = case.gpu_state()
    hp = (0.9, 0.7, 1.0)
    nl.outer_step(case.plan, case.d_phi, case.d_delta, case.d_theta, hp, [], [0])             # no groups
    nl.outer_step(case.plan, case.d_phi, case.d_delta, case.d_theta, hp, [], [0, 0, 0])       # empty groups
    torch.cuda.synchronize()
    after = case.gpu_state()
    for k in before:
        assert np.array_equal(before[k], after[k])
    # an arena with no (or only empty) segments: a valid plan, a step that does nothing
    plan = nl.LaunchPlan(case.d_phi, case.d_delta, case.d_theta, wl.stride, 4, nl.F32, [(5, 0)])
    assert plan.info()["elements_per_worker"] == 0 and plan.info()["num_tiles"] == 0
    nl.outer_step(plan, case.d_phi, case.d_delta, case.d_theta, hp, [0, 1, 2, 3], [0, 2, 4])
    torch.cuda.synchronize()
    after = case.gpu_state()
    for k in before:
        assert np.array_equal(before[k], after[k])


def test_error_paths_launch_nothing():
    wl = workloads.make_small(W=8, layout="tight", count=4, total=3000)
    case = SmallCase(wl, nl, canary=False)
    case.inner_phase(0)
    before = case.gpu_state()
    hp = (0.9, 0.7, 1.0)
    ok_m, ok_o = [0, 1, 2, 3], [0, 2, 4]

    def status_of(fn):
        with pytest.raises(nl.NolocoError) as e:
            fn()
        return e.value.status

    step = lambda m, o, **kw: nl.outer_step(case.plan, kw.get("phi", case.d_phi), case.d_delta,
                                            kw.get("theta", case.d_theta), hp, m, o)
    assert status_of(lambda: step([0, 1, 1, 3], ok_o)) == 3          # duplicate worker
    assert status_of(lambda: step([0, 1, 2, 8], ok_o)) == 3          # id out of range
    assert status_of(lambda: step([0, -1, 2, 3], ok_o)) == 3
    assert status_of(lambda: step(ok_m, [1, 2, 4])) == 3             # offsets must start at 0
    assert status_of(lambda: step(ok_m, [0, 3, 2])) == 3             # decreasing offsets
    assert status_of(lambda: step(ok_m, ok_o, phi=case.d_phi.data_ptr() + 16)) == 5   # misaligned base
    assert status_of(lambda: step(ok_m, ok_o, phi=0)) == 1
    # worker ids are checked against the plan's W
    other = nl.LaunchPlan(case.d_phi, case.d_delta, case.d_theta, wl.stride, 4, nl.F32, wl.segments)
    assert status_of(lambda: nl.outer_step(other, case.d_phi, case.d_delta, case.d_theta, hp,
                                           [0, 1, 2, 3, 4, 5], [0, 6])) == 3
    # an arena whose layout differs from the plan's is refused (raw ABI call: the binding always
    # fills the arena from its plan)
    from paper_2506_10911_amd import binding as B
    for field, value in [("W", 4), ("worker_stride", wl.stride + 64), ("theta_dtype", nl.BF16)]:
        arena = B._Arena.from_buffer_copy(case.plan._arena(case.d_phi, case.d_delta, case.d_theta))
        setattr(arena, field, value)
        m = np.array(ok_m, dtype=np.int32)
        o = np.array(ok_o, dtype=np.int32)
        rc = B._lib.noloco_outer_step(case.plan._handle, C.byref(arena), C.byref(B._HParams(*hp)),
                                      m.ctypes.data, o.ctypes.data, 2, 0)
        assert rc == 2, field
    # layout errors at plan creation
    mk = lambda **kw: nl.LaunchPlan(kw.get("phi", case.d_phi), case.d_delta, case.d_theta,
                                    kw.get("stride", wl.stride), kw.get("W", 8), kw.get("dt", nl.F32),
                                    kw.get("segs", wl.segments))
    assert status_of(lambda: mk(stride=wl.stride + 1)) == 5
    assert status_of(lambda: mk(segs=[(0, 10), (5, 10)])) == 4
    assert status_of(lambda: mk(segs=[(wl.stride - 1, 2)])) == 4
    assert status_of(lambda: mk(W=0)) == 2
    assert status_of(lambda: mk(dt=7)) == 2
    assert status_of(lambda: mk(phi=0)) == 1
    torch.cuda.synchronize()
    after = case.gpu_state()                      # no refused call may have touched the arena
    for k in before:
        assert np.array_equal(before[k].view(np.uint8), after[k].view(np.uint8))
    step(ok_m, ok_o)                              # and the arena is still usable
    torch.cuda.synchronize()
    oracle.outer_step_f32(case.phi, case.delta, case.theta, hp, ok_m, ok_o, segments=wl.segments)
    case.check("after error paths")


def test_group_larger_than_limit_is_unsupported():
    W = 300
    phi, delta, theta = (torch.zeros((W, 64), device="cuda") for _ in range(3))
    plan = nl.LaunchPlan(phi, delta, theta, 64, W, nl.F32, [(0, 64)])
    with pytest.raises(nl.NolocoError) as e:
        nl.outer_step(plan, phi, delta, theta, (0.9, 0.7, 1.0), list(range(W)), [0, W])
    assert e.value.status == 7
    # arrays that alias each other are refused: the step is in place on all three
    for a, b, c in [(phi, phi, theta), (phi, delta, phi), (phi, delta, delta),
                    (phi, phi.data_ptr() + 256, theta)]:
        with pytest.raises(nl.NolocoError) as e:
            nl.outer_step(plan, a, b, c, (0.9, 0.7, 1.0), [0, 1], [0, 2])
        assert e.value.status == 2


def test_resume_and_determinism():
    """5 + 5 steps with a fresh plan object equal 10 steps in one go; a rerun gives the same bits."""
    wl = workloads.make_small(theta_dtype="bf16", W=8, n_schedule=(2, 4), layout="gapped")
    runs = []
    for split in (None, 5, None):
        case = SmallCase(wl, nl)
        for t in range(10):
            if split is not None and t == split:
                case.plan.destroy()
                case.plan = nl.LaunchPlan(case.d_phi, case.d_delta, case.d_theta, wl.stride, wl.W,
                                          nl.BF16, wl.segments)
            case.inner_phase(t)
            members, offsets = nl.plan_groups(wl.seed, t, wl.W, wl.n_at(t))
            case.step(t, members, offsets)
        case.check("after 10 steps")
        runs.append(case.gpu_state())
    for other in runs[1:]:
        for k in other:
            assert np.array_equal(runs[0][k].view(np.uint8), other[k].view(np.uint8))


def test_many_groups_split_over_launches():
    """W = 600 workers in pairs: 300 groups exceed one launch's member table, so the call is split."""
    W = 600
    wl = workloads.make_small(theta_dtype="f32", W=W, layout="gapped", count=5, total=3000)
    case = SmallCase(wl, nl)
    case.inner_phase(0)
    members, offsets = nl.plan_groups(2, 0, W, 2)
    case.step(0, members, offsets)
    case.check("600 workers")


def test_stream_argument_is_honoured():
    wl = workloads.make_small(theta_dtype="f32", W=8, layout="tight")
    case = SmallCase(wl, nl, canary=False)
    case.inner_phase(0)
    members, offsets = nl.plan_groups(0, 0, 8, 2)
    hp = (wl.alpha, wl.beta, wl.gamma)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        nl.outer_step(case.plan, case.d_phi, case.d_delta, case.d_theta, hp, members, offsets)
    s.synchronize()
    oracle.outer_step_f32(case.phi, case.delta, case.theta, hp, members, offsets, segments=wl.segments)
    case.check("side stream")


def test_one_plan_serves_two_threads_on_two_streams():
    """A launch plan is immutable and the step keeps its scratch on the caller's stack, so two host
    threads may step disjoint sets of workers through ONE plan at the same time, each on its own
    stream. 40 steps per thread with changing pairings; the oracle applies the same steps one
    thread after the other (the sets are disjoint, so the interleaving cannot matter)."""
    import threading
    wl = workloads.make_small(theta_dtype="bf16", W=8, layout="gapped")
    case = SmallCase(wl, nl)
    case.inner_phase(0)
    hp = (wl.alpha, wl.beta, wl.gamma)
    halves = ([0, 1, 2, 3], [4, 5, 6, 7])
    rng = np.random.default_rng(5)
    plans = [[rng.permutation(h).tolist() for _ in range(40)] for h in halves]
    errors = []
    torch.cuda.synchronize()

    def work(steps):
        try:
            stream = torch.cuda.Stream()
            for members in steps:
                nl.outer_step(case.plan, case.d_phi, case.d_delta, case.d_theta, hp, members, [0, 2, 4], stream=stream)
            stream.synchronize()
        except Exception as e:            # reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=work, args=(p,)) for p in plans]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for steps in plans:
        for members in steps:
            oracle.outer_step_f32(case.phi, case.delta, case.theta, hp, members, [0, 2, 4], segments=wl.segments)
    case.check("two threads, one plan")


def test_outer_steps_replay_from_a_hip_graph():
    """noloco_outer_step allocates, copies and synchronises nothing, so a window of outer steps can
    be captured into a HIP graph (member tables travel in the kernel arguments and are baked in).
    Three steps with different groupings are captured once and replayed three times, with eager work
    and synchronisation between the replays; every replay is checked against the oracle."""
    wl = workloads.make_small(theta_dtype="bf16", W=8, n_schedule=(2, 4, 8), layout="gapped")
    case = SmallCase(wl, nl)
    hp = (wl.alpha, wl.beta, wl.gamma)
    plans = [nl.plan_groups(wl.seed, t, wl.W, wl.n_at(t)) for t in range(3)]
    case.inner_phase(0)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    snapshot = [t.clone() for t in (case.d_phi, case.d_delta, case.d_theta)]
    with torch.cuda.graph(graph, stream=side):
        for members, offsets in plans:
            nl.outer_step(case.plan, case.d_phi, case.d_delta, case.d_theta, hp, members, offsets)
    # capture does not execute: restore nothing, the arena is still the snapshot
    torch.cuda.synchronize()
    for t, snap in zip((case.d_phi, case.d_delta, case.d_theta), snapshot):
        assert torch.equal(torch.nan_to_num(t.float()), torch.nan_to_num(snap.float()))
    for replay in range(3):
        graph.replay()
        torch.cuda.synchronize()
        for members, offsets in plans:
            oracle.outer_step_f32(case.phi, case.delta, case.theta, hp, members, offsets, segments=wl.segments)
        case.check(f"graph replay {replay}")
        scratch = torch.randn(1 << 16, device="cuda").sum().item()          # eager work between replays
        assert scratch == scratch


def test_probes():
    src = torch.arange(1 << 20, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    nl.copy_probe(dst, src, src.numel() * 4 - 16)
    torch.cuda.synchronize()
    assert torch.equal(dst[:-4], src[:-4]) and float(dst[-4:].abs().sum()) == 0.0
    sink = torch.full((4,), 7.0, device="cuda")
    nl.read_probe(src, src.numel() * 4 - 16, sink)
    nl.fill_probe(dst, dst.numel() * 4 - 32, 2.5)
    torch.cuda.synchronize()
    assert bool((sink == 7.0).all())                            # the read probe writes nothing
    assert bool((dst[:-8] == 2.5).all()) and torch.equal(dst[-8:-4], src[-8:-4])
    for fn in (lambda: nl.copy_probe(dst, src, 24), lambda: nl.fill_probe(dst, -16),
               lambda: nl.read_probe(src, 20, sink)):
        with pytest.raises(nl.NolocoError) as e:
            fn()
        assert e.value.status == 2
    with pytest.raises(nl.NolocoError) as e:
        nl.fill_probe(dst.data_ptr() + 4, 16)
    assert e.value.status == 5


def test_tuning_is_validated_and_automatic_by_default():
    wl = workloads.make_small(W=8, layout="tight", count=4, total=3000)
    case = SmallCase(wl, nl, canary=False)
    # automatic: an arena too small to give every CU eight 4096-column tiles takes the smallest tile;
    # a big one takes 4 vectors per thread for pairs (plans only describe a layout: no memory is touched)
    assert case.plan.info()["tile_elems"] == 1024
    big = nl.LaunchPlan(case.d_phi, case.d_delta, case.d_theta, 1 << 26, 8, nl.F32, [(0, 1 << 26)])
    assert big.info()["tile_elems"] == 4096
    big.destroy()
    for bad in [dict(vectors_per_thread=3), dict(nontemporal=2), dict(group_major=-2), dict(xcd_map=4097)]:
        with pytest.raises(nl.NolocoError) as e:
            case.plan.tune(**bad)
        assert e.value.status == 2
    case.plan.tune(vectors_per_thread=1)
    assert case.plan.info()["tile_elems"] == 1024
    case.plan.tune(vectors_per_thread=4)
    assert case.plan.info()["tile_elems"] == 4096
    case.plan.tune()                                           # back to automatic
    assert case.plan.info()["tile_elems"] == 1024
