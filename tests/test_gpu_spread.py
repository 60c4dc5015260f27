"""GPU parity of noloco_replica_spread against the oracle: whole small arenas for every row-count
path, and the benchmark's full-size arena through small tensors the oracle can do exactly plus a
closed form that holds for every tensor."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from harness import segment_mask, theta_to_device

pytestmark = pytest.mark.gpu

import paper_2506_10911_amd as nl

nl.library_path()

# Primary check: the binary64 DEFINITION (oracle arithmetic 0), within a bound derived from the
# kernel's arithmetic.  Per element the kernel forms, in binary32 (unit roundoff u = 2^-24),
#   mean = (sum of W values) * (1/W),  v = (sum_w (x_w - mean)^2) * (1/W).
# (a) The W squared deviations are non-negative, so the roundings of dev (1), dev*dev (1), the W-1
#     additions and the final product with a rounded 1/W (2) give v a relative error of at most
#     (W + 4) u to first order; (W + 7) u leaves room for the second-order terms.
# (b) An error e in the mean shifts every deviation by the same amount; since the true deviations
#     sum to zero this adds exactly e^2 to v, with |e| <= (W + 1) u max|x| (W-1 additions of partial
#     sums up to W max|x|, then the rounded 1/W).
# Pooling over elements is binary64 on both sides (error ~1e-16 per term), so for a tensor with
# definition value s the kernel's figure lies within
#   sqrt(s^2 (1 + (W+7) u) + ((W+1) u max|x|)^2) - s      of s.
# Secondary check: the oracle's binary32-per-element mode, which repeats the kernel's element
# arithmetic and differs only in the binary64 pooling order: agreement to 1e-12 relative.
U32 = 2.0 ** -24
RTOL_SAME_ARITH = 1e-12


def definition_bound(ref, W, max_abs):
    """Largest |kernel - definition| the arithmetic above allows, per output entry."""
    ref = np.asarray(ref, dtype=np.float64)
    e = (W + 1) * U32 * max_abs
    return np.sqrt(ref * ref * (1.0 + (W + 7) * U32) + e * e) - ref + 1e-15


def max_abs_per_output(x_float, segs):
    """max |x| over each segment's elements (all rows), then over everything, as float64."""
    out = [float(np.abs(x_float[:, o:o + n]).max()) if n > 0 else 0.0 for o, n in segs]
    return np.array(out + [max(out) if out else 0.0])


def run_gpu(plan, x_dev, dtype, num_segments):
    out = torch.full((num_segments + 1,), -1.0, dtype=torch.float64, device="cuda")
    nl.replica_spread(plan, x_dev, dtype, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("theta_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8, 16, 32, 48, 64, 100])
def test_small_arena(theta_dtype, W):
    wl = workloads.make_small(theta_dtype=theta_dtype, W=W, layout="gapped", total=120_000)
    S = wl.stride
    rng = np.random.default_rng(W)
    x = (np.tile(workloads.phi0_cpu(S, 3), (W, 1)) + workloads.drift_cpu((W, S), 3, W, 1e-3)).astype(np.float32)
    segs = list(wl.segments)
    order = rng.permutation(len(segs))
    segs = [segs[i] for i in order] + [(5, 0)]                      # scrambled order, one empty segment
    inside = segment_mask(wl)
    if theta_dtype == "bf16":
        xb = torch.from_numpy(x).to(torch.bfloat16)
        x_host = xb.view(torch.int16).numpy().view(np.uint16).copy()
        x_host[:, ~inside] = 0x7FC0                                # NaN canaries in the gaps
        x_dev = theta_to_device(x_host)
        dt = nl.BF16
    else:
        x_host = x.copy()
        x_host[:, ~inside] = np.nan
        x_dev = torch.from_numpy(x_host).cuda()
        dt = nl.F32
    plan = nl.LaunchPlan(x_dev, x_dev, x_dev, S, W, dt, segs)
    got = run_gpu(plan, x_dev, dt, len(segs))
    ref = oracle.replica_spread(x_host, segs, binary32=False)          # the definition
    same = oracle.replica_spread(x_host, segs, binary32=True)
    assert np.isfinite(got).all()
    x_float = torch.from_numpy(x).to(torch.bfloat16).float().numpy() if theta_dtype == "bf16" else x
    bound = definition_bound(ref, W, max_abs_per_output(x_float, segs))
    assert (np.abs(got - ref) <= bound).all(), (np.abs(got - ref) / bound).max()
    assert (bound[ref > 0] <= 6e-6 * ref[ref > 0]).all()              # the bound itself is tight: (W+7)u/2
    np.testing.assert_allclose(got, same, rtol=RTOL_SAME_ARITH, atol=0)
    assert got[len(segs) - 1] == 0.0                               # the empty segment
    again = run_gpu(plan, x_dev, dt, len(segs))
    assert np.array_equal(got.view(np.uint64), again.view(np.uint64))   # fixed pooling order


def test_errors():
    x = torch.zeros((4, 64), device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    plan = nl.LaunchPlan(x, x, x, 64, 4, nl.F32, [(0, 64)])
    for fn, status in [(lambda: nl.replica_spread(plan, 0, nl.F32, out), 1),
                       (lambda: nl.replica_spread(plan, x, nl.F32, 0), 1),
                       (lambda: nl.replica_spread(plan, x, 5, out), 2),
                       (lambda: nl.replica_spread(plan, x.data_ptr() + 64, nl.F32, out), 5)]:
        with pytest.raises(nl.NolocoError) as e:
            fn()
        assert e.value.status == status
    empty = nl.LaunchPlan(x, x, x, 64, 4, nl.F32, [])
    nl.replica_spread(empty, x, nl.F32, out)
    torch.cuda.synchronize()
    assert float(out[0]) == 0.0


@pytest.mark.parametrize("name,dtype", [("stage6p8b", "f32"), ("stage6p8b", "bf16"), ("ragged_gapped", "f32")])
def test_full_size(name, dtype):
    """The benchmark arena at full size, as float and (the fast weights' storage) as bf16.
    (1) After a fake inner phase: every small tensor (<= 2^16 elements, all W rows) is recomputed by
    the oracle's binary64 definition and must match within the derived bound, and the binary32-per-
    element mode to 1e-12; the overall figure must equal the pooling of the per-tensor figures.
    (2) Rows set to an arithmetic progression x_w = x_0 + w d: every tensor and the total must give
    d sqrt((W^2 - 1) / 12)."""
    wl = workloads.make(name)
    W, S = wl.W, wl.stride
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    item = 4 if dtype == "f32" else 2
    assert W * S * (item + 4.0 / W) * 1.02 + (2 << 30) <= free, \
        f"{name} must fit: {W * S * item / 1e9:.0f} GB needed, {free / 1e9:.0f} GB free"
    print(f"[case] {name} {dtype}: W={W} P={wl.P}", flush=True)
    tdt, code = (torch.float32, nl.F32) if dtype == "f32" else (torch.bfloat16, nl.BF16)
    x = torch.empty((W, S), dtype=tdt, device="cuda")
    row0 = torch.empty((1, S), dtype=torch.float32, device="cuda")
    workloads.fill_phi0_device(row0, wl.seed, wl.init_std)
    for w in range(W):                                                   # common start + drift, row by row
        workloads.fake_inner_phase_device(x[w:w + 1], row0, wl.seed, w, wl.sigma)
    plan = nl.LaunchPlan(x, x, x, S, W, code, wl.segments)
    got = run_gpu(plan, x, code, len(wl.segments))
    small = [i for i, (_, n) in enumerate(wl.segments) if n <= (1 << 16)][:200]
    assert len(small) >= 40
    for i in small:
        o, n = wl.segments[i]
        piece = x[:, o:o + n].cpu()
        host = piece.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else piece.numpy()
        host = np.ascontiguousarray(host)
        ref = oracle.replica_spread(host, binary32=False)[-1]
        bound = definition_bound(ref, W, float(piece.float().abs().max()))
        assert abs(got[i] - ref) <= bound, (i, wl.tensors[i], got[i], ref, bound)
        same = oracle.replica_spread(host, binary32=True)[-1]
        assert got[i] == pytest.approx(same, rel=RTOL_SAME_ARITH), (i, wl.tensors[i])
    numel = np.array([n for _, n in wl.segments], dtype=np.float64)
    pooled = np.sqrt((got[:-1] ** 2 * numel).sum() / numel.sum())
    assert got[-1] == pytest.approx(pooled, rel=1e-12)
    # drift N(0, sigma^2) on top of a common start: population variance over W draws is sigma^2 (W-1)/W
    # (bf16 storage adds rounding noise of about half a percent of that variance)
    expect = wl.sigma * np.sqrt((W - 1) / W)
    assert got[-1] == pytest.approx(expect, rel=2e-3 if dtype == "f32" else 2e-2)
    d = 1.0 / 1024
    if dtype == "bf16":
        x[0].fill_(0.5)            # 0.5 + w / 128 is exact in bf16 for every w < 64
        d = 1.0 / 128
    for w in range(1, W):
        x[w].copy_(x[0])
        x[w].add_(w * d)
    got = run_gpu(plan, x, code, len(wl.segments))
    want = d * np.sqrt((W * W - 1) / 12.0)
    np.testing.assert_allclose(got, want, rtol=2e-4)               # x_0 + w d rounds in binary32
    print(f"[done] {name} {dtype}", flush=True)
    plan.destroy()
    del x, row0
    torch.cuda.empty_cache()
