"""Shared plumbing of the GPU parity tests: device arenas, the oracle run beside them, comparisons.

Nothing here computes any part of the method: the oracle side calls oracle/, the GPU side calls
the C ABI through the binding, inputs come from workloads/.
"""
import numpy as np
import torch

import oracle
import workloads

# Tolerances stated by the benchmark definition for the fp32 state; the bf16 fast weights may be
# off by one bf16 ulp. The tests additionally require bit equality, which the design promises.
RTOL, ATOL = 1e-6, 1e-7


def to_bits(theta_cpu_tensor):
    """torch CPU tensor (float32 or bfloat16) -> numpy float32 / uint16 bit patterns."""
    if theta_cpu_tensor.dtype == torch.bfloat16:
        return theta_cpu_tensor.view(torch.int16).numpy().view(np.uint16)
    return theta_cpu_tensor.numpy()


def theta_to_device(theta_np, device="cuda"):
    if theta_np.dtype == np.uint16:
        return torch.from_numpy(theta_np.view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(theta_np).to(device)


def assert_state_equal(got, want, what, theta_dtype):
    """got / want: dicts of numpy arrays phi, delta (float32) and theta (float32 or bf16 bits)."""
    for k in ("phi", "delta"):
        np.testing.assert_allclose(got[k], want[k], rtol=RTOL, atol=ATOL, equal_nan=True,
                                   err_msg=f"{what}: {k} outside the stated tolerance")
        assert np.array_equal(got[k].view(np.uint32), want[k].view(np.uint32)), \
            f"{what}: {k} within tolerance but not bit-identical"
    if theta_dtype == "bf16":
        g, w = got["theta"].astype(np.int32), want["theta"].astype(np.int32)
        # same sign and at most one step apart in the ordered bf16 bit patterns = within 1 ulp
        assert (np.abs(g - w) <= 1).all(), f"{what}: theta more than 1 bf16 ulp off"
        assert np.array_equal(g, w), f"{what}: theta within 1 ulp but not bit-identical"
    else:
        np.testing.assert_allclose(got["theta"], want["theta"], rtol=RTOL, atol=ATOL, equal_nan=True,
                                   err_msg=f"{what}: theta outside the stated tolerance")
        assert np.array_equal(got["theta"].view(np.uint32), want["theta"].view(np.uint32)), \
            f"{what}: theta not bit-identical"


def segment_mask(wl):
    inside = np.zeros(wl.stride, dtype=bool)
    for o, n in wl.segments:
        inside[o:o + n] = True
    return inside


class SmallCase:
    """A whole small arena on both sides: oracle state in numpy, GPU state in torch tensors."""

    def __init__(self, wl, nl, canary=True):
        self.wl, self.nl = wl, nl
        W, S = wl.W, wl.stride
        self.inside = segment_mask(wl)
        phi0 = workloads.phi0_cpu(S, wl.seed, wl.init_std)
        self.phi = np.tile(phi0, (W, 1))
        self.delta = np.zeros((W, S), dtype=np.float32)
        self.theta = np.zeros((W, S), dtype=np.float32 if wl.theta_dtype == "f32" else np.uint16)
        if canary:
            self.phi[:, ~self.inside] = np.nan
            self.delta[:, ~self.inside] = np.nan
        self.d_phi = torch.from_numpy(self.phi).cuda()
        self.d_delta = torch.from_numpy(self.delta).cuda()
        tdt = torch.float32 if wl.theta_dtype == "f32" else torch.bfloat16
        self.d_theta = torch.zeros((W, S), dtype=tdt, device="cuda")
        self.plan = nl.LaunchPlan(self.d_phi, self.d_delta, self.d_theta, S, W,
                                  nl.F32 if wl.theta_dtype == "f32" else nl.BF16, wl.segments)
        self.canary = canary

    def inner_phase(self, step):
        """theta = cast(phi_oracle + drift): one array, handed bit for bit to both sides."""
        wl = self.wl
        th = workloads.fake_inner_phase_cpu(np.nan_to_num(self.phi), wl.seed, step, wl.sigma, wl.theta_dtype)
        if self.canary:
            th = th.copy()
            th[:, ~self.inside] = 0x7FC0 if wl.theta_dtype == "bf16" else np.nan
        self.theta = np.ascontiguousarray(th)
        self.d_theta.copy_(theta_to_device(self.theta))

    def step(self, step, members, offsets, hp=None):
        wl = self.wl
        hp = hp or (wl.alpha, wl.beta, wl.gamma)
        oracle.outer_step_f32(self.phi, self.delta, self.theta, hp, members, offsets, segments=wl.segments)
        self.nl.outer_step(self.plan, self.d_phi, self.d_delta, self.d_theta, hp, members, offsets)
        torch.cuda.synchronize()

    def gpu_state(self):
        return {"phi": self.d_phi.cpu().numpy(), "delta": self.d_delta.cpu().numpy(),
                "theta": to_bits(self.d_theta.cpu())}

    def oracle_state(self):
        return {"phi": self.phi, "delta": self.delta, "theta": self.theta}

    def check(self, what):
        assert_state_equal(self.gpu_state(), self.oracle_state(), what, self.wl.theta_dtype)
