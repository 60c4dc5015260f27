"""ctypes binding of libnoloco.so: same names as the C ABI, argument marshalling only.

Every step of the method runs in the library's kernels and host code. There is no
fallback: if the shared library has not been built, importing this module raises.
Device buffers are passed as anything with a ``data_ptr()`` method (torch tensors) or as
integer addresses; torch itself is only touched to look up the current stream.
"""
import ctypes as C
import os

import numpy as np

F32, BF16 = 0, 1
MAX_GROUP = 256

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libnoloco.so")


class NolocoError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {strerror(status)} (status {int(status)})")


class _Segment(C.Structure):
    _fields_ = [("offset", C.c_int64), ("numel", C.c_int64)]


class _Arena(C.Structure):
    _fields_ = [("phi", C.c_void_p), ("delta", C.c_void_p), ("theta", C.c_void_p),
                ("worker_stride", C.c_int64), ("W", C.c_int32), ("theta_dtype", C.c_int32),
                ("segments", C.POINTER(_Segment)), ("num_segments", C.c_int32)]


class _HParams(C.Structure):
    _fields_ = [("alpha", C.c_float), ("beta", C.c_float), ("gamma", C.c_float)]


class _Tuning(C.Structure):
    _fields_ = [("vectors_per_thread", C.c_int32), ("nontemporal", C.c_int32),
                ("group_major", C.c_int32), ("xcd_map", C.c_int32)]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2506_10911_amd.build` "
            "(there is no fallback path)")
    # The caller's device buffers come from PyTorch, so the library must bind to the HIP runtime
    # PyTorch has loaded, not to a second copy: import torch first, then the loader reuses it.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(_LIB_PATH)
    L.noloco_plan_groups.restype = C.c_int
    L.noloco_plan_groups.argtypes = [C.c_uint64, C.c_uint64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.noloco_plan_routes.restype = C.c_int
    L.noloco_plan_routes.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p]
    L.noloco_sim_tree_vs_pair.restype = C.c_int
    L.noloco_sim_tree_vs_pair.argtypes = [C.c_uint64, C.c_int32, C.c_double, C.c_double, C.c_int32, C.c_void_p]
    L.noloco_sim_barrier_penalty.restype = C.c_int
    L.noloco_sim_barrier_penalty.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_double, C.c_double, C.c_void_p]
    L.noloco_merge_segments.restype = C.c_int
    L.noloco_merge_segments.argtypes = [C.POINTER(_Segment), C.c_int32, C.c_int64,
                                        C.POINTER(_Segment), C.POINTER(C.c_int32)]
    L.noloco_launch_plan_create.restype = C.c_int
    L.noloco_launch_plan_create.argtypes = [C.POINTER(_Arena), C.POINTER(C.c_void_p)]
    L.noloco_launch_plan_destroy.restype = C.c_int
    L.noloco_launch_plan_destroy.argtypes = [C.c_void_p]
    L.noloco_launch_plan_info.restype = C.c_int
    L.noloco_launch_plan_info.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
    L.noloco_launch_plan_tune.restype = C.c_int
    L.noloco_launch_plan_tune.argtypes = [C.c_void_p, C.POINTER(_Tuning)]
    L.noloco_outer_step.restype = C.c_int
    L.noloco_outer_step.argtypes = [C.c_void_p, C.POINTER(_Arena), C.POINTER(_HParams),
                                    C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    L.noloco_replica_spread.restype = C.c_int
    L.noloco_replica_spread.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    L.noloco_replica_spread_noalloc.restype = C.c_int
    L.noloco_replica_spread_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    L.noloco_copy_probe.restype = C.c_int
    L.noloco_copy_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    L.noloco_read_probe.restype = C.c_int
    L.noloco_read_probe.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    L.noloco_fill_probe.restype = C.c_int
    L.noloco_fill_probe.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_void_p]
    L.noloco_strerror.restype = C.c_char_p
    L.noloco_strerror.argtypes = [C.c_int]
    return L


_lib = _load()

EXPORTS = ("noloco_plan_groups", "noloco_plan_routes", "noloco_merge_segments", "noloco_launch_plan_create",
           "noloco_launch_plan_destroy", "noloco_launch_plan_info", "noloco_launch_plan_tune",
           "noloco_outer_step", "noloco_replica_spread", "noloco_replica_spread_noalloc",
           "noloco_sim_tree_vs_pair",
           "noloco_sim_barrier_penalty", "noloco_copy_probe", "noloco_read_probe", "noloco_fill_probe",
           "noloco_strerror")


def library_path() -> str:
    return _LIB_PATH


def strerror(status) -> str:
    return _lib.noloco_strerror(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise NolocoError(status, where)


def _ptr(x) -> int:
    if x is None:
        return 0
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def _segment_array(segments):
    arr = (_Segment * max(len(segments), 1))()
    for i, (off, numel) in enumerate(segments):
        arr[i].offset, arr[i].numel = int(off), int(numel)
    return arr


def plan_groups(seed: int, step: int, W: int, n: int):
    """noloco_plan_groups: (members int32[W], group_offsets int32[W/n + 1])."""
    members = np.empty(max(int(W), 1), dtype=np.int32)
    groups = int(W) // int(n) if n and n > 0 else 0
    offsets = np.empty(max(groups, 0) + 1, dtype=np.int32)
    _check(_lib.noloco_plan_groups(seed, step, W, n, members.ctypes.data, offsets.ctypes.data),
           "noloco_plan_groups")
    return members[:W], offsets


def plan_routes(seed: int, step: int, microbatch: int, num_stages: int, W: int):
    """noloco_plan_routes: (send_to, recv_from), int32 [num_stages - 1, W] each."""
    b = max(int(num_stages) - 1, 0)
    send_to = np.full((b, max(int(W), 0)), -1, dtype=np.int32)
    recv_from = np.full((b, max(int(W), 0)), -1, dtype=np.int32)
    _check(_lib.noloco_plan_routes(seed, step, microbatch, num_stages, W, send_to.ctypes.data,
                                   recv_from.ctypes.data), "noloco_plan_routes")
    return send_to, recv_from


def merge_segments(segments, worker_stride: int):
    """noloco_merge_segments: list of (offset, numel) runs, sorted and merged."""
    seg = _segment_array(segments)
    out = (_Segment * max(len(segments), 1))()
    count = C.c_int32(0)
    _check(_lib.noloco_merge_segments(seg, len(segments), worker_stride, out, C.byref(count)),
           "noloco_merge_segments")
    return [(out[i].offset, out[i].numel) for i in range(count.value)]


class LaunchPlan:
    """noloco_launch_plan_create / _destroy / _info / _tune for one arena layout."""

    def __init__(self, phi, delta, theta, worker_stride: int, W: int, theta_dtype: int, segments):
        self._handle = C.c_void_p(0)
        self.worker_stride, self.W, self.theta_dtype = int(worker_stride), int(W), int(theta_dtype)
        self._segments = _segment_array(segments)
        self._num_segments = len(segments)
        self._arenas, self._hps = {}, {}       # argument structs by value, never modified once built
        arena = self._arena(phi, delta, theta)
        _check(_lib.noloco_launch_plan_create(C.byref(arena), C.byref(self._handle)),
               "noloco_launch_plan_create")

    def _arena(self, phi, delta, theta):
        """The noloco_arena struct for these base pointers. Structs are kept by pointer triple and
        never changed after they are built, so threads sharing a plan cannot disturb each other."""
        key = (_ptr(phi), _ptr(delta), _ptr(theta))
        arena = self._arenas.get(key)
        if arena is None:
            if len(self._arenas) >= 16:
                self._arenas.clear()
            arena = _Arena(*key, self.worker_stride, self.W, self.theta_dtype, self._segments, self._num_segments)
            self._arenas[key] = arena
        return arena

    def _hparams(self, hparams):
        key = (float(hparams[0]), float(hparams[1]), float(hparams[2]))
        hp = self._hps.get(key)
        if hp is None:
            if len(self._hps) >= 16:
                self._hps.clear()
            hp = _HParams(*key)
            self._hps[key] = hp
        return hp

    def info(self):
        e, r, t, te = C.c_int64(), C.c_int32(), C.c_int64(), C.c_int32()
        _check(_lib.noloco_launch_plan_info(self._handle, C.byref(e), C.byref(r), C.byref(t), C.byref(te)),
               "noloco_launch_plan_info")
        return {"elements_per_worker": e.value, "num_runs": r.value, "num_tiles": t.value,
                "tile_elems": te.value}

    def tune(self, vectors_per_thread=-1, nontemporal=-1, group_major=-1, xcd_map=-1):
        t = _Tuning(int(vectors_per_thread), int(nontemporal), int(group_major), int(xcd_map))
        _check(_lib.noloco_launch_plan_tune(self._handle, C.byref(t)), "noloco_launch_plan_tune")

    def destroy(self):
        if self._handle:
            handle, self._handle = self._handle, C.c_void_p(0)
            _check(_lib.noloco_launch_plan_destroy(handle), "noloco_launch_plan_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _int32_address(values):
    a = np.ascontiguousarray(values, dtype=np.int32)
    return a, a.__array_interface__["data"][0]


def outer_step(plan: LaunchPlan, phi, delta, theta, hparams, members, group_offsets, stream=None):
    """noloco_outer_step: one fused outer step in place, enqueued on `stream` (default: torch's current)."""
    arena = plan._arena(phi, delta, theta)
    hp = plan._hparams(hparams)
    m, m_at = _int32_address(members)
    o, o_at = _int32_address(group_offsets)
    status = _lib.noloco_outer_step(plan._handle, C.byref(arena), C.byref(hp), m_at, o_at, len(o) - 1,
                                    _stream(stream))
    if status != 0:
        raise NolocoError(status, "noloco_outer_step")


def replica_spread(plan: LaunchPlan, x, x_dtype: int, out_std, stream=None):
    """noloco_replica_spread: out_std (device float64 [num_segments + 1]) <- pooled std across the W rows of x."""
    _check(_lib.noloco_replica_spread(plan._handle, _ptr(x), int(x_dtype), _ptr(out_std), _stream(stream)),
           "noloco_replica_spread")


def replica_spread_noalloc(plan: LaunchPlan, x, x_dtype: int, out_std, stream=None):
    """noloco_replica_spread_noalloc: the same pass staged in the library's static per-GPU array."""
    _check(_lib.noloco_replica_spread_noalloc(plan._handle, _ptr(x), int(x_dtype), _ptr(out_std),
                                              _stream(stream)), "noloco_replica_spread_noalloc")


def copy_probe(dst, src, nbytes: int, stream=None):
    """noloco_copy_probe: plain device copy of nbytes (measurement aid)."""
    _check(_lib.noloco_copy_probe(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)),
           "noloco_copy_probe")


def read_probe(src, nbytes: int, sink, stream=None):
    """noloco_read_probe: streams nbytes from src, writes nothing (measurement aid)."""
    _check(_lib.noloco_read_probe(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)),
           "noloco_read_probe")


def fill_probe(dst, nbytes: int, value: float = 0.0, stream=None):
    """noloco_fill_probe: streams nbytes of `value` into dst (measurement aid)."""
    _check(_lib.noloco_fill_probe(_ptr(dst), int(nbytes), float(value), _stream(stream)),
           "noloco_fill_probe")


def sim_tree_vs_pair(seed: int, W: int, mu: float, sigma: float, trials: int):
    """noloco_sim_tree_vs_pair: dict with mean tree / pair times and their standard errors."""
    out = np.zeros(4, dtype=np.float64)
    _check(_lib.noloco_sim_tree_vs_pair(seed, W, mu, sigma, trials, out.ctypes.data),
           "noloco_sim_tree_vs_pair")
    return {"tree": out[0], "tree_se": out[1], "pair": out[2], "pair_se": out[3]}


def sim_barrier_penalty(seed: int, W: int, n: int, inner_steps: int, outer_steps: int, mu: float, sigma: float):
    """noloco_sim_barrier_penalty: (finishing time with a global barrier, with subgroup sync)."""
    out = np.zeros(2, dtype=np.float64)
    _check(_lib.noloco_sim_barrier_penalty(seed, W, n, inner_steps, outer_steps, mu, sigma,
                                           out.ctypes.data), "noloco_sim_barrier_penalty")
    return float(out[0]), float(out[1])
