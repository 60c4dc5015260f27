"""ctypes front end of the CPU oracle (oracle/noloco_oracle.cpp).

TEST INFRASTRUCTURE. Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of
bench.py may import this package; the product (paper_2506_10911_amd) never does, and
this package never imports the product.

Every function here only marshals numpy arrays into the C++ routines; the arithmetic of
the method (arxiv 2506.10911, Eq. 1-3 and the subgroup sampling) is all in the .cpp file.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def load(path):
    """Opens one build of the oracle and declares its signatures (tests load mutated builds this way)."""
    L = C.CDLL(path)
    L.oracle_mix64.restype = C.c_uint64
    L.oracle_mix64.argtypes = [C.c_uint64]
    L.oracle_bounded16.restype = C.c_int32
    L.oracle_bounded16.argtypes = [C.c_uint16, C.c_uint16]
    L.oracle_draw.restype = C.c_uint64
    L.oracle_draw.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
    L.oracle_plan_groups.restype = C.c_int
    L.oracle_plan_groups.argtypes = [C.c_uint64, C.c_uint64, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p]
    L.oracle_bf16_narrow.restype = None
    L.oracle_bf16_narrow.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
    L.oracle_bf16_widen.restype = None
    L.oracle_bf16_widen.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
    L.oracle_outer_step_f32.restype = C.c_int
    L.oracle_outer_step_f32.argtypes = [
        C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32,
        C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_float, C.c_float,
        C.c_void_p, C.c_void_p, C.c_int32]
    L.oracle_outer_step_f64.restype = C.c_int
    L.oracle_outer_step_f64.argtypes = [
        C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
        C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_double, C.c_double,
        C.c_void_p, C.c_void_p, C.c_int32]
    L.oracle_plan_routes.restype = C.c_int
    L.oracle_plan_routes.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p]
    L.oracle_replica_spread.restype = C.c_int
    L.oracle_replica_spread.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_void_p,
                                        C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load(_build.ensure_built())
    return _lib


def mix64(z: int) -> int:
    return int(lib().oracle_mix64(C.c_uint64(z & (2**64 - 1))))


def bounded16(r: int, m: int) -> int:
    """16-bit analogue of the bounded draw's accept rule: r % m, or -1 if r is rejected."""
    return int(lib().oracle_bounded16(r, m))


def draw(seed: int, step: int, k: int) -> int:
    return int(lib().oracle_draw(seed, step, k))


def plan_groups(seed: int, step: int, W: int, n: int):
    """Returns (members int32[W], group_offsets int32[W/n+1]); raises ValueError on a bad (W, n)."""
    members = np.empty(max(W, 1), dtype=np.int32)
    offsets = np.empty(max(W // max(n, 1), 0) + 1 if n >= 1 else 1, dtype=np.int32)
    rc = lib().oracle_plan_groups(seed, step, W, n, members.ctypes.data, offsets.ctypes.data)
    if rc != 0:
        raise ValueError(f"no partition of {W} workers into groups of {n}")
    return members[:W], offsets


def plan_routes(seed: int, step: int, microbatch: int, num_stages: int, W: int):
    """Returns (send_to, recv_from), int32 [num_stages - 1, W] each; raises ValueError on bad sizes."""
    b = max(num_stages - 1, 0)
    send_to = np.full((b, max(W, 0)), -1, dtype=np.int32)
    recv_from = np.full((b, max(W, 0)), -1, dtype=np.int32)
    rc = lib().oracle_plan_routes(seed, step, microbatch, num_stages, W, send_to.ctypes.data,
                                  recv_from.ctypes.data)
    if rc != 0:
        raise ValueError("bad routing sizes")
    return send_to, recv_from


def bf16_narrow(x) -> np.ndarray:
    """float32 array -> bf16 bit patterns (uint16), round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_bf16_narrow(x.ctypes.data, out.ctypes.data, x.size)
    return out


def bf16_widen(h) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 array (exact)."""
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().oracle_bf16_widen(h.ctypes.data, out.ctypes.data, h.size)
    return out


def _segs(segments, stride):
    if segments is None:
        segments = [(0, stride)]
    off = np.ascontiguousarray([s[0] for s in segments], dtype=np.int64)
    ln = np.ascontiguousarray([s[1] for s in segments], dtype=np.int64)
    return off, ln


def _groups(members, group_offsets):
    m = np.ascontiguousarray(members, dtype=np.int32)
    o = np.ascontiguousarray(group_offsets, dtype=np.int32)
    return m, o


def outer_step_f32(phi, delta, theta, hp, members, group_offsets, segments=None):
    """One outer step in binary32, in place.

    phi, delta: float32 [W, stride], C-contiguous. theta: float32 [W, stride], or uint16
    [W, stride] holding bf16 bit patterns. hp = (alpha, beta, gamma). segments: list of
    (offset, numel) inside a row (default: the whole row).
    """
    assert phi.dtype == np.float32 and delta.dtype == np.float32
    assert phi.flags.c_contiguous and delta.flags.c_contiguous and theta.flags.c_contiguous
    assert phi.shape == delta.shape == theta.shape and phi.ndim == 2
    if theta.dtype == np.uint16:
        is_bf16 = 1
    else:
        assert theta.dtype == np.float32
        is_bf16 = 0
    W, stride = phi.shape
    off, ln = _segs(segments, stride)
    assert ((off >= 0) & (off + ln <= stride)).all()
    m, o = _groups(members, group_offsets)
    rc = lib().oracle_outer_step_f32(
        phi.ctypes.data, delta.ctypes.data, theta.ctypes.data, is_bf16, stride, W,
        off.ctypes.data, ln.ctypes.data, len(off), hp[0], hp[1], hp[2],
        m.ctypes.data, o.ctypes.data, len(o) - 1)
    if rc != 0:
        raise ValueError("groups are not a partition of a subset of the workers")


def outer_step_f64(phi, delta, theta, hp, members, group_offsets, segments=None):
    """The same step in binary64 (all three arrays float64 [W, stride]), in place."""
    for a in (phi, delta, theta):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    assert phi.shape == delta.shape == theta.shape and phi.ndim == 2
    W, stride = phi.shape
    off, ln = _segs(segments, stride)
    assert ((off >= 0) & (off + ln <= stride)).all()
    m, o = _groups(members, group_offsets)
    rc = lib().oracle_outer_step_f64(
        phi.ctypes.data, delta.ctypes.data, theta.ctypes.data, stride, W,
        off.ctypes.data, ln.ctypes.data, len(off), hp[0], hp[1], hp[2],
        m.ctypes.data, o.ctypes.data, len(o) - 1)
    if rc != 0:
        raise ValueError("groups are not a partition of a subset of the workers")


def replica_spread(x, segments=None, binary32=False):
    """Pooled standard deviation across the W rows of x (float32 or bf16 bits as uint16, [W, stride]).

    Returns float64 [num_segments + 1]: one value per segment, then the value over all segments.
    binary32=False is the definition in binary64; True does the per-element arithmetic in binary32.
    """
    assert x.ndim == 2 and x.flags.c_contiguous and x.dtype in (np.float32, np.uint16)
    W, stride = x.shape
    off, ln = _segs(segments, stride)
    assert ((off >= 0) & (off + ln <= stride)).all()
    out = np.empty(len(off) + 1, dtype=np.float64)
    rc = lib().oracle_replica_spread(x.ctypes.data, int(x.dtype == np.uint16), stride, W,
                                     off.ctypes.data, ln.ctypes.data, len(off), int(binary32),
                                     out.ctypes.data)
    if rc != 0:
        raise ValueError("bad arguments")
    return out
