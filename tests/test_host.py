"""CPU-only checks of the product's host side: the library loads, exports what the header
declares, and its planner and segment merger agree with the oracle / with plain reasoning."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from conftest import ROOT

import paper_2506_10911_amd as nl

nl.library_path()          # loads libnoloco.so now; a missing library is an error, not a skip


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "noloco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(noloco_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"noloco_plan_groups", "noloco_outer_step", "noloco_launch_plan_create"} <= set(names)
    lib = ctypes.CDLL(nl.library_path())
    for name in names:
        assert hasattr(lib, name), f"{name} declared in noloco.h but not exported"
    assert set(nl.binding.EXPORTS) == set(names)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 and as C++ on its own."""
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "noloco.h"\n'
                   'int probe(void) { noloco_hparams h = {0.9f, 0.7f, 1.0f}; noloco_segment s = {0, 4};\n'
                   '  noloco_tuning t = {-1, -1, -1, -1}; (void)h; (void)s; (void)t;\n'
                   '  return (int)sizeof(noloco_arena) + NOLOCO_MAX_GROUP + (int)NOLOCO_BF16; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, "-c", str(src),
                    "-o", str(tmp_path / "use_c.o")], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-I", inc, "-x", "c++", "-c", str(src),
                    "-o", str(tmp_path / "use_cpp.o")], check=True)


def test_strerror_covers_all_codes():
    seen = {nl.strerror(c) for c in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert nl.strerror(99) == "unknown status"


def divisors(W):
    return [d for d in range(1, W + 1) if W % d == 0]


def test_planner_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(123)
    checked = 0
    for W in range(1, 65):
        for n in divisors(W):
            for _ in range(6):
                seed = int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2))
                step = int(rng.integers(0, 2**40))
                a_m, a_o = nl.plan_groups(seed, step, W, n)
                b_m, b_o = oracle.plan_groups(seed, step, W, n)
                assert a_m.tolist() == b_m.tolist() and a_o.tolist() == b_o.tolist()
                checked += 1
    for seed in range(40):                         # the benchmark's own streams
        for step in range(25):
            for W, n in [(4, 2), (8, 2), (16, 2), (64, 2), (64, 4), (64, 8), (1024, 2), (96, 3)]:
                a_m, a_o = nl.plan_groups(seed, step, W, n)
                b_m, b_o = oracle.plan_groups(seed, step, W, n)
                assert a_m.tolist() == b_m.tolist() and a_o.tolist() == b_o.tolist()
                checked += 1
    assert checked > 9000


def test_planner_errors():
    for W, n, status in [(8, 3, 3), (8, 0, 3), (8, 9, 3), (0, 1, 2), (-4, 2, 2)]:
        with pytest.raises(nl.NolocoError) as e:
            nl.plan_groups(0, 0, W, n)
        assert e.value.status == status
    lib = ctypes.CDLL(nl.library_path())
    lib.noloco_plan_groups.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_void_p, ctypes.c_void_p]
    assert lib.noloco_plan_groups(0, 0, 4, 2, None, None) == 1


def test_route_planner_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(321)
    checked = 0
    for stages in (1, 2, 3, 4, 8):
        for W in (1, 2, 3, 8, 16, 64, 257):
            for _ in range(12):
                seed, step, mb = (int(rng.integers(0, 2**62)) for _ in range(3))
                a = nl.plan_routes(seed, step, mb, stages, W)
                b = oracle.plan_routes(seed, step, mb, stages, W)
                assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
                checked += 1
    for seed in range(10):
        for step in range(20):
            for mb in range(4):
                a = nl.plan_routes(seed, step, mb, 4, 16)
                b = oracle.plan_routes(seed, step, mb, 4, 16)
                assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
                checked += 1
    assert checked > 1000
    for stages, W, status in [(0, 4, 2), (2, 0, 2)]:
        with pytest.raises(nl.NolocoError) as e:
            nl.plan_routes(0, 0, 0, stages, W)
        assert e.value.status == status


def test_merge_segments():
    assert nl.merge_segments([], 64) == []
    assert nl.merge_segments([(0, 64)], 64) == [(0, 64)]
    assert nl.merge_segments([(10, 5), (0, 10), (20, 3), (15, 0), (23, 1)], 64) == [(0, 15), (20, 4)]
    # tight-packed odd sizes collapse into one run
    sizes = [7, 1, 1001, 33, 64]
    segs, off = [], 5
    for s in sizes:
        segs.append((off, s))
        off += s
    assert nl.merge_segments(segs[::-1], 2048) == [(5, sum(sizes))]
    for bad, status in [([(0, 10), (9, 3)], 4), ([(60, 5)], 4), ([(0, 65)], 4), ([(-1, 3)], 2),
                        ([(3, -1)], 2), ([(5, 5), (5, 1)], 4)]:
        with pytest.raises(nl.NolocoError) as e:
            nl.merge_segments(bad, 64)
        assert e.value.status == status, bad
