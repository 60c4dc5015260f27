"""Planted mistakes: each single-line mutation of the oracle's outer step must be caught by the
pins (hand examples, brute force over partitions, DiLoCo reduction, bf16 step), and each
single-line mutation of its planners by theirs (exhaustive 16-bit bounded draw, sorted-partition
validity, uniformity over all partitions, permutation/inverse of the routes).

The mutants are compiled from the oracle's source on the CPU and loaded in place of the real
build; nothing here touches a GPU or the HIP library.
"""
import os
import subprocess

import pytest

import oracle
import test_oracle_planner as planner_pins
import test_oracle_routes as route_pins
import test_oracle_step as pins
from conftest import read_hand_examples

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "noloco_oracle.cpp")

MUTANTS = {
    "outer_gradient_sign": ("const T Delta = p - load_theta(at);", "const T Delta = load_theta(at) - p;"),
    "pull_term_dropped": ("const T d_new = (t1 - t2) - t3;", "const T d_new = (t1 - t2);"),
    "pull_term_sign": ("const T d_new = (t1 - t2) - t3;", "const T d_new = (t1 - t2) + t3;"),
    "gradient_term_sign": ("const T d_new = (t1 - t2) - t3;", "const T d_new = (t1 + t2) - t3;"),
    "sum_not_mean_Delta": ("const T mean_Delta = sum_Delta * inv_n;", "const T mean_Delta = sum_Delta;"),
    "sum_not_mean_phi": ("const T mean_phi = sum_phi * inv_n;", "const T mean_phi = sum_phi;"),
    "pull_wrong_member": ("gamma * (phi_old[a] - mean_phi)", "gamma * (phi_old[0] - mean_phi)"),
    "alpha_beta_swapped": ("const T t1 = alpha * delta[at];", "const T t1 = beta * delta[at];"),
    "momentum_forgotten": ("const T t1 = alpha * delta[at];", "const T t1 = T(0) * delta[at];"),
    "update_sign": ("const T p_new = phi_old[a] + d_new;", "const T p_new = phi_old[a] - d_new;"),
    "update_uses_mean": ("const T p_new = phi_old[a] + d_new;", "const T p_new = mean_phi + d_new;"),
    "restart_dropped": ("store_theta(at, p_new);", "(void)store_theta;"),
    "self_excluded": ("else        { sum_Delta = sum_Delta + Delta; sum_phi = sum_phi + p; }",
                      "else if (a + 1 < n) { sum_Delta = sum_Delta + Delta; sum_phi = sum_phi + p; }"),
    "bf16_truncates": ("u += 0x7FFFu + lsb;", "u += 0u * lsb;"),
}


# Mistakes in the subgroup planner and the routing planner (oracle_plan_groups, oracle_plan_routes).
PLANNER_MUTANTS = {
    # partner drawn from all W positions instead of [0, i]: still a permutation, no longer uniform
    "groups_shuffle_partner_from_all": (
        """    int32_t j = static_cast<int32_t>(s.bounded(static_cast<uint64_t>(i) + 1));
    std::swap(members[i], members[j]);""",
        """    int32_t j = static_cast<int32_t>(s.bounded(static_cast<uint64_t>(W)));
    std::swap(members[i], members[j]);"""),
    "bounded_draw_never_rejects": ("return r >= reject_below;", "return r >= reject_below || true;"),
    "bounded_draw_rejects_wrong_side": ("return r >= reject_below;", "return r > reject_below;"),
    "chunk_left_unsorted": ("std::sort(members + g * n, members + (g + 1) * n);", "(void)0;"),
    "chunk_offsets_off": ("group_offsets[g] = g * n;", "group_offsets[g] = g * n + (g > 0);"),
    "routes_inverse_is_not_the_inverse": ("for (int32_t r = 0; r < W; ++r) from[to[r]] = r;",
                                          "for (int32_t r = 0; r < W; ++r) from[r] = to[r];"),
    "routes_partner_from_all": (
        """      int32_t j = static_cast<int32_t>(s.bounded(static_cast<uint64_t>(i) + 1));
      std::swap(to[i], to[j]);""",
        """      int32_t j = static_cast<int32_t>(s.bounded(static_cast<uint64_t>(W)));
      std::swap(to[i], to[j]);"""),
    "routes_same_stream_for_every_boundary": ("mix64(batch_key ^ mix64(static_cast<uint64_t>(b) + 3 * kGolden))",
                                              "mix64(batch_key ^ mix64(3 * kGolden))"),
}


def run_planner_pins():
    planner_pins.test_bounded_draw_rule_is_exactly_uniform_on_a_16_bit_word()
    for W in (4, 6, 12, 30):
        planner_pins.test_every_plan_is_a_partition_into_sorted_groups(W)
    for W, n, count in ((4, 2, 3), (6, 2, 15), (6, 3, 10), (8, 4, 35)):
        planner_pins.test_partitions_are_uniform(W, n, count)
    planner_pins.test_each_worker_meets_every_peer_equally_often()
    for stages, W in ((2, 2), (2, 8), (3, 5)):
        route_pins.test_every_boundary_is_a_permutation_with_its_inverse(stages, W)
    for W, limit in ((3, 20.5), (4, 49.7)):
        route_pins.test_permutations_are_uniform(W, limit)
    route_pins.test_boundaries_are_independent()


def run_pins():
    for case in read_hand_examples():
        for mode in ("f64", "f32", "bf16"):
            pins.test_hand_examples(case, mode)
    pins.test_brute_force_all_partitions(4, 2)
    pins.test_brute_force_all_partitions(6, 3)
    pins.test_diloco_reduction_against_textbook_momentum()
    pins.test_bf16_theta_step()
    pins.test_bf16_narrow_matches_library_cast_and_ties_to_even()


def test_unmutated_oracle_passes_the_same_pins():
    run_pins()


def test_unmutated_oracle_passes_the_planner_pins():
    run_planner_pins()


@pytest.mark.parametrize("name", sorted(PLANNER_MUTANTS))
def test_planner_mutant_is_caught(name, tmp_path, monkeypatch):
    old, new = PLANNER_MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "mutant.cpp"
    src.write_text(text.replace(old, new))
    so = tmp_path / f"mutant_{name}.so"
    subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-shared", "-fPIC",
                    "-o", str(so), str(src)], check=True)
    monkeypatch.setattr(oracle, "_lib", oracle.load(str(so)))
    with pytest.raises(AssertionError):
        run_planner_pins()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "mutant.cpp"
    src.write_text(text.replace(old, new))
    so = tmp_path / f"mutant_{name}.so"
    subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-shared", "-fPIC",
                    "-o", str(so), str(src)], check=True)
    monkeypatch.setattr(oracle, "_lib", oracle.load(str(so)))
    with pytest.raises(AssertionError):
        run_pins()
