"""Planted mistakes: each single-line mutation of the oracle's outer step must be caught by the
pins (hand examples, brute force over partitions, DiLoCo reduction, bf16 step).

The mutants are compiled from the oracle's source on the CPU and loaded in place of the real
build; nothing here touches a GPU or the HIP library.
"""
import os
import subprocess

import pytest

import oracle
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
