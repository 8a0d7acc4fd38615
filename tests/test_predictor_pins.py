"""Pins for the pipeline-simulator oracle: the numbers Section 4.3 prints, the closed form of the uniform
pipeline, brute-force checks of the schedule's constraints, and invariants."""
import itertools
import os
import random

import pytest

from oracle import predictor_oracle as P

GOLD = {}
for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_section_4_3_numbers.txt")):
    if line.strip() and not line.startswith("#"):
        k, *v = line.split()
        GOLD[k] = [float(t) for t in v] if len(v) > 1 else float(v[0])


def test_theoretical_mfu_is_the_device_weighted_mean_printed_in_the_paper():
    assert P.weighted_mean([GOLD["mfu_nvidia"], GOLD["mfu_accel_a"]], [1, 1]) == pytest.approx(GOLD["mfu_theory_nvidia_a"], abs=5e-3)
    assert P.weighted_mean([GOLD["mfu_amd"], GOLD["mfu_accel_b"]], [1, 1]) == pytest.approx(GOLD["mfu_theory_amd_b"], abs=5e-3)
    # the 120-node cluster: 128 AMD + 640 of the other type
    c = [GOLD["n_amd"], GOLD["n_accel_large"]]
    assert P.weighted_mean([GOLD["mfu_amd"], GOLD["mfu_accel_c"]], c) == pytest.approx(GOLD["mfu_theory_amd_c"], abs=5e-3)
    th = P.weighted_mean([GOLD["tflops_amd_70b"], GOLD["tflops_accel_a_70b"]], c)
    assert 100 * GOLD["tflops_mixed_70b"] / th == pytest.approx(GOLD["ratio_mixed_70b"], abs=2e-2)
    assert 100 * GOLD["mfu_mixed_nvidia_a"] / GOLD["mfu_theory_nvidia_a"] == pytest.approx(GOLD["ratio_nvidia_a"], abs=1e-2)
    assert 100 * GOLD["mfu_mixed_amd_b"] / GOLD["mfu_theory_amd_b"] == pytest.approx(GOLD["ratio_amd_b"], abs=2e-2)
    assert 100 * GOLD["mfu_mixed_amd_c"] / GOLD["mfu_theory_amd_c"] == pytest.approx(GOLD["ratio_amd_c"], abs=1e-2)
    # a swapped weight vector must not reproduce the printed value
    assert abs(P.weighted_mean([GOLD["mfu_amd"], GOLD["mfu_accel_c"]], c[::-1]) - GOLD["mfu_theory_amd_c"]) > 1.0


def test_printed_end_to_end_improvement_and_stage_vectors():
    assert 100 * (GOLD["e2e_uniform_ms"] - GOLD["e2e_nonuniform_ms"]) / GOLD["e2e_uniform_ms"] == pytest.approx(
        GOLD["e2e_improvement_percent"], abs=5e-3)
    assert sum(GOLD["stages_nonuniform"]) == 80 == GOLD["stages_uniform_layers"] * GOLD["stages_uniform_pp"]   # Llama2-70B, Table 1


def test_eq1_eq3_values():
    assert P.p2p_bytes(1, 4096, 12288) == 100663296            # Eq. (3)
    assert P.p2p_bytes(2, 2048, 8192) == 2 * 2048 * 8192 * 2
    # Eq. (1): L*G / (S*T)
    assert P.tgs(4096, 512, 768, 3.0) == pytest.approx(4096 * 512 / 768 / 3.0)


def test_uniform_pipeline_closed_form():
    # equal stages, free links: (M + P - 1) (tf + tb), the textbook makespan of GPipe and 1F1B alike
    for Pn, M, tf, tb in [(1, 1, 2.0, 3.0), (4, 8, 1.0, 2.0), (6, 3, 0.5, 1.25), (3, 16, 2.0, 4.0), (5, 5, 1.0, 1.0)]:
        it, busy, _ = P.simulate([tf] * Pn, [tb] * Pn, [0.0] * (Pn - 1), M)
        assert it == pytest.approx((M + Pn - 1) * (tf + tb))
        assert busy == [pytest.approx(M * (tf + tb))] * Pn


def test_single_slow_stage_bounds_the_iteration():
    tf, tb = [1.0, 1.0, 3.0, 1.0], [2.0, 2.0, 6.0, 2.0]
    M = 32
    it, busy, _ = P.simulate(tf, tb, [0.0] * 3, M)
    assert it >= max(busy)
    assert it <= max(busy) + sum(tf) + sum(tb)        # fill and drain cost at most one pass through all stages
    # balancing the same total work lowers the time
    tot_f, tot_b = sum(tf), sum(tb)
    it_bal, _, _ = P.simulate([tot_f / 4] * 4, [tot_b / 4] * 4, [0.0] * 3, M)
    assert it_bal < it


def test_link_time_delays_by_the_round_trip_through_the_pipeline():
    Pn, M, tf, tb, c = 4, 6, 1.0, 2.0, 0.25
    it0, _, _ = P.simulate([tf] * Pn, [tb] * Pn, [0.0] * (Pn - 1), M)
    it1, _, _ = P.simulate([tf] * Pn, [tb] * Pn, [c] * (Pn - 1), M)
    assert it1 >= it0 + 2 * (Pn - 1) * c - 1e-12       # first forward down and last backward up cross every link
    assert it1 <= it0 + 2 * (Pn - 1) * c * M


def brute_force_makespan(tf, tb, link, M):
    """Longest path through the dependency graph: program order inside a stage and the two data edges."""
    Pn = len(tf)
    orders = [P.one_f_one_b_order(p, Pn, M) for p in range(Pn)]
    finish = {}

    def fin(p, i):
        key = (p, i)
        if key in finish:
            return finish[key]
        kind, m = orders[p][i]
        t = fin(p, i - 1) if i > 0 else 0.0
        if kind == "F" and p > 0:
            j = orders[p - 1].index(("F", m))
            t = max(t, fin(p - 1, j) + link[p - 1])
        if kind == "B" and p < Pn - 1:
            j = orders[p + 1].index(("B", m))
            t = max(t, fin(p + 1, j) + link[p])
        finish[key] = t + (tf[p] if kind == "F" else tb[p])
        return finish[key]

    return max(fin(p, len(orders[p]) - 1) for p in range(Pn))


def test_simulation_equals_longest_path_on_random_small_pipelines():
    rng = random.Random(7)
    for _ in range(60):
        Pn, M = rng.randint(1, 5), rng.randint(1, 7)
        tf = [rng.uniform(0.2, 3.0) for _ in range(Pn)]
        tb = [rng.uniform(0.2, 5.0) for _ in range(Pn)]
        link = [rng.uniform(0.0, 1.0) for _ in range(Pn - 1)]
        it, _, _ = P.simulate(tf, tb, link, M)
        assert it == pytest.approx(brute_force_makespan(tf, tb, link, M))


def test_order_has_every_operation_once_and_backward_after_forward():
    for Pn, M in itertools.product(range(1, 6), range(1, 9)):
        for p in range(Pn):
            ops = P.one_f_one_b_order(p, Pn, M)
            assert sorted(ops) == sorted([("F", m) for m in range(M)] + [("B", m) for m in range(M)])
            for m in range(M):
                assert ops.index(("F", m)) < ops.index(("B", m))
            assert [m for k, m in ops if k == "B"] == list(range(M))      # gradients are summed in ascending order
            assert P.live_micro_batches(p, Pn, M) == min(M, Pn - p)       # at most "the number of stages" (Section 2.3)


def test_stage_memory():
    # 2 layers, 3 live micro-batches
    assert P.stage_peak_bytes(1, 4, 8, 2, 10, 20, 60, 7) == 2 * 90 + 3 * 2 * 7
    assert P.stage_peak_bytes(0, 4, 2, 1, 10, 20, 60, 7) == 90 + 2 * 7


def test_mfu_definition():
    # 2 devices of peak 100 and 300 TFLOP/s run 4e14 flop in 1 s: 200 TFLOP/s per device over a mean peak of 200
    assert P.mfu(4e14, 1.0, [100.0, 300.0], [1, 1]) == pytest.approx(1.0)
    assert P.mfu(4e14, 2.0, [100.0, 300.0], [1, 1]) == pytest.approx(0.5)
