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


# ---- the exhaustive planner (Section 3.3, both rules): compositions, link placement, order choice ----------------

def test_compositions_are_the_ordered_positive_splits():
    from math import comb
    assert list(P.compositions(4, 2)) == [(1, 3), (2, 2), (3, 1)]
    assert list(P.compositions(3, 3)) == [(1, 1, 1)]
    assert list(P.compositions(2, 3)) == []
    assert list(P.compositions(5, 1)) == [(5,)]
    for n, p in [(5, 2), (6, 3), (7, 4), (9, 5), (10, 3)]:
        c = list(P.compositions(n, p))
        assert len(c) == comb(n - 1, p - 1)          # stars and bars
        assert len(set(c)) == len(c)
        assert all(len(t) == p and sum(t) == n and min(t) >= 1 for t in c)


def _group(tf, tb, link, mem=0, saved=0):
    return dict(fwd_ms=tf, bwd_ms=tb, link_ms=link, weight_bytes=0, grad_bytes=0, optimizer_bytes=0,
                saved_act_bytes=saved, memory_bytes=mem)


def test_link_vector_of_each_group_order():
    g = [_group(1.0, 2.0, 0.25), _group(1.0, 2.0, 0.5), _group(1.0, 2.0, 0.125)]
    X = 7.0
    # counts (2, 1): the pair's own link sits between its two stages, the cross link where the groups meet
    st, ln = P.pipeline_of_order(g[:2], [2, 1], (0, 1), X)
    assert [s is g[0] for s in st] == [True, True, False] and ln == [0.25, X]
    st, ln = P.pipeline_of_order(g[:2], [2, 1], (1, 0), X)
    assert [s is g[1] for s in st] == [True, False, False] and ln == [X, 0.25]
    # counts (1, 2)
    assert P.pipeline_of_order(g[:2], [1, 2], (0, 1), X)[1] == [X, 0.5]
    assert P.pipeline_of_order(g[:2], [1, 2], (1, 0), X)[1] == [0.5, X]
    # three groups, counts (2, 1, 3), order (2, 0, 1): 3 + 2 + 1 stages
    st, ln = P.pipeline_of_order(g, [2, 1, 3], (2, 0, 1), X)
    assert [g.index(s) for s in st] == [2, 2, 2, 0, 0, 1]
    assert ln == [0.125, 0.125, X, 0.25, X]
    # a single group has no cross link at all
    assert P.pipeline_of_order(g[:1], [4], (0,), X)[1] == [0.25] * 3


def test_position_of_the_slow_cross_link_alone_decides_the_order():
    # Three stages of one layer each (3 layers: the only split is 1+1+1), every stage forward 1, backward 2,
    # 3 micro-batches, free links inside a group, cross link 5.  1F1B programs:
    #   stage 0: F0 F1 F2 B0 B1 B2   stage 1: F0 F1 B0 F2 B1 B2   stage 2: F0 B0 F1 B1 F2 B2
    # Links (5, 0), i.e. the lone stage first:
    #   stage 0 forwards end at 1, 2, 3.  Stage 1: F0 6-7, F1 7-8.  Stage 2: F0 7-8, B0 8-10, F1 10-11, B1 11-13.
    #   Stage 1: B0 10-12, F2 (arrived at 8) 12-13, B1 13-15.  Stage 2: F2 13-14, B2 14-16.  Stage 1: B2 16-18.
    #   Stage 0: B0 arrives 12+5=17, 17-19; B1 arrives 20, 20-22; B2 arrives 23, 23-25.               => 25
    # Links (0, 5), i.e. the lone stage last:
    #   Stage 1: F0 1-2, F1 2-3.  Stage 2: F0 arrives 7, 7-8, B0 8-10, F1 (arrived 8) 10-11, B1 11-13.
    #   Stage 1: B0 arrives 15, 15-17; F2 17-18; B1 arrives 18, 18-20.  Stage 2: F2 arrives 23, 23-24, B2 24-26.
    #   Stage 1: B2 arrives 31, 31-33.  Stage 0: B0 17-19, B1 20-22, B2 33-35.                        => 35
    assert P.simulate([1.0] * 3, [2.0] * 3, [5.0, 0.0], 3)[0] == pytest.approx(25.0)
    assert P.simulate([1.0] * 3, [2.0] * 3, [0.0, 5.0], 3)[0] == pytest.approx(35.0)
    same = _group(1.0, 2.0, 0.0)
    # group 0 is the pair: putting it first places the slow link last (35); the planner must turn the order round,
    # which is not the first order it tries
    order, layers, it = P.best_order_and_split([same, dict(same)], [2, 1], 5.0, 3, 3)
    assert (order, layers, it) == ([1, 0], [1, 1, 1], pytest.approx(25.0))
    # group 0 is the lone stage: the first order already has the slow link first
    order, layers, it = P.best_order_and_split([same, dict(same)], [1, 2], 5.0, 3, 3)
    assert (order, layers, it) == ([0, 1], [1, 1, 1], pytest.approx(25.0))


def test_order_choice_with_a_slow_type_and_distinct_links_hand_worked():
    # counts (1, 2), 3 layers (1+1+1), 2 micro-batches; type 0: forward 1, backward 2; type 1: forward 2, backward 4,
    # link i between its two stages; cross link c.  Programs: stages 0, 1: F0 F1 B0 B1; stage 2: F0 B0 F1 B1.
    # Order (0, 1), links (c, i):  stage 0 F: 1, 2.  Stage 1: F0 1+c..3+c, F1 ..5+c.  Stage 2: F0 3+c+i..5+c+i,
    #   B0 ..9+c+i, F1 ..11+c+i, B1 ..15+c+i.  Stage 1: B0 9+c+2i..13+c+2i, B1 15+c+2i..19+c+2i.
    #   Stage 0: B0 13+2c+2i..15+2c+2i, B1 19+2c+2i..21+2c+2i.                                => 21 + 2c + 2i
    # Order (1, 0), links (i, c):  stage 0 F: 2, 4.  Stage 1: F0 2+i..4+i, F1 ..6+i.  Stage 2: F0 4+i+c..5+i+c,
    #   B0 ..7+i+c, F1 ..8+i+c, B1 ..10+i+c.  Stage 1: B0 7+i+2c..11+i+2c, B1 ..15+i+2c.
    #   Stage 0: B0 11+2i+2c..15+2i+2c, B1 ..19+2i+2c.                                        => 19 + 2c + 2i
    c, i = 0.75, 0.125
    groups = [_group(1.0, 2.0, 9.0), _group(2.0, 4.0, i)]      # type 0's own link (9) is never used: one stage
    st, ln = P.pipeline_of_order(groups, [1, 2], (0, 1), c)
    assert P.simulate([s["fwd_ms"] for s in st], [s["bwd_ms"] for s in st], ln, 2)[0] == pytest.approx(21 + 2 * c + 2 * i)
    st, ln = P.pipeline_of_order(groups, [1, 2], (1, 0), c)
    assert P.simulate([s["fwd_ms"] for s in st], [s["bwd_ms"] for s in st], ln, 2)[0] == pytest.approx(19 + 2 * c + 2 * i)
    assert P.best_order_and_split(groups, [1, 2], c, 3, 2) == ([1, 0], [1, 1, 1], pytest.approx(19 + 2 * c + 2 * i))


def test_exhaustive_planner_equals_enumeration_with_longest_path_costing():
    # the same search written a second way: explicit stage owners, the longest-path brute force as the cost
    rng = random.Random(11)
    for _ in range(12):
        ng = rng.randint(1, 3)
        counts = [rng.randint(1, 2) for _ in range(ng)]
        groups = [_group(rng.uniform(0.5, 2.0), rng.uniform(0.5, 4.0), rng.uniform(0.0, 0.5)) for _ in range(ng)]
        cross, M = rng.uniform(0.0, 3.0), rng.randint(1, 4)
        Pn = sum(counts)
        total = Pn + rng.randint(0, 3)
        best = None
        for order in itertools.permutations(range(ng)):
            owner = [g for g in order for _ in range(counts[g])]
            link = [groups[owner[p]]["link_ms"] if owner[p] == owner[p + 1] else cross for p in range(Pn - 1)]
            for cuts in itertools.combinations(range(1, total), Pn - 1):
                lay = [b - a for a, b in zip((0,) + cuts, cuts + (total,))]
                t = brute_force_makespan([n * groups[g]["fwd_ms"] for n, g in zip(lay, owner)],
                                         [n * groups[g]["bwd_ms"] for n, g in zip(lay, owner)], link, M)
                if best is None or t < best - 1e-12:
                    best = t
        assert P.best_order_and_split(groups, counts, cross, total, M)[2] == pytest.approx(best)


def test_memory_rule_of_the_exhaustive_planner():
    # 2 stages, 4 layers, 4 micro-batches; saved activations 10 per layer and live micro-batch: stage 0 holds 2 live
    # micro-batches, stage 1 one.  Capacity 45: stage 0 may take at most 2 layers (2*2*10 = 40), stage 1 at most 4.
    g = [_group(1.0, 2.0, 0.0, mem=45, saved=10)]
    order, layers, _ = P.best_order_and_split(g, [2], 0.0, 4, 4)
    assert layers == [2, 2]
    g = [_group(1.0, 2.0, 0.0, mem=25, saved=10)]      # stage 0: one layer (20), stage 1: at most 2 -> 4 layers do not fit
    assert P.best_order_and_split(g, [2], 0.0, 4, 4) is None
    assert P.best_order_and_split(g, [2], 0.0, 3, 4)[1] == [1, 2]


# ---- the whole search tree (Section 3.3: pipeline, data-parallel and tensor-parallel levels) ---------------------

def _cluster_group(nodes, devs, tf, tb, link=0.0, dp=0.0, w=0, g=0, o=0, mem=0, saved=(0, 0, 0, 0)):
    tf, tb = list(tf) + [0.0] * (4 - len(tf)), list(tb) + [0.0] * (4 - len(tb))
    return dict(n_nodes=nodes, devices_per_node=devs, fwd_ms_tp=tf, bwd_ms_tp=tb, saved_act_bytes_tp=list(saved), link_ms=link,
                dp_ms_per_byte=dp, weight_bytes=w, grad_bytes=g, optimizer_bytes=o, memory_bytes=mem)


def test_cluster_plan_one_node_of_two_devices_hand_worked():
    # 2 layers, 4 samples per iteration in micro-batches of 1.  A layer takes 1 + 2 (forward + backward) on a whole
    # device and 0.6 + 1.2 on half of a tensor-parallel pair; fp32 gradient of a layer: 100 bytes.
    #   d=1, t=1: 2 stages of 1 layer, 4 micro-batches: (4 + 2 - 1) * 3            = 15
    #   d=1, t=2: 1 stage of 2 layers, 4 micro-batches: 4 * 2 * 1.8               = 14.4
    #   d=2, t=1: 1 stage of 2 layers, 2 micro-batches: 2 * 2 * 3 = 12, plus the all-reduce 2*(1/2)*100*2 * x = 200 x
    #   d=2, t=2 and d=4 would need 4 devices
    def plan(x, tp2=True, g=100, **kw):
        grp = _cluster_group(1, 2, (1.0, 0.6 if tp2 else 0.0), (2.0, 1.2 if tp2 else 0.0), dp=x, g=g, **kw)
        return P.plan_cluster([grp], 0.0, 2, 4, 1)
    r = plan(0.0075)
    assert (r["d"], r["tp"], r["stages"], r["layers"], r["n_micro"]) == (2, [1], [1], [2], 2)
    assert r["pipeline_ms"] == pytest.approx(12.0) and r["allreduce_ms"] == pytest.approx(1.5) and r["iter_ms"] == pytest.approx(13.5)
    r = plan(0.02)                      # replicas would cost 12 + 4 = 16: the tensor-parallel pair wins
    assert (r["d"], r["tp"], r["stages"], r["layers"], r["n_micro"]) == (1, [2], [1], [2], 4) and r["iter_ms"] == pytest.approx(14.4)
    r = plan(0.02, tp2=False)           # degree 2 not profiled: the two-stage pipeline is left
    assert (r["d"], r["tp"], r["stages"], r["layers"]) == (1, [1], [2], [1, 1]) and r["iter_ms"] == pytest.approx(15.0)
    r = plan(0.012)                     # 12 + 2.4 = 14.4 ties with the pair: the first found (d = 1) is kept
    assert (r["d"], r["tp"]) == (1, [2])
    # memory: weights 10 + gradients 20 + optimizer 60 per layer and device share; capacity 100
    #   d=2,t=1: 2 layers * 90 = 180 does not fit; d=1,t=2: 2 * 45 = 90 fits (14.4); d=1,t=1: 90 per stage fits (15)
    r = plan(0.0, w=10, g=20, o=60, mem=100)
    assert (r["d"], r["tp"]) == (1, [2]) and r["iter_ms"] == pytest.approx(14.4)
    # saved activations of the live micro-batches count too: 6 bytes per layer at t=2 -> 90 + 1 live * 2 layers * 6 = 102
    r = plan(0.0, w=10, g=20, o=60, mem=100, saved=(0, 6, 0, 0))
    assert (r["d"], r["tp"], r["stages"]) == (1, [1], [2])
    assert plan(0.0, w=10, g=20, o=60, mem=80) is None


def test_cluster_plan_two_types_uses_every_device_and_orders_the_types():
    # type 0: one device (1 + 2 per layer); type 1: a node of two devices (2 + 4 per layer each, 1.2 + 2.4 as a pair), link i
    # between its stages; cross link c; 3 layers, 2 samples, micro-batch 1 -> d = 1 only (type 0 has a single device).
    #   t1 = 1: stages (1, 2), the case worked out above: slow type first, 19 + 2c + 2i
    #   t1 = 2: stages (1, 1): 3 layers over 2 stages, 2 micro-batches; with stage times (f0,b0), (f1,b1) and f1+b1 >= f0 the
    #     1F1B iteration is f0 + c + 2 f1 + 2 b1, then stage 0's backwards: B0 ends at max(2 f0, f0+2c+f1+b1) + b0 and B1 at
    #     max(that, f0 + 2c + 2 f1 + 2 b1) + b0.  Order (0,1), layers (2,1): f0=2,b0=4,f1=1.2,b1=2.4: B0: max(4, 5.6+2c)+4,
    #     B1: max(9.6+2c, 9.2+2c)+4 = 13.6+2c.  Layers (1,2): f0=1,b0=2,f1=2.4,b1=4.8: B1 = max(.., 1+2c+14.4)+2 = 17.4+2c.
    #     Order (1,0), layers (1,2) [type 1 first with 1 layer: f0=1.2,b0=2.4; type 0 second with 2: f1=2,b1=4]:
    #     B0 = max(2.4, 1.2+2c+6)+2.4 = 9.6+2c, B1 = max(9.6+2c, 1.2+2c+12)+2.4 = 15.6+2c.  Layers (2,1): f0=2.4,b0=4.8,f1=1,b1=2:
    #     B0 = max(4.8, 2.4+2c+3)+4.8 = 10.2+2c, B1 = max(10.2+2c, 2.4+2c+6)+4.8 = 15+2c.          => best 13.6 + 2c
    c, i = 0.75, 0.125
    groups = [_cluster_group(1, 1, (1.0,), (2.0,), link=9.0), _cluster_group(1, 2, (2.0, 1.2), (4.0, 2.4), link=i)]
    for tf, tb, ln, want in [([2.0, 1.2], [4.0, 2.4], [c], 13.6 + 2 * c), ([1.0, 2.4], [2.0, 4.8], [c], 17.4 + 2 * c),
                             ([1.2, 2.0], [2.4, 4.0], [c], 15.6 + 2 * c), ([2.4, 1.0], [4.8, 2.0], [c], 15.0 + 2 * c)]:
        assert P.simulate(tf, tb, ln, 2)[0] == pytest.approx(want)
    r = P.plan_cluster(groups, c, 3, 2, 1)
    assert (r["d"], r["tp"], r["stages"], r["order"], r["layers"]) == (1, [1, 2], [1, 1], [0, 1], [2, 1])
    assert r["iter_ms"] == pytest.approx(13.6 + 2 * c)
    groups[1]["fwd_ms_tp"][1] = 0.0      # without the pair's profile only t1 = 1 is left
    r = P.plan_cluster(groups, c, 3, 2, 1)
    assert (r["tp"], r["stages"], r["order"], r["layers"]) == ([1, 1], [1, 2], [1, 0], [1, 1, 1])
    assert r["iter_ms"] == pytest.approx(19 + 2 * c + 2 * i)


def test_cluster_plan_data_parallel_degree_must_divide_batch_and_devices():
    g = _cluster_group(2, 2, (1.0, 0.6, 0.0, 0.0), (2.0, 1.2, 0.0, 0.0))
    # 4 devices, 6 samples, micro-batch 1: d in {1, 2, 3, 6} divides the batch, d*t in {1, 2, 4} the devices -> d in {1, 2}
    seen = set()
    for layers in (4, 8):
        r = P.plan_cluster([g], 0.0, layers, 6, 1)
        assert r["d"] in (1, 2) and r["d"] * r["tp"][0] * r["stages"][0] == 4 and r["n_micro"] * r["d"] == 6
        assert sum(r["layers"]) == layers and len(r["layers"]) == r["stages"][0]
        seen.add((r["d"], r["tp"][0]))
    # micro-batch 4 does not divide 6 samples for any d: nothing to search
    assert P.plan_cluster([g], 0.0, 4, 6, 4) is None
