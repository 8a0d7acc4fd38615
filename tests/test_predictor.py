"""The host-side predictor of the library (hh_sim_pipeline, hh_sim_weighted_mean, hh_plan_layers) against the
Python oracle of the same definitions, on seeded random pipelines, plus the planner's own properties.
Runs without a GPU."""
import itertools
import os
import random

import pytest

from oracle import predictor_oracle as O
from paper_2405_16256_amd import binding as hh


def stage(n_layers, fwd, bwd, n_devices=1, peak=1000.0, link=0.0, w=0, g=0, opt=0, act=0, mem=0):
    return hh.hh_sim_stage(n_layers, n_devices, fwd, bwd, peak, link, w, g, opt, act, mem)


def random_pipeline(rng):
    P = rng.randint(1, 9)
    st = []
    for _ in range(P):
        st.append(stage(rng.randint(1, 9), rng.uniform(0.3, 4.0), rng.uniform(0.5, 8.0), rng.choice([1, 2, 8, 16]),
                        rng.choice([312.0, 989.0, 1307.0, 2500.0]), rng.choice([0.0, 2.5, 25.0, 50.0]),
                        rng.randint(1, 10**9), rng.randint(1, 10**9), rng.randint(0, 10**9), rng.randint(1, 10**9)))
    return st


def test_simulator_matches_the_oracle_on_random_pipelines():
    rng = random.Random(2024)
    for _ in range(200):
        st = random_pipeline(rng)
        P = len(st)
        M, B, S, H, dp = rng.randint(1, 24), rng.choice([1, 2, 4]), rng.choice([1024, 2048, 4096]), rng.choice([4096, 8192]), rng.choice([1, 2, 4])
        flop = rng.uniform(1e11, 1e13)
        res, fin, peak = hh.hh_sim_pipeline(st, M, B, S, H, dp, flop)
        tf = [s.n_layers * s.fwd_ms for s in st]
        tb = [s.n_layers * s.bwd_ms for s in st]
        msg = O.p2p_bytes(B, S, H)
        link = [msg / (st[p].link_gbytes_per_s * 1e9) * 1e3 if st[p].link_gbytes_per_s > 0 else 0.0 for p in range(P - 1)]
        it, busy, fo = O.simulate(tf, tb, link, M)
        assert res.iter_ms == pytest.approx(it, rel=1e-12)
        assert fin == pytest.approx(fo, rel=1e-12)
        assert res.bubble_fraction == pytest.approx(1 - max(busy) / it, abs=1e-12)
        for p in range(P):
            assert peak[p] == O.stage_peak_bytes(p, P, M, st[p].n_layers, st[p].weight_bytes, st[p].grad_bytes,
                                                 st[p].optimizer_bytes, st[p].saved_act_bytes)
        counts = [s.n_devices for s in st]
        nd = sum(counts)
        assert res.n_devices == nd
        assert res.tokens_per_s_per_device == pytest.approx(O.tgs(S, M * B * dp, nd, it * 1e-3), rel=1e-12)
        total_flop = flop * sum(s.n_layers for s in st) * M * dp
        assert res.mean_peak_tflops == pytest.approx(O.weighted_mean([s.peak_tflops for s in st], counts), rel=1e-12)
        assert res.mfu == pytest.approx(O.mfu(total_flop, it * 1e-3, [s.peak_tflops for s in st], counts), rel=1e-12)
        assert res.tflops_per_device == pytest.approx(total_flop / (it * 1e-3) / nd / 1e12, rel=1e-12)


def test_uniform_pipeline_closed_form_through_the_library():
    for P, M in [(1, 1), (4, 8), (12, 32), (10, 64)]:
        st = [stage(8, 1.5, 3.0) for _ in range(P)]
        res, fin, _ = hh.hh_sim_pipeline(st, M, 1, 4096, 8192, 1, 1e12)
        assert res.iter_ms == pytest.approx((M + P - 1) * 8 * 4.5)
        assert res.bubble_fraction == pytest.approx((P - 1) / (M + P - 1))


def test_weighted_mean_reproduces_the_figures_of_section_4_3():
    assert hh.hh_sim_weighted_mean([56.4, 45.3], [1, 1]) == pytest.approx(50.85, abs=5e-3)
    assert hh.hh_sim_weighted_mean([38.90, 28.80], [1, 1]) == pytest.approx(33.85, abs=5e-3)
    assert hh.hh_sim_weighted_mean([38.90, 35.30], [128, 640]) == pytest.approx(35.90, abs=5e-3)
    assert 100 * 51.11 / hh.hh_sim_weighted_mean([93.81, 48.08], [128, 640]) == pytest.approx(91.75, abs=2e-2)


def test_argument_checks():
    ok = [stage(2, 1.0, 2.0)]
    for bad in ([stage(0, 1.0, 2.0)], [stage(2, 0.0, 2.0)], [stage(2, 1.0, 2.0, n_devices=0)], [stage(2, 1.0, 2.0, peak=0.0)], []):
        with pytest.raises(hh.HHError) as e:
            hh.hh_sim_pipeline(bad, 4, 1, 128, 256, 1, 1e9)
        assert e.value.code == hh.HH_ERR_INVALID_ARG
    with pytest.raises(hh.HHError):
        hh.hh_sim_pipeline(ok, 0, 1, 128, 256, 1, 1e9)
    with pytest.raises(hh.HHError):
        hh.hh_sim_weighted_mean([1.0, 2.0], [0, 0])
    with pytest.raises(hh.HHError):
        hh.hh_plan_layers(ok * 3, 2, 4, 1, 128, 256, 1, 1e9)       # fewer layers than stages


def best_split_by_enumeration(st, total, M, B, S, H):
    P = len(st)
    best = None
    for cut in itertools.combinations(range(1, total), P - 1):
        layers = [b - a for a, b in zip((0,) + cut, cut + (total,))]
        tf = [n * s.fwd_ms for n, s in zip(layers, st)]
        tb = [n * s.bwd_ms for n, s in zip(layers, st)]
        msg = O.p2p_bytes(B, S, H)
        link = [msg / (st[p].link_gbytes_per_s * 1e9) * 1e3 if st[p].link_gbytes_per_s > 0 else 0.0 for p in range(P - 1)]
        it, _, _ = O.simulate(tf, tb, link, M)
        if best is None or it < best[0] - 1e-12:
            best = (it, layers)
    return best


def test_planner_finds_the_enumerated_optimum_on_small_mixed_pipelines():
    rng = random.Random(5)
    for _ in range(25):
        P = rng.randint(2, 4)
        total = rng.randint(P + 2, 14)
        st = [stage(0, f, 2 * f, link=rng.choice([0.0, 25.0])) for f in (rng.choice([1.0, 1.3, 2.0]) for _ in range(P))]
        M = rng.randint(2, 10)
        layers, res = hh.hh_plan_layers(st, total, M, 1, 2048, 4096, 1, 1e12, slack=total)
        it, _ = best_split_by_enumeration(st, total, M, 1, 2048, 4096)
        assert sum(layers) == total and min(layers) >= 1
        assert res.iter_ms == pytest.approx(it, rel=1e-12)


def test_planner_gives_equal_devices_equal_layers_and_faster_devices_more():
    st = [stage(0, 2.0, 4.0) for _ in range(10)]
    layers, res = hh.hh_plan_layers(st, 80, 64, 1, 4096, 8192, 1, 1e12)
    assert layers == [8] * 10                                         # the uniform split of Section 4.3: PP = 10, 8 layers each
    # twelve stages, four of them on a device that is 7/6 slower: the 80 layers split into sixes and sevens
    slow, fast = stage(0, 7.0 / 6.0, 14.0 / 6.0), stage(0, 1.0, 2.0)
    st = [fast] + [slow] * 4 + [fast] * 7
    layers, res = hh.hh_plan_layers(st, 80, 64, 1, 4096, 8192, 1, 1e12, slack=1)
    assert sum(layers) == 80 and set(layers) <= {6, 7}
    assert sum(layers[1:5]) < 4 * 7                                    # the slow stages carry fewer layers
    uniform8, _, _ = hh.hh_sim_pipeline([stage(8, s.fwd_ms, s.bwd_ms) for s in ([fast] + [slow] * 4 + [fast] * 5)], 64, 1, 4096,
                                        8192, 1, 1e12)
    assert res.iter_ms < uniform8.iter_ms                              # and beat eight layers on each of ten stages


def test_planner_respects_stage_memory():
    # the faster stage would take more layers, but its memory only holds three
    a = stage(0, 1.0, 2.0, w=100, g=200, opt=600, act=50, mem=3 * 900 + 2 * 3 * 50)
    b = stage(0, 2.0, 4.0, w=100, g=200, opt=600, act=50, mem=0)
    layers, _ = hh.hh_plan_layers([a, b], 9, 8, 1, 128, 256, 1, 1e9, slack=9)
    assert layers[0] <= 3 and sum(layers) == 9
    a_small = stage(0, 1.0, 2.0, w=100, g=200, opt=600, act=50, mem=10)
    b_small = stage(0, 2.0, 4.0, w=100, g=200, opt=600, act=50, mem=10)
    with pytest.raises(hh.HHError) as e:
        hh.hh_plan_layers([a_small, b_small], 9, 8, 1, 128, 256, 1, 1e9, slack=9)
    assert e.value.code == hh.HH_ERR_UNSUPPORTED_SHAPE


# ---------------------------------------------------------------- stage order (second rule of the planner)
def group_pair(rng, B, S, H):
    """A library group descriptor and the oracle's view of the same group."""
    fwd = rng.choice([1.0, 1.3, 2.0, 2.6])
    link_gb = rng.choice([0.0, 5.0, 25.0])
    w, g, opt, act = rng.randint(1, 50), rng.randint(1, 50), rng.randint(0, 100), rng.randint(1, 40)
    mem = rng.choice([0, 0, 4000, 9000])
    lib_group = stage(0, fwd, 2 * fwd, link=link_gb, w=w, g=g, opt=opt, act=act, mem=mem)
    msg = O.p2p_bytes(B, S, H)
    link_ms = msg / (link_gb * 1e9) * 1e3 if link_gb > 0 else 0.0
    ora_group = dict(fwd_ms=fwd, bwd_ms=2 * fwd, link_ms=link_ms, weight_bytes=w, grad_bytes=g, optimizer_bytes=opt,
                     saved_act_bytes=act, memory_bytes=mem)
    return lib_group, ora_group


def test_stage_order_matches_exhaustive_search_on_small_mixed_clusters():
    rng = random.Random(11)
    B, S, H = 1, 2048, 4096
    tried = 0
    while tried < 30:
        n_groups = rng.randint(1, 3)
        counts = [rng.randint(1, 2) for _ in range(n_groups)]
        P = sum(counts)
        total = rng.randint(P, P + 6)
        M = rng.randint(2, 8)
        pairs = [group_pair(rng, B, S, H) for _ in range(n_groups)]
        cross_gb = rng.choice([0.0, 2.5, 25.0])
        cross_ms = O.p2p_bytes(B, S, H) / (cross_gb * 1e9) * 1e3 if cross_gb > 0 else 0.0
        want = O.best_order_and_split([o for _, o in pairs], counts, cross_ms, total, M)
        if want is None:
            with pytest.raises(hh.HHError) as e:
                hh.hh_plan_order([l for l, _ in pairs], counts, cross_gb, total, M, B, S, H, 1, 1e12, slack=total)
            assert e.value.code == hh.HH_ERR_UNSUPPORTED_SHAPE
            continue
        order, layers, res = hh.hh_plan_order([l for l, _ in pairs], counts, cross_gb, total, M, B, S, H, 1, 1e12, slack=total)
        assert sorted(order) == list(range(n_groups)) and sum(layers) == total and min(layers) >= 1
        assert res.iter_ms == pytest.approx(want[2], rel=1e-12)
        tried += 1


def test_stage_order_puts_the_memory_tight_type_late_and_keeps_slow_links_few():
    # two accelerator types of equal speed; type 0 has little memory.  Under 1F1B the first stages hold the most
    # live micro-batches, so the small-memory type must come last.
    small = stage(0, 1.0, 2.0, w=10, g=10, opt=10, act=100, mem=4 * 30 + 2 * 4 * 100)   # 4 layers with at most 2 live micro-batches
    big = stage(0, 1.0, 2.0, w=10, g=10, opt=10, act=100, mem=0)
    order, layers, res = hh.hh_plan_order([small, big], [2, 2], 0.0, 16, 8, 1, 128, 256, 1, 1e9, slack=0)
    assert order == [1, 0] and layers == [4, 4, 4, 4]
    # one type, any count: the order is trivial and the result equals the plain layer split
    st = [stage(0, 1.0, 2.0) for _ in range(4)]
    want_layers, want = hh.hh_plan_layers(st, 12, 6, 1, 128, 256, 1, 1e9)
    order, layers, res = hh.hh_plan_order([stage(0, 1.0, 2.0)], [4], 0.0, 12, 6, 1, 128, 256, 1, 1e9)
    assert order == [0] and layers == want_layers and res.iter_ms == want.iter_ms


def test_stage_order_argument_checks():
    g = [stage(0, 1.0, 2.0)]
    with pytest.raises(hh.HHError):
        hh.hh_plan_order(g, [0], 0.0, 4, 2, 1, 128, 256, 1, 1e9)
    with pytest.raises(hh.HHError):
        hh.hh_plan_order(g * 9, [1] * 9, 0.0, 12, 2, 1, 128, 256, 1, 1e9)
    with pytest.raises(hh.HHError):
        hh.hh_plan_order(g, [3], 0.0, 2, 2, 1, 128, 256, 1, 1e9)       # fewer layers than stages
