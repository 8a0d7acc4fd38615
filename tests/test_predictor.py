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


# ---- the whole search tree: data-parallel and tensor-parallel levels above the pipeline level --------------------

def cluster_group(nodes, devs, tf, tb, link=0.0, dp=0.0, w=0, g=0, o=0, mem=0, saved=(0, 0, 0, 0), peak=1000.0):
    tf, tb = list(tf) + [0.0] * (4 - len(tf)), list(tb) + [0.0] * (4 - len(tb))
    return hh.hh_cluster_group(nodes, devs, (hh.C.c_double * 4)(*tf), (hh.C.c_double * 4)(*tb), (hh.C.c_uint64 * 4)(*saved), peak, link, dp,
                               w, g, o, mem)


def oracle_group(g, msg_bytes):
    return dict(n_nodes=g.n_nodes, devices_per_node=g.devices_per_node, fwd_ms_tp=list(g.fwd_ms_tp), bwd_ms_tp=list(g.bwd_ms_tp),
                saved_act_bytes_tp=list(g.saved_act_bytes_tp),
                link_ms=msg_bytes / (g.link_gbytes_per_s * 1e9) * 1e3 if g.link_gbytes_per_s > 0 else 0.0,
                dp_ms_per_byte=1.0 / (g.dp_gbytes_per_s * 1e9) * 1e3 if g.dp_gbytes_per_s > 0 else 0.0,
                weight_bytes=g.weight_bytes, grad_bytes=g.grad_bytes, optimizer_bytes=g.optimizer_bytes, memory_bytes=g.memory_bytes)


def test_cluster_plan_hand_worked_cases_through_the_library():
    # the cases worked out by hand for the oracle (tests/test_predictor_pins.py): one node of two devices, 2 layers, 4 samples
    B, S, H = 1, 16, 8                       # message size is irrelevant here: all links are free
    def plan(dp_gbs, tp2=True, **kw):
        g = cluster_group(1, 2, (1.0, 0.6 if tp2 else 0.0), (2.0, 1.2 if tp2 else 0.0), dp=dp_gbs, g=100, **kw)
        return hh.hh_plan_cluster([g], 0.0, 2, 4, B, S, H, 1e9, slack=4)
    # all-reduce 2*(1/2)*100*2 bytes = 200 bytes at x ms per byte: x ms per byte <-> 1e-6 / x GB/s
    p, layers = plan(1e-6 / 0.0075)
    assert (p.data_parallel, p.tensor_parallel[0], p.stages[0], layers, p.n_micro) == (2, 1, 1, [2], 2)
    assert p.pipeline_ms == pytest.approx(12.0) and p.grad_allreduce_ms == pytest.approx(1.5) and p.sim.iter_ms == pytest.approx(13.5)
    assert p.sim.n_devices == 2 and p.strategies_costed == 3
    # Eq. (1) on the whole iteration: seq * global batch / (devices * time)
    assert p.sim.tokens_per_s_per_device == pytest.approx(S * 4 / (2 * 13.5e-3))
    p, layers = plan(1e-6 / 0.02)
    assert (p.data_parallel, p.tensor_parallel[0], layers) == (1, 2, [2]) and p.sim.iter_ms == pytest.approx(14.4)
    p, layers = plan(1e-6 / 0.02, tp2=False)
    assert (p.data_parallel, p.tensor_parallel[0], layers) == (1, 1, [1, 1]) and p.sim.iter_ms == pytest.approx(15.0)


def test_cluster_plan_matches_exhaustive_search_on_small_random_clusters():
    rng = random.Random(77)
    checked = 0
    for _ in range(40):
        ng = rng.randint(1, 2)
        B, S, H = rng.choice([1, 2]), 128, 64
        msg = O.p2p_bytes(B, S, H)
        groups = []
        for _ in range(ng):
            devs = rng.choice([1, 2, 4])
            tf1, tb1 = rng.uniform(0.5, 2.0), rng.uniform(1.0, 4.0)
            eff = [1.0, rng.uniform(0.55, 0.7), rng.uniform(0.3, 0.45), 0.0]      # time at degree 2^i relative to degree 1
            prof = [rng.random() < 0.8 or i == 0 for i in range(4)]
            tf = [tf1 * e if p else 0.0 for e, p in zip(eff, prof)]
            tb = [tb1 * e if p else 0.0 for e, p in zip(eff, prof)]
            w = rng.randint(50, 150)
            mem = rng.choice([0, 0, rng.randint(400, 2500)])
            groups.append(cluster_group(rng.randint(1, 2), devs, tf, tb, link=rng.choice([0.0, 1e-4, 1e-3]),
                                        dp=rng.choice([0.0, 1e-6, 1e-5]), w=w, g=2 * w, o=6 * w, mem=mem,
                                        saved=tuple(rng.randint(5, 60) // (1 << i) for i in range(4))))
        total = rng.randint(2, 6)
        gb = rng.choice([2, 4, 8]) * B
        cross = rng.choice([0.0, 1e-4, 5e-5])
        want = O.plan_cluster([oracle_group(g, msg) for g in groups], msg / (cross * 1e9) * 1e3 if cross > 0 else 0.0, total, gb, B)
        try:
            p, layers = hh.hh_plan_cluster(groups, cross, total, gb, B, S, H, 1e9, slack=total)
        except hh.HHError as e:
            assert e.code == hh.HH_ERR_UNSUPPORTED_SHAPE and want is None
            continue
        assert want is not None
        checked += 1
        assert p.sim.iter_ms == pytest.approx(want["iter_ms"], rel=1e-9)
        assert p.pipeline_ms == pytest.approx(want["pipeline_ms"], rel=1e-9) and p.grad_allreduce_ms == pytest.approx(want["allreduce_ms"], rel=1e-9, abs=1e-15)
        assert (p.data_parallel, list(p.tensor_parallel)[:ng], list(p.stages)[:ng], p.n_micro) == (want["d"], want["tp"], want["stages"], want["n_micro"])
        assert sum(layers) == total and len(layers) == p.n_stages == sum(want["stages"])
        # every accelerator is used
        assert sum(p.data_parallel * p.tensor_parallel[i] * p.stages[i] for i in range(ng)) == sum(g.n_nodes * g.devices_per_node for g in groups) == p.sim.n_devices
    assert checked >= 25


def test_cluster_plan_for_a_two_speed_cluster_gives_the_slow_type_fewer_layers():
    # a mix in the spirit of Section 4.3, scaled down: one node of 4 of a fast type and two nodes of 4 of a type 1.6x
    # slower, 24 layers, 32 samples per iteration
    fast = cluster_group(1, 4, (1.0, 0.62, 0.40), (2.0, 1.24, 0.80), link=25.0, dp=20.0, w=10**9, g=2 * 10**9, o=6 * 10**9)
    slow = cluster_group(2, 4, (1.6, 1.0, 0.66), (3.2, 2.0, 1.3), link=25.0, dp=20.0, w=10**9, g=2 * 10**9, o=6 * 10**9)
    p, layers = hh.hh_plan_cluster([fast, slow], 2.5, 24, 32, 1, 4096, 8192, 1.7e12, slack=0)
    assert sum(layers) == 24 and p.n_stages == len(layers) and p.sim.search_truncated == 0
    by_type = {0: [], 1: []}
    pos = 0
    for k in range(2):
        g = p.order[k]
        by_type[g] += layers[pos:pos + p.stages[g]]
        pos += p.stages[g]
    # load balance: a stage of the fast type carries more work per unit of its speed-adjusted time, i.e. at least as many
    # layers per accelerator-second as a stage of the slow type
    per_dev_fast = max(by_type[0]) / p.tensor_parallel[0]
    per_dev_slow = min(by_type[1]) / p.tensor_parallel[1]
    assert per_dev_fast >= per_dev_slow
    assert p.data_parallel * p.tensor_parallel[0] * p.stages[0] == 4 and p.data_parallel * p.tensor_parallel[1] * p.stages[1] == 8
    assert p.n_micro * p.data_parallel == 32


def test_layer_split_reports_a_truncated_search():
    # 14 stages with 5 candidate counts each: more leaves than the budget of costed candidates
    st = [stage(0, 1.0 + 0.01 * i, 2.0) for i in range(14)]
    layers, res = hh.hh_plan_layers(st, 70, 2, 1, 128, 64, 1, 1e9, slack=2)
    assert res.search_truncated == 1 and sum(layers) == 70
    layers, res = hh.hh_plan_layers(st[:4], 20, 2, 1, 128, 64, 1, 1e9, slack=2)
    assert res.search_truncated == 0 and sum(layers) == 20


def test_cluster_plan_argument_checks():
    g = cluster_group(1, 2, (1.0,), (2.0,))
    for args in [dict(n=0), dict(total=0), dict(gb=0), dict(mb=0), dict(slack=-1), dict(max_stages=0)]:
        with pytest.raises(hh.HHError) as e:
            hh.hh_plan_cluster([g] * args.get("n", 1), 0.0, args.get("total", 4), args.get("gb", 4), args.get("mb", 1), 128, 64, 1e9,
                               slack=args.get("slack", 2), max_stages=args.get("max_stages", 64))
        assert e.value.code == hh.HH_ERR_INVALID_ARG
    with pytest.raises(hh.HHError) as e:                 # 3 samples in micro-batches of 2: no data-parallel degree fits
        hh.hh_plan_cluster([g], 0.0, 4, 3, 2, 128, 64, 1e9)
    assert e.value.code == hh.HH_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(hh.HHError) as e:                 # the best plan has 2 stages, the caller's array holds 1
        hh.hh_plan_cluster([g], 0.0, 4, 1, 1, 128, 64, 1e9, max_stages=1)    # one sample: no replicas, only degree 1 profiled
    assert e.value.code == hh.HH_ERR_INVALID_ARG
