"""Test infrastructure only: a plain Python model of what the workload simulator of Section 3.2 computes
for one pipeline, written from the definitions so that it can be checked by eye.  Nothing in the
product imports this file.

The paper states what the simulator returns (time of one iteration step and the maximum memory use of a
strategy, Section 3.2), the pipeline discipline (PipeDream-1F1B data constraints, Section 3.3), the
metrics (Eq. 1 throughput, Eq. 2 MFU, Eq. 3 point-to-point volume) and how the "theoretical" figure of a
mixed cluster is formed (the mean over all accelerators, Section 4.3).  It does not give the simulator's
inner model; the reading taken here is the textbook one:

* a stage runs its operations one at a time in the 1F1B order: forward of micro-batches 0 .. w-1
  (w = min(M, P - p) for stage p of P), then backward of m followed by forward of m + w, and the remaining
  backwards;
* forward of micro-batch m on stage p starts when the stage is free and the forward of m on stage p-1 has
  finished and its boundary tensor (Eq. 3 bytes) has crossed the link; backward likewise from stage p+1;
* the iteration ends when every stage has finished its last backward.

All times in milliseconds, sizes in bytes, link speed in bytes per millisecond.
"""
from __future__ import annotations


def one_f_one_b_order(p: int, n_stages: int, n_micro: int):
    """Operation list of stage p: ('F', m) / ('B', m) in execution order (Section 2.3, 1F1B)."""
    w = min(n_micro, n_stages - p)
    ops = [("F", m) for m in range(w)]
    for m in range(n_micro):
        ops.append(("B", m))
        if m + w < n_micro:
            ops.append(("F", m + w))
    return ops


def simulate(fwd_ms, bwd_ms, link_ms, n_micro):
    """fwd_ms[p], bwd_ms[p]: time of one micro-batch on stage p (all its layers); link_ms[p]: transfer time of
    one boundary tensor between stage p and p+1 (len P-1).  Returns (iteration_ms, busy_ms[p], finish[p])."""
    P = len(fwd_ms)
    orders = [one_f_one_b_order(p, P, n_micro) for p in range(P)]
    done = {}                       # (kind, p, m) -> finish time
    nxt = [0] * P                   # next operation index per stage
    free = [0.0] * P                # time the stage becomes free
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for p in range(P):
            while nxt[p] < len(orders[p]):
                kind, m = orders[p][nxt[p]]
                if kind == "F":
                    dep = None if p == 0 else ("F", p - 1, m)
                    lat = 0.0 if p == 0 else link_ms[p - 1]
                    dur = fwd_ms[p]
                else:
                    dep = None if p == P - 1 else ("B", p + 1, m)
                    lat = 0.0 if p == P - 1 else link_ms[p]
                    dur = bwd_ms[p]
                if dep is not None and dep not in done:
                    break
                ready = 0.0 if dep is None else done[dep] + lat
                start = max(free[p], ready)
                free[p] = start + dur
                done[(kind, p, m)] = free[p]
                nxt[p] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlocked")
    busy = [n_micro * (fwd_ms[p] + bwd_ms[p]) for p in range(P)]
    return max(free), busy, list(free)


def live_micro_batches(p: int, n_stages: int, n_micro: int) -> int:
    """Largest number of micro-batches whose activations stage p holds at once under 1F1B."""
    live = peak = 0
    for kind, _ in one_f_one_b_order(p, n_stages, n_micro):
        live += 1 if kind == "F" else -1
        peak = max(peak, live)
    return peak


def stage_peak_bytes(p, n_stages, n_micro, n_layers, weight_bytes, grad_bytes, optimizer_bytes, saved_act_bytes):
    """Parameters, gradients and optimizer state of the stage's layers plus the activations of the live
    micro-batches (per layer figures as in the per-layer profile record)."""
    return n_layers * (weight_bytes + grad_bytes + optimizer_bytes) + \
        live_micro_batches(p, n_stages, n_micro) * n_layers * saved_act_bytes


def p2p_bytes(batch, seq, hidden):
    """Eq. (3): one 16-bit boundary tensor."""
    return batch * seq * hidden * 2


def tgs(seq, global_batch, n_devices, iter_s):
    """Eq. (1): tokens per device per second."""
    return seq * global_batch / (n_devices * iter_s)


def weighted_mean(values, counts):
    """Section 4.3: the theoretical figure of a mixed cluster is the mean over all its accelerators."""
    return sum(v * c for v, c in zip(values, counts)) / sum(counts)


def mfu(model_flop_per_iteration, iter_s, peaks_tflops, counts):
    """Eq. (2): achieved TFLOP/s per device over the mean peak of the cluster's devices."""
    n = sum(counts)
    achieved = model_flop_per_iteration / iter_s / n / 1e12
    return achieved / weighted_mean(peaks_tflops, counts)


def compositions(total, parts):
    """All ways to write total as an ordered sum of `parts` positive integers."""
    if parts == 1:
        if total >= 1:
            yield (total,)
        return
    for first in range(1, total - parts + 2):
        for rest in compositions(total - first, parts - 1):
            yield (first,) + rest


def pipeline_of_order(groups, counts, order, cross_link_ms_per_msg):
    """The stage list and the link list of one order of the accelerator groups (Section 3.3: a group's stages stay
    together).  Stage list: counts[g] copies of groups[g] for each g of `order` in turn.  Link p joins stages p and
    p+1: the group's own link when both belong to the same group, the cross link where two groups meet."""
    owner = [g for g in order for _ in range(counts[g])]
    stages = [groups[g] for g in owner]
    links = [groups[owner[p]]["link_ms"] if owner[p] == owner[p + 1] else cross_link_ms_per_msg
             for p in range(len(owner) - 1)]
    return stages, links


def best_order_and_split(groups, counts, cross_link_ms_per_msg, total_layers, n_micro):
    """Section 3.3, both rules by exhaustion: every order of the accelerator groups along the pipeline (a group's
    stages stay together), every split of the layers over the stages; the fastest iteration wins, the first found
    among equals (orders in lexicographic order of group indices).  groups[g] = dict(fwd_ms, bwd_ms per layer,
    link_ms = transfer time of one boundary tensor inside the group, weight/grad/optimizer/saved_act bytes per layer,
    memory_bytes or 0).  Returns (order, layers, iteration_ms)."""
    import itertools
    best = None
    for order in itertools.permutations(range(len(groups))):
        stages, links = pipeline_of_order(groups, counts, order, cross_link_ms_per_msg)
        P = len(stages)
        for layers in compositions(total_layers, P):
            ok = True
            for p, (st, n) in enumerate(zip(stages, layers)):
                if st["memory_bytes"] and stage_peak_bytes(p, P, n_micro, n, st["weight_bytes"], st["grad_bytes"],
                                                           st["optimizer_bytes"], st["saved_act_bytes"]) > st["memory_bytes"]:
                    ok = False
                    break
            if not ok:
                continue
            it, _, _ = simulate([n * st["fwd_ms"] for n, st in zip(layers, stages)],
                                [n * st["bwd_ms"] for n, st in zip(layers, stages)], links, n_micro)
            if best is None or it < best[2] - 1e-12:
                best = (list(order), list(layers), it)
    return best


def plan_cluster(groups, cross_link_ms_per_msg, total_layers, global_batch, micro_batch):
    """The whole three-level search tree of Section 3.3 by exhaustion.  groups[g] = dict(n_nodes, devices_per_node,
    fwd_ms_tp / bwd_ms_tp / saved_act_bytes_tp: lists indexed by log2 of the tensor-parallel degree (time <= 0: not
    profiled), link_ms, dp_ms_per_byte (ring all-reduce time per byte and device between replicas, 0: free),
    weight_bytes / grad_bytes / optimizer_bytes per whole layer, memory_bytes or 0).

    Level 2: one data-parallel degree d for every stage; level 3: one tensor-parallel degree t_g per group, inside a
    node; every accelerator is used, so group g forms n_nodes*devices_per_node / (d*t_g) stages; level 1 under each such
    leaf: best_order_and_split on the pipeline time.  A leaf costs that pipeline time plus the slowest stage's gradient
    all-reduce between its d replicas, 2 (d-1)/d * grad_bytes/t * layers * dp_ms_per_byte.  The cheapest leaf wins, the
    first found among equals (d ascending, then the t_g ascending with group 0 slowest).
    Returns dict(d, tp, stages, order, layers, n_micro, pipeline_ms, allreduce_ms, iter_ms) or None."""
    import itertools
    best = None
    max_dev = max(g["n_nodes"] * g["devices_per_node"] for g in groups)
    for d in range(1, max_dev + 1):
        if global_batch % (d * micro_batch):
            continue
        n_micro = global_batch // (d * micro_batch)
        options = [[i for i in range(4) if g["devices_per_node"] % (1 << i) == 0 and g["fwd_ms_tp"][i] > 0 and g["bwd_ms_tp"][i] > 0]
                   for g in groups]
        for tp_idx in itertools.product(*options):
            counts, stage_groups = [], []
            for g, i in zip(groups, tp_idx):
                t, dev = 1 << i, g["n_nodes"] * g["devices_per_node"]
                if dev % (d * t) or dev // (d * t) < 1:
                    break
                counts.append(dev // (d * t))
                stage_groups.append(dict(fwd_ms=g["fwd_ms_tp"][i], bwd_ms=g["bwd_ms_tp"][i], link_ms=g["link_ms"],
                                         weight_bytes=g["weight_bytes"] // t, grad_bytes=g["grad_bytes"] // t,
                                         optimizer_bytes=g["optimizer_bytes"] // t, saved_act_bytes=g["saved_act_bytes_tp"][i],
                                         memory_bytes=g["memory_bytes"]))
            else:
                if sum(counts) > total_layers:
                    continue
                r = best_order_and_split(stage_groups, counts, cross_link_ms_per_msg, total_layers, n_micro)
                if r is None:
                    continue
                order, layers, pipe = r
                owner = [g for g in order for _ in range(counts[g])]
                ar = max([2.0 * (d - 1) / d * (groups[g]["grad_bytes"] / (1 << tp_idx[g])) * n * groups[g]["dp_ms_per_byte"]
                          for g, n in zip(owner, layers)] + [0.0]) if d > 1 else 0.0
                if best is None or pipe + ar < best["iter_ms"] - 1e-12:
                    best = dict(d=d, tp=[1 << i for i in tp_idx], stages=counts, order=order, layers=layers, n_micro=n_micro,
                                pipeline_ms=pipe, allreduce_ms=ar, iter_ms=pipe + ar)
    return best
