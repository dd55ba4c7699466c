"""Pins of the scheduling oracle (oracle/sched_oracle.py) to what the paper and plain reasoning fix:
the memory figures Sec. 4.1 and Table 1 print for AlexNet at batch 200 (tests/golden/
alexnet_b200_memory.txt), a hand-worked route of Alg. 1, and brute-force properties of the pool."""
import os
import random

import pytest

from oracle import sched_oracle as so

MiB = float(1 << 20)
HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "alexnet_b200_memory.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


G = _golden()


def test_alexnet_baseline_and_liveness_match_the_paper():
    net = so.alexnet()
    base = so.memory_trace(net, so.BASELINE)
    assert round(base["peak"] / MiB, 3) == G["baseline_mb"] and base["tensors"] == G["baseline_tensors"]
    live = so.memory_trace(net, so.LIVENESS)
    assert round(live["peak"] / MiB, 3) == G["liveness_peak_mb"]
    assert live["peak_step"] == G["liveness_peak_step"]
    # "up to 17 tensors with a peak memory usage of 1489.355MB" is read as: 17 tensors at the peak step
    # (the text itself says the peak of the count lies elsewhere)
    assert live["live"][live["peak_step"] - 1] == G["liveness_peak_tensors"]
    assert live["live"][39 - 1] == G["liveness_live_tensors_at_pool2"]
    # the paper's split of the peak: forward tensors up to CONV5 + what the backward POOL5 holds
    assert round(G["liveness_peak_fwd_part_mb"] + G["liveness_peak_bwd_part_mb"], 3) == G["liveness_peak_mb"]
    b = 200 * 4
    fwd = b * (3 * 96 * 55 * 55 + 96 * 27 * 27 + 3 * 256 * 27 * 27 + 256 * 13 * 13 + 4 * 384 * 13 * 13 + 256 * 13 * 13)
    assert round(fwd / MiB, 3) == G["liveness_peak_fwd_part_mb"]
    assert round(2 * b * (256 * 13 * 13 + 256 * 6 * 6) / MiB, 3) == G["liveness_peak_bwd_part_mb"]
    # liveness never uses more than the baseline, and nothing is live after the last step's frees
    assert max(live["bytes"]) <= base["peak"]


def test_alexnet_offloading_matches_the_paper():
    net = so.alexnet()
    off = so.memory_trace(net, so.OFFLOAD)
    assert off["peak_step"] == G["offload_peak_step"]
    assert off["live"][off["peak_step"] - 1] == G["offload_live_tensors_at_pool2"]
    # 1132.155 is printed; the nine tensors the paper counts at that step add up to 1132.056
    # (RELU1, LRN1, POOL1, CONV2, RELU2, LRN2, POOL2 outputs and the two gradients of the step):
    # a tenth of a MB, 9e-5 of the figure, is left unexplained
    assert abs(off["peak"] / MiB - G["offload_peak_mb"]) <= 0.1
    b = 200 * 4
    nine = b * (2 * 96 * 55 * 55 + 96 * 27 * 27 + 3 * 256 * 27 * 27 + 256 * 13 * 13) + b * (256 * 13 * 13 + 256 * 27 * 27)
    assert off["peak"] == nine


@pytest.mark.parametrize("strategy,name", [(so.SPEED, "speed_centric"), (so.MEMORY, "memory_centric"),
                                           (so.COST_AWARE, "cost_aware")])
def test_alexnet_recomputation_matches_table_1(strategy, name):
    r = so.memory_trace(so.alexnet(), so.RECOMPUTE, strategy)
    assert round(r["peak"] / MiB, 3) == G[name + "_peak_mb"]
    assert r["extra"] == G[name + "_extra"]
    if strategy != so.SPEED:
        assert r["peak_step"] == G["recompute_peak_step"]


def test_segment_costs_closed_form():
    # one kept layer, m cheap layers, one kept layer: speed-centric recomputes m, memory-centric m(m+1)/2
    for m in range(1, 7):
        net = so.Net()
        prev = net.add(so.DATA, 1000)
        prev = net.add(so.CONV, 5000, [prev])
        for _ in range(m):
            prev = net.add(so.ACT, 5000, [prev])
        prev = net.add(so.CONV, 5000, [prev])
        prev = net.add(so.SOFTMAX, 10, [prev])
        assert so.memory_trace(net, so.RECOMPUTE, so.SPEED)["extra"] == m
        assert so.memory_trace(net, so.RECOMPUTE, so.MEMORY)["extra"] == m * (m + 1) // 2
        ca = so.memory_trace(net, so.RECOMPUTE, so.COST_AWARE)
        assert ca["peak"] <= so.memory_trace(net, so.RECOMPUTE, so.MEMORY)["peak"]
        assert m <= ca["extra"] <= m * (m + 1) // 2


def _nested_fans():
    """a -> b -> {c, d}; c -> e; d -> f -> {g, h}; {e, g, h} -> i -> j: two fans, the second inside
    a branch of the first, joined at i."""
    net = so.Net()
    ids = {}
    ids["a"] = net.add(so.DATA, 10)
    ids["b"] = net.add(so.CONV, 10, [ids["a"]])
    ids["c"] = net.add(so.CONV, 10, [ids["b"]])
    ids["d"] = net.add(so.CONV, 10, [ids["b"]])
    ids["e"] = net.add(so.ACT, 10, [ids["c"]])
    ids["f"] = net.add(so.CONV, 10, [ids["d"]])
    ids["g"] = net.add(so.ACT, 10, [ids["f"]])
    ids["h"] = net.add(so.POOL, 10, [ids["f"]])
    ids["i"] = net.add(so.JOIN, 30, [ids["e"], ids["g"], ids["h"]])
    ids["j"] = net.add(so.SOFTMAX, 30, [ids["i"]])
    return net, ids


def test_route_of_nested_fans_by_hand():
    net, ids = _nested_fans()
    names = {v: k for k, v in ids.items()}
    got = "".join(names[i] for i in so.route(net))
    # depth first from a: b, its first branch c, e; i is reached but waits (1 of 3); back to d, f, g; i waits
    # (2 of 3); h; now i runs, then j
    assert got == "abcedfghij"


def test_route_is_a_topological_order_on_random_dags():
    rnd = random.Random(5)
    for _ in range(50):
        n = rnd.randint(2, 25)
        net = so.Net()
        net.add(so.DATA, 1)
        for i in range(1, n):
            k = rnd.randint(1, min(3, i))
            net.add(so.CONV, 1, sorted(rnd.sample(range(i), k)))
        order = so.route(net)
        reach = {0}
        for i in range(1, n):
            if any(p in reach for p in net.layers[i][2]) and all(p in reach for p in net.layers[i][2]):
                reach.add(i)
        seen = set()
        for i in order:
            assert all(p in seen for p in net.layers[i][2])
            assert i not in seen
            seen.add(i)
        assert seen == reach


def test_pool_first_fit_against_a_byte_map():
    rnd = random.Random(11)
    size = 64 * so.BLOCK
    pool = so.Pool(size)
    blocks = [0] * 64            # brute force: owner id per block
    held = {}
    for _ in range(3000):
        if held and (rnd.random() < 0.45 or sum(1 for b in blocks if b) > 56):
            ident = rnd.choice(sorted(held))
            start, n = held.pop(ident)
            pool.free(ident)
            for b in range(start, start + n):
                assert blocks[b] == ident
                blocks[b] = 0
        else:
            nbytes = rnd.randint(1, 9 * so.BLOCK)
            need = -(-nbytes // so.BLOCK)
            # first fit on the byte map: the lowest run of `need` free blocks
            want = None
            run = 0
            for b in range(64):
                run = run + 1 if blocks[b] == 0 else 0
                if run == need:
                    want = b - need + 1
                    break
            got = pool.alloc(nbytes)
            if want is None:
                assert got is None
                continue
            ident, offset = got
            assert offset == want * so.BLOCK and offset % so.BLOCK == 0
            for b in range(want, want + need):
                blocks[b] = ident
            held[ident] = (want, need)
        assert pool.used_blocks == sum(1 for b in blocks if b)
        free_runs, run = [], 0
        for b in blocks + [1]:
            if b == 0:
                run += 1
            elif run:
                free_runs.append(run)
                run = 0
        assert pool.largest_free() == max(free_runs, default=0) * so.BLOCK
