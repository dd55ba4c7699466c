"""The host-side memory scheduling of the library (include/sn_runtime.h, csrc/sn_runtime.cpp) against
the plain-Python oracle (oracle/sched_oracle.py, itself pinned to the paper's AlexNet figures in
test_oracle_sched.py): execution order, pool, memory per step at every level and strategy, on AlexNet
and on seeded random networks with forks and joins.  Integer work: everything must agree exactly.
CPU only; nothing is launched."""
import os
import random
import re

import pytest

import paper_1801_04380_amd as sn
from oracle import sched_oracle as so
from paper_1801_04380_amd import _lib, runtime as rt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MiB = float(1 << 20)


def _mirror(onet):
    """The same network in the library's representation (kinds share their numbering by design of
    the header; checked below)."""
    net = rt.Net()
    for kind, nbytes, prev in onet.layers:
        net.add(kind, nbytes, prev)
    return net


def test_kind_numbers_agree():
    for name in so.KIND_NAMES:
        assert getattr(rt, "SN_L_" + name) == getattr(so, name)
    assert (rt.SN_MEM_BASELINE, rt.SN_MEM_LIVENESS, rt.SN_MEM_OFFLOAD, rt.SN_MEM_RECOMPUTE) == (
        so.BASELINE, so.LIVENESS, so.OFFLOAD, so.RECOMPUTE)
    assert (rt.SN_RECOMP_SPEED, rt.SN_RECOMP_MEMORY, rt.SN_RECOMP_COST_AWARE) == (so.SPEED, so.MEMORY, so.COST_AWARE)


def test_header_symbols_are_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "sn_runtime.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(sn_(?:pool|net)_[a-z0-9_]+)\s*\(", text)))
    assert len(names) >= 17
    lib = _lib.load()
    for name in names:
        assert hasattr(lib, name), name
        assert name in rt.SIGNATURES, "binding lacks " + name


def _levels():
    out = [(so.BASELINE, so.SPEED), (so.LIVENESS, so.SPEED), (so.OFFLOAD, so.SPEED)]
    return out + [(so.RECOMPUTE, s) for s in (so.SPEED, so.MEMORY, so.COST_AWARE)]


def _same_trace(onet):
    net = _mirror(onet)
    assert net.route() == so.route(onet)
    for level, strategy in _levels():
        want = so.memory_trace(onet, level, strategy)
        got = net.memory_trace(level, strategy)
        assert got["bytes"] == want["bytes"], (level, strategy)
        assert got["live"] == want["live"], (level, strategy)
        assert (got["peak"], got["peak_step"], got["tensors"], got["extra"]) == (
            want["peak"], want["peak_step"], want["tensors"], want["extra"]), (level, strategy)
    net.close()


def test_alexnet_matches_the_oracle_and_the_paper():
    onet = so.alexnet()
    _same_trace(onet)
    net = _mirror(onet)
    # the figures Sec. 4.1 and Table 1 print (see tests/golden/alexnet_b200_memory.txt)
    assert round(net.memory_trace(rt.SN_MEM_BASELINE)["peak"] / MiB, 3) == 2189.437
    live = net.memory_trace(rt.SN_MEM_LIVENESS)
    assert (round(live["peak"] / MiB, 3), live["peak_step"], live["live"][31]) == (1489.355, 32, 17)
    off = net.memory_trace(rt.SN_MEM_OFFLOAD)
    assert off["peak_step"] == 39 and off["live"][38] == 9 and abs(off["peak"] / MiB - 1132.155) <= 0.1
    for strategy, peak, extra in ((rt.SN_RECOMP_SPEED, 993.018, 14), (rt.SN_RECOMP_MEMORY, 886.23, 23),
                                  (rt.SN_RECOMP_COST_AWARE, 886.23, 17)):
        r = net.memory_trace(rt.SN_MEM_RECOMPUTE, strategy)
        assert (round(r["peak"] / MiB, 3), r["extra"]) == (peak, extra)
    assert net.memory_trace(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE)["peak_step"] == 44


def _random_net(rnd):
    """A connected network: a chain with forks that rejoin, layer kinds in plausible places."""
    onet = so.Net()
    prev = onet.add(so.DATA, rnd.randint(1, 50) * 1000)
    n = rnd.randint(3, 18)
    open_branches = []
    for _ in range(n):
        r = rnd.random()
        size = rnd.randint(1, 60) * 1000
        if r < 0.15 and len(onet.layers) > 2:
            # fork: two branches from prev that a JOIN closes
            a = onet.add(rnd.choice([so.CONV, so.POOL, so.ACT]), size, [prev])
            b = onet.add(rnd.choice([so.CONV, so.ACT, so.BN]), size, [prev])
            if rnd.random() < 0.5:
                b = onet.add(rnd.choice([so.ACT, so.CONV, so.LRN]), size, [b])
            prev = onet.add(so.JOIN, 2 * size, [a, b])
        else:
            kind = rnd.choice([so.CONV, so.CONV, so.ACT, so.ACT, so.LRN, so.POOL, so.BN, so.FC, so.DROPOUT])
            prev = onet.add(kind, size, [prev])
    onet.add(so.SOFTMAX, 1000, [prev])
    return onet


@pytest.mark.parametrize("seed", range(40))
def test_random_networks_match_the_oracle(seed):
    _same_trace(_random_net(random.Random(seed)))


def test_trace_properties_on_random_networks():
    for seed in range(40, 70):
        onet = _random_net(random.Random(seed))
        net = _mirror(onet)
        base = net.memory_trace(rt.SN_MEM_BASELINE)["peak"]
        live = net.memory_trace(rt.SN_MEM_LIVENESS)
        mem = net.memory_trace(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_MEMORY)
        spd = net.memory_trace(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_SPEED)
        ca = net.memory_trace(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE)
        assert live["peak"] <= base                      # liveness never needs more than the baseline
        assert live["extra"] == 0
        # cost-aware mixes the two per segment (Table 1: between them); on odd networks the whole-segment
        # replay of speed-centric can cost more than memory-centric's targeted one, hence min / max
        assert min(spd["extra"], mem["extra"]) <= ca["extra"] <= max(spd["extra"], mem["extra"])
        assert ca["peak"] <= max(mem["peak"], 1) and ca["l_peak"] == mem["peak"]   # and cost-aware keeps the memory-centric peak
        cap = base
        free = net.step_budgets(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE, cap)
        assert free == [cap - b for b in ca["bytes"]]
        assert net.step_budgets(rt.SN_MEM_LIVENESS, 0, 1) == [0] * net.steps()
        net.close()


def test_route_of_nested_fans():
    onet = so.Net()
    a = onet.add(so.DATA, 10)
    b = onet.add(so.CONV, 10, [a])
    c = onet.add(so.CONV, 10, [b])
    d = onet.add(so.CONV, 10, [b])
    e = onet.add(so.ACT, 10, [c])
    f = onet.add(so.CONV, 10, [d])
    g = onet.add(so.ACT, 10, [f])
    h = onet.add(so.POOL, 10, [f])
    i = onet.add(so.JOIN, 30, [e, g, h])
    j = onet.add(so.SOFTMAX, 30, [i])
    net = _mirror(onet)
    assert net.route() == [a, b, c, e, d, f, g, h, i, j]   # i waits for e, g and h (Alg. 1)
    _same_trace(onet)


def test_pool_matches_the_oracle_pool():
    rnd = random.Random(3)
    size = 200 * rt.SN_POOL_BLOCK + 17
    pool, opool = rt.Pool(size), so.Pool(size)
    held = {}
    for _ in range(5000):
        if held and rnd.random() < 0.48:
            ident = rnd.choice(sorted(held))
            pool.free(ident)
            opool.free(held.pop(ident))
        else:
            nbytes = rnd.choice([0, 1, 1023, 1024, 1025, rnd.randint(1, 30 * 1024)])
            got, want = pool.alloc(nbytes), opool.alloc(nbytes)
            assert (got is None) == (want is None)
            if got:
                assert got[1] == want[1]
                held[got[0]] = want[0]
        assert pool.used_bytes == opool.used_blocks * so.BLOCK
        assert pool.largest_free == opool.largest_free()
    assert pool.peak_bytes == opool.peak_blocks * so.BLOCK
    assert pool.high_water == opool.high_water * so.BLOCK
    with pytest.raises(ValueError):
        pool.free(10 ** 9)


def test_pool_holds_the_tensors_of_a_liveness_schedule():
    """Allocating and freeing AlexNet's tensors step by step through the pool: a pool of the liveness
    peak rounded up to blocks per tensor suffices here, and what is left is the workspace budget."""
    onet = so.alexnet()
    live = so.memory_trace(onet, so.LIVENESS)
    pool = rt.Pool(int(live["peak"] * 1.02))
    assert pool.alloc(int(live["peak"]))            # it fits in one piece
    assert pool.largest_free <= int(live["peak"] * 0.02) + rt.SN_POOL_BLOCK


def test_bad_arguments():
    net = rt.Net()
    with pytest.raises(ValueError):
        net.add(rt.SN_L_CONV, 10, [])          # only a data layer has no input
    d = net.add(rt.SN_L_DATA, 10)
    with pytest.raises(ValueError):
        net.add(rt.SN_L_CONV, 10, [5])         # unknown predecessor
    with pytest.raises(ValueError):
        net.add(rt.SN_L_DATA, 10, [d])
    with pytest.raises(ValueError):
        net.memory_trace(rt.SN_MEM_LIVENESS)   # no layer after the data layer
    c = net.add(rt.SN_L_CONV, 10, [d])
    with pytest.raises(ValueError):
        net.memory_trace(7)
    with pytest.raises(ValueError):
        net.set_conv_shape(d, sn.conv_shape(1, 1, 4, 4, 1, 3, 3))
    net.set_conv_shape(c, sn.conv_shape(1, 1, 4, 4, 1, 3, 3, (1, 1), (1, 1)))


def test_budgets_reach_the_conv_planner():
    """Sec. 3.5: the free bytes of a step are the budget of its CONV call.  VGG-16-shaped convolutions
    at batch 32 in bf16 under a capacity that leaves little at the memory peak: the planner's choice at
    every step needs no more than the step has, and steps with room get a workspace algorithm."""
    from paper_1801_04380_amd import workloads as wl
    cfg = wl.CONFIGS[3]
    N = cfg["N"]
    net = rt.Net()
    prev = net.add(rt.SN_L_DATA, N * 3 * 224 * 224 * 2)
    convs = {}
    for layer in cfg["layers"]:
        P, Q = wl.out_hw(layer)
        out = N * layer.K * P * Q * 2
        prev = net.add(rt.SN_L_CONV, out, [prev])
        convs[prev] = layer
        net.set_conv_shape(prev, sn.conv_shape(N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride,
                                               layer.pad, sn.SN_BF16, sn.SN_BF16))
        prev = net.add(rt.SN_L_BN, out, [prev])
        prev = net.add(rt.SN_L_ACT, out, [prev])
        if layer.pool:
            prev = net.add(rt.SN_L_POOL, out // 4, [prev])
    net.add(rt.SN_L_SOFTMAX, N * 1000 * 2, [prev])
    sn.sn_planner_clear()
    trace = net.memory_trace(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE)
    capacity = trace["peak"] + (1 << 20)
    plans = net.plan_convs(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE, capacity)
    assert [p["layer"] for p in plans] == sorted(convs)
    free = net.step_budgets(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE, capacity)
    staged = 0
    for p in plans:
        assert p["fwd_budget"] == free[p["fwd_step"] - 1] // 256 * 256
        assert p["bwd_budget"] == free[p["bwd_step"] - 1] // 256 * 256
        assert p["ws_fwd"] <= p["fwd_budget"] and p["ws_bwd_data"] <= p["bwd_budget"]
        assert p["ws_bwd_filter"] <= p["bwd_budget"]
        shape = sn.conv_shape(N, *[getattr(convs[p["layer"]], k) for k in ("C", "H", "W", "K", "R", "S")],
                              convs[p["layer"]].stride, convs[p["layer"]].pad, sn.SN_BF16, sn.SN_BF16)
        assert (p["algo_fwd"], p["ws_fwd"]) == sn.sn_conv_plan(shape, sn.SN_CONV_FWD, p["fwd_budget"])[:2]
        staged += p["algo_bwd_filter"] == sn.SN_ALGO_STAGED
    assert staged >= 1
    # with no room at all every call falls back to the zero-workspace algorithm
    for p in net.plan_convs(rt.SN_MEM_RECOMPUTE, rt.SN_RECOMP_COST_AWARE, 0):
        assert (p["algo_fwd"], p["algo_bwd_data"], p["algo_bwd_filter"]) == (sn.SN_ALGO_DIRECT,) * 3
        assert p["ws_fwd"] == p["ws_bwd_data"] == p["ws_bwd_filter"] == 0
