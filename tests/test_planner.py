"""CPU-only property tests of the planner against brute force on made-up timing
tables (Sec. 3.5: skip the algorithms that need more memory than is free, take
the fastest of the rest; more workspace never makes the plan slower)."""
import itertools
import random

import paper_1801_04380_amd as sn

DIRS = (sn.SN_CONV_FWD, sn.SN_CONV_BWD_DATA, sn.SN_CONV_BWD_FILTER)
ALGOS = (sn.SN_ALGO_DIRECT, sn.SN_ALGO_IM2COL_GEMM, sn.SN_ALGO_STAGED, sn.SN_ALGO_WINOGRAD)


def _needs(shape, d):
    out = {}
    for a in ALGOS:
        try:
            out[a] = sn.sn_conv_workspace_query(shape, d, a)
        except sn.SnError as e:
            assert e.status == 2
    return out


def test_cold_start_ranking_is_always_feasible():
    sn.sn_planner_clear()
    shape = sn.conv_shape(8, 64, 28, 28, 64, 3, 3, (1, 1), (1, 1), sn.SN_BF16, sn.SN_BF16)
    for d in DIRS:
        needs = _needs(shape, d)
        for budget in (0, 255, 256, 1 << 16, 1 << 22, 1 << 34):
            algo, used, ms = sn.sn_conv_plan(shape, d, budget)
            assert ms is None
            assert algo in needs and needs[algo][0] <= budget and used <= budget
        assert sn.sn_conv_plan(shape, d, 0)[0] == sn.SN_ALGO_DIRECT


def test_fastest_feasible_matches_brute_force():
    rnd = random.Random(5)
    shape = sn.conv_shape(4, 32, 20, 20, 48, 3, 3, (1, 1), (1, 1), sn.SN_BF16, sn.SN_F32)
    other = sn.conv_shape(4, 32, 20, 20, 48, 3, 3, (2, 2), (1, 1), sn.SN_BF16, sn.SN_F32)
    for trial in range(20):
        sn.sn_planner_clear()
        table = []
        for d in DIRS:
            needs = _needs(shape, d)
            for a, (mn, pf) in needs.items():
                for ws in sorted({mn, pf, (mn + pf) // 2}):
                    if rnd.random() < 0.8:
                        ms = round(rnd.uniform(0.1, 5.0), 3)
                        sn.sn_planner_record(shape, d, a, ws, ms)
                        table.append((d, a, ws, ms))
        # records of another shape must not leak in
        sn.sn_planner_record(other, sn.SN_CONV_FWD, sn.SN_ALGO_DIRECT, 0, 0.001)
        for d in DIRS:
            rows = [r for r in table if r[0] == d]
            budgets = sorted({0, 1 << 40} | {r[2] for r in rows} | {max(r[2] - 1, 0) for r in rows})
            last = None
            for budget in budgets:
                feasible = [r for r in rows if r[2] <= budget]
                algo, used, ms = sn.sn_conv_plan(shape, d, budget)
                if feasible:
                    # the fastest; among the records within 3 % of it the smallest workspace, then the faster
                    fastest = min(r[3] for r in feasible)
                    near = [r for r in feasible if r[3] <= fastest * 1.03 + 1e-9]
                    best = min(near, key=lambda r: (r[2], r[3]))
                    assert abs(ms - best[3]) < 1e-6 and used == best[2] and algo == best[1], (trial, d, budget)
                    assert ms <= fastest * 1.03 + 1e-6
                    if last is not None:
                        assert fastest <= last + 1e-6   # a bigger budget never makes the fastest feasible step slower
                    last = fastest
                else:
                    assert ms is None and used <= budget
    sn.sn_planner_clear()


def test_record_rejects_infeasible_measurements():
    shape = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1))
    mn, _ = sn.sn_conv_workspace_query(shape, sn.SN_CONV_FWD, sn.SN_ALGO_IM2COL_GEMM)
    try:
        sn.sn_planner_record(shape, sn.SN_CONV_FWD, sn.SN_ALGO_IM2COL_GEMM, mn - 1, 1.0)
        assert False
    except sn.SnError as e:
        assert e.status == 3
    try:
        sn.sn_planner_record(shape, sn.SN_CONV_FWD, sn.SN_ALGO_STAGED, 1 << 20, 1.0)
        assert False
    except sn.SnError as e:
        assert e.status == 2
    # overwriting a record keeps one entry
    sn.sn_planner_clear()
    sn.sn_planner_record(shape, sn.SN_CONV_FWD, sn.SN_ALGO_DIRECT, 0, 2.0)
    sn.sn_planner_record(shape, sn.SN_CONV_FWD, sn.SN_ALGO_DIRECT, 0, 1.5)
    assert abs(sn.sn_conv_plan(shape, sn.SN_CONV_FWD, 0)[2] - 1.5) < 1e-6
    sn.sn_planner_clear()


def test_cold_start_on_strided_shapes_counts_the_passes():
    """Without measurements the phase planes are guessed only where they pay (Sec. 3.5 leaves the
    ranking to measurement; this is the stand-in before any exists): backward-data in at most
    two passes, forward only with the whole batch; the zero-workspace kernel otherwise (never the
    explicit algorithm, which is picked on measurement only)."""
    sn.sn_planner_clear()
    shape = sn.conv_shape(64, 128, 56, 56, 128, 3, 3, (2, 2), (1, 1), sn.SN_BF16, sn.SN_BF16)
    mn, pf = sn.sn_conv_workspace_query(shape, sn.SN_CONV_BWD_DATA, sn.SN_ALGO_STAGED)
    assert mn < pf                                     # one image's planes up to the whole batch
    per_image = (pf - mn) // 63
    assert sn.sn_conv_plan(shape, sn.SN_CONV_BWD_DATA, pf)[0] == sn.SN_ALGO_STAGED
    assert sn.sn_conv_plan(shape, sn.SN_CONV_BWD_DATA, mn + 31 * per_image)[0] == sn.SN_ALGO_STAGED     # 32 images: 2 passes
    algo, used, _ = sn.sn_conv_plan(shape, sn.SN_CONV_BWD_DATA, mn + 30 * per_image)                   # 31 images: 3 passes
    assert algo == sn.SN_ALGO_DIRECT and used == 0
    assert sn.sn_conv_plan(shape, sn.SN_CONV_BWD_DATA, 4096)[0] == sn.SN_ALGO_DIRECT
    fmn, fpf = sn.sn_conv_workspace_query(shape, sn.SN_CONV_FWD, sn.SN_ALGO_STAGED)
    assert sn.sn_conv_plan(shape, sn.SN_CONV_FWD, fpf)[0] == sn.SN_ALGO_STAGED
    assert sn.sn_conv_plan(shape, sn.SN_CONV_FWD, fpf - 256)[0] == sn.SN_ALGO_DIRECT


def test_backward_filter_workspace_is_a_range():
    """STAGED backward-filter on the row-stationary kernel runs with a quarter of its slices upward
    (Sec. 3.5: the more workspace, the faster); without measurements the planner guesses it down to
    half of them and the zero-workspace form below that."""
    sn.sn_planner_clear()
    shape = sn.conv_shape(64, 96, 35, 35, 96, 3, 3, (1, 1), (1, 1), sn.SN_BF16, sn.SN_BF16)
    mn, pf = sn.sn_conv_workspace_query(shape, sn.SN_CONV_BWD_FILTER, sn.SN_ALGO_STAGED)
    per = 96 * 96 * 9 * 4
    assert 0 < mn < pf and pf % per < 256 and mn <= pf // 4 + per + 256
    algo, used, _ = sn.sn_conv_plan(shape, sn.SN_CONV_BWD_FILTER, pf)
    assert algo == sn.SN_ALGO_STAGED and used == pf
    half = mn + (pf - mn) // 3
    algo, used, _ = sn.sn_conv_plan(shape, sn.SN_CONV_BWD_FILTER, half + per)
    assert algo == sn.SN_ALGO_STAGED and used == half + per
    assert sn.sn_conv_plan(shape, sn.SN_CONV_BWD_FILTER, half - per)[0] == sn.SN_ALGO_DIRECT
    assert sn.sn_conv_plan(shape, sn.SN_CONV_BWD_FILTER, mn - 256)[0] == sn.SN_ALGO_DIRECT
