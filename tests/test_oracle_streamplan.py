"""Pins for oracle/streamplan.py (Section 5, Algorithm 1 and the cost model of the same section)."""
import itertools
import os
import random

import pytest

from oracle import streamplan as sp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "streamplan_worked.txt")


LEVELING = ([12.0, 5.0, 30.0, 2.0], [4.0, 10.0, 0.05, 0.01], 800, 100, 8, 1500.0, 0.0, 1)


HALF_YES = ([12.0, 30.0], [0.01, 10.0], 800, 100, 2, 1100.0, 0.0, 1)
HALF_NO = ([20.0, 30.0], [0.01, 10.0], 800, 100, 2, 1100.0, 0.0, 1)


def golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or ":" not in line:
            continue
        key, val = line.split(":")
        out[key.strip()] = [float(x) for x in val.split()]
    return out


def test_worked_runs():
    g = golden()
    p = sp.plan_streams([12.0, 30.0, 6.0], [4.0, 10.0, 1.0], 400, 100, 7, 1e9, 0.5, 2)
    assert p.s == [int(x) for x in g["search_s"]]
    assert p.m == [int(x) for x in g["search_m"]]
    assert p.J == g["search_J"][0]
    assert p.accepted == int(g["search_accepted"][0])
    p = sp.plan_streams(*LEVELING)
    assert p.s == [int(x) for x in g["leveling_s"]]
    assert p.m == [int(x) for x in g["leveling_m"]]
    assert p.J == pytest.approx(g["leveling_J"][0], rel=1e-14)
    assert p.accepted == int(g["leveling_accepted"][0])


def test_printed_cost_model():
    # c(m) = max{t0/s0, t1/s1, t2/s2} * m / b0, retyped with numbers: max(12/2, 30/4, 6/1) = 7.5; * 400 / 100 = 30
    assert sp.predicted_cost([12.0, 30.0, 6.0], [2, 4, 1], 400, 100) == 30.0
    # and the planner's J is that cost when all stages share one micro-batch
    p = sp.plan_streams([12.0, 30.0, 6.0], [4.0, 10.0, 1.0], 400, 100, 7, 1e9, 0.5, 2)
    assert p.J == sp.predicted_cost([12.0, 30.0, 6.0], p.s, 400, 100)
    # one stream, the baseline batch: a stage takes its warm-up time
    assert sp.stage_time(7.25, 1, 64, 64) == 7.25


def brute_force_best(t, P, m, b0):
    K = len(t)
    best = None
    for s in itertools.product(range(1, P - K + 2), repeat=K):
        if sum(s) <= P:
            J = max(sp.stage_time(t[k], s[k], m, b0) for k in range(K))
            if best is None or J < best:
                best = J
    return best


def test_greedy_reaches_the_minimal_bottleneck_when_nothing_limits_it():
    rng = random.Random(2509)
    for trial in range(200):
        K = rng.randint(1, 4)
        P = K + rng.randint(0, 6)
        t = [rng.uniform(0.5, 50.0) for _ in range(K)]
        u = [rng.uniform(0.0, 8.0) for _ in range(K)]
        B = rng.randint(1, 5000)
        b0 = rng.randint(1, 512)
        p = sp.plan_streams(t, u, B, b0, P, 1e18, 0.0, 1)
        assert p.m == [B] * K
        # with continuous random times no two stages tie, so the search only stops when raising the bottleneck
        # stage is no longer possible (budget used up): that is the min-max optimum over all allocations
        assert sum(p.s) <= P
        assert p.J == pytest.approx(brute_force_best(t, P, B, b0), rel=1e-12)


def test_invariants_under_tight_budgets():
    rng = random.Random(447)
    for trial in range(300):
        K = rng.randint(1, 5)
        P = K + rng.randint(0, 5)
        t = [rng.uniform(0.1, 20.0) for _ in range(K)]
        u = [rng.choice([0.0, 0.05, 1.0, 3.0, 64.0]) for _ in range(K)]
        B = rng.randint(1, 2000)
        b0 = rng.randint(1, 300)
        per = sum(u)
        M = rng.choice([per * rng.randint(1, 3000) + 0.5, 1e12])
        eps = rng.choice([0.0, 0.01, 0.5, 5.0])
        tau = rng.randint(1, 3)
        p = sp.plan_streams(t, u, B, b0, P, M, eps, tau)
        assert all(x >= 1 for x in p.s) and sum(p.s) <= P
        assert all(1 <= x <= B for x in p.m)
        assert sp.memory_in_use(p.s, p.m, u) <= M
        J1 = max(sp.stage_time(t[k], 1, min(p.m), b0) for k in range(K))  # one stream each, the uniform m
        assert p.J <= 2.0 * J1 + 1e-12     # leveling at most doubles a stage that was at most half the bottleneck
        assert p.accepted <= P - K
        # the uniform micro-batch of step 1 is maximal: one more sample per stage would not fit (or m = B)
        m0 = min(p.m)
        assert m0 == B or sp.memory_in_use([1] * K, [m0 + 1] * K, u) > M


def test_every_accepted_step_gains_more_than_eps():
    t, u = [40.0, 10.0], [1.0, 1.0]
    # raising stage 0: 40 -> 20 (gain 20) -> 13.33 (gain 6.67) -> 10 (gain 3.33), then stage 1 is the bottleneck
    assert sp.plan_streams(t, u, 100, 100, 10, 1e9, 0.0, 1).s == [4, 1]   # (a fifth stream would leave J at 10)
    assert sp.plan_streams(t, u, 100, 100, 10, 1e9, 7.0, 1).s == [2, 1]
    assert sp.plan_streams(t, u, 100, 100, 10, 1e9, 5.0, 1).s == [3, 1]
    assert sp.plan_streams(t, u, 100, 100, 10, 1e9, 25.0, 4).s == [1, 1]


def test_only_stages_at_most_half_the_bottleneck_are_leveled():
    # 10.01 bytes per sample and a cap of 1100: m = 109 (1091.09 bytes).  Stage times at m = 109: t * 1.09.
    # t0 = 12: 13.08, twice that is below 32.7 -> m0 becomes min(800 // 2, 218) = 218 (1.09 bytes more: fits)
    assert sp.plan_streams(*HALF_YES).m == [218, 109]
    # t0 = 20: 21.8, twice that is above 32.7 -> stays
    assert sp.plan_streams(*HALF_NO).m == [109, 109]


def test_a_tie_between_two_bottlenecks_stops_the_search():
    # two equal stages: one more stream on either leaves the maximum where it is, so nothing is accepted
    p = sp.plan_streams([10.0, 10.0, 1.0], [1.0, 1.0, 1.0], 64, 64, 9, 1e9, 0.0, 2)
    assert p.s == [1, 1, 1] and p.accepted == 0 and p.J == 10.0


def test_special_cases():
    p = sp.plan_streams([5.0], [2.0], 1000, 100, 4, 1e9, 0.0, 1)      # one stage takes the whole budget
    assert p.s == [4] and p.m == [1000] and p.J == 5.0 / 4 * 1000 / 100
    p = sp.plan_streams([5.0, 9.0], [2.0, 2.0], 1000, 100, 2, 1e9, 0.0, 1)   # P = K: nothing to hand out
    assert p.s == [1, 1] and p.accepted == 0
    p = sp.plan_streams([5.0, 9.0], [2.0, 2.0], 1000, 100, 8, 4000.0, 0.0, 3)  # memory admits no second stream
    assert p.s == [1, 1] and p.m == [1000, 1000]
    p = sp.plan_streams([5.0, 9.0], [2.0, 2.0], 1000, 100, 8, 3999.0, 0.0, 3)
    assert p.s == [1, 1] and p.m == [999, 999]
    with pytest.raises(ValueError):
        sp.plan_streams([5.0, 9.0], [2.0, 2.0], 1000, 100, 8, 3.0, 0.0, 3)     # not even one sample fits
    with pytest.raises(ValueError):
        sp.plan_streams([5.0, 9.0], [2.0, 2.0], 1000, 100, 1, 1e9, 0.0, 3)     # fewer streams than stages
    with pytest.raises(ValueError):
        sp.plan_streams([5.0, 0.0], [2.0, 2.0], 1000, 100, 4, 1e9, 0.0, 3)


def test_planted_mistakes_are_caught():
    """A plausible slip in the planner fails one of the pins above: shown by planting each in a copy."""
    import inspect
    src = inspect.getsource(sp)
    slips = [("t_k / s_k * m_k / b0", "t_k * s_k * m_k / b0"),            # streams slow a stage down
             ("if delta > gain:", "if delta < gain:"),                     # keeps the worst candidate
             ("m_unit = max(1, B // u_s)", "m_unit = max(1, B // K)"),     # unit from the stage count
             ("m_new = min(m_unit, 2 * m[k])", "m_new = max(m_unit, 2 * m[k])"),
             ("if sum(s2) <= P and", "if"),                                # stream budget ignored
             ("if 2.0 * stage_time(t[k], s[k], m[k], b0) <= J:", "if True:")]
    for old, new in slips:
        assert old in src
        ns = {}
        exec(compile(src.replace(old, new), "<planted>", "exec"), ns)
        plan = ns["plan_streams"]
        bad = False
        try:
            g = golden()
            p = plan([12.0, 30.0, 6.0], [4.0, 10.0, 1.0], 400, 100, 7, 1e9, 0.5, 2)
            bad |= p.s != [int(x) for x in g["search_s"]] or p.J != g["search_J"][0]
            p = plan(*LEVELING)
            bad |= p.m != [int(x) for x in g["leveling_m"]] or p.s != [int(x) for x in g["leveling_s"]]
            bad |= plan(*HALF_NO).m != [109, 109] or plan(*HALF_YES).m != [218, 109]
            p = plan([12.0, 30.0, 6.0], [4.0, 0.5, 0.05], 400, 100, 6, 1500.0, 0.0, 1)
            bad |= ns["memory_in_use"](p.s, p.m, [4.0, 0.5, 0.05]) > 1500.0 or sum(p.s) > 6
        except Exception:
            bad = True
        assert bad, (old, new)
