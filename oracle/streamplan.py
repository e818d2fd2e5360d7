"""Oracle for the adaptive stream / micro-batch planner.  TEST INFRASTRUCTURE ONLY (same rules as
oracle/__init__.py): imported by tests, smoke() and the CPU baseline leg of bench.py, never by the package.

What it follows: Section 5, "Adaptive multi-channel horizontal fusion" and Algorithm 1 (warm-up figures in,
streams per stage s[k] and micro-batch per stage m[k] out), with the cost model printed at the end of Section 5
(predicted bottleneck cost c(m) = max_k(t_k / s_k) * m / b0 for a micro-batch m under a baseline batch b0).
The steps are taken in the algorithm's order and notation.  Where the listing leaves something open, the
reading is stated next to the line that needs it; the same list stands in the design notes.

Arithmetic: IEEE doubles, every expression evaluated left to right as written (no fused multiply-add), so
that an implementation that writes the same expressions in double takes the same integer decisions.

Pins (tests/test_oracle_streamplan.py): a run worked out by hand (tests/golden/streamplan_worked.txt), the
printed cost model on its own, brute force over all stream allocations on small instances (with ample memory
and eps = 0 the greedy search ends on an allocation with the minimal bottleneck whenever no tie stops it),
invariants (budgets respected, every accepted step gains more than eps, the bottleneck never grows) and
special cases (one stage, P = K, memory that admits no second stream).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence


def stage_time(t_k: float, s_k: int, m_k: int, b0: int) -> float:
    """TIME(k, s[k], m[k]) of Algorithm 1 under the cost model of Section 5: a stage whose warm-up time for the
    baseline batch b0 on one stream was t_k takes t_k / s_k * m_k / b0 for a micro-batch m_k on s_k streams."""
    return t_k / s_k * m_k / b0


def predicted_cost(t: Sequence[float], s: Sequence[int], m: int, b0: int) -> float:
    """c(m) = max{t_0/s_0, t_1/s_1, ...} * m / b0, the cost model as printed (Section 5)."""
    return max(t_k / s_k for t_k, s_k in zip(t, s)) * m / b0


def memory_in_use(s: Sequence[int], m: Sequence[int], u: Sequence[float]) -> float:
    """sum_k s[k] * m[k] * u[k]: every stream of a stage holds one micro-batch of that stage."""
    total = 0.0
    for s_k, m_k, u_k in zip(s, m, u):
        total = total + (s_k * m_k) * u_k
    return total


@dataclass
class Plan:
    s: List[int]      # streams per stage
    m: List[int]      # micro-batch per stage
    J: float          # bottleneck latency max_k TIME(k, s[k], m[k]) of the returned plan
    accepted: int     # number of stream increments the search accepted


def plan_streams(t: Sequence[float], u: Sequence[float], B: int, b0: int, P: int, M_cap: float,
                 eps: float, tau: int) -> Plan:
    """Algorithm 1.  t[k]: warm-up time of stage k for a batch of b0 samples on one stream; u[k]: bytes one
    sample occupies in stage k; B: global batch; P: stream budget; M_cap: memory cap in bytes; eps: smallest
    gain worth a stream; tau: stall cap."""
    K = len(t)
    if K < 1 or len(u) != K or B < 1 or b0 < 1 or P < K or tau < 1:
        raise ValueError("bad arguments")
    if any(not (x > 0.0) for x in t) or any(not (x >= 0.0) for x in u) or not (eps >= 0.0):
        raise ValueError("bad arguments")

    # Step 1 (the warm-up itself is the caller's: t and u come in).  One stream per stage, the largest uniform m
    # that fits.  Reading: m is also at most B (a micro-batch cannot exceed the batch); no m >= 1 fits: error.
    s = [1] * K
    per_sample = memory_in_use(s, [1] * K, u)
    m0 = B
    if per_sample > 0.0 and M_cap / per_sample < float(B):
        m0 = int(M_cap / per_sample)  # an estimate: the two loops below settle rounding either way
    while m0 >= 1 and memory_in_use(s, [m0] * K, u) > M_cap:
        m0 -= 1
    while m0 < B and memory_in_use(s, [m0 + 1] * K, u) <= M_cap:
        m0 += 1
    if m0 < 1:
        raise ValueError("not even one sample per stage fits the memory cap")
    m = [m0] * K
    J = max(stage_time(t[k], s[k], m[k], b0) for k in range(K))
    stall = 0
    accepted = 0

    # Step 2: adaptive search.  Reading: a candidate must also respect the global stream cap sum_k s[k] <= P
    # (stated in the text, absent from the listing); ties keep the first stage (strict ">").  When no candidate
    # gains more than eps nothing changes, so the remaining iterations up to the stall cap repeat the same scan.
    while stall < tau:
        gain = 0.0
        best = None
        for k in range(K):
            s2 = list(s)
            s2[k] = s[k] + 1
            if sum(s2) <= P and memory_in_use(s2, m, u) <= M_cap:
                J2 = max(stage_time(t[j], s2[j], m[j], b0) for j in range(K))
                delta = J - J2
                if delta > gain:
                    gain = delta
                    best = s2
        if gain > eps:
            s = best
            J = max(stage_time(t[k], s[k], m[k], b0) for k in range(K))
            stall = 0
            accepted += 1
        else:
            stall += 1

    # Step 3: micro-batch leveling.  Readings: "much faster than the bottleneck" = at most half of it (doubling
    # the micro-batch then does not make the stage the new bottleneck); "memory allows" = the cap still holds
    # with the new m[k]; the text says the micro-batch is increased up to the bound, so a bound below the
    # current m[k] leaves it alone; J is the search's, not recomputed between stages.
    u_s = sum(s)
    m_unit = max(1, B // u_s)
    for k in range(K):
        if 2.0 * stage_time(t[k], s[k], m[k], b0) <= J:
            m_new = min(m_unit, 2 * m[k])
            if m_new > m[k]:
                m2 = list(m)
                m2[k] = m_new
                if memory_in_use(s, m2, u) <= M_cap:
                    m = m2
    J_out = max(stage_time(t[k], s[k], m[k], b0) for k in range(K))
    return Plan(s=list(s), m=list(m), J=J_out, accepted=accepted)
