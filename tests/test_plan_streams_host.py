"""Host logic of the library without a GPU: qrm_plan_streams (Section 5, Algorithm 1) against the oracle."""
import random

import pytest

from oracle import streamplan as sp


@pytest.fixture(scope="module")
def binding():
    from paper_2509_02447_amd import binding as b
    b.load_library()
    return b


def compare(binding, t, u, B, b0, P, M, eps, tau):
    st, s, m, J, acc = binding.qrm_plan_streams(t, u, B, b0, P, M, eps, tau)
    try:
        ref = sp.plan_streams(t, u, B, b0, P, M, eps, tau)
    except ValueError:
        assert st != 0, (t, u, B, b0, P, M, eps, tau)
        return None
    assert st == 0, (st, t, u, B, b0, P, M, eps, tau)
    assert s == ref.s and m == ref.m and acc == ref.accepted, (t, u, B, b0, P, M, eps, tau, s, m, ref)
    assert J == ref.J          # same expressions in double on both sides: bit for bit
    return ref


def test_worked_runs_and_special_cases(binding):
    ref = compare(binding, [12.0, 30.0, 6.0], [4.0, 10.0, 1.0], 400, 100, 7, 1e9, 0.5, 2)
    assert ref.s == [2, 4, 1] and ref.J == 30.0
    ref = compare(binding, [12.0, 5.0, 30.0, 2.0], [4.0, 10.0, 0.05, 0.01], 800, 100, 8, 1500.0, 0.0, 1)
    assert ref.s == [1, 1, 2, 1] and ref.m == [106, 106, 106, 160]
    compare(binding, [12.0, 30.0], [0.01, 10.0], 800, 100, 2, 1100.0, 0.0, 1)
    compare(binding, [20.0, 30.0], [0.01, 10.0], 800, 100, 2, 1100.0, 0.0, 1)
    compare(binding, [10.0, 10.0, 1.0], [1.0, 1.0, 1.0], 64, 64, 9, 1e9, 0.0, 2)
    compare(binding, [5.0], [2.0], 1000, 100, 4, 1e9, 0.0, 1)
    compare(binding, [5.0, 9.0], [2.0, 2.0], 1000, 100, 8, 3999.0, 0.0, 3)
    compare(binding, [5.0, 9.0], [0.0, 0.0], 1000, 100, 8, 0.0, 0.0, 3)            # no memory needed at all


def test_random_instances_equal_the_oracle(binding):
    rng = random.Random(20250902)
    for trial in range(3000):
        K = rng.randint(1, 6)
        P = K + rng.randint(0, 10)
        t = [rng.choice([rng.uniform(1e-4, 0.1), rng.uniform(0.1, 50.0), float(rng.randint(1, 20))]) for _ in range(K)]
        u = [rng.choice([0.0, 0.01, 0.05, 1.0, 3.0, 9.0, 196608.0, rng.uniform(0.0, 1e6)]) for _ in range(K)]
        B = rng.choice([1, 7, 256, 4096, 8192, rng.randint(1, 100000)])
        b0 = rng.choice([1, 64, 8192, rng.randint(1, 10000)])
        per = sum(u)
        M = rng.choice([per * rng.randint(1, max(1, 2 * B)) * rng.choice([1.0, 1.0 + 1e-9, 0.999]), 1e15, per * 0.5])
        eps = rng.choice([0.0, 1e-6, 0.01, 0.5, 5.0])
        tau = rng.randint(1, 3)
        compare(binding, t, u, B, b0, P, M, eps, tau)


def test_errors(binding):
    ok = ([1.0, 2.0], [1.0, 1.0], 100, 10, 4, 1e9, 0.0, 1)
    assert binding.qrm_plan_streams(*ok)[0] == 0
    bad = [([1.0, 0.0], [1.0, 1.0], 100, 10, 4, 1e9, 0.0, 1),          # a stage that takes no time
           ([1.0, float("nan")], [1.0, 1.0], 100, 10, 4, 1e9, 0.0, 1),
           ([1.0, 2.0], [1.0, -1.0], 100, 10, 4, 1e9, 0.0, 1),
           ([1.0, 2.0], [1.0, 1.0], 0, 10, 4, 1e9, 0.0, 1),
           ([1.0, 2.0], [1.0, 1.0], 100, 0, 4, 1e9, 0.0, 1),
           ([1.0, 2.0], [1.0, 1.0], 100, 10, 1, 1e9, 0.0, 1),           # fewer streams than stages
           ([1.0, 2.0], [1.0, 1.0], 100, 10, 4, 1e9, -1.0, 1),
           ([1.0, 2.0], [1.0, 1.0], 100, 10, 4, 1e9, 0.0, 0),
           ([1.0] * 65, [1.0] * 65, 100, 10, 100, 1e9, 0.0, 1)]         # more stages than the library takes
    for args in bad:
        assert binding.qrm_plan_streams(*args)[0] == 1, args
    assert binding.qrm_plan_streams([1.0, 2.0], [1.0, 1.0], 100, 10, 4, 1.5, 0.0, 1)[0] == 2   # nothing fits
