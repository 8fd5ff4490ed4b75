"""Pins of the planner oracle (paper Section 7, inequality group; ``ko_plan_batches``) against
things other than itself: hand-solved cases, the definition checked in exact rational arithmetic
(the returned n satisfies every inequality and n - 1 violates one), the two extreme scenarios
the paper describes, and invariances."""
import math
from fractions import Fraction

import numpy as np

from oracle import ref


def satisfied(n, tA, tG, thot, q, ioA, ioG, ioE, K):
    """The four inequalities as printed, in exact rationals (inputs are doubles: exact)."""
    F = Fraction
    tA, tG, thot, ioA, ioG, ioE = map(F, (tA, tG, thot, ioA, ioG, ioE))
    q = [F(v) for v in q]
    ok = n * tA >= ioG and n * (tA + tG) >= ioG + K * ioE
    if q:
        ok = ok and n * (tA + tG) + thot >= ioG + (K + 1) * ioE
        ok = ok and n * (tA + tG) + thot + sum(q) >= ioG + (K + len(q)) * ioE + ioA
    return ok


def test_hand_solved_cases():
    # only the gate transfer matters: n * 2 >= 7  ->  4; exactly divisible: no rounding up
    assert ref.plan_batches(2.0, 0.0, 0.0, [], 0.0, 7.0, 0.0, 0) == 4
    assert ref.plan_batches(2.0, 0.0, 0.0, [], 0.0, 8.0, 0.0, 0) == 4
    assert ref.plan_batches(2.0, 0.0, 0.0, [], 0.0, 0.0, 0.0, 0) == 1          # n is a positive integer
    # II: n * 2.75 >= 1 + 2 * 21 = 43  ->  16 (15 * 2.75 = 41.25)
    assert ref.plan_batches(2.5, 0.25, 0.0, [], 0.0, 1.0, 21.0, 2) == 16
    # III: n * 2.75 + 5 >= 1 + 3 * 21 = 64 -> n >= 21.45 -> 22;
    # IV: n * 2.75 + 5 + 6 >= 1 + 5 * 21 + 4 = 110 -> n >= 36 exactly -> 36
    assert ref.plan_batches(2.5, 0.25, 5.0, [2.0, 2.0, 2.0], 4.0, 1.0, 21.0, 2) == 36
    # no compute at all cannot hide anything
    assert ref.plan_batches(0.0, 0.0, 0.0, [], 0.0, 1.0, 0.0, 0, n_max=1000) == -1


def test_result_is_the_smallest_n_that_satisfies_the_group_exactly():
    g = np.random.Generator(np.random.PCG64(77))
    for trial in range(300):
        tA, tG = float(g.uniform(0.01, 3.0)), float(g.uniform(0.0, 0.5))
        thot = float(g.uniform(0.0, 4.0))
        q = [float(v) for v in g.uniform(0.0, 2.0, size=int(g.integers(0, 7)))]
        ioA, ioG, ioE = float(g.uniform(0, 5)), float(g.uniform(0, 2)), float(g.uniform(0, 30))
        K = int(g.integers(0, 5))
        n = ref.plan_batches(tA, tG, thot, q, ioA, ioG, ioE, K)
        assert n >= 1 and satisfied(n, tA, tG, thot, q, ioA, ioG, ioE, K), trial
        assert n == 1 or not satisfied(n - 1, tA, tG, thot, q, ioA, ioG, ioE, K), trial


def test_each_inequality_can_be_the_binding_one():
    base = dict(tA=1.0, tG=1.0, thot=0.0, q=[1.0], ioA=0.0, ioG=0.0, ioE=0.0, K=1)

    def n_of(**kw):
        a = dict(base, **kw)
        return ref.plan_batches(a["tA"], a["tG"], a["thot"], a["q"], a["ioA"], a["ioG"], a["ioE"], a["K"])
    assert n_of() == 1
    assert n_of(ioG=10.0) == 10                       # I: n * tA >= ioG (tG does not help here)
    assert n_of(ioE=16.0, K=1, thot=16.0, q=[16.0]) == 8   # II: 2n >= 16; III, IV slack
    assert n_of(ioE=16.0, K=0, thot=0.0, q=[32.0]) == 8    # III: 2n >= (0+1)*16; II needs nothing
    assert n_of(ioA=40.0, q=[1.0, 1.0]) == 19         # IV: 2n + 2 >= 40
    # the attention transfer enters IV only, the queue's compute only IV
    assert n_of(ioA=40.0, q=[30.0, 9.0]) == 1 and n_of(ioA=40.0, thot=38.0, q=[1.0, 1.0]) == 1


def test_best_and_worst_case_of_the_paper():
    # best case: every token on hot experts -> empty queue -> III and IV do not apply, whatever
    # the hot experts' compute or the attention weights' transfer time
    args = (2.5, 0.25)
    assert ref.plan_batches(*args, 100.0, [], 50.0, 1.0, 21.0, 2) == ref.plan_batches(*args, 0.0, [], 0.0, 1.0, 21.0, 2) == 16
    # worst case: nobody picked a hot expert (t_hot = 0): never a smaller n than with hot compute
    for q in ([2.0] * 3, [0.5] * 6):
        assert ref.plan_batches(*args, 0.0, q, 4.0, 1.0, 21.0, 2) >= ref.plan_batches(*args, 5.0, q, 4.0, 1.0, 21.0, 2)


def test_invariances_and_monotonicity():
    g = np.random.Generator(np.random.PCG64(3))
    for _ in range(50):
        a = [float(v) for v in g.uniform(0.05, 4.0, size=6)]
        q = [float(v) for v in g.uniform(0.0, 2.0, size=4)]
        K = int(g.integers(0, 4))
        n = ref.plan_batches(a[0], a[1], a[2], q, a[3], a[4], a[5], K)
        # the unit of time does not matter (a power of two scales every term exactly)
        assert ref.plan_batches(*(8 * v for v in a[:3]), [8 * v for v in q], *(8 * v for v in a[3:]), K) == n
        # the order of the queue does not matter; more compute per batch never needs more batches;
        # slower transfers never need fewer
        assert ref.plan_batches(a[0], a[1], a[2], q[::-1], a[3], a[4], a[5], K) == n
        assert ref.plan_batches(2 * a[0], a[1], a[2], q, a[3], a[4], a[5], K) <= n
        assert ref.plan_batches(a[0], a[1], a[2], q, a[3], a[4], 2 * a[5], K) >= n
