"""The native NPFP** scheduler (behind the C ABI, host code) against the scheduling
oracle: every decision and every table entry identical.  No GPU needed."""
import math
import time

import numpy as np
import pytest

from oracle import npfp_oracle as S
from paper_2505_23317_amd import cfdetr as K

POLICIES = ["C", "CF", "[C]F", "C[F]", "[C][F]"]


def paper_cost(levels=4, nmax=8):
    return [[0.0] + [float(w) if n == 1 else w * n / 2.0 for n in range(1, nmax + 1)]
            for w in range(levels)]


def rand_table(rng, levels, nmax):
    base = np.sort(rng.uniform(0.3, 2.0, levels))
    return [[0.0] + [float(base[l] * (1 + rng.uniform(0.3, 0.9) * (n - 1))) for n in range(1, nmax + 1)]
            for l in range(levels)]


def test_paper_tables_through_the_library():
    C = paper_cost()
    far = 1e9
    order, cuts, dba = K.cfdetr_sched_fine_batches([1, 2, 2, 3], [far] * 4, 0.0, far, C)
    assert dba == [0, 1, 2, 3, 5] and cuts == [(0, 2), (2, 4)]
    order, cuts, dba = K.cfdetr_sched_fine_batches([1, 2, 2, 3, 3], [far] * 5, 0.0, far, C)
    assert dba == [0, 1, 2, 3, 5, 6] and cuts == [(0, 1), (1, 3), (3, 5)]


def test_response_times_match():
    rng = np.random.default_rng(1)
    assert K.cfdetr_sched_response_times([4, 10, 20], [1, 2, 3]) == (True, [4.0, 7.0, 7.0])
    for _ in range(300):
        n = int(rng.integers(1, 9))
        period = np.sort(rng.uniform(2.0, 30.0, n)).tolist()
        c = rng.uniform(0.1, 3.0, n).tolist()
        assert K.cfdetr_sched_response_times(period, c) == S.response_times(period, c)


def test_fine_batches_match_with_constraints_and_unsorted_input():
    rng = np.random.default_rng(2)
    for _ in range(500):
        n = int(rng.integers(0, 13))
        levels = int(rng.integers(1, 4))
        C = rand_table(rng, levels, 12)
        w = rng.integers(0, levels, n).tolist()
        t = float(rng.uniform(0, 10))
        dl = (t + rng.uniform(0.5, 12.0, n)).tolist()
        nxt = t + float(rng.uniform(0.5, 12.0))
        got = K.cfdetr_sched_fine_batches(w, dl, t, nxt, C)
        want = S.fine_batches(w, dl, t, nxt, C)
        assert got[0] == want[0] and got[1] == want[1]
        assert got[2] == want[2]          # same additions in the same order: identical doubles


def test_decisions_match():
    rng = np.random.default_rng(4)
    for _ in range(600):
        n = int(rng.integers(1, 9))
        Cc = [0.0] + np.cumsum(rng.uniform(0.2, 1.0, n)).tolist()
        C = rand_table(rng, 3, n)
        ac = sorted(rng.choice(n, int(rng.integers(0, n + 1)), replace=False).tolist())
        rest = [i for i in range(n) if i not in ac]
        af = sorted(rng.choice(rest, int(rng.integers(0, len(rest) + 1)), replace=False).tolist()) \
            if rest else []
        w = rng.integers(0, 3, len(af)).tolist()
        t = float(rng.uniform(0, 10))
        dl = (t + rng.uniform(0.3, 6.0, len(af))).tolist()
        nxt = t + float(rng.uniform(0.1, 6.0))
        for pol in POLICIES:
            assert K.cfdetr_sched_decide(pol, t, ac, af, w, dl, nxt, Cc, C) == \
                S.decide(pol, t, ac, af, w, dl, nxt, Cc, C), (pol, ac, af)


def test_coarse_batch_rule_and_argument_errors():
    c = [0, 1.0, 1.5, 2.5, 3.0]
    for n, t, nxt in [(4, 10.0, 13.0), (4, 10.0, 12.9), (4, 10.0, 11.4), (1, 0.0, 9.0), (0, 0.0, 9.0),
                      (3, 10.0, 10.5)]:
        assert K.cfdetr_sched_coarse_batch(n, t, nxt, c) == S.coarse_batch_size(n, t, nxt, c)
    assert K.cfdetr_sched_coarse_batch(65, 0.0, 1.0, c) == -1
    with pytest.raises(K.CfdetrError):
        K.cfdetr_sched_response_times([1.0, -2.0], [0.1, 0.1])
    with pytest.raises(K.CfdetrError):      # a workload level the table does not have
        K.cfdetr_sched_fine_batches([0, 5], [9.0, 9.0], 0.0, 9.0, paper_cost(3, 4))
    with pytest.raises(K.CfdetrError):      # table narrower than the batch could get
        K.cfdetr_sched_fine_batches([0, 1, 1], [9.0] * 3, 0.0, 9.0, paper_cost(3, 2))


def test_decision_cost_is_small():
    """The paper wants run-time decisions with minimal overhead: time the worst one here
    (64 active fine subtasks, batched policy) through the C ABI."""
    rng = np.random.default_rng(5)
    lib = K.load_library()
    import ctypes
    n = 64
    C = rand_table(rng, 3, n)
    tab, n_levels, max_size = K._fine_table(C)
    w, dl = K._iarr(rng.integers(0, 3, n).tolist()), K._darr([1e9] * n)
    order, ends = (ctypes.c_int32 * n)(), (ctypes.c_int32 * n)()
    nb = ctypes.c_int32()
    t0 = time.perf_counter()
    reps = 2000
    for _ in range(reps):
        lib.cfdetr_sched_fine_batches(n, w, dl, 0.0, 1e9, tab, n_levels, max_size, order, ends,
                                      ctypes.byref(nb), None)
    us = (time.perf_counter() - t0) / reps * 1e6
    print(f"[sched] dynamic batch assignment of 64 subtasks: {us:.1f} us per call (incl. ctypes)")
    assert us < 200.0
