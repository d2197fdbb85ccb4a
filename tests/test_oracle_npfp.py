"""Pins for the scheduling oracle (Sec. IV): the paper's two worked DP tables, a
response-time example worked by hand, exhaustive search over all contiguous partitions,
and a discrete-event simulation of the lemma that batching never breaks what the offline
test guarantees."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import npfp_oracle as S

GOLD = os.path.join(os.path.dirname(__file__), "golden", "dba_examples.txt")


def paper_cost(levels=4, nmax=8):
    """C_batch of the paper's examples: w alone, w*size/2 in a batch."""
    return [[0.0] + [float(w) if n == 1 else w * n / 2.0 for n in range(1, nmax + 1)]
            for w in range(levels)]


def _gold(name):
    rows, result = [], None
    with open(GOLD) as f:
        for line in f:
            p = line.split()
            if not p or p[0] != name:
                continue
            if p[1] == "result":
                result = (float(p[2]), [tuple(int(v) for v in c.split("-")) for c in p[4:]])
            else:
                rows.append((int(p[1]), int(p[2]), float(p[3]), float(p[4])))
    return rows, result


@pytest.mark.parametrize("name,w", [("T2", [1, 2, 2, 3]), ("T5", [1, 2, 2, 3, 3])])
def test_dp_tables_of_the_paper(name, w):
    rows, (total, cuts) = _gold(name)
    C = paper_cost()
    far = 1e9
    order, got_cuts, dba = S.fine_batches(w, [far] * len(w), 0.0, far, C)
    assert order == list(range(len(w)))
    for k, j, prev, cost in rows:                     # every candidate the table lists
        assert dba[j - 1] == prev
        assert dba[j - 1] + C[w[k - 1]][k - j + 1] == cost
    for k in range(1, len(w) + 1):                    # and each DBA[k] is their minimum
        assert dba[k] == min(c for kk, _, _, c in rows if kk == k)
    assert dba[len(w)] == total and got_cuts == cuts


def test_response_times_by_hand():
    # three tasks, priorities 0 > 1 > 2: C = (1, 2, 3), T = (4, 10, 20)
    # R0 = 1 + B0(3) = 4 <= 4
    # R1: start 2+3 = 5 -> 2+3+ceil(5/4)*1 = 7 -> 2+3+2 = 7: R1 = 7
    # R2: B = 0, start 3 -> 3+1*1+1*2 = 6 -> 3+2+2 = 7 -> 3+2*1+1*2 = 7: R2 = 7
    ok, R = S.response_times([4, 10, 20], [1, 2, 3])
    assert ok and R == [4, 7, 7]
    # a longer low-priority subtask blocks the first one past its period: R0 = 1 + 3.5
    ok, R = S.response_times([4, 10, 20], [1, 2, 3.5])
    assert not ok and R[0] == 4.5
    # interference that keeps growing past the period is reported as unbounded
    ok, R = S.response_times([2, 3], [1.5, 1.0])
    assert not ok and R[1] == math.inf


def test_coarse_batch_rule():
    c = [0, 1.0, 1.5, 2.5, 3.0]
    assert S.coarse_batch_size(4, 10.0, 13.0, c) == 4        # largest that fits (Eq. 5 with =)
    assert S.coarse_batch_size(4, 10.0, 12.9, c) == 3
    assert S.coarse_batch_size(4, 10.0, 11.4, c) == 1        # no batch of two fits: single one
    assert S.coarse_batch_size(1, 10.0, 99.0, c) == 1 and S.coarse_batch_size(0, 0, 9, c) == 0
    # the single subtask runs even when it does not fit (its own guarantee is the offline test)
    assert S.coarse_batch_size(3, 10.0, 10.5, c) == 1


def _best_partition_by_search(w, dl, t, nxt, C):
    """All 2^(N-1) contiguous partitions of every prefix; returns the DBA table."""
    N = len(w)
    best = [0.0] + [math.inf] * N
    for k in range(1, N + 1):
        for bits in itertools.product([0, 1], repeat=k - 1):
            cuts, a = [], 0
            for i, b in enumerate(bits):
                if b:
                    cuts.append((a, i + 1))
                    a = i + 1
            cuts.append((a, k))
            now, ok = t, True
            for a, b in cuts:
                now += C[w[b - 1]][b - a]
                if now > nxt or now > min(dl[a:b]):
                    ok = False
                    break
            if ok:
                best[k] = min(best[k], now - t)
    return best


def test_dp_against_exhaustive_search():
    rng = np.random.default_rng(3)
    C = [[0.0] + [1.0 + 0.2 * l + (0.45 + 0.1 * l) * (n - 1) for n in range(1, 9)] for l in range(3)]
    for trial in range(200):
        N = int(rng.integers(1, 8))
        w = sorted(rng.integers(0, 3, N).tolist())
        t = float(rng.uniform(0, 5))
        dl = (t + rng.uniform(1.0, 8.0, N)).tolist()
        nxt = t + float(rng.uniform(1.0, 8.0))
        order, cuts, dba = S.fine_batches(w, dl, t, nxt, C)
        want = _best_partition_by_search(w, [dl[i] for i in order], t, nxt, C)
        assert dba == pytest.approx(want)
        # the dispatched batches cover a prefix, in order, and meet both constraints
        now, pos = t, 0
        for a, b in cuts:
            assert a == pos and b > a
            pos = b
            now += C[w[b - 1]][b - a]
            assert now <= nxt + 1e-12 and now <= min(dl[i] for i in order[a:b]) + 1e-12
        k = max(i for i in range(N + 1) if dba[i] < math.inf)
        assert pos == k


def test_decision_follows_the_policy():
    Cc = [0, 1.0, 1.5, 2.0]
    Cf = paper_cost()
    # coarse always first; batched only under [C]
    assert S.decide("CF", 0.0, [1, 2], [0], [1], [9.0], 5.0, Cc, Cf) == ("coarse", [1])
    assert S.decide("[C]F", 0.0, [1, 2], [0], [1], [9.0], 5.0, Cc, Cf) == ("coarse", [1, 2])
    # policy C never runs fine subtasks
    assert S.decide("C", 0.0, [], [0], [1], [9.0], 5.0, Cc, Cf) == ("idle", [])
    # F: the highest-priority fine subtask, only if it ends before the next release
    assert S.decide("CF", 0.0, [], [0, 2], [2, 1], [9.0, 9.0], 2.0, Cc, Cf) == ("fine", [[0]])
    assert S.decide("CF", 0.0, [], [0, 2], [2, 1], [9.0, 9.0], 1.9, Cc, Cf) == ("idle", [])
    # [F]: sorted by workload, batches from the DP (S M | M L of Table II)
    kind, batches = S.decide("C[F]", 0.0, [], [0, 1, 2, 3], [3, 2, 1, 2], [99.0] * 4, 99.0, Cc, Cf)
    assert kind == "fine" and batches == [[2, 1], [3, 0]]


def _simulate(policy, period, Cc, Cf, horizon, rng):
    """Discrete-event run: releases at multiples of the period; a coarse subtask decides at
    random whether a fine one follows (with a random workload); every execution takes its
    table WCET.  Returns the number of coarse deadline misses and fine deadline misses."""
    n = len(period)
    t, miss_c, miss_f = 0.0, 0, 0
    pending_c, pending_f = {}, {}          # task -> deadline ; task -> (workload, deadline)
    released = [0] * n
    while t < horizon:
        for i in range(n):
            while released[i] * period[i] <= t + 1e-12:
                if i in pending_c:
                    miss_c += 1
                pending_f.pop(i, None)     # the old job's fine part is dropped at its deadline
                pending_c[i] = (released[i] + 1) * period[i]
                released[i] += 1
        nxt = min(released[i] * period[i] for i in range(n))
        ac, af = sorted(pending_c), sorted(pending_f)
        kind, what = S.decide(policy, t, ac, af, [pending_f[i][0] for i in af],
                              [pending_f[i][1] for i in af], nxt, Cc, Cf)
        if kind == "coarse":
            t += Cc[len(what)]
            for i in what:
                dl = pending_c.pop(i)
                miss_c += t > dl + 1e-9
                if rng.random() < 0.7:
                    pending_f[i] = (int(rng.integers(0, 3)), dl)
        elif kind == "fine":
            for batch in what:
                t += Cf[max(pending_f[i][0] for i in batch)][len(batch)]
                for i in batch:
                    miss_f += t > pending_f.pop(i)[1] + 1e-9
            assert t <= nxt + 1e-9          # fine work never delays a coarse release
        else:
            t = nxt
    return miss_c, miss_f


@pytest.mark.parametrize("policy", ["C", "CF", "[C]F", "C[F]", "[C][F]"])
def test_no_deadline_miss_when_the_offline_test_passes(policy):
    """Lemmas 1 and 2: a task set that passes the response-time test keeps every coarse
    deadline under every policy variant; fine subtasks that are run end by their deadline."""
    rng = np.random.default_rng(17)
    runs = 0
    while runs < 25:
        n = int(rng.integers(2, 6))
        period = sorted(rng.choice([4.0, 5.0, 6.0, 8.0, 10.0, 12.0], n).tolist())
        c1 = float(rng.uniform(0.3, 1.2))
        Cc = [0.0] + [c1 * (1 + 0.55 * (k - 1)) for k in range(1, n + 1)]   # sub-additive
        ok, _ = S.response_times(period, [c1] * n)
        if not ok:
            continue
        runs += 1
        Cf = [[0.0] + [(0.5 + 0.4 * l) * (1 + 0.6 * (k - 1)) for k in range(1, n + 1)]
              for l in range(3)]
        miss_c, miss_f = _simulate(policy, period, Cc, Cf, 200.0, rng)
        assert miss_c == 0 and miss_f == 0
