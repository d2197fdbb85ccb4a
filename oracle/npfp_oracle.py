"""CPU oracle for the NPFP** scheduling decisions of CF-DETR (Sec. IV).

TEST INFRASTRUCTURE ONLY, like the encoder oracle next to it: only the test-suite may
import it; the product's scheduler (C++, behind the C ABI) shares no code with it.

What it computes, and where the paper states it:

* the offline schedulability test of individually executed coarse subtasks: the
  response-time recurrence R(x+1) = C_i + B_i + sum over higher priorities of
  ceil(R(x) / T_h) * C_h, started at C_i + B_i, with B_i the longest lower-priority
  coarse subtask (Lemma 1, Eq. 3-4);
* coarse batch assignment (Algo. 2): among the batches made of the x highest-priority
  active coarse subtasks, the largest x >= 2 whose batch WCET fits before the earliest
  future release (P1, P2, Eq. 5); otherwise the single highest-priority subtask;
* fine batch assignment (Algo. 3, Lemma 3, Eq. 6): sort the active fine subtasks by
  workload, cut the sorted sequence into contiguous batches by dynamic programming,
  DBA[k] = min over j of DBA[j-1] + C_batch(w_k, k-j+1), where a batch that would end
  after the deadline of one of its subtasks or after the earliest future coarse
  release costs infinity;
* the generic decision at a scheduling instant (Algo. 1) for the five policy variants.

Readings where the paper is silent (also listed in the design notes):
  - priorities are the task indices, 0 highest; D_i = T_i;
  - batch WCETs come from tables: coarse by batch size, fine by (workload level of the
    largest member, batch size), as for identical cameras (the paper looks them up in a
    measured table);
  - ties in the DP go to the first minimum met when j runs k, k-1, ..., 1, i.e. the
    shortest last batch (what the paper's five-subtask example shows: S | MM | LL);
  - a batch (j..k) starts when the batches before it are done, at t + DBA[j-1], and
    its end t + DBA[j-1] + C must be <= every deadline in it and <= the next coarse
    release; when DBA[N] is infinite, the longest prefix with a finite DBA[k] is
    dispatched (the paper: "a shorter valid prefix ... or no fine batches");
  - sorting by workload is stable with respect to priority.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

INF = math.inf


def response_times(period: Sequence[float], c_coarse: Sequence[float],
                   max_iter: int = 100000) -> Tuple[bool, List[float]]:
    """Lemma 1 (Eq. 3-4).  Returns (schedulable, R) with R[i] = inf when the
    recurrence passes T_i before it converges."""
    n = len(period)
    R = [0.0] * n
    ok = True
    for i in range(n):
        blocking = max([0.0] + [c_coarse[j] for j in range(i + 1, n)])
        r = c_coarse[i] + blocking
        for _ in range(max_iter):
            nxt = c_coarse[i] + blocking + sum(
                math.ceil(r / period[h]) * c_coarse[h] for h in range(i))
            if nxt == r:
                break
            r = nxt
            if r > period[i]:
                r = INF
                break
        R[i] = r
        ok = ok and r <= period[i]
    return ok, R


def coarse_batch_size(n_active: int, t: float, next_release: float,
                      c_batch_by_size: Sequence[float]) -> int:
    """Algo. 2: how many of the highest-priority active coarse subtasks run now.
    c_batch_by_size[x] is the WCET of a batch of x (index 0 unused, [1] = single)."""
    if n_active >= 2:
        for x in range(n_active, 1, -1):
            if c_batch_by_size[x] <= next_release - t:      # Eq. 5
                return x
    return 1 if n_active >= 1 else 0


def fine_batches(workload: Sequence[int], deadline: Sequence[float], t: float,
                 next_coarse_release: float, c_batch: Sequence[Sequence[float]]):
    """Algo. 3 / Lemma 3.  workload[i] is the level (0 = smallest) of active fine
    subtask i (listed by priority), deadline[i] its absolute deadline;
    c_batch[level][size] the WCET of a batch of `size` padded to `level`.
    Returns (order, cuts, dba): the subtasks sorted by workload (stable), the batches as
    half-open index ranges into `order` covering the dispatched prefix, and the table
    DBA[0..N]."""
    N = len(workload)
    order = sorted(range(N), key=lambda i: workload[i])
    w = [workload[i] for i in order]
    dl = [deadline[i] for i in order]
    dba = [0.0] + [INF] * N
    arg = [0] * (N + 1)
    for k in range(1, N + 1):
        for j in range(k, 0, -1):
            if dba[j - 1] == INF:
                continue
            end = t + dba[j - 1] + c_batch[w[k - 1]][k - j + 1]
            if end > next_coarse_release or end > min(dl[j - 1:k]):
                continue
            cost = dba[j - 1] + c_batch[w[k - 1]][k - j + 1]
            if cost < dba[k]:
                dba[k], arg[k] = cost, j
    k = N
    while k > 0 and dba[k] == INF:
        k -= 1
    cuts: List[Tuple[int, int]] = []
    while k > 0:
        cuts.append((arg[k] - 1, k))
        k = arg[k] - 1
    cuts.reverse()
    return order, cuts, dba


def decide(policy: str, t: float, active_coarse: Sequence[int], active_fine: Sequence[int],
           fine_workload: Sequence[int], fine_deadline: Sequence[float],
           next_release: float, c_coarse_by_size: Sequence[float],
           c_fine: Sequence[Sequence[float]]):
    """Algo. 1 for policy in {"C", "CF", "[C]F", "C[F]", "[C][F]"}.
    active_coarse / active_fine: task indices, ascending = by priority; fine_workload and
    fine_deadline are aligned with active_fine; next_release: earliest future release of
    any task.  Returns ("coarse", [tasks]) | ("fine", [[tasks of batch 1], ...]) |
    ("idle", [])."""
    batched_c = policy.startswith("[C]")
    fine_mode = policy[len("[C]") if batched_c else 1:]
    if active_coarse:
        x = coarse_batch_size(len(active_coarse), t, next_release, c_coarse_by_size) \
            if batched_c else 1
        return "coarse", list(active_coarse[:x])
    if active_fine and fine_mode:
        if fine_mode == "[F]" and len(active_fine) >= 2:
            order, cuts, _ = fine_batches(fine_workload, fine_deadline, t, next_release, c_fine)
            batches = [[active_fine[order[i]] for i in range(a, b)] for a, b in cuts]
            return ("fine", batches) if batches else ("idle", [])
        # a single fine subtask (policy F, or only one active): the highest priority one,
        # if it ends before the next coarse release
        if t + c_fine[fine_workload[0]][1] <= next_release:
            return "fine", [[active_fine[0]]]
    return "idle", []
