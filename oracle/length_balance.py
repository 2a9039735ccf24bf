"""Plain CPU oracle of length-based load balancing before rollout (paper section 3.1.1).

TEST INFRASTRUCTURE ONLY.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this; the library's implementation shares no code with it.

The paper fixes the goal and not the rule: from a predicted generation length per
sample, reorder and distribute the samples so that every worker group's batch has
about the same total predicted length.  Reading taken (a heuristic, so the oracle
takes its steps one by one):

  1. visit the samples by decreasing predicted length, equal lengths in increasing
     sample index;
  2. give each sample to the group whose running total is smallest among the groups
     that still have room, the lowest group index on equal totals;
  3. "room": with equal_count, group g takes at most n // G + (1 if g < n % G else 0)
     samples (synchronous data-parallel workers get equal-sized batches); without
     it every group always has room (longest-processing-time-first list scheduling).

Outputs: group_of[i]; order = the sample indices listed group after group, inside a
group in the order they were given to it; bounds[g]..bounds[g+1] = that group's slice
of order; totals[g] = its summed predicted length.
"""
from __future__ import annotations


def balance_lengths(pred_len, n_groups: int, equal_count: bool):
    """Steps 1-3 above with plain loops; lengths are non-negative Python ints."""
    n = len(pred_len)
    if n_groups < 1:
        raise ValueError("n_groups >= 1")
    if any(int(v) < 0 for v in pred_len):
        raise ValueError("lengths are non-negative")
    visit = sorted(range(n), key=lambda i: (-int(pred_len[i]), i))
    room = [n // n_groups + (1 if g < n % n_groups else 0) if equal_count else n for g in range(n_groups)]
    totals = [0] * n_groups
    members = [[] for _ in range(n_groups)]
    group_of = [-1] * n
    for i in visit:
        best = -1
        for g in range(n_groups):
            if len(members[g]) >= room[g]:
                continue
            if best < 0 or totals[g] < totals[best]:
                best = g
        members[best].append(i)
        totals[best] += int(pred_len[i])
        group_of[i] = best
    order, bounds = [], [0]
    for g in range(n_groups):
        order.extend(members[g])
        bounds.append(len(order))
    return group_of, order, bounds, totals


def makespan(pred_len, group_of, n_groups: int) -> int:
    """Largest group total of an assignment (what the slowest worker group decodes)."""
    t = [0] * n_groups
    for i, g in enumerate(group_of):
        t[g] += int(pred_len[i])
    return max(t) if t else 0
