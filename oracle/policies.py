"""Oracle of the scheduling policies (plain Python over lists).  TEST INFRASTRUCTURE ONLY.

Section 4.5 describes two policies in prose.  Scaling: after a resource grant, chunks are shifted
from the old workers to the new ones (Section 5.3: picked at random from each old task); before a
revocation, the chunks of the workers to be freed are spread round robin over the remaining ones.
Rebalancing: solvers are ranked by their median performance over the last I iterations and chunks
move gradually from slower to faster solvers until the differences are below the estimated
processing time of one chunk.

What the prose leaves open is fixed here (and listed among the readings of the paper):
  * an old solver with m chunks gives away floor(m * (K_new - K_old) / K_new) of them, which leaves
    every solver with about n_chunks / K_new;
  * "random" = the chunks with the smallest caller-supplied random words, so that both
    implementations see the same draws;
  * receivers are served in turn, one chunk each, in the order the chunks are handed over;
  * rebalancing moves one chunk at a time from the solver that would finish last to the one that
    would finish first, lightest chunk first, and at most `max_moves` chunks per call.

Section 2.2 cites that starting with many partitions and reducing them after a few iterations speeds
up convergence, and the summary of the evaluation that such changes pay once convergence slows down.
The paper gives no rule; the one fixed here: a round stalls when it leaves more than `stall_ratio` of
the gap it started from, and `patience` stalled rounds in a row under the current K halve K.
"""
from __future__ import annotations

import statistics
from typing import List, Sequence, Tuple


def scale_out(table: Sequence[int], K_old: int, K_new: int, draw: Sequence[int]) -> List[int]:
    new = list(table)
    n_new = K_new - K_old
    handed = []                                    # in hand-over order
    for k in range(K_old):
        mine = [c for c in range(len(table)) if table[c] == k]
        give = (len(mine) * n_new) // K_new
        by_draw = sorted(mine, key=lambda c: (draw[c], c))
        handed.extend(by_draw[:give])
    for pos, c in enumerate(handed):
        new[c] = K_old + pos % n_new
    return new


def scale_in(table: Sequence[int], K_old: int, K_new: int) -> List[int]:
    new = list(table)
    freed = []
    for k in range(K_new, K_old):
        freed.extend(c for c in range(len(table)) if table[c] == k)
    for pos, c in enumerate(freed):
        new[c] = pos % K_new
    return new


def rebalance(load: Sequence[int], K: int, unit_time: Sequence[Sequence[float]], table: Sequence[int],
              max_moves: int) -> Tuple[List[int], int]:
    """unit_time[i][k]: runtime per unit of load of solver k in the i-th of the last iterations."""
    rate = [statistics.median([row[k] for row in unit_time]) for k in range(K)]
    new = list(table)
    moved = 0
    while moved < max_moves:
        total = [sum(load[c] for c in range(len(new)) if new[c] == k) for k in range(K)]
        time = [rate[k] * float(total[k]) for k in range(K)]
        slow = max(range(K), key=lambda k: (time[k], -k))          # first of the slowest
        fast = min(range(K), key=lambda k: (time[k], k))           # first of the fastest
        if slow == fast:
            break
        mine = [c for c in range(len(new)) if new[c] == slow]
        if not mine:
            break
        pick = min(mine, key=lambda c: (load[c], -c))              # lightest, then larger id
        if not (time[slow] - time[fast] > rate[fast] * float(load[pick])):
            break
        new[pick] = fast
        moved += 1
    return new, moved


def next_solver_count(gaps: Sequence[float], K: int, K_min: int, stall_ratio: float, patience: int,
                      since_change: int) -> int:
    """Number of solvers for the next round, from the gap before the first round and after each round."""
    if K <= K_min or since_change < patience or len(gaps) < patience + 1:
        return K
    recent = range(len(gaps) - patience, len(gaps))
    if all(gaps[t] > stall_ratio * gaps[t - 1] for t in recent):
        return max(K_min, -(-K // 2))
    return K
