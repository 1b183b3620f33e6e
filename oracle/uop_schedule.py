"""Adaptive scheduling and tiling of the uop generator, on the oracle side (Section 4.2, "Adaptive Scheduling and Tiling").

Test infrastructure, not product code; shares nothing with the HIP path.

The paper's generator schedules the DAG of logical operators onto the virtual cores and then chooses the operators'
tilings by removing dominant critical paths one after the other: every operator comes with a set of valid
decompositions into uops, every uop and dependency edge with a cost, a critical path is dominant when its cost exceeds
the average cost per core by more than a threshold, and the operators on such a path get another tiling until the
expected benefit is marginal or no dominant path is left.  The paper gives this in prose only; what is fixed here
(readings, listed in the design notes):

* operator: a matvec of `n_blocks` row blocks whose K range is `nk` tile steps long.  Its decompositions: the K range of
  every row block cut into S = 1 .. `max_parts` ranges (range s = steps [nk s / S, nk (s + 1) / S)), one work item per
  (range, row block), items in that order.  The items of ranges 0 .. S - 2 store partial sums and signal; the item of the
  last range of a row block waits for them, adds them (`group` of them per joining step) and stores the result.
* schedule: the NI = n_blocks * S items of an operator are dealt in contiguous shares, core c taking items
  [NI c / C, NI (c + 1) / C) and its j-th item going to its compute core j mod V.  A compute core is a lane; lanes work
  through their items in order.
* cost model (integers): a tile step costs `step`, every item `item` on top (output region and store), every partial
  joining step `join`, and a dependency edge `edge` between the end of the producing item and the moment
  the joining item may use it.  A joining item first works through its own range, then waits if it must.  The span of
  an operator is the time its last lane ends; its work is the sum of its items' costs without waiting.
* critical path: the longest path through the operator DAG, an operator weighing its span (an operator starts when all
  its predecessors have ended).  Average cost per core: the work of all operators over the number of lanes.
* the loop: while the critical path costs more than (100 + threshold_pct) % of the average, take, among the operators
  on the path and all their finer decompositions, the one that shortens its operator's span most (first found wins
  ties: operators from the source of the path on, coarser before finer); stop when that gain is below min_gain_pct % of
  the path's cost (marginal) or nothing finer is left.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class Op:
    n_blocks: int
    nk: int
    max_parts: int = 1
    preds: tuple = ()           # indices of operators that must have ended before this one starts (all smaller than its own)
    group: int = 1              # partial results that one joining step adds


@dataclass(frozen=True)
class Cost:
    step: int
    item: int
    join: int
    edge: int


def item_lane(i, NI, C, V):
    """The lane (core * V + compute core) of item i when NI items are dealt in contiguous shares over C cores."""
    c = i * C // NI                                     # then settle on the core c with NI c / C <= i < NI (c + 1) / C
    while NI * c // C > i:
        c -= 1
    while NI * (c + 1) // C <= i:
        c += 1
    return c * V + (i - NI * c // C) % V


def op_cost(op, S, C, V, cost):
    """(span, work) of one operator under the decomposition S."""
    NB, nk = op.n_blocks, op.nk
    NI = NB * S
    lane_t = [0] * (C * V)
    finish = [0] * NI
    work = 0
    for i in range(NI):
        s, rb = divmod(i, NB)
        own = (nk * (s + 1) // S - nk * s // S) * cost.step
        lane = item_lane(i, NI, C, V)
        if s < S - 1 or S == 1:
            t = lane_t[lane] + own + cost.item
            work += own + cost.item
        else:
            ready = max(finish[sp * NB + rb] for sp in range(S - 1)) + cost.edge
            joins = -(-(S - 1) // op.group)
            t = max(lane_t[lane] + own, ready) + joins * cost.join + cost.item
            work += own + joins * cost.join + cost.item
        finish[i] = t
        lane_t[lane] = t
    return max(lane_t) if NI else 0, work


def critical_path(spans, preds):
    """Longest path through the DAG, node o weighing spans[o]: (cost, [operators from source to sink]).  Ties: the
    predecessor and the sink with the lowest index."""
    n = len(spans)
    dist, via = [0] * n, [-1] * n
    for o in range(n):
        best, arg = 0, -1
        for p in preds[o]:
            assert 0 <= p < o, "operators are listed in a topological order"
            if dist[p] > best:
                best, arg = dist[p], p
        dist[o], via[o] = best + spans[o], arg
    if n == 0:
        return 0, []
    end = max(range(n), key=lambda o: (dist[o], -o))
    path = []
    o = end
    while o >= 0:
        path.append(o)
        o = via[o]
    return dist[end], path[::-1]


def adaptive_tiling(ops, C, V, cost, threshold_pct=10, min_gain_pct=3):
    """The decomposition S of every operator after the dominant critical paths have been removed, and the log of the
    loop: per look at the graph (path cost, average cost per lane, path, refined operator or -1, its new S, gain)."""
    memo = {}

    def oc(o, S):
        if (o, S) not in memo:
            memo[(o, S)] = op_cost(ops[o], S, C, V, cost)
        return memo[(o, S)]

    parts = [1] * len(ops)
    preds = [op.preds for op in ops]
    log = []
    while True:
        spans = [oc(o, parts[o])[0] for o in range(len(ops))]
        avg = sum(oc(o, parts[o])[1] for o in range(len(ops))) // (C * V)
        pc, path = critical_path(spans, preds)
        if pc * 100 <= avg * (100 + threshold_pct):
            log.append((pc, avg, path, -1, 0, 0))
            break
        best = (0, -1, 0)
        for o in path:
            for S in range(parts[o] + 1, ops[o].max_parts + 1):
                gain = spans[o] - oc(o, S)[0]
                if gain > best[0]:
                    best = (gain, o, S)
        gain, o, S = best
        if gain <= 0 or gain * 100 < pc * min_gain_pct:
            log.append((pc, avg, path, -1, 0, gain))
            break
        log.append((pc, avg, path, o, S, gain))
        parts[o] = S
    return parts, log
