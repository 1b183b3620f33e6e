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
  With `surplus` = T the builder offers every cut a second time for the last T row blocks alone (the blocks that are
  left over when the others go round the compute cores evenly): the first n_blocks - T blocks stay whole and are dealt
  first, in contiguous shares of their own, then the items of the cut blocks.
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
  on the path and all their finer decompositions (a larger S, of the surplus or of all blocks), the one that shortens
  its operator's span most (first found wins ties: operators from the source of the path on, coarser before finer, the
  surplus before all blocks); stop when that gain is below min_gain_pct % of
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
    surplus: int = 0            # T > 0: the builder also offers cuts of the last T row blocks alone (0 < T < n_blocks)


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


def op_cost(op, S, C, V, cost, tail=0):
    """(span, work) of one operator under the decomposition (S, tail): tail = 0 cuts every row block into S ranges, tail = T
    leaves the first n_blocks - T row blocks whole (dealt first, in contiguous shares of their own) and cuts the last T."""
    NB, nk = op.n_blocks, op.nk
    T = (tail if tail else NB) if S > 1 else 0
    NW = NB - T
    NI = T * S
    lane_t = [0] * (C * V)
    work = 0
    for j in range(NW):
        lane_t[item_lane(j, NW, C, V)] += nk * cost.step + cost.item
        work += nk * cost.step + cost.item
    finish = [0] * NI
    for i in range(NI):
        s, rb = divmod(i, T)
        own = (nk * (s + 1) // S - nk * s // S) * cost.step
        lane = item_lane(i, NI, C, V)
        if s < S - 1:
            t = lane_t[lane] + own + cost.item
            work += own + cost.item
        else:
            ready = max(finish[sp * T + rb] for sp in range(S - 1)) + cost.edge
            joins = -(-(S - 1) // op.group)
            t = max(lane_t[lane] + own, ready) + joins * cost.join + cost.item
            work += own + joins * cost.join + cost.item
        finish[i] = t
        lane_t[lane] = t
    return max(lane_t) if NB else 0, work


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
    """The decomposition (S, tail) of every operator after the dominant critical paths have been removed: (parts, tails,
    log), log = per look at the graph (path cost, average cost per lane, path, refined operator or -1, its new S, gain)."""
    memo = {}

    def oc(o, d):
        if (o, d) not in memo:
            memo[(o, d)] = op_cost(ops[o], d[0], C, V, cost, d[1])
        return memo[(o, d)]

    state = [(1, 0)] * len(ops)
    preds = [op.preds for op in ops]
    log = []
    while True:
        spans = [oc(o, state[o])[0] for o in range(len(ops))]
        avg = sum(oc(o, state[o])[1] for o in range(len(ops))) // (C * V)
        pc, path = critical_path(spans, preds)
        if pc * 100 <= avg * (100 + threshold_pct):
            log.append((pc, avg, path, -1, 0, 0))
            break
        best = (0, -1, None)
        for o in path:
            for S in range(state[o][0] + 1, ops[o].max_parts + 1):
                for tail in ([ops[o].surplus] if ops[o].surplus else []) + [0]:
                    gain = spans[o] - oc(o, (S, tail))[0]
                    if gain > best[0]:
                        best = (gain, o, (S, tail))
        gain, o, d = best
        if gain <= 0 or gain * 100 < pc * min_gain_pct:
            log.append((pc, avg, path, -1, 0, gain))
            break
        log.append((pc, avg, path, o, d[0], gain))
        state[o] = d
    return [d[0] for d in state], [d[1] for d in state], log
