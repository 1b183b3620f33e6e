"""The generator's adaptive tiling step (Section 4.2, "Adaptive Scheduling and Tiling") on the oracle side, pinned before
any product code: two examples worked by hand, the cost of a decomposition against a clock-tick simulation of the lanes
that is written from the description and shares no formula with it, the longest path on a graph checked by eye, and what
the loop promises: it ends, it only ever shortens the critical path, it touches operators on dominant paths only, and where
it stops there is either no dominant path or no finer tiling with more than a marginal gain."""
import itertools

import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

from oracle import uop_schedule as S

COMMON = dict(deadline=None, max_examples=150, derandomize=True, suppress_health_check=[HealthCheck.too_slow])


def tick_simulation(op, parts, C, V, cost, tail=0):
    """Every lane works through its items one clock tick at a time.  Whole row blocks come first (with `tail` = T the first
    n_blocks - T blocks stay whole and are dealt in shares of their own), then the items of the cut blocks.  An item of an
    earlier K range is `own` ticks of steps and `item` ticks of storing; the item of the last range does its own steps,
    then stands still until every partial result of its row block has been finished for `edge` ticks, then adds them,
    `group` per joining step, and stores.  Returns the tick at which the last lane has nothing left."""
    NB, nk = op.n_blocks, op.nk
    T = 0 if parts == 1 else (tail or NB)
    NW, NI = NB - T, T * parts
    lanes = [[] for _ in range(C * V)]
    for c in range(C):
        for j, b in enumerate(range(NW * c // C, NW * (c + 1) // C)):
            lanes[c * V + j % V] += [("work", nk * cost.step + cost.item), ("done", ("whole", b))]
    for c in range(C):
        for j, i in enumerate(range(NI * c // C, NI * (c + 1) // C)):
            s, rb = i // T, i % T
            own = (nk * (s + 1) // parts - nk * s // parts) * cost.step
            q = lanes[c * V + j % V]
            if s < parts - 1:
                q += [("work", own + cost.item), ("done", i)]
            else:
                q += [("work", own), ("wait", [sp * T + rb for sp in range(parts - 1)]),
                      ("work", len(range(0, parts - 1, op.group)) * cost.join + cost.item), ("done", i)]
    ptr = [0] * len(lanes)
    rem = [q[0][1] if q else 0 for q in lanes]
    finished = {}
    t = 0
    while True:
        moved = True
        while moved:
            moved = False
            for l, q in enumerate(lanes):
                if ptr[l] >= len(q):
                    continue
                kind, arg = q[ptr[l]]
                go = (kind == "work" and rem[l] == 0) or kind == "done" or \
                     (kind == "wait" and all(p in finished and finished[p] + cost.edge <= t for p in arg))
                if kind == "done" and go:
                    finished[arg] = t
                if go:
                    ptr[l] += 1
                    moved = True
                    if ptr[l] < len(q) and q[ptr[l]][0] == "work":
                        rem[l] = q[ptr[l]][1]
        if all(ptr[l] >= len(q) for l, q in enumerate(lanes)):
            return t
        t += 1
        for l, q in enumerate(lanes):
            if ptr[l] < len(q) and q[ptr[l]][0] == "work" and rem[l] > 0:
                rem[l] -= 1
        assert t < 100000


def test_three_row_blocks_on_two_lanes_worked_by_hand():
    """Two cores of one compute core each, three row blocks of eight steps; a step 10, an item 5, a joined partial 10, an
    edge 0.  Uncut: the lanes hold 1 and 2 blocks of 85: span 170, work 255, average 127, so the path is dominant.  In two
    ranges lane 0 holds the three first halves (45 each: done at 45, 90, 135) and lane 1 the three joining items: own steps
    until 40, the partial is there at 45, +10 +5 = 60; 60 + 40 = 100 against 90, +15 = 115; 155 against 135, +15 = 170: no
    gain.  In four ranges (2 steps = 20 per range, partial items 25) lane 0 ends its six items at 25 .. 150, lane 1 holds
    the third ranges (25, 50, 75) and the joining items: 95 against max(25, 100, 25) = 100, +30 +5 = 135; 155 against 125,
    +35 = 190; 210 against max(75, 150, 75), +35 = 245.  In three ranges (2, 3, 3 steps; partial items 25 and 35) the nine
    items are dealt four and five: lane 0 ends (0, 0) (0, 1) (0, 2) (1, 0) at 25, 50, 75, 110; lane 1 ends (1, 1) (1, 2) at
    35, 70, then the joining items: block 0 has its own steps done at 100 and waits for 110, +20 +5 = 135; block 1: 165
    against max(50, 35), +25 = 190; block 2: 220, +25 = 245.  Nothing is shorter than 170: the tiling stays as it is."""
    op = S.Op(3, 8, 4)
    cost = S.Cost(step=10, item=5, join=10, edge=0)
    assert S.op_cost(op, 1, 2, 1, cost) == (170, 255)
    assert S.op_cost(op, 2, 2, 1, cost)[0] == 170
    assert S.op_cost(op, 4, 2, 1, cost)[0] == 245
    assert S.op_cost(op, 3, 2, 1, cost)[0] == 245
    parts, tails, log = S.adaptive_tiling([op], 2, 1, cost, threshold_pct=10, min_gain_pct=3)
    assert parts == [1]
    assert log == [(170, 127, [0], -1, 0, 0)]


def test_the_surplus_block_alone_is_cut_worked_by_hand():
    """The first example again, but the builder also offers cuts of the one row block that is left over when the other two
    have gone round the two lanes.  Whole blocks 0 and 1 end at 85 on either lane.  Block 2 in two ranges: its first half on
    lane 0, 85 + 45 = 130; the joining item on lane 1 has its own steps done at 125, waits for 130, +10 +5 = 145: a gain of
    25 of 170, taken.  (All blocks in two ranges: 170, as before.  The surplus in three ranges, 2, 3, 3 steps: lane 0 ends
    range 0 at 110; lane 1 range 1 at 120 and the joining item at 150 + 20 + 5 = 175.  In four: lane 0 ends ranges 0 and 1
    at 110 and 135, lane 1 range 2 at 110, the joining item waits from 130 to 135, +30 +5 = 170.)  After the cut the work is
    255 + 5 + 10 = 270, the average 135, and 145 is within 10 % of it: the loop ends."""
    op = S.Op(3, 8, 4, (), 1, 1)
    cost = S.Cost(step=10, item=5, join=10, edge=0)
    assert S.op_cost(op, 2, 2, 1, cost, 1) == (145, 270)
    assert S.op_cost(op, 2, 2, 1, cost, 0)[0] == 170
    assert S.op_cost(op, 3, 2, 1, cost, 1)[0] == 175
    assert S.op_cost(op, 4, 2, 1, cost, 1)[0] == 170
    assert S.adaptive_tiling([op], 2, 1, cost) == ([2], [1], [(170, 127, [0], 0, 2, 25), (145, 135, [0], -1, 0, 0)])


def test_six_row_blocks_on_four_lanes_worked_by_hand():
    """Four cores of one compute core, six row blocks of eight steps of 10, nothing else costs.  Uncut the cores hold 1, 2, 1,
    2 blocks: span 160, work 480, average 120: dominant (160 > 132).  In two ranges twelve items of 40 are dealt three a
    lane; lanes 2 and 3 hold the joining items, whose partial results (done at 40, 80, 120 on lanes 0 and 1) are there the
    moment their own steps end: span 120, a gain of 40 of 160.  With 120 against an average of 120 nothing is dominant."""
    op = S.Op(6, 8, 2)
    cost = S.Cost(step=10, item=0, join=0, edge=0)
    assert S.op_cost(op, 1, 4, 1, cost) == (160, 480)
    assert S.op_cost(op, 2, 4, 1, cost) == (120, 480)
    parts, tails, log = S.adaptive_tiling([op], 4, 1, cost)
    assert parts == [2]
    assert log == [(160, 120, [0], 0, 2, 40), (120, 120, [0], -1, 0, 0)]


def test_longest_path_of_a_graph_checked_by_eye():
    """0 -> 1 -> 3, 0 -> 2 -> 3, 4 alone.  Weights 5, 2, 7, 1, 13: the paths cost 5 + 2 + 1 = 8, 5 + 7 + 1 = 13 and 13; of
    two equally long ones the one that ends at the lower index is taken."""
    preds = [(), (0,), (0,), (1, 2), ()]
    assert S.critical_path([5, 2, 7, 1, 13], preds) == (13, [0, 2, 3])
    assert S.critical_path([5, 2, 7, 1, 14], preds) == (14, [4])
    assert S.critical_path([5, 7, 7, 1, 1], preds) == (13, [0, 1, 3])          # equal predecessors: the lower index
    assert S.critical_path([], []) == (0, [])


def test_items_are_dealt_in_contiguous_shares():
    for NI, C, V in itertools.product([1, 2, 5, 7, 12, 64, 65], [1, 2, 3, 8], [1, 2]):
        want = {}
        for c in range(C):
            for j, i in enumerate(range(NI * c // C, NI * (c + 1) // C)):
                want[i] = c * V + j % V
        assert [S.item_lane(i, NI, C, V) for i in range(NI)] == [want[i] for i in range(NI)]


@settings(**COMMON)
@given(nb=st.integers(1, 9), nk=st.integers(1, 9), parts=st.integers(1, 5), C=st.integers(1, 4), V=st.integers(1, 2),
       step=st.integers(1, 4), item=st.integers(0, 3), join=st.integers(0, 3), edge=st.integers(0, 5), group=st.integers(1, 4),
       tail=st.integers(0, 8))
def test_cost_of_a_decomposition_equals_a_tick_by_tick_simulation(nb, nk, parts, C, V, step, item, join, edge, group, tail):
    parts = min(parts, nk)
    tail = tail if tail < nb else 0
    op, cost = S.Op(nb, nk, parts, (), group, tail), S.Cost(step, item, join, edge)
    span, work = S.op_cost(op, parts, C, V, cost, tail)
    assert span == tick_simulation(op, parts, C, V, cost, tail)
    # work: every step once, every item its store, the partial results of a cut row block joined `group` at a time
    cut = 0 if parts == 1 else (tail or nb)
    assert work == nb * nk * step + (nb - cut + cut * parts) * item + cut * -(-(parts - 1) // group) * join


def test_closed_forms_of_the_uncut_operator():
    """One compute core per core and C cores: the fullest core holds ceil(NB / C) blocks."""
    cost = S.Cost(step=7, item=3, join=100, edge=100)
    for NB, nk, C in [(1, 1, 1), (5, 3, 2), (64, 9, 8), (65, 9, 8), (7, 2, 16)]:
        span, work = S.op_cost(S.Op(NB, nk), 1, C, 1, cost)
        assert span == -(-NB // C) * (nk * 7 + 3) and work == NB * (nk * 7 + 3)


@settings(**COMMON)
@given(data=st.data(), n_ops=st.integers(1, 5), C=st.integers(1, 6), V=st.integers(1, 2), thr=st.integers(0, 40), mg=st.integers(0, 20))
def test_what_the_loop_promises(data, n_ops, C, V, thr, mg):
    ops = []
    for o in range(n_ops):
        nk = data.draw(st.integers(1, 12))
        preds = tuple(p for p in range(o) if data.draw(st.booleans()))
        nb = data.draw(st.integers(1, 14))
        ops.append(S.Op(nb, nk, data.draw(st.integers(1, min(nk, 6))), preds, data.draw(st.integers(1, 3)), nb % (C * V) if nb > C * V else 0))
    cost = S.Cost(data.draw(st.integers(1, 9)), data.draw(st.integers(0, 9)), data.draw(st.integers(0, 9)), data.draw(st.integers(0, 20)))
    parts, tails, log = S.adaptive_tiling(ops, C, V, cost, thr, mg)
    assert all(1 <= p <= op.max_parts and t in (0, op.surplus) and (p > 1 or t == 0) for p, t, op in zip(parts, tails, ops))
    assert len(log) <= 1 + sum(op.max_parts - 1 for op in ops)
    # every look but the last refined one operator on the path it saw, and the path it saw next was never longer
    state = [(1, 0)] * n_ops

    def finer(q):
        return [(s2, t2) for s2 in range(state[q][0] + 1, ops[q].max_parts + 1) for t2 in {0, ops[q].surplus}]

    for (pc, avg, path, o, s_new, gain), nxt in zip(log, log[1:] + [None]):
        spans = [tick_simulation(op, d[0], C, V, cost, d[1]) for op, d in zip(ops, state)]
        assert (pc, path) == S.critical_path(spans, [op.preds for op in ops])
        if nxt is None:
            assert o == -1
            if pc * 100 > avg * (100 + thr):      # it stopped although a path is dominant: nothing finer gains more than the margin
                for q in path:
                    for s2, t2 in finer(q):
                        g = spans[q] - tick_simulation(ops[q], s2, C, V, cost, t2)
                        assert g <= 0 or g * 100 < pc * mg
        else:
            assert pc * 100 > avg * (100 + thr) and o in path and s_new > state[o][0] and gain > 0 and gain * 100 >= pc * mg
            took = [d for d in finer(o) if d[0] == s_new and spans[o] - tick_simulation(ops[o], d[0], C, V, cost, d[1]) == gain]
            assert took                                                   # the gain it names is the gain of a decomposition it offers
            for q in path:                                                # and nothing finer on the path gains more
                for s2, t2 in finer(q):
                    assert spans[q] - tick_simulation(ops[q], s2, C, V, cost, t2) <= gain
            state[o] = (s_new, ops[o].surplus if (s_new, ops[o].surplus) in took else 0)
            assert nxt[0] <= pc
    assert [d[0] for d in state] == parts and [d[1] for d in state] == tails
    touched = {e[3] for e in log if e[3] >= 0}
    on_paths = set().union(*[set(e[2]) for e in log])
    assert touched <= on_paths


def test_an_even_deal_is_left_alone_and_an_uneven_one_is_cut():
    cost = S.Cost(step=100, item=40, join=120, edge=300)
    # 1024 row blocks on 256 x 2 lanes: two a lane, nothing dominant, no look beyond the first
    parts, tails, log = S.adaptive_tiling([S.Op(1024, 512, 16)], 256, 2, cost)
    assert parts == [1] and len(log) == 1
    # 768 row blocks: lanes hold 1 or 2 blocks of 32 steps, half of them idle half of the time
    parts, tails, log = S.adaptive_tiling([S.Op(768, 32, 8)], 256, 2, cost)
    assert parts[0] >= 2 and log[-1][0] < log[0][0]
    # offered the 256 surplus blocks alone, it cuts those: a whole block and a half item a lane instead of three half items
    parts, tails, log2 = S.adaptive_tiling([S.Op(768, 32, 8, (), 16, 256)], 256, 2, cost)
    assert tails == [256] and parts[0] >= 2 and log2[-1][0] < log[-1][0]
    # an operator off the critical path keeps its tiling however uneven it is
    parts, _, _ = S.adaptive_tiling([S.Op(768, 32, 8), S.Op(3, 2, 2)], 256, 2, cost)
    assert parts[1] == 1


def test_topological_order_is_required():
    with pytest.raises(AssertionError):
        S.critical_path([1, 1], [(1,), ()])
