"""The library's adaptive tiling step (vdc_schedule; Section 4.2, "Adaptive Scheduling and Tiling") against the oracle
side's, look for look, and what the matvec tiler does with it: the cut of K it takes for a dense shape is the oracle's
choice under the library's cost model, and the programs it then writes (several work items per compute core, partial
results and joining items of one row block on different cores or on the same one) are validated, run on the interpreter
under a random schedule and equal the fp64 GEMV.  Host logic only: no GPU."""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

import paper_2605_03190_amd as vdc
from oracle import gemv_ref, uop_machine as UM, uop_schedule as S

COMMON = dict(deadline=None, max_examples=80, derandomize=True, suppress_health_check=[HealthCheck.too_slow])


def library_cost(tile_bytes):
    """The cost model the header documents for the tilers: nanoseconds for tiles of tile_bytes."""
    step = 510 + tile_bytes // 20
    return S.Cost(step=step, item=1500, join=step + 1200, edge=16000)


@settings(**COMMON)
@given(data=st.data(), n_ops=st.integers(0, 6), C=st.integers(1, 7), V=st.integers(1, 2), thr=st.integers(1, 40), mg=st.integers(1, 20))
def test_the_library_takes_the_looks_the_oracle_takes(data, n_ops, C, V, thr, mg):
    ops, preds = [], []
    for o in range(n_ops):
        nk = data.draw(st.integers(1, 40))
        nb = data.draw(st.integers(1, 40))
        ops.append((nb, nk, data.draw(st.integers(1, min(nk, 8))), data.draw(st.integers(1, 5)), nb % (C * V) if nb > C * V else 0))
        preds.append(tuple(p for p in range(o) if data.draw(st.booleans())))
    cost = tuple(data.draw(st.integers(lo, 50)) for lo in (1, 0, 0, 0))
    want_parts, want_tails, want_log = S.adaptive_tiling([S.Op(nb, nk, mp, pr, g, su) for (nb, nk, mp, g, su), pr in zip(ops, preds)], C, V,
                                                         S.Cost(*cost), thr, mg)
    with vdc.Executor(device=-1, n_cores=C, vcc_per_core=V, sched_threshold_pct=thr, sched_min_gain_pct=mg) as ex:
        parts, tails, log = ex.schedule(ops, preds, cost)
        assert parts == want_parts and tails == want_tails
        assert log == [(pc, avg, o, s, g) for pc, avg, _, o, s, g in want_log]
        if all(not p for p in preds):
            assert ex.schedule(ops, None, cost) == (parts, tails, log)


def test_malformed_graphs_are_refused():
    with vdc.Executor(device=-1, n_cores=4) as ex:
        for ops, preds, cost in [([(0, 4, 1)], None, (1, 0, 0, 0)), ([(4, 0, 1)], None, (1, 0, 0, 0)), ([(4, 4, 5)], None, (1, 0, 0, 0)),
                                 ([(4, 4, 0)], None, (1, 0, 0, 0)), ([(4, 4, 2)], None, (0, 0, 0, 0)), ([(4, 4, 2)], None, (1, -1, 0, 0)),
                                 ([(4, 4, 2), (4, 4, 2)], [(1,), ()], (1, 0, 0, 0)), ([(4, 4, 2)], [(0,)], (1, 0, 0, 0)),
                                 ([(1 << 23, 8, 4)], None, (1, 0, 0, 0)), ([(4, 4, 2, -1)], None, (1, 0, 0, 0)),
                                 ([(4, 4, 2, 1, 4)], None, (1, 0, 0, 0)), ([(4, 4, 2, 1, -1)], None, (1, 0, 0, 0))]:
            with pytest.raises(vdc.VdcError) as e:
                ex.schedule(ops, preds, cost)
            assert e.value.code == vdc.VDC_EINVAL
        with pytest.raises(vdc.VdcError):
            ex.schedule([(4, 4, 2)], None, None, tile_bytes=100)
    for bad in (dict(sched_threshold_pct=-1), dict(sched_min_gain_pct=101), dict(sched_force_parts=17), dict(sched_force_parts=100), dict(sched_force_parts=117)):
        with pytest.raises(vdc.VdcError):
            vdc.Executor(device=-1, **bad)


@settings(**COMMON)
@given(rows=st.integers(1, 4000), nk=st.integers(1, 64), B=st.sampled_from([1, 2, 8]), tile=st.sampled_from([4096, 8192, 16384]),
       C=st.sampled_from([3, 16, 256]))
def test_the_matvec_tiler_takes_the_cut_the_oracle_would(rows, nk, B, tile, C):
    with vdc.Executor(device=-1, n_cores=C) as ex:
        R, Kt, NB, nk_, s_max, s, tail = ex.matvec_tiling(rows, 256 * nk, B, tile)
        assert NB == -(-rows // R) and nk_ == -(-256 * nk // Kt) and 1 <= s <= s_max
        # what the builder offers: the surplus row blocks alone where there are any; at least four steps a range, a depId per
        # cut row block, a short stream of cut items per core
        lanes = 2 * C
        surplus = NB % lanes if NB > lanes and R % 4 == 0 and R <= Kt and min(16, nk_ // 4, 8 * lanes // (NB % lanes or NB)) >= 2 else 0
        cut = surplus or NB
        assert s_max == 1 or (s_max <= min(16, nk_ // 4) and cut <= 4096 and s_max * cut <= max(cut, 8 * lanes) and R % 4 == 0 and R <= Kt)
        want, want_tail, _ = S.adaptive_tiling([S.Op(NB, nk_, s_max, (), Kt // R, surplus)], C, 2, library_cost(tile))
        assert ([s], [tail]) == (want, want_tail) and tail in (0, surplus)


def test_shapes_of_the_benchmark_configurations_and_awkward_ones():
    with vdc.Executor(device=-1, n_cores=256) as ex:
        assert ex.matvec_tiling(32768, 65536, 8, 16384)[2:] == (1024, 512, 4, 1, 0)     # two row blocks a compute core: left alone
        assert ex.matvec_tiling(8192, 8192, 1, 8192)[2:] == (1024, 32, 4, 1, 0)
        R, Kt, NB, nk, s_max, s, tail = ex.matvec_tiling(9216, 16384, 1, 16384)        # 64 blocks over: those alone are cut
        assert (NB, nk, tail) == (576, 64, 64) and s >= 4
        assert ex.matvec_tiling(12288, 8192, 1, 16384)[2:] == (768, 32, 8, 1, 0)       # 256 over, short rows: no cut is worth its dependency
        R, Kt, NB, nk, s_max, s, tail = ex.matvec_tiling(1024, 16384, 1, 16384)        # an eighth of the compute cores busy: cut
        assert NB == 64 and s >= 4 and tail == 0


def _run(ex, rows, K, B, tile, ncores, slot, nslots, seed):
    w, sb, d = ex.matvec_program(rows, K, K, B, tile)
    ws = ex.matvec_workspace(rows, K, K, B, tile)
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    sizes = [M.nbytes, X.nbytes, B * rows * 4] + ([ws.nbytes] if ws.size else [])
    rc, msg = ex.program_validate(w, sb, d, sizes)
    assert rc == vdc.VDC_OK, msg
    Y = np.full((B, rows), np.nan, np.float32)
    m = UM.Machine(w, sb, d, [M, X, Y] + ([ws] if ws.size else []), n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=4096)
    m.run("random", seed)
    m.check_final()
    Yr, Ya = gemv_ref.gemv_dense(M, X)
    assert np.all(np.abs(Y - Yr) <= 2e-6 * Ya + 1e-30)
    signals = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.STORE) - (-(-rows // ex.matvec_tiling(rows, K, B, tile)[0]))
    return signals


CUT_SEEN = []


@settings(**COMMON)
@given(blocks_x2=st.integers(1, 15), extra=st.integers(0, 3), nk=st.integers(8, 200), B=st.sampled_from([1, 2, 3]), ncores=st.integers(1, 4),
       seed=st.integers(0, 1000))
def test_programs_of_cut_shapes_equal_the_gemv(blocks_x2, extra, nk, B, ncores, seed):
    """Row-block counts around half-integer multiples of the number of compute cores (where the adaptive step cuts K), with a
    ragged last block; tiles of 2 KB = 4 rows x 128 columns."""
    slot, nslots, tile = 2048, 16, 2048
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots) as ex:
        R, Kt = ex.matvec_tiling(4, 128 * nk, B, tile)[:2]
        rows = max(1, blocks_x2 * ncores * R - extra)                # NB = blocks_x2 / 2 per compute core, give or take
        s, tail = ex.matvec_tiling(rows, Kt * nk, B, tile)[5:]
        signals = _run(ex, rows, Kt * nk, B, tile, ncores, slot, nslots, seed)
        assert signals == (s - 1) * (tail or -(-rows // R))          # every partial result is one more store
        CUT_SEEN.append((s, tail))


def test_the_adaptive_step_did_cut_some_of_those_shapes():
    assert CUT_SEEN and max(s for s, _ in CUT_SEEN) >= 2 and min(s for s, _ in CUT_SEEN) == 1
    assert any(t > 0 for _, t in CUT_SEEN) and any(s > 1 and t == 0 for s, t in CUT_SEEN)       # the surplus alone, and all blocks


@pytest.mark.parametrize("ncores,force,rows,nk,B,tile,slot,nslots", [
    (1, 2, 24, 8, 2, 2048, 2048, 16), (1, 4, 8, 16, 2, 2048, 2048, 16), (2, 3, 28, 12, 2, 2048, 2048, 16), (3, 16, 36, 64, 2, 2048, 2048, 16),
    (2, 2, 4, 9, 2, 2048, 2048, 16),
    (2, 16, 70, 64, 8, 16384, 8192, 19),      # tiles of 32 rows x 128 columns: four partial results per joining step, fifteen to join
    (3, 7, 100, 30, 8, 16384, 8192, 19),      # ... six: a full step and a short one
    # the surplus row blocks alone: whole blocks first (looped or unrolled form), then the items of the cut blocks
    (2, 102, 27, 16, 2, 2048, 2048, 16),      # 7 row blocks on 4 compute cores: 4 whole, 3 cut in two
    (1, 104, 90, 16, 1, 2048, 2048, 16),      # 23 on 2: 22 whole (the looped form), 1 cut in four
    (3, 103, 50, 12, 3, 2048, 2048, 16),      # 13 on 6, a ragged last block among the cut ones
    (2, 116, 200, 64, 8, 16384, 8192, 19),    # 7 on 4 with tiles of 32 rows: 3 cut in sixteen, four joining steps
])
def test_forced_cuts_with_partial_and_joining_items_on_one_core(ncores, force, rows, nk, B, tile, slot, nslots):
    """sched_force_parts takes the scheduler out: every K cut the builder offers can be run, also where it would not pay."""
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots, sched_force_parts=force) as ex:
        R, Kt, NB, nk_, s_max, s, tail = ex.matvec_tiling(rows, 128 * nk, B, tile)
        assert s == min(force % 100, s_max) and s >= 2 and (tail > 0) == (force > 100)
        signals = _run(ex, rows, 128 * nk, B, tile, ncores, slot, nslots, rows)
        assert signals == (s - 1) * (tail or NB)


@pytest.mark.parametrize("rows,nk,tile,ncores", [(200, 8, 16384, 2), (100, 6, 8192, 3), (64, 4, 16384, 1)])
def test_eight_vectors_take_a_vector_tile_over_two_steps_on_request(rows, nk, tile, ncores):
    """Eight vectors, tiles of 32 (16) rows x 128 columns, few row blocks per compute core, an even number of steps: with
    issue_flags bit 1 the tiler gives a MATVEC vector tiles that hold the pieces of two steps (8 rows of two pieces, one
    slot): validated, run under a random schedule, the GEMV; half as many vector loads as matrix loads.  Without the bit it
    keeps the step-by-step form, with the same bits in the result."""
    K = 128 * nk
    out = []
    for fl in (2, 0):
        with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=8192, n_slots=19, issue_flags=fl, sched_force_parts=1) as ex:
            w, sb, d = ex.matvec_program(rows, K, K, 8, tile)
            rng = np.random.default_rng(rows)
            M = rng.standard_normal((rows, K)).astype(np.float32)
            X = rng.standard_normal((8, K)).astype(np.float32)
            rc, msg = ex.program_validate(w, sb, d, [M.nbytes, X.nbytes, 8 * rows * 4])
            assert rc == vdc.VDC_OK, msg
        Y = np.full((8, rows), np.nan, np.float32)
        m = UM.Machine(w, sb, d, [M, X, Y], n_cores=ncores, slot_bytes=8192, n_slots=19)
        m.run("random", 5)
        m.check_final()
        Yr, Ya = gemv_ref.gemv_dense(M, X)
        assert np.all(np.abs(Y - Yr) <= 1e-6 * Ya + 1e-30)
        loads_x = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 1)
        loads_m = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
        xspans = {(int(x[3]) >> 8) & 0x7F for x in w[(w[:, 0] & 0xFF) == 16]}
        assert (xspans == {2} and 2 * loads_x == loads_m) if fl == 2 else (xspans == {0} and loads_x == loads_m)
        out.append(Y)
    assert np.array_equal(out[0], out[1])
