"""Pins of the decode-attention oracle (oracle/attn_ref.py) and of the attn / attn_merge uops of the interpreter.

The paper prints neither a formula nor a worked example for its `attn` uop (Section 4.1; Section 6.2, "Dynamic
Attention Length"), so the reference is tied to what the mathematics fixes: closed forms of the softmax-weighted mean
(equal scores, two rows, one dominant row), its invariances (a common shift of the scores, the order of the context
rows), and a library routine (scipy's softmax followed by a matrix product).  The interpreter's tiled, running-maximum
uops must then reproduce the reference for every way of cutting a context into tiles and items.
"""
import numpy as np
import pytest
import scipy.special

from oracle import attn_ref, uop_asm as A, uop_machine as UM


def _case(lengths, d, seed):
    rng = np.random.default_rng(seed)
    row_off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    n = int(row_off[-1])
    Q = rng.standard_normal((len(lengths), d)).astype(np.float32)
    K = rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    return Q, K, V, row_off


def test_equal_scores_give_the_mean_of_the_value_rows():
    Q, K, V, ro = _case([7, 1, 30], 8, 0)
    K[:] = K[0]                                   # every row of a context scores alike
    O, A_, S = attn_ref.attn_decode(Q, K, V, ro, 0.37)
    for s in range(3):
        assert np.allclose(O[s], V[ro[s]:ro[s + 1]].astype(np.float64).mean(axis=0), rtol=1e-13, atol=1e-15)
    Q[:] = 0                                      # and so does a zero query, whatever the keys
    K = np.random.default_rng(1).standard_normal(K.shape).astype(np.float32)
    O, _, _ = attn_ref.attn_decode(Q, K, V, ro, 2.0)
    assert np.allclose(O[2], V[ro[2]:ro[3]].astype(np.float64).mean(axis=0), rtol=1e-13)


def test_two_rows_are_the_logistic_mixture():
    Q, K, V, ro = _case([2], 4, 2)
    scale = 0.5
    O, _, _ = attn_ref.attn_decode(Q, K, V, ro, scale)
    s0, s1 = (scale * float(np.dot(Q[0].astype(np.float64), K[i].astype(np.float64))) for i in (0, 1))
    w0 = 1.0 / (1.0 + np.exp(s1 - s0))
    assert np.allclose(O[0], w0 * V[0].astype(np.float64) + (1.0 - w0) * V[1].astype(np.float64), rtol=1e-13)


def test_a_dominant_row_is_returned_and_huge_scores_do_not_overflow():
    Q, K, V, ro = _case([50], 16, 3)
    K[:] = 0
    K[17] = 1000.0 * Q[0]                          # score about 1000 |q|^2: exp() of it overflows unless the maximum is taken out
    O, _, _ = attn_ref.attn_decode(Q, K, V, ro, 1.0)
    assert np.all(np.isfinite(O)) and np.allclose(O[0], V[17].astype(np.float64), rtol=1e-12)


def test_invariances_shift_of_all_scores_and_order_of_rows():
    Q, K, V, ro = _case([33, 5], 8, 4)
    O, _, _ = attn_ref.attn_decode(Q, K, V, ro, 0.3)
    # adding the same vector u to every key of a request shifts all its scores by scale * q.u
    K64, u = K.astype(np.float64), np.arange(8) / 4.0
    O2, _, _ = attn_ref.attn_decode(Q, K64 + u, V, ro, 0.3)
    assert np.allclose(O, O2, rtol=1e-11, atol=1e-13)
    perm = np.concatenate([np.random.default_rng(5).permutation(33), 33 + np.arange(5)[::-1]])
    O3, _, _ = attn_ref.attn_decode(Q, K[perm], V[perm], ro, 0.3)
    assert np.allclose(O, O3, rtol=1e-12, atol=1e-14)


def test_against_the_library_softmax():
    Q, K, V, ro = _case([1, 100, 64, 257], 32, 6)
    scale = 1.0 / np.sqrt(32)
    O, A_, S = attn_ref.attn_decode(Q, K, V, ro, scale)
    for s in range(4):
        k, v = K[ro[s]:ro[s + 1]].astype(np.float64), V[ro[s]:ro[s + 1]].astype(np.float64)
        p = scipy.special.softmax(scale * (k @ Q[s].astype(np.float64)))
        assert np.allclose(O[s], p @ v, rtol=1e-12, atol=1e-14)
        assert np.allclose(A_[s], p @ np.abs(v), rtol=1e-12)
        assert np.isclose(S[s], (scale * np.abs(k * Q[s].astype(np.float64)).sum(axis=1)).max(), rtol=1e-12)
    with pytest.raises(ValueError):
        attn_ref.attn_decode(Q, K, V, np.array([0, 0, 5, 6, 7]), scale)


# ---- the uops of the interpreter ---------------------------------------------------------------------
def _run(lengths, d, R, chunk, seed, schedule="program", sseed=0, ncores=2, slot=1024, nslots=12):
    Q, K, V, ro = _case(lengths, d, seed)
    p, n_items = A.attn_decode_program(ro, d, R, slot, ncores, chunk_tiles=chunk)
    w, sb, ds = p.finish()
    O = np.full((len(lengths), d), np.nan, np.float32)
    W = np.full((n_items, d + 4), np.nan, np.float32)
    m = UM.Machine(w, sb, ds, [K, V, Q, O, W], n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=64).run(schedule, sseed)
    m.check_final()
    return (Q, K, V, ro), O, W, m


@pytest.mark.parametrize("lengths,d,R,chunk", [
    ([1], 8, 4, 1),
    ([4, 9, 1, 23], 8, 4, 2),          # tails, one item and several items per request
    ([100, 3, 64], 16, 8, 3),
    ([300], 32, 8, 5),                 # one long request cut into eight items
    ([5, 5, 5, 5, 5, 5, 5], 8, 16, 4), # more requests than compute cores, a tile larger than every context
])
def test_attn_program_equals_the_reference_for_any_tiling(lengths, d, R, chunk):
    (Q, K, V, ro), O, W, m = _run(lengths, d, R, chunk, seed=sum(lengths))
    Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, 1.0 / np.sqrt(d))
    # the interpreter computes in fp64 and rounds the partial rows and the result to fp32
    assert np.all(np.abs(O - Or) <= 4e-7 * Ar + 1e-30)
    # the same inputs cut differently give the same result to that rounding
    (_, _, _, _), O2, _, _ = _run(lengths, d, R, chunk + 2, seed=sum(lengths))
    assert np.all(np.abs(O2.astype(np.float64) - O) <= 8e-7 * Ar + 1e-30)


def test_partial_rows_are_the_running_maximum_sum_and_weighted_values():
    (Q, K, V, ro), O, W, m = _run([40], 8, 4, 3, seed=9)      # 10 tiles, items of 3 tiles: rows 0..11, 12..23, 24..35, 36..39
    scale = 1.0 / np.sqrt(8)
    for i, (a, b) in enumerate([(0, 12), (12, 24), (24, 36), (36, 40)]):
        s = scale * (K[a:b].astype(np.float64) @ Q[0].astype(np.float64))
        assert np.isclose(W[i, 8], s.max(), rtol=1e-6)
        assert np.isclose(W[i, 9], np.exp(s - s.max()).sum(), rtol=1e-6)
        assert np.allclose(W[i, :8], np.exp(s - s.max()) @ V[a:b].astype(np.float64), rtol=1e-5, atol=1e-6)
        assert W[i, 10] == 0 and W[i, 11] == 0


def test_every_schedule_gives_the_same_image_and_the_query_tile_goes_back_last():
    ref = None
    for i in range(30):
        _, O, W, m = _run([37, 12, 70], 8, 4, 4, seed=1, schedule="program" if i == 0 else "random", sseed=i)
        got = (O.tobytes(), W.tobytes(), m.trace_vmc, m.trace_vcc)
        ref = ref or got
        assert got == ref
    # one request on one compute core: the query tile is the first allocation of the item and is freed after
    # the key and value tiles that were allocated later (slots come back in another order than they went out)
    _, O, W, m = _run([12], 8, 4, 8, seed=2, ncores=1)
    first_alloc = m.alloc_log[0][0][2]
    frees = [p for (p, n) in m.cores[0].free_log]
    assert frees.index(first_alloc) == 6          # after three key tiles and three value tiles


def _run_whole(lengths, d, R, chunk, seed, schedule="program", sseed=0, ncores=2, slot=1024, nslots=12, Q=None):
    Q0, K, V, ro = _case(lengths, d, seed)
    Q = Q0 if Q is None else Q
    p, n_items = A.attn_decode_program(ro, d, R, slot, ncores, chunk_tiles=chunk, whole=True)
    w, sb, ds = p.finish()
    O = np.full((len(lengths), d), np.nan, np.float32)
    W = np.full((max(n_items, 1), d + 4), np.nan, np.float32)
    m = UM.Machine(w, sb, ds, [K, V, Q, O, W], n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=64).run(schedule, sseed)
    m.check_final()
    return (Q, K, V, ro), O, W, n_items, m


def test_an_attn_uop_that_sees_a_whole_context_writes_the_result_itself():
    # Section 4.1 names one attn uop.  Given a region of d values instead of a partial row it writes o / l, the request's
    # result, and nothing is merged.  Contexts of one item and contexts cut into several, in one batch.
    lengths, d, R, chunk = [9, 4, 40, 1, 16, 23], 8, 4, 4          # tiles: 3, 1, 10, 1, 4, 6 -> whole, whole, cut, whole, whole, cut
    (Q, K, V, ro), O, W, n_items, m = _run_whole(lengths, d, R, chunk, seed=77)
    assert n_items == 3 + 2                                          # partial rows only for the two cut contexts
    Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, 1.0 / np.sqrt(d))
    assert np.all(np.abs(O - Or) <= 4e-7 * Ar + 1e-30)
    # a whole context's result is one rounding of the fp64 result (with the scale as the uop carries it, in fp32):
    # closer than the merged form's bound
    Or32 = attn_ref.attn_decode(Q, K, V, ro, float(np.float32(1.0 / np.sqrt(d))))[0]
    for s in (0, 1, 3, 4):
        assert np.all(np.abs(O[s] - Or32[s]) <= 2.0 ** -24 * (1 + 1e-6) * np.abs(Or32[s]))
    # the merged form of the same batch agrees to the rounding of its partial rows
    (_, _, _, _), O2, _, _ = _run(lengths, d, R, chunk, seed=77)
    assert np.all(np.abs(O2.astype(np.float64) - O) <= 8e-7 * Ar + 1e-30)
    # every schedule gives the same image
    for i in range(10):
        _, O3, W3, _, m3 = _run_whole(lengths, d, R, chunk, seed=77, schedule="random", sseed=i)
        assert O3.tobytes() == O.tobytes() and W3.tobytes() == W.tobytes() and m3.trace_vcc == m.trace_vcc


def test_whole_context_result_in_closed_form():
    # a zero query scores every row alike: the result is the mean of the value rows, whatever the keys are
    lengths, d = [12, 3], 8
    (Q, K, V, ro), O, W, n_items, m = _run_whole(lengths, d, 4, 4, seed=5, Q=np.zeros((2, 8), np.float32))
    assert n_items == 0 and np.all(np.isnan(W))
    for s in range(2):
        mean = V[ro[s]:ro[s + 1]].astype(np.float64).mean(axis=0)
        assert np.all(np.abs(O[s] - mean) <= 2.0 ** -24 * (1 + 1e-6) * np.abs(mean))
    # one row: the result is that value row, bit for bit
    (Q, K, V, ro), O, W, n_items, m = _run_whole([1], d, 4, 4, seed=6)
    assert np.array_equal(O[0], V[0])


def test_attn_rejects_an_output_region_of_another_shape():
    Q, K, V, ro = _case([4], 8, 1)
    p, _ = A.attn_decode_program(ro, 8, 4, 1024, 1, chunk_tiles=4, whole=True)
    # the STORE's region becomes two rows of d values
    bad = p.desc(3, 2, 8 * 4, 8 * 4, 8 * 4)
    vm = p.vmc(0)
    for i, wd in enumerate(vm):
        u = UM.decode(wd)
        if u.opcode == UM.STORE:
            vm[i] = A.word(UM.STORE, UM.F_SEND | UM.F_RECV, vflow=u.vflow, vcc=u.vcc, nslots=u.nslots, size=2, imm=u.imm, desc=bad)
    w, sb, ds = p.finish()
    O = np.zeros((2, 8), np.float32)
    with pytest.raises(UM.ProgramError):
        UM.Machine(w, sb, ds, [K, V, Q, O, np.zeros((1, 12), np.float32)], n_cores=1, slot_bytes=1024, n_slots=12, n_dep_ids=64).run()


def _run_join(lengths, d, R, chunk, seed, schedule="program", sseed=0, ncores=2, slot=1024, nslots=12, Q=None, whole=True):
    Q0, K, V, ro = _case(lengths, d, seed)
    Q = Q0 if Q is None else Q
    p, n_items = A.attn_decode_program(ro, d, R, slot, ncores, chunk_tiles=chunk, whole=whole, join=True)
    w, sb, ds = p.finish()
    O = np.full((len(lengths), d), np.nan, np.float32)
    W = np.full((max(n_items, 1), d + 4), np.nan, np.float32)
    m = UM.Machine(w, sb, ds, [K, V, Q, O, W], n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=64).run(schedule, sseed)
    m.check_final()
    return (Q, K, V, ro), O, W, n_items, (w, m)


@pytest.mark.parametrize("lengths,d,R,chunk", [
    ([40], 8, 4, 3),                   # four items: three partial rows joined by the first
    ([4, 9, 1, 23], 8, 4, 2),
    ([100, 3, 64], 16, 8, 3),
    ([300], 32, 8, 5),                 # eight items
    ([37, 12, 70, 5], 8, 4, 4),
])
def test_an_attn_uop_joins_the_partial_rows_of_the_other_items(lengths, d, R, chunk):
    # a cut context without ATTN_MERGE: its first item takes the other items' partial rows behind its last pair
    (Q, K, V, ro), O, W, n_items, (w, m) = _run_join(lengths, d, R, chunk, seed=sum(lengths))
    ops = np.array([UM.decode(x).opcode for x in w])
    assert (ops == UM.ATTN_MERGE).sum() == 0
    tiles = [-(-L // R) for L in lengths]
    assert n_items == sum(-(-t // chunk) - 1 for t in tiles)            # one partial row per item but the joining one
    Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, 1.0 / np.sqrt(d))
    assert np.all(np.abs(O - Or) <= 4e-7 * Ar + 1e-30)
    # the merged form of the same cut agrees to the rounding of the partial rows
    (_, _, _, _), O2, _, _ = _run(lengths, d, R, chunk, seed=sum(lengths))
    assert np.all(np.abs(O2.astype(np.float64) - O) <= 8e-7 * Ar + 1e-30)
    # every schedule gives the same image and the same traces
    for i in range(8):
        _, O3, W3, _, (_, m3) = _run_join(lengths, d, R, chunk, seed=sum(lengths), schedule="random", sseed=i)
        assert O3.tobytes() == O.tobytes() and W3.tobytes() == W.tobytes() and m3.trace_vcc == m.trace_vcc


def test_joined_result_in_closed_form():
    # a zero query weighs every row alike whatever the cut: the mean of all value rows of the context
    lengths, d = [29, 50], 8
    (Q, K, V, ro), O, W, n_items, _ = _run_join(lengths, d, 4, 3, seed=11, Q=np.zeros((2, 8), np.float32))
    for s in range(2):
        mean = V[ro[s]:ro[s + 1]].astype(np.float64).mean(axis=0)
        assert np.all(np.abs(O[s] - mean) <= 3 * 2.0 ** -24 * np.abs(mean) + 1e-9)
    # the partial rows of the other items: maximum 0, sum = rows of the item
    assert np.all(W[:, 8] == 0)
    assert sorted(W[:, 9].tolist()) == sorted([12.0, 5.0, 12.0, 12.0, 12.0, 2.0])
    # a dominant key row in an item that is not the joining one carries the result: its value row
    Q, K, V, ro = _case([40], 8, 3)
    K[:] = 0
    K[30] = 50.0 * Q[0] / np.dot(Q[0], Q[0])                 # score 50 / sqrt(8) against zeros elsewhere
    p, n_items = A.attn_decode_program(ro, 8, 4, 1024, 2, chunk_tiles=3, join=True)
    w, sb, ds = p.finish()
    O = np.full((1, 8), np.nan, np.float32)
    W = np.full((n_items, 12), np.nan, np.float32)
    UM.Machine(w, sb, ds, [K, V, Q, O, W], n_cores=2, slot_bytes=1024, n_slots=12, n_dep_ids=64).run()
    assert np.allclose(O[0], V[30], rtol=1e-5, atol=1e-6)


def test_attn_join_rejects_wrong_tiles():
    Q, K, V, ro = _case([40], 8, 3)
    for what in ("rows", "out"):
        p, n_items = A.attn_decode_program(ro, 8, 4, 1024, 2, chunk_tiles=3, join=True)
        for core in range(2):
            vm = p.vmc(core)
            for i, wd in enumerate(vm):
                u = UM.decode(wd)
                if what == "rows" and u.opcode == UM.LOAD and (u.flags & UM.F_DEP_RECV):
                    bad = p.desc(4, 2, 12 * 4, 12 * 4, 12 * 4)      # two partial rows where the uop expects three
                    vm[i] = A.word(UM.LOAD, u.flags, vflow=u.vflow, vcc=u.vcc, nslots=u.nslots, size=2, dep_id=u.dep_id, dep_count=3, imm=u.imm, desc=bad)
        if what == "out":
            # the joining uop is handed a partial-row region instead of a result row
            for core in range(2):
                vm = p.vmc(core)
                for i, wd in enumerate(vm):
                    u = UM.decode(wd)
                    if u.opcode == UM.STORE and not (u.flags & UM.F_DEP_SEND):
                        bad = p.desc(4, 1, 12 * 4, 12 * 4, 12 * 4)
                        vm[i] = A.word(UM.STORE, u.flags, vflow=u.vflow, vcc=u.vcc, nslots=u.nslots, size=1, imm=0, desc=bad)
        w, sb, ds = p.finish()
        O = np.zeros((1, 8), np.float32)
        W = np.zeros((max(n_items, 1) + 1, 12), np.float32)
        with pytest.raises(UM.ProgramError):
            UM.Machine(w, sb, ds, [K, V, Q, O, W], n_cores=2, slot_bytes=1024, n_slots=12, n_dep_ids=64).run()
