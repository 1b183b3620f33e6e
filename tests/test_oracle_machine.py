"""Pins of the sequential interpreter of the decoupled abstract machine (oracle/uop_machine.py).

The paper prints no worked example of the machine, so the interpreter is tied to what the
paper and the mathematics fix: the result of a matvec program is the textbook product
(Section 3); the machine is a FIFO dataflow network without cyclic dependencies
(Section 4.3, "Dependency Resolving", "Avoiding Deadlock"), hence every legal schedule gives the
same memory image and the same per-unit traces; the allocator returns the first contiguous free
position (Section 4.3, "Virtual Memory Core"); in-order allocation that over-commits the slots
deadlocks (Section 4.3, "Avoiding Deadlock"); dynamic addresses are the literal address plus an
accumulator advanced by control uops (Section 5, "Dynamic address generation").
"""
import numpy as np
import pytest

from oracle import gemv_ref, uop_asm as A, uop_machine as UM


def _run(p, tensors, schedule="program", seed=0, **kw):
    w, sb, d = p.finish()
    m = UM.Machine(w, sb, d, tensors, n_cores=p.n_cores, vcc_per_core=p.V, **kw)
    return m.run(schedule, seed)


def _inputs(rows, K, B, seed, ld=None):
    rng = np.random.default_rng(seed)
    ld = K if ld is None else ld
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    return M, X, np.full((B, rows), np.nan, np.float32)


def _check_result(M, X, Y, ld=None):
    Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
    # the interpreter accumulates in fp64 and rounds once to fp32 at the copy-out
    assert np.all(np.abs(Y.astype(np.float64) - Yr) <= 6e-8 * np.abs(Yr) + 1e-12 * Ya + 1e-45)


# ---- allocator -----------------------------------------------------------------------------------
def test_first_fit_against_string_search_all_16bit_masks():
    for n in (1, 2, 3, 4):
        for mask in range(1 << 16):
            s = format(mask, "016b")[::-1]                 # s[i] = bit i
            assert UM.first_fit(mask, n, 16) == s.find("0" * n)


def test_first_fit_sampled_32bit_masks_and_limits():
    rng = np.random.default_rng(0)
    masks = rng.integers(0, 1 << 32, 200000, dtype=np.uint64)
    # mix in dense masks, where long runs are rare
    masks[::2] |= rng.integers(0, 1 << 32, 100000, dtype=np.uint64)
    for mask in masks[:60000]:
        mask = int(mask)
        for n in (1, 2, 4):
            for n_slots in (32, 19):
                s = format(mask, "032b")[::-1][:n_slots]
                assert UM.first_fit(mask, n, n_slots) == s.find("0" * n)
    assert UM.first_fit(0, 32, 32) == 0 and UM.first_fit(1, 32, 32) == -1
    assert UM.first_fit(0b0110, 1, 4) == 0 and UM.first_fit(0b0111, 1, 4) == 3
    assert UM.first_fit(0b0111, 2, 4) == -1          # no wrap-around


# ---- word layout ----------------------------------------------------------------------------------
def test_decode_inverts_the_assembler_field_by_field():
    rng = np.random.default_rng(3)
    for _ in range(2000):
        f = dict(opcode=int(rng.integers(256)), flags=int(rng.integers(256)), vflow=int(rng.integers(16)),
                 vcc=int(rng.integers(4)), acc=int(rng.integers(8)), nslots=int(rng.integers(64)),
                 size=int(rng.integers(65536)), dep_id=int(rng.integers(65536)),
                 imm=int(rng.integers(-(1 << 47), 1 << 47)), desc=int(rng.integers(256)),
                 dep_count=int(rng.integers(256)))
        u = UM.decode(A.word(**f))
        assert {k: getattr(u, k) for k in f} == f
    # extreme immediates
    for imm in (-(1 << 47), (1 << 47) - 1, -1, 0, 1, 1 << 33, -(1 << 33) - 5):
        assert UM.decode(A.word(A.ADD, imm=imm)).imm == imm


def _golden_words():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "uop_words.txt")
    names = ("opcode", "flags", "vflow", "vcc", "acc", "nslots", "size", "dep_id", "imm", "desc", "dep_count")
    out = []
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        left, right = line.split("|")
        name, *hexw = left.split()
        out.append((name, tuple(int(h, 16) for h in hexw), dict(zip(names, (int(x) for x in right.split())))))
    return out


def test_hand_written_instruction_words():
    """The bit layout is fixed by words written out by hand (tests/golden/uop_words.txt), not by the assembler and the
    decoder agreeing with each other: the assembler must produce exactly these words and the decoder exactly these
    fields.  A field moved by a bit, a swapped pair of words or a wrong sign extension fails here."""
    cases = _golden_words()
    assert {c[2]["opcode"] for c in cases} >= {A.HALT, A.LOOP, A.REPEAT, A.SET, A.LOAD, A.STORE, A.MATVEC}
    assert any(c[2]["imm"] < 0 for c in cases) and any(c[2]["dep_count"] for c in cases)
    for name, words, f in cases:
        assert len(words) == 4
        assert tuple(A.word(**f)) == words, name
        u = UM.decode(words)
        assert {k: getattr(u, k) for k in f} == f, name


# ---- result = textbook product -------------------------------------------------------------------
@pytest.mark.parametrize("rows,K,B,R,Kt,slot,ncores", [
    (16, 64, 1, 8, 64, 4096, 1),
    (50, 200, 3, 8, 64, 4096, 3),        # ragged tail in rows and in K
    (33, 100, 8, 4, 32, 1024, 2),
    (7, 8, 2, 16, 128, 8192, 2),         # a single partial tile
    (128, 128, 1, 8, 128, 4096, 4),
])
def test_dense_program_equals_gemv(rows, K, B, R, Kt, slot, ncores):
    M, X, Y = _inputs(rows, K, B, seed=rows + K)
    p = A.dense_matvec_program(rows, K, K, B, R, Kt, slot, ncores)
    _run(p, [M, X, Y], slot_bytes=slot, n_slots=12)
    _check_result(M, X, Y)


@pytest.mark.parametrize("rows,K,R,Kt,slot,ncores,xspan,B", [
    (40, 512, 8, 64, 2048, 2, 2, 3),     # three vectors: a vector tile is three rows of two pieces side by side
    (33, 448, 8, 64, 4096, 3, 4, 4),     # seven steps: the second vector tile holds three pieces a row
    (64, 1024, 32, 128, 8192, 1, 2, 8),  # the shape of the headline workload's tiles: 8 vectors, 32 rows x 128 columns
])
def test_a_vector_tile_over_several_steps_with_several_vectors(rows, K, R, Kt, slot, ncores, xspan, B):
    """The same with B > 1: the vector tile holds B rows of xspan pieces as they lie in memory.  The textbook product, the
    bits of the step-by-step program, every schedule the same image, single entries of the matrix against vectors whose
    every entry is different (a slip in row or piece would pick another value), the load counts."""
    M, X, Y = _inputs(rows, K, B, seed=rows + K + xspan)
    p = A.dense_matvec_program(rows, K, K, B, R, Kt, slot, ncores, xspan=xspan)
    m = _run(p, [M, X, Y], slot_bytes=slot, n_slots=12)
    _check_result(M, X, Y)
    Y1 = np.full_like(Y, np.nan)
    _run(A.dense_matvec_program(rows, K, K, B, R, Kt, slot, ncores), [M, X, Y1], slot_bytes=slot, n_slots=12)
    assert np.array_equal(Y, Y1)
    for seed in range(5):
        Y2 = np.full_like(Y, np.nan)
        w, sb, d = p.finish()
        UM.Machine(w, sb, d, [M, X, Y2], n_cores=ncores, slot_bytes=slot, n_slots=12).run("random", seed).check_final()
        assert np.array_equal(Y, Y2)
    X0 = (np.arange(1, K + 1, dtype=np.float32)[None, :] + 4096.0 * np.arange(B, dtype=np.float32)[:, None])
    for (i, j) in [(0, 0), (rows - 1, K - 1), (rows // 2, Kt + 1), (3, K - Kt)]:
        M0 = np.zeros((rows, K), np.float32)
        M0[i, j] = 2.0
        Y0 = np.full((B, rows), np.nan, np.float32)
        _run(p, [M0, X0, Y0], slot_bytes=slot, n_slots=12)
        exp = np.zeros((B, rows), np.float32)
        exp[:, i] = 2.0 * X0[:, j]
        assert np.array_equal(Y0, exp)
    loads_x = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 1)
    loads_m = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
    nk, nrb = K // Kt, -(-rows // R)
    assert loads_m == nk * nrb and loads_x == -(-nk // xspan) * nrb
    # a vector tile with a row too few, or with rows too short for the steps it is popped for, is refused
    w, sb, d = p.finish()
    ix = [k for k in range(len(w)) if (w[k, 0] & 0xFF) == A.LOAD and d[UM.decode(w[k]).desc][0] == 1]
    w2 = np.array(w, copy=True)
    w2[ix[0], 1] = (w2[ix[0], 1] & 0xFFFF0000) | (B - 1)
    with pytest.raises(UM.ProgramError):
        UM.Machine(w2, sb, d, [M, X, Y], n_cores=ncores, slot_bytes=slot, n_slots=12).run()
    d2 = np.array(d, copy=True)
    d2[UM.decode(w[ix[0]]).desc][2] = Kt * 4             # one piece a row where the uop needs xspan
    with pytest.raises(UM.ProgramError):
        UM.Machine(w, sb, d2, [M, X, Y], n_cores=ncores, slot_bytes=slot, n_slots=12).run()


@pytest.mark.parametrize("rows,K,R,Kt,slot,ncores,xspan", [
    (40, 512, 8, 64, 2048, 2, 8),        # eight steps: one vector tile for the whole row block
    (40, 512, 8, 64, 2048, 2, 4),        # two vector tiles of four steps
    (33, 448, 8, 64, 1024, 3, 4),        # seven steps: the second vector tile holds three
    (16, 256, 4, 128, 4096, 1, 2),
])
def test_a_vector_tile_over_several_steps_equals_gemv(rows, K, R, Kt, slot, ncores, xspan):
    """MATVEC with one vector tile per xspan steps (B = 1): the textbook product, and also the bits of the program that
    loads the vector step by step (the same products in the same order); every schedule gives the same image; a single
    non-zero entry lands where it belongs (a slip in the row of the vector tile would move or lose it)."""
    M, X, Y = _inputs(rows, K, 1, seed=rows + K + xspan)
    p = A.dense_matvec_program(rows, K, K, 1, R, Kt, slot, ncores, xspan=xspan)
    m = _run(p, [M, X, Y], slot_bytes=slot, n_slots=12)
    _check_result(M, X, Y)
    Y1 = np.full_like(Y, np.nan)
    _run(A.dense_matvec_program(rows, K, K, 1, R, Kt, slot, ncores), [M, X, Y1], slot_bytes=slot, n_slots=12)
    assert np.array_equal(Y, Y1)
    for seed in range(10):
        Y2 = np.full_like(Y, np.nan)
        w, sb, d = p.finish()
        UM.Machine(w, sb, d, [M, X, Y2], n_cores=ncores, slot_bytes=slot, n_slots=12).run("random", seed).check_final()
        assert np.array_equal(Y, Y2)
    for (i, j) in [(0, 0), (rows - 1, K - 1), (rows // 2, Kt + 1), (3, K - Kt)]:
        M0 = np.zeros((rows, K), np.float32)
        M0[i, j] = 2.0
        X0 = np.arange(1, K + 1, dtype=np.float32)[None, :]
        Y0 = np.full((1, rows), np.nan, np.float32)
        _run(p, [M0, X0, Y0], slot_bytes=slot, n_slots=12)
        exp = np.zeros(rows, np.float32)
        exp[i] = 2.0 * (j + 1)
        assert np.array_equal(Y0[0], exp)
    # fewer vector loads than steps, and the vector tile goes back after the matrix tiles of its steps
    loads_x = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 1)
    loads_m = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
    nk, nrb = K // Kt, -(-rows // R)
    assert loads_m == nk * nrb and loads_x == -(-nk // xspan) * nrb


def test_a_vector_tile_over_several_steps_must_hold_the_pieces_of_its_steps():
    M, X, Y = _inputs(16, 256, 2, seed=1)
    p = A.dense_matvec_program(16, 256, 256, 2, 8, 64, 2048, 1)
    w, sb, d = p.finish()
    w = np.array(w, copy=True)
    i = int(np.flatnonzero((w[:, 0] & 0xFF) == A.MATVEC)[0])
    w[i, 3] |= 2 << 8                                    # xspan = 2 in imm[47:40] on a B = 2 uop whose vector tiles hold one piece a row
    with pytest.raises(UM.ProgramError):
        UM.Machine(w, sb, d, [M, X, Y], n_cores=1, slot_bytes=2048, n_slots=12).run()
    # a vector tile that holds fewer rows than the steps it is popped for
    M, X, Y = _inputs(16, 512, 1, seed=2)
    p = A.dense_matvec_program(16, 512, 512, 1, 8, 64, 2048, 1, xspan=4)
    w, sb, d = p.finish()
    w = np.array(w, copy=True)
    ix = [k for k in range(len(w)) if (w[k, 0] & 0xFF) == A.LOAD and UM.decode(w[k]).size == 4 and d[UM.decode(w[k]).desc][0] == 1]
    w[ix[0], 1] = (w[ix[0], 1] & 0xFFFF0000) | 3         # only three valid rows
    with pytest.raises(UM.ProgramError):
        UM.Machine(w, sb, d, [M, X, Y], n_cores=1, slot_bytes=2048, n_slots=12).run()


@pytest.mark.parametrize("row_off,K,B,R,Kt,slot,ncores,span", [
    ([0, 200], 64, 1, 8, 64, 2048, 2, 8),            # dense, one vector: 25 blocks in groups of 8, the last of one block
    ([0, 77], 32, 3, 4, 32, 1024, 3, 4),             # dense, three vectors, a row tail inside the last group
    ([0, 40, 47, 170, 186], 128, 1, 16, 128, 8192, 2, 8),   # ragged: segments of 40, 7, 123 and 16 rows, each its own vector
    ([0, 9, 300], 100, 1, 8, 32 * 4, 4096, 1, 2),    # K tail inside the only tile (K < Kt)
])
def test_matvec_over_several_row_blocks_equals_gemv(row_off, K, B, R, Kt, slot, ncores, span):
    """MATVEC over `span` row blocks that share one vector tile (K fits a tile): the textbook product per segment, the bits
    of the one-block-per-uop program (the same products in the same order), the same image under every schedule, a single
    non-zero entry lands in its own row (a slip in the block's row offset inside the output region would move it), one
    vector load and one store per group instead of per block, and no slot is left behind."""
    rows, n_seg = row_off[-1], len(row_off) - 1
    ragged = n_seg > 1
    rng = np.random.default_rng(rows + K + span)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((n_seg if ragged else B, K)).astype(np.float32)
    Y = np.full((rows,) if ragged else (B, rows), np.nan, np.float32)
    p = A.rowspan_matvec_program(row_off, K, K, B, R, Kt, slot, ncores, span)
    m = _run(p, [M, X, Y], slot_bytes=slot, n_slots=14)
    m.check_final()
    if ragged:
        Yr, Ya = gemv_ref.gemv_ragged(M, np.array(row_off, dtype=np.int64), X)
    else:
        Yr, Ya = gemv_ref.gemv_dense(M, X)
    assert np.all(np.abs(Y.astype(np.float64) - Yr) <= 6e-8 * np.abs(Yr) + 1e-12 * Ya + 1e-45)
    # one block per uop (span is only the program builder's grouping; a group of one block is the listing's uop)
    Y1 = np.full_like(Y, np.nan)
    p1 = A.Program(ncores)
    g = 0
    for s in range(n_seg):
        for r in range(row_off[s], row_off[s + 1], R):
            core, v = (g % (ncores * 2)) // 2, g % 2
            rv = min(R, row_off[s + 1] - r)
            p1.vmc(core).append(A.word(A.LOAD, A.F_SEND, vflow=2 * v, vcc=v, nslots=-(-R * Kt * 4 // slot), size=rv, imm=r * K * 4,
                                       desc=p1.desc(0, R, K * 4, Kt * 4, K * 4)))
            p1.vmc(core).append(A.word(A.LOAD, A.F_SEND, vflow=2 * v + 1, vcc=v, nslots=-(-B * Kt * 4 // slot), size=B,
                                       imm=(s * K * 4 if ragged else 0), desc=p1.desc(1, B, K * 4, Kt * 4, K * 4)))
            p1.vmc(core).append(A.word(A.STORE, A.F_SEND | A.F_RECV, vflow=4 + v, vcc=v, nslots=-(-B * R * 4 // slot), size=B, imm=r * 4,
                                       desc=p1.desc(2, B, rv * 4, R * 4, (0 if ragged else rows) * 4)))
            p1.vcc(core, v).append(A.word(A.MATVEC, size=1, imm=A.matvec_imm(B, R, Kt // 4)))
            g += 1
    _run(p1, [M, X, Y1], slot_bytes=slot, n_slots=14)
    assert np.array_equal(Y, Y1)
    for seed in range(10):
        Y2 = np.full_like(Y, np.nan)
        w, sb, d = p.finish()
        UM.Machine(w, sb, d, [M, X, Y2], n_cores=ncores, slot_bytes=slot, n_slots=14).run("random", seed).check_final()
        assert np.array_equal(Y, Y2)
    for (i, j) in [(0, 0), (rows - 1, K - 1), (rows // 2, 1), (min(rows - 1, R + 1), K // 2)]:
        M0 = np.zeros((rows, K), np.float32)
        M0[i, j] = 2.0
        X0 = np.tile(np.arange(1, K + 1, dtype=np.float32)[None, :], (X.shape[0], 1))
        Y0 = np.full_like(Y, np.nan)
        _run(p, [M0, X0, Y0], slot_bytes=slot, n_slots=14)
        exp = np.zeros_like(Y0)
        exp[..., i] = 2.0 * (j + 1)
        assert np.array_equal(Y0, exp)
    # per group: one vector load and one store
    groups = sum(-(-(row_off[s + 1] - row_off[s]) // (span * R)) for s in range(n_seg))
    blocks = sum(-(-(row_off[s + 1] - row_off[s]) // R) for s in range(n_seg))
    loads_x = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 1)
    loads_m = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
    stores = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.STORE)
    assert loads_m == blocks and loads_x == groups and stores == groups


def test_matvec_over_several_row_blocks_needs_one_step_and_a_fitting_region():
    M = np.ones((32, 64), np.float32)
    X = np.ones((1, 64), np.float32)
    Y = np.zeros((1, 32), np.float32)
    p = A.rowspan_matvec_program([0, 32], 64, 64, 1, 8, 64, 2048, 1, 4)
    w, sb, d = p.finish()
    bad = np.array(w, copy=True)
    i = int(np.flatnonzero((bad[:, 0] & 0xFF) == A.MATVEC)[0])
    bad[i, 1] = (bad[i, 1] & 0xFFFF0000) | 2             # two tile steps on a uop over several row blocks
    with pytest.raises(UM.ProgramError):
        UM.Machine(bad, sb, d, [M, X, Y], n_cores=1, slot_bytes=2048, n_slots=14).run()
    bad = np.array(w, copy=True)
    bad[i, 3] = (bad[i, 3] & ~np.uint32(0xFF << 16)) | np.uint32(2 << 16)   # says two blocks: the region of four is too wide
    with pytest.raises(UM.ProgramError):
        UM.Machine(bad, sb, d, [M, X, Y], n_cores=1, slot_bytes=2048, n_slots=14).run()


def test_leading_dimension():
    M, X, Y = _inputs(24, 40, 2, seed=9, ld=52)
    p = A.dense_matvec_program(24, 40, 52, 2, 8, 16, 1024, 2)
    _run(p, [M, X, Y], slot_bytes=1024, n_slots=8)
    _check_result(M, X, Y, ld=52)


def test_closed_forms_through_the_machine():
    rows, K = 64, 256
    M = np.repeat((np.arange(rows) % 1024).astype(np.float32)[:, None], K, axis=1)
    X = np.ones((1, K), np.float32)
    Y = np.zeros((1, rows), np.float32)
    _run(A.dense_matvec_program(rows, K, K, 1, 8, 64, 2048, 3), [M, X, Y], slot_bytes=2048, n_slots=9)
    assert np.array_equal(Y[0], K * (np.arange(rows) % 1024).astype(np.float32))
    # a single non-zero entry picks one term: any indexing slip moves or loses it
    for (i, j) in [(0, 0), (63, 255), (17, 130)]:
        M = np.zeros((rows, K), np.float32)
        M[i, j] = 2.0
        X = np.arange(1, K + 1, dtype=np.float32)[None, :]
        Y = np.full((1, rows), np.nan, np.float32)
        _run(A.dense_matvec_program(rows, K, K, 1, 8, 64, 2048, 3), [M, X, Y], slot_bytes=2048, n_slots=9)
        exp = np.zeros(rows, np.float32)
        exp[i] = 2.0 * (j + 1)
        assert np.array_equal(Y[0], exp)


# ---- determinacy under every legal schedule -------------------------------------------------------
def test_every_schedule_gives_the_same_image_and_traces():
    rows, K, B = 40, 96, 2
    M, X, _ = _inputs(rows, K, B, seed=4)
    p = A.dense_matvec_program(rows, K, K, B, 8, 32, 1024, 2)
    ref = None
    for i in range(101):
        Y = np.full((B, rows), np.nan, np.float32)
        m = _run(p, [M, X, Y], "program" if i == 0 else "random", seed=i, slot_bytes=1024, n_slots=6)
        got = (Y.tobytes(), m.trace_vmc, m.trace_vcc)
        if ref is None:
            ref = got
        assert got == ref
    _check_result(M, X, Y)


def test_allocation_log_lowest_feasible_and_never_overlapping():
    M, X, Y = _inputs(64, 128, 2, seed=5)
    p = A.dense_matvec_program(64, 128, 128, 2, 8, 32, 1024, 2)
    for seed in range(5):
        m = _run(p, [M, X, Y], "random", seed=seed, slot_bytes=1024, n_slots=7)
        for core in range(2):
            assert m.alloc_log[core]
            for before, n, pos in m.alloc_log[core]:
                s = format(before, "032b")[::-1][:7]
                assert pos == s.find("0" * n) and pos >= 0
            assert m.cores[core].mask == 0 and 1 <= m.cores[core].peak_slots <= 7


# ---- dynamic address generation -------------------------------------------------------------------
def test_looped_program_trace_is_the_arithmetic_progression():
    rows, K, B, R, Kt, ncores = 64, 96, 2, 4, 32, 2
    M, X, Y = _inputs(rows, K, B, seed=6)
    p = A.looped_matvec_program(rows, K, K, B, R, Kt, 1024, ncores)
    m = _run(p, [M, X, Y], slot_bytes=1024, n_slots=6)
    _check_result(M, X, Y)
    nk, per = K // Kt, rows // R // (ncores * 2)
    for core in range(ncores):
        exp = []
        for v in range(2):
            first = (core * 2 + v) * per
            for rb in range(first, first + per):
                for kt in range(nk):
                    exp.append((A.LOAD, 0, (rb * R * K + kt * Kt) * 4, R))     # desc 0: matrix
                    exp.append((A.LOAD, 1, kt * Kt * 4, B))                    # desc 1: vector
                exp.append((A.STORE, 2, rb * R * 4, B))                        # desc 2: result
        got = [(op, d, off, n) for (_pc, op, d, off, n) in m.trace_vmc[core]]
        assert got == exp
    # the per-uop program counters repeat with the loop body: only 3 distinct memory uops per compute core
    assert len({pc for (pc, *_r) in m.trace_vmc[0]}) == 6


def test_looped_and_literal_programs_touch_the_same_addresses():
    rows, K, B, R, Kt, ncores = 32, 64, 1, 4, 16, 2
    M, X, Y1 = _inputs(rows, K, B, seed=7)
    Y2 = Y1.copy()
    a = _run(A.looped_matvec_program(rows, K, K, B, R, Kt, 256, ncores), [M, X, Y1], slot_bytes=256, n_slots=6)
    b = _run(A.dense_matvec_program(rows, K, K, B, R, Kt, 256, ncores), [M, X, Y2], slot_bytes=256, n_slots=6)
    assert Y1.tobytes() == Y2.tobytes()
    strip = lambda tr: sorted((op, off, n) for (_pc, op, _d, off, n) in tr)
    assert sorted(sum((strip(t) for t in a.trace_vmc), [])) == sorted(sum((strip(t) for t in b.trace_vmc), []))


def test_control_uops():
    p = A.Program(1, 2)
    vm = p.vmc(0)
    vm += [A.word(A.SET, acc=3, imm=-5), A.word(A.LOOP, imm=3), A.word(A.LOOP, imm=4), A.word(A.ADD, acc=1, imm=10),
           A.word(A.REPEAT, acc=2, imm=1), A.word(A.REPEAT, acc=3, imm=100)]
    w, sb, d = p.finish()
    m = UM.Machine(w, sb, d, [], n_cores=1).run()
    acc = m.cores[0].vmc.acc
    assert acc[1] == 120 and acc[2] == 12 and acc[3] == 295 and acc[0] == 0
    for bad in ([A.word(A.REPEAT)], [A.word(A.LOOP, imm=2), A.word(A.HALT)], [A.word(A.LOOP, imm=0)],
                [A.word(A.LOOP, imm=1)] * 5, [A.word(A.MATVEC)]):
        p = A.Program(1, 2)
        p.vmc(0).extend(bad)
        w, sb, d = p.finish()
        with pytest.raises(UM.ProgramError):
            UM.Machine(w, sb, d, [], n_cores=1).run()


def test_continue_if_leaves_the_loop_when_its_register_reaches_the_bound():
    """Traces written out by hand.  A loop of ten trips loads 64-byte rows at acc 0 = 0, 64, 128, ... and adds 64 per
    trip; CONTINUE_IF acc 0 < 192 stands between the ADD and the REPEAT.  Trip 1 loads at 0 (acc becomes 64: goes on),
    trip 2 at 64 (128: goes on), trip 3 at 128 (192: not below 192, the loop is left) - three loads, not ten, and the
    REPEAT's own addition to acc 1 happened exactly twice.  The load behind the loop then sees acc 0 = 192."""
    X = np.arange(256, dtype=np.float32)
    p = A.Program(1, 1)
    d = p.desc(0, 1, 64, 64, 64)
    vm, vc = p.vmc(0), p.vcc(0, 0)
    vm += [A.word(A.LOOP, imm=10),
           A.word(A.LOAD, A.F_SEND | A.F_DYNAMIC, vflow=0, vcc=0, acc=0, nslots=1, size=1, imm=0, desc=d),
           A.word(A.ADD, acc=0, imm=64),
           A.word(A.CONTINUE_IF, acc=0, imm=192, size=1),
           A.word(A.REPEAT, acc=1, imm=1000),
           A.word(A.LOAD, A.F_SEND | A.F_DYNAMIC, vflow=0, vcc=0, acc=0, nslots=1, size=1, imm=4, desc=d)]
    # the compute core's own loop is cut short the same way: four regions are dropped one at a time
    vc += [A.word(A.LOOP, imm=100), A.word(A.DROP, size=1), A.word(A.ADD, acc=5, imm=1),
           A.word(A.CONTINUE_IF, acc=5, imm=4, size=1), A.word(A.REPEAT, acc=6, imm=7)]
    w, sb, dd = p.finish()
    for seed in range(5):
        m = UM.Machine(w, sb, dd, [X], n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=4).run("random", seed)
        assert [(r[0], r[3]) for r in m.trace_vmc[0]] == [(1, 0), (1, 64), (1, 128), (5, 196)]     # (pc, byte offset)
        assert m.cores[0].vmc.acc[0] == 192 and m.cores[0].vmc.acc[1] == 2000 and not m.cores[0].vmc.loops
        assert m.cores[0].vccs[0].acc[5] == 4 and m.cores[0].vccs[0].acc[6] == 21 and len(m.trace_vcc[0][0]) == 4
    # inside a nest only the innermost loop is left; the distance skips a whole inner loop
    p = A.Program(1, 1)
    p.vmc(0).extend([A.word(A.LOOP, imm=3), A.word(A.SET, acc=0, imm=0), A.word(A.LOOP, imm=50), A.word(A.ADD, acc=0, imm=1),
                     A.word(A.CONTINUE_IF, acc=0, imm=5, size=4), A.word(A.LOOP, imm=2), A.word(A.ADD, acc=2, imm=1),
                     A.word(A.REPEAT, acc=7, imm=0), A.word(A.REPEAT, acc=3, imm=1), A.word(A.REPEAT, acc=4, imm=1)])
    w, sb, dd = p.finish()
    m = UM.Machine(w, sb, dd, [], n_cores=1, vcc_per_core=1).run()
    acc = m.cores[0].vmc.acc
    # per outer trip: acc 0 counts 1..5; trips 1..4 run the inner pair of ADDs and the middle REPEAT, the fifth leaves
    assert acc[0] == 5 and acc[2] == 3 * 4 * 2 and acc[3] == 3 * 4 and acc[4] == 3
    # malformed: outside a loop; a distance that does not end on a REPEAT; a distance that cuts an inner loop open
    for bad in ([A.word(A.CONTINUE_IF, acc=0, imm=1, size=1), A.word(A.REPEAT)],
                [A.word(A.LOOP, imm=2), A.word(A.CONTINUE_IF, acc=0, imm=1, size=1), A.word(A.ADD), A.word(A.REPEAT)],
                [A.word(A.LOOP, imm=2), A.word(A.CONTINUE_IF, acc=0, imm=1, size=0), A.word(A.REPEAT)],
                [A.word(A.LOOP, imm=2), A.word(A.CONTINUE_IF, acc=0, imm=1, size=2), A.word(A.LOOP, imm=2), A.word(A.REPEAT), A.word(A.REPEAT)]):
        p = A.Program(1, 1)
        p.vmc(0).extend(bad)
        w, sb, dd = p.finish()
        with pytest.raises(UM.ProgramError):
            UM.Machine(w, sb, dd, [], n_cores=1, vcc_per_core=1).run()


# ---- deadlock --------------------------------------------------------------------------------------
def test_in_order_over_allocation_deadlocks():
    # the matrix tile takes both slots of a two-slot pool; the vector tile that the compute core needs
    # next can never be allocated, and the matrix tile is only returned after that vector tile was used
    M, X, Y = _inputs(8, 64, 1, seed=8)
    p = A.dense_matvec_program(8, 64, 64, 1, 8, 64, 1024, 1, vcc_per_core=1)     # matrix tile = 2 KB = 2 slots
    w, sb, d = p.finish()
    with pytest.raises(UM.DeadlockError):
        UM.Machine(w, sb, d, [M, X, Y], n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=2).run()
    for seed in range(10):                   # one more slot and every schedule completes
        UM.Machine(w, sb, d, [M, X, Y], n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=3).run("random", seed)
    _check_result(M, X, Y)


def test_wrong_send_order_is_rejected_by_the_compute_uop():
    # m2c delivers in program order of the send uops; two matrix tiles in a row break the listing's a, b, a, b
    M, X, Y = _inputs(8, 64, 1, seed=8)
    p = A.Program(1, 1)
    dm, dx, dy = p.desc(0, 8, 128, 128, 256), p.desc(1, 1, 128, 128, 256), p.desc(2, 1, 32, 32, 32)
    p.vmc(0).extend([A.word(A.LOAD, A.F_SEND, vflow=0, nslots=1, size=8, imm=0, desc=dm),
                     A.word(A.LOAD, A.F_SEND, vflow=0, nslots=1, size=8, imm=128, desc=dm),
                     A.word(A.LOAD, A.F_SEND, vflow=1, nslots=1, size=1, imm=0, desc=dx),
                     A.word(A.LOAD, A.F_SEND, vflow=1, nslots=1, size=1, imm=128, desc=dx),
                     A.word(A.STORE, A.F_SEND | A.F_RECV, vflow=2, nslots=1, size=1, imm=0, desc=dy)])
    p.vcc(0, 0).append(A.word(A.MATVEC, size=2, imm=A.matvec_imm(1, 8, 8)))
    w, sb, d = p.finish()
    with pytest.raises(UM.ProgramError):
        UM.Machine(w, sb, d, [M, X, Y], n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=5).run()


def test_missing_send_deadlocks():
    M, X, Y = _inputs(8, 32, 1, seed=10)
    p = A.dense_matvec_program(8, 32, 32, 1, 8, 32, 1024, 1, vcc_per_core=1)
    vm = p.vmc(0)
    u = UM.decode(vm[1])
    vm[1] = A.word(A.LOAD, 0, vflow=u.vflow, vcc=u.vcc, nslots=u.nslots, size=u.size, imm=u.imm, desc=u.desc)
    w, sb, d = p.finish()
    with pytest.raises(UM.DeadlockError):
        UM.Machine(w, sb, d, [M, X, Y], n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=4).run()


# ---- depId between memory cores --------------------------------------------------------------------
def test_dep_id_orders_a_store_before_a_dependent_load():
    # core 0 computes t = M1 x and signals depId 5; core 1 loads t with load.dep and computes y = M2 t
    rng = np.random.default_rng(12)
    M1 = rng.standard_normal((8, 16)).astype(np.float32)
    M2 = rng.standard_normal((4, 8)).astype(np.float32)
    x = rng.standard_normal((1, 16)).astype(np.float32)
    for seed in range(20):
        t = np.full((1, 8), np.nan, np.float32)
        y = np.full((1, 4), np.nan, np.float32)
        p = A.Program(2, 1)
        d_m1, d_x, d_t = p.desc(0, 8, 64, 64, 64), p.desc(1, 1, 64, 64, 64), p.desc(2, 1, 32, 32, 32)
        d_m2, d_t_in, d_y = p.desc(3, 4, 32, 32, 32), p.desc(2, 1, 32, 32, 32), p.desc(4, 1, 16, 16, 16)
        p.vmc(0).extend([A.word(A.LOAD, A.F_SEND, vflow=0, nslots=1, size=8, desc=d_m1),
                         A.word(A.LOAD, A.F_SEND, vflow=1, nslots=1, size=1, desc=d_x),
                         A.word(A.STORE, A.F_SEND | A.F_RECV | A.F_DEP_SEND, vflow=2, nslots=1, size=1, desc=d_t,
                                dep_id=5)])
        p.vcc(0, 0).append(A.word(A.MATVEC, size=1, imm=A.matvec_imm(1, 8, 4)))
        p.vmc(1).extend([A.word(A.LOAD, A.F_SEND, vflow=0, nslots=1, size=4, desc=d_m2),
                         A.word(A.LOAD, A.F_SEND | A.F_DEP_RECV, vflow=1, nslots=1, size=1, desc=d_t_in, dep_id=5,
                                dep_count=1),
                         A.word(A.STORE, A.F_SEND | A.F_RECV, vflow=2, nslots=1, size=1, desc=d_y)])
        p.vcc(1, 0).append(A.word(A.MATVEC, size=1, imm=A.matvec_imm(1, 4, 2)))
        w, sb, d = p.finish()
        m = UM.Machine(w, sb, d, [M1, x, t, M2, y], n_cores=2, vcc_per_core=1, slot_bytes=512, n_slots=4)
        m.run("random", seed)
        t_ref, _ = gemv_ref.gemv_dense(M1, x)
        assert np.array_equal(t, t_ref.astype(np.float32))
        y_ref, _ = gemv_ref.gemv_dense(M2, t)
        assert np.array_equal(y, y_ref.astype(np.float32))
        assert m.dep[5] == 1


def _golden_constants():
    import os
    out = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "deployment_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = int(line[1])
    return out


def test_paper_deployment_constants_are_the_defaults():
    # the values the paper prints (tests/golden/deployment_constants.txt, each with the passage that states it):
    # one VMC and two VCCs per core, 8 KB slots, a 32-bit slot mask
    import inspect
    g = _golden_constants()
    sig = inspect.signature(UM.Machine.__init__).parameters
    assert sig["vcc_per_core"].default == g["vcc_per_core"] == 2 and sig["slot_bytes"].default == g["slot_bytes"] == 8192
    assert g["mask_bits"] == 32 and g["vmc_per_core"] == 1
    with pytest.raises(AssertionError):
        UM.Machine(np.zeros((1, 4), np.uint32), np.zeros(4, np.uint32), np.zeros((1, 8), np.uint32), [],
                   n_cores=1, n_slots=g["mask_bits"] + 1)
    # Section 3's example: four core pairs, the matrix cut along its rows, every pair one row block; the product comes out
    rows, K = 4 * 8, 64
    M, X, Y = _inputs(rows, K, 1, seed=3)
    m = _run(A.dense_matvec_program(rows, K, K, 1, 8, 64, 8192, g["example_cores"], vcc_per_core=1), [M, X, Y], slot_bytes=8192, n_slots=8)
    _check_result(M, X, Y)
    assert [sum(1 for r in t if r[1] == UM.STORE) for t in m.trace_vmc] == [1] * g["example_cores"]


# ---- memory uops with no arithmetic behind them (Section 6.3, "Memory virtual core overhead") -------
# Closed forms: a copy leaves the destination equal to the source byte for byte and touches nothing past
# the range; a fill leaves copies of one word; a read leaves memory as it was.  The traces are the blocks
# of the range in order, which is written out here by hand and not taken from the assembler.
@pytest.mark.parametrize("nbytes,tile,ncores", [(4096, 1024, 2), (7 * 1024 + 512, 2048, 2), (48, 1024, 1), (64 * 1024 + 16, 4096, 3)])
def test_copy_program_is_the_identity_on_its_range(nbytes, tile, ncores):
    rng = np.random.default_rng(nbytes)
    src = rng.integers(0, 256, nbytes + 64, dtype=np.uint8)
    for i in range(4):
        dst = np.full(nbytes + 64, 0xA5, np.uint8)
        p = A.stream_program("copy", nbytes, tile, 1024, ncores, row_bytes=512)
        m = _run(p, [src, dst], "program" if i == 0 else "random", seed=i, slot_bytes=1024, n_slots=9)
        assert np.array_equal(dst[:nbytes], src[:nbytes]) and np.all(dst[nbytes:] == 0xA5)
        m.check_final()


def test_fill_and_read_programs():
    nbytes, tile = 9 * 1024 + 32, 2048
    dst = np.full(nbytes + 32, 0x11, np.uint8)
    p = A.stream_program("fill", nbytes, tile, 1024, 2, value=0xDEADBEEF, row_bytes=1024)
    m = _run(p, [dst], "random", seed=1, slot_bytes=1024, n_slots=5)
    assert np.all(dst[:nbytes].view(np.uint32) == 0xDEADBEEF) and np.all(dst[nbytes:] == 0x11)
    m.check_final()
    src = np.arange(nbytes, dtype=np.uint8)
    keep = src.copy()
    p = A.stream_program("read", nbytes, tile, 1024, 2, row_bytes=1024)
    m = _run(p, [src], "random", seed=2, slot_bytes=1024, n_slots=5)
    assert np.array_equal(src, keep)
    m.check_final()
    # the loads of all cores together cover the range exactly once, block by block
    got = sorted((off, rows) for core in m.trace_vmc for (_pc, op, _d, off, rows) in core if op == UM.LOAD)
    want = [(o, min(tile, nbytes - 32 - o) // 1024) for o in range(0, nbytes - 32, tile)] + [(nbytes - 32, 1)]
    assert got == want
    assert sum(u[2] for core in m.trace_vcc for s in core for u in s) == len(want)


def test_stream_uops_reject_more_bytes_than_the_region_holds():
    p = A.Program(1, 1)
    d = p.desc(0, 1, 64, 64, 64)
    p.vmc(0).append(A.word(A.STORE, A.F_SEND | A.F_RECV, vflow=4, nslots=1, size=1, imm=0, desc=d))
    p.vcc(0, 0).append(A.word(A.FILL, size=1, imm=A.fill_imm(1, 2048)))
    with pytest.raises(UM.ProgramError):
        _run(p, [np.zeros(64, np.uint8)], slot_bytes=1024, n_slots=4)


# ---- several operators in one graph, ordered by depIds between their tiles (Section 4.1) ---------------
def _chain_case(dims, B, seed):
    rng = np.random.default_rng(seed)
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(len(dims) - 1)]
    X = rng.standard_normal((B, dims[0])).astype(np.float32)
    return Ms, X


def _chain_run(dims, B, R, Kt, Ms, X, schedule="program", seed=0, ncores=2, n_slots=8):
    p, w_off, a_off = A.chain_matvec_program(dims, B, R, Kt, 1024, ncores)
    W = np.concatenate([m.ravel() for m in Ms])
    Abuf = np.full(sum(B * d for d in dims), np.nan, np.float32)
    Abuf[:B * dims[0]] = X.ravel()
    w, sb, ds = p.finish()
    m = UM.Machine(w, sb, ds, [W, Abuf, Abuf], n_cores=ncores, slot_bytes=1024, n_slots=n_slots, n_dep_ids=256).run(schedule, seed)
    m.check_final()
    Ys = [Abuf[a_off[l + 1] // 4:a_off[l + 1] // 4 + B * dims[l + 1]].reshape(B, dims[l + 1]) for l in range(len(dims) - 1)]
    return Ys, Abuf, m


def test_chain_of_matvecs_equals_layer_by_layer_gemv():
    dims, B, R, Kt = (64, 96, 32, 64), 2, 8, 32
    Ms, X = _chain_case(dims, B, 1)
    Ys, _, m = _chain_run(dims, B, R, Kt, Ms, X)
    prev = X
    for l, Y in enumerate(Ys):
        # every layer against the fp64 product of its own (fp32) input
        Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
        assert np.all(np.abs(Y.astype(np.float64) - Yr) <= 6e-8 * np.abs(Yr) + 1e-12 * Ya + 1e-45), l
        prev = Y
    # closed form: identity matrices hand the vectors through unchanged, bit for bit
    eye = [np.eye(64, dtype=np.float32)] * 3
    Ys, _, _ = _chain_run((64, 64, 64, 64), B, R, Kt, eye, X)
    assert all(np.array_equal(Y, X) for Y in Ys)


def test_chain_is_determinate_and_never_reads_a_tile_before_it_is_written():
    dims, B, R, Kt = (64, 64, 128, 32), 1, 8, 32
    Ms, X = _chain_case(dims, B, 2)
    ref = None
    for i in range(40):
        # the activations start as NaN: a tile read before its producers have stored would poison the result
        Ys, Abuf, m = _chain_run(dims, B, R, Kt, Ms, X, "program" if i == 0 else "random", seed=i, ncores=3, n_slots=6)
        assert not np.isnan(Abuf).any()
        got = (Abuf.tobytes(), m.trace_vmc, m.trace_vcc)
        ref = ref or got
        assert got == ref


def test_chain_without_its_dependency_flags_reads_too_early_under_some_schedule():
    """The pin of the pin: strip DEP_RECV from the loads and some legal schedule computes from tiles that are not there yet."""
    dims, B, R, Kt = (32, 64, 32), 1, 8, 32
    Ms, X = _chain_case(dims, B, 3)
    p, w_off, a_off = A.chain_matvec_program(dims, B, R, Kt, 1024, 2)
    w, sb, ds = p.finish()
    w = w.copy()
    is_dep_load = ((w[:, 0] & 0xFF) == A.LOAD) & (((w[:, 0] >> 8) & A.F_DEP_RECV) != 0)
    w[is_dep_load, 0] &= ~np.uint32(A.F_DEP_RECV << 8)
    bad = 0
    for i in range(20):
        Abuf = np.full(sum(B * d for d in dims), np.nan, np.float32)
        Abuf[:B * dims[0]] = X.ravel()
        UM.Machine(w, sb, ds, [np.concatenate([m.ravel() for m in Ms]), Abuf, Abuf], n_cores=2, slot_bytes=1024, n_slots=8,
                   n_dep_ids=256).run("random", i)
        bad += int(np.isnan(Abuf).any())
    assert bad > 0
