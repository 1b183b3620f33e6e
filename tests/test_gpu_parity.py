"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bar: integer work (allocator positions, per-unit uop traces with their generated addresses) bit-exact against
the oracle interpreter; floating point |Y_gpu - Y_ref| <= 1e-5 * sum_j |M_ij X_bj| per output against the fp64
GEMV (products and sums in fp64).  Any accumulation order within that bound is a correct result.
"""
import numpy as np
import pytest
import torch

import paper_2605_03190_amd as vdc
import workloads
from oracle import attn_ref, gemv_ref, rope_ref, uop_asm as A, uop_machine as UM

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _check(Y_gpu, Yr, Ya, what=""):
    err = np.abs(Y_gpu.astype(np.float64) - Yr)
    bound = TOL * Ya + 1e-30
    worst = float((err / bound).max())
    assert worst <= 1.0, "%s: error is %.3g times the bound" % (what, worst)
    return worst


@pytest.fixture(scope="module")
def ex():
    e = vdc.Executor()
    yield e
    e.destroy()


def test_slot_allocator_matches_first_fit_bit_exactly(ex):
    rng = np.random.default_rng(0)
    n = 20000
    masks = rng.integers(0, 1 << 32, n, dtype=np.uint64)
    masks[::3] |= rng.integers(0, 1 << 32, len(masks[::3]), dtype=np.uint64)      # denser masks
    masks[:64] = [(1 << i) - 1 for i in range(32)] + [0xFFFFFFFF ^ (1 << i) for i in range(32)]
    masks = masks.astype(np.uint32)
    for n_slots in (32, 19, 7):
        ns = rng.integers(1, 5, n).astype(np.int32)
        ns[:8] = [1, 2, 3, 4, 8, 16, 19, 32]
        pos = ex.debug_alloc(_dev(masks.view(np.int32)), _dev(ns), n_slots).cpu().numpy()
        exp = np.array([UM.first_fit(int(m), int(k), n_slots) for m, k in zip(masks, ns)], dtype=np.int32)
        assert np.array_equal(pos, exp)


DENSE_CASES = [
    # rows, K, ld, B, tile_bytes
    (128, 128, 128, 1, 4096),          # configuration 1
    (1000, 1000, 1000, 1, 4096),       # row and K tails everywhere
    (517, 2052, 2060, 3, 8192),        # leading dimension, odd sizes, B = 3
    (2048, 4096, 4096, 8, 16384),
    (70000, 128, 128, 2, 8192),        # many row blocks per core, one K tile: MATVECs over several row blocks
    (131077, 64, 72, 3, 4096),         # the same form with a leading dimension, a row tail and three vectors
    (200003, 256, 256, 1, 8192),       # ... with tile rows as wide as a wave
    (100001, 128, 128, 4, 8192),       # ... with the most vectors the form takes
    (100001, 128, 128, 5, 8192),       # one vector more: a MATVEC per row block
    (3, 8, 8, 1, 2048),                # less than one tile
    (4096, 512, 512, 5, 2048),
    (1024, 8192, 8192, 7, 16384),
    # few row blocks, long rows: K is cut into ranges chained by depId signals between memory cores
    (64, 65536, 65536, 1, 16384),
    (256, 32768, 32768, 3, 8192),
    (100, 8200, 8204, 2, 4096),        # row tail and K tail in a split program
    (16, 4096, 4096, 8, 16384),
    # more row blocks than compute cores and some left over: the adaptive tiling step cuts K of the surplus blocks alone
    (10240, 8192, 8192, 1, 16384),     # 640 row blocks on 512 compute cores: 128 cut in four
    (9216, 16392, 16400, 1, 16384),    # ... a K tail and a leading dimension in the last range; 64 cut in eight
    (8180, 8192, 8192, 8, 16384),      # half as many row blocks as compute cores, eight vectors, a ragged last block: all cut in two
]


@pytest.mark.parametrize("rows,K,ld,B,T", DENSE_CASES)
def test_dense_matvec_against_fp64_gemv(ex, rows, K, ld, B, T):
    rng = np.random.default_rng(rows + K + B)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    dM, dX = _dev(M), _dev(X)
    dY = torch.full((B, rows), float("nan"), device="cuda")
    ex.matvec(dM, dX, dY, T, K=K)
    ex.check()
    Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
    _check(dY.cpu().numpy(), Yr, Ya, "dense %s" % ((rows, K, ld, B, T),))


@pytest.mark.parametrize("cfg,shape", [
    (dict(sched_force_parts=3, n_cores=7), (100, 4096, 4100, 2, 4096)),       # five or six items per core: partial results and joining items share cores
    (dict(sched_force_parts=2, n_cores=1), (16, 2048, 2048, 1, 2048)),        # everything on one core
    (dict(sched_force_parts=16, n_cores=64), (300, 16384, 16384, 3, 8192)),   # the finest cut the builder offers
    (dict(sched_force_parts=1), (64, 65536, 65536, 1, 16384)),                # and none at all where the scheduler would cut
    (dict(sched_threshold_pct=300), (12288, 8192, 8192, 1, 16384)),           # a threshold nothing exceeds: left uncut
    (dict(sched_force_parts=103, n_cores=8), (300, 4096, 4100, 2, 4096)),     # 38 row blocks on 16 compute cores: 32 whole, 6 cut in three
    (dict(sched_force_parts=116), (9200, 16384, 16384, 1, 16384)),            # 575 on 512: the 63 surplus blocks in sixteen ranges
])
def test_cuts_of_k_the_scheduler_would_not_take(cfg, shape):
    """Every decomposition the builder offers gives the GEMV, whatever the cost model thinks of it (sched_force_parts), with
    several work items per compute core and producers and consumers of partial results on the same core."""
    rows, K, ld, B, T = shape
    rng = np.random.default_rng(rows + K)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    with vdc.Executor(**cfg) as e:
        s_max, s, tail = e.matvec_tiling(rows, K, B, T)[4:]
        if "sched_force_parts" in cfg:
            assert s == min(cfg["sched_force_parts"] % 100, s_max) and (tail > 0) == (cfg["sched_force_parts"] > 100)
        else:
            assert s == 1 and s_max > 1
        dY = torch.full((B, rows), float("nan"), device="cuda")
        e.matvec(_dev(M), _dev(X), dY, T, K=K)
        e.check()
        Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
        _check(dY.cpu().numpy(), Yr, Ya, "dense %s with %s" % (shape, cfg))


@pytest.mark.parametrize("cfg", [
    dict(n_ldu=1), dict(n_ldu=2), dict(vcc_per_core=1), dict(vcc_per_core=1, n_ldu=1), dict(n_slots=6), dict(n_cores=7),
    dict(slot_bytes=4096, n_slots=32), dict(slot_bytes=16384), dict(tile_rows=64), dict(n_cores=128),
    dict(n_stu=2), dict(n_stu=2, n_ldu=2, n_cores=100),
])
def test_other_deployment_constants(cfg):
    """The executor with fewer load units, one compute core per memory core, few slots, odd core counts, other slot
    sizes, another tile shape, half the chip, two store units per core: same results (dense with tails, ragged, split along K, fused rope)."""
    rng = np.random.default_rng(31)
    with vdc.Executor(**cfg) as e:
        for rows, K, ld, B, T in ((1000, 1000, 1000, 1, 4096), (517, 2052, 2060, 3, 8192), (2048, 4096, 4096, 8, 16384), (64, 32768, 32768, 2, 16384)):
            if T < e.cfg.slot_bytes and cfg.get("slot_bytes") == 16384 and B * 256 * 4 > 16384:
                continue
            M = rng.standard_normal((rows, ld)).astype(np.float32)
            X = rng.standard_normal((B, K)).astype(np.float32)
            dY = torch.full((B, rows), float("nan"), device="cuda")
            e.matvec(_dev(M), _dev(X), dY, T, K=K)
            e.check()
            Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
            _check(dY.cpu().numpy(), Yr, Ya, "dense %s with %s" % ((rows, K, ld, B, T), cfg))
        K = 128
        row_off = np.array([0, 700, 700, 716, 5000, 5001, 9000, 20000], dtype=np.int64)
        M = rng.standard_normal((20000, K)).astype(np.float32)
        X = rng.standard_normal((7, K)).astype(np.float32)
        dY = torch.full((20000,), float("nan"), device="cuda")
        e.matvec_ragged(_dev(M), row_off, _dev(X), dY, 8192)
        e.check()
        Yr, Ya = gemv_ref.gemv_ragged(M, row_off, X)
        _check(dY.cpu().numpy(), Yr, Ya, "ragged with %s" % (cfg,))
        rows, K, B = 516, 1028, 3
        M = rng.standard_normal((rows, K)).astype(np.float32)
        X = rng.standard_normal((B, K)).astype(np.float32)
        Tt = rope_ref.table(rng.uniform(-3, 3, (B, rows // 2)))
        dY = torch.full((B, rows), float("nan"), device="cuda")
        e.matvec_rope(_dev(M), _dev(X), _dev(Tt), dY, 8192)
        e.check()
        O, Oa = gemv_ref.gemv_dense(M, X)
        Rr, Ra = rope_ref.rope(O, Tt)
        scale = np.empty_like(Oa)
        scale[:, 0::2] = Oa[:, 0::2] + Oa[:, 1::2]
        scale[:, 1::2] = scale[:, 0::2]
        _check(dY.cpu().numpy(), Rr, scale + Ra, "rope with %s" % (cfg,))


def test_closed_forms_on_the_gpu(ex):
    rows, K = 3000, 1536
    M = np.repeat((np.arange(rows) % 1024).astype(np.float32)[:, None], K, axis=1)
    dY = torch.empty((1, rows), device="cuda")
    ex.matvec(_dev(M), torch.ones((1, K), device="cuda"), dY, 8192)
    ex.check()
    assert np.array_equal(dY.cpu().numpy()[0], (K * (np.arange(rows) % 1024)).astype(np.float32))   # exact in fp32
    # identity block: y = x bit for bit
    x = np.random.default_rng(1).standard_normal((2, 256)).astype(np.float32)
    dY = torch.empty((2, 256), device="cuda")
    ex.matvec(torch.eye(256, device="cuda"), _dev(x), dY, 4096)
    ex.check()
    assert np.array_equal(dY.cpu().numpy(), x)


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_uop_traces_and_result_match_the_interpreter(name):
    """Configurations 1 and 2: the address trace of every unit is bit-exact against the sequential interpreter
    running the same uop graph, and the result matches the fp64 GEMV."""
    cfg = workloads.CONFIGS[name]
    w_ = workloads.make(cfg, device="cuda")
    M, X = w_.M.cpu().numpy(), w_.X.cpu().numpy()
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        nc, ns = ex.cfg.n_cores, ex.cfg.n_slots
        words, sb, descs = ex.matvec_program(cfg.rows, cfg.K, cfg.K, cfg.B, cfg.tile_bytes)
        prog = ex.program_create(words, sb, descs, [M.nbytes, X.nbytes, cfg.B * cfg.rows * 4])
        dY = torch.full((cfg.B, cfg.rows), float("nan"), device="cuda")
        cap = 4096
        trace, count = ex.run(prog, [w_.M, w_.X, dY], trace_cap=cap)
        ex.check()
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
    Yo = np.full((cfg.B, cfg.rows), np.nan, np.float32)
    m = UM.Machine(words, sb, descs, [M, X, Yo], n_cores=nc, slot_bytes=cfg.slot_bytes, n_slots=ns).run()
    V = 2
    for core in range(nc):
        s = core * (1 + V)
        exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
        assert count[s] == len(exp) <= cap
        assert [tuple(int(x) for x in r) for r in trace[s, :len(exp)]] == exp
        for v in range(V):
            exp = [(pc, op | (n << 16), imm & 0xFFFFFFFF, imm >> 32) for (pc, op, n, imm) in m.trace_vcc[core][v]]
            assert count[s + 1 + v] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[s + 1 + v, :len(exp)]] == exp
    Yr, Ya = gemv_ref.gemv_dense(M, X)
    _check(dY.cpu().numpy(), Yr, Ya, name)
    _check(Yo, Yr, Ya, name + " (interpreter)")


@pytest.mark.parametrize("cfg,shape", [
    (dict(sched_force_parts=4), (96, 8192, 8192, 2, 4096)),          # all 12 row blocks in four ranges on 16 compute cores
    (dict(sched_force_parts=103), (300, 4096, 4100, 2, 4096)),       # 38 row blocks: 32 whole, the 6 left over in three ranges
    (dict(sched_force_parts=16), (160, 8192 + 36, 8192 + 36, 8, 16384)),    # 5 blocks of 32 rows, 15 partial results joined four a step, a K tail
])
def test_uop_traces_of_cut_programs_match_the_interpreter(cfg, shape):
    """Programs in which the adaptive tiling step's decompositions are forced (K cut for all row blocks, for the surplus
    alone): every unit's trace (pc, uop, generated address), the depId waits among them, is bit-exact against the interpreter
    running the same graph, and the result is the fp64 GEMV."""
    rows, K, ld, B, T = shape
    rng = np.random.default_rng(rows + K)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    with vdc.Executor(n_cores=8, **cfg) as ex:
        nc, ns, slot = ex.cfg.n_cores, ex.cfg.n_slots, ex.cfg.slot_bytes
        s, tail = ex.matvec_tiling(rows, K, B, T)[5:]
        assert s == cfg["sched_force_parts"] % 100 and (tail > 0) == (cfg["sched_force_parts"] > 100)
        words, sb, descs = ex.matvec_program(rows, K, ld, B, T)
        ws = ex.matvec_workspace(rows, K, ld, B, T)
        assert ws.size
        prog = ex.program_create(words, sb, descs, [((rows - 1) * ld + K) * 4, X.nbytes, B * rows * 4, ws.nbytes])
        dY = torch.full((B, rows), float("nan"), device="cuda")
        cap = 8192
        trace, count = ex.run(prog, [_dev(M), _dev(X), dY, _dev(ws)], trace_cap=cap)
        ex.check()
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
    Yo = np.full((B, rows), np.nan, np.float32)
    m = UM.Machine(words, sb, descs, [M, X, Yo, ws.copy()], n_cores=nc, slot_bytes=slot, n_slots=ns).run()
    V = 2
    for core in range(nc):
        st = core * (1 + V)
        exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
        assert count[st] == len(exp) <= cap
        assert [tuple(int(x) for x in r) for r in trace[st, :len(exp)]] == exp
        for v in range(V):
            exp = [(pc, op | (n << 16), imm & 0xFFFFFFFF, imm >> 32) for (pc, op, n, imm) in m.trace_vcc[core][v]]
            assert count[st + 1 + v] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[st + 1 + v, :len(exp)]] == exp
    Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
    _check(dY.cpu().numpy(), Yr, Ya, "cut %s %s" % (cfg, shape))
    _check(Yo, Yr, Ya, "cut %s %s (interpreter)" % (cfg, shape))


@pytest.mark.parametrize("rows,nk,T", [(2048, 64, 16384), (1000, 32, 8192)])
def test_eight_vectors_with_a_vector_tile_over_two_steps(rows, nk, T):
    """issue_flags bit 1: eight vectors take vector tiles that hold the pieces of two steps (a loop body of six memory uops
    on every memory core).  Run once with traces (the front end's general path), every unit's trace bit for bit the
    interpreter's, and once without (the loop body replayed as one batch of six): both results are the fp64 GEMV, and both
    have the bits of the step-by-step program's result."""
    K, B = 128 * nk, 8
    rng = np.random.default_rng(rows)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    dM, dX = _dev(M), _dev(X)
    res = {}
    for fl in (2, 0):
        with vdc.Executor(n_cores=16, issue_flags=fl, sched_force_parts=1) as ex:
            nc, ns, slot = ex.cfg.n_cores, ex.cfg.n_slots, ex.cfg.slot_bytes
            words, sb, descs = ex.matvec_program(rows, K, K, B, T)
            xspans = {(int(x[3]) >> 8) & 0x7F for x in words[(words[:, 0] & 0xFF) == 16]}
            assert xspans == ({2} if fl == 2 else {0})
            prog = ex.program_create(words, sb, descs, [M.nbytes, X.nbytes, B * rows * 4])
            dY = torch.full((B, rows), float("nan"), device="cuda")
            ex.run(prog, [dM, dX, dY])
            ex.check()
            res[fl] = dY.cpu().numpy()
            if fl == 2:
                dY2 = torch.full((B, rows), float("nan"), device="cuda")
                cap = 8192
                trace, count = ex.run(prog, [dM, dX, dY2], trace_cap=cap)
                ex.check()
                trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
                assert np.array_equal(dY2.cpu().numpy(), res[2])
                Yo = np.full((B, rows), np.nan, np.float32)
                m = UM.Machine(words, sb, descs, [M, X, Yo], n_cores=nc, slot_bytes=slot, n_slots=ns).run()
                V = 2
                for core in range(nc):
                    st = core * (1 + V)
                    exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
                    assert count[st] == len(exp) <= cap
                    assert [tuple(int(x) for x in r) for r in trace[st, :len(exp)]] == exp
                    for v in range(V):
                        exp = [(pc, op | (n << 16), imm & 0xFFFFFFFF, imm >> 32) for (pc, op, n, imm) in m.trace_vcc[core][v]]
                        assert count[st + 1 + v] == len(exp)
                        assert [tuple(int(x) for x in r) for r in trace[st + 1 + v, :len(exp)]] == exp
    Yr, Ya = gemv_ref.gemv_dense(M, X)
    _check(res[2], Yr, Ya, "vector tile over two steps")
    _check(Yo, Yr, Ya, "vector tile over two steps (interpreter)")
    assert np.array_equal(res[0], res[2])


def test_programs_assembled_by_the_oracle_side_run_on_the_gpu():
    """uop graphs that no product code produced (oracle-side assembler), through vdc_program_create / vdc_run."""
    rng = np.random.default_rng(3)
    with vdc.Executor(n_cores=8, slot_bytes=2048, n_slots=16) as ex:
        for build, (rows, K, B, R, Kt) in [(A.dense_matvec_program, (200, 328, 3, 16, 64)),
                                           (A.looped_matvec_program, (512, 384, 2, 8, 128)),
                                           (A.dense_matvec_program, (64, 2048, 1, 1, 1024))]:
            M = rng.standard_normal((rows, K)).astype(np.float32)
            X = rng.standard_normal((B, K)).astype(np.float32)
            p = build(rows, K, K, B, R, Kt, 2048, 8, nt=True)
            words, sb, descs = p.finish()
            prog = ex.program_create(words, sb, descs, [M.nbytes, X.nbytes, B * rows * 4])
            dY = torch.full((B, rows), float("nan"), device="cuda")
            trace, count = ex.run(prog, [_dev(M), _dev(X), dY], trace_cap=2048)
            ex.check()
            Yr, Ya = gemv_ref.gemv_dense(M, X)
            _check(dY.cpu().numpy(), Yr, Ya, build.__name__)
            Yo = np.zeros((B, rows), np.float32)
            m = UM.Machine(words, sb, descs, [M, X, Yo], n_cores=8, slot_bytes=2048, n_slots=16).run()
            trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
            for core in range(8):
                exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
                assert count[core * 3] == len(exp)
                assert [tuple(int(x) for x in r) for r in trace[core * 3, :len(exp)]] == exp
            prog.destroy()


def test_continue_if_cuts_loops_short_on_the_gpu():
    """continue_if (Section 4.1) on both kinds of core: every row block's sweep over K is a LOOP of 1000 trips that the
    memory core leaves when its offset register reaches the end of the row (so the trip count comes from a register, not
    from the LOOP), with store and second row block behind it; the compute core's stream is cut short the same way.
    Result against the fp64 product, the memory cores' traces against the interpreter's."""
    rng = np.random.default_rng(21)
    rows, K, B, R, Kt, C, slot = 96, 640, 2, 8, 128, 4, 4096
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    p = A.Program(C, 2)
    dm, dx = p.desc(0, R, Kt * 4, Kt * 4, K * 4), p.desc(1, B, Kt * 4, Kt * 4, K * 4)
    dy = p.desc(2, B, R * 4, R * 4, rows * 4)
    nk = K // Kt
    for rb in range(rows // R):
        unit = rb % (C * 2)
        core, v = unit // 2, unit % 2
        vm = p.vmc(core)
        vm += [A.word(A.SET, acc=2, imm=0), A.word(A.LOOP, imm=1000),
               A.word(A.LOAD, A.F_SEND | A.F_DYNAMIC | A.F_NT, vflow=v, vcc=v, acc=2, nslots=1, size=R, imm=rb * R * K * 4, desc=dm),
               A.word(A.LOAD, A.F_SEND | A.F_DYNAMIC, vflow=2 + v, vcc=v, acc=2, nslots=1, size=B, imm=0, desc=dx),
               A.word(A.ADD, acc=2, imm=Kt * 4),
               A.word(A.CONTINUE_IF, acc=2, imm=K * 4, size=1),
               A.word(A.REPEAT, acc=7, imm=0),
               A.word(A.STORE, A.F_SEND | A.F_RECV, vflow=4 + v, vcc=v, nslots=1, size=B, imm=rb * R * 4, desc=dy)]
        vc = p.vcc(core, v)
        # one MATVEC per trip of a loop that a register ends after the first trip
        vc += [A.word(A.SET, acc=1, imm=0), A.word(A.LOOP, imm=50), A.word(A.MATVEC, size=nk, imm=A.matvec_imm(B, R, Kt // 4)),
               A.word(A.ADD, acc=1, imm=1), A.word(A.CONTINUE_IF, acc=1, imm=1, size=1), A.word(A.REPEAT, acc=0, imm=0)]
    words, sb, descs = p.finish()
    with vdc.Executor(n_cores=C, slot_bytes=slot, n_slots=12) as ex:
        prog = ex.program_create(words, sb, descs, [M.nbytes, X.nbytes, B * rows * 4])
        dY = torch.full((B, rows), float("nan"), device="cuda")
        trace, count = ex.run(prog, [_dev(M), _dev(X), dY], trace_cap=1024)
        ex.check()
        Yr, Ya = gemv_ref.gemv_dense(M, X)
        _check(dY.cpu().numpy(), Yr, Ya, "continue_if")
        Yo = np.zeros((B, rows), np.float32)
        m = UM.Machine(words, sb, descs, [M, X, Yo], n_cores=C, slot_bytes=slot, n_slots=12).run()
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
        for core in range(C):
            exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
            blocks = sum(1 for rb in range(rows // R) if (rb % (C * 2)) // 2 == core)
            assert len(exp) == blocks * (2 * nk + 1)      # per row block: nk trips of two loads (not 1000), one store
            assert count[core * 3] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[core * 3, :len(exp)]] == exp
        prog.destroy()


def test_graphs_lowered_by_the_library_run_on_the_gpu():
    """Graphs go through the library's lowering steps (vdc_graph_lower: placement, flows, reordering, depIds) and then
    through vdc_program_create / vdc_run: the running example against the fp64 product turned by the fp64 rotation, a chain
    against the layer-by-layer product, a stream that over-commits the slots as written against the product."""
    from oracle import uop_lower as L
    from test_host_logic import _graph_arrays
    rng = np.random.default_rng(31)
    # matvec -> rope, the intermediate kept in local memory by the placement step
    rows, K, B, R, Kt, slot, C = 384, 512, 4, 16, 128, 8192, 6
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    T = rope_ref.table(rng.uniform(-np.pi, np.pi, (B, rows // 2)))
    g = L.matvec_rope_graph(rows, K, B, R, Kt, slot, C)
    with vdc.Executor(n_cores=C, slot_bytes=slot, n_slots=12) as ex:
        nb = [M.nbytes, X.nbytes, B * rows * 4, T.nbytes, B * rows * 4]
        w, sb, d, stats = ex.graph_lower(*_graph_arrays(g), nb, temp_tensors=1 << 4, geom_tensor=2)
        assert stats[0] == rows // R
        prog = ex.program_create(w, sb, d, nb)
        dY = torch.full((B, rows), float("nan"), device="cuda")
        dO = torch.full((B, rows), float("nan"), device="cuda")
        ex.run(prog, [_dev(M), _dev(X), dY, _dev(T), dO])
        ex.check()
        assert bool(torch.isnan(dO).all())                       # the intermediate never reached memory
        O, Oa = gemv_ref.gemv_dense(M, X)
        Rr, Ra = rope_ref.rope(O, T)
        assert np.all(np.abs(dY.cpu().numpy() - Rr) <= 1e-5 * (Ra + Oa) + 1e-30)
        prog.destroy()
    # a chain of three layers with per-tile dependencies
    dims, B, R, Kt, slot, C = (256, 512, 256, 128), 2, 16, 128, 8192, 3
    Ls = len(dims) - 1
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(Ls)]
    W = np.concatenate([m.ravel() for m in Ms])
    X = rng.standard_normal((B, dims[0])).astype(np.float32)
    g = L.chain_graph(dims, B, R, Kt, slot, C)
    with vdc.Executor(n_cores=C, slot_bytes=slot, n_slots=12) as ex:
        nA = B * sum(dims)
        w, sb, d, stats = ex.graph_lower(*_graph_arrays(g), [W.nbytes, nA * 4, nA * 4])
        assert stats[2] == sum(dims[l + 1] // Kt for l in range(Ls - 1)) and stats[4] > 0
        prog = ex.program_create(w, sb, d, [W.nbytes, nA * 4, nA * 4])
        for rnd in range(2):                                     # twice over the same buffers: the counters start from zero again
            dA = torch.full((nA,), float("nan"), device="cuda")
            dA[:B * dims[0]] = _dev((X * (rnd + 1)).ravel())
            ex.run(prog, [_dev(W), dA, dA])
            ex.check()
            a = dA.cpu().numpy()
            x, off = (X * (rnd + 1)).astype(np.float32), B * dims[0]
            for l in range(Ls):
                Yr, Ya = gemv_ref.gemv_dense(Ms[l], x)
                got = a[off:off + B * dims[l + 1]].reshape(B, dims[l + 1])
                _check(got, Yr, Ya, "lowered chain, layer %d" % l)
                x = got
                off += B * dims[l + 1]
        prog.destroy()


ROPE_CASES = [
    # rows, K, ld, B, tile_bytes
    (128, 128, 128, 1, 4096),
    (1000, 1000, 1000, 1, 4096),       # row tail and K tail
    (516, 2052, 2060, 3, 8192),
    (2048, 4096, 4096, 8, 16384),
    (70000, 128, 128, 2, 8192),        # many row blocks per compute core: the looped form
    (4096, 8192, 8192, 5, 16384),
]


@pytest.mark.parametrize("rows,K,ld,B,T", ROPE_CASES)
def test_fused_matvec_rope_against_the_two_oracles(ex, rows, K, ld, B, T):
    """R = rope(M X, T) with M X kept in local memory (store.local / load.local) against fp64 gemv followed by the fp64
    rotation.  The intermediate is fp32 on the device, so its rounding scale is part of the bound."""
    rng = np.random.default_rng(rows + K + B)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    Tt = rope_ref.table(rng.uniform(-np.pi, np.pi, (B, rows // 2)))
    dY = torch.full((B, rows), float("nan"), device="cuda")
    ex.matvec_rope(_dev(M), _dev(X), _dev(Tt), dY, T, K=K)
    ex.check()
    O, Oa = gemv_ref.gemv_dense(M, X, ld=ld)
    Rr, Ra = rope_ref.rope(O, Tt)
    # |error| <= 1e-5 * (sum of magnitudes behind each of the two values that are combined)
    scale = np.empty_like(Oa)
    scale[:, 0::2] = Oa[:, 0::2] + Oa[:, 1::2]
    scale[:, 1::2] = scale[:, 0::2]
    _check(dY.cpu().numpy(), Rr, scale + Ra, "rope %s" % ((rows, K, ld, B, T),))


def test_fused_program_assembled_by_the_oracle_side_runs_on_the_gpu():
    rows, K, B, R, Kt = 64, 128, 2, 16, 64
    rng = np.random.default_rng(77)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    Tt = rope_ref.table(rng.uniform(-np.pi, np.pi, (B, rows // 2)))
    with vdc.Executor(n_cores=2, slot_bytes=4096) as e2:
        w, sb, d = A.dense_matvec_program(rows, K, K, B, R, Kt, 4096, n_cores=2, rope=True).finish()
        prog = e2.program_create(w, sb, d, [M.nbytes, X.nbytes, 4 * B * rows, Tt.nbytes])
        dY = torch.full((B, rows), float("nan"), device="cuda")
        e2.run(prog, [_dev(M), _dev(X), dY, _dev(Tt)])
        e2.check()
        Y = np.full((B, rows), np.nan, np.float32)
        UM.Machine(w, sb, d, [M, X, Y, Tt], n_cores=2, slot_bytes=4096, n_slots=e2.cfg.n_slots).run("random", 5)
        # the interpreter keeps the intermediate in fp32 as well: the two agree to fp32 rounding of the rotation
        assert np.allclose(dY.cpu().numpy(), Y, rtol=0, atol=2e-5)
        prog.destroy()


STREAM_CASES = [
    # mode, bytes, tile_bytes
    ("copy", 64 << 20, 16384),
    ("copy", (5 << 20) + 7 * 1024 + 48, 8192),     # uneven runs, a short block and a short row
    ("copy", 3 * 4096, 4096),                      # fewer blocks than compute cores
    ("copy", 48, 2048),                            # less than one row
    ("copy", (1 << 20) + 256, 256),                # tiles below a row of 1 KB
    ("fill", (9 << 20) + 1024 + 16, 16384),
    ("fill", 1 << 20, 4096),
    ("read", (33 << 20) + 2048 - 16, 16384),
]


@pytest.mark.parametrize("mode,nbytes,T", STREAM_CASES)
def test_memory_uops_alone_move_every_byte_exactly(ex, mode, nbytes, T):
    """Byte work: bit-exact.  The expected image is the closed form (copy: the source; fill: the word; read: nothing
    changes), and bytes past the range stay as they were."""
    g = torch.Generator(device="cuda").manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, device="cuda", generator=g)
    keep = src.clone()
    dst = torch.full((nbytes + 64,), 0xEE, dtype=torch.uint8, device="cuda")
    for _ in range(2):                       # the second run takes the cached program
        ex.stream(mode, src if mode != "fill" else None, dst if mode != "read" else None, nbytes, T, value=0xC0FFEE11)
        ex.check()
    assert torch.equal(src, keep)
    if mode == "copy":
        assert torch.equal(dst[:nbytes], src[:nbytes])
    if mode == "fill":
        assert bool((dst[:nbytes].view(torch.int32) == np.int32(np.uint32(0xC0FFEE11).view(np.int32))).all())
    if mode == "read":
        assert bool((dst == 0xEE).all())
    assert bool((dst[nbytes:] == 0xEE).all())


def test_plain_kernel_the_memory_uops_are_measured_against(ex):
    nbytes = (3 << 20) + 16 * 37
    g = torch.Generator(device="cuda").manual_seed(5)
    src = torch.randint(0, 256, (nbytes + 16,), dtype=torch.uint8, device="cuda", generator=g)
    keep = src.clone()
    dst = torch.full((nbytes + 16,), 0xEE, dtype=torch.uint8, device="cuda")
    ex.raw_stream("copy", src, dst, nbytes)
    assert torch.equal(dst[:nbytes], src[:nbytes]) and bool((dst[nbytes:] == 0xEE).all())
    ex.raw_stream("fill", None, dst, nbytes, value=0x01020304)
    assert bool((dst[:nbytes].view(torch.int32) == 0x01020304).all()) and bool((dst[nbytes:] == 0xEE).all())
    ex.raw_stream("read", src, None, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(src, keep)
    with pytest.raises(vdc.VdcError):
        ex.raw_stream("copy", src, dst, 24)


def test_stream_traces_match_the_interpreter_and_oracle_assembled_streams_run():
    """The per-unit traces of a copy are bit-exact against the interpreter running the same uops; then stream programs
    that the oracle-side assembler built (no product tiler) run on the GPU."""
    nbytes, T = 300 * 1024 + 512 + 32, 4096
    rng = np.random.default_rng(11)
    src = rng.integers(0, 256, nbytes, dtype=np.uint8)
    with vdc.Executor(n_cores=8, slot_bytes=2048, n_slots=12) as ex:
        words, sb, descs = ex.stream_program("copy", nbytes, T)
        prog = ex.program_create(words, sb, descs, [nbytes, nbytes])
        dsrc, ddst = _dev(src), torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        trace, count = ex.run(prog, [dsrc, ddst], trace_cap=1024)
        ex.check()
        assert np.array_equal(ddst.cpu().numpy(), src)
        out = np.zeros(nbytes, np.uint8)
        m = UM.Machine(words, sb, descs, [src, out], n_cores=8, slot_bytes=2048, n_slots=12).run()
        assert np.array_equal(out, src)
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
        for core in range(8):
            exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
            assert count[core * 3] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[core * 3, :len(exp)]] == exp
            for v in range(2):
                exp = [(pc, op | (n << 16), imm & 0xFFFFFFFF, imm >> 32) for (pc, op, n, imm) in m.trace_vcc[core][v]]
                assert count[core * 3 + 1 + v] == len(exp)
                assert [tuple(int(x) for x in r) for r in trace[core * 3 + 1 + v, :len(exp)]] == exp
        prog.destroy()
        for mode in ("copy", "fill", "read"):
            p = A.stream_program(mode, nbytes, T, 2048, 8, value=0x0BADF00D, row_bytes=512)
            words, sb, descs = p.finish()
            prog = ex.program_create(words, sb, descs, [nbytes, nbytes] if mode == "copy" else [nbytes])
            ddst = torch.full((nbytes,), 0x77, dtype=torch.uint8, device="cuda")
            ex.run(prog, {"copy": [dsrc, ddst], "fill": [ddst], "read": [dsrc]}[mode])
            ex.check()
            got = ddst.cpu().numpy()
            if mode == "copy":
                assert np.array_equal(got, src)
            elif mode == "fill":
                assert np.all(got.view(np.uint32) == 0x0BADF00D)
            else:
                assert np.all(got == 0x77)
            assert np.array_equal(dsrc.cpu().numpy(), src)
            prog.destroy()


def _attn_inputs(lengths, seed, d=128):
    rng = np.random.default_rng(seed)
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    Q = rng.standard_normal((len(lengths), d)).astype(np.float32)
    K = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
    V = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
    return Q, K, V, ro


def _check_attn(O_gpu, Q, K, V, ro, scale, what):
    """|O - O_ref| <= (2 * 1e-5 * S + 2e-5) * A: S bounds the rounding of a score (it enters through exp, twice: in
    the weight and in the normalisation), A = sum_r p_r |V_rt| is the scale of the weighted sum itself."""
    Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, scale)
    bound = (2.0 * TOL * S[:, None] + 2e-5) * Ar + 1e-30
    worst = float((np.abs(O_gpu.astype(np.float64) - Or) / bound).max())
    assert worst <= 1.0, "%s: error is %.3g times the bound" % (what, worst)


ATTN_CASES = [
    # context lengths, tile_bytes
    ([1], 4096),
    ([40, 7, 300, 9, 64], 4096),                   # tails; one request shared by several compute cores
    ([600], 8192),
    ([33] * 9, 16384),
    ([512], 16384),                                # the paper's regimes: 1 x 512,
    ([512] * 64, 16384),                           # 64 x 512,
    ("rand", 16384),                               # 64 x random[256, 1024],
    ([65536], 16384),                              # 1 x 65536
    ([5000, 1, 17], 8192),
    ([700, 3, 64, 2000], 16384, 64),               # head dimension 64: tiles of 64, 32, 16 context rows
    ([333, 90], 8192, 64),
    ([40, 41, 42, 43], 4096, 64),
]


@pytest.mark.parametrize("case", ATTN_CASES)
def test_decode_attention_against_the_fp64_definition(ex, case):
    lengths, T, d = case if len(case) == 3 else (case[0], case[1], 128)
    if lengths == "rand":
        lengths = list(np.random.default_rng(64).integers(256, 1025, 64))
    Q, K, V, ro = _attn_inputs(lengths, seed=len(lengths) + T, d=d)
    dO = torch.full((len(lengths), d), float("nan"), device="cuda")
    dQ, dK, dV = _dev(Q), _dev(K), _dev(V)
    for _ in range(2):                             # the second run takes the cached program
        ex.attn_decode(dQ, dK, dV, ro, dO, T)
        ex.check()
    _check_attn(dO.cpu().numpy(), Q, K, V, ro, d ** -0.5, "attention %s d %d" % (lengths[:4], d))


def test_attention_traces_match_the_interpreter_and_oracle_assembled_programs_run():
    lengths = [70, 9, 130, 33]
    Q, K, V, ro = _attn_inputs(lengths, seed=8)
    d = 128
    with vdc.Executor(n_cores=4, slot_bytes=4096, n_slots=12) as ex:
        words, sb, descs, n_items = ex.attn_decode_program(ro, d, 4096)
        prog = ex.program_create(words, sb, descs, [K.nbytes, V.nbytes, Q.nbytes, Q.nbytes, n_items * (d + 4) * 4])
        dO = torch.full((len(lengths), d), float("nan"), device="cuda")
        dW = torch.full((n_items, d + 4), float("nan"), device="cuda")
        trace, count = ex.run(prog, [_dev(K), _dev(V), _dev(Q), dO, dW], trace_cap=512)
        ex.check()
        _check_attn(dO.cpu().numpy(), Q, K, V, ro, d ** -0.5, "tiler program")
        Oo, Wo = np.zeros((len(lengths), d), np.float32), np.zeros((n_items, d + 4), np.float32)
        m = UM.Machine(words, sb, descs, [K, V, Q, Oo, Wo], n_cores=4, slot_bytes=4096, n_slots=12, n_dep_ids=1024).run()
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
        for core in range(4):
            exp = [(pc, op | (dd << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, dd, off, n) in m.trace_vmc[core]]
            assert count[core * 3] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[core * 3, :len(exp)]] == exp
            for v in range(2):
                exp = [(pc, op | (n << 16), imm & 0xFFFFFFFF, imm >> 32) for (pc, op, n, imm) in m.trace_vcc[core][v]]
                assert count[core * 3 + 1 + v] == len(exp)
                assert [tuple(int(x) for x in r) for r in trace[core * 3 + 1 + v, :len(exp)]] == exp
        # the partial rows agree with the interpreter's (same tiling, fp32 against fp64 arithmetic)
        Wg = dW.cpu().numpy()
        assert np.allclose(Wg[:, 128:130], Wo[:, 128:130], rtol=1e-4, atol=1e-5) and np.all(Wg[:, 130:] == 0)
        prog.destroy()
        # a program from the oracle-side assembler (another way of cutting and dealing the work)
        p, n_items = A.attn_decode_program(ro, d, 8, 4096, 4, chunk_tiles=3)
        words, sb, descs = p.finish()
        prog = ex.program_create(words, sb, descs, [K.nbytes, V.nbytes, Q.nbytes, Q.nbytes, n_items * (d + 4) * 4])
        dO.fill_(float("nan"))
        dW = torch.full((n_items, d + 4), float("nan"), device="cuda")
        ex.run(prog, [_dev(K), _dev(V), _dev(Q), dO, dW])
        ex.check()
        _check_attn(dO.cpu().numpy(), Q, K, V, ro, d ** -0.5, "oracle-assembled program")
        prog.destroy()
        # the oracle-side assembler's other forms: contexts of one item write their result themselves, and the first item
        # of a cut context joins the others' partial rows (no ATTN_MERGE)
        for chunk in (3, 6):
            p, n_items = A.attn_decode_program(ro, d, 8, 4096, 4, chunk_tiles=chunk, whole=True, join=True)
            words, sb, descs = p.finish()
            assert not any((int(w0) & 0xFF) == A.ATTN_MERGE for w0 in np.asarray(words).reshape(-1, 4)[:, 0])
            n_w = max(n_items, 1)
            prog = ex.program_create(words, sb, descs, [K.nbytes, V.nbytes, Q.nbytes, Q.nbytes, n_w * (d + 4) * 4])
            dO.fill_(float("nan"))
            dW = torch.full((n_w, d + 4), float("nan"), device="cuda")
            ex.run(prog, [_dev(K), _dev(V), _dev(Q), dO, dW])
            ex.check()
            _check_attn(dO.cpu().numpy(), Q, K, V, ro, d ** -0.5, "oracle-assembled program, whole contexts and joins, items of %d tiles" % chunk)
            prog.destroy()


def test_attention_shares_at_their_limits():
    # more contexts than tiles in a share (most compute cores hold several whole contexts, some none); one context over
    # more compute cores than a request may have partial rows (it is cut into 65 equal items instead of at the shares)
    rng = np.random.default_rng(12)
    for lengths, T, ncores, d in ((list(rng.integers(1, 4, 700)), 4096, 0, 128), ([40000], 4096, 40, 128), ([9000, 5, 30000], 8192, 48, 64)):
        Q, K, V, ro = _attn_inputs(lengths, seed=len(lengths), d=d)
        with (vdc.Executor() if ncores == 0 else vdc.Executor(n_cores=ncores)) as ex:
            words, sb, descs, n_items = ex.attn_decode_program(ro, d, T)
            ops = np.asarray(words).reshape(-1, 4)[:, 0] & 0xFF
            joins = (np.asarray(words).reshape(-1, 4)[:, 3] >> 16) & 0xFF
            assert int(joins[ops == A.ATTN].max()) <= 64
            if lengths == [40000]:
                assert int(joins[ops == A.ATTN].max()) == 64 and int((ops == A.ATTN).sum()) == 65
            dO = torch.full((len(lengths), d), float("nan"), device="cuda")
            ex.attn_decode(_dev(Q), _dev(K), _dev(V), ro, dO, T)
            ex.check()
            _check_attn(dO.cpu().numpy(), Q, K, V, ro, d ** -0.5, "attention at the limits of the shares, %d contexts" % len(lengths))


def test_attention_refuses_what_it_does_not_support(ex):
    Q, K, V, ro = _attn_inputs([10, 20], seed=1)
    dQ, dK, dV, dO = _dev(Q), _dev(K), _dev(V), torch.zeros((2, 128), device="cuda")
    for bad in (dict(T=2048), dict(ro=np.array([0, 10, 10])), dict(ro=np.array([1, 10, 30]))):
        a = dict(T=4096, ro=ro)
        a.update(bad)
        with pytest.raises(vdc.VdcError):
            ex.attn_decode(dQ, dK, dV, a["ro"], dO, a["T"])
    with pytest.raises(vdc.VdcError):
        ex.attn_decode(dQ[:, :32].contiguous(), dK, dV, ro, dO, 4096)      # d = 32


CHAIN_CASES = [
    # dims = (K_0, rows_0, rows_1, ...), B, tile_bytes
    ((4096, 4096, 4096, 4096), 1, 16384),
    ((1024, 4096, 1024), 4, 8192),
    ((1000, 516, 2052, 12), 2, 4096),            # K tails and row tails; a last layer of one row block
    ((8192, 32768, 8192), 1, 16384),             # several row blocks per compute core: later ones follow the waiting loads
    ((2048, 2048, 2048, 2048, 2048, 2048, 2048, 2048, 2048), 8, 16384),
]


@pytest.mark.parametrize("dims,B,T", CHAIN_CASES)
def test_chain_of_matvecs_in_one_launch(ex, dims, B, T):
    """Every layer against the fp64 product of its own input as the GPU stored it (so the bar of a single matvec applies
    per layer).  The chain runs twice on the same buffers with different X: a tile that was read from a cache left over
    from the first run, or before its producers had stored it, would show in the second."""
    rng = np.random.default_rng(sum(dims) + B)
    L = len(dims) - 1
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L)]
    dW = _dev(np.concatenate([m.ravel() for m in Ms]))
    a_off = np.concatenate([[0], np.cumsum([B * x for x in dims])])
    dA = torch.full((int(a_off[-1]),), float("nan"), device="cuda")
    for rep in range(2):
        X = rng.standard_normal((B, dims[0])).astype(np.float32)
        dA[:B * dims[0]] = _dev(X.ravel())
        ex.matvec_chain(dW, dA, dims, B, T)
        ex.check()
        Ah = dA.cpu().numpy()
        assert not np.isnan(Ah).any()
        prev = X
        for l in range(L):
            Y = Ah[a_off[l + 1]:a_off[l + 2]].reshape(B, dims[l + 1])
            Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
            _check(Y, Yr, Ya, "chain %s layer %d run %d" % (dims, l, rep))
            prev = Y


def test_two_store_units_serve_the_other_operators_too():
    """Attention (partials and merges signal through depId from both store units), the stream uops and a chain of
    matvecs on an executor with two store units per core, to the same bars as with one."""
    with vdc.Executor(n_stu=2) as e:
        assert e.cfg.n_stu == 2
        for lengths, T, d in (([40, 7, 300, 9, 64], 4096, 128), ([5000, 1, 17], 8192, 128), ([700, 3, 64, 2000], 16384, 64)):
            Q, K, V, ro = _attn_inputs(lengths, seed=11 + T, d=d)
            dO = torch.full((len(lengths), d), float("nan"), device="cuda")
            e.attn_decode(_dev(Q), _dev(K), _dev(V), ro, dO, T)
            e.check()
            _check_attn(dO.cpu().numpy(), Q, K, V, ro, d ** -0.5, "attention %s, two store units" % (lengths,))
        for mode, nbytes, T in (("copy", (5 << 20) + 7 * 1024 + 48, 8192), ("fill", (9 << 20) + 1024 + 16, 16384), ("copy", (1 << 20) + 256, 256)):
            g = torch.Generator(device="cuda").manual_seed(nbytes)
            src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, device="cuda", generator=g)
            dst = torch.full((nbytes + 64,), 0xEE, dtype=torch.uint8, device="cuda")
            e.stream(mode, src if mode != "fill" else None, dst, nbytes, T, value=0xC0FFEE11)
            e.check()
            if mode == "copy":
                assert torch.equal(dst[:nbytes], src[:nbytes])
            else:
                assert bool((dst[:nbytes].view(torch.int32) == np.int32(np.uint32(0xC0FFEE11).view(np.int32))).all())
            assert bool((dst[nbytes:] == 0xEE).all())
        dims, B, T = (1000, 516, 2052, 12), 2, 4096
        rng = np.random.default_rng(3)
        L = len(dims) - 1
        Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L)]
        dW = _dev(np.concatenate([m.ravel() for m in Ms]))
        a_off = np.concatenate([[0], np.cumsum([B * x for x in dims])])
        dA = torch.full((int(a_off[-1]),), float("nan"), device="cuda")
        X = rng.standard_normal((B, dims[0])).astype(np.float32)
        dA[:B * dims[0]] = _dev(X.ravel())
        e.matvec_chain(dW, dA, dims, B, T)
        e.check()
        Ah = dA.cpu().numpy()
        prev = X
        for l in range(L):
            Y = Ah[a_off[l + 1]:a_off[l + 2]].reshape(B, dims[l + 1])
            Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
            _check(Y, Yr, Ya, "chain layer %d, two store units" % l)
            prev = Y


def test_role_placement_changes_no_result(ex):
    """Which units share a SIMD is a matter of speed alone: the same program under every placement gives the same bits
    (the order of every sum is fixed by the program), and the library refuses a placement it does not know."""
    rng = np.random.default_rng(12)
    for rows, K, B, T in ((3000, 128, 1, 8192), (9001, 2052, 3, 8192)):
        M = rng.standard_normal((rows, K)).astype(np.float32)
        X = rng.standard_normal((B, K)).astype(np.float32)
        dM, dX = _dev(M), _dev(X)
        w, sb, d = ex.matvec_program(rows, K, K, B, T)
        prog = ex.program_create(w, sb, d, [M.nbytes, X.nbytes, B * rows * 4])
        try:
            got = []
            for placement in (0, 1, 2):
                prog.set_placement(placement)
                dY = torch.full((B, rows), float("nan"), device="cuda")
                ex.run(prog, [dM, dX, dY])
                ex.check()
                got.append(dY.cpu().numpy())
            assert np.array_equal(got[0], got[1]) and np.array_equal(got[0], got[2])
            Yr, Ya = gemv_ref.gemv_dense(M, X)
            _check(got[1], Yr, Ya, "placement 1 %s" % ((rows, K, B, T),))
            with pytest.raises(vdc.VdcError) as e:
                prog.set_placement(3)
            assert e.value.code == vdc.VDC_EINVAL
        finally:
            prog.destroy()


def test_chain_traces_match_the_interpreter():
    dims, B, T = (256, 512, 128, 256), 2, 4096
    rng = np.random.default_rng(12)
    L = len(dims) - 1
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L)]
    W = np.concatenate([m.ravel() for m in Ms])
    X = rng.standard_normal((B, dims[0])).astype(np.float32)
    with vdc.Executor(n_cores=4, slot_bytes=4096, n_slots=12) as ex:
        words, sb, descs = ex.matvec_chain_program(dims, B, T)
        nA = B * sum(dims)
        prog = ex.program_create(words, sb, descs, [W.nbytes, nA * 4, nA * 4])
        dA = torch.full((nA,), float("nan"), device="cuda")
        dA[:B * dims[0]] = _dev(X.ravel())
        trace, count = ex.run(prog, [_dev(W), dA, dA], trace_cap=1024)
        ex.check()
        Ao = np.full(nA, np.nan, np.float32)
        Ao[:B * dims[0]] = X.ravel()
        m = UM.Machine(words, sb, descs, [W, Ao, Ao], n_cores=4, slot_bytes=4096, n_slots=12, n_dep_ids=1024).run()
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
        for core in range(4):
            exp = [(pc, op | (dd << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, dd, off, n) in m.trace_vmc[core]]
            assert count[core * 3] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[core * 3, :len(exp)]] == exp
        # fp32 on the GPU against fp64 in the interpreter, through three layers
        assert np.allclose(dA.cpu().numpy(), Ao, rtol=1e-4, atol=1e-5)
        prog.destroy()
        # the oracle-side assembler's chain (a dependency on every vector tile, row blocks dealt round-robin), twice
        p, w_off, a_off = A.chain_matvec_program(dims, B, 8, 128, 4096, 4)
        words, sb, descs = p.finish()
        prog = ex.program_create(words, sb, descs, [W.nbytes, nA * 4, nA * 4])
        for rep in range(2):
            X2 = rng.standard_normal((B, dims[0])).astype(np.float32)
            dA.fill_(float("nan"))
            dA[:B * dims[0]] = _dev(X2.ravel())
            ex.run(prog, [_dev(W), dA, dA])
            ex.check()
            Ah = dA.cpu().numpy()
            prev = X2
            for l in range(L):
                Y = Ah[a_off[l + 1] // 4:a_off[l + 1] // 4 + B * dims[l + 1]].reshape(B, dims[l + 1])
                Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
                _check(Y, Yr, Ya, "oracle-assembled chain layer %d run %d" % (l, rep))
                prev = Y
        prog.destroy()


def test_runs_can_be_captured_in_a_hip_graph_and_replayed(ex):
    """vdc_run enqueues one kernel (the depId counters are put back to zero by the core that leaves last), so a caller may
    capture it; every replay, with eager work and synchronisations in between, must equal the eager result."""
    rows, K, B, T = 1024, 2048, 2, 8192
    rng = np.random.default_rng(9)
    dM = _dev(rng.standard_normal((rows, K)).astype(np.float32))
    dY = torch.full((B, rows), float("nan"), device="cuda")
    dY2 = torch.full((B, 64), float("nan"), device="cuda")              # a second, split-K run in the same graph (uses depIds)
    dM2 = _dev(rng.standard_normal((64, 16384)).astype(np.float32))
    dX2 = _dev(rng.standard_normal((B, 16384)).astype(np.float32))
    xs = [_dev(rng.standard_normal((B, K)).astype(np.float32)) for _ in range(3)]
    dX = xs[0].clone()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ex.matvec(dM, dX, dY, T, stream=s)                              # builds and caches the programs outside the capture
        ex.matvec(dM2, dX2, dY2, 16384, stream=s)
        ex.check(s)
        eager2 = dY2.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            ex.matvec(dM, dX, dY, T, stream=s)
            ex.matvec(dM2, dX2, dY2, 16384, stream=s)
    torch.cuda.synchronize()
    for x in xs:
        dX.copy_(x)
        dY.fill_(float("nan")); dY2.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ex.check()
        want = torch.empty_like(dY)
        ex.matvec(dM, x, want, T)                                       # eager, between the replays
        ex.check()
        assert torch.equal(dY, want)
        assert torch.equal(dY2, eager2)


def test_attention_and_stream_runs_replay_from_a_hip_graph(ex):
    """The depId counters are put back to zero at the end of every run, so a captured attention run can be replayed; every
    replay is checked against the eager result, with eager work in between."""
    Q, K, V, ro = _attn_inputs([300, 40, 700], seed=3)
    dQ, dK, dV = _dev(Q), _dev(K), _dev(V)
    dO = torch.zeros((3, 128), device="cuda")
    src = torch.randint(0, 256, (1 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    ex.attn_decode(dQ, dK, dV, ro, dO, 8192)            # builds and caches the programs outside the capture
    ex.stream("copy", src, dst, 1 << 20, 8192)
    ex.check()
    eager = dO.clone()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            ex.attn_decode(dQ, dK, dV, ro, dO, 8192, stream=s)
            ex.stream("copy", src, dst, 1 << 20, 8192, stream=s)
    torch.cuda.current_stream().wait_stream(s)
    for i in range(3):
        dO.fill_(float("nan"))
        dst.zero_()
        src.add_(1)                                      # eager work between the replays; the copy must see the new bytes
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ex.check()
        assert torch.equal(dO, eager) and torch.equal(dst, src)


def test_ragged_batch(ex):
    rng = np.random.default_rng(4)
    K = 128
    row_off = np.array([0, 700, 700, 716, 5000, 5001, 9000, 20000], dtype=np.int64)
    M = rng.standard_normal((20000, K)).astype(np.float32)
    X = rng.standard_normal((7, K)).astype(np.float32)
    dY = torch.full((20000,), float("nan"), device="cuda")
    ex.matvec_ragged(_dev(M), row_off, _dev(X), dY, 8192)
    ex.check()
    Yr, Ya = gemv_ref.gemv_ragged(M, row_off, X)
    _check(dY.cpu().numpy(), Yr, Ya, "ragged")


def test_matvec_over_several_row_blocks_traces_and_ragged_result():
    """K fits one tile and there are many row blocks per compute core: the tiler's MATVECs cover several row blocks.  On a
    small executor the traces of every unit are bit-exact against the interpreter running the same graph (dense, three
    vectors, a row tail); on the full executor a ragged batch with empty, tiny and long segments matches the fp64 GEMV, with
    one and with two store units."""
    rng = np.random.default_rng(11)
    rows, K, B, T = 3001, 64, 3, 4096
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    with vdc.Executor(n_cores=6, slot_bytes=4096) as ex:
        nc, ns = ex.cfg.n_cores, ex.cfg.n_slots
        words, sb, descs = ex.matvec_program(rows, K, K, B, T)
        spans = {(int(x[3]) >> 16) & 0xFF for x in words[(words[:, 0] & 0xFF) == A.MATVEC]}
        assert max(spans) >= 2
        prog = ex.program_create(words, sb, descs, [M.nbytes, X.nbytes, B * rows * 4])
        dY = torch.full((B, rows), float("nan"), device="cuda")
        cap = 4096
        trace, count = ex.run(prog, [_dev(M), _dev(X), dY], trace_cap=cap)
        ex.check()
        trace, count = trace.cpu().numpy().view(np.uint32), count.cpu().numpy()
    Yo = np.full((B, rows), np.nan, np.float32)
    m = UM.Machine(words, sb, descs, [M, X, Yo], n_cores=nc, slot_bytes=4096, n_slots=ns).run()
    for core in range(nc):
        s = core * 3
        exp = [(pc, op | (d << 8) | (n << 16), off & 0xFFFFFFFF, off >> 32) for (pc, op, d, off, n) in m.trace_vmc[core]]
        assert count[s] == len(exp) <= cap
        assert [tuple(int(x) for x in r) for r in trace[s, :len(exp)]] == exp
        for v in range(2):
            exp = [(pc, op | (n << 16), imm & 0xFFFFFFFF, imm >> 32) for (pc, op, n, imm) in m.trace_vcc[core][v]]
            assert count[s + 1 + v] == len(exp)
            assert [tuple(int(x) for x in r) for r in trace[s + 1 + v, :len(exp)]] == exp
    Yr, Ya = gemv_ref.gemv_dense(M, X)
    _check(dY.cpu().numpy(), Yr, Ya, "several row blocks per uop")
    _check(Yo, Yr, Ya, "several row blocks per uop (interpreter)")
    K = 128
    lengths = [0, 5, 70000, 16, 1, 33000, 17, 0, 250, 9000]
    row_off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = int(row_off[-1])
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((len(lengths), K)).astype(np.float32)
    Yr, Ya = gemv_ref.gemv_ragged(M, row_off, X)
    dM, dX = _dev(M), _dev(X)
    for n_stu in (1, 2):
        with vdc.Executor(n_stu=n_stu) as ex:
            words, _, _ = ex.matvec_program(rows, K, K, 1, 8192, row_off=row_off)
            assert max((int(x[3]) >> 16) & 0xFF for x in words[(words[:, 0] & 0xFF) == A.MATVEC]) >= 2
            dY = torch.full((rows,), float("nan"), device="cuda")
            ex.matvec_ragged(dM, row_off, dX, dY, 8192)
            ex.check()
            _check(dY.cpu().numpy(), Yr, Ya, "ragged, several row blocks per uop, %d store unit(s)" % n_stu)


def test_dep_id_chain_between_two_memory_cores():
    """y = M2 (M1 x): core 0 stores t = M1 x and signals depId 5; core 1 waits for it with load.dep."""
    rng = np.random.default_rng(12)
    M1 = rng.standard_normal((64, 64)).astype(np.float32)
    M2 = rng.standard_normal((64, 64)).astype(np.float32)
    x = rng.standard_normal((1, 64)).astype(np.float32)
    p = A.Program(2, 1)
    d_m1, d_x, d_t = p.desc(0, 64, 256, 256, 256), p.desc(1, 1, 256, 256, 256), p.desc(2, 1, 256, 256, 256)
    d_m2, d_y = p.desc(3, 64, 256, 256, 256), p.desc(4, 1, 256, 256, 256)
    p.vmc(0).extend([A.word(A.LOAD, A.F_SEND, vflow=0, nslots=4, size=64, desc=d_m1),
                     A.word(A.LOAD, A.F_SEND, vflow=1, nslots=1, size=1, desc=d_x),
                     A.word(A.STORE, A.F_SEND | A.F_RECV | A.F_DEP_SEND, vflow=2, nslots=1, size=1, desc=d_t, dep_id=5)])
    p.vcc(0, 0).append(A.word(A.MATVEC, size=1, imm=A.matvec_imm(1, 64, 16)))
    p.vmc(1).extend([A.word(A.LOAD, A.F_SEND, vflow=0, nslots=4, size=64, desc=d_m2),
                     A.word(A.LOAD, A.F_SEND | A.F_DEP_RECV, vflow=1, nslots=1, size=1, desc=d_t, dep_id=5, dep_count=1),
                     A.word(A.STORE, A.F_SEND | A.F_RECV, vflow=2, nslots=1, size=1, desc=d_y)])
    p.vcc(1, 0).append(A.word(A.MATVEC, size=1, imm=A.matvec_imm(1, 64, 16)))
    words, sb, descs = p.finish()
    with vdc.Executor(n_cores=2, vcc_per_core=1, slot_bytes=4096, n_slots=20) as ex:
        prog = ex.program_create(words, sb, descs, [M1.nbytes, x.nbytes, 256, M2.nbytes, 256])
        for _ in range(5):
            dt = torch.full((1, 64), float("nan"), device="cuda")
            dy = torch.full((1, 64), float("nan"), device="cuda")
            ex.run(prog, [_dev(M1), _dev(x), dt, _dev(M2), dy])
            ex.check()
            t = dt.cpu().numpy()
            tr, ta = gemv_ref.gemv_dense(M1, x)
            _check(t, tr, ta, "t")
            yr, ya = gemv_ref.gemv_dense(M2, t)          # from the t the device actually produced
            _check(dy.cpu().numpy(), yr, ya, "y")


def test_watchdog_reports_deadlock_and_the_grid_drains():
    """A spin limit of two polls, far below the latency of a tile load: some unit gives up, every wave leaves its loop, the
    kernel ends normally and the error comes back through the status word; the device stays usable."""
    rng = np.random.default_rng(7)
    M = rng.standard_normal((4096, 4096)).astype(np.float32)
    X = rng.standard_normal((1, 4096)).astype(np.float32)
    dM, dX = _dev(M), _dev(X)
    dY = torch.zeros((1, 4096), device="cuda")
    with vdc.Executor(watchdog_spins=2) as ex:
        ex.matvec(dM, dX, dY, 8192)
        rc, info = ex.sync_status()
        assert rc == vdc.VDC_EDEADLOCK, (rc, info)
        rc, info = ex.sync_status()              # the status was cleared
        assert rc == vdc.VDC_OK
    with vdc.Executor() as ex:
        ex.matvec(dM, dX, dY, 8192)
        ex.check()
        Yr, Ya = gemv_ref.gemv_dense(M, X)
        _check(dY.cpu().numpy(), Yr, Ya, "after watchdog")


def test_invalid_arguments_are_refused(ex):
    dM = torch.zeros((64, 64), device="cuda")
    dX = torch.zeros((1, 64), device="cuda")
    dY = torch.zeros((1, 64), device="cuda")
    L = vdc.lib()
    s = 0
    assert L.vdc_matvec(ex.handle, dM.data_ptr(), 64, 64, 64, dX.data_ptr(), dY.data_ptr(), 1, 5000, s) == vdc.VDC_EINVAL
    assert L.vdc_matvec(ex.handle, dM.data_ptr(), 64, 62, 64, dX.data_ptr(), dY.data_ptr(), 1, 4096, s) == vdc.VDC_EINVAL
    assert L.vdc_matvec(ex.handle, dM.data_ptr() + 4, 64, 60, 64, dX.data_ptr(), dY.data_ptr(), 1, 4096, s) == vdc.VDC_EINVAL
    assert L.vdc_matvec(ex.handle, dM.data_ptr(), 64, 64, 64, dX.data_ptr(), dY.data_ptr(), 9, 4096, s) == vdc.VDC_EINVAL
    assert L.vdc_matvec(ex.handle, None, 64, 64, 64, dX.data_ptr(), dY.data_ptr(), 1, 4096, s) == vdc.VDC_EINVAL
    assert L.vdc_matvec(ex.handle, dM.data_ptr(), 0, 64, 64, dX.data_ptr(), dY.data_ptr(), 1, 4096, s) == vdc.VDC_EINVAL
