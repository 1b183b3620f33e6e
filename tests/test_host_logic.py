"""CPU tests of the library's host side: the C ABI loads and exports every declared symbol, the matvec tiler's
uop graphs run to the right result on the oracle interpreter, and the validator accepts / rejects what it should.
No compute call needs a GPU here: the executor is created host-only (device = -1)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_03190_amd as vdc
import workloads
from oracle import gemv_ref, rope_ref, uop_asm as A, uop_machine as UM

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vdcores.h")).read()
    declared = set(re.findall(r"\b(vdc_[a-z_]+)\s*\(", header))
    declared -= {"vdc_config"}
    assert declared == set(vdc.EXPORTS), declared ^ set(vdc.EXPORTS)
    L = ctypes.CDLL(vdc.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


def test_strerror_and_defaults_are_the_paper_deployment():
    assert vdc.strerror(0) == "ok" and "watchdog" in vdc.strerror(vdc.VDC_EDEADLOCK)
    with vdc.Executor(device=-1) as ex:
        c = ex.cfg
        # the values the paper prints (tests/golden/deployment_constants.txt): 1 VMC + 2 VCCs per CU, 8 KB slots,
        # 128 threads per execution unit, a 32-bit mask
        g = {}
        for line in open(os.path.join(ROOT, "tests", "golden", "deployment_constants.txt")):
            line = line.split("#")[0].split()
            if len(line) == 2:
                g[line[0]] = int(line[1])
        assert (c.vcc_per_core, c.slot_bytes, c.threads_per_eu) == (g["vcc_per_core"], g["slot_bytes"], g["threads_per_eu"]) == (2, 8192, 128)
        assert c.n_slots <= g["mask_bits"]
        assert 1 <= c.n_slots <= 32 and c.n_slots * c.slot_bytes <= 160 * 1024
        assert c.n_cores == 256 and c.n_ldu == 4 and c.n_stu == 1


def test_bad_configs_are_rejected():
    for bad in (dict(slot_bytes=3000), dict(n_slots=33), dict(vcc_per_core=3), dict(threads_per_eu=64),
                dict(n_ldu=3), dict(slot_bytes=16384, n_slots=11)):
        with pytest.raises(vdc.VdcError) as e:
            vdc.Executor(device=-1, **bad)
        assert e.value.code == vdc.VDC_EINVAL


CASES = [
    # rows, K, ld, B, tile_bytes, n_cores, slot_bytes, n_slots
    (128, 128, 128, 1, 4096, 4, 4096, 12),      # cfg1 shape on four cores
    (100, 200, 212, 3, 4096, 3, 4096, 12),      # row tail, K tail, leading dimension
    (37, 1000, 1000, 8, 2048, 2, 2048, 16),
    (300, 64, 64, 2, 4096, 5, 4096, 8),
    (64, 2048, 2048, 1, 16384, 2, 8192, 10),
    (5, 12, 12, 1, 2048, 4, 1024, 8),           # fewer row blocks than compute cores
    # few row blocks, long rows: K is cut as finely as the builder offers (the adaptive step is taken out: on problems this
    # small its cost model would leave K whole) and the partial sums are chained through depId signals
    (32, 4096, 4096, 1, 4096, 8, 4096, 12),
    (16, 8192, 8200, 3, 8192, 8, 8192, 10),     # one row block
    (38, 2000, 2000, 2, 4096, 6, 4096, 12),     # row tail and K tail in a split program
]


@pytest.mark.parametrize("rows,K,ld,B,T,ncores,slot,nslots", CASES)
def test_tiler_program_on_the_oracle_interpreter(rows, K, ld, B, T, ncores, slot, nslots):
    rng = np.random.default_rng(rows * 7 + K)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    Y = np.full((B, rows), np.nan, np.float32)
    cut = rows <= 38 and K >= 2000
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots, sched_force_parts=16 if cut else 1) as ex:
        w, sb, d = ex.matvec_program(rows, K, ld, B, T)
        ws0 = ex.matvec_workspace(rows, K, ld, B, T)
        sizes = [((rows - 1) * ld + K) * 4, X.nbytes, Y.nbytes] + ([ws0.nbytes] if ws0.size else [])
        rc, msg = ex.program_validate(w, sb, d, sizes)
        assert rc == vdc.VDC_OK, msg
    split = ws0.size > 0
    assert split == cut
    if split:
        ops = np.asarray(w)[:, 0] & 0xFF
        flags = (np.asarray(w)[:, 0] >> 8) & 0xFF
        assert ((ops == 8) & ((flags & 32) != 0)).any() and ((ops == 9) & ((flags & 16) != 0)).any()   # load.dep and signalling stores
    for sched, seed in (("program", 0), ("random", 1)):
        Y[:] = np.nan
        ws = ws0.copy()
        UM.Machine(w, sb, d, [M, X, Y] + ([ws] if split else []), n_cores=ncores, slot_bytes=slot, n_slots=nslots).run(sched, seed)
        Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
        # partial sums pass through fp32 once per K range
        assert np.all(np.abs(Y - Yr) <= (2e-6 if split else 1e-7) * Ya + 1e-30)


@pytest.mark.parametrize("rows,K,ld,B,T,ncores,slot,nslots", [
    (128, 128, 128, 1, 4096, 4, 4096, 12),
    (100, 200, 212, 3, 4096, 3, 4096, 12),      # row tail (a multiple of 4), K tail, leading dimension
    (640, 64, 64, 2, 4096, 2, 4096, 10),        # many row blocks per compute core: the looped form
    (64, 1024, 1024, 8, 16384, 2, 8192, 10),
])
def test_fused_matvec_rope_program_on_the_oracle_interpreter(rows, K, ld, B, T, ncores, slot, nslots):
    rng = np.random.default_rng(rows + 3 * K)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    Tt = rope_ref.table(rng.uniform(-3.0, 3.0, (B, rows // 2)))
    Y = np.full((B, rows), np.nan, np.float32)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots) as ex:
        w, sb, d = ex.matvec_rope_program(rows, K, ld, B, T)
        rc, msg = ex.program_validate(w, sb, d, [((rows - 1) * ld + K) * 4, X.nbytes, Y.nbytes, Tt.nbytes])
        assert rc == vdc.VDC_OK, msg
        with pytest.raises(vdc.VdcError):
            ex.matvec_rope_program(rows + 2, K, ld, B, T)          # rows must be a multiple of 4
    ops, flags = w[:, 0] & 0xFF, (w[:, 0] >> 8) & 0xFF
    assert (ops == A.ROPE).any() and ((ops == A.STORE) & ((flags & A.F_LOCAL) != 0)).any() and ((ops == A.LOAD) & ((flags & A.F_LOCAL) != 0)).any()
    O, Oa = gemv_ref.gemv_dense(M, X, ld=ld)
    Rr, Ra = rope_ref.rope(O, Tt)
    for sched, seed in (("program", 0), ("random", 1)):
        Y[:] = np.nan
        m = UM.Machine(w, sb, d, [M, X, Y, Tt], n_cores=ncores, slot_bytes=slot, n_slots=nslots)
        m.run(sched, seed)
        m.check_final()
        assert np.all(np.abs(Y - Rr) <= 1e-6 * (Ra + Oa) + 1e-30)


def test_two_store_units_per_core():
    """With two store units each receives the return queue of one compute core: the tilers' programs (plain and fused)
    run to the same result on the interpreter under random schedules, and a STORE moved to the other unit is refused
    by the validator and by the interpreter."""
    rng = np.random.default_rng(77)
    rows, K, B, T = 200, 300, 3, 4096
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    Tt = rope_ref.table(rng.uniform(-3.0, 3.0, (B, rows // 2)))
    O, Oa = gemv_ref.gemv_dense(M, X)
    Rr, Ra = rope_ref.rope(O, Tt)
    kw = dict(n_cores=3, slot_bytes=4096, n_slots=12)
    with vdc.Executor(device=-1, n_stu=2, **kw) as ex:
        assert ex.cfg.n_stu == 2
        w, sb, d = ex.matvec_program(rows, K, K, B, T)
        assert ex.program_validate(w, sb, d, [M.nbytes, X.nbytes, O.size * 4])[0] == vdc.VDC_OK
        wr, sbr, dr = ex.matvec_rope_program(rows, K, K, B, T)
        assert ex.program_validate(wr, sbr, dr, [M.nbytes, X.nbytes, O.size * 4, Tt.nbytes])[0] == vdc.VDC_OK
        # the first STORE of compute core 1 on the flow of compute core 0's store unit
        bad = np.array(w, copy=True)
        ops, vcc = bad[:, 0] & 0xFF, (bad[:, 0] >> 20) & 3
        i = int(np.flatnonzero((ops == A.STORE) & (vcc == 1))[0])
        bad[i, 0] ^= 1 << 16
        rc, msg = ex.program_validate(bad, sb, d, [M.nbytes, X.nbytes, O.size * 4])
        assert rc == vdc.VDC_EPROGRAM and "store unit" in msg
    for seed in range(3):
        Y = np.full((B, rows), np.nan, np.float32)
        m = UM.Machine(w, sb, d, [M, X, Y], n_stu=2, **kw)
        m.run("random", seed)
        m.check_final()
        assert np.all(np.abs(Y - O) <= 1e-7 * Oa + 1e-30)
        Y[:] = np.nan
        m = UM.Machine(wr, sbr, dr, [M, X, Y, Tt], n_stu=2, **kw)
        m.run("random", seed)
        m.check_final()
        assert np.all(np.abs(Y - Rr) <= 1e-6 * (Ra + Oa) + 1e-30)
    with pytest.raises(UM.ProgramError):
        UM.Machine(bad, sb, d, [M, X, np.zeros((B, rows), np.float32)], n_stu=2, **kw).run()
    with pytest.raises(vdc.VdcError):
        vdc.Executor(device=-1, n_stu=3)
    with pytest.raises(vdc.VdcError):
        vdc.Executor(device=-1, n_stu=2, vcc_per_core=1)


def test_ragged_tiler_program_on_the_oracle_interpreter():
    rng = np.random.default_rng(5)
    K = 64
    row_off = np.array([0, 5, 5, 40, 41, 100, 260, 277], dtype=np.int64)
    M = rng.standard_normal((277, K)).astype(np.float32)
    X = rng.standard_normal((7, K)).astype(np.float32)
    Y = np.full(277, np.nan, np.float32)
    with vdc.Executor(device=-1, n_cores=4, slot_bytes=4096, n_slots=12) as ex:
        w, sb, d = ex.matvec_program(277, K, K, 1, 4096, row_off=row_off)
        rc, msg = ex.program_validate(w, sb, d, [M.nbytes, X.nbytes, Y.nbytes])
        assert rc == vdc.VDC_OK, msg
    UM.Machine(w, sb, d, [M, X, Y], n_cores=4, slot_bytes=4096, n_slots=12).run("random", 2)
    Yr, Ya = gemv_ref.gemv_ragged(M, row_off, X)
    assert np.all(np.abs(Y - Yr) <= 1e-7 * Ya + 1e-30)


def test_zipf_ragged_program_balances_bytes_over_cores():
    # the config-4 recipe on 16 cores: every core gets the same number of row blocks, within one
    row_off = workloads.zipf_segments(1 << 14, 64, 1.1, 3)
    with vdc.Executor(device=-1, n_cores=16, slot_bytes=8192, n_slots=19) as ex:
        w, sb, d = ex.matvec_program(1 << 14, 128, 128, 1, 8192, row_off=row_off)
        rc, msg = ex.program_validate(w, sb, d, [(1 << 14) * 512, 64 * 512, (1 << 14) * 4])
        assert rc == vdc.VDC_OK, msg
    M = np.zeros((1 << 14, 128), np.float32)
    X = np.zeros((64, 128), np.float32)
    Y = np.zeros(1 << 14, np.float32)
    m = UM.Machine(w, sb, d, [M, X, Y], n_cores=16, slot_bytes=8192, n_slots=19).run()
    loads = [sum(1 for r in t if r[1] == UM.LOAD and r[2] == 0 or r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
             for t in m.trace_vmc]
    assert max(loads) - min(loads) <= 1


def test_validator_rejects_broken_programs():
    with vdc.Executor(device=-1, n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=4) as ex:
        M, X, Y = 16 * 64 * 4, 64 * 4, 16 * 4

        def check(mutate, expect_ok=False):
            p = A.dense_matvec_program(16, 64, 64, 1, 16, 32, 1024, 1, vcc_per_core=1)
            mutate(p)
            w, sb, d = p.finish()
            rc, msg = ex.program_validate(w, sb, d, [M, X, Y])
            assert (rc == vdc.VDC_OK) == expect_ok, msg
            return msg

        check(lambda p: None, expect_ok=True)
        # address beyond the tensor
        def far(p):
            u = UM.decode(p.vmc(0)[0])
            p.vmc(0)[0] = A.word(A.LOAD, u.flags, vflow=u.vflow, vcc=u.vcc, nslots=u.nslots, size=u.size, imm=M - 64, desc=u.desc)
        assert "beyond" in check(far)
        # a send removed: the compute core starves
        def nosend(p):
            u = UM.decode(p.vmc(0)[1])
            p.vmc(0)[1] = A.word(A.LOAD, 0, vflow=u.vflow, vcc=u.vcc, nslots=u.nslots, size=u.size, imm=u.imm, desc=u.desc)
        check(nosend)
        # wrong slot count
        def slots(p):
            u = UM.decode(p.vmc(0)[0])
            p.vmc(0)[0] = A.word(A.LOAD, u.flags, vflow=u.vflow, vcc=u.vcc, nslots=3, size=u.size, imm=u.imm, desc=u.desc)
        assert "nslots" in check(slots)
        # matvec geometry that no handler exists for (7 chunks per row)
        def geom(p):
            p.vcc(0, 0)[0] = A.word(A.MATVEC, size=2, imm=A.matvec_imm(1, 16, 7))
        check(geom)
        # continue_if outside a loop, and one whose distance does not end on its loop's REPEAT
        assert "CONTINUE_IF" in check(lambda p: p.vmc(0).insert(0, A.word(A.CONTINUE_IF, acc=0, imm=1, size=1)))
        assert "CONTINUE_IF" in check(lambda p: [p.vmc(0).insert(0, w_) for w_ in reversed(
            [A.word(A.LOOP, imm=2), A.word(A.CONTINUE_IF, acc=0, imm=1, size=2), A.word(A.ADD), A.word(A.ADD), A.word(A.REPEAT)])])
        # and a well-formed one is accepted
        check(lambda p: [p.vmc(0).insert(0, w_) for w_ in reversed(
            [A.word(A.LOOP, imm=2), A.word(A.CONTINUE_IF, acc=0, imm=1, size=2), A.word(A.ADD), A.word(A.REPEAT)])], expect_ok=True)
        # REPEAT without LOOP, memory opcode on a compute core
        check(lambda p: p.vmc(0).insert(0, A.word(A.REPEAT)))
        check(lambda p: p.vcc(0, 0).insert(0, A.word(A.LOAD)))
    # over-committed slots: the matrix tile takes the whole pool (the deadlock case of Section 4.3)
    with vdc.Executor(device=-1, n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=2) as ex:
        p = A.dense_matvec_program(8, 64, 64, 1, 8, 64, 1024, 1, vcc_per_core=1)      # matrix tile = 2 KB = both slots
        w, sb, d = p.finish()
        rc, msg = ex.program_validate(w, sb, d, [8 * 64 * 4, 64 * 4, 32])
        assert rc == vdc.VDC_EPROGRAM and "deadlock" in msg


def test_validator_bounds_arithmetic_cannot_wrap():
    """A row pitch or an accumulator chosen so that 64-bit arithmetic wraps must not slip a box past the tensor's end."""
    with vdc.Executor(device=-1, n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=4) as ex:
        M, X, Y = 16 * 64 * 4, 64 * 4, 16 * 4

        def check(mutate):
            p = A.dense_matvec_program(16, 64, 64, 1, 16, 32, 1024, 1, vcc_per_core=1)
            mutate(p)
            w, sb, d = p.finish()
            rc, msg = ex.program_validate(w, sb, d, [M, X, Y])
            return rc, msg

        assert check(lambda p: None)[0] == vdc.VDC_OK
        # a pitch of 2^63 bytes: (rows - 1) * pitch is 0 modulo 2^64 for an odd number of further rows pairs
        for pitch in (1 << 63, (1 << 63) + 16, (1 << 62), (1 << 64) - 16):
            def huge_pitch(p, pitch=pitch):
                u = UM.decode(p.vmc(0)[0])
                t, box_rows, row_bytes, lds_pitch = p.descs[u.desc][:4]
                p.descs[u.desc] = (t, box_rows, row_bytes, lds_pitch, pitch & 0xFFFFFFFF, pitch >> 32, 0, 0)
            rc, msg = check(huge_pitch)
            assert rc == vdc.VDC_EPROGRAM and "beyond" in msg, (hex(pitch), msg)
        # an accumulator driven past 2^63 by repeated additions of the largest immediate
        def acc_overflow(p):
            big = (1 << 47) - 16
            pre = [A.word(A.LOOP, imm=70000), A.word(A.LOOP, imm=1000)] + [A.word(A.ADD, acc=1, imm=big)] + [A.word(A.REPEAT, acc=1, imm=big), A.word(A.REPEAT, acc=1, imm=big)]
            for i, w_ in enumerate(pre):
                p.vmc(0).insert(i, w_)
        rc, msg = check(acc_overflow)
        assert rc == vdc.VDC_EPROGRAM and "overflow" in msg, msg


def test_device_entry_points_refuse_a_host_only_executor():
    with vdc.Executor(device=-1, n_cores=2) as ex:
        w, sb, d = ex.matvec_program(64, 64, 64, 1, 4096)
        with pytest.raises(vdc.VdcError) as e:
            ex.program_create(w, sb, d, [64 * 64 * 4, 256, 256])
        assert e.value.code == vdc.VDC_EINVAL


# ---- memory uops with nothing to compute behind them (Section 6.3, "Memory virtual core overhead") ----
@pytest.mark.parametrize("mode,nbytes,T,ncores,slot,nslots", [
    ("copy", 64 * 1024, 4096, 2, 4096, 8),                 # whole blocks, looped
    ("copy", 37 * 4096 + 3 * 1024 + 48, 4096, 3, 4096, 6),  # uneven runs, a short block and a short row
    ("copy", 48, 1024, 2, 1024, 4),                        # less than one row
    ("copy", 5 * 256, 256, 1, 1024, 4),                    # tiles below a row of 1 KB
    ("fill", 21 * 8192 + 1024 + 16, 8192, 2, 8192, 5),
    ("read", 33 * 2048 + 2048 - 16, 2048, 2, 2048, 4),
])
def test_stream_program_on_the_oracle_interpreter(mode, nbytes, T, ncores, slot, nslots):
    rng = np.random.default_rng(nbytes)
    src = rng.integers(0, 256, nbytes + 32, dtype=np.uint8)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots) as ex:
        w, sb, d = ex.stream_program(mode, nbytes, T, value=0x01020304)
        rc, msg = ex.program_validate(w, sb, d, [nbytes, nbytes] if mode == "copy" else [nbytes])
        assert rc == vdc.VDC_OK, msg
    ops = w[:, 0] & 0xFF
    assert (ops == {"read": A.DROP, "fill": A.FILL, "copy": A.COPY}[mode]).any()
    for sched, seed in (("program", 0), ("random", 1)):
        dst = np.full(nbytes + 32, 0xEE, np.uint8)
        keep = src.copy()
        tensors = {"read": [src], "fill": [dst], "copy": [src, dst]}[mode]
        m = UM.Machine(w, sb, d, tensors, n_cores=ncores, slot_bytes=slot, n_slots=nslots)
        m.run(sched, seed)
        m.check_final()
        assert np.array_equal(src, keep)
        if mode == "copy":
            assert np.array_equal(dst[:nbytes], src[:nbytes])
        if mode == "fill":
            assert np.all(dst[:nbytes].view(np.uint32) == 0x01020304)
        assert np.all(dst[nbytes:] == 0xEE)
        # every byte of the range is moved exactly once
        for op in ([A.LOAD] if mode != "fill" else []) + ([A.STORE] if mode != "read" else []):
            seen = np.zeros(nbytes, np.uint8)
            for core in m.trace_vmc:
                for (_pc, o, di, off, rows) in core:
                    if o == op:
                        seen[off:off + rows * int(d[di][2])] += 1
            assert np.all(seen == 1)


def test_stream_program_rejects_bad_arguments():
    with vdc.Executor(device=-1, n_cores=2, slot_bytes=4096, n_slots=4) as ex:
        for bad in (dict(nbytes=0), dict(nbytes=40), dict(T=3000), dict(T=128), dict(T=65536)):
            a = dict(nbytes=4096, T=4096)
            a.update(bad)
            with pytest.raises(vdc.VdcError):
                ex.stream_program("copy", a["nbytes"], a["T"])
        with pytest.raises(vdc.VdcError):
            ex.stream_program("copy", 1 << 20, 16384)      # an input and an output region of 16 KB need eight slots
        ex.stream_program("read", 1 << 20, 16384)


# ---- decode attention over ragged contexts (Section 6.2, "Dynamic Attention Length") -----------------
@pytest.mark.parametrize("lengths,T,ncores,slot,nslots,d", [
    ([1], 4096, 1, 4096, 8, 128),
    ([40, 7, 300, 9, 64], 4096, 2, 4096, 10, 128),     # one long request shared by the compute cores, short ones whole
    ([600], 8192, 4, 8192, 8, 128),                    # a single request on eight compute cores
    ([33] * 9, 16384, 2, 8192, 10, 128),               # more requests than compute cores; a tile holds most of a context
    ([70, 5, 400], 4096, 2, 4096, 10, 64),             # head dimension 64
    ([129], 16384, 3, 8192, 8, 64),
])
def test_attention_program_on_the_oracle_interpreter(lengths, T, ncores, slot, nslots, d):
    from oracle import attn_ref
    rng = np.random.default_rng(sum(lengths))
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    Q = rng.standard_normal((len(lengths), d)).astype(np.float32)
    K = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
    V = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots) as ex:
        w, sb, ds, n_items = ex.attn_decode_program(ro, d, T)
        rc, msg = ex.program_validate(w, sb, ds, [K.nbytes, V.nbytes, Q.nbytes, Q.nbytes, n_items * (d + 4) * 4])
        assert rc == vdc.VDC_OK, msg
        for bad in (dict(d=32), dict(T=2048), dict(ro=np.array([0, 5, 5]))):
            a = dict(ro=ro, d=d, T=T)
            a.update(bad)
            with pytest.raises(vdc.VdcError):
                ex.attn_decode_program(a["ro"], a["d"], a["T"])
    ops, flags = w[:, 0] & 0xFF, (w[:, 0] >> 8) & 0xFF
    # every context has one item that writes the result itself: a context inside one compute core's share is that item
    # alone; a context that is cut has one partial row per other item, which the first item joins (no ATTN_MERGE)
    partial = int(((ops == A.STORE) & ((flags & A.F_DEP_SEND) != 0)).sum())
    assert n_items == max(partial, 1) and (ops == A.ATTN_MERGE).sum() == 0
    assert (ops == A.ATTN).sum() == partial + len(lengths)
    joined = int(sum(int((x >> 16) & 0xFF) for x, o in zip(w[:, 3], ops) if o == A.ATTN))      # the descriptor field of the attn uops
    assert joined == partial
    Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, d ** -0.5)
    for sched, seed in (("program", 0), ("random", 1)):
        O = np.full((len(lengths), d), np.nan, np.float32)
        W = np.full((n_items, d + 4), np.nan, np.float32)
        m = UM.Machine(w, sb, ds, [K, V, Q, O, W], n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=1024)
        m.run(sched, seed)
        m.check_final()
        assert np.all(np.abs(O - Or) <= 4e-7 * Ar + 1e-30)


def test_attention_items_balance_over_the_compute_cores():
    # the uneven regime: 64 requests of 256..1024 rows on 16 cores; and one long request alone
    rng = np.random.default_rng(3)
    for lengths in (rng.integers(256, 1025, 64), np.array([65536])):
        ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
        with vdc.Executor(device=-1, n_cores=16) as ex:
            w, sb, ds, n_items = ex.attn_decode_program(ro, 128, 16384)
        ops, size = w[:, 0] & 0xFF, w[:, 1] & 0xFFFF
        per_vcc = []
        for c in range(16):
            for v in range(2):
                a, b = sb[c * 3 + 1 + v], sb[c * 3 + 2 + v]
                per_vcc.append(int(size[a:b][ops[a:b] == A.ATTN].sum()))
        total = sum(-(-int(L) // 32) for L in lengths)
        assert sum(per_vcc) == total
        assert max(per_vcc) <= total / 32 + max(1, -(-total // 128)) + 1


# ---- a chain of matvec operators in one uop graph (Section 3; Section 4.1, depId dependencies) ---------
@pytest.mark.parametrize("dims,B,T,ncores,slot,nslots", [
    ((256, 256), 1, 4096, 2, 4096, 8),                      # one layer: nothing waits
    ((128, 256, 64, 192), 2, 4096, 2, 4096, 10),            # three layers, more than one row block per compute core
    ((200, 100, 36), 1, 4096, 3, 4096, 8),                  # K tails and row tails in a chain
    ((512, 128, 128, 128, 128), 3, 8192, 4, 8192, 8),       # fewer row blocks than compute cores from layer 0 on
])
def test_chain_program_on_the_oracle_interpreter(dims, B, T, ncores, slot, nslots):
    rng = np.random.default_rng(sum(dims))
    L = len(dims) - 1
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L)]
    X = rng.standard_normal((B, dims[0])).astype(np.float32)
    W = np.concatenate([m.ravel() for m in Ms])
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots) as ex:
        w, sb, d = ex.matvec_chain_program(dims, B, T)
        a_bytes = 4 * B * sum(dims)
        rc, msg = ex.program_validate(w, sb, d, [W.nbytes, a_bytes, a_bytes])
        assert rc == vdc.VDC_OK, msg
    ops, flags = w[:, 0] & 0xFF, (w[:, 0] >> 8) & 0xFF
    if L > 1:
        assert ((ops == A.LOAD) & ((flags & A.F_DEP_RECV) != 0)).any() and ((ops == A.STORE) & ((flags & A.F_DEP_SEND) != 0)).any()
    else:
        assert not (flags & (A.F_DEP_RECV | A.F_DEP_SEND)).any()
    a_off = np.concatenate([[0], np.cumsum([B * x for x in dims])])
    ref = None
    for sched, seed in (("program", 0), ("random", 1), ("random", 2)):
        Abuf = np.full(B * sum(dims), np.nan, np.float32)      # a tile read before it is written poisons the result
        Abuf[:B * dims[0]] = X.ravel()
        m = UM.Machine(w, sb, d, [W, Abuf, Abuf], n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=1024)
        m.run(sched, seed)
        m.check_final()
        assert not np.isnan(Abuf).any()
        prev = X
        for l in range(L):
            Y = Abuf[a_off[l + 1]:a_off[l + 2]].reshape(B, dims[l + 1])
            Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
            assert np.all(np.abs(Y - Yr) <= 1e-7 * Ya + 1e-30), (sched, l)
            prev = Y
        ref = ref if ref is not None else Abuf.tobytes()
        assert Abuf.tobytes() == ref


def test_chain_program_rejects_what_it_cannot_chain():
    with vdc.Executor(device=-1, n_cores=2, n_dep_ids=1) as ex:
        with pytest.raises(vdc.VdcError):
            ex.matvec_chain_program((4096, 4096, 4096), 1, 16384)      # two groups of vector tiles in layer 1, one depId
        with pytest.raises(vdc.VdcError):
            ex.matvec_chain_program((4096, 4098), 1, 16384)            # not a multiple of 4
        ex.matvec_chain_program((4096, 4096), 1, 16384)


# ---- the generator's lowering steps (Section 4.2): the library's against the oracle side's, word for word -------------
def _graph_arrays(g):
    """An oracle-side graph (oracle/uop_lower.py) in the arrays vdc_graph_lower takes: the memory uops in the order they
    were written down, the descriptor table, the edges, the compute streams."""
    from oracle import uop_lower as L
    ops_list = sorted((m for c in range(g.n_cores) for v in range(g.V) for m in g.mem[c][v]), key=lambda m: m.seq)
    index = {id(m): i for i, m in enumerate(ops_list)}
    descs, ops = [], np.zeros(len(ops_list), dtype=vdc.Executor.GRAPH_MEMOP)
    for i, m in enumerate(ops_list):
        if m.desc not in descs:
            descs.append(m.desc)
        ops[i] = (m.op, m.core, m.vcc, descs.index(m.desc), m.offset, m.rows, m.nslots, m.group, int(m.nt))
    edges = np.array([(index[id(s)], index[id(l)]) for s, l in g.edges], dtype=np.int64).reshape(-1, 2)
    comp, begin = [], [0]
    for c in range(g.n_cores):
        for v in range(g.V):
            comp.extend(g.comp[c][v])
            begin.append(len(comp))
    dtab = np.array([A.descriptor(*d) for d in descs], dtype=np.uint32)
    return ops, edges, np.array(comp, dtype=np.uint32).reshape(-1, 4), np.array(begin, dtype=np.uint32), dtab


def test_graph_lowering_matches_the_oracle_side_word_for_word():
    """The same graphs through the library's lowering steps and through the oracle side's: identical bytecode (integer
    work: bit for bit), for the running example (placement), for a chain (flows, depIds, removed waits) and for a stream
    that over-commits the slots as written (reordering)."""
    from oracle import uop_lower as L
    # the running example of Section 3: matvec, then rope, the intermediate through a temporary tensor
    rows, K, B, R, Kt, slot, C = 96, 256, 3, 8, 64, 1024, 3
    nb = [rows * K * 4, B * K * 4, B * rows * 4, B * rows * 4, B * rows * 4]
    g = L.matvec_rope_graph(rows, K, B, R, Kt, slot, C)
    arrays = _graph_arrays(g)
    assert L.place_local(g) == rows // R
    L.assign_flows(g)
    L.embed_deps(g)
    w_ref, sb_ref, d_ref = L.assemble(g).finish()
    with vdc.Executor(device=-1, n_cores=C, slot_bytes=slot, n_slots=12) as ex:
        w, sb, d, stats = ex.graph_lower(*arrays, nb, temp_tensors=1 << 4, geom_tensor=2)
        assert list(stats) == [rows // R, 0, 0, 0, 0]
        assert np.array_equal(w, w_ref) and np.array_equal(sb, sb_ref) and np.array_equal(d, d_ref)
        # and without permission to keep tensor 4 out of memory nothing is placed: every pair needs its wait
        w2, sb2, d2, stats2 = ex.graph_lower(*arrays, nb, temp_tensors=0, geom_tensor=2)
        assert list(stats2) == [0, 0, rows // R, rows // R, 0]
    # a chain of three layers: one depId per vector tile, the waits that flow order implies removed
    dims, B, R, Kt, slot, C = (128, 192, 128, 64), 2, 8, 64, 1024, 3
    g = L.chain_graph(dims, B, R, Kt, slot, C)
    arrays = _graph_arrays(g)
    L.assign_flows(g)
    n_ids, kept, dropped = L.embed_deps(g)
    w_ref, sb_ref, d_ref = L.assemble(g).finish()
    nA = B * sum(dims) * 4
    with vdc.Executor(device=-1, n_cores=C, slot_bytes=slot, n_slots=12) as ex:
        w, sb, d, stats = ex.graph_lower(*arrays, [sum(dims[l] * dims[l + 1] for l in range(3)) * 4, nA, nA])
        assert list(stats) == [0, 0, n_ids, kept, dropped] and dropped > 0
        assert np.array_equal(w, w_ref) and np.array_equal(sb, sb_ref) and np.array_equal(d, d_ref)
    # one memory core, two compute cores, uops written down strictly alternating: two slots are over-committed
    rows, K, B, R, Kt, slot = 32, 128, 1, 8, 64, 2048
    g = L.new_graph(1, 2, slot)
    dm, dx, dy = (0, R, Kt * 4, Kt * 4, K * 4), (1, B, Kt * 4, Kt * 4, K * 4), (2, B, R * 4, R * 4, rows * 4)
    per_v = [[], []]
    for rb in range(rows // R):
        v = rb % 2
        grp = (per_v[v][-1].group + 1) if per_v[v] else 0
        for kt in range(K // Kt):
            per_v[v] += [L.MemOp(A.LOAD, 0, v, dm, (rb * R * K + kt * Kt) * 4, R, 1, grp), L.MemOp(A.LOAD, 0, v, dx, kt * Kt * 4, B, 1, grp)]
            grp += 1
        per_v[v].append(L.MemOp(A.STORE, 0, v, dy, rb * R * 4, B, 1, grp))
        g.comp[0][v].append(A.word(A.MATVEC, size=K // Kt, imm=A.matvec_imm(B, R, Kt // 4)))
    for i in range(max(len(per_v[0]), len(per_v[1]))):          # written down in the starving order
        for v in (0, 1):
            if i < len(per_v[v]):
                g.add(per_v[v][i])
    arrays = _graph_arrays(g)
    nb = [rows * K * 4, B * K * 4, B * rows * 4]
    L.assign_flows(g)
    assert L.schedule(g, nb, 2) is True
    w_ref, sb_ref, d_ref = L.assemble(g).finish()
    with vdc.Executor(device=-1, n_cores=1, slot_bytes=slot, n_slots=2) as ex:
        w, sb, d, stats = ex.graph_lower(*arrays, nb)
        assert list(stats) == [0, 1, 0, 0, 0]
        assert np.array_equal(w, w_ref) and np.array_equal(sb, sb_ref) and np.array_equal(d, d_ref)
    with vdc.Executor(device=-1, n_cores=1, slot_bytes=slot, n_slots=6) as ex:      # with room the written order stays
        assert list(ex.graph_lower(*arrays, nb)[3]) == [0, 0, 0, 0, 0]
    with vdc.Executor(device=-1, n_cores=1, slot_bytes=slot, n_slots=1) as ex:      # no order fits one slot
        with pytest.raises(vdc.VdcError) as e:
            ex.graph_lower(*arrays, nb)
        assert e.value.code == vdc.VDC_EPROGRAM


def test_fused_rope_program_comes_from_the_placement_step():
    """vdc_matvec_rope's tiler writes the two operators as they come; the placement step must have turned every
    store / load pair of the intermediate into a local pair, and nothing may name the temporary tensor any more."""
    for rows, K, B, T, C in ((1000, 1000, 1, 4096, 3), (70000, 128, 2, 8192, 4), (512, 4096, 8, 16384, 2)):
        rows -= rows % 4
        with vdc.Executor(device=-1, n_cores=C, slot_bytes=min(T, 8192)) as ex:
            w, sb, d = ex.matvec_rope_program(rows, K, K, B, T)
        ops, flags, di = w[:, 0] & 0xFF, (w[:, 0] >> 8) & 0xFF, (w[:, 3] >> 16) & 0xFF
        mem = (ops == A.LOAD) | (ops == A.STORE)
        local_st = (ops == A.STORE) & ((flags & A.F_LOCAL) != 0)
        local_ld = (ops == A.LOAD) & ((flags & A.F_LOCAL) != 0)
        assert local_st.sum() == local_ld.sum() >= 1
        assert np.all(local_ld[1:][local_st[:-1]])                                  # every store.local is followed by its load.local
        assert not np.any(d[di[mem & ((flags & A.F_LOCAL) == 0)], 0] == 4)          # no memory uop touches tensor 4
