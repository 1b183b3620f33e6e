"""The host tilers on random shapes: every program the library would run is validated, run on the oracle's interpreter
under a random legal schedule and compared with the plain definitions (fp64 GEMV, fp64 softmax attention, byte images).

Host logic only (no GPU): the library is created without a device.  Shapes are drawn by hypothesis from ranges that
cross every branch of the tilers: row and K tails, fewer row blocks than compute cores (K split), looped and unrolled
forms, ragged batches with empty segments, contexts shorter than a tile, ranges shorter than a block.
"""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

import paper_2605_03190_amd as vdc
from oracle import attn_ref, gemv_ref, uop_machine as UM

COMMON = dict(deadline=None, max_examples=60, derandomize=True, suppress_health_check=[HealthCheck.too_slow])


def _machine(w, sb, d, tensors, ncores, slot, nslots, seed):
    m = UM.Machine(w, sb, d, tensors, n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=1024)
    m.run("random", seed)
    m.check_final()
    return m


@settings(**COMMON)
@given(rows=st.integers(1, 300), k4=st.integers(1, 300), B=st.integers(1, 8), tile=st.sampled_from([2048, 4096, 8192]),
       ncores=st.integers(1, 5), pad=st.integers(0, 3), seed=st.integers(0, 1000))
def test_dense_matvec_programs(rows, k4, B, tile, ncores, pad, seed):
    K, ld = 4 * k4, 4 * (k4 + pad)
    slot, nslots = 2048, 16
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots) as ex:
        try:
            w, sb, d = ex.matvec_program(rows, K, ld, B, tile)
        except vdc.VdcError:
            return                                           # a geometry the compute uop does not have (B too large for the tile)
        ws = ex.matvec_workspace(rows, K, ld, B, tile)
        sizes = [((rows - 1) * ld + K) * 4, X.nbytes, B * rows * 4] + ([ws.nbytes] if ws.size else [])
        rc, msg = ex.program_validate(w, sb, d, sizes)
        assert rc == vdc.VDC_OK, msg
    Y = np.full((B, rows), np.nan, np.float32)
    _machine(w, sb, d, [M, X, Y] + ([ws] if ws.size else []), ncores, slot, nslots, seed)
    Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
    assert np.all(np.abs(Y - Yr) <= 2e-6 * Ya + 1e-30)


@settings(**COMMON)
@given(rows=st.integers(1, 200), nk=st.integers(2, 24), tile=st.sampled_from([2048, 4096, 8192]), ncores=st.integers(1, 4),
       n_stu=st.sampled_from([1, 2]), seed=st.integers(0, 1000))
def test_one_vector_programs_with_vector_tiles_over_several_steps(rows, nk, tile, ncores, n_stu, seed):
    """One right-hand vector and K a whole number of tiles: where the tiler lets a vector tile serve several steps
    (few row blocks per compute core, an even number of steps) the MATVEC uops say so, there are fewer vector loads than
    matrix loads, and the result is the GEMV either way; also with two store units per core."""
    slot, nslots = 2048, 16
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_stu=n_stu) as ex:
        Kt = None
        for cand in (256, 128, 64, 32, 16):
            try:
                w, sb, d = ex.matvec_program(rows, cand * nk, cand * nk, 1, tile)
            except vdc.VdcError:
                continue
            mv = w[(w[:, 0] & 0xFF) == 16]
            if ((int(mv[0, 2]) >> 24) | ((int(mv[0, 3]) & 0xFF) << 8)) * 4 == cand:      # lpr * 4 = the tile's width
                Kt = cand
                break
        assert Kt is not None
        K = Kt * nk
        ws = ex.matvec_workspace(rows, K, K, 1, tile)
        sizes = [rows * K * 4, K * 4, rows * 4] + ([ws.nbytes] if ws.size else [])
        rc, msg = ex.program_validate(w, sb, d, sizes)
        assert rc == vdc.VDC_OK, msg
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((1, K)).astype(np.float32)
    Y = np.full((1, rows), np.nan, np.float32)
    m = UM.Machine(w, sb, d, [M, X, Y] + ([ws] if ws.size else []), n_cores=ncores, slot_bytes=slot, n_slots=nslots, n_dep_ids=1024, n_stu=n_stu)
    m.run("random", seed)
    m.check_final()
    Yr, Ya = gemv_ref.gemv_dense(M, X)
    assert np.all(np.abs(Y - Yr) <= 2e-6 * Ya + 1e-30)
    xspans = {(int(x[3]) >> 8) & 0x7F for x in w[(w[:, 0] & 0xFF) == 16]}
    loads_x = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 1)
    loads_m = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
    if max(xspans) >= 2:
        assert loads_x < loads_m          # (a program may mix the forms: row blocks in a loop keep a vector tile per step)
    else:
        assert loads_x >= loads_m or ws.size


@settings(**COMMON)
@given(lengths=st.lists(st.integers(0, 90), min_size=1, max_size=9), k4=st.integers(1, 80), tile=st.sampled_from([2048, 4096]),
       ncores=st.integers(1, 4), seed=st.integers(0, 1000))
def test_ragged_matvec_programs(lengths, k4, tile, ncores, seed):
    K = 4 * k4
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = int(ro[-1])
    if rows == 0:
        return
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((len(lengths), K)).astype(np.float32)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=2048, n_slots=12) as ex:
        w, sb, d = ex.matvec_program(rows, K, K, 1, tile, row_off=ro)
        rc, msg = ex.program_validate(w, sb, d, [M.nbytes, X.nbytes, rows * 4])
        assert rc == vdc.VDC_OK, msg
    Y = np.full(rows, np.nan, np.float32)
    _machine(w, sb, d, [M, X, Y], ncores, 2048, 12, seed)
    Yr, Ya = gemv_ref.gemv_ragged(M, ro, X)
    assert np.all(np.abs(Y - Yr) <= 1e-6 * Ya + 1e-30)


@settings(**COMMON)
@given(lengths=st.lists(st.integers(1, 400), min_size=1, max_size=6), k4=st.integers(1, 32), B=st.integers(1, 4),
       tile=st.sampled_from([2048, 4096]), ncores=st.integers(1, 2), n_stu=st.sampled_from([1, 2]), seed=st.integers(0, 1000))
def test_short_k_programs_cover_several_row_blocks_per_uop(lengths, k4, B, tile, ncores, n_stu, seed):
    """K fits one tile and there are many row blocks per compute core: the tiler lets a MATVEC cover several row blocks
    that share a vector tile and a STORE (the count stands in the uop's descriptor field).  Dense (the lengths added up,
    B vectors) and ragged (one vector per segment): validated, run under a random schedule, equal to the GEMV, and with
    fewer stores and vector loads than row blocks wherever the form is used."""
    K = 4 * k4
    rng = np.random.default_rng(seed)
    for ragged in (False, True):
        ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64) if ragged else np.array([0, sum(lengths)], np.int64)
        rows, Bv = int(ro[-1]), (1 if ragged else B)
        M = rng.standard_normal((rows, K)).astype(np.float32)
        X = rng.standard_normal((len(ro) - 1 if ragged else Bv, K)).astype(np.float32)
        with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=2048, n_slots=14, n_stu=n_stu) as ex:
            try:
                w, sb, d = ex.matvec_program(rows, K, K, Bv, tile, row_off=ro if ragged else None)
            except vdc.VdcError:
                continue
            ws = ex.matvec_workspace(rows, K, K, Bv, tile) if not ragged else np.zeros(0, np.float32)
            rc, msg = ex.program_validate(w, sb, d, [M.nbytes, X.nbytes, Bv * rows * 4] + ([ws.nbytes] if ws.size else []))
            assert rc == vdc.VDC_OK, msg
        Y = np.full((rows,) if ragged else (Bv, rows), np.nan, np.float32)
        m = UM.Machine(w, sb, d, [M, X, Y] + ([ws] if ws.size else []), n_cores=ncores, slot_bytes=2048, n_slots=14, n_dep_ids=1024, n_stu=n_stu)
        m.run("random", seed)
        m.check_final()
        Yr, Ya = gemv_ref.gemv_ragged(M, ro, X) if ragged else gemv_ref.gemv_dense(M, X)
        assert np.all(np.abs(Y - Yr) <= 2e-6 * Ya + 1e-30)
        # the MATVECs as executed (a stretch of whole groups is a loop): their words through the compute cores' traces
        V = 2
        mv = [w[sb[c * (1 + V) + 1 + v] + r[0]] for c in range(ncores) for v in range(V) for r in m.trace_vcc[c][v] if r[1] == 16]
        spans = [(int(x[3]) >> 16) & 0xFF for x in mv]
        if max(spans) >= 2:
            loads_x = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 1)
            loads_m = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.LOAD and m.descs[r[2]].tensor == 0)
            stores = sum(1 for t in m.trace_vmc for r in t if r[1] == UM.STORE)
            assert loads_x == len(mv) and stores == len(mv) and loads_m == sum(max(1, x) for x in spans) and len(mv) < loads_m


@settings(**COMMON)
@given(lengths=st.lists(st.integers(1, 200), min_size=1, max_size=7), tile=st.sampled_from([4096, 8192, 16384]),
       ncores=st.integers(1, 4), seed=st.integers(0, 1000), d=st.sampled_from([64, 128]))
def test_attention_programs(lengths, tile, ncores, seed, d):
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((len(lengths), d)).astype(np.float32)
    K = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
    V = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=4096, n_slots=16) as ex:
        w, sb, ds, n_items = ex.attn_decode_program(ro, d, tile)
        rc, msg = ex.program_validate(w, sb, ds, [K.nbytes, V.nbytes, Q.nbytes, Q.nbytes, n_items * (d + 4) * 4])
        assert rc == vdc.VDC_OK, msg
    O = np.full((len(lengths), d), np.nan, np.float32)
    W = np.full((n_items, d + 4), np.nan, np.float32)
    _machine(w, sb, ds, [K, V, Q, O, W], ncores, 4096, 16, seed)
    Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, d ** -0.5)
    assert np.all(np.abs(O - Or) <= 4e-7 * Ar + 1e-30)


@settings(**COMMON)
@given(mode=st.sampled_from(["read", "fill", "copy"]), n16=st.integers(1, 3000), tile=st.sampled_from([256, 1024, 4096]),
       ncores=st.integers(1, 4), seed=st.integers(0, 1000))
def test_stream_programs(mode, n16, tile, ncores, seed):
    nbytes = 16 * n16
    rng = np.random.default_rng(seed)
    src = rng.integers(0, 256, nbytes + 16, dtype=np.uint8)
    keep = src.copy()
    dst = np.full(nbytes + 16, 0xEE, np.uint8)
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=1024, n_slots=12) as ex:
        w, sb, d = ex.stream_program(mode, nbytes, tile, value=0x5A5A0F0F)
        rc, msg = ex.program_validate(w, sb, d, [nbytes, nbytes] if mode == "copy" else [nbytes])
        assert rc == vdc.VDC_OK, msg
    _machine(w, sb, d, {"read": [src], "fill": [dst], "copy": [src, dst]}[mode], ncores, 1024, 12, seed)
    assert np.array_equal(src, keep) and np.all(dst[nbytes:] == 0xEE)
    if mode == "copy":
        assert np.array_equal(dst[:nbytes], src[:nbytes])
    if mode == "fill":
        assert np.all(dst[:nbytes].view(np.uint32) == 0x5A5A0F0F)


@settings(**COMMON)
@given(dims4=st.lists(st.integers(1, 60), min_size=2, max_size=5), B=st.integers(1, 4), tile=st.sampled_from([2048, 4096]),
       ncores=st.integers(1, 4), seed=st.integers(0, 1000))
def test_chain_programs(dims4, B, tile, ncores, seed):
    dims = [4 * x for x in dims4]
    L = len(dims) - 1
    rng = np.random.default_rng(seed)
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L)]
    X = rng.standard_normal((B, dims[0])).astype(np.float32)
    W = np.concatenate([m.ravel() for m in Ms])
    with vdc.Executor(device=-1, n_cores=ncores, slot_bytes=2048, n_slots=16) as ex:
        try:
            w, sb, d = ex.matvec_chain_program(dims, B, tile)
        except vdc.VdcError:
            return                                           # a shape the tiler does not chain (a row block wider than the next layer's tile)
        a_bytes = 4 * B * sum(dims)
        rc, msg = ex.program_validate(w, sb, d, [W.nbytes, a_bytes, a_bytes])
        assert rc == vdc.VDC_OK, msg
    Abuf = np.full(B * sum(dims), np.nan, np.float32)
    Abuf[:B * dims[0]] = X.ravel()
    _machine(w, sb, d, [W, Abuf, Abuf], ncores, 2048, 16, seed)
    a_off = np.concatenate([[0], np.cumsum([B * x for x in dims])])
    prev = X
    for l in range(L):
        Y = Abuf[a_off[l + 1]:a_off[l + 2]].reshape(B, dims[l + 1])
        Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
        assert np.all(np.abs(Y - Yr) <= 1e-7 * Ya + 1e-30), l
        prev = Y
