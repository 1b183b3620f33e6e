"""Contracts of the generator's lowering steps (Section 4.2), pinned on the interpreter before any product code:
every step leaves the results of the graph alone, whatever the schedule; a store -> load pair that is rewritten to
store.local / load.local gives the bits of the program that was written fused by hand; an order of the memory core's
stream that over-commits the slots deadlocks before the reordering step and completes after it; removing the waits that
flow order implies removes waits and nothing else (and a wait that is NOT implied cannot be removed)."""
import copy

import numpy as np
import pytest

from oracle import gemv_ref, rope_ref, uop_asm as A, uop_lower as L, uop_machine as UM


def _run(g, tensors, n_slots, schedule="program", seed=0):
    w, sb, d = L.assemble(g).finish()
    ts = [t.copy() for t in tensors]
    m = UM.Machine(w, sb, d, ts, n_cores=g.n_cores, vcc_per_core=g.V, slot_bytes=g.slot_bytes, n_slots=n_slots).run(schedule, seed)
    return m, ts


def _rope_inputs(rows, K, B, seed):
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    T = rope_ref.table(rng.uniform(-np.pi, np.pi, (B, rows // 2))).astype(np.float32)
    return M, X, T


def _semantics(words, descs):
    """A program's memory and compute uops without the numbering of the descriptor table."""
    out = []
    for w in words:
        u = UM.decode(w)
        d = tuple(int(x) for x in descs[u.desc][:6]) if u.opcode in (A.LOAD, A.STORE) else None
        out.append((u.opcode, u.flags, u.vflow, u.vcc, u.acc, u.nslots, u.size, u.dep_id, u.imm, u.dep_count, d))
    return out


def test_store_load_pair_becomes_the_fused_program_written_by_hand():
    """The running example of Section 3.  Unfused, O = M X goes through memory (a temporary tensor) and rope reads it back;
    the placement step keeps it in local memory.  The rewritten graph is, uop for uop, the fused program that the
    assembler writes directly, its result has the same bits as the unfused graph's, and both are the fp64 product turned by
    the fp64 rotation within the bound."""
    rows, K, B, R, Kt, slot, C = 96, 256, 3, 8, 64, 1024, 3
    M, X, T = _rope_inputs(rows, K, B, 5)
    tensors = [M, X, np.full((B, rows), np.nan, np.float32), T, np.full((B, rows), np.nan, np.float32)]
    unfused = L.matvec_rope_graph(rows, K, B, R, Kt, slot, C)
    L.assign_flows(unfused)
    assert L.embed_deps(copy.deepcopy(unfused))[1] == rows // R          # left alone, every pair would need a wait of its own
    fused = L.matvec_rope_graph(rows, K, B, R, Kt, slot, C)
    assert L.place_local(fused) == rows // R and not fused.edges
    L.assign_flows(fused)
    assert L.embed_deps(fused) == (0, 0, 0)
    # the unfused graph needs its dependency: the store must have landed before the load reads (same core, other unit)
    g0 = copy.deepcopy(unfused)
    L.embed_deps(g0)
    _, t0 = _run(g0, tensors, 12)
    _, t1 = _run(fused, tensors, 12)
    assert np.array_equal(t0[2], t1[2]) and np.isfinite(t1[2]).all()
    assert np.isnan(t1[4]).all() and np.isfinite(t0[4]).all()             # fused: the intermediate never reaches memory
    O, Oa = gemv_ref.gemv_dense(M, X)
    Rr, Ra = rope_ref.rope(O, T)
    assert np.all(np.abs(t1[2] - Rr) <= 1e-6 * (Ra + Oa) + 1e-30)         # the intermediate passes through fp32 once
    # uop for uop the program the assembler writes fused by hand
    w1, sb1, d1 = L.assemble(fused).finish()
    w2, sb2, d2 = A.dense_matvec_program(rows, K, K, B, R, Kt, slot, C, nt=True, rope=True).finish()
    assert np.array_equal(sb1, sb2)
    assert _semantics(w1, d1) == _semantics(w2, d2)
    # determinate under random schedules, before and after the step
    for g in (g0, fused):
        for seed in range(25):
            _, t = _run(g, tensors, 12, "random", seed)
            assert np.array_equal(t[2], t1[2])
    # a pair that is not one-to-one stays in memory: a second reader of the same store
    g = L.matvec_rope_graph(rows, K, B, R, Kt, slot, C)
    s, l = g.edges[0]
    extra = L.MemOp(A.LOAD, l.core, l.vcc, l.desc, l.offset, l.rows, l.nslots)
    g.edges.append((s, extra))
    assert L.place_local(g) == rows // R - 1 and len(g.edges) == 2


def _two_core_matvec_graph(rows, K, B, R, Kt, slot):
    """One memory core, two compute cores, a row block each per round; memory uops written down the way that starves:
    the matrix tile of compute core 0, the matrix tile of compute core 1, and only then the vector tiles."""
    g = L.new_graph(1, 2, slot)
    nk = K // Kt
    dm, dx, dy = (0, R, Kt * 4, Kt * 4, K * 4), (1, B, Kt * 4, Kt * 4, K * 4), (2, B, R * 4, R * 4, rows * 4)
    sl = lambda nb: -(-nb // slot)
    per_v = [[], []]
    for rb in range(rows // R):
        v = rb % 2
        grp = (g.mem[0][v][-1].group + 1) if g.mem[0][v] else 0
        for kt in range(nk):
            a = g.add(L.MemOp(A.LOAD, 0, v, dm, (rb * R * K + kt * Kt) * 4, R, sl(R * Kt * 4), grp))
            b = g.add(L.MemOp(A.LOAD, 0, v, dx, kt * Kt * 4, B, sl(B * Kt * 4), grp))
            per_v[v] += [a, b]
            grp += 1
        per_v[v].append(g.add(L.MemOp(A.STORE, 0, v, dy, rb * R * 4, B, sl(B * R * 4), grp)))
        g.comp[0][v].append(A.word(A.MATVEC, size=nk, imm=A.matvec_imm(B, R, Kt // 4)))
    # the starving order: strictly alternate single uops of the two compute cores
    bad = []
    for i in range(max(len(per_v[0]), len(per_v[1]))):
        for v in (0, 1):
            if i < len(per_v[v]):
                bad.append(per_v[v][i])
    g.order = [bad]
    return g


def test_over_committed_order_deadlocks_before_the_reordering_step_and_completes_after():
    rows, K, B, R, Kt, slot = 32, 128, 1, 8, 64, 2048             # a matrix tile is one slot, a vector tile one slot
    rng = np.random.default_rng(9)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    tensors = [M, X, np.full((B, rows), np.nan, np.float32)]
    nbytes = [t.nbytes for t in tensors]
    g = _two_core_matvec_graph(rows, K, B, R, Kt, slot)
    L.assign_flows(g)
    # two slots: a0 and A0 take both; neither compute core ever gets its vector tile
    with pytest.raises(UM.DeadlockError):
        _run(g, tensors, 2)
    assert not L.completes(g, nbytes, 2)
    before = [id(m) for m in g.stream(0)]
    assert L.schedule(g, nbytes, 2) is True
    after = g.stream(0)
    assert sorted(id(m) for m in after) == sorted(before) and [id(m) for m in after] != before
    for v in (0, 1):                                              # every compute core still sees its own order
        assert [m for m in after if m.vcc == v] == g.mem[0][v]
    Yr, Ya = gemv_ref.gemv_dense(M, X)
    for seed in range(100):
        _, t = _run(g, tensors, 2, "random", seed)
        assert np.all(np.abs(t[2] - Yr) <= 1e-5 * Ya)
        if seed == 0:
            first = t[2]
        assert np.array_equal(t[2], first)
    # with room for it the written order is fine and the step changes nothing
    g2 = _two_core_matvec_graph(rows, K, B, R, Kt, slot)
    L.assign_flows(g2)
    assert L.schedule(g2, nbytes, 6) is False
    _, t = _run(g2, tensors, 6)
    assert np.array_equal(t[2], first)
    # a pool that no order can serve is reported, not looped on
    g3 = _two_core_matvec_graph(rows, K, B, R, Kt, slot)
    L.assign_flows(g3)
    with pytest.raises(UM.DeadlockError):
        L.schedule(g3, nbytes, 1)


def test_chain_dependencies_embedded_and_implied_waits_removed():
    dims, B, R, Kt, slot, C = (128, 192, 128, 64), 2, 8, 64, 1024, 3
    rng = np.random.default_rng(4)
    L_ = len(dims) - 1
    Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L_)]
    W = np.concatenate([m.ravel() for m in Ms])
    X = rng.standard_normal((B, dims[0])).astype(np.float32)
    Aact = np.full(B * sum(dims), np.nan, np.float32)
    Aact[:B * dims[0]] = X.ravel()

    def run(g, schedule="program", seed=0):
        w, sb, d = L.assemble(g).finish()
        a = Aact.copy()
        UM.Machine(w, sb, d, [W, a, a], n_cores=C, slot_bytes=slot, n_slots=12).run(schedule, seed)
        return a

    # the layer-by-layer product in fp64
    refs, x = [], X.astype(np.float64)
    for l in range(L_):
        x = x @ Ms[l].astype(np.float64).T
        refs.append(x)
    full = L.chain_graph(dims, B, R, Kt, slot, C)
    L.assign_flows(full)
    n_ids, kept_all, dropped_all = L.embed_deps(full, eliminate=False)
    lean = L.chain_graph(dims, B, R, Kt, slot, C)
    L.assign_flows(lean)
    n_ids2, kept, dropped = L.embed_deps(lean, eliminate=True)
    assert n_ids == n_ids2 == sum(dims[l + 1] // Kt for l in range(L_ - 1))          # one depId per vector tile of layers 1..
    assert dropped_all == 0 and dropped > 0 and kept + dropped == kept_all
    a0 = run(full)
    for g in (full, lean):
        for seed in range(50):
            assert np.array_equal(run(g, "random", seed), a0, equal_nan=True)
    off = B * dims[0]
    for l in range(L_):
        got = a0[off:off + B * dims[l + 1]].reshape(B, dims[l + 1])
        assert np.all(np.abs(got - refs[l]) <= 1e-4 * (np.abs(refs[l]) + 1.0))
        off += B * dims[l + 1]
    # the same bytecode as the assembler's own chain program, up to the waits that flow order implies
    w1, sb1, d1 = L.assemble(full).finish()
    w2, sb2, d2 = A.chain_matvec_program(dims, B, R, Kt, slot, C)[0].finish()
    strip = lambda sem: [(o, f, vf, v, a, ns, sz, imm, d) for (o, f, vf, v, a, ns, sz, dep, imm, dc, d) in sem]
    assert strip(_semantics(w1, d1)) == strip(_semantics(w2, d2))
    # the waits that were kept are NOT implied by anything: without them some schedule reads a tile before it is written
    broken = L.chain_graph(dims, B, R, Kt, slot, C)
    L.assign_flows(broken)
    L.embed_deps(broken)
    for core in range(C):
        for m in broken.stream(core):
            m.dep_wait = None
    assert any(not np.array_equal(run(broken, "random", seed), a0, equal_nan=True) for seed in range(40))
