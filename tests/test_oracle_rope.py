"""Pins of the rope oracle and of the interpreter's fused matvec + rope program (store.local / load.local)."""
import numpy as np
import pytest

from oracle import gemv_ref, rope_ref, uop_asm as A, uop_machine as UM


def _angles(rng, B, pairs):
    return rng.uniform(-np.pi, np.pi, (B, pairs))


def test_zero_angle_is_the_identity_and_quarter_turn_swaps_with_a_sign():
    rng = np.random.default_rng(0)
    O = rng.standard_normal((2, 10))
    R, _ = rope_ref.rope(O, rope_ref.table(np.zeros((2, 5))))
    assert np.array_equal(R, O)
    T = np.zeros((2, 10)); T[:, 1::2] = 1.0                  # cos 0, sin 1 exactly: a quarter turn
    R, _ = rope_ref.rope(O, T)
    assert np.array_equal(R[:, 0::2], -O[:, 1::2]) and np.array_equal(R[:, 1::2], O[:, 0::2])


def test_equals_multiplication_by_a_unit_complex_number():
    rng = np.random.default_rng(1)
    O = rng.standard_normal((3, 64))
    a = _angles(rng, 3, 32)
    T = np.empty((3, 64)); T[:, 0::2] = np.cos(a); T[:, 1::2] = np.sin(a)
    R, _ = rope_ref.rope(O, T)
    z = (O[:, 0::2] + 1j * O[:, 1::2]) * np.exp(1j * a)
    assert np.allclose(R[:, 0::2], z.real, rtol=0, atol=1e-14) and np.allclose(R[:, 1::2], z.imag, rtol=0, atol=1e-14)


def test_pairs_keep_their_length_and_turns_add_up():
    rng = np.random.default_rng(2)
    O = rng.standard_normal((2, 32))
    a, b = _angles(rng, 2, 16), _angles(rng, 2, 16)
    def tab(x):
        T = np.empty((2, 32)); T[:, 0::2] = np.cos(x); T[:, 1::2] = np.sin(x); return T
    Ra, _ = rope_ref.rope(O, tab(a))
    assert np.allclose(Ra[:, 0::2] ** 2 + Ra[:, 1::2] ** 2, O[:, 0::2] ** 2 + O[:, 1::2] ** 2, rtol=1e-13)
    Rab, _ = rope_ref.rope(Ra, tab(b))
    Rsum, _ = rope_ref.rope(O, tab(a + b))
    assert np.allclose(Rab, Rsum, rtol=0, atol=1e-13)
    # a transposed pair or a flipped sign would turn the other way: the inverse turn undoes it only with the right signs
    Rback, _ = rope_ref.rope(Ra, tab(-a))
    assert np.allclose(Rback, O, rtol=0, atol=1e-13)


def test_each_vector_uses_its_own_angles():
    O = np.ones((2, 4))
    T = rope_ref.table(np.array([[0.0, 0.0], [np.pi, np.pi]]))
    R, _ = rope_ref.rope(O, T)
    assert np.allclose(R[0], 1.0) and np.allclose(R[1], -1.0, atol=1e-6)


@pytest.mark.parametrize("rows,K,B,R,Kt,slot,ncores", [(40, 96, 3, 8, 32, 1024, 3), (64, 64, 1, 16, 64, 4096, 2), (24, 40, 8, 8, 16, 512, 5)])
def test_fused_program_on_the_interpreter(rows, K, B, R, Kt, slot, ncores):
    """O = M X stays on chip (store.local / load.local), rope turns it: same result under the fixed sweep and under
    random legal schedules, equal to the two oracles applied one after the other, no slot left allocated."""
    rng = np.random.default_rng(rows + K)
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    T = rope_ref.table(_angles(rng, B, rows // 2))
    w, sb, d = A.dense_matvec_program(rows, K, K, B, R, Kt, slot, n_cores=ncores, rope=True).finish()
    O, Oa = gemv_ref.gemv_dense(M, X)
    Rr, Ra = rope_ref.rope(O, T)
    images, traces = [], []
    for sched, seed in [("program", 0)] + [("random", s) for s in range(1, 21)]:
        Y = np.full((B, rows), np.nan, np.float32)
        m = UM.Machine(w, sb, d, [M, X, Y, T], n_cores=ncores, slot_bytes=slot, n_slots=12)
        m.run(sched, seed)
        m.check_final()
        # the intermediate O passes through fp32 once: its rounding is part of the bound
        assert np.all(np.abs(Y - Rr) <= 1e-6 * (Ra + Oa) + 1e-30)
        images.append(Y.copy())
        traces.append((m.trace_vmc, m.trace_vcc))
        assert all(c.mask == 0 and not any(c.parked) for c in m.cores)
    assert all(np.array_equal(images[0], im) for im in images[1:])
    assert all(traces[0] == t for t in traces[1:])
    ops = w[:, 0] & 0xFF
    flags = (w[:, 0] >> 8) & 0xFF
    assert ((ops == A.STORE) & ((flags & A.F_LOCAL) != 0)).sum() == -(-rows // R)
    assert ((ops == A.LOAD) & ((flags & A.F_LOCAL) != 0)).sum() == -(-rows // R)


def test_a_load_local_without_its_store_local_deadlocks():
    p = A.Program(1, 1)
    d = p.desc(0, 1, 16, 16, 16)
    p.vmc(0).append(A.word(A.LOAD, A.F_SEND | A.F_LOCAL, vflow=0, vcc=0, nslots=0, size=1, desc=d))
    w, sb, ds = p.finish()
    m = UM.Machine(w, sb, ds, [np.zeros(4, np.float32)], n_cores=1, vcc_per_core=1, slot_bytes=1024, n_slots=4)
    with pytest.raises(UM.DeadlockError):
        m.run("program", 0)
