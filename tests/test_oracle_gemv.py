"""Pins of the fp64 GEMV oracle (oracle/gemv_ref.c) against what the mathematics fixes.

The hot path reaches exactly the matrix-vector product of the paper's running example
(Section 3, O = M @ N), so the oracle is that definition; these tests tie it to closed
forms, invariants, a library routine and exact rational brute force, chosen so that a
dropped term, a transposed operand or a wrong stride fails at least one of them.
"""
from fractions import Fraction

import numpy as np
import pytest

import workloads
from oracle import gemv_ref


def test_all_ones_gives_K():
    for rows, K, B in [(3, 1, 1), (17, 129, 2), (5, 4096, 8)]:
        Y, Ya = gemv_ref.gemv_dense(np.ones((rows, K), np.float32), np.ones((B, K), np.float32))
        assert Y.shape == (B, rows)
        assert np.all(Y == K) and np.all(Ya == K)


def test_identity_returns_x_exactly():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((3, 64)).astype(np.float32)
    Y, _ = gemv_ref.gemv_dense(np.eye(64, dtype=np.float32), X)
    assert np.array_equal(Y, X.astype(np.float64))


def test_row_index_pattern_closed_form():
    rows, K = 2500, 333
    M = np.repeat((np.arange(rows) % 1024).astype(np.float32)[:, None], K, axis=1)
    Y, _ = gemv_ref.gemv_dense(M, np.ones((1, K), np.float32))
    assert np.array_equal(Y[0], K * (np.arange(rows) % 1024).astype(np.float64))


def test_column_weights_catch_transposition():
    # M[i][j] = i + 1, X[j] = j + 1: Y[i] = (i + 1) K (K + 1) / 2; the transposed product differs
    rows, K = 7, 11
    M = np.repeat(np.arange(1, rows + 1, dtype=np.float32)[:, None], K, axis=1)
    X = np.arange(1, K + 1, dtype=np.float32)[None, :]
    Y, _ = gemv_ref.gemv_dense(M, X)
    assert np.array_equal(Y[0], np.arange(1, rows + 1) * (K * (K + 1) / 2.0))


def test_single_nonzero_selects_one_term():
    rows, K, B = 37, 53, 3
    rng = np.random.default_rng(2)
    X = rng.random((B, K), dtype=np.float32) + 1.0
    for (i, j) in [(0, 0), (36, 52), (5, 40), (20, 1)]:
        M = np.zeros((rows, K), np.float32)
        M[i, j] = 3.0
        Y, _ = gemv_ref.gemv_dense(M, X)
        exp = np.zeros((B, rows))
        exp[:, i] = 3.0 * X[:, j].astype(np.float64)
        assert np.array_equal(Y, exp)


def test_leading_dimension_skips_padding():
    rng = np.random.default_rng(3)
    rows, K, ld = 9, 20, 28
    Mp = rng.standard_normal((rows, ld)).astype(np.float32)
    X = rng.standard_normal((2, K)).astype(np.float32)
    Y1, _ = gemv_ref.gemv_dense(Mp, X, ld=ld)
    Y2, _ = gemv_ref.gemv_dense(Mp[:, :K].copy(), X)
    assert np.array_equal(Y1, Y2)


def test_matches_library_matmul_fp64():
    w = workloads.make("cfg1")
    M, X = w.M.numpy(), w.X.numpy()
    Y, Ya = gemv_ref.gemv_dense(M, X)
    ref = X.astype(np.float64) @ M.astype(np.float64).T
    assert np.allclose(Y, ref, rtol=1e-13, atol=0)
    assert np.allclose(Ya, np.abs(X.astype(np.float64)) @ np.abs(M.astype(np.float64)).T, rtol=1e-13)
    rng = np.random.default_rng(5)
    M = rng.standard_normal((61, 97)).astype(np.float32)
    X = rng.standard_normal((8, 97)).astype(np.float32)
    Y, Ya = gemv_ref.gemv_dense(M, X)
    ref = X.astype(np.float64) @ M.astype(np.float64).T
    assert np.all(np.abs(Y - ref) <= 1e-13 * Ya)


def test_exact_rational_brute_force():
    rng = np.random.default_rng(7)
    rows, K, B = 6, 9, 2
    M = rng.standard_normal((rows, K)).astype(np.float32)
    X = rng.standard_normal((B, K)).astype(np.float32)
    Y, _ = gemv_ref.gemv_dense(M, X)
    for b in range(B):
        for i in range(rows):
            exact = sum(Fraction(float(M[i, j])) * Fraction(float(X[b, j])) for j in range(K))
            assert abs(Fraction(float(Y[b, i])) - exact) <= abs(exact) * Fraction(1, 10**13) + Fraction(1, 10**18)


def test_linearity_and_row_permutation():
    rng = np.random.default_rng(11)
    M = rng.integers(-8, 9, (33, 45)).astype(np.float32)       # small integers: everything exact
    x1 = rng.integers(-8, 9, (1, 45)).astype(np.float32)
    x2 = rng.integers(-8, 9, (1, 45)).astype(np.float32)
    Y1, _ = gemv_ref.gemv_dense(M, x1)
    Y2, _ = gemv_ref.gemv_dense(M, x2)
    Y12, _ = gemv_ref.gemv_dense(M, 2 * x1 - 3 * x2)
    assert np.array_equal(Y12, 2 * Y1 - 3 * Y2)
    perm = rng.permutation(33)
    Yp, _ = gemv_ref.gemv_dense(M[perm], x1)
    assert np.array_equal(Yp[0], Y1[0][perm])


def test_ragged_equals_dense_per_segment():
    rng = np.random.default_rng(13)
    K = 24
    row_off = np.array([0, 5, 5, 17, 18, 40], dtype=np.int64)     # includes an empty segment
    M = rng.standard_normal((40, K)).astype(np.float32)
    X = rng.standard_normal((5, K)).astype(np.float32)
    Y, Ya = gemv_ref.gemv_ragged(M, row_off, X)
    for s in range(5):
        a, b = row_off[s], row_off[s + 1]
        if a == b:
            continue
        Yd, Yad = gemv_ref.gemv_dense(M[a:b], X[s:s + 1])
        assert np.array_equal(Y[a:b], Yd[0]) and np.array_equal(Ya[a:b], Yad[0])


def test_ragged_uses_the_segments_own_vector():
    K = 8
    row_off = np.array([0, 2, 5], dtype=np.int64)
    M = np.ones((5, K), np.float32)
    X = np.stack([np.full(K, 2.0, np.float32), np.full(K, 5.0, np.float32)])
    Y, _ = gemv_ref.gemv_ragged(M, row_off, X)
    assert np.array_equal(Y, np.array([16, 16, 40, 40, 40], dtype=np.float64))


def test_zipf_segments_recipe():
    ro = workloads.zipf_segments(1 << 19, 64, 1.1, 3)
    L = np.diff(ro)
    assert ro[0] == 0 and ro[-1] == 1 << 19 and len(L) == 64 and L.min() >= 16
    assert 0.2 < L.max() / L.sum() < 0.3                      # the longest holds about a quarter
    ranked = np.sort(L)[::-1].astype(np.float64)
    fit = np.polyfit(np.log(np.arange(2, 65)), np.log(ranked[1:]), 1)[0]
    assert abs(fit + 1.1) < 0.02                              # rank-length slope is -s
