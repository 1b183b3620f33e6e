"""Seeded random shapes on the GPU, each against the oracle: the same operators as the other parity tests, on shapes nobody
picked by hand (tails in every dimension, odd leading dimensions, ragged batches with empty segments, contexts from one
row to several tiles, byte ranges with short rests, chains of uneven layers).  The launch configuration bench.py times, and the same
with two store units per core."""
import numpy as np
import pytest
import torch

import paper_2605_03190_amd as vdc
from oracle import attn_ref, gemv_ref

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.fixture(scope="module", params=[dict(), dict(n_stu=2)], ids=["default", "two-store-units"])
def ex(request):
    e = vdc.Executor(**request.param)
    yield e
    e.destroy()


def test_random_dense_and_ragged_matvecs(ex):
    rng = np.random.default_rng(2605)
    for case in range(40):
        B = int(rng.integers(1, 9))
        tile = int(rng.choice([2048, 4096, 8192, 16384]))
        rows, K = int(rng.integers(1, 3000)), 4 * int(rng.integers(1, 1200))
        ld = K + 4 * int(rng.integers(0, 3))
        M = rng.standard_normal((rows, ld)).astype(np.float32)
        X = rng.standard_normal((B, K)).astype(np.float32)
        Y = torch.full((B, rows), float("nan"), device="cuda")
        try:
            ex.matvec(_dev(M), _dev(X), Y, tile, K=K)
        except vdc.VdcError as e:
            assert e.code == vdc.VDC_EINVAL                  # a (B, tile) pair the compute uop has no geometry for
            continue
        ex.check()
        Yr, Ya = gemv_ref.gemv_dense(M, X, ld=ld)
        worst = float((np.abs(Y.cpu().numpy() - Yr) / (1e-5 * Ya + 1e-30)).max())
        assert worst <= 1.0, "dense case %d: rows %d K %d ld %d B %d tile %d: %.3g" % (case, rows, K, ld, B, tile, worst)
    # one vector, K a whole number of tiles: the form with vector tiles over several steps
    for case in range(16):
        tile = int(rng.choice([2048, 4096, 8192, 16384]))
        rows, K = int(rng.integers(1, 20000)), 256 * int(rng.integers(2, 40))
        M = rng.standard_normal((rows, K)).astype(np.float32)
        X = rng.standard_normal((1, K)).astype(np.float32)
        Y = torch.full((1, rows), float("nan"), device="cuda")
        ex.matvec(_dev(M), _dev(X), Y, tile)
        ex.check()
        Yr, Ya = gemv_ref.gemv_dense(M, X)
        worst = float((np.abs(Y.cpu().numpy() - Yr) / (1e-5 * Ya + 1e-30)).max())
        assert worst <= 1.0, "one-vector case %d: rows %d K %d tile %d: %.3g" % (case, rows, K, tile, worst)
    for case in range(12):
        n_seg = int(rng.integers(1, 40))
        lengths = rng.integers(0, 400, n_seg)
        lengths[rng.integers(0, n_seg)] = 0
        ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
        rows, K = int(ro[-1]), 4 * int(rng.integers(1, 300))
        if rows == 0:
            continue
        tile = int(rng.choice([2048, 4096, 8192]))
        M = rng.standard_normal((rows, K)).astype(np.float32)
        X = rng.standard_normal((n_seg, K)).astype(np.float32)
        Y = torch.full((rows,), float("nan"), device="cuda")
        ex.matvec_ragged(_dev(M), ro, _dev(X), Y, tile)
        ex.check()
        Yr, Ya = gemv_ref.gemv_ragged(M, ro, X)
        worst = float((np.abs(Y.cpu().numpy() - Yr) / (1e-5 * Ya + 1e-30)).max())
        assert worst <= 1.0, "ragged case %d: %.3g" % (case, worst)


def test_random_attention_batches(ex):
    rng = np.random.default_rng(31)
    for case in range(12):
        n = int(rng.integers(1, 30))
        lengths = np.maximum(1, (rng.pareto(1.2, n) * 40).astype(np.int64))       # a few long contexts among short ones
        lengths = np.minimum(lengths, 5000)
        ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
        tile = int(rng.choice([4096, 8192, 16384]))
        d = int(rng.choice([64, 128]))
        Q = rng.standard_normal((n, d)).astype(np.float32)
        K = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
        V = rng.standard_normal((int(ro[-1]), d)).astype(np.float32)
        O = torch.full((n, d), float("nan"), device="cuda")
        ex.attn_decode(_dev(Q), _dev(K), _dev(V), ro, O, tile)
        ex.check()
        Or, Ar, S = attn_ref.attn_decode(Q, K, V, ro, d ** -0.5)
        worst = float((np.abs(O.cpu().numpy() - Or) / ((2e-5 * S[:, None] + 2e-5) * Ar + 1e-30)).max())
        assert worst <= 1.0, "attention case %d (%d contexts, %d rows, tile %d): %.3g" % (case, n, int(ro[-1]), tile, worst)


def test_random_byte_ranges(ex):
    rng = np.random.default_rng(7)
    for case in range(15):
        mode = ["read", "fill", "copy"][case % 3]
        nbytes = 16 * int(rng.integers(1, 400000))
        tile = int(rng.choice([256, 1024, 4096, 16384]))
        src = torch.randint(0, 256, (nbytes + 16,), dtype=torch.uint8, device="cuda")
        keep = src.clone()
        dst = torch.full((nbytes + 16,), 0xEE, dtype=torch.uint8, device="cuda")
        ex.stream(mode, src if mode != "fill" else None, dst if mode != "read" else None, nbytes, tile, value=0x12345678)
        ex.check()
        assert torch.equal(src, keep) and bool((dst[nbytes:] == 0xEE).all()), (case, mode, nbytes, tile)
        if mode == "copy":
            assert torch.equal(dst[:nbytes], src[:nbytes]), (case, nbytes, tile)
        if mode == "fill":
            assert bool((dst[:nbytes].view(torch.int32) == 0x12345678).all()), (case, nbytes, tile)


def test_random_chains(ex):
    rng = np.random.default_rng(11)
    done = 0
    for case in range(12):
        L = int(rng.integers(2, 6))
        dims = [4 * int(rng.integers(8, 900)) for _ in range(L + 1)]
        B = int(rng.integers(1, 5))
        tile = int(rng.choice([4096, 8192, 16384]))
        Ms = [(rng.standard_normal((dims[l + 1], dims[l])) / np.sqrt(dims[l])).astype(np.float32) for l in range(L)]
        X = rng.standard_normal((B, dims[0])).astype(np.float32)
        a_off = np.concatenate([[0], np.cumsum([B * x for x in dims])])
        dA = torch.full((int(a_off[-1]),), float("nan"), device="cuda")
        dA[:B * dims[0]] = _dev(X.ravel())
        try:
            ex.matvec_chain(_dev(np.concatenate([m.ravel() for m in Ms])), dA, dims, B, tile)
        except vdc.VdcError as e:
            assert e.code == vdc.VDC_EINVAL
            continue
        ex.check()
        done += 1
        Ah = dA.cpu().numpy()
        prev = X
        for l in range(L):
            Y = Ah[a_off[l + 1]:a_off[l + 2]].reshape(B, dims[l + 1])
            Yr, Ya = gemv_ref.gemv_dense(Ms[l], prev)
            worst = float((np.abs(Y - Yr) / (1e-5 * Ya + 1e-30)).max())
            assert worst <= 1.0, "chain case %d dims %s layer %d: %.3g" % (case, dims, l, worst)
            prev = Y
    assert done >= 6
