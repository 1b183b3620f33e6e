"""Parity at the full benchmark sizes, in the launch configuration bench.py times (one core per CU, default units).

The fp64 oracle computes every output of cfg3, cfg4 and cfg5 (B = 8 and B = 1; the 8 GiB matrix goes through the host in
row blocks, one per thread).  Properties that hold at any size come on top: an all-rows closed form that is exact in fp32,
and single non-zero entries at byte offsets beyond 2^32.
"""
import numpy as np
import pytest
import torch

import paper_2605_03190_amd as vdc
import workloads
from oracle import gemv_ref

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _worst(Y_gpu, Yr, Ya):
    return float((np.abs(Y_gpu.astype(np.float64) - Yr) / (TOL * Ya + 1e-30)).max())


def _free():
    import gc
    gc.collect()
    torch.cuda.empty_cache()


def test_cfg3_every_output():
    cfg = workloads.CONFIGS["cfg3"]
    w = workloads.make(cfg, device="cuda")
    Y = torch.full((cfg.B, cfg.rows), float("nan"), device="cuda")
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        ex.matvec(w.M, w.X, Y, cfg.tile_bytes)
        ex.check()
    Yr, Ya = gemv_ref.gemv_dense(w.M.cpu().numpy(), w.X.cpu().numpy())
    assert _worst(Y.cpu().numpy(), Yr, Ya) <= 1.0
    _free()


def test_cfg4_ragged_every_output():
    cfg = workloads.CONFIGS["cfg4"]
    w = workloads.make(cfg, device="cuda")
    Y = torch.full((cfg.rows,), float("nan"), device="cuda")
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        ex.matvec_ragged(w.M, w.row_off, w.X, Y, cfg.tile_bytes)
        ex.check()
    Yr, Ya = gemv_ref.gemv_ragged(w.M.cpu().numpy(), w.row_off, w.X.cpu().numpy())
    assert _worst(Y.cpu().numpy(), Yr, Ya) <= 1.0
    _free()


def _oracle_dense_all_rows(M_dev, Xh, threads=16):
    """The fp64 oracle on every row of a matrix that lives on the GPU: row blocks go through the host one at a time per
    thread (the C loops run outside the interpreter lock), so the 8 GiB matrix is never held twice."""
    import concurrent.futures
    rows = M_dev.shape[0]
    blk = -(-rows // threads)

    def part(i):
        a, b = i * blk, min(rows, (i + 1) * blk)
        return gemv_ref.gemv_dense(M_dev[a:b].cpu().numpy(), Xh)

    with concurrent.futures.ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(part, range(threads)))
    return np.concatenate([p[0] for p in parts], axis=1), np.concatenate([p[1] for p in parts], axis=1)


@pytest.mark.parametrize("name", ["cfg5", "cfg5_b1"])
def test_cfg5_every_output_against_the_oracle(name):
    """All 32768 x B outputs of the headline configuration against the fp64 definition, in the launch configuration
    bench.py times."""
    cfg = workloads.CONFIGS[name]
    w = workloads.make(cfg, device="cuda")
    Y = torch.full((cfg.B, cfg.rows), float("nan"), device="cuda")
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        ex.matvec(w.M, w.X, Y, cfg.tile_bytes)
        ex.check()
    Yh = Y.cpu().numpy()
    assert np.isfinite(Yh).all(), "an output was never written"
    Yr, Ya = _oracle_dense_all_rows(w.M, w.X.cpu().numpy())
    assert Yr.shape == Yh.shape
    assert _worst(Yh, Yr, Ya) <= 1.0
    del w, Y
    _free()


def test_cfg5_row_pattern_is_exact_for_every_output():
    """M[i][j] = i mod 1024 and X[b] = 2^b: Y[b][i] = 2^b * K * (i mod 1024), exactly representable at every step of
    any summation tree whose leaves are whole numbers of equal-length runs, so every one of the 8 x 32768 outputs is
    compared bit for bit (catches a wrong row anywhere, at offsets up to 8 GiB)."""
    cfg = workloads.CONFIGS["cfg5"]
    a = (torch.arange(cfg.rows, device="cuda") % 1024).to(torch.float32)
    M = a[:, None].expand(cfg.rows, cfg.K).contiguous()
    X = (2.0 ** torch.arange(cfg.B, device="cuda", dtype=torch.float32))[:, None].expand(cfg.B, cfg.K).contiguous()
    Y = torch.full((cfg.B, cfg.rows), float("nan"), device="cuda")
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        ex.matvec(M, X, Y, cfg.tile_bytes)
        ex.check()
    exp = (2.0 ** np.arange(cfg.B))[:, None] * (cfg.K * (np.arange(cfg.rows) % 1024))[None, :]
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), exp)
    del M, X, Y
    _free()


def test_cfg5_single_entries_beyond_4_gib():
    """One non-zero entry at a time, x[j] = j + 1: the result is j* + 1 in row i* and zero everywhere else."""
    cfg = workloads.CONFIGS["cfg5_b1"]
    M = torch.zeros((cfg.rows, cfg.K), device="cuda")
    X = (torch.arange(cfg.K, device="cuda", dtype=torch.float32) + 1.0)[None, :].contiguous()
    Y = torch.empty((1, cfg.rows), device="cuda")
    spots = [(0, 0), (cfg.rows - 1, cfg.K - 1), (16384, 1), (16385, 65535), (20000, 12345), (32767, 0), (24575, 255), (24576, 256)]
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        for (i, j) in spots:
            assert i * cfg.K * 4 + j * 4 >= (1 << 32) or i < 16384
            M[i, j] = 1.0
            Y.fill_(float("nan"))
            ex.matvec(M, X, Y, cfg.tile_bytes)
            ex.check()
            Yh = Y.cpu().numpy()[0]
            exp = np.zeros(cfg.rows, dtype=np.float32)
            exp[i] = j + 1
            assert np.array_equal(Yh, exp), (i, j)
            M[i, j] = 0.0
    del M, X, Y
    _free()


# ---- decode attention at the benchmark's sizes (bench.py --workload attn_*: 8 heads per request) ---------------
@pytest.mark.parametrize("regime", ["attn_0.5k_b", "attn_64k", "attn_rand"])
def test_attention_regimes_at_benchmark_size(regime):
    """Every context against the fp64 definition, and properties that hold for every output: value rows that are all equal come back whatever the weights are,
    up to the rounding of the sums; every output lies between the smallest and largest value it
    averages."""
    from oracle import attn_ref
    import bench
    d, heads = 128, 8
    lengths = np.repeat(bench.ATTN_REGIMES[regime][1](), heads)
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = int(ro[-1])
    g = torch.Generator(device="cuda").manual_seed(rows)
    Q = torch.randn((len(lengths), d), device="cuda", generator=g)
    K = torch.randn((rows, d), device="cuda", generator=g)
    V = torch.randn((rows, d), device="cuda", generator=g)
    O = torch.full((len(lengths), d), float("nan"), device="cuda")
    with vdc.Executor() as ex:
        ex.attn_decode(Q, K, V, ro, O, 16384)
        ex.check()
        Og = O.cpu().numpy()
        assert np.all(np.isfinite(Og))
        # every context of the batch against the fp64 definition
        Or, Ar, S = attn_ref.attn_decode(Q.cpu().numpy(), K.cpu().numpy(), V.cpu().numpy(), ro, d ** -0.5)
        bad = np.abs(Og - Or) > (2e-5 * S[:, None] + 2e-5) * Ar + 1e-30
        assert not bad.any(), "contexts %s" % sorted(set(np.nonzero(bad)[0].tolist()))[:8]
        # every output is a weighted mean of its context's value rows
        seg = torch.repeat_interleave(torch.arange(len(lengths), device="cuda"), torch.from_numpy(lengths).cuda())
        lo = torch.full((len(lengths), d), float("inf"), device="cuda").scatter_reduce(0, seg[:, None].expand(-1, d), V, "amin")
        hi = torch.full((len(lengths), d), float("-inf"), device="cuda").scatter_reduce(0, seg[:, None].expand(-1, d), V, "amax")
        assert bool(((O >= lo - 1e-5) & (O <= hi + 1e-5)).all())
        # constant value rows per context: the result is that row, whatever the scores
        Vc = (seg.to(torch.float32) * 0.25 + 1.0)[:, None].expand(-1, d).contiguous()
        ex.attn_decode(Q, K, Vc, ro, O, 16384)
        ex.check()
        want = (torch.arange(len(lengths), device="cuda", dtype=torch.float32) * 0.25 + 1.0)[:, None].expand(-1, d)
        assert bool((torch.abs(O - want) <= 1e-5 * want).all())
    _free()


@pytest.mark.parametrize("n_stu", [1, 2])
def test_memory_uops_over_the_sweep_range(n_stu):
    """The block-size sweep's own range and launch configurations (4 GiB, 16 KB and 32 KB blocks, one and two store units):
    every byte of a copy and of a fill, and nothing past the range."""
    _free()
    nbytes = 4096 << 20
    g = torch.Generator(device="cuda").manual_seed(7)
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, ((nbytes + 64) // 4,), dtype=torch.int32, device="cuda", generator=g).view(torch.uint8)
    dst = torch.full((nbytes + 64,), 0xEE, dtype=torch.uint8, device="cuda")
    with vdc.Executor(n_stu=n_stu) as ex:
        for T in (16384, 32768):
            dst.fill_(0xEE)
            ex.stream("copy", src, dst, nbytes, T)
            ex.check()
            assert torch.equal(dst[:nbytes], src[:nbytes]) and bool((dst[nbytes:] == 0xEE).all())
        ex.stream("fill", None, dst, nbytes, 16384, value=0x5A5A1234)
        ex.check()
        assert bool((dst[:nbytes].view(torch.int32) == 0x5A5A1234).all()) and bool((dst[nbytes:] == 0xEE).all())
    del src, dst
    _free()
