"""Parity at the full benchmark sizes, in the launch configuration bench.py times (one core per CU, default units).

cfg3 and cfg4 are small enough for the fp64 oracle to compute every output.  For cfg5 (8 GiB matrix) the oracle
computes sampled rows one by one, and properties that hold at any size cover every output: an all-rows closed form
that is exact in fp32, and single non-zero entries at byte offsets beyond 2^32.
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


@pytest.mark.parametrize("name", ["cfg5", "cfg5_b1"])
def test_cfg5_sampled_rows_against_the_oracle(name):
    cfg = workloads.CONFIGS[name]
    w = workloads.make(cfg, device="cuda")
    Y = torch.full((cfg.B, cfg.rows), float("nan"), device="cuda")
    with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
        ex.matvec(w.M, w.X, Y, cfg.tile_bytes)
        ex.check()
        n_cores = ex.cfg.n_cores
    Yh = Y.cpu().numpy()
    assert np.isfinite(Yh).all(), "an output was never written"
    # rows: first and last row of every core's share, both ends of the matrix, and a seeded random sample
    per = cfg.rows // n_cores
    rows = {0, cfg.rows - 1}
    for c in range(n_cores):
        rows.update((c * per, c * per + per - 1))
    rng = np.random.default_rng(cfg.seed)
    rows.update(int(r) for r in rng.integers(0, cfg.rows, 160))
    rows = np.array(sorted(rows))
    Ms = w.M[torch.from_numpy(rows).cuda()].cpu().numpy()
    Yr, Ya = gemv_ref.gemv_dense(Ms, w.X.cpu().numpy())
    assert _worst(Yh[:, rows], Yr, Ya) <= 1.0
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
    """Sampled contexts against the fp64 definition (the first, the last, the longest and the shortest of the batch, one
    by one), and properties that hold for every output: value rows that are all equal come back whatever the weights are,
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
        pick = sorted({0, len(lengths) - 1, int(np.argmax(lengths)), int(np.argmin(lengths))})
        for s in pick:
            a, b = int(ro[s]), int(ro[s + 1])
            Or, Ar, S = attn_ref.attn_decode(Q[s:s + 1].cpu().numpy(), K[a:b].cpu().numpy(), V[a:b].cpu().numpy(), np.array([0, b - a]), d ** -0.5)
            assert np.all(np.abs(Og[s] - Or[0]) <= (2e-5 * S[0] + 2e-5) * Ar[0] + 1e-30), "context %d" % s
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
