"""The entry point that allocates nothing on the device (vdc_matvec_noalloc): its results against vdc_matvec's and the
oracle's, on calls in a row that share the static scratch array, the later ones with smaller inputs.  Collected last
on purpose: a failure here must not hide the tests of the hot path proper."""
import ctypes

import numpy as np
import pytest

import paper_2605_03190_amd as vdc
from oracle import gemv_ref

pytestmark = pytest.mark.gpu


def _case(torch, rows, K, B, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    M = torch.randn((rows, K), device="cuda", generator=g)
    X = torch.randn((B, K), device="cuda", generator=g)
    return M, X


def _raw_noalloc(ex, M, X, Y, tile, stream):
    """The C ABI itself, not the binding's wrapper."""
    rows, ld = M.shape
    B, K = X.shape
    return vdc.lib().vdc_matvec_noalloc(ex.handle, ctypes.c_void_p(M.data_ptr()), rows, K, ld, ctypes.c_void_p(X.data_ptr()),
                                        ctypes.c_void_p(Y.data_ptr()), B, tile, ctypes.c_void_p(stream.cuda_stream or 0))


def test_noalloc_matches_matvec_on_calls_that_share_the_scratch():
    import torch
    stream = torch.cuda.current_stream()
    # (rows, K, B, tile): the first is cut along K as well (few row blocks: partial sums through the workspace and depId
    # counters, all of which live in the scratch array), then a smaller one of the same kind, then a plain one, then
    # the first again (rebuilt over what the others left), twice (the second time the program is reused in place)
    shapes = [(256, 16384, 2, 8192), (64, 4096, 1, 8192), (1000, 1500 // 4 * 4, 4, 8192), (256, 16384, 2, 8192), (256, 16384, 2, 8192)]
    with vdc.Executor() as ex:
        for i, (rows, K, B, tile) in enumerate(shapes):
            M, X = _case(torch, rows, K, B, 100 + i)
            Yn = torch.full((B, rows), float("nan"), device="cuda")
            Ym = torch.full((B, rows), float("nan"), device="cuda")
            rc = _raw_noalloc(ex, M, X, Yn, tile, stream)
            assert rc == vdc.VDC_OK, (i, vdc.strerror(rc))
            ex.check(stream)
            ex.matvec(M, X, Ym, tile, stream=stream)
            ex.check(stream)
            yn, ym = Yn.cpu().numpy(), Ym.cpu().numpy()
            # the same program on the same kernels: the two entry points agree to the bit
            assert np.array_equal(yn, ym), "call %d: %s differs from vdc_matvec" % (i, (rows, K, B, tile))
            Yr, Ya = gemv_ref.gemv_dense(M.cpu().numpy(), X.cpu().numpy())
            assert np.all(np.abs(yn - Yr) <= 1e-5 * Ya), "call %d against the oracle" % i


def test_noalloc_two_executors_take_turns_on_one_stream():
    """The array is per GPU, not per executor: another executor's call replaces the program, and the first executor's
    next call must notice and put its own back."""
    import torch
    stream = torch.cuda.current_stream()
    with vdc.Executor() as a, vdc.Executor(slot_bytes=4096) as b:
        M1, X1 = _case(torch, 128, 8192, 1, 7)
        M2, X2 = _case(torch, 96, 2048, 3, 8)
        for rnd in range(2):
            for ex, (M, X), tile in ((a, (M1, X1), 8192), (b, (M2, X2), 4096)):
                B, rows = X.shape[0], M.shape[0]
                Y = torch.full((B, rows), float("nan"), device="cuda")
                assert _raw_noalloc(ex, M, X, Y, tile, stream) == vdc.VDC_OK
                ex.check(stream)
                Yr, Ya = gemv_ref.gemv_dense(M.cpu().numpy(), X.cpu().numpy())
                assert np.all(np.abs(Y.cpu().numpy() - Yr) <= 1e-5 * Ya), (rnd, tile)


def test_noalloc_refuses_what_does_not_fit_and_leaves_the_output_alone():
    import torch
    stream = torch.cuda.current_stream()
    with vdc.Executor() as ex:
        # some dense shape whose program image is larger than the array (many row blocks per core in unrolled form)
        big = None
        for rows, K, B, tile in [(32768, 512, 1, 8192), (16384, 1024, 1, 4096), (8192, 2048, 1, 2048)]:
            w, sb, d = ex.matvec_program(rows, K, K, B, tile)
            if w.nbytes + sb.nbytes + d.nbytes > vdc.NOALLOC_SCRATCH_BYTES - 16384:
                big = (rows, K, B, tile)
                break
        assert big is not None, "no test shape exceeds the scratch array any more: pick a larger one"
        rows, K, B, tile = big
        M, X = _case(torch, rows, K, B, 5)
        Y = torch.full((B, rows), 7.0, device="cuda")
        rc = _raw_noalloc(ex, M, X, Y, tile, stream)
        assert rc == vdc.VDC_ETOOBIG and "scratch" in vdc.strerror(rc)
        torch.cuda.synchronize()
        assert bool((Y == 7.0).all())
        # bad arguments are refused as by vdc_matvec
        assert _raw_noalloc(ex, M, X, Y, 1000, stream) == vdc.VDC_EINVAL
        # and the call after a refusal works
        M, X = _case(torch, 64, 4096, 1, 6)
        Y = torch.full((1, 64), float("nan"), device="cuda")
        assert _raw_noalloc(ex, M, X, Y, 8192, stream) == vdc.VDC_OK
        ex.check(stream)
        Yr, Ya = gemv_ref.gemv_dense(M.cpu().numpy(), X.cpu().numpy())
        assert np.all(np.abs(Y.cpu().numpy() - Yr) <= 1e-5 * Ya)
