"""The resident form of the executor (Section 4.3: the virtual cores are launched once and uop graphs are streamed to them).

Graphs that go through one resident launch give, bit for bit, what the same graphs give as separate launches, also when a
graph reads what the one before wrote and when graphs use depId counters; the cores leave by themselves when the host posts
nothing (the wait is forced to end from the host, by a small idle limit), after a graph that ended in an error (forced by a
spin limit of two polls), and on vdc_resident_stop; calls that do not fit the state are refused.  Every kernel in this file
exits normally.
"""
import time

import numpy as np
import pytest
import torch

import paper_2605_03190_amd as vdc
from oracle import gemv_ref

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _graph(ex, rows, K, B, tile, M, X, Y):
    """A matvec program and its tensors (with the workspace of a program that is also cut along K)."""
    words, sb, descs = ex.matvec_program(rows, K, K, B, tile)
    ws = ex.matvec_workspace(rows, K, K, B, tile)
    sizes = [rows * K * 4, B * K * 4, B * rows * 4] + ([ws.nbytes] if ws.size else [])
    prog = ex.program_create(words, sb, descs, sizes)
    tensors = [M, X, Y] + ([_dev(ws)] if ws.size else [])
    return prog, tensors


def test_graphs_streamed_to_resident_cores_equal_separate_launches():
    """Twelve graphs (more than the mailbox holds) from five programs, each with an output buffer of its own; two of them read
    what the graph before them wrote; two programs use depId counters and a workspace, which every run must find clean.  The
    results are read after the cores have left (while they are up, other work of the process on the GPU may wait for them)."""
    rng = np.random.default_rng(2605)
    shapes = [(2048, 4096, 8, 16384), (1000, 1000, 1, 4096), (64, 65536, 1, 16384), (70000, 128, 2, 8192), (512, 2048, 8, 8192),
              (300, 2048, 8, 8192)]              # the last one takes its vectors from a result of the first
    order = [0, 5, 1, 2, 3, 4, 2, 0, 5, 1, 3, 2]
    with vdc.Executor() as ex:
        progs, mats, vecs = [], [], []
        for (rows, K, B, tile) in shapes:
            mats.append(_dev(rng.standard_normal((rows, K)).astype(np.float32)))
            vecs.append(_dev(rng.standard_normal((B, K)).astype(np.float32)))
            words, sb, descs = ex.matvec_program(rows, K, K, B, tile)
            ws = ex.matvec_workspace(rows, K, K, B, tile)
            sizes = [rows * K * 4, B * K * 4, B * rows * 4] + ([ws.nbytes] if ws.size else [])
            progs.append((ex.program_create(words, sb, descs, sizes), [_dev(ws)] if ws.size else []))

        def jobs():
            """(program, tensors) per graph of `order`, every graph with a fresh output buffer."""
            out, last0 = [], None
            for g in order:
                rows, K, B, tile = shapes[g]
                Y = torch.full((B, rows), float("nan"), device="cuda")
                X = last0 if g == 5 else vecs[g]
                if g == 0:
                    last0 = Y
                out.append((progs[g][0], [mats[g], X, Y] + progs[g][1]))
            return out

        ref_jobs, res_jobs = jobs(), jobs()
        torch.cuda.synchronize()
        for prog, tensors in ref_jobs:                       # separate launches
            ex.run(prog, tensors)
            ex.check()
        assert ex.resident_state() == (0, 0)
        ex.resident_start(idle_ms=1000)                      # the same graphs through one resident launch
        tickets = [ex.resident_submit(prog, tensors) for prog, tensors in res_jobs]
        assert tickets == list(range(1, len(order) + 1))
        for t in (tickets[3], tickets[-1], tickets[0]):
            rc, info = ex.resident_wait(t)
            assert rc == vdc.VDC_OK, (rc, info)
        assert ex.resident_state() == (1, len(order))
        ex.resident_stop()
        assert ex.resident_state()[0] == 0
        for i, ((_, a), (_, b)) in enumerate(zip(ref_jobs, res_jobs)):
            ya, yb = a[2].cpu().numpy(), b[2].cpu().numpy()
            assert not np.isnan(ya).any()
            assert np.array_equal(ya, yb), "graph %d (shape %d) differs from its separate launch" % (i, order[i])
        # and the executor is back in its ordinary state
        prog, tensors = res_jobs[2]
        tensors[2].fill_(float("nan"))
        ex.run(prog, tensors)
        ex.check()
        assert np.array_equal(tensors[2].cpu().numpy(), ref_jobs[2][1][2].cpu().numpy())


def test_resident_cores_leave_by_themselves_when_the_host_goes_quiet():
    rng = np.random.default_rng(3)
    M = rng.standard_normal((1024, 1024)).astype(np.float32)
    X = rng.standard_normal((2, 1024)).astype(np.float32)
    dM, dX = _dev(M), _dev(X)
    dY = torch.full((2, 1024), float("nan"), device="cuda")
    with vdc.Executor() as ex:
        prog, tensors = _graph(ex, 1024, 1024, 2, 8192, dM, dX, dY)
        ex.resident_start(idle_ms=20)
        t = ex.resident_submit(prog, tensors)
        rc, info = ex.resident_wait(t)
        assert rc == vdc.VDC_OK, (rc, info)
        t0 = time.time()
        while ex.resident_state()[0] != 2 and time.time() - t0 < 10.0:
            time.sleep(0.01)
        assert ex.resident_state() == (2, 1), "the cores did not leave on their own"
        with pytest.raises(vdc.VdcError) as e:
            ex.resident_submit(prog, tensors)
        assert e.value.code == vdc.VDC_ESTATE
        ex.resident_stop()
        Yr, Ya = gemv_ref.gemv_dense(M, X)
        assert np.all(np.abs(dY.cpu().numpy() - Yr) <= 1e-5 * Ya)
        # a new residency on the same executor
        dY.fill_(float("nan"))
        ex.resident_start(idle_ms=1000)
        rc, info = ex.resident_wait(ex.resident_submit(prog, tensors))
        assert rc == vdc.VDC_OK, (rc, info)
        ex.resident_stop()
        assert np.all(np.abs(dY.cpu().numpy() - Yr) <= 1e-5 * Ya)


def test_a_graph_that_ends_in_an_error_ends_the_residency():
    """A spin limit of two polls, far below the latency of a tile load: the graph's units give up, the error comes back
    through vdc_resident_wait, the cores leave, and the executor works again afterwards."""
    dM = torch.zeros((4096, 4096), device="cuda")
    dX = torch.ones((1, 4096), device="cuda")
    dY = torch.zeros((1, 4096), device="cuda")
    with vdc.Executor(watchdog_spins=2) as ex:
        prog, tensors = _graph(ex, 4096, 4096, 1, 8192, dM, dX, dY)
        ex.resident_start(idle_ms=1000)
        t = ex.resident_submit(prog, tensors)
        rc, info = ex.resident_wait(t)
        assert rc == vdc.VDC_EDEADLOCK, (rc, info)
        t0 = time.time()
        while ex.resident_state()[0] != 2 and time.time() - t0 < 10.0:
            time.sleep(0.01)
        assert ex.resident_state()[0] == 2
        ex.resident_stop()
        rc, info = ex.sync_status()
        assert rc == vdc.VDC_OK
    with vdc.Executor() as ex:
        ex.matvec(dM, dX, dY, 8192)
        ex.check()


def test_resident_calls_that_do_not_fit_the_state_are_refused():
    dM = torch.zeros((256, 256), device="cuda")
    dX = torch.ones((1, 256), device="cuda")
    dY = torch.zeros((1, 256), device="cuda")
    with vdc.Executor() as ex:
        prog, tensors = _graph(ex, 256, 256, 1, 4096, dM, dX, dY)
        with pytest.raises(vdc.VdcError) as e:
            ex.resident_submit(prog, tensors)
        assert e.value.code == vdc.VDC_ESTATE
        with pytest.raises(vdc.VdcError) as e:
            ex.resident_stop()
        assert e.value.code == vdc.VDC_ESTATE
        ex.resident_start(idle_ms=1000)
        with pytest.raises(vdc.VdcError) as e:
            ex.resident_start()
        assert e.value.code == vdc.VDC_ESTATE
        with pytest.raises(vdc.VdcError) as e:
            ex.run(prog, tensors)
        assert e.value.code == vdc.VDC_ESTATE
        assert vdc.lib().vdc_program_destroy(prog.handle) == vdc.VDC_ESTATE
        with pytest.raises(vdc.VdcError) as e:                    # programs are created before the cores go resident
            _graph(ex, 256, 256, 1, 4096, dM, dX, dY)
        assert e.value.code == vdc.VDC_ESTATE
        assert ex.resident_wait(5)[0] == vdc.VDC_ESTATE          # never posted
        ex.resident_stop()                                        # no graph at all: the cores just leave
        ex.run(prog, tensors)
        ex.check()
        assert float(dY.sum()) == 0.0
