"""Graphs streamed to resident cores against a launch per graph (on the GPU).

    python -m paper_2605_03190_amd.resident_bench [--graphs 200] [cfg1 cfg2 cfg3 ...]

Section 4.3 launches the virtual cores once and streams uop graphs to them.  For each workload the same matvec graph is run
`--graphs` times back to back, once as that many vdc_run calls queued on one stream (a kernel launch per graph) and once
posted to the resident cores (vdc_resident_submit), and the time per graph is printed for both, host clock from the first
call to the completion of the last graph.
"""
import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workloads", nargs="*", default=["cfg1", "cfg2", "cfg3"])
    ap.add_argument("--graphs", type=int, default=200)
    args = ap.parse_args()
    import torch
    import paper_2605_03190_amd as vdc
    import workloads

    print("%-8s %22s %22s %8s" % ("workload", "launch per graph (us)", "resident cores (us)", "ratio"))
    for name in args.workloads:
        cfg = workloads.CONFIGS[name]
        w = workloads.make(cfg, device="cuda")
        Y = torch.zeros((cfg.B, cfg.rows), device="cuda")
        with vdc.Executor(slot_bytes=cfg.slot_bytes) as ex:
            words, sb, descs = ex.matvec_program(cfg.rows, cfg.K, cfg.K, cfg.B, cfg.tile_bytes)
            ws = ex.matvec_workspace(cfg.rows, cfg.K, cfg.K, cfg.B, cfg.tile_bytes)
            sizes = [w.M.numel() * 4, w.X.numel() * 4, Y.numel() * 4] + ([ws.nbytes] if ws.size else [])
            prog = ex.program_create(words, sb, descs, sizes)
            tensors = [w.M, w.X, Y] + ([torch.from_numpy(ws).cuda()] if ws.size else [])
            for _ in range(20):
                ex.run(prog, tensors)
            ex.check()
            t0 = time.perf_counter()
            for _ in range(args.graphs):
                ex.run(prog, tensors)
            ex.check()
            t_launch = (time.perf_counter() - t0) / args.graphs * 1e6
            ex.resident_start(idle_ms=1000)
            for _ in range(20):
                t = ex.resident_submit(prog, tensors)
            rc, info = ex.resident_wait(t)
            assert rc == vdc.VDC_OK, (rc, info)
            t0 = time.perf_counter()
            for _ in range(args.graphs):
                t = ex.resident_submit(prog, tensors)
            rc, info = ex.resident_wait(t)
            t_res = (time.perf_counter() - t0) / args.graphs * 1e6
            assert rc == vdc.VDC_OK, (rc, info)
            ex.resident_stop()
        print("%-8s %22.2f %22.2f %8.2f" % (name, t_launch, t_res, t_launch / t_res), flush=True)


if __name__ == "__main__":
    main()
