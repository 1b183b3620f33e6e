#!/usr/bin/env python3
"""Benchmark of the hot path: one step = one pass of the whole uop graph of the matvec operator
(vdc_matvec: fetch/decode, address generation, slot allocation, tile loads, matvec uops, result stores) over the
resident synthetic inputs of one configuration.  Prints ONE JSON line on stdout; everything else goes to stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg5_b1|cfg3|cfg4|cfg2|cfg1]
    python bench.py --workload attn_0.5k|attn_0.5k_b|attn_64k|attn_rand [--heads 8]     (decode attention, see below)

metric  = matrix elements per second on one GPU (one element = one fp32 matrix entry, each used for B vectors)
roofline = algorithmic HBM bytes of one launch / mean duration of the executor kernel, against 8 TB/s
cpu_baseline = the oracle (plain fp64 C loops, one thread) timed on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published peak HBM3E bandwidth

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the factors a plain copy
# kernel of known size gives): workload -> (bytes, the file under profiles/ that holds the counter runs).  The figure is
# reported only for the exact configuration it was measured on (no --tile-bytes / --slot-bytes / --n-stu / --tile-rows
# override); every other run prints null.
MEASURED_TRAFFIC = {
    "cfg5": (8650709316, "profiles/vdc_executor_kernel_cfg5_hbm_traffic.txt"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(rows, K, B, n_x_rows):
    """Bytes one launch must move through HBM: every matrix entry once, the vectors once, the result once.
    (Vector tiles re-read by other cores come from the L2 / Infinity Cache and are not counted.)"""
    return 4 * rows * K + 4 * n_x_rows * K + 4 * B * rows


# The four regimes of the paper's uneven-context study (Section 6.2, "Dynamic Attention Length"): context rows per request.
ATTN_REGIMES = {
    "attn_0.5k": ("1 x 512", lambda: [512]),
    "attn_0.5k_b": ("64 x 512", lambda: [512] * 64),
    "attn_64k": ("1 x 65536", lambda: [65536]),
    "attn_rand": ("64 x random[256,1024]", lambda: list(np.random.default_rng(2605).integers(256, 1025, 64))),
}


def bench_attention(args):
    """Decode attention with one query per request (vdc_attn_decode) on one regime.  The paper does not say how many
    heads its model has: every request has `heads` key/value heads of 128 values with one query head each, and every
    (request, head) pair is one context of the ragged batch.  One element = one fp32 key or value entry, read once."""
    import torch
    import paper_2605_03190_amd as vdc
    vdc.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    label, make = ATTN_REGIMES[args.workload]
    d = 128
    lengths = np.repeat(make(), args.heads)
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = int(ro[-1])
    tile = args.tile_bytes or 16384
    g = torch.Generator(device="cuda").manual_seed(rows)
    # batches that fit the Infinity Cache are rotated over several copies so that every launch reads from HBM
    n_copies = max(1, min(8, (2 << 30) // (2 * rows * d * 4))) if 2 * rows * d * 4 <= 512 << 20 else 1
    Q = torch.randn((len(lengths), d), device="cuda", generator=g)
    Ks = [torch.randn((rows, d), device="cuda", generator=g) for _ in range(n_copies)]
    Vs = [torch.randn((rows, d), device="cuda", generator=g) for _ in range(n_copies)]
    O = torch.full((len(lengths), d), float("nan"), device="cuda")
    ex = vdc.Executor(slot_bytes=args.slot_bytes or 8192, n_stu=args.n_stu)
    stream = torch.cuda.current_stream()
    for i in range(args.warmup):
        ex.attn_decode(Q, Ks[i % n_copies], Vs[i % n_copies], ro, O, tile, stream=stream)
    ex.check(stream)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(args.steps):
        starts[i].record(stream)
        ex.attn_decode(Q, Ks[i % n_copies], Vs[i % n_copies], ro, O, tile, stream=stream)
        ends[i].record(stream)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_begin
    ex.check(stream)
    kern_ms = [s.elapsed_time(e) for s, e in zip(starts, ends)]
    kern_avg_ms = float(np.mean(kern_ms))
    elements = 2 * rows * d
    alg = 4 * elements + 2 * 4 * len(lengths) * d
    achieved = alg / (kern_avg_ms * 1e-3) / 1e9
    value = elements * args.steps / t_total
    log("%s: %d contexts, %d rows; per step %.4f ms, kernel avg %.4f ms (min %.4f max %.4f)  %.1f GB/s = %.1f%% of %.0f"
        % (args.workload, len(lengths), rows, t_total * 1e3 / args.steps, kern_avg_ms, min(kern_ms), max(kern_ms), achieved,
           100 * achieved / HBM_PEAK_GBS, HBM_PEAK_GBS))
    out = {
        "metric": "decode-attention key/value elements/sec at 1 GPU", "value": value, "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_total * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: decode attention, %s context rows per request, %d heads of %d, fp32, %d KB tiles" % (
            args.workload, label, args.heads, d, tile // 1024), "contexts": len(lengths), "rows": rows, "tile_bytes": tile},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "kernel": "vdc_executor_kernel", "kernel_avg_ms": kern_avg_ms, "algorithmic_bytes": alg},
    }
    if not args.no_cpu_baseline:
        from oracle import attn_ref
        # bounded sample: the leading contexts of the batch, whole, up to about 64K rows
        n = max(1, int(np.searchsorted(ro, 65536, side="right")) - 1)
        last = (args.steps - 1) % n_copies
        r1 = int(ro[n])
        Qh, Kh, Vh = Q[:n].cpu().numpy(), Ks[last][:r1].cpu().numpy(), Vs[last][:r1].cpu().numpy()
        t = time.perf_counter()
        Or, Ar, S = attn_ref.attn_decode(Qh, Kh, Vh, ro[:n + 1], d ** -0.5)
        tc = time.perf_counter() - t
        worst = float((np.abs(O[:n].cpu().numpy() - Or) / ((2e-5 * S[:, None] + 2e-5) * Ar + 1e-30)).max())
        log("oracle sample: %d contexts, %d rows in %.2f s; GPU vs oracle on the sample: error = %.3g of the bound" % (n, r1, tc, worst))
        if worst > 1.0:
            log("PARITY FAILURE on the sampled contexts")
            sys.exit(1)
        out["cpu_baseline"] = {"value": 2 * r1 * d / tc, "unit": "elements/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d of %d contexts (%d rows); fp64 definition in numpy, one thread; %.1f s" % (n, len(lengths), r1, tc)}
    ex.destroy()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--tile-bytes", type=int, default=0, help="override the configuration's tile (I/O block) size: 2048, 4096, 8192 or 16384")
    ap.add_argument("--slot-bytes", type=int, default=0, help="override the configuration's slot size")
    ap.add_argument("--n-stu", type=int, default=0, help="store units per core: 1 or 2 (0: the library's default)")
    ap.add_argument("--tile-rows", type=int, default=0, help="rows per matrix tile (0: the tiler's choice)")
    ap.add_argument("--heads", type=int, default=8, help="attention workloads: key/value heads per request")
    ap.add_argument("--per-launch", action="store_true", help="log the duration of every timed launch (stderr)")
    ap.add_argument("--fixed-warmup", action="store_true", help="exactly --warmup untimed steps, also when the launch times have not settled yet")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run a plain device-to-device copy of MIB mebibytes --steps times: "
                         "the known traffic that the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus %d is not supported. "
            "The number to quote is the one-GPU throughput." % args.gpus)
        sys.exit(2)

    if args.workload in ATTN_REGIMES:
        return bench_attention(args)

    import torch
    import paper_2605_03190_amd as vdc
    import workloads
    vdc.lib()                                  # fails loudly when the HIP extension is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = workloads.CONFIGS[args.workload]
    if args.tile_bytes or args.slot_bytes:
        import dataclasses
        cfg = dataclasses.replace(cfg, tile_bytes=args.tile_bytes or cfg.tile_bytes, slot_bytes=args.slot_bytes or cfg.slot_bytes)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        log("copied %d bytes %d times (each copy reads and writes that many bytes): %.3f ms per copy, %.0f GB/s read + %.0f GB/s written"
            % (n, args.steps, dt * 1e3, n / dt / 1e9, n / dt / 1e9))
        return
    t0 = time.time()
    w = workloads.make(cfg, device=dev)
    rows, K, B = cfg.rows, cfg.K, cfg.B
    ragged = w.row_off is not None
    Y = torch.full((rows,) if ragged else (B, rows), float("nan"), device=dev)
    # configurations whose matrix fits the 256 MB Infinity Cache are rotated over several copies so that every
    # launch reads from HBM ("cold")
    n_copies = 1
    if w.M.numel() * 4 <= 512 << 20:
        n_copies = max(1, min(8, (2 << 30) // (w.M.numel() * 4)))
    Ms = [w.M] + [w.M.clone() for _ in range(n_copies - 1)]
    torch.cuda.synchronize()
    log("inputs: %s rows=%d K=%d B=%d tile=%d ragged=%s copies=%d (%.1f s)" % (cfg.name, rows, K, B, cfg.tile_bytes, ragged, n_copies, time.time() - t0))

    ex = vdc.Executor(slot_bytes=cfg.slot_bytes, n_stu=args.n_stu, tile_rows=args.tile_rows)
    stream = torch.cuda.current_stream()

    # What the memory system gives a plain kernel on the same bytes in this very run ("achievable"): the matrix read
    # once by an ordinary grid-stride kernel of 128-bit loads (vdc_raw_stream, no virtual cores).  Measured before the
    # benchmark proper: about 50 ms of reads, which also takes the clocks out of their idle state (after an idle period
    # the first twenty-odd launches of anything run 5 to 15 % slower, see profiles/).
    m_bytes = w.M.numel() * 4
    n_raw = int(max(10, min(400, 0.05 / (m_bytes / 6.0e12 + 5e-6))))
    for i in range(3):
        ex.raw_stream("read", Ms[i % n_copies], None, m_bytes, stream=stream)
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record(stream)
    for i in range(n_raw):
        ex.raw_stream("read", Ms[i % n_copies], None, m_bytes, stream=stream)
    r1.record(stream)
    r1.synchronize()
    raw_ms = r0.elapsed_time(r1) / n_raw
    achievable = m_bytes / (raw_ms * 1e-3) / 1e9
    log("plain read-stream kernel on the matrix: %.4f ms per pass over %d launches, %.1f GB/s = %.1f%% of %.0f" % (
        raw_ms, n_raw, achievable, 100 * achievable / HBM_PEAK_GBS, HBM_PEAK_GBS))

    # The second reference of Section 6.3 ("Memory virtual core overhead"): the same bytes moved by the executor's own
    # memory uops with nothing to compute behind them (vdc_stream in read mode, same block size).  It is the same
    # kernel as the benchmark's, bound by instruction issue like it, so these launches also bring the shader clock to
    # where the timed launches will hold it.
    vmc_read = None
    vmc_tile = min(cfg.tile_bytes, 2 * cfg.slot_bytes)
    try:
        for i in range(3):
            ex.stream("read", Ms[i % n_copies], None, m_bytes, vmc_tile, stream=stream)
        r0.record(stream)
        for i in range(n_raw):
            ex.stream("read", Ms[i % n_copies], None, m_bytes, vmc_tile, stream=stream)
        r1.record(stream)
        r1.synchronize()
        ex.check(stream)
        vmc_read = m_bytes / (r0.elapsed_time(r1) / n_raw * 1e-3) / 1e9
        log("memory uops alone (read, %d-byte blocks): %.1f GB/s = %.1f%% of %.0f" % (vmc_tile, vmc_read, 100 * vmc_read / HBM_PEAK_GBS, HBM_PEAK_GBS))
    except vdc.VdcError as e:
        log("memory uops alone: not run (%s)" % e)

    def step(i):
        M = Ms[i % n_copies]
        if ragged:
            ex.matvec_ragged(M, w.row_off, w.X, Y, cfg.tile_bytes, stream=stream)
        else:
            ex.matvec(M, w.X, Y, cfg.tile_bytes, stream=stream)

    for i in range(args.warmup):
        step(i)
    ex.check(stream)
    # The first launches of this kernel after any change of load run up to 20 % slower than the later ones (measured:
    # 1.61 ms falling to 1.32 ms over about twenty launches on cfg5, also right after 100 ms of other kernels on the same
    # data; the power management settles the clocks for the new load).  Unless --fixed-warmup is given the warm-up
    # therefore goes on, untimed, until three launches in a row are within 1 % of each other (at most 60 more).
    warmup_done = args.warmup
    if not args.fixed_warmup:
        last = []
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(60):
            e0.record(stream)
            step(args.warmup + i)
            e1.record(stream)
            e1.synchronize()
            last = (last + [e0.elapsed_time(e1)])[-3:]
            warmup_done += 1
            if len(last) == 3 and max(last) <= 1.01 * min(last):
                break
        log("warm-up: %d launches in all, the last three %s ms" % (warmup_done, " ".join("%.4f" % x for x in last)))

    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(args.steps):
        starts[i].record(stream)
        step(i)
        ends[i].record(stream)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_begin
    ex.check(stream)
    kern_ms = [s.elapsed_time(e) for s, e in zip(starts, ends)]
    kern_avg_ms = float(np.mean(kern_ms))
    ms_per_step = t_total * 1e3 / args.steps
    if args.per_launch:
        log("per launch, ms: " + " ".join("%.4f" % x for x in kern_ms))
    elements = rows * K
    value = elements * args.steps / t_total
    alg = algorithmic_bytes(rows, K, B, w.X.shape[0])
    achieved = alg / (kern_avg_ms * 1e-3) / 1e9
    log("steps=%d total=%.3f ms  per step %.4f ms  kernel avg %.4f ms (min %.4f max %.4f)  %.3e elements/s  %.1f GB/s = %.1f%% of %.0f"
        % (args.steps, t_total * 1e3, ms_per_step, kern_avg_ms, min(kern_ms), max(kern_ms), value, achieved,
           100 * achieved / HBM_PEAK_GBS, HBM_PEAK_GBS))

    overridden = bool(args.tile_bytes or args.slot_bytes or args.n_stu or args.tile_rows)
    traffic, traffic_source = (None, None) if overridden else MEASURED_TRAFFIC.get(cfg.name, (None, None))
    out = {
        "metric": "hot-path matrix elements/sec at 1 GPU",
        "value": value,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "warmup_done": warmup_done,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %s %dx%d fp32, B=%d, %d KB tiles, %d KB slots, seed %d" % (
            cfg.name, "ragged %d segments" % cfg.n_seg if ragged else "dense", rows, K, B, cfg.tile_bytes // 1024,
            cfg.slot_bytes // 1024, cfg.seed), "rows": rows, "K": K, "B": B, "tile_bytes": cfg.tile_bytes},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "vdc_executor_kernel", "kernel_avg_ms": kern_avg_ms, "algorithmic_bytes": alg,
                     "achievable": achievable, "achievable_kernel": "raw_stream_kernel<read> (plain 128-bit loads, same matrix, same run)",
                     "frac_of_achievable": achieved / achievable, "memory_uops_alone": vmc_read},
    }

    if not args.no_cpu_baseline:
        from oracle import gemv_ref
        gemv_ref.build()
        # bounded sample: the first rows of the matrix (of the first segments when ragged), all K columns, all B vectors
        Xh = w.X.cpu().numpy()
        probe = min(rows, 64)

        def run_oracle(n):
            Mh = w.M[:n].cpu().numpy()
            t = time.perf_counter()
            if ragged:
                ro = np.minimum(w.row_off, n)
                Yr, Ya = gemv_ref.gemv_ragged(Mh, ro, Xh)
            else:
                Yr, Ya = gemv_ref.gemv_dense(Mh, Xh)
            return time.perf_counter() - t, Yr, Ya

        tp, _, _ = run_oracle(probe)
        n = int(min(rows, max(probe, probe * args.cpu_seconds / max(tp, 1e-6))))
        if not ragged:
            n = max(probe, n // 64 * 64)
        tc, Yr, Ya = run_oracle(n)
        Yg = Y[:n].cpu().numpy() if ragged else Y[:, :n].cpu().numpy()
        worst = float((np.abs(Yg - Yr) / (1e-5 * Ya + 1e-30)).max())
        log("oracle sample: %d rows in %.2f s -> %.3e elements/s; GPU vs oracle on the sample: error = %.3g of the bound" % (n, tc, n * K / tc, worst))
        if worst > 1.0:
            log("PARITY FAILURE on the sampled rows")
            sys.exit(1)
        out["cpu_baseline"] = {"value": n * K / tc, "unit": "elements/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d of %d rows, all %d columns, B=%d; plain fp64 C loops, one thread; %.1f s" % (n, rows, K, B, tc)}
        if not ragged:
            # the same oracle on all the host cores this process may use: the sample's rows split into one block per
            # thread (the C loops run outside the interpreter lock); a second line of the baseline, not a tuned kernel
            import concurrent.futures
            cores = max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)))
            n_all = min(rows, n * cores) // (64 * cores) * (64 * cores)
            if cores > 1 and n_all >= 64 * cores:
                Mh = w.M[:n_all].cpu().numpy()
                blk = n_all // cores
                t = time.perf_counter()
                with concurrent.futures.ThreadPoolExecutor(cores) as pool:
                    parts = list(pool.map(lambda i: gemv_ref.gemv_dense(Mh[i * blk:(i + 1) * blk], Xh), range(cores)))
                ta = time.perf_counter() - t
                Yall = np.concatenate([p_[0] for p_ in parts], axis=1)
                Aall = np.concatenate([p_[1] for p_ in parts], axis=1)
                worst_all = float((np.abs(Y[:, :n_all].cpu().numpy() - Yall) / (1e-5 * Aall + 1e-30)).max())
                log("oracle on %d threads: %d rows in %.2f s -> %.3e elements/s; GPU vs oracle: error = %.3g of the bound" % (cores, n_all, ta, n_all * K / ta, worst_all))
                if worst_all > 1.0:
                    log("PARITY FAILURE on the rows of the all-cores sample")
                    sys.exit(1)
                out["cpu_baseline_all_cores"] = {"value": n_all * K / ta, "unit": "elements/s", "cores": cores, "kind": "oracle",
                                                 "sample": "first %d of %d rows in %d row blocks, one thread each; plain fp64 C loops; %.1f s" % (n_all, rows, cores, ta)}
    ex.destroy()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
