"""Memory uops alone, by I/O block size, against plain load/store instructions (on the GPU).

    python -m paper_2605_03190_amd.vmc_sweep [--mib 4096] [--steps 5]

The measurement of Section 6.3 ("Memory virtual core overhead") on this machine: a byte range is read, filled or
copied once by memory uops of a given block size with nothing to compute behind them (vdc_stream), and once by an
ordinary grid-stride kernel of 128-bit loads and stores (vdc_raw_stream).  The ratio says at which block size the cost
of the virtual memory core is amortised.  A slot is as large as the block, up to 8 KB, so that small blocks do not
waste local memory.  Rates count the bytes of the range once for read and fill, twice (read + written) for copy.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

TILES = [256, 512, 1024, 2048, 4096, 8192, 16384, 32768]
MODES = ["read", "fill", "copy"]
HBM_PEAK_GBS = 8000.0


def time_ms(fn, steps, warmup=2):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b))
    ts.sort()
    return ts[len(ts) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=4096, help="size of the range in MiB")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--n-stu", type=int, default=0, help="store units per core: 1 or 2 (0: the library's default)")
    args = ap.parse_args()
    import torch
    import paper_2605_03190_amd as vdc

    nbytes = args.mib << 20
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    moved = {"read": nbytes, "fill": nbytes, "copy": 2 * nbytes}
    raw = {}
    with vdc.Executor() as ex:
        for mode in MODES:
            s, d = (src if mode != "fill" else None), (dst if mode != "read" else None)
            ms = time_ms(lambda: ex.raw_stream(mode, s, d, nbytes, value=7), args.steps)
            raw[mode] = moved[mode] / ms / 1e6
    print("range %d MiB, median of %d runs; GB/s (fraction of the plain kernel's rate)" % (args.mib, args.steps))
    print("%-12s" % "block" + "".join("%22s" % m for m in MODES))
    print("%-12s" % "plain kernel" + "".join("%15.0f (%3.0f%%)" % (raw[m], 100.0 * raw[m] / HBM_PEAK_GBS) for m in MODES) + "   (of 8 TB/s)")
    for T in TILES:
        slot = max(1024, min(T, 8192))
        row = "%-12s" % ("%d B" % T)
        with vdc.Executor(slot_bytes=slot, n_stu=args.n_stu) as ex:
            for mode in MODES:
                s, d = (src if mode != "fill" else None), (dst if mode != "read" else None)
                try:
                    ex.stream(mode, s, d, nbytes, T, value=7)
                    ex.check()
                except vdc.VdcError as e:
                    row += "%22s" % "n/a"
                    continue
                ms = time_ms(lambda: ex.stream(mode, s, d, nbytes, T, value=7), args.steps)
                ex.check()
                rate = moved[mode] / ms / 1e6
                row += "%15.0f (%3.0f%%)" % (rate, 100.0 * rate / raw[mode])
        print(row, flush=True)


if __name__ == "__main__":
    main()
