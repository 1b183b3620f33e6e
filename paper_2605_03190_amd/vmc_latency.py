"""Runtime latency metrics of the virtual memory core and an ablation of its issue path (on the GPU).

    python -m paper_2605_03190_amd.vmc_latency [--uops 4096] [--steps 7] [--no-ablation]

The runtime table of Section 6.3 ("Memory virtual core overhead") on this machine, with every figure taken from whole
launches timed by HIP events (median of --steps), so that nothing is instrumented:

  start-up latency      the launch of a graph whose streams hold nothing but HALT (cores start, find nothing to do, drain
                        and leave) and of a graph with one 1 KB load per compute core (the first uop through the whole
                        path: fetch, decode, allocation, dispatch, load, delivery, hand-back); their difference is what
                        the first uop adds
  uop interval          what a memory core spends per uop in the steady state: duration of a long graph of small memory
                        uops / uops per core.  load = 1 KB reads handed to a compute core that drops them, store = 1 KB
                        regions filled by a compute core and written back, control = a loop of ADD uops on the front end
                        alone; "initiation interval" = the load figure at the smallest block (256 B), where nothing but
                        the issue path is left
  ablation              the load figure with 1, 2 and 4 load units, with the front end held to 1, 2, 4 or 8 memory uops
                        per dispatch (issue_batch) and with or without its replay of decoded loop bodies (issue_flags)

Clock: the figures are wall-clock nanoseconds; cycles are quoted at the 2.4 GHz the chip is specified with.
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

GHZ = 2.4
OP_HALT, OP_LOOP, OP_REPEAT, OP_ADD = 0, 1, 2, 3


def word(opcode, acc=0, imm=0):
    """A control uop in the library's 16-byte layout (include/vdcores.h names the file that defines it)."""
    q = imm & ((1 << 48) - 1)
    return (opcode | (acc << 22), 0, q & 0xFFFFFFFF, q >> 32)


def median_ms(fn, steps, warmup=3):
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
    return float(np.median(ts))


def control_program(ex, trips, adds):
    """Every memory core runs LOOP trips { ADD x adds } REPEAT; the compute cores halt at once."""
    V = ex.cfg.vcc_per_core
    words, sb = [], [0]
    for _ in range(ex.cfg.n_cores):
        words += [word(OP_LOOP, imm=trips)] + [word(OP_ADD, acc=1, imm=16)] * adds + [word(OP_REPEAT, acc=0, imm=0), word(OP_HALT)]
        sb.append(len(words))
        for _ in range(V):
            words.append(word(OP_HALT))
            sb.append(len(words))
    return ex.program_create(np.array(words, dtype=np.uint32), np.array(sb, dtype=np.uint32), np.array([[0, 1, 16, 16, 16, 0, 0, 0]], dtype=np.uint32), [16])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--uops", type=int, default=4096, help="memory uops per core in the steady-state graphs")
    ap.add_argument("--steps", type=int, default=7)
    ap.add_argument("--no-ablation", action="store_true")
    args = ap.parse_args()
    import torch
    import paper_2605_03190_amd as vdc

    assert torch.cuda.is_available(), "vmc_latency needs a GPU"
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")

    def per_uop_ns(ex, mode, block, src, dst):
        """Steady state: ns per memory uop and core."""
        nbytes = args.uops * ex.cfg.n_cores * block
        s, d = (src if mode != "fill" else None), (dst if mode != "read" else None)
        ex.stream(mode, s, d, nbytes, block, value=7)
        ex.check()
        ms = median_ms(lambda: ex.stream(mode, s, d, nbytes, block, value=7), args.steps)
        ex.check()
        return ms * 1e6 / args.uops

    cap = args.uops * 256 * 1024
    src = torch.randint(0, 256, (cap,), dtype=torch.uint8, device="cuda")
    dst = torch.empty(cap, dtype=torch.uint8, device="cuda")
    print("Runtime latency metrics of the virtual memory core (median of %d launches; %d uops per core in the steady-state graphs)" % (args.steps, args.uops))
    with vdc.Executor(slot_bytes=1024) as ex:
        nc, V = ex.cfg.n_cores, ex.cfg.vcc_per_core
        halt = np.array([word(OP_HALT)] * (nc * (1 + V)), dtype=np.uint32)
        empty = ex.program_create(halt, np.arange(nc * (1 + V) + 1, dtype=np.uint32), np.array([[0, 1, 16, 16, 16, 0, 0, 0]], dtype=np.uint32), [16])
        t_empty = median_ms(lambda: ex.run(empty, [dummy]), args.steps) * 1e3
        ex.check()
        one = nc * V * 1024                                  # one 1 KB block per compute core
        t_first = median_ms(lambda: ex.stream("read", src, None, one, 1024), args.steps) * 1e3
        ex.check()
        print("%-58s %8.2f us" % ("start-up: launch of an empty graph (start, drain, leave)", t_empty))
        print("%-58s %8.2f us   (%+.2f us for the first uop)" % ("start-up: launch of a graph with one 1 KB load per compute core", t_first, t_first - t_empty))
        trips, adds = 20000, 6
        ctl = control_program(ex, trips, adds)
        t_ctl = median_ms(lambda: ex.run(ctl, [dummy]), args.steps) * 1e6
        ex.check()
        ns_ctl = (t_ctl - t_empty * 1e3) / (trips * (adds + 1))
        ld1k = per_uop_ns(ex, "read", 1024, src, dst)
        st1k = per_uop_ns(ex, "fill", 1024, src, dst)
    with vdc.Executor(slot_bytes=1024) as ex:
        ii = per_uop_ns(ex, "read", 256, src, dst)
    rows = [("uop initiation interval (256 B loads, per core)", ii), ("average memory load uop (1 KB, per core)", ld1k),
            ("average memory store uop (1 KB, per core)", st1k), ("average control uop (front end alone)", ns_ctl)]
    for name, ns in rows:
        print("%-58s %8.1f ns   (%5.0f cycles at %.1f GHz)" % (name, ns, ns * GHZ, GHZ))
    if args.no_ablation:
        return
    print()
    print("Issue-path ablation: ns per 1 KB load uop and core (reads handed to a compute core that drops them)")
    print("%-34s" % "load units x uops per dispatch" + "".join("%10s" % ("batch %d" % b) for b in (1, 2, 4, 8)))
    for n_ldu in (1, 2, 4):
        for flags, label in ((0, "loop bodies replayed"), (1, "every trip decoded again")):
            line = "%-34s" % ("%d load unit%s, %s" % (n_ldu, "s" if n_ldu > 1 else "", label))
            for batch in (1, 2, 4, 8):
                with vdc.Executor(slot_bytes=1024, n_ldu=n_ldu, issue_batch=batch, issue_flags=flags) as ex:
                    line += "%10.1f" % per_uop_ns(ex, "read", 1024, src, dst)
            print(line, flush=True)


if __name__ == "__main__":
    main()
