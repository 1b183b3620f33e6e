"""The adaptive tiling step on the GPU: dense matvecs whose row-block count does not fill the compute cores evenly, run with
every cut of K the builder offers (sched_force_parts) and with the cut the scheduler takes from its cost model.

    python -m paper_2605_03190_amd.sched_bench [--steps 30]

Per shape: microseconds (median) per forced cut S of all row blocks, and (second line) of the surplus row blocks alone
where the shape has a surplus; the scheduler's choice (S, and "s" when it cuts the surplus only), its time, what the choice
gains over the uncut operator, how it compares with the best forced cut, and the host time of the scheduling step.  Matrices that fit the last-level cache are rotated over several copies so that every run reads from
memory.  Results are checked against a float64 product of a few rows on the host.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

CASES = [  # rows, K, B, tile_bytes
    (12288, 8192, 1, 16384),
    (10240, 8192, 1, 16384),
    (9216, 16384, 1, 16384),
    (20480, 8192, 1, 16384),
    (14336, 4096, 1, 16384),
    (4096, 14336, 1, 16384),
    (1024, 16384, 1, 16384),
    (2048, 2048, 1, 16384),
    (8192, 8192, 1, 8192),
    (12288, 8192, 8, 16384),
    (8192, 8192, 8, 16384),
    (24576, 16384, 8, 16384),
]


def time_us(fn, steps):
    import torch
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b) * 1e3)
    return sorted(ts)[len(ts) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=30)
    args = ap.parse_args()
    import torch
    import paper_2605_03190_amd as vdc

    import time
    forced = [1, 2, 3, 4, 6, 8, 12, 16]
    print("median of %d runs, microseconds; S = ranges K is cut into; '-' = the builder does not offer the cut" % args.steps)
    print("%-22s %2s %6s %5s %4s | %s | %6s %8s %7s %7s %9s" % ("rows x K", "B", "tile", "NB", "nk", " ".join("S=%-5d" % s for s in forced),
                                                            "chosen", "us", "vs S=1", "vs best", "sched us"))
    auto = vdc.Executor()
    for rows, K, B, tile in CASES:
        g = torch.Generator(device="cuda").manual_seed(rows + K)
        n_copies = max(1, min(6, (1 << 30) // (rows * K * 4)))
        Ms = [torch.randn(rows, K, device="cuda", generator=g) * K ** -0.5 for _ in range(n_copies)]
        X = torch.randn(B, K, device="cuda", generator=g)
        Y = torch.full((B, rows), float("nan"), device="cuda")
        t0 = time.perf_counter()
        R, Kt, NB, nk, s_max, s_auto, tail_auto = auto.matvec_tiling(rows, K, B, tile)
        t_sched = (time.perf_counter() - t0) * 1e6
        sample = torch.arange(0, rows, max(1, rows // 61), device="cuda")
        want = (X.double() @ Ms[0][sample].double().T).float()
        turn = [0]

        def check(ex):
            Y.fill_(float("nan"))
            ex.matvec(Ms[0], X, Y, tile)
            ex.check()
            assert not torch.isnan(Y).any()
            err = float((Y[:, sample] - want).abs().max())
            assert err < 1e-3, err

        def run_on(ex):
            def fn():
                turn[0] += 1
                ex.matvec(Ms[turn[0] % n_copies], X, Y, tile)
            return fn

        lanes = 2 * auto.cfg.n_cores
        has_surplus = NB > lanes and NB % lanes != 0 and s_max >= 2
        times, times_s = {}, {}
        for fam, out in ((0, times), (100, times_s)):
            if fam and not has_surplus:
                continue
            for s in forced:
                if s > s_max or (fam and s == 1):
                    continue
                with vdc.Executor(sched_force_parts=fam + s) as ex:
                    assert ex.matvec_tiling(rows, K, B, tile)[5:] == (s, (NB % lanes if fam else 0) if s > 1 else 0)
                    check(ex)
                    out[s] = time_us(run_on(ex), args.steps)
                    ex.check()
        check(auto)
        t_auto = time_us(run_on(auto), args.steps)
        auto.check()
        cells = " ".join(("%-7.1f" % times[s]) if s in times else "%-7s" % "-" for s in forced)
        best = min(list(times.values()) + list(times_s.values()))
        print("%-22s %2d %6d %5d %4d | %s | %6s %8.1f %6.2fx %6.2fx %9.0f" % ("%d x %d" % (rows, K), B, tile, NB, nk, cells,
                                                                           "%d%s" % (s_auto, "s" if tail_auto else ""), t_auto,
                                                                           times[1] / t_auto, best / t_auto, t_sched), flush=True)
        if times_s:
            cells = " ".join(("%-7.1f" % times_s[s]) if s in times_s else "%-7s" % "-" for s in forced)
            print("%-22s %2s %6s %5d %4s | %s |" % ("  surplus blocks alone", "", "", NB % lanes, "", cells), flush=True)
        del Ms, X, Y
    auto.destroy()


if __name__ == "__main__":
    main()
