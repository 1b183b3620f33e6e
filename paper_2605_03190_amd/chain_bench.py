"""A chain of matvec layers as one uop graph against the same layers as separate launches (on the GPU).

    python -m paper_2605_03190_amd.chain_bench [--steps 30]

Y_0 = M_0 X, Y_l = M_l Y_(l-1): vdc_matvec_chain runs all layers in one launch, every layer starting on a vector tile
as soon as the row blocks of the layer before that produce it have been stored (depId dependencies between memory
uops); the comparison runs one vdc_matvec per layer on the same stream, with a kernel boundary between layers.
Weights are seeded standard-normal fp32 scaled by 1/sqrt(K); the bytes counted are the weights, read once.
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

CASES = [  # dims = (K_0, rows_0, ...), B
    ((2048,) * 9, 1),
    ((4096,) * 9, 1),
    ((4096, 14336, 4096, 14336, 4096), 1),
    ((8192,) * 5, 1),
    ((8192,) * 5, 8),
    ((16384,) * 5, 1),
]


def time_ms(fn, steps):
    import torch
    for _ in range(3):
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
    return sorted(ts)[len(ts) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--tile-bytes", type=int, default=16384)
    args = ap.parse_args()
    import torch
    import paper_2605_03190_amd as vdc

    print("median of %d runs; tiles of %d bytes; GB/s = weight bytes / time" % (args.steps, args.tile_bytes))
    print("%-44s %2s %9s | %10s %8s | %10s %8s | %7s" % ("layers", "B", "MiB", "one graph", "GB/s", "L launches", "GB/s", "ratio"))
    with vdc.Executor() as ex:
        for dims, B in CASES:
            L = len(dims) - 1
            g = torch.Generator(device="cuda").manual_seed(sum(dims))
            w_elems = sum(dims[l + 1] * dims[l] for l in range(L))
            W = torch.randn(w_elems, device="cuda", generator=g)
            off = 0
            Ms = []
            for l in range(L):
                n = dims[l + 1] * dims[l]
                W[off:off + n] *= dims[l] ** -0.5
                Ms.append(W[off:off + n].view(dims[l + 1], dims[l]))
                off += n
            A = torch.zeros(B * sum(dims), device="cuda")
            A[:B * dims[0]] = torch.randn(B * dims[0], device="cuda", generator=g)
            a_off = np.concatenate([[0], np.cumsum([B * x for x in dims])])
            acts = [A[a_off[l]:a_off[l + 1]].view(B, dims[l]) for l in range(L + 1)]

            def chain():
                ex.matvec_chain(W, A, dims, B, args.tile_bytes)

            def separate():
                for l in range(L):
                    ex.matvec(Ms[l], acts[l], acts[l + 1], args.tile_bytes)

            separate()
            ex.check()
            want = A.clone()
            chain()
            ex.check()
            # the two differ only in rounding order (a single matvec of few row blocks also splits K)
            err = float((A - want).abs().max() / want.abs().max())
            assert err < 1e-4, err
            t1 = time_ms(chain, args.steps)
            t2 = time_ms(separate, args.steps)
            ex.check()
            nbytes = 4 * w_elems
            name = "x".join(str(d) for d in dims) if len(set(dims)) > 1 else "%d layers of %d x %d" % (L, dims[0], dims[0])
            print("%-44s %2d %9.0f | %8.1f us %8.0f | %8.1f us %8.0f | %6.2fx" % (name, B, nbytes / 2**20, t1 * 1e3, nbytes / t1 / 1e6,
                                                                               t2 * 1e3, nbytes / t2 / 1e6, t2 / t1), flush=True)


if __name__ == "__main__":
    main()
