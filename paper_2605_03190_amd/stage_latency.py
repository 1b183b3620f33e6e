"""Stage latencies of the allocate -> load -> consume -> recycle loop, measured on the GPU with the observer build.

    python paper_2605_03190_amd/build.py --observer          # once, on the CPU
    python -m paper_2605_03190_amd.stage_latency [workload]  # on the GPU; workload = a dense name from workloads.CONFIGS,
                                                             # or attn_64k: decode attention, 8 contexts of 65536 rows

The observer build (-DVDC_PROFILE) adds one wave to core 0 that only reads: it samples the control words of the core
(ring heads and tails, slot mask) and one progress word per unit, and logs every change with a time stamp.  This
script turns the log into the median time a matrix tile spends in each stage.  The sampling period (printed) bounds
the resolution; the instrumented kernel is about 25 % slower than the product build, so the figures are upper bounds.
"""
import ctypes
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

CAP = 65536          # events the observer keeps
# words of the log: 0..7 uq_head, 8 slot mask, 12..19 uq_tail, 36 + w = progress word of wave w
W_HEAD, W_MASK, W_TAIL, W_PROGRESS = 0, 8, 12, 36


def first_reach(t, word, val, wd, f=lambda b: b):
    """time at which counter word wd was first seen >= k, for every k"""
    sel = word == wd
    out, prev = {}, 0
    for a, b in zip(t[sel], val[sel]):
        b = f(int(b))
        for k in range(prev + 1, b + 1):
            out[k] = a
        prev = max(prev, b)
    return out


def read_log(vdc, ex):
    """The observer's log as (time, word, value) arrays, times from the first event."""
    buf = np.zeros(2 * CAP + 1, dtype=np.uint64)
    L = vdc.lib()
    L.vdc_prof_events.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    if L.vdc_prof_events(ex.handle, ctypes.c_void_p(buf.ctypes.data)) != 0:
        raise SystemExit("could not read the observer log")
    n = min(int(buf[-1]), CAP)
    ev = buf[:2 * n].reshape(n, 2)
    t = ev[:, 0].astype(np.int64)
    t -= t[0]
    word = (ev[:, 1] & np.uint64(0xFFFFFFFF)).astype(np.int64)
    val = (ev[:, 1] >> np.uint64(32)).astype(np.int64)
    return n, t, word, val


def slots_in_use(t, word, val, n_slots):
    sel = word == W_MASK
    used = np.array([bin(int(x)).count("1") for x in val[sel]])
    dur = np.diff(t[sel])
    if len(dur):
        print("slots in use, time-weighted mean %.2f of %d" % ((used[:-1] * dur).sum() / dur.sum(), n_slots))


def attention(vdc, torch):
    """Decode attention, 8 contexts of 65536 rows, 16 KB tiles: the stages of a (key tile, value tile) pair.  Key tiles of
    compute core v travel on load unit v, value tiles on load unit 2 + v; the first ticket of an item is its query tile."""
    lengths = np.repeat([65536], 8)
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows, d = int(ro[-1]), 128
    Q, K, V = (torch.randn(sh, device="cuda") for sh in ((len(lengths), d), (rows, d), (rows, d)))
    O = torch.empty((len(lengths), d), device="cuda")
    ex = vdc.Executor()
    for _ in range(3):
        ex.attn_decode(Q, K, V, ro, O, 16384)
    ex.check()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ex.attn_decode(Q, K, V, ro, O, 16384)
    e1.record()
    torch.cuda.synchronize()
    n, t, word, val = read_log(vdc, ex)
    print("attn_64k: instrumented kernel %.3f ms; %d events, sampling period (median) %d cycles" % (e0.elapsed_time(e1), n, np.median(np.diff(np.unique(t)))))
    for v in range(2):
        uk, uv = v, 2 + v
        disp, issued, deliv = (first_reach(t, word, val, w + uk) for w in (W_TAIL, W_HEAD, W_PROGRESS + 1))
        vdisp, vissued, vdeliv = (first_reach(t, word, val, w + uv) for w in (W_TAIL, W_HEAD, W_PROGRESS + 1))
        popped = first_reach(t, word, val, W_PROGRESS + 6 + 2 * v)
        back = first_reach(t, word, val, W_PROGRESS + 10 + v)
        rows_ = []
        for k in range(3, 31):      # the pairs of the core's first item (the query tile is record 1 of the value tiles' unit)
            try:
                rows_.append((issued[k] - disp[k], deliv[k] - issued[k], vissued[k + 1] - vdisp[k + 1], vdeliv[k + 1] - vissued[k + 1],
                              popped[1 + 2 * k] - max(deliv[k], vdeliv[k + 1]), back[1 + 2 * k] - popped[1 + 2 * k], disp[k + 2] - back[1 + 2 * k],
                              disp[k + 1] - disp[k], back[1 + 2 * k] - disp[k]))
            except KeyError:
                pass
        if not rows_:
            continue
        r = np.array(rows_)
        print("compute core %d: %d pairs; cycles: median / mean / 90th percentile" % (v, len(r)))
        for i, nm in enumerate(["key tile: dispatched -> loads issued", "key tile: issued -> delivered", "value tile: dispatched -> loads issued",
                                "value tile: issued -> delivered", "both delivered -> popped", "popped -> slots back (the uop's work)",
                                "slots back -> dispatch of pair k + 2", "period (pair k -> k + 1)", "lifetime of the key tile's slots"]):
            print("   %-44s %7.0f %7.0f %7.0f" % (nm, np.median(r[:, i]), r[:, i].mean(), np.percentile(r[:, i], 90)))
    slots_in_use(t, word, val, ex.cfg.n_slots)
    ex.destroy()


def main():
    import torch
    import paper_2605_03190_amd as vdc
    from paper_2605_03190_amd.build import SO_OBSERVER
    import workloads
    if not os.path.exists(SO_OBSERVER):
        raise SystemExit("build the observer library first: python paper_2605_03190_amd/build.py --observer")
    vdc.LIB_PATH = SO_OBSERVER
    name = sys.argv[1] if len(sys.argv) > 1 else "cfg5"
    if name == "attn_64k":
        return attention(vdc, torch)
    cfg = workloads.CONFIGS[name]
    if cfg.n_seg:
        raise SystemExit("dense workloads only")
    w = workloads.make(cfg, device="cuda")
    ex = vdc.Executor(slot_bytes=cfg.slot_bytes)
    Y = torch.zeros((cfg.B, cfg.rows), device="cuda")
    for _ in range(3):
        ex.matvec(w.M, w.X, Y, cfg.tile_bytes)
    ex.check()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ex.matvec(w.M, w.X, Y, cfg.tile_bytes)
    e1.record()
    torch.cuda.synchronize()
    n, t, word, val = read_log(vdc, ex)
    ut = np.unique(t)
    print("%s: instrumented kernel %.3f ms; %d events, sampling period (median) %d cycles" % (name, e0.elapsed_time(e1), n, np.median(np.diff(ut))))
    n_ldu = ex.cfg.n_ldu
    for v in range(ex.cfg.vcc_per_core):
        # matrix tiles of compute core v travel on load unit v, its vector tiles on load unit V + v (mod n_ldu)
        um, ux = v % n_ldu, (ex.cfg.vcc_per_core + v) % n_ldu
        disp = first_reach(t, word, val, W_TAIL + um)
        issued = first_reach(t, word, val, W_HEAD + um)
        deliv = first_reach(t, word, val, W_PROGRESS + 1 + um)
        xdisp = first_reach(t, word, val, W_TAIL + ux)
        xdeliv = first_reach(t, word, val, W_PROGRESS + 1 + ux)
        popped = first_reach(t, word, val, W_PROGRESS + 6 + 2 * v)     # tickets popped by the first wave
        back = first_reach(t, word, val, W_PROGRESS + 10 + v)          # tickets whose regions went back to the pool
        rows = []
        for k in range(100, 500):
            try:
                rows.append((issued[k] - disp[k], deliv[k] - issued[k], xdeliv[k] - xdisp[k], popped[2 * k] - max(deliv[k], xdeliv[k]),
                             back[2 * k] - popped[2 * k], disp[k + 3] - back[2 * k], disp[k + 1] - disp[k], back[2 * k] - disp[k]))
            except KeyError:
                pass
        if not rows:
            continue
        r = np.array(rows)
        print("compute core %d, tile steps 100..500 (%d complete), cycles: median / mean / 90th percentile" % (v, len(r)))
        for i, nm in enumerate(["matrix tile: dispatched -> loads issued", "matrix tile: issued -> landed and delivered", "vector tile: dispatched -> delivered",
                                "both delivered -> popped by the compute core", "popped -> both waves done, slots back in the pool",
                                "slots back -> dispatch of the step three later", "period (dispatch of step k -> k + 1)",
                                "lifetime of a matrix tile's slots"]):
            print("   %-52s %7.0f %7.0f %7.0f" % (nm, np.median(r[:, i]), r[:, i].mean(), np.percentile(r[:, i], 90)))
    slots_in_use(t, word, val, ex.cfg.n_slots)
    ex.destroy()


if __name__ == "__main__":
    main()
