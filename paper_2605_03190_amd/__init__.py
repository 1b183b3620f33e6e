"""Python binding of libvdcores.so (the C ABI declared in include/vdcores.h).

Argument marshalling only: every step of the hot path runs in the library's HIP kernels.
PyTorch is used by callers for device memory and streams; this module never computes.
If the library has not been built, importing the binding's functions fails loudly; there is
no CPU fallback.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvdcores.so")

VDC_OK, VDC_EINVAL, VDC_ENOMEM, VDC_EPROGRAM, VDC_EDEVICE, VDC_EDEADLOCK, VDC_ELEAK, VDC_ETOOBIG = 0, -1, -2, -3, -4, -5, -6, -7
VDC_ESTATE, VDC_ETIMEOUT = -8, -9
NOALLOC_SCRATCH_BYTES = 256 * 1024


class VdcError(RuntimeError):
    def __init__(self, code, what=""):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (what, strerror(code), code))


class vdc_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "device", "n_cores", "vcc_per_core", "threads_per_eu", "slot_bytes", "n_slots", "n_ldu", "n_stu",
        "n_dep_ids", "watchdog_spins", "tile_rows", "issue_batch", "issue_flags", "sched_threshold_pct", "sched_min_gain_pct",
        "sched_force_parts")]


class vdc_sched_op(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int64), ("nk", ctypes.c_int64), ("max_parts", ctypes.c_int32), ("join_group", ctypes.c_int32),
                ("surplus", ctypes.c_int64)]


class vdc_cost_model(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("step", "item", "join", "edge")]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built (python -m paper_2605_03190_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libvdcores.so is not built: run `python paper_2605_03190_amd/build.py` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        pp = ctypes.POINTER(ctypes.c_void_p)
        sig = {
            "vdc_create": [pp, ctypes.POINTER(vdc_config)],
            "vdc_destroy": [vp],
            "vdc_get_config": [vp, ctypes.POINTER(vdc_config)],
            "vdc_program_create": [vp, vp, i64, vp, vp, i32, vp, i32, pp],
            "vdc_program_validate": [vp, vp, i64, vp, vp, i32, vp, i32, ctypes.c_char_p, i32],
            "vdc_program_destroy": [vp],
            "vdc_program_set_placement": [vp, i32],
            "vdc_run": [vp, vp, vp, i32, vp],
            "vdc_run_traced": [vp, vp, vp, i32, vp, vp, i32, vp],
            "vdc_sync_status": [vp, vp, vp],
            "vdc_resident_start": [vp, i32],
            "vdc_resident_submit": [vp, vp, vp, i32, ctypes.POINTER(ctypes.c_uint32)],
            "vdc_resident_wait": [vp, ctypes.c_uint32, i32, vp],
            "vdc_resident_state": [vp, ctypes.POINTER(ctypes.c_uint32)],
            "vdc_resident_stop": [vp],
            "vdc_matvec": [vp, vp, i64, i64, i64, vp, vp, i32, i32, vp],
            "vdc_matvec_noalloc": [vp, vp, i64, i64, i64, vp, vp, i32, i32, vp],
            "vdc_matvec_ragged": [vp, vp, vp, i32, i64, vp, vp, i32, vp],
            "vdc_matvec_program": [vp, i64, i64, i64, i32, i32, vp, i32, vp, ctypes.POINTER(i64), vp, vp,
                                   ctypes.POINTER(i32)],
            "vdc_matvec_rope": [vp, vp, i64, i64, i64, vp, vp, vp, i32, i32, vp],
            "vdc_matvec_rope_program": [vp, i64, i64, i64, i32, i32, vp, ctypes.POINTER(i64), vp, vp, ctypes.POINTER(i32)],
            "vdc_matvec_workspace": [vp, i64, i64, i64, i32, i32, vp, ctypes.POINTER(i64)],
            "vdc_matvec_chain": [vp, vp, vp, vp, i32, i32, i32, vp],
            "vdc_matvec_chain_program": [vp, vp, i32, i32, i32, vp, ctypes.POINTER(i64), vp, vp, ctypes.POINTER(i32)],
            "vdc_attn_decode": [vp, vp, vp, vp, vp, i32, i32, ctypes.c_float, vp, i32, vp],
            "vdc_attn_decode_program": [vp, vp, i32, i32, ctypes.c_float, i32, vp, ctypes.POINTER(i64), vp, vp, ctypes.POINTER(i32),
                                        ctypes.POINTER(i64)],
            "vdc_stream": [vp, i32, vp, vp, i64, ctypes.c_uint32, i32, vp],
            "vdc_raw_stream": [vp, i32, vp, vp, i64, ctypes.c_uint32, vp],
            "vdc_stream_program": [vp, i32, i64, ctypes.c_uint32, i32, vp, ctypes.POINTER(i64), vp, vp, ctypes.POINTER(i32)],
            "vdc_debug_alloc": [vp, vp, vp, i32, vp, i32, vp],
            "vdc_graph_lower": [vp, vp, i64, vp, i64, vp, vp, vp, i32, ctypes.c_uint32, i32, vp, i32, vp, ctypes.POINTER(i64), vp, vp,
                                ctypes.POINTER(i32), vp],
            "vdc_schedule": [vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, ctypes.POINTER(i32)],
            "vdc_matvec_tiling": [vp, i64, i64, i32, i32, vp],
        }
        for name, args in sig.items():
            f = getattr(L, name)
            f.argtypes = args
            f.restype = ctypes.c_int
        L.vdc_strerror.argtypes = [ctypes.c_int]
        L.vdc_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


EXPORTS = ["vdc_create", "vdc_destroy", "vdc_get_config", "vdc_program_create", "vdc_program_validate",
           "vdc_program_destroy", "vdc_program_set_placement", "vdc_run", "vdc_run_traced", "vdc_sync_status",
           "vdc_resident_start", "vdc_resident_submit", "vdc_resident_wait", "vdc_resident_state", "vdc_resident_stop", "vdc_matvec", "vdc_matvec_noalloc", "vdc_matvec_ragged",
           "vdc_matvec_program", "vdc_matvec_rope", "vdc_matvec_rope_program", "vdc_matvec_workspace", "vdc_matvec_chain", "vdc_matvec_chain_program", "vdc_attn_decode", "vdc_attn_decode_program",
           "vdc_stream", "vdc_raw_stream",
           "vdc_stream_program", "vdc_debug_alloc", "vdc_graph_lower", "vdc_schedule", "vdc_matvec_tiling", "vdc_strerror"]


def strerror(code):
    return lib().vdc_strerror(int(code)).decode()


def _check(rc, what):
    if rc != VDC_OK:
        raise VdcError(rc, what)


def _np_ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _stream_ptr(stream):
    """hipStream_t of a torch stream (None: torch's current stream)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(getattr(stream, "cuda_stream", stream) or 0)


class Program:
    def __init__(self, ex, handle):
        self.ex, self.handle = ex, handle

    def destroy(self):
        if self.handle:
            _check(lib().vdc_program_destroy(self.handle), "vdc_program_destroy")
            self.handle = None

    def set_placement(self, placement):
        _check(lib().vdc_program_set_placement(self.handle, placement), "vdc_program_set_placement")


class Executor:
    """vdc_create / vdc_destroy and the calls that take the executor."""

    def __init__(self, **cfg):
        c = vdc_config()
        for k, v in cfg.items():
            setattr(c, k, v)
        h = ctypes.c_void_p()
        _check(lib().vdc_create(ctypes.byref(h), ctypes.byref(c)), "vdc_create")
        self.handle = h
        got = vdc_config()
        _check(lib().vdc_get_config(self.handle, ctypes.byref(got)), "vdc_get_config")
        self.cfg = got

    def destroy(self):
        if self.handle:
            _check(lib().vdc_destroy(self.handle), "vdc_destroy")
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.destroy()

    @property
    def n_streams(self):
        return self.cfg.n_cores * (1 + self.cfg.vcc_per_core)

    # ---- low level -------------------------------------------------------------------------------
    @staticmethod
    def _prog_arrays(words, stream_begin, descs, tensor_bytes):
        words = np.ascontiguousarray(words, dtype=np.uint32).reshape(-1, 4)
        sb = np.ascontiguousarray(stream_begin, dtype=np.uint32)
        descs = np.ascontiguousarray(descs, dtype=np.uint32).reshape(-1, 8)
        tb = np.ascontiguousarray(tensor_bytes, dtype=np.int64)
        return words, sb, descs, tb

    def program_create(self, words, stream_begin, descs, tensor_bytes):
        words, sb, descs, tb = self._prog_arrays(words, stream_begin, descs, tensor_bytes)
        if len(sb) != self.n_streams + 1:
            raise VdcError(VDC_EINVAL, "vdc_program_create (stream_begin length)")
        h = ctypes.c_void_p()
        _check(lib().vdc_program_create(self.handle, _np_ptr(words), len(words), _np_ptr(sb), _np_ptr(descs), len(descs),
                                        _np_ptr(tb), len(tb), ctypes.byref(h)), "vdc_program_create")
        return Program(self, h)

    def program_validate(self, words, stream_begin, descs, tensor_bytes):
        """Returns (code, message)."""
        words, sb, descs, tb = self._prog_arrays(words, stream_begin, descs, tensor_bytes)
        if len(sb) != self.n_streams + 1:
            return VDC_EINVAL, "stream_begin length"
        buf = ctypes.create_string_buffer(256)
        rc = lib().vdc_program_validate(self.handle, _np_ptr(words), len(words), _np_ptr(sb), _np_ptr(descs), len(descs),
                                        _np_ptr(tb), len(tb), buf, 256)
        return rc, buf.value.decode()

    def run(self, prog, tensors, stream=None, trace_cap=0):
        """tensors: torch CUDA tensors.  With trace_cap > 0 returns (trace, trace_count) device tensors."""
        import torch
        bases = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
        if trace_cap:
            trace = torch.zeros((self.n_streams, trace_cap, 4), dtype=torch.int32, device=tensors[0].device)
            count = torch.zeros((self.n_streams,), dtype=torch.int32, device=tensors[0].device)
            _check(lib().vdc_run_traced(self.handle, prog.handle, bases, len(tensors), trace.data_ptr(), count.data_ptr(),
                                        trace_cap, _stream_ptr(stream)), "vdc_run_traced")
            return trace, count
        _check(lib().vdc_run(self.handle, prog.handle, bases, len(tensors), _stream_ptr(stream)), "vdc_run")
        return None

    # ---- the resident form ----------------------------------------------------------------------
    def resident_start(self, idle_ms=0):
        _check(lib().vdc_resident_start(self.handle, idle_ms), "vdc_resident_start")

    def resident_submit(self, prog, tensors):
        """Posts one graph; returns its ticket."""
        bases = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
        ticket = ctypes.c_uint32(0)
        _check(lib().vdc_resident_submit(self.handle, prog.handle, bases, len(tensors), ctypes.byref(ticket)), "vdc_resident_submit")
        return ticket.value

    def resident_wait(self, ticket, timeout_ms=10000):
        """Returns (code, info[4])."""
        info = (ctypes.c_uint32 * 4)()
        rc = lib().vdc_resident_wait(self.handle, ticket, timeout_ms, info)
        return rc, list(info)

    def resident_state(self):
        """Returns (state, completed): state 0 not started, 1 up, 2 the cores have left."""
        done = ctypes.c_uint32(0)
        return lib().vdc_resident_state(self.handle, ctypes.byref(done)), done.value

    def resident_stop(self):
        _check(lib().vdc_resident_stop(self.handle), "vdc_resident_stop")

    def sync_status(self, stream=None):
        """Waits for the stream; returns (code, info[4])."""
        info = (ctypes.c_uint32 * 4)()
        rc = lib().vdc_sync_status(self.handle, _stream_ptr(stream), info)
        return rc, list(info)

    def check(self, stream=None):
        rc, info = self.sync_status(stream)
        if rc != VDC_OK:
            raise VdcError(rc, "device run (core %d role %#x pc %d detail %#x)" % tuple(info))

    # ---- high level ------------------------------------------------------------------------------
    def matvec(self, M, X, Y, tile_bytes, K=None, stream=None):
        """Y[b][i] = sum_j M[i][j] X[b][j].  M: [rows, ld] fp32 CUDA (K <= ld columns used), X: [B, K], Y: [B, rows]."""
        rows, ld = M.shape
        B, Kx = X.shape
        K = Kx if K is None else K
        assert M.is_cuda and X.is_cuda and Y.is_cuda and M.is_contiguous() and X.is_contiguous() and Y.is_contiguous()
        assert M.dtype == X.dtype == Y.dtype and str(M.dtype) == "torch.float32"
        assert Kx == K and tuple(Y.shape) == (B, rows)
        _check(lib().vdc_matvec(self.handle, M.data_ptr(), rows, K, ld, X.data_ptr(), Y.data_ptr(), B, tile_bytes,
                                _stream_ptr(stream)), "vdc_matvec")

    def matvec_noalloc(self, M, X, Y, tile_bytes, K=None, stream=None):
        """matvec() through the entry point that allocates nothing on the device (program and workspace in the
        library's static scratch array); VdcError(VDC_ETOOBIG) when the program does not fit it."""
        rows, ld = M.shape
        B, Kx = X.shape
        K = Kx if K is None else K
        assert M.is_cuda and X.is_cuda and Y.is_cuda and M.is_contiguous() and X.is_contiguous() and Y.is_contiguous()
        assert M.dtype == X.dtype == Y.dtype and str(M.dtype) == "torch.float32"
        assert Kx == K and tuple(Y.shape) == (B, rows)
        _check(lib().vdc_matvec_noalloc(self.handle, M.data_ptr(), rows, K, ld, X.data_ptr(), Y.data_ptr(), B, tile_bytes,
                                        _stream_ptr(stream)), "vdc_matvec_noalloc")

    def matvec_rope(self, M, X, T, Y, tile_bytes, K=None, stream=None):
        """Y = rope(M X, T): T and Y are [B, rows]; T holds (cos, sin) for every pair of rows."""
        rows, ld = M.shape
        B, Kx = X.shape
        K = Kx if K is None else K
        assert all(t.is_cuda and t.is_contiguous() and str(t.dtype) == "torch.float32" for t in (M, X, T, Y))
        assert Kx == K and tuple(Y.shape) == (B, rows) and tuple(T.shape) == (B, rows)
        _check(lib().vdc_matvec_rope(self.handle, M.data_ptr(), rows, K, ld, X.data_ptr(), T.data_ptr(), Y.data_ptr(), B, tile_bytes,
                                     _stream_ptr(stream)), "vdc_matvec_rope")

    def matvec_ragged(self, M, row_off, X, Y, tile_bytes, stream=None):
        """Segment s = rows row_off[s]..row_off[s+1]-1 of M ([sum rows, K]) times X[s] ([n_seg, K]); Y: [sum rows]."""
        row_off = np.ascontiguousarray(row_off, dtype=np.int64)
        n_seg, K = X.shape
        assert M.is_cuda and X.is_cuda and Y.is_cuda and M.is_contiguous() and X.is_contiguous() and Y.is_contiguous()
        assert str(M.dtype) == "torch.float32" and M.shape[1] == K and len(row_off) == n_seg + 1
        assert int(row_off[-1]) == M.shape[0] == Y.numel()
        _check(lib().vdc_matvec_ragged(self.handle, M.data_ptr(), _np_ptr(row_off), n_seg, K, X.data_ptr(), Y.data_ptr(),
                                       tile_bytes, _stream_ptr(stream)), "vdc_matvec_ragged")

    def matvec_rope_program(self, rows, K, ld, B, tile_bytes):
        """The uop graph matvec_rope would run."""
        n_w, n_d = ctypes.c_int64(0), ctypes.c_int32(0)
        f = lib().vdc_matvec_rope_program
        _check(f(self.handle, rows, K, ld, B, tile_bytes, None, ctypes.byref(n_w), None, None, ctypes.byref(n_d)), "vdc_matvec_rope_program (sizing)")
        words = np.zeros((n_w.value, 4), dtype=np.uint32)
        descs = np.zeros((n_d.value, 8), dtype=np.uint32)
        sb = np.zeros(self.n_streams + 1, dtype=np.uint32)
        _check(f(self.handle, rows, K, ld, B, tile_bytes, _np_ptr(words), ctypes.byref(n_w), _np_ptr(sb), _np_ptr(descs), ctypes.byref(n_d)),
               "vdc_matvec_rope_program")
        return words, sb, descs

    def matvec_program(self, rows, K, ld, B, tile_bytes, row_off=None):
        """The uop graph the matvec operator would run: (words[n,4], stream_begin, descs[n,8]) as numpy uint32."""
        n_w, n_d = ctypes.c_int64(0), ctypes.c_int32(0)
        ro = None if row_off is None else np.ascontiguousarray(row_off, dtype=np.int64)
        ro_p = None if ro is None else _np_ptr(ro)
        n_seg = 0 if ro is None else len(ro) - 1
        rc = lib().vdc_matvec_program(self.handle, rows, K, ld, B, tile_bytes, ro_p, n_seg, None, ctypes.byref(n_w), None,
                                      None, ctypes.byref(n_d))
        _check(rc, "vdc_matvec_program (sizing)")
        words = np.zeros((n_w.value, 4), dtype=np.uint32)
        descs = np.zeros((n_d.value, 8), dtype=np.uint32)
        sb = np.zeros(self.n_streams + 1, dtype=np.uint32)
        rc = lib().vdc_matvec_program(self.handle, rows, K, ld, B, tile_bytes, ro_p, n_seg, _np_ptr(words), ctypes.byref(n_w),
                                      _np_ptr(sb), _np_ptr(descs), ctypes.byref(n_d))
        _check(rc, "vdc_matvec_program")
        return words, sb, descs

    def matvec_workspace(self, rows, K, ld, B, tile_bytes):
        """Initial content (numpy float32, possibly empty) of tensor 3 of the program matvec_program returns."""
        n = ctypes.c_int64(0)
        _check(lib().vdc_matvec_workspace(self.handle, rows, K, ld, B, tile_bytes, None, ctypes.byref(n)), "vdc_matvec_workspace (sizing)")
        ws = np.zeros(n.value // 4, dtype=np.float32)
        if n.value:
            _check(lib().vdc_matvec_workspace(self.handle, rows, K, ld, B, tile_bytes, _np_ptr(ws), ctypes.byref(n)), "vdc_matvec_workspace")
        return ws

    def matvec_tiling(self, rows, K, B, tile_bytes):
        """vdc_matvec_tiling: (rows per tile, tile width, row blocks, steps along K, finest K cut offered, K cut taken,
        trailing row blocks it is taken on or 0 for all)."""
        out = np.zeros(7, dtype=np.int64)
        _check(lib().vdc_matvec_tiling(self.handle, rows, K, B, tile_bytes, _np_ptr(out)), "vdc_matvec_tiling")
        return tuple(int(x) for x in out)

    def schedule(self, ops, preds=None, cost=None, tile_bytes=16384):
        """vdc_schedule: ops = [(n_blocks, nk, max_parts[, join_group[, surplus]])], preds = per operator the operators it
        waits for, cost = (step, item, join, edge) or None for the library's model.  Returns (parts, tails, log) with log =
        [(path cost, average, refined operator or -1, new S, gain)]."""
        n = len(ops)
        arr = (vdc_sched_op * max(n, 1))()
        for o, op in enumerate(ops):
            arr[o] = vdc_sched_op(op[0], op[1], op[2], op[3] if len(op) > 3 else 0, op[4] if len(op) > 4 else 0)
        pb = pr = None
        if preds is not None:
            pb = np.zeros(n + 1, dtype=np.int32)
            pb[1:] = np.cumsum([len(p) for p in preds])
            pr = np.array([q for p in preds for q in p] + [0], dtype=np.int32)
        cm = vdc_cost_model(*cost) if cost is not None else None
        parts = np.zeros(max(n, 1), dtype=np.int32)
        tails = np.zeros(max(n, 1), dtype=np.int32)
        cap = 2 + sum(op[2] for op in ops)
        log = np.zeros((cap, 5), dtype=np.int64)
        looks = ctypes.c_int32(cap)
        _check(lib().vdc_schedule(self.handle, ctypes.cast(arr, ctypes.c_void_p), n, _np_ptr(pb) if pb is not None else None,
                                  _np_ptr(pr) if pr is not None else None, ctypes.cast(ctypes.pointer(cm), ctypes.c_void_p) if cm else None,
                                  tile_bytes, _np_ptr(parts), _np_ptr(tails), _np_ptr(log), ctypes.byref(looks)), "vdc_schedule")
        return [int(x) for x in parts[:n]], [int(x) for x in tails[:n]], [tuple(int(x) for x in r) for r in log[:looks.value]]

    def matvec_chain(self, W, A, dims, B, tile_bytes, stream=None):
        """Y_0 = M_0 X, Y_l = M_l Y_(l-1) in one launch.  W: the matrices back to back; A: X then every Y_l, back to back
        (CUDA fp32 tensors); dims = (K_0, rows_0, rows_1, ...).  Asynchronous."""
        d = np.ascontiguousarray(dims, dtype=np.int64)
        _check(lib().vdc_matvec_chain(self.handle, W.data_ptr(), A.data_ptr(), _np_ptr(d), len(d) - 1, B, tile_bytes, _stream_ptr(stream)),
               "vdc_matvec_chain")

    def matvec_chain_program(self, dims, B, tile_bytes):
        """The uop graph matvec_chain would run."""
        d = np.ascontiguousarray(dims, dtype=np.int64)
        n_w, n_d = ctypes.c_int64(0), ctypes.c_int32(0)
        f = lib().vdc_matvec_chain_program
        _check(f(self.handle, _np_ptr(d), len(d) - 1, B, tile_bytes, None, ctypes.byref(n_w), None, None, ctypes.byref(n_d)), "vdc_matvec_chain_program (sizing)")
        words = np.zeros((n_w.value, 4), dtype=np.uint32)
        descs = np.zeros((n_d.value, 8), dtype=np.uint32)
        sb = np.zeros(self.n_streams + 1, dtype=np.uint32)
        _check(f(self.handle, _np_ptr(d), len(d) - 1, B, tile_bytes, _np_ptr(words), ctypes.byref(n_w), _np_ptr(sb), _np_ptr(descs), ctypes.byref(n_d)),
               "vdc_matvec_chain_program")
        return words, sb, descs

    def attn_decode(self, Q, K, V, row_off, O, tile_bytes, scale=None, stream=None):
        """O[s] = softmax(scale * K_s Q[s]) V_s per request s; Q, O: [n_seg][d], K, V: [rows][d] CUDA fp32 tensors;
        row_off: host offsets (n_seg + 1).  Asynchronous."""
        ro = np.ascontiguousarray(row_off, dtype=np.int64)
        d = Q.shape[1]
        scale = 0.0 if scale is None else float(scale)     # 0: the library takes d ** -0.5
        _check(lib().vdc_attn_decode(self.handle, Q.data_ptr(), K.data_ptr(), V.data_ptr(), _np_ptr(ro), len(ro) - 1, d, scale,
                                     O.data_ptr(), tile_bytes, _stream_ptr(stream)), "vdc_attn_decode")

    def attn_decode_program(self, row_off, d, tile_bytes, scale=None):
        """The uop graph attn_decode would run: (words, stream_begin, descs, n_items)."""
        ro = np.ascontiguousarray(row_off, dtype=np.int64)
        scale = 0.0 if scale is None else float(scale)     # 0: the library takes d ** -0.5
        n_w, n_d, n_i = ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_int64(0)
        f = lib().vdc_attn_decode_program
        _check(f(self.handle, _np_ptr(ro), len(ro) - 1, d, scale, tile_bytes, None, ctypes.byref(n_w), None, None, ctypes.byref(n_d),
                 ctypes.byref(n_i)), "vdc_attn_decode_program (sizing)")
        words = np.zeros((n_w.value, 4), dtype=np.uint32)
        descs = np.zeros((n_d.value, 8), dtype=np.uint32)
        sb = np.zeros(self.n_streams + 1, dtype=np.uint32)
        _check(f(self.handle, _np_ptr(ro), len(ro) - 1, d, scale, tile_bytes, _np_ptr(words), ctypes.byref(n_w), _np_ptr(sb), _np_ptr(descs),
                 ctypes.byref(n_d), ctypes.byref(n_i)), "vdc_attn_decode_program")
        return words, sb, descs, n_i.value

    STREAM_MODES = {"read": 0, "fill": 1, "copy": 2}

    def stream(self, mode, src, dst, nbytes, tile_bytes, value=0, stream=None):
        """Memory uops with nothing to compute behind them: mode "read" (src), "fill" (dst, value) or "copy" (src, dst);
        src, dst: CUDA tensors or None.  Asynchronous."""
        _check(lib().vdc_stream(self.handle, self.STREAM_MODES[mode], src.data_ptr() if src is not None else None,
                                dst.data_ptr() if dst is not None else None, nbytes, value, tile_bytes, _stream_ptr(stream)), "vdc_stream")

    def raw_stream(self, mode, src, dst, nbytes, value=0, stream=None):
        """The same bytes as stream(), moved by an ordinary grid-stride kernel: what stream() is measured against."""
        _check(lib().vdc_raw_stream(self.handle, self.STREAM_MODES[mode], src.data_ptr() if src is not None else None,
                                    dst.data_ptr() if dst is not None else None, nbytes, value, _stream_ptr(stream)), "vdc_raw_stream")

    GRAPH_MEMOP = np.dtype([("op", "<i4"), ("core", "<i4"), ("vcc", "<i4"), ("desc", "<i4"), ("offset", "<i8"), ("rows", "<i4"),
                            ("nslots", "<i4"), ("group", "<i4"), ("nt", "<i4")])

    def graph_lower(self, ops, edges, comp_words, comp_begin, descs, tensor_bytes, temp_tensors=0, geom_tensor=0):
        """vdc_graph_lower: ops = array of GRAPH_MEMOP, edges = [n, 2] int64 (store, load), comp_words [n, 4] uint32 with
        comp_begin offsets per compute core, descs [n, 8] uint32.  Returns (words, stream_begin, descs, stats)."""
        ops = np.ascontiguousarray(ops, dtype=self.GRAPH_MEMOP)
        edges = np.ascontiguousarray(edges, dtype=np.int64).reshape(-1, 2)
        comp_words = np.ascontiguousarray(comp_words, dtype=np.uint32).reshape(-1, 4)
        comp_begin = np.ascontiguousarray(comp_begin, dtype=np.uint32)
        descs = np.ascontiguousarray(descs, dtype=np.uint32).reshape(-1, 8)
        tb = np.ascontiguousarray(tensor_bytes, dtype=np.int64)
        n_w, n_d = ctypes.c_int64(0), ctypes.c_int32(0)
        stats = np.zeros(5, dtype=np.int32)
        f = lib().vdc_graph_lower
        args = (self.handle, _np_ptr(ops), len(ops), _np_ptr(edges) if len(edges) else None, len(edges), _np_ptr(comp_words), _np_ptr(comp_begin),
                _np_ptr(descs), len(descs), temp_tensors, geom_tensor, _np_ptr(tb), len(tb))
        rc = f(*args, None, ctypes.byref(n_w), None, None, ctypes.byref(n_d), _np_ptr(stats))
        _check(rc, "vdc_graph_lower (sizing)")
        words = np.zeros((n_w.value, 4), dtype=np.uint32)
        out_descs = np.zeros((n_d.value, 8), dtype=np.uint32)
        sb = np.zeros(self.n_streams + 1, dtype=np.uint32)
        _check(f(*args, _np_ptr(words), ctypes.byref(n_w), _np_ptr(sb), _np_ptr(out_descs), ctypes.byref(n_d), _np_ptr(stats)), "vdc_graph_lower")
        return words, sb, out_descs, stats

    def stream_program(self, mode, nbytes, tile_bytes, value=0):
        """The uop graph stream() would run."""
        n_w, n_d = ctypes.c_int64(0), ctypes.c_int32(0)
        f, m = lib().vdc_stream_program, self.STREAM_MODES[mode]
        _check(f(self.handle, m, nbytes, value, tile_bytes, None, ctypes.byref(n_w), None, None, ctypes.byref(n_d)), "vdc_stream_program (sizing)")
        words = np.zeros((n_w.value, 4), dtype=np.uint32)
        descs = np.zeros((n_d.value, 8), dtype=np.uint32)
        sb = np.zeros(self.n_streams + 1, dtype=np.uint32)
        _check(f(self.handle, m, nbytes, value, tile_bytes, _np_ptr(words), ctypes.byref(n_w), _np_ptr(sb), _np_ptr(descs), ctypes.byref(n_d)),
               "vdc_stream_program")
        return words, sb, descs

    def debug_alloc(self, masks, nslots, n_slots, stream=None):
        """masks (int32/uint32 CUDA tensor), nslots (int32 CUDA tensor) -> positions (int32 CUDA tensor)."""
        import torch
        pos = torch.empty(masks.numel(), dtype=torch.int32, device=masks.device)
        _check(lib().vdc_debug_alloc(self.handle, masks.data_ptr(), nslots.data_ptr(), n_slots, pos.data_ptr(),
                                     masks.numel(), _stream_ptr(stream)), "vdc_debug_alloc")
        return pos
