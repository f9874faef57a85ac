"""ctypes front end of libhag: argument marshalling only.

Function names follow include/hag.h.  Host arrays are numpy; device arrays are
torch tensors used purely as device memory (data_ptr) and for the current
stream.  Every step of the aggregation path runs in the library's HIP kernels;
there is no fallback: if libhag.so is missing or fails to load, importing a
symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("HAG_LIB", os.path.join(_HERE, "libhag.so"))

HAG_SUM, HAG_MEAN, HAG_MAX, HAG_GCN = 0, 1, 2, 3
HAG_F32, HAG_I32 = 0, 1
HAG_OK, HAG_EINVAL, HAG_ENOMEM, HAG_EHIP, HAG_ESTATE, HAG_ETIMEOUT = 0, -1, -2, -3, -4, -5
HAG_OPT_ONE_LAUNCH_MAX_ITEMS, HAG_OPT_SPIN_LIMIT, HAG_OPT_TEST_WAIT_UNREACHABLE, HAG_OPT_DETERMINISTIC_MAX_BACKWARD = 1, 2, 3, 4
HAG_OPT_SEQ_ONE_LAUNCH = 6
HAG_OPT_PARTITION_SHIFT = 5
HAG_SEARCH_CANONICAL, HAG_SEARCH_DEDUP, HAG_SEARCH_DEVICE = 1, 2, 4
HAG_PHASE_LEVELS, HAG_PHASE_GATHER, HAG_PHASE_FOLD, HAG_PHASE_ALL = 1, 2, 4, 7
OPS = {"sum": HAG_SUM, "mean": HAG_MEAN, "max": HAG_MAX, "gcn": HAG_GCN}

EXPORTS = [
    "hag_search", "hag_search_batched", "hag_from_merges", "hag_prefix", "hag_free", "hag_stats",
    "hag_get_merges", "hag_get_forward", "hag_upload", "hag_workspace_bytes", "hag_forward",
    "hag_backward", "hag_forward_phases", "hag_backward_phases", "hag_naive_forward", "hag_naive_backward",
    "hag_algorithmic_bytes", "hag_last_error", "hag_forward_static_scratch", "hag_probe_rows", "hag_probe_copy", "hag_probe_mfma_f32", "hag_set_option", "hag_check", "hag_seq_search",
    "hag_seq_create", "hag_seq_free", "hag_seq_cells", "hag_seq_ranks", "hag_seq_launches", "hag_seq_get_plan", "hag_seq_set_option", "hag_seq_check", "hag_seq_train_workspace_bytes", "hag_seq_lstm_forward_train", "hag_seq_lstm_backward", "hag_seq_merges", "hag_seq_upload", "hag_seq_workspace_bytes",
    "hag_seq_lstm_forward",
]
HAG_STATIC_SCRATCH_BYTES = 64 << 20


class HagError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libhag error {code}: {msg}")
        self.code = code


class hag_stats_t(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in (
        "n", "e", "a", "levels", "h", "e_hag", "aggr_naive", "aggr_hag", "xfer_naive", "xfer_hag",
        "max_degree", "max_hag_degree", "stages", "components")]


_lib = None


def lib():
    """Load libhag.so (built by paper_1906_03707_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_1906_03707_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32
        L.hag_search.argtypes = [i64, vp, vp, i64, u32, i32, ctypes.POINTER(vp)]
        L.hag_search_batched.argtypes = [i64, vp, vp, i64, vp, ctypes.c_double, u32, i32, ctypes.POINTER(vp)]
        L.hag_from_merges.argtypes = [i64, vp, vp, i64, vp, vp, u32, ctypes.POINTER(vp)]
        L.hag_prefix.argtypes = [vp, i64, ctypes.POINTER(vp)]
        L.hag_free.argtypes = [vp]
        L.hag_free.restype = None
        L.hag_stats.argtypes = [vp, ctypes.POINTER(hag_stats_t)]
        L.hag_get_merges.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp)]
        L.hag_get_forward.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                      ctypes.POINTER(i32), ctypes.POINTER(vp), ctypes.POINTER(vp)]
        L.hag_upload.argtypes = [vp, vp]
        L.hag_workspace_bytes.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64]
        L.hag_workspace_bytes.restype = ctypes.c_size_t
        for name in ("hag_forward", "hag_naive_forward"):
            getattr(L, name).argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, vp, vp, vp, vp, vp]
        for name in ("hag_backward", "hag_naive_backward"):
            getattr(L, name).argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, vp, vp, vp, vp, vp]
        for name in ("hag_forward_phases", "hag_backward_phases"):
            getattr(L, name).argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, vp, vp, vp, vp, vp, u32]
        L.hag_algorithmic_bytes.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64]
        L.hag_algorithmic_bytes.restype = i64
        L.hag_last_error.restype = ctypes.c_char_p
        L.hag_forward_static_scratch.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, vp, vp, vp, vp]
        L.hag_probe_rows.argtypes = [vp, i64, i64, i64, i32, i64, vp, vp]
        L.hag_probe_rows.restype = i64
        L.hag_probe_copy.argtypes = [vp, vp, i64, vp]
        L.hag_probe_mfma_f32.argtypes = [i64, i64, vp, vp]
        L.hag_probe_mfma_f32.restype = i64
        L.hag_seq_search.argtypes = [i64, vp, vp, i64, ctypes.POINTER(i64), vp, vp, vp, vp, vp]
        L.hag_seq_create.argtypes = [i64, vp, vp, i64, ctypes.POINTER(vp)]
        L.hag_seq_free.argtypes = [vp]
        L.hag_seq_free.restype = None
        for name in ("hag_seq_cells", "hag_seq_ranks", "hag_seq_launches", "hag_seq_merges"):
            getattr(L, name).argtypes = [vp]
            getattr(L, name).restype = i64
        L.hag_seq_upload.argtypes = [vp]
        L.hag_seq_get_plan.argtypes = [vp, i32] + [vp] * 8
        L.hag_seq_set_option.argtypes = [vp, i32, i64]
        L.hag_seq_check.argtypes = [vp, vp]
        L.hag_seq_train_workspace_bytes.argtypes = [vp, i64, i64]
        L.hag_seq_train_workspace_bytes.restype = ctypes.c_size_t
        L.hag_seq_lstm_forward_train.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp, vp]
        L.hag_seq_lstm_backward.argtypes = [vp, i64, i64] + [vp] * 10
        L.hag_seq_workspace_bytes.argtypes = [vp, i64, i64]
        L.hag_seq_workspace_bytes.restype = ctypes.c_size_t
        L.hag_seq_lstm_forward.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp, vp]
        L.hag_set_option.argtypes = [vp, i32, i64]
        L.hag_check.argtypes = [vp, vp]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise HagError(rc, lib().hag_last_error().decode())


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _view(ptr, count, dtype):
    if count == 0 or not ptr:
        return np.zeros(0, dtype=dtype)
    ct = {np.int32: ctypes.c_int32, np.int64: ctypes.c_int64}[dtype]
    return np.ctypeslib.as_array(ctypes.cast(ptr, ctypes.POINTER(ct)), shape=(count,)).copy()


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return HAG_F32
    if t.dtype == torch.int32:
        return HAG_I32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device tensors must be contiguous and on the GPU")
    return ctypes.c_void_p(t.data_ptr())


class Hag:
    """Owner of one hag_t handle."""

    def __init__(self, handle):
        self._h = ctypes.c_void_p(handle)
        self._ws = {}
        self._n = None

    def __del__(self):
        try:
            if self._h:
                lib().hag_free(self._h)
                self._h = None
        except Exception:
            pass

    # ---- host side ---------------------------------------------------------------------------
    def stats(self) -> dict:
        s = hag_stats_t()
        _check(lib().hag_stats(self._h, ctypes.byref(s)))
        return {k: getattr(s, k) for k, _ in s._fields_}

    def get_merges(self):
        n = ctypes.c_int64()
        l, r, red = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        _check(lib().hag_get_merges(self._h, ctypes.byref(n), ctypes.byref(l), ctypes.byref(r), ctypes.byref(red)))
        return _view(l.value, n.value, np.int32), _view(r.value, n.value, np.int32), _view(red.value, n.value, np.int32)

    def get_forward(self):
        st = self.stats()
        l, r, lp, hp, hc = (ctypes.c_void_p() for _ in range(5))
        nl = ctypes.c_int32()
        _check(lib().hag_get_forward(self._h, ctypes.byref(l), ctypes.byref(r), ctypes.byref(lp), ctypes.byref(nl),
                                     ctypes.byref(hp), ctypes.byref(hc)))
        return dict(agg_left=_view(l.value, st["a"], np.int32), agg_right=_view(r.value, st["a"], np.int32),
                    level_ptr=_view(lp.value, nl.value + 1, np.int32), n_levels=nl.value,
                    hrowptr=_view(hp.value, st["n"] + 1, np.int64), hcol=_view(hc.value, st["h"], np.int32))

    def prefix(self, n_merges) -> "Hag":
        out = ctypes.c_void_p()
        _check(lib().hag_prefix(self._h, int(n_merges), ctypes.byref(out)))
        return Hag(out.value)

    def algorithmic_bytes(self, which, op, d) -> int:
        return int(lib().hag_algorithmic_bytes(self._h, which, OPS[op], int(d)))

    # ---- device side -------------------------------------------------------------------------
    def upload(self):
        _check(lib().hag_upload(self._h, _stream_ptr()))
        return self

    def set_option(self, option, value):
        _check(lib().hag_set_option(self._h, int(option), int(value)))
        return self

    def check(self):
        """Synchronises the current stream; raises HagError(HAG_ETIMEOUT) if a one-launch pass gave up waiting."""
        _check(lib().hag_check(self._h, _stream_ptr()))

    def workspace_bytes(self, op, dtype_code, d) -> int:
        return int(lib().hag_workspace_bytes(self._h, OPS[op], dtype_code, int(d)))

    def _workspace(self, op, t):
        import torch
        nbytes = self.workspace_bytes(op, _dtype_code(t), t.shape[1])
        # one buffer per (device, stream): calls enqueued on different streams may overlap
        key = (t.device.index, torch.cuda.current_stream(t.device).cuda_stream)
        ws = self._ws.get(key)
        if ws is None or ws.numel() < nbytes:
            ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=t.device)
            self._ws[key] = ws
        return ws

    def _check_args(self, what, a, op, out, argmax, workspace, needs_argmax):
        """Everything the C ABI cannot check from raw pointers: the library takes no row count, so a
        matrix with too few rows, a narrower dtype or a short workspace would make a kernel read or
        write out of bounds."""
        import torch
        if op not in OPS:
            raise ValueError(f"unknown op {op!r}")
        if self._n is None:
            self._n = self.stats()["n"]
        if a.dim() != 2 or a.shape[0] != self._n:
            raise ValueError(f"{what} must have shape [{self._n}, d], got {tuple(a.shape)}")
        code = _dtype_code(a)
        for name, t in (("output", out),):
            if t is not None and (t.shape != a.shape or t.dtype != a.dtype or t.device != a.device):
                raise ValueError(f"{name} must match {what}: shape {tuple(a.shape)}, dtype {a.dtype}, device {a.device}; "
                                 f"got {tuple(t.shape)}, {t.dtype}, {t.device}")
        if argmax is not None and (argmax.shape != a.shape or argmax.dtype != torch.int32 or argmax.device != a.device):
            raise ValueError(f"argmax must be int32 of shape {tuple(a.shape)} on {a.device}, got {argmax.dtype} "
                             f"{tuple(argmax.shape)} on {argmax.device}")
        if needs_argmax and argmax is None:
            raise ValueError("argmax is required for max")
        if workspace is not None:
            need = self.workspace_bytes(op, code, a.shape[1])
            have = workspace.numel() * workspace.element_size()
            if have < need or workspace.device != a.device:
                raise ValueError(f"workspace holds {have} bytes on {workspace.device}, {need} needed on {a.device}")

    def _fwd(self, fn, x, op, y, argmax, workspace, *extra):
        import torch
        self._check_args("x", x, op, y, argmax, workspace, False)
        n, d = x.shape
        if y is None:
            y = torch.empty_like(x)
        if op == "max" and argmax is None:
            argmax = torch.empty((n, d), dtype=torch.int32, device=x.device)
        ws = workspace if workspace is not None else self._workspace(op, x)
        _check(fn(self._h, OPS[op], _dtype_code(x), d, _dev_ptr(x), _dev_ptr(y), _dev_ptr(argmax), _dev_ptr(ws),
                  _stream_ptr(), *extra))
        return (y, argmax) if op == "max" else y

    def _bwd(self, fn, gy, op, argmax, gx, workspace, *extra):
        import torch
        self._check_args("gy", gy, op, gx, argmax, workspace, op == "max")
        n, d = gy.shape
        if gx is None:
            gx = torch.empty_like(gy)
        ws = workspace if workspace is not None else self._workspace(op, gy)
        _check(fn(self._h, OPS[op], _dtype_code(gy), d, _dev_ptr(gy), _dev_ptr(argmax), _dev_ptr(gx), _dev_ptr(ws),
                  _stream_ptr(), *extra))
        return gx

    def forward(self, x, op="sum", y=None, argmax=None, workspace=None):
        return self._fwd(lib().hag_forward, x, op, y, argmax, workspace)

    def backward(self, gy, op="sum", argmax=None, gx=None, workspace=None):
        return self._bwd(lib().hag_backward, gy, op, argmax, gx, workspace)

    def forward_static_scratch(self, x, op="sum", y=None, argmax=None):
        """hag_forward with the library's fixed scratch array as workspace (no workspace argument)."""
        import torch
        self._check_args("x", x, op, y, argmax, None, False)
        n, d = x.shape
        if y is None:
            y = torch.empty_like(x)
        if op == "max" and argmax is None:
            argmax = torch.empty((n, d), dtype=torch.int32, device=x.device)
        _check(lib().hag_forward_static_scratch(self._h, OPS[op], _dtype_code(x), d, _dev_ptr(x), _dev_ptr(y),
                                                _dev_ptr(argmax), _stream_ptr()))
        return (y, argmax) if op == "max" else y

    def forward_phases(self, x, phases, op="sum", y=None, argmax=None, workspace=None):
        return self._fwd(lib().hag_forward_phases, x, op, y, argmax, workspace, int(phases))

    def backward_phases(self, gy, phases, op="sum", argmax=None, gx=None, workspace=None):
        return self._bwd(lib().hag_backward_phases, gy, op, argmax, gx, workspace, int(phases))

    def naive_forward(self, x, op="sum", y=None, argmax=None, workspace=None):
        return self._fwd(lib().hag_naive_forward, x, op, y, argmax, workspace)

    def naive_backward(self, gy, op="sum", argmax=None, gx=None, workspace=None):
        return self._bwd(lib().hag_naive_backward, gy, op, argmax, gx, workspace)


def hag_search(rowptr, col, capacity, flags=HAG_SEARCH_CANONICAL, max_depth=0) -> Hag:
    rowptr, col = _np(rowptr, np.int64), _np(col, np.int32)
    out = ctypes.c_void_p()
    _check(lib().hag_search(rowptr.size - 1, rowptr.ctypes.data, col.ctypes.data, int(capacity), flags, max_depth,
                            ctypes.byref(out)))
    return Hag(out.value)


def hag_search_batched(rowptr, col, graph_ptr, capacity_fraction, flags=HAG_SEARCH_CANONICAL, max_depth=0) -> Hag:
    rowptr, col, graph_ptr = _np(rowptr, np.int64), _np(col, np.int32), _np(graph_ptr, np.int64)
    out = ctypes.c_void_p()
    _check(lib().hag_search_batched(rowptr.size - 1, rowptr.ctypes.data, col.ctypes.data, graph_ptr.size - 1,
                                    graph_ptr.ctypes.data, float(capacity_fraction), flags, max_depth,
                                    ctypes.byref(out)))
    return Hag(out.value)


def hag_from_merges(rowptr, col, left, right, flags=0) -> Hag:
    rowptr, col = _np(rowptr, np.int64), _np(col, np.int32)
    left, right = _np(left, np.int32), _np(right, np.int32)
    out = ctypes.c_void_p()
    _check(lib().hag_from_merges(rowptr.size - 1, rowptr.ctypes.data, col.ctypes.data, left.size,
                                 left.ctypes.data, right.ctypes.data, flags, ctypes.byref(out)))
    return Hag(out.value)


def probe_rows(src, n_rows, d, reads, from_lds, workgroups, sink) -> int:
    """hag_probe_rows on torch device tensors; returns the row bytes the launch reads."""
    if src.numel() < n_rows * d or sink.numel() < workgroups * 1024:
        raise ValueError("probe buffers too small")
    rc = lib().hag_probe_rows(_dev_ptr(src), int(n_rows), int(d), int(reads), int(from_lds), int(workgroups),
                              _dev_ptr(sink), _stream_ptr())
    if rc < 0:
        _check(rc)
    return int(rc)


def probe_copy(src, dst, nbytes):
    if src.numel() * src.element_size() < nbytes or dst.numel() * dst.element_size() < nbytes:
        raise ValueError("copy buffers too small")
    _check(lib().hag_probe_copy(_dev_ptr(src), _dev_ptr(dst), int(nbytes), _stream_ptr()))


def probe_mfma_f32(iters, workgroups, sink) -> int:
    """hag_probe_mfma_f32; returns the flops of the launch."""
    if sink.numel() * sink.element_size() < workgroups * 1024:
        raise ValueError("sink too small")
    rc = lib().hag_probe_mfma_f32(int(iters), int(workgroups), _dev_ptr(sink), _stream_ptr())
    if rc < 0:
        _check(int(rc))
    return int(rc)


def hag_seq_search(rowptr, col, capacity):
    """Algorithm 3 for a sequential Aggregate (ordered lists): (left, right, redundancy, hrowptr, hcol)."""
    rowptr, col = _np(rowptr, np.int64), _np(col, np.int32)
    n, e = rowptr.size - 1, int(rowptr[-1]) if rowptr.size else 0
    cap = int(min(max(capacity, 0), e))
    left, right, red = (np.zeros(max(cap, 1), dtype=np.int32) for _ in range(3))
    hrowptr = np.zeros(n + 1, dtype=np.int64)
    hcol = np.zeros(max(e, 1), dtype=np.int32)
    a = ctypes.c_int64()
    _check(lib().hag_seq_search(n, rowptr.ctypes.data, col.ctypes.data, int(capacity), ctypes.byref(a), left.ctypes.data,
                                right.ctypes.data, red.ctypes.data, hrowptr.ctypes.data, hcol.ctypes.data))
    return left[:a.value], right[:a.value], red[:a.value], hrowptr, hcol[:hrowptr[n]]


class SeqHag:
    """Plan of an LSTM aggregator over ordered neighbour lists (hag_seq_create): a prefix HAG when capacity > 0,
    the plain lists when capacity == 0."""

    def __init__(self, rowptr, col, capacity):
        rowptr, col = _np(rowptr, np.int64), _np(col, np.int32)
        self.n = rowptr.size - 1
        h = ctypes.c_void_p()
        _check(lib().hag_seq_create(self.n, rowptr.ctypes.data, col.ctypes.data, int(capacity), ctypes.byref(h)))
        self._h = h
        self._ws = {}

    def __del__(self):
        try:                                # at interpreter shutdown the module's globals may be gone already
            if getattr(self, "_h", None):
                lib().hag_seq_free(self._h)
                self._h = None
        except Exception:
            pass

    @property
    def cells(self) -> int:
        return int(lib().hag_seq_cells(self._h))

    @property
    def ranks(self) -> int:
        return int(lib().hag_seq_ranks(self._h))

    @property
    def launches(self) -> int:
        return int(lib().hag_seq_launches(self._h))

    @property
    def merges(self) -> int:
        return int(lib().hag_seq_merges(self._h))

    def plan(self, order=0):
        """(n_states, paths [n_paths, 4], step_x, step_out, level_ptr, final_state) as copies (hag_seq_get_plan);
        order 0: paths grouped by level, 1: by the depth of their start state (the one-launch pass)."""
        i64, p32, p64 = ctypes.c_int64, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        ns, npaths, nl = i64(), i64(), i64()
        paths, sx, so, fs, lp = p32(), p32(), p32(), p32(), p64()
        _check(lib().hag_seq_get_plan(self._h, int(order), ctypes.byref(ns), ctypes.byref(npaths), ctypes.byref(paths), ctypes.byref(sx),
                                      ctypes.byref(so), ctypes.byref(nl), ctypes.byref(lp), ctypes.byref(fs)))
        take = lambda ptr, count, dt: (np.ctypeslib.as_array(ptr, shape=(count,)).astype(dt, copy=True) if count else np.zeros(0, dt))
        cells = self.cells
        return (ns.value, take(paths, 4 * npaths.value, np.int32).reshape(-1, 4), take(sx, cells, np.int32), take(so, cells, np.int32),
                take(lp, nl.value + 1, np.int64), take(fs, self.n, np.int32))

    def upload(self):
        _check(lib().hag_seq_upload(self._h))
        return self

    def set_option(self, option, value):
        _check(lib().hag_seq_set_option(self._h, int(option), int(value)))
        return self

    def train_workspace_bytes(self, d, hidden) -> int:
        return int(lib().hag_seq_train_workspace_bytes(self._h, int(d), int(hidden)))

    def lstm_forward_train(self, x, w_ih, w_hh, b, workspace=None):
        """As lstm_forward, keeping what lstm_backward needs; returns (a [n, H], workspace)."""
        import torch
        hidden, d = int(w_hh.shape[1]), int(x.shape[1])
        for name, t, shape in (("x", x, (self.n, d)), ("w_ih", w_ih, (4 * hidden, d)), ("w_hh", w_hh, (4 * hidden, hidden)),
                               ("b", b, (4 * hidden,))):
            if tuple(t.shape) != shape or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
                raise ValueError(f"{name} must be a contiguous float32 device tensor of shape {shape}")
        need = self.train_workspace_bytes(d, hidden)
        if need == 0:
            raise ValueError("d must be a multiple of 4, hidden a multiple of 8 up to 128, d + hidden at most 256")
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
        elif workspace.numel() * workspace.element_size() < need or workspace.device != x.device:
            raise ValueError("workspace too small or on another device")
        out = torch.empty((self.n, hidden), dtype=torch.float32, device=x.device)
        _check(lib().hag_seq_lstm_forward_train(self._h, d, hidden, _dev_ptr(x), _dev_ptr(w_ih), _dev_ptr(w_hh), _dev_ptr(b),
                                                _dev_ptr(out), _dev_ptr(workspace), _stream_ptr()))
        return out, workspace

    def lstm_backward(self, x, w_ih, w_hh, g_a, workspace):
        """Gradients (g_x, g_w_ih, g_w_hh, g_b) of a loss with gradient g_a [n, H] at a_out, after lstm_forward_train with
        the same x, w_ih, w_hh and workspace."""
        import torch
        hidden, d = int(w_hh.shape[1]), int(x.shape[1])
        for name, t, shape in (("x", x, (self.n, d)), ("w_ih", w_ih, (4 * hidden, d)), ("w_hh", w_hh, (4 * hidden, hidden)),
                               ("g_a", g_a, (self.n, hidden))):
            if tuple(t.shape) != shape or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
                raise ValueError(f"{name} must be a contiguous float32 device tensor of shape {shape}")
        need = self.train_workspace_bytes(d, hidden)
        if need == 0 or workspace.numel() * workspace.element_size() < need or workspace.device != x.device:
            raise ValueError("workspace too small or on another device")
        new = lambda *shape: torch.empty(shape, dtype=torch.float32, device=x.device)
        g_x, g_w_ih, g_w_hh, g_b = new(self.n, d), new(4 * hidden, d), new(4 * hidden, hidden), new(4 * hidden)
        _check(lib().hag_seq_lstm_backward(self._h, d, hidden, _dev_ptr(x), _dev_ptr(w_ih), _dev_ptr(w_hh), _dev_ptr(g_a), _dev_ptr(g_x),
                                           _dev_ptr(g_w_ih), _dev_ptr(g_w_hh), _dev_ptr(g_b), _dev_ptr(workspace), _stream_ptr()))
        return g_x, g_w_ih, g_w_hh, g_b

    def check(self):
        """Synchronise the current stream; raises HagError(HAG_ETIMEOUT) if a wait of a one-launch pass gave up."""
        _check(lib().hag_seq_check(self._h, _stream_ptr()))

    def workspace_bytes(self, d, hidden) -> int:
        return int(lib().hag_seq_workspace_bytes(self._h, int(d), int(hidden)))

    def lstm_forward(self, x, w_ih, w_hh, b, out=None, workspace=None):
        """a [n, H] = LSTM aggregate of every node's ordered list; torch float32 device tensors."""
        import torch
        hidden, d = int(w_hh.shape[1]), int(x.shape[1])
        for name, t, shape in (("x", x, (self.n, d)), ("w_ih", w_ih, (4 * hidden, d)), ("w_hh", w_hh, (4 * hidden, hidden)),
                               ("b", b, (4 * hidden,))):
            if tuple(t.shape) != shape or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
                raise ValueError(f"{name} must be a contiguous float32 device tensor of shape {shape}")
        if out is None:
            out = torch.empty((self.n, hidden), dtype=torch.float32, device=x.device)
        elif tuple(out.shape) != (self.n, hidden) or out.dtype != torch.float32 or not out.is_contiguous() or out.device != x.device:
            raise ValueError("out must be a contiguous float32 tensor [n, hidden] on x's device")
        need = self.workspace_bytes(d, hidden)
        if workspace is None:
            key = (x.device, torch.cuda.current_stream(x.device).cuda_stream, d, hidden)
            workspace = self._ws.get(key)
            if workspace is None:
                workspace = self._ws[key] = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
        elif workspace.numel() * workspace.element_size() < need or workspace.device != x.device:
            raise ValueError("workspace too small or on another device")
        _check(lib().hag_seq_lstm_forward(self._h, d, hidden, _dev_ptr(x), _dev_ptr(w_ih), _dev_ptr(w_hh), _dev_ptr(b),
                                          _dev_ptr(out), _dev_ptr(workspace), _stream_ptr()))
        return out
