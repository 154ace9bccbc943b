"""Thin ctypes binding of libsprnn.so: argument marshalling only.

The names mirror the C ABI in ``include/sprnn.h``.  PyTorch is used for device memory and streams;
every step of the recurrent path runs inside the HIP library.  If the library is missing this module
raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SPRNN_LIBRARY") or os.path.join(_HERE, "libsprnn.so")   # override: A/B of builds

SPRNN_OK = 0
SPRNN_ERR_INVALID = -1
SPRNN_ERR_CAPACITY = -2
SPRNN_ERR_HIP = -3
SPRNN_ERR_UNSUPPORTED = -4
SPRNN_ERR_STATE = -5

CELLS = {"relu": 0, "tanh": 1, "identity": 2, "lstm": 3, "gru": 4, "lstm_backward": 5, "gru_backward": 6}
GATES = {"lstm": 4, "gru": 3}
SYNC = {"auto": 0, "tagged": 1, "barrier": 2}
LAYOUT = {"auto": 0, "row_groups": 1, "lane_pool": 2}
GATHER = {"auto": 0, "wide": 1, "narrow": 2}
ACTIVATIONS = {"auto": 0, "binary32": 1, "binary16": 2}
XCD = {"auto": 0, "spread": 1, "one": 2}
LAUNCH = {"auto": 0, "ordinary": 1, "cooperative": 2}

EXPORTS = ["sprnn_create", "sprnn_create_ex", "sprnn_forward", "sprnn_forward_noalloc", "sprnn_forward_lstm", "sprnn_forward_lstm_train", "sprnn_forward_gru",
           "sprnn_forward_stepwise", "sprnn_backward_lstm", "sprnn_backward_lstm_with_weights", "sprnn_forward_gru_train",
           "sprnn_backward_gru", "sprnn_backward_gru_with_weights",
           "sprnn_project", "sprnn_backward", "sprnn_backward_with_weights", "sprnn_weight_gradient", "sprnn_transpose_csr",
           "sprnn_get_info", "sprnn_read_timeline", "sprnn_check", "sprnn_pack_host", "sprnn_free_host", "sprnn_status_string",
           "sprnn_destroy"]


class Options(ctypes.Structure):
    _fields_ = [("grid", ctypes.c_int), ("waves", ctypes.c_int), ("lanes_per_row", ctypes.c_int),
                ("sync", ctypes.c_int), ("bank_aware", ctypes.c_int), ("balance", ctypes.c_int),
                ("poll_delay", ctypes.c_int), ("spin_limit", ctypes.c_int), ("timeline", ctypes.c_int),
                ("fill_waves", ctypes.c_int), ("launch", ctypes.c_int), ("jitter", ctypes.c_int), ("compact", ctypes.c_int), ("layout", ctypes.c_int),
                ("gather", ctypes.c_int), ("xcd", ctypes.c_int), ("overlap", ctypes.c_int), ("activations", ctypes.c_int)]


class Info(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int), ("rows", ctypes.c_int), ("batch", ctypes.c_int), ("cell", ctypes.c_int),
                ("grid", ctypes.c_int), ("block", ctypes.c_int), ("waves", ctypes.c_int),
                ("lanes_per_row", ctypes.c_int), ("sync", ctypes.c_int), ("bank_aware", ctypes.c_int),
                ("balance", ctypes.c_int), ("poll_delay", ctypes.c_int),
                ("words_per_lane_max", ctypes.c_int), ("template_words", ctypes.c_int),
                ("lds_bytes", ctypes.c_int), ("resident_capacity", ctypes.c_int),
                ("nnz", ctypes.c_int64), ("padded_words", ctypes.c_int64), ("ring_bytes", ctypes.c_int64),
                ("lds_pass_factor", ctypes.c_double), ("compact", ctypes.c_int), ("layout", ctypes.c_int),
                ("gather_waves", ctypes.c_int), ("one_xcd", ctypes.c_int), ("overlap_rounds", ctypes.c_int),
                ("overlap_words", ctypes.c_int), ("activations", ctypes.c_int), ("reserved", ctypes.c_int * 1)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


class SprnnError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (what, status_string(code), code))


_lib = None


def hip_runtimes_mapped() -> set:
    """Paths of the HIP runtime libraries (libamdhip64) mapped into this process."""
    found = set()
    try:
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    found.add(line.split()[-1])
    except OSError:
        pass
    return found


def load_with_one_runtime(path: str) -> ctypes.CDLL:
    """dlopen a HIP library of this package so that the process keeps ONE HIP runtime (see load_library)."""
    if not hip_runtimes_mapped():
        import torch  # noqa: F401  (maps torch's bundled HIP runtime before the library asks for one)
    lib = ctypes.CDLL(path)
    runtimes = hip_runtimes_mapped()
    if len(runtimes) > 1:
        raise ImportError("two HIP runtimes are mapped into this process (%s): load %s after the runtime the "
                          "application uses, e.g. import torch first" % (", ".join(sorted(runtimes)), os.path.basename(path)))
    return lib


def load_library() -> ctypes.CDLL:
    """Load libsprnn.so from the package directory; fails loudly when it has not been built.

    One HIP runtime per process: libsprnn.so depends on libamdhip64.so.7 and the dynamic linker gives it the copy the
    process already holds.  PyTorch ships its own copy, and this binding hands torch's streams and device pointers to
    the library, so torch has to be in the process first; with no runtime mapped yet it is imported here, and a process
    that ends up with two different runtimes is refused.
    """
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libsprnn.so is missing: build it with `python -m paper_1804_10223_amd.build` "
                          "(there is no fallback path)")
    lib = load_with_one_runtime(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    i32p, u16p, u32pp, i32pp = (ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint16),
                                ctypes.POINTER(ctypes.POINTER(ctypes.c_uint32)),
                                ctypes.POINTER(ctypes.POINTER(ctypes.c_int32)))
    lib.sprnn_create.restype = ci
    lib.sprnn_create.argtypes = [ctypes.POINTER(vp), ci, ci, ci, i32p, i32p, u16p, ci]
    lib.sprnn_create_ex.restype = ci
    lib.sprnn_create_ex.argtypes = [ctypes.POINTER(vp), ci, ci, ci, i32p, i32p, u16p, ci, ctypes.POINTER(Options)]
    lib.sprnn_forward.restype = ci
    lib.sprnn_forward.argtypes = [vp, ci, vp, vp, vp, vp]
    lib.sprnn_forward_noalloc.restype = ci
    lib.sprnn_forward_noalloc.argtypes = [vp, ci, vp, vp, vp, vp]
    lib.sprnn_forward_lstm.restype = ci
    lib.sprnn_forward_lstm.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp]
    lib.sprnn_forward_lstm_train.restype = ci
    lib.sprnn_forward_lstm_train.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.sprnn_backward_lstm.restype = ci
    lib.sprnn_backward_lstm.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.sprnn_backward_lstm_with_weights.restype = ci
    lib.sprnn_backward_lstm_with_weights.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.sprnn_forward_gru_train.restype = ci
    lib.sprnn_forward_gru_train.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp]
    lib.sprnn_backward_gru.restype = ci
    lib.sprnn_backward_gru.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.sprnn_backward_gru_with_weights.restype = ci
    lib.sprnn_backward_gru_with_weights.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.sprnn_forward_gru.restype = ci
    lib.sprnn_forward_gru.argtypes = [vp, ci, vp, vp, vp, vp, vp]
    lib.sprnn_backward.restype = ci
    lib.sprnn_backward.argtypes = [vp, ci, vp, vp, vp, vp, vp]
    lib.sprnn_weight_gradient.restype = ci
    lib.sprnn_weight_gradient.argtypes = [vp, ci, vp, vp, vp, vp, vp]
    lib.sprnn_transpose_csr.restype = ci
    lib.sprnn_transpose_csr.argtypes = [ci, ci, i32p, i32p, u16p, i32p, i32p, u16p, i32p]
    lib.sprnn_backward_with_weights.restype = ci
    lib.sprnn_backward_with_weights.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.sprnn_forward_stepwise.restype = ci
    lib.sprnn_forward_stepwise.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp]
    lib.sprnn_project.restype = ci
    lib.sprnn_project.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp]
    lib.sprnn_get_info.restype = ci
    lib.sprnn_get_info.argtypes = [vp, ctypes.POINTER(Info)]
    lib.sprnn_check.restype = ci
    lib.sprnn_check.argtypes = [vp]
    lib.sprnn_read_timeline.restype = ci
    lib.sprnn_read_timeline.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), ci, ctypes.POINTER(ctypes.c_double)]
    lib.sprnn_pack_host.restype = ci
    lib.sprnn_pack_host.argtypes = [ci, ci, ci, i32p, i32p, u16p, ctypes.POINTER(Options), ci, u32pp, i32pp, i32pp,
                                    ctypes.POINTER(Info)]
    lib.sprnn_free_host.restype = None
    lib.sprnn_free_host.argtypes = [vp]
    lib.sprnn_status_string.restype = ctypes.c_char_p
    lib.sprnn_status_string.argtypes = [ci]
    lib.sprnn_destroy.restype = ci
    lib.sprnn_destroy.argtypes = [vp]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().sprnn_status_string(int(code)).decode()


def make_options(**kw) -> Options:
    o = Options()
    for k, v in kw.items():
        if k == "sync" and isinstance(v, str):
            v = SYNC[v]
        if k == "layout" and isinstance(v, str):
            v = LAYOUT[v]
        if k == "gather" and isinstance(v, str):
            v = GATHER[v]
        if k == "xcd" and isinstance(v, str):
            v = XCD[v]
        if k == "activations" and isinstance(v, str):
            v = ACTIVATIONS[v]
        if k == "launch" and isinstance(v, str):
            v = LAUNCH[v]
        if not hasattr(o, k):
            raise TypeError("unknown option %r" % k)
        setattr(o, k, int(v))
    return o


def _csr_args(row_ptr, col_idx, val_bits):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    val_bits = np.ascontiguousarray(val_bits, dtype=np.uint16)
    keep = (row_ptr, col_idx, val_bits)
    i32p, u16p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint16)
    cp = col_idx.ctypes.data_as(i32p) if col_idx.size else ctypes.cast(None, i32p)
    vp = val_bits.ctypes.data_as(u16p) if val_bits.size else ctypes.cast(None, u16p)
    return keep, row_ptr.ctypes.data_as(i32p), cp, vp


def pack_host(hidden: int, batch: int, cell: str, row_ptr, col_idx, val_bits, num_cus: int = 256, **options):
    """sprnn_pack_host: the packed register image as numpy arrays (no GPU needed).

    Returns (words [grid, template_words, block] uint32, lane_row [grid, block] int32,
    lane_words [grid, block] int32, info dict).
    """
    lib = load_library()
    keep, rp, cp, vp = _csr_args(row_ptr, col_idx, val_bits)
    opt = make_options(**options)
    words = ctypes.POINTER(ctypes.c_uint32)()
    lane_row = ctypes.POINTER(ctypes.c_int32)()
    lane_words = ctypes.POINTER(ctypes.c_int32)()
    info = Info()
    rc = lib.sprnn_pack_host(hidden, batch, CELLS[cell], rp, cp, vp, ctypes.byref(opt), num_cus,
                             ctypes.byref(words), ctypes.byref(lane_row), ctypes.byref(lane_words), ctypes.byref(info))
    if rc != SPRNN_OK:
        raise SprnnError(rc, "sprnn_pack_host")
    try:
        g, nw, blk = info.grid, info.template_words, info.block
        w = np.ctypeslib.as_array(words, shape=(g, nw, blk)).copy()
        lr = np.ctypeslib.as_array(lane_row, shape=(g, blk)).copy()
        lw = np.ctypeslib.as_array(lane_words, shape=(g, blk)).copy()
    finally:
        lib.sprnn_free_host(ctypes.cast(words, ctypes.c_void_p))
        lib.sprnn_free_host(ctypes.cast(lane_row, ctypes.c_void_p))
        lib.sprnn_free_host(ctypes.cast(lane_words, ctypes.c_void_p))
    return w, lr, lw, info.as_dict()


def _dev_ptr(t, shape, what):
    import torch
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 CUDA tensor" % what)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (what, tuple(shape), tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


class SparseRNN:
    """Owner of one sprnn handle.  ``cell`` is "relu" | "tanh" | "identity" | "lstm"."""

    def __init__(self, hidden: int, batch: int, cell: str, row_ptr, col_idx, val_bits, device: int = 0, **options):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.hidden, self.batch, self.cell = int(hidden), int(batch), cell
        self.rows = self.hidden * GATES.get(cell, 1)
        self.device = int(device)
        keep, rp, cp, vp = _csr_args(row_ptr, col_idx, val_bits)
        opt = make_options(**options)
        rc = self._lib.sprnn_create_ex(ctypes.byref(self._h), self.hidden, self.batch, CELLS[cell], rp, cp, vp,
                                       self.device, ctypes.byref(opt))
        if rc != SPRNN_OK:
            self._h = ctypes.c_void_p()
            raise SprnnError(rc, "sprnn_create_ex")

    # -- life cycle
    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.sprnn_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- queries
    def info(self) -> dict:
        i = Info()
        rc = self._lib.sprnn_get_info(self._h, ctypes.byref(i))
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_get_info")
        return i.as_dict()

    def read_timeline(self):
        """sprnn_read_timeline: (ticks [grid, 16] uint64, ticks_per_second); clears the accumulators."""
        g = self.info()["grid"]
        buf = np.zeros((g, 16), dtype=np.uint64)
        hz = ctypes.c_double()
        rc = self._lib.sprnn_read_timeline(self._h, buf.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), g * 16,
                                           ctypes.byref(hz))
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_read_timeline")
        return buf, hz.value

    def _nnz(self) -> int:
        if getattr(self, "_nnz_cached", None) is None:
            self._nnz_cached = int(self.info()["nnz"])
        return self._nnz_cached

    def check(self) -> int:
        """sprnn_check: synchronise and return the status code (SPRNN_OK or SPRNN_ERR_STATE)."""
        return int(self._lib.sprnn_check(self._h))

    # -- forward passes (enqueue on torch's current stream of the handle's device)
    def _stream(self):
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)

    def _alloc(self, T):
        import torch
        return torch.empty((T, self.batch, self.hidden), dtype=torch.float32, device="cuda:%d" % self.device)

    def forward(self, x, h0=None, h_out=None):
        """sprnn_forward: x [T, B, H] -> h_out [T, B, H] (vanilla cells)."""
        T = int(x.shape[0])
        if h_out is None:
            h_out = self._alloc(T)
        rc = self._lib.sprnn_forward(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                     _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                     _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward")
        return h_out

    def forward_noalloc(self, x, h0, h_out):
        """sprnn_forward_noalloc: as forward, exchange ring in the library's static device array; h_out is the caller's."""
        T = int(x.shape[0])
        rc = self._lib.sprnn_forward_noalloc(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                             _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                             _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward_noalloc")
        return h_out

    def forward_lstm(self, x, h0=None, c0=None, h_out=None, c_out=None):
        """sprnn_forward_lstm: x [T, B, 4H] -> (h_out, c_out), each [T, B, H]."""
        T = int(x.shape[0])
        if h_out is None:
            h_out = self._alloc(T)
        if c_out is None:
            c_out = self._alloc(T)
        rc = self._lib.sprnn_forward_lstm(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                          _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                          _dev_ptr(c0, (self.batch, self.hidden), "c0"),
                                          _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"),
                                          _dev_ptr(c_out, (T, self.batch, self.hidden), "c_out"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward_lstm")
        return h_out, c_out

    def forward_lstm_train(self, x, h0=None, c0=None, h_out=None, c_out=None, gates=None):
        """sprnn_forward_lstm_train: x [T, B, 4H] -> (h_out, c_out [T, B, H], gates [T, B, 4H] after their activations).
        Outputs the caller does not pass are allocated here."""
        import torch
        T = int(x.shape[0])
        h_out = self._alloc(T) if h_out is None else h_out
        c_out = self._alloc(T) if c_out is None else c_out
        if gates is None:
            gates = torch.empty((T, self.batch, self.rows), dtype=torch.float32, device="cuda:%d" % self.device)
        rc = self._lib.sprnn_forward_lstm_train(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                                _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                                _dev_ptr(c0, (self.batch, self.hidden), "c0"),
                                                _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"),
                                                _dev_ptr(c_out, (T, self.batch, self.hidden), "c_out"),
                                                _dev_ptr(gates, (T, self.batch, self.rows), "gates_out"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward_lstm_train")
        return h_out, c_out, gates

    def backward_lstm(self, dh_ext, gates, c_fwd, c0=None, want_dh0=True, want_dc0=True, d_bprime=None, dh0=None, dc0=None):
        """sprnn_backward_lstm on a "lstm_backward" handle (the TRANSPOSED [H][4H] matrix):
        (d_bprime [T, B, 4H], dh0 [B, H] or None, dc0 [B, H] or None).  Outputs the caller does not pass are allocated here."""
        import torch
        T = int(dh_ext.shape[0])
        dev = "cuda:%d" % self.device
        if d_bprime is None:
            d_bprime = torch.empty((T, self.batch, 4 * self.hidden), dtype=torch.float32, device=dev)
        if dh0 is None and want_dh0:
            dh0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        if dc0 is None and want_dc0:
            dc0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        rc = self._lib.sprnn_backward_lstm(self._h, T, _dev_ptr(dh_ext, (T, self.batch, self.hidden), "dh_ext"),
                                           _dev_ptr(gates, (T, self.batch, 4 * self.hidden), "gates"),
                                           _dev_ptr(c_fwd, (T, self.batch, self.hidden), "c_fwd"),
                                           _dev_ptr(c0, (self.batch, self.hidden), "c0"),
                                           _dev_ptr(d_bprime, (T, self.batch, 4 * self.hidden), "d_bprime"),
                                           _dev_ptr(dh0, (self.batch, self.hidden), "dh0"),
                                           _dev_ptr(dc0, (self.batch, self.hidden), "dc0"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_backward_lstm")
        return d_bprime, dh0, dc0

    def backward_lstm_with_weights(self, dh_ext, gates, c_fwd, h_fwd, c0=None, h0=None, want_dh0=True, want_dc0=True,
                                   d_bprime=None, dh0=None, dc0=None, dU=None):
        """sprnn_backward_lstm_with_weights on a "lstm_backward" handle:
        (d_bprime [T, B, 4H], dh0, dc0 [B, H] or None, dU [nnz] in the transposed matrix's CSR order).
        Outputs the caller does not pass are allocated here (dU: at least max(nnz, 1) elements)."""
        import torch
        T = int(dh_ext.shape[0])
        dev = "cuda:%d" % self.device
        nnz = self._nnz()
        if d_bprime is None:
            d_bprime = torch.empty((T, self.batch, 4 * self.hidden), dtype=torch.float32, device=dev)
        if dh0 is None and want_dh0:
            dh0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        if dc0 is None and want_dc0:
            dc0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        if dU is None:
            dU = torch.empty((max(nnz, 1),), dtype=torch.float32, device=dev)
        rc = self._lib.sprnn_backward_lstm_with_weights(
            self._h, T, _dev_ptr(dh_ext, (T, self.batch, self.hidden), "dh_ext"),
            _dev_ptr(gates, (T, self.batch, 4 * self.hidden), "gates"), _dev_ptr(c_fwd, (T, self.batch, self.hidden), "c_fwd"),
            _dev_ptr(c0, (self.batch, self.hidden), "c0"), _dev_ptr(h_fwd, (T, self.batch, self.hidden), "h_fwd"),
            _dev_ptr(h0, (self.batch, self.hidden), "h0"), _dev_ptr(d_bprime, (T, self.batch, 4 * self.hidden), "d_bprime"),
            _dev_ptr(dh0, (self.batch, self.hidden), "dh0"), _dev_ptr(dc0, (self.batch, self.hidden), "dc0"),
            ctypes.c_void_p(dU.data_ptr()), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_backward_lstm_with_weights")
        return d_bprime, dh0, dc0, dU[:nnz]

    def forward_gru(self, x, b_hn=None, h0=None, h_out=None):
        """sprnn_forward_gru: x [T, B, 3H] (blocks r|z|n), b_hn [H] or None -> h_out [T, B, H]."""
        T = int(x.shape[0])
        if h_out is None:
            h_out = self._alloc(T)
        rc = self._lib.sprnn_forward_gru(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                         _dev_ptr(b_hn, (self.hidden,), "b_hn"),
                                         _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                         _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward_gru")
        return h_out

    def forward_gru_train(self, x, b_hn=None, h0=None, h_out=None, gates=None):
        """sprnn_forward_gru_train: x [T, B, 3H] -> (h_out [T, B, H], gates [T, B, 4H] = r | z | n | q).
        Outputs the caller does not pass are allocated here."""
        import torch
        T = int(x.shape[0])
        if h_out is None:
            h_out = self._alloc(T)
        if gates is None:
            gates = torch.empty((T, self.batch, 4 * self.hidden), dtype=torch.float32, device="cuda:%d" % self.device)
        rc = self._lib.sprnn_forward_gru_train(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                               _dev_ptr(b_hn, (self.hidden,), "b_hn"), _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                               _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"),
                                               _dev_ptr(gates, (T, self.batch, 4 * self.hidden), "gates_out"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward_gru_train")
        return h_out, gates

    def backward_gru(self, dh_ext, gates, h_fwd, h0=None, want_dh0=True, want_recurrent=True, d_bprime=None, d_recurrent=None, dh0=None):
        """sprnn_backward_gru on a "gru_backward" handle (the TRANSPOSED [H][3H] matrix):
        (d_bprime [T, B, 3H], d_recurrent [T, B, 3H] or None, dh0 [B, H] or None).  Outputs the caller does not pass are
        allocated here."""
        import torch
        T = int(dh_ext.shape[0])
        dev = "cuda:%d" % self.device
        if d_bprime is None:
            d_bprime = torch.empty((T, self.batch, 3 * self.hidden), dtype=torch.float32, device=dev)
        d_rec = d_recurrent
        if d_rec is None and want_recurrent:
            d_rec = torch.empty((T, self.batch, 3 * self.hidden), dtype=torch.float32, device=dev)
        if dh0 is None and want_dh0:
            dh0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        rc = self._lib.sprnn_backward_gru(self._h, T, _dev_ptr(dh_ext, (T, self.batch, self.hidden), "dh_ext"),
                                          _dev_ptr(gates, (T, self.batch, 4 * self.hidden), "gates"),
                                          _dev_ptr(h_fwd, (T, self.batch, self.hidden), "h_fwd"),
                                          _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                          _dev_ptr(d_bprime, (T, self.batch, 3 * self.hidden), "d_bprime"),
                                          _dev_ptr(d_rec, (T, self.batch, 3 * self.hidden), "d_recurrent"),
                                          _dev_ptr(dh0, (self.batch, self.hidden), "dh0"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_backward_gru")
        return d_bprime, d_rec, dh0

    def backward_gru_with_weights(self, dh_ext, gates, h_fwd, h0=None, want_dh0=True, want_recurrent=True,
                                  d_bprime=None, d_recurrent=None, dh0=None, dU=None):
        """sprnn_backward_gru_with_weights on a "gru_backward" handle:
        (d_bprime [T, B, 3H], d_recurrent or None, dh0 or None, dU [nnz] in the transposed matrix's CSR order).
        Outputs the caller does not pass are allocated here (dU: at least max(nnz, 1) elements)."""
        import torch
        T = int(dh_ext.shape[0])
        dev = "cuda:%d" % self.device
        nnz = self._nnz()
        if d_bprime is None:
            d_bprime = torch.empty((T, self.batch, 3 * self.hidden), dtype=torch.float32, device=dev)
        d_rec = d_recurrent
        if d_rec is None and want_recurrent:
            d_rec = torch.empty((T, self.batch, 3 * self.hidden), dtype=torch.float32, device=dev)
        if dh0 is None and want_dh0:
            dh0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        if dU is None:
            dU = torch.empty((max(nnz, 1),), dtype=torch.float32, device=dev)
        rc = self._lib.sprnn_backward_gru_with_weights(
            self._h, T, _dev_ptr(dh_ext, (T, self.batch, self.hidden), "dh_ext"),
            _dev_ptr(gates, (T, self.batch, 4 * self.hidden), "gates"), _dev_ptr(h_fwd, (T, self.batch, self.hidden), "h_fwd"),
            _dev_ptr(h0, (self.batch, self.hidden), "h0"), _dev_ptr(d_bprime, (T, self.batch, 3 * self.hidden), "d_bprime"),
            _dev_ptr(d_rec, (T, self.batch, 3 * self.hidden), "d_recurrent"), _dev_ptr(dh0, (self.batch, self.hidden), "dh0"),
            ctypes.c_void_p(dU.data_ptr()), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_backward_gru_with_weights")
        return d_bprime, d_rec, dh0, dU[:nnz]

    def backward(self, dh_ext, h_fwd, d_bprime=None, want_dh0=True, dh0=None):
        """sprnn_backward on a handle that holds the TRANSPOSED matrix: (delta [T, B, H], dh0 [B, H] or None)."""
        import torch
        T = int(dh_ext.shape[0])
        if d_bprime is None:
            d_bprime = self._alloc(T)
        if dh0 is None and want_dh0:
            dh0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device="cuda:%d" % self.device)
        rc = self._lib.sprnn_backward(self._h, T, _dev_ptr(dh_ext, (T, self.batch, self.hidden), "dh_ext"),
                                      _dev_ptr(h_fwd, (T, self.batch, self.hidden), "h_fwd"),
                                      _dev_ptr(d_bprime, (T, self.batch, self.hidden), "d_bprime"),
                                      _dev_ptr(dh0, (self.batch, self.hidden), "dh0"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_backward")
        return d_bprime, dh0

    def backward_with_weights(self, dh_ext, h_fwd, h0=None, d_bprime=None, want_dh0=True, dh0=None, dU=None):
        """sprnn_backward_with_weights on a handle that holds the TRANSPOSED matrix:
        (delta [T, B, H], dh0 [B, H] or None, dU [nnz] in the transposed matrix's CSR order)."""
        import torch
        T = int(dh_ext.shape[0])
        nnz = self._nnz()
        if d_bprime is None:
            d_bprime = self._alloc(T)
        dev = "cuda:%d" % self.device
        if dh0 is None and want_dh0:
            dh0 = torch.empty((self.batch, self.hidden), dtype=torch.float32, device=dev)
        if dU is None:
            dU = torch.empty((max(nnz, 1),), dtype=torch.float32, device=dev)
        rc = self._lib.sprnn_backward_with_weights(self._h, T, _dev_ptr(dh_ext, (T, self.batch, self.hidden), "dh_ext"),
                                                   _dev_ptr(h_fwd, (T, self.batch, self.hidden), "h_fwd"),
                                                   _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                                   _dev_ptr(d_bprime, (T, self.batch, self.hidden), "d_bprime"),
                                                   _dev_ptr(dh0, (self.batch, self.hidden), "dh0"),
                                                   ctypes.c_void_p(dU.data_ptr()), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_backward_with_weights")
        return d_bprime, dh0, dU[:nnz]

    def weight_gradient(self, d_bprime, h_fwd, h0=None, dU=None):
        """sprnn_weight_gradient on the FORWARD handle: dU [nnz] float32 in CSR order."""
        import torch
        T = int(d_bprime.shape[0])
        nnz = self._nnz()
        if dU is None:
            dU = torch.empty((max(nnz, 1),), dtype=torch.float32, device="cuda:%d" % self.device)
        rc = self._lib.sprnn_weight_gradient(self._h, T, _dev_ptr(d_bprime, (T, self.batch, self.rows), "d_bprime"),
                                             _dev_ptr(h_fwd, (T, self.batch, self.hidden), "h_fwd"),
                                             _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                             ctypes.c_void_p(dU.data_ptr()), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_weight_gradient")
        return dU[:nnz]

    def project(self, x_in, w_in_bits, bias=None, b_prime=None):
        """sprnn_project: x_in [T, B, I] float32, w_in_bits [R, I] binary16 (float16 tensor, or its bits as int16/uint16),
        bias [R] or None -> b' [T, B, R], the ``x`` argument of the forward calls."""
        import torch
        T, I = int(x_in.shape[0]), int(x_in.shape[-1])
        if not (isinstance(w_in_bits, torch.Tensor) and w_in_bits.is_cuda and w_in_bits.is_contiguous()
                and w_in_bits.element_size() == 2 and tuple(w_in_bits.shape) == (self.rows, I)):
            raise TypeError("w_in_bits must be a contiguous 16-bit CUDA tensor of shape %s" % ((self.rows, I),))
        if b_prime is None:
            b_prime = torch.empty((T, self.batch, self.rows), dtype=torch.float32, device="cuda:%d" % self.device)
        rc = self._lib.sprnn_project(self._h, T, I, _dev_ptr(x_in, (T, self.batch, I), "x_in"),
                                     ctypes.c_void_p(w_in_bits.data_ptr()), _dev_ptr(bias, (self.rows,), "bias"),
                                     _dev_ptr(b_prime, (T, self.batch, self.rows), "b_prime"), self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_project")
        return b_prime

    def forward_stepwise(self, x, h0=None, c0=None, h_out=None, c_out=None):
        """sprnn_forward_stepwise: the one-launch-per-timestep comparison path; returns (h_out, c_out or None)."""
        T = int(x.shape[0])
        lstm = self.cell == "lstm"
        if h_out is None:
            h_out = self._alloc(T)
        if lstm and c_out is None:
            c_out = self._alloc(T)
        rc = self._lib.sprnn_forward_stepwise(self._h, T, _dev_ptr(x, (T, self.batch, self.rows), "x"),
                                              _dev_ptr(h0, (self.batch, self.hidden), "h0"),
                                              _dev_ptr(c0, (self.batch, self.hidden), "c0") if lstm else None,
                                              _dev_ptr(h_out, (T, self.batch, self.hidden), "h_out"),
                                              _dev_ptr(c_out, (T, self.batch, self.hidden), "c_out") if lstm else None,
                                              self._stream())
        if rc != SPRNN_OK:
            raise SprnnError(rc, "sprnn_forward_stepwise")
        return h_out, c_out


def transpose_csr(rows: int, cols: int, row_ptr, col_idx, val_bits, with_source: bool = False):
    """sprnn_transpose_csr on numpy arrays: (t_row_ptr [cols + 1], t_col_idx, t_val_bits[, t_source])."""
    lib = load_library()
    keep, rp, cp, vp = _csr_args(row_ptr, col_idx, val_bits)
    nnz = int(np.asarray(row_ptr)[rows])
    t_rp = np.zeros(cols + 1, dtype=np.int32)
    t_ci = np.zeros(max(nnz, 1), dtype=np.int32)
    t_vb = np.zeros(max(nnz, 1), dtype=np.uint16)
    t_src = np.zeros(max(nnz, 1), dtype=np.int32)
    rc = lib.sprnn_transpose_csr(rows, cols, rp, cp, vp, t_rp.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 t_ci.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 t_vb.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                                 t_src.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != SPRNN_OK:
        raise SprnnError(rc, "sprnn_transpose_csr")
    if with_source:
        return t_rp, t_ci[:nnz], t_vb[:nnz], t_src[:nnz]
    return t_rp, t_ci[:nnz], t_vb[:nnz]
