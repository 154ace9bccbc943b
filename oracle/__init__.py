"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``liboracle.so`` built from ``sprnn_oracle.c`` (plain C, gcc) and exposes
the oracle's functions on numpy arrays.  Nothing in the product package may
import this module; only ``tests/``, the smoke check and the benchmark's
CPU-baseline leg do.  It imports nothing from the product package.

Cells and equations: see the header of ``sprnn_oracle.c`` (Eq. 2 of the paper
for the vanilla cell; Appendix B's four-gate LSTM; a three-gate GRU; the backward pass
through time of the vanilla cell; Section 3.1's input projection b' = W x + b).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sprnn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

ACT = {"relu": 0, "tanh": 1, "identity": 2}

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add contraction) and return the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-fopenmp", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        ci = ctypes.c_int
        lib.oracle_half_bits_to_float.restype = ctypes.c_float
        lib.oracle_half_bits_to_float.argtypes = [ctypes.c_uint16]
        lib.oracle_rnn_forward.restype = ci
        lib.oracle_rnn_forward.argtypes = [ci, ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, ci]
        lib.oracle_rnn_forward_f64.restype = ci
        lib.oracle_rnn_forward_f64.argtypes = [ci, ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f64p, ci]
        lib.oracle_lstm_forward.restype = ci
        lib.oracle_lstm_forward.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f32p, f32p, ci]
        lib.oracle_lstm_forward_f64.restype = ci
        lib.oracle_lstm_forward_f64.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f64p, f64p, ci]
        lib.oracle_lstm_forward_saved.restype = ci
        lib.oracle_lstm_forward_saved.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f32p, f32p, f32p, ci]
        lib.oracle_lstm_backward_f64.restype = ci
        lib.oracle_lstm_backward_f64.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f32p, f32p, f32p,
                                                 f64p, f64p, f64p, f64p]
        lib.oracle_gru_forward.restype = ci
        lib.oracle_gru_forward.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f32p, ci]
        lib.oracle_gru_forward_saved.restype = ci
        lib.oracle_gru_forward_saved.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f32p, f32p, ci]
        lib.oracle_gru_backward_f64.restype = ci
        lib.oracle_gru_backward_f64.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f32p, f64p, f64p, f64p, f64p, f64p]
        lib.oracle_gru_forward_f64.restype = ci
        lib.oracle_gru_forward_f64.argtypes = [ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f64p, ci]
        lib.oracle_rnn_backward_f64.restype = ci
        lib.oracle_rnn_backward_f64.argtypes = [ci, ci, ci, ci, i32p, i32p, u16p, f32p, f32p, f32p, f64p, f64p, f64p]
        lib.oracle_input_projection_f64.restype = ci
        lib.oracle_input_projection_f64.argtypes = [ci, ci, ci, u16p, f32p, f32p, f64p, ci]
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _csr(row_ptr, col_idx, val_bits, rows, cols):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    val_bits = np.ascontiguousarray(val_bits, dtype=np.uint16)
    if row_ptr.shape != (rows + 1,) or row_ptr[0] != 0 or np.any(np.diff(row_ptr) < 0):
        raise ValueError("malformed row_ptr")
    nnz = int(row_ptr[-1])
    if col_idx.shape != (nnz,) or val_bits.shape != (nnz,):
        raise ValueError("col_idx / val_bits length differs from row_ptr[-1]")
    if nnz and (col_idx.min() < 0 or col_idx.max() >= cols):
        raise ValueError("column index out of range")
    # keep ctypes happy for empty arrays
    if nnz == 0:
        col_idx = np.zeros(1, dtype=np.int32)
        val_bits = np.zeros(1, dtype=np.uint16)
    return row_ptr, col_idx, val_bits


def half_bits_to_float(bits) -> np.ndarray:
    """Decode binary16 bit patterns with the oracle's own decoder (element by element)."""
    lib = _load()
    bits = np.asarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    flat_in, flat_out = bits.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = lib.oracle_half_bits_to_float(int(flat_in[i]))
    return out


def rnn_forward(hidden: int, batch: int, act: str, row_ptr, col_idx, val_bits, x, h0=None,
                f64: bool = False, threads: int = 1) -> np.ndarray:
    """All hidden states [T, B, H] of the vanilla cell (Eq. 2); float32, or float64 for the twin."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, hidden, hidden)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    if x.shape != (T, batch, hidden):
        raise ValueError("x must be [T, B, H]")
    if h0 is not None:
        h0 = np.ascontiguousarray(h0, dtype=np.float32)
        if h0.shape != (batch, hidden):
            raise ValueError("h0 must be [B, H]")
    out = np.empty((T, batch, hidden), dtype=np.float64 if f64 else np.float32)
    fn = lib.oracle_rnn_forward_f64 if f64 else lib.oracle_rnn_forward
    rc = fn(hidden, batch, T, ACT[act], _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
            _ptr(val_bits, ctypes.c_uint16), _ptr(x, ctypes.c_float), _ptr(h0, ctypes.c_float),
            _ptr(out, ctypes.c_double if f64 else ctypes.c_float), int(threads))
    if rc != 0:
        raise RuntimeError("oracle_rnn_forward failed")
    return out


def lstm_forward(hidden: int, batch: int, row_ptr, col_idx, val_bits, x, h0=None, c0=None,
                 f64: bool = False, threads: int = 1):
    """(h [T, B, H], c [T, B, H]) of the four-gate LSTM cell; gate row blocks i | f | g | o."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, 4 * hidden, hidden)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    if x.shape != (T, batch, 4 * hidden):
        raise ValueError("x must be [T, B, 4H]")
    if h0 is not None:
        h0 = np.ascontiguousarray(h0, dtype=np.float32)
    if c0 is not None:
        c0 = np.ascontiguousarray(c0, dtype=np.float32)
    dt = np.float64 if f64 else np.float32
    ct = ctypes.c_double if f64 else ctypes.c_float
    h = np.empty((T, batch, hidden), dtype=dt)
    c = np.empty((T, batch, hidden), dtype=dt)
    fn = lib.oracle_lstm_forward_f64 if f64 else lib.oracle_lstm_forward
    rc = fn(hidden, batch, T, _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
            _ptr(val_bits, ctypes.c_uint16), _ptr(x, ctypes.c_float), _ptr(h0, ctypes.c_float),
            _ptr(c0, ctypes.c_float), _ptr(h, ct), _ptr(c, ct), int(threads))
    if rc != 0:
        raise RuntimeError("oracle_lstm_forward failed")
    return h, c


def gru_forward(hidden: int, batch: int, row_ptr, col_idx, val_bits, x, b_hn=None, h0=None,
                f64: bool = False, threads: int = 1) -> np.ndarray:
    """h [T, B, H] of the GRU cell; gate row blocks r | z | n; b_hn [H] is the candidate's recurrent bias."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, 3 * hidden, hidden)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    if x.shape != (T, batch, 3 * hidden):
        raise ValueError("x must be [T, B, 3H]")
    if b_hn is not None:
        b_hn = np.ascontiguousarray(b_hn, dtype=np.float32)
        if b_hn.shape != (hidden,):
            raise ValueError("b_hn must be [H]")
    if h0 is not None:
        h0 = np.ascontiguousarray(h0, dtype=np.float32)
        if h0.shape != (batch, hidden):
            raise ValueError("h0 must be [B, H]")
    out = np.empty((T, batch, hidden), dtype=np.float64 if f64 else np.float32)
    fn = lib.oracle_gru_forward_f64 if f64 else lib.oracle_gru_forward
    rc = fn(hidden, batch, T, _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
            _ptr(val_bits, ctypes.c_uint16), _ptr(x, ctypes.c_float), _ptr(b_hn, ctypes.c_float),
            _ptr(h0, ctypes.c_float), _ptr(out, ctypes.c_double if f64 else ctypes.c_float), int(threads))
    if rc != 0:
        raise RuntimeError("oracle_gru_forward failed")
    return out


def gru_forward_saved(hidden: int, batch: int, row_ptr, col_idx, val_bits, x, b_hn=None, h0=None, threads: int = 1):
    """The binary32 GRU forward pass, also returning what a backward pass needs:
    (h [T, B, H], gates [T, B, 4H] with blocks r | z | n | q, q = U_n h_{t-1} + b_hn)."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, 3 * hidden, hidden)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    if x.shape != (T, batch, 3 * hidden):
        raise ValueError("x must be [T, B, 3H]")
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
    b_hn, h0 = f32(b_hn), f32(h0)
    h = np.empty((T, batch, hidden), dtype=np.float32)
    gates = np.empty((T, batch, 4 * hidden), dtype=np.float32)
    f = ctypes.c_float
    rc = lib.oracle_gru_forward_saved(hidden, batch, T, _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
                                      _ptr(val_bits, ctypes.c_uint16), _ptr(x, f), _ptr(b_hn, f), _ptr(h0, f),
                                      _ptr(h, f), _ptr(gates, f), int(threads))
    if rc != 0:
        raise RuntimeError("oracle_gru_forward_saved failed")
    return h, gates


def gru_backward(hidden: int, batch: int, row_ptr, col_idx, val_bits, gates, h_fwd, dh_ext, h0=None):
    """Backward pass through time of the GRU cell for L = sum_t <dh_ext[t], h_t>, binary64, from the quantities kept
    by the forward pass.  Returns (d_bprime [T, B, 3H] = dp_r | dp_z | da, d_rec [T, B, 3H] = dp_r | dp_z | dq,
    dh0 [B, H], dU [nnz] in CSR order of the [3H][H] matrix, db_hn [H])."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, 3 * hidden, hidden)
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
    gates, h_fwd, dh_ext, h0 = map(f32, (gates, h_fwd, dh_ext, h0))
    T = h_fwd.shape[0]
    if gates.shape != (T, batch, 4 * hidden):
        raise ValueError("gates must be [T, B, 4H]")
    if h_fwd.shape != (T, batch, hidden) or dh_ext.shape != (T, batch, hidden):
        raise ValueError("h_fwd and dh_ext must be [T, B, H]")
    if h0 is not None and h0.shape != (batch, hidden):
        raise ValueError("h0 must be [B, H]")
    nnz = int(row_ptr[-1])
    d_bprime = np.empty((T, batch, 3 * hidden), dtype=np.float64)
    d_rec = np.empty((T, batch, 3 * hidden), dtype=np.float64)
    dh0 = np.empty((batch, hidden), dtype=np.float64)
    dU = np.empty(max(nnz, 1), dtype=np.float64)
    db_hn = np.empty(hidden, dtype=np.float64)
    f, d = ctypes.c_float, ctypes.c_double
    rc = lib.oracle_gru_backward_f64(hidden, batch, T, _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
                                     _ptr(val_bits, ctypes.c_uint16), _ptr(gates, f), _ptr(h_fwd, f), _ptr(h0, f),
                                     _ptr(dh_ext, f), _ptr(d_bprime, d), _ptr(d_rec, d), _ptr(dh0, d), _ptr(dU, d), _ptr(db_hn, d))
    if rc != 0:
        raise RuntimeError("oracle_gru_backward_f64 failed")
    return d_bprime, d_rec, dh0, dU[:nnz], db_hn


def rnn_backward(hidden: int, batch: int, act: str, row_ptr, col_idx, val_bits, h_fwd, dh_ext, h0=None):
    """Backward pass through time of the vanilla cell for L = sum_t <dh_ext[t], h_t>, binary64.
    Returns (d_bprime [T, B, H], dh0 [B, H], dU [nnz] in CSR order)."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, hidden, hidden)
    h_fwd = np.ascontiguousarray(h_fwd, dtype=np.float32)
    dh_ext = np.ascontiguousarray(dh_ext, dtype=np.float32)
    T = h_fwd.shape[0]
    if h_fwd.shape != (T, batch, hidden) or dh_ext.shape != (T, batch, hidden):
        raise ValueError("h_fwd and dh_ext must be [T, B, H]")
    if h0 is not None:
        h0 = np.ascontiguousarray(h0, dtype=np.float32)
        if h0.shape != (batch, hidden):
            raise ValueError("h0 must be [B, H]")
    nnz = int(row_ptr[-1])
    d_bprime = np.empty((T, batch, hidden), dtype=np.float64)
    dh0 = np.empty((batch, hidden), dtype=np.float64)
    dU = np.empty(max(nnz, 1), dtype=np.float64)
    rc = lib.oracle_rnn_backward_f64(hidden, batch, T, ACT[act], _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
                                     _ptr(val_bits, ctypes.c_uint16), _ptr(h_fwd, ctypes.c_float), _ptr(h0, ctypes.c_float),
                                     _ptr(dh_ext, ctypes.c_float), _ptr(d_bprime, ctypes.c_double), _ptr(dh0, ctypes.c_double),
                                     _ptr(dU, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("oracle_rnn_backward_f64 failed")
    return d_bprime, dh0, dU[:nnz]


def lstm_forward_saved(hidden: int, batch: int, row_ptr, col_idx, val_bits, x, h0=None, c0=None, threads: int = 1):
    """The binary32 LSTM forward pass, also returning what a backward pass needs:
    (h [T, B, H], c [T, B, H], gates [T, B, 4H] after their activations, blocks i | f | g | o)."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, 4 * hidden, hidden)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    if x.shape != (T, batch, 4 * hidden):
        raise ValueError("x must be [T, B, 4H]")
    if h0 is not None:
        h0 = np.ascontiguousarray(h0, dtype=np.float32)
    if c0 is not None:
        c0 = np.ascontiguousarray(c0, dtype=np.float32)
    h = np.empty((T, batch, hidden), dtype=np.float32)
    c = np.empty((T, batch, hidden), dtype=np.float32)
    gates = np.empty((T, batch, 4 * hidden), dtype=np.float32)
    f = ctypes.c_float
    rc = lib.oracle_lstm_forward_saved(hidden, batch, T, _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
                                       _ptr(val_bits, ctypes.c_uint16), _ptr(x, f), _ptr(h0, f), _ptr(c0, f),
                                       _ptr(h, f), _ptr(c, f), _ptr(gates, f), int(threads))
    if rc != 0:
        raise RuntimeError("oracle_lstm_forward_saved failed")
    return h, c, gates


def lstm_backward(hidden: int, batch: int, row_ptr, col_idx, val_bits, gates, c_fwd, h_fwd, dh_ext, h0=None, c0=None):
    """Backward pass through time of the LSTM cell for L = sum_t <dh_ext[t], h_t>, binary64, from the gate values,
    cell states and outputs kept by the forward pass.
    Returns (d_bprime [T, B, 4H], dh0 [B, H], dc0 [B, H], dU [nnz] in CSR order of the [4H][H] matrix)."""
    lib = _load()
    row_ptr, col_idx, val_bits = _csr(row_ptr, col_idx, val_bits, 4 * hidden, hidden)
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
    gates, c_fwd, h_fwd, dh_ext, h0, c0 = map(f32, (gates, c_fwd, h_fwd, dh_ext, h0, c0))
    T = h_fwd.shape[0]
    if gates.shape != (T, batch, 4 * hidden):
        raise ValueError("gates must be [T, B, 4H]")
    for a in (c_fwd, h_fwd, dh_ext):
        if a.shape != (T, batch, hidden):
            raise ValueError("c_fwd, h_fwd and dh_ext must be [T, B, H]")
    for a in (h0, c0):
        if a is not None and a.shape != (batch, hidden):
            raise ValueError("h0 and c0 must be [B, H]")
    nnz = int(row_ptr[-1])
    d_bprime = np.empty((T, batch, 4 * hidden), dtype=np.float64)
    dh0 = np.empty((batch, hidden), dtype=np.float64)
    dc0 = np.empty((batch, hidden), dtype=np.float64)
    dU = np.empty(max(nnz, 1), dtype=np.float64)
    f, d = ctypes.c_float, ctypes.c_double
    rc = lib.oracle_lstm_backward_f64(hidden, batch, T, _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
                                      _ptr(val_bits, ctypes.c_uint16), _ptr(gates, f), _ptr(c_fwd, f), _ptr(c0, f),
                                      _ptr(h_fwd, f), _ptr(h0, f), _ptr(dh_ext, f), _ptr(d_bprime, d), _ptr(dh0, d),
                                      _ptr(dc0, d), _ptr(dU, d))
    if rc != 0:
        raise RuntimeError("oracle_lstm_backward_f64 failed")
    return d_bprime, dh0, dc0, dU[:nnz]


def input_projection(w_bits, x, bias=None, threads: int = 1) -> np.ndarray:
    """b' = W x + b of Section 3.1 for every input vector: w_bits [R, I] binary16 bits, x [..., I] float32,
    bias [R] float32 or None; returns float64 [..., R]."""
    lib = _load()
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    if w_bits.ndim != 2:
        raise ValueError("w_bits must be [R, I]")
    R, I = w_bits.shape
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.shape[-1] != I:
        raise ValueError("last axis of x must be I")
    lead = x.shape[:-1]
    M = int(np.prod(lead, dtype=np.int64))
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.shape != (R,):
            raise ValueError("bias must be [R]")
    out = np.empty((M, R), dtype=np.float64)
    rc = lib.oracle_input_projection_f64(R, I, M, _ptr(w_bits, ctypes.c_uint16), _ptr(x.reshape(M, I), ctypes.c_float),
                                         _ptr(bias, ctypes.c_float), _ptr(out, ctypes.c_double), int(threads))
    if rc != 0:
        raise RuntimeError("oracle_input_projection_f64 failed")
    return out.reshape(*lead, R)
