"""Parity of the input projection (sprnn_project, Section 3.1's b' = W x + b) against the CPU oracle, through the C ABI.

Tolerance, written out: products are exact in the matrix cores and the sums are binary32, so with K = input size
    |b'_gpu - b'_exact| <= (K + 8) * 2^-24 * (sum_k |W[r][k] x[k]| + |bias[r]|) + 2^-26 * sum_k |W[r][k]|
(the first term is the worst case of K binary32 additions plus the split of x into two binary16 halves, exact to 2^-21 = 8 * 2^-24; the second is the absolute
floor of the split for inputs below the smallest normal binary16 number).  Typical errors are ~sqrt(K) smaller.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1804_10223_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def bound(p, K):
    W = p.w_bits.view(np.float16).astype(np.float64)
    absw = np.abs(W)
    return (K + 8) * 2.0 ** -24 * (np.abs(p.x_in.astype(np.float64)) @ absw.T + np.abs(p.bias.astype(np.float64))) \
        + 2.0 ** -26 * absw.sum(axis=1)


def tiny_matrix(hidden, cell):
    """A handle only fixes (hidden, batch, cell) for the projection; its recurrent matrix is irrelevant here."""
    rows = hidden * (4 if cell == "lstm" else 1)
    row_ptr = np.arange(rows + 1, dtype=np.int32)
    col_idx = (np.arange(rows, dtype=np.int32) % hidden).astype(np.int32)
    vals = np.full(rows, 0.5, dtype=np.float16).view(np.uint16)
    return row_ptr, col_idx, vals


def run_project(hidden, batch, cell, p, use_bias=True, **options):
    row_ptr, col_idx, vals = tiny_matrix(hidden, cell)
    with binding.SparseRNN(hidden, batch, cell, row_ptr, col_idx, vals, poll_delay=-1, **options) as rnn:
        x = torch.from_numpy(p.x_in).cuda()
        w = torch.from_numpy(p.w_bits.view(np.int16)).cuda()
        b = torch.from_numpy(p.bias).cuda() if use_bias else None
        out = rnn.project(x, w, b)
        torch.cuda.synchronize()
        return out.cpu().numpy()


CASES = [
    # cell, hidden, batch, T, input size: ragged in every direction; K % 4 != 0 takes the element-wise loads
    ("relu", 100, 2, 37, 77),
    ("relu", 100, 2, 37, 72),      # K % 8 == 0: all vector loads
    ("relu", 100, 2, 37, 68),      # K % 4 == 0 only: x by vectors, W element-wise
    ("relu", 1, 1, 1, 1),
    ("relu", 300, 4, 50, 200),     # several tiles in m and n, ragged tails
    ("relu", 129, 1, 65, 64),      # one row / one column past a tile edge
    ("lstm", 64, 8, 9, 130),       # R = 4H
    ("tanh", 1152, 4, 16, 1152),   # 8 x 9 tiles: the XCD-aware tile order is in use
]


@pytest.mark.parametrize("cell,hidden,batch,T,I", CASES)
def test_projection_matches_oracle(cell, hidden, batch, T, I):
    rows = hidden * (4 if cell == "lstm" else 1)
    p = wl.make_projection(rows, I, T, batch, seed=hidden + I)
    print("case", cell, hidden, batch, T, I, flush=True)
    got = run_project(hidden, batch, cell, p)
    want = oracle.input_projection(p.w_bits, p.x_in, p.bias, threads=8)
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= bound(p, I)), float((err / bound(p, I)).max())
    # far tighter than the worst case in practice; a transposed or shifted operand is nowhere near
    assert err.max() <= 2e-5 * max(1.0, np.abs(want).max())


def test_projection_without_bias_and_input_scales():
    for scale in (1.0, 1e3, 1e-2, 1e-5):
        p = wl.make_projection(200, 96, 10, 4, seed=3, x_scale=scale)
        print("scale", scale, flush=True)
        got = run_project(200, 4, "relu", p, use_bias=False)
        p.bias[:] = 0
        want = oracle.input_projection(p.w_bits, p.x_in, None, threads=8)
        err = np.abs(got.astype(np.float64) - want)
        assert np.all(err <= bound(p, 96)), (scale, float((err / bound(p, 96)).max()))


def test_projection_closed_forms_bit_exact():
    # identity W and inputs with few significant bits: b' = x + b with one binary32 rounding, exactly
    rng = np.random.default_rng(2)
    H, B, T = 160, 2, 21
    x = rng.integers(-2000, 2000, size=(T, B, H)).astype(np.float32) / np.float32(8.0)
    bias = rng.integers(-64, 64, size=H).astype(np.float32) / np.float32(4.0)
    p = wl.Projection(rows=H, input_size=H, w_bits=np.eye(H, dtype=np.float16).view(np.uint16).copy(), bias=bias, x_in=x)
    got = run_project(H, B, "relu", p)
    assert np.array_equal(got, x + bias)
    assert np.array_equal(got.astype(np.float64), oracle.input_projection(p.w_bits, x, bias))
    # a single entry W[r, k] = 0.5
    W = np.zeros((H, H), dtype=np.float16)
    W[7, 150] = 0.5
    p = wl.Projection(rows=H, input_size=H, w_bits=W.view(np.uint16).copy(), bias=np.zeros(H, np.float32), x_in=x)
    got = run_project(H, B, "relu", p)
    want = np.zeros((T, B, H), np.float32)
    want[..., 7] = 0.5 * x[..., 150]
    assert np.array_equal(got, want)


def test_projection_at_the_headline_shape():
    """hidden 2304, batch 4, T 256 with input size 2304: every output against the oracle."""
    p = wl.make_projection(2304, 2304, 256, 4, seed=0)
    got = run_project(2304, 4, "relu", p)
    print("gpu done", flush=True)
    want = oracle.input_projection(p.w_bits, p.x_in, p.bias, threads=16)
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= bound(p, 2304)), float((err / bound(p, 2304)).max())
    assert err.max() <= 2e-5 * np.abs(want).max()


@pytest.mark.parametrize("name", ["cfg2", "cfg5"])
def test_whole_layer_from_raw_inputs(name):
    """sprnn_project feeding the persistent kernel on one stream against the oracle's projection + recurrence."""
    w = wl.make_config(name, steps=24)
    lstm = w.cell == "lstm"
    p = wl.make_projection(w.rows, w.hidden, w.steps, w.batch, seed=5,
                           forget_block=(w.hidden, 2 * w.hidden) if lstm else None)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x_in = torch.from_numpy(p.x_in).cuda()
        w_in = torch.from_numpy(p.w_bits.view(np.int16)).cuda()
        bias = torch.from_numpy(p.bias).cuda()
        bp = rnn.project(x_in, w_in, bias)
        if lstm:
            h, _ = rnn.forward_lstm(bp)
        else:
            h = rnn.forward(bp)
        torch.cuda.synchronize()
        assert rnn.check() == 0
        h = h.cpu().numpy()
    bp_ref = oracle.input_projection(p.w_bits, p.x_in, p.bias, threads=8).astype(np.float32)
    if lstm:
        ref, _ = oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, bp_ref, f64=True, threads=8)
    else:
        ref = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, bp_ref, f64=True, threads=8)
    for t in range(w.steps):
        assert np.abs(h[t] - ref[t]).max() <= 1e-3 * np.abs(ref[t]).max(), t


def test_projection_keeps_subnormal_weights_and_tiny_inputs():
    """Binary16 subnormal weights (multiples of 2^-24) and inputs below the binary16 normal range contribute exactly."""
    rng = np.random.default_rng(4)
    H, B, T = 96, 2, 5
    w_bits = rng.integers(1, 1024, size=(H, H)).astype(np.uint16)        # exponent field 0: all subnormal, positive
    w_bits[::2] |= 0x8000                                                # every other row negative
    x = rng.integers(-8, 9, size=(T, B, H)).astype(np.float32)
    p = wl.Projection(rows=H, input_size=H, w_bits=w_bits, bias=np.zeros(H, np.float32), x_in=x)
    got = run_project(H, B, "relu", p)
    want = oracle.input_projection(w_bits, x, None)                      # integers times 2^-24: exact in binary32 too
    assert np.array_equal(got.astype(np.float64), want)
    # inputs of magnitude 2^-20 .. 2^-17 with 6 significant bits against weights that are small integers
    x_tiny = (rng.integers(-63, 64, size=(T, B, H)).astype(np.float32) * np.float32(2.0 ** -23))
    w_int = rng.integers(-4, 5, size=(H, H)).astype(np.float16)
    p = wl.Projection(rows=H, input_size=H, w_bits=w_int.view(np.uint16).copy(), bias=np.zeros(H, np.float32), x_in=x_tiny)
    got = run_project(H, B, "relu", p)
    assert np.array_equal(got.astype(np.float64), oracle.input_projection(p.w_bits, x_tiny, None))


def test_two_stacked_layers_from_raw_inputs():
    """Layer 2 takes layer 1's h_t as its input: project -> recurrence -> project -> recurrence, all enqueued on one
    stream without a host synchronisation in between, against the same chain of oracle calls."""
    H, B, T, I = 384, 4, 20, 200
    w1 = wl.make_workload("l1", "tanh", H, B, T, 0.2, seed=11)
    w2 = wl.make_workload("l2", "relu", H, B, T, 0.1, seed=12, row_nnz="poisson")
    p1 = wl.make_projection(H, I, T, B, seed=13)
    p2 = wl.make_projection(H, H, T, B, seed=14)
    with binding.SparseRNN(H, B, "tanh", w1.row_ptr, w1.col_idx, w1.val_bits) as l1, \
            binding.SparseRNN(H, B, "relu", w2.row_ptr, w2.col_idx, w2.val_bits) as l2:
        dev = lambda a, view=None: torch.from_numpy(a if view is None else a.view(view)).cuda()
        h1 = l1.forward(l1.project(dev(p1.x_in), dev(p1.w_bits, np.int16), dev(p1.bias)))
        h2 = l2.forward(l2.project(h1, dev(p2.w_bits, np.int16), dev(p2.bias)))
        torch.cuda.synchronize()
        assert l1.check() == 0 and l2.check() == 0
        h1, h2 = h1.cpu().numpy(), h2.cpu().numpy()
    b1 = oracle.input_projection(p1.w_bits, p1.x_in, p1.bias, threads=8).astype(np.float32)
    r1 = oracle.rnn_forward(H, B, "tanh", w1.row_ptr, w1.col_idx, w1.val_bits, b1, f64=True, threads=8)
    b2 = oracle.input_projection(p2.w_bits, r1.astype(np.float32), p2.bias, threads=8).astype(np.float32)
    r2 = oracle.rnn_forward(H, B, "relu", w2.row_ptr, w2.col_idx, w2.val_bits, b2, f64=True, threads=8)
    for t in range(T):
        assert np.abs(h1[t] - r1[t]).max() <= 1e-3 * np.abs(r1[t]).max(), t
        assert np.abs(h2[t] - r2[t]).max() <= 1e-3 * np.abs(r2[t]).max(), t
