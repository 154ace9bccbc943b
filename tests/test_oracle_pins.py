"""Pins for the CPU oracle: everything here checks ``oracle/`` against something that is NOT the oracle.

The paper prints no worked numeric example for the recurrent step (Eq. 2), so the oracle is pinned by
  * a hand-evaluated integer example of Eq. 2 (tests/golden/eq2_hand_example.json),
  * the dense special case against numpy float64 matmul and torch.nn.RNNCell / LSTMCell,
  * closed forms: identity matrix (running sum), permutation matrices (bit exact), zero weights,
  * exact rational brute force on tiny sizes,
  * invariants: positive homogeneity, batch independence, time composition, fp64 twin bound,
  * exhaustive binary16 decode against numpy.
The input projection b' = W x + b (Section 3.1) is pinned by a hand-evaluated non-square example with a
bias (tests/golden/eq1_hand_example.json), numpy's float64 matrix product, identity / single-entry closed
forms (bit exact), exact rational brute force, and checks that a transposed operand or a dropped bias fails.
The GRU cell (three gates; the paper gives no equations) is pinned against torch.nn.GRUCell, which fixes the gate
order r, z, n and the place of the candidate's recurrent bias, and by closed forms and invariants.
The backward passes (vanilla cell, LSTM, GRU) are pinned against torch autograd of the same dense cell in float64
(torch.nn.LSTMCell and torch.nn.GRUCell for the gated cells), single-step closed forms, zero weights, and finite differences of the forward oracle.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_1804_10223_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def f16bits(a):
    return np.asarray(a, dtype=np.float16).view(np.uint16)


def dense_csr(w16):
    """CSR that stores EVERY entry of the float16 matrix (also zeros), density 1.0."""
    rows, cols = w16.shape
    row_ptr = (np.arange(rows + 1) * cols).astype(np.int32)
    col_idx = np.tile(np.arange(cols, dtype=np.int32), rows)
    return row_ptr, col_idx, w16.reshape(-1).view(np.uint16).copy()


# ----------------------------------------------------------------------------- binary16 decode
def test_half_decode_exhaustive_matches_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.half_bits_to_float(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))  # bit exact, incl. -0 and subnormals


# ----------------------------------------------------------------------------- hand example (golden)
def test_golden_hand_example_eq2():
    with open(os.path.join(HERE, "golden", "eq2_hand_example.json")) as f:
        g = json.load(f)
    w16 = np.array(g["U_r"], dtype=np.float16)
    row_ptr, col_idx, vals = wl.csr_from_dense(w16)
    x = np.array(g["b_prime"], dtype=np.float32)
    h0 = np.array(g["h0"], dtype=np.float32)
    h = oracle.rnn_forward(g["hidden"], g["batch"], "relu", row_ptr, col_idx, vals, x, h0)
    assert np.array_equal(h, np.array(g["h"], dtype=np.float32))


# ----------------------------------------------------------------------------- dense special case
@pytest.mark.parametrize("act", ["relu", "tanh", "identity"])
def test_dense_matches_float64_matmul(act):
    rng = np.random.default_rng(11)
    H, B, T = 37, 3, 5
    w16 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float16)
    row_ptr, col_idx, vals = dense_csr(w16)
    x = rng.standard_normal((T, B, H)).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    got = oracle.rnn_forward(H, B, act, row_ptr, col_idx, vals, x, h0)
    W = w16.astype(np.float64)
    h = h0.astype(np.float64)
    f = {"relu": lambda z: np.maximum(z, 0.0), "tanh": np.tanh, "identity": lambda z: z}[act]
    for t in range(T):
        h = f(h @ W.T + x[t].astype(np.float64))   # row i of W dotted with h: NOT the transpose
        np.testing.assert_allclose(got[t], h, rtol=0, atol=2e-5 * max(1.0, np.abs(h).max()))
    # a transposed operand must be far outside that tolerance (the pin is sensitive to it)
    hT = f(h0.astype(np.float64) @ W + x[0].astype(np.float64))
    assert np.abs(hT - got[0]).max() > 1e-2


def test_dense_matches_torch_rnncell():
    rng = np.random.default_rng(5)
    H, B, T = 24, 2, 4
    w16 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float16)
    row_ptr, col_idx, vals = dense_csr(w16)
    x = rng.standard_normal((T, B, H)).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    got = oracle.rnn_forward(H, B, "relu", row_ptr, col_idx, vals, x, h0)
    cell = torch.nn.RNNCell(H, H, bias=False, nonlinearity="relu").double()
    with torch.no_grad():
        cell.weight_hh.copy_(torch.from_numpy(w16.astype(np.float64)))
        cell.weight_ih.copy_(torch.eye(H, dtype=torch.float64))
        h = torch.from_numpy(h0.astype(np.float64))
        for t in range(T):
            h = cell(torch.from_numpy(x[t].astype(np.float64)), h)
            np.testing.assert_allclose(got[t], h.numpy(), rtol=0, atol=2e-5)


def test_dense_lstm_matches_torch_lstmcell_gate_order_and_equations():
    rng = np.random.default_rng(6)
    H, B, T = 19, 3, 4
    w16 = (rng.standard_normal((4 * H, H)) / np.sqrt(H)).astype(np.float16)
    row_ptr, col_idx, vals = dense_csr(w16)
    x = rng.standard_normal((T, B, 4 * H)).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    gh, gc = oracle.lstm_forward(H, B, row_ptr, col_idx, vals, x, h0, c0)
    cell = torch.nn.LSTMCell(4 * H, H, bias=False).double()   # gate order i, f, g, o
    with torch.no_grad():
        cell.weight_hh.copy_(torch.from_numpy(w16.astype(np.float64)))
        cell.weight_ih.copy_(torch.eye(4 * H, dtype=torch.float64))
        h = torch.from_numpy(h0.astype(np.float64))
        c = torch.from_numpy(c0.astype(np.float64))
        for t in range(T):
            h, c = cell(torch.from_numpy(x[t].astype(np.float64)), (h, c))
            np.testing.assert_allclose(gh[t], h.numpy(), rtol=0, atol=2e-5)
            np.testing.assert_allclose(gc[t], c.numpy(), rtol=0, atol=2e-5)
    # swapping two gate blocks must be visible at this tolerance
    xs = x.copy()
    xs[:, :, 0:H], xs[:, :, H:2 * H] = x[:, :, H:2 * H], x[:, :, 0:H]
    sh, _ = oracle.lstm_forward(H, B, row_ptr, col_idx, vals, xs, h0, c0)
    assert np.abs(sh - gh).max() > 1e-2


# ----------------------------------------------------------------------------- closed forms
def test_identity_matrix_is_running_sum():
    rng = np.random.default_rng(2)
    H, B, T = 50, 2, 7
    row_ptr = np.arange(H + 1, dtype=np.int32)
    col_idx = np.arange(H, dtype=np.int32)
    vals = f16bits(np.ones(H))
    x = rng.integers(0, 5, size=(T, B, H)).astype(np.float32)        # x >= 0: ReLU never clips
    h0 = rng.integers(0, 5, size=(B, H)).astype(np.float32)
    got = oracle.rnn_forward(H, B, "relu", row_ptr, col_idx, vals, x, h0)
    want = h0[None] + np.cumsum(x, axis=0)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("H", [7, 4099, 65535])
def test_permutation_matrix_moves_values_bit_exactly(H):
    rng = np.random.default_rng(H)
    perm = rng.permutation(H).astype(np.int32)          # row i reads column perm[i]
    row_ptr = np.arange(H + 1, dtype=np.int32)
    vals = f16bits(np.ones(H))
    B, T = 2, 3
    x = np.zeros((T, B, H), dtype=np.float32)
    h0 = np.abs(rng.standard_normal((B, H))).astype(np.float32)
    got = oracle.rnn_forward(H, B, "relu", row_ptr, perm, vals, x, h0)
    cur = h0
    for t in range(T):
        cur = cur[:, perm]
        assert np.array_equal(got[t].view(np.uint32), cur.view(np.uint32))


def test_permutation_cycle_returns_to_start():
    H = 12
    perm = np.roll(np.arange(H, dtype=np.int32), 1)      # one 12-cycle
    row_ptr = np.arange(H + 1, dtype=np.int32)
    x = np.zeros((H, 1, H), dtype=np.float32)
    h0 = np.arange(1, H + 1, dtype=np.float32)[None]
    got = oracle.rnn_forward(H, 1, "relu", row_ptr, perm, f16bits(np.ones(H)), x, h0)
    assert np.array_equal(got[-1], h0)
    assert not np.array_equal(got[0], h0)


@pytest.mark.parametrize("act", ["relu", "tanh", "identity"])
def test_zero_weights_give_act_of_x(act):
    rng = np.random.default_rng(3)
    H, B, T = 33, 2, 3
    x = rng.standard_normal((T, B, H)).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    f = {"relu": lambda z: np.maximum(z, np.float32(0)), "tanh": np.tanh, "identity": lambda z: z}[act]
    # (a) no stored entries at all, (b) stored zeros
    empty = (np.zeros(H + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16))
    stored = dense_csr(np.zeros((H, H), dtype=np.float16))
    for row_ptr, col_idx, vals in (empty, stored):
        got = oracle.rnn_forward(H, B, act, row_ptr, col_idx, vals, x, h0)
        if act == "tanh":
            np.testing.assert_allclose(got, f(x.astype(np.float64)), rtol=0, atol=1e-6)
        else:
            assert np.array_equal(got, f(x))


def test_zero_weight_lstm_closed_form():
    rng = np.random.default_rng(4)
    H, B, T = 9, 2, 3
    x = rng.standard_normal((T, B, 4 * H))
    c0 = rng.standard_normal((B, H))
    row_ptr = np.zeros(4 * H + 1, dtype=np.int32)
    gh, gc = oracle.lstm_forward(H, B, row_ptr, np.zeros(0, np.int32), np.zeros(0, np.uint16),
                                 x.astype(np.float32), None, c0.astype(np.float32))
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    c = c0.astype(np.float32).astype(np.float64)
    x = x.astype(np.float32).astype(np.float64)
    for t in range(T):
        i, f, g, o = (x[t][:, k * H:(k + 1) * H] for k in range(4))
        c = sig(f) * c + sig(i) * np.tanh(g)
        h = sig(o) * np.tanh(c)
        np.testing.assert_allclose(gc[t], c, rtol=0, atol=1e-6)
        np.testing.assert_allclose(gh[t], h, rtol=0, atol=1e-6)


# ----------------------------------------------------------------------------- exact brute force
def _brute_force_rnn(W, x, h0, relu):
    """Eq. 2 in exact rational arithmetic from the dense matrix (pure Python)."""
    H = len(W)
    T, B = len(x), len(x[0])
    h = [[Fraction(v) for v in row] for row in h0]
    out = []
    for t in range(T):
        new = []
        for b in range(B):
            row = []
            for i in range(H):
                s = sum(Fraction(W[i][j]) * h[b][j] for j in range(H)) + Fraction(x[t][b][i])
                row.append(max(s, Fraction(0)) if relu else s)
            new.append(row)
        h = new
        out.append(h)
    return out


@pytest.mark.parametrize("seed", range(6))
def test_exact_rational_brute_force_tiny(seed):
    rng = np.random.default_rng(100 + seed)
    H = int(rng.integers(1, 9)); B = int(rng.integers(1, 3)); T = int(rng.integers(1, 4))
    relu = bool(seed % 2 == 0)
    # dyadic values with few bits: every product and sum is exact in binary32, so equality is bit exact
    W = (rng.integers(-8, 9, size=(H, H)) / 8.0) * (rng.random((H, H)) < 0.6)
    x = rng.integers(-16, 17, size=(T, B, H)) / 4.0
    h0 = rng.integers(-8, 9, size=(B, H)) / 2.0
    w16 = W.astype(np.float16)
    assert np.array_equal(w16.astype(np.float64), W)
    row_ptr, col_idx, vals = wl.csr_from_dense(w16)
    got = oracle.rnn_forward(H, B, "relu" if relu else "identity", row_ptr, col_idx, vals,
                             x.astype(np.float32), h0.astype(np.float32))
    want = _brute_force_rnn(W.tolist(), x.tolist(), h0.tolist(), relu)
    for t in range(T):
        for b in range(B):
            for i in range(H):
                assert Fraction(float(got[t, b, i])) == want[t][b][i], (t, b, i)


# ----------------------------------------------------------------------------- invariants
def _small_sparse(seed=0, cell="relu", H=96, B=3, T=6, density=0.2):
    return wl.make_workload("t", cell, H, B, T, density, seed=seed, h0_std=0.5)


def test_relu_positive_homogeneity_is_bit_exact():
    w = _small_sparse(1)
    a = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0)
    for k in (-3, 5):
        s = np.float32(2.0 ** k)
        b = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x * s, w.h0 * s)
        assert np.array_equal(b, a * s)


def test_batch_columns_are_independent():
    w = _small_sparse(2)
    full = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0)
    for b in range(w.batch):
        one = oracle.rnn_forward(w.hidden, 1, "relu", w.row_ptr, w.col_idx, w.val_bits,
                                 w.x[:, b:b + 1].copy(), w.h0[b:b + 1].copy())
        assert np.array_equal(one[:, 0], full[:, b])


def test_time_composition():
    w = _small_sparse(3, T=9)
    full = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0)
    first = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x[:4].copy(), w.h0)
    second = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x[4:].copy(), first[-1].copy())
    assert np.array_equal(np.concatenate([first, second]), full)


def test_lstm_time_composition_and_batch_independence():
    w = _small_sparse(4, cell="lstm", H=40, B=2, T=6)
    h, c = oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, None)
    h1, c1 = oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x[:2].copy(), w.h0, None)
    h2, c2 = oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x[2:].copy(), h1[-1].copy(), c1[-1].copy())
    assert np.array_equal(np.concatenate([h1, h2]), h) and np.array_equal(np.concatenate([c1, c2]), c)
    hb, cb = oracle.lstm_forward(w.hidden, 1, w.row_ptr, w.col_idx, w.val_bits, w.x[:, 1:2].copy(), w.h0[1:2].copy(), None)
    assert np.array_equal(hb[:, 0], h[:, 1]) and np.array_equal(cb[:, 0], c[:, 1])


@pytest.mark.parametrize("cell", ["relu", "tanh", "lstm"])
def test_fp64_twin_bounds_fp32_rounding(cell):
    w = wl.make_workload("t", cell, 256, 2, 12, 0.3, seed=7, h0_std=0.3, gain=0.9 if cell != "lstm" else 1.0)
    if cell == "lstm":
        a, ac = oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, None)
        d, dc = oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, None, f64=True)
        pairs = [(a, d), (ac, dc)]
    else:
        a = oracle.rnn_forward(w.hidden, w.batch, cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0)
        d = oracle.rnn_forward(w.hidden, w.batch, cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, f64=True)
        pairs = [(a, d)]
    for got, ref in pairs:
        for t in range(w.steps):
            assert np.abs(got[t] - ref[t]).max() <= 2e-5 * np.abs(ref[t]).max()   # 50x inside the 1e-3 parity bound


def test_fp64_twin_on_dense_float64_reference():
    # the twin itself is pinned against numpy float64 to ~1e-13
    rng = np.random.default_rng(8)
    H, B, T = 31, 2, 4
    w16 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float16)
    row_ptr, col_idx, vals = dense_csr(w16)
    x = rng.standard_normal((T, B, H)).astype(np.float32)
    got = oracle.rnn_forward(H, B, "tanh", row_ptr, col_idx, vals, x, None, f64=True)
    h = np.zeros((B, H))
    for t in range(T):
        h = np.tanh(h @ w16.astype(np.float64).T + x[t].astype(np.float64))
        np.testing.assert_allclose(got[t], h, rtol=0, atol=1e-12)


def test_openmp_rows_do_not_change_results():
    w = _small_sparse(9, H=200, T=5)
    a = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=1)
    b = oracle.rnn_forward(w.hidden, w.batch, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=4)
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------- generator sanity
def test_generator_shapes_and_determinism():
    a = wl.make_config("cfg1")
    b = wl.make_config("cfg1")
    assert a.hidden == 256 and a.batch == 1 and a.steps == 16 and a.h0 is None
    assert np.all(np.diff(a.row_ptr) == 26)
    assert np.array_equal(a.col_idx, b.col_idx) and np.array_equal(a.val_bits, b.val_bits) and np.array_equal(a.x, b.x)
    for r in range(a.rows):
        cols = a.col_idx[a.row_ptr[r]:a.row_ptr[r + 1]]
        assert np.all(np.diff(cols) > 0) and cols.min() >= 0 and cols.max() < a.hidden
    l = wl.make_workload("l", "lstm", 16, 2, 3, 0.25, seed=1)
    assert l.x.shape == (3, 2, 64) and l.row_ptr.shape == (65,)
    assert abs(float(l.x[:, :, 16:32].mean()) - 1.0) < 0.5      # forget-gate bias folded into b'


# ----------------------------------------------------------------------------- input projection (Section 3.1)
def test_golden_hand_example_input_projection():
    with open(os.path.join(HERE, "golden", "eq1_hand_example.json")) as f:
        g = json.load(f)
    W = f16bits(np.array(g["W"], dtype=np.float16))
    x = np.array(g["x"], dtype=np.float32)
    b = np.array(g["b"], dtype=np.float32)
    got = oracle.input_projection(W, x, b)
    assert got.shape == (2, 2, g["rows"])
    assert np.array_equal(got, np.array(g["b_prime"], dtype=np.float64))
    # without the bias the hand values are missed by exactly b
    assert np.array_equal(oracle.input_projection(W, x, None), np.array(g["b_prime"], dtype=np.float64) - b.astype(np.float64))


def test_input_projection_matches_float64_matmul_and_is_not_its_transpose():
    rng = np.random.default_rng(5)
    R, I, T, B = 29, 41, 4, 3
    w16 = (rng.standard_normal((R, I)) / np.sqrt(I)).astype(np.float16)
    x = rng.standard_normal((T, B, I)).astype(np.float32)
    b = rng.standard_normal(R).astype(np.float32)
    got = oracle.input_projection(f16bits(w16), x, b)
    want = x.astype(np.float64) @ w16.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    assert np.array_equal(got, oracle.input_projection(f16bits(w16), x, b, threads=3))
    # square case: the transposed operand is far away
    ws = (rng.standard_normal((I, I)) / np.sqrt(I)).astype(np.float16)
    g2 = oracle.input_projection(f16bits(ws), x, None)
    assert np.abs(g2 - x.astype(np.float64) @ ws.astype(np.float64)).max() > 1e-2
    np.testing.assert_allclose(g2, x.astype(np.float64) @ ws.astype(np.float64).T, rtol=0, atol=1e-13)


def test_input_projection_closed_forms_bit_exact():
    rng = np.random.default_rng(6)
    I = 17
    x = rng.standard_normal((5, 2, I)).astype(np.float32)
    b = rng.standard_normal(I).astype(np.float32)
    eye = np.eye(I, dtype=np.float16)
    assert np.array_equal(oracle.input_projection(f16bits(eye), x, b), x.astype(np.float64) + b.astype(np.float64))
    # one entry W[r, k] = 0.5 picks half of input k into output r and nothing else
    W = np.zeros((3, I), dtype=np.float16)
    W[2, 11] = 0.5
    got = oracle.input_projection(f16bits(W), x, None)
    want = np.zeros((5, 2, 3))
    want[..., 2] = 0.5 * x[..., 11].astype(np.float64)
    assert np.array_equal(got, want)
    # zero weights leave the bias
    assert np.array_equal(oracle.input_projection(f16bits(np.zeros((3, I), dtype=np.float16)), x, b[:3]),
                          np.broadcast_to(b[:3].astype(np.float64), (5, 2, 3)))


def test_input_projection_exact_rational_brute_force():
    rng = np.random.default_rng(7)
    R, I, M = 4, 6, 3
    w16 = rng.standard_normal((R, I)).astype(np.float16)
    x = rng.standard_normal((M, I)).astype(np.float32)
    b = rng.standard_normal(R).astype(np.float32)
    got = oracle.input_projection(f16bits(w16), x, b)
    for m in range(M):
        for r in range(R):
            exact = sum((Fraction(float(w16[r, k])) * Fraction(float(x[m, k])) for k in range(I)), Fraction(0)) + Fraction(float(b[r]))
            scale = sum(abs(float(w16[r, k]) * float(x[m, k])) for k in range(I)) + abs(float(b[r]))
            assert abs(Fraction(float(got[m, r])) - exact) <= Fraction(scale) * Fraction(I + 1, 2 ** 52)


# ----------------------------------------------------------------------------- GRU cell
def test_dense_gru_matches_torch_grucell_gate_order_and_bias_placement():
    rng = np.random.default_rng(21)
    H, B, T = 19, 3, 6
    w16 = (rng.standard_normal((3 * H, H)) / np.sqrt(H)).astype(np.float16)
    row_ptr, col_idx, vals = dense_csr(w16)
    x = rng.standard_normal((T, B, 3 * H)).astype(np.float32)
    b_hh = rng.standard_normal(3 * H).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    # b_hr and b_hz are additive and travel inside x; b_hn must stay inside the reset product
    xb = x.copy()
    xb[:, :, :2 * H] += b_hh[:2 * H]
    got = oracle.gru_forward(H, B, row_ptr, col_idx, vals, xb, b_hh[2 * H:], h0)
    cell = torch.nn.GRUCell(3 * H, H, bias=True).double()   # gate order r, z, n
    with torch.no_grad():
        cell.weight_hh.copy_(torch.from_numpy(w16.astype(np.float64)))
        cell.weight_ih.copy_(torch.eye(3 * H, dtype=torch.float64))
        cell.bias_ih.zero_()
        cell.bias_hh.copy_(torch.from_numpy(b_hh.astype(np.float64)))
        h = torch.from_numpy(h0.astype(np.float64))
        for t in range(T):
            h = cell(torch.from_numpy(x[t].astype(np.float64)), h)
            np.testing.assert_allclose(got[t], h.numpy(), rtol=0, atol=2e-5)
    g64 = oracle.gru_forward(H, B, row_ptr, col_idx, vals, xb, b_hh[2 * H:], h0, f64=True)
    np.testing.assert_allclose(g64[-1], h.numpy(), rtol=0, atol=1e-6)   # x + b_hr, x + b_hz were rounded to binary32
    # the candidate's recurrent bias outside the reset product, or two gate blocks swapped, must be visible
    xo = xb.copy()
    xo[:, :, 2 * H:] += b_hh[2 * H:]
    assert np.abs(oracle.gru_forward(H, B, row_ptr, col_idx, vals, xo, None, h0) - got).max() > 1e-2
    xs = xb.copy()
    xs[:, :, 0:H], xs[:, :, H:2 * H] = xb[:, :, H:2 * H], xb[:, :, 0:H]
    assert np.abs(oracle.gru_forward(H, B, row_ptr, col_idx, vals, xs, b_hh[2 * H:], h0) - got).max() > 1e-2


def test_gru_closed_forms():
    rng = np.random.default_rng(22)
    H, B, T = 11, 2, 4
    zero = np.zeros(3 * H + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    b_hn = rng.standard_normal(H).astype(np.float32)
    x = rng.standard_normal((T, B, 3 * H)).astype(np.float32)
    # update gate saturated at 1 (sigmoid(40) == 1 in binary32): the state never changes
    xk = x.copy()
    xk[:, :, H:2 * H] = 40.0
    got = oracle.gru_forward(H, B, *zero, xk, b_hn, h0)
    assert np.array_equal(got, np.broadcast_to(h0, (T, B, H)))
    # update gate saturated at 0, reset gate at 1, zero weights: h_t = tanh(x_n + b_hn) whatever came before
    xf = x.copy()
    xf[:, :, H:2 * H] = -120.0
    xf[:, :, 0:H] = 40.0
    got = oracle.gru_forward(H, B, *zero, xf, b_hn, h0, f64=True)
    np.testing.assert_allclose(got, np.tanh(xf[:, :, 2 * H:].astype(np.float64) + b_hn.astype(np.float64)), rtol=0, atol=1e-15)
    # reset gate at 0: the candidate ignores the recurrent term (a one-entry weight in the n block has no effect)
    xr = x.copy()
    xr[:, :, 0:H] = -120.0
    rp = np.zeros(3 * H + 1, dtype=np.int32)
    rp[2 * H + 1:] = 1                       # row 2H (candidate of unit 0) reads column 3
    a = oracle.gru_forward(H, B, rp, np.array([3], np.int32), f16bits([1.5]), xr, None, h0, f64=True)
    b = oracle.gru_forward(H, B, *zero, xr, None, h0, f64=True)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-30)


def test_gru_time_composition_batch_independence_and_twin():
    rng = np.random.default_rng(23)
    H, B, T = 40, 2, 9
    parts = [wl.make_workload("g", "relu", H, B, 1, 0.3, seed=s) for s in (1, 2, 3)]
    row_ptr = np.concatenate([[0], np.cumsum(np.concatenate([np.diff(p.row_ptr) for p in parts]))]).astype(np.int32)
    col_idx = np.concatenate([p.col_idx for p in parts])
    vals = np.concatenate([p.val_bits for p in parts])
    x = rng.standard_normal((T, B, 3 * H)).astype(np.float32)
    b_hn = rng.standard_normal(H).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    full = oracle.gru_forward(H, B, row_ptr, col_idx, vals, x, b_hn, h0)
    first = oracle.gru_forward(H, B, row_ptr, col_idx, vals, x[:4], b_hn, h0)
    rest = oracle.gru_forward(H, B, row_ptr, col_idx, vals, x[4:], b_hn, first[-1])
    assert np.array_equal(full, np.concatenate([first, rest]))
    one = oracle.gru_forward(H, 1, row_ptr, col_idx, vals, x[:, 1:2], b_hn, h0[1:2])
    assert np.array_equal(one[:, 0], full[:, 1])
    twin = oracle.gru_forward(H, B, row_ptr, col_idx, vals, x, b_hn, h0, f64=True)
    assert np.abs(full - twin).max() < 2e-5
    assert np.array_equal(full, oracle.gru_forward(H, B, row_ptr, col_idx, vals, x, b_hn, h0, threads=3))


# ----------------------------------------------------------------------------- backward pass through time
@pytest.mark.parametrize("act", ["relu", "tanh", "identity"])
def test_backward_matches_torch_autograd(act):
    rng = np.random.default_rng(31)
    H, B, T = 23, 3, 6
    w = wl.make_workload("b", act, H, B, T, 0.4, seed=5, row_nnz="poisson", h0_std=0.5)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h_fwd = oracle.rnn_forward(H, B, act, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, f64=True).astype(np.float32)
    d_b, dh0, dU = oracle.rnn_backward(H, B, act, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    # the same cell, dense, in torch float64 with autograd
    U = np.zeros((H, H))
    for i in range(H):
        for k in range(w.row_ptr[i], w.row_ptr[i + 1]):
            U[i, w.col_idx[k]] = float(np.array(w.val_bits[k], dtype=np.uint16).view(np.float16))
    Ut = torch.tensor(U, dtype=torch.float64, requires_grad=True)
    xt = torch.tensor(w.x.astype(np.float64), requires_grad=True)
    h0t = torch.tensor(w.h0.astype(np.float64), requires_grad=True)
    f = {"relu": torch.relu, "tanh": torch.tanh, "identity": lambda z: z}[act]
    h, loss = h0t, 0.0
    for t in range(T):
        h = f(h @ Ut.T + xt[t])
        loss = loss + (torch.tensor(e[t].astype(np.float64)) * h).sum()
    loss.backward()
    # the oracle takes g' from the binary32 forward outputs, torch from its own binary64 ones
    np.testing.assert_allclose(d_b, xt.grad.numpy(), rtol=0, atol=2e-6 * np.abs(xt.grad.numpy()).max())
    np.testing.assert_allclose(dh0, h0t.grad.numpy(), rtol=0, atol=2e-6 * np.abs(h0t.grad.numpy()).max())
    dense = Ut.grad.numpy()
    want = np.array([dense[i, w.col_idx[k]] for i in range(H) for k in range(w.row_ptr[i], w.row_ptr[i + 1])])
    np.testing.assert_allclose(dU, want, rtol=0, atol=2e-6 * np.abs(want).max())
    # a transposed matrix in the recurrence is far away
    bad = oracle.rnn_backward(H, B, act, *wl.csr_from_dense(U.T.astype(np.float16)), h_fwd, e, w.h0)[0]
    assert np.abs(bad - d_b).max() > 1e-2


def test_backward_single_step_closed_form_and_zero_weights():
    rng = np.random.default_rng(32)
    H, B = 9, 2
    w = wl.make_workload("b", "tanh", H, B, 1, 0.5, seed=6, h0_std=1.0)
    e = rng.standard_normal((1, B, H)).astype(np.float32)
    h1 = oracle.rnn_forward(H, B, "tanh", w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0)
    d_b, dh0, dU = oracle.rnn_backward(H, B, "tanh", w.row_ptr, w.col_idx, w.val_bits, h1, e, w.h0)
    delta = (1.0 - h1[0].astype(np.float64) ** 2) * e[0]
    assert np.array_equal(d_b[0], delta)
    U = np.zeros((H, H))
    for i in range(H):
        for k in range(w.row_ptr[i], w.row_ptr[i + 1]):
            U[i, w.col_idx[k]] = float(np.array(w.val_bits[k], dtype=np.uint16).view(np.float16))
    np.testing.assert_allclose(dh0, delta @ U, rtol=0, atol=1e-14)
    k = 0
    for i in range(H):
        for kk in range(w.row_ptr[i], w.row_ptr[i + 1]):
            np.testing.assert_allclose(dU[k], (delta[:, i] * w.h0[:, w.col_idx[kk]].astype(np.float64)).sum(), rtol=0, atol=1e-14)
            k += 1
    # zero weights: nothing flows back through time
    zero = np.zeros(H + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16)
    T = 4
    hf = rng.standard_normal((T, B, H)).astype(np.float32)
    ee = rng.standard_normal((T, B, H)).astype(np.float32)
    d_b, dh0, dU = oracle.rnn_backward(H, B, "relu", *zero, hf, ee, None)
    assert np.array_equal(d_b, np.where(hf > 0, ee.astype(np.float64), 0.0))
    assert not dh0.any() and dU.size == 0


def test_backward_agrees_with_finite_differences_of_the_forward_oracle():
    rng = np.random.default_rng(33)
    H, B, T = 7, 1, 4
    w = wl.make_workload("b", "tanh", H, B, T, 0.6, seed=7, h0_std=0.5)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    fwd = lambda x, h0: oracle.rnn_forward(H, B, "tanh", w.row_ptr, w.col_idx, w.val_bits, x, h0, f64=True)
    h_fwd = fwd(w.x, w.h0).astype(np.float32)
    d_b, dh0, _ = oracle.rnn_backward(H, B, "tanh", w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    loss = lambda x, h0: float((fwd(x, h0) * e).sum())
    eps = 2.0 ** -7                             # exactly representable steps of binary32 inputs
    for (t, j) in ((0, 1), (2, 4), (3, 6)):
        xp, xm = w.x.copy(), w.x.copy()
        xp[t, 0, j] += eps
        xm[t, 0, j] -= eps
        fd = (loss(xp, w.h0) - loss(xm, w.h0)) / (float(xp[t, 0, j]) - float(xm[t, 0, j]))
        assert abs(fd - d_b[t, 0, j]) < 2e-3 * max(1.0, abs(fd))
    hp, hm = w.h0.copy(), w.h0.copy()
    hp[0, 3] += eps
    hm[0, 3] -= eps
    fd = (loss(w.x, hp) - loss(w.x, hm)) / (float(hp[0, 3]) - float(hm[0, 3]))
    assert abs(fd - dh0[0, 3]) < 2e-3 * max(1.0, abs(fd))


# ----------------------------------------------------------------------------- backward pass through time, LSTM
def _dense_from_csr(rows, cols, row_ptr, col_idx, val_bits):
    U = np.zeros((rows, cols))
    for i in range(rows):
        for k in range(row_ptr[i], row_ptr[i + 1]):
            U[i, col_idx[k]] = float(np.array(val_bits[k], dtype=np.uint16).view(np.float16))
    return U


def test_lstm_saved_forward_is_the_forward_and_its_gates_reproduce_the_states():
    H, B, T = 19, 2, 5
    w = wl.make_workload("l", "lstm", H, B, T, 0.4, seed=8, h0_std=0.5)
    c0 = np.random.default_rng(40).standard_normal((B, H)).astype(np.float32)
    h, c = oracle.lstm_forward(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
    hs, cs, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
    assert np.array_equal(h, hs) and np.array_equal(c, cs)
    i, f, g, o = (gates[:, :, k * H:(k + 1) * H].astype(np.float64) for k in range(4))
    c_prev = np.concatenate([c0[None], c[:-1]]).astype(np.float64)
    np.testing.assert_allclose(f * c_prev + i * g, c, rtol=0, atol=1e-6)
    np.testing.assert_allclose(o * np.tanh(c.astype(np.float64)), h, rtol=0, atol=1e-6)
    assert (i > 0).all() and (i < 1).all() and (np.abs(g) < 1).all()          # sigmoid and tanh ranges


def test_lstm_backward_matches_torch_autograd_of_lstmcell():
    rng = np.random.default_rng(41)
    H, B, T = 17, 3, 6
    w = wl.make_workload("l", "lstm", H, B, T, 0.4, seed=9, row_nnz="poisson", h0_std=0.5)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
    d_b, dh0, dc0, dU = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
    U = _dense_from_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    cell = torch.nn.LSTMCell(4 * H, H, bias=False).double()                   # gate order i, f, g, o
    with torch.no_grad():
        cell.weight_hh.copy_(torch.from_numpy(U))
        cell.weight_ih.copy_(torch.eye(4 * H, dtype=torch.float64))
    cell.weight_ih.requires_grad_(False)
    xt = torch.tensor(w.x.astype(np.float64), requires_grad=True)
    h0t = torch.tensor(w.h0.astype(np.float64), requires_grad=True)
    c0t = torch.tensor(c0.astype(np.float64), requires_grad=True)
    ht, ct, loss = h0t, c0t, 0.0
    for t in range(T):
        ht, ct = cell(xt[t], (ht, ct))
        loss = loss + (torch.tensor(e[t].astype(np.float64)) * ht).sum()
    loss.backward()
    # the oracle starts from the binary32 forward quantities, torch from its own binary64 ones
    tol = lambda a: 5e-6 * np.abs(a).max()
    np.testing.assert_allclose(d_b, xt.grad.numpy(), rtol=0, atol=tol(xt.grad.numpy()))
    np.testing.assert_allclose(dh0, h0t.grad.numpy(), rtol=0, atol=tol(h0t.grad.numpy()))
    np.testing.assert_allclose(dc0, c0t.grad.numpy(), rtol=0, atol=tol(c0t.grad.numpy()))
    dense = cell.weight_hh.grad.numpy()
    want = np.array([dense[i, w.col_idx[k]] for i in range(4 * H) for k in range(w.row_ptr[i], w.row_ptr[i + 1])])
    np.testing.assert_allclose(dU, want, rtol=0, atol=tol(want))
    # every block of d_bprime carries signal, and two swapped gate blocks are far away
    for k in range(4):
        assert np.abs(d_b[:, :, k * H:(k + 1) * H]).max() > 1e-3
    sw = gates.copy()
    sw[:, :, 0:H], sw[:, :, 3 * H:4 * H] = gates[:, :, 3 * H:4 * H], gates[:, :, 0:H]
    bad = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, sw, c, h, e, w.h0, c0)[0]
    assert np.abs(bad - d_b).max() > 1e-2


def test_lstm_backward_single_step_closed_form_and_zero_weights():
    rng = np.random.default_rng(42)
    H, B = 6, 2
    w = wl.make_workload("l", "lstm", H, B, 1, 0.5, seed=10, h0_std=1.0)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    e = rng.standard_normal((1, B, H)).astype(np.float32)
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
    d_b, dh0, dc0, dU = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
    i, f, g, o = (gates[0][:, k * H:(k + 1) * H].astype(np.float64) for k in range(4))
    tc = np.tanh(c[0].astype(np.float64))
    dc = e[0] * o * (1 - tc * tc)
    want = np.concatenate([dc * g * i * (1 - i), dc * c0 * f * (1 - f), dc * i * (1 - g * g), e[0] * tc * o * (1 - o)], axis=1)
    np.testing.assert_allclose(d_b[0], want, rtol=0, atol=1e-15)
    np.testing.assert_allclose(dc0, dc * f, rtol=0, atol=1e-15)
    U = _dense_from_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    np.testing.assert_allclose(dh0, want @ U, rtol=0, atol=1e-14)
    k = 0
    for r in range(4 * H):
        for kk in range(w.row_ptr[r], w.row_ptr[r + 1]):
            np.testing.assert_allclose(dU[k], (want[:, r] * w.h0[:, w.col_idx[kk]].astype(np.float64)).sum(), rtol=0, atol=1e-14)
            k += 1
    # zero weights: only the cell state carries gradient through time
    zero = np.zeros(4 * H + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16)
    T = 3
    x = rng.standard_normal((T, B, 4 * H)).astype(np.float32)
    ee = rng.standard_normal((T, B, H)).astype(np.float32)
    hz, cz, gz = oracle.lstm_forward_saved(H, B, *zero, x, None, c0)
    d_b, dh0, dc0, dU = oracle.lstm_backward(H, B, *zero, gz, cz, hz, ee, None, c0)
    assert not dh0.any() and dU.size == 0
    fz, oz = gz[:, :, H:2 * H].astype(np.float64), gz[:, :, 3 * H:].astype(np.float64)
    tz = np.tanh(cz.astype(np.float64))
    run = np.zeros((B, H))
    for t in range(T - 1, -1, -1):
        dct = run + ee[t] * oz[t] * (1 - tz[t] ** 2)
        np.testing.assert_allclose(d_b[t][:, 3 * H:], ee[t] * tz[t] * oz[t] * (1 - oz[t]), rtol=0, atol=1e-15)
        run = dct * fz[t]
    np.testing.assert_allclose(dc0, run, rtol=0, atol=1e-15)


def test_lstm_backward_agrees_with_finite_differences_of_the_forward_oracle():
    rng = np.random.default_rng(43)
    H, B, T = 5, 1, 4
    w = wl.make_workload("l", "lstm", H, B, T, 0.6, seed=11, h0_std=0.5)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    fwd = lambda x, h0, cc: oracle.lstm_forward(H, B, w.row_ptr, w.col_idx, w.val_bits, x, h0, cc, f64=True)[0]
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
    d_b, dh0, dc0, _ = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
    loss = lambda x, h0, cc: float((fwd(x, h0, cc) * e).sum())
    eps = 2.0 ** -7
    for (t, r) in ((0, 1), (1, H + 2), (2, 2 * H + 4), (3, 3 * H)):
        xp, xm = w.x.copy(), w.x.copy()
        xp[t, 0, r] += eps
        xm[t, 0, r] -= eps
        fd = (loss(xp, w.h0, c0) - loss(xm, w.h0, c0)) / (float(xp[t, 0, r]) - float(xm[t, 0, r]))
        assert abs(fd - d_b[t, 0, r]) < 2e-3 * max(1.0, abs(fd))
    for (arr, grad, which) in ((w.h0, dh0, 0), (c0, dc0, 1)):
        ap, am = arr.copy(), arr.copy()
        ap[0, 3] += eps
        am[0, 3] -= eps
        args_p = (w.x, ap, c0) if which == 0 else (w.x, w.h0, ap)
        args_m = (w.x, am, c0) if which == 0 else (w.x, w.h0, am)
        fd = (loss(*args_p) - loss(*args_m)) / (float(ap[0, 3]) - float(am[0, 3]))
        assert abs(fd - grad[0, 3]) < 2e-3 * max(1.0, abs(fd))


# ----------------------------------------------------------------------------- backward pass through time, GRU
def test_gru_saved_forward_is_the_forward_and_its_gates_reproduce_the_outputs():
    H, B, T = 19, 2, 5
    w = wl.make_workload("g", "gru", H, B, T, 0.4, seed=12, h0_std=0.5)
    h = oracle.gru_forward(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0)
    hs, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0)
    assert np.array_equal(h, hs)
    r, z, n, q = (gates[:, :, k * H:(k + 1) * H].astype(np.float64) for k in range(4))
    h_prev = np.concatenate([w.h0[None], h[:-1]]).astype(np.float64)
    np.testing.assert_allclose((1 - z) * n + z * h_prev, h, rtol=0, atol=1e-6)
    np.testing.assert_allclose(np.tanh(w.x[:, :, 2 * H:] + r * q), n, rtol=0, atol=1e-6)
    U = _dense_from_csr(3 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    np.testing.assert_allclose(h_prev @ U[2 * H:].T + w.b_hn, q, rtol=0, atol=1e-5)


def test_gru_backward_matches_torch_autograd_of_grucell():
    rng = np.random.default_rng(51)
    H, B, T = 17, 3, 6
    w = wl.make_workload("g", "gru", H, B, T, 0.4, seed=13, row_nnz="poisson", h0_std=0.5)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0)
    d_b, d_rec, dh0, dU, db_hn = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, h, e, w.h0)
    U = _dense_from_csr(3 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    cell = torch.nn.GRUCell(3 * H, H, bias=True).double()                     # gate order r, z, n
    with torch.no_grad():
        cell.weight_hh.copy_(torch.from_numpy(U))
        cell.weight_ih.copy_(torch.eye(3 * H, dtype=torch.float64))
        cell.bias_ih.zero_()
        cell.bias_hh.zero_()
        cell.bias_hh[2 * H:].copy_(torch.from_numpy(w.b_hn.astype(np.float64)))
    cell.weight_ih.requires_grad_(False)
    xt = torch.tensor(w.x.astype(np.float64), requires_grad=True)
    h0t = torch.tensor(w.h0.astype(np.float64), requires_grad=True)
    ht, loss = h0t, 0.0
    for t in range(T):
        ht = cell(xt[t], ht)
        loss = loss + (torch.tensor(e[t].astype(np.float64)) * ht).sum()
    loss.backward()
    tol = lambda a: 5e-6 * np.abs(a).max()
    np.testing.assert_allclose(d_b, xt.grad.numpy(), rtol=0, atol=tol(xt.grad.numpy()))
    np.testing.assert_allclose(dh0, h0t.grad.numpy(), rtol=0, atol=tol(h0t.grad.numpy()))
    dense = cell.weight_hh.grad.numpy()
    want = np.array([dense[i, w.col_idx[k]] for i in range(3 * H) for k in range(w.row_ptr[i], w.row_ptr[i + 1])])
    np.testing.assert_allclose(dU, want, rtol=0, atol=tol(want))
    want_b = cell.bias_hh.grad.numpy()
    np.testing.assert_allclose(db_hn, want_b[2 * H:], rtol=0, atol=tol(want_b))
    # the r and z blocks of the two outputs agree and the bias gradients of b_hr, b_hz are their sums; the candidate
    # blocks differ by the reset gate
    assert np.array_equal(d_b[:, :, :2 * H], d_rec[:, :, :2 * H])
    np.testing.assert_allclose(d_rec[:, :, :2 * H].sum(axis=(0, 1)), want_b[:2 * H], rtol=0, atol=tol(want_b))
    np.testing.assert_allclose(d_rec[:, :, 2 * H:], d_b[:, :, 2 * H:] * gates[:, :, :H], rtol=0, atol=1e-15)
    # two swapped gate blocks are far away
    sw = gates.copy()
    sw[:, :, 0:H], sw[:, :, H:2 * H] = gates[:, :, H:2 * H], gates[:, :, 0:H]
    bad = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, sw, h, e, w.h0)[0]
    assert np.abs(bad - d_b).max() > 1e-2


def test_gru_backward_single_step_closed_form_and_zero_weights():
    rng = np.random.default_rng(52)
    H, B = 6, 2
    w = wl.make_workload("g", "gru", H, B, 1, 0.5, seed=14, h0_std=1.0)
    e = rng.standard_normal((1, B, H)).astype(np.float32)
    h, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0)
    d_b, d_rec, dh0, dU, db_hn = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, h, e, w.h0)
    r, z, n, q = (gates[0][:, k * H:(k + 1) * H].astype(np.float64) for k in range(4))
    da = e[0] * (1 - z) * (1 - n * n)
    want = np.concatenate([da * q * r * (1 - r), e[0] * (w.h0 - n) * z * (1 - z), da], axis=1)
    np.testing.assert_allclose(d_b[0], want, rtol=0, atol=1e-15)
    v = np.concatenate([want[:, :2 * H], da * r], axis=1)
    np.testing.assert_allclose(d_rec[0], v, rtol=0, atol=1e-15)
    U = _dense_from_csr(3 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    np.testing.assert_allclose(dh0, e[0] * z + v @ U, rtol=0, atol=1e-14)
    np.testing.assert_allclose(db_hn, (da * r).sum(axis=0), rtol=0, atol=1e-14)
    k = 0
    for row in range(3 * H):
        for kk in range(w.row_ptr[row], w.row_ptr[row + 1]):
            np.testing.assert_allclose(dU[k], (v[:, row] * w.h0[:, w.col_idx[kk]].astype(np.float64)).sum(), rtol=0, atol=1e-14)
            k += 1
    # zero weights: only the update gate's direct path carries gradient through time
    zero = np.zeros(3 * H + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.uint16)
    T = 3
    x = rng.standard_normal((T, B, 3 * H)).astype(np.float32)
    ee = rng.standard_normal((T, B, H)).astype(np.float32)
    hz, gz = oracle.gru_forward_saved(H, B, *zero, x, None, w.h0)
    d_b, d_rec, dh0, dU, db_hn = oracle.gru_backward(H, B, *zero, gz, hz, ee, w.h0)
    zz = gz[:, :, H:2 * H].astype(np.float64)
    run = np.zeros((B, H))
    for t in range(T - 1, -1, -1):
        dh = ee[t] + run
        np.testing.assert_allclose(d_b[t][:, 2 * H:], dh * (1 - zz[t]) * (1 - gz[t][:, 2 * H:3 * H].astype(np.float64) ** 2), rtol=0, atol=1e-15)
        run = dh * zz[t]
    np.testing.assert_allclose(dh0, run, rtol=0, atol=1e-15)
    assert dU.size == 0 and not d_b[:, :, :H].any()      # q = 0: the reset gate gets no gradient


def test_gru_backward_agrees_with_finite_differences_of_the_forward_oracle():
    rng = np.random.default_rng(53)
    H, B, T = 5, 1, 4
    w = wl.make_workload("g", "gru", H, B, T, 0.6, seed=15, h0_std=0.5)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    fwd = lambda x, h0, b: oracle.gru_forward(H, B, w.row_ptr, w.col_idx, w.val_bits, x, b, h0, f64=True)
    h, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0)
    d_b, _, dh0, _, db_hn = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, h, e, w.h0)
    loss = lambda x, h0, b: float((fwd(x, h0, b) * e).sum())
    eps = 2.0 ** -7
    for (t, r) in ((0, 1), (1, H + 2), (3, 2 * H + 4)):
        xp, xm = w.x.copy(), w.x.copy()
        xp[t, 0, r] += eps
        xm[t, 0, r] -= eps
        fd = (loss(xp, w.h0, w.b_hn) - loss(xm, w.h0, w.b_hn)) / (float(xp[t, 0, r]) - float(xm[t, 0, r]))
        assert abs(fd - d_b[t, 0, r]) < 2e-3 * max(1.0, abs(fd))
    hp, hm = w.h0.copy(), w.h0.copy()
    hp[0, 3] += eps
    hm[0, 3] -= eps
    fd = (loss(w.x, hp, w.b_hn) - loss(w.x, hm, w.b_hn)) / (float(hp[0, 3]) - float(hm[0, 3]))
    assert abs(fd - dh0[0, 3]) < 2e-3 * max(1.0, abs(fd))
    bp, bm = w.b_hn.copy(), w.b_hn.copy()
    bp[2] += eps
    bm[2] -= eps
    fd = (loss(w.x, w.h0, bp) - loss(w.x, w.h0, bm)) / (float(bp[2]) - float(bm[2]))
    assert abs(fd - db_hn[2]) < 2e-3 * max(1.0, abs(fd))
