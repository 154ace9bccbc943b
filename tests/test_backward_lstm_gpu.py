"""Parity of the LSTM's training path (sprnn_forward_lstm_train, sprnn_backward_lstm, sprnn_weight_gradient on an
LSTM handle) against the CPU oracle, through the C ABI.

Both sides of a backward comparison get the same inputs: the gate values, cell states and outputs kept by the oracle's
own binary32 forward pass, and seeded e_t = dL/dh_t.  Bar, as everywhere: per timestep
max|got - want| <= 1e-3 * max|want|, for dL/db'_t (all four gate blocks together), dL/dh_0 and dL/dc_0.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1804_10223_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

REL_TOL = 1e-3


def _dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _workload(H, B, T, dens, rownnz, seed):
    w = wl.make_workload("lb", "lstm", H, B, T, dens, seed=seed, row_nnz=rownnz, h0_std=0.5)
    rng = np.random.default_rng(seed + 1000)
    c0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    return w, c0, e


def _close(got, want, what):
    assert np.all(np.isfinite(got)), what
    assert np.abs(got - want).max() <= REL_TOL * np.abs(want).max() + 1e-30, what


def run_backward(w, c0, e, **options):
    H, B, T = w.hidden, w.batch, w.steps
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0, threads=8)
    want_d, want_dh0, want_dc0, want_dU = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
    t_rp, t_ci, t_vb = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb, **options) as rnn:
        info = rnn.info()
        print("case lstm_backward H", H, "B", B, "T", T, options,
              {k: info[k] for k in ("grid", "block", "lanes_per_row", "sync", "compact", "template_words")}, flush=True)
        got_d, got_dh0, got_dc0 = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0))
        assert rnn.check() == binding.SPRNN_OK
        got_d, got_dh0, got_dc0 = got_d.cpu().numpy(), got_dh0.cpu().numpy(), got_dc0.cpu().numpy()
        # second call on the same handle, without the initial-state gradients (one step fewer)
        again, n1, n2 = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0), want_dh0=False, want_dc0=False)
        assert n1 is None and n2 is None and np.array_equal(again.cpu().numpy(), got_d)
        assert rnn.check() == binding.SPRNN_OK
    for t in range(T):
        _close(got_d[t], want_d[t], "d_bprime[%d]" % t)
    _close(got_dh0, want_dh0, "dh0")
    _close(got_dc0, want_dc0, "dc0")
    return h, got_d, want_d, want_dU


@pytest.mark.parametrize("H,B,T,dens,rownnz,opts", [
    (96, 4, 9, 0.3, "fixed", {}),
    (257, 1, 7, 0.2, "poisson", {}),
    (130, 8, 5, 0.1, "poisson", {}),
    (333, 2, 6, 0.15, "poisson", {"balance": 1}),
    (32, 4, 8, 0.4, "fixed", {"grid": 1}),
    (48, 8, 6, 0.5, "fixed", {"grid": 1}),
    (320, 4, 10, 0.3, "fixed", {"sync": "barrier"}),
    (1500, 4, 6, 0.004, "poisson", {"compact": 1}),
    (576, 4, 32, 0.1, "fixed", {}),
    (512, 8, 12, 0.2, "fixed", {"jitter": 5}),
])
def test_lstm_backward_matches_oracle(H, B, T, dens, rownnz, opts):
    w, c0, e = _workload(H, B, T, dens, rownnz, seed=H + T)
    run_backward(w, c0, e, **opts)


@pytest.mark.parametrize("B", [1, 4])
def test_lstm_backward_at_the_largest_hidden_size(B):
    # H = 16383: 4H = 65532 gate rows, the most a 16-bit column index of the transposed matrix reaches.  H of the 4H
    # rows of U hold a single 1.0, one per column, so dL/dh_{t-1} = e_{t-1} + (one gate gradient each): parity with
    # the oracle as everywhere, and dL/dh_0 must be the chosen entries of dL/db'_0 bit for bit.
    H, T = 16383, 3
    rng = np.random.default_rng(16383 + B)
    chosen = np.sort(rng.permutation(4 * H)[:H]).astype(np.int64)      # the rows of U that are not empty
    cols = rng.permutation(H).astype(np.int32)                         # row chosen[k] reads column cols[k]
    counts = np.zeros(4 * H, dtype=np.int64)
    counts[chosen] = 1
    row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    x = rng.standard_normal((T, B, 4 * H)).astype(np.float32)
    h0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    c0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h, c, gates = oracle.lstm_forward_saved(H, B, row_ptr, cols, ones, x, h0, c0, threads=8)
    want_d, want_dh0, want_dc0, _ = oracle.lstm_backward(H, B, row_ptr, cols, ones, gates, c, h, e, h0, c0)
    t_rp, t_ci, t_vb = binding.transpose_csr(4 * H, H, row_ptr, cols, ones)
    gate_row_of_column = np.empty(H, dtype=np.int64)
    gate_row_of_column[cols] = chosen
    assert np.array_equal(t_ci[:H], gate_row_of_column) and t_ci.max() >= 4 * H - 40
    with binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb) as rnn:
        info = rnn.info()
        print("case lstm_backward at the index limit, B", B, {k: info[k] for k in ("grid", "block", "compact", "lds_bytes")}, flush=True)
        got_d, got_dh0, got_dc0 = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0))
        assert rnn.check() == binding.SPRNN_OK
        got_d, got_dh0, got_dc0 = got_d.cpu().numpy(), got_dh0.cpu().numpy(), got_dc0.cpu().numpy()
    for t in range(T):
        _close(got_d[t], want_d[t], "d_bprime[%d]" % t)
    _close(got_dh0, want_dh0, "dh0")
    _close(got_dc0, want_dc0, "dc0")
    moved = got_d[0][:, gate_row_of_column] + np.float32(0)
    assert np.array_equal(got_dh0.view(np.uint32), moved.view(np.uint32))
    with pytest.raises(binding.SprnnError) as err:                      # one more and the index no longer fits
        binding.SparseRNN(H + 1, B, "lstm_backward", np.zeros(H + 2, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16))
    assert err.value.code == binding.SPRNN_ERR_UNSUPPORTED


def test_lstm_backward_single_timestep_and_one_wanted_initial_gradient():
    H, B, T = 150, 2, 1
    w, c0, e = _workload(H, B, T, 0.3, "poisson", seed=21)
    run_backward(w, c0, e)
    # only one of the two initial-state gradients asked for: the other costs nothing and is not written
    H, B, T = 210, 4, 7
    w, c0, e = _workload(H, B, T, 0.2, "fixed", seed=22)
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
    want_d, want_dh0, want_dc0, _ = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
    t_csr = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(H, B, "lstm_backward", *t_csr) as rnn:
        d1, dh0, none = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0), want_dc0=False)
        d2, none2, dc0 = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0), want_dh0=False)
        d3, _, dc0_zero = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), None)          # c_0 = 0: dp_f of the first step is 0
        assert rnn.check() == binding.SPRNN_OK
    assert none is None and none2 is None and np.array_equal(d1.cpu().numpy(), d2.cpu().numpy())
    _close(dh0.cpu().numpy(), want_dh0, "dh0 alone")
    _close(dc0.cpu().numpy(), want_dc0, "dc0 alone")
    assert not d3.cpu().numpy()[0][:, H:2 * H].any()
    _close(dc0_zero.cpu().numpy(), want_dc0, "dc0 with c0 = 0")      # dc_1 f_1 does not depend on c_0


def test_lstm_backward_zero_weights_closed_form():
    # nothing flows through h: dp_o = e tanh(c) o (1 - o) exactly as binary32 products, dL/dh_0 = 0
    H, B, T = 200, 4, 5
    rng = np.random.default_rng(2)
    gates = rng.uniform(0.05, 0.95, size=(T, B, 4 * H)).astype(np.float32)
    c = rng.standard_normal((T, B, H)).astype(np.float32)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    zero = np.zeros(4 * H + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16)
    want_d, want_dh0, want_dc0, _ = oracle.lstm_backward(H, B, *zero, gates, c, np.zeros_like(c), e, None, c0)
    with binding.SparseRNN(H, B, "lstm_backward", np.zeros(H + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16)) as rnn:
        d, dh0, dc0 = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0))
        assert rnn.check() == binding.SPRNN_OK
    assert not dh0.cpu().numpy().any()
    np.testing.assert_allclose(d.cpu().numpy(), want_d, rtol=0, atol=2e-6 * np.abs(want_d).max())
    np.testing.assert_allclose(dc0.cpu().numpy(), want_dc0, rtol=0, atol=2e-6 * np.abs(want_dc0).max())
    assert not want_dh0.any()


def test_lstm_training_forward_keeps_the_gate_values():
    H, B, T = 300, 4, 12
    w, c0, _ = _workload(H, B, T, 0.2, "poisson", seed=77)
    want_h, want_c, want_g = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0, threads=8)
    with binding.SparseRNN(H, B, "lstm", w.row_ptr, w.col_idx, w.val_bits) as rnn:
        h, c, g = rnn.forward_lstm_train(_dev(w.x), _dev(w.h0), _dev(c0))
        h2, c2 = rnn.forward_lstm(_dev(w.x), _dev(w.h0), _dev(c0))
        assert rnn.check() == binding.SPRNN_OK
        h, c, g = h.cpu().numpy(), c.cpu().numpy(), g.cpu().numpy()
        assert np.array_equal(h, h2.cpu().numpy()) and np.array_equal(c, c2.cpu().numpy())   # the same arithmetic
    for t in range(T):
        _close(h[t], want_h[t], "h[%d]" % t)
        _close(c[t], want_c[t], "c[%d]" % t)
        for q in range(4):   # each gate block against its own scale
            _close(g[t][:, q * H:(q + 1) * H], want_g[t][:, q * H:(q + 1) * H], "gates[%d] block %d" % (t, q))


def test_lstm_training_step_at_the_lstm_config_shape():
    # forward (keeping gates), backward and weight gradient, all on the GPU, against the oracle's whole chain
    w = wl.make_config("cfg5", steps=24)
    H, B, T = w.hidden, w.batch, w.steps
    rng = np.random.default_rng(5)
    c0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h, got_d, want_d, want_dU = run_backward(w, c0, e)
    # the gradient of the 0.84 M recurrent weights on the forward handle, from the oracle's dp (rounded to binary32)
    with binding.SparseRNN(H, B, "lstm", w.row_ptr, w.col_idx, w.val_bits) as fwd:
        got_dU = fwd.weight_gradient(_dev(want_d.astype(np.float32)), _dev(h), _dev(w.h0)).cpu().numpy()
        assert fwd.check() == binding.SPRNN_OK
        _close(got_dU, want_dU, "dU")
        # the whole chain on the GPU: its own forward quantities feed its backward pass
        gh, gc, gg = fwd.forward_lstm_train(_dev(w.x), _dev(w.h0), _dev(c0))
        t_rp, t_ci, t_vb = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
        with binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb) as bwd:
            d, dh0, dc0 = bwd.backward_lstm(_dev(e), gg, gc, _dev(c0))
            assert bwd.check() == binding.SPRNN_OK
        dU = fwd.weight_gradient(d, gh, _dev(w.h0)).cpu().numpy()
        assert fwd.check() == binding.SPRNN_OK
    d = d.cpu().numpy()
    for t in range(T):
        _close(d[t], want_d[t], "chain d_bprime[%d]" % t)
    _close(dU, want_dU, "chain dU")


def test_lstm_weight_gradient_small_shapes():
    for (H, B, T, dens, opts) in ((96, 4, 7, 0.3, {}), (130, 8, 5, 0.2, {}), (75, 1, 6, 0.4, {}), (24, 2, 5, 0.5, {"grid": 1})):
        w, c0, e = _workload(H, B, T, dens, "poisson", seed=H)
        h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0)
        want_d, _, _, want_dU = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
        with binding.SparseRNN(H, B, "lstm", w.row_ptr, w.col_idx, w.val_bits, **opts) as fwd:
            print("case lstm weight gradient H", H, "B", B, opts, flush=True)
            got = fwd.weight_gradient(_dev(want_d.astype(np.float32)), _dev(h), _dev(w.h0)).cpu().numpy()
            assert fwd.check() == binding.SPRNN_OK
        _close(got, want_dU, "dU H=%d" % H)


def test_lstm_backward_wrong_handles_are_refused():
    H, B, T = 64, 4, 3
    w, c0, e = _workload(H, B, T, 0.3, "fixed", seed=9)
    z = torch.zeros((T, B, H), device="cuda")
    z4 = torch.zeros((T, B, 4 * H), device="cuda")
    with binding.SparseRNN(H, B, "lstm", w.row_ptr, w.col_idx, w.val_bits) as fwd:
        with pytest.raises(binding.SprnnError) as err:
            fwd.backward_lstm(z, z4, z)
        assert err.value.code == binding.SPRNN_ERR_UNSUPPORTED
    t_rp, t_ci, t_vb = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb) as bwd:
        for call in (lambda: bwd.forward(z), lambda: bwd.backward(z, z), lambda: bwd.forward_stepwise(z),
                     lambda: bwd.weight_gradient(z, z)):
            with pytest.raises(binding.SprnnError) as err:
                call()
            assert err.value.code == binding.SPRNN_ERR_UNSUPPORTED
        # T = 0: nothing flows back
        d, dh0, dc0 = bwd.backward_lstm(z[:0], z4[:0], z[:0])
        assert d.shape[0] == 0 and not dh0.cpu().numpy().any() and not dc0.cpu().numpy().any()


@pytest.mark.parametrize("H,B,T,dens,rownnz,opts", [
    (96, 4, 9, 0.3, "fixed", {}),
    (257, 1, 7, 0.2, "poisson", {}),
    (130, 8, 5, 0.1, "poisson", {}),
    (333, 2, 6, 0.15, "poisson", {"balance": 1}),
    (32, 4, 8, 0.4, "fixed", {"grid": 1}),
    (320, 4, 10, 0.3, "fixed", {"sync": "barrier"}),
    (576, 4, 32, 0.1, "fixed", {"jitter": 7}),
])
def test_lstm_backward_with_weights_matches_oracle(H, B, T, dens, rownnz, opts):
    w, c0, e = _workload(H, B, T, dens, rownnz, seed=H + T + 1)
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, c0, threads=8)
    want_d, want_dh0, want_dc0, want_dU = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, w.h0, c0)
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits, with_source=True)
    with binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb, **opts) as rnn:
        info = rnn.info()
        print("case fused lstm_backward H", H, "B", B, "T", T, opts,
              {k: info[k] for k in ("grid", "block", "lanes_per_row", "template_words")}, flush=True)
        try:
            d, dh0, dc0, dU_t = rnn.backward_lstm_with_weights(_dev(e), _dev(gates), _dev(c), _dev(h), _dev(c0), _dev(w.h0))
        except binding.SprnnError as err:
            if err.code == binding.SPRNN_ERR_UNSUPPORTED:
                pytest.skip("mapping too wide for the fused instantiation: %s" % err)
            raise
        assert rnn.check() == binding.SPRNN_OK
        # the plain backward pass on the same handle gives the same gradients, bit for bit
        d2, dh02, dc02 = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0))
        assert np.array_equal(d2.cpu().numpy(), d.cpu().numpy()) and np.array_equal(dh02.cpu().numpy(), dh0.cpu().numpy())
        assert np.array_equal(dc02.cpu().numpy(), dc0.cpu().numpy())
        # without the initial-state gradients the extra step still runs (it pairs dp_1 with h_0)
        d3, n1, n2, dU_t3 = rnn.backward_lstm_with_weights(_dev(e), _dev(gates), _dev(c), _dev(h), _dev(c0), _dev(w.h0),
                                                          want_dh0=False, want_dc0=False)
        assert n1 is None and n2 is None and np.array_equal(dU_t3.cpu().numpy(), dU_t.cpu().numpy())
        assert np.array_equal(d3.cpu().numpy(), d.cpu().numpy())
        assert rnn.check() == binding.SPRNN_OK
    d, dU_t = d.cpu().numpy(), dU_t.cpu().numpy()
    for t in range(T):
        _close(d[t], want_d[t], "d_bprime[%d]" % t)
    _close(dh0.cpu().numpy(), want_dh0, "dh0")
    _close(dc0.cpu().numpy(), want_dc0, "dc0")
    dU = np.empty_like(dU_t)
    dU[t_src] = dU_t                       # back to the forward matrix's CSR order
    _close(dU, want_dU, "dU")


def test_lstm_backward_with_weights_at_the_lstm_config_shape():
    w = wl.make_config("cfg5", steps=20)
    H, B, T = w.hidden, w.batch, w.steps
    rng = np.random.default_rng(6)
    c0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h, c, gates = oracle.lstm_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, None, c0, threads=8)
    want_d, want_dh0, _, want_dU = oracle.lstm_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, c, h, e, None, c0)
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits, with_source=True)
    with binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb) as rnn:
        d, dh0, _, dU_t = rnn.backward_lstm_with_weights(_dev(e), _dev(gates), _dev(c), _dev(h), _dev(c0), None)
        assert rnn.check() == binding.SPRNN_OK
    d, dU_t = d.cpu().numpy(), dU_t.cpu().numpy()
    for t in range(T):
        _close(d[t], want_d[t], "d_bprime[%d]" % t)
    _close(dh0.cpu().numpy(), want_dh0, "dh0")
    dU = np.empty_like(dU_t)
    dU[t_src] = dU_t
    _close(dU, want_dU, "dU")
