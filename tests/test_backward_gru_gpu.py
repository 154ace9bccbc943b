"""Parity of the GRU's training path (sprnn_forward_gru_train, sprnn_backward_gru, sprnn_weight_gradient on a GRU
handle) against the CPU oracle, through the C ABI.

Both sides of a backward comparison get the same inputs: r, z, n, q and the outputs kept by the oracle's own binary32
forward pass, and seeded e_t = dL/dh_t.  Bar, as everywhere: per timestep max|got - want| <= 1e-3 * max|want|.
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


def _close(got, want, what):
    assert np.all(np.isfinite(got)), what
    assert np.abs(got - want).max() <= REL_TOL * np.abs(want).max() + 1e-30, what


def run_backward(w, e, **options):
    H, B, T = w.hidden, w.batch, w.steps
    h, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0, threads=8)
    want_d, want_v, want_dh0, want_dU, want_db = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, h, e, w.h0)
    t_csr = binding.transpose_csr(3 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(H, B, "gru_backward", *t_csr, **options) as rnn:
        info = rnn.info()
        print("case gru_backward H", H, "B", B, "T", T, options,
              {k: info[k] for k in ("grid", "block", "lanes_per_row", "sync", "compact", "template_words")}, flush=True)
        d, v, dh0 = rnn.backward_gru(_dev(e), _dev(gates), _dev(h), _dev(w.h0))
        assert rnn.check() == binding.SPRNN_OK
        d, v, dh0 = d.cpu().numpy(), v.cpu().numpy(), dh0.cpu().numpy()
        # second call on the same handle, without the optional outputs (one step fewer)
        again, n1, n2 = rnn.backward_gru(_dev(e), _dev(gates), _dev(h), _dev(w.h0), want_dh0=False, want_recurrent=False)
        assert n1 is None and n2 is None and np.array_equal(again.cpu().numpy(), d)
        assert rnn.check() == binding.SPRNN_OK
    for t in range(T):
        _close(d[t], want_d[t], "d_bprime[%d]" % t)
        _close(v[t], want_v[t], "d_recurrent[%d]" % t)
    _close(dh0, want_dh0, "dh0")
    assert np.array_equal(d[:, :, :2 * H], v[:, :, :2 * H])          # the r and z blocks are the same numbers
    _close(v[:, :, 2 * H:].sum(axis=(0, 1), dtype=np.float64), want_db, "db_hn from d_recurrent")
    return h, want_v, want_dU


@pytest.mark.parametrize("B", [1, 2])
def test_gru_backward_at_the_largest_hidden_size(B):
    # H = 21845: 3H = 65535 gate rows, the most a 16-bit column index of the transposed matrix reaches.  H of the 3H
    # rows of U hold a single 1.0, one per column, the last row among them: a wrong index moves a whole gate gradient
    # to the wrong place, far outside the bar.
    H, T = 21845, 3
    rng = np.random.default_rng(21845 + B)
    chosen = np.sort(np.concatenate([rng.permutation(3 * H - 1)[:H - 1], [3 * H - 1]])).astype(np.int64)
    cols = rng.permutation(H).astype(np.int32)
    counts = np.zeros(3 * H, dtype=np.int64)
    counts[chosen] = 1
    row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    x = rng.standard_normal((T, B, 3 * H)).astype(np.float32)
    b_hn = (rng.standard_normal(H) * 0.1).astype(np.float32)
    h0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    h, gates = oracle.gru_forward_saved(H, B, row_ptr, cols, ones, x, b_hn, h0, threads=8)
    want_d, want_v, want_dh0, _, _ = oracle.gru_backward(H, B, row_ptr, cols, ones, gates, h, e, h0)
    t_csr = binding.transpose_csr(3 * H, H, row_ptr, cols, ones)
    assert t_csr[1].max() == 3 * H - 1 == 65534
    with binding.SparseRNN(H, B, "gru_backward", *t_csr) as rnn:
        info = rnn.info()
        print("case gru_backward at the index limit, B", B, {k: info[k] for k in ("grid", "block", "compact", "lds_bytes")}, flush=True)
        d, v, dh0 = rnn.backward_gru(_dev(e), _dev(gates), _dev(h), _dev(h0))
        assert rnn.check() == binding.SPRNN_OK
        d, v, dh0 = d.cpu().numpy(), v.cpu().numpy(), dh0.cpu().numpy()
    for t in range(T):
        _close(d[t], want_d[t], "d_bprime[%d]" % t)
        _close(v[t], want_v[t], "d_recurrent[%d]" % t)
    _close(dh0, want_dh0, "dh0")
    # element by element too: every entry of dL/dh_0 holds one moved gate gradient of size O(1)
    assert np.abs(dh0 - want_dh0).max() <= REL_TOL * max(1.0, np.abs(want_dh0).max())
    with pytest.raises(binding.SprnnError) as err:                      # one more and the index no longer fits
        binding.SparseRNN(H + 1, B, "gru_backward", np.zeros(H + 2, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16))
    assert err.value.code == binding.SPRNN_ERR_UNSUPPORTED


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
    (150, 2, 1, 0.3, "poisson", {}),
])
def test_gru_backward_matches_oracle(H, B, T, dens, rownnz, opts):
    w = wl.make_workload("gb", "gru", H, B, T, dens, seed=H + T, gain=1.0, row_nnz=rownnz, h0_std=0.5)
    e = np.random.default_rng(H).standard_normal((T, B, H)).astype(np.float32)
    run_backward(w, e, **opts)


def test_gru_training_forward_keeps_the_gate_values():
    H, B, T = 300, 4, 12
    w = wl.make_workload("gf", "gru", H, B, T, 0.2, seed=78, gain=1.0, row_nnz="poisson", h0_std=0.5)
    want_h, want_g = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0, threads=8)
    with binding.SparseRNN(H, B, "gru", w.row_ptr, w.col_idx, w.val_bits) as rnn:
        h, g = rnn.forward_gru_train(_dev(w.x), _dev(w.b_hn), _dev(w.h0))
        h2 = rnn.forward_gru(_dev(w.x), _dev(w.b_hn), _dev(w.h0))
        assert rnn.check() == binding.SPRNN_OK
        h, g = h.cpu().numpy(), g.cpu().numpy()
        assert np.array_equal(h, h2.cpu().numpy())                    # the same arithmetic
    for t in range(T):
        _close(h[t], want_h[t], "h[%d]" % t)
        for q in range(4):   # each block against its own scale
            _close(g[t][:, q * H:(q + 1) * H], want_g[t][:, q * H:(q + 1) * H], "gates[%d] block %d" % (t, q))


def test_gru_training_step_on_the_gpu_alone_and_its_weight_gradient():
    # hidden 1024, density 20 %, batch 4 (the cells table's shape): backward and weight gradient against the oracle,
    # then the whole chain on the GPU, its own forward quantities feeding its backward pass
    H, B, T = 1024, 4, 24
    w = wl.make_workload("gt", "gru", H, B, T, 0.20, seed=0, gain=1.0, h0_std=0.3)
    e = np.random.default_rng(7).standard_normal((T, B, H)).astype(np.float32)
    h, want_v, want_dU = run_backward(w, e)
    with binding.SparseRNN(H, B, "gru", w.row_ptr, w.col_idx, w.val_bits) as fwd:
        got_dU = fwd.weight_gradient(_dev(want_v.astype(np.float32)), _dev(h), _dev(w.h0)).cpu().numpy()
        assert fwd.check() == binding.SPRNN_OK
        _close(got_dU, want_dU, "dU")
        gh, gg = fwd.forward_gru_train(_dev(w.x), _dev(w.b_hn), _dev(w.h0))
        t_csr = binding.transpose_csr(3 * H, H, w.row_ptr, w.col_idx, w.val_bits)
        with binding.SparseRNN(H, B, "gru_backward", *t_csr) as bwd:
            d, v, dh0 = bwd.backward_gru(_dev(e), gg, gh, _dev(w.h0))
            assert bwd.check() == binding.SPRNN_OK
        dU = fwd.weight_gradient(v, gh, _dev(w.h0)).cpu().numpy()
        assert fwd.check() == binding.SPRNN_OK
    v = v.cpu().numpy()
    for t in range(T):
        _close(v[t], want_v[t], "chain d_recurrent[%d]" % t)
    _close(dU, want_dU, "chain dU")


def test_gru_weight_gradient_small_shapes():
    for (H, B, T, dens, opts) in ((96, 4, 7, 0.3, {}), (130, 8, 5, 0.2, {}), (75, 1, 6, 0.4, {}), (24, 2, 5, 0.5, {"grid": 1})):
        w = wl.make_workload("gw", "gru", H, B, T, dens, seed=H, gain=1.0, row_nnz="poisson", h0_std=0.5)
        e = np.random.default_rng(H).standard_normal((T, B, H)).astype(np.float32)
        h, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0)
        _, want_v, _, want_dU, _ = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, h, e, w.h0)
        with binding.SparseRNN(H, B, "gru", w.row_ptr, w.col_idx, w.val_bits, **opts) as fwd:
            print("case gru weight gradient H", H, "B", B, opts, flush=True)
            got = fwd.weight_gradient(_dev(want_v.astype(np.float32)), _dev(h), _dev(w.h0)).cpu().numpy()
            assert fwd.check() == binding.SPRNN_OK
        _close(got, want_dU, "dU H=%d" % H)


def test_gru_backward_zero_weights_and_wrong_handles():
    H, B, T = 64, 4, 3
    rng = np.random.default_rng(3)
    gates = rng.uniform(0.05, 0.95, size=(T, B, 4 * H)).astype(np.float32)
    hf = rng.standard_normal((T, B, H)).astype(np.float32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    zero3 = np.zeros(3 * H + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16)
    want_d, want_v, want_dh0, _, _ = oracle.gru_backward(H, B, *zero3, gates, hf, e, h0)
    with binding.SparseRNN(H, B, "gru_backward", np.zeros(H + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16)) as bwd:
        d, v, dh0 = bwd.backward_gru(_dev(e), _dev(gates), _dev(hf), _dev(h0))
        assert bwd.check() == binding.SPRNN_OK
        np.testing.assert_allclose(d.cpu().numpy(), want_d, rtol=0, atol=2e-6 * np.abs(want_d).max())
        np.testing.assert_allclose(v.cpu().numpy(), want_v, rtol=0, atol=2e-6 * np.abs(want_v).max())
        np.testing.assert_allclose(dh0.cpu().numpy(), want_dh0, rtol=0, atol=2e-6 * np.abs(want_dh0).max())
        z, z3, z4 = torch.zeros((T, B, H), device="cuda"), torch.zeros((T, B, 3 * H), device="cuda"), torch.zeros((T, B, 4 * H), device="cuda")
        for call in (lambda: bwd.forward(z), lambda: bwd.backward(z, z), lambda: bwd.backward_lstm(z, z4, z),
                     lambda: bwd.weight_gradient(z, z)):
            with pytest.raises(binding.SprnnError) as err:
                call()
            assert err.value.code == binding.SPRNN_ERR_UNSUPPORTED
        d0, v0, dh00 = bwd.backward_gru(z[:0], z4[:0], z[:0])          # T = 0: nothing flows back
        assert d0.shape[0] == 0 and not dh00.cpu().numpy().any()
    w = wl.make_workload("gx", "gru", H, B, T, 0.3, seed=1, gain=1.0)
    with binding.SparseRNN(H, B, "gru", w.row_ptr, w.col_idx, w.val_bits) as fwd:
        with pytest.raises(binding.SprnnError) as err:
            fwd.backward_gru(z, z4, z)
        assert err.value.code == binding.SPRNN_ERR_UNSUPPORTED


@pytest.mark.parametrize("H,B,T,dens,rownnz,opts", [
    (96, 4, 9, 0.3, "fixed", {}),
    (257, 1, 7, 0.2, "poisson", {}),
    (130, 8, 5, 0.1, "poisson", {}),
    (333, 2, 6, 0.15, "poisson", {"balance": 1}),
    (32, 4, 8, 0.4, "fixed", {"grid": 1}),
    (320, 4, 10, 0.3, "fixed", {"sync": "barrier"}),
    (576, 4, 32, 0.1, "fixed", {"jitter": 7}),
    (1024, 8, 16, 0.2, "fixed", {}),
])
def test_gru_backward_with_weights_matches_oracle(H, B, T, dens, rownnz, opts):
    w = wl.make_workload("gbw", "gru", H, B, T, dens, seed=H + T + 1, gain=1.0, row_nnz=rownnz, h0_std=0.5)
    e = np.random.default_rng(H + 1).standard_normal((T, B, H)).astype(np.float32)
    h, gates = oracle.gru_forward_saved(H, B, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0, threads=8)
    want_d, want_v, want_dh0, want_dU, _ = oracle.gru_backward(H, B, w.row_ptr, w.col_idx, w.val_bits, gates, h, e, w.h0)
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(3 * H, H, w.row_ptr, w.col_idx, w.val_bits, with_source=True)
    with binding.SparseRNN(H, B, "gru_backward", t_rp, t_ci, t_vb, **opts) as rnn:
        info = rnn.info()
        print("case fused gru_backward H", H, "B", B, "T", T, opts,
              {k: info[k] for k in ("grid", "block", "lanes_per_row", "template_words")}, flush=True)
        try:
            d, v, dh0, dU_t = rnn.backward_gru_with_weights(_dev(e), _dev(gates), _dev(h), _dev(w.h0))
        except binding.SprnnError as err:
            if err.code == binding.SPRNN_ERR_UNSUPPORTED:
                pytest.skip("mapping too wide for the fused instantiation: %s" % err)
            raise
        assert rnn.check() == binding.SPRNN_OK
        # the plain backward pass on the same handle gives the same gradients, bit for bit
        d2, v2, dh02 = rnn.backward_gru(_dev(e), _dev(gates), _dev(h), _dev(w.h0))
        assert np.array_equal(d2.cpu().numpy(), d.cpu().numpy()) and np.array_equal(v2.cpu().numpy(), v.cpu().numpy())
        assert np.array_equal(dh02.cpu().numpy(), dh0.cpu().numpy())
        d3, n1, n2, dU_t3 = rnn.backward_gru_with_weights(_dev(e), _dev(gates), _dev(h), _dev(w.h0), want_dh0=False, want_recurrent=False)
        assert n1 is None and n2 is None and np.array_equal(dU_t3.cpu().numpy(), dU_t.cpu().numpy())
        assert rnn.check() == binding.SPRNN_OK
    d, v, dU_t = d.cpu().numpy(), v.cpu().numpy(), dU_t.cpu().numpy()
    for t in range(T):
        _close(d[t], want_d[t], "d_bprime[%d]" % t)
        _close(v[t], want_v[t], "d_recurrent[%d]" % t)
    _close(dh0.cpu().numpy(), want_dh0, "dh0")
    dU = np.empty_like(dU_t)
    dU[t_src] = dU_t                       # back to the forward matrix's CSR order
    _close(dU, want_dU, "dU")
