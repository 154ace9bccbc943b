"""Parity of the backward pass through time (sprnn_backward) against the CPU oracle, through the C ABI.

Both sides get the same inputs: the oracle's own forward outputs h_t (binary32) and seeded e_t = dL/dh_t.
Bar, as for the forward pass: per timestep  max|delta_gpu - delta_oracle| <= 1e-3 * max|delta_oracle|, same for dL/dh_0.
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


def assert_weight_gradient(dU, want, row_ptr, what=""):
    """dL/dU against the oracle: one max-norm over all nonzeros, and row by row at each row's own scale (a row whose
    gradients are small must be right at ITS size; the floor of 1e-5 of the largest entry covers rows that cancel to
    almost nothing)."""
    assert dU.shape == want.shape and np.all(np.isfinite(dU)), what
    top = np.abs(want).max() if want.size else 0.0
    assert np.abs(dU - want).max() <= REL_TOL * top + 1e-30, what
    err = np.abs(dU - want)
    starts = np.asarray(row_ptr[:-1], dtype=np.int64)
    nonempty = np.diff(row_ptr) > 0
    if not nonempty.any():
        return
    row_err = np.maximum.reduceat(err, starts[nonempty])
    row_top = np.maximum.reduceat(np.abs(want), starts[nonempty])
    worst = int(np.argmax(row_err - (REL_TOL * row_top + 1e-5 * top)))
    assert np.all(row_err <= REL_TOL * row_top + 1e-5 * top), "%s: row %d err %.3e at scale %.3e" % (what, worst, row_err[worst], row_top[worst])


def run_case(w, e, **options):
    h_fwd = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    want_d, want_dh0, _ = oracle.rnn_backward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    t_rp, t_ci, t_vb = binding.transpose_csr(w.hidden, w.hidden, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, t_rp, t_ci, t_vb, **options) as rnn:
        info = rnn.info()
        print("case", w.cell, "H", w.hidden, "B", w.batch, "T", w.steps, options, {k: info[k] for k in ("grid", "block", "lanes_per_row", "sync")}, flush=True)
        got_d, got_dh0 = rnn.backward(_dev(e), _dev(h_fwd))
        assert rnn.check() == binding.SPRNN_OK
        got_d, got_dh0 = got_d.cpu().numpy(), got_dh0.cpu().numpy()
        again, none = rnn.backward(_dev(e), _dev(h_fwd), want_dh0=False)     # second call on the same handle, no dh0
        assert none is None and np.array_equal(again.cpu().numpy(), got_d)
        assert rnn.check() == binding.SPRNN_OK
    assert np.all(np.isfinite(got_d)) and np.all(np.isfinite(got_dh0))
    for t in range(w.steps):
        scale = np.abs(want_d[t]).max()
        assert np.abs(got_d[t] - want_d[t]).max() <= REL_TOL * scale + 1e-30, t
    assert np.abs(got_dh0 - want_dh0).max() <= REL_TOL * np.abs(want_dh0).max() + 1e-30
    return got_d


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts", [
    ("relu", 96, 4, 9, 0.3, "fixed", {}),
    ("tanh", 257, 1, 7, 0.2, "poisson", {}),
    ("identity", 130, 8, 5, 0.1, "poisson", {}),
    ("relu", 333, 2, 6, 0.15, "poisson", {"balance": 1}),
    ("tanh", 64, 4, 8, 0.4, "fixed", {"grid": 1}),
    ("relu", 640, 4, 10, 0.3, "fixed", {"sync": "barrier"}),
    ("relu", 2000, 4, 6, 0.01, "poisson", {"compact": 1}),
    ("tanh", 1152, 4, 32, 0.1, "fixed", {}),
    ("tanh", 640, 4, 12, 0.2, "fixed", {"xcd": "one"}),
    ("tanh", 1000, 2, 6, 0.4, "fixed", {"overlap": 2, "waves": 2, "lanes_per_row": 32}),   # (a forward-only option: the backward kernels read the same words in one go)
])
def test_backward_matches_oracle(cell, H, B, T, dens, rownnz, opts):
    w = wl.make_workload("bwd", cell, H, B, T, dens, seed=H + T, row_nnz=rownnz, h0_std=0.5)
    e = np.random.default_rng(H).standard_normal((T, B, H)).astype(np.float32)
    run_case(w, e, **opts)


def test_backward_relu_mask_and_zero_weights_bit_exact():
    # zero weights: delta_t = [h_t > 0] e_t exactly, dL/dh_0 = 0
    H, B, T = 300, 4, 5
    rng = np.random.default_rng(1)
    hf = rng.standard_normal((T, B, H)).astype(np.float32)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    with binding.SparseRNN(H, B, "relu", np.zeros(H + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16)) as rnn:
        d, dh0 = rnn.backward(_dev(e), _dev(hf))
        assert rnn.check() == binding.SPRNN_OK
        assert np.array_equal(d.cpu().numpy(), np.where(hf > 0, e, np.float32(0)))
        assert not dh0.cpu().numpy().any()


def test_backward_at_the_headline_shape():
    w = wl.make_config("cfg3", steps=64)
    e = np.random.default_rng(3).standard_normal((w.steps, w.batch, w.hidden)).astype(np.float32)
    run_case(w, e)
    # and the gradient of its 1.6 M weights
    h_fwd = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    delta, _, want = oracle.rnn_backward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, poll_delay=-1) as rnn:
        got = rnn.weight_gradient(_dev(delta.astype(np.float32)), _dev(h_fwd), _dev(w.h0)).cpu().numpy()
    assert_weight_gradient(got, want, w.row_ptr, "headline shape")


def test_backward_through_a_permutation_at_the_largest_hidden_size_is_bit_exact():
    # H = 65535 (the last size a 16-bit column index reaches), one sample, column compaction.  With U a permutation matrix
    # of ones, delta_t = [h_t > 0] (e_t + P^T delta_{t+1}): one exact addition per element, so binary32 numpy gives the
    # very bits the kernel must produce.
    H, B, T = 65535, 1, 4
    rng = np.random.default_rng(65535)
    perm = rng.permutation(H).astype(np.int32)                   # forward: row i reads column perm[i]
    row_ptr = np.arange(H + 1, dtype=np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    hf = rng.standard_normal((T, B, H)).astype(np.float32)       # only its sign matters here
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    t_rp, t_ci, t_vb = binding.transpose_csr(H, H, row_ptr, perm, ones)
    inv = np.empty(H, dtype=np.int64)
    inv[perm] = np.arange(H)                                      # transposed row j reads column inv[j]
    assert np.array_equal(t_ci[:H], inv)
    with binding.SparseRNN(H, B, "relu", t_rp, t_ci, t_vb) as rnn:
        info = rnn.info()
        print("case relu backward permutation", {k: info[k] for k in ("grid", "block", "compact", "lds_bytes")}, flush=True)
        assert info["compact"] == 1
        d, dh0 = rnn.backward(_dev(e), _dev(hf))
        assert rnn.check() == binding.SPRNN_OK
        d, dh0 = d.cpu().numpy(), dh0.cpu().numpy()
    back = np.zeros((B, H), dtype=np.float32)
    for t in range(T - 1, -1, -1):
        want = np.where(hf[t] > 0, e[t] + back, np.float32(0))
        assert np.array_equal((d[t] + np.float32(0)).view(np.uint32), (want + np.float32(0)).view(np.uint32)), t
        back = want[:, inv] + np.float32(0)
    assert np.array_equal(dh0.view(np.uint32), back.view(np.uint32))


def test_backward_is_refused_for_gated_cells_and_bad_arguments():
    w = wl.make_config("cfg5", steps=2)
    with binding.SparseRNN(w.hidden, w.batch, "lstm", w.row_ptr, w.col_idx, w.val_bits, poll_delay=-1) as rnn:
        z = torch.zeros((2, w.batch, w.hidden), device="cuda")
        with pytest.raises(binding.SprnnError):
            rnn.backward(z, z)


# ------------------------------------------------------------------ gradient of the recurrent weights
@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts", [
    ("relu", 96, 4, 9, 0.3, "fixed", {}),
    ("tanh", 257, 1, 7, 0.2, "poisson", {}),
    ("identity", 130, 8, 5, 0.1, "poisson", {}),
    ("relu", 333, 2, 6, 0.15, "poisson", {"balance": 1}),
    ("tanh", 64, 4, 8, 0.4, "fixed", {"grid": 1}),
    ("relu", 640, 4, 10, 0.5, "fixed", {"lanes_per_row": 8}),
    ("tanh", 1152, 4, 32, 0.1, "fixed", {}),
])
def test_weight_gradient_matches_oracle(cell, H, B, T, dens, rownnz, opts):
    w = wl.make_workload("wg", cell, H, B, T, dens, seed=H + T, row_nnz=rownnz, h0_std=0.5)
    e = np.random.default_rng(H).standard_normal((T, B, H)).astype(np.float32)
    h_fwd = oracle.rnn_forward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    delta, _, want = oracle.rnn_backward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    delta32 = delta.astype(np.float32)
    # cross-check that rounding delta to binary32 for the call does not matter at this bar
    hp = np.concatenate([w.h0[None].astype(np.float64), h_fwd[:-1].astype(np.float64)])
    rows = np.repeat(np.arange(H), np.diff(w.row_ptr))
    want32 = np.einsum("tbk,tbk->k", delta32.astype(np.float64)[:, :, rows], hp[:, :, w.col_idx])
    assert np.abs(want32 - want).max() <= 1e-5 * np.abs(want).max()
    with binding.SparseRNN(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, poll_delay=-1, **opts) as rnn:
        got = rnn.weight_gradient(_dev(delta32), _dev(h_fwd), _dev(w.h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    assert_weight_gradient(got, want, w.row_ptr, "weight gradient")


def test_weight_gradient_closed_forms_bit_exact():
    # one timestep, small integers: every product and sum is exact, each nonzero gets exactly its own pair
    H, B = 200, 4
    rng = np.random.default_rng(8)
    w = wl.make_workload("wg", "identity", H, B, 1, 0.1, seed=1, row_nnz="poisson")
    delta = rng.integers(-4, 5, size=(1, B, H)).astype(np.float32)
    h0 = rng.integers(-4, 5, size=(B, H)).astype(np.float32)
    hf = np.zeros((1, B, H), dtype=np.float32)
    rows = np.repeat(np.arange(H), np.diff(w.row_ptr))
    want = (delta[0][:, rows] * h0[:, w.col_idx]).sum(axis=0)
    with binding.SparseRNN(H, B, "identity", w.row_ptr, w.col_idx, w.val_bits, poll_delay=-1) as rnn:
        got = rnn.weight_gradient(_dev(delta), _dev(hf), _dev(h0)).cpu().numpy()
        assert np.array_equal(got, want)
        # without h0 the first step contributes nothing
        assert not rnn.weight_gradient(_dev(delta), _dev(hf), None).cpu().numpy().any()


def test_weight_gradient_is_refused_where_the_forward_mapping_cannot_serve():
    w = wl.make_workload("wg", "relu", 2000, 4, 2, 0.01, seed=2, row_nnz="poisson")
    z = torch.zeros((2, 4, 2000), device="cuda")
    with binding.SparseRNN(2000, 4, "relu", w.row_ptr, w.col_idx, w.val_bits, poll_delay=-1, compact=1) as rnn:
        with pytest.raises(binding.SprnnError):
            rnn.weight_gradient(z, z)


# ------------------------------------------------------------------ backward pass with the weight gradient fused in
@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts", [
    ("relu", 96, 4, 9, 0.3, "fixed", {}),
    ("tanh", 257, 1, 7, 0.2, "poisson", {}),
    ("identity", 130, 8, 5, 0.1, "poisson", {}),
    ("relu", 333, 2, 6, 0.15, "poisson", {"balance": 1}),
    ("tanh", 64, 4, 8, 0.4, "fixed", {"grid": 1}),
    ("relu", 640, 4, 10, 0.3, "fixed", {"sync": "barrier"}),
    ("relu", 640, 4, 10, 0.5, "fixed", {"lanes_per_row": 8}),      # 40 words per lane: the 512-thread instantiation
    ("tanh", 1152, 4, 32, 0.1, "fixed", {}),
])
def test_backward_with_weights_matches_oracle(cell, H, B, T, dens, rownnz, opts):
    w = wl.make_workload("bw", cell, H, B, T, dens, seed=H + T, row_nnz=rownnz, h0_std=0.5)
    e = np.random.default_rng(H).standard_normal((T, B, H)).astype(np.float32)
    h_fwd = oracle.rnn_forward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    want_d, want_dh0, want_dU = oracle.rnn_backward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(H, H, w.row_ptr, w.col_idx, w.val_bits, with_source=True)
    with binding.SparseRNN(H, B, cell, t_rp, t_ci, t_vb, **opts) as rnn:
        info = rnn.info()
        print("case", cell, H, B, T, opts, {k: info[k] for k in ("grid", "block", "lanes_per_row", "template_words")}, flush=True)
        try:
            d, dh0, dU_t = rnn.backward_with_weights(_dev(e), _dev(h_fwd), _dev(w.h0))
        except binding.SprnnError as err:
            if err.code == binding.SPRNN_ERR_UNSUPPORTED:
                pytest.skip("mapping too wide for the fused instantiation: %s" % err)
            raise
        assert rnn.check() == binding.SPRNN_OK
        d, dh0, dU_t = d.cpu().numpy(), dh0.cpu().numpy(), dU_t.cpu().numpy()
        # the plain backward pass on the same handle gives the same delta, bit for bit
        d2, _ = rnn.backward(_dev(e), _dev(h_fwd))
        assert np.array_equal(d2.cpu().numpy(), d)
    for t in range(T):
        assert np.abs(d[t] - want_d[t]).max() <= REL_TOL * np.abs(want_d[t]).max() + 1e-30, t
    assert np.abs(dh0 - want_dh0).max() <= REL_TOL * np.abs(want_dh0).max() + 1e-30
    dU = np.empty_like(dU_t)
    dU[t_src] = dU_t                       # back to the forward matrix's CSR order
    assert_weight_gradient(dU, want_dU, w.row_ptr, "fused weight gradient")


def test_backward_with_weights_at_the_headline_shape_and_without_h0():
    w = wl.make_config("cfg3", steps=48)
    e = np.random.default_rng(5).standard_normal((w.steps, w.batch, w.hidden)).astype(np.float32)
    h_fwd = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, None, threads=8)
    want_d, want_dh0, want_dU = oracle.rnn_backward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, None)
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(w.hidden, w.hidden, w.row_ptr, w.col_idx, w.val_bits, with_source=True)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, t_rp, t_ci, t_vb) as rnn:
        d, dh0, dU_t = rnn.backward_with_weights(_dev(e), _dev(h_fwd), None, want_dh0=False)
        assert rnn.check() == binding.SPRNN_OK and dh0 is None
        d, dU_t = d.cpu().numpy(), dU_t.cpu().numpy()
    for t in range(w.steps):
        assert np.abs(d[t] - want_d[t]).max() <= REL_TOL * np.abs(want_d[t]).max() + 1e-30, t
    dU = np.empty_like(dU_t)
    dU[t_src] = dU_t
    assert_weight_gradient(dU, want_dU, w.row_ptr, "fused weight gradient, headline shape")


def test_backward_with_random_pauses_in_the_hand_off_is_unchanged():
    w = wl.make_workload("bj", "tanh", 768, 4, 40, 0.1, seed=4, h0_std=0.3)
    rng = np.random.default_rng(6)
    e = rng.standard_normal((w.steps, w.batch, w.hidden)).astype(np.float32)
    hf = rng.standard_normal((w.steps, w.batch, w.hidden)).astype(np.float32) * np.float32(0.5)
    t_rp, t_ci, t_vb = binding.transpose_csr(w.hidden, w.hidden, w.row_ptr, w.col_idx, w.val_bits)
    outs = []
    for jitter in (0, 5, 11):
        with binding.SparseRNN(w.hidden, w.batch, "tanh", t_rp, t_ci, t_vb, jitter=jitter, lanes_per_row=16) as rnn:   # (pinned: the lanes of a row fix the order of its sums)
            d, dh0, dU = rnn.backward_with_weights(_dev(e), _dev(hf), _dev(w.h0))
            assert rnn.check() == binding.SPRNN_OK
            outs.append((d.cpu().numpy(), dh0.cpu().numpy(), dU.cpu().numpy()))
    for a in outs[1:]:
        for x, y in zip(outs[0], a):
            assert np.array_equal(x, y)
