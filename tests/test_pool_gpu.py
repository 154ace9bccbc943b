"""GPU parity of the lane-pool layout (options.layout = "lane_pool": rows take groups of `batch` lanes out of a pool of
gathering wavefronts, separate wavefronts own b', g and the stores) against the CPU oracle, through the C ABI.

Same bar as the default layout: per timestep  max|h_gpu - h_oracle| <= 1e-3 * max|h_oracle|; index handling bit exact.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1804_10223_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

REL_TOL = 1e-3
POOL = {"layout": "lane_pool"}


def _dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _assert_parity(got, want, what):
    assert got.shape == want.shape and np.all(np.isfinite(got)), what
    for t in range(want.shape[0]):
        scale = np.abs(want[t]).max()
        assert np.abs(got[t] - want[t]).max() <= REL_TOL * scale + 1e-30, "%s step %d" % (what, t)


def _forward(w, **options):
    want = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **POOL, **options) as rnn:
        info = rnn.info()
        print("case", w.name, w.cell, "H", w.hidden, "B", w.batch, "T", w.steps, options,
              {k: info[k] for k in ("grid", "block", "gather_waves", "template_words", "words_per_lane_max", "layout")}, flush=True)
        assert info["layout"] == 2
        got = rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy()
        again = rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy()      # the ring's step counter carries over between calls
        assert rnn.check() == binding.SPRNN_OK
    assert np.array_equal(got, again)
    _assert_parity(got, want, w.name)
    return got


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts", [
    ("relu", 96, 4, 12, 0.3, "fixed", {}),
    ("tanh", 200, 2, 9, 0.2, "poisson", {}),
    ("relu", 300, 1, 7, 0.1, "fixed", {}),
    ("identity", 130, 8, 6, 0.25, "poisson", {}),
    ("relu", 1152, 4, 20, 0.1, "fixed", {}),
    ("relu", 1152, 4, 20, 0.1, "fixed", {"sync": "barrier"}),
    ("relu", 640, 4, 10, 0.5, "fixed", {"waves": 7}),              # seven gathering wavefronts, two per SIMD
    ("tanh", 777, 2, 8, 0.3, "poisson", {"grid": 19}),              # ragged rows, odd grid, rows straddle wavefronts
    ("relu", 512, 4, 9, 0.2, "fixed", {"bank_aware": 2}),           # CSR order inside the lanes
    ("relu", 2304, 4, 16, 0.3, "fixed", {}),                        # headline shape: 25 words per lane in 28 slots
    ("relu", 5760, 2, 8, 0.1, "poisson", {}),                       # the large ragged layer: 59 words per lane
])
def test_forward_matches_oracle(cell, H, B, T, dens, rownnz, opts):
    w = wl.make_workload("pool", cell, H, B, T, dens, seed=H + B + T, row_nnz=rownnz, h0_std=0.2)
    _forward(w, **opts)


def test_permutation_matrix_is_bit_exact():
    # one nonzero of value 1.0 per row: h_t[i] = h_{t-1}[perm[i]] exactly (identity activation), empty groups included
    H, B, T = 1500, 4, 6
    rng = np.random.default_rng(9)
    perm = rng.permutation(H).astype(np.int32)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    with binding.SparseRNN(H, B, "identity", np.arange(H + 1, dtype=np.int32), perm, np.full(H, 0x3C00, np.uint16), **POOL) as rnn:
        print("case permutation", rnn.info()["grid"], flush=True)
        got = rnn.forward(torch.zeros((T, B, H), device="cuda"), _dev(h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    want = h0
    for t in range(T):
        want = want[:, perm] + np.float32(0.0)
        assert np.array_equal(got[t].view(np.uint32), want.view(np.uint32)), t


def test_empty_rows_and_zero_matrix():
    H, B, T = 400, 4, 5
    w = wl.make_workload("holes", "relu", H, B, T, 0.2, seed=3, row_nnz="poisson")
    # knock out every third row completely
    keep = np.ones(w.nnz, dtype=bool)
    for r in range(0, H, 3):
        keep[w.row_ptr[r]:w.row_ptr[r + 1]] = False
    counts = np.diff(w.row_ptr)
    counts[0::3] = 0
    w.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    w.col_idx, w.val_bits = w.col_idx[keep], w.val_bits[keep]
    _forward(w)
    zero = wl.make_workload("zero", "relu", H, B, T, 0.2, seed=4)
    zero.row_ptr = np.zeros(H + 1, np.int32); zero.col_idx = zero.col_idx[:0]; zero.val_bits = zero.val_bits[:0]
    got = _forward(zero, grid=8)
    assert np.array_equal(got, np.maximum(zero.x, 0) + np.float32(0))


def test_random_pauses_in_the_hand_off_change_nothing():
    w = wl.make_workload("jit", "tanh", 768, 4, 40, 0.1, seed=4, h0_std=0.3)
    outs = []
    for jitter in (0, 5, 11):
        with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, jitter=jitter, **POOL) as rnn:
            print("case jitter", jitter, flush=True)
            outs.append(rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy())
            assert rnn.check() == binding.SPRNN_OK
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz", [
    ("relu", 96, 4, 9, 0.3, "fixed"),
    ("tanh", 257, 1, 7, 0.2, "poisson"),
    ("identity", 130, 8, 5, 0.1, "poisson"),
    ("tanh", 1152, 4, 24, 0.1, "fixed"),
])
def test_backward_and_fused_weight_gradient_match_oracle(cell, H, B, T, dens, rownnz):
    w = wl.make_workload("pool-bwd", cell, H, B, T, dens, seed=H + T, row_nnz=rownnz, h0_std=0.5)
    e = np.random.default_rng(H).standard_normal((T, B, H)).astype(np.float32)
    h_fwd = oracle.rnn_forward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    want_d, want_dh0, want_dU = oracle.rnn_backward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, h_fwd, e, w.h0)
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(H, H, w.row_ptr, w.col_idx, w.val_bits, with_source=True)
    with binding.SparseRNN(H, B, cell, t_rp, t_ci, t_vb, **POOL) as rnn:
        info = rnn.info()
        print("case backward", cell, H, B, T, {k: info[k] for k in ("grid", "block", "template_words")}, flush=True)
        d, dh0 = rnn.backward(_dev(e), _dev(h_fwd))
        d2, dh02, dU_t = rnn.backward_with_weights(_dev(e), _dev(h_fwd), _dev(w.h0))
        assert rnn.check() == binding.SPRNN_OK
        d, dh0, d2, dh02, dU_t = (a.cpu().numpy() for a in (d, dh0, d2, dh02, dU_t))
    assert np.array_equal(d, d2) and np.array_equal(dh0, dh02)
    _assert_parity(d, want_d.astype(np.float32), "delta")
    assert np.abs(dh0 - want_dh0).max() <= REL_TOL * np.abs(want_dh0).max() + 1e-30
    dU = np.empty_like(dU_t)
    dU[t_src] = dU_t
    assert np.abs(dU - want_dU).max() <= REL_TOL * np.abs(want_dU).max()


def test_layout_is_refused_where_it_does_not_apply():
    l = wl.make_workload("l", "lstm", 64, 4, 2, 0.2, seed=0)
    with pytest.raises(binding.SprnnError) as e:
        binding.SparseRNN(l.hidden, l.batch, "lstm", l.row_ptr, l.col_idx, l.val_bits, **POOL)
    assert e.value.code == binding.SPRNN_ERR_UNSUPPORTED
    # one nonzero per row in a very long layer: the rows of a workgroup outnumber the lanes that could own their outputs
    H = 30000
    with pytest.raises(binding.SprnnError) as e:
        binding.SparseRNN(H, 4, "relu", np.arange(H + 1, dtype=np.int32), np.arange(H, dtype=np.int32), np.full(H, 0x3C00, np.uint16), **POOL)
    assert e.value.code == binding.SPRNN_ERR_CAPACITY
