"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: per timestep  max|h_gpu - h_oracle| <= 1e-3 * max|h_oracle|  (same for c_t of the LSTM); index and
sparsity-pattern handling bit exact (permutation matrices, zero weights).
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


def oracle_run(w, threads=8):
    if w.cell == "lstm":
        return oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, w.c0, threads=threads)
    if w.cell == "gru":
        return oracle.gru_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x, w.b_hn, w.h0, threads=threads), None
    return oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=threads), None


def gpu_run(rnn, w, stepwise=False):
    x, h0, c0 = _dev(w.x), _dev(w.h0), _dev(w.c0)
    if stepwise:
        h, c = rnn.forward_stepwise(x, h0, c0)
    elif w.cell == "lstm":
        h, c = rnn.forward_lstm(x, h0, c0)
    elif w.cell == "gru":
        h, c = rnn.forward_gru(x, _dev(w.b_hn), h0), None
    else:
        h, c = rnn.forward(x, h0), None
    assert rnn.check() == binding.SPRNN_OK
    return h.cpu().numpy(), (None if c is None else c.cpu().numpy())


def assert_parity(got, want, what=""):
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), what
    for t in range(want.shape[0]):
        scale = np.abs(want[t]).max()
        err = np.abs(got[t] - want[t]).max()
        assert err <= REL_TOL * scale + 1e-30, "%s step %d: err %.3e scale %.3e" % (what, t, err, scale)


def check_workload(w, stepwise_too=True, **options):
    want_h, want_c = oracle_run(w)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **options) as rnn:
        info = rnn.info()
        print("case", w.name, w.cell, "H", w.hidden, "B", w.batch, "T", w.steps, options, {k: info[k] for k in ("grid", "block", "lanes_per_row", "template_words", "sync", "balance")}, flush=True)
        got_h, got_c = gpu_run(rnn, w)
        assert_parity(got_h, want_h, "h persistent")
        if want_c is not None:
            assert_parity(got_c, want_c, "c persistent")
        if stepwise_too and w.cell != "gru":      # the per-timestep comparison path is not offered for the GRU
            s_h, s_c = gpu_run(rnn, w, stepwise=True)
            assert_parity(s_h, want_h, "h stepwise")
            if want_c is not None:
                assert_parity(s_c, want_c, "c stepwise")
    return info


# ------------------------------------------------------------------ small shapes: several tiles, ragged tails
SMALL = [
    ("relu", 96, 4, 9, 0.3, "fixed", {}),
    ("relu", 257, 1, 7, 0.2, "fixed", {}),
    ("relu", 333, 2, 6, 0.15, "poisson", {}),
    ("tanh", 200, 4, 8, 0.25, "fixed", {}),
    ("identity", 130, 8, 5, 0.1, "poisson", {}),
    ("relu", 1000, 4, 12, 0.05, "poisson", {"grid": 13}),
    ("relu", 640, 4, 10, 0.5, "fixed", {"lanes_per_row": 64}),
    ("relu", 640, 4, 10, 0.5, "fixed", {"lanes_per_row": 8}),
    ("relu", 640, 1, 10, 0.1, "fixed", {"lanes_per_row": 1}),
    ("relu", 640, 2, 10, 0.1, "fixed", {"lanes_per_row": 2}),
    ("identity", 300, 8, 6, 0.2, "fixed", {"lanes_per_row": 8}),
    ("relu", 300, 8, 6, 0.5, "poisson", {"lanes_per_row": 32}),
    ("relu", 500, 4, 10, 0.2, "poisson", {"balance": 1}),
    ("relu", 500, 4, 10, 0.2, "poisson", {"balance": 2}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"bank_aware": 2}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"sync": "barrier"}),
    ("relu", 500, 1, 10, 0.2, "fixed", {"sync": "barrier", "grid": 6}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"poll_delay": -1}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"xcd": "one"}),                                 # every workgroup on one XCD, exchange through its L2
    ("relu", 500, 4, 10, 0.2, "fixed", {"xcd": "one", "sync": "barrier", "grid": 7}),
    ("tanh", 1152, 4, 20, 0.1, "fixed", {"xcd": "one", "grid": 32, "jitter": 3}),
    ("relu", 1000, 2, 12, 0.05, "poisson", {"xcd": "one", "compact": 1, "grid": 13}),
    ("lstm", 100, 4, 7, 0.2, "poisson", {"xcd": "one"}),
    ("lstm", 256, 8, 9, 0.125, "fixed", {"xcd": "one", "poll_delay": 1}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"xcd": "spread"}),
    ("relu", 640, 4, 12, 0.8, "fixed", {"overlap": 2, "waves": 2, "lanes_per_row": 32}),   # copy of h consumed in two parts, early words during the second
    ("tanh", 1000, 2, 9, 0.4, "fixed", {"overlap": 2, "waves": 2, "jitter": 3}),
    ("tanh", 1024, 1, 7, 0.9, "poisson", {"overlap": 2, "waves": 2, "lanes_per_row": 16, "jitter": 5}),
    ("relu", 1200, 4, 40, 0.6, "fixed", {"overlap": 2, "waves": 4, "lanes_per_row": 32, "jitter": 7}),
    ("relu", 1000, 2, 9, 0.4, "poisson", {"overlap": 2, "waves": 2, "lanes_per_row": 32}),
    ("relu", 1152, 4, 20, 0.3, "fixed", {"overlap": 2, "xcd": "one", "grid": 32, "lanes_per_row": 16}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"gather": "narrow"}),                       # one 4-byte LDS read per sample (ablation rung)
    ("tanh", 1152, 4, 12, 0.1, "fixed", {"gather": "narrow", "sync": "barrier", "bank_aware": 2}),   # the ablation's first rung
    ("relu", 500, 4, 10, 0.2, "fixed", {"launch": "cooperative"}),
    ("relu", 500, 4, 10, 0.2, "fixed", {"compact": 1}),
    ("relu", 2000, 4, 8, 0.01, "poisson", {"compact": 1, "grid": 50}),
    ("tanh", 1500, 2, 8, 0.01, "fixed", {"compact": 1, "grid": 40}),
    ("identity", 3000, 1, 8, 0.005, "poisson", {"compact": 1, "grid": 30}),
    ("relu", 1200, 8, 8, 0.02, "fixed", {"compact": 1, "grid": 64}),
    ("relu", 1200, 8, 8, 0.02, "fixed", {"compact": 1, "grid": 64, "sync": "barrier"}),
    ("relu", 2000, 4, 6, 0.02, "fixed", {"compact": 1, "waves": 2}),
    ("relu", 4000, 4, 5, 0.02, "fixed", {"compact": 1, "waves": 2}),
    ("lstm", 600, 8, 7, 0.02, "fixed", {"compact": 1}),
    ("lstm", 700, 2, 7, 0.01, "poisson", {"compact": 1, "grid": 20}),
    ("lstm", 64, 8, 9, 0.3, "fixed", {}),
    ("lstm", 40, 2, 9, 0.3, "fixed", {"grid": 1, "sync": "barrier"}),
    ("tanh", 88, 4, 9, 0.3, "poisson", {"grid": 1}),
    ("relu", 192, 4, 9, 0.2, "poisson", {"grid": 2}),
    ("lstm", 100, 4, 7, 0.2, "poisson", {}),
    ("lstm", 77, 1, 6, 0.4, "fixed", {"lanes_per_row": 4}),
    ("lstm", 150, 2, 6, 0.3, "fixed", {"lanes_per_row": 16, "sync": "barrier"}),
]


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts", SMALL)
def test_small_shapes_match_oracle(cell, H, B, T, dens, rownnz, opts):
    w = wl.make_workload("small", cell, H, B, T, dens, seed=H + B + T, row_nnz=rownnz, h0_std=0.5,
                         gain=1.0 if cell == "lstm" else 0.9)
    if cell == "lstm":
        w.c0 = (np.random.default_rng(1).standard_normal((B, H)) * 0.5).astype(np.float32)
    check_workload(w, **opts)


def test_very_large_sparse_layer_fits_through_column_compaction():
    # hidden 11520 at batch 4 (the largest layer of Section 5.3): h is 184 KB, more than a CU's LDS; every
    # workgroup copies only the columns its rows read
    w = wl.make_workload("huge", "relu", 11520, 4, 5, 0.01, seed=14, h0_std=0.5)
    info = check_workload(w, stepwise_too=False)
    assert info["compact"] == 1 and info["lds_bytes"] < 11520 * 16
    with pytest.raises(binding.SprnnError) as e:
        binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, compact=2)
    assert e.value.code == binding.SPRNN_ERR_CAPACITY


@pytest.mark.parametrize("H,B", [(4099, 2), (20000, 1), (9000, 4), (65535, 1), (65535, 2)])   # 65535: the largest hidden size a 16-bit column index reaches
def test_permutation_matrix_bit_exact_with_column_compaction(H, B):
    rng = np.random.default_rng(H)
    perm = rng.permutation(H).astype(np.int32)
    row_ptr = np.arange(H + 1, dtype=np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    T = 4
    x = np.zeros((T, B, H), dtype=np.float32)
    h0 = np.abs(rng.standard_normal((B, H))).astype(np.float32) + np.float32(0.01)
    with binding.SparseRNN(H, B, "relu", row_ptr, perm, ones, compact=1) as rnn:
        assert rnn.info()["compact"] == 1
        h = rnn.forward(_dev(x), _dev(h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    cur = h0
    for t in range(T):
        cur = cur[:, perm]
        assert np.array_equal(h[t].view(np.uint32), cur.view(np.uint32)), t


def test_large_layer_whose_columns_need_scaled_indices():
    # h of 4608 x 4 samples is 72 KB: byte offsets of columns no longer fit 16 bits, the packed index counts columns
    w = wl.make_workload("big", "relu", 4608, 4, 6, 0.02, seed=11, h0_std=0.5)
    info = check_workload(w, stepwise_too=False)
    assert info["lds_bytes"] == 4608 * 16


# ------------------------------------------------------------------ degenerate cases
def test_zero_steps_and_single_step():
    w = wl.make_workload("t1", "relu", 128, 4, 1, 0.2, seed=1, h0_std=0.3)
    check_workload(w)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        empty = torch.empty((0, 4, 128), dtype=torch.float32, device="cuda")
        out = rnn.forward(empty, None)
        assert out.shape == (0, 4, 128) and rnn.check() == binding.SPRNN_OK


@pytest.mark.parametrize("cell", ["relu", "identity"])
def test_zero_weights_bit_exact(cell):
    H, B, T = 300, 4, 5
    rng = np.random.default_rng(0)
    x = rng.standard_normal((T, B, H)).astype(np.float32)
    row_ptr = np.zeros(H + 1, dtype=np.int32)
    with binding.SparseRNN(H, B, cell, row_ptr, np.zeros(0, np.int32), np.zeros(0, np.uint16)) as rnn:
        h = rnn.forward(_dev(x), None).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    want = np.maximum(x, np.float32(0)) if cell == "relu" else x
    assert np.array_equal(h, want + np.float32(0))       # +0: a -0.0 result is written as +0.0


def test_workgroups_that_read_nothing_of_each_other_stay_in_step():
    # zero weights with column compaction: no workgroup needs any column of h, so only the flow-control entries of
    # the copy lists keep the workgroups within one step of each other (without them a fast workgroup would
    # overwrite ring slots that a slow one has not read); pauses widen the window, many steps give it room
    H, B, T = 3000, 2, 400
    rng = np.random.default_rng(5)
    x = rng.standard_normal((T, B, H)).astype(np.float32)
    row_ptr = np.zeros(H + 1, dtype=np.int32)
    for seed in (0, 7):
        with binding.SparseRNN(H, B, "relu", row_ptr, np.zeros(0, np.int32), np.zeros(0, np.uint16), compact=1, jitter=seed, grid=60) as rnn:
            assert rnn.info()["compact"] == 1
            h = rnn.forward(_dev(x), None).cpu().numpy()
            assert rnn.check() == binding.SPRNN_OK
        assert np.array_equal(h, np.maximum(x, np.float32(0)) + np.float32(0))
    # block-diagonal weights: every workgroup reads only its own rows' columns
    w = wl.make_workload("blk", "relu", 1920, 4, 300, 0.02, seed=15, h0_std=0.4)
    keep = (w.col_idx // 64) == (np.repeat(np.arange(1920), np.diff(w.row_ptr)) // 64)
    counts = np.add.reduceat(keep.astype(np.int64), w.row_ptr[:-1])
    w.col_idx, w.val_bits = w.col_idx[keep], w.val_bits[keep]
    w.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    want, _ = oracle_run(w)
    for seed in (0, 3):
        with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, compact=1, jitter=seed, grid=30) as rnn:
            got, _ = gpu_run(rnn, w)
        assert_parity(got, want, "block diagonal, jitter %d" % seed)


def test_empty_rows_and_stored_zeros():
    H, B, T = 90, 2, 6
    w = wl.make_workload("e", "relu", H, B, T, 0.2, seed=2, h0_std=0.5)
    # empty every third row, and store explicit zeros in some places
    keep = np.ones(w.nnz, dtype=bool)
    for r in range(0, H, 3):
        keep[w.row_ptr[r]:w.row_ptr[r + 1]] = False
    counts = np.array([keep[w.row_ptr[r]:w.row_ptr[r + 1]].sum() for r in range(H)])
    w.col_idx, w.val_bits = w.col_idx[keep], w.val_bits[keep].copy()
    w.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    w.val_bits[::7] = 0
    w.val_bits[3::11] = 0x8000
    check_workload(w)


@pytest.mark.parametrize("H,B", [(7, 4), (4099, 2), (16384, 1), (4100, 4), (9000, 2), (20000, 1), (5000, 8), (65535, 1)])
def test_permutation_matrix_bit_exact(H, B):
    rng = np.random.default_rng(H)
    perm = rng.permutation(H).astype(np.int32)
    row_ptr = np.arange(H + 1, dtype=np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    T = 4
    x = np.zeros((T, B, H), dtype=np.float32)
    h0 = np.abs(rng.standard_normal((B, H))).astype(np.float32) + np.float32(0.01)
    with binding.SparseRNN(H, B, "relu", row_ptr, perm, ones) as rnn:
        h = rnn.forward(_dev(x), _dev(h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
        s, _ = rnn.forward_stepwise(_dev(x), _dev(h0))
        s = s.cpu().numpy()
    cur = h0
    for t in range(T):
        cur = cur[:, perm]
        assert np.array_equal(h[t].view(np.uint32), cur.view(np.uint32)), t
        assert np.array_equal(s[t].view(np.uint32), cur.view(np.uint32)), t


def test_subnormal_and_extreme_fp16_weights_are_not_flushed():
    H, B, T = 64, 4, 3
    rng = np.random.default_rng(3)
    w = wl.make_workload("sub", "identity", H, B, T, 0.5, seed=3)
    bits = w.val_bits.copy()
    bits[0::3] = rng.integers(1, 0x3FF, size=bits[0::3].shape).astype(np.uint16)            # positive subnormals
    bits[1::3] = (0x8000 | rng.integers(1, 0x3FF, size=bits[1::3].shape)).astype(np.uint16)  # negative subnormals
    w.val_bits = bits
    w.x = np.zeros_like(w.x)
    w.h0 = (rng.standard_normal((B, H)) * 1e4).astype(np.float32)
    want, _ = oracle_run(w)
    assert np.abs(want[0]).max() > 0
    with binding.SparseRNN(H, B, "identity", w.row_ptr, w.col_idx, w.val_bits) as rnn:
        got, _ = gpu_run(rnn, w)
    assert_parity(got, want, "subnormal")


# ------------------------------------------------------------------ handle reuse: the ring keeps its timestep numbering
def test_consecutive_forwards_and_time_composition():
    w = wl.make_workload("c", "relu", 400, 4, 11, 0.2, seed=4, h0_std=0.5)
    want, _ = oracle_run(w)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x, h0 = _dev(w.x), _dev(w.h0)
        for rep in range(3):                      # 11 steps each: the ring slot phase differs every time
            h = rnn.forward(x, h0)
            assert rnn.check() == binding.SPRNN_OK
            assert_parity(h.cpu().numpy(), want, "rep %d" % rep)
        a = rnn.forward(x[:5].contiguous(), h0)
        b = rnn.forward(x[5:].contiguous(), a[-1].contiguous())
        assert rnn.check() == binding.SPRNN_OK
        both = torch.cat([a, b]).cpu().numpy()
        assert_parity(both, want, "split 5+6")
        # run-to-run determinism of the persistent path
        h1 = rnn.forward(x, h0).cpu().numpy()
        h2 = rnn.forward(x, h0).cpu().numpy()
        assert np.array_equal(h1, h2)


@pytest.mark.parametrize("cell,H,B,opts", [
    ("relu", 1152, 4, {}),
    ("relu", 3000, 4, {"compact": 1, "grid": 150}),
    ("lstm", 800, 4, {"compact": 1}),
    ("relu", 1152, 4, {"sync": "barrier"}),
    ("relu", 2000, 2, {"grid": 250, "poll_delay": 2}),
    ("lstm", 512, 8, {}),
    ("tanh", 96, 4, {"grid": 1}),
])
def test_random_pauses_in_the_hand_off_do_not_change_results(cell, H, B, opts):
    # every wavefront pauses pseudo-randomly before publishing, before polling and after copying h, differently in
    # every step: any race in the hand-off (ring re-arm, single LDS copy, barrier placement) would show as a mismatch
    T = 160
    w = wl.make_workload("jit", cell, H, B, T, 0.1, seed=12, gain=1.0 if cell == "lstm" else 0.9, h0_std=0.3)
    want_h, want_c = oracle_run(w)
    ref = None
    # (the lanes of a row fix the order of its sums; with nothing pinned the library may measure its way to another count
    # from one handle to the next, so the count the first handle arrived at is asked for in the others)
    pinned = dict(opts)
    for seed in (0, 1, 2, 3):
        with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, jitter=seed, **pinned) as rnn:
            pinned.setdefault("lanes_per_row", rnn.info()["lanes_per_row"])
            got_h, got_c = gpu_run(rnn, w)
        assert_parity(got_h, want_h, "jitter %d" % seed)
        if want_c is not None:
            assert_parity(got_c, want_c, "jitter %d (c)" % seed)
        if ref is None:
            ref = got_h
        else:
            assert np.array_equal(ref, got_h), "jitter seed %d changed the result" % seed


def test_long_sequence_is_deterministic_and_matches_in_pieces():
    w = wl.make_workload("long", "relu", 1024, 4, 3000, 0.1, seed=13)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x = _dev(w.x)
        a = rnn.forward(x, None).cpu().numpy()
        b = rnn.forward(x, None).cpu().numpy()
        p1 = rnn.forward(x[:1234].contiguous(), None)
        p2 = rnn.forward(x[1234:].contiguous(), p1[-1].contiguous())
        assert rnn.check() == binding.SPRNN_OK
    assert np.array_equal(a, b)
    assert np.array_equal(a, torch.cat([p1, p2]).cpu().numpy())
    want = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, np.ascontiguousarray(w.x[:64]), None, threads=8)
    assert_parity(a[:64], want, "first 64 steps")


def test_two_handles_interleaved_on_one_stream():
    w1 = wl.make_workload("a", "relu", 256, 4, 8, 0.2, seed=5)
    w2 = wl.make_workload("b", "lstm", 96, 2, 8, 0.3, seed=6, gain=1.0)
    want1, _ = oracle_run(w1)
    want2h, want2c = oracle_run(w2)
    with binding.SparseRNN(w1.hidden, w1.batch, w1.cell, w1.row_ptr, w1.col_idx, w1.val_bits) as r1, \
            binding.SparseRNN(w2.hidden, w2.batch, w2.cell, w2.row_ptr, w2.col_idx, w2.val_bits) as r2:
        h1 = r1.forward(_dev(w1.x), None)
        h2, c2 = r2.forward_lstm(_dev(w2.x), None, None)
        h1b = r1.forward(_dev(w1.x), None)
        assert r1.check() == binding.SPRNN_OK and r2.check() == binding.SPRNN_OK
        assert_parity(h1.cpu().numpy(), want1)
        assert_parity(h1b.cpu().numpy(), want1)
        assert_parity(h2.cpu().numpy(), want2h)
        assert_parity(c2.cpu().numpy(), want2c)


def test_side_stream():
    w = wl.make_workload("s", "relu", 300, 2, 9, 0.2, seed=7)
    want, _ = oracle_run(w)
    st = torch.cuda.Stream()
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x = _dev(w.x)
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            h = rnn.forward(x, None)
        st.synchronize()
        assert rnn.check() == binding.SPRNN_OK
        assert_parity(h.cpu().numpy(), want)


def test_a_large_h_gets_the_wavefront_count_with_fewer_surplus_loads():
    # 3072 x batch 4: h is 3072 pieces of 16 bytes.  Eight wavefronts copy it in six rounds and issue eight; twelve copy
    # it in four exactly.  With nothing asked for, both mappings are measured; whichever is kept gives the oracle's
    # result, and a caller who fixes the count gets that count.
    w = wl.make_workload("w", "relu", 3072, 4, 6, 0.1, seed=31, h0_std=0.3)
    want, _ = oracle_run(w)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, fill_waves=8) as rnn:
        assert rnn.info()["block"] == 512
        got, _ = gpu_run(rnn, w)
        assert_parity(got, want)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        info = rnn.info()
        print("case kept", info["grid"], "x", info["block"], flush=True)
        assert info["block"] % 64 == 0 and info["block"] <= 768, info
        got, _ = gpu_run(rnn, w)
        assert_parity(got, want)


def test_two_full_size_handles_on_two_streams_take_turns():
    # Each of the two layers needs every compute unit, and their workgroups spin on each other: started side by side
    # they would wait for each other's compute units until the watchdog ends both.  The library orders its persistent
    # launches on a device, whatever streams they go to, so alternating launches on two streams without any host
    # synchronisation in between must give the same results as one after the other.
    wa = wl.make_workload("a", "relu", 2304, 4, 24, 0.3, seed=21, h0_std=0.3)
    wb = wl.make_workload("b", "tanh", 2048, 4, 24, 0.3, seed=22, h0_std=0.3)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    with binding.SparseRNN(wa.hidden, wa.batch, wa.cell, wa.row_ptr, wa.col_idx, wa.val_bits, lanes_per_row=64) as ra, \
            binding.SparseRNN(wb.hidden, wb.batch, wb.cell, wb.row_ptr, wb.col_idx, wb.val_bits, lanes_per_row=64) as rb:
        print("case grids", ra.info()["grid"], rb.info()["grid"], flush=True)
        assert ra.info()["grid"] + rb.info()["grid"] > 256
        xa, ha, xb, hb = _dev(wa.x), _dev(wa.h0), _dev(wb.x), _dev(wb.h0)
        want_a = ra.forward(xa, ha).cpu().numpy()
        want_b = rb.forward(xb, hb).cpu().numpy()
        outs = []
        torch.cuda.synchronize()
        for i in range(6):
            with torch.cuda.stream(s1):
                oa = ra.forward(xa, ha)
            with torch.cuda.stream(s2):
                ob = rb.forward(xb, hb)
            outs.append((oa, ob))
        torch.cuda.synchronize()
        assert ra.check() == binding.SPRNN_OK and rb.check() == binding.SPRNN_OK
        for oa, ob in outs:
            assert np.array_equal(oa.cpu().numpy(), want_a) and np.array_equal(ob.cpu().numpy(), want_b)
    want, _ = oracle_run(wa)
    assert_parity(want_a, want)


def test_a_full_size_layer_beside_other_work_on_another_stream():
    # Ordinary kernels on another stream may hold compute units when the persistent kernel starts: its workgroups that
    # are already resident wait (bounded) for the others, which get their compute units as the other work drains.
    # The result must be the same as on an idle device.
    w = wl.make_workload("busy", "relu", 2304, 4, 32, 0.3, seed=41, h0_std=0.3)
    side, main = torch.cuda.Stream(), torch.cuda.Stream()
    a = torch.randn((4096, 4096), device="cuda")
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, lanes_per_row=64) as rnn:
        assert rnn.info()["grid"] == 256
        x, h0 = _dev(w.x), _dev(w.h0)
        want = rnn.forward(x, h0).cpu().numpy()
        torch.cuda.synchronize()
        outs = []
        for i in range(4):
            with torch.cuda.stream(side):
                b = a
                for _ in range(6):
                    b = torch.mm(b, a) * 1e-3     # a few milliseconds of work that fills the device
            with torch.cuda.stream(main):
                outs.append(rnn.forward(x, h0))
        torch.cuda.synchronize()
        assert rnn.check() == binding.SPRNN_OK
        for o in outs:
            assert np.array_equal(o.cpu().numpy(), want)
    assert_parity(want, oracle_run(w)[0])


def test_two_host_threads_with_a_handle_each():
    # different handles from different host threads at the same time, each thread on a stream of its own: the
    # library's per-device launch order is the only state they share
    import threading
    ws = [wl.make_workload("t%d" % i, "relu", 2048, 4, 16, 0.2, seed=50 + i, h0_std=0.3) for i in range(2)]
    rnns = [binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) for w in ws]
    try:
        ins = [(_dev(w.x), _dev(w.h0)) for w in ws]
        wants = [r.forward(x, h0).cpu().numpy() for r, (x, h0) in zip(rnns, ins)]
        torch.cuda.synchronize()
        results, errors = [[], []], []

        def work(i):
            try:
                st = torch.cuda.Stream()
                with torch.cuda.stream(st):
                    for _ in range(25):
                        results[i].append(rnns[i].forward(*ins[i]))
                st.synchronize()
            except Exception as e:  # noqa: BLE001  (reported by the asserting thread)
                errors.append(e)

        threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        assert not errors, errors
        torch.cuda.synchronize()
        for i in range(2):
            assert rnns[i].check() == binding.SPRNN_OK
            assert len(results[i]) == 25
            for o in results[i]:
                assert np.array_equal(o.cpu().numpy(), wants[i])
            assert_parity(wants[i], oracle_run(ws[i])[0])
    finally:
        for r in rnns:
            r.close()


# ------------------------------------------------------------------ error paths that need a device
def test_one_xcd_mode_repeated_calls_and_refusal():
    # many launches on one handle (the placement counters alternate between two sets and are cleared by the launch in
    # between), results identical to the spread mapping's bit for bit; refused where 8 x grid workgroups cannot be resident
    w = wl.make_workload("x", "relu", 768, 4, 10, 0.1, seed=7, h0_std=0.3)
    x, h0 = _dev(w.x), _dev(w.h0)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, xcd="spread") as rnn:
        want = rnn.forward(x, h0).cpu().numpy()
        lanes = rnn.info()["lanes_per_row"]
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, xcd="one") as rnn:
        info = rnn.info()
        print("case one xcd", {k: info[k] for k in ("grid", "block", "one_xcd", "poll_delay")}, flush=True)
        assert info["one_xcd"] == 1
        for i in range(7):
            assert np.array_equal(rnn.forward(x, h0).cpu().numpy(), want), i
        out = torch.empty_like(x)
        rnn.forward_noalloc(x, h0, out)
        assert np.array_equal(out.cpu().numpy(), want)
        assert rnn.check() == binding.SPRNN_OK
    big = wl.make_config("cfg3", steps=2)
    with pytest.raises(binding.SprnnError) as e:
        binding.SparseRNN(big.hidden, big.batch, big.cell, big.row_ptr, big.col_idx, big.val_bits, xcd="one")
    assert e.value.code == binding.SPRNN_ERR_UNSUPPORTED
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:   # auto: measured at create time
        print("case auto", rnn.info()["one_xcd"], rnn.info()["poll_delay"], rnn.info()["lanes_per_row"], flush=True)
        got = rnn.forward(x, h0).cpu().numpy()
        if rnn.info()["lanes_per_row"] == lanes:   # the same lanes per row add up in the same order
            assert np.array_equal(got, want)
        assert_parity(got, oracle_run(w)[0])


@pytest.mark.parametrize("cell,H,B,dens", [("relu", 1152, 4, 0.10), ("tanh", 1280, 2, 0.10), ("lstm", 640, 4, 0.1)])
def test_layers_a_little_larger_than_one_xcd_are_also_tried_as_fewer_larger_workgroups(cell, H, B, dens):
    # With nothing asked for, sprnn_create builds the mapping of its own choice and, where the same rows fit the CUs of
    # one XCD as larger workgroups, that one too, and keeps the faster.  Whichever it keeps must give the oracle's result;
    # a caller who fixes any part of the mapping gets exactly the mapping asked for.
    w = wl.make_workload("f", cell, H, B, 12, dens, seed=11, gain=1.0 if cell == "lstm" else 0.9, h0_std=0.3)
    want, wantc = oracle_run(w)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, xcd="spread") as rnn:
        own = rnn.info()
    assert own["grid"] > 32, own          # (the shapes are chosen so that the library's own mapping exceeds one XCD)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        info = rnn.info()
        print("case", cell, H, B, "own grid", own["grid"], "x", own["block"], "kept", info["grid"], "x", info["block"],
              "one xcd", info["one_xcd"], flush=True)
        assert info["grid"] <= info["resident_capacity"] and (not info["one_xcd"] or info["grid"] <= 32), info
        got, gotc = gpu_run(rnn, w)
        assert_parity(got, want)
        if cell == "lstm":
            assert_parity(gotc, wantc)


def test_narrow_gathers_are_refused_where_not_built():
    w = wl.make_workload("n", "relu", 200, 2, 2, 0.2, seed=0)
    with pytest.raises(binding.SprnnError) as e:
        binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, gather="narrow")
    assert e.value.code == binding.SPRNN_ERR_UNSUPPORTED


def test_wrong_cell_call_and_bad_arguments():
    w = wl.make_workload("s", "relu", 64, 2, 3, 0.2, seed=8)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x = _dev(w.x)
        with pytest.raises(binding.SprnnError) as e:
            rnn.forward_lstm(x, None, None)
        assert e.value.code == binding.SPRNN_ERR_UNSUPPORTED
        with pytest.raises(ValueError):
            rnn.forward(x[:, :1].contiguous())
    with pytest.raises(binding.SprnnError) as e:
        binding.SparseRNN(64, 2, "relu", w.row_ptr, w.col_idx, w.val_bits, device=99)
    assert e.value.code == binding.SPRNN_ERR_INVALID


def test_watchdog_trip_is_reported_and_every_kernel_exits():
    # a spin limit of one poll makes the kernel's own bounded wait give up almost immediately;
    # the kernel must still drain, the trip must be reported, and the handle must refuse further work
    w = wl.make_workload("wd", "relu", 1024, 4, 64, 0.05, seed=9)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, grid=64, spin_limit=1,
                           poll_delay=-1) as rnn:
        rnn.forward(_dev(w.x), None)
        code = rnn.check()
        assert code in (binding.SPRNN_OK, binding.SPRNN_ERR_STATE)
        if code == binding.SPRNN_ERR_STATE:
            with pytest.raises(binding.SprnnError) as e:
                rnn.forward(_dev(w.x), None)
            assert e.value.code == binding.SPRNN_ERR_STATE


# ------------------------------------------------------------------ the five measured configurations, full size
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_full_configs_match_oracle(name):
    w = wl.make_config(name)
    info = check_workload(w, stepwise_too=(name in ("cfg1", "cfg2", "cfg5")))
    assert info["grid"] <= info["resident_capacity"]


def test_two_part_copy_at_the_headline_shape_and_with_random_pauses():
    # options.overlap at full size (cfg3, cfg4), where the second part really is in flight while the early words are
    # worked through; random pauses must not change a bit, and a backward pass on the same handle ignores the option
    for name in ("cfg3", "cfg4"):
        w = wl.make_config(name, steps=48)
        info = check_workload(w, stepwise_too=False, overlap=2)
        assert info["overlap_rounds"] == 2 and info["overlap_words"] >= 4
    w = wl.make_config("cfg3", steps=64)
    outs = []
    for jitter in (0, 5, 11):
        with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, overlap=2, jitter=jitter) as rnn:
            outs.append(rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy())
            assert rnn.check() == binding.SPRNN_OK
            if jitter == 0:
                h = torch.from_numpy(outs[0]).cuda()
                e = torch.ones_like(h)
                d, dh0 = rnn.backward(e, h)        # (the matrix as it is: any square matrix serves as "the transposed one")
                assert rnn.check() == binding.SPRNN_OK and bool(torch.isfinite(d).all()) and bool(torch.isfinite(dh0).all())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ------------------------------------------------------------------ GRU cell
@pytest.mark.parametrize("H,B,T,dens,rownnz,opts", [
    (48, 4, 9, 0.3, "fixed", {}),
    (100, 1, 7, 0.2, "poisson", {}),
    (130, 2, 6, 0.25, "poisson", {"lanes_per_row": 16}),
    (64, 8, 5, 0.5, "fixed", {}),
    (300, 4, 8, 0.1, "poisson", {"balance": 1}),
    (40, 4, 6, 0.4, "fixed", {"grid": 1}),
    (512, 4, 12, 0.1, "fixed", {"sync": "barrier"}),
    (600, 2, 10, 0.02, "poisson", {"compact": 1}),
    (1024, 8, 16, 0.2, "fixed", {}),
])
def test_gru_matches_oracle(H, B, T, dens, rownnz, opts):
    w = wl.make_workload("gru", "gru", H, B, T, dens, seed=H + B, gain=1.0, row_nnz=rownnz, h0_std=0.5)
    check_workload(w, **opts)


def test_gru_time_composition_null_arguments_and_wrong_calls():
    w = wl.make_workload("gru", "gru", 256, 4, 20, 0.2, seed=9, gain=1.0, h0_std=0.3)
    with binding.SparseRNN(w.hidden, w.batch, "gru", w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x, h0, bhn = _dev(w.x), _dev(w.h0), _dev(w.b_hn)
        full = rnn.forward_gru(x, bhn, h0)
        first = rnn.forward_gru(x[:7].contiguous(), bhn, h0)
        rest = rnn.forward_gru(x[7:].contiguous(), bhn, first[-1].contiguous())
        torch.cuda.synchronize()
        assert torch.equal(full, torch.cat([first, rest]))
        # no b_hn, no h0: zeros
        got = rnn.forward_gru(x).cpu().numpy()
        want = oracle.gru_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, w.x, None, None, threads=8)
        assert_parity(got, want, "gru without b_hn / h0")
        with pytest.raises(binding.SprnnError):
            rnn.forward(x)
        with pytest.raises(binding.SprnnError):
            rnn.forward_stepwise(x)
        assert rnn.check() == binding.SPRNN_OK
    v = wl.make_workload("v", "relu", 64, 4, 1, 0.2)
    with binding.SparseRNN(64, 4, "relu", v.row_ptr, v.col_idx, v.val_bits) as rnn:
        with pytest.raises(binding.SprnnError):
            rnn.forward_gru(torch.zeros((1, 4, 64), device="cuda"))


def test_gru_with_random_pauses_is_unchanged():
    w = wl.make_workload("gru", "gru", 768, 4, 40, 0.1, seed=3, gain=1.0, h0_std=0.3)
    outs = []
    for jitter in (0, 5, 11):
        with binding.SparseRNN(w.hidden, w.batch, "gru", w.row_ptr, w.col_idx, w.val_bits, jitter=jitter, lanes_per_row=16) as rnn:   # (pinned: the lanes of a row fix the order of its sums)
            outs.append(rnn.forward_gru(_dev(w.x), _dev(w.b_hn), _dev(w.h0)).cpu().numpy())
            assert rnn.check() == binding.SPRNN_OK
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ------------------------------------------------------------------ a fixed draw of odd shapes and forced mappings
def _drawn_cases(n=36, seed=2024):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        cell = ["relu", "tanh", "identity", "lstm", "gru"][int(rng.integers(0, 5))]
        B = [1, 2, 4, 8][int(rng.integers(0, 4))]
        H = int(rng.integers(3, 700))
        T = int(rng.integers(1, 12))
        dens = float(rng.choice([0.02, 0.1, 0.3, 0.7, 1.0]))
        rownnz = ["fixed", "poisson"][int(rng.integers(0, 2))]
        opts = {}
        pick = int(rng.integers(0, 6))
        if pick == 0:
            opts["sync"] = "barrier"
        elif pick == 1:
            opts["balance"] = int(rng.integers(1, 3))
        elif pick == 2:
            opts["compact"] = 1
        elif pick == 3:
            opts["bank_aware"] = 2
        elif pick == 4:
            lmax = 16 if cell in ("lstm", "gru") else 64
            opts["lanes_per_row"] = int(min(lmax, max(B, 2 ** int(rng.integers(0, 7)))))
        cases.append((cell, H, B, T, dens, rownnz, opts))
    return cases


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts", _drawn_cases())
def test_drawn_shapes_match_oracle(cell, H, B, T, dens, rownnz, opts):
    w = wl.make_workload("drawn", cell, H, B, T, dens, seed=H * 7 + T, gain=1.0 if cell in ("lstm", "gru") else 0.9,
                         row_nnz=rownnz, h0_std=0.4)
    try:
        check_workload(w, **opts)
    except binding.SprnnError as err:
        # a forced mapping may not fit (too many words per lane for the lanes asked for): that must be a clean refusal
        assert err.code in (binding.SPRNN_ERR_CAPACITY, binding.SPRNN_ERR_INVALID), err
        assert opts, "the library's own choice of mapping must always fit these sizes"
