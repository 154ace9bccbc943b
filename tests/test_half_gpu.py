"""binary16 activations (options.activations = 2; Section 6 names lower-precision activations as future work): h travels
between workgroups and sits in LDS as binary16, rounded to nearest once per step before it is published; products,
sums, b' and h_out stay binary32.

Bars: (1) the same bound as everywhere against the plain binary32 oracle, max|h - h_oracle| <= 1e-3 max|h_oracle| per
timestep (the rounding leaves a few 1e-4, so this bar is met with a small margin, not a large one); (2) against the
oracle run one step at a time with h rounded to binary16 between steps (numpy's round-to-nearest conversion), which is
what the mode computes: in the first three steps the median element within 1e-5 and 99 % within 2e-4 (the two sides'
sums and activation functions differ by a few 1e-7, which makes about one rounding in a thousand fall the other way,
and each such flip of 2^-11 shifts the following steps' sums, so the two drift apart slowly), all steps within 1e-3; (3) bit-exact where no
rounding happens (permutation matrices of binary16-representable values).
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


def _stepwise_rounded_oracle(w):
    """(h_out as the mode defines it, the rounded state after the last step): the oracle one step at a time, h rounded to
    binary16 between steps; h_out[t] is the unrounded output of step t."""
    H, B = w.hidden, w.batch
    cur = (np.zeros((B, H), np.float32) if w.h0 is None else w.h0).astype(np.float16).astype(np.float32)
    out = np.empty((w.steps, B, H), np.float32)
    for t in range(w.steps):
        out[t] = oracle.rnn_forward(H, B, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x[t:t + 1], cur)[0]
        cur = out[t].astype(np.float16).astype(np.float32)
    return out


CASES = [
    ("relu", 96, 9, 0.3, "fixed", {}),                                   # one workgroup: h stays in LDS
    ("tanh", 640, 12, 0.3, "fixed", {"waves": 2}),
    ("identity", 300, 8, 0.2, "poisson", {}),
    ("tanh", 1000, 30, 0.1, "poisson", {"jitter": 3}),
    ("relu", 500, 10, 0.2, "fixed", {"sync": "barrier"}),
    ("relu", 500, 10, 0.2, "fixed", {"xcd": "one"}),
    ("tanh", 333, 7, 0.25, "poisson", {"balance": 1}),                   # odd hidden size: the last 16-byte piece is half used
    ("relu", 1152, 20, 0.1, "fixed", {"lanes_per_row": 64, "jitter": 5}),
    ("relu", 640, 10, 0.5, "fixed", {"lanes_per_row": 8, "bank_aware": 2}),       # 40 words per lane: the 48-slot kernel
    ("tanh", 4608, 6, 0.02, "fixed", {}),                                # 36 KB of binary16 h: more than two copy rounds
    ("relu", 3000, 6, 0.01, "poisson", {"compact": 1}),                  # column compaction: two columns per 16-byte piece
    ("tanh", 2000, 6, 0.02, "fixed", {"compact": 1, "grid": 125, "jitter": 2}),
]
# batch 8: a column is eight binary16 values, one 16-byte read; the eight owner lanes of a row pack it
CASES_8 = [
    ("relu", 96, 9, 0.3, "fixed", {}),                                   # one workgroup
    ("tanh", 640, 12, 0.3, "fixed", {"waves": 2}),
    ("identity", 300, 8, 0.2, "poisson", {"jitter": 3}),
    ("relu", 500, 10, 0.2, "fixed", {"sync": "barrier"}),
    ("relu", 500, 10, 0.2, "fixed", {"xcd": "one"}),
    ("tanh", 333, 7, 0.25, "poisson", {"balance": 1, "lanes_per_row": 8}),
    ("relu", 1760, 12, 0.12, "fixed", {"lanes_per_row": 32, "jitter": 5}),
    ("tanh", 3072, 6, 0.05, "fixed", {}),                                # 48 KB of binary16 h
    ("relu", 2000, 6, 0.02, "fixed", {"compact": 1, "grid": 100}),       # column compaction: one column per 16-byte piece
    ("relu", 11520, 4, 0.01, "fixed", {}),                               # 180 KB of binary16 h: runs compacted
]


@pytest.mark.parametrize("B,cell,H,T,dens,rownnz,opts", [(4,) + c for c in CASES] + [(8,) + c for c in CASES_8])
def test_binary16_activations_match_both_oracles(B, cell, H, T, dens, rownnz, opts):
    w = wl.make_workload("half", cell, H, B, T, dens, seed=H + T, row_nnz=rownnz, h0_std=0.5)
    plain = oracle.rnn_forward(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    rounded = _stepwise_rounded_oracle(w)
    with binding.SparseRNN(H, B, cell, w.row_ptr, w.col_idx, w.val_bits, activations="binary16", **opts) as rnn:
        info = rnn.info()
        got = rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
        again = rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy()          # second call on the same handle
        assert rnn.check() == binding.SPRNN_OK and np.array_equal(got, again)
    assert info["activations"] == 2 and np.all(np.isfinite(got))
    worst = 0.0
    for t in range(T):
        scale = np.abs(plain[t]).max()
        worst = max(worst, np.abs(got[t] - plain[t]).max() / scale)
        assert np.abs(got[t] - plain[t]).max() <= REL_TOL * scale, t
        # against the rounded oracle only a rounding that falls the other way (the two sides' sums differ in the last
        # binary32 bits) separates the two, and what such a flip of 2^-11 does to the next steps' sums
        diff = np.abs(got[t] - rounded[t])
        if t < 3:   # (the flips add up over the steps of a recurrence: the tight comparison is for the first ones)
            assert np.median(diff) <= 1e-5 * scale and np.quantile(diff, 0.99) <= 2e-4 * scale, (t, np.median(diff) / scale, np.quantile(diff, 0.99) / scale)
        assert diff.max() <= REL_TOL * scale, t
    print("case batch", B, cell, H, T, dens, rownnz, opts, {k: info[k] for k in ("grid", "block", "lanes_per_row", "lds_bytes")},
          "worst step against the binary32 oracle: %.2e of max|h|" % worst, flush=True)


@pytest.mark.parametrize("H,B", [(7, 4), (1000, 4), (4099, 4), (16384, 4), (7, 8), (1000, 8), (4099, 8), (9999, 8)])   # (the largest h that fits in LDS)
def test_permutation_of_binary16_values_is_bit_exact(H, B):
    rng = np.random.default_rng(H)
    perm = rng.permutation(H).astype(np.int32)
    row_ptr = np.arange(H + 1, dtype=np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    T = 5
    x = np.zeros((T, B, H), dtype=np.float32)
    h0 = (rng.integers(1, 2048, (B, H)) / 64.0).astype(np.float32)      # exactly representable in binary16, never zero
    with binding.SparseRNN(H, B, "relu", row_ptr, perm, ones, activations=2) as rnn:
        h = rnn.forward(_dev(x), _dev(h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    cur = h0
    for t in range(T):
        cur = cur[:, perm]
        assert np.array_equal(h[t].view(np.uint32), cur.view(np.uint32)), t


def test_tiny_negative_results_do_not_become_the_not_written_mark():
    # identity cell, results around -1e-9: they round to -0.0 in binary16, which is the mark of an unwritten element; the
    # kernel must publish +0.0 instead (a mark would make every reader wait until the watchdog trips)
    H, T = 256, 6
    rng = np.random.default_rng(2)
    row_ptr = np.arange(H + 1, dtype=np.int32)
    col = rng.permutation(H).astype(np.int32)
    ones = np.full(H, 0x3C00, dtype=np.uint16)
    x = np.full((T, 4, H), -1e-9, dtype=np.float32)
    with binding.SparseRNN(H, 4, "identity", row_ptr, col, ones, activations=2, grid=4, spin_limit=200000) as rnn:
        h = rnn.forward(_dev(x), None).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    assert np.all(np.abs(h) < 1e-8) and np.all(np.isfinite(h))


def test_headline_shape_and_the_largest_layer_with_binary16_activations():
    w = wl.make_config("cfg3", steps=64)
    plain = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=16)
    outs = []
    for jitter in (0, 7):
        with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, activations=2, jitter=jitter, lanes_per_row=64) as rnn:   # (pinned: the lanes of a row fix the order of its sums)
            outs.append(rnn.forward(_dev(w.x), _dev(w.h0)).cpu().numpy())
            assert rnn.check() == binding.SPRNN_OK
    assert np.array_equal(outs[0], outs[1])                               # random pauses change nothing
    for t in range(w.steps):
        assert np.abs(outs[0][t] - plain[t]).max() <= REL_TOL * np.abs(plain[t]).max(), t
    # hidden 11520 at batch 4 and 1 %: 92 KB of binary16 activations fit in LDS where binary32 needs column compaction
    big = wl.make_workload("huge", "relu", 11520, 4, 5, 0.01, seed=14, h0_std=0.5)
    want = oracle.rnn_forward(11520, 4, "relu", big.row_ptr, big.col_idx, big.val_bits, big.x, big.h0, threads=16)
    with binding.SparseRNN(11520, 4, "relu", big.row_ptr, big.col_idx, big.val_bits, activations=2) as rnn:
        info = rnn.info()
        assert info["compact"] == 0 and info["lds_bytes"] == 11520 * 8
        got = rnn.forward(_dev(big.x), _dev(big.h0)).cpu().numpy()
        assert rnn.check() == binding.SPRNN_OK
    for t in range(5):
        assert np.abs(got[t] - want[t]).max() <= REL_TOL * np.abs(want[t]).max(), t


def test_calls_that_are_not_built_for_binary16_activations_are_refused():
    w = wl.make_workload("r", "relu", 512, 4, 3, 0.2, seed=1)
    with binding.SparseRNN(512, 4, "relu", w.row_ptr, w.col_idx, w.val_bits, activations=2) as rnn:
        x = _dev(w.x)
        for call in (lambda: rnn.forward_noalloc(x, None, torch.empty_like(x)), lambda: rnn.backward(x, x), lambda: rnn.backward_with_weights(x, x),
                     lambda: rnn.weight_gradient(x, x)):
            with pytest.raises(binding.SprnnError) as e:
                call()
            assert e.value.code == binding.SPRNN_ERR_UNSUPPORTED
        s, _ = rnn.forward_stepwise(x, None)                                # the comparison path is binary32 throughout
        want = oracle.rnn_forward(512, 4, "relu", w.row_ptr, w.col_idx, w.val_bits, w.x, None)
        assert np.abs(s.cpu().numpy() - want).max() <= 1e-5 * np.abs(want).max()
        assert rnn.check() == binding.SPRNN_OK
