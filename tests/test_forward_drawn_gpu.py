"""A fixed draw of shapes, densities and cells for the forward pass with NOTHING fixed about the mapping: sprnn_create
then measures its candidate mappings on the device and keeps one, and whichever it keeps must give the oracle's result.
Same bar as the other parity tests (per timestep, max-norm 1e-3)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1804_10223_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

REL_TOL = 1e-3


def _dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _drawn(n=36, seed=1804):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        cell = ["relu", "tanh", "identity", "lstm", "gru"][int(rng.integers(0, 5))]
        B = [1, 2, 4, 8][int(rng.integers(0, 4))]
        H = int(rng.choice([int(rng.integers(1, 200)), int(rng.integers(200, 1500)), int(rng.integers(1500, 4000))]))
        if cell in ("lstm", "gru"):
            H = min(H, 1200)
        dens = float(rng.choice([0.0, 0.01, 0.05, 0.2, 0.5]))
        T = int(rng.integers(1, 12))
        cases.append((cell, H, B, T, dens, ["fixed", "poisson"][int(rng.integers(0, 2))]))
    return cases


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz", _drawn())
def test_drawn_forward_shapes_with_the_librarys_own_mapping(cell, H, B, T, dens, rownnz):
    w = wl.make_workload("drawn", cell, H, B, T, dens, seed=H + 7 * T, gain=1.0 if cell in ("lstm", "gru") else 0.9,
                         row_nnz=rownnz, h0_std=0.4)
    print("case", cell, "H", H, "B", B, "T", T, dens, rownnz, flush=True)
    csr = (w.row_ptr, w.col_idx, w.val_bits)
    try:
        rnn = binding.SparseRNN(H, B, cell, *csr)
    except binding.SprnnError as e:
        # the only legitimate refusal here: a gated layer whose nonzeros do not fit in the register files (one unit per
        # wavefront at most 16 lanes per row: beyond 32 nonzeros per lane only four wavefronts fit a workgroup)
        assert e.code == binding.SPRNN_ERR_CAPACITY and cell in ("lstm", "gru") and w.nnz > 1_500_000, (e, w.nnz)
        return
    with rnn:
        info = rnn.info()
        print("   kept", info["grid"], "x", info["block"], "lanes", info["lanes_per_row"], "one xcd", info["one_xcd"],
              "compact", info["compact"], flush=True)
        if cell == "lstm":
            want, want_c = oracle.lstm_forward(H, B, *csr, w.x, w.h0, w.c0, threads=8)
            got, got_c = rnn.forward_lstm(_dev(w.x), _dev(w.h0), _dev(w.c0))
        elif cell == "gru":
            want, want_c = oracle.gru_forward(H, B, *csr, w.x, w.b_hn, w.h0, threads=8), None
            got, got_c = rnn.forward_gru(_dev(w.x), _dev(w.b_hn), _dev(w.h0)), None
        else:
            want, want_c = oracle.rnn_forward(H, B, cell, *csr, w.x, w.h0, threads=8), None
            got, got_c = rnn.forward(_dev(w.x), _dev(w.h0)), None
        assert rnn.check() == binding.SPRNN_OK
    for a, b, what in ((got, want, "h"), (got_c, want_c, "c")):
        if b is None:
            continue
        a = a.cpu().numpy()
        assert a.shape == b.shape and np.all(np.isfinite(a))
        for t in range(T):
            assert np.abs(a[t] - b[t]).max() <= REL_TOL * np.abs(b[t]).max() + 1e-30, (what, t)
