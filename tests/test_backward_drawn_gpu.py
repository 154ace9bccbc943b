"""A fixed draw of odd shapes and forced mappings for the backward passes of all cells (plain and with the weight
gradient fused in), against the CPU oracle through the C ABI.  Same bar as the other backward tests."""
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


def _drawn_cases(n=30, seed=4711):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        cell = ["relu", "tanh", "lstm", "gru"][int(rng.integers(0, 4))]
        B = [1, 2, 4, 8][int(rng.integers(0, 4))]
        H = int(rng.integers(3, 500))
        T = int(rng.integers(1, 10))
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
            opts["lanes_per_row"] = int(min(64, max(B, 2 ** int(rng.integers(0, 7)))))
        cases.append((cell, H, B, T, dens, rownnz, opts, bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("cell,H,B,T,dens,rownnz,opts,fused", _drawn_cases())
def test_drawn_backward_shapes_match_oracle(cell, H, B, T, dens, rownnz, opts, fused):
    w = wl.make_workload("drawn", cell, H, B, T, dens, seed=H * 5 + T, gain=1.0 if cell in ("lstm", "gru") else 0.9,
                         row_nnz=rownnz, h0_std=0.4)
    rng = np.random.default_rng(H + B + T)
    e = rng.standard_normal((T, B, H)).astype(np.float32)
    c0 = (rng.standard_normal((B, H)) * 0.5).astype(np.float32)
    csr = (w.row_ptr, w.col_idx, w.val_bits)
    print("case", cell, "H", H, "B", B, "T", T, dens, rownnz, opts, "fused" if fused else "plain", flush=True)
    if cell == "lstm":
        h, c, gates = oracle.lstm_forward_saved(H, B, *csr, w.x, w.h0, c0)
        want = dict(zip(("d", "dh0", "dc0", "dU"), oracle.lstm_backward(H, B, *csr, gates, c, h, e, w.h0, c0)))
    elif cell == "gru":
        h, gates = oracle.gru_forward_saved(H, B, *csr, w.x, w.b_hn, w.h0)
        want = dict(zip(("d", "v", "dh0", "dU", "db"), oracle.gru_backward(H, B, *csr, gates, h, e, w.h0)))
    else:
        h = oracle.rnn_forward(H, B, cell, *csr, w.x, w.h0)
        want = dict(zip(("d", "dh0", "dU"), oracle.rnn_backward(H, B, cell, *csr, h, e, w.h0)))
    t_rp, t_ci, t_vb, t_src = binding.transpose_csr(w.rows, H, *csr, with_source=True)
    kind = {"lstm": "lstm_backward", "gru": "gru_backward"}.get(cell, cell)
    def run(options, with_weights):
        out = {}
        with binding.SparseRNN(H, B, kind, t_rp, t_ci, t_vb, **options) as rnn:
            if cell == "lstm":
                if with_weights:
                    out["d"], out["dh0"], out["dc0"], out["dU_t"] = rnn.backward_lstm_with_weights(_dev(e), _dev(gates), _dev(c), _dev(h), _dev(c0), _dev(w.h0))
                else:
                    out["d"], out["dh0"], out["dc0"] = rnn.backward_lstm(_dev(e), _dev(gates), _dev(c), _dev(c0))
            elif cell == "gru":
                if with_weights:
                    out["d"], out["v"], out["dh0"], out["dU_t"] = rnn.backward_gru_with_weights(_dev(e), _dev(gates), _dev(h), _dev(w.h0))
                else:
                    out["d"], out["v"], out["dh0"] = rnn.backward_gru(_dev(e), _dev(gates), _dev(h), _dev(w.h0))
            else:
                if with_weights:
                    out["d"], out["dh0"], out["dU_t"] = rnn.backward_with_weights(_dev(e), _dev(h), _dev(w.h0))
                else:
                    out["d"], out["dh0"] = rnn.backward(_dev(e), _dev(h))
            assert rnn.check() == binding.SPRNN_OK
            return {k: v.cpu().numpy() for k, v in out.items()}

    # A forced mapping may not fit, and the fused kernels are not built for every mapping.  Such a draw must be refused
    # cleanly, and then runs without the part that was refused (first the fusion, then the forced option), so that every
    # draw is compared with the oracle; the library's own mapping must always work.
    got = None
    for options, with_weights in ((opts, fused), (opts, False), ({}, fused), ({}, False)):
        try:
            got = run(options, with_weights)
            print("   ran with", options, "fused" if with_weights else "plain", flush=True)
            break
        except binding.SprnnError as err:
            assert err.code in (binding.SPRNN_ERR_CAPACITY, binding.SPRNN_ERR_INVALID, binding.SPRNN_ERR_UNSUPPORTED), err
            assert options or with_weights, "the library's own choice of mapping must always fit these sizes"
    assert got is not None
    for t in range(T):
        _close(got["d"][t], want["d"][t], "d_bprime[%d]" % t)
        if "v" in got:
            _close(got["v"][t], want["v"][t], "d_recurrent[%d]" % t)
    _close(got["dh0"], want["dh0"], "dh0")
    if "dc0" in got:
        _close(got["dc0"], want["dc0"], "dc0")
    if "dU_t" in got and want["dU"].size:
        dU = np.empty_like(got["dU_t"])
        dU[t_src] = got["dU_t"]
        _close(dU, want["dU"], "dU")


@pytest.mark.parametrize("cell,H,B,opts,code", [
    ("relu", 100, 8, {"lanes_per_row": 4}, binding.SPRNN_ERR_INVALID),            # fewer lanes per row than samples
    ("lstm_backward", 100, 4, {"lanes_per_row": 3}, binding.SPRNN_ERR_INVALID),   # not a power of two
    ("gru_backward", 200, 4, {"waves": 13}, binding.SPRNN_ERR_INVALID),           # more wavefronts than a workgroup may have
    ("relu", 3000, 4, {"compact": 2, "grid": 1}, binding.SPRNN_ERR_CAPACITY),     # one workgroup cannot hold two copies of h ... and all rows
    ("lstm_backward", 20000, 1, {}, binding.SPRNN_ERR_UNSUPPORTED),               # 4H columns exceed 16-bit indices
])
def test_mappings_that_cannot_be_served_are_refused_cleanly(cell, H, B, opts, code):
    gates = {"lstm_backward": 4, "gru_backward": 3}.get(cell, 1)
    rows = H
    row_ptr = np.arange(rows + 1, dtype=np.int32)
    col = (np.arange(rows, dtype=np.int64) % (gates * H)).astype(np.int32)
    with pytest.raises(binding.SprnnError) as err:
        binding.SparseRNN(H, B, cell, row_ptr, col, np.full(rows, 0x3C00, np.uint16), **opts)
    assert err.value.code == code, err.value


@pytest.mark.parametrize("cell,H,B,T,dens", [
    ("lstm", 2560, 4, 4, 0.004),      # 4H x B x 4 bytes = 160 KB of gate gradients: only the chunks a workgroup reads fit in LDS
    ("gru", 5000, 2, 3, 0.004),
    ("lstm", 3000, 8, 3, 0.01),
])
def test_large_gated_backward_layers_run_through_column_compaction(cell, H, B, T, dens):
    w = wl.make_workload("big", cell, H, B, T, dens, seed=1, gain=1.0, row_nnz="poisson", h0_std=0.3)
    e = np.random.default_rng(1).standard_normal((T, B, H)).astype(np.float32)
    csr = (w.row_ptr, w.col_idx, w.val_bits)
    t_csr = binding.transpose_csr(w.rows, H, *csr)
    with binding.SparseRNN(H, B, cell + "_backward", *t_csr) as rnn:
        info = rnn.info()
        print("case", cell, H, B, {k: info[k] for k in ("grid", "block", "lds_bytes", "compact", "template_words")}, flush=True)
        assert info["compact"] == 1
        if cell == "lstm":
            h, c, g = oracle.lstm_forward_saved(H, B, *csr, w.x, w.h0, None, threads=8)
            want = oracle.lstm_backward(H, B, *csr, g, c, h, e, w.h0, None)[:3]
            got = rnn.backward_lstm(_dev(e), _dev(g), _dev(c))
        else:
            h, g = oracle.gru_forward_saved(H, B, *csr, w.x, w.b_hn, w.h0, threads=8)
            want = oracle.gru_backward(H, B, *csr, g, h, e, w.h0)[:3]
            got = rnn.backward_gru(_dev(e), _dev(g), _dev(h), _dev(w.h0))
        assert rnn.check() == binding.SPRNN_OK
    for a, b, what in zip(got, want, ("first output", "second output", "third output")):
        a = a.cpu().numpy()
        if a.ndim == 3:
            for t in range(T):
                _close(a[t], b[t], "%s[%d]" % (what, t))
        else:
            _close(a, b, what)
