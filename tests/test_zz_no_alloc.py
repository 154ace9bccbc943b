"""GPU test of sprnn_forward_noalloc (the entry point that allocates nothing: its exchange ring and control words live
in a static device array that every call on one GPU shares).

Two calls in a row through the C ABI, the second on a smaller layer, so that the second one meets the array as the
first one left it; each result must be bit-identical to sprnn_forward's on the same handle (same kernels, same
arithmetic) and within the parity bar of the oracle.  Layers whose ring does not fit are refused.
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


def _both_ways(w, **options):
    """h_t from sprnn_forward and from sprnn_forward_noalloc on one handle, plus the oracle's."""
    want = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **options) as rnn:
        x, h0 = _dev(w.x), _dev(w.h0)
        print("case", w.name, "H", w.hidden, "B", w.batch, "T", w.steps, options, flush=True)
        ref = rnn.forward(x, h0)
        out = torch.full((w.steps, w.batch, w.hidden), float("nan"), dtype=torch.float32, device="cuda")
        rnn.forward_noalloc(x, h0, out)
        assert rnn.check() == binding.SPRNN_OK
        return ref.cpu().numpy(), out.cpu().numpy(), want


def _assert_same(ref, got, want, what):
    assert np.array_equal(ref.view(np.uint32), got.view(np.uint32)), what + ": differs from sprnn_forward"
    for t in range(want.shape[0]):
        scale = np.abs(want[t]).max()
        assert np.abs(got[t] - want[t]).max() <= REL_TOL * scale + 1e-30, "%s step %d" % (what, t)


def test_noalloc_two_calls_second_smaller():
    big = wl.make_workload("noalloc-big", "relu", 1152, 4, 40, 0.1, seed=11, h0_std=0.1)
    small = wl.make_workload("noalloc-small", "relu", 320, 2, 24, 0.2, seed=12)
    _assert_same(*_both_ways(big), "first call (1152 x batch 4)")
    _assert_same(*_both_ways(small), "second call (320 x batch 2)")


def test_noalloc_interleaved_with_own_ring_and_barrier_mode():
    # the same handle alternates between its own ring and the shared array; then the grid-barrier variant, whose
    # counters also live in the array
    w = wl.make_workload("noalloc-mix", "tanh", 512, 4, 16, 0.1, seed=13, h0_std=0.2)
    want = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, w.x, w.h0, threads=8)
    for sync in ("tagged", "barrier"):
        with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, sync=sync) as rnn:
            x, h0 = _dev(w.x), _dev(w.h0)
            print("case", w.name, sync, flush=True)
            outs = []
            for i in range(4):
                out = torch.empty((w.steps, w.batch, w.hidden), dtype=torch.float32, device="cuda")
                (rnn.forward_noalloc(x, h0, out) if i % 2 else rnn.forward(x, h0, out))
                outs.append(out.cpu().numpy())
            assert rnn.check() == binding.SPRNN_OK
        for o in outs:
            _assert_same(outs[0], o, want, "alternating calls, " + sync)


def test_noalloc_refuses_a_ring_beyond_the_static_array():
    # batch * hidden above 65 472: four ring slots no longer fit in 1 MiB; one nonzero per row keeps the layer cheap
    H, B = 20000, 4
    row_ptr = np.arange(H + 1, dtype=np.int32)
    col = ((np.arange(H, dtype=np.int64) * 7919 + 3) % H).astype(np.int32)
    val = np.full(H, 0x3C00, dtype=np.uint16)
    with binding.SparseRNN(H, B, "relu", row_ptr, col, val) as rnn:
        x = torch.zeros((2, B, H), dtype=torch.float32, device="cuda")
        out = torch.empty_like(x)
        print("case refuse H", H, "B", B, flush=True)
        with pytest.raises(binding.SprnnError) as e:
            rnn.forward_noalloc(x, None, out)
        assert e.value.code == binding.SPRNN_ERR_CAPACITY
        rnn.forward(x, None, out)        # the handle itself still works
        assert rnn.check() == binding.SPRNN_OK


@pytest.mark.parametrize("H,dens,opts", [(2304, 0.05, {}), (1152, 0.1, {"xcd": "one", "grid": 32})])
def test_noalloc_call_captured_in_a_graph_and_replayed(H, dens, opts):
    # What the entry point is for: a caller under stream capture.  The captured call (a fill kernel that re-marks the
    # ring, then the persistent kernel as an ordinary launch) is replayed several times with new inputs, with eager work
    # of the same handle and synchronisations in between; every replay must equal the eager result for that input.
    w = wl.make_workload("graph", "tanh", H, 4, 24, dens, seed=17, h0_std=0.3)
    rng = np.random.default_rng(3)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **opts) as rnn:
        x, h0 = _dev(w.x), _dev(w.h0)
        out = torch.empty_like(x)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            rnn.forward_noalloc(x, h0, out)            # warm-up outside the capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            rnn.forward_noalloc(x, h0, out)
        for i in range(4):
            new_x = torch.from_numpy((rng.standard_normal(w.x.shape) * 0.5).astype(np.float32)).cuda()
            x.copy_(new_x)
            out.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            eager = rnn.forward(new_x, h0).cpu().numpy()            # the handle's own ring, between two replays
            assert rnn.check() == binding.SPRNN_OK
            assert np.array_equal(got.view(np.uint32), eager.view(np.uint32)), "replay %d" % i
        want = oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, new_x.cpu().numpy(), w.h0, threads=8)
        for t in range(w.steps):
            assert np.abs(got[t] - want[t]).max() <= REL_TOL * np.abs(want[t]).max() + 1e-30, t


def test_calls_on_the_handles_own_ring_are_refused_under_capture():
    # a launch on the handle's own ring carries the handle's position in that ring: replayed, it would accept the last
    # replay's values as its own, so it is refused while the stream is being captured (and works again afterwards)
    w = wl.make_workload("cap", "relu", 512, 4, 6, 0.2, seed=19)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits) as rnn:
        x = _dev(w.x)
        out = torch.empty_like(x)
        want = rnn.forward(x, None).cpu().numpy()
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        refused = None
        with torch.cuda.graph(graph, stream=side):
            try:
                rnn.forward(x, None, out)
            except binding.SprnnError as e:
                refused = e.code
            rnn.forward_noalloc(x, None, out)
        assert refused == binding.SPRNN_ERR_UNSUPPORTED
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want)
        assert np.array_equal(rnn.forward(x, None).cpu().numpy(), want) and rnn.check() == binding.SPRNN_OK
