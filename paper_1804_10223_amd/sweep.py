#!/usr/bin/env python3
"""Ablation and parameter sweeps of the persistent sparse recurrent kernel on synthetic layers.

    python -m paper_1804_10223_amd.sweep [--what ablation,density,size,constnnz,batch,steps,placement,activations,thinned,exchange,cells,training,casestudy] [--reps 8]
    python -m paper_1804_10223_amd.sweep --what rung --config cfg2 --rung naive|wide|bank_aware|tagged|pool|two_part|spread32|one_xcd32
                                                                  (one variant alone in the process, for counter passes)

Mirrors the structure of the paper's evaluation on this library's own kernels (its comparison systems are
closed libraries on other hardware and are not reproduced):

  ablation   Table 1's shape (hidden 1152, batch 4, density 10 %, T 256) and the headline shape (2304, 30 %):
             per-timestep launches -> persistent with 4-byte gathers, CSR-order nonzeros and a grid barrier ->
             wide gathers -> bank-aware ordering -> tagged hand-off (Table 1's four rungs), with the packer's LDS pass
             model as the bank-conflict figure; then the two layouts side by side.
  density / size / batch / steps
             the four axes of Section 5.2 around its base point (hidden 1792, density 10 %, batch 4, T 256).
  constnnz   Section 5.3's last experiment: about 1.32 M nonzeros spread over layers of 2304 to 11520 units.
  placement  small layers with their workgroups spread over all XCDs against confined to one XCD (options.xcd).
  activations  binary32 against binary16 activations on layers of 1152 to 11520 units (options.activations).
  cells      the four cells (ReLU, tanh, LSTM, GRU) on one layer shape: hidden 1024, density 20 %, T 256, batch 4 and 8.
  training   the launches of one training step (forward, backward pass through time, weight gradient) of a ReLU cell,
             the LSTM and the GRU on the same layer shape.
  casestudy  the layer shapes of Appendix B's two tables (machine translation LSTMs at 4-12.5 % density, speech
             recognition layers at 12 %) with random unstructured patterns, as the paper itself does for the speech
             layers; milliseconds per 256-timestep sequence beside the paper's own figure (another GPU: context).

Prints markdown tables on stdout.  Needs a GPU; every number comes from the HIP library.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np


def _time_us_per_step(torch, run, T, reps):
    for _ in range(2):
        run()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / T)
    return float(np.median(ts))


def measure(torch, w, reps, stepwise=False, want_output=False, **options):
    """Microseconds per timestep of one workload (whole launch / T) and the mapping the library chose (and, on request,
    the output h of the last run as a numpy array)."""
    from . import binding
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    x, h0, c0 = dev(w.x), dev(w.h0), dev(w.c0)
    T = w.steps
    h_out = torch.empty((T, w.batch, w.hidden), dtype=torch.float32, device="cuda")
    c_out = torch.empty_like(h_out) if w.cell == "lstm" else None
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **options) as rnn:
        info = rnn.info()
        if stepwise:
            run = lambda: rnn.forward_stepwise(x, h0, c0, h_out, c_out)
        elif w.cell == "lstm":
            run = lambda: rnn.forward_lstm(x, h0, c0, h_out, c_out)
        elif w.cell == "gru":
            b_hn = dev(w.b_hn)
            run = lambda: rnn.forward_gru(x, b_hn, h0, h_out)
        else:
            run = lambda: rnn.forward(x, h0, h_out)
        us = _time_us_per_step(torch, run, T, max(3, reps // 2) if stepwise else reps)
        if rnn.check() != 0:
            raise RuntimeError("spin watchdog tripped")
        out = h_out.cpu().numpy() if want_output else None
    return (us, info, out) if want_output else (us, info)


# The rungs of Table 1, each on top of the one before: no wide loads and a grid barrier ("naive"), wide loads
# (Section 4.1), bank-aware order of a row's nonzeros (Section 4.1, Appendix A), validity carried by the data instead
# of a barrier (Section 4.2's Lamport timestamps).
RUNGS = [
    ("naive", dict(sync="barrier", bank_aware=2, gather="narrow")),
    ("wide", dict(sync="barrier", bank_aware=2, gather="wide")),
    ("bank_aware", dict(sync="barrier", bank_aware=1, gather="wide")),
    ("tagged", dict(sync="tagged", bank_aware=1, gather="wide")),
]


def ablation(torch, wl, reps):
    print("## Ablation (cf. Table 1): microseconds per timestep, whole launch / T (layout: one lane group per row)\n")
    print("The rungs share one mapping (the one the packer picks first); the last column is what `sprnn_create` arrives at when it may also\nmeasure a second mapping and the XCD placement.\n")
    print("| shape | per-timestep launches | persistent: 4-byte gathers, CSR order, grid barrier | + wide gathers | + bank-aware order | + tagged hand-off | tagged hand-off with CSR order | modelled LDS cycles per gather: CSR order / bank-aware | the library's own choice (grid x block) |")
    print("|---|---|---|---|---|---|---|---|---|")
    for name in ("cfg2", "cfg3"):
        w = wl.make_config(name)
        step, _ = measure(torch, w, reps, stepwise=True)
        got = {}
        for rung, opts in RUNGS:
            got[rung] = measure(torch, w, reps, layout=1, **opts)
        tn, _ = measure(torch, w, reps, layout=1, sync="tagged", bank_aware=2)
        own, io = measure(torch, w, reps)
        print("| %s: hidden %d, batch %d, density %.0f %%, T %d | %.2f | %.2f | %.2f | %.2f | %.2f | %.2f | %.2f / %.2f | %.2f (%d x %d%s) |" % (
            name, w.hidden, w.batch, 100 * w.meta["density"], w.steps, step, got["naive"][0], got["wide"][0], got["bank_aware"][0],
            got["tagged"][0], tn, got["wide"][1]["lds_pass_factor"], got["bank_aware"][1]["lds_pass_factor"],
            own, io["grid"], io["block"], ", one XCD" if io["one_xcd"] else ""), flush=True)
    print()
    w = wl.make_config("cfg4")
    b1, i1 = measure(torch, w, reps, balance=1)
    b2, i2 = measure(torch, w, reps, balance=2)
    print("Load balance (cf. Section 6), cfg4 (hidden 5760, batch 2, Poisson(576) rows): rows dealt by nonzero count "
          "%.2f us/step with %.1f %% padding; contiguous rows %.2f us/step with %.1f %% padding.\n" % (
              b1, 100.0 * (i1["padded_words"] / max(i1["nnz"], 1) - 1), b2, 100.0 * (i2["padded_words"] / max(i2["nnz"], 1) - 1)), flush=True)
    print("Layout (cf. Section 6, load balancing by nonzero count): one lane group per row against the lane pool\n")
    print("| shape | one lane group per row us/step | lane pool us/step | lane pool grid x block, words per lane | modelled LDS cycles per gather: groups / pool |")
    print("|---|---|---|---|---|")
    for name in ("cfg2", "cfg3", "cfg4"):
        w = wl.make_config(name)
        a, ia = measure(torch, w, reps, layout=1)
        try:
            b, ib = measure(torch, w, reps, layout=2)
            print("| %s | %.2f | %.2f | %d x %d, %d | %.2f / %.2f |" % (name, a, b, ib["grid"], ib["block"], ib["words_per_lane_max"],
                                                                 ia["lds_pass_factor"], ib["lds_pass_factor"]), flush=True)
        except Exception as e:
            print("| %s | %.2f | refused: %s | | |" % (name, a, e), flush=True)
    print()
    print("Copy of h consumed in two parts, early words during the second (cf. Section 4.2, work during the load stage)\n")
    print("| shape | one copy, then all words us/step | two parts us/step | copy rounds in the first part, early words of the words per lane | modelled LDS cycles per gather: one copy / two parts |")
    print("|---|---|---|---|---|")
    for name in ("cfg3", "cfg4"):
        w = wl.make_config(name)
        a, ia = measure(torch, w, reps, overlap=1)
        try:
            b, ib = measure(torch, w, reps, overlap=2)
            print("| %s | %.2f | %.2f | %d, %d of %d | %.2f / %.2f |" % (name, a, b, ib["overlap_rounds"], ib["overlap_words"], ib["words_per_lane_max"],
                                                                  ia["lds_pass_factor"], ib["lds_pass_factor"]), flush=True)
        except Exception as e:
            print("| %s | %.2f | refused: %s | | |" % (name, a, e), flush=True)
    print()


# further variants that --what rung can run alone: the lane-pool layout and the two-part copy
VARIANTS = dict(RUNGS, pool=dict(layout=2), two_part=dict(overlap=2),
                # 32 workgroups (cfg2 fits them) spread over all XCDs or confined to one
                spread32=dict(grid=32, xcd="spread", poll_delay=1), one_xcd32=dict(grid=32, xcd="one", poll_delay=1))


def one_rung(torch, wl, reps, config, rung):
    """One rung of the ablation (or one variant) alone in this process, so that a counter pass of the profiler sees only
    its launches; the back-off is fixed, so there are no calibration launches either."""
    opts = dict(layout=1, poll_delay=3)
    opts.update(VARIANTS[rung])
    w = wl.make_config(config)
    us, info = measure(torch, w, reps, **opts)
    print("rung %s on %s: %.3f us/step, grid %d x %d, modelled LDS cycles per gather %.3f" % (
        rung, config, us, info["grid"], info["block"], info["lds_pass_factor"]), flush=True)


def axis(torch, wl, reps, title, cases):
    print("## %s\n" % title)
    print("| hidden | batch | density | T | nonzeros | persistent us/step | per-timestep launches us/step | ratio | grid x block | lanes/row | back-off | LDS for h | one XCD |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for (H, B, dens, T) in cases:
        w = wl.make_workload("sweep", "relu", H, B, T, dens, seed=0)
        try:
            us, info = measure(torch, w, reps)
        except Exception as e:  # a shape that does not fit on chip is part of the picture
            print("| %d | %d | %.1f %% | %d | %d | does not fit: %s | | | | | | | |" % (H, B, 100 * dens, T, w.nnz, e), flush=True)
            continue
        st, _ = measure(torch, w, reps, stepwise=True)
        print("| %d | %d | %.1f %% | %d | %d | %.2f | %.2f | %.1fx | %d x %d | %d | %d | %d KB%s | %s |" % (
            H, B, 100 * dens, T, w.nnz, us, st, st / us, info["grid"], info["block"], info["lanes_per_row"], info["poll_delay"],
            info["lds_bytes"] // 1024, " (compacted)" if info["compact"] else "", "yes" if info["one_xcd"] else ""), flush=True)
    print()


def placement(torch, wl, reps):
    """Small layers (at most 32 workgroups): workgroups spread over all XCDs against the one-XCD mode, and what the
    calibration at create time picks by itself."""
    print("## XCD placement of small layers: microseconds per timestep, T 256\n")
    print("| layer | grid x block | spread over all XCDs | one XCD | chosen at create time (one XCD?) |")
    print("|---|---|---|---|---|")
    cases = [("cfg2 with 32 workgroups", wl.make_config("cfg2"), dict(grid=32)),
             ("relu 1792, 1 %, batch 4", wl.make_workload("p", "relu", 1792, 4, 256, 0.01, seed=0), {}),
             ("relu 1792, 5 %, batch 4", wl.make_workload("p", "relu", 1792, 4, 256, 0.05, seed=0), {}),
             ("relu 1792, 10 %, batch 4, 28 workgroups of 8 lanes per row", wl.make_workload("p", "relu", 1792, 4, 256, 0.10, seed=0), dict(grid=28, lanes_per_row=8)),
             ("relu 1024, 10 %, batch 4", wl.make_workload("p", "relu", 1024, 4, 256, 0.10, seed=0), {}),
             ("lstm 256, 12.5 %, batch 4", wl.make_workload("p", "lstm", 256, 4, 256, 0.125, seed=0, gain=1.0), {}),
             ("lstm 1024, 4.7 %, batch 1", wl.make_workload("p", "lstm", 1024, 1, 256, 0.047, seed=0, gain=1.0), {})]
    for name, w, opts in cases:
        try:
            a, ia = measure(torch, w, reps, xcd="spread", **opts)
            b, _ = measure(torch, w, reps, xcd="one", **opts)
            c, ic = measure(torch, w, reps, **opts)
            print("| %s | %d x %d | %.2f | %.2f | %.2f (%s) |" % (name, ia["grid"], ia["block"], a, b, c, "yes" if ic["one_xcd"] else "no"), flush=True)
        except Exception as e:
            print("| %s | | refused: %s | | |" % (name, e), flush=True)
    print()


def activations(torch, wl, reps):
    """binary32 against binary16 activations (options.activations): half the exchange and LDS traffic, and the worst
    difference between the two outputs as a fraction of max|h| per timestep."""
    import numpy as np
    print("## Activations exchanged as binary32 or binary16 (cf. Section 6, future work): batch 4 and 8, T 256\n")
    print("| hidden | batch | density | binary32 us/step | binary16 us/step | LDS for h | worst step difference / max abs h |")
    print("|---|---|---|---|---|---|---|")
    for (H, B, dens) in [(1152, 4, 0.10), (2304, 4, 0.30), (3072, 4, 0.10), (4096, 4, 0.10), (5120, 4, 0.10), (7168, 4, 0.026), (11520, 4, 0.01),
                         (1024, 8, 0.20), (1760, 8, 0.12), (2560, 8, 0.12), (3072, 8, 0.12), (5120, 8, 0.05)]:
        w = wl.make_workload("sweep", "relu", H, B, 256, dens, seed=0)
        a, ia, oa = measure(torch, w, reps, want_output=True)
        b, ib, ob = measure(torch, w, reps, want_output=True, activations=2)
        diff = max(float(np.abs(oa[t] - ob[t]).max() / np.abs(oa[t]).max()) for t in range(w.steps))
        print("| %d | %d | %.1f %% | %.2f | %.2f | %d KB%s / %d KB | %.1e |" % (H, B, 100 * dens, a, b, ia["lds_bytes"] // 1024,
              " (compacted)" if ia["compact"] else "", ib["lds_bytes"] // 1024, diff), flush=True)
    print()


def thinned(torch, wl, reps):
    """How much of a step is the operate stage: the same layer on the same mapping with every row cut down to a part of
    its nonzeros, down to none.  What remains with none is the exchange of h, the reduction and the epilogue."""
    import copy
    print("## Step time against the part of every row's nonzeros kept (mapping and back-off fixed): what the operate stage costs\n")
    print("| shape | grid x block, lanes per row | all | 3/4 | 1/2 | 1/4 | none | operate stage = all - none | LDS bound of the operate stage (16 B per gather at the measured 152 TB/s, on the CUs the mapping uses) |")
    print("|---|---|---|---|---|---|---|---|---|")
    for name, opts in (("cfg3", dict(lanes_per_row=64, waves=9, grid=256, poll_delay=3)),
                       ("cfg5", dict(lanes_per_row=16, waves=4, fill_waves=8, grid=256, poll_delay=5)),
                       ("cfg2", dict(lanes_per_row=16, grid=32, xcd="one", poll_delay=1))):
        full = wl.make_config(name)
        got = []
        info = None
        for keep in (1.0, 0.75, 0.5, 0.25, 0.0):
            w = copy.copy(full)
            counts = ((full.row_ptr[1:] - full.row_ptr[:-1]) * keep).astype(np.int64)
            sel = np.concatenate([np.arange(a, a + n) for a, n in zip(full.row_ptr[:-1], counts)]) if counts.sum() else np.zeros(0, np.int64)
            w.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
            w.col_idx, w.val_bits = full.col_idx[sel.astype(np.int64)], full.val_bits[sel.astype(np.int64)]
            us, i = measure(torch, w, reps, **opts)
            info = info or i
            got.append(us)
        planes = 2 if full.batch == 8 else 1
        bound = full.nnz * 16.0 * planes / (152e12 * min(info["grid"], 256) / 256.0) * 1e6   # (the CUs the mapping uses)
        print("| %s | %d x %d, %d | %.2f | %.2f | %.2f | %.2f | %.2f | %.2f | %.2f |" % (
            name, info["grid"], info["block"], info["lanes_per_row"], got[0], got[1], got[2], got[3], got[4], got[0] - got[4], bound), flush=True)
    print()


def exchange(torch, wl, reps):
    """The hand-off alone: a matrix with no nonzeros at all (every row empty), so a step is publish, exchange of h,
    reduction of zeros and epilogue, against the number of workgroups that take part and the bytes of h."""
    from . import binding
    print("## The exchange alone (a matrix without nonzeros): microseconds per timestep against participants and bytes of h, T 256\n")
    print("| hidden | batch | h | grid x block | placement | us/step |")
    print("|---|---|---|---|---|---|")
    cases = [(2304, 4, dict(grid=256, waves=9, lanes_per_row=64, xcd="spread")),
             (2304, 4, dict(grid=128, waves=9, lanes_per_row=32, xcd="spread")),
             (2304, 4, dict(grid=64, waves=9, lanes_per_row=16, xcd="spread")),
             (2304, 4, dict(grid=32, waves=9, lanes_per_row=8, xcd="spread")),
             (2304, 4, dict(grid=32, waves=9, lanes_per_row=8, xcd="one")),
             (2304, 4, dict(grid=16, waves=9, lanes_per_row=4, xcd="one")),
             (256, 4, dict(grid=256, waves=1, lanes_per_row=64, xcd="spread")),
             (2304, 2, dict(grid=256, waves=9, lanes_per_row=64, xcd="spread")),
             (4096, 4, dict(grid=256, waves=8, lanes_per_row=32, xcd="spread")),
             (2304, 8, dict(grid=256, waves=9, lanes_per_row=64, xcd="spread"))]
    for H, B, opts in cases:
        w = wl.make_workload("x", "relu", H, B, 256, 0.0, seed=0)
        try:
            us, info = measure(torch, w, reps, **opts)
            print("| %d | %d | %d KB | %d x %d | %s | %.2f |" % (H, B, H * B * 4 // 1024, info["grid"], info["block"],
                                                             "one XCD" if info["one_xcd"] else "all XCDs", us), flush=True)
        except Exception as e:
            print("| %d | %d | %d KB | | refused: %s | |" % (H, B, H * B * 4 // 1024, e), flush=True)
    print()


def cells(torch, wl, reps):
    print("## Cells: hidden 1024, density 20 %, T 256\n")
    print("| cell | gate rows | batch | nonzeros | persistent us/step | grid x block | lanes/row | back-off |")
    print("|---|---|---|---|---|---|---|---|")
    for B in (4, 8):
        for cell in ("relu", "tanh", "lstm", "gru"):
            w = wl.make_workload("cells", cell, 1024, B, 256, 0.20, seed=0, gain=1.0 if cell in ("lstm", "gru") else 0.9)
            us, info = measure(torch, w, reps)
            print("| %s | %d | %d | %d | %.2f | %d x %d | %d | %d |" % (
                cell, w.rows // w.hidden, B, w.nnz, us, info["grid"], info["block"], info["lanes_per_row"], info["poll_delay"]), flush=True)
    print()


def training(torch, wl, reps):
    from . import binding
    print("## Training step: hidden 1024, density 20 %, T 256 (microseconds per timestep of each launch)\n")
    print("| cell | batch | forward | backward through time | weight gradient | backward with weight gradient fused in | backward grid x block |")
    print("|---|---|---|---|---|---|---|")
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for B in (4, 8):
        for cell in ("relu", "lstm", "gru"):
            w = wl.make_workload("train", cell, 1024, B, 256, 0.20, seed=0, gain=0.9 if cell == "relu" else 1.0)
            H, T = w.hidden, w.steps
            x = dev(w.x)
            e = torch.randn((T, B, H), device="cuda")
            t_csr = binding.transpose_csr(w.rows, H, w.row_ptr, w.col_idx, w.val_bits)
            fused = None
            with binding.SparseRNN(H, B, cell, w.row_ptr, w.col_idx, w.val_bits) as fwd, \
                    binding.SparseRNN(H, B, {"lstm": "lstm_backward", "gru": "gru_backward"}.get(cell, cell), *t_csr) as bwd:
                if cell == "lstm":
                    f_us = _time_us_per_step(torch, lambda: fwd.forward_lstm_train(x), T, reps)
                    h, c, g = fwd.forward_lstm_train(x)
                    b_us = _time_us_per_step(torch, lambda: bwd.backward_lstm(e, g, c), T, reps)
                    d = bwd.backward_lstm(e, g, c)[0]
                    try:
                        fused = _time_us_per_step(torch, lambda: bwd.backward_lstm_with_weights(e, g, c, h), T, reps)
                    except binding.SprnnError:
                        pass
                elif cell == "gru":
                    b_hn = dev(w.b_hn)
                    f_us = _time_us_per_step(torch, lambda: fwd.forward_gru_train(x, b_hn), T, reps)
                    h, g = fwd.forward_gru_train(x, b_hn)
                    b_us = _time_us_per_step(torch, lambda: bwd.backward_gru(e, g, h), T, reps)
                    d = bwd.backward_gru(e, g, h)[1]          # the recurrent sums' gradient feeds the weight gradient
                    try:
                        fused = _time_us_per_step(torch, lambda: bwd.backward_gru_with_weights(e, g, h), T, reps)
                    except binding.SprnnError:
                        pass
                else:
                    h = fwd.forward(x)
                    f_us = _time_us_per_step(torch, lambda: fwd.forward(x, None, h), T, reps)
                    b_us = _time_us_per_step(torch, lambda: bwd.backward(e, h), T, reps)
                    d = bwd.backward(e, h)[0]
                    try:
                        fused = _time_us_per_step(torch, lambda: bwd.backward_with_weights(e, h), T, reps)
                    except binding.SprnnError:
                        pass
                w_us = _time_us_per_step(torch, lambda: fwd.weight_gradient(d, h), T, reps)
                if fwd.check() != 0 or bwd.check() != 0:
                    raise RuntimeError("spin watchdog tripped")
                bi = bwd.info()
            print("| %s | %d | %.2f | %.2f | %.2f | %s | %d x %d |" % (
                cell, B, f_us, b_us, w_us, "-" if fused is None else "%.2f" % fused, bi["grid"], bi["block"]), flush=True)
    print()


def casestudy(torch, wl, reps):
    print("## Case-study layer shapes (cf. Appendix B, both tables): random unstructured pattern, T 256\n")
    print("| layer | cell | hidden | density | batch | persistent us/step | ms per 256 steps | per-timestep launches ms | paper's sparse persistent ms (V100, its batch) | grid x block | lanes/row |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    nmt = [(256, 0.125, 0.33), (512, 0.0625, 0.37), (768, 0.0417, 0.48), (1024, 0.047, 0.55), (1024, 0.125, 0.63), (1448, 0.047, 0.78)]
    ds2 = [(1760, 0.12, 0.72), (2560, 0.12, 0.89), (3072, 0.12, 0.94)]
    cases = [("translation", "lstm", H, d, B, ms) for (H, d, ms) in nmt for B in (1, 4)] + \
            [("speech", "relu", H, d, B, ms) for (H, d, ms) in ds2 for B in (1, 8)]
    for (what, cell, H, dens, B, paper_ms) in cases:
        w = wl.make_workload("case", cell, H, B, 256, dens, seed=0, gain=1.0 if cell == "lstm" else 0.9)
        us, info = measure(torch, w, reps)
        st, _ = measure(torch, w, reps, stepwise=True)
        print("| %s | %s | %d | %.2f %% | %d | %.2f | %.3f | %.2f | %.2f | %d x %d | %d |" % (
            what, cell, H, 100 * dens, B, us, us * 256e-3, st * 256e-3, paper_ms, info["grid"], info["block"], info["lanes_per_row"]), flush=True)
    print()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--what", default="ablation,density,size,constnnz,batch,steps,placement,activations,thinned,exchange,cells,training,casestudy")
    ap.add_argument("--reps", type=int, default=8)
    ap.add_argument("--rung", default="", help="with --what rung: naive | wide | bank_aware | tagged | pool | two_part | spread32 | one_xcd32")
    ap.add_argument("--config", default="cfg2", help="with --what rung: the configuration")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("sweep: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    from . import workloads as wl
    what = args.what.split(",")
    if "rung" in what:
        one_rung(torch, wl, args.reps, args.config, args.rung)
    if "ablation" in what:
        ablation(torch, wl, args.reps)
    if "density" in what:
        axis(torch, wl, args.reps, "Density (cf. Section 5.2, first sweep): hidden 1792, batch 4, T 256",
             [(1792, 4, d, 256) for d in (0.01, 0.05, 0.10, 0.20, 0.30)])
    if "size" in what:
        axis(torch, wl, args.reps, "Layer size (cf. Sections 5.2 and 5.3): density 10 %, batch 4, T 256",
             [(H, 4, 0.10, 256) for H in (1024, 1792, 2304, 3072, 4096, 5120)] + [(5760, 2, 0.10, 256), (11520, 1, 0.01, 256)])
    if "constnnz" in what:
        axis(torch, wl, args.reps, "Constant number of nonzeros (cf. Section 5.3): about 1.32 M, batch 4, T 256",
             [(2304, 4, 0.25, 256), (3072, 4, 0.14, 256), (4096, 4, 0.079, 256), (5760, 4, 0.04, 256), (7168, 4, 0.026, 256),
              (11520, 4, 0.01, 256)])
    if "placement" in what:
        placement(torch, wl, args.reps)
    if "activations" in what:
        activations(torch, wl, args.reps)
    if "thinned" in what:
        thinned(torch, wl, args.reps)
    if "exchange" in what:
        exchange(torch, wl, args.reps)
    if "cells" in what:
        cells(torch, wl, args.reps)
    if "training" in what:
        training(torch, wl, args.reps)
    if "casestudy" in what:
        casestudy(torch, wl, args.reps)
    if "batch" in what:
        axis(torch, wl, args.reps, "Batch size: hidden 1792, density 10 %, T 256", [(1792, B, 0.10, 256) for B in (1, 2, 4, 8)])
    if "steps" in what:
        axis(torch, wl, args.reps, "Timesteps: hidden 1792, batch 4, density 10 %", [(1792, 4, 0.10, T) for T in (16, 64, 256, 1024)])


if __name__ == "__main__":
    main()
