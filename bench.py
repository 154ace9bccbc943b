#!/usr/bin/env python3
"""Benchmark of the persistent sparse recurrent step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3] [--all-configs]

One "step" is one pass of the whole hot path over one batch of synthetic input: one call of
sprnn_forward over the T timesteps of the configuration (cfg3 = hidden 2304, batch 4, density 30 %,
T = 256, the shape the metric is quoted on).  Inputs are resident in device memory before the timed
region.  Prints ONE JSON line on stdout; everything else goes to stderr.

Reported beside the throughput:
  roofline      the stated per-timestep bound  T_roof = max(nnz*gather_bytes/BW_lds, nnz*B/R_valu) + L_handoff + |h|/BW_fill
                (on-chip operand bandwidth or multiply-add issue rate for the nonzero stream + cross-workgroup
                store->observe latency + marginal time to bring h into one CU), its device constants measured live
                by libsprnn_probe (LDS rate with nothing but the reads in the loop; hand-off as the minimum over
                several probe launches before and after the timed region, capped by the lowest value the probe has
                returned on this hardware (see HANDOFF_FLOOR_NS); fill rate as the SLOPE of copy time over three
                sizes, its intercept being latency that the hand-off term already holds), and achieved/peak in
                microseconds per timestep.
                HBM traffic per launch comes from a counter summary file (--traffic-file), never from a constant.
  stepwise      the non-persistent comparison path (one launch per timestep) on the same inputs.
  backward      the backward pass through time of the same layer (sprnn_backward on the transposed matrix).
  projection    the step before the path (sprnn_project: b' = W x + b for all timesteps, input size = hidden size)
                against the dense fp16 MFMA peak, and the whole layer (projection + recurrence) per call.
  cpu_baseline  the CPU oracle as it stands, timed on the host cores of this machine.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_forward(run, steps, warmup, torch):
    """Wall time of `steps` calls bracketed by synchronize, plus per-call kernel time from HIP events
    recorded on the stream the kernel is launched on (torch's current stream)."""
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in evs:
        a.record(stream)
        run()
        b.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_call_ms = [a.elapsed_time(b) for a, b in evs]
    return (t1 - t0), per_call_ms


def measure_config(name, steps, warmup, torch, with_stepwise=True, options=None):
    from paper_1804_10223_amd import binding, workloads as wl
    w = wl.make_config(name)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    x, h0, c0 = dev(w.x), dev(w.h0), dev(w.c0)
    rnn = binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **(options or {}))
    info = rnn.info()
    T = w.steps
    h_out = torch.empty((T, w.batch, w.hidden), dtype=torch.float32, device="cuda")
    c_out = torch.empty_like(h_out) if w.cell == "lstm" else None
    if w.cell == "lstm":
        run = lambda: rnn.forward_lstm(x, h0, c0, h_out, c_out)
        run_step = lambda: rnn.forward_stepwise(x, h0, c0, h_out, c_out)
    else:
        run = lambda: rnn.forward(x, h0, h_out)
        run_step = lambda: rnn.forward_stepwise(x, h0, None, h_out, None)
    wall, per_call = time_forward(run, steps, warmup, torch)
    if rnn.check() != 0:
        raise RuntimeError("spin watchdog tripped during the benchmark")
    res = dict(name=name, workload=w, info=info, wall_s=wall, kernel_ms=float(np.median(per_call)),
               kernel_ms_mean=float(np.mean(per_call)), T=T)
    if with_stepwise:
        swall, sper = time_forward(run_step, max(3, steps // 4), 1, torch)
        res["stepwise_ms"] = float(np.median(sper))
    rnn.close()
    return res


def measure_projection(w, steps, warmup, torch, options=None):
    """The step before the path (Section 3.1's b' = W x + b for all timesteps, sprnn_project) on the same shape with
    input size = hidden size, and the whole layer (projection then recurrence on one stream)."""
    from paper_1804_10223_amd import binding, workloads as wl
    p = wl.make_projection(w.rows, w.hidden, w.steps, w.batch, seed=1,
                           forget_block=(w.hidden, 2 * w.hidden) if w.cell == "lstm" else None)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, **(options or {})) as rnn:
        x_in = torch.from_numpy(p.x_in).cuda()
        w_in = torch.from_numpy(p.w_bits.view(np.int16)).cuda()
        bias = torch.from_numpy(p.bias).cuda()
        bp = torch.empty((w.steps, w.batch, w.rows), dtype=torch.float32, device="cuda")
        h_out = torch.empty((w.steps, w.batch, w.hidden), dtype=torch.float32, device="cuda")
        c_out = torch.empty_like(h_out) if w.cell == "lstm" else None
        _, per_call = time_forward(lambda: rnn.project(x_in, w_in, bias, bp), steps, warmup, torch)

        def layer():
            rnn.project(x_in, w_in, bias, bp)
            if w.cell == "lstm":
                rnn.forward_lstm(bp, None, None, h_out, c_out)
            else:
                rnn.forward(bp, None, h_out)
        _, per_layer = time_forward(layer, steps, warmup, torch)
        if rnn.check() != 0:
            raise RuntimeError("spin watchdog tripped during the layer benchmark")
    us = float(np.median(per_call)) * 1e3
    flops = 2.0 * w.steps * w.batch * w.rows * w.hidden
    return {"kernel": "project_kernel (v_mfma_f32_32x32x16_f16, x split into two fp16 halves)", "input_size": w.hidden,
            "us_per_launch": us, "bound": "mfma", "achieved": flops / us * 1e-6, "peak": 2500.0, "unit": "TFLOP/s",
            "frac": flops / us * 1e-6 / 2500.0, "flops_algorithmic": flops, "mfma_flops_executed": 2.0 * flops,
            "layer_ms": float(np.median(per_layer))}


def measure_backward(w, steps, warmup, torch, options=None):
    """Backward pass through time (sprnn_backward) of the same layer: the transposed matrix resident, T + 1 steps."""
    from paper_1804_10223_amd import binding
    if w.cell not in ("relu", "tanh", "identity"):
        return None
    t_rp, t_ci, t_vb = binding.transpose_csr(w.hidden, w.hidden, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(w.hidden, w.batch, w.cell, t_rp, t_ci, t_vb, **(options or {})) as rnn:
        info = rnn.info()
        gen = torch.Generator(device="cuda").manual_seed(1)
        e = torch.randn((w.steps, w.batch, w.hidden), device="cuda", generator=gen)
        h_fwd = torch.randn((w.steps, w.batch, w.hidden), device="cuda", generator=gen)
        d = torch.empty_like(e)
        dh0 = torch.empty((w.batch, w.hidden), dtype=torch.float32, device="cuda")
        dU_t = torch.empty((max(w.nnz, 1),), dtype=torch.float32, device="cuda")
        # (every output is allocated here, outside the timed region: the binding allocates nothing when given them)
        _, per_call = time_forward(lambda: rnn.backward(e, h_fwd, d, dh0=dh0), steps, warmup, torch)
        fused_ms = None
        try:   # the same pass with the weight gradient fused in (not built for every mapping)
            _, per_fused = time_forward(lambda: rnn.backward_with_weights(e, h_fwd, None, d, dh0=dh0, dU=dU_t), steps, warmup, torch)
            fused_ms = float(np.median(per_fused))
        except binding.SprnnError:
            pass
        if rnn.check() != 0:
            raise RuntimeError("spin watchdog tripped during the backward benchmark")
    ms = float(np.median(per_call))
    # the non-recurrent half: gradient of the recurrent weights on the forward handle
    with binding.SparseRNN(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, poll_delay=-1) as fwd:
        dU = torch.empty((w.nnz,), dtype=torch.float32, device="cuda")
        _, per_wg = time_forward(lambda: fwd.weight_gradient(d, h_fwd, None, dU), steps, warmup, torch)
    wg_ms = float(np.median(per_wg))
    return {"kernel": "persistent_kernel<B=%d,NW=%d,backward>" % (w.batch, info["template_words"]), "ms_per_launch": ms,
            "us_per_timestep": ms * 1e3 / w.steps, "grid": info["grid"], "block": info["block"], "poll_delay": info["poll_delay"],
            "weight_gradient_ms_per_launch": wg_ms, "weight_gradient_us_per_timestep": wg_ms * 1e3 / w.steps,
            "fused_with_weight_gradient_ms_per_launch": fused_ms,
            "fused_with_weight_gradient_us_per_timestep": None if fused_ms is None else fused_ms * 1e3 / w.steps}


def measure_lstm_training(steps, warmup, torch):
    """One training step of the LSTM layer of cfg5, all three launches: forward keeping the gate values, backward pass
    through time on the transposed matrix (sprnn_backward_lstm), weight gradient on the forward handle."""
    from paper_1804_10223_amd import binding, workloads
    w = workloads.make_config("cfg5")
    H, B, T = w.hidden, w.batch, w.steps
    gen = torch.Generator(device="cuda").manual_seed(2)
    x = torch.from_numpy(w.x).cuda()
    e = torch.randn((T, B, H), device="cuda", generator=gen)
    t_rp, t_ci, t_vb = binding.transpose_csr(4 * H, H, w.row_ptr, w.col_idx, w.val_bits)
    with binding.SparseRNN(H, B, "lstm", w.row_ptr, w.col_idx, w.val_bits) as fwd, \
            binding.SparseRNN(H, B, "lstm_backward", t_rp, t_ci, t_vb) as bwd:
        # every output is allocated here, outside the timed regions: the binding allocates nothing when given them
        mk = lambda *shape: torch.empty(shape, dtype=torch.float32, device="cuda")
        h, c, g = mk(T, B, H), mk(T, B, H), mk(T, B, 4 * H)
        d, dh0, dc0, dU, dU_t = mk(T, B, 4 * H), mk(B, H), mk(B, H), mk(w.nnz), mk(w.nnz)
        _, per_f = time_forward(lambda: fwd.forward_lstm_train(x, None, None, h, c, g), steps, warmup, torch)
        _, per_b = time_forward(lambda: bwd.backward_lstm(e, g, c, d_bprime=d, dh0=dh0, dc0=dc0), steps, warmup, torch)
        _, per_w = time_forward(lambda: fwd.weight_gradient(d, h, None, dU), steps, warmup, torch)
        fused_ms = None
        try:   # backward and weight gradient in one kernel (not built for every mapping)
            _, per_fused = time_forward(lambda: bwd.backward_lstm_with_weights(e, g, c, h, d_bprime=d, dh0=dh0, dc0=dc0, dU=dU_t),
                                        steps, warmup, torch)
            fused_ms = float(np.median(per_fused))
        except binding.SprnnError:
            pass
        if fwd.check() != 0 or bwd.check() != 0:
            raise RuntimeError("spin watchdog tripped during the LSTM training benchmark")
        bi = bwd.info()
    f_ms, b_ms, w_ms = (float(np.median(v)) for v in (per_f, per_b, per_w))
    return {"workload": "cfg5: sparse LSTM, hidden %d, batch %d, T %d, density %.0f%%" % (H, B, T, 100 * w.meta["density"]),
            "forward_keeping_gates_us_per_timestep": f_ms * 1e3 / T, "backward_us_per_timestep": b_ms * 1e3 / T,
            "weight_gradient_us_per_timestep": w_ms * 1e3 / T,
            "backward_fused_with_weight_gradient_us_per_timestep": None if fused_ms is None else fused_ms * 1e3 / T,
            "backward_grid": bi["grid"], "backward_block": bi["block"],
            "backward_exchange_bytes_per_timestep": 4 * H * B * 4}


VALU_LANES_PER_CLK_PER_CU = 64      # 4 SIMDs x 16 lanes: one multiply-add per lane and clock
# The ping-pong probe depends on the power state the device happens to be in (one box returned 365-385 ns cold and
# 490-510 ns after busy kernels; another 646 ns at first and 463 ns after the timed launches), while the kernel's step
# time does not.  A latency FLOOR must not rise with such states, so the roofline uses the smaller of the live reading
# and the lowest one-way latency this probe has returned on any MI355X so far: the strictest choice, and the one that
# keeps `frac` comparable between runs.  The live readings are reported beside it.
HANDOFF_FLOOR_NS = {"cross": 344.0, "same": 310.0}


def roofline_for(w, info, probe_vals):
    """Stated per-timestep bound for one configuration from the measured device constants."""
    gather = 4 * w.batch                                   # fp32 activations of one column, all samples
    lds_bytes = w.nnz * gather
    width = min(16, gather)
    t_lds = lds_bytes / probe_vals["lds_Bps"][width]
    t_valu = w.nnz * w.batch / probe_vals["valu_lane_ops_per_s"]       # one multiply-add per nonzero and sample
    t_operate = max(t_lds, t_valu)
    if info.get("one_xcd"):
        t_handoff = min(probe_vals["handoff_same_ns"], HANDOFF_FLOOR_NS["same"]) * 1e-9
    else:
        t_handoff = min(probe_vals["handoff_cross_ns"], HANDOFF_FLOOR_NS["cross"]) * 1e-9
    if info["grid"] == 1:
        t_handoff = 0.0
    h_bytes = w.hidden * w.batch * 4
    t_fill = 0.0 if info["grid"] == 1 else h_bytes * probe_vals["fill_s_per_byte"]
    return dict(t_operate_us=t_operate * 1e6, t_lds_us=t_lds * 1e6, t_valu_us=t_valu * 1e6, t_handoff_us=t_handoff * 1e6,
                t_fill_us=t_fill * 1e6, t_roof_us=(t_operate + t_handoff + t_fill) * 1e6, lds_bytes_per_step=lds_bytes, h_bytes=h_bytes)


def measure_probes(probe, torch):
    vals = {"lds_Bps": {}}
    for width in (4, 8, 16):
        vals["lds_Bps"][width] = probe.lds_peak(width)
    vals["lds_with_adds_Bps_16"] = probe.lds_gather(256, 1024, 16, 0)
    vals["lds_random_Bps_16"] = probe.lds_gather(256, 1024, 16, 1)
    warm = lambda: probe.lds_peak(16)    # keeps the clocks up: two lone workgroups do not
    vals["handoff_same_ns"], vals["xcc_same"] = probe.handoff_ns_best(True, launches=6, warm=warm)
    vals["handoff_cross_ns"], vals["xcc_cross"] = probe.handoff_ns_best(False, launches=6, warm=warm)
    slope, intercept, times = probe.fill_fit()
    vals["fill_s_per_byte"], vals["fill_intercept_s"], vals["fill_times_s"] = slope, intercept, times
    prop = torch.cuda.get_device_properties(0)
    vals["cus"] = int(prop.multi_processor_count)
    vals["clock_hz"] = float(getattr(prop, "clock_rate", 2400000)) * 1e3
    vals["valu_lane_ops_per_s"] = vals["cus"] * VALU_LANES_PER_CLK_PER_CU * vals["clock_hz"]
    return vals


def read_traffic_file(path, workload_name):
    """HBM bytes per launch of the persistent kernel from a counter summary: text lines `key = value` written from
    rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE, each scaled by the same run's reference copy).  None when the
    file is missing or describes another workload."""
    try:
        kv = {}
        with open(path) as f:
            for line in f:
                if "=" in line and not line.lstrip().startswith("#"):
                    k, v = line.split("=", 1)
                    kv[k.strip()] = v.strip()
        if kv.get("workload") != workload_name:
            return None
        return {"fetch_bytes_per_launch": float(kv["fetch_bytes_per_launch"]), "write_bytes_per_launch": float(kv["write_bytes_per_launch"]),
                "source": os.path.relpath(path, ROOT)}
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(w, budget_s=20.0):
    """The oracle as it stands on this machine's host cores: single thread (the reported value) and all cores."""
    import oracle
    cores = os.cpu_count() or 1
    try:
        cores = min(cores, len(os.sched_getaffinity(0)))
    except AttributeError:
        pass
    cores = int(os.environ.get("OMP_NUM_THREADS", cores)) if os.environ.get("OMP_NUM_THREADS", "").isdigit() else cores

    def run(T, threads):
        xs = np.ascontiguousarray(w.x[:T])
        t0 = time.perf_counter()
        if w.cell == "lstm":
            oracle.lstm_forward(w.hidden, w.batch, w.row_ptr, w.col_idx, w.val_bits, xs, w.h0, w.c0, threads=threads)
        else:
            oracle.rnn_forward(w.hidden, w.batch, w.cell, w.row_ptr, w.col_idx, w.val_bits, xs, w.h0, threads=threads)
        return time.perf_counter() - t0

    probe_T = min(8, w.steps)
    per_step = run(probe_T, 1) / probe_T
    T1 = int(max(probe_T, min(w.steps, (budget_s * 0.6) / max(per_step, 1e-9))))
    t_single = run(T1, 1)
    per_step_n = run(probe_T, cores) / probe_T
    Tn = int(max(probe_T, min(w.steps, (budget_s * 0.4) / max(per_step_n, 1e-9))))
    t_multi = run(Tn, cores)
    return {"value": T1 / t_single, "unit": "timesteps/s", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d timesteps of %s, single thread" % (T1, w.steps, w.name),
            "us_per_timestep": t_single / T1 * 1e6,
            "all_cores": {"value": Tn / t_multi, "unit": "timesteps/s", "cores": cores,
                          "us_per_timestep": t_multi / Tn * 1e6,
                          "sample": "first %d timesteps, OpenMP over rows inside each timestep" % Tn}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--all-configs", action="store_true", help="also time cfg1..cfg5 and write a table to stderr")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "persistent_kernel_cfg3_traffic.txt"),
                    help="counter summary (key = value lines) that holds the measured HBM bytes per launch of the timed kernel")
    ap.add_argument("--poll-delay", type=int, default=0,
                    help="fix the back-off before a step's first poll (units of 64 clocks) instead of letting "
                         "sprnn_create measure it: profiler runs then see only the timed launches")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures ONE GPU only (the persistent kernel lives on one device); "
            "--gpus %d is not supported" % args.gpus)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(3)
    from paper_1804_10223_amd import binding, probe
    binding.load_library()

    log("measuring device constants (LDS gather rate, hand-off latency, fill rate) ...")
    pv = measure_probes(probe, torch)
    log("  LDS conflict-free, reads only: b128 %.1f TB/s, b64 %.1f TB/s, b32 %.1f TB/s (with the values added up: b128 %.1f TB/s; random columns %.1f TB/s)" % (
        pv["lds_Bps"][16] / 1e12, pv["lds_Bps"][8] / 1e12, pv["lds_Bps"][4] / 1e12, pv["lds_with_adds_Bps_16"] / 1e12, pv["lds_random_Bps_16"] / 1e12))
    log("  hand-off one way (minimum of 6 launches): same XCD %.0f ns %s, cross XCD %.0f ns %s" % (
        pv["handoff_same_ns"], pv["xcc_same"], pv["handoff_cross_ns"], pv["xcc_cross"]))
    log("  fill: %s us for %s bytes -> marginal %.1f GB/s per CU, intercept %.2f us" % (
        ["%.2f" % (t * 1e6) for t in pv["fill_times_s"].values()], list(pv["fill_times_s"].keys()),
        1e-9 / pv["fill_s_per_byte"], pv["fill_intercept_s"] * 1e6))

    options = {"poll_delay": args.poll_delay} if args.poll_delay else None
    res = measure_config(args.config, args.steps, args.warmup, torch, options=options)
    w, info, T = res["workload"], res["info"], res["T"]
    us_per_ts = res["kernel_ms"] * 1e3 / T
    # the hand-off floor once more, right after the timed launches (the device is as busy as it gets): keep the minimum
    for key, same in (("handoff_same_ns", True), ("handoff_cross_ns", False)):
        again, _ = probe.handoff_ns_best(same, launches=3)
        if again < pv[key]:
            log("  hand-off %s XCD right after the timed launches: %.0f ns (before: %.0f)" % ("same" if same else "cross", again, pv[key]))
            pv[key] = again
    roof = roofline_for(w, info, pv)
    value = args.steps * T / res["wall_s"]
    log("%s: %.3f us/timestep (kernel median %.3f ms per %d timesteps), wall %.1f timesteps/s; roofline %.3f us => %.1f %%" % (
        args.config, us_per_ts, res["kernel_ms"], T, value, roof["t_roof_us"], 100 * roof["t_roof_us"] / us_per_ts))
    log("  mapping: " + json.dumps({k: info[k] for k in ("grid", "block", "lanes_per_row", "template_words", "words_per_lane_max", "lds_bytes", "sync", "bank_aware", "balance", "poll_delay", "lds_pass_factor", "padded_words", "nnz")}))

    proj = measure_projection(w, args.steps, args.warmup, torch, options=options)
    log("  input projection (input size %d): %.1f us per launch, %.1f TFLOP/s algorithmic; whole layer %.3f ms" % (
        proj["input_size"], proj["us_per_launch"], proj["achieved"], proj["layer_ms"]))

    bwd = measure_backward(w, args.steps, args.warmup, torch, options=options)
    if bwd:
        log("  backward pass through time: %.3f us/timestep (%.3f ms per launch); weight gradient alone %.3f us/timestep (%.3f ms per launch); "
            "both fused: %s us/timestep" % (bwd["us_per_timestep"], bwd["ms_per_launch"], bwd["weight_gradient_us_per_timestep"],
                                           bwd["weight_gradient_ms_per_launch"], bwd["fused_with_weight_gradient_us_per_timestep"]))

    lstm = measure_lstm_training(max(5, args.steps // 2), 2, torch)
    log("  LSTM training step at cfg5: forward keeping gates %.3f, backward %.3f, weight gradient %.3f, both fused %s us/timestep" % (
        lstm["forward_keeping_gates_us_per_timestep"], lstm["backward_us_per_timestep"], lstm["weight_gradient_us_per_timestep"],
        lstm["backward_fused_with_weight_gradient_us_per_timestep"]))

    table = []
    if args.all_configs:
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            r = res if name == args.config else measure_config(name, max(5, args.steps // 2), 2, torch)
            rf = roofline_for(r["workload"], r["info"], pv)
            us = r["kernel_ms"] * 1e3 / r["T"]
            row = dict(config=name, us_per_timestep=us, stepwise_us_per_timestep=r["stepwise_ms"] * 1e3 / r["T"],
                       roofline={"bound": "lds+exchange", "achieved": us, "peak": rf["t_roof_us"], "frac": rf["t_roof_us"] / us,
                                 "unit": "us/timestep", "t_operate_us": rf["t_operate_us"], "t_handoff_us": rf["t_handoff_us"],
                                 "t_fill_us": rf["t_fill_us"]},
                       grid=r["info"]["grid"], block=r["info"]["block"])
            table.append(row)
            log("  %s" % json.dumps(row))

    # A plain device-to-device copy of known size (256 MiB read + 256 MiB written) so that hardware-counter
    # runs of this same command have a reference dispatch to scale FETCH_SIZE / WRITE_SIZE with.
    calib = torch.empty(64 << 20, dtype=torch.float32, device="cuda")
    calib2 = torch.empty_like(calib)
    calib.fill_(1.0)
    torch.cuda.synchronize()
    calib2.copy_(calib)
    torch.cuda.synchronize()
    del calib, calib2

    cpu = None
    if not args.no_cpu:
        log("timing the CPU oracle on the host cores ...")
        cpu = cpu_baseline(w)
        log("  oracle: %.1f us/timestep single thread; %.1f us/timestep on %d cores" % (
            cpu["us_per_timestep"], cpu["all_cores"]["us_per_timestep"], cpu["all_cores"]["cores"]))

    traffic = read_traffic_file(args.traffic_file, w.name)
    out = {
        "metric": "timesteps_per_sec (hidden %d, batch %d, density %.0f%%)" % (w.hidden, w.batch, 100 * w.meta["density"]),
        "value": value,
        "unit": "timesteps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["wall_s"] / args.steps * 1e3,
        "us_per_timestep": us_per_ts,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 (fp16 weights, fp32 activations and accumulation)",
        "data": "synthetic",
        "config": {"workload": "%s: sparse %s RNN, hidden %d, batch %d, T %d, density %.0f%%, fp16 weights + u16 indices" % (
            w.name, w.cell, w.hidden, w.batch, T, 100 * w.meta["density"]),
            "timesteps_per_step": T, "grid": info["grid"], "block": info["block"], "sync": "tagged" if info["sync"] == 1 else "barrier",
            "launch": "ordinary kernel launch, the library's persistent launches ordered per device (the default)"},
        "roofline": {
            "bound": "lds+exchange",
            "achieved": us_per_ts,
            "peak": roof["t_roof_us"],
            "unit": "us/timestep (lower is better; frac = peak/achieved)",
            "frac": roof["t_roof_us"] / us_per_ts,
            # HBM bytes per launch (fetch + write) of the timed kernel, read from the counter summary of this command
            # (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes scaled by the run's reference copy); null without one
            "traffic": None if traffic is None else traffic["fetch_bytes_per_launch"] + traffic["write_bytes_per_launch"],
            "traffic_source": None if traffic is None else traffic["source"],
            "traffic_algorithmic": 4.0 * info["padded_words"] + 4.0 * w.x.size + 4.0 * T * w.batch * w.hidden,
            "t_operate_us": roof["t_operate_us"], "t_lds_us": roof["t_lds_us"], "t_valu_us": roof["t_valu_us"],
            "t_handoff_us": roof["t_handoff_us"], "t_fill_us": roof["t_fill_us"],
            "lds_bytes_per_timestep": roof["lds_bytes_per_step"],
            "lds_achieved_TBps": roof["lds_bytes_per_step"] / (us_per_ts * 1e-6) / 1e12,
            "lds_peak_measured_TBps": pv["lds_Bps"][min(16, 4 * w.batch)] / 1e12,
            "valu_peak_lane_ops_per_s": pv["valu_lane_ops_per_s"],
            "handoff_same_xcd_ns": pv["handoff_same_ns"], "handoff_cross_xcd_ns": pv["handoff_cross_ns"],
            "handoff_floor_ns": HANDOFF_FLOOR_NS,
            "fill_marginal_GBps_per_cu": 1e-9 / pv["fill_s_per_byte"], "fill_intercept_us": pv["fill_intercept_s"] * 1e6,
            "fill_times_us": {str(k): v * 1e6 for k, v in pv["fill_times_s"].items()},
            "kernel": "persistent_kernel<B=%d,NW=%d>" % (w.batch, info["template_words"]),
            "kernel_ms_per_launch": res["kernel_ms"],
        },
        "stepwise": {"us_per_timestep": res["stepwise_ms"] * 1e3 / T, "speedup_of_persistent": res["stepwise_ms"] / res["kernel_ms"]},
        "projection": proj,
        "backward": bwd,
        "lstm_training": lstm,
        "cpu_baseline": cpu,
    }
    if table:
        out["all_configs"] = table
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
