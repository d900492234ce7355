#!/usr/bin/env python3
"""Benchmark of the CSB-RNN hot path on one MI355X.

Headline workload (BASELINE "configs[1]"): single-layer LSTM, input 153, hidden 512
(W 2048 x 665), CSB block 32 x 32, 10x pruning, batch 1, T = 100, synthetic, seed 0.
One "step" is one csb_rnn_forward over the whole T-frame sequence (pack / plan / upload
are done once, before the timed region, as the paper loads weights and instructions once
before streaming frames, Sec. 6.1).  The metric is microseconds per timestep (lower is
better) with the algorithmic GB/s beside it.

Also reported on the same JSON line:
  roofline      -- the dominant kernel of the headline workload
  streaming_path-- the same workload without the resident layout (weights re-streamed per step)
  rnn_configs   -- the other batch-1 workloads per timestep; csb_spmv on every RNN matrix, warm / cold
  spmv_stress   -- csb_spmv on the 8192 x 8192 heavy-tailed matrix (the HBM-bound case),
                   warm (matrix resident in the Infinity Cache) and cold (rotating over
                   distinct device copies of the matrix, > 512 MB in total), launches queued
                   behind a long kernel so that the host's call overhead does not show
  spmv_tall     -- the same on a matrix four times as tall (the streaming rate away from the
                   launch floor), next to a plain read of the same number of bytes
  batched       -- csb_spmm on the matrix cores (8192^2 x 128, cfg4 x 64) and the cfg4 model at batch 64
  projection, lstmp_sr1, cells, weights_16bit -- the rows built after the hot path
  cpu_baseline  -- the CPU oracle timed on this machine's host cores on the same workload
--only <leg> runs one leg alone and prints that leg's JSON (for rocprofv3 runs whose summaries
are kept under profiles/).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3


def load_traffic():
    """HBM-side bytes per launch of the roofline kernels, from the committed summary of the
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/hbm_traffic_pmc.txt: lines
    'traffic <key> read_bytes=<n> written_bytes=<n>', already scaled by the readings of a plain
    copy of known size; the file has the commands and the raw readings).  No file, no figure."""
    table = {}
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")) as f:
            for line in f:
                w = line.split()
                if len(w) >= 4 and w[0] == "traffic":
                    kv = dict(t.split("=", 1) for t in w[2:] if "=" in t)
                    table[w[1]] = int(float(kv["read_bytes"])) + int(float(kv["written_bytes"]))
    except (OSError, KeyError, ValueError):
        pass
    return table


TRAFFIC_BYTES = load_traffic()
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def spmv_alg_bytes(view, batch=1, value_bytes=4):
    """Algorithmic bytes of one CSB mat-vec: values (4 bytes, or 2 in a 16-bit format), one byte
    per row/column index, two count bytes per block, x read once, y written once."""
    nb = int(view["nbr"]) * int(view["nbc"])
    return (value_bytes * int(view["nnz"]) + len(view["rowidx"]) + len(view["colidx"]) + 2 * nb
            + 4 * int(view["cols"]) * batch + 4 * int(view["rows"]) * batch)


def rnn_step_alg_bytes(views, cell, hidden, batch=1):
    G = 4 if cell == 0 else 3
    total = 0
    for v in views:
        total += spmv_alg_bytes(v, batch) + 4 * G * hidden + 8 * hidden * batch + 4 * hidden * batch
    return total


def time_region(fn, reps, torch):
    """Milliseconds for `reps` calls of fn on the current stream, HIP events on that stream."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop)


def graph_replay_ms(fn, reps, torch):
    """Milliseconds per replay of `fn` captured once into a HIP graph (fn must be launches only
    and have run once before, so that nothing is set up inside the capture)."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        fn()
    torch.cuda.synchronize()
    graph.replay()
    return time_region(graph.replay, reps, torch) / reps


def time_each(fn, reps, torch):
    """One event pair per repetition: (median, min) in ms."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    torch.cuda.synchronize()
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2], ts[0]


_blocker = {}


def time_queued(calls, reps, torch):
    """Microseconds per call with every launch queued behind a long kernel, so that the host's
    launch rate (several microseconds per call from Python) does not show: two large matrix
    products go first, the start event sits behind them, and by the time they end the
    launches are all in the queue.  HIP events on the current stream."""
    if "a" not in _blocker:
        _blocker["a"] = torch.randn(6144, 6144, device="cuda")
        _blocker["c"] = torch.empty(6144, 6144, device="cuda")
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    torch.mm(_blocker["a"], _blocker["a"], out=_blocker["c"])
    torch.mm(_blocker["a"], _blocker["a"], out=_blocker["c"])
    start.record()
    for _ in range(reps):
        for c in calls:
            c()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1000.0 / (reps * len(calls))


def stream_read_leg(torch, stream_read):
    """Measured HBM read bandwidth of this GPU: a plain streaming read of 2 GiB (8 x the
    Infinity Cache), the practical roofline the mat-vec figures are also quoted against."""
    buf = torch.ones(512 * 1024 * 1024, dtype=torch.float32, device="cuda")
    out = stream_read(buf)
    for _ in range(2):
        stream_read(buf, out)
    n = 10
    ms = time_region(lambda: stream_read(buf, out), n, torch) / n
    gbps = buf.numel() * 4 / (ms * 1e-3) / 1e9
    del buf
    res = {"bytes": 512 * 1024 * 1024 * 4, "ms": round(ms, 4), "gbps": round(gbps, 1),
           "frac_of_nominal_peak": round(gbps / HBM_PEAK_GBS, 4)}
    return res


def plain_read_cold_us(torch, stream_read, nbytes, total=700e6):
    """A plain read of `nbytes` per launch, cold: distinct buffers in turn (more than 2 x the
    Infinity Cache in all), launches queued -- what one launch of that size costs when all it
    does is read."""
    n4 = max(64, int(nbytes) // 16)
    bufs = [torch.ones(n4 * 4, dtype=torch.float32, device="cuda") for _ in range(max(3, int(total / (n4 * 16)) + 1))]
    out = stream_read(bufs[0])
    for b in bufs:
        stream_read(b, out)
    us = time_queued([lambda b=b: stream_read(b, out) for b in bufs], 4, torch)
    return {"bytes": n4 * 16, "us": round(us, 3), "gbps": round(n4 * 16 / us / 1e3, 1), "buffers": len(bufs)}


ONLY = ["headline", "hbm_stream_read", "rnn_configs", "resident_batches", "spmv_stress", "spmv_cfg5", "spmv_tall",
        "batched", "spmm_cfg5", "projection", "lstmp_sr1", "cells", "weights_16bit", "spmv_cfg5_bf16", "spmm_bfloat",
        "calib_copy", "cpu_baseline"]


def only_leg(args, torch, np, csb_inputs, CsbMatrix, CsbRnn, stream_read):
    """One leg by name; legs that quote a fraction of the measured stream read run without it."""
    o = args.only
    if o == "hbm_stream_read":
        return stream_read_leg(torch, stream_read)
    if o == "rnn_configs":
        return rnn_configs_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, stream_read, None)
    if o == "resident_batches":
        return resident_batches_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn)
    if o == "spmv_stress":
        return stress_leg(torch, np, csb_inputs, CsbMatrix, stream_read)
    if o == "spmv_cfg5":          # cold launches of the default plan only
        return stress_leg(torch, np, csb_inputs, CsbMatrix, stream_read, names=("cfg5",), modes=((0, "default_plan"),), cold_only=True)
    if o == "spmv_tall":
        return tall_leg(torch, np, csb_inputs, CsbMatrix, stream_read)
    if o == "batched":
        return batched_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn)
    if o == "spmm_cfg5":
        return batched_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, cases=(("cfg5", 128),), with_rnn=False)
    if o == "projection":
        return projection_leg(torch, np, None, False)
    if o == "lstmp_sr1":
        return lstmp_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, not args.no_cpu)
    if o == "cells":
        return cells_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, not args.no_cpu)
    if o == "weights_16bit":
        return val16_leg(torch, np, csb_inputs, CsbMatrix, None)
    if o == "spmv_cfg5_bf16":
        return val16_leg(torch, np, csb_inputs, CsbMatrix, None, formats=("bf16",), cold_only=True, what=("spmv",))
    if o == "spmm_bfloat":
        return val16_leg(torch, np, csb_inputs, CsbMatrix, None, formats=("bf16",), what=("spmm_bfloat",))
    if o == "calib_copy":
        return calib_copy_leg(torch)
    if o == "cpu_baseline":
        cfg = csb_inputs.CONFIGS[args.workload]
        return cpu_leg(cfg, csb_inputs.make_rnn(cfg))
    raise ValueError(o)


def calib_copy_leg(torch):
    """Plain 256 MiB device copies: the known-size kernel that scales rocprofv3's FETCH_SIZE /
    WRITE_SIZE readings."""
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    return {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "launches": 5}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-stress", action="store_true", help="skip the 8192^2 SpMV stress leg")
    ap.add_argument("--only", default=None, choices=ONLY,
                    help="run one leg alone (its kernels are then the only ones of their kind in a rocprofv3 trace) "
                         "and print that leg's JSON; the contract line needs the default run")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run plain 256 MiB device copies: the known-size kernel that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(no collectives, no sharding in this path)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import csb_inputs
    from paper_2005_05758_amd import CsbMatrix, CsbRnn, stream_read

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.only and args.only != "headline":
        print(json.dumps({"only": args.only, args.only: only_leg(args, torch, np, csb_inputs, CsbMatrix, CsbRnn, stream_read)}))
        return
    cfg = csb_inputs.CONFIGS[args.workload]
    wl = csb_inputs.make_rnn(cfg)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, bias)
    rnn.upload()                      # resident layout: one launch runs all T steps
    views = [w.view() for w in Ws]
    xd = torch.from_numpy(wl.x).cuda()
    T, B = cfg.T, cfg.batch

    def step():
        rnn.forward(xd, want_hseq=True)

    for _ in range(args.warmup):
        step()
    ms = time_region(step, args.steps, torch)
    ms_per_step = ms / args.steps
    ms_median, ms_min = time_each(step, args.steps, torch)
    us_per_t = ms_per_step * 1000.0 / T
    bytes_step = rnn_step_alg_bytes(views, cfg.cell, cfg.hidden, B)
    gbps = bytes_step / (us_per_t * 1e-6) / 1e9

    # dominant kernel of the headline workload: the resident kernel IS the timed region (one
    # launch per sequence), so its launch duration is ms_per_step
    st = rnn.stats()
    ach = bytes_step * T / (ms_per_step * 1e-3) / 1e9
    roofline = {"kernel": f"csb::rnn_resident_kernel<{st['slots_per_lane']}, true>", "bound": "hbm",
                "achieved": round(ach, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 5),
                "traffic": TRAFFIC_BYTES.get("rnn_resident_cfg2") if args.workload == "cfg2" else None,
                "us_per_launch": round(ms_per_step * 1e3, 3), "alg_bytes_per_launch": bytes_step * T,
                "units_per_launch": T,
                "note": "weights stay in registers for all T steps (read from HBM once per launch); a step is "
                        "bound by the h_t exchange latency between workgroups, not by HBM: the figure is the "
                        "algorithmic bytes of T re-streamed mat-vecs over the launch time, as the metric defines it",
                "resident_plan": st,
                # the paper's own engine schedule on the same matrix, for context (Sec. 6.3.2: 4 x 4
                # PEGroups of 4 x 4 PEs); here every lane issues the same number of multiply-adds
                # and slot_fill is the share of them that is useful
                "paper_schedule_model": {k: round(v, 4) for k, v in Ws[0].sharing_model(4, 4, 4, 4).items()
                                         if k.startswith("eff_")}}

    # the same workload with the weights re-streamed every step (one mat-vec launch per step)
    Ws2 = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn2 = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws2, bias)
    for w in Ws2:
        w.upload()
    for _ in range(2):
        rnn2.forward(xd, want_hseq=True)
    ms2 = time_region(lambda: rnn2.forward(xd, want_hseq=True), 5, torch) / 5
    streaming = {"us_per_timestep": round(ms2 * 1000.0 / T, 3),
                 "gbps_algorithmic": round(bytes_step / (ms2 * 1e-3 / T) / 1e9, 2),
                 "note": "csb_rnn_forward without the resident layout: one csb spmv launch per step and layer, which also "
                         "finishes the cells of its units; timed in a loop over the same buffers, where the call replays "
                         "the HIP graph of its launches that the handle keeps"}
    # the same call captured once into a HIP graph and replayed (the streaming path is kernel
    # launches only: nothing in it depends on the host)
    ms3 = graph_replay_ms(lambda: rnn2.forward(xd, want_hseq=True), 5, torch)
    streaming["graph_replay_us_per_timestep"] = round(ms3 * 1000.0 / T, 3)

    out = {
        "metric": "us_per_timestep_csb_lstm_batch1",
        "value": round(us_per_t, 4),
        "unit": "us/timestep",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {'LSTM' if cfg.cell == 0 else 'GRU'} {cfg.input}->{cfg.hidden} x{cfg.n_layers}, "
                               f"W {wl.W[0].rows}x{wl.W[0].cols}, CSB block {cfg.block}, {cfg.rate:g}x pruning, "
                               f"batch {B}, T={T}, seed {cfg.seed}",
                   "timesteps_per_step": T, "alg_bytes_per_timestep": bytes_step},
        "us_per_timestep_median": round(ms_median * 1000.0 / T, 4),
        "us_per_timestep_min": round(ms_min * 1000.0 / T, 4),
        "gbps_algorithmic": round(gbps, 3),
        "pct_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBS, 4),
        "roofline": roofline,
        "streaming_path": streaming,
    }

    if args.calib_copy:
        out["calib_copy"] = calib_copy_leg(torch)
    if args.only == "headline":
        print(json.dumps(out))
        return
    if not args.no_stress:
        sr = stream_read_leg(torch, stream_read)
        out["hbm_stream_read"] = sr
        out["pct_of_measured_stream_read"] = round(100.0 * gbps / sr["gbps"], 4)
        out["rnn_configs"] = rnn_configs_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, stream_read, args.workload)
        out["resident_batches"] = resident_batches_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn)
        out["spmv_stress"] = stress_leg(torch, np, csb_inputs, CsbMatrix, stream_read, sr["gbps"])
        out["spmv_tall"] = tall_leg(torch, np, csb_inputs, CsbMatrix, stream_read)
        out["batched"] = batched_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn)
        out["projection"] = projection_leg(torch, np, sr["gbps"], not args.no_cpu)
        out["lstmp_sr1"] = lstmp_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, not args.no_cpu)
        out["cells"] = cells_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, not args.no_cpu)
        out["weights_16bit"] = val16_leg(torch, np, csb_inputs, CsbMatrix, sr["gbps"])
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_leg(cfg, wl)
    print(json.dumps(out))


def rnn_configs_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, stream_read, headline):
    """The other batch-1 workloads (the headline one is timed above): microseconds per timestep
    with the resident layout and streaming, and csb_spmv on the first layer's matrix of every
    batch-1 workload, warm (back to back) and cold (a 2 GiB streaming read between launches
    empties the caches; one event pair around each launch, median)."""
    res = {}
    flush = torch.ones(512 * 1024 * 1024, dtype=torch.float32, device="cuda")
    sink = stream_read(flush)
    for name in ("cfg1", "cfg2", "cfg3"):
        cfg = csb_inputs.CONFIGS[name]
        wl = csb_inputs.make_rnn(cfg)
        entry = {"workload": f"{'LSTM' if cfg.cell == 0 else 'GRU'} {cfg.input}->{cfg.hidden} x{cfg.n_layers}, block {cfg.block}, "
                             f"{cfg.rate:g}x, T={cfg.T}"}
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        views = [w.view() for w in Ws]
        bytes_step = rnn_step_alg_bytes(views, cfg.cell, cfg.hidden, 1)
        entry["alg_bytes_per_timestep"] = bytes_step
        if name != headline:
            bias = [torch.from_numpy(b).cuda() for b in wl.bias]
            xd = torch.from_numpy(wl.x).cuda()
            for mode in ("resident", "streaming"):
                rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, bias)
                if mode == "resident":
                    rnn.upload()
                else:
                    for w in Ws:
                        w.upload()
                for _ in range(5):
                    rnn.forward(xd, want_hseq=True)
                n = 30
                us = time_region(lambda: rnn.forward(xd, want_hseq=True), n, torch) * 1000.0 / (n * cfg.T)
                entry[f"{mode}_us_per_timestep"] = round(us, 3)
                entry[f"{mode}_gbps_algorithmic"] = round(bytes_step / us / 1e3, 1)
                del rnn
        M = CsbMatrix(wl.W[0].A, wl.W[0].br, wl.W[0].bc)
        M.plan()
        M.upload()
        ab = spmv_alg_bytes(M.view())
        x = torch.from_numpy(csb_inputs.make_vectors(5, wl.W[0].cols, 1)).cuda()
        y = torch.empty(wl.W[0].rows, dtype=torch.float32, device="cuda")
        for _ in range(10):
            M.spmv(x, y)
        us_warm = time_queued([lambda: M.spmv(x, y)] * 50, 4, torch)
        # cold: a 2 GiB read before every launch, one event pair around each launch; nothing waits
        # for the host in between (the read is long enough for the next calls to be queued)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(15)]
        torch.cuda.synchronize()
        for a, b in pairs:
            stream_read(flush, sink)
            a.record()
            M.spmv(x, y)
            b.record()
        torch.cuda.synchronize()
        cold = [a.elapsed_time(b) * 1000.0 for a, b in pairs]
        cold.sort()
        us_cold = cold[len(cold) // 2]
        entry["spmv_layer0"] = {"shape": [int(wl.W[0].rows), int(wl.W[0].cols)], "nnz": int(M.view()["nnz"]), "alg_bytes": ab,
                                "us_warm": round(us_warm, 2), "us_cold": round(us_cold, 2),
                                "gbps_cold": round(ab / us_cold / 1e3, 1)}
        res[name] = entry
    res["note"] = ("at these sizes a mat-vec launch is a fixed chain of dependent phases (about 3 us warm and 6.4 us "
                   "cold whatever the matrix holds; an empty launch takes 2.6): the resident kernel exists because of that")
    return res


def resident_batches_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn):
    """Batches of the batch-1 workloads: the sequences of a batch are independent, so a model that
    leaves XCDs free runs them as instances of the resident kernel side by side.  Per workload and
    batch: the path csb_rnn_forward picks by itself, and each of the two paths when named."""
    import os
    res = {}
    old = os.environ.get("CSB_RNN_BATCH_PATH")
    try:
        for name in ("cfg1", "cfg2", "cfg3", "cfg4"):
            cfg = csb_inputs.CONFIGS[name]
            wl = csb_inputs.make_rnn(cfg, batch=1)
            Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
            rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias])
            rnn.upload()
            for w in Ws:
                w.upload()
            entry = {"workgroups_per_instance": rnn.stats()["n_workgroups"], "T": cfg.T}
            for B in (8, 64):
                xd = torch.from_numpy(np.random.default_rng(B).uniform(-1, 1, (cfg.T, B, cfg.input)).astype(np.float32)).cuda()
                row = {}
                for path in ("resident", "batched", None):
                    if path is None:
                        os.environ.pop("CSB_RNN_BATCH_PATH", None)
                    else:
                        os.environ["CSB_RNN_BATCH_PATH"] = path
                    for _ in range(3):
                        rnn.forward(xd, want_hseq=True)
                    n = 10
                    ms = time_region(lambda: rnn.forward(xd, want_hseq=True), n, torch) / n
                    row[path or "picked"] = {"ms_per_batch": round(ms, 4), "us_per_timestep": round(ms * 1e3 / cfg.T, 3),
                                             "sequences_per_s": round(B / (ms * 1e-3))}
                entry[f"batch{B}"] = row
            # the resident layout planned for the batch (csb_rnn_plan_resident): smaller instances, fewer rounds
            os.environ["CSB_RNN_BATCH_PATH"] = "resident"
            for B in (8, 64):
                rnn.plan_resident(B)
                rnn.upload()
                st = rnn.stats()
                xd = torch.from_numpy(np.random.default_rng(B).uniform(-1, 1, (cfg.T, B, cfg.input)).astype(np.float32)).cuda()
                for _ in range(3):
                    rnn.forward(xd, want_hseq=True)
                n = 10
                ms = time_region(lambda: rnn.forward(xd, want_hseq=True), n, torch) / n
                entry[f"batch{B}"]["resident_planned_for_batch"] = {
                    "workgroups_per_instance": st["n_workgroups"], "slots_per_lane": st["slots_per_lane"],
                    "ms_per_batch": round(ms, 4), "us_per_timestep": round(ms * 1e3 / cfg.T, 3),
                    "sequences_per_s": round(B / (ms * 1e-3))}
            res[name] = entry
            del rnn
    finally:
        if old is None:
            os.environ.pop("CSB_RNN_BATCH_PATH", None)
        else:
            os.environ["CSB_RNN_BATCH_PATH"] = old
    return res


def wave_spread(stamps, np):
    """Largest / mean time a wavefront (a workgroup) spends multiplying, from the clock stamps of
    one launch: [workgroups][16 wavefronts][8 stamps] for the row-owned kernel (stamp 3 = first
    segment in LDS, 4 = products done), [workgroups][stamps] for the tile kernel."""
    sp = stamps.cpu().numpy().astype(np.float64)
    wv = sp[:, :, 4] - sp[:, :, 3] if sp.ndim == 3 else sp[:, 10::3] - sp[:, 8::3]
    wg = wv.max(axis=1)
    return round(float(wv.max() / wv.mean()), 4), round(float(wg.max() / wg.mean()), 4)


def stress_leg(torch, np, csb_inputs, CsbMatrix, stream_read, stream_gbps=None, names=("cfg5", "cfg5_diag"),
               modes=((0, "default_plan"), (2, "equal_split")), cold_only=False):
    """csb_spmv on the 8192^2 heavy-tailed matrices (the HBM-bound case): warm (matrix in the
    Infinity Cache) and cold (rotating over distinct device copies, > 512 MB in all), for
    the default plan (row-owned layout) and the tile-based equal-split plan (mode 2).  Launches
    are queued behind a long kernel, so the figures are the device's, not the host's."""
    res = {}
    for name in names:
        m = csb_inputs.make_mat(csb_inputs.CONFIGS[name])
        x = torch.from_numpy(csb_inputs.make_vectors(5, m.cols, 1)).cuda()
        y = torch.empty(m.rows, dtype=torch.float32, device="cuda")
        for mode, tag in modes:
            M = CsbMatrix(m.A, m.br, m.bc)
            st = M.plan(0, mode)
            M.upload()
            v = M.view()
            ab = spmv_alg_bytes(v)
            entry = {"nnz": int(v["nnz"]), "alg_bytes": ab,
                     "kernel": (f"csb::spmv_rows_kernel<2, 0, {1 if st['rounds'] > 1 else 0}>" if st["row_owned"]
                                else "csb::spmv_kernel<0, false>"),
                     "image_bytes_per_launch": int(st["matvec_bytes"]),
                     "image_over_algorithmic": round(st["matvec_bytes"] / ab, 4),
                     "wave_max_over_mean": round(st["work_max"] / st["work_mean"], 4),
                     "workgroup_max_over_mean": round(st["chunk_max_over_mean"], 4),
                     "nosplit_max_over_mean": round(st["nosplit_max_over_mean"], 4),
                     "lane_fill": round(st["lane_fill"], 4), "n_chunks": st["n_chunks"], "rounds": st["rounds"],
                     "shared_tiles": st["n_shared_tiles"]}
            if not cold_only:
                for _ in range(10):
                    M.spmv(x, y)
                us_warm = time_queued([lambda: M.spmv(x, y)] * 20, 5, torch)
                # dynamic balance: clocks each wavefront spends on its share (stamps of one launch)
                _, stamps = M.spmv_stamps(x)
                torch.cuda.synchronize()
                dw, dg = wave_spread(stamps, np)
                entry.update({"us_warm": round(us_warm, 3), "gbps_warm": round(ab / us_warm / 1e3, 1),
                              "dyn_wave_max_over_mean": dw, "dyn_workgroup_max_over_mean": dg})
                if mode == 0:
                    # the paper's own schedule on the same matrix (4 x 4 PEGroups of 4 x 4 PEs, Sec. 6.3.2),
                    # next to this partition's efficiency (mean / largest wavefront work)
                    sm = M.sharing_model(4, 4, 4, 4)
                    entry["paper_schedule_model"] = {k: round(v, 4) for k, v in sm.items() if k.startswith("eff_")}
                    entry["partition_efficiency"] = round(st["work_mean"] / st["work_max"], 4)
            if name == "cfg5":
                # cold: rotate over distinct device copies so that every launch streams from HBM
                copies = [M]
                n_copies = 24
                for _ in range(n_copies - 1):
                    c = CsbMatrix(m.A, m.br, m.bc)
                    c.plan(0, mode)
                    c.upload()
                    copies.append(c)
                for c in copies:
                    c.spmv(x, y)
                us_cold = time_queued([lambda c=c: c.spmv(x, y) for c in copies], 5, torch)
                entry.update({"us_cold": round(us_cold, 3), "gbps_cold": round(ab / us_cold / 1e3, 1),
                              "frac_hbm_cold": round(ab / us_cold / 1e3 / HBM_PEAK_GBS, 4),
                              "cold_copies": n_copies, "cold_bytes_total": n_copies * M.device_bytes()})
                if stream_gbps:
                    entry["frac_of_measured_stream_read_cold"] = round(ab / us_cold / 1e3 / stream_gbps, 4)
                if not cold_only:
                    # against a plain cold read of the same number of bytes in one launch
                    pr = plain_read_cold_us(torch, stream_read, st["matvec_bytes"])
                    entry["plain_read_of_image_size"] = pr
                    entry["plain_read_over_time"] = round(pr["us"] / us_cold, 3)
                del copies
            res[f"{name}_{tag}"] = entry
            del M
    colds = [e for k, e in res.items() if k.startswith("cfg5_") and "us_cold" in e]
    if colds:
        best = min(colds, key=lambda e: e["us_cold"])
        res["roofline"] = {"kernel": best["kernel"], "bound": "hbm", "achieved": best["gbps_cold"], "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": best["frac_hbm_cold"], "traffic": TRAFFIC_BYTES.get("spmv_cfg5"),
                           "us_per_launch": best["us_cold"], "alg_bytes_per_launch": best["alg_bytes"],
                           "note": "cold: every launch reads a different device copy of the matrix"}
    return res


def tall_leg(torch, np, csb_inputs, CsbMatrix, stream_read, rows=32768):
    """csb_spmv on a matrix four times as tall as the stress matrix (32768 x 8192, same block,
    rate and heavy-tailed recipe, seed 0): 95 MB of algorithmic bytes per launch, so the fixed
    part of a launch weighs a quarter as much and the figure shows the streaming rate."""
    cfg = csb_inputs.MatConfig("tall", rows, 8192, 32, 12.0, "heavy", 0.05, 0)
    m = csb_inputs.make_mat(cfg)
    x = torch.from_numpy(csb_inputs.make_vectors(5, m.cols, 1)).cuda()
    y = torch.empty(m.rows, dtype=torch.float32, device="cuda")
    copies = []
    for _ in range(7):
        c = CsbMatrix(m.A, m.br, m.bc)
        st = c.plan()
        c.upload()
        copies.append(c)
    for c in copies:
        c.spmv(x, y)
    ab = spmv_alg_bytes(copies[0].view())
    us_cold = time_queued([lambda c=c: c.spmv(x, y) for c in copies], 6, torch)
    us_warm = time_queued([lambda: copies[0].spmv(x, y)] * 8, 4, torch)
    pr = plain_read_cold_us(torch, stream_read, st["matvec_bytes"])
    return {"shape": [int(m.rows), int(m.cols)], "nnz": int(copies[0].view()["nnz"]), "alg_bytes": ab,
            "image_bytes_per_launch": int(st["matvec_bytes"]), "image_over_algorithmic": round(st["matvec_bytes"] / ab, 4),
            "n_chunks": st["n_chunks"], "rounds": st["rounds"], "row_owned": st["row_owned"],
            "wave_max_over_mean": round(st["work_max"] / st["work_mean"], 4),
            "us_cold": round(us_cold, 3), "gbps_cold": round(ab / us_cold / 1e3, 1),
            "frac_hbm_cold": round(ab / us_cold / 1e3 / HBM_PEAK_GBS, 4), "us_warm": round(us_warm, 3),
            "cold_copies": len(copies), "plain_read_of_image_size": pr, "plain_read_over_time": round(pr["us"] / us_cold, 3)}


def val16_leg(torch, np, csb_inputs, CsbMatrix, stream_gbps, formats=("f16", "bf16"), cold_only=False, what=("spmv", "spmm", "spmm_bfloat")):
    """csb_spmv and csb_spmm on the 8192^2 matrix with the kernel values stored in 16 bits
    (the paper's engine works on 16-bit weights): half the value bytes on the HBM-bound path.
    Cold as in the 32-bit leg (rotating device copies)."""
    from paper_2005_05758_amd import VAL_F16, VAL_BF16
    res = {}
    m = csb_inputs.make_mat(csb_inputs.CONFIGS["cfg5"])
    x = torch.from_numpy(csb_inputs.make_vectors(5, m.cols, 1)).cuda()
    y = torch.empty(m.rows, dtype=torch.float32, device="cuda")
    for fmt, name in ((VAL_F16, "f16"), (VAL_BF16, "bf16")):
        if name not in formats:
            continue
        n_copies = 40 if "spmv" in what else 1
        copies = []
        for _ in range(n_copies):
            c = CsbMatrix(m.A, m.br, m.bc)
            c.set_value_format(fmt)
            c.plan()
            c.upload()
            copies.append(c)
        M = copies[0]
        ab = spmv_alg_bytes(M.view(), value_bytes=2)
        for c in copies:
            c.spmv(x, y)
        entry = {"alg_bytes": ab, "device_bytes": M.device_bytes()}
        if "spmv" in what:
            if not cold_only:
                entry["us_warm"] = round(time_queued([lambda: M.spmv(x, y)] * 20, 5, torch), 3)
            us_cold = time_queued([lambda c=c: c.spmv(x, y) for c in copies], 4, torch)
            entry.update({"us_cold": round(us_cold, 3), "gbps_cold": round(ab / us_cold / 1e3, 1),
                          "frac_hbm_cold": round(ab / us_cold / 1e3 / HBM_PEAK_GBS, 4),
                          "cold_copies": n_copies, "cold_bytes_total": n_copies * M.device_bytes()})
            if stream_gbps:
                entry["frac_of_measured_stream_read_cold"] = round(ab / us_cold / 1e3 / stream_gbps, 4)
        if name == "bf16" and "spmm" in what:
            B = 128
            X = torch.from_numpy(csb_inputs.make_vectors(6, m.cols, B).reshape(m.cols, B)).cuda()
            Y = torch.empty((m.rows, B), dtype=torch.float32, device="cuda")
            for _ in range(3):
                M.spmm(X, Y)
            n = 20
            us = time_region(lambda: M.spmm(X, Y), n, torch) * 1000.0 / n
            nnz = int(M.view()["nnz"])
            entry["spmm_b128"] = {"us": round(us, 2), "tflops_algorithmic": round(2.0 * nnz * B / us / 1e6, 3),
                                  "note": "bfloat16 kernel values, float32 right-hand sides, f32 matrix cores (csb_spmm)"}
        if name == "bf16" and "spmm_bfloat" in what:
            # bfloat16 right-hand sides too: csb_spmm_bfloat on the bf16 matrix cores
            n = 20
            nnz = int(M.view()["nnz"])
            bf = {}
            for Bb in (128, 512):
                Xb = torch.from_numpy(csb_inputs.make_vectors(6, m.cols, Bb).reshape(m.cols, Bb)).cuda().to(torch.bfloat16)
                Yb = torch.empty((m.rows, Bb), dtype=torch.float32, device="cuda")
                for _ in range(3):
                    M.spmm_bfloat(Xb, Yb)
                us = time_region(lambda: M.spmm_bfloat(Xb, Yb), n, torch) * 1000.0 / n
                tf = 2.0 * nnz * Bb / us / 1e6
                bf[f"batch{Bb}"] = {"us": round(us, 2), "tflops_algorithmic": round(tf, 3)}
            tf = bf["batch512"]["tflops_algorithmic"]
            entry["spmm_bfloat"] = dict(bf, roofline={
                "kernel": "csb::spmm_reg16_kernel<16, 2, 2>", "bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s",
                "frac": round(tf / 2500.0, 5), "traffic": None,
                "note": "dense bf16 MFMA peak as the nominal roof; one 16-column MFMA step per block, part and tile of 16 "
                        "right-hand sides: the launch is bound by its loads and its instruction stream, not by the matrix cores"})
        res[f"spmv_cfg5_{name}"] = entry
        del copies, M
    return res


def batched_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, cases=(("cfg5", 128), ("cfg4", 64)), with_rnn=True):
    """The batched (matrix-core) path: csb_spmm on the 8192^2 matrix with 128 right-hand sides
    and on a cfg4 layer matrix with 64, then the whole cfg4 workload (2-layer LSTM, batch 64,
    T = 256) through csb_rnn_forward.  Flops are the algorithmic 2 * nnz * batch."""
    res = {}
    for name, batch in cases:
        if name == "cfg5":
            m = csb_inputs.make_mat(csb_inputs.CONFIGS[name])
        else:
            m = csb_inputs.make_rnn(csb_inputs.CONFIGS[name], T=1, batch=1).W[0]
        M = CsbMatrix(m.A, m.br, m.bc)
        M.plan()
        M.upload()
        X = torch.from_numpy(csb_inputs.make_vectors(5, m.cols, batch)).cuda()
        Y = torch.empty((m.rows, batch), dtype=torch.float32, device="cuda")
        for _ in range(3):
            M.spmm(X, Y)
        n = 20
        us = time_region(lambda: M.spmm(X, Y), n, torch) * 1000.0 / n
        v = M.view()
        fl = 2.0 * int(v["nnz"]) * batch
        # what the kernel's access pattern pulls through L2 -> L1: every block gathers the rows of X
        # of its own kept columns (no reuse inside a workgroup), plus the kernel values once
        gather = 4.0 * float(np.asarray(v["ncols"], dtype=np.int64).sum()) * batch + 4.0 * int(v["nnz"])
        res[f"spmm_{name}_b{batch}"] = {"shape": [int(m.rows), int(m.cols)], "nnz": int(v["nnz"]), "batch": batch,
                                        "us": round(us, 2), "tflops_algorithmic": round(fl / us / 1e6, 3),
                                        "frac_fp32_mfma_peak": round(fl / us / 1e6 / MFMA_F32_PEAK_TFLOPS, 4),
                                        "l2_gather_bytes": int(gather), "l2_gather_gbps": round(gather / us / 1e3, 1)}
        del M
    best = res.get("spmm_cfg5_b128")
    if best:
        res["roofline"] = {"kernel": "csb::spmm_reg_kernel<false, 16, 2, 0>", "bound": "mfma", "achieved": best["tflops_algorithmic"],
                           "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": best["frac_fp32_mfma_peak"],
                           "traffic": TRAFFIC_BYTES.get("spmm_cfg5_b128"),
                           "us_per_launch": best["us"], "flops_per_launch": 2.0 * best["nnz"] * best["batch"],
                           "note": "the matrix cores are the roof; counters (profiles/spmm_cfg5_b128_pmc.txt): the matrix pipe is "
                                   "busy about half of the launch, with 1.65 x the MFMAs of the kernel-row form (rows are "
                                   "scattered to their tile rows in the operand, which keeps the results in registers); the "
                                   "gather of X rows is not the bound (all gathers pointed at one row: 3 % faster)"}
    if not with_rnn:
        return res
    cfg = csb_inputs.CONFIGS["cfg4"]
    wl = csb_inputs.make_rnn(cfg)
    Ws = [CsbMatrix(w.A, w.br, w.bc) for w in wl.W]
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, bias)
    for w in Ws:
        w.upload()
    xd = torch.from_numpy(wl.x).cuda()
    rnn.forward(xd, want_hseq=False)
    n = 3
    ms = time_region(lambda: rnn.forward(xd, want_hseq=False), n, torch) / n
    fl_step = sum(2.0 * int(w.view()["nnz"]) * cfg.batch for w in Ws)
    res["rnn_cfg4"] = {"workload": f"{cfg.name}: {cfg.n_layers} x LSTM {cfg.input}->{cfg.hidden}, block {cfg.block}, "
                                   f"{cfg.rate:g}x, batch {cfg.batch}, T={cfg.T}",
                       "us_per_timestep": round(ms * 1000.0 / cfg.T, 2),
                       "tflops_algorithmic": round(fl_step / (ms * 1e-3 / cfg.T) / 1e12, 3),
                       "sequences_per_s": round(cfg.batch / (ms * 1e-3), 1),
                       "note": "the matrix-core path (csb_spmm per diagonal); the same workload as instances of the resident "
                               "kernel laid out for this batch is timed in resident_batches.cfg4.batch64"}
    # the same call captured into a HIP graph and replayed (kernel launches only)
    msg = graph_replay_ms(lambda: rnn.forward(xd, want_hseq=False), n, torch)
    res["rnn_cfg4"]["graph_replay_us_per_timestep"] = round(msg * 1000.0 / cfg.T, 2)
    return res


def projection_leg(torch, np, stream_gbps, with_cpu):
    """csb_project (RowPrune / ColumnPrune of Algorithm 1) on a dense 8192 x 8192 Gaussian matrix,
    block 32, 12x: the matrix the stress leg's shape comes from.  Algorithmic bytes: one read
    of W and one write of Z."""
    from paper_2005_05758_amd import project
    rows = cols = 8192
    rng = np.random.default_rng(0)
    Wh = rng.normal(0, 0.05, (rows, cols)).astype(np.float32)
    W = torch.from_numpy(Wh).cuda()
    Z = torch.empty_like(W)
    for _ in range(2):
        project(W, 32, 32, 12.0, out=Z)
    n = 10
    ms = time_region(lambda: project(W, 32, 32, 12.0, out=Z), n, torch) / n
    ab = 2 * rows * cols * 4
    res = {"shape": [rows, cols], "block": 32, "rate": 12.0, "ms": round(ms, 4), "alg_bytes": ab,
           "gbps_algorithmic": round(ab / (ms * 1e-3) / 1e9, 1),
           "roofline": {"kernel": "csb_project (5 kernels: row sums, select, column sums, select, masked copy)",
                        "bound": "hbm", "achieved": round(ab / (ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                        "frac_of_measured_stream_read": round(ab / (ms * 1e-3) / 1e9 / stream_gbps, 4) if stream_gbps else None},
           "density_out": round(float((Z != 0).float().mean()), 5)}
    if with_cpu:
        import oracle
        t0 = time.perf_counter()
        oracle.csb_project(Wh, 32, 32, 12.0)
        res["cpu_baseline"] = {"value": round((time.perf_counter() - t0) * 1e3, 1), "unit": "ms", "cores": 1, "kind": "oracle",
                               "sample": "one projection of the same matrix (single-threaded C: float32 sums, qsort per block-column / block-row)"}
    return res


def lstmp_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, with_cpu):
    """The shape of the paper's speech model SR1 (Table 1): two LSTMP layers, 153 -> 1024 and
    512 -> 1024 with a 512-wide projection, 13x in 32 x 32 blocks, synthetic weights.  Batch 1
    (one frame at a time: streaming, two CSB mat-vec launches per layer and frame; and resident) and batch 32
    on the matrix cores.  The paper's FPGA figure for its trained SR1 is 6.58 us per frame
    (another machine, 16-bit fixed point: context, not a baseline)."""
    from paper_2005_05758_amd import CELL_LSTMP
    res = {}
    for batch, T in ((1, 100), (32, 100)):
        wl = csb_inputs.make_lstmp(0, 2, 153, 1024, 512, 32, 13.0, T, batch)
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        Ps = [CsbMatrix(m.A, m.br, m.bc) for m in wl.Wp]
        bias = [torch.from_numpy(b).cuda() for b in wl.bias]
        rnn = CsbRnn(CELL_LSTMP, 153, 1024, Ws, bias, proj=512, Wp=Ps)
        for m in Ws + Ps:
            m.upload()
        xd = torch.from_numpy(wl.x).cuda()
        for _ in range(3):              # (steady state: a streaming call that repeats its arguments records its launches once)
            rnn.forward(xd, want_hseq=True)
        n = 3
        ms = time_region(lambda: rnn.forward(xd, want_hseq=True), n, torch) / n
        nnz = sum(int(m.view()["nnz"]) for m in Ws + Ps)
        key = f"batch{batch}" + ("_streaming" if batch == 1 else "")
        res[key] = {"us_per_frame": round(ms * 1000.0 / T, 2), "frames_per_s": round(batch * T / (ms * 1e-3), 1),
                    "nnz": nnz, "tflops_algorithmic": round(2.0 * nnz * batch / (ms * 1e-3 / T) / 1e12, 4)}
        if batch == 1:          # the same call replayed from a HIP graph (launches only)
            res[key]["graph_replay_us_per_frame"] = round(graph_replay_ms(lambda: rnn.forward(xd, want_hseq=True), n, torch) * 1000.0 / T, 2)
        if batch == 1:
            # the resident layout: one launch for the whole sequence
            rnn2 = CsbRnn(CELL_LSTMP, 153, 1024, [CsbMatrix(m.A, m.br, m.bc) for m in wl.W], bias, proj=512,
                          Wp=[CsbMatrix(m.A, m.br, m.bc) for m in wl.Wp])
            rnn2.upload()
            for _ in range(3):
                rnn2.forward(xd, want_hseq=True)
            n2 = 20
            ms2 = time_region(lambda: rnn2.forward(xd, want_hseq=True), n2, torch) / n2
            res["batch1_resident"] = {"us_per_frame": round(ms2 * 1000.0 / T, 3), "frames_per_s": round(T / (ms2 * 1e-3), 1),
                                      "resident_plan": rnn2.stats()}
        if with_cpu and batch == 1:
            import oracle
            W, Wp = [m.A for m in wl.W], [m.A for m in wl.Wp]
            t0 = time.perf_counter()
            reps = 0
            while time.perf_counter() - t0 < 5.0:
                oracle.lstmp_forward(W, Wp, wl.bias, wl.x, 153, 1024, 512)
                reps += 1
            res["cpu_baseline"] = {"value": round((time.perf_counter() - t0) / (reps * T) * 1e6, 2), "unit": "us/frame",
                                   "cores": oracle.num_threads(), "kind": "oracle",
                                   "sample": f"{reps} sequences of T={T}, batch 1 (float64 dense masked products + gates)"}
    return res


def cells_leg(torch, np, csb_inputs, CsbMatrix, CsbRnn, with_cpu):
    """The shapes of two more of the paper's speech models (Table 1), synthetic weights, batch 1:
    SR3 = two Li-GRU layers 39 -> 512 -> 512 at 7.1x (resident and streaming path), and SR2 =
    two GRU layers 39 -> 1024 -> 1024 at 21.7x in the reset-before form (two dependent CSB
    products per step) next to the reset-after form, each on the streaming and the resident path.  The
    paper's FPGA figure for its trained SR2 is 5.18 us per frame (context, not a baseline)."""
    from paper_2005_05758_amd import CELL_LIGRU, CELL_GRU_RB, CELL_GRU
    T = 100
    res = {}

    def timed(rnn, xd, n):
        for _ in range(2):
            rnn.forward(xd, want_hseq=True)
        return round(time_region(lambda: rnn.forward(xd, want_hseq=True), n, torch) / n * 1000.0 / T, 3)

    def cpu(cell, wl, I, H):
        import oracle
        W = [m.A for m in wl.W]
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 4.0:
            oracle.rnn_forward(cell, W, wl.bias, wl.x, I, H)
            reps += 1
        return {"value": round((time.perf_counter() - t0) / (reps * T) * 1e6, 2), "unit": "us/frame",
                "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"{reps} sequences of T={T}, batch 1 (float64 dense masked products + gates)"}

    # SR3 shape, Li-GRU
    cfg = csb_inputs.RnnConfig("sr3", csb_inputs.LIGRU, 2, 39, 512, 32, 7.1, "binomial", 0.05, 1, T, 0)
    wl = csb_inputs.make_rnn(cfg)
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    xd = torch.from_numpy(wl.x).cuda()
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rs = CsbRnn(CELL_LIGRU, 39, 512, Ws, bias)
    for m in Ws:
        m.upload()
    rr = CsbRnn(CELL_LIGRU, 39, 512, [CsbMatrix(m.A, m.br, m.bc) for m in wl.W], bias)
    rr.upload()
    res["ligru_sr3"] = {"batch1_streaming_us_per_frame": timed(rs, xd, 3),
                        "batch1_streaming_graph_replay_us_per_frame": round(graph_replay_ms(lambda: rs.forward(xd, want_hseq=True), 3, torch) * 1000.0 / T, 3),
                        "batch1_resident_us_per_frame": timed(rr, xd, 20),
                        "nnz": sum(int(m.view()["nnz"]) for m in Ws), "resident_plan": rr.stats()}
    if with_cpu:
        res["ligru_sr3"]["cpu_baseline"] = cpu(csb_inputs.LIGRU, wl, 39, 512)
    # SR2 shape, GRU in both forms
    cfg = csb_inputs.RnnConfig("sr2", csb_inputs.GRU_RB, 2, 39, 1024, 32, 21.7, "binomial", 0.05, 1, T, 0)
    wl = csb_inputs.make_rnn(cfg)
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    xd = torch.from_numpy(wl.x).cuda()
    Was, Uns = [], []
    for l, m in enumerate(wl.W):
        Wa, Un = csb_inputs.split_gru_rb(m.A, 39 if l == 0 else 1024, 1024)
        Was.append(CsbMatrix(Wa, m.br, m.bc))
        Uns.append(CsbMatrix(Un, m.br, m.bc))
    rb = CsbRnn(CELL_GRU_RB, 39, 1024, Was, bias, Wp=Uns)
    for m in Was + Uns:
        m.upload()
    rbr = CsbRnn(CELL_GRU_RB, 39, 1024, [CsbMatrix(m.unpack(), m.br, m.bc) for m in Was], bias,
                 Wp=[CsbMatrix(m.unpack(), m.br, m.bc) for m in Uns])
    rbr.upload()
    Wg = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    ga = CsbRnn(CELL_GRU, 39, 1024, Wg, bias)
    for m in Wg:
        m.upload()
    gr = CsbRnn(CELL_GRU, 39, 1024, [CsbMatrix(m.A, m.br, m.bc) for m in wl.W], bias)
    gr.upload()
    res["gru_sr2"] = {"reset_before_streaming_us_per_frame": timed(rb, xd, 3),
                      "reset_before_resident_us_per_frame": timed(rbr, xd, 20),
                      "reset_before_resident_plan": rbr.stats(),
                      "reset_before_streaming_graph_replay_us_per_frame": round(graph_replay_ms(lambda: rb.forward(xd, want_hseq=True), 3, torch) * 1000.0 / T, 3),
                      "reset_after_streaming_us_per_frame": timed(ga, xd, 3),
                      "reset_after_streaming_graph_replay_us_per_frame": round(graph_replay_ms(lambda: ga.forward(xd, want_hseq=True), 3, torch) * 1000.0 / T, 3),
                      "reset_after_resident_us_per_frame": timed(gr, xd, 20),
                      "nnz": sum(int(m.view()["nnz"]) for m in Wg), "resident_plan": gr.stats()}
    if with_cpu:
        res["gru_sr2"]["cpu_baseline_reset_before"] = cpu(csb_inputs.GRU_RB, wl, 39, 1024)
    return res


def cpu_leg(cfg, wl):
    """The CPU oracle as it stands, on the host cores of this machine: float64 LSTM/GRU on the
    decompressed dense matrix, whole T-frame sequences until about 10 s have passed; beside it
    the oracle's float32 mat-vec on the CSB arrays (what a CPU does with the same format)."""
    import oracle
    W = [m.A for m in wl.W]
    oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x[:2], cfg.input, cfg.hidden)   # warm-up
    t0 = time.perf_counter()
    reps = 0
    while True:
        oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 or reps >= 20000:
            break
    us = dt / (reps * cfg.T) * 1e6
    res = {"value": round(us, 3), "unit": "us/timestep", "cores": oracle.num_threads(), "kind": "oracle",
           "sample": f"{reps} full sequences of T={cfg.T} (float64 dense masked mat-vec + gates, OpenMP over rows)"}
    # the same on one core (a few sequences), for the per-core figure
    all_threads = oracle.num_threads()
    try:
        oracle.set_threads(1)
        t0 = time.perf_counter()
        r1 = 0
        while time.perf_counter() - t0 < 3.0:
            oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
            r1 += 1
        res["one_core_us_per_timestep"] = round((time.perf_counter() - t0) / (r1 * cfg.T) * 1e6, 3)
    finally:
        oracle.set_threads(all_threads)
    # like for like: the oracle's float32 CSB-MVM on the encoded arrays (mat-vec only, no gates),
    # on this workload's first layer and on the 8192^2 stress matrix, all cores and one core
    def time_csb(enc, x, budget):
        oracle.csb_matvec_f32(enc, x)
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < budget:
            oracle.csb_matvec_f32(enc, x)
            n += 1
        return round((time.perf_counter() - t0) / n * 1e6, 2)
    import csb_inputs
    big = csb_inputs.make_mat(csb_inputs.CONFIGS["cfg5"])
    cases = {f"{cfg.name}_layer0": (wl.W[0].A, wl.W[0].br, wl.W[0].bc), "cfg5": (big.A, big.br, big.bc)}
    res["csb_f32_matvec"] = {}
    for name, (A, br, bc) in cases.items():
        enc = oracle.csb_encode(A, br, bc)
        x = csb_inputs.make_vectors(5, A.shape[1], 1)
        entry = {"nnz": int(enc.nnz), "us_all_cores": time_csb(enc, x, 1.5)}
        try:
            oracle.set_threads(1)
            entry["us_one_core"] = time_csb(enc, x, 1.5)
        finally:
            oracle.set_threads(all_threads)
        res["csb_f32_matvec"][name] = entry
    return res


if __name__ == "__main__":
    main()
