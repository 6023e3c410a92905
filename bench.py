#!/usr/bin/env python3
"""Benchmark of the batched CTC cost + gradient on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--dtype f32|bf16]
                    [--mode grad|loss|align]

A step is one ctc_loss_and_grad call (host launcher + all kernels) over one synthetic
minibatch whose activations already sit in HBM.  The default workload is the English-shaped
per-GPU minibatch (config index 1: B=64, A=29, T<=750).  Prints one JSON line.
--mode loss times the cost-only call (grads == NULL), --mode align the most probable
alignment (ctc_best_path); the default, grad, is the headline metric.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
# One non-packed, non-fused VALU operation per lane per clock: 256 CUs x 64 lanes x 2.4 GHz.
# (The published 157.3 TFLOP/s fp32 vector figure counts 2 for packing and 2 for FMA on top.)
ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
# Algorithmic lane-operations of one step of one (blank, label) state pair in one direction, priced
# for the log-space recursion that defines the path: two two-term log-sum-exps = 4 transcendentals
# (two exp2, two log2) at quarter rate (= 16) + 25 plain operations.  The kernel itself recurs on
# probabilities with a per-lane exponent and issues about a third of that (see LANE_OPS_EXECUTED),
# so `achieved` is the rate at which the defined work gets done, not the ALU's busy rate.
LANE_OPS_PER_PAIR_STEP = 41
# What the linear-domain kernel executes per pair-step: 2 fused multiply-adds, 1 addition,
# 2 multiplications, 2 conversions of emissions, 2 DPP moves, 1 pack, 1 address, and about 3 for
# the renewal of the exponents every 8 steps.
LANE_OPS_EXECUTED = 14
# The max recursion of the alignment has no transcendentals: compares, selects, two fp64 adds.
LANE_OPS_PER_PAIR_STEP_ALIGN = 22


# HBM bytes per launch as the counters saw them (FETCH_SIZE + WRITE_SIZE, each scaled by what the same
# counter reads for a plain copy of known size): profiles/hbm_traffic.json, written from the rocprofv3 --pmc
# runs whose summaries sit beside it.  Each entry names the sources it was measured on; a figure measured
# on other sources than the ones in the tree is reported with "traffic_current": false.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")

# What the paper reports for this computation (Section 4.2, Table "gpucpuctc"): seconds per epoch spent in
# the CTC cost and gradient, on its CPU implementation and on its GPU implementation.  Other hardware, other
# workload unit (an epoch of its corpora): context, not a baseline for `value`.
PAPER_CONTEXT = {
    "source": "Section 4.2, Table gpucpuctc: CTC time in seconds per epoch, 5-layer 3-RNN model",
    "hardware": "NVIDIA Titan X GPUs (count for this run not stated; 8 per node, 8 or 16 typical) vs. the node's "
                "two Intel CPUs (model not stated), fp32",
    "english": {"cpu_ctc_s_per_epoch": 5888.12, "gpu_ctc_s_per_epoch": 203.56, "speedup": 28.9},
    "mandarin": {"cpu_ctc_s_per_epoch": 1688.01, "gpu_ctc_s_per_epoch": 135.05, "speedup": 12.5},
    "note": "with about 8 M utterances per English epoch (11,940 h at about 7 s each: an estimate, the paper gives "
            "no count for this table) the GPU figure is roughly 39 k utterances/s over all its GPUs",
}


def source_digest():
    """sha256 (first 16 hex digits) over the library's sources: ties a counter measurement to the code."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1512_02595_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(config, dtype, kernel):
    """(bytes per launch, measured on the current sources?) from profiles/hbm_traffic.json, or (None, None)."""
    try:
        with open(TRAFFIC_FILE) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None, None
    entry = table.get("config%d/%s" % (config, dtype))
    if not entry or kernel not in entry.get("kernels", {}):
        return None, None
    k = entry["kernels"][kernel]
    return float(k["read_bytes"] + k["written_bytes"]), entry.get("source_digest") == source_digest()


def kernel_bytes(batch, elem, mode="grad"):
    """Algorithmic HBM bytes of each kernel for one launch on `batch`: what the kernel must read and
    write once, per frame, per row of the tensor and per lattice cell, as the comments below state."""
    frames = batch.frames
    A = batch.A
    pairs = int((batch.input_lengths.astype(np.int64) * (batch.label_lengths.astype(np.int64) + 1)).sum())
    cells = batch.lattice_cells
    full = batch.T * batch.B * A * elem
    if mode != "grad":
        # cost only / alignment: the activations are read once; the chain reads one emission per
        # state pair and frame (4 bytes) and, for the alignment, writes one byte of choices per pair
        # and frame, which the backtrace reads along the path (at most 64 per frame) before it
        # writes one int32 per frame of the tensor
        out = {"ctc_softmax": frames * A * elem + frames * 4,
               "ctc_lattice": pairs * 4 + (pairs if mode == "align" else 0)}
        if mode == "align":
            out["ctc_backtrace"] = frames * 64 + batch.T * batch.B * 4
        else:
            out["ctc_gradient"] = 0
        return out, pairs
    if A > 2048:
        # wide alphabets: the softmax launch also writes the dense gradient (y, or zeros for
        # padding); the gradient launch only rewrites the label columns and the blank
        touched = int((batch.input_lengths.astype(np.int64) * (batch.label_lengths.astype(np.int64) + 2)).sum())
        soft, grad = frames * A * elem + full, 2 * touched * elem
    else:
        # read every valid row once, write one statistic per row / read the rows again and write
        # the whole gradient tensor
        soft, grad = frames * A * elem + frames * 4, frames * A * elem + full
    return {
        "ctc_softmax": soft,
        # one alpha and one beta value per lattice cell, 4 bytes each, written once
        "ctc_lattice": cells * 8,
        "ctc_gradient": grad,
    }, pairs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="0..4: the five headline workloads (1 = the metric's); 5: bigram alphabet")
    ap.add_argument("--dtype", choices=("f32", "bf16"), default="f32")
    ap.add_argument("--mode", choices=("grad", "loss", "align"), default="grad",
                    help="grad: cost + gradient (headline); loss: cost only; align: most probable alignment")
    ap.add_argument("--metadata", choices=("host", "device"), default="host",
                    help="device: ctc_loss_and_grad_device (lengths and labels resident on the GPU, workspace "
                         "sized by bounds)")
    ap.add_argument("--graph", action="store_true",
                    help="with --metadata device: record each minibatch's call into a HIP graph and time replays")
    ap.add_argument("--buffers", type=int, default=4, help="distinct minibatches rotated through")
    ap.add_argument("--profile-steps", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", type=int, default=-1,
                    help="0: write the whole gradient in a launch of its own even where the lattice launch has idle "
                         "compute units; 1..100: ctc_debug_set_overlap; default: the library's setting")
    ap.add_argument("--sequential-chains", action="store_true",
                    help="measurement of the paper's order: the forward recursion's launch, then the backward one's "
                         "(ctc_debug_set_sequential_chains); the JSON line says so and is no headline figure")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (reference for HBM counters)")
    args = ap.parse_args()

    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path needs no collective; "
                 "utterances would simply be split across ranks). Use --gpus 1.")

    import torch
    from paper_1512_02595_amd import ctc, harness, workloads

    dev = harness.require_gpu()
    if args.calibrate_copy:
        n = 256 << 20                                   # 256 MiB read + 256 MiB written per copy
        src = torch.ones(n // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize(dev)
        ms = e0.elapsed_time(e1) / 20
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_copy": n, "bytes_written_per_copy": n,
                          "copies": 25, "ms_per_copy": round(ms, 4),
                          "copy_GBps_read_plus_write": round(2 * n / (ms * 1e-3) / 1e9, 1)}), flush=True)
        return
    ctc.load()
    if args.overlap >= 0:
        ctc.debug_set_overlap(args.overlap)
    if args.sequential_chains:
        ctc.debug_set_sequential_chains(True)
    dtype = ctc.DTYPE_F32 if args.dtype == "f32" else ctc.DTYPE_BF16
    elem = 4 if dtype == ctc.DTYPE_F32 else 2

    batches = [workloads.make_config(args.config, seed=workloads.BASE_SEED + args.config + 1000 * i)
               for i in range(args.buffers)]
    stream = torch.cuda.current_stream(dev).cuda_stream
    if args.metadata == "device":
        if args.mode == "align":
            sys.exit("bench.py: --metadata device covers the grad and loss modes")
        max_label = max(int(b.label_lengths.max()) for b in batches)
        dbs = []
        for b in batches:
            d = harness.DeviceMetaBatch(b.T, b.B, b.A, max_label, b.blank, dtype, dev)
            d.load(b)
            dbs.append(d)
        want_grad = args.mode == "grad"
        if args.graph:
            side = torch.cuda.Stream()
            graphs = {}
            for d in dbs:
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    d.run(stream=side.cuda_stream, want_grad=want_grad)          # warm-up outside the capture
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize(dev)
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    d.run(stream=torch.cuda.current_stream().cuda_stream, want_grad=want_grad)
                graphs[id(d)] = g

            def step(d, stream, kernel_ms=None):
                graphs[id(d)].replay()
            args.profile_steps = 0                 # (a replay has no events inside it)
        else:
            def step(d, stream, kernel_ms=None):
                d.run(stream, want_grad=want_grad, kernel_ms=kernel_ms)
    else:
        if args.graph:
            sys.exit("bench.py: --graph needs --metadata device (the host-metadata call reads host memory)")
        dbs = [harness.DeviceBatch(b, dtype, dev, poison=False) for b in batches]
        step = {"grad": harness.DeviceBatch.run, "loss": harness.DeviceBatch.run_loss,
                "align": harness.DeviceBatch.run_best_path}[args.mode]

    for i in range(args.warmup):
        step(dbs[i % len(dbs)], stream)
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(dbs[i % len(dbs)], stream)
    torch.cuda.synchronize(dev)
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # The same loop once more with an event pair around every call (median and minimum of the
    # device time of single calls), and on one minibatch only (cache-warm: its buffers may still
    # sit in the 256 MB infinity cache from the call before).
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        step(dbs[i % len(dbs)], stream)
        e1.record()
    torch.cuda.synchronize(dev)
    per_call = np.array([e0.elapsed_time(e1) for e0, e1 in evs])
    torch.cuda.synchronize(dev)
    w0 = time.perf_counter()
    for i in range(args.steps):
        step(dbs[0], stream)
    torch.cuda.synchronize(dev)
    warm_ms = (time.perf_counter() - w0) * 1e3 / args.steps

    B = batches[0].B
    frames = float(np.mean([b.frames for b in batches]))
    if args.mode == "grad":
        compulsory = float(np.mean([b.compulsory_bytes(elem) for b in batches]))
    else:       # the valid activations once; the alignment also writes one int32 per frame of the tensor
        compulsory = float(np.mean([b.frames * b.A * elem for b in batches]))
        if args.mode == "align":
            compulsory += batches[0].T * batches[0].B * 4

    # Per-kernel device time, HIP events on the launch stream (ctc_profile_kernels).
    kms = np.zeros((args.profile_steps, ctc.NUM_KERNELS), dtype=np.float32)
    for i in range(args.profile_steps):
        step(dbs[i % len(dbs)], stream, kernel_ms=kms[i])
    kavg = [float(v) for v in kms.mean(axis=0)] if args.profile_steps else [1e-9] * ctc.NUM_KERNELS
    names = [ctc.kernel_name(i) for i in range(ctc.NUM_KERNELS)]
    if args.mode == "align":
        names[2] = ctc.kernel_name(ctc.KERNEL_BACKTRACE)
    kb = [kernel_bytes(b, elem, args.mode) for b in batches]
    kernels = {}
    for i, n in enumerate(names):
        byt = float(np.mean([k[0][n] for k in kb]))
        kernels[n] = {"ms": round(kavg[i], 5) if args.profile_steps else None, "algorithmic_bytes": int(byt),
                      "GBps": round(byt / (kavg[i] * 1e-3) / 1e9, 2) if args.profile_steps and kavg[i] > 0 else None}
    dom = int(np.argmax(kavg))
    dom_name = names[dom]
    if args.profile_steps == 0:
        dom_name = None
    traffic, traffic_current = (measured_traffic(args.config, args.dtype, dom_name)
                                if args.mode == "grad" and dom_name else (None, None))
    if dom_name is None:
        roofline = None
    else:
        # The dominant kernel against the HBM roofline: its algorithmic bytes (kernel_bytes) over its
        # measured duration.
        achieved = kernels[dom_name]["GBps"]
        roofline = {"kernel": dom_name, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic,
                    "traffic_current": traffic_current}
        if dom_name == "ctc_lattice":
            # The recursion is a chain of dependent steps and moves few bytes: what limits it is the rate
            # at which a wavefront issues the step's instructions.  For orientation, the same kernel
            # against the vector ALUs, in lane-operations per second: the operations it executes, and
            # the operations of the log-space recursion that defines the path (which it does not run).
            directions = 2.0 if args.mode == "grad" else 1.0
            priced = LANE_OPS_PER_PAIR_STEP_ALIGN if args.mode == "align" else LANE_OPS_PER_PAIR_STEP
            executed = LANE_OPS_PER_PAIR_STEP_ALIGN if args.mode == "align" else LANE_OPS_EXECUTED
            pair_steps = directions * float(np.mean([k[1] for k in kb]))
            per_s = pair_steps / (kavg[dom] * 1e-3) / 1e12
            roofline["alu_orientation"] = {
                "peak_T_lane_ops_per_s": round(ALU_PEAK_TOPS, 2),
                "executed_lane_ops_per_pair_step": executed,
                "executed_frac_of_peak": round(per_s * executed / ALU_PEAK_TOPS, 5),
                "log_space_lane_ops_per_pair_step": priced,
                "log_space_equivalent_frac_of_peak": round(per_s * priced / ALU_PEAK_TOPS, 5),
                "note": "peak = one non-packed, non-fused VALU operation per lane and clock (256 CUs x 64 lanes x "
                        "2.4 GHz); the executed count is the linear-domain step's, the log-space count prices the "
                        "defining recursion (a transcendental as 4)"}

    out = {
        "metric": {"grad": "ctc_loss_grad_utterances_per_s", "loss": "ctc_loss_only_utterances_per_s",
                   "align": "ctc_best_path_utterances_per_s"}[args.mode],
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "utterances/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_call_median": round(float(np.median(per_call)), 5),
        "ms_per_call_min": round(float(per_call.min()), 5),
        "ms_per_step_cache_warm": round(warm_ms, 5),
        "rotating_bytes": int(sum(d.x.numel() * d.x.element_size() * 2 + d.ws_bytes for d in dbs)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64 lattice state (probabilities with a per-lane exponent), %s activations" % args.dtype,
        "data": "synthetic",
        "config": {"workload": "config[%d] %s: B=%d A=%d T=%d, %d rotating minibatches"
                   % (args.config, batches[0].name, B, batches[0].A, batches[0].T, len(batches)),
                   "mode": args.mode, "metadata": args.metadata, "graph": bool(args.graph),
                   "sequential_chains": bool(args.sequential_chains)},
        "activation_frames_per_s": round(frames / (ms_per_step * 1e-3), 1),
        "hbm_roofline_frac_end_to_end": round(compulsory / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
        "compulsory_bytes": int(compulsory),
        "kernels": kernels,
        "roofline": roofline,
        "paper_context": PAPER_CONTEXT,
    }

    if not args.no_cpu_baseline:
        from oracle import ctc_oracle as orc
        b = batches[0]
        x64 = b.logits.astype(np.float64) if dtype == ctc.DTYPE_F32 else workloads.to_bf16_grid(b.logits).astype(np.float64)
        nb = b.B
        # Bounded sample: whole minibatch if its lattice is small enough, else its first utterances.
        budget_cells = 60e6
        if b.lattice_cells + b.frames * b.A > budget_cells:
            w = b.input_lengths.astype(np.int64) * (2 * b.label_lengths.astype(np.int64) + 1 + b.A)
            nb = max(1, int(np.searchsorted(np.cumsum(w), budget_cells)))
        nlab = int(b.label_lengths[:nb].sum())
        xs = np.ascontiguousarray(x64[:, :nb, :])
        # About 15 core-seconds of oracle work: time one run, then size the repetitions.
        cores = orc.max_threads()
        if args.mode == "align":
            def oracle_call():
                orc.ctc_best_path(xs, b.flat_labels[:nlab], b.label_lengths[:nb], b.input_lengths[:nb], b.blank)
        else:
            def oracle_call():
                orc.ctc_loss_and_grad(xs, b.flat_labels[:nlab], b.label_lengths[:nb], b.input_lengths[:nb],
                                      b.blank, want_grad=(args.mode == "grad"))
        c0 = time.perf_counter()
        oracle_call()
        first = time.perf_counter() - c0
        reps = int(min(200, max(3, np.ceil(15.0 / max(first * cores, 1e-6)))))
        times = []
        for _ in range(reps):
            c0 = time.perf_counter()
            oracle_call()
            times.append(time.perf_counter() - c0)
        tmed = float(np.median(times))
        c0 = time.perf_counter()
        if args.mode == "align":
            orc.ctc_best_path(xs, b.flat_labels[:nlab], b.label_lengths[:nb], b.input_lengths[:nb], b.blank,
                              nthreads=1)
        else:
            orc.ctc_loss_and_grad(xs, b.flat_labels[:nlab], b.label_lengths[:nb], b.input_lengths[:nb],
                                  b.blank, want_grad=(args.mode == "grad"), nthreads=1)
        t_single = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(nb / tmed, 2), "unit": "utterances/s",
                               "cores": cores, "kind": "oracle",
                               "single_thread_value": round(nb / t_single, 2),
                               "sample": "first %d of %d utterances of minibatch 0, median of %d runs, %.3f s each"
                                         % (nb, b.B, reps, tmed),
                               "activation_frames_per_s": round(float(b.input_lengths[:nb].sum()) / tmed, 1)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
