#!/usr/bin/env python3
"""Benchmark of the LF-MMI forward-backward hot path on one MI355X.

A step is one lfmmi_forward_backward call (emission, alpha/beta recursion,
scale scan, occupancy + gradient) over one synthetic batch already resident in
HBM. Default workload: the WSJ-monophone-shaped case the headline metric is
quoted on (2,000-state / 20,000-arc denominator graph, 84 pdfs, B = 64,
T in [100, 500]). Prints one JSON line.
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

# MI355X: 256 CUs x 128 B/clk LDS x 2.4 GHz (4-byte reads; the datasheet formula)
LDS_PEAK_GBPS = 256 * 128 * 2.4
# ... and what `lfmmi_microbench lds` measures over the whole chip for conflict-free 4-byte
# reads, at the 2.13 GHz the shader clock settles at under that load (profiles/lds_peak.txt)
LDS_PEAK_MEASURED_GBPS = 68800.0
HBM_PEAK_GBPS = 8000.0
# HBM bytes of the recursion kernel per step (all its launches), from rocprofv3 FETCH_SIZE /
# WRITE_SIZE scaled by a plain copy of known size (profiles/hbm_traffic_<workload>.txt)
# (e2e_num_den: the denominator's recursion, the kernel the roofline object describes)
REC_TRAFFIC_BYTES = {"wsj_mono_2k": 362.4e6, "biphone_10k": 4245.5e6, "long_unequal_5k": 1224.1e6,
                     "e2e_num_den": 641.8e6, "hmm_den_2k": 345.6e6, "wsj_den_7398": 2347.2e6}


def phase_timers(config, torch, binding, workloads):
    """Clocks per phase of k_occ_planes (thread 0 of every workgroup, s_memtime), from the
    counters a library built with -DLFMMI_PHASE_TIMERS keeps."""
    import ctypes
    lib = ctypes.CDLL(binding.LIB_PATH)
    if not hasattr(lib, "lfmmi_phase_timers_read"):
        print("bench.py: the library was not built with -DLFMMI_PHASE_TIMERS", file=sys.stderr)
        return 2
    os.environ["LFMMI_BUCKETS"] = "1"
    wl = workloads.make_workload(config)
    x = torch.from_numpy(wl["logits"]).cuda()
    B, T, P = x.shape
    h = binding.lfmmi_graph_create(wl["den"])
    objf = torch.empty(B, device="cuda")
    grad = torch.empty((B, T, P), device="cuda")
    status = torch.zeros(B, dtype=torch.int32, device="cuda")
    out = (ctypes.c_ulonglong * 81)()
    for k in range(4):  # the last call is the one that is read
        if k == 3 and lib.lfmmi_phase_timers_read(out, 1) != 0:
            return 1
        binding.lfmmi_forward_backward(h, x, wl["lengths"], wl["leak"], 1.0, False, objf, grad, status)
    if lib.lfmmi_phase_timers_read(out, 1) != 0:
        return 1
    names = ["start of the workgroup", "scales of the group", "barrier", "staging", "barrier",
             "gathers", "barrier", "sums, pdfs with few rows", "sums, pdfs with many rows"]
    v = list(out)
    total = float(sum(v[:9]))
    print("%s: %d workgroups, %d frame groups; clocks of thread 0 per frame group" %
          (wl["name"], v[14], v[15]))
    for i, n in enumerate(names):
        print("  %-28s %9.0f  %5.1f %%" % (n, v[i] / max(v[15], 1), 100.0 * v[i] / max(total, 1.0)))
    steps = v[80]
    if steps:
        info = binding.lfmmi_graph_ordering_info
        slots = [[0] * 16, [0] * 16]
        for o in (0, 1):
            d = binding.lfmmi_graph_ordering_copy(h, 0, o)
            for w in range(d["waves"]):
                slots[o][w] = int(d["slice_off"][d["wave_first"][w + 1]] - d["slice_off"][d["wave_first"][w]])
        print("k_rec, arcs in registers: clocks per step and wave (mean over both directions; "
              "%d steps); slots of the wave in the alpha / beta ordering" % steps)
        print("  wave   head  slots   tail   wait at the barrier   total   slots alpha/beta")
        for w in range(16):
            c = [v[16 + 4 * w + q] / steps for q in range(4)]
            print("  %4d %6.0f %6.0f %6.0f %6.0f %21.0f   %d/%d" %
                  (w, c[0], c[1], c[2], c[3], sum(c), slots[0][w], slots[1][w]))
    h.close()
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2,
                    help="workload 1..5 (2 is the metric); 6: the HMM-expanded graph; "
                         "7: the paper's own denominator size and batch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="BYTES",
                    help="only run plain device-to-device copies of BYTES (to calibrate the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--phase-timers", action="store_true",
                    help="one call with the whole batch as one launch on a library built with "
                         "-DLFMMI_PHASE_TIMERS: where a frame group of the occupancy kernel "
                         "spends its clocks; prints a table and exits")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; sequences are independent, so "
              "several GPUs would each take a share of the batch with no communication. "
              "Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2005_09824_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.copy_probe > 0:
        n = args.copy_probe // 4
        a = torch.ones(n, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(4):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": n * 4, "copies": 4}))
        return 0
    if args.phase_timers:
        return phase_timers(args.config, torch, binding, workloads)
    wl = workloads.make_workload(args.config)
    lengths, leak = wl["lengths"], wl["leak"]
    frames = int(lengths.sum())
    B, T, P = wl["logits"].shape
    x = torch.from_numpy(wl["logits"]).cuda()
    den = binding.lfmmi_graph_create(wl["den"])
    num = binding.lfmmi_graph_create_batch(wl["num"]) if args.config == 5 else None
    S, A = wl["den"]["num_states"], len(wl["den"]["src"])
    objf = torch.empty(B, dtype=torch.float32, device="cuda")
    grad = torch.empty((B, T, P), dtype=torch.float32, device="cuda")
    status = torch.zeros(B, dtype=torch.int32, device="cuda")

    def step():
        if num is not None:  # Eq. 2 / Eq. 3: numerator minus denominator
            binding.lfmmi_loss(num, den, x, lengths, leak, objf, grad, status)
        else:
            binding.lfmmi_forward_backward(den, x, lengths, leak, 1.0, False, objf, grad, status)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The library keeps the HIP events of profiled calls and uses them again: as many
    # untimed profiled steps as timed ones, so that no event is created inside the
    # timed region
    binding.lfmmi_profile_enable(den, 2)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    binding.lfmmi_profile_read(den)
    # HIP events around the recursion launches (the dominant kernel) of every timed step
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kern = binding.lfmmi_profile_read(den)
    binding.lfmmi_profile_enable(den, False)
    # the other kernels' launch durations: a few more steps outside the timed region
    binding.lfmmi_profile_enable(den, 1)
    for _ in range(min(args.steps, 10)):
        step()
    torch.cuda.synchronize()
    others = binding.lfmmi_profile_read(den)
    binding.lfmmi_profile_enable(den, False)
    kern["emit"], kern["occ"] = others["emit"], others["occ"]
    if int(status.abs().sum().item()) != 0:
        print("bench.py: a sequence was flagged", file=sys.stderr)
        return 1

    # Outside the timed region: single calls bracketed by HIP events on the stream
    # the call is ordered on (torch's current stream), for the median and the spread
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(max(20, min(args.steps, 50)))]
    for a, b in evs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    call_ms = sorted(a.elapsed_time(b) for a, b in evs)

    # For reference, outside the timed region: the same work with the whole batch
    # as one bucket, i.e. one recursion launch over all 2B workgroups and nothing
    # overlapping it. The library reads LFMMI_BUCKETS at every call.
    os.environ["LFMMI_BUCKETS"] = "1"
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    binding.lfmmi_profile_enable(den, True)
    t0 = time.perf_counter()
    for _ in range(10):
        step()
    torch.cuda.synchronize()
    one_dt = (time.perf_counter() - t0) / 10
    one = binding.lfmmi_profile_read(den)
    binding.lfmmi_profile_enable(den, False)
    del os.environ["LFMMI_BUCKETS"]

    ms_per_step = dt / args.steps * 1e3
    fps = frames / (dt / args.steps)

    # dominant kernel: the alpha/beta recursion. Algorithmic LDS bytes per frame:
    # per arc and direction two 4-byte gathers (state vector, emission), per state
    # and direction 12 bytes (write, re-read for the rescale, write back).
    # A call cuts its sequences into buckets that run concurrently, each with a
    # recursion launch of its own: bytes and duration below are per launch (means).
    launches_per_call = kern["launches"] / max(kern["calls"], 1)
    rec_bytes = frames * (16.0 * A + 24.0 * S) / launches_per_call
    rec_s = kern["rec"] * 1e-3
    achieved = rec_bytes / rec_s / 1e9
    info = binding.lfmmi_graph_info(den)
    # the whole call against the same peak: the recursion's bytes of all launches of a
    # step, and the bytes of the whole path (forward, backward and occupancy: 24 per
    # arc and 28 per state and frame), over the time of a step
    step_s = dt / args.steps
    rec_step_gbps = frames * (16.0 * A + 24.0 * S) / step_s / 1e9
    path_step_gbps = frames * (24.0 * A + 28.0 * S) / step_s / 1e9
    out = {
        "metric": "LF-MMI forward-backward frames/sec (loss+grad), 2k-state den graph, B=64",
        "value": fps,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl["name"], "states": S, "arcs": A, "pdfs": P, "batch": B,
                   "frames": frames, "max_len": T, "leak": leak,
                   "numerators": num is not None},
        "roofline": {"bound": "lds", "kernel": "k_rec", "achieved": achieved,
                     "peak": LDS_PEAK_GBPS, "unit": "GB/s", "frac": achieved / LDS_PEAK_GBPS,
                     "peak_measured": LDS_PEAK_MEASURED_GBPS,
                     "frac_of_measured_peak": achieved / LDS_PEAK_MEASURED_GBPS,
                     # not per launch: all launches of a step over the time of a step
                     "whole_call": {"recursion_bytes": {"achieved": rec_step_gbps,
                                                        "frac": rec_step_gbps / LDS_PEAK_GBPS,
                                                        "frac_of_measured_peak":
                                                            rec_step_gbps / LDS_PEAK_MEASURED_GBPS},
                                    "path_bytes": {"achieved": path_step_gbps,
                                                   "frac": path_step_gbps / LDS_PEAK_GBPS,
                                                   "frac_of_measured_peak":
                                                       path_step_gbps / LDS_PEAK_MEASURED_GBPS}},
                     "traffic": (REC_TRAFFIC_BYTES[wl["name"]] / launches_per_call
                                 if wl["name"] in REC_TRAFFIC_BYTES else None),
                     "kernel_ms": kern["rec"], "launches_per_step": launches_per_call,
                     # a launch holds one compute unit per workgroup (the launches of a
                     # step overlap on different ones): the same against their LDS peak
                     "workgroups_per_launch": 2 * B / launches_per_call, "compute_units": 256,
                     "frac_of_occupied_cus": achieved / (LDS_PEAK_GBPS *
                                                         min(2 * B / launches_per_call, 256) / 256.0),
                     "hbm_frac": (REC_TRAFFIC_BYTES.get(wl["name"], 0.0) / launches_per_call
                                  / rec_s / 1e9) / HBM_PEAK_GBPS,
                     # one launch for the whole batch (LFMMI_BUCKETS=1), not the timed path
                     "one_launch": {"kernel_ms": one["rec"], "ms_per_step": one_dt * 1e3,
                                    "achieved": frames * (16.0 * A + 24.0 * S) / (one["rec"] * 1e-3) / 1e9,
                                    "frac": frames * (16.0 * A + 24.0 * S) / (one["rec"] * 1e-3) / 1e9
                                            / LDS_PEAK_GBPS}},
        "kernels_ms": {k: kern[k] for k in ("emit", "rec", "scan", "occ")},
        # single calls between HIP events, outside the timed region
        "call_ms_hip_events": {"calls": len(call_ms), "median": call_ms[len(call_ms) // 2],
                               "min": call_ms[0], "max": call_ms[-1]},
        "arc_updates_per_s": 2.0 * A * fps,
        "workspace_bytes": info["workspace_bytes"],
    }

    if not args.no_cpu_baseline:
        from oracle import lfmmi_oracle as oracle
        threads = oracle.max_threads()
        t0 = time.perf_counter()
        if num is not None:
            oracle.loss(wl["num"], wl["den"], wl["logits"], lengths, leak)
        else:
            oracle.forward_backward(wl["den"], wl["logits"], lengths, leak)
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": frames / cdt, "unit": "frames/s", "cores": threads,
                               "kind": "oracle",
                               "sample": "the whole batch once (%d frames), fp64 log-domain, "
                                         "OpenMP over sequences" % frames}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
