#!/usr/bin/env python3
"""Benchmark of the detector's hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic
telemetry resident in HBM: gd_score_batch over all T steps of the workload,
gd_update_window, gd_flags and gd_topk_nodes.  The workload is the 65 536-rank
configuration (65 536 ranks x 4 096 steps x 8 metrics fp32, 8 GiB).

Prints one JSON line: telemetry samples scored per second, the scoring
kernel's achieved HBM bandwidth against the 8 TB/s peak (algorithmic bytes /
HIP-event time per launch), the CPU oracle timed on a bounded sample of the
same workload, and the streaming per-step latency on the 32 768-rank shape.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_per_launch(R: int, M: int, T: int) -> int:
    """What one gd_score_batch call must move: every fp32 sample read once, plus
    per step: med+mad, mask bytes, rank bits, primary node score, node mask, node bits."""
    N = R // 8
    per_step = 4 * M * R + 8 * M + R + R // 8 + 4 * N + N + N // 8
    return per_step * T


def _score_source_hash() -> str:
    import hashlib
    src = os.path.join(ROOT, "paper_2605_17879_amd", "csrc", "score.hip")
    return hashlib.sha256(open(src, "rb").read()).hexdigest()


def _profile_record(name: str):
    """A committed counter record under profiles/, or None when the kernel source has
    changed since it was taken (the figures would no longer describe this kernel)."""
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", name)))
        if rec.get("score_hip_sha256") == _score_source_hash():
            return rec
    except (OSError, ValueError, KeyError):
        pass
    return None


def measured_traffic():
    """HBM bytes per scoring launch from the committed counter runs, or None."""
    rec = _profile_record("score_kernel_c3_traffic.json")
    return rec["hbm_bytes_per_launch"] if rec else None


def issue_view(torch, samples: int, score_ms: float) -> dict:
    """Why the HBM fraction is what it is: the share of all SIMD cycles of the chip (compute
    units x 4 SIMDs at the device's clock, one 64-lane vector instruction per 4 cycles)
    that the scoring launch spends issuing vector instructions -- instruction count per
    sample from the committed counter profile (null once the kernel has changed since),
    time from this run."""
    rec = _profile_record("score_kernel_c3_counters.json")
    prop = torch.cuda.get_device_properties(0)
    clock_hz = float(getattr(prop, "clock_rate", 2400000)) * 1e3       # kHz
    simds = prop.multi_processor_count * 4
    out = {"valu_instructions_per_sample": None, "simd_cycles_issuing_valu": None,
           "clock_hz": clock_hz, "simds": simds,
           "what": "instruction count from rocprofv3 counters (profiles/score_kernel_c3_counters.json), time from this run"}
    if rec:
        vps = rec["valu_instructions_per_sample"]
        out["valu_instructions_per_sample"] = vps
        out["simd_cycles_issuing_valu"] = vps * samples / 64 * 4 / (score_ms * 1e-3 * clock_hz * simds)
    return out


def make_detector(w):
    from paper_2605_17879_amd import Config, Detector
    return Detector(Config(n_ranks=w.R, n_metrics=w.M, window=w.W, persist_k=w.k,
                           primary_metric=w.primary, min_signals=w.min_signals, topk=w.topk,
                           z_threshold=w.thr, direction=tuple(w.directions)))


def cpu_baseline(w, x_dev, sample_steps: int) -> dict:
    """The oracle, as it stands, on the first `sample_steps` steps of the same tensor."""
    import oracle
    xs = x_dev[:sample_steps].cpu().numpy()
    p = oracle.Params(R=w.R, M=w.M, W=w.W, k=w.k, thr=w.thr, directions=tuple(w.directions),
                      primary=w.primary, min_signals=w.min_signals)
    t0 = time.perf_counter()
    oracle.detect(p, xs, topk_k=w.topk, want_z=False)
    dt = time.perf_counter() - t0
    cores = oracle.num_threads()
    # one core, on a sample sized to take a few seconds
    one_steps = max(1, min(sample_steps, sample_steps * 4 // max(cores, 1) // 4))
    oracle.set_threads(1)
    t1 = time.perf_counter()
    oracle.detect(p, xs[:one_steps], topk_k=w.topk, want_z=False)
    dt1 = time.perf_counter() - t1
    oracle.set_threads(cores)
    return {"value": xs.size / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample_steps} of {w.T} steps ({xs.size} samples, {dt:.2f} s wall)",
            "single_thread": {"value": xs[:one_steps].size / dt1, "unit": "samples/s",
                              "sample": f"first {one_steps} steps, {dt1:.2f} s wall"}}


def streaming_latency(torch, n_steps: int) -> dict:
    """Per-call latency of score + window + flags + top-64 with one step appended
    per call on the 32 768-rank x 8-metric shape (100 000 steps by default, the input
    made on the device 1 000 steps at a time), host wall clock incl. stream sync."""
    from workloads import generate, workload
    w = workload(4, T=n_steps)
    det = make_detector(w)
    out, fl, tk = det.alloc_outputs(1), det.alloc_flags(), det.alloc_topk(w.topk)
    out["med"].zero_(); out["mad"].zero_()
    det.set_streaming_hints(out["med"].view(-1), out["mad"].view(-1))   # each call starts from the last one's results
    stream = torch.cuda.Stream()
    lat = []
    chunk = 1000
    for c0 in range(0, n_steps, chunk):
        x = generate(w, seed=4, t0=c0, t1=min(n_steps, c0 + chunk), device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for t in range(x.shape[0]):
                t0 = time.perf_counter()
                det.score_batch(x[t:t + 1], out, stream)
                det.update_window(out, 1, stream=stream)
                det.flags(fl, stream)
                det.topk_nodes(w.topk, tk, stream)
                stream.synchronize()
                lat.append(time.perf_counter() - t0)
    lat = sorted(lat[50:])                      # the first calls warm up
    det.close()
    return {"workload": f"{w.R} ranks x {w.M} metrics, 1 step per call, W={w.W}",
            "calls": len(lat), "p50_us": 1e6 * lat[len(lat) // 2],
            "p99_us": 1e6 * lat[int(len(lat) * 0.99)]}


def detection_report(torch, det, w, x, out, fl) -> dict:
    """What the detector says at the end of the batch against the faults the generator
    injected (reported, not gated: small slowdowns are not detectable by design)."""
    from workloads.telemetry import faults
    torch.cuda.synchronize()
    truth = sorted({f.rank_lo // w.G for f in faults(w, 3)})
    flagged = torch.nonzero(fl["node_flag"] != 0).flatten().cpu().tolist()
    hit = len(set(flagged) & set(truth))
    sev = det.alloc_severity()
    det.severity(x, out, sev)
    torch.cuda.synchronize()
    tiers = torch.bincount(sev["tier"].to(torch.int64), minlength=4).cpu().tolist()
    return {"injected_slow_nodes": len(truth), "flagged_nodes": len(flagged), "true_positives": hit,
            "recall": hit / max(1, len(truth)), "precision": hit / max(1, len(flagged)),
            "nodes_per_severity_tier": {"not_flagged": tiers[0], "no_observable_impact": tiers[1],
                                        "moderate": tiers[2], "severe": tiers[3]}}


def z_variant(torch, det, w, x, stream, alg_bytes: int) -> dict:
    """The scoring launch with the optional full z output (4 more bytes written per
    sample): timed on its own, not part of `value`."""
    out = det.alloc_outputs(w.T, want_z=True)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(4)]
    with torch.cuda.stream(stream):
        for s0, s1 in ev:
            s0.record(stream)
            det.score_batch(x, out, stream)
            s1.record(stream)
        torch.cuda.synchronize()
    ms = sorted(s0.elapsed_time(s1) for s0, s1 in ev[1:])[1]
    nbytes = alg_bytes + 4 * w.samples
    del out
    return {"what": "gd_score_batch writing z[T][M][R] as well", "ms": ms, "algorithmic_bytes": nbytes,
            "GB/s": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def c2_leg(torch, stream, host_input: bool = False) -> dict:
    """The 16 384-rank configuration (16 384 ranks x 10 000 steps x 4 metrics, another register
    tiling of the same kernel) in one gd_score_batch call: launch time by HIP events on the
    launch stream, algorithmic bytes, fraction of the HBM peak.  Not part of `value`."""
    from workloads import generate, workload
    w = workload(2)
    # (the same bytes either way; made on the host and uploaded when a counter profiler is
    # attached, which does not survive this recipe's device-side generation)
    x = generate(w, seed=2, device="cpu").cuda() if host_input else generate(w, seed=2, device="cuda")
    det = make_detector(w)
    out = det.alloc_outputs(w.T)
    # (this leg starts on freshly allocated buffers, and after the CPU leg the GPU has idled for
    # seconds: the first launches run up to a tenth slower, so ten go untimed)
    n_warm, n_timed = 10, 10
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_timed)]
    torch.cuda.synchronize()                        # the input is made on the default stream
    with torch.cuda.stream(stream):
        for _ in range(n_warm):
            det.score_batch(x, out, stream)
        for s0, s1 in ev:
            s0.record(stream)
            det.score_batch(x, out, stream)
            s1.record(stream)
        torch.cuda.synchronize()
    ms = sorted(s0.elapsed_time(s1) for s0, s1 in ev)
    avg = sum(ms) / len(ms)
    alg = algorithmic_bytes_per_launch(w.R, w.M, w.T)
    det.close()
    del x, out
    return {"workload": f"{w.R} ranks x {w.T} steps x {w.M} metrics fp32",
            "kernel": "score_kernel<256,16,11,true,false,false>", "launches": n_timed, "warmup": n_warm,
            "avg_launch_ms": avg,
            "algorithmic_bytes": alg, "bytes_per_sample": alg / w.samples,
            "achieved_GB/s": alg / (avg * 1e-3) / 1e9, "frac": alg / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "samples_per_s": w.samples / (avg * 1e-3)}


def ledger_leg(torch, det, w, out, stream) -> dict:
    """The bookkeeping beyond the default rule on the same resident scoring outputs
    (persistence per indicator, windowed score sums and their ranking, recurrence):
    not part of `value`, timed on its own."""
    det.alloc_ledger(w.T)
    lf, tk = det.alloc_ledger_flags(), det.alloc_topk(w.topk)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
    with torch.cuda.stream(stream):
        for s0, s1 in ev:
            s0.record(stream)
            det.update_ledger(out, w.T, stream=stream)
            det.ledger_flags(lf, stream)
            det.topk_nodes_mean(w.topk, tk, stream)
            s1.record(stream)
        torch.cuda.synchronize()
    ms = sorted(s0.elapsed_time(s1) for s0, s1 in ev)[2]
    N = w.R // w.G
    read = w.T * (w.R + N) + min(w.T, w.W) * N * 4          # exceed bytes of ranks and nodes, the window's node scores
    return {"what": "update_ledger + ledger_flags + topk_nodes_mean on the batch's scoring outputs",
            "ms": ms, "input_bytes": read, "GB/s": read / (ms * 1e-3) / 1e9}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--cpu-sample-steps", type=int, default=1024)
    ap.add_argument("--stream-steps", type=int, default=100000)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-stream", action="store_true", help="skip the streaming-latency leg")
    ap.add_argument("--only-batch", action="store_true",
                    help="only the timed batch steps and the read probe (for profiler runs): no CPU, streaming, z or ledger legs")
    ap.add_argument("--with-c2", action="store_true",
                    help="with --only-batch: run the 16 384-rank leg as well (for profiler runs)")
    ap.add_argument("--c2-host-input", action="store_true",
                    help="make the 16 384-rank leg's input on the host and upload it (for counter-profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 2 GiB elementwise copy kernel (known traffic) for counter calibration")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1 "
              "(sharding by step across GPUs exists as a design only)", file=sys.stderr)
        return 2
    import torch
    from workloads import generate, workload
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    w = workload(3)
    x = generate(w, seed=3, device="cuda")          # [T][M][R] fp32, resident in HBM
    det = make_detector(w)
    out, fl, tk = det.alloc_outputs(w.T), det.alloc_flags(), det.alloc_topk(w.topk)
    stream = torch.cuda.Stream()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(a.steps)]

    def step(i, timed):
        if timed:
            ev[i][0].record(stream)
        det.score_batch(x, out, stream)
        if timed:
            ev[i][1].record(stream)
        det.update_window(out, w.T, stream=stream)
        det.flags(fl, stream)
        det.topk_nodes(w.topk, tk, stream)

    with torch.cuda.stream(stream):
        for i in range(a.warmup):
            step(i, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(a.steps):
            step(i, True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    if a.calibrate_copy:        # a plain copy kernel of known size, for scaling HBM counters
        src = x[:1024].reshape(-1)                  # 2 GiB read ...
        dst = torch.empty_like(src)                 # ... 2 GiB written
        for _ in range(3):
            torch.add(src, 1.0, out=dst)            # one elementwise kernel: read src, write dst
        torch.cuda.synchronize()
        del dst
    # the ceiling of a single pass: the scoring kernel's loads alone over the same tensor
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
    with torch.cuda.stream(stream):
        for s0, s1 in pe:
            s0.record(stream)
            det.probe_read(x, sink, stream)
            s1.record(stream)
        torch.cuda.synchronize()
    read_ms = sorted(s0.elapsed_time(s1) for s0, s1 in pe)[2]
    ms_per_step = 1e3 * dt / a.steps
    score_ms = sum(s.elapsed_time(e) for s, e in ev) / a.steps
    alg = algorithmic_bytes_per_launch(w.R, w.M, w.T)
    achieved = alg / (score_ms * 1e-3) / 1e9
    res = {
        "metric": "telemetry samples scored/sec", "value": w.samples / (ms_per_step * 1e-3),
        "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.R} ranks x {w.T} steps x {w.M} metrics fp32 "
                               f"(heavy-tailed noise, W={w.W}, k={w.k}, top-{w.topk}); "
                               "score_batch + update_window + flags + topk_nodes per step"},
        "roofline": {"bound": "hbm", "kernel": "score_kernel<1024,16,12,true,false,false>", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(), "algorithmic_bytes": alg,
                     "avg_launch_ms": score_ms,
                     "read_only_ceiling": {"GB/s": x.numel() * 4 / (read_ms * 1e-3) / 1e9, "ms": read_ms,
                                           "what": "the same loads with no arithmetic (gd_probe_read)"},
                     "limited_by": "vector-instruction issue and the barrier-separated phases of the selection, "
                                   "not HBM: counter traffic equals the algorithmic bytes (see issue_view)",
                     "issue_view": issue_view(torch, w.samples, score_ms)},
    }
    res["detection"] = detection_report(torch, det, w, x, out, fl)
    if not a.only_batch:
        res["with_z"] = z_variant(torch, det, w, x, stream, alg)
        res["ledger"] = ledger_leg(torch, det, w, out, stream)
    if not a.no_cpu and not a.only_batch:
        res["cpu_baseline"] = cpu_baseline(w, x, a.cpu_sample_steps)
    del x, out
    torch.cuda.empty_cache()
    if not a.only_batch or a.with_c2:
        res["c2"] = c2_leg(torch, stream, a.c2_host_input)
        torch.cuda.empty_cache()
    if not a.no_stream and not a.only_batch:
        res["streaming"] = streaming_latency(torch, a.stream_steps)
    det.close()
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
